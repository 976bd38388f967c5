"""The five workloads' op sequences run on the oracle alone: properties that must hold whatever
the implementation (pool restored bit-exactly, onloaded bytes equal the originals, counts)."""
import numpy as np
import pytest

from backends import OracleBackend
from workloads import make_workload, flows


@pytest.mark.parametrize("cfg", [1, 3, 4])
def test_match_roundtrip_restores_pool(cfg):
    wl = make_workload(cfg, "small")
    be = OracleBackend()
    keep_fill = None
    tr = flows.flow_match_roundtrip(wl, be)
    assert len(tr["pages"]) > 0
    assert np.array_equal(tr["before"], tr["after"])
    from workloads import fill_pool_numpy
    assert np.array_equal(be.pool, fill_pool_numpy(wl.geom, wl.kv_dtype, wl.cfg))
    for s in tr["staged_samples"]:
        assert not np.all(s == flows.CANARY)


def test_offload_onload_small_cfg2():
    wl = make_workload(2, "small")
    be = OracleBackend()
    tr = flows.flow_offload_onload(wl, be)
    assert len(tr["onload_slots"]) > 0
    assert np.array_equal(tr["onloaded"], tr["onloaded_from"])
    assert np.all(tr["still_canary"] == flows.CANARY)
    for j, i in enumerate(tr["sample"]):
        assert np.array_equal(tr["staged"][j], tr["original_of_sample"][int(i)])
    ev, miss = tr["counters_evict"]
    assert miss == 0 and ev == len(tr["cold_keys"]) // 10
    assert tr["count"] == wl.n_live_target - ev
    assert np.all(tr["match_len"] <= np.diff(wl.blk_off))
    assert np.any(tr["match_len"] < np.diff(wl.blk_off))


def test_stress_small_cfg5():
    wl = make_workload(5, "small")
    be = OracleBackend()
    tr = flows.flow_stress(wl, be, n_rounds=4, q=512)
    assert tr["counters_evict"][0] == 4 * 512 and tr["counters_evict"][1] == 0
    assert tr["counters_insert"][2] == 0
    assert len(tr["round_values"]) == 4
