"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2504_03648_amd import binding
    return binding.load()


def _declared():
    text = open(os.path.join(ROOT, "include", "aibx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aibx_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2504_03648_amd import binding
    names = _declared()
    assert len(names) >= 16
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_version_and_strerror(lib):
    assert lib.aibx_version() >= 100 and lib.aibx_hash_version() == 1
    assert lib.aibx_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -99):
        assert len(lib.aibx_strerror(code)) > 0


def test_storage_bytes_rules(lib):
    out = C.c_size_t()
    assert lib.aibx_index_storage_bytes(1 << 20, C.byref(out)) == 0 and out.value == 21 << 20
    assert lib.aibx_index_storage_bytes(8, C.byref(out)) == 0 and out.value == 168
    for bad in (0, 4, 12, 1000, (1 << 20) + 8, 1 << 40):
        assert lib.aibx_index_storage_bytes(bad, C.byref(out)) == -3
    assert lib.aibx_index_storage_bytes(64, None) == -1


def test_argument_errors_are_raised_before_any_launch(lib):
    from paper_2504_03648_amd.binding import PoolDesc
    fake = C.c_void_p(0x1000)         # never dereferenced: every call below must fail on the host
    odd = C.c_void_p(0x1004)
    # block hash
    assert lib.aibx_block_hash(fake, fake, fake, -1, 0, 16, 0, fake, None) == -1
    assert lib.aibx_block_hash(fake, fake, fake, 1, 1, 0, 0, fake, None) == -1
    assert lib.aibx_block_hash(fake, fake, fake, 1, 1, 1025, 0, fake, None) == -1
    assert lib.aibx_block_hash(None, fake, fake, 1, 1, 16, 0, fake, None) == -1
    assert lib.aibx_block_hash(fake, odd, fake, 1, 1, 16, 0, fake, None) == -2
    assert lib.aibx_block_hash(fake, fake, fake, 0, 0, 16, 0, fake, None) == 0      # empty batch
    # index
    h = C.c_void_p()
    assert lib.aibx_index_create(None, 1 << 20, 64, None, C.byref(h)) == -1
    assert lib.aibx_index_create(fake, 1 << 20, 100, None, C.byref(h)) == -3
    assert lib.aibx_index_create(fake, 16, 64, None, C.byref(h)) == -1               # storage too small
    assert lib.aibx_index_create(odd, 1 << 20, 64, None, C.byref(h)) == -2
    assert lib.aibx_index_insert(None, fake, fake, 1, None, None) == -1
    assert lib.aibx_index_evict(None, fake, 1, None, None, None) == -1
    assert lib.aibx_prefix_match(None, fake, fake, 1, 1, None, fake, None) == -1
    assert lib.aibx_index_destroy(None) == 0
    assert lib.aibx_index_touch(None, fake, 1, 0, None) == -1
    assert lib.aibx_index_age(None, None) == -1
    assert lib.aibx_index_stats(None, fake, None) == -1
    assert lib.aibx_index_rebuild(None, None, None, None) == -1
    assert lib.aibx_index_select_victims(None, 2, 5, fake, fake, 1, fake, None) == -1
    assert lib.aibx_hash_match(None, fake, fake, fake, 1, 1, 16, 0, fake, fake, fake, None) == -1
    # routing straight from the tokens
    f = lib.aibx_hash_match_route
    h1 = C.c_void_p(0x2000)   # stands for an index handle; never dereferenced before the checks below fail
    assert f(None, fake, fake, fake, 1, 1, 16, 0, 8, fake, 1, 2, fake, fake, None) == -1
    assert f(h1, fake, fake, fake, 1, 1, 16, 0, 0, fake, 1, 2, fake, fake, None) == -1
    assert f(h1, fake, fake, fake, 1, 1, 16, 0, 64, fake, 1, 2, fake, fake, None) == -1
    assert f(h1, fake, fake, fake, 1, 1, 16, 0, 8, fake, 1, 0, fake, fake, None) == -1
    assert f(h1, fake, fake, fake, 1, 1, 16, 0, 8, None, 1, 2, fake, fake, None) == -1
    assert f(h1, fake, odd, fake, 1, 1, 16, 0, 8, fake, 1, 2, fake, fake, None) == -2
    assert f(h1, fake, fake, fake, 1, 1, 24, 0, 8, fake, 1, 2, fake, fake, None) == -3
    assert f(h1, fake, fake, fake, 0, 0, 16, 0, 8, fake, 1, 2, fake, fake, None) == 0
    # routing
    assert lib.aibx_route(fake, fake, 1, 1, 0, fake, 1, 2, fake, fake, None) == -1
    assert lib.aibx_route(fake, fake, 1, 1, 64, fake, 1, 2, fake, fake, None) == -1
    assert lib.aibx_route(fake, fake, 1, 1, 8, fake, 1, 0, fake, fake, None) == -1
    assert lib.aibx_route(fake, fake, 0, 0, 8, fake, 1, 2, fake, fake, None) == 0
    assert lib.aibx_route(fake, odd, 1, 1, 8, fake, 1, 2, fake, fake, None) == -2
    # copies
    d = PoolDesc(0x1000, 2, 1 << 20, 4096, 4096, 16)
    assert lib.aibx_kv_gather(C.byref(d), fake, None, -1, fake, 8192, None, None) == -1
    assert lib.aibx_kv_gather(C.byref(d), fake, None, 0, fake, 8192, None, None) == 0
    assert lib.aibx_kv_gather(None, fake, None, 1, fake, 8192, None, None) == -1
    assert lib.aibx_kv_gather(C.byref(d), fake, None, 1, fake, 4096, None, None) == -1  # stride < block
    assert lib.aibx_kv_gather(C.byref(d), fake, None, 1, fake, 8200, None, None) == -2
    assert lib.aibx_kv_scatter(C.byref(d), fake, None, 1, odd, 8192, None, None) == -2
    for f in (lib.aibx_kv_gather_fill, lib.aibx_kv_scatter_fill):
        assert f(C.byref(d), fake, None, fake, -1, fake, 8192, None, None) == -1
        assert f(C.byref(d), fake, None, fake, 0, fake, 8192, None, None) == 0
        assert f(None, fake, None, fake, 1, fake, 8192, None, None) == -1
        assert f(C.byref(d), fake, None, C.c_void_p(0x1002), 1, fake, 8192, None, None) == -2   # fill counts are int32
        assert f(C.byref(d), fake, None, fake, 1, fake, 4096, None, None) == -1     # stride < block
    for f in (lib.aibx_kv_offload, lib.aibx_kv_onload):
        assert f(C.byref(d), fake, -1, fake, 8192, None, None) == -1
        assert f(C.byref(d), fake, 0, fake, 8192, None, None) == 0
        assert f(None, fake, 1, fake, 8192, None, None) == -1
        assert f(C.byref(d), fake, 1, None, 8192, None, None) == -1
        assert f(C.byref(d), fake, 1, fake, 4096, None, None) == -1      # host stride < block
        assert f(C.byref(d), fake, 1, odd, 8192, None, None) == -2
        assert f(C.byref(d), fake, 1, fake, 8200, None, None) == -2
        # an address that is not pinned host memory is refused before any launch
        assert f(C.byref(d), fake, 1, fake, 8192, None, None) == -1
    from paper_2504_03648_amd.binding import PoolRunsDesc
    rd = PoolRunsDesc(0x1000, 4, 16, 2048, 16 * 4 * 2048, 4 * 2048, 2048, 8)      # token-major, 128 KiB pages
    for f in (lib.aibx_kv_gather_runs, lib.aibx_kv_scatter_runs):
        assert f(C.byref(rd), fake, None, -1, fake, 1 << 17, None, None) == -1
        assert f(C.byref(rd), fake, None, 0, fake, 1 << 17, None, None) == 0
        assert f(None, fake, None, 1, fake, 1 << 17, None, None) == -1
        assert f(C.byref(rd), fake, None, 1, fake, (1 << 17) - 16, None, None) == -1   # stride < block
        assert f(C.byref(rd), fake, None, 1, odd, 1 << 17, None, None) == -2
        assert f(C.byref(PoolRunsDesc(0x1000, 4, 0, 2048, 1 << 17, 8192, 2048, 8)), fake, None, 1, fake, 1 << 17, None, None) == -1
        assert f(C.byref(PoolRunsDesc(0x1000, 4, 16, 2048, 1 << 17, 8192, 2040, 8)), fake, None, 1, fake, 1 << 17, None, None) == -2
        assert f(C.byref(PoolRunsDesc(0x1000, 4, 16, 2048, 1 << 17, 1024, 2048, 8)), fake, None, 1, fake, 1 << 17, None, None) == -1  # runs overlap
        assert f(C.byref(PoolRunsDesc(0x1000, 1, 1 << 20, 4096, 1 << 32, 4096, 4096, 8)), fake, None, 1, fake, 1 << 32, None, None) == -3  # segment of 4 GiB
    bad = PoolDesc(0x1000, 2, 1 << 20, 4096, 4100, 16)
    assert lib.aibx_kv_gather(C.byref(bad), fake, None, 1, fake, 8208, None, None) == -1  # page_stride < seg
    bad = PoolDesc(0x1000, 2, 1 << 20, 4112, 4104, 16)
    assert lib.aibx_kv_gather(C.byref(bad), fake, None, 1, fake, 8208, None, None) == -2
    bad = PoolDesc(0x1000, 0, 1 << 20, 4096, 4096, 16)
    assert lib.aibx_kv_scatter(C.byref(bad), fake, None, 1, fake, 8192, None, None) == -1


def test_copy_launch_split_respects_the_grid_limit(lib):
    """A launch holds at most 2^32 - 1 threads (256 per workgroup, one workgroup per 4 KiB tile):
    calls that move 64 GiB or more are split, entries are never cut, nothing is left out."""
    from paper_2504_03648_amd.binding import PoolDesc, aibx_kv_copy_launches
    max_groups = ((2**32 - 1) // 256) & ~7
    cases = [
        (160, 32768, 16384),      # half of the 160 GiB pool of the 70B-shaped config: 80 GiB
        (160, 32768, 32768),      # all of it
        (64, 32768, 4608),        # one batch of the 8B-shaped config: a single launch
        (1, 4497408, 17408),      # page-major latent pages (ragged last tile per segment)
        (61, 73728, 17408),
        (1, 16, 1 << 26),         # 16-byte segments: one tile per entry
        (3, 4096 * 5_000_000, 3), # a block of 15 M tiles: one entry per launch
    ]
    for n_seg, seg_bytes, n in cases:
        d = PoolDesc(0x1000, n_seg, 1 << 40, seg_bytes, seg_bytes, 1 << 30)
        tpb = -(-seg_bytes // 4096) * n_seg
        plan, k = aibx_kv_copy_launches(d, n, capacity=64)
        assert k == len(plan) >= 1
        nxt = 0
        for first, cnt, grid in plan:
            assert first == nxt and cnt >= 1
            assert grid % 8 == 0 and grid * 256 < 2**32 and grid <= max_groups
            assert cnt * tpb <= grid < cnt * tpb + 8
            nxt = first + cnt
        assert nxt == n
        assert all(c == plan[0][1] for _, c, _ in plan[:-1])          # equal launches, then the rest
        assert k == -(-n // (max_groups // tpb))
    plan, k = aibx_kv_copy_launches(PoolDesc(0x1000, 160, 1 << 30, 32768, 32768, 32768), 16384)
    assert k == 2                                                      # 80 GiB: two launches
    plan, k = aibx_kv_copy_launches(PoolDesc(0x1000, 1, 0, 16, 16, 8), 0)
    assert (plan, k) == ([], 0)
    plan, k = aibx_kv_copy_launches(PoolDesc(0x1000, 1, 0, 16, 16, 8), 1 << 30, capacity=4)
    assert k == -(-(1 << 30) // max_groups) and len(plan) == 4         # more launches than asked for
    big = PoolDesc(0x1000, 8, 1 << 50, 4096 * 3_000_000, 4096 * 3_000_000, 8)   # 24 M tiles in one block
    assert lib.aibx_kv_copy_launches(C.byref(big), 1, None, None, None, 0) == -3
    assert lib.aibx_kv_gather(C.byref(big), C.c_void_p(0x1000), None, 1, C.c_void_p(0x1000), 8 * 4096 * 3_000_000,
                              None, None) == -3
    assert lib.aibx_kv_copy_launches(None, 1, None, None, None, 0) == -1


def test_calibration_kernel_rejects_bad_arguments(lib):
    fake = C.c_void_p(0x1000)
    f = lib.aibx_calib_random_reads
    assert f(None, 1 << 20, 128, 8, 10, 0, fake, None) == -1
    assert f(fake, 1 << 20, 128, 8, -1, 0, fake, None) == -1
    assert f(fake, 1 << 20, 100, 8, 10, 0, fake, None) == -1          # line size not a power of two
    assert f(fake, (1 << 20) + 128, 128, 8, 10, 0, fake, None) == -1  # table size not a power of two
    assert f(fake, 1 << 20, 64, 128, 10, 0, fake, None) == -1         # read longer than a line
    assert f(fake, 1 << 20, 128, 24, 10, 0, fake, None) == -1
    assert f(C.c_void_p(0x1040), 1 << 20, 128, 8, 10, 0, fake, None) == -2
    assert f(fake, 1 << 20, 128, 8, 0, 0, fake, None) == 0
