"""Pins for the oracle's chained block hash: worked vectors, an independent big-integer closed
form, and the invariants a prefix hash must have. None of these call the HIP library."""
import os

import numpy as np
import pytest

import oracle
from workloads import make_workload, make_tokens

M = (1 << 64) - 1
K0, K1, K2, K3 = 0x9E3779B97F4A7C15, 0x6A09E667F3BCC909, 0xBB67AE8584CAA73B, 0x3C6EF372FE94F82B

TOKEN_RULES = {
    "iota32": list(range(32)),
    "zeros32": [0] * 32,
    "iota64": list(range(64)),
    "desc48from31999": [31999 - i for i in range(48)],
}


def _h(tokens, B, seed=0):
    t = np.asarray(tokens, dtype=np.int32)
    return oracle.block_hash(t, [0, len(t)], [0, len(t) // B], B, seed)


def test_golden_vectors():
    path = os.path.join(os.path.dirname(__file__), "golden", "hash_vectors.txt")
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        left, right = line.split("|")
        B, seed, rule = left.split()
        want = [int(x, 16) for x in right.split()]
        got = _h(TOKEN_RULES[rule], int(B), int(seed, 16))
        assert [int(x) for x in got] == want, rule
        n += 1
    assert n == 4


# --- independent evaluation: Python ints, closed form of the affine chain ----------------------
def _F(x):
    x ^= x >> 32
    x = (x * K1) & M
    x ^= x >> 29
    x = (x * K2) & M
    return x ^ (x >> 32)


def _digest(block):
    c = 0
    for i, t in enumerate(block):
        y = (((int(t) & 0xFFFFFFFF) ^ (K0 * (i + 1))) * K1) & M
        c += y ^ (y >> 32)
    return _F(c & M)


def _closed_form(tokens, B, seed):
    """s_j = K2^(j+1) s_-1 + sum_{k<=j} K2^(j-k) d_k, every power taken with pow(.,.,2^64)."""
    n = len(tokens) // B
    d = [_digest(tokens[j * B:(j + 1) * B]) for j in range(n)]
    s0 = _F((seed ^ K3) & M)
    out = []
    for j in range(n):
        s = (pow(K2, j + 1, 1 << 64) * s0 + sum(pow(K2, j - k, 1 << 64) * d[k] for k in range(j + 1))) & M
        h = _F(s ^ K3)
        out.append(h ^ K0 if h in (0, M) else h)
    return out


@pytest.mark.parametrize("B,n_tok,seed", [(16, 16 * 37 + 5, 0), (64, 64 * 9, 12345), (1, 23, 7),
                                           (5, 64, M), (1024, 2048 + 100, 1 << 63)])
def test_closed_form_bigint(B, n_tok, seed):
    rng = np.random.default_rng(B * 1000 + n_tok)
    tok = rng.integers(-2**31, 2**31, size=n_tok, dtype=np.int64).astype(np.int32)
    assert [int(x) for x in _h(tok, B, seed)] == _closed_form([int(t) for t in tok], B, seed)


def test_negative_token_is_its_bit_pattern():
    a = _h([-1] * 16, 16)
    b = _closed_form([0xFFFFFFFF] * 16, 16, 0)
    assert int(a[0]) == b[0]


# --- invariants -------------------------------------------------------------------------------
def test_equal_prefixes_equal_hashes_on_every_config():
    for cfg in (1, 2, 3, 4, 5):
        wl = make_workload(cfg, "small")
        h = oracle.block_hash(wl.tokens, wl.tok_off, wl.blk_off, wl.block_size, 0)
        B = wl.block_size
        assert not np.any(h == 0) and not np.any(h == np.uint64(M))
        rng = np.random.default_rng(cfg)
        for _ in range(40):
            r, q = rng.integers(0, wl.n_req, size=2)
            tr = wl.tokens[wl.tok_off[r]:wl.tok_off[r + 1]]
            tq = wl.tokens[wl.tok_off[q]:wl.tok_off[q + 1]]
            m = min(len(tr), len(tq))
            neq = np.flatnonzero(tr[:m] != tq[:m])
            lcp = int(neq[0]) if len(neq) else m
            k = lcp // B
            hr = h[wl.blk_off[r]:wl.blk_off[r + 1]]
            hq = h[wl.blk_off[q]:wl.blk_off[q + 1]]
            assert np.array_equal(hr[:k], hq[:k])                      # H1
            nb = min(len(hr), len(hq))
            assert not np.any(hr[k:nb] == hq[k:nb])                    # H3: chain keeps them apart


def test_truncation_and_extension_do_not_change_earlier_blocks():
    rng = np.random.default_rng(1)
    tok = rng.integers(0, 32000, size=16 * 20 + 9, dtype=np.int32)
    full = _h(tok, 16)
    for cut in (16, 16 * 7, 16 * 7 + 15, 16 * 19):
        assert np.array_equal(_h(tok[:cut], 16), full[: cut // 16])    # H2
    assert len(_h(tok[:15], 16)) == 0                                   # shorter than a block


def test_order_sensitivity_and_seed():
    rng = np.random.default_rng(2)
    tok = rng.integers(0, 32000, size=64, dtype=np.int32)
    base = _h(tok, 16)
    t = tok.copy()
    t[3], t[9] = tok[9], tok[3]                                         # swap inside block 0
    assert _h(t, 16)[0] != base[0]
    t = tok.copy()
    t[0:16], t[16:32] = tok[16:32], tok[0:16]                           # swap blocks 0 and 1
    sw = _h(t, 16)
    assert sw[0] != base[0] and sw[1] != base[1]
    assert _h(tok, 16, seed=1)[0] != base[0]                            # H7
    # a change in block 2 leaves blocks 0,1 and changes 2,3
    t = tok.copy()
    t[40] ^= 1
    ch = _h(t, 16)
    assert np.array_equal(ch[:2], base[:2]) and ch[2] != base[2] and ch[3] != base[3]


def test_ragged_batch_equals_one_by_one():
    tok, tok_off, blk_off = make_tokens(5, 0, 40)
    h = oracle.block_hash(tok, tok_off, blk_off, 16, 99)
    for r in (0, 7, 39):
        one = _h(tok[tok_off[r]:tok_off[r + 1]], 16, 99)
        assert np.array_equal(one, h[blk_off[r]:blk_off[r + 1]])


def test_no_collisions_and_spread():
    rng = np.random.default_rng(3)
    tok = rng.integers(0, 32000, size=16 * 200000, dtype=np.int32)
    n = len(tok) // 16
    # every block its own request: 200k independent first-block hashes
    off = np.arange(n + 1, dtype=np.int64)
    h = oracle.block_hash(tok, off * 16, off, 16, 0)
    assert len(np.unique(h)) == n
    for shift in (0, 54):                                               # low and high 10 bits
        cnt = np.bincount(((h >> np.uint64(shift)) & np.uint64(1023)).astype(np.int64), minlength=1024)
        assert abs(cnt - n / 1024).max() < 6 * np.sqrt(n / 1024)


def test_invalid_arguments_are_rejected():
    tok = np.zeros(32, dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.block_hash(tok, [0, 32], [0, 2], 0, 0)
    with pytest.raises(ValueError):
        oracle.block_hash(tok, [0, 32], [0, 2], 1025, 0)
    with pytest.raises(ValueError):
        oracle.block_hash(tok, [0, 32], [0, 3], 16, 0)                  # wrong block count
    assert len(oracle.block_hash(tok[:0], [0], [0], 16, 0)) == 0        # zero requests


def test_finaliser_is_a_bijection_with_known_inverse():
    """Undo each step with the modular inverses of the two odd multipliers and the xor-shift
    inverses; the round trip must return the input."""
    i1, i2 = pow(K1, -1, 1 << 64), pow(K2, -1, 1 << 64)

    def unshift(x, s):
        y = x
        for _ in range(64 // s + 1):
            y = x ^ (y >> s)
        return y

    rng = np.random.default_rng(4)
    for x in [0, 1, M, 1 << 63] + [int(v) for v in rng.integers(0, M, size=200, dtype=np.uint64)]:
        y = oracle.finalise(x)
        assert y == _F(x)
        z = unshift(y, 32)
        z = (z * i2) & M
        z = unshift(z, 29)
        z = (z * i1) & M
        z = unshift(z, 32)
        assert z == x


def test_reserved_values_are_remapped():
    assert oracle.avoid_reserved(0) == K0
    assert oracle.avoid_reserved(M) == M ^ K0
    for v in (1, M - 1, K0, 12345):
        assert oracle.avoid_reserved(v) == v


def test_token_term_matches_definition():
    for t, i in [(0, 0), (31999, 15), (-1, 63), (-2**31, 1023), (7, 3)]:
        y = (((t & 0xFFFFFFFF) ^ (K0 * (i + 1))) * K1) & M
        assert oracle.token_term(t, i) == y ^ (y >> 32)
