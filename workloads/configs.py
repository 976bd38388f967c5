"""The five synthetic workloads (multi-turn chat and shared-system-prompt serving shapes).

They stand in for the traffic the paper's distributed KV cache targets (Section 3.2.5: multi-turn
applications with overlapping token sequences) and for its Bird-SQL run, whose items are not
reproduced here. Everything is drawn from numpy's PCG64 with entropy 0 and a spawn key
(config, replica, stream), so every consumer sees the same bytes.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

VOCAB = 32000

CONFIG_NAMES = {
    1: "tiny-16req-pagemajor-bf16",
    2: "llama3-8b-64req-4096tok-bf16",
    3: "llama3-70b-256req-zipf-bf16",
    4: "mla-128req-16384tok-latent-bf16",
    5: "stress-1024req-lognormal-fp8",
}

# spawn-key stream ids
_S_LEN, _S_SHARED, _S_TAIL, _S_PAGES, _S_FILL, _S_OPS, _S_KV, _S_PICK = range(8)


def _rng(cfg: int, replica: int, stream: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence(0, spawn_key=(cfg, replica, stream)))


@dataclass
class Geometry:
    """Paged KV pool: n_seg planes, each n_pages x seg_bytes; a block is its n_seg segments."""
    n_seg: int
    seg_bytes: int
    n_pages: int
    layout: str = "layer-major"        # "layer-major": plane-strided; "page-major": n_seg == 1

    @property
    def blk_bytes(self) -> int:
        return self.n_seg * self.seg_bytes

    @property
    def page_stride(self) -> int:
        return self.seg_bytes

    @property
    def seg_stride(self) -> int:
        return self.n_pages * self.seg_bytes

    @property
    def pool_bytes(self) -> int:
        return self.n_seg * self.n_pages * self.seg_bytes

    def as_tuple(self):
        return (self.n_seg, self.seg_stride, self.page_stride, self.seg_bytes, self.n_pages)

    def page_major(self) -> "Geometry":
        """Same bytes per block held as one contiguous segment per page."""
        return Geometry(1, self.blk_bytes, self.n_pages, "page-major")


@dataclass
class Workload:
    cfg: int
    name: str
    scale: str
    block_size: int
    hash_seed: int
    tokens: np.ndarray                 # int32[T], requests concatenated
    tok_off: np.ndarray                # int64[R+1]
    blk_off: np.ndarray                # int64[R+1], floor(len/B) prefix sums
    n_slots: int                       # index capacity (power of two)
    load_factor: float                 # live keys / n_slots after preload
    geom: Geometry
    kv_dtype: str                      # "bf16" | "fp8"
    batch_pages: int                   # pages per gather/scatter call
    page_perm: np.ndarray              # int32[n_pages] random permutation (block rank -> page)
    preload_requests: Optional[int] = None   # cfg 1: only these first requests are indexed
    extra: dict = field(default_factory=dict)

    @property
    def n_req(self) -> int:
        return len(self.tok_off) - 1

    @property
    def n_blocks(self) -> int:
        return int(self.blk_off[-1])

    @property
    def n_live_target(self) -> int:
        return int(self.n_slots * self.load_factor)


def zipf_sample(rng: np.random.Generator, n: int, k: int, s: float) -> np.ndarray:
    """n draws from P(i) ~ (i+1)^-s over i in [0, k), by inverse CDF."""
    w = np.arange(1, k + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    return np.minimum(np.searchsorted(cdf, rng.random(n), side="left"), k - 1).astype(np.int64)


def _tok(rng, n):
    return rng.integers(0, VOCAB, size=int(n), dtype=np.int32)


def _request_lengths_and_prefixes(cfg: int, replica: int, n_req: int):
    """Returns (lengths int64[R], prefix_id int64[R], prefix_tokens list, shared_len int64[R])."""
    r_len, r_sh = _rng(cfg, replica, _S_LEN), _rng(cfg, replica, _S_SHARED)
    if cfg == 1:
        lens = r_len.integers(256, 1025, size=n_req)
        pid = np.arange(n_req) % 4
        prefixes = [_tok(r_sh, 512) for _ in range(4)]
        shared = np.minimum(lens, 512)
    elif cfg == 2:
        lens = np.full(n_req, 4096)
        pid = np.arange(n_req) // 8
        prefixes = [_tok(r_sh, 2048) for _ in range(int(pid.max()) + 1)]
        shared = np.full(n_req, 2048)
    elif cfg == 3:
        lens = r_len.integers(2048, 8193, size=n_req)
        pid = zipf_sample(r_len, n_req, 512, 1.1)
        prefixes = [_tok(r_sh, 1024) for _ in range(512)]
        shared = np.full(n_req, 1024)
    elif cfg == 4:
        lens = np.full(n_req, 16384)
        pid = np.arange(n_req) // 16
        prefixes = [_tok(r_sh, 8192) for _ in range(int(pid.max()) + 1)]
        shared = np.full(n_req, 8192)
    elif cfg == 5:
        lens = np.exp(r_len.normal(np.log(2048.0), 1.0, size=n_req)).astype(np.int64)
        lens = np.clip(lens, 16, 32768)
        n_prompts = 10000
        pid = zipf_sample(r_len, n_req, n_prompts, 1.0)
        plen = r_sh.integers(16, 129, size=n_prompts) * 16            # 256 .. 2048 step 16
        used = np.unique(pid)
        table = {int(p): _tok(np.random.default_rng(
            np.random.SeedSequence(0, spawn_key=(cfg, replica, _S_SHARED, int(p)))), plen[p])
            for p in used}
        prefixes = table
        shared = np.minimum(lens, plen[pid])
    else:
        raise ValueError(f"unknown config {cfg}")
    return lens.astype(np.int64), pid.astype(np.int64), prefixes, shared.astype(np.int64)


_DEFAULT_REQ = {1: 16, 2: 64, 3: 256, 4: 128, 5: 1024}
_BLOCK = {1: 16, 2: 16, 3: 16, 4: 64, 5: 16}


def make_tokens(cfg: int, replica: int = 0, n_req: Optional[int] = None):
    """Token streams of one replica of config `cfg`: (tokens int32[T], tok_off, blk_off)."""
    n_req = _DEFAULT_REQ[cfg] if n_req is None else int(n_req)
    lens, pid, prefixes, shared = _request_lengths_and_prefixes(cfg, replica, n_req)
    r_tail = _rng(cfg, replica, _S_TAIL)
    tok_off = np.zeros(n_req + 1, dtype=np.int64)
    np.cumsum(lens, out=tok_off[1:])
    tokens = _tok(r_tail, tok_off[-1])                    # unique tails everywhere ...
    for r in range(n_req):                                # ... then the shared prefix on top
        k = int(shared[r])
        tokens[tok_off[r]:tok_off[r] + k] = prefixes[int(pid[r])][:k]
    blk_off = np.zeros(n_req + 1, dtype=np.int64)
    np.cumsum(lens // _BLOCK[cfg], out=blk_off[1:])
    return tokens, tok_off, blk_off


def make_scaled_tokens(cfg: int, min_blocks: int, n_req: Optional[int] = None):
    """Replicas 0, 1, 2, ... of the config's request mix concatenated until at least `min_blocks`
    blocks are covered (the scaled batch on which hash+match throughput is measured)."""
    toks, lens, blks = [], [], []
    total, k = 0, 0
    while total < min_blocks or k == 0:
        t, to, bo = make_tokens(cfg, k, n_req)
        toks.append(t)
        lens.append(np.diff(to))
        blks.append(np.diff(bo))
        total += int(bo[-1])
        k += 1
    lens, blks = np.concatenate(lens), np.concatenate(blks)
    tok_off = np.zeros(len(lens) + 1, dtype=np.int64)
    np.cumsum(lens, out=tok_off[1:])
    blk_off = np.zeros(len(blks) + 1, dtype=np.int64)
    np.cumsum(blks, out=blk_off[1:])
    return np.concatenate(toks), tok_off, blk_off


def _geometry(cfg: int, scale: str) -> tuple:
    """(Geometry, kv_dtype, n_slots, load_factor, batch_pages)."""
    small = scale == "small"
    if cfg == 1:      # one page = [K/V=2, 4 layers, 16 tok, 8 heads, 128] bf16, page-major
        g = Geometry(1, 2 * 4 * 16 * 8 * 128 * 2, 256 if small else 2048, "page-major")
        return g, "bf16", 4096, 0.0, g.n_pages
    if cfg == 2:      # 32 layers x {K,V}; segment = 16 tok x 8 heads x 128 x bf16
        g = Geometry(4 if small else 64, 16 * 8 * 128 * 2, 2560 if small else 20000)
        return g, "bf16", (1 << 14) if small else (1 << 20), 0.5, 4608
    if cfg == 3:      # 80 layers x {K,V}
        g = Geometry(10 if small else 160, 16 * 8 * 128 * 2, 2048 if small else 32768)
        return g, "bf16", (1 << 16) if small else (1 << 22), 0.7, 256 if small else 4096
    if cfg == 4:      # 61 layers, latent 512 + rope 64, 64-token pages
        g = Geometry(3 if small else 61, 64 * (512 + 64) * 2, 768 if small else 17408)
        return g, "bf16", (1 << 15) if small else (1 << 22), 0.5, 128 if small else 2048
    if cfg == 5:      # 32 layers x {K,V}, fp8 bytes
        g = Geometry(4 if small else 64, 16 * 8 * 128 * 1, 4096 if small else 131072)
        return g, "fp8", (1 << 17) if small else (1 << 24), 0.75, 256 if small else 4096
    raise ValueError(f"unknown config {cfg}")


_SMALL_REQ = {1: 16, 2: 16, 3: 24, 4: 16, 5: 64}


def make_workload(cfg: int, scale: str = "full", layout: Optional[str] = None) -> Workload:
    """Config `cfg` (1..5). scale="small" keeps block size, segment size, sharing pattern and
    length distribution but cuts requests, layers, pages and index slots so that a CPU run of the
    oracle finishes in seconds. layout="page-major" folds each block into one segment."""
    assert scale in ("full", "small")
    n_req = _SMALL_REQ[cfg] if scale == "small" else _DEFAULT_REQ[cfg]
    tokens, tok_off, blk_off = make_tokens(cfg, 0, n_req)
    geom, kv_dtype, n_slots, lf, batch = _geometry(cfg, scale)
    if layout == "page-major":
        geom = geom.page_major()
    perm = _rng(cfg, 0, _S_PAGES).permutation(geom.n_pages).astype(np.int32)
    return Workload(cfg=cfg, name=CONFIG_NAMES[cfg], scale=scale, block_size=_BLOCK[cfg],
                    hash_seed=0, tokens=tokens, tok_off=tok_off, blk_off=blk_off, n_slots=n_slots,
                    load_factor=lf, geom=geom, kv_dtype=kv_dtype, batch_pages=batch,
                    page_perm=perm, preload_requests=8 if cfg == 1 else None)


def filler_keys(cfg: int, n: int) -> tuple:
    """n distinct random index keys (never 0 or 2^64-1) with values 2^63 | k ("held elsewhere")."""
    rng = _rng(cfg, 0, _S_FILL)
    keys = rng.integers(1, np.iinfo(np.uint64).max, size=int(n * 1.01) + 16, dtype=np.uint64)
    keys = keys[np.sort(np.unique(keys, return_index=True)[1])][:n]
    assert len(keys) == n
    values = (np.uint64(1) << np.uint64(63)) | np.arange(n, dtype=np.uint64)
    return keys, values


def ops_rng(cfg: int, tag: int = 0) -> np.random.Generator:
    """Stream for op-sequence choices (which keys to evict, which pages to move)."""
    return np.random.default_rng(np.random.SeedSequence(0, spawn_key=(cfg, 0, _S_OPS, tag)))


def _f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = x.astype(np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16          # round to nearest even
    return u.astype(np.uint16)


def fill_pool_numpy(geom: Geometry, kv_dtype: str, cfg: int) -> np.ndarray:
    """Host pool bytes: bf16 N(0,1) values, or uniform random bytes standing in for fp8 e4m3."""
    rng = _rng(cfg, 0, _S_KV)
    n = geom.pool_bytes
    if kv_dtype == "bf16":
        out = np.empty(n // 2, dtype=np.uint16)
        step = 1 << 22
        for i in range(0, len(out), step):
            m = min(step, len(out) - i)
            out[i:i + m] = _f32_to_bf16_bits(rng.standard_normal(m, dtype=np.float32))
        return out.view(np.uint8)
    return rng.integers(0, 256, size=n, dtype=np.uint8)


def fill_pool_torch(pool, kv_dtype: str, cfg: int) -> None:
    """Device pool bytes, in place (`pool`: 1-D uint8 torch tensor on the GPU). Same distributions
    as fill_pool_numpy, drawn by torch's generator in 256 MiB pieces."""
    import torch
    gen = torch.Generator(device=pool.device)
    gen.manual_seed(1000 + cfg)
    step = 1 << 28
    for i in range(0, pool.numel(), step):
        piece = pool[i:i + step]
        if kv_dtype == "bf16":
            v = torch.randn(piece.numel() // 2, device=pool.device, dtype=torch.float32,
                            generator=gen).to(torch.bfloat16)
            piece.copy_(v.view(torch.uint8))
        else:
            piece.copy_(torch.randint(0, 256, (piece.numel(),), device=pool.device,
                                      dtype=torch.uint8, generator=gen))
