"""Seeded synthetic inputs shaped like relQuery serving batches.

This module holds no arithmetic of the layer step: it only draws random
numbers, lays out page tables and converts fp32 draws to bf16 bit patterns.
Both the CPU oracle's tests and the GPU path's tests/benchmark take their
inputs from here so that the two sides see the same bits.

Workload structure (Sec. 2.2 Def. 2.1: the requests of one relQuery are one
template filled with different rows, hence a long shared token prefix and a
short private suffix; Sec. 5.1 "Datasets and Workloads": inputs of a few
hundred tokens, outputs of 5-100 tokens, 1-100 requests per relQuery).  The
datasets and trained weights themselves are replaced by random draws.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace

import numpy as np


# ----------------------------------------------------------------------------
# bf16 bit patterns (format conversion only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# shapes
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class LayerShape:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp_dim: int
    page_size: int = 16
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def qkv_dim(self) -> int:
        return self.q_dim + 2 * self.kv_dim

    @property
    def params(self) -> int:
        H, I = self.hidden, self.mlp_dim
        return self.qkv_dim * H + H * self.q_dim + 3 * I * H + 2 * H


TINY = LayerShape(256, 4, 4, 64, 688)
TINY_GQA = LayerShape(256, 8, 2, 64, 688)
TINY_D128 = LayerShape(256, 2, 1, 128, 688)
TINY_G5 = LayerShape(256, 10, 2, 64, 688)        # 5 query heads per kv head: the group does not divide a 128-row tile
TINY_G3_D128 = LayerShape(256, 6, 2, 128, 688)
LLAMA_13B = LayerShape(5120, 40, 40, 128, 13824)
LLAMA_70B = LayerShape(8192, 64, 8, 128, 28672)
LLAMA_70B_TP4 = LayerShape(8192, 16, 2, 128, 7168)     # one GPU's share of the 70B layer under 4-way tensor parallelism (Sec. 5.1)
QWEN_32B_TP2 = LayerShape(5120, 20, 4, 128, 13824)     # one GPU's share of the 32B layer under 2-way tensor parallelism
QWEN_32B = LayerShape(5120, 40, 8, 128, 27648)   # Sec. 5.1: the 32B model of the evaluation (grouped-query, 5 heads per kv head)


# ----------------------------------------------------------------------------
# batch descriptor
# ----------------------------------------------------------------------------
@dataclass
class Batch:
    """Host-side batch descriptor (what the scheduler hands to the GPU worker)."""
    q_start: np.ndarray        # int32 [B+1]
    ctx_len: np.ndarray        # int32 [B], sequence length after this step's append
    block_table: np.ndarray    # int32 [B, max_blocks]
    prefix_id: np.ndarray      # int32 [B], -1 = no shared prefix
    prefix_len: np.ndarray     # int32 [num_prefixes], multiples of the page size
    num_pages: int
    name: str = ""

    @property
    def num_reqs(self) -> int:
        return int(len(self.ctx_len))

    @property
    def T(self) -> int:
        return int(self.q_start[-1])

    @property
    def q_len(self) -> np.ndarray:
        return np.diff(self.q_start).astype(np.int32)

    @property
    def past(self) -> np.ndarray:
        return (self.ctx_len - self.q_len).astype(np.int32)

    def select(self, reqs) -> "Batch":
        """Sub-batch holding the given requests (same pages, same cache)."""
        reqs = np.asarray(reqs, dtype=np.int64)
        ql = self.q_len[reqs]
        qs = np.zeros(len(reqs) + 1, np.int32)
        qs[1:] = np.cumsum(ql)
        return replace(self, q_start=qs, ctx_len=self.ctx_len[reqs].copy(),
                       block_table=np.ascontiguousarray(self.block_table[reqs]),
                       prefix_id=self.prefix_id[reqs].copy())

    def token_rows(self, reqs) -> np.ndarray:
        """Packed row indices (in THIS batch) of the query tokens of the given requests."""
        out = [np.arange(self.q_start[r], self.q_start[r + 1]) for r in reqs]
        return np.concatenate(out).astype(np.int64) if out else np.zeros(0, np.int64)


class PagePool:
    """Hands out page ids in a seeded random order (non-contiguous on purpose)."""

    def __init__(self, num_pages: int, rng: np.random.Generator):
        self.order = rng.permutation(num_pages).astype(np.int32)
        self.next = 0
        self.num_pages = num_pages

    def take(self, n: int) -> np.ndarray:
        if self.next + n > self.num_pages:
            raise ValueError("page pool exhausted")
        out = self.order[self.next:self.next + n]
        self.next += n
        return out


def build_batch(shape: LayerShape, q_len, ctx_len, prefix_id=None, prefix_len=(), seed: int = 0,
                spare_pages: int = 3, name: str = "") -> Batch:
    """Lay out block tables: one page run per shared prefix, private pages for the rest."""
    P = shape.page_size
    q_len = np.asarray(q_len, np.int32)
    ctx_len = np.asarray(ctx_len, np.int32)
    B = len(q_len)
    prefix_id = np.full(B, -1, np.int32) if prefix_id is None else np.asarray(prefix_id, np.int32)
    prefix_len = np.asarray(prefix_len, np.int32).reshape(-1)
    assert np.all(prefix_len % P == 0)
    blocks = (ctx_len + P - 1) // P
    max_blocks = int(blocks.max()) if B else 1
    shared = prefix_len // P
    shared_of = np.zeros(B, np.int64)
    if len(shared):
        shared_of = np.where(prefix_id >= 0, shared[np.maximum(prefix_id, 0)], 0)
    priv = blocks - shared_of
    assert np.all(priv >= 0)
    num_pages = int(shared.sum() + priv.sum() + spare_pages)
    rng = np.random.default_rng(seed ^ 0x5EED)
    pool = PagePool(num_pages, rng)
    prefix_pages = [pool.take(int(n)) for n in shared]
    bt = np.full((B, max_blocks), -1, np.int32)
    for r in range(B):
        n0 = 0
        if prefix_id[r] >= 0:
            pp = prefix_pages[prefix_id[r]]
            bt[r, :len(pp)] = pp
            n0 = len(pp)
        bt[r, n0:blocks[r]] = pool.take(int(blocks[r] - n0))
    qs = np.zeros(B + 1, np.int32)
    qs[1:] = np.cumsum(q_len)
    # unused tail entries point at page 0: harmless, never dereferenced by a correct reader
    bt[bt < 0] = 0
    return Batch(qs, ctx_len, bt, prefix_id, prefix_len, num_pages, name)


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------
def make_weights(shape: LayerShape, seed: int, n_layers: int = 0) -> dict:
    """bf16 bit patterns: projections ~N(0, 0.02), norm weights 1 + N(0, 0.02).

    n_layers > 0 selects the depth-scaled random init used for the 13B / 70B shaped
    layers: the two projections that write into the residual stream (w_o, w_down)
    get std 0.02 / sqrt(2 n_layers), as a stack of that depth is initialised, so that
    one layer moves the stream by a fraction of its magnitude instead of doubling it.
    """
    rng = np.random.default_rng(seed)
    H, I = shape.hidden, shape.mlp_dim
    out_std = 0.02 / np.sqrt(2.0 * n_layers) if n_layers > 0 else 0.02

    def proj(n, k, std=0.02):
        return f32_to_bf16_bits(rng.standard_normal((n, k), dtype=np.float32) * np.float32(std))

    def norm():
        return f32_to_bf16_bits(np.float32(1.0) + rng.standard_normal(H, dtype=np.float32) * np.float32(0.02))

    return {"w_in_norm": norm(), "w_qkv": proj(shape.qkv_dim, H), "w_o": proj(H, shape.q_dim, out_std),
            "w_post_norm": norm(), "w_gate_up": proj(2 * I, H), "w_down": proj(H, I, out_std)}


def e4m3_code_values() -> np.ndarray:
    """Value of each of the 256 codes of the 8-bit floating point format (1 sign, 4 exponent, 3 mantissa bits, bias 7;
    0x7f / 0xff are NaN).  A format table, no arithmetic of the method."""
    c = np.arange(256)
    e, m = (c >> 3) & 15, c & 7
    mag = np.where(e == 0, m * 2.0 ** -9, (8 + m) * 2.0 ** (e - 10.0))
    v = np.where(c & 128, -mag, mag).astype(np.float32)
    v[[0x7F, 0xFF]] = np.nan
    return v


def nearest_e4m3_codes(a: np.ndarray) -> np.ndarray:
    """Codes whose values are nearest to the entries of `a` (magnitudes above 448 give 448).  Used to DRAW inputs
    (weight codes); which way a tie falls does not matter here."""
    mags = e4m3_code_values()[:0x7F].astype(np.float64)            # 0 .. 448, increasing with the code
    mid = (mags[1:] + mags[:-1]) / 2
    a = np.asarray(a, np.float32)
    code = np.searchsorted(mid, np.abs(a).astype(np.float64)).astype(np.uint8)
    return code | (np.signbit(a).astype(np.uint8) << 7)


# Scales of the four projections' inputs in the quantised-projection variant (static, per tensor, as an engine would
# calibrate them offline): normed activations have unit RMS (room for 8 sigma); attention outputs are averages of
# values (room for 6); silu(g) * u has RMS ~1 with a long tail (room for 24).
W8A8_INPUT_SCALES = {"a_qkv": 8.0 / 448.0, "a_o": 6.0 / 448.0, "a_gate_up": 8.0 / 448.0, "a_down": 24.0 / 448.0}


def make_weights_w8a8(shape: LayerShape, seed: int, n_layers: int = 0) -> dict:
    """The layer of make_weights with its four projections as 8-bit codes: each output row is scaled so that its
    largest magnitude maps to 448 (s_* = the fp32 scale of every row), the norm weights stay bf16."""
    w = make_weights(shape, seed, n_layers)
    out = {"w_in_norm": w["w_in_norm"], "w_post_norm": w["w_post_norm"], **{k: np.float32(v) for k, v in W8A8_INPUT_SCALES.items()}}
    for name in ("qkv", "o", "gate_up", "down"):
        f = bf16_bits_to_f32(w["w_" + name])
        s = (np.abs(f).max(axis=1) / np.float32(448.0)).astype(np.float32)
        s[s == 0] = np.float32(1.0)
        out["w_" + name] = nearest_e4m3_codes(f / s[:, None])
        out["s_" + name] = s
    return out


def make_model(shape: LayerShape, n_layers: int, vocab: int, seed: int, scaled: bool = True) -> dict:
    """Random-init stack: embedding ~N(0, 1) (so that the residual stream has unit scale like the
    activations of the single-layer workloads), layers as make_weights, output layer ~N(0, 0.02)."""
    rng = np.random.default_rng(seed + 31337)
    H = shape.hidden
    emb = f32_to_bf16_bits(rng.standard_normal((vocab, H), dtype=np.float32))
    head = f32_to_bf16_bits(rng.standard_normal((vocab, H), dtype=np.float32) * np.float32(0.02))
    fin = f32_to_bf16_bits(np.float32(1.0) + rng.standard_normal(H, dtype=np.float32) * np.float32(0.02))
    layers = [make_weights(shape, seed + 101 * (i + 1), n_layers if scaled else 0) for i in range(n_layers)]
    return {"embedding": emb, "layers": layers, "w_final_norm": fin, "w_lm_head": head}


def make_model_w8a8(shape: LayerShape, n_layers: int, vocab: int, seed: int, scaled: bool = True, depth: int = 0) -> dict:
    """make_model with every layer as make_weights_w8a8 (embedding, final norm and output layer stay bf16).  depth: the
    depth of the stack the n_layers are a slice of (sets the scale of the projections that write the stream)."""
    m = make_model(shape, 0, vocab, seed, scaled)
    m["layers"] = [make_weights_w8a8(shape, seed + 101 * (i + 1), (depth or n_layers) if scaled else 0) for i in range(n_layers)]
    return m


def make_token_ids(T: int, vocab: int, seed: int) -> np.ndarray:
    return np.random.default_rng(seed + 4242).integers(0, vocab, T).astype(np.int32)


def make_activations(T: int, H: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed + 7919)
    return f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))


def make_cache(shape: LayerShape, num_pages: int, seed: int, fill: bool = True):
    """K and V page pools [num_pages, P, n_kv, d] as bf16 bits.

    With fill=True every slot (used or not) holds an N(0,1) draw: it stands in
    for the keys and values of earlier steps, and makes a read of a slot that
    the block tables do not name show up as a mismatch.
    """
    shp = (num_pages, shape.page_size, shape.n_kv_heads, shape.head_dim)
    if not fill:
        return np.zeros(shp, np.uint16), np.zeros(shp, np.uint16)
    rng = np.random.default_rng(seed + 104729)
    k = f32_to_bf16_bits(rng.standard_normal(shp, dtype=np.float32))
    v = f32_to_bf16_bits(rng.standard_normal(shp, dtype=np.float32))
    return k, v


def make_cache_fp8(shape: LayerShape, num_pages: int, seed: int):
    """K and V page pools [num_pages, P, n_kv, d] of 8-bit floating point codes (1-4-3 bits), every slot filled:
    uniformly drawn codes with the two NaN patterns (0x7f, 0xff) replaced.  A format detail only, no arithmetic."""
    shp = (num_pages, shape.page_size, shape.n_kv_heads, shape.head_dim)
    rng = np.random.default_rng(seed + 15485863)
    # codes below exponent field 12 (magnitudes under 32): a cache of unit-scale keys and values
    k = (rng.integers(0, 96, shp, dtype=np.uint8) | (rng.integers(0, 2, shp, dtype=np.uint8) << 7)).astype(np.uint8)
    v = (rng.integers(0, 96, shp, dtype=np.uint8) | (rng.integers(0, 2, shp, dtype=np.uint8) << 7)).astype(np.uint8)
    return k, v


# ----------------------------------------------------------------------------
# the benchmark configurations
# ----------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    shape: LayerShape
    batch: Batch
    seed: int
    n_layers: int = 0          # depth of the stack the layer is cut from (0: plain N(0, 0.02) init)
    notes: str = ""
    extra: dict = field(default_factory=dict)

    def weights(self) -> dict:
        return make_weights(self.shape, self.seed, self.n_layers)


def workload_tiny(seed: int = 1000, shape: LayerShape = TINY) -> Workload:
    """2 prefill rows of 64 tokens (no past) + 6 decode rows of context 128."""
    q_len = [64, 64] + [1] * 6
    ctx = [64, 64] + [128] * 6
    b = build_batch(shape, q_len, ctx, seed=seed, name="tiny")
    return Workload("tiny", shape, b, seed)


def workload_tiny_prefix(seed: int = 1001, shape: LayerShape = TINY) -> Workload:
    """Test-only: a 32-token shared prefix, continuing chunks and decode rows mixed."""
    P = shape.page_size
    pl = 2 * P
    q_len = [40, 1, 17, 1, 1, 33, 5]
    ctx = [pl + 40, pl + 9, pl + 30, pl + 1, 70, 33 + 64, pl + 5]
    pid = [0, 0, 0, 0, -1, -1, 0]
    b = build_batch(shape, q_len, ctx, pid, [pl], seed=seed, name="tiny_prefix")
    return Workload("tiny_prefix", shape, b, seed)


def workload_tiny_long_prefixes(seed: int = 1011, shape: LayerShape = TINY) -> Workload:
    """Test-only: two shared prefixes of very different lengths (33 and 6 pages: many key blocks with a ragged last
    one) under few rows; prefill chunks and decode rows behind both."""
    P = shape.page_size
    pa, pb = 33 * P, 6 * P
    q_len = [23, 1, 1, 9, 1, 1, 1, 30, 1]
    ctx = [pa + 23, pa + 4, pa + 1, pb + 9, pb + 12, pa + 40, 50, 30, pb + 1]
    pid = [0, 0, 0, 1, 1, 0, -1, -1, 1]
    b = build_batch(shape, q_len, ctx, pid, [pa, pb], seed=seed, name="tiny_long_prefixes")
    return Workload("tiny_long_prefixes", shape, b, seed)


def workload_relquery_13b(seed: int = 1001, n_rows: int = 200, n_prefill: int = 16,
                          prefix: int = 512, shape: LayerShape = LLAMA_13B) -> Workload:
    """One relQuery: rows share a template prefix; a few rows prefill their suffix, the rest decode."""
    rng = np.random.default_rng(seed)
    suffix = rng.integers(30, 121, n_rows)
    gen = rng.integers(1, 17, n_rows)
    q_len = np.where(np.arange(n_rows) < n_prefill, suffix, 1)
    ctx = np.where(np.arange(n_rows) < n_prefill, prefix + suffix, prefix + suffix + gen)
    b = build_batch(shape, q_len, ctx, np.zeros(n_rows, np.int32), [prefix], seed=seed,
                    name="relquery_13b")
    return Workload("relquery_13b_16p184d", shape, b, seed, n_layers=40)


def workload_relquery_32b(seed: int = 1006) -> Workload:
    """The relQuery batch of workload_relquery_13b on the 32B layer shape (64 layers deep)."""
    wl = workload_relquery_13b(seed=seed, shape=QWEN_32B)
    return Workload("relquery_32b_16p184d", QWEN_32B, wl.batch, seed, n_layers=64)


def workload_tp_share(which: str = "70b_tp4", seed: int = 1008) -> Workload:
    """The relQuery batch of workload_relquery_13b on one GPU's share of a tensor-parallel layer: heads and MLP columns
    divided by the parallel degree, hidden size whole (the all-reduces between the shares are not part of this build)."""
    shape, depth = {"70b_tp4": (LLAMA_70B_TP4, 80), "32b_tp2": (QWEN_32B_TP2, 64)}[which]
    wl = workload_relquery_13b(seed=seed, shape=shape)
    return Workload(f"relquery_{which}_share", shape, wl.batch, seed, n_layers=depth)


def workload_decode_heavy_70b(seed: int = 1002, with_chunk: bool = True, n_rel: int = 4,
                              rows_per_rel: int = 64, prefix: int = 768, chunk: int = 2048,
                              shape: LayerShape = LLAMA_70B) -> Workload:
    """256 decode rows from 4 relQueries (own prefix each) and, optionally, one prefill chunk."""
    rng = np.random.default_rng(seed)
    n = n_rel * rows_per_rel
    ctx = rng.integers(600, 1501, n)
    ctx = np.maximum(ctx, prefix + 1)            # a member has left its template behind
    pid = np.repeat(np.arange(n_rel), rows_per_rel)
    q_len = np.ones(n, np.int64)
    if with_chunk:
        ctx = np.append(ctx, chunk)
        q_len = np.append(q_len, chunk)
        pid = np.append(pid, -1)
    b = build_batch(shape, q_len, ctx, pid, [prefix] * n_rel, seed=seed, name="decode_heavy_70b")
    return Workload("decode_heavy_70b" + ("_chunk2048" if with_chunk else "_decode_only"), shape, b, seed, n_layers=80)


def workload_prefill_only_13b(seed: int = 1003, n_req: int = 64, total: int = 8192, prefix: int = 1024,
                              lo: int = 50, hi: int = 200, shape: LayerShape = LLAMA_13B) -> Workload:
    """64 suffix prefills (sum 8192 tokens) behind one cached 1024-token template prefix."""
    rng = np.random.default_rng(seed)
    s = rng.integers(lo, hi + 1, n_req)
    i = 0
    while s.sum() != total:                      # nudge round-robin, inside the bounds
        step = 1 if s.sum() < total else -1
        if lo <= s[i % n_req] + step <= hi:
            s[i % n_req] += step
        i += 1
    b = build_batch(shape, s, prefix + s, np.zeros(n_req, np.int32), [prefix], seed=seed,
                    name="prefill_only_13b")
    return Workload("prefill_only_13b", shape, b, seed, n_layers=40)


def workload_decode_plus_chunk_13b(chunk: int, seed: int = 1004, n_dec: int = 128, ctx: int = 1024,
                                   shape: LayerShape = LLAMA_13B) -> Workload:
    """128 decode rows of context 1024 and one prefill chunk of `chunk` tokens (0 = none)."""
    q_len = [1] * n_dec + ([chunk] if chunk else [])
    c = [ctx] * n_dec + ([chunk] if chunk else [])
    b = build_batch(shape, q_len, c, seed=seed, name=f"decode128_chunk{chunk}")
    return Workload(f"decode{n_dec}_chunk{chunk}_13b" if n_dec else f"prefill_chunk{chunk}_13b", shape, b, seed, n_layers=40)


# ----------------------------------------------------------------------------
# batches for fitting the batch-duration model (Sec. 4.2, Eq. 9)
# ----------------------------------------------------------------------------
def prefill_tokens(b: Batch) -> tuple:
    """(utok, total) of a batch's prefill rows: the query tokens they compute, and all their prompt tokens
    including the ones the prefix cache serves (the two abscissae the paper compares)."""
    pre = b.q_len > 1
    return int(b.q_len[pre].sum()), int(b.ctx_len[pre].sum())


def duration_sweep_prefill(n_batches: int, seed: int = 1100, max_tokens: int = 8192, max_reqs: int = 256,
                           shape: LayerShape = LLAMA_13B) -> list:
    """Prefill batches as a serving run meets them: requests of one to three relQueries (template prefix
    of 256-1024 tokens, private suffix of 30-120), each request either finding its template in the prefix
    cache (it computes its suffix only) or not (it computes the whole prompt into private pages).  The
    batch's token budget and its cache hit rate are drawn per batch so that the sweep covers the range of
    uncached tokens and decorrelates them from the total."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n_batches):
        budget = int(rng.integers(256, max_tokens + 1))
        hit = float(rng.random())
        prefixes = [int(p) for p in rng.choice([256, 512, 768, 1024], int(rng.integers(1, 4)))]
        q_len, ctx, pid = [], [], []
        utok = 0
        while len(q_len) < max_reqs:
            rel = len(q_len) % len(prefixes)
            suffix = int(rng.integers(30, 121))
            cached = bool(rng.random() < hit)
            q = suffix if cached else prefixes[rel] + suffix
            if q_len and utok + q > budget:
                break
            q_len.append(q)
            ctx.append(prefixes[rel] + suffix)
            pid.append(rel if cached else -1)
            utok += q
        used = sorted({p for p in pid if p >= 0})
        remap = {p: j for j, p in enumerate(used)}
        pid = [remap[p] if p >= 0 else -1 for p in pid]
        out.append(build_batch(shape, q_len, ctx, pid, [prefixes[p] for p in used], seed=seed + i,
                               name=f"duration_prefill_{i}"))
    return out


def duration_sweep_decode(sizes, seed: int = 1200, shape: LayerShape = LLAMA_13B) -> list:
    """Decode batches of the given request counts: members of relQueries of 1-100 requests behind their
    template (256-1024 tokens), suffix 30-120, 1-16 tokens generated so far."""
    rng = np.random.default_rng(seed)
    out = []
    for i, n in enumerate(sizes):
        ctx, pid, prefixes = [], [], []
        while len(ctx) < n:
            members = min(int(rng.integers(1, 101)), n - len(ctx))
            prefixes.append(int(rng.choice([256, 512, 768, 1024])))
            for _ in range(members):
                ctx.append(prefixes[-1] + int(rng.integers(30, 121)) + int(rng.integers(1, 17)))
                pid.append(len(prefixes) - 1)
        out.append(build_batch(shape, [1] * n, ctx, pid, prefixes, seed=seed + i, name=f"duration_decode_{n}"))
    return out


# ----------------------------------------------------------------------------
# relQuery traces for the serving loop (Sec. 5.1 "Datasets and Workloads")
# ----------------------------------------------------------------------------
@dataclass
class RelQuerySpec:
    rid: int
    arrival: float        # seconds
    prefix: int           # template tokens shared by all requests
    suffix: list          # private tokens per request
    out_len: int          # OL(R)
    template: int = -1    # relQueries with the same template id share its tokens (-1: its own)


def poisson_trace(n_relqueries: int, rate: float, seed: int = 0, max_requests: int = 100, out_lens=(5, 50),
                  n_templates: int = 0) -> list:
    """Seeded synthetic trace shaped like Sec. 5.1's workloads: Poisson arrivals, 1-100 requests per relQuery,
    a template of 256-1024 tokens, suffixes of 30-120 tokens, output lengths of 5 or 50 tokens.  With n_templates > 0
    the relQueries draw their template (and its length) from that many shared ones."""
    rng = np.random.default_rng(seed)
    lens = [int(x) for x in rng.choice([256, 512, 768, 1024], max(n_templates, 1))]
    t, out = 0.0, []
    for rid in range(n_relqueries):
        t += float(rng.exponential(1.0 / rate))
        n = int(rng.integers(1, max_requests + 1))
        prefix = int(rng.choice([256, 512, 768, 1024]))
        suffix = [int(x) for x in rng.integers(30, 121, n)]
        ol = int(rng.choice(out_lens))
        tmpl = -1
        if n_templates > 0:
            tmpl = int(rng.integers(0, n_templates))
            prefix = lens[tmpl]
        out.append(RelQuerySpec(rid, t, prefix, suffix, ol, tmpl))
    return out


def sample_positions(seed: int):
    """The random draws of Eq. 11's sample, as a function both the scheduler and its oracle are handed:
    draw(rid, key, n, k) -> k distinct positions in range(n), a pure function of its arguments and the seed."""
    def draw(rid: int, key: int, n: int, k: int) -> list:
        rng = np.random.default_rng([seed, rid, key, n, k])
        return sorted(int(x) for x in rng.choice(n, k, replace=False))
    return draw

