"""Seeded synthetic inputs for absorbed MLA decode.

This module only *produces inputs*: random tensors of the benchmark shapes,
RoPE applied to the decoupled key / query parts (the kernels and the CPU
oracle both receive them already rotated), rounding to the storage dtype,
per-token fp8 quantisation of the cache, and the page pool / page table.
It contains none of the attention arithmetic and is imported by tests and
benchmarks on both the GPU side and the oracle side.

Storage conventions (numpy):
  fp32  -> float32 arrays
  bf16  -> uint16 arrays holding bfloat16 bit patterns
  fp8   -> uint8 arrays holding OCP e4m3 codes + float32 per-token scale

RoPE follows Sec. 3.1, Eq. 1 of the paper: interleaved (real, imaginary)
pairs (2k-1, 2k), angle theta_k = base^(-2(k-1)/d).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

F32, BF16, FP8_E4M3 = "f32", "bf16", "fp8_e4m3"

BF16_NAN = np.uint16(0x7FC0)
E4M3_NAN = np.uint8(0x7F)
E4M3_MAX = 448.0


# --------------------------------------------------------------------------
# RNG: one independent counter-based stream per (seed, tensor id)
# --------------------------------------------------------------------------

def stream(seed: int, tensor_id: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(tensor_id)]))


def normal(rng: np.random.Generator, shape, std: float = 1.0) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x


# --------------------------------------------------------------------------
# RoPE (Sec. 3.1, Eq. 1)
# --------------------------------------------------------------------------

def rope(x: np.ndarray, positions, base: float = 10000.0) -> np.ndarray:
    """Rotate the last axis of x (even length d) at the given positions.

    x: [..., n, d]; positions: scalar or [n].  Pair k (0-based) = elements
    (2k, 2k+1) = (real, imaginary); angle = pos * base^(-2k/d).
    Computed in float64, returned in x's dtype."""
    x = np.asarray(x)
    d = x.shape[-1]
    assert d % 2 == 0
    pos = np.asarray(positions, dtype=np.float64)
    theta = base ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)
    ang = pos[..., None] * theta  # [n, d/2] or [d/2]
    c, s = np.cos(ang), np.sin(ang)
    xr = x[..., 0::2].astype(np.float64)
    xi = x[..., 1::2].astype(np.float64)
    out = np.empty(x.shape, dtype=np.float64)
    out[..., 0::2] = xr * c - xi * s
    out[..., 1::2] = xi * c + xr * s
    return out.astype(x.dtype)


# --------------------------------------------------------------------------
# storage codecs (encoders only; decoding belongs to whoever consumes them)
# --------------------------------------------------------------------------

def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round to nearest even; NaN -> 0x7FC0."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r[nan] = BF16_NAN
    return r


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Inverse view used only to hand bf16 inputs to float-consuming helpers."""
    return (np.ascontiguousarray(bits).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quant_e4m3_per_token(x: np.ndarray):
    """Per-row (token) absmax scaling to OCP e4m3: scale = absmax/448
    (1 when the row is all zero), code = RNE(x/scale) saturated to +-448.

    x: [n, row] float32 -> (codes uint8 [n, row], scale float32 [n])."""
    import torch
    x = np.ascontiguousarray(x, dtype=np.float32)
    absmax = np.abs(x).max(axis=-1)
    scale = (absmax / np.float32(E4M3_MAX)).astype(np.float32)
    scale[absmax == 0] = np.float32(1.0)
    y = np.clip(x / scale[..., None], -E4M3_MAX, E4M3_MAX).astype(np.float32)
    codes = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    return codes, scale


def encode_e4m3(x: np.ndarray) -> np.ndarray:
    """Plain saturating RNE encode of float32 values to e4m3 codes (no scale)."""
    import torch
    y = np.clip(np.ascontiguousarray(x, dtype=np.float32), -E4M3_MAX, E4M3_MAX)
    return torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == BF16:
        return to_bf16_bits(x)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# workload description
# --------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    B: int
    H: int
    d_head: int
    d_c: int
    d_rope: int
    page_size: int
    io_dtype: str
    cache_dtype: str
    softmax_scale: float
    num_splits: int
    seq_lens: np.ndarray            # int32 [B]
    page_table: np.ndarray          # int32 [B, max_pages_per_seq], unused = -1
    pool: np.ndarray                # [num_pages, page_size, d_c+d_rope] storage dtype
    kv_scale: Optional[np.ndarray]  # float32 [num_pages, page_size] (fp8 only)
    q_nope: np.ndarray              # [B, H, d_head] storage (io) dtype
    q_rope: np.ndarray              # [B, H, d_rope]
    W_UK: np.ndarray                # [H, d_head, d_c]
    W_UV: np.ndarray                # [H, d_c, d_head]
    meta: dict = field(default_factory=dict)

    @property
    def num_pages(self) -> int:
        return int(self.pool.shape[0])

    @property
    def max_pages_per_seq(self) -> int:
        return int(self.page_table.shape[1])

    @property
    def tokens(self) -> int:
        return int(self.seq_lens.sum())

    @property
    def row_bytes(self) -> int:
        return int(self.pool.shape[2] * self.pool.dtype.itemsize)

    @property
    def cache_bytes_per_step(self) -> int:
        """Bytes of cache one decode step must read: every cached token's
        [c_kv | k_rope] row once (+ its fp32 scale for fp8)."""
        per_tok = self.row_bytes + (4 if self.cache_dtype == FP8_E4M3 else 0)
        return self.tokens * per_tok


def build_paged_cache(seq_lens: Sequence[int], d_c: int, d_rope: int,
                      page_size: int, cache_dtype: str, seed: int,
                      placement: str = "random", free_frac: float = 0.0,
                      k_rope_gain: float = 1.0, rope_base: float = 10000.0,
                      max_pages_per_seq: Optional[int] = None,
                      poison: bool = True, tensor_id_base: int = 1000):
    """Fill a page pool with per-sequence N(0,1) rows [c_kv | RoPE(k_rope)].

    Free pages and the unused tail slots of each last page hold NaN
    (poison=True) so that any read of them shows up in the output."""
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    B = len(seq_lens)
    row = d_c + d_rope
    n_pages_b = (seq_lens.astype(np.int64) + page_size - 1) // page_size
    n_used = int(n_pages_b.sum())
    pool_pages = max(1, n_used if free_frac <= 0 else int(math.ceil(n_used / (1.0 - free_frac))))
    if max_pages_per_seq is None:
        max_pages_per_seq = max(1, int(n_pages_b.max()) if B else 1)
    assert max_pages_per_seq >= (int(n_pages_b.max()) if B else 0)
    prng = stream(seed, tensor_id_base - 1)
    order = prng.permutation(pool_pages) if placement == "random" else np.arange(pool_pages)
    order = order.astype(np.int32)

    if cache_dtype == F32:
        pool = np.full((pool_pages, page_size, row), np.nan if poison else 0.0, dtype=np.float32)
        kv_scale = None
    elif cache_dtype == BF16:
        pool = np.full((pool_pages, page_size, row), BF16_NAN if poison else 0, dtype=np.uint16)
        kv_scale = None
    elif cache_dtype == FP8_E4M3:
        pool = np.full((pool_pages, page_size, row), E4M3_NAN if poison else 0, dtype=np.uint8)
        kv_scale = np.full((pool_pages, page_size), np.nan if poison else 1.0, dtype=np.float32)
    else:
        raise ValueError(cache_dtype)

    page_table = np.full((B, max_pages_per_seq), -1, dtype=np.int32)
    cursor = 0
    for b in range(B):
        L, npg = int(seq_lens[b]), int(n_pages_b[b])
        pages = order[cursor:cursor + npg]
        cursor += npg
        page_table[b, :npg] = pages
        if L == 0:
            continue
        x = normal(stream(seed, tensor_id_base + b), (L, row))
        if d_rope:
            if k_rope_gain != 1.0:
                x[:, d_c:] *= np.float32(k_rope_gain)
            x[:, d_c:] = rope(x[:, d_c:], np.arange(L), rope_base)
        flat = pool.reshape(pool_pages * page_size, row)
        rows = (pages.astype(np.int64)[:, None] * page_size + np.arange(page_size)[None, :]).reshape(-1)[:L]
        if cache_dtype == F32:
            flat[rows] = x
        elif cache_dtype == BF16:
            flat[rows] = to_bf16_bits(x)
        else:
            codes, sc = quant_e4m3_per_token(x)
            flat[rows] = codes
            kv_scale.reshape(-1)[rows] = sc
    return pool, kv_scale, page_table, seq_lens


def make_workload(name: str, *, B: int, H: int, d_head: int, d_c: int, d_rope: int,
                  seq_lens: Sequence[int], io_dtype: str, cache_dtype: str,
                  page_size: int = 64, placement: str = "random", free_frac: float = 0.0,
                  k_rope_gain: float = 1.0, num_splits: int = 1, seed: int = 0,
                  max_pages_per_seq: Optional[int] = None, rope_base: float = 10000.0,
                  softmax_scale: Optional[float] = None, poison: bool = True) -> Workload:
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    assert len(seq_lens) == B
    if softmax_scale is None:
        softmax_scale = 1.0 / math.sqrt(d_head + d_rope)
    pool, kv_scale, page_table, seq_lens = build_paged_cache(
        seq_lens, d_c, d_rope, page_size, cache_dtype, seed, placement, free_frac,
        k_rope_gain, rope_base, max_pages_per_seq, poison)
    q_nope = normal(stream(seed, 1), (B, H, d_head))
    q_rope = normal(stream(seed, 2), (B, H, d_rope))
    if d_rope:
        pos = np.maximum(seq_lens.astype(np.int64) - 1, 0)
        q_rope = rope(q_rope.transpose(1, 0, 2), pos, rope_base).transpose(1, 0, 2)
    # weights ~ N(0, variance 1/d_c)
    std = 1.0 / math.sqrt(d_c)
    W_UK = normal(stream(seed, 3), (H, d_head, d_c), std)
    W_UV = normal(stream(seed, 4), (H, d_c, d_head), std)
    return Workload(
        name=name, B=B, H=H, d_head=d_head, d_c=d_c, d_rope=d_rope, page_size=page_size,
        io_dtype=io_dtype, cache_dtype=cache_dtype, softmax_scale=float(softmax_scale),
        num_splits=num_splits, seq_lens=seq_lens, page_table=page_table, pool=pool,
        kv_scale=kv_scale, q_nope=store(q_nope, io_dtype),
        q_rope=store(np.ascontiguousarray(q_rope), io_dtype),
        W_UK=store(W_UK, io_dtype), W_UV=store(W_UV, io_dtype),
        meta={"seed": seed, "placement": placement, "free_frac": free_frac,
              "k_rope_gain": k_rope_gain})


def multi_queries(w: Workload, q_len: int, seed: Optional[int] = None, rope_base: float = 10000.0):
    """Queries of the q_len newest tokens of every sequence of `w` (multi-token prediction /
    speculative decoding): the cache of `w` is taken to hold those tokens' rows already, token i
    sits at position seq_len - q_len + i and its decoupled part is rotated there.

    Returns (q_nope [B, q_len, H, d_head], q_rope [B, q_len, H, d_rope]) in w's io storage dtype."""
    seed = w.meta.get("seed", 0) if seed is None else seed
    q_nope = normal(stream(seed, 21), (w.B, q_len, w.H, w.d_head))
    q_rope = normal(stream(seed, 22), (w.B, q_len, w.H, w.d_rope))
    if w.d_rope:
        pos = w.seq_lens.astype(np.int64)[:, None] - q_len + np.arange(q_len)[None, :]      # [B, q_len]
        pos = np.maximum(pos, 0).reshape(-1)
        flat = q_rope.reshape(w.B * q_len, w.H, w.d_rope).transpose(1, 0, 2)                 # [H, B*q_len, d]
        q_rope = rope(flat, pos, rope_base).transpose(1, 0, 2).reshape(w.B, q_len, w.H, w.d_rope)
    return store(q_nope, w.io_dtype), store(np.ascontiguousarray(q_rope), w.io_dtype)


# --------------------------------------------------------------------------
# the five benchmark configurations (and scaled-down versions of them)
# --------------------------------------------------------------------------

def config(name: str, seed: int = 0, shrink: int = 1) -> Workload:
    """name in {"C1".."C5"}.  shrink > 1 divides the context lengths (and, for
    the wide batches, the batch) so a CPU can finish the case in seconds; the
    head / latent / page shapes stay the real ones."""
    s = max(1, int(shrink))
    if name == "C1":
        return make_workload("C1", B=1, H=32, d_head=128, d_c=512, d_rope=64,
                             seq_lens=[max(1, 1024 // s)], io_dtype=F32, cache_dtype=F32,
                             placement="identity", num_splits=4 if s == 1 else 2, seed=seed)
    if name == "C2":
        B = 16 if s == 1 else max(2, 16 // s)
        return make_workload("C2", B=B, H=32, d_head=128, d_c=512, d_rope=64,
                             seq_lens=[max(1, 8192 // s)] * B, io_dtype=BF16, cache_dtype=BF16,
                             placement="random", num_splits=16 if s == 1 else 4, seed=seed)
    if name == "C3":
        B = 64 if s == 1 else max(3, 64 // s)
        lens = stream(seed, 50).integers(max(1, 1024 // s), 32768 // s, size=B, endpoint=True)
        return make_workload("C3", B=B, H=32, d_head=128, d_c=512, d_rope=64,
                             seq_lens=lens, io_dtype=BF16, cache_dtype=BF16,
                             placement="random", free_frac=0.1, k_rope_gain=4.0,
                             max_pages_per_seq=max(1, 512 // s), num_splits=16 if s == 1 else 4,
                             seed=seed)
    if name == "C4":
        B = 128 if s == 1 else max(2, 128 // s)
        return make_workload("C4", B=B, H=28, d_head=128, d_c=256, d_rope=64,
                             seq_lens=[max(1, 4096 // s)] * B, io_dtype=BF16, cache_dtype=BF16,
                             placement="random", num_splits=2, seed=seed)
    if name == "C5":
        B = 4 if s == 1 else 2
        return make_workload("C5", B=B, H=32, d_head=128, d_c=512, d_rope=64,
                             seq_lens=[max(1, 131072 // s)] * B, io_dtype=BF16,
                             cache_dtype=FP8_E4M3, placement="random", num_splits=32, seed=seed)
    raise KeyError(name)


# --------------------------------------------------------------------------
# calibration inputs of the offline conversion (Sec. 4.2, 4.3, App. B-D)
# --------------------------------------------------------------------------

def calibration(n: int, D: int, g: int, d: int, seed: int = 0, decay: float = 0.7,
                key_gain: float = 3.0, outliers: int = 4, floor: float = 0.0):
    """Synthetic stand-in for the hidden states of a calibration corpus and for the
    key/value projections of one GQA layer, all float64.

    X [n, D]: Gaussian factors with a power-law spectrum (factor k scaled by
    (k+1)^-decay, plus `floor`), mixed by a random matrix, with a few outlier channels
    scaled by 8 (large-magnitude channels are typical of transformer hidden states).
    W_K, W_V [g*d, D] ~ N(0, 1/D), W_K times `key_gain` (keys carry larger norms than
    values, the situation Sec. 4.3 balances)."""
    k = min(n, D)
    Z = stream(seed, 40).standard_normal((n, k))
    s = (1.0 + np.arange(k)) ** (-decay) + floor
    B = stream(seed, 41).standard_normal((k, D)) / np.sqrt(k)
    X = (Z * s) @ B
    ch = stream(seed, 42).choice(D, size=min(outliers, D), replace=False)
    X[:, ch] *= 8.0
    W_K = stream(seed, 43).standard_normal((g * d, D)) * (key_gain / np.sqrt(D))
    W_V = stream(seed, 44).standard_normal((g * d, D)) / np.sqrt(D)
    return X, W_K, W_V


def start_block(m: int, p: int, seed: int = 0) -> np.ndarray:
    """Gaussian start block of the block power iteration (random numbers are drawn here, not by the library)."""
    return stream(seed, 45).standard_normal((m, p))
