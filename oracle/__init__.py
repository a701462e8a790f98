"""CPU oracle for absorbed MLA decode -- TEST INFRASTRUCTURE ONLY.

Thin ctypes/numpy wrapper over ``mla_oracle.c`` (plain C, fp64).  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the product path never does, and this package imports nothing from
the product.  All arithmetic lives in the C file; this module only widens
stored values exactly to fp64 and marshals pointers.

Functions follow the paper's Sec. 3.3: ``decode_explicit`` is the
"MHA paradigm" equation (materialise keys and values from the latent),
``absorb_q`` / ``decode_absorbed`` / ``out_proj`` are the three lines of the
"MQA paradigm" (Absorb) equation, ``decode_split`` / ``merge_lse`` are the
same softmax evaluated chunk by chunk and merged by log-sum-exp.

Parity pins (tests/test_oracle_pins.py): absorbed == explicit; reduction to
textbook MHA / GQA / MQA under selector-identity projections (Sec. 4.1,
App. A.2.1); closed forms of softmax; invariances; scalar brute force;
codec tables.  The absolute output values on the five benchmark shapes are
"parity unpinned" by any printed number: the paper prints none.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "mla_oracle.c"
_LIB = _HERE / "libmla_oracle.so"

F32, BF16, FP8_E4M3 = 0, 1, 2

_lib = None


def build(force: bool = False) -> Path:
    """Compile the C oracle with gcc (OpenMP over (b, h) only)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-std=c11",
               "-Wall", "-Wextra", "-o", str(_LIB), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _c():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        lib.oracle_widen_bf16.restype = ctypes.c_double
        lib.oracle_widen_bf16.argtypes = [ctypes.c_uint16]
        lib.oracle_widen_e4m3.restype = ctypes.c_double
        lib.oracle_widen_e4m3.argtypes = [ctypes.c_uint8]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_encode_bf16.restype = ctypes.c_uint16
        lib.oracle_encode_bf16.argtypes = [ctypes.c_float]
        lib.oracle_encode_e4m3.restype = ctypes.c_uint8
        lib.oracle_encode_e4m3.argtypes = [ctypes.c_float]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_c().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads for the (b, h) loops; 0 restores the default."""
    _c().oracle_set_num_threads(ctypes.c_int(int(n)))


# --------------------------------------------------------------------------
# exact widening of stored values
# --------------------------------------------------------------------------

def widen_bf16_bits(bits: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float64, exactly."""
    u = np.ascontiguousarray(bits).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def widen_e4m3_code(code: int) -> float:
    return float(_c().oracle_widen_e4m3(int(code)))


def widen_bf16_code(bits: int) -> float:
    return float(_c().oracle_widen_bf16(int(bits)))


def widen(x) -> np.ndarray:
    """float32 / float64 / bf16 (torch.bfloat16 tensor or uint16 bits) -> float64."""
    if hasattr(x, "detach"):  # torch tensor, without importing torch here
        t = x.detach().cpu().contiguous()
        name = str(t.dtype)
        if name == "torch.bfloat16":
            return widen_bf16_bits(t.view(_torch().int16).numpy().view(np.uint16))
        return t.double().numpy()
    a = np.asarray(x)
    if a.dtype == np.uint16:
        return widen_bf16_bits(a)
    return np.ascontiguousarray(a, dtype=np.float64)


def _torch():
    import torch
    return torch


# --------------------------------------------------------------------------
# marshalling helpers
# --------------------------------------------------------------------------

def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _ip(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _vp(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _pool_args(pool, kv_scale):
    """pool: ndarray [num_pages, page_size, d_c+d_rope] of float32, uint16
    (bf16 bits) or uint8 (e4m3 codes, kv_scale required)."""
    pool = np.ascontiguousarray(pool)
    if pool.dtype == np.float32:
        dt = F32
    elif pool.dtype == np.uint16:
        dt = BF16
    elif pool.dtype == np.uint8:
        dt = FP8_E4M3
        if kv_scale is None:
            raise ValueError("fp8 cache needs kv_scale")
    else:
        raise TypeError(f"unsupported cache dtype {pool.dtype}")
    sc = None if kv_scale is None else np.ascontiguousarray(kv_scale, dtype=np.float32)
    return pool, sc, dt


# --------------------------------------------------------------------------
# oracle entry points
# --------------------------------------------------------------------------

def gather_paged(pool, page_table, seq_lens, max_len: int) -> np.ndarray:
    """Byte-exact logical view: uint8 [B, max_len, row_bytes]; rows past
    seq_len are zero bytes."""
    pool = np.ascontiguousarray(pool)
    page_size = pool.shape[1]
    row_bytes = pool.shape[2] * pool.dtype.itemsize
    pt, sl = _i32(page_table), _i32(seq_lens)
    B = sl.shape[0]
    dense = np.empty((B, max_len, row_bytes), dtype=np.uint8)
    _c().oracle_gather_paged(_vp(pool), _ip(pt), _ip(sl), _vp(dense),
                             ctypes.c_int(B), ctypes.c_int(max_len),
                             ctypes.c_int(row_bytes), ctypes.c_int(page_size),
                             ctypes.c_int(pt.shape[1]))
    return dense


def absorb_q(q_nope, W_UK) -> np.ndarray:
    """q_abs[b,h,:] = q_nope[b,h,:] . W_UK[h]   (first line of Eq. "mqa")."""
    q, W = widen(q_nope), widen(W_UK)
    B, H, d_head = q.shape
    d_c = W.shape[2]
    assert W.shape == (H, d_head, d_c)
    out = np.empty((B, H, d_c), dtype=np.float64)
    _c().oracle_absorb_q(_dp(q), _dp(W), _dp(out), B, H, d_head, d_c)
    return out


def out_proj(o_lat, W_UV) -> np.ndarray:
    """out[b,h,:] = o_lat[b,h,:] . W_UV[h]   (last line of Eq. "mqa", inside the brackets)."""
    o, W = widen(o_lat), widen(W_UV)
    B, H, d_c = o.shape
    d_head = W.shape[2]
    assert W.shape == (H, d_c, d_head)
    out = np.empty((B, H, d_head), dtype=np.float64)
    _c().oracle_out_proj(_dp(o), _dp(W), _dp(out), B, H, d_c, d_head)
    return out


def decode_explicit(q_nope, q_rope, W_UK, W_UV, pool, kv_scale, page_table,
                    seq_lens, softmax_scale: float, d_c: int,
                    b_sel=None, h_sel=None, return_probs: bool = False):
    """The definition: Eq. "mha" with K, V materialised from the latent.

    Returns (out [n_b, n_h, d_head], lse [n_b, n_h][, probs [n_b, n_h, max_len]])."""
    qn, qr, Wk, Wv = widen(q_nope), widen(q_rope), widen(W_UK), widen(W_UV)
    pool, sc, dt = _pool_args(pool, kv_scale)
    pt, sl = _i32(page_table), _i32(seq_lens)
    B, H, d_head = qn.shape
    d_rope = pool.shape[2] - d_c
    assert qr.shape == (B, H, d_rope) or d_rope == 0
    if d_rope == 0:
        qr = np.zeros((B, H, 0))
    bs = None if b_sel is None else _i32(b_sel)
    hs = None if h_sel is None else _i32(h_sel)
    n_b = B if bs is None else len(bs)
    n_h = H if hs is None else len(hs)
    out = np.empty((n_b, n_h, d_head), dtype=np.float64)
    lse = np.empty((n_b, n_h), dtype=np.float64)
    max_len = int(sl.max()) if len(sl) else 0
    probs = np.zeros((n_b, n_h, max(max_len, 1)), dtype=np.float64) if return_probs else None
    _c().oracle_decode_explicit(
        _dp(qn), _dp(qr), _dp(Wk), _dp(Wv), _vp(pool), _vp(sc), _ip(pt), _ip(sl),
        _dp(out), _dp(lse), None if probs is None else _dp(probs),
        ctypes.c_int(max(max_len, 1)), B, H, d_head, d_c, d_rope,
        pool.shape[1], pt.shape[1], ctypes.c_double(softmax_scale), dt,
        None if bs is None else _ip(bs), n_b, None if hs is None else _ip(hs), n_h)
    if return_probs:
        return out, lse, probs
    return out, lse


def decode_absorbed(q_abs, q_rope, pool, kv_scale, page_table, seq_lens,
                    softmax_scale: float):
    """Second line of Eq. "mqa": scores of [q_abs; q_rope] against
    [c_kv; k_rope], softmax over the cached tokens, weights applied to c_kv.

    Returns (o_lat [B,H,d_c], lse [B,H])."""
    qa, qr = widen(q_abs), widen(q_rope)
    pool, sc, dt = _pool_args(pool, kv_scale)
    pt, sl = _i32(page_table), _i32(seq_lens)
    B, H, d_c = qa.shape
    d_rope = pool.shape[2] - d_c
    if d_rope == 0:
        qr = np.zeros((B, H, 0))
    assert qr.shape == (B, H, d_rope)
    o = np.empty((B, H, d_c), dtype=np.float64)
    lse = np.empty((B, H), dtype=np.float64)
    _c().oracle_decode_absorbed(
        _dp(qa), _dp(qr), _vp(pool), _vp(sc), _ip(pt), _ip(sl), _dp(o), _dp(lse),
        B, H, d_c, d_rope, pool.shape[1], pt.shape[1],
        ctypes.c_double(softmax_scale), dt)
    return o, lse


def decode_absorbed_multi(q_abs, q_rope, pool, kv_scale, page_table, seq_lens,
                          softmax_scale: float):
    """Eq. "mqa" for the T newest positions of every sequence at once (multi-token
    prediction / speculative decoding): query token i of T sits at position
    seq_len - T + i and sees the cached rows up to and including its own.

    q_abs [B,T,H,d_c], q_rope [B,T,H,d_rope] -> (o_lat [B,T,H,d_c], lse [B,T,H])."""
    qa, qr = widen(q_abs), widen(q_rope)
    pool, sc, dt = _pool_args(pool, kv_scale)
    pt, sl = _i32(page_table), _i32(seq_lens)
    B, T, H, d_c = qa.shape
    d_rope = pool.shape[2] - d_c
    if d_rope == 0:
        qr = np.zeros((B, T, H, 0))
    assert qr.shape == (B, T, H, d_rope)
    o = np.empty((B, T, H, d_c), dtype=np.float64)
    lse = np.empty((B, T, H), dtype=np.float64)
    _c().oracle_decode_absorbed_multi(
        _dp(qa), _dp(qr), _vp(pool), _vp(sc), _ip(pt), _ip(sl), _dp(o), _dp(lse),
        B, T, H, d_c, d_rope, pool.shape[1], pt.shape[1],
        ctypes.c_double(softmax_scale), dt)
    return o, lse


def prefill_explicit(q_nope, q_rope, W_UK, W_UV, pool, kv_scale, page_table, seq_lens,
                     softmax_scale: float, d_c: int):
    """Eq. "mha" (the MHA paradigm of Sec. 3.3) for the T newest positions of every sequence:
    keys [W_UK c_j ; k_rope_j] and values W_UV c_j materialised per head, query token i of T at
    position seq_len - T + i attends to the keys up to and including its own.  T = seq_len is the
    prefill of a whole prompt.

    q_nope [B,T,H,d_head], q_rope [B,T,H,d_rope] -> (out [B,T,H,d_head], lse [B,T,H])."""
    qn, qr = widen(q_nope), widen(q_rope)
    Wk, Wv = widen(W_UK), widen(W_UV)
    pool, sc, dt = _pool_args(pool, kv_scale)
    pt, sl = _i32(page_table), _i32(seq_lens)
    B, T, H, d_head = qn.shape
    d_rope = pool.shape[2] - d_c
    if d_rope == 0:
        qr = np.zeros((B, T, H, 0))
    assert qr.shape == (B, T, H, d_rope)
    assert Wk.shape == (H, d_head, d_c) and Wv.shape == (H, d_c, d_head)
    out = np.empty((B, T, H, d_head), dtype=np.float64)
    lse = np.empty((B, T, H), dtype=np.float64)
    _c().oracle_prefill_explicit(
        _dp(qn), _dp(qr), _dp(Wk), _dp(Wv), _vp(pool), _vp(sc), _ip(pt), _ip(sl), _dp(out), _dp(lse),
        B, T, H, d_head, d_c, d_rope, pool.shape[1], pt.shape[1],
        ctypes.c_double(softmax_scale), dt)
    return out, lse


def decode_split(q_abs, q_rope, pool, kv_scale, page_table, seq_lens,
                 softmax_scale: float, n_splits: int, chunk_pages: int,
                 return_partials: bool = False):
    """Chunk-local softmax over page-aligned chunks + log-sum-exp merge."""
    qa, qr = widen(q_abs), widen(q_rope)
    pool, sc, dt = _pool_args(pool, kv_scale)
    pt, sl = _i32(page_table), _i32(seq_lens)
    B, H, d_c = qa.shape
    d_rope = pool.shape[2] - d_c
    if d_rope == 0:
        qr = np.zeros((B, H, 0))
    o = np.empty((B, H, d_c), dtype=np.float64)
    lse = np.empty((B, H), dtype=np.float64)
    op = np.empty((B, H, n_splits, d_c), dtype=np.float64) if return_partials else None
    lp = np.empty((B, H, n_splits), dtype=np.float64) if return_partials else None
    _c().oracle_decode_split(
        _dp(qa), _dp(qr), _vp(pool), _vp(sc), _ip(pt), _ip(sl), _dp(o), _dp(lse),
        None if op is None else _dp(op), None if lp is None else _dp(lp),
        B, H, d_c, d_rope, pool.shape[1], pt.shape[1], n_splits, chunk_pages,
        ctypes.c_double(softmax_scale), dt)
    if return_partials:
        return o, lse, op, lp
    return o, lse


def merge_lse(o_part, lse_part):
    """o_part [S, d_c], lse_part [S] -> (o [d_c], lse)."""
    op, lp = _f64(o_part), _f64(lse_part)
    S, d_c = op.shape
    o = np.empty(d_c, dtype=np.float64)
    l = ctypes.c_double(0.0)
    _c().oracle_merge_lse(_dp(op), _dp(lp), S, d_c, _dp(o), ctypes.byref(l))
    return o, float(l.value)


def mla_step(q_nope, q_rope, W_UK, W_UV, pool, kv_scale, page_table, seq_lens,
             softmax_scale: float):
    """The three absorbed calls chained in fp64 with no intermediate rounding.

    Returns dict(q_abs, o_lat, lse, out)."""
    q_abs = absorb_q(q_nope, W_UK)
    o_lat, lse = decode_absorbed(q_abs, q_rope, pool, kv_scale, page_table,
                                 seq_lens, softmax_scale)
    out = out_proj(o_lat, W_UV)
    return {"q_abs": q_abs, "o_lat": o_lat, "lse": lse, "out": out}


# --------------------------------------------------------------------------
# cache append (Sec. 3.3 MLA equations: c^{KV} = W^{DKV} x, k^R = RoPE(W^{KR} x, t))
# --------------------------------------------------------------------------

def rope(v, pos: float, base: float = 10000.0) -> np.ndarray:
    """Sec. 3.1 Eq. 1 on the last axis of v (even length) at position pos; fp64."""
    out = _f64(v).copy()
    flat = out.reshape(-1, out.shape[-1])
    for i in range(flat.shape[0]):
        r = np.ascontiguousarray(flat[i])
        rc = _c().oracle_rope(_dp(r), ctypes.c_int(r.shape[0]), ctypes.c_double(pos), ctypes.c_double(base))
        if rc != 0:
            raise ValueError("rope needs an even length")
        flat[i] = r
    return out


def encode_bf16(x32) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    a = np.ascontiguousarray(x32, dtype=np.float32)
    f = _c().oracle_encode_bf16
    return np.array([f(ctypes.c_float(float(v))) for v in a.ravel()], dtype=np.uint16).reshape(a.shape)


def encode_e4m3(x32) -> np.ndarray:
    """float32 -> OCP e4m3 codes (uint8): nearest, ties to even, saturating."""
    a = np.ascontiguousarray(x32, dtype=np.float32)
    f = _c().oracle_encode_e4m3
    return np.array([f(ctypes.c_float(float(v))) for v in a.ravel()], dtype=np.uint8).reshape(a.shape)


def encode_row(row32, dtype: int):
    """One token's fp32 row -> (stored row, scale or None)."""
    r = np.ascontiguousarray(row32, dtype=np.float32)
    n = r.shape[0]
    dst = np.empty(n, dtype={F32: np.float32, BF16: np.uint16, FP8_E4M3: np.uint8}[dtype])
    sc = ctypes.c_float(0.0)
    _c().oracle_encode_row(r.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), ctypes.c_int(n), ctypes.c_int(dtype),
                           _vp(dst), ctypes.byref(sc))
    return dst, (float(np.float32(sc.value)) if dtype == FP8_E4M3 else None)


def cache_append(x, W, pool, kv_scale, page_table, positions, d_c: int, rope_base: float = 10000.0):
    """Append one token per sequence.  x [B, D], W [D, d_c + d_rope] (stored dtypes or floats;
    widened exactly), pool / kv_scale / page_table as for the decode.  Returns
    (new pool, new kv_scale or None, fp64 rows [B, d_c + d_rope]); the inputs are not modified."""
    pool, sc, dt = _pool_args(pool, kv_scale)
    pool = pool.copy()
    sc = None if sc is None else sc.copy()
    xw, Ww = _f64(widen(x)), _f64(widen(W))
    B, D = xw.shape
    n = Ww.shape[1]
    assert Ww.shape[0] == D and n == pool.shape[2]
    pt, ps = _i32(page_table), _i32(positions)
    rows = np.empty((B, n), dtype=np.float64)
    rc = _c().oracle_cache_append(
        _dp(xw), _dp(Ww), _vp(pool), None if sc is None else sc.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
        ctypes.c_int(dt), _ip(pt), _ip(ps), ctypes.c_int(B), ctypes.c_int(D), ctypes.c_int(d_c),
        ctypes.c_int(n - d_c), ctypes.c_int(pool.shape[1]), ctypes.c_int(pool.shape[0]),
        ctypes.c_int(pt.shape[1]), ctypes.c_double(rope_base), _dp(rows))
    if rc != 0:
        raise RuntimeError("oracle_cache_append failed")
    return pool, sc, rows
