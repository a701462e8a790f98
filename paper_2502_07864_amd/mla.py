"""Python binding of the gfx950 MLA decode library (``include/mla_gfx950.h``).

Argument marshalling only: every function takes torch tensors that already
live on the GPU, passes their device pointers and the current HIP stream to
the C entry point of the same name, and returns the output tensor.  torch is
used for device memory and streams; no arithmetic happens here and there is
no fallback path: a missing library or a failing call raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional

import torch

_LIB_PATH = Path(__file__).resolve().parent / "libmla_gfx950.so"
_lib = None

F32, BF16, FP8_E4M3 = 0, 1, 2
FLAG_DEFAULT, FLAG_PORTABLE_KERNEL, FLAG_SKIP_MERGE, FLAG_BALANCED = 0, 1, 2, 4

EXPORTS = ("mla_status_string", "mla_version", "mla_absorb_q", "mla_out_proj",
           "mla_decode_workspace_bytes", "mla_decode_paged", "mla_merge_partials",
           "mla_merge_out_proj", "mla_gather_paged", "mla_append_workspace_bytes", "mla_cache_append",
           "mla_decode_paged_multi", "mla_merge_out_proj_multi", "mla_prefill_workspace_bytes", "mla_prefill_mha",
           "mla_static_scratch_bytes", "mla_decode_paged_static", "mla_diag_stream_tiles")


class MlaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def lib() -> ctypes.CDLL:
    """Load libmla_gfx950.so (built in-tree by ``python -m paper_2502_07864_amd.build``)."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2502_07864_amd.build`")
        L = ctypes.CDLL(str(_LIB_PATH))
        vp, i, u, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint, ctypes.c_float
        L.mla_status_string.restype = ctypes.c_char_p
        L.mla_status_string.argtypes = [i]
        L.mla_version.restype = ctypes.c_char_p
        L.mla_version.argtypes = []
        L.mla_absorb_q.restype = i
        L.mla_absorb_q.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
        L.mla_out_proj.restype = i
        L.mla_out_proj.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
        L.mla_decode_workspace_bytes.restype = ctypes.c_size_t
        L.mla_decode_workspace_bytes.argtypes = [i, i, i, i]
        L.mla_decode_paged.restype = i
        L.mla_decode_paged.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t,
                                       i, i, i, i, i, i, i, i, f, i, i, u, vp]
        L.mla_static_scratch_bytes.restype = ctypes.c_size_t
        L.mla_static_scratch_bytes.argtypes = []
        L.mla_decode_paged_static.restype = i
        L.mla_decode_paged_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp,
                                              i, i, i, i, i, i, i, i, f, i, i, u, vp]
        L.mla_decode_paged_multi.restype = i
        L.mla_decode_paged_multi.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t,
                                             i, i, i, i, i, i, i, i, i, f, i, i, u, vp]
        L.mla_merge_out_proj_multi.restype = i
        L.mla_merge_out_proj_multi.argtypes = [vp, ctypes.c_size_t, vp, vp, vp, vp, i, i, i, i, i, i, i, u, vp]
        L.mla_prefill_workspace_bytes.restype = ctypes.c_size_t
        L.mla_prefill_workspace_bytes.argtypes = [i, i, i, i]
        L.mla_prefill_mha.restype = i
        L.mla_prefill_mha.argtypes = [vp] * 10 + [ctypes.c_size_t] + [i] * 9 + [f, i, i, vp]
        L.mla_merge_partials.restype = i
        L.mla_merge_partials.argtypes = [vp, ctypes.c_size_t, vp, vp, i, i, i, i, i, u, vp]
        L.mla_merge_out_proj.restype = i
        L.mla_merge_out_proj.argtypes = [vp, ctypes.c_size_t, vp, vp, vp, vp, i, i, i, i, i, i, u, vp]
        L.mla_gather_paged.restype = i
        L.mla_gather_paged.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, vp]
        L.mla_diag_stream_tiles.restype = i
        L.mla_diag_stream_tiles.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
        L.mla_append_workspace_bytes.restype = ctypes.c_size_t
        L.mla_append_workspace_bytes.argtypes = [i, i, i, i, i]
        L.mla_cache_append.restype = i
        L.mla_cache_append.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t,
                                       i, i, i, i, i, i, i, f, i, i, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().mla_status_string(int(status)).decode()


def version() -> str:
    return lib().mla_version().decode()


def _io_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"io dtype must be float32 or bfloat16, got {t.dtype}")


def _cache_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype in (torch.uint8, torch.float8_e4m3fn):
        return FP8_E4M3
    raise TypeError(f"cache dtype must be float32, bfloat16, uint8 or float8_e4m3fn, got {t.dtype}")


def _dev(t: Optional[torch.Tensor], name: str):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream(t: torch.Tensor):
    return torch.cuda.current_stream(t.device).cuda_stream


def _check(status: int, where: str):
    if status != 0:
        raise MlaError(status, where)


def absorb_q(q_nope: torch.Tensor, W_UK: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """q_abs[b,h,:] = q_nope[b,h,:] . W_UK[h];  q_nope [B,H,d_head], W_UK [H,d_head,d_c]."""
    B, H, d_head = q_nope.shape
    H2, d_head2, d_c = W_UK.shape
    if (H2, d_head2) != (H, d_head) or W_UK.dtype != q_nope.dtype:
        raise ValueError("W_UK must be [H, d_head, d_c] of q_nope's dtype")
    if out is None:
        out = torch.empty((B, H, d_c), dtype=q_nope.dtype, device=q_nope.device)
    _check(lib().mla_absorb_q(_dev(q_nope, "q_nope"), _dev(W_UK, "W_UK"), _dev(out, "out"),
                              B, H, d_head, d_c, _io_code(q_nope), _stream(q_nope)), "mla_absorb_q")
    return out


def out_proj(o_lat: torch.Tensor, W_UV: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """out[b,h,:] = o_lat[b,h,:] . W_UV[h];  o_lat [B,H,d_c], W_UV [H,d_c,d_head]."""
    B, H, d_c = o_lat.shape
    H2, d_c2, d_head = W_UV.shape
    if (H2, d_c2) != (H, d_c) or W_UV.dtype != o_lat.dtype:
        raise ValueError("W_UV must be [H, d_c, d_head] of o_lat's dtype")
    if out is None:
        out = torch.empty((B, H, d_head), dtype=o_lat.dtype, device=o_lat.device)
    _check(lib().mla_out_proj(_dev(o_lat, "o_lat"), _dev(W_UV, "W_UV"), _dev(out, "out"),
                              B, H, d_c, d_head, _io_code(o_lat), _stream(o_lat)), "mla_out_proj")
    return out


def decode_workspace_bytes(B: int, H: int, d_c: int, num_splits: int) -> int:
    return int(lib().mla_decode_workspace_bytes(B, H, d_c, num_splits))


def decode_paged(q_abs: torch.Tensor, q_rope: Optional[torch.Tensor], kv_cache: torch.Tensor,
                 page_table: torch.Tensor, seq_lens: torch.Tensor, softmax_scale: float,
                 num_splits: int = 1, kv_scale: Optional[torch.Tensor] = None,
                 workspace: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                 lse: Optional[torch.Tensor] = None, return_lse: bool = False, flags: int = 0):
    """Paged absorbed decode.  kv_cache [num_pages, page_size, d_c+d_rope];
    page_table int32 [B, max_pages_per_seq]; seq_lens int32 [B].
    Returns o_lat [B,H,d_c] (and lse [B,H] fp32 if return_lse or lse given)."""
    B, H, d_c = q_abs.shape
    num_pages, page_size, row = kv_cache.shape
    d_rope = row - d_c
    if d_rope < 0:
        raise ValueError("cache rows are shorter than d_c")
    if d_rope and (q_rope is None or tuple(q_rope.shape) != (B, H, d_rope) or q_rope.dtype != q_abs.dtype):
        raise ValueError("q_rope must be [B, H, d_rope] of q_abs's dtype")
    if page_table.dtype != torch.int32 or seq_lens.dtype != torch.int32:
        raise TypeError("page_table and seq_lens must be int32")
    if page_table.dim() != 2 or page_table.shape[0] != B or seq_lens.shape != (B,):
        raise ValueError("page_table must be [B, max_pages_per_seq], seq_lens [B]")
    if kv_scale is not None and (kv_scale.dtype != torch.float32 or tuple(kv_scale.shape) != (num_pages, page_size)):
        raise ValueError("kv_scale must be float32 [num_pages, page_size]")
    need = decode_workspace_bytes(B, H, d_c, num_splits)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q_abs.device)
    skip_merge = bool(flags & FLAG_SKIP_MERGE)
    if out is None and not skip_merge:
        out = torch.empty((B, H, d_c), dtype=q_abs.dtype, device=q_abs.device)
    if lse is None and return_lse:
        lse = torch.empty((B, H), dtype=torch.float32, device=q_abs.device)
    _check(lib().mla_decode_paged(
        _dev(q_abs, "q_abs"), _dev(q_rope, "q_rope"), _dev(kv_cache, "kv_cache"),
        _dev(kv_scale, "kv_scale"), _dev(page_table, "page_table"), _dev(seq_lens, "seq_lens"),
        _dev(out, "out"), _dev(lse, "lse"), _dev(workspace, "workspace"),
        workspace.numel() * workspace.element_size(), B, H, d_c, d_rope, page_size, num_pages,
        page_table.shape[1], num_splits, float(softmax_scale), _io_code(q_abs),
        _cache_code(kv_cache), int(flags), _stream(q_abs)), "mla_decode_paged")
    if skip_merge:
        return workspace
    return (out, lse) if lse is not None else out


def static_scratch_bytes() -> int:
    return int(lib().mla_static_scratch_bytes())


def decode_paged_static(q_abs: torch.Tensor, q_rope: Optional[torch.Tensor], kv_cache: torch.Tensor,
                        page_table: torch.Tensor, seq_lens: torch.Tensor, softmax_scale: float,
                        out: torch.Tensor, num_splits: int = 1, kv_scale: Optional[torch.Tensor] = None,
                        lse: Optional[torch.Tensor] = None, flags: int = 0):
    """decode_paged without a workspace (the partials live in the library's static device array) and
    without any allocation: the caller passes `out` [B,H,d_c] (and `lse` [B,H] fp32 if wanted).
    The tensors' device must be the current device."""
    B, H, d_c = q_abs.shape
    num_pages, page_size, row = kv_cache.shape
    d_rope = row - d_c
    if d_rope < 0:
        raise ValueError("cache rows are shorter than d_c")
    if d_rope and (q_rope is None or tuple(q_rope.shape) != (B, H, d_rope) or q_rope.dtype != q_abs.dtype):
        raise ValueError("q_rope must be [B, H, d_rope] of q_abs's dtype")
    if page_table.dtype != torch.int32 or seq_lens.dtype != torch.int32:
        raise TypeError("page_table and seq_lens must be int32")
    if page_table.dim() != 2 or page_table.shape[0] != B or seq_lens.shape != (B,):
        raise ValueError("page_table must be [B, max_pages_per_seq], seq_lens [B]")
    if tuple(out.shape) != (B, H, d_c) or out.dtype != q_abs.dtype:
        raise ValueError("out must be [B, H, d_c] of q_abs's dtype")
    if lse is not None and (tuple(lse.shape) != (B, H) or lse.dtype != torch.float32):
        raise ValueError("lse must be float32 [B, H]")
    if q_abs.device.index != torch.cuda.current_device():
        raise ValueError("the tensors' device must be the current device")
    _check(lib().mla_decode_paged_static(
        _dev(q_abs, "q_abs"), _dev(q_rope, "q_rope"), _dev(kv_cache, "kv_cache"),
        _dev(kv_scale, "kv_scale"), _dev(page_table, "page_table"), _dev(seq_lens, "seq_lens"),
        _dev(out, "out"), _dev(lse, "lse"), B, H, d_c, d_rope, page_size, num_pages,
        page_table.shape[1], num_splits, float(softmax_scale), _io_code(q_abs),
        _cache_code(kv_cache), int(flags), _stream(q_abs)), "mla_decode_paged_static")
    return out


def decode_paged_multi(q_abs: torch.Tensor, q_rope: Optional[torch.Tensor], kv_cache: torch.Tensor,
                       page_table: torch.Tensor, seq_lens: torch.Tensor, softmax_scale: float,
                       num_splits: int = 1, kv_scale: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                       lse: Optional[torch.Tensor] = None, return_lse: bool = False, flags: int = 0):
    """Paged absorbed decode of q_len query tokens per sequence in one pass over the cache.
    q_abs [B,q_len,H,d_c], q_rope [B,q_len,H,d_rope]; the cache already holds the query tokens'
    own rows (the last q_len of each sequence) and token i sees rows < seq_len - (q_len-1-i).
    Returns o_lat [B,q_len,H,d_c] (and lse [B,q_len,H] fp32 if return_lse or lse given)."""
    B, T, H, d_c = q_abs.shape
    num_pages, page_size, row = kv_cache.shape
    d_rope = row - d_c
    if d_rope < 0:
        raise ValueError("cache rows are shorter than d_c")
    if d_rope and (q_rope is None or tuple(q_rope.shape) != (B, T, H, d_rope) or q_rope.dtype != q_abs.dtype):
        raise ValueError("q_rope must be [B, q_len, H, d_rope] of q_abs's dtype")
    if page_table.dtype != torch.int32 or seq_lens.dtype != torch.int32:
        raise TypeError("page_table and seq_lens must be int32")
    if page_table.dim() != 2 or page_table.shape[0] != B or seq_lens.shape != (B,):
        raise ValueError("page_table must be [B, max_pages_per_seq], seq_lens [B]")
    if kv_scale is not None and (kv_scale.dtype != torch.float32 or tuple(kv_scale.shape) != (num_pages, page_size)):
        raise ValueError("kv_scale must be float32 [num_pages, page_size]")
    need = decode_workspace_bytes(B, T * H, d_c, num_splits)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q_abs.device)
    skip_merge = bool(flags & FLAG_SKIP_MERGE)
    if out is None and not skip_merge:
        out = torch.empty((B, T, H, d_c), dtype=q_abs.dtype, device=q_abs.device)
    if lse is None and return_lse:
        lse = torch.empty((B, T, H), dtype=torch.float32, device=q_abs.device)
    _check(lib().mla_decode_paged_multi(
        _dev(q_abs, "q_abs"), _dev(q_rope, "q_rope"), _dev(kv_cache, "kv_cache"),
        _dev(kv_scale, "kv_scale"), _dev(page_table, "page_table"), _dev(seq_lens, "seq_lens"),
        _dev(out, "out"), _dev(lse, "lse"), _dev(workspace, "workspace"),
        workspace.numel() * workspace.element_size(), B, T, H, d_c, d_rope, page_size, num_pages,
        page_table.shape[1], num_splits, float(softmax_scale), _io_code(q_abs),
        _cache_code(kv_cache), int(flags), _stream(q_abs)), "mla_decode_paged_multi")
    if skip_merge:
        return workspace
    return (out, lse) if lse is not None else out


def merge_out_proj_multi(workspace: torch.Tensor, W_UV: torch.Tensor, B: int, q_len: int, num_splits: int,
                         o_lat: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                         lse: Optional[torch.Tensor] = None, return_lse: bool = False, flags: int = 0):
    """merge_out_proj after decode_paged_multi(flags=FLAG_SKIP_MERGE).
    Returns (o_lat [B,q_len,H,d_c], out [B,q_len,H,d_head][, lse [B,q_len,H]])."""
    H, d_c, d_head = W_UV.shape
    if o_lat is None:
        o_lat = torch.empty((B, q_len, H, d_c), dtype=W_UV.dtype, device=W_UV.device)
    if out is None:
        out = torch.empty((B, q_len, H, d_head), dtype=W_UV.dtype, device=W_UV.device)
    if lse is None and return_lse:
        lse = torch.empty((B, q_len, H), dtype=torch.float32, device=W_UV.device)
    _check(lib().mla_merge_out_proj_multi(_dev(workspace, "workspace"),
                                          workspace.numel() * workspace.element_size(), _dev(W_UV, "W_UV"),
                                          _dev(o_lat, "o_lat"), _dev(lse, "lse"), _dev(out, "out"), B, q_len, H,
                                          d_c, d_head, num_splits, _io_code(W_UV), int(flags),
                                          _stream(workspace)), "mla_merge_out_proj_multi")
    return (o_lat, out, lse) if lse is not None else (o_lat, out)


def prefill_workspace_bytes(B: int, heads: int, d_c: int, max_pages_per_seq: int) -> int:
    return int(lib().mla_prefill_workspace_bytes(B, heads, d_c, max_pages_per_seq))


def prefill_mha(q_nope: torch.Tensor, q_rope: torch.Tensor, W_UK: torch.Tensor, W_UV: torch.Tensor,
                kv_cache: torch.Tensor, page_table: torch.Tensor, seq_lens: torch.Tensor, softmax_scale: float,
                workspace: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                lse: Optional[torch.Tensor] = None, return_lse: bool = False):
    """Prefill in the MHA paradigm: keys [W_UK c ; k_rope] and values W_UV c materialised per head,
    causal attention of the q_len newest tokens of every sequence (the cache holds their rows).
    q_nope [B,q_len,H,d_head], q_rope [B,q_len,H,d_rope] -> out [B,q_len,H,d_head] (and lse [B,q_len,H])."""
    B, T, H, d_head = q_nope.shape
    H2, d_head2, d_c = W_UK.shape
    num_pages, page_size, row = kv_cache.shape
    d_rope = row - d_c
    if (H2, d_head2) != (H, d_head) or tuple(W_UV.shape) != (H, d_c, d_head):
        raise ValueError("W_UK must be [H, d_head, d_c] and W_UV [H, d_c, d_head]")
    if tuple(q_rope.shape) != (B, T, H, d_rope) or q_rope.dtype != q_nope.dtype:
        raise ValueError("q_rope must be [B, q_len, H, d_rope] of q_nope's dtype")
    if page_table.dtype != torch.int32 or seq_lens.dtype != torch.int32:
        raise TypeError("page_table and seq_lens must be int32")
    if page_table.dim() != 2 or page_table.shape[0] != B or seq_lens.shape != (B,):
        raise ValueError("page_table must be [B, max_pages_per_seq], seq_lens [B]")
    if workspace is None:
        workspace = torch.empty(max(256, prefill_workspace_bytes(B, H, d_c, page_table.shape[1])),
                                dtype=torch.uint8, device=q_nope.device)
    if out is None:
        out = torch.empty((B, T, H, d_head), dtype=q_nope.dtype, device=q_nope.device)
    if lse is None and return_lse:
        lse = torch.empty((B, T, H), dtype=torch.float32, device=q_nope.device)
    _check(lib().mla_prefill_mha(
        _dev(q_nope, "q_nope"), _dev(q_rope, "q_rope"), _dev(W_UK, "W_UK"), _dev(W_UV, "W_UV"),
        _dev(kv_cache, "kv_cache"), _dev(page_table, "page_table"), _dev(seq_lens, "seq_lens"),
        _dev(out, "out"), _dev(lse, "lse"), _dev(workspace, "workspace"),
        workspace.numel() * workspace.element_size(), B, T, H, d_head, d_c, d_rope, page_size, num_pages,
        page_table.shape[1], float(softmax_scale), _io_code(q_nope), _cache_code(kv_cache),
        _stream(q_nope)), "mla_prefill_mha")
    return (out, lse) if lse is not None else out


def merge_partials(workspace: torch.Tensor, B: int, H: int, d_c: int, num_splits: int,
                   dtype: torch.dtype, out: Optional[torch.Tensor] = None,
                   lse: Optional[torch.Tensor] = None, return_lse: bool = False, flags: int = 0):
    """Merge the per-chunk partials left in `workspace` by decode_paged(flags=FLAG_SKIP_MERGE);
    pass FLAG_BALANCED here iff the decode call had it."""
    if out is None:
        out = torch.empty((B, H, d_c), dtype=dtype, device=workspace.device)
    if lse is None and return_lse:
        lse = torch.empty((B, H), dtype=torch.float32, device=workspace.device)
    _check(lib().mla_merge_partials(_dev(workspace, "workspace"),
                                    workspace.numel() * workspace.element_size(),
                                    _dev(out, "out"), _dev(lse, "lse"), B, H, d_c, num_splits,
                                    _io_code(out), int(flags), _stream(workspace)), "mla_merge_partials")
    return (out, lse) if lse is not None else out


def merge_out_proj(workspace: torch.Tensor, W_UV: torch.Tensor, B: int, num_splits: int,
                   o_lat: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                   lse: Optional[torch.Tensor] = None, return_lse: bool = False, flags: int = 0):
    """Merge the partials left by decode_paged(flags=FLAG_SKIP_MERGE) and apply W_UV [H,d_c,d_head]
    (pass FLAG_BALANCED here iff the decode call had it).
    Returns (o_lat [B,H,d_c], out [B,H,d_head][, lse])."""
    H, d_c, d_head = W_UV.shape
    if o_lat is None:
        o_lat = torch.empty((B, H, d_c), dtype=W_UV.dtype, device=W_UV.device)
    if out is None:
        out = torch.empty((B, H, d_head), dtype=W_UV.dtype, device=W_UV.device)
    if lse is None and return_lse:
        lse = torch.empty((B, H), dtype=torch.float32, device=W_UV.device)
    _check(lib().mla_merge_out_proj(_dev(workspace, "workspace"),
                                    workspace.numel() * workspace.element_size(), _dev(W_UV, "W_UV"),
                                    _dev(o_lat, "o_lat"), _dev(lse, "lse"), _dev(out, "out"), B, H, d_c,
                                    d_head, num_splits, _io_code(W_UV), int(flags), _stream(workspace)),
           "mla_merge_out_proj")
    return (o_lat, out, lse) if lse is not None else (o_lat, out)


def gather_paged(kv_cache: torch.Tensor, page_table: torch.Tensor, seq_lens: torch.Tensor,
                 max_len: int) -> torch.Tensor:
    """Logical view of the cache: uint8 [B, max_len, row_bytes], rows past seq_len zeroed."""
    num_pages, page_size, row = kv_cache.shape
    row_bytes = row * kv_cache.element_size()
    B = seq_lens.shape[0]
    dense = torch.empty((B, max_len, row_bytes), dtype=torch.uint8, device=kv_cache.device)
    _check(lib().mla_gather_paged(_dev(kv_cache, "kv_cache"), _dev(page_table, "page_table"),
                                  _dev(seq_lens, "seq_lens"), _dev(dense, "dense"), B, max_len,
                                  row_bytes, page_size, num_pages, page_table.shape[1],
                                  _stream(kv_cache)), "mla_gather_paged")
    return dense


def diag_stream_tiles(kv_cache: torch.Tensor, page_table: torch.Tensor, seq_lens: torch.Tensor,
                      num_splits: int) -> None:
    """Diagnostic: the bf16 decode kernel's tile requests, waits and barriers over the cached rows,
    with no arithmetic and no output (what streaming the cache once costs in that launch shape)."""
    num_pages, page_size, row = kv_cache.shape
    if kv_cache.dtype != torch.bfloat16 or page_size != 64:
        raise ValueError("diag_stream_tiles takes a bf16 cache with pages of 64 rows")
    _check(lib().mla_diag_stream_tiles(_dev(kv_cache, "kv_cache"), _dev(page_table, "page_table"),
                                       _dev(seq_lens, "seq_lens"), seq_lens.shape[0], row - 64, num_pages,
                                       page_table.shape[1], num_splits, _stream(kv_cache)),
           "mla_diag_stream_tiles")


def append_workspace_bytes(B: int, D: int, d_c: int, d_rope: int, io_dtype: torch.dtype = torch.bfloat16) -> int:
    code = F32 if io_dtype == torch.float32 else BF16
    return int(lib().mla_append_workspace_bytes(B, D, d_c, d_rope, code))


def cache_append(x: torch.Tensor, W_DKVR: torch.Tensor, kv_cache: torch.Tensor, page_table: torch.Tensor,
                 positions: torch.Tensor, d_c: int, kv_scale: Optional[torch.Tensor] = None,
                 rope_base: float = 10000.0, workspace: Optional[torch.Tensor] = None) -> None:
    """Writes row [x . W[:, :d_c] | RoPE(x . W[:, d_c:], positions)] of one new token per sequence
    into kv_cache (in place) at logical position positions[b];  x [B, D], W_DKVR [D, d_c + d_rope]."""
    B, D = x.shape
    D2, n = W_DKVR.shape
    num_pages, page_size, row = kv_cache.shape
    if D2 != D or n != row or W_DKVR.dtype != x.dtype:
        raise ValueError("W_DKVR must be [D, d_c + d_rope] of x's dtype, matching the cache row")
    d_rope = n - d_c
    if workspace is None:
        workspace = torch.empty(max(16, append_workspace_bytes(B, D, d_c, d_rope, x.dtype)),
                                dtype=torch.uint8, device=x.device)
    _check(lib().mla_cache_append(_dev(x, "x"), _dev(W_DKVR, "W_DKVR"), _dev(kv_cache, "kv_cache"),
                                  _dev(kv_scale, "kv_scale"), _dev(page_table, "page_table"),
                                  _dev(positions, "positions"), _dev(workspace, "workspace"),
                                  workspace.numel(), B, D, d_c, d_rope, page_size, num_pages,
                                  page_table.shape[1], float(rope_base), _io_code(x),
                                  _cache_code(kv_cache), _stream(x)), "mla_cache_append")
