"""Host-side checks of the C-ABI that need no GPU: the library loads, exports
every function the public header declares, and rejects bad arguments before
touching the HIP runtime (so no launch can happen here)."""
import ctypes
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parents[1]
HEADERS = sorted((ROOT / "include").glob("*.h"))
LIBPATH = ROOT / "paper_2502_07864_amd" / "libmla_gfx950.so"

OK, E_NULL, E_SHAPE, E_UNSUP, E_WS, E_HIP, E_SCRATCH = 0, -1, -2, -3, -4, -6, -7
F32, BF16, FP8 = 0, 1, 2


@pytest.fixture(scope="module")
def lib():
    if not LIBPATH.exists():
        from paper_2502_07864_amd.build import build_library
        build_library()
    L = ctypes.CDLL(str(LIBPATH))
    vp, i, u, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint, ctypes.c_float
    L.mla_status_string.restype = ctypes.c_char_p
    L.mla_version.restype = ctypes.c_char_p
    L.mla_absorb_q.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
    L.mla_out_proj.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
    L.mla_decode_workspace_bytes.restype = ctypes.c_size_t
    L.mla_decode_workspace_bytes.argtypes = [i, i, i, i]
    L.mla_decode_paged.argtypes = [vp] * 9 + [ctypes.c_size_t] + [i] * 8 + [f, i, i, u, vp]
    L.mla_static_scratch_bytes.restype = ctypes.c_size_t
    L.mla_static_scratch_bytes.argtypes = []
    L.mla_decode_paged_static.argtypes = [vp] * 8 + [i] * 8 + [f, i, i, u, vp]
    L.mla_decode_paged_multi.argtypes = [vp] * 9 + [ctypes.c_size_t] + [i] * 9 + [f, i, i, u, vp]
    L.mla_merge_out_proj_multi.argtypes = [vp, ctypes.c_size_t, vp, vp, vp, vp] + [i] * 7 + [u, vp]
    L.mla_prefill_workspace_bytes.restype = ctypes.c_size_t
    L.mla_prefill_workspace_bytes.argtypes = [i, i, i, i]
    L.mla_prefill_mha.argtypes = [vp] * 10 + [ctypes.c_size_t] + [i] * 9 + [f, i, i, vp]
    L.mla_gather_paged.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, vp]
    L.mla_diag_stream_tiles.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
    L.mla_append_workspace_bytes.restype = ctypes.c_size_t
    L.mla_append_workspace_bytes.argtypes = [i, i, i, i, i]
    L.mla_cache_append.argtypes = [vp] * 7 + [ctypes.c_size_t] + [i] * 7 + [f, i, i, vp]
    return L


def declared_functions():
    names = set()
    for header in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", header.read_text(), flags=re.S)
        names |= set(re.findall(r"\b(mla_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_functions_are_exported(lib):
    names = declared_functions()
    assert {"mla_absorb_q", "mla_decode_paged", "mla_out_proj", "mla_decode_workspace_bytes",
            "mla_gather_paged", "mla_status_string", "mla_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"


def test_binding_lists_the_same_entry_points():
    src = "".join((ROOT / "paper_2502_07864_amd" / f).read_text() for f in ("mla.py", "convert.py"))
    for n in declared_functions():
        assert n in src, f"{n} has no Python binding"


def test_status_strings(lib):
    assert lib.mla_status_string(OK) == b"MLA_OK"
    for code, key in [(E_NULL, b"NULL"), (E_SHAPE, b"SHAPE"), (E_UNSUP, b"UNSUPPORTED"),
                      (E_WS, b"WORKSPACE"), (E_HIP, b"HIP")]:
        assert key in lib.mla_status_string(code)
    assert b"unknown" in lib.mla_status_string(-99)
    assert lib.mla_version().startswith(b"mla-gfx950")


def test_workspace_bytes(lib):
    n = lib.mla_decode_workspace_bytes(16, 32, 512, 16)
    assert n >= 16 * 16 * 32 * 513 * 4 and n % 256 == 0
    assert lib.mla_decode_workspace_bytes(0, 32, 512, 16) == 0
    assert lib.mla_decode_workspace_bytes(16, 32, 512, 0) == 0
    assert lib.mla_decode_workspace_bytes(1, 1, 8, 1) >= 36


P = 0x1000  # a non-null, 256-aligned fake pointer: validation must fail before it is ever used


def test_projection_validation(lib):
    for fn in (lib.mla_absorb_q, lib.mla_out_proj):
        assert fn(None, P, P, 1, 1, 8, 8, F32, None) == E_NULL
        assert fn(P, None, P, 1, 1, 8, 8, F32, None) == E_NULL
        assert fn(P, P, None, 1, 1, 8, 8, F32, None) == E_NULL
        assert fn(P, P, P, 0, 1, 8, 8, F32, None) == E_SHAPE
        assert fn(P, P, P, 1, -1, 8, 8, F32, None) == E_SHAPE
        assert fn(P, P, P, 1, 1, 0, 8, F32, None) == E_SHAPE
        assert fn(P, P, P, 1, 1, 8, 8, FP8, None) == E_UNSUP
        assert fn(P, P, P, 1, 1, 8, 8, 7, None) == E_UNSUP


def decode_args(**kw):
    a = dict(q_abs=P, q_rope=P, kv=P, kv_scale=None, table=P, lens=P, o=P, lse=None, ws=P,
             ws_bytes=1 << 30, B=2, H=32, d_c=512, d_rope=64, page=64, num_pages=8, max_pages=4,
             splits=2, scale=0.07, io=BF16, cache=BF16, flags=0, stream=None)
    a.update(kw)
    return [a[k] for k in ("q_abs", "q_rope", "kv", "kv_scale", "table", "lens", "o", "lse", "ws",
                           "ws_bytes", "B", "H", "d_c", "d_rope", "page", "num_pages", "max_pages",
                           "splits", "scale", "io", "cache", "flags", "stream")]


@pytest.mark.parametrize("kw,want", [
    (dict(q_abs=None), E_NULL), (dict(q_rope=None), E_NULL), (dict(kv=None), E_NULL),
    (dict(table=None), E_NULL), (dict(lens=None), E_NULL), (dict(o=None), E_NULL),
    (dict(cache=FP8), E_NULL),                       # fp8 cache without scales
    (dict(kv_scale=P), E_SHAPE),                     # scales with a non-fp8 cache
    (dict(B=0), E_SHAPE), (dict(H=0), E_SHAPE), (dict(d_c=0), E_SHAPE), (dict(d_rope=-8), E_SHAPE),
    (dict(page=0), E_SHAPE), (dict(num_pages=0), E_SHAPE), (dict(max_pages=0), E_SHAPE),
    (dict(splits=0), E_SHAPE), (dict(scale=float("nan")), E_SHAPE),
    (dict(max_pages=1 << 30, page=64), E_SHAPE),
    (dict(io=FP8), E_UNSUP), (dict(cache=5), E_UNSUP), (dict(io=BF16, cache=F32), E_UNSUP),
    (dict(H=1025), E_UNSUP), (dict(d_c=520), E_UNSUP), (dict(d_c=12), E_UNSUP),
    (dict(d_rope=72), E_UNSUP), (dict(d_rope=4), E_UNSUP), (dict(B=70000), E_UNSUP),
    (dict(ws=None), E_WS), (dict(ws_bytes=1024), E_WS), (dict(ws=P + 8), E_WS),
])
def test_decode_validation(lib, kw, want):
    assert lib.mla_decode_paged(*decode_args(**kw)) == want


def static_args(**kw):
    a = decode_args(**kw)
    del a[8:10]                  # no workspace, no workspace_bytes
    return a


@pytest.mark.parametrize("kw,want", [
    (dict(q_abs=None), E_NULL), (dict(o=None), E_NULL), (dict(cache=FP8), E_NULL),
    (dict(B=0), E_SHAPE), (dict(splits=0), E_SHAPE), (dict(io=FP8), E_UNSUP), (dict(d_c=520), E_UNSUP),
    (dict(flags=2), E_UNSUP),                                   # MLA_FLAG_SKIP_MERGE
    (dict(flags=4, io=F32, cache=F32), E_UNSUP),                # balanced partition without the matrix-core kernel
    (dict(B=64, splits=16), E_SCRATCH),                         # 64 x 17 x 32 x 513 x 4 B = 71 MB
    (dict(B=16, H=64, splits=16), E_SCRATCH),
])
def test_static_scratch_decode_validation(lib, kw, want):
    """Everything, the scratch limit included, is rejected before the first HIP call."""
    assert lib.mla_decode_paged_static(*static_args(**kw)) == want


def test_static_scratch_limit(lib):
    n = lib.mla_static_scratch_bytes()
    assert n == 32 << 20
    assert lib.mla_decode_workspace_bytes(16, 32, 512, 16) <= n     # the headline shape fits
    assert b"SCRATCH" in lib.mla_status_string(E_SCRATCH)


@pytest.mark.parametrize("kw,q_len,want", [
    (dict(), 0, E_SHAPE), (dict(), -2, E_SHAPE), (dict(H=0), 2, E_SHAPE),
    (dict(H=32), 33, E_UNSUP), (dict(H=128), 9, E_UNSUP),       # more than 1024 query rows per sequence
    (dict(q_abs=None), 2, E_NULL), (dict(lens=None), 4, E_NULL),
    (dict(ws_bytes=2 * 3 * 32 * 513 * 4), 2, E_WS),             # sized for one query token only
    (dict(d_c=12), 2, E_UNSUP),
])
def test_multi_token_decode_validation(lib, kw, q_len, want):
    a = decode_args(**kw)
    a.insert(11, q_len)          # ..., B, q_len, heads, ...
    assert lib.mla_decode_paged_multi(*a) == want


def test_multi_token_tail_validation(lib):
    f = lib.mla_merge_out_proj_multi
    def call(**kw):
        d = dict(ws=P, ws_bytes=1 << 30, W=P, o=P, lse=None, out=P, B=2, q_len=2, H=32, d_c=512, d_head=128,
                 splits=2, io=BF16, flags=0, stream=None)
        d.update(kw)
        return f(*[d[k] for k in ("ws", "ws_bytes", "W", "o", "lse", "out", "B", "q_len", "H", "d_c", "d_head",
                                  "splits", "io", "flags", "stream")])
    assert call(W=None) == E_NULL and call(o=None) == E_NULL and call(out=None) == E_NULL
    assert call(q_len=0) == E_SHAPE and call(B=0) == E_SHAPE and call(d_head=0) == E_SHAPE
    assert call(io=FP8) == E_UNSUP and call(d_c=6) == E_UNSUP and call(B=40000, q_len=2) == E_UNSUP
    assert call(ws=None) == E_WS and call(ws_bytes=4096) == E_WS


def test_merge_row_count_that_overflows_32_bits_is_refused(lib):
    """65535 x 65535 output rows (x 2 column blocks) do not fit the merge kernels' 32-bit wavefront
    index: refused on the host, whatever the workspace size claims."""
    lib.mla_merge_partials.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_uint, ctypes.c_void_p]
    huge = (1 << 63) - 1
    assert lib.mla_merge_partials(P, huge, P, None, 65535, 65535, 512, 1, BF16, 0, None) == E_UNSUP
    f = lib.mla_merge_out_proj_multi
    assert f(P, huge, P, P, None, P, 65535, 1, 65535, 512, 128, 1, BF16, 0, None) == E_UNSUP


def prefill_args(**kw):
    a = dict(q_nope=P, q_rope=P, W_UK=P, W_UV=P, kv=P, table=P, lens=P, out=P, lse=None, ws=P, ws_bytes=1 << 40,
             B=2, q_len=100, H=32, d_head=128, d_c=512, d_rope=64, page=64, num_pages=8, max_pages=4, scale=0.07,
             io=BF16, cache=BF16, stream=None)
    a.update(kw)
    return [a[k] for k in ("q_nope", "q_rope", "W_UK", "W_UV", "kv", "table", "lens", "out", "lse", "ws", "ws_bytes",
                           "B", "q_len", "H", "d_head", "d_c", "d_rope", "page", "num_pages", "max_pages", "scale",
                           "io", "cache", "stream")]


@pytest.mark.parametrize("kw,want", [
    (dict(q_nope=None), E_NULL), (dict(q_rope=None), E_NULL), (dict(W_UK=None), E_NULL), (dict(W_UV=None), E_NULL),
    (dict(kv=None), E_NULL), (dict(table=None), E_NULL), (dict(lens=None), E_NULL), (dict(out=None), E_NULL),
    (dict(B=0), E_SHAPE), (dict(q_len=0), E_SHAPE), (dict(H=-1), E_SHAPE), (dict(d_c=0), E_SHAPE),
    (dict(max_pages=0), E_SHAPE), (dict(scale=float("nan")), E_SHAPE), (dict(max_pages=1 << 30), E_SHAPE),
    (dict(io=F32, cache=F32), E_UNSUP), (dict(cache=FP8), E_UNSUP), (dict(d_head=64), E_UNSUP),
    (dict(d_c=384), E_UNSUP), (dict(d_rope=32), E_UNSUP), (dict(page=16), E_UNSUP), (dict(B=4096), E_UNSUP),
    (dict(ws=None), E_WS), (dict(ws_bytes=1 << 20), E_WS), (dict(ws=P + 16), E_WS),
])
def test_prefill_validation(lib, kw, want):
    assert lib.mla_prefill_mha(*prefill_args(**kw)) == want


def test_prefill_workspace_bytes(lib):
    n = lib.mla_prefill_workspace_bytes(2, 32, 512, 4)
    assert n % 256 == 0
    assert n >= 32 * 256 * 512 * 2 + 2 * 32 * 4 * 64 * 320 * 2 + 2 * 32 * 4 * 4 + 2 * 32 * 4
    assert lib.mla_prefill_workspace_bytes(0, 32, 512, 4) == 0


def test_gather_validation(lib):
    g = lib.mla_gather_paged
    assert g(None, P, P, P, 1, 4, 64, 4, 2, 1, None) == E_NULL
    assert g(P, P, P, None, 1, 4, 64, 4, 2, 1, None) == E_NULL
    assert g(P, P, P, P, 0, 4, 64, 4, 2, 1, None) == E_SHAPE
    assert g(P, P, P, P, 1, 0, 64, 4, 2, 1, None) == E_SHAPE
    assert g(P, P, P, P, 1, 4, 0, 4, 2, 1, None) == E_SHAPE
    assert g(P, P, P, P, 1, 4, 6, 4, 2, 1, None) == E_UNSUP


def test_stream_probe_validation(lib):
    g = lib.mla_diag_stream_tiles
    assert g(None, P, P, 1, 512, 8, 4, 2, None) == E_NULL
    assert g(P, None, P, 1, 512, 8, 4, 2, None) == E_NULL
    assert g(P, P, None, 1, 512, 8, 4, 2, None) == E_NULL
    assert g(P, P, P, 0, 512, 8, 4, 2, None) == E_SHAPE
    assert g(P, P, P, 1, 512, 0, 4, 2, None) == E_SHAPE
    assert g(P, P, P, 1, 512, 8, 0, 2, None) == E_SHAPE
    assert g(P, P, P, 1, 512, 8, 4, 0, None) == E_SHAPE
    assert g(P, P, P, 1, 128, 8, 4, 2, None) == E_UNSUP
    assert g(P, P, P, 70000, 512, 8, 4, 2, None) == E_UNSUP


def append_args(**kw):
    a = dict(x=P, W=P, kv=P, kv_scale=None, table=P, pos=P, ws=P, ws_bytes=1 << 30, B=4, D=4096,
             d_c=512, d_rope=64, page=64, num_pages=8, max_pages=4, base=10000.0, io=BF16, cache=BF16,
             stream=None)
    a.update(kw)
    return [a[k] for k in ("x", "W", "kv", "kv_scale", "table", "pos", "ws", "ws_bytes", "B", "D", "d_c",
                           "d_rope", "page", "num_pages", "max_pages", "base", "io", "cache", "stream")]


@pytest.mark.parametrize("kw,want", [
    (dict(x=None), E_NULL), (dict(W=None), E_NULL), (dict(kv=None), E_NULL), (dict(table=None), E_NULL),
    (dict(pos=None), E_NULL), (dict(cache=FP8), E_NULL), (dict(kv_scale=P), E_NULL),
    (dict(B=0), E_SHAPE), (dict(D=0), E_SHAPE), (dict(d_c=0), E_SHAPE), (dict(d_rope=-2), E_SHAPE),
    (dict(d_rope=63), E_SHAPE), (dict(page=0), E_SHAPE), (dict(num_pages=0), E_SHAPE),
    (dict(max_pages=0), E_SHAPE), (dict(base=0.0), E_SHAPE), (dict(base=float("nan")), E_SHAPE),
    (dict(max_pages=1 << 30), E_SHAPE),
    (dict(io=FP8), E_UNSUP), (dict(cache=9), E_UNSUP), (dict(d_c=1000), E_UNSUP),
    (dict(ws=None), E_WS), (dict(ws_bytes=64), E_WS), (dict(ws=P + 4), E_WS),
])
def test_append_validation(lib, kw, want):
    assert lib.mla_cache_append(*append_args(**kw)) == want


def test_append_workspace_bytes(lib):
    n = lib.mla_append_workspace_bytes(16, 4096, 512, 64, BF16)
    assert n % 256 == 0 and n >= 16 * 576 * 4            # at least one fp32 partial row per sequence
    assert n <= 16 * (4096 // 32) * 576 * 4 + 256        # at most one per 32 model dimensions
    assert lib.mla_append_workspace_bytes(0, 4096, 512, 64, BF16) == 0
    assert lib.mla_append_workspace_bytes(16, 4096, 512, 64, FP8) == 0
    assert lib.mla_append_workspace_bytes(3, 100, 40, 8, F32) >= 3 * 48 * 4


def test_product_path_does_not_use_the_oracle():
    """The library, its binding and its build script never reference the test oracle."""
    pkg = ROOT / "paper_2502_07864_amd"
    for f in list(pkg.glob("*.py")) + list((pkg / "csrc").glob("*")):
        if not f.is_file():
            continue
        text = f.read_text()
        assert "oracle" not in text.lower(), f"{f} mentions the oracle"
        assert "workloads" not in text, f"{f} reaches for the input generator"
    # the input generator serves both sides and imports neither
    for f in (ROOT / "workloads").glob("*.py"):
        t = f.read_text()
        assert "import oracle" not in t and "from oracle" not in t and "paper_2502_07864_amd" not in t
    for f in (ROOT / "oracle").glob("*"):
        if f.suffix in (".py", ".c"):
            t = f.read_text()
            assert "paper_2502_07864_amd" not in t and "mla_gfx950" not in t and "workloads" not in t


# ------------------------------------------------------------------ offline conversion (mla_convert_gfx950.h)

def conv_lib(lib):
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.mla_conv_project.argtypes = [vp, vp, vp, i, i, i, i, vp]
    lib.mla_conv_rope_moments.argtypes = [vp, vp, i, i, i, i, vp]
    lib.mla_conv_sym_eig_workspace_bytes.restype = sz
    lib.mla_conv_sym_eig_workspace_bytes.argtypes = [i, i]
    lib.mla_conv_sym_eig.argtypes = [vp, vp, vp, sz, vp, i, i, i, vp]
    lib.mla_conv_rotate_rows.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
    lib.mla_conv_kv_balance.argtypes = [vp, i, vp, i, vp, vp, i, i, i, vp]
    lib.mla_conv_joint_moment.argtypes = [vp, i, vp, i, vp, vp, vp, i, i, i, vp]
    lib.mla_conv_top_eig_workspace_bytes.restype = sz
    lib.mla_conv_top_eig_workspace_bytes.argtypes = [i, i]
    lib.mla_conv_top_eig.argtypes = [vp, vp, vp, vp, vp, sz, vp, i, i, i, i, vp]
    lib.mla_conv_apply_workspace_bytes.restype = sz
    lib.mla_conv_apply_workspace_bytes.argtypes = [i, i]
    lib.mla_conv_apply.argtypes = [vp, vp, vp, vp, sz, i, i, vp]
    lib.mla_convert_layer_workspace_bytes.restype = sz
    lib.mla_convert_layer_workspace_bytes.argtypes = [i, i, i, i, i, i, i, i, i]
    lib.mla_convert_layer.argtypes = [vp] * 14 + [vp, sz, vp] + [i] * 10 + [vp]
    return lib


P = 0x1000   # a non-NULL pointer value; every call below is rejected before it could be used


def test_conversion_header_is_scanned():
    assert {"mla_conv_project", "mla_conv_sym_eig", "mla_conv_top_eig", "mla_convert_layer"} <= set(declared_functions())


def test_conversion_step_validation(lib):
    L = conv_lib(lib)
    assert L.mla_conv_project(None, P, P, 4, 4, 4, 4, None) == E_NULL
    assert L.mla_conv_project(P, P, P, 4, 4, 4, 3, None) == E_SHAPE          # ldy < m
    assert L.mla_conv_project(P, P, P, 0, 4, 4, 4, None) == E_SHAPE
    assert L.mla_conv_rope_moments(P, None, 8, 2, 8, 1, None) == E_NULL
    assert L.mla_conv_rope_moments(P, P, 8, 2, 7, 1, None) == E_SHAPE        # odd head dimension
    assert L.mla_conv_rope_moments(P, P, 8, 2, 8, 3, None) == E_SHAPE        # 4 pairs do not fold by 3
    assert L.mla_conv_rope_moments(P, P, 8, 32, 128, 8, None) == E_UNSUP     # M g = 256 > 128
    assert L.mla_conv_rotate_rows(P, P, P, 2, 8, 1, 1, 16, None) == E_SHAPE     # in place is not allowed
    assert L.mla_conv_rotate_rows(P, P, P + 64, 2, 8, 1, 1, 0, None) == E_SHAPE
    assert L.mla_conv_rotate_rows(P, P, P + 64, 2, 8, 2, 3, 16, None) == E_SHAPE  # keep > M
    assert L.mla_conv_rotate_rows(P, P, P + 64, 2, 8, 2, 0, 16, None) == E_SHAPE  # keep < 1
    assert L.mla_conv_kv_balance(P, 4, P, 4, None, P, 8, 4, 4, None) == E_NULL
    assert L.mla_conv_kv_balance(P, 3, P, 4, P, P, 8, 4, 4, None) == E_SHAPE  # ldk < a
    assert L.mla_conv_joint_moment(P, 4, P, 4, P, P, None, 8, 4, 4, None) == E_NULL
    assert L.mla_conv_joint_moment(P, 4, P, 4, P, P, P, 0, 4, 4, None) == E_SHAPE


def test_conversion_eigensolver_validation(lib):
    L = conv_lib(lib)
    need = L.mla_conv_sym_eig_workspace_bytes(3, 32)
    assert 3 * 32 * 32 * 8 <= need <= 3 * 32 * 32 * 8 + (1 << 16)
    assert L.mla_conv_sym_eig_workspace_bytes(1, 1) == 0 and L.mla_conv_sym_eig_workspace_bytes(1, 2049) == 0
    assert L.mla_conv_sym_eig(P, P, P, 1 << 20, None, 1, 8, 30, None) == E_NULL
    assert L.mla_conv_sym_eig(P, P, P, 1 << 20, P, 1, 1, 30, None) == E_SHAPE
    assert L.mla_conv_sym_eig(P, P, P, 1 << 30, P, 1, 4096, 30, None) == E_UNSUP
    assert L.mla_conv_sym_eig(P, P, P, L.mla_conv_sym_eig_workspace_bytes(1, 8) - 1, P, 1, 8, 30, None) == E_WS
    assert L.mla_conv_sym_eig(P, P, None, 0, P, 1, 8, 30, None) == E_WS
    n = L.mla_conv_top_eig_workspace_bytes(8064, 576)
    assert n >= 2 * 8064 * 576 * 8 + 4 * 576 * 576 * 8 and n % 256 == 0
    assert L.mla_conv_top_eig_workspace_bytes(100, 101) == 0 and L.mla_conv_top_eig_workspace_bytes(4096, 2048) == 0
    assert L.mla_conv_top_eig(P, P, P, P, P, 1 << 30, P, 100, 20, 10, 5, None) == E_SHAPE      # p < r
    assert L.mla_conv_top_eig(P, P, P, P, P, 1 << 30, P, 100, 20, 101, 5, None) == E_SHAPE     # p > m
    assert L.mla_conv_top_eig(P, P, P, P, P, 1 << 40, P, 4096, 20, 2048, 5, None) == E_UNSUP   # p > 1024
    assert L.mla_conv_top_eig(P, P, P, P, P, 16, P, 100, 20, 30, 5, None) == E_WS
    assert L.mla_conv_top_eig(P, None, P, P, P, 1 << 30, P, 100, 20, 30, 5, None) == E_NULL
    assert L.mla_conv_apply(P, P, None, None, 0, 8, 4, None) == E_NULL
    assert L.mla_conv_apply(P, P, P, None, 0, 8, 4, None) == E_SHAPE       # in place is not allowed
    assert L.mla_conv_apply(P, P, P + 64, None, 0, 8, 0, None) == E_SHAPE
    assert L.mla_conv_apply_workspace_bytes(8064, 576) == 4 * 8064 * 576 * 8


def test_conversion_chain_validation(lib):
    L = conv_lib(lib)
    ok = dict(n=256, D=64, g=4, h=8, d=16, M=1, keep=1, r_kv=24, p=32, iters=10)

    def call(ws_bytes=1 << 40, null_at=None, **kw):
        a = dict(ok, **kw)
        ptrs = [P] * 14
        if null_at is not None:
            ptrs[null_at] = None
        return L.mla_convert_layer(*ptrs, P, ws_bytes, P, a["n"], a["D"], a["g"], a["h"], a["d"], a["M"], a["keep"],
                                   a["r_kv"], a["p"], a["iters"], None)

    need = L.mla_convert_layer_workspace_bytes(256, 64, 4, 8, 16, 1, 1, 24, 32)
    assert need > 256 * (7 * 16) * 8 and need % 256 == 0
    assert call(null_at=0) == E_NULL and call(null_at=13) == E_NULL
    assert call(h=6) == E_SHAPE            # h not a multiple of g
    assert call(d=15) == E_SHAPE
    assert call(M=3, keep=3) == E_SHAPE    # 8 pairs do not fold by 3
    assert call(M=2, keep=3) == E_SHAPE    # more kept components than the group has pairs
    assert call(M=2, keep=1, p=121) == E_SHAPE   # p > 2 g d - d_rope = 120
    assert call(M=2, keep=1, p=120, ws_bytes=16) == E_WS   # a valid shape: only the workspace is wrong
    assert call(r_kv=40) == E_SHAPE        # r_kv > p
    assert call(p=200) == E_SHAPE          # p > (2g-1)d = 112
    assert call(g=1, h=8) == E_SHAPE       # nothing to merge
    assert call(g=32, h=32, d=128, M=8, keep=8, D=4096, r_kv=512, p=576) == E_UNSUP   # M g > 128
    assert call(ws_bytes=need - 1) == E_WS
    assert L.mla_convert_layer_workspace_bytes(256, 64, 4, 6, 16, 1, 1, 24, 32) == 0
