// C-ABI entry points: host-side argument validation, then kernel launches.
// Validation never touches the HIP runtime, so every error path can be
// exercised on a machine without a GPU.
#include "mla_internal.h"

#include <mutex>

using namespace mla;

namespace {

bool io_ok(mla_dtype t) { return t == MLA_F32 || t == MLA_BF16; }

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Chunks actually used for a request of num_splits chunks per sequence: when the batch is too
// small for num_splits chunks to give every CU a workgroup, each requested chunk is cut again
// (x2 or x4).  Every entry point derives the workspace layout from this same rule.
int effective_splits(int B, int num_splits)
{
    int m = 1;
    while (m < 4 && (long)B * num_splits * m < 256) m *= 2;
    return num_splits * m;
}

// Workspace: partial outputs, partial log-sum-exps, plan.  Sized for B * (S + 1) partial slots:
// the uniform partition uses B * S of them ([B, H, S, d_c]), the balanced one up to B * S + B - 1
// ([slot, H, d_c]); the plan ([B, 2] int32) is written and read by the balanced partition only.
struct WsLayout {
    size_t lse_off, plan_off, total;
};

WsLayout ws_layout(int B, int H, int d_c, int eff_splits)
{
    const size_t slots = (size_t)B * (eff_splits + 1);
    WsLayout l;
    l.lse_off = align_up(slots * H * d_c * sizeof(float), 256);
    l.plan_off = l.lse_off + align_up(slots * H * sizeof(float), 256);
    l.total = l.plan_off + align_up((size_t)B * 2 * sizeof(int32_t), 256);
    return l;
}

void fill_merge_params(MergeParams& m, const void* workspace, int B, int H, int d_c, int eff_splits,
                       bool balanced)
{
    const WsLayout l = ws_layout(B, H, d_c, eff_splits);
    m.o_part = static_cast<const float*>(workspace);
    m.lse_part = reinterpret_cast<const float*>(static_cast<const char*>(workspace) + l.lse_off);
    m.plan = balanced ? reinterpret_cast<const int32_t*>(static_cast<const char*>(workspace) + l.plan_off)
                      : nullptr;
    m.B = B; m.H = H; m.d_c = d_c; m.num_splits = eff_splits;
}

// The merge kernels index their wavefronts (one per output row and block of 256 columns) with 32-bit
// integers: sizes whose row count would not fit are refused rather than wrapped.
bool merge_rows_overflow(long long B, long long H, int d_c)
{
    return B * H * ((d_c + 255) / 256) > 0x7FFFFFFFLL;
}

// Arguments of one decode call (mla_decode_paged_multi's, without the workspace).
struct DecodeCall {
    const void* q_abs; const void* q_rope; const void* kv_cache; const float* kv_scale;
    const int32_t* page_table; const int32_t* seq_lens; void* o_lat; float* lse;
    int B, q_len, heads, d_c, d_rope, page_size, num_pages, max_pages_per_seq, num_splits;
    float softmax_scale;
    mla_dtype io_dtype, cache_dtype;
    unsigned flags;
    void* hip_stream;
};

// whether the call runs on the matrix-core kernels
bool uses_mfma(const DecodeCall& c)
{
    DecodeParams p = {};
    p.B = c.B; p.H = c.q_len * c.heads; p.d_c = c.d_c; p.d_rope = c.d_rope; p.page_size = c.page_size;
    p.num_splits = effective_splits(c.B, c.num_splits);
    return !(c.flags & MLA_FLAG_PORTABLE_KERNEL) && decode_mfma_supported(p, c.io_dtype, c.cache_dtype);
}

// host-side validation of everything but the workspace; touches no HIP call
int decode_validate(const DecodeCall& c)
{
    const bool skip_merge = (c.flags & MLA_FLAG_SKIP_MERGE) != 0;
    if (!c.q_abs || !c.kv_cache || !c.page_table || !c.seq_lens || (!c.o_lat && !skip_merge)) return MLA_ERR_NULL;
    if (c.d_rope > 0 && !c.q_rope) return MLA_ERR_NULL;
    if (c.B <= 0 || c.q_len <= 0 || c.heads <= 0 || c.d_c <= 0 || c.d_rope < 0 || c.page_size <= 0 ||
        c.num_pages <= 0 || c.max_pages_per_seq <= 0 || c.num_splits <= 0)
        return MLA_ERR_SHAPE;
    if ((long long)c.max_pages_per_seq * c.page_size > 0x7FFFFFFFLL) return MLA_ERR_SHAPE;
    if (!(c.softmax_scale == c.softmax_scale)) return MLA_ERR_SHAPE;
    if ((long long)c.q_len * c.heads > 1024) return MLA_ERR_UNSUPPORTED;
    if (!io_ok(c.io_dtype)) return MLA_ERR_UNSUPPORTED;
    if (c.cache_dtype != MLA_F32 && c.cache_dtype != MLA_BF16 && c.cache_dtype != MLA_FP8_E4M3)
        return MLA_ERR_UNSUPPORTED;
    if (c.cache_dtype == MLA_F32 && c.io_dtype != MLA_F32) return MLA_ERR_UNSUPPORTED;
    if (c.cache_dtype == MLA_FP8_E4M3 && !c.kv_scale) return MLA_ERR_NULL;
    if (c.cache_dtype != MLA_FP8_E4M3 && c.kv_scale) return MLA_ERR_SHAPE;
    if (c.d_c > 512 || c.d_c % 8 || c.d_rope > 64 || c.d_rope % 8) return MLA_ERR_UNSUPPORTED;
    if (c.B > 65535 || c.num_splits > 16383) return MLA_ERR_UNSUPPORTED;
    if (c.flags & MLA_FLAG_BALANCED) {
        // only the matrix-core kernel has this partition; grid size; page counts are summed in 32 bits
        if (!uses_mfma(c)) return MLA_ERR_UNSUPPORTED;
        const int S = effective_splits(c.B, c.num_splits);
        if ((long long)c.B * S > 0x3FFFFF || (long long)c.B * c.max_pages_per_seq > 0x7FFFFFFFLL)
            return MLA_ERR_UNSUPPORTED;
    }
    return MLA_OK;
}

// launches of a validated call; `workspace` is large enough and 256-byte aligned
int decode_launch(const DecodeCall& c, void* workspace)
{
    const bool skip_merge = (c.flags & MLA_FLAG_SKIP_MERGE) != 0;
    const int B = c.B, H = c.q_len * c.heads;   // query rows per sequence
    hipStream_t stream = static_cast<hipStream_t>(c.hip_stream);
    DecodeParams p;
    p.q_abs = c.q_abs; p.q_rope = c.q_rope; p.kv = c.kv_cache; p.kv_scale = c.kv_scale;
    p.page_table = c.page_table; p.seq_lens = c.seq_lens;
    p.o_part = static_cast<float*>(workspace);
    const int S = effective_splits(B, c.num_splits);
    const WsLayout wl = ws_layout(B, H, c.d_c, S);
    p.lse_part = reinterpret_cast<float*>(static_cast<char*>(workspace) + wl.lse_off);
    p.plan = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + wl.plan_off);
    p.B = B; p.H = H; p.d_c = c.d_c; p.d_rope = c.d_rope; p.page_size = c.page_size;
    p.num_pages = c.num_pages; p.max_pages = c.max_pages_per_seq; p.num_splits = S;
    p.chunk_pages = (c.max_pages_per_seq + S - 1) / S;
    p.q_len = c.q_len; p.heads = c.heads;
    p.q_inner = 1; p.o_final = nullptr; p.lse_final = nullptr;
    p.scale = c.softmax_scale;

    const bool balanced = (c.flags & MLA_FLAG_BALANCED) != 0;
    const bool mfma = uses_mfma(c);
    hipError_t e;
    if (mfma && !balanced && decode_mfma_wide_supported(p, c.io_dtype, c.cache_dtype))
        e = launch_decode_mfma_wide(p, stream);
    else if (mfma) e = launch_decode_mfma(p, c.cache_dtype, stream, balanced);
    else      e = launch_decode_portable(p, c.io_dtype, c.cache_dtype, stream);
    if (e != hipSuccess) return MLA_ERR_HIP;
    if (skip_merge) return MLA_OK;

    MergeParams m;
    fill_merge_params(m, workspace, B, H, c.d_c, S, balanced);
    m.o_lat = c.o_lat; m.lse = c.lse;
    e = launch_merge(m, c.io_dtype, stream);
    return e == hipSuccess ? MLA_OK : MLA_ERR_HIP;
}

}  // namespace

// ---- scratch of mla_decode_paged_static: split-KV partials in a device array of the library's own.
// Every GPU the library runs on holds its own copy of the array, at its own address, until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the address that
// goes into kernel arguments is looked up once per device, with that device current.
static constexpr size_t STATIC_SCRATCH_BYTES = (size_t)32 << 20;
static constexpr int MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
static std::mutex scratch_mutex;
static void* scratch_ptr[MAX_DEVICES];   // device address of `scratch` on device i (nullptr: not looked up yet)

static void* static_scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        scratch_ptr[dev] = ptr;
    }
    return scratch_ptr[dev];
}

extern "C" {

const char* mla_status_string(int status)
{
    switch (status) {
        case MLA_OK:              return "MLA_OK";
        case MLA_ERR_NULL:        return "MLA_ERR_NULL: a required pointer is NULL";
        case MLA_ERR_SHAPE:       return "MLA_ERR_SHAPE: a size is non-positive or inconsistent";
        case MLA_ERR_UNSUPPORTED: return "MLA_ERR_UNSUPPORTED: shape or dtype combination not implemented";
        case MLA_ERR_WORKSPACE:   return "MLA_ERR_WORKSPACE: workspace missing, misaligned or too small";
        case MLA_ERR_HIP:         return "MLA_ERR_HIP: a HIP runtime call failed";
        case MLA_ERR_SCRATCH_LIMIT:
            return "MLA_ERR_SCRATCH_LIMIT: the call needs more scratch than the library's static array holds "
                   "(mla_static_scratch_bytes)";
        default:                  return "unknown mla status";
    }
}

const char* mla_version(void) { return "mla-gfx950 0.1"; }

int mla_absorb_q(const void* q_nope, const void* W_UK, void* q_abs, int B, int H, int d_head,
                 int d_c, mla_dtype io_dtype, void* hip_stream)
{
    if (!q_nope || !W_UK || !q_abs) return MLA_ERR_NULL;
    if (B <= 0 || H <= 0 || d_head <= 0 || d_c <= 0) return MLA_ERR_SHAPE;
    if (!io_ok(io_dtype)) return MLA_ERR_UNSUPPORTED;
    if (H > 65535 || (B + 15) / 16 > 65535) return MLA_ERR_UNSUPPORTED;
    hipError_t e = launch_head_gemm(q_nope, W_UK, q_abs, B, H, d_head, d_c, io_dtype,
                                    static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MLA_OK : MLA_ERR_HIP;
}

int mla_out_proj(const void* o_lat, const void* W_UV, void* out, int B, int H, int d_c,
                 int d_head, mla_dtype io_dtype, void* hip_stream)
{
    if (!o_lat || !W_UV || !out) return MLA_ERR_NULL;
    if (B <= 0 || H <= 0 || d_head <= 0 || d_c <= 0) return MLA_ERR_SHAPE;
    if (!io_ok(io_dtype)) return MLA_ERR_UNSUPPORTED;
    if (H > 65535 || (B + 15) / 16 > 65535) return MLA_ERR_UNSUPPORTED;
    hipError_t e = launch_head_gemm(o_lat, W_UV, out, B, H, d_c, d_head, io_dtype,
                                    static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MLA_OK : MLA_ERR_HIP;
}

size_t mla_decode_workspace_bytes(int B, int H, int d_c, int num_splits)
{
    if (B <= 0 || H <= 0 || d_c <= 0 || num_splits <= 0) return 0;
    const int S = effective_splits(B, num_splits);
    return ws_layout(B, H, d_c, S).total;
}

int mla_decode_paged(const void* q_abs, const void* q_rope, const void* kv_cache,
                     const float* kv_scale, const int32_t* page_table, const int32_t* seq_lens,
                     void* o_lat, float* lse, void* workspace, size_t workspace_bytes, int B, int H,
                     int d_c, int d_rope, int page_size, int num_pages, int max_pages_per_seq,
                     int num_splits, float softmax_scale, mla_dtype io_dtype, mla_dtype cache_dtype,
                     unsigned flags, void* hip_stream)
{
    return mla_decode_paged_multi(q_abs, q_rope, kv_cache, kv_scale, page_table, seq_lens, o_lat, lse,
                                  workspace, workspace_bytes, B, 1, H, d_c, d_rope, page_size, num_pages,
                                  max_pages_per_seq, num_splits, softmax_scale, io_dtype, cache_dtype,
                                  flags, hip_stream);
}

int mla_decode_paged_multi(const void* q_abs, const void* q_rope, const void* kv_cache,
                           const float* kv_scale, const int32_t* page_table, const int32_t* seq_lens,
                           void* o_lat, float* lse, void* workspace, size_t workspace_bytes, int B,
                           int q_len, int heads, int d_c, int d_rope, int page_size, int num_pages,
                           int max_pages_per_seq, int num_splits, float softmax_scale,
                           mla_dtype io_dtype, mla_dtype cache_dtype, unsigned flags, void* hip_stream)
{
    const DecodeCall c = {q_abs, q_rope, kv_cache, kv_scale, page_table, seq_lens, o_lat, lse, B, q_len, heads,
                          d_c, d_rope, page_size, num_pages, max_pages_per_seq, num_splits, softmax_scale,
                          io_dtype, cache_dtype, flags, hip_stream};
    const int st = decode_validate(c);
    if (st != MLA_OK) return st;
    const size_t need = mla_decode_workspace_bytes(B, q_len * heads, d_c, num_splits);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return MLA_ERR_WORKSPACE;
    return decode_launch(c, workspace);
}

size_t mla_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int mla_decode_paged_static(const void* q_abs, const void* q_rope, const void* kv_cache,
                            const float* kv_scale, const int32_t* page_table, const int32_t* seq_lens,
                            void* o_lat, float* lse, int B, int H, int d_c, int d_rope, int page_size,
                            int num_pages, int max_pages_per_seq, int num_splits, float softmax_scale,
                            mla_dtype io_dtype, mla_dtype cache_dtype, unsigned flags, void* hip_stream)
{
    if (flags & MLA_FLAG_SKIP_MERGE) return MLA_ERR_UNSUPPORTED;   // the partials would stay in the library's own array
    const DecodeCall c = {q_abs, q_rope, kv_cache, kv_scale, page_table, seq_lens, o_lat, lse, B, 1, H,
                          d_c, d_rope, page_size, num_pages, max_pages_per_seq, num_splits, softmax_scale,
                          io_dtype, cache_dtype, flags, hip_stream};
    const int st = decode_validate(c);
    if (st != MLA_OK) return st;
    if (mla_decode_workspace_bytes(B, H, d_c, num_splits) > STATIC_SCRATCH_BYTES) return MLA_ERR_SCRATCH_LIMIT;
    void* ptr = static_scratch_of_current_device();
    if (!ptr) return MLA_ERR_HIP;
    return decode_launch(c, ptr);
}

int mla_merge_partials(const void* workspace, size_t workspace_bytes, void* o_lat, float* lse,
                       int B, int H, int d_c, int num_splits, mla_dtype io_dtype, unsigned flags,
                       void* hip_stream)
{
    if (!o_lat) return MLA_ERR_NULL;
    if (B <= 0 || H <= 0 || d_c <= 0 || num_splits <= 0) return MLA_ERR_SHAPE;
    if (!io_ok(io_dtype)) return MLA_ERR_UNSUPPORTED;
    if (H > 65535 || B > 65535 || d_c % 4 || d_c > 2048) return MLA_ERR_UNSUPPORTED;
    if (merge_rows_overflow(B, H, d_c)) return MLA_ERR_UNSUPPORTED;
    const size_t need = mla_decode_workspace_bytes(B, H, d_c, num_splits);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return MLA_ERR_WORKSPACE;
    MergeParams m;
    fill_merge_params(m, workspace, B, H, d_c, effective_splits(B, num_splits), (flags & MLA_FLAG_BALANCED) != 0);
    m.o_lat = o_lat; m.lse = lse;
    hipError_t e = launch_merge(m, io_dtype, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MLA_OK : MLA_ERR_HIP;
}

int mla_merge_out_proj(const void* workspace, size_t workspace_bytes, const void* W_UV, void* o_lat,
                       float* lse, void* out, int B, int H, int d_c, int d_head, int num_splits,
                       mla_dtype io_dtype, unsigned flags, void* hip_stream)
{
    return mla_merge_out_proj_multi(workspace, workspace_bytes, W_UV, o_lat, lse, out, B, 1, H, d_c, d_head,
                                    num_splits, io_dtype, flags, hip_stream);
}

int mla_merge_out_proj_multi(const void* workspace, size_t workspace_bytes, const void* W_UV, void* o_lat,
                             float* lse, void* out, int B, int q_len, int heads, int d_c, int d_head,
                             int num_splits, mla_dtype io_dtype, unsigned flags, void* hip_stream)
{
    if (!o_lat || !W_UV || !out) return MLA_ERR_NULL;
    if (B <= 0 || q_len <= 0 || heads <= 0 || d_c <= 0 || d_head <= 0 || num_splits <= 0) return MLA_ERR_SHAPE;
    if (!io_ok(io_dtype)) return MLA_ERR_UNSUPPORTED;
    if ((long long)q_len * heads > 65535 || (long long)B * q_len > 65535 || d_c % 4 || d_c > 2048)
        return MLA_ERR_UNSUPPORTED;
    if (merge_rows_overflow(B, q_len * heads, d_c)) return MLA_ERR_UNSUPPORTED;
    const size_t need = mla_decode_workspace_bytes(B, q_len * heads, d_c, num_splits);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return MLA_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool balanced = (flags & MLA_FLAG_BALANCED) != 0;
    const int S = effective_splits(B, num_splits);
    // The partials of (sequence b, query token i, head h) lie where those of sequence b * q_len + i,
    // head h of a batch of B * q_len one-token sequences would: the merge and the projection see
    // that batch.  Only the balanced partition's plan is per sequence; with it and q_len > 1 the
    // merge runs over the q_len * heads rows of each sequence and the projection follows it.
    MergeParams m;
    fill_merge_params(m, workspace, B, q_len * heads, d_c, S, balanced);
    m.o_lat = o_lat; m.lse = lse;
    if (!(balanced && q_len > 1)) { m.B = B * q_len; m.H = heads; }
    hipError_t e;
    if (m.H == heads && merge_out_proj_supported(m, d_head, io_dtype)) {
        e = launch_merge_out_proj(m, W_UV, out, stream);
    } else {
        e = launch_merge(m, io_dtype, stream);
        if (e == hipSuccess)
            e = launch_head_gemm(o_lat, W_UV, out, B * q_len, heads, d_c, d_head, io_dtype, stream);
    }
    return e == hipSuccess ? MLA_OK : MLA_ERR_HIP;
}

namespace {
struct PrefillWs {
    size_t pool_off, table_off, lens_off, total;
};
PrefillWs prefill_ws(int B, int heads, int d_c, int max_pages)
{
    PrefillWs w;
    w.pool_off = align_up((size_t)heads * 256 * d_c * 2, 256);                                   // after Wcat
    w.table_off = w.pool_off + align_up((size_t)B * heads * max_pages * 64 * 320 * 2, 256);      // after the pool
    w.lens_off = w.table_off + align_up((size_t)B * heads * max_pages * sizeof(int32_t), 256);
    w.total = w.lens_off + align_up((size_t)B * heads * sizeof(int32_t), 256);
    return w;
}
}  // namespace

size_t mla_prefill_workspace_bytes(int B, int heads, int d_c, int max_pages_per_seq)
{
    if (B <= 0 || heads <= 0 || d_c <= 0 || max_pages_per_seq <= 0) return 0;
    return prefill_ws(B, heads, d_c, max_pages_per_seq).total;
}

int mla_prefill_mha(const void* q_nope, const void* q_rope, const void* W_UK, const void* W_UV,
                    const void* kv_cache, const int32_t* page_table, const int32_t* seq_lens, void* out,
                    float* lse, void* workspace, size_t workspace_bytes, int B, int q_len, int heads,
                    int d_head, int d_c, int d_rope, int page_size, int num_pages, int max_pages_per_seq,
                    float softmax_scale, mla_dtype io_dtype, mla_dtype cache_dtype, void* hip_stream)
{
    if (!q_nope || !q_rope || !W_UK || !W_UV || !kv_cache || !page_table || !seq_lens || !out) return MLA_ERR_NULL;
    if (B <= 0 || q_len <= 0 || heads <= 0 || d_head <= 0 || d_c <= 0 || d_rope < 0 || page_size <= 0 ||
        num_pages <= 0 || max_pages_per_seq <= 0)
        return MLA_ERR_SHAPE;
    if ((long long)max_pages_per_seq * page_size > 0x7FFFFFFFLL) return MLA_ERR_SHAPE;
    if (!(softmax_scale == softmax_scale)) return MLA_ERR_SHAPE;
    if (!io_ok(io_dtype)) return MLA_ERR_UNSUPPORTED;
    if (cache_dtype != MLA_F32 && cache_dtype != MLA_BF16 && cache_dtype != MLA_FP8_E4M3) return MLA_ERR_UNSUPPORTED;
    if (!prefill_supported(d_head, d_c, d_rope, page_size, io_dtype, cache_dtype)) return MLA_ERR_UNSUPPORTED;
    const long long pseudo = (long long)B * heads;                     // (sequence, head) pairs
    if (pseudo > 65535 || max_pages_per_seq > 65535 * 16 || pseudo * max_pages_per_seq > 0x7FFFFFFFLL ||
        (pseudo + 7) / 8 * 8 * ((q_len + 63) / 64) > 0x7FFFFFFFLL)
        return MLA_ERR_UNSUPPORTED;
    const PrefillWs wl = prefill_ws(B, heads, d_c, max_pages_per_seq);
    if (!workspace || workspace_bytes < wl.total || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return MLA_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    void* pool2 = ws + wl.pool_off;
    int32_t* table2 = reinterpret_cast<int32_t*>(ws + wl.table_off);
    int32_t* lens2 = reinterpret_cast<int32_t*>(ws + wl.lens_off);
    hipError_t e = launch_prefill_materialise(kv_cache, page_table, seq_lens, W_UK, W_UV, ws, pool2, table2, lens2,
                                              B, heads, d_c, num_pages, max_pages_per_seq, stream);
    if (e != hipSuccess) return MLA_ERR_HIP;
    // the attention: every (sequence, head) pair is a sequence of q_len query rows over its own rows
    DecodeParams p;
    p.q_abs = q_nope; p.q_rope = q_rope; p.kv = pool2; p.kv_scale = nullptr;
    p.page_table = table2; p.seq_lens = lens2;
    p.o_part = nullptr; p.lse_part = nullptr; p.plan = nullptr;
    p.B = (int)pseudo; p.H = q_len; p.d_c = d_head; p.d_rope = d_rope; p.page_size = page_size;
    p.num_pages = (int)(pseudo * max_pages_per_seq); p.max_pages = max_pages_per_seq;
    p.num_splits = 1; p.chunk_pages = max_pages_per_seq;
    p.q_len = q_len; p.heads = 1; p.q_inner = heads; p.o_final = out; p.lse_final = lse;
    p.scale = softmax_scale;
    e = launch_prefill_attention(p, stream);
    return e == hipSuccess ? MLA_OK : MLA_ERR_HIP;
}

size_t mla_append_workspace_bytes(int B, int D, int d_c, int d_rope, mla_dtype io_dtype)
{
    if (B <= 0 || D <= 0 || d_c <= 0 || d_rope < 0 || !io_ok(io_dtype)) return 0;
    const int n = d_c + d_rope;
    return align_up((size_t)B * append_slices(B, D, n, io_dtype) * n * sizeof(float), 256);
}

int mla_cache_append(const void* x, const void* W_DKVR, void* kv_cache, float* kv_scale,
                     const int32_t* page_table, const int32_t* positions, void* workspace,
                     size_t workspace_bytes, int B, int D, int d_c, int d_rope, int page_size,
                     int num_pages, int max_pages_per_seq, float rope_base, mla_dtype io_dtype,
                     mla_dtype cache_dtype, void* hip_stream)
{
    if (!x || !W_DKVR || !kv_cache || !page_table || !positions) return MLA_ERR_NULL;
    if (B <= 0 || D <= 0 || d_c <= 0 || d_rope < 0 || page_size <= 0 || num_pages <= 0 ||
        max_pages_per_seq <= 0 || !(rope_base > 0.f))
        return MLA_ERR_SHAPE;
    if (d_rope % 2) return MLA_ERR_SHAPE;                    // RoPE turns pairs
    if (!io_ok(io_dtype)) return MLA_ERR_UNSUPPORTED;
    if (cache_dtype != MLA_F32 && cache_dtype != MLA_BF16 && cache_dtype != MLA_FP8_E4M3)
        return MLA_ERR_UNSUPPORTED;
    if ((cache_dtype == MLA_FP8_E4M3) != (kv_scale != nullptr)) return MLA_ERR_NULL;
    if (d_c + d_rope > 1024 || B > 65535 * 16) return MLA_ERR_UNSUPPORTED;
    if ((long)max_pages_per_seq * page_size > 0x7FFFFFFFL) return MLA_ERR_SHAPE;
    const size_t need = mla_append_workspace_bytes(B, D, d_c, d_rope, io_dtype);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15))
        return MLA_ERR_WORKSPACE;
    AppendParams p;
    p.x = x; p.W = W_DKVR; p.part = static_cast<float*>(workspace);
    p.kv = kv_cache; p.kv_scale = kv_scale; p.page_table = page_table; p.positions = positions;
    p.B = B; p.D = D; p.d_c = d_c; p.d_rope = d_rope; p.page_size = page_size;
    p.num_pages = num_pages; p.max_pages = max_pages_per_seq;
    p.slices = append_slices(B, D, d_c + d_rope, io_dtype);
    p.rope_base = rope_base;
    if (p.slices > 65535) return MLA_ERR_UNSUPPORTED;
    hipError_t e = launch_cache_append(p, io_dtype, cache_dtype, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MLA_OK : MLA_ERR_HIP;
}

int mla_gather_paged(const void* kv_cache, const int32_t* page_table, const int32_t* seq_lens,
                     void* dense, int B, int max_len, int row_bytes, int page_size, int num_pages,
                     int max_pages_per_seq, void* hip_stream)
{
    if (!kv_cache || !page_table || !seq_lens || !dense) return MLA_ERR_NULL;
    if (B <= 0 || max_len <= 0 || row_bytes <= 0 || page_size <= 0 || num_pages <= 0 ||
        max_pages_per_seq <= 0)
        return MLA_ERR_SHAPE;
    if ((long long)max_pages_per_seq * page_size > 0x7FFFFFFFLL) return MLA_ERR_SHAPE;
    if (row_bytes % 4 || B > 65535) return MLA_ERR_UNSUPPORTED;
    hipError_t e = launch_gather(kv_cache, page_table, seq_lens, dense, B, max_len, row_bytes,
                                 page_size, num_pages, max_pages_per_seq,
                                 static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MLA_OK : MLA_ERR_HIP;
}

int mla_diag_stream_tiles(const void* kv_cache, const int32_t* page_table, const int32_t* seq_lens,
                          int B, int d_c, int num_pages, int max_pages_per_seq, int num_splits,
                          void* hip_stream)
{
    if (!kv_cache || !page_table || !seq_lens) return MLA_ERR_NULL;
    if (B <= 0 || num_pages <= 0 || max_pages_per_seq <= 0 || num_splits <= 0) return MLA_ERR_SHAPE;
    if ((long long)max_pages_per_seq * 64 > 0x7FFFFFFFLL) return MLA_ERR_SHAPE;
    if ((d_c != 256 && d_c != 512) || B > 65535 || num_splits > 65535) return MLA_ERR_UNSUPPORTED;
    DecodeParams p = {};
    p.kv = kv_cache; p.page_table = page_table; p.seq_lens = seq_lens;
    p.B = B; p.H = 32; p.heads = 32; p.q_len = 1; p.q_inner = 1;
    p.d_c = d_c; p.d_rope = 64; p.page_size = 64; p.num_pages = num_pages; p.max_pages = max_pages_per_seq;
    p.num_splits = min(num_splits, max_pages_per_seq);
    p.chunk_pages = (max_pages_per_seq + p.num_splits - 1) / p.num_splits;
    hipError_t e = launch_decode_stream_probe(p, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MLA_OK : MLA_ERR_HIP;
}

}  // extern "C"
