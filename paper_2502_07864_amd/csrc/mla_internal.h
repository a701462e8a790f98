// Internal declarations shared by the library's translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "mla_gfx950.h"

namespace mla {

// Everything a decode kernel needs; passed by value as the kernel argument.
// Several query tokens per sequence (q_len > 1) are handled as more query rows: H counts the rows
// of one sequence, token-major (row = token * heads + head), and the row of query token i sees
// the cached rows below seq_len - (q_len - 1 - i) only (Eq. "mqa": the sum runs up to the query's
// own position).
struct DecodeParams {
    const void* q_abs;          // [B,H,d_c]      io dtype
    const void* q_rope;         // [B,H,d_rope]   io dtype
    const void* kv;             // [num_pages, page_size, d_c+d_rope] cache dtype
    const float* kv_scale;      // [num_pages, page_size] (fp8 cache) or nullptr
    const int32_t* page_table;  // [B, max_pages]
    const int32_t* seq_lens;    // [B]
    void* o_part;               // [B, H, S, d_c]  chunk-normalised partial outputs, stored in the io dtype
                                // (fp32 io: fp32; bf16 io: bf16 -- half the bytes to write and to merge)
    float* lse_part;            // [B, H, S]       natural-log LSE per chunk (-inf = empty)
    int32_t* plan;              // balanced partition only: [B, 2] first partial slot and count per
                                // sequence (the partials are then [slot, H, d_c] / [slot, H])
    int B, H, d_c, d_rope, page_size, num_pages, max_pages, num_splits, chunk_pages;
    int q_len, heads;           // H = q_len * heads
    int q_inner;                // 1; prefill: heads of the model (sequence b stands for (b / q_inner, b % q_inner))
    void* o_final;              // prefill only: [.., d_head] io dtype, rows indexed like the query rows
    float* lse_final;           // prefill only, may be nullptr
    float scale;
};

// cached rows of a sequence of L rows that query row h may see
__host__ __device__ __forceinline__ int visible_rows(const DecodeParams& p, int L, int h)
{
    return L - (p.q_len - 1 - h / p.heads);
}

struct MergeParams {
    const void* o_part;    // partial outputs in the io dtype (see DecodeParams)
    const float* lse_part;
    const int32_t* plan;   // nullptr, or (balanced partition) [B, 2] first slot and count per sequence
    void* o_lat;   // [B,H,d_c] io dtype
    float* lse;    // [B,H] or nullptr
    int B, H, d_c, num_splits;
};

// Index of chunk s of (sequence b, head h) in the partial buffers: all chunks of one (b, h) are
// adjacent, so the merge reads one contiguous block per output row.
__host__ __device__ __forceinline__ size_t part_index(int b, int h, int s, int H, int S)
{
    return ((size_t)b * H + h) * S + s;
}

// ---- small device helpers ------------------------------------------------

// value of v on lane `lane` (wave-uniform index), as a uniform value on every lane
__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Split-KV merge weights of one output row.  Lane s of the wave holds the log-sum-exp of
// chunk s (-inf for s >= S and for empty chunks).  Every lane computes the same reference
// (the maximum) and normaliser by reading the S values lane by lane, 16 at a time with
// compile-time offsets and in index order: no chain of cross-lane shuffles, and a result that
// does not depend on which wave computes it.  lse = m + log z (z = 0: every chunk empty).
struct ChunkWeights {
    float m, z;      // maximum and sum_s e^{lse_s - m}
    float ref, inv;  // m (0 if every chunk is empty) and 1/z (0 if z = 0)
};

__device__ __forceinline__ ChunkWeights chunk_weights(float ls, int S)
{
    ChunkWeights cw;
    cw.m = -INFINITY;
    for (int s0 = 0; s0 < S; s0 += 16) {
#pragma unroll
        for (int i = 0; i < 16; ++i) cw.m = fmaxf(cw.m, lane_value(ls, s0 + i));
    }
    cw.ref = cw.m == -INFINITY ? 0.f : cw.m;
    cw.z = 0.f;
    for (int s0 = 0; s0 < S; s0 += 16) {
#pragma unroll
        for (int i = 0; i < 16; ++i) cw.z += __expf(lane_value(ls, s0 + i) - cw.ref);   // e^{-inf} = 0
    }
    cw.inv = cw.z > 0.f ? 1.f / cw.z : 0.f;
    return cw;
}

// weight e^{lse_s - lse} of chunk s (s < 64; 0 for s >= S and for empty chunks), on every lane
__device__ __forceinline__ float chunk_weight_at(const ChunkWeights& cw, float ls, int s)
{
    return __expf(lane_value(ls, s) - cw.ref) * cw.inv;
}

// Where the S partials of one (sequence, query row) lie: chunk s has its log-sum-exp at
// lse_part[first + s * step] and its row at element (first + s * step) * d_c of o_part.  Uniform
// partition: S adjacent entries; balanced partition: the slots the plan names, one every H entries
// ([slot, H] / [slot, H, d_c]), S of them (0 for an empty sequence; any number otherwise).
struct ChunkSpan {
    size_t first, step;
    int S;
};

// (a plan entry that does not fit the workspace's slots -- a workspace no balanced decode call has
// written -- reads as an empty sequence)
__device__ __forceinline__ ChunkSpan planned_span(int first_slot, int count, const MergeParams& p, int h)
{
    const long long slots = (long long)p.B * (p.num_splits + 1);
    if (first_slot < 0 || count < 0 || (long long)first_slot + count > slots) { first_slot = 0; count = 0; }
    return ChunkSpan{(size_t)first_slot * p.H + h, (size_t)p.H, count};
}

// log-sum-exp of chunk blk + lane of a span (-inf at and past S), blk a multiple of 64
__device__ __forceinline__ float span_lse(const float* lse_part, const ChunkSpan& c, int blk, int lane)
{
    const int s = blk + lane;
    return s < c.S ? lse_part[c.first + (size_t)s * c.step] : -INFINITY;
}

// chunk_weights for a span of any length: the same operations in the same order over blocks of 64
// chunks (ls0 = span_lse of block 0), so that up to 64 chunks the result is chunk_weights' bit for bit
__device__ __forceinline__ ChunkWeights span_weights(const float* lse_part, const ChunkSpan& c, float ls0, int lane)
{
    ChunkWeights cw;
    cw.m = -INFINITY;
    for (int blk = 0; blk < c.S; blk += 64) {
        const float ls = blk ? span_lse(lse_part, c, blk, lane) : ls0;
        for (int s0 = 0; s0 < min(64, c.S - blk); s0 += 16) {
#pragma unroll
            for (int i = 0; i < 16; ++i) cw.m = fmaxf(cw.m, lane_value(ls, s0 + i));
        }
    }
    cw.ref = cw.m == -INFINITY ? 0.f : cw.m;
    cw.z = 0.f;
    for (int blk = 0; blk < c.S; blk += 64) {
        const float ls = blk ? span_lse(lse_part, c, blk, lane) : ls0;
        for (int s0 = 0; s0 < min(64, c.S - blk); s0 += 16) {
#pragma unroll
            for (int i = 0; i < 16; ++i) cw.z += __expf(lane_value(ls, s0 + i) - cw.ref);
        }
    }
    cw.inv = cw.z > 0.f ? 1.f / cw.z : 0.f;
    return cw;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16)
{
    return __uint_as_float(bits16 << 16);
}

// Four consecutive values of a partial output row (element index a multiple of 4); the rows are
// stored in the io dtype: BF16 = true reads 8 bytes, false 16.
template <bool BF16> __device__ __forceinline__ float4 load_part4(const void* base, size_t elem)
{
    if constexpr (BF16) {
        const uint2 v = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(base) + elem);
        return make_float4(bf16_bits_to_f32(v.x & 0xFFFFu), __uint_as_float(v.x & 0xFFFF0000u),
                           bf16_bits_to_f32(v.y & 0xFFFFu), __uint_as_float(v.y & 0xFFFF0000u));
    } else {
        return *reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem);
    }
}

// fp32 -> bf16 bits, round to nearest even, NaN kept quiet.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// OCP e4m3 code -> fp32 (bias 7, subnormals m*2^-9, S.1111.111 = NaN).
__device__ __forceinline__ float e4m3_to_f32(uint32_t code)
{
    uint32_t sign = (code & 0x80u) << 24;
    uint32_t em = code & 0x7Fu;
    float mag;
    if (em == 0x7Fu)      mag = __uint_as_float(0x7FC00000u);
    else if (em < 8u)     mag = (float)em * 0.001953125f;                 // m * 2^-9
    else                  mag = __uint_as_float((em << 20) + (120u << 23)); // rebias 7 -> 127
    return __uint_as_float(__float_as_uint(mag) | sign);
}

// ---- launchers (each returns hipGetLastError() of its launch) --------------

hipError_t launch_decode_portable(const DecodeParams& p, mla_dtype io, mla_dtype cache, hipStream_t s);
bool       decode_mfma_supported(const DecodeParams& p, mla_dtype io, mla_dtype cache);
hipError_t launch_decode_mfma(const DecodeParams& p, mla_dtype cache, hipStream_t s, bool balanced = false);
// uniform chunks of at most 32 tiles, bf16 caches: the kernel with separate requesting and consuming
// wavefronts (same grid as launch_decode_mfma's)
hipError_t launch_decode_stream(const DecodeParams& p, dim3 grid, hipStream_t s);
// the same kernel under the balanced partition (needs p.plan; launch_decode_mfma's balanced grid)
hipError_t launch_decode_stream_balanced(const DecodeParams& p, dim3 grid, hipStream_t s);
// the same kernel's tile requests, waits and barriers alone (diagnostic: no query rows, arithmetic or output)
hipError_t launch_decode_stream_probe(const DecodeParams& p, hipStream_t s);
// uniform chunks, fp8 caches: wavefronts that turn tiles into softmax weights beside wavefronts that
// contract the tile before with them (same grid as launch_decode_mfma's)
hipError_t launch_decode_stream_fp8(const DecodeParams& p, dim3 grid, hipStream_t s, bool balanced);
bool       decode_mfma_wide_supported(const DecodeParams& p, mla_dtype io, mla_dtype cache);
hipError_t launch_decode_mfma_wide(const DecodeParams& p, hipStream_t s);   // 64 query rows per workgroup
hipError_t launch_prefill_attention(const DecodeParams& p, hipStream_t s);  // causal attention over materialised keys / values
// prefill: materialise [W_UK c ; k_rope | W_UV c] per (sequence, head) into a pool of its own
bool       prefill_supported(int d_head, int d_c, int d_rope, int page_size, mla_dtype io, mla_dtype cache);
hipError_t launch_prefill_materialise(const void* kv, const int32_t* page_table, const int32_t* seq_lens,
                                      const void* W_UK, const void* W_UV, void* Wcat, void* pool2, int32_t* table2,
                                      int32_t* lens2, int B, int heads, int d_c, int num_pages, int max_pages,
                                      hipStream_t s);
hipError_t launch_merge(const MergeParams& p, mla_dtype io, hipStream_t s);
hipError_t launch_gather(const void* kv, const int32_t* page_table, const int32_t* seq_lens,
                         void* dense, int B, int max_len, int row_bytes, int page_size,
                         int num_pages, int max_pages, hipStream_t s);
bool       merge_out_proj_supported(const MergeParams& p, int d_head, mla_dtype io);
hipError_t launch_merge_out_proj(const MergeParams& p, const void* W_UV, void* out, hipStream_t s);
// Y[b,h,n] = sum_k X[b,h,k] * W[h,k,n]
// (y_f32: Y is fp32 whatever the io dtype)
hipError_t launch_head_gemm(const void* X, const void* W, void* Y, int B, int H, int K, int N,
                            mla_dtype io, hipStream_t s, bool y_f32 = false);

// Cache append.  The projection x . W is cut into `slices` slices of the model dimension (fp32
// partial rows [B, slices, n] in the workspace); the finishing kernel adds them, rotates the
// rope part and stores one row per sequence.
struct AppendParams {
    const void* x;              // [B, D] io dtype
    const void* W;              // [D, n] io dtype, n = d_c + d_rope
    float* part;                // [B, slices, n] fp32 (workspace)
    void* kv;                   // cache pool
    float* kv_scale;            // [num_pages, page_size] (fp8 cache) or nullptr
    const int32_t* page_table;  // [B, max_pages]
    const int32_t* positions;   // [B]
    int B, D, d_c, d_rope, page_size, num_pages, max_pages, slices;
    float rope_base;
};
int        append_slices(int B, int D, int n, mla_dtype io);
hipError_t launch_cache_append(const AppendParams& p, mla_dtype io, mla_dtype cache, hipStream_t s);

}  // namespace mla
