// Portable (scalar-FMA, fp32) kernels: paged decode for every supported dtype
// pair and shape, the split-KV merge, and the page gather test hook.
//
// The decode kernel is the library's reference GPU path: it is the only path
// for fp32 and fp8 caches and for shapes the matrix-core kernel does not
// cover.  One workgroup handles (chunk, sequence, group of 8 heads): a tile of
// 16 cached rows is widened to fp32 in LDS, scored against the 8 query rows,
// folded into a running softmax (second line of the absorbed attention
// equation, Sec. 3.3 of the paper) and accumulated into the latent output.
#include "mla_internal.h"
#include <type_traits>

namespace mla {
namespace {

constexpr int PT_THREADS = 256;
constexpr int PT_HG = 8;        // heads per workgroup
constexpr int PT_TOK = 16;      // cached rows per tile
constexpr int PT_MAX_ROW = 576; // max d_c + d_rope
constexpr int PT_PAD = 4;       // LDS row padding (floats): rows stay 16-byte aligned (128-bit reads) and
                                // consecutive rows start one 16-byte unit apart
constexpr int PT_MAX_COLS = 2;  // d_c <= 512 = 2 * 256 threads

template <typename T> struct Load8;

template <> struct Load8<float> {
    static __device__ __forceinline__ void run(const void* base, size_t elem, const float*, size_t, float* out)
    {
        const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem);
        float4 a = p[0], b = p[1];
        out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
        out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
    }
};

struct bf16_tag {};
template <> struct Load8<bf16_tag> {
    static __device__ __forceinline__ void run(const void* base, size_t elem, const float*, size_t, float* out)
    {
        uint4 v = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + elem);
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i]     = bf16_bits_to_f32(w[i] & 0xFFFFu);
            out[2 * i + 1] = bf16_bits_to_f32(w[i] >> 16);
        }
    }
};

struct fp8_tag {};
template <> struct Load8<fp8_tag> {
    static __device__ __forceinline__ void run(const void* base, size_t elem, const float* scale, size_t row, float* out)
    {
        uint2 v = *reinterpret_cast<const uint2*>(static_cast<const uint8_t*>(base) + elem);
        float s = scale[row];
        uint32_t w[2] = {v.x, v.y};
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = e4m3_to_f32((w[i >> 2] >> (8 * (i & 3))) & 0xFFu) * s;
    }
};

// four consecutive query values (element index a multiple of 4)
template <typename QT> __device__ __forceinline__ float4 load_q4(const void* p, size_t i);
template <> __device__ __forceinline__ float4 load_q4<float>(const void* p, size_t i)
{
    return *reinterpret_cast<const float4*>(static_cast<const float*>(p) + i);
}
template <> __device__ __forceinline__ float4 load_q4<bf16_tag>(const void* p, size_t i)
{
    const uint2 v = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(p) + i);
    return make_float4(bf16_bits_to_f32(v.x & 0xFFFFu), bf16_bits_to_f32(v.x >> 16),
                       bf16_bits_to_f32(v.y & 0xFFFFu), bf16_bits_to_f32(v.y >> 16));
}

template <typename QT, typename CT>
__global__ __launch_bounds__(PT_THREADS) void decode_portable_kernel(DecodeParams p)
{
    __shared__ __attribute__((aligned(16))) float q_s[PT_HG][PT_MAX_ROW + PT_PAD];
    __shared__ __attribute__((aligned(16))) float k_s[PT_TOK][PT_MAX_ROW + PT_PAD];
    __shared__ __attribute__((aligned(16))) float s_s[PT_HG][PT_TOK];
    __shared__ __attribute__((aligned(16))) float p_s[PT_TOK][PT_HG];     // weights, token-major: the 8 heads of a token are adjacent
    __shared__ __attribute__((aligned(16))) float alpha_s[PT_HG];
    __shared__ float m_s[PT_HG], l_s[PT_HG];
    __shared__ int valid_s[PT_TOK];

    const int tid = threadIdx.x;
    const int split = blockIdx.x, b = blockIdx.y, h0 = blockIdx.z * PT_HG;
    const int row = p.d_c + p.d_rope;
    const int nh = min(PT_HG, p.H - h0);

    int L = p.seq_lens[b];
    L = max(0, min(L, p.max_pages * p.page_size));
    const long chunk_tok = (long)p.chunk_pages * p.page_size;
    const long j0l = min((long)L, (long)split * chunk_tok);
    const long j1l = min((long)L, j0l + chunk_tok);
    const int j0 = (int)j0l, j1 = (int)j1l;
    if (j0 >= j1) {  // empty chunk: weight zero in the merge, partial output never read
        if (tid < nh) p.lse_part[part_index(b, h0 + tid, split, p.H, p.num_splits)] = -INFINITY;
        return;
    }

    // query rows [q_abs | q_rope] of this head group -> LDS (fp32), four values per load, all of a
    // thread's loads requested before the first is used (one after the other they would each wait
    // out the memory latency)
    {
        constexpr int PT_NQ = (PT_HG * (PT_MAX_ROW / 4) + PT_THREADS - 1) / PT_THREADS;   // 5
        const int q4_per_row = row / 4;
        float4 qv[PT_NQ];
#pragma unroll
        for (int i = 0; i < PT_NQ; ++i) {
            const int idx = tid + i * PT_THREADS;
            const int h = idx / q4_per_row, k = (idx % q4_per_row) * 4;
            qv[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (h < nh) {
                const size_t bh = (size_t)b * p.H + h0 + h;
                qv[i] = k < p.d_c ? load_q4<QT>(p.q_abs, bh * p.d_c + k)
                                  : load_q4<QT>(p.q_rope, bh * p.d_rope + (k - p.d_c));
            }
        }
#pragma unroll
        for (int i = 0; i < PT_NQ; ++i) {
            const int idx = tid + i * PT_THREADS;
            const int h = idx / q4_per_row, k = (idx % q4_per_row) * 4;
            if (h < PT_HG) *static_cast<float4*>(__builtin_assume_aligned(&q_s[h][k], 16)) = qv[i];
        }
    }
    if (tid < PT_HG) { m_s[tid] = -INFINITY; l_s[tid] = 0.f; }

    float acc[PT_MAX_COLS][PT_HG];
#pragma unroll
    for (int i = 0; i < PT_MAX_COLS; ++i)
#pragma unroll
        for (int h = 0; h < PT_HG; ++h) acc[i][h] = 0.f;

    const int chunks_per_row = row / 8;
    // softmax step (16 threads per head): the head's own upper limit of the sum (several query
    // tokens per sequence)
    const int my_limit = visible_rows(p, L, h0 + min(tid / PT_TOK, PT_HG - 1));
    // ---- tile staging, one tile ahead in registers: a thread owns up to PT_NIT pieces (8 values of one
    // row) of every tile; the next tile's pieces are requested before the current tile is used, so
    // their latency runs under its arithmetic.  Rows outside the chunk or on a bad page are zero.
    constexpr int PT_NIT = (PT_TOK * (PT_MAX_ROW / 8) + PT_THREADS - 1) / PT_THREADS;   // 5
    int st_t[PT_NIT], st_c[PT_NIT];          // row of the tile and first column of each piece (-1: none)
#pragma unroll
    for (int i = 0; i < PT_NIT; ++i) {
        const int idx = tid + i * PT_THREADS;
        st_t[i] = idx < PT_TOK * chunks_per_row ? idx / chunks_per_row : -1;
        st_c[i] = (idx % chunks_per_row) * 8;
    }
    float st_v[PT_NIT][8];
    bool st_ok[PT_NIT];
    auto fetch = [&](int t0) {
#pragma unroll
        for (int i = 0; i < PT_NIT; ++i) {
#pragma unroll
            for (int e = 0; e < 8; ++e) st_v[i][e] = 0.f;
            const int j = t0 + st_t[i];
            bool ok = st_t[i] >= 0 && j < j1;
            if (ok) {
                const int page = p.page_table[(size_t)b * p.max_pages + j / p.page_size];
                ok = page >= 0 && page < p.num_pages;
                if (ok) {
                    const size_t r = (size_t)page * p.page_size + (j % p.page_size);
                    Load8<CT>::run(p.kv, r * row + st_c[i], p.kv_scale, r, st_v[i]);
                }
            }
            st_ok[i] = ok;
        }
    };
    fetch(j0);
    for (int t0 = j0; t0 < j1; t0 += PT_TOK) {
        __syncthreads();  // previous tile fully consumed (and q_s / m_s written)
#pragma unroll
        for (int i = 0; i < PT_NIT; ++i) {
            if (st_t[i] >= 0) {
                if (st_c[i] == 0) valid_s[st_t[i]] = st_ok[i] ? 1 : 0;
                float4* dst = static_cast<float4*>(__builtin_assume_aligned(&k_s[st_t[i]][st_c[i]], 16));
                dst[0] = make_float4(st_v[i][0], st_v[i][1], st_v[i][2], st_v[i][3]);
                dst[1] = make_float4(st_v[i][4], st_v[i][5], st_v[i][6], st_v[i][7]);
            }
        }
        if (t0 + PT_TOK < j1) fetch(t0 + PT_TOK);
        __syncthreads();
        // ---- scores: (head, token) pair per two threads, each half of the row
        if (tid < PT_HG * PT_TOK * 2) {
            int pair = tid >> 1, half = tid & 1;
            int h = pair / PT_TOK, t = pair % PT_TOK;
            int kb = half * (row / 2), ke = kb + row / 2;
            // 128-bit LDS reads (an LDS instruction costs the wavefront ~17 cycles of issue whatever
            // its width), four partial sums
            float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
#pragma unroll 8
            for (int k = kb; k < ke; k += 4) {
                // (rows are 16-byte aligned and row / 2 is a multiple of 4 values: said out loud, or the
                // compiler falls back to 64-bit reads)
                const float4 qv = *static_cast<const float4*>(__builtin_assume_aligned(&q_s[h][k], 16));
                const float4 kv4 = *static_cast<const float4*>(__builtin_assume_aligned(&k_s[t][k], 16));
                d0 = fmaf(qv.x, kv4.x, d0); d1 = fmaf(qv.y, kv4.y, d1);
                d2 = fmaf(qv.z, kv4.z, d2); d3 = fmaf(qv.w, kv4.w, d3);
            }
            float dot = (d0 + d1) + (d2 + d3);
            dot += __shfl_xor(dot, 1);
            if (half == 0) s_s[h][t] = valid_s[t] ? dot * p.scale : -INFINITY;
        }
        __syncthreads();
        // ---- running softmax: one thread per (head, token) of the tile, the 16 lanes of a head side
        // by side in one wavefront (maximum and sum by lane shuffles)
        if (tid < PT_HG * PT_TOK) {
            const int h = tid / PT_TOK, t = tid % PT_TOK;
            const float sv = t0 + t < my_limit ? s_s[h][t] : -INFINITY;
            float tmax = sv;
#pragma unroll
            for (int o = PT_TOK / 2; o > 0; o >>= 1) tmax = fmaxf(tmax, __shfl_xor(tmax, o));
            const float m_old = m_s[h];
            const float m_new = fmaxf(m_old, tmax);
            const float e = m_new == -INFINITY ? 0.f : expf(sv - m_new);
            p_s[t][h] = e;
            float sum = e;
#pragma unroll
            for (int o = PT_TOK / 2; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
            if (t == 0) {
                const float a = m_new == -INFINITY ? 1.f : expf(m_old - m_new);  // exp(-inf) = 0 on the first tile
                alpha_s[h] = a;
                l_s[h] = l_s[h] * a + sum;
                m_s[h] = m_new;
            }
        }
        __syncthreads();
        // ---- latent values: thread owns columns tid, tid+256
#pragma unroll
        for (int i = 0; i < PT_MAX_COLS; ++i) {
            int c = tid + i * PT_THREADS;
            if (c < p.d_c) {
                static_assert(PT_HG == 8, "two 128-bit reads fetch the weights of a token");
                {
                    const float4 a0 = *reinterpret_cast<const float4*>(&alpha_s[0]);
                    const float4 a1 = *reinterpret_cast<const float4*>(&alpha_s[4]);
                    acc[i][0] *= a0.x; acc[i][1] *= a0.y; acc[i][2] *= a0.z; acc[i][3] *= a0.w;
                    acc[i][4] *= a1.x; acc[i][5] *= a1.y; acc[i][6] *= a1.z; acc[i][7] *= a1.w;
                }
#pragma unroll
                for (int t = 0; t < PT_TOK; ++t) {
                    const float v = k_s[t][c];
                    const float4 w0 = *reinterpret_cast<const float4*>(&p_s[t][0]);
                    const float4 w1 = *reinterpret_cast<const float4*>(&p_s[t][4]);
                    acc[i][0] = fmaf(w0.x, v, acc[i][0]); acc[i][1] = fmaf(w0.y, v, acc[i][1]);
                    acc[i][2] = fmaf(w0.z, v, acc[i][2]); acc[i][3] = fmaf(w0.w, v, acc[i][3]);
                    acc[i][4] = fmaf(w1.x, v, acc[i][4]); acc[i][5] = fmaf(w1.y, v, acc[i][5]);
                    acc[i][6] = fmaf(w1.z, v, acc[i][6]); acc[i][7] = fmaf(w1.w, v, acc[i][7]);
                }
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PT_MAX_COLS; ++i) {
        int c = tid + i * PT_THREADS;
        if (c < p.d_c) {
            for (int h = 0; h < nh; ++h) {
                float l = l_s[h];
                const float val = l > 0.f ? acc[i][h] / l : 0.f;
                const size_t at = part_index(b, h0 + h, split, p.H, p.num_splits) * p.d_c + c;
                if constexpr (std::is_same<QT, bf16_tag>::value) static_cast<uint16_t*>(p.o_part)[at] = (uint16_t)f32_to_bf16_bits(val);
                else                                             static_cast<float*>(p.o_part)[at] = val;
            }
        }
    }
    if (tid < nh) {
        float l = l_s[tid];
        p.lse_part[part_index(b, h0 + tid, split, p.H, p.num_splits)] = l > 0.f ? m_s[tid] + logf(l) : -INFINITY;
    }
}

// ---- split-KV merge: lse = log sum_s e^{lse_s}, o = sum_s e^{lse_s - lse} o_s ----
// General kernel: any number of chunks, any d_c (multiple of 4), both partitions.  One workgroup
// per (head, sequence): the chunk weights are computed once into LDS (up to MG_MAXS chunks; more
// than that are handled MG_MAXS at a time with a running reference), then every thread streams
// its four columns with eight partial rows in flight.
constexpr int MG_MAXS = 1024;

template <bool OUT_BF16>
__global__ __launch_bounds__(128) void merge_kernel(MergeParams p)
{
    __shared__ float w_s[MG_MAXS];
    __shared__ float red_s[2];
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    // chunks of (b, h): uniform partition: S adjacent entries; balanced partition: the slots the
    // plan names, one every H entries ([slot, H] / [slot, H, d_c])
    const bool planned = p.plan != nullptr;
    const int S = planned ? p.plan[2 * b + 1] : p.num_splits;
    const size_t first = planned ? (size_t)p.plan[2 * b] * p.H + h : part_index(b, h, 0, p.H, p.num_splits);
    const size_t step = planned ? (size_t)p.H : 1;
    const float* lp = p.lse_part + first;

    auto block_max = [&](float v) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
        __syncthreads();
        if ((tid & 63) == 0) red_s[tid >> 6] = v;
        __syncthreads();
        return fmaxf(red_s[0], red_s[1]);
    };
    auto block_sum = [&](float v) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        __syncthreads();
        if ((tid & 63) == 0) red_s[tid >> 6] = v;
        __syncthreads();
        return red_s[0] + red_s[1];
    };

    // reference = the maximum over all chunks, normaliser = sum of e^{lse_s - max}
    float m = -INFINITY;
    for (int s = tid; s < S; s += 128) m = fmaxf(m, lp[s * step]);
    m = block_max(m);
    float z = 0.f;
    if (m != -INFINITY)
        for (int s = tid; s < S; s += 128) z += expf(lp[s * step] - m);  // exp(-inf) = 0
    z = block_sum(z);
    const float inv = z > 0.f ? 1.f / z : 0.f;

    float4 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = 0; s0 < S; s0 += MG_MAXS) {
        const int ns = min(MG_MAXS, S - s0);
        __syncthreads();
        for (int s = tid; s < ns; s += 128) {
            const float ls = lp[(s0 + s) * step];
            w_s[s] = ls == -INFINITY ? 0.f : expf(ls - m) * inv;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {             // columns tid*4 + i*512 (d_c <= 2048 per pass)
            const int c = tid * 4 + i * 512;
            if (c >= p.d_c) break;
            const size_t src = (first + (size_t)s0 * step) * p.d_c + c;   // element index into the partial rows
            for (int s = 0; s < ns; s += 8) {
                float4 v[8];
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    v[j] = load_part4<OUT_BF16>(p.o_part, src + (size_t)min(s + j, ns - 1) * step * p.d_c);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    // weight 0 for empty chunks (their rows were never written: discarded by the
                    // select, not multiplied) and past the last chunk
                    const float w = s + j < ns ? w_s[s + j] : 0.f;
                    const bool live = w != 0.f;
                    acc[i].x = fmaf(w, live ? v[j].x : 0.f, acc[i].x); acc[i].y = fmaf(w, live ? v[j].y : 0.f, acc[i].y);
                    acc[i].z = fmaf(w, live ? v[j].z : 0.f, acc[i].z); acc[i].w = fmaf(w, live ? v[j].w : 0.f, acc[i].w);
                }
            }
        }
    }
    const size_t out_base = ((size_t)b * p.H + h) * p.d_c;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid * 4 + i * 512;
        if (c >= p.d_c) break;
        if (OUT_BF16) {
            uint2 o;
            o.x = f32_to_bf16_bits(acc[i].x) | (f32_to_bf16_bits(acc[i].y) << 16);
            o.y = f32_to_bf16_bits(acc[i].z) | (f32_to_bf16_bits(acc[i].w) << 16);
            *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.o_lat) + out_base + c) = o;
        } else {
            *reinterpret_cast<float4*>(static_cast<float*>(p.o_lat) + out_base + c) = acc[i];
        }
    }
    if (p.lse && tid == 0) p.lse[(size_t)b * p.H + h] = z > 0.f ? m + logf(z) : -INFINITY;
}

// Streaming variant for d_c a multiple of 256: one wavefront per (sequence, head, block of 256
// columns).  Lane s owns the log-sum-exp of chunk s; every lane streams one float4 per chunk with
// the loads of up to 16 chunks in flight.  PLAN = false: uniform partition, at most 64 chunks.
// PLAN = true: the chunks the balanced partition's plan names for the sequence, any number of
// them, 64 at a time.
template <bool OUT_BF16, bool PLAN>
__global__ __launch_bounds__(256) void merge_wave_kernel(MergeParams p)
{
    const int lane = threadIdx.x & 63;
    const int blocks_per_row = p.d_c / 256;
    const int total = p.B * p.H * blocks_per_row;
    const int wid = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (wid >= total) return;
    const int cb = wid % blocks_per_row;
    const int bh = wid / blocks_per_row;
    const int b = bh / p.H, h = bh % p.H;
    const ChunkSpan c = PLAN ? planned_span(p.plan[2 * b], p.plan[2 * b + 1], p, h)
                             : ChunkSpan{part_index(b, h, 0, p.H, p.num_splits), 1, p.num_splits};
    const int S = c.S;

    // Start streaming the first chunks' partial rows before their weights are known.  Rows of
    // empty chunks were never written: whatever is read there is discarded by a select, not
    // multiplied by zero.
    constexpr int BATCH = 16;
    const size_t stride = c.step * (size_t)p.d_c;
    const size_t base = c.first * p.d_c + cb * 256 + lane * 4;   // element index
    const float ls0 = span_lse(p.lse_part, c, 0, lane);
    float4 v[BATCH];
    // rows past the last chunk re-read it (weight zero); a sequence without chunks reads its first slot's row
    auto row = [&](int s) { return base + (size_t)max(0, min(s, S - 1)) * stride; };
#pragma unroll
    for (int i = 0; i < BATCH; ++i) v[i] = load_part4<OUT_BF16>(p.o_part, row(i));

    const ChunkWeights cw = PLAN ? span_weights(p.lse_part, c, ls0, lane) : chunk_weights(ls0, S);

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int blk = 0; blk < S; blk += 64) {
        const float ls = blk ? span_lse(p.lse_part, c, blk, lane) : ls0;
        for (int s0 = 0; s0 < min(64, S - blk); s0 += BATCH) {
            if (blk + s0 > 0) {
#pragma unroll
                for (int i = 0; i < BATCH; ++i) v[i] = load_part4<OUT_BF16>(p.o_part, row(blk + s0 + i));
            }
#pragma unroll
            for (int i = 0; i < BATCH; ++i) {
                const float ws = chunk_weight_at(cw, ls, s0 + i);   // 0 at and past S
                const bool live = ws != 0.f;
                acc.x = fmaf(ws, live ? v[i].x : 0.f, acc.x); acc.y = fmaf(ws, live ? v[i].y : 0.f, acc.y);
                acc.z = fmaf(ws, live ? v[i].z : 0.f, acc.z); acc.w = fmaf(ws, live ? v[i].w : 0.f, acc.w);
            }
        }
    }
    const size_t o = (size_t)bh * p.d_c + cb * 256 + lane * 4;
    if (OUT_BF16) {
        uint2 r;
        r.x = f32_to_bf16_bits(acc.x) | (f32_to_bf16_bits(acc.y) << 16);
        r.y = f32_to_bf16_bits(acc.z) | (f32_to_bf16_bits(acc.w) << 16);
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.o_lat) + o) = r;
    } else {
        *reinterpret_cast<float4*>(static_cast<float*>(p.o_lat) + o) = acc;
    }
    if (p.lse && cb == 0 && lane == 0) p.lse[bh] = cw.z > 0.f ? cw.m + logf(cw.z) : -INFINITY;
}

// ---- page gather (byte exact) ---------------------------------------------
__global__ __launch_bounds__(256) void gather_kernel(const uint32_t* kv, const int32_t* page_table,
                                                     const int32_t* seq_lens, uint32_t* dense,
                                                     int max_len, int row_words, int page_size,
                                                     int num_pages, int max_pages)
{
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= max_len) return;
    int L = min(seq_lens[b], max_pages * page_size);
    const uint32_t* src = nullptr;
    if (j < L) {
        int page = page_table[(size_t)b * max_pages + j / page_size];
        if (page >= 0 && page < num_pages)
            src = kv + ((size_t)page * page_size + (j % page_size)) * row_words;
    }
    uint32_t* dst = dense + ((size_t)b * max_len + j) * row_words;
    for (int w = lane; w < row_words; w += 64) dst[w] = src ? src[w] : 0u;
}

}  // namespace

hipError_t launch_decode_portable(const DecodeParams& p, mla_dtype io, mla_dtype cache, hipStream_t s)
{
    dim3 grid(p.num_splits, p.B, (p.H + PT_HG - 1) / PT_HG), block(PT_THREADS);
    if (io == MLA_F32 && cache == MLA_F32)
        decode_portable_kernel<float, float><<<grid, block, 0, s>>>(p);
    else if (io == MLA_F32 && cache == MLA_BF16)
        decode_portable_kernel<float, bf16_tag><<<grid, block, 0, s>>>(p);
    else if (io == MLA_F32 && cache == MLA_FP8_E4M3)
        decode_portable_kernel<float, fp8_tag><<<grid, block, 0, s>>>(p);
    else if (io == MLA_BF16 && cache == MLA_BF16)
        decode_portable_kernel<bf16_tag, bf16_tag><<<grid, block, 0, s>>>(p);
    else if (io == MLA_BF16 && cache == MLA_FP8_E4M3)
        decode_portable_kernel<bf16_tag, fp8_tag><<<grid, block, 0, s>>>(p);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_merge(const MergeParams& p, mla_dtype io, hipStream_t s)
{
    if (p.d_c % 256 == 0 && (p.plan || p.num_splits <= 64)) {
        const int waves = p.B * p.H * (p.d_c / 256);
        dim3 grid((waves + 3) / 4), block(256);
        if (io == MLA_BF16) {
            if (p.plan) merge_wave_kernel<true, true><<<grid, block, 0, s>>>(p);
            else        merge_wave_kernel<true, false><<<grid, block, 0, s>>>(p);
        } else {
            if (p.plan) merge_wave_kernel<false, true><<<grid, block, 0, s>>>(p);
            else        merge_wave_kernel<false, false><<<grid, block, 0, s>>>(p);
        }
        return hipGetLastError();
    }
    dim3 grid(p.H, p.B), block(128);
    if (io == MLA_BF16) merge_kernel<true><<<grid, block, 0, s>>>(p);
    else                merge_kernel<false><<<grid, block, 0, s>>>(p);
    return hipGetLastError();
}

hipError_t launch_gather(const void* kv, const int32_t* page_table, const int32_t* seq_lens,
                         void* dense, int B, int max_len, int row_bytes, int page_size,
                         int num_pages, int max_pages, hipStream_t s)
{
    dim3 grid((max_len + 3) / 4, B), block(256);
    gather_kernel<<<grid, block, 0, s>>>(static_cast<const uint32_t*>(kv), page_table, seq_lens,
                                         static_cast<uint32_t*>(dense), max_len, row_bytes / 4,
                                         page_size, num_pages, max_pages);
    return hipGetLastError();
}

}  // namespace mla
