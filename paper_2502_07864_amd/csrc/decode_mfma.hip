// Matrix-core paged decode for a bf16 latent cache (gfx950 / CDNA4).
//
// Second line of the absorbed attention equation (Sec. 3.3 of the paper): all
// H heads score against the ONE shared row k_hat_j = [c_j ; k^R_j] and weight
// the same latent rows c_j, so per 64-token page both contractions are dense:
//     S^T [64 tok x 32 heads] = K [64 x (d_c+64)] . Q^T [(d_c+64) x 32]
//     O^T [d_c x 32 heads]   += V^T [d_c x 64 tok] . P^T [64 x 32]
// with V = the first d_c columns of the very same LDS tile as K.
//
// Work decomposition (one workgroup = 4 wavefronts per (chunk, sequence)):
//   wave = (hg, tg): head group hg (16 heads) x token half tg (32 of the 64
//   rows of each page).  Each wave runs a complete, private online softmax for
//   its 16 heads over its own rows, so the only workgroup barrier per page is
//   the one that hands over the LDS tile; the two token halves are merged once
//   at the end.  The page goes HBM -> LDS once (direct-to-LDS 128-bit loads,
//   double buffered) and is read from LDS by both head groups.
//
// Operand layouts (v_mfma_f32_16x16x32_bf16, lane = 16*g + n):
//   A holds row n, k = 8g..8g+7; B holds column n, k = 8g..8g+7;
//   D holds rows 4g..4g+3 of column n.
// Transposed formulation: S^T puts heads on the D columns, so every lane owns
// ONE head: row max / sum need two cross-lane steps, the rescale factor is a
// per-lane scalar, and the exponentiated scores are already the B operand of
// the second contraction if its k-slots are ordered (4g+i, 16+4g+i).  The A
// operand V^T (token-contiguous per lane) comes from ds_read_b64_tr_b16, which
// transposes 4x16 blocks of 16-bit elements while reading LDS.
//
// LDS layout: row r of the tile occupies bytes [r*ROWB, (r+1)*ROWB); inside a
// row, 16-byte chunk c is stored at chunk position c ^ ((r >> 1) & 7).  With
// ROWB = 1152 or 640 bytes (= 32 banks mod 64) this makes both the row-wise
// 128-bit reads of 16 consecutive rows and the transposing reads conflict free.
#include "mla_internal.h"

namespace mla {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

#define LDS_AS __attribute__((address_space(3)))
#define CONST_AS __attribute__((address_space(4)))

constexpr int MF_THREADS = 256;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

template <int D_C>
__global__ __launch_bounds__(MF_THREADS, 1) void decode_mfma_bf16_kernel(DecodeParams p)
{
    constexpr int ROW = D_C + 64;               // elements per cache row
    constexpr int ROWB = ROW * 2;               // bytes per row
    constexpr int CPR = ROWB / 16;              // 16-byte chunks per row (72 / 40)
    constexpr int TILE_B = 64 * ROWB;           // bytes per page
    constexpr int NLOAD = TILE_B / (MF_THREADS * 16);  // 16-byte loads per thread per page
    constexpr int NKS = ROW / 32;               // k-steps of the score contraction
    constexpr int NCT = D_C / 16;               // column tiles of the value contraction
    static_assert(TILE_B % (MF_THREADS * 16) == 0, "page must split evenly over the loads");
    static_assert(CPR % 8 == 0, "chunk swizzle needs rows of whole 128-byte groups");

    __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * TILE_B];
    LDS_AS unsigned char* lds = (LDS_AS unsigned char*)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hg = wave & 1, tg = wave >> 1;
    const int n = lane & 15, g = lane >> 4;
    const int split = blockIdx.x, b = blockIdx.y;

    // Read-only tables go through the scalar cache: scalar loads do not count against the
    // vector-memory counter, so looking up a page id never waits on an in-flight page prefetch.
    const CONST_AS int32_t* seq_lens_c = (const CONST_AS int32_t*)p.seq_lens;
    const CONST_AS int32_t* ptab = (const CONST_AS int32_t*)(p.page_table + (size_t)b * p.max_pages);
    int L = seq_lens_c[b];
    L = max(0, min(L, p.max_pages * 64));
    const int n_pages = (L + 63) >> 6;
    const int pg0 = split * p.chunk_pages;
    const int pg1 = min(pg0 + p.chunk_pages, n_pages);
    const size_t part = ((size_t)b * p.num_splits + split) * p.H;
    if (pg0 >= pg1) {  // empty chunk: weight zero in the merge, partial output never read
        if (tid < p.H) p.lse_part[part + tid] = -INFINITY;
        return;
    }

    // ---- this wave's 16 query rows as B operands, resident for the whole chunk
    const int head = hg * 16 + n;
    bf16x8 qreg[NKS];
    {
        const uint16_t* qa = static_cast<const uint16_t*>(p.q_abs) + ((size_t)b * p.H + head) * D_C;
        const uint16_t* qr = static_cast<const uint16_t*>(p.q_rope) + ((size_t)b * p.H + head) * 64;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (head < p.H) {
                const uint16_t* src = ks < D_C / 32 ? qa + ks * 32 + g * 8 : qr + (ks - D_C / 32) * 32 + g * 8;
                v = *reinterpret_cast<const uint4*>(src);
            }
            qreg[ks] = __builtin_bit_cast(bf16x8, v);
        }
    }

    // ---- page staging: HBM -> registers (128-bit loads, issued one page ahead) -> LDS.
    // Load k of wave w covers LDS chunks [(4k+w)*64, +64) (contiguous per wave: conflict-free
    // 128-bit LDS stores); LDS chunk P = row r, position pc holds the row's chunk pc ^ ((r>>1)&7),
    // so a wave still reads whole 128-byte lines from HBM.
    uint32_t goff[NLOAD];   // byte offset of this thread's chunk inside a page
    uint32_t grow[NLOAD];   // its row, for the ragged last page
#pragma unroll
    for (int k = 0; k < NLOAD; ++k) {
        int P = (k * 4 + wave) * 64 + lane;
        int r = P / CPR, pc = P % CPR;
        goff[k] = (uint32_t)(r * ROWB + ((pc ^ ((r >> 1) & 7)) << 4));
        grow[k] = (uint32_t)r;
    }
    const uint32_t st_off = (uint32_t)(wave * 1024 + lane * 16);  // + k*4096: where load k lands in a tile

    const unsigned char* kv = static_cast<const unsigned char*>(p.kv);
    u32x4 stg[NLOAD];

    // rows of page pg that belong to the sequence (0 if its page id is outside the pool)
    auto rows_valid = [&](int pg) {
        int page = ptab[pg];
        return (page >= 0 && page < p.num_pages) ? min(64, L - pg * 64) : 0;
    };
    // Rows past the end of the sequence are never fetched: they become zeros in LDS, so
    // whatever those slots hold (NaN included) cannot reach the accumulators.
    auto fetch_tile = [&](int pg) {
        const int nv = rows_valid(pg);
        const unsigned char* src = kv + (size_t)(nv > 0 ? ptab[pg] : 0) * TILE_B;
        if (nv == 64) {  // whole page (the common case): no per-lane predicate
#pragma unroll
            for (int k = 0; k < NLOAD; ++k) stg[k] = *reinterpret_cast<const u32x4*>(src + goff[k]);
        } else {
#pragma unroll
            for (int k = 0; k < NLOAD; ++k) {
                u32x4 v = (u32x4){0u, 0u, 0u, 0u};
                if ((int)grow[k] < nv) v = *reinterpret_cast<const u32x4*>(src + goff[k]);
                stg[k] = v;
            }
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int k = 0; k < NLOAD; ++k)
            *(LDS_AS u32x4*)(lds + buf * TILE_B + k * 4096 + st_off) = stg[k];
    };

    // ---- running softmax state: this lane's head = column n of the D tiles
    float m_run = -INFINITY;   // running max of scaled scores, in log2 units
    float l_run = 0.f;         // this lane's share of the running sum (its 8 rows per page)
    f32x4 oacc[NCT];
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) oacc[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const float sc = p.scale * LOG2E;
    // LDS byte offsets that do not depend on the page.  A swizzled chunk index splits into a
    // per-lane part (low 3 bits, xor-ed with the row key) and a compile-time part (high bits).
    // score A operand: row 32tg + n (+16), chunk 4ks + g
    const uint32_t a_row = (uint32_t)((tg * 32 + n) * ROWB);
    const uint32_t a_key = (uint32_t)(n >> 1);
    uint32_t a_base[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) a_base[e] = a_row + ((((uint32_t)(4 * e + g)) ^ a_key) << 4);
    // value A operand (transposing read): the lane supplies row 32tg + 4g + (n>>2) (+16),
    // 8 bytes at element column 16ct + 4(n&3), i.e. chunk 2ct + ((n&3)>>1), half (n&1)
    const uint32_t v_row = (uint32_t)((tg * 32 + g * 4 + (n >> 2)) * ROWB);
    const uint32_t v_key = (uint32_t)((2 * g + (n >> 3)) & 7);
    uint32_t v_base[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
        v_base[e] = v_row + ((((uint32_t)(2 * e) + (uint32_t)((n & 3) >> 1)) ^ v_key) << 4) + (uint32_t)((n & 1) * 8);

    fetch_tile(pg0);
    store_tile(0);
    if (pg0 + 1 < pg1) fetch_tile(pg0 + 1);

    for (int pg = pg0; pg < pg1; ++pg) {
        const int buf = (pg - pg0) & 1;
        // the tile of this page is complete in LDS, and every wave has finished reading the
        // other buffer (which receives the next page at the end of this iteration)
        __syncthreads();
        const int n_valid = rows_valid(pg);
        LDS_AS unsigned char* tile = lds + buf * TILE_B;

        // ---- S^T = K . Q^T for this wave's 32 rows x 16 heads
        f32x4 sacc[2] = {(f32x4){0.f, 0.f, 0.f, 0.f}, (f32x4){0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            LDS_AS unsigned char* ap = tile + a_base[ks & 1] + (ks >> 1) * 128;
            bf16x8 a0 = *(LDS_AS bf16x8*)(ap);
            bf16x8 a1 = *(LDS_AS bf16x8*)(ap + 16 * ROWB);
            sacc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qreg[ks], sacc[0], 0, 0, 0);
            sacc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qreg[ks], sacc[1], 0, 0, 0);
        }

        // ---- online softmax for head n over rows {32tg + 16mt + 4g + i}
        float x[8];
        float tmax = -INFINITY;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int tok = tg * 32 + mt * 16 + g * 4 + i;
                float v = tok < n_valid ? sacc[mt][i] * sc : -INFINITY;
                x[mt * 4 + i] = v;
                tmax = fmaxf(tmax, v);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = fast_exp2(m_run - m_use);
        uint32_t pw[4];
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t w = pack_bf16x2(fast_exp2(x[2 * i] - m_use), fast_exp2(x[2 * i + 1] - m_use));
            pw[i] = w;
            psum += bf16_bits_to_f32(w & 0xFFFFu) + bf16_bits_to_f32(w >> 16);  // sum what is multiplied
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        const bf16x8 pb = __builtin_bit_cast(bf16x8, (u32x4){pw[0], pw[1], pw[2], pw[3]});

        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) oacc[ct] *= alpha;
        }

        // ---- O^T += V^T . P^T
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            LDS_AS unsigned char* vp = tile + v_base[ct & 3] + (ct >> 2) * 128;
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(vp));
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(vp + 16 * ROWB));
            s16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            oacc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), pb, oacc[ct], 0, 0, 0);
        }

        // ---- hand the prefetched page to the other buffer, start fetching the one after it
        if (pg + 1 < pg1) {
            store_tile(buf ^ 1);
            if (pg + 2 < pg1) fetch_tile(pg + 2);
        }
    }

    // ---- merge the two token halves of each head group, normalise, write the partial
    float l_w = l_run + __shfl_xor(l_run, 16);
    l_w += __shfl_xor(l_w, 32);
    __syncthreads();  // tiles no longer needed: reuse LDS as exchange space
    constexpr int XCH = NCT * 1024 + 512;  // per head group: O tiles + m + l
    LDS_AS unsigned char* xch = lds + hg * XCH;
    if (tg == 1) {
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) *(LDS_AS f32x4*)(xch + (ct * 64 + lane) * 16) = oacc[ct];
        *(LDS_AS float*)(xch + NCT * 1024 + lane * 4) = m_run;
        *(LDS_AS float*)(xch + NCT * 1024 + 256 + lane * 4) = l_w;
    }
    __syncthreads();
    if (tg == 0) {
        const float m1 = *(LDS_AS float*)(xch + NCT * 1024 + lane * 4);
        const float l1 = *(LDS_AS float*)(xch + NCT * 1024 + 256 + lane * 4);
        const float m_all = fmaxf(m_run, m1);
        const float m_use = m_all == -INFINITY ? 0.f : m_all;
        const float w0 = fast_exp2(m_run - m_use), w1 = fast_exp2(m1 - m_use);
        const float lt = l_w * w0 + l1 * w1;
        const float inv = lt > 0.f ? 1.f / lt : 0.f;
        if (head < p.H) {
            float* dst = p.o_part + (part + head) * D_C + g * 4;
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                f32x4 o1 = *(LDS_AS f32x4*)(xch + (ct * 64 + lane) * 16);
                f32x4 o = (oacc[ct] * w0 + o1 * w1) * inv;
                *reinterpret_cast<f32x4*>(dst + ct * 16) = o;
            }
            if (g == 0) p.lse_part[part + head] = lt > 0.f ? (m_all + __builtin_amdgcn_logf(lt)) * LN2 : -INFINITY;
        }
    }
}

}  // namespace

bool decode_mfma_supported(const DecodeParams& p, mla_dtype io, mla_dtype cache)
{
    return io == MLA_BF16 && cache == MLA_BF16 && p.page_size == 64 && p.d_rope == 64 &&
           (p.d_c == 256 || p.d_c == 512) && p.H >= 1 && p.H <= 32;
}

hipError_t launch_decode_mfma(const DecodeParams& p, hipStream_t s)
{
    dim3 grid(p.num_splits, p.B), block(MF_THREADS);
    if (p.d_c == 512)      decode_mfma_bf16_kernel<512><<<grid, block, 0, s>>>(p);
    else if (p.d_c == 256) decode_mfma_bf16_kernel<256><<<grid, block, 0, s>>>(p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace mla
