// Per-head batched projections of the absorbed attention equation (Sec. 3.3):
//   absorb   : q_abs[b,h,:] = q_nope[b,h,:] . W_UK[h]     (K = d_head, N = d_c)
//   out-proj : out[b,h,:]   = o_lat[b,h,:]  . W_UV[h]     (K = d_c,    N = d_head)
// Both are Y[b,h,n] = sum_k X[b,h,k] W[h,k,n]: H independent skinny GEMMs whose
// cost is reading W once.  A workgroup owns NT (64, 32 or 16) output columns of one head
// for up to 16 batch rows; its four wavefronts split k, and inside a wavefront 64 / NT lane
// groups split it further, each lane streaming one column of W (coalesced along n) against
// the batch rows held in LDS; the partial sums are reduced through LDS.  The narrower tiles
// give a small problem (one batch row, 128 output columns) a workgroup per CU.
#include "mla_internal.h"

namespace mla {
namespace {

constexpr int HG_THREADS = 256;
constexpr int HG_BT = 16;     // batch rows per workgroup
constexpr int HG_NT = 64;     // widest tile of output columns per workgroup
constexpr int HG_KC = 512;    // k staged in LDS per pass

template <bool BF16>
__device__ __forceinline__ float ld(const void* p, size_t i)
{
    if (BF16) return bf16_bits_to_f32(static_cast<const uint16_t*>(p)[i]);
    return static_cast<const float*>(p)[i];
}

template <bool BF16, bool Y_F32, int NT>
__global__ __launch_bounds__(HG_THREADS) void head_gemm_kernel(const void* X, const void* W, void* Y,
                                                                int B, int H, int K, int N)
{
    constexpr int KS = 64 / NT;          // k slices inside a wavefront
    constexpr int NSL = 4 * KS;          // k slices in all
    // batch rows of one k adjacent: a 128-bit LDS read fetches four of them (an LDS instruction
    // costs the wavefront ~17 cycles of issue whatever its width), and groups of four rows past
    // the batch are not read at all
    __shared__ __attribute__((aligned(16))) float x_t[HG_KC][HG_BT];
    __shared__ float red_s[NSL][HG_BT][NT];

    const int tid = threadIdx.x, lane = tid & 63, col = lane % NT;
    const int kg = (tid >> 6) * KS + lane / NT;      // this lane's k slice
    const int n = blockIdx.x * NT + col;
    const int h = blockIdx.y;
    const int b0 = blockIdx.z * HG_BT;
    const int nb = min(HG_BT, B - b0);
    const int nb4 = (nb + 3) / 4;      // groups of four batch rows in use

    float acc[HG_BT];
#pragma unroll
    for (int i = 0; i < HG_BT; ++i) acc[i] = 0.f;

    for (int k0 = 0; k0 < K; k0 += HG_KC) {
        const int kc = min(HG_KC, K - k0);
        __syncthreads();
        for (int idx = tid; idx < HG_BT * kc; idx += HG_THREADS) {
            int bb = idx / kc, k = idx % kc;
            x_t[k][bb] = bb < nb ? ld<BF16>(X, ((size_t)(b0 + bb) * H + h) * K + k0 + k) : 0.f;
        }
        __syncthreads();
        if (n < N) {
            const int per = (kc + NSL - 1) / NSL;
            const int kb = kg * per, ke = min(kc, kb + per);
            auto step = [&](int k, float w) {
#pragma unroll
                for (int g4 = 0; g4 < HG_BT / 4; ++g4) {
                    if (g4 < nb4) {
                        const float4 xv = *reinterpret_cast<const float4*>(&x_t[k][g4 * 4]);
                        acc[g4 * 4 + 0] = fmaf(xv.x, w, acc[g4 * 4 + 0]);
                        acc[g4 * 4 + 1] = fmaf(xv.y, w, acc[g4 * 4 + 1]);
                        acc[g4 * 4 + 2] = fmaf(xv.z, w, acc[g4 * 4 + 2]);
                        acc[g4 * 4 + 3] = fmaf(xv.w, w, acc[g4 * 4 + 3]);
                    }
                }
            };
            // eight weight loads in flight per lane: with one at a time the loop runs at the speed
            // of the memory latency (a skinny batch gives the chip few wavefronts to hide it)
            int k = kb;
            for (; k + 8 <= ke; k += 8) {
                float w[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) w[j] = ld<BF16>(W, ((size_t)h * K + k0 + k + j) * N + n);
#pragma unroll
                for (int j = 0; j < 8; ++j) step(k + j, w[j]);
            }
            for (; k < ke; ++k) step(k, ld<BF16>(W, ((size_t)h * K + k0 + k) * N + n));
        }
    }
#pragma unroll
    for (int i = 0; i < HG_BT; ++i) red_s[kg][i][col] = acc[i];
    __syncthreads();
    for (int idx = tid; idx < HG_BT * NT; idx += HG_THREADS) {
        int bb = idx / NT, nn = idx % NT;
        int oc = blockIdx.x * NT + nn;
        if (bb < nb && oc < N) {
            float v = 0.f;
#pragma unroll
            for (int sl = 0; sl < NSL; sl += 4)      // slices of one wavefront group first, as the 64-column tile always did
                v += (red_s[sl][bb][nn] + red_s[sl + 1][bb][nn]) + (red_s[sl + 2][bb][nn] + red_s[sl + 3][bb][nn]);
            size_t o = ((size_t)(b0 + bb) * H + h) * N + oc;
            if (BF16 && !Y_F32) static_cast<uint16_t*>(Y)[o] = (uint16_t)f32_to_bf16_bits(v);
            else                static_cast<float*>(Y)[o] = v;
        }
    }
}

// ---- matrix-core variant (bf16) ---------------------------------------------------------
// One workgroup = one head x NT output columns x up to 64 batch rows (one 16-row tile per
// wavefront).  The whole [K x NT] slab of W[h] is staged in LDS once with coalesced 128-bit
// loads and shared by the four wavefronts.  v_mfma_f32_16x16x32_bf16 wants, per lane, eight
// consecutive k of one column: W is stored k-major, so the B operand is read with the
// transposing LDS load (two 4-row reads per k-step); the A operand (8 consecutive k of one
// batch row) comes straight from global memory, X being tiny.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
#define LDS_AS __attribute__((address_space(3)))

constexpr int HM_LDS_BYTES = 40 * 1024;

template <int NT, bool Y_F32>
__global__ __launch_bounds__(256) void head_gemm_mfma_kernel(const uint16_t* X, const uint16_t* W, void* Y,
                                                             int B, int H, int K, int N)
{
    constexpr int RS = NT * 2 + 16;          // LDS row stride in bytes (padded: rows shift banks)
    constexpr int CPR = NT / 8;              // 16-byte chunks per slab row
    __shared__ __attribute__((aligned(16))) unsigned char smem[HM_LDS_BYTES];
    LDS_AS unsigned char* lds = (LDS_AS unsigned char*)smem;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, g = lane >> 4;
    // consecutive workgroup ids go to different XCDs: keep the column tiles of one head on
    // one XCD (ids that differ by a multiple of H) so they share its L2 lines of W[h]
    const int h = blockIdx.x % H;
    const int n0 = (blockIdx.x / H) * NT;
    const int brow = (blockIdx.y * 4 + wave) * 16 + n;    // batch row of this lane's A operand

    // A operands of every k-step (K <= 512), requested before the slab so both are in flight
    const bool active = (blockIdx.y * 4 + wave) * 16 < B;
    const bool live = brow < B;
    const uint16_t* xrow = X + ((size_t)min(brow, B - 1) * H + h) * K + g * 8;
    const int nks = K / 32;
    u32x4 areg[16];
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
        areg[ks] = (u32x4){0u, 0u, 0u, 0u};
        if (active && live && ks < nks) areg[ks] = *reinterpret_cast<const u32x4*>(xrow + ks * 32);
    }

    // stage W[h][0:K][n0:n0+NT]
    const uint16_t* Wh = W + ((size_t)h * K) * N + n0;
    for (int c = tid; c < K * CPR; c += 256) {
        int r = c / CPR, cc = c % CPR;
        u32x4 v = *reinterpret_cast<const u32x4*>(Wh + (size_t)r * N + cc * 8);
        *(LDS_AS u32x4*)(lds + r * RS + cc * 16) = v;
    }
    __syncthreads();
    if (!active) return;

    f32x4 acc[NT / 16];
#pragma unroll
    for (int j = 0; j < NT / 16; ++j) acc[j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // transposing read: the lane supplies row 8g + (n>>2) (+4), 8 bytes at column 4(n&3)
    const uint32_t tr_off = (uint32_t)((g * 8 + (n >> 2)) * RS + (n & 3) * 8);
#pragma unroll
    for (int ks = 0; ks < 16; ++ks) {
        if (ks < nks) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, areg[ks]);
#pragma unroll
            for (int j = 0; j < NT / 16; ++j) {
                LDS_AS unsigned char* bp = lds + ks * 32 * RS + tr_off + j * 32;
                s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(bp));
                s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4*)(bp + 4 * RS));
                s16x8 bb = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, bb), acc[j], 0, 0, 0);
            }
        }
    }
    // D: lane holds rows 4g..4g+3 (batch) of column n
#pragma unroll
    for (int j = 0; j < NT / 16; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int bb = (blockIdx.y * 4 + wave) * 16 + g * 4 + i;
            if (bb < B) {
                const size_t o = ((size_t)bb * H + h) * N + n0 + j * 16 + n;
                if (Y_F32) static_cast<float*>(Y)[o] = acc[j][i];
                else       static_cast<uint16_t*>(Y)[o] = (uint16_t)f32_to_bf16_bits(acc[j][i]);
            }
        }
}

template <int NT>
bool try_launch_mfma(const void* X, const void* W, void* Y, int B, int H, int K, int N, bool y_f32,
                     hipStream_t s, hipError_t* err)
{
    if (N % NT || K % 32 || K > 512 || (size_t)K * (NT * 2 + 16) > (size_t)HM_LDS_BYTES) return false;
    dim3 grid(H * (N / NT), (B + 63) / 64), block(256);
    const uint16_t* x = static_cast<const uint16_t*>(X);
    const uint16_t* w = static_cast<const uint16_t*>(W);
    if (y_f32) head_gemm_mfma_kernel<NT, true><<<grid, block, 0, s>>>(x, w, Y, B, H, K, N);
    else       head_gemm_mfma_kernel<NT, false><<<grid, block, 0, s>>>(x, w, Y, B, H, K, N);
    *err = hipGetLastError();
    return true;
}

}  // namespace

hipError_t launch_head_gemm(const void* X, const void* W, void* Y, int B, int H, int K, int N,
                            mla_dtype io, hipStream_t s, bool y_f32)
{
    if (io == MLA_BF16 && (size_t)H * (N / 16 + 1) < 60000) {
        // widest column tile that still gives the chip a workgroup per CU
        const long by = (B + 63) / 64;
        hipError_t err = hipSuccess;
        if (N % 64 == 0 && (long)H * (N / 64) * by >= 256 && try_launch_mfma<64>(X, W, Y, B, H, K, N, y_f32, s, &err)) return err;
        if (N % 32 == 0 && (long)H * (N / 32) * by >= 256 && try_launch_mfma<32>(X, W, Y, B, H, K, N, y_f32, s, &err)) return err;
        if (try_launch_mfma<16>(X, W, Y, B, H, K, N, y_f32, s, &err)) return err;
        if (try_launch_mfma<32>(X, W, Y, B, H, K, N, y_f32, s, &err)) return err;
        if (try_launch_mfma<64>(X, W, Y, B, H, K, N, y_f32, s, &err)) return err;
    }
    // widest column tile that still gives the chip a workgroup per CU
    const long per_col_tile = (long)H * ((B + HG_BT - 1) / HG_BT);
    int nt = HG_NT;
    while (nt > 16 && (long)((N + nt - 1) / nt) * per_col_tile < 256) nt /= 2;
    dim3 grid((N + nt - 1) / nt, H, (B + HG_BT - 1) / HG_BT), block(HG_THREADS);
#define MLA_HEAD_GEMM(NT_)                                                                                          \
    do {                                                                                                            \
        if (io == MLA_BF16 && y_f32) head_gemm_kernel<true, true, NT_><<<grid, block, 0, s>>>(X, W, Y, B, H, K, N); \
        else if (io == MLA_BF16)     head_gemm_kernel<true, false, NT_><<<grid, block, 0, s>>>(X, W, Y, B, H, K, N); \
        else                         head_gemm_kernel<false, false, NT_><<<grid, block, 0, s>>>(X, W, Y, B, H, K, N); \
    } while (0)
    if (nt == 64) MLA_HEAD_GEMM(64);
    else if (nt == 32) MLA_HEAD_GEMM(32);
    else MLA_HEAD_GEMM(16);
#undef MLA_HEAD_GEMM
    return hipGetLastError();
}

}  // namespace mla
