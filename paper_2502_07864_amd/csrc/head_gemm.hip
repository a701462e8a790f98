// Per-head batched projections of the absorbed attention equation (Sec. 3.3):
//   absorb   : q_abs[b,h,:] = q_nope[b,h,:] . W_UK[h]     (K = d_head, N = d_c)
//   out-proj : out[b,h,:]   = o_lat[b,h,:]  . W_UV[h]     (K = d_c,    N = d_head)
// Both are Y[b,h,n] = sum_k X[b,h,k] W[h,k,n]: H independent skinny GEMMs whose
// cost is reading W once.  A workgroup owns 64 output columns of one head for
// up to 16 batch rows; its four wavefronts split k, each lane streaming one
// column of W (coalesced along n) against the batch rows held in LDS, and the
// four partial sums are reduced through LDS.
#include "mla_internal.h"

namespace mla {
namespace {

constexpr int HG_THREADS = 256;
constexpr int HG_BT = 16;     // batch rows per workgroup
constexpr int HG_NT = 64;     // output columns per workgroup
constexpr int HG_KC = 512;    // k staged in LDS per pass

template <bool BF16>
__device__ __forceinline__ float ld(const void* p, size_t i)
{
    if (BF16) return bf16_bits_to_f32(static_cast<const uint16_t*>(p)[i]);
    return static_cast<const float*>(p)[i];
}

template <bool BF16>
__global__ __launch_bounds__(HG_THREADS) void head_gemm_kernel(const void* X, const void* W, void* Y,
                                                                int B, int H, int K, int N)
{
    __shared__ float x_s[HG_BT][HG_KC];
    __shared__ float red_s[4][HG_BT][HG_NT];

    const int tid = threadIdx.x, lane = tid & 63, kg = tid >> 6;
    const int n = blockIdx.x * HG_NT + lane;
    const int h = blockIdx.y;
    const int b0 = blockIdx.z * HG_BT;
    const int nb = min(HG_BT, B - b0);

    float acc[HG_BT];
#pragma unroll
    for (int i = 0; i < HG_BT; ++i) acc[i] = 0.f;

    for (int k0 = 0; k0 < K; k0 += HG_KC) {
        const int kc = min(HG_KC, K - k0);
        __syncthreads();
        for (int idx = tid; idx < HG_BT * kc; idx += HG_THREADS) {
            int bb = idx / kc, k = idx % kc;
            x_s[bb][k] = bb < nb ? ld<BF16>(X, ((size_t)(b0 + bb) * H + h) * K + k0 + k) : 0.f;
        }
        __syncthreads();
        if (n < N) {
            const int per = (kc + 3) / 4;
            const int kb = kg * per, ke = min(kc, kb + per);
            for (int k = kb; k < ke; ++k) {
                float w = ld<BF16>(W, ((size_t)h * K + k0 + k) * N + n);
#pragma unroll
                for (int i = 0; i < HG_BT; ++i) acc[i] = fmaf(x_s[i][k], w, acc[i]);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < HG_BT; ++i) red_s[kg][i][lane] = acc[i];
    __syncthreads();
    for (int idx = tid; idx < HG_BT * HG_NT; idx += HG_THREADS) {
        int bb = idx / HG_NT, nn = idx % HG_NT;
        int col = blockIdx.x * HG_NT + nn;
        if (bb < nb && col < N) {
            float v = (red_s[0][bb][nn] + red_s[1][bb][nn]) + (red_s[2][bb][nn] + red_s[3][bb][nn]);
            size_t o = ((size_t)(b0 + bb) * H + h) * N + col;
            if (BF16) static_cast<uint16_t*>(Y)[o] = (uint16_t)f32_to_bf16_bits(v);
            else      static_cast<float*>(Y)[o] = v;
        }
    }
}

}  // namespace

hipError_t launch_head_gemm(const void* X, const void* W, void* Y, int B, int H, int K, int N,
                            mla_dtype io, hipStream_t s)
{
    dim3 grid((N + HG_NT - 1) / HG_NT, H, (B + HG_BT - 1) / HG_BT), block(HG_THREADS);
    if (io == MLA_BF16) head_gemm_kernel<true><<<grid, block, 0, s>>>(X, W, Y, B, H, K, N);
    else                head_gemm_kernel<false><<<grid, block, 0, s>>>(X, W, Y, B, H, K, N);
    return hipGetLastError();
}

}  // namespace mla
