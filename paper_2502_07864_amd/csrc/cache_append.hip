// Cache append: the row the decode reads, produced for one new token per sequence
// (Sec. 3.3, MLA equations, left column):
//     c^{KV}_t = W^{DKV} x_t        k^R_t = RoPE(W^{KR} x_t, t)        row = [c^{KV}_t ; k^R_t]
// with RoPE as in Sec. 3.1, Eq. 1 (consecutive pairs (real, imaginary), pair i turned by
// t * base^(-2i/d^R)).  The two projections are one skinny GEMM x . [W^{DKV} ; W^{KR}]^T whose cost
// is reading the weights once: it runs on the per-head GEMM kernels with the model dimension cut
// into slices that play the part of the heads (fp32 partial rows), so that enough workgroups
// stream the weights.  One small kernel per sequence then adds the slices in a fixed order,
// rotates the rope part (angles in fp64: positions reach 10^5 radians), rounds the row to the
// cache dtype (fp8: one scale per token, absmax / 448, codes by round-to-nearest-even,
// saturating) and writes it through the page table.
#include "mla_internal.h"

namespace mla {
namespace {

constexpr int AP_MAXN = 1024;   // longest cache row the finishing kernel holds in LDS

// fp32 -> OCP e4m3 code: nearest, ties to even, magnitudes above 448 saturate, NaN -> S.1111.111
__device__ __forceinline__ uint32_t f32_to_e4m3_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    const uint32_t sign = (u >> 24) & 0x80u;
    u &= 0x7FFFFFFFu;
    if (u > 0x7F800000u) return sign | 0x7Fu;
    const float a = __uint_as_float(u);
    if (a >= 448.f) return sign | 0x7Eu;
    if (a < 0.015625f) return sign | (uint32_t)rintf(a * 512.f);   // subnormals m * 2^-9; 8 is 2^-6
    // normal: keep 3 mantissa bits, round to nearest even (a carry moves into the exponent)
    u += 0x7FFFFu + ((u >> 20) & 1u);
    return sign | ((u >> 20) - (120u << 3));
}

template <int CACHE>   // mla_dtype of the cache
__global__ __launch_bounds__(256) void append_finish_kernel(AppendParams p)
{
    __shared__ float row[AP_MAXN];
    __shared__ float wmax[4];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int n = p.d_c + p.d_rope;
    const int pos = p.positions[b];   // requested now, needed after the sums

    // Slices added in index order.  The loads do not depend on the position or the page, so they
    // go out first: sixteen slices of each of this thread's columns at a time (slices past the
    // last re-read it and are not added; columns past the row likewise).
    {
        constexpr int NC = AP_MAXN / 256;
        float acc[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[c] = 0.f;
        const float* base = p.part + (size_t)b * p.slices * n;
        for (int s0 = 0; s0 < p.slices; s0 += 16) {
            float v[NC][16];
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    v[c][i] = base[(size_t)min(s0 + i, p.slices - 1) * n + min(tid + c * 256, n - 1)];
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[c] += s0 + i < p.slices ? v[c][i] : 0.f;
        }
#pragma unroll
        for (int c = 0; c < NC; ++c)
            if (tid + c * 256 < n) row[tid + c * 256] = acc[c];
    }
    if (pos < 0 || pos >= p.max_pages * p.page_size) return;          // outside the table
    const int page = p.page_table[(size_t)b * p.max_pages + pos / p.page_size];
    if (page < 0 || page >= p.num_pages) return;                      // outside the pool
    const size_t r = (size_t)page * p.page_size + (size_t)(pos % p.page_size);
    __syncthreads();
    if (tid < p.d_rope / 2) {
        const double theta = pow((double)p.rope_base, -2.0 * (double)tid / (double)p.d_rope);
        double sn, cs;
        sincos((double)pos * theta, &sn, &cs);
        const double re = row[p.d_c + 2 * tid], im = row[p.d_c + 2 * tid + 1];
        row[p.d_c + 2 * tid]     = (float)(re * cs - im * sn);
        row[p.d_c + 2 * tid + 1] = (float)(re * sn + im * cs);
    }
    __syncthreads();

    if (CACHE == MLA_F32) {
        float* dst = static_cast<float*>(p.kv) + r * n;
        for (int j = tid; j < n; j += 256) dst[j] = row[j];
    } else if (CACHE == MLA_BF16) {
        uint16_t* dst = static_cast<uint16_t*>(p.kv) + r * n;
        for (int j = tid; j < n; j += 256) dst[j] = (uint16_t)f32_to_bf16_bits(row[j]);
    } else {
        float amax = 0.f;
        for (int j = tid; j < n; j += 256) amax = fmaxf(amax, fabsf(row[j]));
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
        if ((tid & 63) == 0) wmax[tid >> 6] = amax;
        __syncthreads();
        amax = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
        const float scale = amax > 0.f ? amax / 448.0f : 1.0f;
        uint8_t* dst = static_cast<uint8_t*>(p.kv) + r * n;
        for (int j = tid; j < n; j += 256) dst[j] = (uint8_t)f32_to_e4m3_bits(row[j] / scale);
        if (tid == 0) p.kv_scale[r] = scale;
    }
}

}  // namespace

// Slices of the model dimension: the widest slice (fewest partial rows) that still gives the
// chip a workgroup per CU, the narrowest if none does.  Slices of a multiple of 32 up to 512
// rows suit the matrix-core GEMM; anything else runs as one slice on the scalar-FMA kernel.
int append_slices(int B, int D, int n, mla_dtype io)
{
    if (io != MLA_BF16 || D % 32 || n % 16) return (D > 512 && D % 512 == 0) ? D / 512 : 1;
    const long per_slice = (long)((n + 63) / 64) * ((B + 63) / 64);
    int best = 0;
    for (int ks = 512; ks >= 32; ks >>= 1) {
        if (D % ks) continue;
        best = D / ks;
        if ((long)best * per_slice >= 256) break;
    }
    return best > 0 ? best : 1;
}

hipError_t launch_cache_append(const AppendParams& p, mla_dtype io, mla_dtype cache, hipStream_t s)
{
    const int n = p.d_c + p.d_rope;
    // x [B, D] = [B, slices, D/slices] and W [D, n] = [slices, D/slices, n]: the slices are the "heads"
    hipError_t e = launch_head_gemm(p.x, p.W, p.part, p.B, p.slices, p.D / p.slices, n, io, s,
                                    /*y_f32=*/true);
    if (e != hipSuccess) return e;
    dim3 grid(p.B), block(256);
    if (cache == MLA_F32)       append_finish_kernel<MLA_F32><<<grid, block, 0, s>>>(p);
    else if (cache == MLA_BF16) append_finish_kernel<MLA_BF16><<<grid, block, 0, s>>>(p);
    else                        append_finish_kernel<MLA_FP8_E4M3><<<grid, block, 0, s>>>(p);
    return hipGetLastError();
}

}  // namespace mla
