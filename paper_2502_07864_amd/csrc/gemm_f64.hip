// fp64 matrix product on the gfx950 matrix cores, used by the offline conversion
// (activations X W^T, second moments C^T C, block power iteration S Q, the low-rank
// projections R^T W and W R of App. D.2).
//
// Workgroup tile 128 x 128, K step 16, eight wavefronts in 4 x 2, each 32 x 64 =
// 2 x 4 tiles of v_mfma_f64_16x16x4_f64 (64 accumulator registers), two workgroups per
// CU = four wavefronts per SIMD: the matrix pipe of a SIMD always has a wavefront that
// is not waiting at the barrier or for LDS.  Lane l of a wavefront supplies
// A[l % 16][l / 16] and B[l / 16][l % 16] and receives D[4 r + l / 16][l % 16] in
// element r of the result vector.  Both operands are staged k-major in LDS
// ([k][m] and [k][n]) whichever way they lie in memory, so the inner loop is the
// same for all four transpose combinations; the next K step is fetched into
// registers while the current one is multiplied.
#include "convert_internal.h"
#include <algorithm>
#include <cmath>

namespace mla {
namespace conv {
namespace {

typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int THREADS = 512;                  // eight wavefronts in 4 x 2, each 32 x 64 = 2 x 4 tiles
constexpr int EPT = BM * BK / THREADS;        // elements of one operand tile per thread (4)
constexpr int LD = 132;                       // row pitch of a staged k-row, in doubles: 264 dwords = 8 (mod 64), so
                                              // the 16 k-rows a wavefront writes at once fall on different banks
constexpr int STAGE = BK * LD;                // one operand, one buffer

// Fetch the 128 x 16 tile of an operand whose (mn, k) element is P[mn*s_mn + k*s_k].
// K_CONTIG: s_k == 1, sixteen lanes read 128 consecutive bytes of one row;
// otherwise s_mn == 1 and 128 lanes read consecutive elements of one k-row.
template <bool K_CONTIG>
__device__ __forceinline__ void fetch(const double* __restrict__ P, long s_mn, long s_k,
                                      int mn0, int k0, int MN, int K, int tid, double (&r)[EPT]) {
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        int mn, k;
        if (K_CONTIG) { k = k0 + (tid & 15); mn = mn0 + (tid >> 4) + (THREADS / 16) * i; }
        else          { mn = mn0 + (tid & 127); k = k0 + (tid >> 7) + (THREADS / 128) * i; }
        r[i] = (mn < MN && k < K) ? P[(long)mn * s_mn + (long)k * s_k] : 0.0;
    }
}

template <bool K_CONTIG>
__device__ __forceinline__ void stage(double* S, int tid, const double (&r)[EPT]) {
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        if (K_CONTIG) S[(tid & 15) * LD + (tid >> 4) + (THREADS / 16) * i] = r[i];
        else          S[((tid >> 7) + (THREADS / 128) * i) * LD + (tid & 127)] = r[i];
    }
}

template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(THREADS, 2) void gemm_f64_kernel(GemmF64 g, int tiles_n, int tiles, int splits, int kt_per) {
    extern __shared__ double lds[];            // As[2][BK][LD], Bs[2][BK][LD]
    double* As = lds;
    double* Bs = lds + 2 * STAGE;

    // consecutive tiles (same rows of A) share an XCD: workgroup ids 8 apart run on one XCD
    const int total = tiles * splits;
    const int per = (total + 7) / 8;
    const int item = (int)(blockIdx.x % 8) * per + (int)(blockIdx.x / 8);
    if (item >= total) return;
    const int tile = item % tiles, z = item / tiles;     // z: slice of the K range
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
    const int nk_all = (g.K + BK - 1) / BK;
    const int kt0 = z * kt_per, kt1 = min(nk_all, kt0 + kt_per);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 32, wn = (wave & 1) * 64;
    const int li = lane & 15, kq = lane >> 4;
    // a wavefront whose 64 x 64 part lies outside the matrix (edge tiles) stages data but multiplies nothing
    const bool inside = m0 + wm < g.M && n0 + wn < g.N;

    f64x4 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = (f64x4){0.0, 0.0, 0.0, 0.0};

    double ra[EPT], rb[EPT];
    fetch<A_KC>(g.A, g.sAm, g.sAk, m0, kt0 * BK, g.M, g.K, tid, ra);
    fetch<B_KC>(g.B, g.sBn, g.sBk, n0, kt0 * BK, g.N, g.K, tid, rb);
    stage<A_KC>(As, tid, ra);
    stage<B_KC>(Bs, tid, rb);
    __syncthreads();

    for (int kt = kt0; kt < kt1; ++kt) {
        const int buf = (kt - kt0) & 1;
        const bool more = kt + 1 < kt1;
        if (more) {
            fetch<A_KC>(g.A, g.sAm, g.sAk, m0, (kt + 1) * BK, g.M, g.K, tid, ra);
            fetch<B_KC>(g.B, g.sBn, g.sBk, n0, (kt + 1) * BK, g.N, g.K, tid, rb);
        }
        const double* a_s = As + buf * STAGE + wm + li;
        const double* b_s = Bs + buf * STAGE + wn + li;
#pragma unroll
        for (int ks = 0; inside && ks < BK / 4; ++ks) {
            double a[2], b[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (t < 2) a[t] = a_s[(ks * 4 + kq) * LD + t * 16];
                b[t] = b_s[(ks * 4 + kq) * LD + t * 16];
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            stage<A_KC>(As + (buf ^ 1) * STAGE, tid, ra);
            stage<B_KC>(Bs + (buf ^ 1) * STAGE, tid, rb);
        }
        __syncthreads();
    }

    if (splits > 1) {                                    // raw slice product; the reduction kernel scales
        double* part = g.partial + (size_t)z * g.M * g.N;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = m0 + wm + i * 16 + 4 * r + kq;
                    const int col = n0 + wn + j * 16 + li;
                    if (row < g.M && col < g.N) part[(size_t)row * g.N + col] = acc[i][j][r];
                }
        return;
    }
    double scale = g.alpha;
    if (g.dev_mode == 1) scale *= *g.alpha_dev;
    else if (g.dev_mode == 2) scale /= *g.alpha_dev;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = m0 + wm + i * 16 + 4 * r + kq;
                const int col = n0 + wn + j * 16 + li;
                if (row < g.M && col < g.N) {
                    double* c = g.C + (long)row * g.ldc + col;
                    *c = g.accumulate ? *c + scale * acc[i][j][r] : scale * acc[i][j][r];
                }
            }
}

// C (=|+=) scale * sum over the K slices, slices added in index order
__global__ __launch_bounds__(256) void gemm_f64_reduce_kernel(GemmF64 g, int splits) {
    const long total = (long)g.M * g.N;
    double scale = g.alpha;
    if (g.dev_mode == 1) scale *= *g.alpha_dev;
    else if (g.dev_mode == 2) scale /= *g.alpha_dev;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        double a = 0.0;
        for (int z = 0; z < splits; ++z) a += g.partial[(size_t)z * total + idx];
        double* c = g.C + (idx / g.N) * g.ldc + idx % g.N;
        *c = g.accumulate ? *c + scale * a : scale * a;
    }
}

template <bool A_KC, bool B_KC>
hipError_t run(const GemmF64& g, hipStream_t s) {
    constexpr size_t lds_bytes = 4 * STAGE * sizeof(double);
    hipError_t e0 = allow_dynamic_lds(reinterpret_cast<const void*>(&gemm_f64_kernel<A_KC, B_KC>), (int)lds_bytes);
    if (e0 != hipSuccess) return e0;
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const int tiles = tiles_m * tiles_n;
    const int nk = (g.K + BK - 1) / BK;
    // K slices: only when scratch is there, the tiles leave most of the 256 CUs idle and every slice
    // still has at least 4 K steps
    int splits = 1;
    if (g.partial && nk >= 8) {
        const size_t fit = g.partial_doubles / ((size_t)g.M * g.N);
        const int most = (int)std::min<size_t>(std::min<size_t>(fit, 16), nk / 4);
        if (tiles <= 64) {
            splits = std::min(most, 256 / tiles);
        } else if (tiles < 1024) {
            // pick the fewest slices that keep at least 85 % of the CUs busy in the last round
            auto fill = [&](int sp) { const double r = (double)tiles * sp / 256.0; return r / std::ceil(r); };
            for (int sp = 1; sp <= std::min(most, 4); ++sp)
                if (fill(sp) > fill(splits) + 0.05) { splits = sp; if (fill(sp) >= 0.85) break; }
        }
        if (splits < 2) splits = 1;
    }
    int kt_per = (nk + splits - 1) / splits;
    splits = (nk + kt_per - 1) / kt_per;                 // no empty slice
    const int total = tiles * splits;
    const int grid = ((total + 7) / 8) * 8;
    gemm_f64_kernel<A_KC, B_KC><<<grid, THREADS, lds_bytes, s>>>(g, tiles_n, tiles, splits, kt_per);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || splits == 1) return e;
    const long cells = (long)g.M * g.N;
    gemm_f64_reduce_kernel<<<(int)std::min<long>((cells + 255) / 256, 4096), 256, 0, s>>>(g, splits);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_f64(const GemmF64& g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
    const bool a_kc = g.sAk == 1, b_kc = g.sBk == 1;
    if ((!a_kc && g.sAm != 1) || (!b_kc && g.sBn != 1)) return hipErrorInvalidValue;
    if (a_kc && b_kc) return run<true, true>(g, s);
    if (a_kc) return run<true, false>(g, s);
    if (b_kc) return run<false, true>(g, s);
    return run<false, false>(g, s);
}

}  // namespace conv
}  // namespace mla
