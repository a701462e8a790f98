// Internal declarations of the fp64 conversion kernels (Sec. 4, App. B-D).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

namespace mla {
namespace conv {

// C[m, n] = scale * sum_k A(m, k) B(k, n), where A(m, k) = A[m*sAm + k*sAk] and
// B(k, n) = B[k*sBk + n*sBn]; for each operand one of the two strides is 1.
// scale = alpha, times *alpha_dev (dev_mode 1) or divided by it (dev_mode 2).
// accumulate: C += instead of C =.
// partial / partial_doubles: optional scratch; when the tile count alone cannot fill the chip and K is
// deep, the K range is cut into slices whose products go to the scratch and are summed in a fixed order.
struct GemmF64 {
    const double* A; long sAm, sAk;
    const double* B; long sBk, sBn;
    double* C; long ldc;
    int M, N, K;
    double alpha;
    const double* alpha_dev; int dev_mode;
    int accumulate;
    double* partial; size_t partial_doubles;
};
hipError_t launch_gemm_f64(const GemmF64& g, hipStream_t s);

// Raise a kernel's dynamic-LDS limit; done once per (kernel, device), safe to call from several threads.
hipError_t allow_dynamic_lds(const void* kernel, int bytes);

// limits the host checks before launching
constexpr int MOMENT_MAX_MG = 128;   // M*g of a FreqFold group
constexpr int EIG_MAX_M = 2048;      // Jacobi: matrix order
constexpr int TOP_MAX_P = 1024;      // block power iteration: block width

hipError_t launch_rope_moments(const double* K, double* sigma, int n, int g, int d, int M, hipStream_t s);
hipError_t launch_rotate_rows(const double* W, const double* U, double* W_out, int g, int d, int M, int keep, int cols, hipStream_t s);
hipError_t launch_row_norms(const double* K, int ldk, int a, const double* V, int ldv, int b, double* norms, int n, hipStream_t s);
hipError_t launch_alpha(const double* norms, double* alpha, int n, hipStream_t s);
// C[t, 0:a] = K[t, 0:a] / *alpha, C[t, a:a+b] = V[t, 0:b]   (in place allowed)
hipError_t launch_balance(const double* K, int ldk, const double* V, int ldv, const double* alpha, double* C, int n, int a, int b, hipStream_t s);
// work: jacobi_work_bytes(batch, m) bytes
size_t jacobi_work_bytes(int batch, int m);
hipError_t launch_jacobi(double* A, double* evals, double* work, int* info, int batch, int m, int max_sweeps, hipStream_t s);
// G (p x p, symmetric positive definite) -> lower Cholesky factor in place (blocks above the diagonal
// are left undefined), X = its inverse (zero above the diagonal); *bad += clamped pivots.
// tmp: chol_tmp_doubles(p) doubles of scratch.
inline size_t chol_tmp_doubles(int p) { return 8 + (size_t)64 * p + (size_t)16 * 64 * p; }
hipError_t launch_chol_inverse(double* G, double* X, double* tmp, int p, int* bad, hipStream_t s);
hipError_t launch_symmetrise(double* T, int p, hipStream_t s);
hipError_t launch_fill_int(int* dst, int value, int count, hipStream_t s);
// dst[r, c] = src[r*lds + c] * f, f = 1, *scale (mode 1) or 1 / *scale (mode 2)
hipError_t launch_copy_scaled(const double* src, long lds_, double* dst, long ldd, int rows, int cols, const double* scale, int mode, hipStream_t s);
// E [g*d, h*d]: E[j*d + b, i*d + b] = 1 when j is the group of query head i (Sec. 4.1), else 0
hipError_t launch_selector(double* E, int g, int h, int d, hipStream_t s);
// W_UV[i, rho, b] = R[nope + group(i)*d + b, rho]   (nope: rows of the NoPE key in front of the values)
hipError_t launch_gather_w_uv(const double* R, double* W_UV, int g, int h, int d, int nope, int r, hipStream_t s);

}  // namespace conv
}  // namespace mla
