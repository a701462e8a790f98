// Kernels of the offline GQA -> MLA conversion other than the matrix product:
// per-group second moments (App. B, App. C), row rotation (Sec. 4.2), balancing
// (Sec. 4.3), the batched Jacobi eigensolver, and the Cholesky step of the block
// power iteration (App. D.2).  All fp64.
#include "convert_internal.h"

namespace mla {
namespace conv {
namespace {

// ------------------------------------------------------------------ block reductions
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Sum over the workgroup; every thread gets the result.  red: >= 16 doubles of LDS.
__device__ __forceinline__ double block_sum(double v, double* red) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_sum(v);
    __syncthreads();                       // red may still be read from a previous call
    if (lane == 0) red[wave] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < nw; ++w) t += red[w];
    return t;
}

// ------------------------------------------------------------------ App. B / App. C: second moments
// One workgroup per FreqFold group.  Sixteen tokens at a time are staged in LDS
// (their M*g real and M*g imaginary components); thread t owns entries
// t, t + 256, ... of the (M g) x (M g) result.
constexpr int MT = 16;
__global__ __launch_bounds__(256) void rope_moments_kernel(const double* __restrict__ K, double* __restrict__ sigma,
                                                           int n, int g, int d, int M) {
    __shared__ double xs[MT][MOMENT_MAX_MG], ys[MT][MOMENT_MAX_MG];
    const int G = blockIdx.x, Mg = M * g, tid = threadIdx.x;
    const long ldk = (long)g * d;
    const int nout = Mg * Mg, nq = (nout + 255) / 256;
    double acc[64];
#pragma unroll
    for (int q = 0; q < 64; ++q) acc[q] = 0.0;
    for (int t0 = 0; t0 < n; t0 += MT) {
        for (int idx = tid; idx < MT * Mg; idx += 256) {
            const int tt = idx / Mg, c = idx % Mg;
            const int p = c / g, j = c % g;
            const long col = (long)j * d + 2 * (G * M + p);
            const int t = t0 + tt;
            xs[tt][c] = t < n ? K[t * ldk + col] : 0.0;
            ys[tt][c] = t < n ? K[t * ldk + col + 1] : 0.0;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 64; ++q) {
            if (q < nq) {
                const int o = tid + 256 * q;
                if (o < nout) {
                    const int c1 = o / Mg, c2 = o % Mg;
                    double a = acc[q];
#pragma unroll
                    for (int tt = 0; tt < MT; ++tt) a += xs[tt][c1] * xs[tt][c2] + ys[tt][c1] * ys[tt][c2];
                    acc[q] = a;
                }
            }
        }
        __syncthreads();
    }
    const double inv_n = 1.0 / (double)n;
#pragma unroll
    for (int q = 0; q < 64; ++q) {
        const int o = tid + 256 * q;
        if (q < nq && o < nout) sigma[(long)G * nout + o] = acc[q] * inv_n;
    }
}

// ------------------------------------------------------------------ Sec. 4.2: rotation of rows
// grid (2 * groups, column tiles of 32): part 0 rotates the real rows, part 1 the imaginary rows.
__global__ __launch_bounds__(256) void rotate_rows_kernel(const double* __restrict__ W, const double* __restrict__ U,
                                                          double* __restrict__ W_out, int g, int d, int M, int cols) {
    __shared__ double ws[MOMENT_MAX_MG][33];
    const int part = blockIdx.x & 1, G = blockIdx.x >> 1, Mg = M * g, tid = threadIdx.x;
    const int col0 = blockIdx.y * 32;
    for (int idx = tid; idx < Mg * 32; idx += 256) {
        const int c = idx >> 5, cc = idx & 31;
        const long row = (long)(c % g) * d + 2 * (G * M + c / g) + part;
        ws[c][cc] = col0 + cc < cols ? W[row * cols + col0 + cc] : 0.0;
    }
    __syncthreads();
    const int cc = tid & 31;
    const double* Ug = U + (long)G * Mg * Mg;
    for (int r = tid >> 5; r < Mg; r += 8) {
        double a = 0.0;
        for (int c = 0; c < Mg; ++c) a += Ug[c * Mg + r] * ws[c][cc];
        const long row = (long)(r / M) * d + 2 * (G * M + r % M) + part;
        if (col0 + cc < cols) W_out[row * cols + col0 + cc] = a;
    }
}

// ------------------------------------------------------------------ Sec. 4.3: alpha
// One wavefront per token: Euclidean norms of its NoPE-key row and of its value row.
__global__ __launch_bounds__(256) void row_norms_kernel(const double* __restrict__ K, int ldk, int a,
                                                        const double* __restrict__ V, int ldv, int b,
                                                        double* __restrict__ norms, int n) {
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (t >= n) return;
    double sk = 0.0, sv = 0.0;
    for (int c = lane; c < a; c += 64) { const double v = K[(long)t * ldk + c]; sk += v * v; }
    for (int c = lane; c < b; c += 64) { const double v = V[(long)t * ldv + c]; sv += v * v; }
    sk = wave_sum(sk);
    sv = wave_sum(sv);
    if (lane == 0) { norms[t] = sqrt(sk); norms[n + t] = sqrt(sv); }
}

__global__ __launch_bounds__(1024) void alpha_kernel(const double* __restrict__ norms, double* __restrict__ alpha, int n) {
    __shared__ double red[16];
    double sk = 0.0, sv = 0.0;
    for (int t = threadIdx.x; t < n; t += 1024) { sk += norms[t]; sv += norms[n + t]; }
    sk = block_sum(sk, red);
    sv = block_sum(sv, red);
    if (threadIdx.x == 0) *alpha = sk / sv;       // the 1/n of the two means cancels
}

__global__ __launch_bounds__(256) void balance_kernel(const double* K, int ldk, const double* V, int ldv,
                                                      const double* __restrict__ alpha, double* C, int n, int a, int b) {
    const double inv = 1.0 / *alpha;
    const long total = (long)n * (a + b);
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const long t = idx / (a + b);
        const int c = (int)(idx % (a + b));
        C[idx] = c < a ? K[t * ldk + c] * inv : V[t * ldv + (c - a)];
    }
}

// ------------------------------------------------------------------ batched Jacobi eigensolver
// One workgroup per matrix.  A sweep is m - 1 (m even; else m) steps of a round-robin
// schedule; a step rotates m/2 disjoint index pairs at once: first the rows of A
// (A <- J^T A), then the columns of A and of V (A <- A J, V <- V J), J being the
// product of the step's plane rotations.  Small matrices live in LDS, larger
// ones in global memory (the waves of a workgroup share one vector cache, so a barrier
// orders their accesses).  At the end the eigenvalues are ranked in descending order
// and the columns of V are written over A in that order.
struct JacobiLds {
    int pp[1024], qq[1024];
    double cc[1024], ss[1024];
    double red[16];
    int flag;
};

__global__ __launch_bounds__(1024) void jacobi_kernel(double* A_all, double* evals_all, double* V_all, int* info,
                                                      int m, int max_sweeps, int in_lds) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    JacobiLds& L = *reinterpret_cast<JacobiLds*>(smem);
    double* lds_mat = reinterpret_cast<double*>(smem + ((sizeof(JacobiLds) + 15) & ~size_t(15)));
    const int tid = threadIdx.x, nt = blockDim.x;
    double* Ag = A_all + (long)blockIdx.x * m * m;
    double* Vg = V_all + (long)blockIdx.x * m * m;
    double* A = in_lds ? lds_mat : Ag;
    double* V = in_lds ? lds_mat + (long)m * m : Vg;

    double tot = 0.0;
    for (int idx = tid; idx < m * m; idx += nt) {
        const double v = Ag[idx];
        if (in_lds) A[idx] = v;
        V[idx] = (idx / m == idx % m) ? 1.0 : 0.0;
        tot += v * v;
    }
    tot = block_sum(tot, L.red);                       // squared Frobenius norm (orthogonal similarity keeps it)
    const double tol2 = 1e-26 * tot;

    const int mp = m + (m & 1), half = mp / 2;        // odd m: index m is a bye
    int used = -1;
    for (int sweep = 0; sweep <= max_sweeps; ++sweep) {
        double off = 0.0;
        for (int idx = tid; idx < m * m; idx += nt)
            if (idx / m != idx % m) { const double v = A[idx]; off += v * v; }
        off = block_sum(off, L.red);
        if (off <= tol2) { used = sweep > 0 ? sweep : 1; break; }
        if (sweep == max_sweeps) break;
        for (int step = 0; step < mp - 1; ++step) {
            for (int k = tid; k < half; k += nt) {
                int p, q;
                if (k == 0) { p = mp - 1; q = step; }
                else { p = (step + k) % (mp - 1); q = (step - k + (mp - 1)) % (mp - 1); }
                if (p > q) { const int t = p; p = q; q = t; }
                double c = 1.0, s = 0.0;
                if (q < m) {
                    const double apq = A[(long)p * m + q];
                    const double app = A[(long)p * m + p], aqq = A[(long)q * m + q];
                    if (fabs(apq) > 1e-300 && fabs(apq) > 1e-18 * sqrt(fabs(app * aqq))) {
                        const double theta = (aqq - app) / (2.0 * apq);
                        const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                        c = 1.0 / sqrt(t * t + 1.0);
                        s = t * c;
                    }
                } else {
                    q = p;                              // bye: nothing to rotate
                }
                L.pp[k] = p; L.qq[k] = q; L.cc[k] = c; L.ss[k] = s;
            }
            __syncthreads();
            // rows p and q of A
            for (int idx = tid; idx < half * m; idx += nt) {
                const int k = idx / m, j = idx % m;
                const double s = L.ss[k];
                if (s != 0.0) {
                    const double c = L.cc[k];
                    const long ip = (long)L.pp[k] * m + j, iq = (long)L.qq[k] * m + j;
                    const double ap = A[ip], aq = A[iq];
                    A[ip] = c * ap - s * aq;
                    A[iq] = s * ap + c * aq;
                }
            }
            __syncthreads();
            // columns p and q of A and of V
            for (int idx = tid; idx < half * m; idx += nt) {
                const int k = idx % half, i = idx / half;
                const double s = L.ss[k];
                if (s != 0.0) {
                    const double c = L.cc[k];
                    const long ip = (long)i * m + L.pp[k], iq = (long)i * m + L.qq[k];
                    const double ap = A[ip], aq = A[iq];
                    // the rotation was chosen to annihilate A[p][q] and A[q][p]: store exact zeros there
                    A[ip] = i == L.qq[k] ? 0.0 : c * ap - s * aq;
                    A[iq] = i == L.pp[k] ? 0.0 : s * ap + c * aq;
                    const double vp = V[ip], vq = V[iq];
                    V[ip] = c * vp - s * vq;
                    V[iq] = s * vp + c * vq;
                }
            }
            __syncthreads();
        }
    }

    // rank the diagonal in descending order (ties: lower index first); cc doubles as the diagonal store
    double* diag = L.cc;                               // m <= 2048 entries: cc and ss are adjacent, 2048 doubles
    int* rank = L.pp;                                  // pp and qq are adjacent, 2048 ints
    __syncthreads();
    for (int i = tid; i < m; i += nt) diag[i] = A[(long)i * m + i];
    __syncthreads();
    for (int i = tid; i < m; i += nt) {
        const double di = diag[i];
        int r = 0;
        for (int j = 0; j < m; ++j) { const double dj = diag[j]; r += (dj > di) || (dj == di && j < i); }
        rank[i] = r;
        evals_all[(long)blockIdx.x * m + r] = di;
    }
    __syncthreads();
    for (int idx = tid; idx < m * m; idx += nt) {
        const int i = idx / m, c = idx % m;
        Ag[(long)i * m + rank[c]] = V[idx];
    }
    if (tid == 0) info[blockIdx.x] = used;
}

// ------------------------------------------------------------------ Cholesky factor and its inverse
// One workgroup of 1024 threads on a p x p matrix in global memory (p <= 1024).
// Right-looking: scale column j, then subtract its outer product from the trailing
// lower triangle.  A pivot that is not above 1e-13 of the largest diagonal entry is clamped
// to that floor and counted.  Then X = L^{-1}, one thread per column by forward substitution.
__global__ __launch_bounds__(1024) void chol_inverse_kernel(double* G, double* X, int p, int* bad) {
    __shared__ double piv, red[16], colj[TOP_MAX_P];
    __shared__ int nbad;
    const int tid = threadIdx.x, tx = tid & 31, ty = tid >> 5;
    double mx = 0.0;
    for (int i = tid; i < p; i += 1024) mx = fmax(mx, G[(long)i * p + i]);
    // block maximum through the sum helper's LDS: take the max per wave, then over waves
    for (int o = 32; o > 0; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o));
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    if (tid == 0) nbad = 0;
    __syncthreads();
    mx = 0.0;
    for (int w = 0; w < 16; ++w) mx = fmax(mx, red[w]);
    const double floor_v = fmax(mx * 1e-13, 1e-300);

    for (int j = 0; j < p; ++j) {
        if (tid == 0) {
            double v = G[(long)j * p + j];
            if (!(v > floor_v)) { v = floor_v; ++nbad; }
            v = sqrt(v);
            G[(long)j * p + j] = v;
            piv = v;
        }
        __syncthreads();
        const double inv = 1.0 / piv;
        for (int i = j + 1 + tid; i < p; i += 1024) {
            const double v = G[(long)i * p + j] * inv;
            G[(long)i * p + j] = v;
            colj[i] = v;
        }
        __syncthreads();
        const int cnt = p - j - 1;
        for (int ii = ty; ii < cnt; ii += 32) {
            const long i = j + 1 + ii;
            const double lij = colj[i];
            for (int kk = tx; kk <= ii; kk += 32) {
                const long k = j + 1 + kk;
                G[i * p + k] -= lij * colj[k];
            }
        }
        __syncthreads();
    }
    // X = L^{-1}: column c solves L x = e_c
    for (int c = tid; c < p; c += 1024) {
        for (int i = 0; i < c; ++i) X[(long)i * p + c] = 0.0;
        X[(long)c * p + c] = 1.0 / G[(long)c * p + c];
    }
    __syncthreads();
    for (int i = 1; i < p; ++i) {
        // row i of X for all columns c < i:  x_ic = -(sum_{k=c}^{i-1} L_ik x_kc) / L_ii
        const double lii = G[(long)i * p + i];
        for (int c = tid; c < i; c += 1024) {
            double a = 0.0;
            for (int k = c; k < i; ++k) a += G[(long)i * p + k] * X[(long)k * p + c];
            X[(long)i * p + c] = -a / lii;
        }
        // column c only reads its own earlier entries: no barrier needed between rows
    }
    if (tid == 0 && nbad) atomicAdd(bad, nbad);
}

__global__ __launch_bounds__(256) void symmetrise_kernel(double* T, int p) {
    const long total = (long)p * p;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const int i = (int)(idx / p), j = (int)(idx % p);
        if (i < j) {
            const double v = 0.5 * (T[idx] + T[(long)j * p + i]);
            T[idx] = v;
            T[(long)j * p + i] = v;
        }
    }
}

__global__ void fill_int_kernel(int* dst, int value, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = value;
}

__global__ __launch_bounds__(256) void copy_scaled_kernel(const double* __restrict__ src, long lds_, double* __restrict__ dst, long ldd,
                                                          int rows, int cols, const double* __restrict__ scale, int mode) {
    const double f = mode == 1 ? *scale : (mode == 2 ? 1.0 / *scale : 1.0);
    const long total = (long)rows * cols;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const long r = idx / cols, c = idx % cols;
        dst[r * ldd + c] = src[r * lds_ + c] * f;
    }
}

__global__ __launch_bounds__(256) void selector_kernel(double* __restrict__ E, int g, int h, int d) {
    const long total = (long)g * d * h * d;
    const int per = h / g;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const long row = idx / ((long)h * d), col = idx % ((long)h * d);
        const int j = (int)(row / d), b = (int)(row % d), i = (int)(col / d), b2 = (int)(col % d);
        E[idx] = (j == i / per && b == b2) ? 1.0 : 0.0;
    }
}

__global__ __launch_bounds__(256) void gather_w_uv_kernel(const double* __restrict__ R, double* __restrict__ W_UV,
                                                          int g, int h, int d, int r) {
    const long total = (long)h * r * d;
    const int per = h / g;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const int b = (int)(idx % d), rho = (int)((idx / d) % r), i = (int)(idx / ((long)d * r));
        W_UV[idx] = R[((long)(g - 1) * d + (long)(i / per) * d + b) * r + rho];
    }
}

inline int grid_for(long total) {
    const long b = (total + 255) / 256;
    return (int)(b < 1 ? 1 : (b > 65535 ? 65535 : b));
}

}  // namespace

hipError_t launch_rope_moments(const double* K, double* sigma, int n, int g, int d, int M, hipStream_t s) {
    rope_moments_kernel<<<d / (2 * M), 256, 0, s>>>(K, sigma, n, g, d, M);
    return hipGetLastError();
}

hipError_t launch_rotate_rows(const double* W, const double* U, double* W_out, int g, int d, int M, int cols, hipStream_t s) {
    dim3 grid(2 * (d / (2 * M)), (cols + 31) / 32);
    rotate_rows_kernel<<<grid, 256, 0, s>>>(W, U, W_out, g, d, M, cols);
    return hipGetLastError();
}

hipError_t launch_row_norms(const double* K, int ldk, int a, const double* V, int ldv, int b, double* norms, int n, hipStream_t s) {
    row_norms_kernel<<<(n + 3) / 4, 256, 0, s>>>(K, ldk, a, V, ldv, b, norms, n);
    return hipGetLastError();
}

hipError_t launch_alpha(const double* norms, double* alpha, int n, hipStream_t s) {
    alpha_kernel<<<1, 1024, 0, s>>>(norms, alpha, n);
    return hipGetLastError();
}

hipError_t launch_balance(const double* K, int ldk, const double* V, int ldv, const double* alpha, double* C, int n, int a, int b, hipStream_t s) {
    balance_kernel<<<grid_for((long)n * (a + b)), 256, 0, s>>>(K, ldk, V, ldv, alpha, C, n, a, b);
    return hipGetLastError();
}

hipError_t launch_jacobi(double* A, double* evals, double* work, int* info, int batch, int m, int max_sweeps, hipStream_t s) {
    const size_t head = (sizeof(JacobiLds) + 15) & ~size_t(15);
    const size_t mats = 2 * (size_t)m * m * sizeof(double);
    const int in_lds = head + mats <= 128 * 1024;
    const size_t bytes = head + (in_lds ? mats : 0);
    static bool configured = false;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&jacobi_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        if (e != hipSuccess) return e;
        configured = true;
    }
    const int threads = m <= 64 ? 256 : 1024;
    jacobi_kernel<<<batch, threads, bytes, s>>>(A, evals, work, info, m, max_sweeps, in_lds);
    return hipGetLastError();
}

hipError_t launch_chol_inverse(double* G, double* X, int p, int* bad, hipStream_t s) {
    chol_inverse_kernel<<<1, 1024, 0, s>>>(G, X, p, bad);
    return hipGetLastError();
}

hipError_t launch_symmetrise(double* T, int p, hipStream_t s) {
    symmetrise_kernel<<<grid_for((long)p * p), 256, 0, s>>>(T, p);
    return hipGetLastError();
}

hipError_t launch_fill_int(int* dst, int value, int count, hipStream_t s) {
    fill_int_kernel<<<(count + 255) / 256, 256, 0, s>>>(dst, value, count);
    return hipGetLastError();
}

hipError_t launch_copy_scaled(const double* src, long lds_, double* dst, long ldd, int rows, int cols, const double* scale, int mode, hipStream_t s) {
    copy_scaled_kernel<<<grid_for((long)rows * cols), 256, 0, s>>>(src, lds_, dst, ldd, rows, cols, scale, mode);
    return hipGetLastError();
}

hipError_t launch_selector(double* E, int g, int h, int d, hipStream_t s) {
    selector_kernel<<<grid_for((long)g * d * h * d), 256, 0, s>>>(E, g, h, d);
    return hipGetLastError();
}

hipError_t launch_gather_w_uv(const double* R, double* W_UV, int g, int h, int d, int r, hipStream_t s) {
    gather_w_uv_kernel<<<grid_for((long)h * r * d), 256, 0, s>>>(R, W_UV, g, h, d, r);
    return hipGetLastError();
}

}  // namespace conv
}  // namespace mla
