// Kernels of the offline GQA -> MLA conversion other than the matrix product:
// per-group second moments (App. B, App. C), row rotation (Sec. 4.2), balancing
// (Sec. 4.3), the batched Jacobi eigensolver, and the Cholesky step of the block
// power iteration (App. D.2).  All fp64.
#include "convert_internal.h"
#include <algorithm>
#include <mutex>
#include <set>
#include <utility>

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
// Output rows: the RoPE key first (component r < keep of group G at pair G * keep + r), then the NoPE
// key (component r >= keep at pair (r - keep) * groups + G).
__global__ __launch_bounds__(256) void rotate_rows_kernel(const double* __restrict__ W, const double* __restrict__ U,
                                                          double* __restrict__ W_out, int g, int d, int M, int keep, int cols) {
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
        const int groups = d / (2 * M);
        const long row = (r < keep ? 2L * (G * keep + r) : 2L * keep * groups + 2L * ((long)(r - keep) * groups + G)) + part;
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

// ------------------------------------------------------------------ Jacobi eigensolver, one large matrix
// The same rotations as above, spread over the chip, one launch per step (one workgroup per index
// pair: pending column rotations of the previous step on its two rows, then its own angle and row
// rotation).  Launch order on the stream is the only synchronisation.  A sweep
// starts with a norm launch that raises `done` once the off-diagonal part is small; later launches
// then return at once, so the host can enqueue the maximum number of sweeps without reading back.
struct WideState { double tot; int done, sweeps; };

__device__ __forceinline__ void round_robin_pair(int k, int step, int mp, int& p, int& q) {
    if (k == 0) { p = mp - 1; q = step; }
    else { p = (step + k) % (mp - 1); q = (step - k + (mp - 1)) % (mp - 1); }
    if (p > q) { const int t = p; p = q; q = t; }
}

__global__ __launch_bounds__(256) void jw_init_kernel(double* __restrict__ V, int m, WideState* st) {
    const long total = (long)m * m;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256)
        V[idx] = (idx / m == idx % m) ? 1.0 : 0.0;
    if (blockIdx.x == 0 && threadIdx.x == 0) { st->tot = 0.0; st->done = 0; st->sweeps = -1; }
}

__global__ __launch_bounds__(1024) void jw_norm_kernel(const double* __restrict__ A, int m, int sweep, WideState* st) {
    __shared__ double red[16];
    if (st->done) return;
    double off = 0.0, dia = 0.0;
    for (int idx = threadIdx.x; idx < m * m; idx += 1024) {
        const double v = A[idx];
        if (idx / m == idx % m) dia += v * v; else off += v * v;
    }
    off = block_sum(off, red);
    dia = block_sum(dia, red);
    if (threadIdx.x == 0) {
        if (sweep == 0) st->tot = off + dia;
        if (off <= 1e-26 * st->tot) { st->done = 1; st->sweeps = sweep > 0 ? sweep : 1; }
    }
}

// One step in one launch.  The workgroup of pair (p, q) first applies the column rotations of the
// PREVIOUS step (all its pairs, angles in cs_prev) to its own two rows of A and V -- every row belongs to
// exactly one pair of the current step, so every row gets them exactly once -- then derives its own angle,
// publishes it in cs_next and rotates its two rows of A.  The column rotations of the last step before a
// norm check are flushed by jw_cols_kernel.
__global__ __launch_bounds__(256) void jw_step_kernel(double* A, double* V, int m, int mp, int step, int has_prev,
                                                      const double* __restrict__ cs_prev, double* __restrict__ cs_next,
                                                      const WideState* st) {
    if (st->done) return;
    const int k = blockIdx.x, half = mp / 2;
    int p, q;
    round_robin_pair(k, step, mp, p, q);
    const int nrows = q < m ? 2 : 1;                   // a bye: only row p exists
    if (has_prev) {
        const int prev = (step + mp - 2) % (mp - 1);
        for (int idx = threadIdx.x; idx < nrows * half; idx += 256) {
            const int i = idx < half ? p : q, kk = idx < half ? idx : idx - half;
            const double c = cs_prev[2 * kk], s = cs_prev[2 * kk + 1];
            if (s != 0.0) {
                int pp, qq;
                round_robin_pair(kk, prev, mp, pp, qq);
                const long ip = (long)i * m + pp, iq = (long)i * m + qq;
                const double ap = A[ip], aq = A[iq];
                A[ip] = i == qq ? 0.0 : c * ap - s * aq;        // the annihilated pair gets exact zeros
                A[iq] = i == pp ? 0.0 : s * ap + c * aq;
                const double vp = V[ip], vq = V[iq];
                V[ip] = c * vp - s * vq;
                V[iq] = s * vp + c * vq;
            }
        }
        __syncthreads();
    }
    double c = 1.0, s = 0.0;
    if (q < m) {
        const double apq = A[(long)p * m + q], app = A[(long)p * m + p], aqq = A[(long)q * m + q];
        if (fabs(apq) > 1e-300 && fabs(apq) > 1e-18 * sqrt(fabs(app * aqq))) {
            const double theta = (aqq - app) / (2.0 * apq);
            const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
            c = 1.0 / sqrt(t * t + 1.0);
            s = t * c;
        }
    }
    __syncthreads();                                   // every thread holds the angle before a row changes
    if (threadIdx.x == 0) { cs_next[2 * k] = c; cs_next[2 * k + 1] = s; }
    if (s == 0.0) return;
    for (int j = threadIdx.x; j < m; j += 256) {
        const long ip = (long)p * m + j, iq = (long)q * m + j;
        const double ap = A[ip], aq = A[iq];
        A[ip] = c * ap - s * aq;
        A[iq] = s * ap + c * aq;
    }
}

__global__ __launch_bounds__(256) void jw_cols_kernel(double* A, double* V, int m, int mp, int step,
                                                      const double* __restrict__ cs, const WideState* st) {
    if (st->done) return;
    const int half = mp / 2;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)half * m) return;
    const int k = (int)(idx % half), i = (int)(idx / half);
    const double c = cs[2 * k], s = cs[2 * k + 1];
    if (s == 0.0) return;
    int p, q;
    round_robin_pair(k, step, mp, p, q);
    const long ip = (long)i * m + p, iq = (long)i * m + q;
    const double ap = A[ip], aq = A[iq];
    A[ip] = i == q ? 0.0 : c * ap - s * aq;            // the annihilated pair gets exact zeros
    A[iq] = i == p ? 0.0 : s * ap + c * aq;
    const double vp = V[ip], vq = V[iq];
    V[ip] = c * vp - s * vq;
    V[iq] = s * vp + c * vq;
}

__global__ __launch_bounds__(1024) void jw_rank_kernel(const double* __restrict__ A, int m, double* __restrict__ evals,
                                                       int* __restrict__ rank, const WideState* st, int* info) {
    __shared__ double diag[EIG_MAX_M];
    for (int i = threadIdx.x; i < m; i += 1024) diag[i] = A[(long)i * m + i];
    __syncthreads();
    for (int i = threadIdx.x; i < m; i += 1024) {
        const double di = diag[i];
        int r = 0;
        for (int j = 0; j < m; ++j) { const double dj = diag[j]; r += (dj > di) || (dj == di && j < i); }
        rank[i] = r;
        evals[r] = di;
    }
    if (threadIdx.x == 0) *info = st->done ? st->sweeps : -1;
}

__global__ __launch_bounds__(256) void jw_permute_kernel(double* __restrict__ A_out, const double* __restrict__ V,
                                                         const int* __restrict__ rank, int m) {
    const long total = (long)m * m;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256)
        A_out[(idx / m) * m + rank[idx % m]] = V[idx];
}

// ------------------------------------------------------------------ Cholesky factor and its inverse
// Blocked, 64 columns at a time; the matrix products between the blocks run on the matrix-core
// kernel, the 64 x 64 pieces below in LDS.
constexpr int NB = 64;

// floor for the pivots: 1e-13 of the largest diagonal entry
__global__ __launch_bounds__(1024) void max_diag_kernel(const double* __restrict__ G, int p, double* __restrict__ floor_out) {
    __shared__ double red[16];
    double mx = 0.0;
    for (int i = threadIdx.x; i < p; i += 1024) mx = fmax(mx, G[(long)i * p + i]);
    for (int o = 32; o > 0; o >>= 1) mx = fmax(mx, __shfl_xor(mx, o));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        mx = 0.0;
        for (int w = 0; w < 16; ++w) mx = fmax(mx, red[w]);
        *floor_out = fmax(mx * 1e-13, 1e-300);
    }
}

// Block column k0, step 1: one workgroup factors the nb x nb diagonal block in LDS.
__global__ __launch_bounds__(256) void chol_diag_kernel(double* G, int p, int k0, int nb,
                                                        const double* __restrict__ floor_in, int* bad) {
    __shared__ double D[NB][NB + 1];
    __shared__ double piv;
    __shared__ int nbad;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    for (int idx = tid; idx < nb * nb; idx += 256) D[idx / nb][idx % nb] = G[(long)(k0 + idx / nb) * p + k0 + idx % nb];
    if (tid == 0) nbad = 0;
    const double floor_v = *floor_in;
    __syncthreads();
    for (int j = 0; j < nb; ++j) {
        if (tid == 0) {
            double v = D[j][j];
            if (!(v > floor_v)) { v = floor_v; ++nbad; }
            v = sqrt(v);
            D[j][j] = v;
            piv = v;
        }
        __syncthreads();
        const double inv = 1.0 / piv;
        for (int i = j + 1 + tid; i < nb; i += 256) D[i][j] *= inv;
        __syncthreads();
        for (int i = j + 1 + ty; i < nb; i += 16) {
            const double lij = D[i][j];
            for (int k = j + 1 + tx; k <= i; k += 16) D[i][k] -= lij * D[k][j];
        }
        __syncthreads();
    }
    for (int idx = tid; idx < nb * nb; idx += 256) {
        const int i = idx / nb, k = idx % nb;
        G[(long)(k0 + i) * p + k0 + k] = k <= i ? D[i][k] : 0.0;
    }
    if (tid == 0 && nbad) atomicAdd(bad, nbad);
}

// Step 2: workgroup w solves 64 rows of the panel below the factored block: L_rows = A_rows L_kk^{-T}.
__global__ __launch_bounds__(256) void chol_solve_kernel(double* G, int p, int k0, int nb) {
    __shared__ double D[NB][NB + 1], P[NB][NB + 1];
    const int tid = threadIdx.x;
    for (int idx = tid; idx < nb * nb; idx += 256) D[idx / nb][idx % nb] = G[(long)(k0 + idx / nb) * p + k0 + idx % nb];
    const int r0 = k0 + nb + blockIdx.x * NB;
    const int nr = min(NB, p - r0);
    for (int idx = tid; idx < nr * nb; idx += 256) P[idx / nb][idx % nb] = G[(long)(r0 + idx / nb) * p + k0 + idx % nb];
    __syncthreads();
    if (tid < nr) {
        for (int c = 0; c < nb; ++c) {
            double v = P[tid][c];
            for (int u = 0; u < c; ++u) v -= P[tid][u] * D[c][u];
            P[tid][c] = v / D[c][c];
        }
    }
    __syncthreads();
    for (int idx = tid; idx < nr * nb; idx += 256) G[(long)(r0 + idx / nb) * p + k0 + idx % nb] = P[idx / nb][idx % nb];
}

// The same two steps for full 64 x 64 blocks with the rows held in registers (every loop unrolled, so all
// register indices are static).  Factorisation: one wavefront, lane i owns row i; per step every lane
// publishes its entry of column j in LDS and reads the others back as broadcasts, so a step is one LDS
// round trip and no barrier (a single wavefront's LDS accesses complete in order).  Entries above
// the diagonal are scratch.
__global__ __launch_bounds__(64) void chol_diag64_kernel(double* G, int p, int k0,
                                                         const double* __restrict__ floor_in, int* bad) {
    __shared__ double col[NB];
    const int i = threadIdx.x;
    double* mine = G + (long)(k0 + i) * p + k0;
    double row[NB];
#pragma unroll
    for (int k = 0; k < NB; ++k) row[k] = mine[k];
    const double floor_v = *floor_in;
    int nbad = 0;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        col[i] = row[j];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        double d = col[j];
        if (!(d > floor_v)) { d = floor_v; ++nbad; }
        const double piv = sqrt(d), inv = 1.0 / piv;
        row[j] = i == j ? piv : row[j] * inv;
#pragma unroll
        for (int k = j + 1; k < NB; ++k) row[k] -= row[j] * (col[k] * inv);   // col[k] * inv: the bits lane k stores
        __builtin_amdgcn_wave_barrier();
    }
#pragma unroll
    for (int k = 0; k < NB; ++k) mine[k] = k <= i ? row[k] : 0.0;
    if (i == 0 && nbad) atomicAdd(bad, nbad);
}

// Panel solve: one wavefront per 64 rows, lane = row, the factored block (and the reciprocals of its
// diagonal) broadcast from LDS.
__global__ __launch_bounds__(64) void chol_solve64_kernel(double* G, int p, int k0) {
    __shared__ double D[NB][NB], Dinv[NB];
    const int tid = threadIdx.x;
#pragma unroll 8
    for (int idx = tid; idx < NB * NB; idx += 64) D[idx / NB][idx % NB] = G[(long)(k0 + idx / NB) * p + k0 + idx % NB];
    __syncthreads();
    Dinv[tid] = 1.0 / D[tid][tid];
    __syncthreads();
    const int r = k0 + NB + blockIdx.x * NB + tid;
    if (r >= p) return;
    double* mine = G + (long)r * p + k0;
    double x[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) x[c] = mine[c];
#pragma unroll
    for (int c = 0; c < NB; ++c) {
        double v0 = x[c], v1 = 0.0;                    // two chains: the sums are short but dependent
#pragma unroll
        for (int u = 0; u + 1 < c; u += 2) { v0 -= x[u] * D[c][u]; v1 -= x[u + 1] * D[c][u + 1]; }
        if (c & 1) v0 -= x[c - 1] * D[c][c - 1];
        x[c] = (v0 + v1) * Dinv[c];
    }
#pragma unroll
    for (int c = 0; c < NB; ++c) mine[c] = x[c];
}

// X_jj = L_jj^{-1} for every diagonal block j (one workgroup each); thread c solves L x = e_c.
__global__ __launch_bounds__(64) void tri_inverse_diag_kernel(const double* __restrict__ G, double* __restrict__ X, int p) {
    __shared__ double D[NB][NB + 1], Y[NB][NB + 1];
    const int k0 = blockIdx.x * NB, nb = min(NB, p - k0), c = threadIdx.x;
    for (int idx = c; idx < nb * nb; idx += 64) D[idx / nb][idx % nb] = G[(long)(k0 + idx / nb) * p + k0 + idx % nb];
    __syncthreads();
    if (c < nb) {
        for (int i = 0; i < c; ++i) Y[i][c] = 0.0;
        Y[c][c] = 1.0 / D[c][c];
        for (int i = c + 1; i < nb; ++i) {
            double a = 0.0;
            for (int k = c; k < i; ++k) a += D[i][k] * Y[k][c];
            Y[i][c] = -a / D[i][i];
        }
    }
    __syncthreads();
    for (int idx = c; idx < nb * nb; idx += 64) X[(long)(k0 + idx / nb) * p + k0 + idx % nb] = Y[idx / nb][idx % nb];
}

__global__ __launch_bounds__(256) void fill_double_kernel(double* dst, double value, long count) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < count; i += (long)gridDim.x * 256) dst[i] = value;
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
                                                          int g, int h, int d, int nope, int r) {
    const long total = (long)h * r * d;
    const int per = h / g;
    for (long idx = (long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long)gridDim.x * 256) {
        const int b = (int)(idx % d), rho = (int)((idx / d) % r), i = (int)(idx / ((long)d * r));
        W_UV[idx] = R[((long)nope + (long)(i / per) * d + b) * r + rho];
    }
}

inline int grid_for(long total) {
    const long b = (total + 255) / 256;
    return (int)(b < 1 ? 1 : (b > 65535 ? 65535 : b));
}

}  // namespace

hipError_t allow_dynamic_lds(const void* kernel, int bytes) {
    static std::mutex lock;
    static std::set<std::pair<const void*, int>> done;
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> hold(lock);
    if (done.count({kernel, device})) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.insert({kernel, device});
    return e;
}

hipError_t launch_rope_moments(const double* K, double* sigma, int n, int g, int d, int M, hipStream_t s) {
    rope_moments_kernel<<<d / (2 * M), 256, 0, s>>>(K, sigma, n, g, d, M);
    return hipGetLastError();
}

hipError_t launch_rotate_rows(const double* W, const double* U, double* W_out, int g, int d, int M, int keep, int cols, hipStream_t s) {
    dim3 grid(2 * (d / (2 * M)), (cols + 31) / 32);
    rotate_rows_kernel<<<grid, 256, 0, s>>>(W, U, W_out, g, d, M, keep, cols);
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

// scratch behind the batch of V matrices: angles, ranks, state of the wide solver
constexpr size_t JACOBI_EXTRA_BYTES = 2 * (2 * 1024 * sizeof(double)) + EIG_MAX_M * sizeof(int) + 256;
size_t jacobi_work_bytes(int batch, int m) { return (size_t)batch * m * m * sizeof(double) + JACOBI_EXTRA_BYTES; }

static hipError_t launch_jacobi_wide(double* A, double* evals, double* V, void* extra, int* info, int m, int max_sweeps, hipStream_t s) {
    double* cs[2] = {static_cast<double*>(extra), static_cast<double*>(extra) + 2 * 1024};   // angles of step parity
    int* rank = reinterpret_cast<int*>(cs[1] + 2 * 1024);
    WideState* st = reinterpret_cast<WideState*>(rank + EIG_MAX_M);
    const int mp = m + (m & 1), half = mp / 2;
    hipError_t e;
    jw_init_kernel<<<grid_for((long)m * m), 256, 0, s>>>(V, m, st);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int col_grid = (int)(((long)half * m + 255) / 256);
    for (int sweep = 0; sweep <= max_sweeps; ++sweep) {
        jw_norm_kernel<<<1, 1024, 0, s>>>(A, m, sweep, st);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (sweep == max_sweeps) break;
        for (int step = 0; step < mp - 1; ++step)
            jw_step_kernel<<<half, 256, 0, s>>>(A, V, m, mp, step, step > 0, cs[(step + 1) & 1], cs[step & 1], st);
        // the column rotations of the sweep's last step, before the norm is taken
        jw_cols_kernel<<<col_grid, 256, 0, s>>>(A, V, m, mp, mp - 2, cs[(mp - 2) & 1], st);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    jw_rank_kernel<<<1, 1024, 0, s>>>(A, m, evals, rank, st, info);
    jw_permute_kernel<<<grid_for((long)m * m), 256, 0, s>>>(A, V, rank, m);
    return hipGetLastError();
}

hipError_t launch_jacobi(double* A, double* evals, double* work, int* info, int batch, int m, int max_sweeps, hipStream_t s) {
    if (m > 128) {                                     // large matrices: the whole chip works on one at a time
        void* extra = work + (size_t)batch * m * m;
        const int sweeps = std::min(max_sweeps, 16);   // every sweep enqueued costs its launches even after convergence
        for (int b = 0; b < batch; ++b) {
            hipError_t e = launch_jacobi_wide(A + (size_t)b * m * m, evals + (size_t)b * m, work + (size_t)b * m * m,
                                              extra, info + b, m, sweeps, s);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    const size_t head = (sizeof(JacobiLds) + 15) & ~size_t(15);
    const size_t mats = 2 * (size_t)m * m * sizeof(double);
    const int in_lds = head + mats <= 128 * 1024;
    const size_t bytes = head + (in_lds ? mats : 0);
    hipError_t e0 = allow_dynamic_lds(reinterpret_cast<const void*>(&jacobi_kernel), 128 * 1024);
    if (e0 != hipSuccess) return e0;
    const int threads = m <= 64 ? 256 : 1024;
    jacobi_kernel<<<batch, threads, bytes, s>>>(A, evals, work, info, m, max_sweeps, in_lds);
    return hipGetLastError();
}

hipError_t launch_chol_inverse(double* G, double* X, double* tmp, int p, int* bad, hipStream_t s) {
    double* floor_v = tmp;                 // one double
    double* T = tmp + 8;                   // 64 x p
    double* part = T + (size_t)NB * p;     // K slices of the products below: 16 x 64 x p
    hipError_t e;
    max_diag_kernel<<<1, 1024, 0, s>>>(G, p, floor_v);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int nblk = (p + NB - 1) / NB;
    // right-looking factorisation: panel, then trailing block  A22 -= L21 L21^T
    for (int k = 0; k < nblk; ++k) {
        const int k0 = k * NB, nb = std::min(NB, p - k0), rest = p - k0 - nb;
        if (nb == NB) chol_diag64_kernel<<<1, 64, 0, s>>>(G, p, k0, floor_v, bad);
        else chol_diag_kernel<<<1, 256, 0, s>>>(G, p, k0, nb, floor_v, bad);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (rest > 0) {
            if (nb == NB) chol_solve64_kernel<<<(rest + NB - 1) / NB, 64, 0, s>>>(G, p, k0);
            else chol_solve_kernel<<<(rest + NB - 1) / NB, 256, 0, s>>>(G, p, k0, nb);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            const double* L21 = G + (long)(k0 + nb) * p + k0;
            GemmF64 g{L21, p, 1, L21, 1, p, G + (long)(k0 + nb) * (p + 1), p, rest, rest, nb, -1.0, nullptr, 0, 1, nullptr, 0};
            if ((e = launch_gemm_f64(g, s)) != hipSuccess) return e;
        }
    }
    // X = L^{-1}: diagonal blocks, then block row i:  X[i, :i] = -X_ii (L[i, :i] X[:i, :i])
    fill_double_kernel<<<grid_for((long)p * p), 256, 0, s>>>(X, 0.0, (long)p * p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    tri_inverse_diag_kernel<<<nblk, 64, 0, s>>>(G, X, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    for (int i = 1; i < nblk; ++i) {
        const int i0 = i * NB, nb = std::min(NB, p - i0);
        GemmF64 t{G + (long)i0 * p, p, 1, X, p, 1, T, p, nb, i0, i0, 1.0, nullptr, 0, 0, part, (size_t)16 * NB * p};
        if ((e = launch_gemm_f64(t, s)) != hipSuccess) return e;
        GemmF64 x{X + (long)i0 * (p + 1), p, 1, T, p, 1, X + (long)i0 * p, p, nb, i0, nb, -1.0, nullptr, 0, 0, nullptr, 0};
        if ((e = launch_gemm_f64(x, s)) != hipSuccess) return e;
    }
    return hipSuccess;
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

hipError_t launch_gather_w_uv(const double* R, double* W_UV, int g, int h, int d, int nope, int r, hipStream_t s) {
    gather_w_uv_kernel<<<grid_for((long)h * r * d), 256, 0, s>>>(R, W_UV, g, h, d, nope, r);
    return hipGetLastError();
}

}  // namespace conv
}  // namespace mla
