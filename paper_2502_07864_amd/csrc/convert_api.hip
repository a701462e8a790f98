// C ABI of the offline GQA -> MLA conversion (include/mla_convert_gfx950.h):
// argument checks on the host, then launches on the caller's stream.
#include "mla_convert_gfx950.h"
#include "convert_internal.h"
#include <algorithm>

using namespace mla::conv;

namespace {

constexpr int JACOBI_MAX_SWEEPS = 60;
// Rayleigh-Ritz matrix of the power iteration (chip-wide solver above order 128): 6-8 sweeps are what it
// takes; the sweeps enqueued beyond convergence still cost their launches (2.5 us each, 1150 per sweep at
// order 576), so the cap is kept close.  A matrix that needs more is reported through info (-1).
constexpr int RITZ_MAX_SWEEPS = 10;

inline size_t align256(size_t b) { return (b + 255) & ~size_t(255); }
inline int st(hipError_t e) { return e == hipSuccess ? MLA_OK : MLA_ERR_HIP; }

// C = scale * op(A) op(B) helpers on row-major matrices
inline GemmF64 gemm_nt(const double* A, long lda, const double* B, long ldb, double* C, long ldc, int M, int N, int K, double alpha) {
    return GemmF64{A, lda, 1, B, 1, ldb, C, ldc, M, N, K, alpha, nullptr, 0};   // C = A B^T
}
inline GemmF64 gemm_nn(const double* A, long lda, const double* B, long ldb, double* C, long ldc, int M, int N, int K, double alpha) {
    return GemmF64{A, lda, 1, B, ldb, 1, C, ldc, M, N, K, alpha, nullptr, 0};   // C = A B
}
inline GemmF64 gemm_tn(const double* A, long lda, const double* B, long ldb, double* C, long ldc, int M, int N, int K, double alpha) {
    return GemmF64{A, 1, lda, B, ldb, 1, C, ldc, M, N, K, alpha, nullptr, 0};   // C = A^T B (A is K x M)
}

constexpr int GRAM_SLICES = 16;     // K slices of the p x p products of tall blocks
struct TopWs { double *Y, *Q, *G, *X, *T, *Z, *tmp, *part; size_t part_doubles; size_t bytes; };
TopWs top_ws(void* base, int m, int p) {
    TopWs w{};
    size_t off = 0;
    auto take = [&](size_t count) { double* ptr = base ? reinterpret_cast<double*>(static_cast<char*>(base) + off) : nullptr;
                                    off += align256(count * sizeof(double)); return ptr; };
    w.Y = take((size_t)m * p);
    w.Q = take((size_t)m * p);
    w.G = take((size_t)p * p);
    w.X = take((size_t)p * p);
    w.T = take((size_t)p * p);
    w.Z = take(jacobi_work_bytes(1, p) / sizeof(double));
    w.tmp = take(chol_tmp_doubles(p));
    w.part_doubles = std::max((size_t)GRAM_SLICES * p * p, (size_t)4 * m * p);
    w.part = take(w.part_doubles);
    w.bytes = off;
    return w;
}

// Q <- Y L^{-T} with L L^T = Y^T Y  (one Cholesky-QR pass); the result lands in `out`
int chol_qr(const double* Y, double* out, const TopWs& w, int m, int p, int* bad, hipStream_t s) {
    GemmF64 gram = gemm_tn(Y, p, Y, p, w.G, p, p, p, m, 1.0);
    gram.partial = w.part;
    gram.partial_doubles = w.part_doubles;
    hipError_t e = launch_gemm_f64(gram, s);
    if (e != hipSuccess) return MLA_ERR_HIP;
    e = launch_chol_inverse(w.G, w.X, w.tmp, p, bad, s);
    if (e != hipSuccess) return MLA_ERR_HIP;
    return st(launch_gemm_f64(gemm_nt(Y, p, w.X, p, out, p, m, p, p, 1.0), s));
}

int top_eig(const double* S, const double* Q0, double* evals, double* R, const TopWs& w, int* info,
            int m, int r, int p, int iters, hipStream_t s) {
    hipError_t e = launch_fill_int(info, 0, 2, s);
    if (e != hipSuccess) return MLA_ERR_HIP;
    int rc;
    // orthonormal start block (two passes: the start block is the caller's and may be badly conditioned)
    if ((rc = chol_qr(Q0, w.Y, w, m, p, info, s)) != MLA_OK) return rc;
    if ((rc = chol_qr(w.Y, w.Q, w, m, p, info, s)) != MLA_OK) return rc;
    for (int it = 0; it < iters; ++it) {
        GemmF64 sq = gemm_nn(S, m, w.Q, p, w.Y, p, m, p, m, 1.0);
        sq.partial = w.part;
        sq.partial_doubles = w.part_doubles;
        e = launch_gemm_f64(sq, s);
        if (e != hipSuccess) return MLA_ERR_HIP;
        if ((rc = chol_qr(w.Y, w.Q, w, m, p, info, s)) != MLA_OK) return rc;
    }
    // second pass restores orthonormality to rounding level before the Rayleigh-Ritz step
    if ((rc = chol_qr(w.Q, w.Y, w, m, p, info, s)) != MLA_OK) return rc;
    e = launch_copy_scaled(w.Y, p, w.Q, p, m, p, nullptr, 0, s);
    if (e != hipSuccess) return MLA_ERR_HIP;
    // T = Q^T S Q, T = Z diag(evals) Z^T, R = Q Z[:, :r]
    GemmF64 sq = gemm_nn(S, m, w.Q, p, w.Y, p, m, p, m, 1.0);
    sq.partial = w.part;
    sq.partial_doubles = w.part_doubles;
    e = launch_gemm_f64(sq, s);
    if (e != hipSuccess) return MLA_ERR_HIP;
    GemmF64 ritz = gemm_tn(w.Q, p, w.Y, p, w.T, p, p, p, m, 1.0);
    ritz.partial = w.part;
    ritz.partial_doubles = w.part_doubles;
    e = launch_gemm_f64(ritz, s);
    if (e != hipSuccess) return MLA_ERR_HIP;
    e = launch_symmetrise(w.T, p, s);
    if (e != hipSuccess) return MLA_ERR_HIP;
    e = launch_jacobi(w.T, evals, w.Z, info + 1, 1, p, p > 128 ? RITZ_MAX_SWEEPS : JACOBI_MAX_SWEEPS, s);
    if (e != hipSuccess) return MLA_ERR_HIP;
    return st(launch_gemm_f64(gemm_nn(w.Q, p, w.T, p, R, r, m, r, p, 1.0), s));
}

struct LayerWs {
    double *K, *sigma_work, *W_K_rot, *E, *E_rot, *C, *norms, *S, *W_cat;
    void* top; size_t top_bytes;
    size_t bytes;
};
LayerWs layer_ws(void* base, int n, int D, int g, int h, int d, int M, int keep, int p) {
    LayerWs w{};
    size_t off = 0;
    auto take = [&](size_t count) { double* ptr = base ? reinterpret_cast<double*>(static_cast<char*>(base) + off) : nullptr;
                                    off += align256(count * sizeof(double)); return ptr; };
    const size_t gd = (size_t)g * d, mj = 2 * gd - (size_t)keep * (d / M), Mg = (size_t)M * g;
    w.K = take((size_t)n * gd);
    w.sigma_work = take(jacobi_work_bytes(d / (2 * M), (int)Mg) / sizeof(double));
    w.W_K_rot = take(gd * D);
    w.E = take(gd * (size_t)h * d);
    w.E_rot = take(gd * (size_t)h * d);
    w.C = take((size_t)n * mj);
    w.norms = take(2 * (size_t)n);
    w.S = take(mj * mj);
    w.W_cat = take(mj * D);
    w.top_bytes = top_ws(nullptr, (int)mj, p).bytes;
    w.top = base ? static_cast<char*>(base) + off : nullptr;
    off += w.top_bytes;
    w.bytes = off;
    return w;
}

bool layer_shape_ok(int n, int D, int g, int h, int d, int M, int keep, int r_kv, int p) {
    if (n <= 0 || D <= 0 || g <= 0 || h <= 0 || d <= 0 || M <= 0 || r_kv <= 0 || p <= 0) return false;
    if (d % 2 || (d / 2) % M || h % g || g < 2 || keep < 1 || keep > M) return false;
    const long mj = 2L * g * d - (long)keep * (d / M);
    return r_kv <= p && p <= mj;
}

}  // namespace

extern "C" {

int mla_conv_project(const double* X, const double* W, double* Y, int n, int D, int m, int ldy, void* hip_stream) {
    if (!X || !W || !Y) return MLA_ERR_NULL;
    if (n <= 0 || D <= 0 || m <= 0 || ldy < m) return MLA_ERR_SHAPE;
    return st(launch_gemm_f64(gemm_nt(X, D, W, D, Y, ldy, n, m, D, 1.0), static_cast<hipStream_t>(hip_stream)));
}

int mla_conv_rope_moments(const double* K, double* sigma, int n, int g, int d, int M, void* hip_stream) {
    if (!K || !sigma) return MLA_ERR_NULL;
    if (n <= 0 || g <= 0 || d <= 0 || M <= 0 || d % 2 || (d / 2) % M) return MLA_ERR_SHAPE;
    if ((long)M * g > MOMENT_MAX_MG) return MLA_ERR_UNSUPPORTED;
    return st(launch_rope_moments(K, sigma, n, g, d, M, static_cast<hipStream_t>(hip_stream)));
}

size_t mla_conv_sym_eig_workspace_bytes(int batch, int m) {
    if (batch <= 0 || m < 2 || m > EIG_MAX_M) return 0;
    return jacobi_work_bytes(batch, m);
}

int mla_conv_sym_eig(double* A, double* evals, double* work, size_t work_bytes, int* info,
                     int batch, int m, int max_sweeps, void* hip_stream) {
    if (!A || !evals || !info) return MLA_ERR_NULL;
    if (batch <= 0 || m < 2 || max_sweeps <= 0) return MLA_ERR_SHAPE;
    if (m > EIG_MAX_M || batch > 65535) return MLA_ERR_UNSUPPORTED;
    if (!work || work_bytes < mla_conv_sym_eig_workspace_bytes(batch, m)) return MLA_ERR_WORKSPACE;
    return st(launch_jacobi(A, evals, work, info, batch, m, max_sweeps, static_cast<hipStream_t>(hip_stream)));
}

int mla_conv_rotate_rows(const double* W, const double* U, double* W_out, int g, int d, int M, int keep, int cols, void* hip_stream) {
    if (!W || !U || !W_out) return MLA_ERR_NULL;
    if (g <= 0 || d <= 0 || M <= 0 || cols <= 0 || d % 2 || (d / 2) % M || keep < 1 || keep > M || W == W_out) return MLA_ERR_SHAPE;
    if ((long)M * g > MOMENT_MAX_MG || (cols + 31) / 32 > 65535) return MLA_ERR_UNSUPPORTED;
    return st(launch_rotate_rows(W, U, W_out, g, d, M, keep, cols, static_cast<hipStream_t>(hip_stream)));
}

int mla_conv_kv_balance(const double* K_nope, int ldk, const double* V, int ldv, double* alpha,
                        double* row_norms, int n, int a, int b, void* hip_stream) {
    if (!K_nope || !V || !alpha || !row_norms) return MLA_ERR_NULL;
    if (n <= 0 || a <= 0 || b <= 0 || ldk < a || ldv < b) return MLA_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipError_t e = launch_row_norms(K_nope, ldk, a, V, ldv, b, row_norms, n, s);
    if (e != hipSuccess) return MLA_ERR_HIP;
    return st(launch_alpha(row_norms, alpha, n, s));
}

int mla_conv_joint_moment(const double* K_nope, int ldk, const double* V, int ldv, const double* alpha,
                          double* C, double* S, int n, int a, int b, void* hip_stream) {
    if (!K_nope || !V || !alpha || !C || !S) return MLA_ERR_NULL;
    if (n <= 0 || a <= 0 || b <= 0 || ldk < a || ldv < b) return MLA_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const int m = a + b;
    hipError_t e = launch_balance(K_nope, ldk, V, ldv, alpha, C, n, a, b, s);
    if (e != hipSuccess) return MLA_ERR_HIP;
    return st(launch_gemm_f64(gemm_tn(C, m, C, m, S, m, m, m, n, 1.0 / (double)n), s));
}

size_t mla_conv_top_eig_workspace_bytes(int m, int p) {
    if (m <= 0 || p <= 0 || p > m || p > TOP_MAX_P) return 0;
    return top_ws(nullptr, m, p).bytes;
}

int mla_conv_top_eig(const double* S, const double* Q0, double* evals, double* R,
                     void* workspace, size_t workspace_bytes, int* info,
                     int m, int r, int p, int iters, void* hip_stream) {
    if (!S || !Q0 || !evals || !R || !info) return MLA_ERR_NULL;
    if (m <= 0 || r <= 0 || p < r || p > m || iters < 0 || p < 2) return MLA_ERR_SHAPE;
    if (p > TOP_MAX_P) return MLA_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < mla_conv_top_eig_workspace_bytes(m, p)) return MLA_ERR_WORKSPACE;
    return top_eig(S, Q0, evals, R, top_ws(workspace, m, p), info, m, r, p, iters, static_cast<hipStream_t>(hip_stream));
}

size_t mla_conv_apply_workspace_bytes(int m, int p) {
    if (m <= 0 || p <= 0) return 0;
    return (size_t)4 * m * p * sizeof(double);
}

int mla_conv_apply(const double* S, const double* Q, double* Y, void* workspace, size_t workspace_bytes,
                   int m, int p, void* hip_stream) {
    if (!S || !Q || !Y) return MLA_ERR_NULL;
    if (m <= 0 || p <= 0 || Q == Y) return MLA_ERR_SHAPE;
    GemmF64 g = gemm_nn(S, m, Q, p, Y, p, m, p, m, 1.0);
    if (workspace && workspace_bytes >= 2 * (size_t)m * p * sizeof(double)) {
        g.partial = static_cast<double*>(workspace);
        g.partial_doubles = workspace_bytes / sizeof(double);
    }
    return st(launch_gemm_f64(g, static_cast<hipStream_t>(hip_stream)));
}

size_t mla_convert_layer_workspace_bytes(int n, int D, int g, int h, int d, int M, int keep, int r_kv, int p) {
    if (!layer_shape_ok(n, D, g, h, d, M, keep, r_kv, p) || p > TOP_MAX_P || (long)M * g > MOMENT_MAX_MG) return 0;
    return layer_ws(nullptr, n, D, g, h, d, M, keep, p).bytes;
}

int mla_convert_layer(const double* X, const double* W_K, const double* W_V, const double* Q0,
                      double* W_KR, double* W_QR, double* W_DKV, double* W_UK, double* W_UV,
                      double* alpha, double* evals_rope, double* U, double* evals_joint, double* R_KV,
                      void* workspace, size_t workspace_bytes, int* info,
                      int n, int D, int g, int h, int d, int M, int keep, int r_kv, int p, int iters,
                      void* hip_stream) {
    if (!X || !W_K || !W_V || !Q0 || !W_KR || !W_QR || !W_DKV || !W_UK || !W_UV || !alpha || !evals_rope ||
        !U || !evals_joint || !R_KV || !info) return MLA_ERR_NULL;
    if (!layer_shape_ok(n, D, g, h, d, M, keep, r_kv, p) || iters < 0 || p < 2) return MLA_ERR_SHAPE;
    if (p > TOP_MAX_P || (long)M * g > MOMENT_MAX_MG || (long)M * g < 2) return MLA_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < mla_convert_layer_workspace_bytes(n, D, g, h, d, M, keep, r_kv, p)) return MLA_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const LayerWs w = layer_ws(workspace, n, D, g, h, d, M, keep, p);
    const int gd = g * d, hd = h * d, groups = d / (2 * M), Mg = M * g;
    const int d_rope = keep * (d / M);        // width of the RoPE key
    const int a = gd - d_rope, mj = a + gd;   // NoPE key, joint NoPE-key + value space
    hipError_t e;
#define MLA_TRY(call) do { e = (call); if (e != hipSuccess) return MLA_ERR_HIP; } while (0)
    // Sec. 4.1 / App. B: key activations before RoPE, their per-group moments, the bases U
    MLA_TRY(launch_gemm_f64(gemm_nt(X, D, W_K, D, w.K, gd, n, gd, D, 1.0), s));
    MLA_TRY(launch_rope_moments(w.K, U, n, g, d, M, s));
    MLA_TRY(launch_jacobi(U, evals_rope, w.sigma_work, info, groups, Mg, JACOBI_MAX_SWEEPS, s));
    // Sec. 4.2: rotate W^K and the selector matrices (W^UK_i)^T, stacked as [g d, h d]
    MLA_TRY(launch_rotate_rows(W_K, U, w.W_K_rot, g, d, M, keep, D, s));
    MLA_TRY(launch_selector(w.E, g, h, d, s));
    MLA_TRY(launch_rotate_rows(w.E, U, w.E_rot, g, d, M, keep, hd, s));
    // the RoPE key: W_KR = the first d_rope rows of the rotated W^K; W_QR[i][a][b] = E_rot[a][i d + b]
    MLA_TRY(launch_copy_scaled(w.W_K_rot, D, W_KR, D, d_rope, D, nullptr, 0, s));
    for (int i = 0; i < h; ++i)
        MLA_TRY(launch_copy_scaled(w.E_rot + (size_t)i * d, hd, W_QR + (size_t)i * d_rope * d, d, d_rope, d, nullptr, 0, s));
    // Sec. 4.3: activations of the NoPE key and of the values, alpha
    MLA_TRY(launch_gemm_f64(gemm_nt(X, D, w.W_K_rot + (size_t)d_rope * D, D, w.C, mj, n, a, D, 1.0), s));
    MLA_TRY(launch_gemm_f64(gemm_nt(X, D, W_V, D, w.C + a, mj, n, gd, D, 1.0), s));
    MLA_TRY(launch_row_norms(w.C, mj, a, w.C + a, mj, gd, w.norms, n, s));
    MLA_TRY(launch_alpha(w.norms, alpha, n, s));
    // App. D.2: balanced activations, their moment, its leading eigenvectors
    MLA_TRY(launch_balance(w.C, mj, w.C + a, mj, alpha, w.C, n, a, gd, s));
    MLA_TRY(launch_gemm_f64(gemm_tn(w.C, mj, w.C, mj, w.S, mj, mj, mj, n, 1.0 / (double)n), s));
    int rc = top_eig(w.S, Q0, evals_joint, R_KV, top_ws(w.top, mj, p), info + groups, mj, r_kv, p, iters, s);
    if (rc != MLA_OK) return rc;
    // W^DKV' = R^T [W^DK_NoPE / alpha ; W^DV]
    MLA_TRY(launch_copy_scaled(w.W_K_rot + (size_t)d_rope * D, D, w.W_cat, D, a, D, alpha, 2, s));
    MLA_TRY(launch_copy_scaled(W_V, D, w.W_cat + (size_t)a * D, D, gd, D, nullptr, 0, s));
    MLA_TRY(launch_gemm_f64(gemm_tn(R_KV, r_kv, w.W_cat, D, W_DKV, D, r_kv, D, mj, 1.0), s));
    // W^UK'_i = alpha W^UK_NoPE,i R_K for all heads at once: (E_rot[d_rope:, :])^T R_K -> [h d, r_kv]
    GemmF64 uk = gemm_tn(w.E_rot + (size_t)d_rope * hd, hd, R_KV, r_kv, W_UK, r_kv, hd, r_kv, a, 1.0);
    uk.alpha_dev = alpha;
    uk.dev_mode = 1;
    MLA_TRY(launch_gemm_f64(uk, s));
    // W^UV'_i = W^UV_i R_V: the rows of R_V that belong to the group of head i, transposed
    MLA_TRY(launch_gather_w_uv(R_KV, W_UV, g, h, d, a, r_kv, s));
#undef MLA_TRY
    return MLA_OK;
}

}  // extern "C"
