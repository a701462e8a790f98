/*
 * mla_convert_gfx950.h -- C ABI of the offline GQA -> MLA conversion (Sec. 4 of
 * the paper, App. B-D) on AMD MI355X (gfx950), run once per layer on calibration
 * activations.  It produces the tensors the decode calls of mla_gfx950.h consume.
 *
 * Notation: g key/value heads of d dimensions (d even), h query heads (h % g == 0),
 * model dimension D, n calibration tokens.  Inside a head, RoPE pair l (from 0) is
 * dimension 2l (real part) and 2l+1 (imaginary part).  M adjacent pairs form one
 * FreqFold group (App. C); M = 1 is plain RoRoPE.  A "merged key" is the g*d vector
 * of all key heads side by side (Sec. 4.1).
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer to fp64 (IEEE binary64) data unless the
 *    comment says otherwise; all arithmetic is fp64.  Matrices are dense, row-major,
 *    8-byte aligned; a leading dimension "ld" is the distance between rows in elements.
 *  - The caller owns every buffer including workspaces; the library allocates
 *    nothing and keeps no state.  hip_stream is a hipStream_t as void*; all work is
 *    enqueued on it and the call returns without waiting.
 *  - Return value: MLA_OK or a negative mla_status (mla_gfx950.h); arguments are
 *    validated on the host before the first launch.  Numerical trouble that only the
 *    device can see is reported through an int "info" buffer the caller reads after
 *    synchronising (0 = fine).
 *  - Second moments are NOT mean-centred (App. B defines sigma = K^T K) and are divided
 *    by n.  Eigenvectors are unique only up to sign and up to a rotation inside a
 *    repeated eigenvalue.
 */
#ifndef MLA_CONVERT_GFX950_H
#define MLA_CONVERT_GFX950_H

#include "mla_gfx950.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Activations of a projection (Sec. 4.1, first equation; App. D.2 step 1):
 *   Y[t, 0:m] = W x_t      X [n, D], W [m, D], Y [n, ldy] (ldy >= m; other columns untouched)
 */
int mla_conv_project(const double* X, const double* W, double* Y,
                     int n, int D, int m, int ldy, void* hip_stream);

/*
 * Summed second moments of the real and imaginary key components per FreqFold group
 * (App. B: sigma_x + sigma_y; App. C: the M pairs of a group are concatenated).
 *   K      [n, g*d]  key activations BEFORE RoPE
 *   sigma  [d/(2M), M*g, M*g]; entry (p*g + j, p'*g + j') of group G is
 *          (1/n) sum_t  K[t, j*d + 2(GM+p)] K[t, j'*d + 2(GM+p')] + the same one column to the right
 * Requires (d/2) % M == 0.
 */
int mla_conv_rope_moments(const double* K, double* sigma,
                          int n, int g, int d, int M, void* hip_stream);

/*
 * Batched symmetric eigendecomposition (App. B: the columns of U are the eigenvectors
 * by descending eigenvalue; also the PCA of App. D.2).  Cyclic Jacobi rotations, one
 * workgroup per matrix up to m = 128; a larger matrix is spread over the chip, one launch per
 * rotation step, the batch is then processed one matrix after the other, and at most 16 sweeps are run.
 *   A      [batch, m, m]  in: symmetric matrices; out: eigenvectors in the COLUMNS, column c
 *                         belonging to evals[c]
 *   evals  [batch, m]     eigenvalues, descending
 *   work                  scratch of mla_conv_sym_eig_workspace_bytes(batch, m) bytes
 *   info   [batch] int    out: sweeps used (>= 1), or -1 if the off-diagonal part did not fall
 *                         below 1e-13 of the Frobenius norm within max_sweeps
 * 2 <= m <= 2048.
 */
size_t mla_conv_sym_eig_workspace_bytes(int batch, int m);
int mla_conv_sym_eig(double* A, double* evals, double* work, size_t work_bytes, int* info,
                     int batch, int m, int max_sweeps, void* hip_stream);

/*
 * Rotation of the rows of W^K, and of (W^UK_i)^T, by the RoRoPE bases (Sec. 4.2; the same
 * matrix on the real and on the imaginary vector of a group, Eq. "rorope"):
 *   for every group G and component r:
 *     W_out[row_x(G, r), :] = sum_c U[G][c, r] W[col_x(G, c), :]        (k' = U^T k)
 *     and the same for the imaginary rows (row + 1),
 *   col_x(G, c = p*g + j) = j*d + 2(GM+p).
 *   Output rows: first the RoPE key, the `keep` leading components of every group (1 <= keep <= M),
 *   d_rope = keep * d / M rows:  row_x(G, r) = 2 (G keep + r)  for r < keep;  then the NoPE key:
 *   row_x(G, r) = d_rope + 2 ((r - keep) d/(2M) + G)  for r >= keep.
 *   keep = M: the RoPE key is a whole head of d dimensions whose pair G M + r carries a component of
 *   the group that owns that pair, so ordinary RoPE of width d applies to it.  keep = 1: one pair per
 *   group, ordinary RoPE of width d / M applies (its pair G turns with the first frequency of group G,
 *   the effective frequency of App. C's example).  The paper fixes neither; Table 1's most compressed
 *   LLaMA-2-7B setting keeps 576 = r_kv + d^R values per token, which 512 + 64 (M = 2, keep = 1) meets.
 *   W, W_out [g*d, cols] (distinct buffers), U [d/(2M), M*g, M*g].
 */
int mla_conv_rotate_rows(const double* W, const double* U, double* W_out,
                         int g, int d, int M, int keep, int cols, void* hip_stream);

/*
 * Key/value balancing factor (Sec. 4.3):  alpha = mean_t ||K_nope[t]||_2 / mean_t ||V[t]||_2
 *   K_nope [n, ldk] (a columns used), V [n, ldv] (b columns used), alpha: one double,
 *   row_norms [2, n]: out, ||K_nope[t]||_2 then ||V[t]||_2 (summed in a fixed order: the
 *   result does not vary from run to run).
 */
int mla_conv_kv_balance(const double* K_nope, int ldk, const double* V, int ldv, double* alpha,
                        double* row_norms, int n, int a, int b, void* hip_stream);

/*
 * Second-moment matrix of the balanced activations c_t = [k_NoPE,t / alpha ; v_t] (App. D.2,
 * steps 1-2).   C [n, a+b] receives the c_t, S [(a+b), (a+b)] = C^T C / n.   alpha is the
 * DEVICE scalar written by mla_conv_kv_balance.  K_nope may be C and V may be C + a (with
 * ldk = ldv = a + b): the balancing is then done in place.
 */
int mla_conv_joint_moment(const double* K_nope, int ldk, const double* V, int ldv, const double* alpha,
                          double* C, double* S, int n, int a, int b, void* hip_stream);

/*
 * Leading eigenvectors of a symmetric positive semi-definite matrix (App. D.2: R_KV) by
 * block power iteration: Q <- orth(S Q), iters times, from the caller's start block Q0
 * (random numbers are the caller's), then one Rayleigh-Ritz step on the p-dimensional block.
 * The error of the r leading vectors falls like (lambda_{p+1} / lambda_r)^iters.
 *   S      [m, m]
 *   Q0     [m, p]   start block of full column rank, r <= p <= min(m, 1024)
 *   evals  [p]      Ritz values, descending (the first r are the estimates asked for)
 *   R      [m, r]   Ritz vectors of the r largest, in columns
 *   info   [2] int  info[0]: 0, or the number of Cholesky pivots that had to be clamped (the block
 *                   lost rank); info[1]: sweeps of the final eigendecomposition, -1 if not converged
 *                   (within 10 sweeps for p > 128)
 */
size_t mla_conv_top_eig_workspace_bytes(int m, int p);
/* One application of the moment matrix to a block, Y = S Q (the product each step of the
 * iteration above spends its time in; with Q = R it gives the residual S R - R diag(evals)).
 *   S [m, m], Q [m, p], Y [m, p] (distinct from Q).
 *   workspace: optional scratch of mla_conv_apply_workspace_bytes(m, p) bytes (NULL, 0: none).  With
 *   it, a product whose output tiles alone would leave CUs idle in the last round is computed in
 *   slices of the K range that are summed in a fixed order, as inside mla_conv_top_eig. */
size_t mla_conv_apply_workspace_bytes(int m, int p);
int mla_conv_apply(const double* S, const double* Q, double* Y, void* workspace, size_t workspace_bytes,
                   int m, int p, void* hip_stream);
int mla_conv_top_eig(const double* S, const double* Q0, double* evals, double* R,
                     void* workspace, size_t workspace_bytes, int* info,
                     int m, int r, int p, int iters, void* hip_stream);

/*
 * The whole chain for one layer (Sec. 4.1 merged head -> Sec. 4.2 RoRoPE with M-fold FreqFold
 * -> Sec. 4.3 balancing -> App. D.2 joint low-rank projections), on calibration tokens X.
 *   keep components per group stay under RoPE (see mla_conv_rotate_rows): d_rope = keep * d / M,
 *   and the joint space of NoPE key and values has m_j = 2 g d - d_rope dimensions.
 *   in : X [n, D], W_K [g*d, D], W_V [g*d, D], Q0 [m_j, p] start block for the joint basis
 *   out: W_KR   [d_rope, D]   k_rope = RoPE(W_KR x), RoPE of width d_rope   (the RoPE key)
 *        W_QR   [h, d_rope, d]  q_rope_i = RoPE(W_QR[i] q_i)
 *        W_DKV  [r_kv, D]     c_kv = W_DKV x                   (App. D.2: R^T [W^DK_NoPE/alpha ; W^DV])
 *        W_UK   [h, d, r_kv]  q_abs_i = q_i . W_UK[i]          (alpha W^UK_NoPE,i R_K)
 *        W_UV   [h, r_kv, d]  o_i = o_lat_i . W_UV[i]          ((W^UV_i R_V)^T)
 *        alpha  [1], evals_rope [d/(2M), M*g], U [d/(2M), M*g, M*g], evals_joint [p],
 *        R_KV [m_j, r_kv]
 *        info   [d/(2M) + 2] int: per-group sweeps of the RoRoPE bases, then the two entries of
 *               mla_conv_top_eig
 * The softmax scale of the converted layer stays 1/sqrt(d) (Eq. "qk_rope").
 */
size_t mla_convert_layer_workspace_bytes(int n, int D, int g, int h, int d, int M, int keep, int r_kv, int p);
int mla_convert_layer(const double* X, const double* W_K, const double* W_V, const double* Q0,
                      double* W_KR, double* W_QR, double* W_DKV, double* W_UK, double* W_UV,
                      double* alpha, double* evals_rope, double* U, double* evals_joint, double* R_KV,
                      void* workspace, size_t workspace_bytes, int* info,
                      int n, int D, int g, int h, int d, int M, int keep, int r_kv, int p, int iters,
                      void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MLA_CONVERT_GFX950_H */
