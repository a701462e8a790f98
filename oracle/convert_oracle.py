"""CPU oracle for the offline GQA -> MLA conversion -- TEST INFRASTRUCTURE ONLY.

Plain numpy in fp64, one function per step of the paper's conversion, in the
paper's order and notation.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import this module; the product path never
does, and this module imports nothing from the product.

Notation (Sec. 4, App. B-D): g key/value heads of d dimensions, h query
heads, model dimension D, n calibration tokens; inside a head the RoPE pair
l (0-based here) is made of dimension 2l (real part) and 2l+1 (imaginary
part); M adjacent pairs form one FreqFold group (M = 1: plain RoRoPE).

Steps
  merged_projections    Sec. 4.1        selector-identity W^UK_i, W^UV_i
  group_columns         App. C          which merged-key dimensions form the real / imaginary
                                        vectors of a FreqFold group
  rope_moments          App. B          sigma_x + sigma_y per group
  rorope_basis          App. B          U = eigenvectors, eigenvalues descending
  placement_columns     Sec. 4.2        where component r of a group is stored (RoPE key first)
  rotate_rows           Sec. 4.2        W^K and (W^UK)^T rotated by the same U
  kv_balance            Sec. 4.3        alpha
  joint_moment          App. D.2        second-moment matrix of [k_NoPE / alpha ; v]
  joint_basis           App. D.2        R_KV = leading r_kv eigenvectors
  low_rank_projections  App. D.2        W^DKV' = R^T W^DKV,  W^UKV' = W^UKV R
  convert_layer         the chain, returning the tensors the decode path consumes

Readings taken where the paper leaves a choice (each listed in the design notes):
  * Moments are NOT mean-centred: App. B defines sigma = K^T K, and App. D.2 says
    "covariance" without a centring step; the proposition of App. C holds for
    either.  A common factor 1/n does not change eigenvectors; moments here are
    divided by n.
  * App. C's example counts a "2g-dimensional segment" per pair, App. B fixes that one
    g x g matrix must act on the real and on the imaginary vector alike.  Here U of
    a group is (M g) x (M g) and acts identically on the real vector and on the
    imaginary vector of the group (the only reading under which Eq. "rorope" holds).
  * Where the components go.  Of every group the `keep` leading components (eigenvalues
    descending, 1 <= keep <= M) stay under RoPE; they form the RoPE key, a head of
    d_rope = 2 * keep * (d / 2M) dimensions in which component r of group G is pair
    G * keep + r.  With keep = M that is a whole head of d dimensions in which every
    component sits on one of its group's own M pairs, so ordinary RoPE of width d applies
    (exactly for M = 1, up to FreqFold's approximation otherwise).  With keep = 1 the
    RoPE key has one pair per group and ordinary RoPE of width d / M applies: its pair G
    turns with theta_{G M}, the first frequency of the group (the "effective frequency"
    of App. C's example).  All other components lose RoPE and form the NoPE key, component
    r >= keep of group G at NoPE pair (r - keep) * (d / 2M) + G.
  * Eigenvectors are unique up to sign (and up to a rotation inside a repeated
    eigenvalue): callers compare what is unique (eigenvalues, projectors,
    products that do not depend on the sign).

Parity pins: tests/test_convert_oracle_pins.py (index sets of App. C's worked
example, Eq. "rorope" invariance by brute-force RoPE, optimality of the
eigenbasis, the App. C proposition, exact conversion of a layer whose keys are
rank one across heads, exact recovery at full rank, closed-form 2x2 cases).
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------
# Sec. 4.1: merged key/value head with selector-identity up-projections
# --------------------------------------------------------------------------

def merged_projections(g: int, h: int, d: int):
    """W^UK_i, W^UV_i in R^{d x g d}: identity on the columns of query head i's
    group j = i // (h/g), zero elsewhere.  Returns (W_UK [h,d,gd], W_UV [h,d,gd])."""
    assert h % g == 0
    W_UK = np.zeros((h, d, g * d))
    for i in range(h):
        j = i // (h // g)
        W_UK[i, :, j * d:(j + 1) * d] = np.eye(d)
    return W_UK, W_UK.copy()


# --------------------------------------------------------------------------
# App. C: dimensions of a FreqFold group
# --------------------------------------------------------------------------

def group_columns(g: int, d: int, M: int):
    """Columns of the merged key (g d wide) that form group G's real and imaginary vectors.

    Returns (col_x, col_y), each [d/(2M), M*g] int: entry c = p*g + j is pair
    G*M + p of head j, i.e. column j*d + 2*(G*M+p) (real) and that + 1 (imaginary)."""
    assert d % 2 == 0 and (d // 2) % M == 0
    n_groups = d // (2 * M)
    col_x = np.empty((n_groups, M * g), dtype=np.int64)
    for G in range(n_groups):
        for p in range(M):
            for j in range(g):
                col_x[G, p * g + j] = j * d + 2 * (G * M + p)
    return col_x, col_x + 1


def rope_moments(K: np.ndarray, g: int, d: int, M: int = 1) -> np.ndarray:
    """sigma_x + sigma_y of every group (App. B), divided by n.  K: [n, g*d] key
    activations BEFORE RoPE.  Returns [d/(2M), M*g, M*g]."""
    K = np.asarray(K, dtype=np.float64)
    n = K.shape[0]
    col_x, col_y = group_columns(g, d, M)
    out = np.empty((col_x.shape[0], M * g, M * g))
    for G in range(col_x.shape[0]):
        Kx, Ky = K[:, col_x[G]], K[:, col_y[G]]
        out[G] = (Kx.T @ Kx + Ky.T @ Ky) / n
    return out


def sym_eig_desc(A: np.ndarray):
    """Symmetric eigendecomposition with eigenvalues in descending order and the
    eigenvectors in the columns (LAPACK through numpy)."""
    w, U = np.linalg.eigh(np.asarray(A, dtype=np.float64))
    return w[..., ::-1].copy(), U[..., ::-1].copy()


def rorope_basis(sigma: np.ndarray):
    """App. B: the trace of the leading m x m block of U^T sigma U is largest, for every m,
    when the columns of U are the eigenvectors by descending eigenvalue."""
    return sym_eig_desc(sigma)


# --------------------------------------------------------------------------
# Sec. 4.2: rotation of W^K and W^UK
# --------------------------------------------------------------------------

def rope_width(d: int, M: int, keep=None) -> int:
    """d_rope: dimensions of the RoPE key when `keep` components per group stay under RoPE."""
    keep = M if keep is None else keep
    assert 1 <= keep <= M
    return 2 * keep * (d // (2 * M))


def placement_columns(g: int, d: int, M: int, keep=None):
    """Rows of the rotated key: the RoPE key first (d_rope rows), then the NoPE key.
    Component r of group G: r < keep -> RoPE pair G*keep + r; else NoPE pair
    (r - keep) * n_groups + G, i.e. row d_rope + 2 * that (real), + 1 (imaginary)."""
    keep = M if keep is None else keep
    n_groups = d // (2 * M)
    d_rope = rope_width(d, M, keep)
    out_x = np.empty((n_groups, M * g), dtype=np.int64)
    for G in range(n_groups):
        for r in range(M * g):
            out_x[G, r] = 2 * (G * keep + r) if r < keep else d_rope + 2 * ((r - keep) * n_groups + G)
    return out_x, out_x + 1


def rotate_rows(W: np.ndarray, U: np.ndarray, g: int, d: int, M: int = 1, keep=None) -> np.ndarray:
    """Rows of W ([g*d, anything]) are indexed like the merged key.  The real vector
    and the imaginary vector of every group are replaced by U_G^T times themselves
    (k' = U^T k) and stored at the placement rows.  W^K is rotated as it stands;
    W^UK_i is rotated through its transpose (rows = merged key dimensions)."""
    W = np.asarray(W, dtype=np.float64)
    col_x, col_y = group_columns(g, d, M)
    out_x, out_y = placement_columns(g, d, M, keep)
    out = np.empty_like(W)
    for G in range(col_x.shape[0]):
        out[out_x[G]] = U[G].T @ W[col_x[G]]
        out[out_y[G]] = U[G].T @ W[col_y[G]]
    return out


# --------------------------------------------------------------------------
# Sec. 4.3 / App. D.1: key-value balancing
# --------------------------------------------------------------------------

def kv_balance(K_nope: np.ndarray, V: np.ndarray) -> float:
    """alpha = mean_t ||k_NoPE,t||_2 / mean_t ||v_t||_2."""
    kn = np.sqrt((np.asarray(K_nope, dtype=np.float64) ** 2).sum(axis=1)).mean()
    vn = np.sqrt((np.asarray(V, dtype=np.float64) ** 2).sum(axis=1)).mean()
    return float(kn / vn)


# --------------------------------------------------------------------------
# App. D.2: joint low-rank approximation
# --------------------------------------------------------------------------

def joint_moment(K_nope: np.ndarray, V: np.ndarray, alpha: float) -> np.ndarray:
    """Second-moment matrix of c_NoPE,t = [k_NoPE,t / alpha ; v_t], divided by n."""
    C = np.concatenate([np.asarray(K_nope, dtype=np.float64) / alpha,
                        np.asarray(V, dtype=np.float64)], axis=1)
    return C.T @ C / C.shape[0]


def joint_basis(S: np.ndarray, r_kv: int):
    """R_KV: the r_kv leading eigenvectors of S in columns, and all eigenvalues (descending)."""
    w, U = sym_eig_desc(S)
    return w, U[:, :r_kv].copy()


def low_rank_projections(W_DK_nope, W_DV, W_UK_nope, W_UV, alpha: float, R_KV: np.ndarray):
    """W^DKV' = R^T [W^DK_NoPE / alpha ; W^DV]          [r_kv, D]
    W^UK'_i = (alpha W^UK_NoPE,i) R_K                   [h, d, r_kv]   (R_K: first (g-1)d rows of R)
    W^UV'_i = W^UV_i R_V                                [h, d, r_kv]   (R_V: last g d rows of R)."""
    nk = W_DK_nope.shape[0]
    W_DKV = np.concatenate([np.asarray(W_DK_nope, dtype=np.float64) / alpha,
                            np.asarray(W_DV, dtype=np.float64)], axis=0)
    W_DKV_p = R_KV.T @ W_DKV
    W_UK_p = alpha * np.einsum("hdk,kr->hdr", W_UK_nope, R_KV[:nk])
    W_UV_p = np.einsum("hdk,kr->hdr", W_UV, R_KV[nk:])
    return W_DKV_p, W_UK_p, W_UV_p


# --------------------------------------------------------------------------
# the chain
# --------------------------------------------------------------------------

def convert_layer(X, W_K, W_V, g: int, h: int, d: int, M: int, r_kv: int, keep=None):
    """GQA layer (W_K, W_V: [g*d, D]) -> MLA layer, calibrated on the rows of X [n, D].
    keep (default M): components per FreqFold group that stay under RoPE; d_rope = keep * d / M.

    Returns a dict:
      W_KR   [d_rope, D]   key projection of the RoPE key (k_rope = RoPE(W_KR x), RoPE of width d_rope)
      W_QR   [h, d_rope, d]  q_rope_i = RoPE(W_QR[i] q_i)        (= (W^UK_RoPE,i)^T)
      W_DKV  [r_kv, D]     c_kv = W_DKV x
      W_UK   [h, d, r_kv]  q_abs_i = W_UK[i]^T q_i               (scores against c_kv)
      W_UV   [h, r_kv, d]  o_i = W_UV[i]^T-free form: o_i = o_lat_i @ W_UV[i]
      alpha, evals_rope [groups, M*g], evals_joint [2gd - d_rope], U [groups, Mg, Mg], R_KV."""
    X = np.asarray(X, dtype=np.float64)
    W_K = np.asarray(W_K, dtype=np.float64)
    W_V = np.asarray(W_V, dtype=np.float64)
    W_UK, W_UV = merged_projections(g, h, d)                       # Sec. 4.1
    K = X @ W_K.T                                                  # key activations before RoPE
    evals_rope, U = rorope_basis(rope_moments(K, g, d, M))         # App. B (+ App. C grouping)
    d_rope = rope_width(d, M, keep)
    W_K_rot = rotate_rows(W_K, U, g, d, M, keep)                   # Sec. 4.2
    W_UK_rot = np.stack([rotate_rows(W_UK[i].T, U, g, d, M, keep).T for i in range(h)])
    W_KR, W_DK_nope = W_K_rot[:d_rope], W_K_rot[d_rope:]           # the RoPE key, the NoPE key
    W_QR = np.stack([W_UK_rot[i][:, :d_rope].T for i in range(h)])
    W_UK_nope = W_UK_rot[:, :, d_rope:]
    K_nope, V = X @ W_DK_nope.T, X @ W_V.T
    alpha = kv_balance(K_nope, V)                                  # Sec. 4.3
    evals_joint, R_KV = joint_basis(joint_moment(K_nope, V, alpha), r_kv)   # App. D.2
    W_DKV_p, W_UK_p, W_UV_p = low_rank_projections(W_DK_nope, W_V, W_UK_nope, W_UV, alpha, R_KV)
    return dict(W_KR=W_KR, W_QR=W_QR, W_DKV=W_DKV_p, W_UK=W_UK_p,
                W_UV=np.ascontiguousarray(W_UV_p.transpose(0, 2, 1)),
                alpha=alpha, evals_rope=evals_rope, evals_joint=evals_joint, U=U, R_KV=R_KV)
