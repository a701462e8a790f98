"""GPU parity of the offline conversion (include/mla_convert_gfx950.h) against the numpy
oracle (oracle/convert_oracle.py), entry point by entry point and as a chain, through
the C ABI.  Eigenvectors are unique up to sign (and inside a repeated eigenvalue up to a
rotation), so those tests compare eigenvalues, projectors and sign-free products, and
check orthonormality and the eigen-equation directly.

Tolerances (fp64 on both sides; the two differ in summation order only): 1e-11 relative
for sums of at most a few thousand products, 1e-9 for eigenvalues and for quantities that
pass through an eigenbasis (error ~ rounding / relative gap)."""
import numpy as np
import pytest

from oracle import convert_oracle as co
from workloads import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cv():
    import torch
    assert torch.cuda.is_available()
    from paper_2502_07864_amd import convert
    convert.lib()
    return convert


def dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float64)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def rel(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ matrix product (activations)

@pytest.mark.parametrize("n,D,m", [(300, 200, 150), (1, 7, 3), (128, 16, 128), (129, 17, 257), (1000, 513, 64)])
def test_project_matches_numpy(cv, n, D, m):
    r = rng(n + D)
    X, W = r.standard_normal((n, D)), r.standard_normal((m, D))
    got = host(cv.project(dev(X), dev(W)))
    assert rel(got, X @ W.T) < 1e-12


# ------------------------------------------------------------------ App. B / C moments

@pytest.mark.parametrize("g,d,M,n", [(4, 16, 1, 100), (4, 16, 2, 37), (3, 12, 3, 64), (8, 64, 4, 200),
                                     (32, 128, 1, 130), (32, 128, 4, 48), (2, 8, 1, 1)])
def test_rope_moments(cv, g, d, M, n):
    K = rng(g * d + M).standard_normal((n, g * d))
    got = host(cv.rope_moments(dev(K), g, d, M))
    want = co.rope_moments(K, g, d, M)
    assert got.shape == want.shape and rel(got, want) < 1e-12


# ------------------------------------------------------------------ eigensolver

def check_eig(A, evals, U, info, tol=1e-10):
    m = A.shape[-1]
    for b in range(A.shape[0]):
        scale = max(np.linalg.norm(A[b]), 1e-300)
        w_ref, _ = co.sym_eig_desc(A[b])
        assert info[b] >= 1, f"matrix {b}: not converged"
        assert np.abs(evals[b] - w_ref).max() <= tol * scale
        assert (np.diff(evals[b]) <= 0).all()
        assert np.abs(U[b].T @ U[b] - np.eye(m)).max() < 1e-12 * m
        assert np.abs(A[b] @ U[b] - U[b] * evals[b]).max() <= tol * scale


@pytest.mark.parametrize("batch,m", [(3, 2), (4, 5), (64, 32), (5, 64), (2, 80), (2, 96), (3, 128), (2, 130),
                                     (1, 257), (1, 512)])
def test_sym_eig_random(cv, batch, m):
    r = rng(m)
    A = r.standard_normal((batch, m, m))
    A = A + A.transpose(0, 2, 1)
    if batch > 1:                                      # one positive semi-definite, rank-deficient member
        B = r.standard_normal((m, max(1, m // 2)))
        A[1] = B @ B.T
    evals, U, info = cv.sym_eig(dev(A))
    check_eig(A, host(evals), host(U), host(info))


def test_sym_eig_degenerate_cases(cv):
    m = 12
    r = rng(99)
    Q, _ = np.linalg.qr(r.standard_normal((m, m)))
    A = np.stack([np.eye(m) * 3.0,                                   # all eigenvalues equal
                  np.zeros((m, m)),                                  # zero matrix
                  np.diag(np.arange(m, dtype=np.float64)),           # already diagonal, ascending
                  Q @ np.diag([5.0] * 4 + [2.0] * 4 + [-1.0] * 4) @ Q.T,   # repeated eigenvalues
                  np.full((m, m), 1.0)])                             # rank one
    evals, U, info = cv.sym_eig(dev(A))
    check_eig(A, host(evals), host(U), host(info))
    assert np.allclose(host(evals)[2], np.arange(m)[::-1], atol=1e-13)


def test_sym_eig_rorope_bases_have_the_oracles_projectors(cv):
    """The use made of it in App. B: bases of the per-group moments of synthetic key activations."""
    g, d, M, n = 8, 32, 2, 256
    X, W_K, _ = synth.calibration(n, 96, g, d, seed=3)
    sigma = co.rope_moments(X @ W_K.T, g, d, M)
    evals, U, info = cv.sym_eig(dev(sigma))
    evals, U = host(evals), host(U)
    w_ref, U_ref = co.rorope_basis(sigma)
    check_eig(sigma, evals, U, host(info))
    for G in range(sigma.shape[0]):
        for c in range(M * g):                          # distinct eigenvalues: columns agree up to sign
            assert abs(abs(U[G][:, c] @ U_ref[G][:, c]) - 1.0) < 1e-8


# ------------------------------------------------------------------ Sec. 4.2 / 4.3 / D.2 steps

@pytest.mark.parametrize("g,d,M,keep,cols", [(4, 16, 1, 1, 50), (4, 16, 2, 2, 33), (4, 16, 2, 1, 33), (3, 12, 3, 2, 7),
                                             (8, 64, 4, 4, 100), (8, 64, 4, 1, 100), (32, 128, 1, 1, 40), (32, 128, 2, 1, 40)])
def test_rotate_rows(cv, g, d, M, keep, cols):
    r = rng(g + d + M)
    W = r.standard_normal((g * d, cols))
    U = r.standard_normal((d // (2 * M), M * g, M * g))
    got = host(cv.rotate_rows(dev(W), dev(U), g, d, M, keep))
    assert rel(got, co.rotate_rows(W, U, g, d, M, keep)) < 1e-12


@pytest.mark.parametrize("n,a,b", [(100, 48, 64), (1, 3, 5), (333, 130, 7)])
def test_kv_balance_and_joint_moment(cv, n, a, b):
    r = rng(n + a)
    K_nope, V = 2.5 * r.standard_normal((n, a)), r.standard_normal((n, b))
    alpha, norms = cv.kv_balance(dev(K_nope), dev(V))
    want = co.kv_balance(K_nope, V)
    assert abs(host(alpha)[0] - want) < 1e-13 * want
    assert rel(host(norms)[0], np.linalg.norm(K_nope, axis=1)) < 1e-13
    S, C = cv.joint_moment(dev(K_nope), dev(V), alpha)
    assert rel(host(S), co.joint_moment(K_nope, V, want)) < 1e-12
    assert rel(host(C), np.concatenate([K_nope / want, V], axis=1)) < 1e-13


def projector_gap(R, R_ref):
    return np.abs(R @ R.T - R_ref @ R_ref.T).max()


@pytest.mark.parametrize("m,r,p,iters", [(60, 8, 16, 40), (200, 40, 64, 60), (300, 17, 33, 60), (40, 40, 40, 2),
                                         (700, 130, 160, 120), (1500, 64, 200, 30)])
def test_top_eig_against_full_eigendecomposition(cv, m, r, p, iters):
    rs = rng(m + r)
    Q, _ = np.linalg.qr(rs.standard_normal((m, m)))
    lam = (1.0 + np.arange(m)) ** -1.5
    S = (Q * lam) @ Q.T
    S = 0.5 * (S + S.T)
    evals, R, info = cv.top_eig(dev(S), dev(synth.start_block(m, p, seed=m)), r, iters)
    evals, R, info = host(evals), host(R), host(info)
    w_ref, R_ref = co.joint_basis(S, r)
    assert info[0] == 0 and info[1] >= 1
    assert np.abs(R.T @ R - np.eye(r)).max() < 1e-12
    assert np.abs(evals[:r] - w_ref[:r]).max() < 1e-10 * w_ref[0]
    assert projector_gap(R, R_ref) < 1e-8
    assert np.abs(S @ R - R * evals[:r]).max() < 1e-9 * w_ref[0]
    assert rel(host(cv.apply(dev(S), dev(R))), S @ R) < 1e-12


def test_apply_with_k_slices_matches_the_plain_product(cv):
    """A tall block on a matrix large enough that the library slices the K range when given scratch."""
    import torch
    m, p = 2304, 192                                    # 18 x 2 tiles: under a third of the CUs without slices
    rs = rng(5)
    S = rs.standard_normal((m, m))
    S = S + S.T
    Q = rs.standard_normal((m, p))
    ws = torch.empty(cv.apply_workspace_bytes(m, p), dtype=torch.uint8, device="cuda")
    want = S @ Q
    assert rel(host(cv.apply(dev(S), dev(Q), workspace=ws)), want) < 1e-12
    assert rel(host(cv.apply(dev(S), dev(Q))), want) < 1e-12


# ------------------------------------------------------------------ the chain

def chain_case(g, h, d, D, n, M, keep, r_kv, p, seed):
    X, W_K, W_V = synth.calibration(n, D, g, d, seed=seed)
    Q0 = synth.start_block(2 * g * d - co.rope_width(d, M, keep), p, seed=seed)
    return X, W_K, W_V, Q0


@pytest.mark.parametrize("g,h,d,D,n,M,keep,r_kv,p", [(4, 8, 16, 96, 512, 1, 1, 40, 56), (4, 8, 16, 96, 512, 2, 2, 40, 56),
                                                     (4, 8, 16, 96, 512, 2, 1, 40, 56), (2, 6, 8, 40, 200, 4, 4, 12, 20),
                                                     (2, 6, 8, 40, 200, 4, 1, 12, 20), (8, 8, 32, 128, 300, 1, 1, 64, 96),
                                                     (8, 8, 32, 128, 300, 4, 2, 64, 96)])
def test_convert_layer_against_the_oracle_chain(cv, g, h, d, D, n, M, keep, r_kv, p):
    X, W_K, W_V, Q0 = chain_case(g, h, d, D, n, M, keep, r_kv, p, seed=g + M)
    out = cv.convert_layer(dev(X), dev(W_K), dev(W_V), dev(Q0), g, h, d, M, r_kv, iters=80, keep=keep)
    got = {k: host(v) for k, v in out.items()}
    want = co.convert_layer(X, W_K, W_V, g, h, d, M, r_kv, keep)
    groups = d // (2 * M)
    d_rope = co.rope_width(d, M, keep)
    assert got["W_KR"].shape == (d_rope, D) and got["W_QR"].shape == (h, d_rope, d)
    assert (got["info"][:groups] >= 1).all() and got["info"][groups] == 0 and got["info"][groups + 1] >= 1
    assert abs(got["alpha"][0] - want["alpha"]) < 1e-11 * want["alpha"]
    assert rel(got["evals_rope"], want["evals_rope"]) < 1e-10
    assert np.abs(got["evals_joint"][:r_kv] - want["evals_joint"][:r_kv]).max() < 1e-9 * want["evals_joint"][0]
    # A sign flip of a RoRoPE basis vector flips one coordinate of the rotated key, hence one row of
    # R_KV: undo those flips (read off the two sets of bases) before comparing the projectors.
    sign = np.sign(np.einsum("gcr,gcr->gr", got["U"], want["U"]))
    out_x, out_y = co.placement_columns(g, d, M, keep)
    flip = np.ones(2 * g * d - d_rope)
    for G in range(groups):
        for r in range(M * g):
            for row in (out_x[G, r], out_y[G, r]):
                if row >= d_rope:
                    flip[row - d_rope] = sign[G, r]
    assert projector_gap(got["R_KV"] * flip[:, None], want["R_KV"]) < 1e-7
    # sign-free products.  Rope head: row a of W_QR[i] and row a of W_KR flip together.
    for i in range(h):
        assert rel(np.einsum("ab,ac->abc", got["W_QR"][i], got["W_KR"]),
                   np.einsum("ab,ac->abc", want["W_QR"][i], want["W_KR"])) < 1e-8
        # latent: W_UK[i] W_DKV and W_UV[i]^T W_DKV depend on the projector R R^T only
        assert rel(got["W_UK"][i] @ got["W_DKV"], want["W_UK"][i] @ want["W_DKV"]) < 1e-7
        assert rel(got["W_UV"][i].T @ got["W_DKV"], want["W_UV"][i].T @ want["W_DKV"]) < 1e-7
    # and the properties that hold whatever the oracle says
    R = got["R_KV"]
    assert np.abs(R.T @ R - np.eye(r_kv)).max() < 1e-11
    for G in range(groups):
        assert np.abs(got["U"][G].T @ got["U"][G] - np.eye(M * g)).max() < 1e-11


# ------------------------------------------------------------------ converted layer through the decode calls

def decode_converted_layer_on_gpu(out, X_ctx, q, d, pos_new, theta, page_size=64):
    """Cache rows and queries of the converted layer (built here in numpy from the GPU's converted
    weights: plain projections and RoPE, the inputs of the decode calls), then mla_absorb_q ->
    mla_decode_paged -> mla_out_proj in fp32 on the GPU."""
    import torch
    from paper_2502_07864_amd import mla
    from test_convert_oracle_pins import rope_hat
    W = {k: host(v) for k, v in out.items()}
    h = q.shape[0]
    L = len(X_ctx)
    d_r = W["W_KR"].shape[0]                                    # width of the RoPE key; theta: its d_r / 2 frequencies
    assert len(theta) == d_r // 2
    c_kv = X_ctx @ W["W_DKV"].T
    k_rope = np.stack([rope_hat(W["W_KR"] @ X_ctx[t], t, d_r, theta) for t in range(L)])
    q_rope = np.stack([rope_hat(W["W_QR"][i] @ q[i], pos_new, d_r, theta) for i in range(h)])
    d_c = c_kv.shape[1]
    pages = (L + page_size - 1) // page_size
    pool = np.zeros((pages + 1, page_size, d_c + d_r), dtype=np.float32)
    order = np.arange(pages)[::-1] + 1                          # pages stored in reverse, page 0 unused
    for t in range(L):
        pool[order[t // page_size], t % page_size] = np.concatenate([c_kv[t], k_rope[t]])
    f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    q_abs = mla.absorb_q(f32(q[None]), f32(W["W_UK"]))
    o_lat = mla.decode_paged(q_abs, f32(q_rope[None]), f32(pool), torch.from_numpy(order[None].astype(np.int32)).cuda(),
                             torch.tensor([L], dtype=torch.int32, device="cuda"), 1.0 / np.sqrt(d), num_splits=2)
    return host(mla.out_proj(o_lat, f32(W["W_UV"])))[0].astype(np.float64)


def test_gpu_conversion_then_gpu_decode_reproduces_gqa_when_nothing_is_lost(cv):
    """Positions zero (RoPE is the identity) and r_kv = (2g-1)d: the layer converted on the GPU and
    decoded by the GPU's absorbed path must give the textbook GQA attention output."""
    from test_convert_oracle_pins import gqa_attention
    g, h, d, D, n, L = 2, 4, 8, 12, 64, 70
    r = rng(37)
    X = r.standard_normal((n, D))
    W_Q, W_K, W_V = (r.standard_normal((m, D)) / np.sqrt(D) for m in (h * d, g * d, g * d))
    theta = np.zeros(d // 2)
    mj = (2 * g - 1) * d
    out = cv.convert_layer(dev(X), dev(W_K), dev(W_V), dev(synth.start_block(mj, mj, seed=2)), g, h, d, 1, mj, iters=2)
    X_ctx = r.standard_normal((L, D))
    want = gqa_attention(X_ctx[-1], X_ctx, W_Q, W_K, W_V, g, h, d, L - 1, theta)
    got = decode_converted_layer_on_gpu(out, X_ctx, (W_Q @ X_ctx[-1]).reshape(h, d), d, L - 1, theta)
    assert np.abs(got - want).max() < 2e-5 * max(1.0, np.abs(want).max())


@pytest.mark.parametrize("M,keep", [(1, 1), (2, 2), (2, 1)])
def test_gpu_converted_layer_decodes_like_the_oracles_converted_layer(cv, M, keep):
    """Truncated rank and real positions: the attention output of the converted layer does not depend on
    the signs of the bases, so GPU conversion + GPU decode must match numpy conversion + the decode oracle.
    The RoPE key takes ordinary RoPE of its own width (d for keep = M, d / M for keep = 1)."""
    from test_convert_oracle_pins import mla_attention_through_the_decode_oracle, std_theta
    g, h, d, D, n, L, r_kv, p = 4, 8, 16, 64, 400, 150, 40, 56
    X, W_K, W_V = synth.calibration(n, D, g, d, seed=11 + M)
    r = rng(43)
    W_Q = r.standard_normal((h * d, D)) / np.sqrt(D)
    X_ctx = synth.calibration(L, D, g, d, seed=13)[0]
    d_rope = co.rope_width(d, M, keep)
    theta = std_theta(d_rope)
    mj = 2 * g * d - d_rope
    out = cv.convert_layer(dev(X), dev(W_K), dev(W_V), dev(synth.start_block(mj, p, seed=3)), g, h, d, M, r_kv, iters=80,
                           keep=keep)
    ref = co.convert_layer(X, W_K, W_V, g, h, d, M, r_kv, keep)
    want = mla_attention_through_the_decode_oracle(ref, X_ctx[-1], X_ctx, W_Q, h, d, L - 1, theta)
    got = decode_converted_layer_on_gpu(out, X_ctx, (W_Q @ X_ctx[-1]).reshape(h, d), d, L - 1, theta)
    assert np.abs(got - want).max() < 2e-5 * max(1.0, np.abs(want).max())


# ------------------------------------------------------------------ the benchmark shape, by properties

def test_convert_layer_at_the_llama2_7b_layer_shape_by_properties(cv):
    """One layer at the shape bench.py times (g = h = 32, d = 128, D = 4096, 4096 tokens, 2-fold FreqFold
    with one RoPE pair per group, r_kv = 512 -- the 512 + 64 row of the decode path --, block 768,
    20 iterations).  The oracle's eigensolver would take minutes here, so the GPU result is
    checked against what must hold at any size, with the moments recomputed in numpy:
    orthogonal bases that diagonalise the per-group moments, Eq. "rorope" on sampled scores (with the
    group's frequency on all its components, FreqFold's premise), alpha, an orthonormal R_KV whose
    columns are eigenpairs of the numpy moment matrix to the iteration's accuracy, Ritz values above
    every Rayleigh quotient of random directions, and the App. D.2 products."""
    from test_convert_oracle_pins import rope_by_component, rope_hat, std_theta
    g = h = 32
    d, D, n, M, keep, r_kv, p, iters = 128, 4096, 4096, 2, 1, 512, 768, 20
    d_rope = co.rope_width(d, M, keep)
    a_nope = g * d - d_rope
    mj = a_nope + g * d
    X, W_K, W_V = synth.calibration(n, D, g, d, seed=0)
    out = cv.convert_layer(dev(X), dev(W_K), dev(W_V), dev(synth.start_block(mj, p, seed=0)), g, h, d, M, r_kv, iters,
                           keep=keep)
    got = {k: host(v) for k, v in out.items()}
    assert got["W_KR"].shape == (64, D) and got["W_DKV"].shape == (512, D)
    assert (got["info"][:-2] >= 1).all() and got["info"][-2] == 0 and got["info"][-1] >= 1
    U, ev = got["U"], got["evals_rope"]
    # App. B: orthogonal, descending, and diagonalising the moments of the numpy activations
    K = X @ W_K.T
    sigma = co.rope_moments(K, g, d, M)
    for G in (0, 17, 31):
        assert np.abs(U[G].T @ U[G] - np.eye(M * g)).max() < 1e-12
        assert (np.diff(ev[G]) <= 0).all()
        assert np.abs(U[G].T @ sigma[G] @ U[G] - np.diag(ev[G])).max() < 1e-10 * ev[G][0]
    # Eq. "rorope" under FreqFold's premise: sampled scores of the rotated merged query / key equal the unrotated ones
    r = rng(3)
    theta = std_theta(d)
    theta_folded = np.repeat(theta[::M], M)
    folded = lambda G, rr: theta[G * M]
    W_K_rot = co.rotate_rows(W_K, U, g, d, M, keep)
    assert rel(got["W_KR"], W_K_rot[:d_rope]) < 1e-12
    for trial in range(3):
        x_k, q_hat = X[r.integers(n)], r.standard_normal(g * d)
        q_rot = co.rotate_rows(q_hat[:, None], U, g, d, M, keep)[:, 0]
        t, j = int(r.integers(4096)), int(r.integers(4096))
        want = rope_hat(q_hat, t, d, theta_folded) @ rope_hat(W_K @ x_k, j, d, theta_folded)
        have = rope_by_component(q_rot, t, g, d, M, keep, folded) @ rope_by_component(W_K_rot @ x_k, j, g, d, M, keep, folded)
        assert abs(have - want) < 1e-9 * (1 + abs(want))
    # Sec. 4.3 and App. D.2 against numpy moments
    K_nope, V = X @ W_K_rot[d_rope:].T, X @ W_V.T
    alpha = co.kv_balance(K_nope, V)
    assert abs(got["alpha"][0] - alpha) < 1e-11 * alpha
    S = co.joint_moment(K_nope, V, alpha)
    R, lam = got["R_KV"], got["evals_joint"]
    assert R.shape == (mj, r_kv)
    assert np.abs(R.T @ R - np.eye(r_kv)).max() < 1e-11
    assert (np.diff(lam) <= 0).all()
    resid = np.linalg.norm(S @ R - R * lam[:r_kv], axis=0).max() / lam[0]
    assert resid < 1e-8, resid                       # what 20 iterations of a 768-wide block leave on this spectrum
    assert lam[:r_kv].sum() <= np.trace(S) * (1 + 1e-12)
    Qr, _ = np.linalg.qr(r.standard_normal((mj, 8)))
    assert (np.einsum("ij,ij->j", Qr, S @ Qr) <= lam[0] * (1 + 1e-9)).all()
    # the products of App. D.2 from the GPU's own R_KV (exact identities, whatever the basis)
    W_cat = np.concatenate([W_K_rot[d_rope:] / alpha, W_V])
    assert rel(got["W_DKV"], R.T @ W_cat) < 1e-11
    i = 5
    E_i = np.zeros((g * d, d))
    E_i[i * d:(i + 1) * d] = np.eye(d)                # (W^UK_i)^T for h = g
    E_rot = co.rotate_rows(E_i, U, g, d, M, keep)
    assert rel(got["W_UK"][i], alpha * E_rot[d_rope:].T @ R[:a_nope]) < 1e-11
    assert rel(got["W_QR"][i], E_rot[:d_rope]) < 1e-12
    assert rel(got["W_UV"][i], R[a_nope + i * d:a_nope + (i + 1) * d].T) == 0.0


def test_whole_pipeline_on_the_gpu_conversion_append_decode(cv):
    """Conversion, cache append (projection + RoPE + paged store) and absorbed decode all on the GPU,
    token by token for three sequences of different lengths, against numpy conversion + numpy cache
    rows + the decode oracle.  The attention output is independent of the signs of the bases."""
    import torch
    from paper_2502_07864_amd import mla
    from test_convert_oracle_pins import mla_attention_through_the_decode_oracle, rope_hat, std_theta
    g, h, d, D, n, r_kv, p, M = 4, 8, 16, 64, 400, 40, 56, 1
    lens = [70, 33, 1]
    B = len(lens)
    X, W_K, W_V = synth.calibration(n, D, g, d, seed=21)
    r = rng(47)
    W_Q = r.standard_normal((h * d, D)) / np.sqrt(D)
    ctx = [synth.calibration(L, D, g, d, seed=30 + b)[0] for b, L in enumerate(lens)]
    theta = std_theta(d)
    mj = (2 * g - 1) * d
    out = cv.convert_layer(dev(X), dev(W_K), dev(W_V), dev(synth.start_block(mj, p, seed=4)), g, h, d, M, r_kv, iters=80)
    f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    # cache rows through mla_cache_append: W_DKVR = [W_DKV^T | W_KR^T]
    W_DKVR = torch.cat([out["W_DKV"].T, out["W_KR"].T], dim=1).to(torch.float32).contiguous()
    pages_per_seq = 2
    pool = torch.full((B * pages_per_seq + 1, 64, r_kv + d), float("nan"), dtype=torch.float32, device="cuda")
    table = torch.tensor([[5, 2], [1, 6], [4, 3]], dtype=torch.int32, device="cuda")
    for t in range(max(lens)):
        x_t = np.stack([ctx[b][t] if t < lens[b] else np.zeros(D) for b in range(B)])
        pos = torch.tensor([t if t < lens[b] else -1 for b in range(B)], dtype=torch.int32, device="cuda")
        mla.cache_append(f32(x_t), W_DKVR, pool, table, pos, r_kv)
    # queries of the newest token of every sequence
    q = np.stack([(W_Q @ ctx[b][-1]).reshape(h, d) for b in range(B)])
    W_QR = host(out["W_QR"])
    q_rope = np.stack([[rope_hat(W_QR[i] @ q[b, i], lens[b] - 1, d, theta) for i in range(h)] for b in range(B)])
    q_abs = mla.absorb_q(f32(q), out["W_UK"].to(torch.float32).contiguous())
    o_lat = mla.decode_paged(q_abs, f32(q_rope), pool, table, torch.tensor(lens, dtype=torch.int32, device="cuda"),
                             1.0 / np.sqrt(d), num_splits=2)
    got = host(mla.out_proj(o_lat, out["W_UV"].to(torch.float32).contiguous())).astype(np.float64)
    ref = co.convert_layer(X, W_K, W_V, g, h, d, M, r_kv)
    for b in range(B):
        want = mla_attention_through_the_decode_oracle(ref, ctx[b][-1], ctx[b], W_Q, h, d, lens[b] - 1, theta)
        assert np.abs(got[b] - want).max() < 5e-5 * max(1.0, np.abs(want).max()), b


# ------------------------------------------------------------------ error reporting through info (forced from the host)

def test_top_eig_reports_a_start_block_that_lacks_rank(cv):
    """Two equal columns in the caller's start block: the Cholesky pivot of the second is clamped and
    counted in info[0]; nothing hangs and nothing is NaN."""
    m, r, p = 96, 8, 16
    rs = rng(71)
    B = rs.standard_normal((m, m))
    S = B @ B.T / m
    Q0 = synth.start_block(m, p, seed=9)
    Q0[:, 5] = Q0[:, 4]
    evals, R, info = cv.top_eig(dev(S), dev(Q0), r, 10)
    assert host(info)[0] >= 1
    assert np.isfinite(host(evals)).all() and np.isfinite(host(R)).all()


def test_sym_eig_reports_a_sweep_limit_that_is_too_low(cv):
    """One sweep does not diagonalise a random matrix: info = -1, the output is still an orthogonal matrix."""
    for m in (24, 200):                                 # single-workgroup path and chip-wide path
        A = rng(m).standard_normal((1, m, m))
        A = A + A.transpose(0, 2, 1)
        evals, U, info = cv.sym_eig(dev(A), max_sweeps=1)
        assert host(info)[0] == -1
        U = host(U)[0]
        assert np.abs(U.T @ U - np.eye(m)).max() < 1e-12
        evals_ok, _, info_ok = cv.sym_eig(dev(A), max_sweeps=40)
        assert host(info_ok)[0] >= 2
        assert np.abs(host(evals_ok)[0] - co.sym_eig_desc(A[0])[0]).max() < 1e-10 * np.linalg.norm(A[0])


def test_convert_layer_with_the_widest_fold(cv):
    """M g = 128, the limit of the per-group kernels (32 heads folded by 4)."""
    g, h, d, D, n, M, r_kv, p = 32, 32, 16, 160, 300, 4, 96, 112
    X, W_K, W_V = synth.calibration(n, D, g, d, seed=8)
    out = cv.convert_layer(dev(X), dev(W_K), dev(W_V), dev(synth.start_block((2 * g - 1) * d, p, seed=8)),
                           g, h, d, M, r_kv, iters=60)
    got = {k: host(v) for k, v in out.items()}
    want = co.convert_layer(X, W_K, W_V, g, h, d, M, r_kv)
    assert (got["info"][:-2] >= 1).all() and got["info"][-2] == 0 and got["info"][-1] >= 1
    assert rel(got["evals_rope"], want["evals_rope"]) < 1e-10
    assert abs(got["alpha"][0] - want["alpha"]) < 1e-11 * want["alpha"]
    assert np.abs(got["evals_joint"][:r_kv] - want["evals_joint"][:r_kv]).max() < 1e-9 * want["evals_joint"][0]
    for i in (0, 13, 31):
        assert rel(got["W_UK"][i] @ got["W_DKV"], want["W_UK"][i] @ want["W_DKV"]) < 1e-6
        assert rel(np.einsum("ab,ac->abc", got["W_QR"][i], got["W_KR"]),
                   np.einsum("ab,ac->abc", want["W_QR"][i], want["W_KR"])) < 1e-7


def test_folding_never_captures_less_than_separate_bases_on_the_gpu(cv):
    """Proposition of App. C on the GPU's own moments and eigenvalues: the M leading eigenvalues of a folded
    group's moment sum to at least the leading eigenvalues of its M pairs taken separately."""
    g, d, n = 8, 32, 500
    X, W_K, _ = synth.calibration(n, 96, g, d, seed=17)
    K = cv.project(dev(X), dev(W_K))
    w1 = host(cv.sym_eig(cv.rope_moments(K, g, d, 1))[0])
    for M in (2, 4, 8):
        wM = host(cv.sym_eig(cv.rope_moments(K, g, d, M))[0])
        for G in range(d // (2 * M)):
            assert wM[G, :M].sum() >= w1[G * M:(G + 1) * M, 0].sum() * (1 - 1e-12)
        # folding moves energy between components, not in or out: the traces agree
        assert abs(wM.sum() - w1.sum()) < 1e-10 * w1.sum()


def test_matrix_product_random_shapes(cv):
    """Ragged sizes through the three transpose cases the chain uses (X W^T, C^T C, S Q with and without K
    slices): primes, single rows and columns, sizes straddling the 128 x 128 x 16 tile."""
    import torch
    r = rng(2024)
    for case in range(12):
        n, D, m = (int(v) for v in r.choice([1, 2, 3, 15, 16, 17, 31, 127, 128, 129, 257, 400], size=3))
        X, W = r.standard_normal((n, D)), r.standard_normal((m, D))
        assert rel(host(cv.project(dev(X), dev(W))), X @ W.T) < 1e-12, (case, n, D, m)
        a, b = max(1, m // 2), m - m // 2 if m > 1 else 1
        Kn, V = r.standard_normal((n, a)), r.standard_normal((n, b))
        S, _ = cv.joint_moment(dev(Kn), dev(V), dev(np.array([1.0])))
        C = np.concatenate([Kn, V], axis=1)
        assert rel(host(S), C.T @ C / n) < 1e-12, (case, n, a, b)
        mm, p = D, max(1, m // 3)
        A = r.standard_normal((mm, mm))
        Q = r.standard_normal((mm, p))
        ws = torch.empty(max(256, cv.apply_workspace_bytes(mm, p)), dtype=torch.uint8, device="cuda")
        assert rel(host(cv.apply(dev(A), dev(Q))), A @ Q) < 1e-12, (case, mm, p)
        assert rel(host(cv.apply(dev(A), dev(Q), workspace=ws)), A @ Q) < 1e-12, (case, mm, p)


def test_largest_orders_the_solvers_take(cv):
    """Order 2048 for the eigensolver (its limit) and block width 1024 for the power iteration (its limit)."""
    m = 2048
    r = rng(77)
    B = r.standard_normal((m, 300))
    A = (B @ B.T / 300 + np.diag(np.linspace(0.0, 2.0, m)))[None]
    evals, U, info = cv.sym_eig(dev(A), max_sweeps=16)
    evals, U = host(evals)[0], host(U)[0]
    assert host(info)[0] >= 1
    w_ref = np.linalg.eigvalsh(A[0])[::-1]
    assert np.abs(evals - w_ref).max() < 1e-10 * w_ref[0]
    assert np.abs(U.T @ U - np.eye(m)).max() < 1e-11
    assert np.abs(A[0] @ U - U * evals).max() < 1e-10 * w_ref[0]
    m2, r2, p2 = 1300, 600, 1024
    Qo, _ = np.linalg.qr(r.standard_normal((m2, m2)))
    lam = (1.0 + np.arange(m2)) ** -1.2
    S = (Qo * lam) @ Qo.T
    S = 0.5 * (S + S.T)
    ev2, R, info2 = cv.top_eig(dev(S), dev(synth.start_block(m2, p2, seed=12)), r2, 40)
    ev2, R = host(ev2), host(R)
    assert host(info2)[0] == 0 and host(info2)[1] >= 1
    assert np.abs(ev2[:r2] - lam[:r2]).max() < 1e-10
    assert np.abs(R.T @ R - np.eye(r2)).max() < 1e-11
    assert np.abs(S @ R - R * ev2[:r2]).max() < 1e-9


def test_converted_gqa_layer_runs_on_the_matrix_core_decode_path(cv):
    """A GQA layer with 128-dimensional heads (g = 8 key/value heads, h = 32 query heads, as LLaMA-3-8B has
    them) converted with 2-fold FreqFold and one RoPE pair per group lands exactly on the decode path's
    headline shape: latent 512 + RoPE key 64, 32 heads of 128.  Conversion in fp64 on the GPU, weights
    rounded to bf16, cache rows written by mla_cache_append into a bf16 paged cache, decode on the
    matrix-core kernels -- against the numpy conversion fed to the decode oracle (the attention output
    does not depend on the signs of the bases).  bf16 bar of the decode path: 2e-2."""
    import torch
    from helpers import max_abs_rel, to_torch, widen_gpu
    from paper_2502_07864_amd import mla
    from test_convert_oracle_pins import mla_attention_through_the_decode_oracle, rope_hat, std_theta
    g, h, d, D, n, M, keep, r_kv, p = 8, 32, 128, 1024, 2048, 2, 1, 512, 640
    d_rope = co.rope_width(d, M, keep)
    assert d_rope == 64
    mj = 2 * g * d - d_rope
    lens = [300, 129, 64]
    B = len(lens)
    bf16 = lambda a: synth.bf16_bits_to_f32(synth.to_bf16_bits(np.asarray(a, dtype=np.float32))).astype(np.float64)
    X, W_K, W_V = synth.calibration(n, D, g, d, seed=23)
    r = rng(59)
    W_Q = r.standard_normal((h * d, D)) / np.sqrt(D)
    ctx = [bf16(synth.calibration(L, D, g, d, seed=40 + b)[0]) for b, L in enumerate(lens)]   # hidden states as stored
    theta = std_theta(d_rope)
    out = cv.convert_layer(dev(X), dev(W_K), dev(W_V), dev(synth.start_block(mj, p, seed=6)), g, h, d, M, r_kv, iters=40,
                           keep=keep)
    info = host(out["info"])
    assert (info[:-2] >= 1).all() and info[-2] == 0 and info[-1] >= 1
    tb = lambda t: t.to(torch.bfloat16).contiguous()
    W_DKVR = tb(torch.cat([out["W_DKV"].T, out["W_KR"].T], dim=1))              # [D, 512 + 64]
    pages_per_seq = 5
    pool = torch.full((B * pages_per_seq + 1, 64, r_kv + d_rope), float("nan"), dtype=torch.bfloat16, device="cuda")
    table = torch.from_numpy(rng(5).permutation(B * pages_per_seq).reshape(B, pages_per_seq).astype(np.int32) + 1).cuda()
    for t in range(max(lens)):
        x_t = np.stack([ctx[b][t] if t < lens[b] else np.zeros(D) for b in range(B)])
        pos = torch.tensor([t if t < lens[b] else -1 for b in range(B)], dtype=torch.int32, device="cuda")
        mla.cache_append(to_torch(synth.to_bf16_bits(x_t.astype(np.float32)), "bf16"), W_DKVR, pool, table, pos, r_kv)
    q = np.stack([bf16((W_Q @ ctx[b][-1]).reshape(h, d)) for b in range(B)])     # queries as stored
    W_QR = host(out["W_QR"])
    q_rope = np.stack([[rope_hat(W_QR[i] @ q[b, i], lens[b] - 1, d_rope, theta) for i in range(h)] for b in range(B)])
    as_bf16 = lambda a: to_torch(synth.to_bf16_bits(np.asarray(a, dtype=np.float32)), "bf16")
    q_abs = mla.absorb_q(as_bf16(q), tb(out["W_UK"]))
    ws = mla.decode_paged(q_abs, as_bf16(q_rope), pool, table, torch.tensor(lens, dtype=torch.int32, device="cuda"),
                          1.0 / np.sqrt(d), num_splits=4, flags=mla.FLAG_SKIP_MERGE)
    _, got = mla.merge_out_proj(ws, tb(out["W_UV"]), B, 4)
    got = widen_gpu(got)
    ref = co.convert_layer(X, W_K, W_V, g, h, d, M, r_kv, keep)
    want = np.stack([mla_attention_through_the_decode_oracle(ref, None, ctx[b], None, h, d, lens[b] - 1, theta, q=q[b])
                     for b in range(B)])
    assert np.isfinite(got).all()
    assert max_abs_rel(got, want) <= 2e-2, max_abs_rel(got, want)
