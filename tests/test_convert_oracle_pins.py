"""Pins for the conversion oracle (oracle/convert_oracle.py): each test checks it
against something other than itself -- index sets printed in App. C, brute-force
RoPE written out with loops, properties that characterise an eigenbasis, the
inequality of App. C's proposition, closed forms, and two constructions under
which the converted layer must reproduce the GQA layer exactly (textbook
attention written in this file)."""
import math
from pathlib import Path

import numpy as np
import pytest

import oracle
from oracle import convert_oracle as co
from test_oracle_pins import dense_cache, textbook_attention

GOLDEN = Path(__file__).parent / "golden"


def rng(seed):
    return np.random.default_rng(seed)


def random_orthogonal(r, m):
    q, t = np.linalg.qr(r.standard_normal((m, m)))
    return q * np.sign(np.diag(t))


def rope_hat(v, pos, d, theta):
    """The merged RoPE of Sec. 4.1 with explicit loops: the same rotation on every
    block of d dimensions; pair l = dimensions (2l, 2l+1) of a block."""
    out = np.array(v, dtype=np.float64)
    for blk in range(len(v) // d):
        for l in range(d // 2):
            a = pos * theta[l]
            x, y = v[blk * d + 2 * l], v[blk * d + 2 * l + 1]
            out[blk * d + 2 * l] = x * math.cos(a) - y * math.sin(a)
            out[blk * d + 2 * l + 1] = x * math.sin(a) + y * math.cos(a)
    return out


def std_theta(d, base=10000.0):
    return np.array([base ** (-2.0 * l / d) for l in range(d // 2)])


def rope_by_component(v, pos, g, d, M, keep, theta_of):
    """RoPE on a ROTATED merged vector, component by component: the pair stored for component r of
    group G turns by pos * theta_of(G, r); theta_of returning None leaves the pair alone (NoPE)."""
    out_x, out_y = co.placement_columns(g, d, M, keep)
    out = np.array(v, dtype=np.float64)
    for G in range(out_x.shape[0]):
        for r in range(M * g):
            th = theta_of(G, r)
            if th is None:
                continue
            a = pos * th
            x, y = v[out_x[G, r]], v[out_y[G, r]]
            out[out_x[G, r]] = x * math.cos(a) - y * math.sin(a)
            out[out_y[G, r]] = x * math.sin(a) + y * math.cos(a)
    return out


# ------------------------------------------------------------- App. C index example

def test_group_columns_are_the_index_sets_of_the_worked_example():
    g, d = 2, 8
    seen = 0
    for line in (GOLDEN / "freqfold_index_example.txt").read_text().splitlines():
        if not line.strip() or line.startswith("#"):
            continue
        head, dims = line.split(":")
        M, G = (int(t) for t in head.split())
        want = sorted(int(t) for t in dims.split())
        col_x, col_y = co.group_columns(g, d, M)
        got = sorted((np.concatenate([col_x[G - 1], col_y[G - 1]]) + 1).tolist())
        assert got == want, (M, G)
        seen += 1
    assert seen == 6


def test_group_and_placement_columns_are_permutations_with_head_major_segments():
    for g, d, M in [(2, 8, 1), (2, 8, 2), (4, 16, 4), (3, 12, 3), (8, 64, 2)]:
        col_x, col_y = co.group_columns(g, d, M)
        out_x, out_y = co.placement_columns(g, d, M)
        for keep in range(1, M + 1):       # any number of kept components: a permutation, RoPE key first
            kx, ky = co.placement_columns(g, d, M, keep)
            assert sorted(np.concatenate([kx.ravel(), ky.ravel()]).tolist()) == list(range(g * d))
            d_rope = co.rope_width(d, M, keep)
            assert d_rope == keep * d // M
            assert (kx[:, :keep] < d_rope).all() and (kx[:, keep:] >= d_rope).all()
            assert (kx[:, :keep] // 2 == np.arange(d // (2 * M))[:, None] * keep + np.arange(keep)[None, :]).all()
        for a, b in [(col_x, col_y), (out_x, out_y)]:
            assert sorted(np.concatenate([a.ravel(), b.ravel()]).tolist()) == list(range(g * d))
            assert (a % 2 == 0).all() and (b == a + 1).all()
        # segment of pair p inside a group lists the heads in order (App. C: S_phi = head 1, head 2, ..)
        for G in range(col_x.shape[0]):
            for p in range(M):
                assert (col_x[G, p * g:(p + 1) * g] // d == np.arange(g)).all()
                assert ((col_x[G, p * g:(p + 1) * g] % d) // 2 == G * M + p).all()
        # the M leading components of every group land in the first head, each on a pair of the group
        first = out_x[:, :M]
        assert (first < d).all()
        assert sorted((first.ravel() // 2).tolist()) == list(range(d // 2))


# ------------------------------------------------------------- Eq. "rorope"

@pytest.mark.parametrize("g,d", [(2, 8), (4, 8), (3, 4)])
def test_rope_inner_product_is_invariant_under_one_rotation_per_pair(g, d):
    r = rng(7 + g)
    theta = std_theta(d)
    q_hat, k = r.standard_normal(g * d), r.standard_normal(g * d)
    U = np.stack([random_orthogonal(r, g) for _ in range(d // 2)])
    q2 = co.rotate_rows(q_hat[:, None], U, g, d, 1)[:, 0]
    k2 = co.rotate_rows(k[:, None], U, g, d, 1)[:, 0]
    for t, j in [(0, 0), (5, 2), (117, 3), (40, 40)]:
        want = rope_hat(q_hat, t, d, theta) @ rope_hat(k, j, d, theta)
        got = rope_hat(q2, t, d, theta) @ rope_hat(k2, j, d, theta)
        assert abs(got - want) < 1e-11 * (1 + abs(want))
    # a different matrix on the real and on the imaginary vector breaks it (App. B): the pin has teeth
    U_bad = np.stack([random_orthogonal(r, g) for _ in range(d // 2)])
    col_x, col_y = co.group_columns(g, d, 1)
    k3 = k2.copy()
    for G in range(d // 2):
        k3[col_y[G]] = U_bad[G].T @ k[col_y[G]]
    assert abs(rope_hat(q2, 9, d, theta) @ rope_hat(k3, 4, d, theta)
               - rope_hat(q_hat, 9, d, theta) @ rope_hat(k, 4, d, theta)) > 1e-3


@pytest.mark.parametrize("M", [2, 4])
def test_folded_groups_are_invariant_when_their_pairs_share_one_frequency(M):
    """App. C: FreqFold treats the M pairs of a group as one frequency.  With a RoPE whose
    frequency IS constant inside each group the rotation by any (M g) x (M g) orthogonal
    matrix is exact when every component keeps that frequency; giving the components the M
    different frequencies of their group's pairs instead is not."""
    g, d = 3, 8
    r = rng(11 + M)
    theta = std_theta(d)
    theta_folded = np.repeat(theta[::M], M)
    q_hat, k = r.standard_normal(g * d), r.standard_normal(g * d)
    U = np.stack([random_orthogonal(r, M * g) for _ in range(d // (2 * M))])
    q2 = co.rotate_rows(q_hat[:, None], U, g, d, M)[:, 0]
    k2 = co.rotate_rows(k[:, None], U, g, d, M)[:, 0]
    want = rope_hat(q_hat, 31, d, theta_folded) @ rope_hat(k, 6, d, theta_folded)
    folded = lambda G, rr: theta[G * M]
    got = rope_by_component(q2, 31, g, d, M, M, folded) @ rope_by_component(k2, 6, g, d, M, M, folded)
    assert abs(got - want) < 1e-11 * (1 + abs(want))
    own = lambda G, rr: theta[G * M + rr % M]
    assert abs(rope_by_component(q2, 31, g, d, M, M, own) @ rope_by_component(k2, 6, g, d, M, M, own)
               - rope_hat(q_hat, 31, d, theta) @ rope_hat(k, 6, d, theta)) > 1e-4


# ------------------------------------------------------------- App. B: moments and eigenbasis

def test_rope_moments_by_explicit_loops():
    g, d, M, n = 3, 8, 2, 5
    K = rng(3).standard_normal((n, g * d))
    got = co.rope_moments(K, g, d, M)
    for G in range(d // (2 * M)):
        for p1 in range(M):
            for j1 in range(g):
                for p2 in range(M):
                    for j2 in range(g):
                        a = j1 * d + 2 * (G * M + p1)
                        b = j2 * d + 2 * (G * M + p2)
                        want = sum(K[t, a] * K[t, b] + K[t, a + 1] * K[t, b + 1] for t in range(n)) / n
                        assert abs(got[G, p1 * g + j1, p2 * g + j2] - want) < 1e-13


def test_basis_is_orthogonal_diagonalises_and_maximises_every_leading_trace():
    r = rng(5)
    m = 6
    A = r.standard_normal((4, 40, m))
    sigma = np.einsum("bni,bnj->bij", A, A) / 40
    w, U = co.rorope_basis(sigma)
    for b in range(4):
        assert np.allclose(U[b].T @ U[b], np.eye(m), atol=1e-12)
        D = U[b].T @ sigma[b] @ U[b]
        assert np.allclose(D, np.diag(w[b]), atol=1e-12)
        assert (np.diff(w[b]) <= 1e-14).all()
        for trial in range(50):                       # trace objective of App. B, every m
            Q = random_orthogonal(r, m)
            T = Q.T @ sigma[b] @ Q
            for k in range(1, m + 1):
                assert np.trace(T[:k, :k]) <= w[b, :k].sum() + 1e-12


def test_two_by_two_closed_form():
    a, b, c = 2.0, 0.5, 1.0       # [[a, b], [b, c]]
    w, U = co.sym_eig_desc(np.array([[a, b], [b, c]]))
    mean, rad = (a + c) / 2, math.hypot((a - c) / 2, b)
    assert np.allclose(w, [mean + rad, mean - rad], atol=1e-14)
    ang = 0.5 * math.atan2(2 * b, a - c)
    assert abs(abs(U[:, 0] @ np.array([math.cos(ang), math.sin(ang)])) - 1) < 1e-14


@pytest.mark.parametrize("M,keep", [(1, 1), (2, 2), (2, 1), (4, 1), (4, 3)])
def test_rotated_key_projection_puts_the_eigenvalues_on_the_placement_slots(M, keep):
    """After rotating W^K with the basis of its own activations, the energy (real^2 + imaginary^2,
    averaged over the tokens) of the pair that stores component r of group G is eigenvalue r of
    group G, and different components of a group are uncorrelated.  The RoPE key (the `keep`
    leading components of every group) therefore holds the largest eigenvalues."""
    g, d, D, n = 4, 8, 10, 64
    r = rng(17)
    X, W_K = r.standard_normal((n, D)), r.standard_normal((g * d, D))
    w, U = co.rorope_basis(co.rope_moments(X @ W_K.T, g, d, M))
    K2 = X @ co.rotate_rows(W_K, U, g, d, M, keep).T
    out_x, out_y = co.placement_columns(g, d, M, keep)
    for G in range(d // (2 * M)):
        for c in range(M * g):
            e = (K2[:, out_x[G, c]] ** 2 + K2[:, out_y[G, c]] ** 2).mean()
            assert abs(e - w[G, c]) < 1e-11
        cross = (K2[:, out_x[G, 0]] * K2[:, out_x[G, 1]] + K2[:, out_y[G, 0]] * K2[:, out_y[G, 1]]).mean()
        assert abs(cross) < 1e-11
    d_rope = co.rope_width(d, M, keep)
    assert abs((K2[:, :d_rope] ** 2).sum() / n - w[:, :keep].sum()) < 1e-10
    if keep == M:      # a whole head: at least as much energy as any head had before
        K = X @ W_K.T
        assert (K2[:, :d] ** 2).sum() >= max((K[:, j * d:(j + 1) * d] ** 2).sum() for j in range(g))


def test_folding_captures_at_least_the_separate_leading_eigenvalues():
    """Proposition of App. C: V2 (M leading eigenvalues of the folded moment) >= V1 (sum of the
    leading eigenvalue of each pair's own moment)."""
    g, d, n = 4, 16, 200
    for seed in range(5):
        K = rng(seed).standard_normal((n, g * d)) @ np.diag(rng(seed + 50).uniform(0.2, 3.0, g * d))
        w1, _ = co.rorope_basis(co.rope_moments(K, g, d, 1))
        for M in (2, 4, 8):
            wM, _ = co.rorope_basis(co.rope_moments(K, g, d, M))
            for G in range(d // (2 * M)):
                V1 = w1[G * M:(G + 1) * M, 0].sum()
                V2 = wM[G, :M].sum()
                assert V2 >= V1 - 1e-12


# ------------------------------------------------------------- Sec. 4.3: alpha

def test_alpha_closed_form_and_score_equivalence():
    r = rng(23)
    K_nope = r.standard_normal((9, 5))
    K_nope *= 3.0 / np.linalg.norm(K_nope, axis=1, keepdims=True)
    V = r.standard_normal((9, 7))
    V *= 1.5 / np.linalg.norm(V, axis=1, keepdims=True)
    assert abs(co.kv_balance(K_nope, V) - 2.0) < 1e-14
    K2, V2 = r.standard_normal((30, 6)), r.standard_normal((30, 4))
    al = co.kv_balance(K2, V2)
    assert abs(np.linalg.norm(K2 / al, axis=1).mean() - np.linalg.norm(V2, axis=1).mean()) < 1e-13


# ------------------------------------------------------------- App. D.2

def test_joint_moment_blocks_and_basis_properties():
    r = rng(29)
    K_nope, V, al = r.standard_normal((50, 6)), r.standard_normal((50, 4)), 1.7
    S = co.joint_moment(K_nope, V, al)
    assert np.allclose(S[:6, :6], K_nope.T @ K_nope / 50 / al ** 2, atol=1e-13)
    assert np.allclose(S[:6, 6:], K_nope.T @ V / 50 / al, atol=1e-13)
    assert np.allclose(S[6:, 6:], V.T @ V / 50, atol=1e-13)
    w, R = co.joint_basis(S, 3)
    assert R.shape == (10, 3) and np.allclose(R.T @ R, np.eye(3), atol=1e-12)
    assert np.allclose(S @ R, R * w[:3], atol=1e-12)
    assert abs(w.sum() - np.trace(S)) < 1e-12 and (np.diff(w) <= 1e-14).all()
    # captured second moment is the largest possible (Ky Fan): no random 3-dimensional subspace beats it
    for _ in range(100):
        Q = random_orthogonal(r, 10)[:, :3]
        assert np.trace(Q.T @ S @ Q) <= w[:3].sum() + 1e-12


def test_low_rank_is_exact_when_the_activations_have_that_rank():
    """If the calibration tokens span r0 <= r_kv dimensions, keys and values rebuilt from the
    latent equal the originals on every calibration token."""
    g, h, d, D, n, r0 = 3, 6, 4, 12, 40, 5
    r = rng(31)
    X = r.standard_normal((n, r0)) @ r.standard_normal((r0, D))
    W_DK_nope, W_DV = r.standard_normal(((g - 1) * d, D)), r.standard_normal((g * d, D))
    W_UK_nope, W_UV = r.standard_normal((h, d, (g - 1) * d)), r.standard_normal((h, d, g * d))
    Kn, V = X @ W_DK_nope.T, X @ W_DV.T
    al = co.kv_balance(Kn, V)
    _, R = co.joint_basis(co.joint_moment(Kn, V, al), r0)
    W_DKV_p, W_UK_p, W_UV_p = co.low_rank_projections(W_DK_nope, W_DV, W_UK_nope, W_UV, al, R)
    assert W_DKV_p.shape == (r0, D) and W_UK_p.shape == (h, d, r0) and W_UV_p.shape == (h, d, r0)
    C = X @ W_DKV_p.T
    for i in range(h):
        assert np.allclose(C @ W_UK_p[i].T, Kn @ W_UK_nope[i].T, atol=1e-10)
        assert np.allclose(C @ W_UV_p[i].T, V @ W_UV[i].T, atol=1e-10)


# ------------------------------------------------------------- the chain against textbook GQA

def gqa_attention(x_new, X_ctx, W_Q, W_K, W_V, g, h, d, pos_new, theta):
    """Textbook GQA decode with RoPE (Sec. 3.2): one new token against its context (itself included)."""
    q = W_Q @ x_new
    outs = []
    for i in range(h):
        j = i // (h // g)
        qi = rope_hat(q[i * d:(i + 1) * d], pos_new, d, theta)
        Kj = np.stack([rope_hat(W_K[j * d:(j + 1) * d] @ X_ctx[t], t, d, theta) for t in range(len(X_ctx))])
        Vj = X_ctx @ W_V[j * d:(j + 1) * d].T
        outs.append(textbook_attention(qi, Kj, Vj, 1.0 / math.sqrt(d))[0])
    return np.stack(outs)


def mla_attention_through_the_decode_oracle(cv, x_new, X_ctx, W_Q, h, d, pos_new, theta, q=None):
    """Feed the converted tensors to the absorbed-decode oracle in the layout the decode path consumes.
    theta: the frequencies of the RoPE key, one per pair of its d_rope dimensions.  q: the query heads
    [h, d] if the caller has them already (else W_Q x_new)."""
    L = len(X_ctx)
    if q is None:
        q = (W_Q @ x_new).reshape(h, d)
    d_r = cv["W_KR"].shape[0]
    assert len(theta) == d_r // 2
    c_kv = X_ctx @ cv["W_DKV"].T
    k_rope = np.stack([rope_hat(cv["W_KR"] @ X_ctx[t], t, d_r, theta) for t in range(L)])
    q_rope = np.stack([rope_hat(cv["W_QR"][i] @ q[i], pos_new, d_r, theta) for i in range(h)])
    pool, table, lens = dense_cache([c_kv], [k_rope], page_size=4, seed=1)
    q_abs = oracle.absorb_q(q[None], cv["W_UK"])
    o_lat, _ = oracle.decode_absorbed(q_abs, q_rope[None], pool, None, table, lens, 1.0 / math.sqrt(d))
    return oracle.out_proj(o_lat, cv["W_UV"])[0]


def test_conversion_is_exact_at_full_rank_when_rope_is_the_identity():
    """Positions all zero make every RoPE rotation the identity, so dropping RoPE from
    the other heads loses nothing; with r_kv = (2g-1)d nothing is truncated either: the
    converted layer (RoRoPE, alpha, joint basis, absorbed decode) must reproduce GQA."""
    g, h, d, D, n, L = 2, 4, 8, 12, 64, 9
    r = rng(37)
    X = r.standard_normal((n, D))
    W_Q, W_K, W_V = (r.standard_normal((m, D)) / math.sqrt(D) for m in (h * d, g * d, g * d))
    theta = np.zeros(d // 2)
    for M, keep in ((1, 1), (2, 2), (2, 1), (4, 1), (4, 2)):
        d_r = co.rope_width(d, M, keep)
        cv = co.convert_layer(X, W_K, W_V, g, h, d, M, 2 * g * d - d_r, keep)
        assert cv["W_KR"].shape == (d_r, D) and cv["W_QR"].shape == (h, d_r, d)
        X_ctx = r.standard_normal((L, D))
        want = gqa_attention(X_ctx[-1], X_ctx, W_Q, W_K, W_V, g, h, d, L - 1, theta)
        got = mla_attention_through_the_decode_oracle(cv, X_ctx[-1], X_ctx, W_Q, h, d, L - 1, theta[:d_r // 2])
        assert np.abs(got - want).max() < 2e-6        # the oracle's pool stores float32


def test_rope_head_alone_is_exact_when_keys_are_rank_one_across_heads():
    """If, for every pair, the heads' key rows are multiples of one (real, imaginary) row pair, the
    summed moment has rank one, every component but the first is zero, and the score of the first
    head under ordinary RoPE equals the GQA score of the query's own group -- real positions."""
    g, h, d, D, n = 3, 6, 8, 10, 32
    r = rng(41)
    base_rows = r.standard_normal((d, D))
    s = r.uniform(0.5, 2.0, (g, d // 2)) * r.choice([-1.0, 1.0], (g, d // 2))
    W_K = np.concatenate([np.repeat(s[j], 2)[:, None] * base_rows for j in range(g)])
    X = r.standard_normal((n, D))
    w, U = co.rorope_basis(co.rope_moments(X @ W_K.T, g, d, 1))
    assert (w[:, 1:] < 1e-12 * w[:, :1]).all()
    W_K_rot = co.rotate_rows(W_K, U, g, d, 1)
    assert np.abs(X @ W_K_rot[d:].T).max() < 1e-12
    W_UK, _ = co.merged_projections(g, h, d)
    theta = std_theta(d)
    x_q, x_k, t, j = r.standard_normal(D), r.standard_normal(D), 57, 12
    W_Q = r.standard_normal((h * d, D))
    for i in range(h):
        q_i = W_Q[i * d:(i + 1) * d] @ x_q
        W_QR_i = co.rotate_rows(W_UK[i].T, U, g, d, 1)[:d]
        got = rope_hat(W_QR_i @ q_i, t, d, theta) @ rope_hat(W_K_rot[:d] @ x_k, j, d, theta)
        grp = i // (h // g)
        want = rope_hat(q_i, t, d, theta) @ rope_hat(W_K[grp * d:(grp + 1) * d] @ x_k, j, d, theta)
        assert abs(got - want) < 1e-11 * (1 + abs(want))


@pytest.mark.parametrize("M", [2, 4])
def test_one_pair_per_group_is_exact_for_rank_one_groups_under_folded_frequencies(M):
    """keep = 1: the RoPE key has one pair per FreqFold group and takes ordinary RoPE of width d / M,
    whose pair G turns with theta_{G M}.  If the original layer's RoPE has that frequency on all M pairs
    of group G (FreqFold's premise) and the group's keys are rank one (all its M g real coordinates
    multiples of one row, likewise the imaginary ones), every other component vanishes and the RoPE-key
    score equals the score of the query's own group in the original layer -- at real positions."""
    g, h, d, D, n = 3, 6, 8, 10, 32
    n_groups = d // (2 * M)
    r = rng(53 + M)
    col_x, col_y = co.group_columns(g, d, M)
    W_K = np.zeros((g * d, D))
    for G in range(n_groups):
        a_row, b_row = r.standard_normal(D), r.standard_normal(D)
        s = r.uniform(0.5, 2.0, M * g) * r.choice([-1.0, 1.0], M * g)
        W_K[col_x[G]] = s[:, None] * a_row
        W_K[col_y[G]] = s[:, None] * b_row
    X = r.standard_normal((n, D))
    w, U = co.rorope_basis(co.rope_moments(X @ W_K.T, g, d, M))
    assert (w[:, 1:] < 1e-12 * w[:, :1]).all()
    d_r = co.rope_width(d, M, 1)
    assert d_r == d // M
    W_K_rot = co.rotate_rows(W_K, U, g, d, M, 1)
    assert np.abs(X @ W_K_rot[d_r:].T).max() < 1e-12          # the NoPE key is empty
    W_UK, _ = co.merged_projections(g, h, d)
    theta = std_theta(d)
    theta_folded = np.repeat(theta[::M], M)                   # the original layer under FreqFold's premise
    theta_key = std_theta(d_r)                                # ordinary RoPE of the narrower key
    assert np.allclose(theta_key, theta[::M], rtol=1e-14)
    x_q, x_k, t, j = r.standard_normal(D), r.standard_normal(D), 57, 12
    W_Q = r.standard_normal((h * d, D))
    for i in range(h):
        q_i = W_Q[i * d:(i + 1) * d] @ x_q
        W_QR_i = co.rotate_rows(W_UK[i].T, U, g, d, M, 1)[:d_r]
        got = rope_hat(W_QR_i @ q_i, t, d_r, theta_key) @ rope_hat(W_K_rot[:d_r] @ x_k, j, d_r, theta_key)
        grp = i // (h // g)
        want = rope_hat(q_i, t, d, theta_folded) @ rope_hat(W_K[grp * d:(grp + 1) * d] @ x_k, j, d, theta_folded)
        assert abs(got - want) < 1e-11 * (1 + abs(want))


def test_merged_projections_select_the_group_of_each_query_head():
    """Sec. 4.1: W^UK_i is the identity on the columns of group ceil(i / (h/g)) - 1 (i from 1)."""
    g, h, d = 2, 6, 3
    W_UK, W_UV = co.merged_projections(g, h, d)
    for i1 in range(1, h + 1):
        j = math.ceil(i1 / (h / g)) - 1
        want = np.zeros((d, g * d))
        want[:, j * d:(j + 1) * d] = np.eye(d)
        assert (W_UK[i1 - 1] == want).all() and (W_UV[i1 - 1] == want).all()
