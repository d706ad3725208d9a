"""Pins of the float64 oracle to things other than itself: library optimizers the
method reduces to, closed forms, invariants, brute force on tiny inputs and a
library SVD.  Each test names the passage of the paper that fixes the value."""
import os

import numpy as np
import pytest
import torch

from oracle import lordo_oracle as orc
from paper_2602_04396_amd import synth

TOL = 1e-12


def rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def rng_of(i):
    return np.random.default_rng(synth.seed_for(0, i))


# ---------------------------------------------------------------------------
# local step
# ---------------------------------------------------------------------------
def test_reduces_to_library_adam_when_Q_is_identity():
    """Sec. 2: with r = p and Q = I the low-rank update is the full-rank Adam update.
    Library routine: torch.optim.Adam in float64 (eps outside the root, bias corrected)."""
    rng = rng_of(1)
    p, q = 12, 9
    W0 = rng.standard_normal((p, q))
    hp = orc.Hyper(beta1=0.9, beta2=0.999, eps=1e-8)
    st = orc.init_state(W0, p, np.eye(p))
    Wt = torch.tensor(W0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([Wt], lr=1e-3, betas=(0.9, 0.999), eps=1e-8)
    W = W0.copy()
    for t in range(7):
        G = rng.standard_normal((p, q))
        W = orc.local_step(st, W, G, 1e-3, hp)
        Wt.grad = torch.tensor(G, dtype=torch.float64)
        opt.step()
    assert rel(W, Wt.detach().numpy()) < 1e-13
    s = opt.state[Wt]
    assert rel(st.u, s["exp_avg"].numpy()) < 1e-13
    assert rel(st.v, s["exp_avg_sq"].numpy()) < 1e-13


def test_projections_against_triple_loops():
    """Sec. 2: g = Q^T G is r x q with g[i][j] = sum_k Q[k][i] G[k][j];
    Q N is p x q with (QN)[k][j] = sum_i Q[k][i] N[i][j].  Brute force, tiny."""
    rng = rng_of(2)
    p, q, r = 5, 4, 3
    Q = rng.standard_normal((p, r))
    G = rng.standard_normal((p, q))
    N = rng.standard_normal((r, q))
    g = np.zeros((r, q))
    for i in range(r):
        for j in range(q):
            for k in range(p):
                g[i, j] += Q[k, i] * G[k, j]
    up = np.zeros((p, q))
    for k in range(p):
        for j in range(q):
            for i in range(r):
                up[k, j] += Q[k, i] * N[i, j]
    assert rel(orc.project_down(Q, G), g) < 1e-14
    assert rel(orc.project_up(Q, N), up) < 1e-14


def test_first_step_closed_form():
    """Sec. 2 with bias correction: from zero state u_hat = g and v_hat = g*g, so the
    first update is W_1 = W_0 - eta Q [g / (|g| + eps)]."""
    rng = rng_of(3)
    p, q, r = 20, 14, 5
    Q = synth.orthonormal(rng, p, r)
    W0 = rng.standard_normal((p, q))
    G = rng.standard_normal((p, q))
    hp = orc.Hyper()
    st = orc.init_state(W0, r, Q)
    W1 = orc.local_step(st, W0, G, 0.01, hp)
    g = Q.T @ G
    expect = W0 - 0.01 * Q @ (g / (np.abs(g) + 1e-8))
    assert rel(W1, expect) < 1e-13


def test_constant_gradient_closed_form_and_rank():
    """A constant gradient keeps u_hat = g and v_hat = g*g at every t, so after T steps
    W_T = W_0 - (sum eta_t) Q [g/(|g|+eps)]; and with a fixed Q the change W_T - W_0 has
    rank at most r (App. A.2, pseudo-gradient with a fixed projection)."""
    rng = rng_of(4)
    p, q, r = 24, 18, 4
    Q = synth.orthonormal(rng, p, r)
    W0 = rng.standard_normal((p, q))
    G = rng.standard_normal((p, q))
    hp = orc.Hyper()
    st = orc.init_state(W0, r, Q)
    W = W0.copy()
    etas = [1e-3 * (1 + 0.1 * k) for k in range(10)]
    for eta in etas:
        W = orc.local_step(st, W, G, eta, hp)
    g = Q.T @ G
    expect = W0 - sum(etas) * Q @ (g / (np.abs(g) + 1e-8))
    assert rel(W - W0, expect - W0) < 1e-9
    sv = np.linalg.svd(W - W0, compute_uv=False)
    assert sv[r] < 1e-12 * sv[0]


def test_varying_gradient_change_has_rank_at_most_r():
    rng = rng_of(5)
    p, q, r = 16, 20, 3
    Q = synth.orthonormal(rng, p, r)
    W0 = rng.standard_normal((p, q))
    st = orc.init_state(W0, r, Q)
    W = W0.copy()
    for _ in range(6):
        W = orc.local_step(st, W, rng.standard_normal((p, q)), 1e-2, orc.Hyper())
    sv = np.linalg.svd(W - W0, compute_uv=False)
    assert sv[r] < 1e-12 * sv[0] and sv[r - 1] > 1e-6 * sv[0]


def test_no_bias_correction_flag():
    """Alg. 1 as printed (bias correction omitted): first step is
    u = (1-b1) g, v = (1-b2) g^2, N = u / (sqrt v + eps)."""
    rng = rng_of(6)
    p, q, r = 10, 8, 4
    Q = synth.orthonormal(rng, p, r)
    W0 = rng.standard_normal((p, q))
    G = rng.standard_normal((p, q))
    hp = orc.Hyper(bias_correction=False)
    st = orc.init_state(W0, r, Q)
    W1 = orc.local_step(st, W0, G, 0.5, hp)
    g = Q.T @ G
    N = (0.1 * g) / (np.sqrt(0.001 * g * g) + 1e-8)
    assert rel(W1, W0 - 0.5 * Q @ N) < 1e-13


def test_grad_scale_is_a_plain_prefactor():
    rng = rng_of(7)
    p, q, r = 10, 8, 4
    Q = synth.orthonormal(rng, p, r)
    W0 = rng.standard_normal((p, q))
    G = rng.standard_normal((p, q))
    a = orc.init_state(W0, r, Q)
    b = orc.init_state(W0, r, Q)
    Wa = orc.local_step(a, W0, G, 0.1, orc.Hyper(), grad_scale=0.25)
    Wb = orc.local_step(b, W0, 0.25 * G, 0.1, orc.Hyper())
    assert rel(Wa, Wb) < 1e-14 and rel(a.v, b.v) < 1e-14


def test_exact_reconstruction_when_rank_le_r():
    """rank(G) <= r and range(G) inside span(Q)  =>  Q Q^T G = G."""
    rng = rng_of(8)
    p, q, r = 30, 22, 6
    G = rng.standard_normal((p, r)) @ rng.standard_normal((r, q))
    Q = orc.range_finder(G, rng.standard_normal((q, r)), 1)
    assert rel(orc.project_up(Q, orc.project_down(Q, G)), G) < 1e-12


# ---------------------------------------------------------------------------
# optional variants: error feedback and quasi-hyperbolic momentum
# ---------------------------------------------------------------------------
def test_error_feedback_telescopes_and_is_orthogonal_to_Q():
    """Alg. 1 error-feedback lines: E_t = G_t + E_{t-1} - Q g_t with g_t = Q^T(G_t + E_{t-1})
    gives sum_t G_t = sum_t Q g_t + E_T and, for orthonormal Q, Q^T E_t = 0."""
    rng = rng_of(9)
    p, q, r = 18, 12, 4
    Q = synth.orthonormal(rng, p, r)
    W = rng.standard_normal((p, q))
    hp = orc.Hyper(error_feedback=True)
    st = orc.init_state(W, r, Q)
    sumG = np.zeros((p, q))
    sumQg = np.zeros((p, q))
    for _ in range(5):
        G = rng.standard_normal((p, q))
        W = orc.local_step(st, W, G, 1e-3, hp)
        sumG += G
        sumQg += Q @ st.last_g
        assert np.abs(Q.T @ st.E).max() < 1e-13
    assert rel(sumQg + st.E, sumG) < 1e-13


def test_local_variant_projection_sees_the_error_buffer():
    """Alg. 2: Q = ComputeProjection(G_t + E_{t-1}).  Build a gradient and a residual whose SUM has
    rank r while each alone has full rank: the step after the refresh then leaves E_t = 0 (the new
    span holds all of G + E), which a projection computed from G alone would not give."""
    rng = rng_of(31)
    p, q, r = 20, 14, 3
    hp = orc.Hyper(error_feedback=True, power_iters=2)
    W = rng.standard_normal((p, q))
    st = orc.init_state(W, r)                                   # Q_0 = identity columns (Alg. 2, Require)
    W = orc.local_step(st, W, rng.standard_normal((p, q)), 1e-3, hp)
    assert np.linalg.matrix_rank(st.E) > r
    low = rng.standard_normal((p, r)) @ rng.standard_normal((r, q))
    G = (low - st.E) / 0.5                                      # 0.5 * G + E = low
    assert np.linalg.matrix_rank(G) > r
    src = orc.local_variant_source(st, G, grad_scale=0.5)
    assert rel(src, low) < 1e-12
    orc.refresh_subspace(st, src, rng.standard_normal((q, r)), hp)
    W = orc.local_step(st, W, G, 1e-3, hp, grad_scale=0.5)
    assert np.abs(st.E).max() < 1e-10 * np.abs(low).max()
    # same construction, projection from the gradient alone: the residual survives
    st2 = orc.init_state(W, r)
    orc.local_step(st2, W, rng.standard_normal((p, q)), 1e-3, hp)
    G2 = (low - st2.E) / 0.5
    orc.refresh_subspace(st2, 0.5 * G2, rng.standard_normal((q, r)), hp)
    orc.local_step(st2, W, G2, 1e-3, hp, grad_scale=0.5)
    assert np.abs(st2.E).max() > 1e-3 * np.abs(low).max()


@pytest.mark.parametrize("kw", [dict(), dict(qhm_mode="low", omega=0.6), dict(error_feedback=True)])
def test_uplink_buffer_rebuilds_the_dense_pseudo_gradient(kw):
    """App. A.5.1: over a window with a fixed Q the dense pseudo-gradient x_{t-K} - x_t equals
    Q sum_tau eta_tau alpha_tau, so the r x q buffer carries all of it (no QHM and low-rank QHM)."""
    rng = rng_of(41)
    p, q, r = 17, 11, 4
    hp = orc.Hyper(uplink_buffer=True, **kw)
    W = rng.standard_normal((p, q))
    st = orc.init_state(W, r, synth.orthonormal(rng, p, r))
    for k in range(5):
        W = orc.local_step(st, W, rng.standard_normal((p, q)), 1e-3 * (1 + k), hp)      # a learning-rate schedule
    assert rel(st.Q @ st.A, orc.pseudo_gradient(st, W)) < 1e-12
    assert np.linalg.matrix_rank(orc.pseudo_gradient(st, W), tol=1e-10) == r


@pytest.mark.parametrize("outer", [dict(outer_lr=1.0), dict(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True),
                                   dict(outer_lr=0.5, outer_momentum=0.8)])
def test_outer_step_from_averaged_buffers_equals_dense_outer_step(outer):
    """Workers that share Q: the outer step fed the mean of the r x q buffers gives the model and
    momentum of the outer step fed the mean of the dense pseudo-gradients, over two windows."""
    rng = rng_of(42)
    p, q, r, M = 14, 9, 3, 3
    hp = orc.Hyper(uplink_buffer=True, **outer)
    Q = synth.orthonormal(rng, p, r)
    W0 = rng.standard_normal((p, q))
    low = [orc.init_state(W0, r, Q) for _ in range(M)]
    dense = [orc.init_state(W0, r, Q) for _ in range(M)]
    W_low = [W0.copy() for _ in range(M)]
    W_dense = [W0.copy() for _ in range(M)]
    for window in range(2):
        for k in range(3):
            for m in range(M):
                G = rng.standard_normal((p, q))
                W_low[m] = orc.local_step(low[m], W_low[m], G, 2e-3, hp)
                W_dense[m] = orc.local_step(dense[m], W_dense[m], G, 2e-3, hp)
        mean_A = sum(st.A for st in low) / M
        mean_D = sum(orc.pseudo_gradient(dense[m], W_dense[m]) for m in range(M)) / M
        for m in range(M):
            W_low[m] = orc.outer_step_lowrank(low[m], mean_A, hp)
            W_dense[m] = orc.outer_step(dense[m], mean_D, hp)
            assert rel(W_low[m], W_dense[m]) < 1e-12
            assert np.abs(low[m].b - dense[m].b).max() < 1e-12
            assert not low[m].A.any()


@pytest.mark.parametrize("mode", ["low", "full"])
def test_qhm_omega_one_is_no_qhm(mode):
    """Alg. 1: at omega = 1 both QHM cases are the "No QHM" case."""
    rng = rng_of(10)
    p, q, r = 14, 10, 3
    Q = synth.orthonormal(rng, p, r)
    W0 = rng.standard_normal((p, q))
    a = orc.init_state(W0, r, Q)
    b = orc.init_state(W0, r, Q)
    Wa, Wb = W0.copy(), W0.copy()
    for _ in range(4):
        G = rng.standard_normal((p, q))
        Wa = orc.local_step(a, Wa, G, 1e-2, orc.Hyper())
        Wb = orc.local_step(b, Wb, G, 1e-2, orc.Hyper(qhm_mode=mode, omega=1.0))
    assert rel(Wa, Wb) < 1e-14


def test_full_rank_qhm_omega_zero_is_column_scaled_sgd():
    """Sec. 3.2: at omega = 0 the full-rank form is G_hat / mu(sqrt(v_hat) + eps), with mu the mean
    over the r rank indices of a column; at step one v_hat = g*g, so the scale of column j
    is mean_i |g_ij| + eps."""
    rng = rng_of(11)
    p, q, r = 9, 7, 3
    Q = synth.orthonormal(rng, p, r)
    W0 = rng.standard_normal((p, q))
    G = rng.standard_normal((p, q))
    st = orc.init_state(W0, r, Q)
    W1 = orc.local_step(st, W0, G, 0.1, orc.Hyper(qhm_mode="full", omega=0.0))
    g = Q.T @ G
    scale = np.abs(g).mean(axis=0) + 1e-8
    assert rel(W1, W0 - 0.1 * G / scale[None, :]) < 1e-13


def test_full_rank_qhm_between_the_endpoints_written_out():
    """Sec. 3.2 at an interior omega, after several steps (so that v_hat is not g*g), written out with plain loops:
    W_ij <- W_ij - eta [ (1 - omega) G_ij / s_j + omega (Q N)_ij ],  s_j = (1/r) sum_k (sqrt(v_hat_kj) + eps),
    N = u_hat / (sqrt(v_hat) + eps).  The moments do not depend on omega, so they come from a plain chain run on the
    same gradients; the update is then also the affine combination of the two endpoint updates."""
    rng = rng_of(13)
    p, q, r, eta, om, eps = 8, 6, 3, 0.05, 0.35, 1e-8
    Q = synth.orthonormal(rng, p, r)
    W0 = rng.standard_normal((p, q))
    hp = orc.Hyper(qhm_mode="full", omega=om)
    st, plain = orc.init_state(W0, r, Q), orc.init_state(W0, r, Q)
    ends = [orc.init_state(W0, r, Q), orc.init_state(W0, r, Q)]
    W = W0.copy()
    for t in range(1, 4):
        G = rng.standard_normal((p, q))
        orc.local_step(plain, W0, G, eta, orc.Hyper())
        W_prev = W.copy()
        W = orc.local_step(st, W_prev, G, eta, hp)
        u_hat = plain.u / (1 - 0.9 ** t)
        v_hat = plain.v / (1 - 0.999 ** t)
        expect = W_prev.copy()
        for j in range(q):
            s_j = sum(np.sqrt(v_hat[k, j]) + eps for k in range(r)) / r
            for i in range(p):
                qn = sum(Q[i, k] * u_hat[k, j] / (np.sqrt(v_hat[k, j]) + eps) for k in range(r))
                expect[i, j] -= eta * ((1 - om) * G[i, j] / s_j + om * qn)
        assert rel(W, expect) < 1e-13
        W_end = [orc.local_step(ends[e], W_prev, G, eta, orc.Hyper(qhm_mode="full", omega=float(e))) for e in (0, 1)]
        assert rel(W, (1 - om) * W_end[0] + om * W_end[1]) < 1e-13


def test_low_rank_qhm_stays_in_span_full_rank_qhm_leaves_it():
    """App. A.4: the low-rank QHM update stays in span(Q); the full-rank one does not."""
    rng = rng_of(12)
    p, q, r = 16, 12, 3
    Q = synth.orthonormal(rng, p, r)
    W0 = rng.standard_normal((p, q))
    G = rng.standard_normal((p, q))
    P_perp = np.eye(p) - Q @ Q.T
    lo = orc.local_step(orc.init_state(W0, r, Q), W0, G, 0.1, orc.Hyper(qhm_mode="low", omega=0.7))
    fu = orc.local_step(orc.init_state(W0, r, Q), W0, G, 0.1, orc.Hyper(qhm_mode="full", omega=0.7))
    assert np.linalg.norm(P_perp @ (lo - W0)) < 1e-13
    assert np.linalg.norm(P_perp @ (fu - W0)) > 1e-3


# ---------------------------------------------------------------------------
# subspace refresh
# ---------------------------------------------------------------------------
def test_orth_is_orthonormal_same_span_positive_diagonal():
    rng = rng_of(13)
    Y = rng.standard_normal((40, 7)) @ np.diag(np.logspace(0, -3, 7))
    Qo = orc.orth(Y)
    assert np.abs(Qo.T @ Qo - np.eye(7)).max() < 1e-13
    R = Qo.T @ Y
    assert np.abs(np.tril(R, -1)).max() < 1e-12 * np.abs(R).max()
    assert (np.diag(R) > 0).all()
    assert rel(Qo @ R, Y) < 1e-13


def test_svd_projection_is_top_left_singular_subspace():
    """Sec. 2 default ComputeProjection: Q = U[:, :r].  Checked through the variational
    property it must have: ||Q^T A||_F^2 = sum of the r largest eigenvalues of A A^T
    (a different library routine: symmetric eigensolver)."""
    rng = rng_of(14)
    A = rng.standard_normal((15, 11))
    r = 4
    Q = orc.svd_projection(A, r)
    assert np.abs(Q.T @ Q - np.eye(r)).max() < 1e-13
    ev = np.sort(np.linalg.eigvalsh(A @ A.T))[::-1]
    assert abs(np.sum((Q.T @ A) ** 2) - ev[:r].sum()) < 1e-10
    # and no other r-dimensional subspace captures more (random trials)
    for _ in range(20):
        B = synth.orthonormal(rng, 15, r)
        assert np.sum((B.T @ A) ** 2) <= ev[:r].sum() + 1e-10


def _c1_source(seed_idx=0):
    rng = np.random.default_rng(synth.seed_for(1, seed_idx))
    S = synth.c1_signal(rng)
    G = synth.c1_gradient(S, rng).astype(np.float64)
    Om = synth.omega(rng, 256, 16).astype(np.float64)
    return S, G, Om


def test_range_finder_converges_to_svd_subspace_on_config1():
    """Config 1 (rank-8 signal, sigma 10..1, noise 0.01, r = 16): the range finder's span must
    close in on the top-8 left singular subspace of G, the residual shrinking per power iteration
    at least as fast as the textbook rate of block power iteration, (sigma_9 / sigma_8)^2."""
    _, G, Om = _c1_source()
    U, sv, _ = np.linalg.svd(G, full_matrices=False)
    U8 = U[:, :8]
    rate = (sv[8] / sv[7]) ** 2
    res = []
    for it in range(5):
        Q = orc.range_finder(G, Om, it)
        assert np.abs(Q.T @ Q - np.eye(16)).max() < 1e-12
        res.append(np.linalg.norm(U8 - Q @ (Q.T @ U8)))
    for k in range(4):
        assert res[k + 1] < 1.05 * rate * res[k]
    assert res[2] < 1e-2 and res[4] < 1e-4


def test_range_finder_reaches_svd_projector_with_a_gap():
    """With a spectral gap at r, enough power iterations give the projector U_r U_r^T
    of the paper's default SVD projection."""
    rng = rng_of(15)
    p, q, r = 48, 40, 5
    A = (synth.orthonormal(rng, p, p)[:, :q] * np.concatenate([np.linspace(9, 5, r), 0.5 * rng.random(q - r)])) \
        @ synth.orthonormal(rng, q, q).T
    Q = orc.range_finder(A, rng.standard_normal((q, r)), 12)
    Qs = orc.svd_projection(A, r)
    assert np.linalg.norm(Q @ Q.T - Qs @ Qs.T) < 1e-9


def test_rayleigh_ritz_gives_the_ordered_singular_vectors_of_the_svd_projection():
    """With a gap at r and a converged range finder, the Rayleigh-Ritz step turns the basis into the columns of
    U[:, :r] of the paper's SVD projection (Sec. 2), in its order, up to the sign of each column, and returns
    the leading singular values.  The full SVD of A by the library is the external reference."""
    rng = rng_of(41)
    p, q, r = 48, 40, 5
    sv = np.concatenate([np.array([9.0, 7.5, 6.5, 5.5, 5.0]), 0.5 * rng.random(q - r)])
    A = (synth.orthonormal(rng, p, p)[:, :q] * sv) @ synth.orthonormal(rng, q, q).T
    Q = orc.range_finder(A, rng.standard_normal((q, r)), 12)
    Qr, S = orc.rayleigh_ritz(Q, A)
    U, S_full, _ = np.linalg.svd(A, full_matrices=False)
    assert np.allclose(S, S_full[:r], rtol=1e-10)
    overlaps = np.abs(np.sum(Qr * U[:, :r], axis=0))           # |<column i, u_i>|
    assert np.all(overlaps > 1 - 1e-9)
    # a transposed small factor or an unsorted order would fail here: column 0 must be u_1, not any other
    assert abs(Qr[:, 0] @ U[:, 0]) > 1 - 1e-9 and abs(Qr[:, 0] @ U[:, 1]) < 1e-6
    # sign convention: the entry of largest magnitude of every column is positive
    assert np.all(Qr[np.argmax(np.abs(Qr), axis=0), np.arange(r)] > 0)


def test_rayleigh_ritz_keeps_the_span_and_diagonalises_the_restricted_matrix():
    """For ANY orthonormal Q (no convergence assumed): same projector, orthonormal columns, Q'^T A A^T Q' diagonal
    with the squared Ritz values in descending order, and their sum equal to the energy ||Q^T A||_F^2 the
    subspace captures."""
    rng = rng_of(42)
    p, q, r = 37, 29, 6
    A = rng.standard_normal((p, q))
    Q = synth.orthonormal(rng, p, r)
    Qr, S = orc.rayleigh_ritz(Q, A)
    assert np.linalg.norm(Qr @ Qr.T - Q @ Q.T) < 1e-12
    assert np.abs(Qr.T @ Qr - np.eye(r)).max() < 1e-12
    D = Qr.T @ A @ A.T @ Qr
    assert np.abs(D - np.diag(S * S)).max() < 1e-10
    assert np.all(np.diff(S) <= 0)
    assert abs(np.sum(S * S) - np.linalg.norm(Q.T @ A) ** 2) < 1e-10
    # refresh_subspace applies it when asked to
    hp = orc.Hyper(power_iters=1, rayleigh_ritz=True)
    st = orc.init_state(np.zeros((p, q)), r)
    Om = rng.standard_normal((q, r))
    Qn = orc.refresh_subspace(st, A, Om, hp)
    Qplain = orc.range_finder(A, Om, 1)
    assert np.linalg.norm(Qn @ Qn.T - Qplain @ Qplain.T) < 1e-12
    Dn = Qn.T @ A @ A.T @ Qn
    assert np.abs(Dn - np.diag(np.diag(Dn))).max() < 1e-10 and np.all(np.diff(np.diag(Dn)) <= 1e-12)


def test_stable_rank_closed_forms():
    """sr = ||A||_F^2 / ||A||_2^2 (Sec. 5.1): n for an orthogonal n x n matrix, 1 for rank one, 25/16 for diag(3, 4),
    invariant under orthogonal factors and scaling, never above the rank."""
    rng = rng_of(43)
    assert abs(orc.stable_rank(synth.orthonormal(rng, 12, 12)) - 12.0) < 1e-10
    assert abs(orc.stable_rank(np.outer(rng.standard_normal(9), rng.standard_normal(7))) - 1.0) < 1e-12
    assert abs(orc.stable_rank(np.diag([3.0, 4.0])) - 25.0 / 16.0) < 1e-12
    A = rng.standard_normal((14, 9))
    B = 3.5 * synth.orthonormal(rng, 14, 14) @ A @ synth.orthonormal(rng, 9, 9)
    assert abs(orc.stable_rank(A) - orc.stable_rank(B)) < 1e-10
    low = rng.standard_normal((14, 3)) @ rng.standard_normal((3, 9))
    assert 1.0 <= orc.stable_rank(low) <= 3.0 + 1e-12


def test_spectral_gap_closed_forms_and_its_estimate():
    """sigma_r - sigma_{r+1} (Sec. 5.1) on matrices with known singular values; the deflated block iteration reaches
    sigma_{r+1} when it is separated from the rest, and stays below the norm of the deflated matrix always."""
    rng = rng_of(44)
    assert abs(orc.spectral_gap(np.diag([5.0, 3.0, 1.0]), 1) - 2.0) < 1e-12
    assert abs(orc.spectral_gap(np.diag([5.0, 3.0, 1.0]), 2) - 2.0) < 1e-12
    assert abs(orc.spectral_gap(np.diag([5.0, 3.0, 1.0]), 3) - 1.0) < 1e-12          # no sigma_4
    p, q, r = 40, 31, 4
    sv = np.concatenate([[9.0, 8.0, 7.0, 6.0, 4.0], 0.3 * rng.random(q - 5)])
    U, V = synth.orthonormal(rng, p, p)[:, :q], synth.orthonormal(rng, q, q)
    A = (U * sv) @ V.T
    assert abs(orc.spectral_gap(A, r) - 2.0) < 1e-10
    est = orc.next_singular_value_estimate(A, U[:, :r], rng.standard_normal((q, r)), iters=8)
    assert abs(est - 4.0) < 1e-9
    # a basis that misses part of the leading subspace: the estimate sees what is left of it (here sigma_1 = 9)
    est_wrong = orc.next_singular_value_estimate(A, U[:, 1:r + 1], rng.standard_normal((q, r)), iters=8)
    assert abs(est_wrong - 9.0) < 1e-9
    # no separation (Gaussian matrix), few iterations: a lower bound, and not a poor one
    G = rng.standard_normal((60, 50))
    Ug, sg, _ = np.linalg.svd(G, full_matrices=False)
    e2 = orc.next_singular_value_estimate(G, Ug[:, :6], rng.standard_normal((50, 6)), iters=2)
    assert 0.85 * sg[6] < e2 <= sg[6] * (1 + 1e-12)
    # 2r > min(p, q): the deflated matrix has fewer than r directions; the estimate must stay below its norm
    # (the completion of the block by the orthonormalisation is not orthogonal to the basis)
    A2 = (synth.orthonormal(rng, 30, 30)[:, :20] * np.concatenate([np.linspace(9, 5, 12), 0.4 * rng.random(8)])) \
        @ synth.orthonormal(rng, 20, 20).T
    Q2 = orc.range_finder(A2, rng.standard_normal((20, 12)), 1)
    norm_deflated = np.linalg.svd(A2 - Q2 @ (Q2.T @ A2), compute_uv=False)[0]
    e3 = orc.next_singular_value_estimate(A2, Q2, rng.standard_normal((20, 12)), iters=2)
    assert 0.5 * norm_deflated < e3 <= norm_deflated * (1 + 1e-12)


def test_range_finder_rank_deficient_source_still_reconstructs():
    """rank(A) < r: the basis is completed arbitrarily; only Q^T Q = I and Q Q^T A = A are fixed."""
    rng = rng_of(16)
    p, q, r = 30, 25, 8
    A = rng.standard_normal((p, 3)) @ rng.standard_normal((3, q))
    Q = orc.range_finder(A, rng.standard_normal((q, r)), 1)
    assert np.abs(Q.T @ Q - np.eye(r)).max() < 1e-12
    assert rel(Q @ (Q.T @ A), A) < 1e-12


# ---------------------------------------------------------------------------
# moment rotation
# ---------------------------------------------------------------------------
def _moments(rng, r, q, t, hp):
    """Moments as t steps of EMA on random low-rank gradients would leave them."""
    u = np.zeros((r, q))
    v = np.zeros((r, q))
    for _ in range(t):
        g = rng.standard_normal((r, q))
        u, v = orc.update_moments(u, v, g, hp.beta1, hp.beta2)
    return u, v


def test_rotation_identity_when_basis_unchanged():
    """Alg. 1 rotation lines with Q_new = Q_old: R = I, u unchanged and
    v = c2 |v_hat - u_hat^2 + u_hat^2| = v."""
    rng = rng_of(17)
    hp = orc.Hyper()
    Q = synth.orthonormal(rng, 20, 5)
    u, v = _moments(rng, 5, 9, 6, hp)
    un, vn = orc.rotate_moments(Q, Q, u, v, 6, hp)
    assert rel(un, u) < TOL and rel(vn, v) < TOL


def test_rotation_permutation_and_sign_flip():
    """Q_new = Q_old Pi permutes the rows of u and v; Q_new = Q_old diag(+-1) flips the
    signs of rows of u and leaves v alone."""
    rng = rng_of(18)
    hp = orc.Hyper()
    r, q = 5, 8
    Q = synth.orthonormal(rng, 17, r)
    u, v = _moments(rng, r, q, 4, hp)
    perm = np.array([2, 0, 4, 1, 3])
    un, vn = orc.rotate_moments(Q[:, perm], Q, u, v, 4, hp)
    assert rel(un, u[perm]) < TOL and rel(vn, v[perm]) < TOL
    s = np.array([1, -1, -1, 1, -1.0])
    un, vn = orc.rotate_moments(Q * s, Q, u, v, 4, hp)
    assert rel(un, u * s[:, None]) < TOL and rel(vn, v) < TOL


def test_rotation_within_span_keeps_full_space_momentum():
    """Q_new = Q_old O with O orthogonal: Q_new u_new = Q_old u (the momentum seen in the
    full space does not move)."""
    rng = rng_of(19)
    hp = orc.Hyper()
    r, q = 6, 7
    Q = synth.orthonormal(rng, 25, r)
    O = synth.orthonormal(rng, r, r)
    u, v = _moments(rng, r, q, 3, hp)
    un, vn = orc.rotate_moments(Q @ O, Q, u, v, 3, hp)
    assert rel((Q @ O) @ un, Q @ u) < TOL
    assert (vn >= 0).all()


def test_rotation_to_orthogonal_subspace_clears_moments():
    rng = rng_of(20)
    hp = orc.Hyper()
    B = synth.orthonormal(rng, 30, 8)
    u, v = _moments(rng, 4, 6, 5, hp)
    un, vn = orc.rotate_moments(B[:, 4:], B[:, :4], u, v, 5, hp)
    assert np.abs(un).max() < 1e-14 and np.abs(vn).max() < 1e-14


def test_second_moment_rotation_hadamard_reading_brute_force():
    """Reading of the squares in the second-moment rotation as elementwise: for one column,
    new_v_i = c2 | sum_j R_ij^2 (v_hat_j - u_hat_j^2) + (sum_j R_ij u_hat_j)^2 |, i.e. a
    variance pushed through the linear map R plus the squared rotated mean."""
    rng = rng_of(21)
    hp = orc.Hyper()
    r, q, t = 4, 3, 5
    Qo = synth.orthonormal(rng, 12, r)
    Qn = synth.orthonormal(rng, 12, r)
    u, v = _moments(rng, r, q, t, hp)
    un, vn = orc.rotate_moments(Qn, Qo, u, v, t, hp)
    c1, c2 = 1 - 0.9 ** t, 1 - 0.999 ** t
    R = np.zeros((r, r))
    for i in range(r):
        for j in range(r):
            for k in range(12):
                R[i, j] += Qn[k, i] * Qo[k, j]
    for col in range(q):
        for i in range(r):
            var = sum(R[i, j] ** 2 * (v[j, col] / c2 - (u[j, col] / c1) ** 2) for j in range(r))
            mean = sum(R[i, j] * u[j, col] / c1 for j in range(r))
            assert abs(vn[i, col] - c2 * abs(var + mean ** 2)) < 1e-14
            assert abs(un[i, col] - sum(R[i, j] * u[j, col] for j in range(r))) < 1e-14


def test_refresh_before_first_step_keeps_zero_moments():
    _, G, Om = _c1_source()
    st = orc.init_state(np.zeros((256, 256)), 16)
    orc.refresh_subspace(st, G, Om, orc.Hyper())
    assert st.t == 0 and not st.u.any() and not st.v.any()
    assert np.abs(st.Q.T @ st.Q - np.eye(16)).max() < 1e-12


def test_mssv_limits():
    """Sec. 5.1 Metrics: same basis -> 1, orthogonal bases -> 0."""
    rng = rng_of(22)
    B = synth.orthonormal(rng, 20, 8)
    assert abs(orc.mssv(B[:, :4], B[:, :4]) - 1) < 1e-13
    assert orc.mssv(B[:, :4], B[:, 4:]) < 1e-26
    sv = np.linalg.svd(B[:, 2:6].T @ B[:, :4], compute_uv=False)
    assert abs(orc.mssv(B[:, 2:6], B[:, :4]) - np.mean(sv ** 2)) < 1e-13


# ---------------------------------------------------------------------------
# outer step
# ---------------------------------------------------------------------------
def test_outer_default_is_worker_average():
    """Alg. 1: OuterOpt is averaging by default: with eta_s = 1 and no momentum the new model
    is the mean of the workers' models."""
    rng = rng_of(23)
    anchor = rng.standard_normal((6, 5))
    workers = [anchor + 0.1 * rng.standard_normal((6, 5)) for _ in range(4)]
    st = orc.init_state(anchor, 2)
    deltas = [orc.pseudo_gradient(st, w) for w in workers]
    x = orc.outer_step(st, np.mean(deltas, axis=0), orc.Hyper())
    assert rel(x, np.mean(workers, axis=0)) < 1e-14
    assert rel(st.anchor, x) < 1e-15


@pytest.mark.parametrize("nesterov", [True, False])
def test_outer_momentum_matches_library_sgd(nesterov):
    """App. D.4/D.5: Nesterov outer optimizer as in DiLoCo = SGD with (Nesterov) momentum fed the
    pseudo-gradient.  Library routine: torch.optim.SGD in float64."""
    rng = rng_of(24)
    x0 = rng.standard_normal((7, 4))
    hp = orc.Hyper(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=nesterov)
    st = orc.init_state(x0, 2)
    xt = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([xt], lr=0.7, momentum=0.9, nesterov=nesterov)
    for _ in range(5):
        D = rng.standard_normal((7, 4))
        x = orc.outer_step(st, D, hp)
        xt.grad = torch.tensor(D)
        opt.step()
        assert rel(x, xt.detach().numpy()) < 1e-13


def test_outer_nesterov_closed_form_two_steps():
    """From b = 0: first step is eta_s (1 + mu) Delta; a second step with the same Delta is
    eta_s (1 + mu + mu^2) Delta."""
    rng = rng_of(25)
    x0 = rng.standard_normal((5, 5))
    D = rng.standard_normal((5, 5))
    hp = orc.Hyper(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True)
    st = orc.init_state(x0, 2)
    x1 = orc.outer_step(st, D, hp)
    assert rel(x1, x0 - 0.7 * 1.9 * D) < 1e-14
    x2 = orc.outer_step(st, D, hp)
    assert rel(x2, x1 - 0.7 * (1 + 0.9 + 0.81) * D) < 1e-14


def test_config1_chain_closed_form():
    """Config 1 with a constant gradient: 10 local steps at eta = 1e-3 then one Nesterov outer step
    (eta_s 0.7, mu 0.9) on the worker's own pseudo-gradient: W = W_0 - 0.7 * 1.9 * 1e-2 * Q N,
    N = g / (|g| + eps)."""
    S, G, Om = _c1_source()
    rng = np.random.default_rng(synth.seed_for(1, 99))
    W0 = synth.weights(rng, 256, 256).astype(np.float64)
    hp = orc.Hyper(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True, power_iters=2)
    st = orc.init_state(W0, 16)
    orc.refresh_subspace(st, G, Om, hp)
    W = W0.copy()
    for _ in range(10):
        W = orc.local_step(st, W, G, 1e-3, hp)
    D = orc.pseudo_gradient(st, W)
    W = orc.outer_step(st, D, hp)
    g = st.Q.T @ G
    expect = W0 - 0.7 * 1.9 * 1e-2 * st.Q @ (g / (np.abs(g) + 1e-8))
    assert rel(W - W0, expect - W0) < 1e-9


# ---------------------------------------------------------------------------
# Sec. 3.3 communication ratios (used by the sharding note only)
# ---------------------------------------------------------------------------
def test_comm_ratios_golden():
    here = os.path.dirname(__file__)
    quoted = {}
    with open(os.path.join(here, "golden", "comm_ratios.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, val, tol = line.split()
                quoted[name] = (float(val), float(tol))
    K, r, p, q = 32, 256, 2048, 2048
    lowrank = 1.0 / ((1 + r / q) / K + 1 / K + 1 / K)
    fullrank = 1.0 / ((1 + r / q) / K + r / (K * p) + r / (K * p))
    val, tol = quoted["vs_lowrank_ddp"]
    assert abs(lowrank - val) / val < tol
    val, tol = quoted["vs_fullrank_ddp"]
    assert abs(fullrank - val) / val < tol


# ---------------------------------------------------------------------------------------------
# projection on the right (Sec. 2 applied to the transposed matrix)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("qhm", ["none", "low", "low_ef", "full", "full_ef"])
def test_right_projection_is_the_method_on_the_transpose(qhm):
    """The explicit right-side formulas (g = G Q, W -= lr N Q^T; full-rank QHM: the gradient term scaled per ROW of W)
    against the left-side functions run on W^T, G^T: two code paths, one result, over steps and a refresh."""
    rng = np.random.default_rng(77)
    p, q, r = 23, 11, 4
    ef = qhm.endswith("_ef")
    qhm = qhm.split("_")[0]
    hp = orc.Hyper(qhm_mode=qhm, omega=0.7 if qhm != "none" else 1.0, power_iters=1, error_feedback=ef)
    W = rng.standard_normal((p, q))
    Q0 = np.linalg.qr(rng.standard_normal((q, r)))[0]
    a, b = orc.init_state(W.T, r, Q0), orc.init_state(W.T, r, Q0)
    Wa, Wb = W.copy(), W.T.copy()
    for t in range(3):
        G = rng.standard_normal((p, q))
        Wa = orc.local_step_right(a, Wa, G, 1e-2, hp, grad_scale=0.5)
        Wb = orc.local_step(b, Wb, G.T, 1e-2, hp, grad_scale=0.5)
        np.testing.assert_allclose(Wa, Wb.T, rtol=0, atol=1e-14)
        np.testing.assert_allclose(a.last_N, b.last_N, rtol=0, atol=1e-13)
        if ef:          # the residual is orthogonal to the basis on the right, and the books balance (sum of gradients = projected part + E)
            np.testing.assert_allclose(a.E, b.E, rtol=0, atol=1e-14)
            assert np.linalg.norm(a.E.T @ a.Q) <= 1e-12
    Src, Om = rng.standard_normal((p, q)), rng.standard_normal((p, r))
    Qa = orc.refresh_subspace_right(a, Src, Om, hp)
    Qb = orc.refresh_subspace(b, Src.T, Om, hp)
    np.testing.assert_allclose(Qa, Qb, rtol=0, atol=1e-14)
    # the new basis spans the top right singular vectors' neighbourhood: Src Q Q^T keeps more of Src than any r coordinates
    assert Qa.shape == (q, r) and np.allclose(Qa.T @ Qa, np.eye(r), atol=1e-12)
    np.testing.assert_allclose(a.u, b.u, rtol=0, atol=1e-14)


def test_right_projection_full_rank_identity_is_adam():
    """r = q and Q = I: the right-projected step is Adam on the full gradient; first step in closed form
    (bias-corrected moments equal g and g^2, so N = g / (|g| + eps))."""
    rng = np.random.default_rng(78)
    p, q = 9, 5
    hp = orc.Hyper()
    W, G = rng.standard_normal((p, q)), rng.standard_normal((p, q))
    st = orc.init_state(W.T, q, np.eye(q))
    W1 = orc.local_step_right(st, W, G, 1e-3, hp)
    np.testing.assert_allclose(W1, W - 1e-3 * G / (np.abs(G) + hp.eps), rtol=1e-12, atol=1e-15)
    # a gradient orthogonal to the columns of Q projects to rounding noise (which eps = 1e-8 in the denominator
    # turns into at most 1e-8 per element of N): W stays where it is
    Q = np.linalg.qr(rng.standard_normal((q, 2)))[0]
    st = orc.init_state(W.T, 2, Q)
    G_perp = rng.standard_normal((p, q)) @ (np.eye(q) - Q @ Q.T)
    np.testing.assert_allclose(orc.local_step_right(st, W, G_perp, 1e-3, hp), W, rtol=0, atol=1e-9)


# ---------------------------------------------------------------------------
# the generator of the blocks the method draws itself (Alg. 1 Require: random initial projection)
# ---------------------------------------------------------------------------
def test_philox_matches_the_published_known_answers():
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for words in rows:
        w = [int(x, 16) for x in words]
        out = orc.philox4x32_10(np.array([w[0:4]], dtype=np.uint32), np.array([w[4:6]], dtype=np.uint32))[0]
        assert [int(x) for x in out] == w[6:10]


def test_gaussian_block_is_box_muller_of_the_philox_words_and_standard_normal():
    seed, mat, draw = 0x1234567812345678, 3, 2
    Z = orc.gaussian_block(seed, mat, draw, 5, 3)               # 15 elements: a ragged last quad
    # element 6 = output 2 of quad 1, element 7 = output 3: one Box-Muller pair, here through the complex exponential
    x = orc.philox4x32_10(np.array([[1, 0, mat, draw]], dtype=np.uint32),
                          np.array([[seed & 0xFFFFFFFF, seed >> 32]], dtype=np.uint32))[0]
    u0, u1 = ((int(x[2]) >> 8) + 0.5) / 2 ** 24, ((int(x[3]) >> 8) + 0.5) / 2 ** 24
    z = np.sqrt(-2 * np.log(u0)) * np.exp(2j * np.pi * u1)
    assert abs(Z.reshape(-1)[6] - z.real) < 1e-14 and abs(Z.reshape(-1)[7] - z.imag) < 1e-14
    # a prefix property: the block of a larger shape starts with the same numbers (element index is the counter)
    assert np.array_equal(orc.gaussian_block(seed, mat, draw, 1, 15).reshape(-1), Z.reshape(-1))
    # other matrix, other draw, other seed: other numbers
    for other in (orc.gaussian_block(seed, mat + 1, draw, 5, 3), orc.gaussian_block(seed, mat, draw + 1, 5, 3),
                  orc.gaussian_block(seed + 1, mat, draw, 5, 3)):
        assert np.min(np.abs(other - Z)) > 0
    big = orc.gaussian_block(99, 0, 0, 2000, 256)
    n = big.size
    assert abs(big.mean()) < 4 / np.sqrt(n) and abs(big.var() - 1) < 4 * np.sqrt(2 / n)
    assert abs(np.mean(big ** 4) - 3) < 4 * np.sqrt(96 / n) and np.abs(big).max() < 6.2
    # columns are uncorrelated: the Gram matrix of the block is n_rows * I up to sampling noise
    Gm = big.T @ big / 2000
    assert np.linalg.norm(Gm - np.eye(256), 2) < 2.5 * (np.sqrt(256 / 2000) * 2 + 256 / 2000)


# ---------------------------------------------------------------------------
# bf16 storage of the weights
# ---------------------------------------------------------------------------
def test_round_to_bf16_is_round_to_nearest_even_once():
    """Against an independent route: for float32-representable inputs the bit-level rounding of the input generator
    (add 0x7FFF + lsb, shift) is the same rounding; plus hand-made ties, the error bound, idempotence, and a
    double-rounding trap (float64 -> float32 -> bf16 would go the other way)."""
    rng = rng_of(70)
    x32 = (rng.standard_normal(20000) * 10.0 ** rng.uniform(-6, 3, 20000)).astype(np.float32)
    assert np.array_equal(orc.round_to_bf16(x32.astype(np.float64)), synth.bf16_round(x32).astype(np.float64))
    # ties go to the even neighbour: spacing at 1.0 is 2^-7
    assert orc.round_to_bf16(np.array([1 + 2.0 ** -8]))[0] == 1.0
    assert orc.round_to_bf16(np.array([1 + 3 * 2.0 ** -8]))[0] == 1 + 2.0 ** -6
    assert orc.round_to_bf16(np.array([-(1 + 2.0 ** -8)]))[0] == -1.0
    assert orc.round_to_bf16(np.array([0.0, 2.0 ** -20, -0.375]))[1] == 2.0 ** -20
    # just above a tie in float64, but a tie after a first rounding to float32: one rounding decides correctly
    x = 1 + 2.0 ** -8 + 2.0 ** -40
    assert np.float32(x) == np.float32(1 + 2.0 ** -8) and orc.round_to_bf16(np.array([x]))[0] == 1 + 2.0 ** -7
    y = rng.standard_normal(5000) * 10.0 ** rng.uniform(-5, 5, 5000)
    r = orc.round_to_bf16(y)
    ulp = 2.0 ** (np.floor(np.log2(np.abs(y))) - 7)
    assert np.all(np.abs(r - y) <= 0.5 * ulp) and np.array_equal(orc.round_to_bf16(r), r)


def test_bf16_weight_steps_are_the_full_precision_steps_rounded_once():
    """The local and the outer step for bf16-stored weights equal the float64 step from the same stored value, rounded
    once (Alg. 1 update lines; OuterOpt); the low-rank state does not depend on the weights at all."""
    rng = rng_of(71)
    p, q, r = 24, 18, 5
    W0 = orc.round_to_bf16(0.02 * rng.standard_normal((p, q)))
    Q = synth.orthonormal(rng, p, r)
    hp = orc.Hyper(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True)
    a, b = orc.init_state(W0, r, Q), orc.init_state(W0, r, Q)
    Wa, Wb = W0.copy(), W0.copy()
    for t in range(4):
        G = rng.standard_normal((p, q)) * 1e-2
        full = orc.local_step(b, Wa, G, 1e-2, hp)                  # from the STORED value of the other chain
        Wa = orc.local_step_bf16_weights(a, Wa, G, 1e-2, hp)
        assert np.array_equal(Wa, orc.round_to_bf16(full))
        assert np.array_equal(a.u, b.u) and np.array_equal(a.v, b.v) and np.array_equal(a.last_N, b.last_N)
    D = orc.pseudo_gradient(a, Wa)
    b.anchor, b.b = a.anchor.copy(), a.b.copy()
    full = orc.outer_step(b, D, hp)
    Wn = orc.outer_step_bf16_weights(a, D, hp)
    assert np.array_equal(Wn, orc.round_to_bf16(full)) and np.array_equal(a.anchor, Wn)
    assert np.array_equal(a.b, b.b)


def test_bf16_residual_step_is_the_error_feedback_step_rounded_once():
    """Alg. 1 error-feedback lines with a bf16-stored residual: from the same stored E the projected matrix, g, the
    moments and the weights are those of the full-precision step, and the new residual is that step's residual
    G_hat + E - Q g (written out here) rounded once; it is orthogonal to Q up to that rounding."""
    rng = rng_of(72)
    p, q, r = 20, 14, 4
    Q = synth.orthonormal(rng, p, r)
    W0 = rng.standard_normal((p, q))
    hp = orc.Hyper(error_feedback=True, qhm_mode="low", omega=0.8)
    a, b = orc.init_state(W0, r, Q), orc.init_state(W0, r, Q)
    Wa = W0.copy()
    for t in range(4):
        G = rng.standard_normal((p, q)) * 1e-2
        b.E = a.E.copy()                                           # the other chain starts from the STORED residual
        E_before = a.E.copy()
        Wb = orc.local_step(b, Wa, G, 1e-2, hp, 0.9)
        Wa = orc.local_step_bf16_residual(a, Wa, G, 1e-2, hp, 0.9)
        A = 0.9 * G + E_before
        assert np.array_equal(a.E, orc.round_to_bf16(A - Q @ (Q.T @ A)))
        assert np.array_equal(a.E, orc.round_to_bf16(b.E)) and np.array_equal(Wa, Wb)
        assert np.array_equal(a.u, b.u) and np.array_equal(a.v, b.v)
        assert np.linalg.norm(Q.T @ a.E) <= 2.0 ** -8 * np.linalg.norm(a.E)
        assert np.array_equal(orc.round_to_bf16(a.E), a.E)
