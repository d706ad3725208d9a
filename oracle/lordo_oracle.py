"""Float64 CPU oracle for the LoRDO per-matrix optimizer path.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
HIP library must compute; it is imported by tests/, by the smoke check and by
the benchmark's cpu_baseline leg and by nothing else.  It shares no code with
the HIP path and never sees a value produced by it, except where a test hands
it a basis on purpose (teacher forcing of the sign/rotation-ambiguous basis)
and, in the tests' first-step handling, the sign of an update whose argument is
zero to working precision (tests/harness.py checks that value against the
closed form before it is taken).

Every function is the paper's formula written out with numpy in float64, one
statement per line of the formula, no blocking, fusion or reordering.  Library
primitives used as steps: `@` (matmul), `numpy.linalg.qr`, `numpy.linalg.svd`.

Notation is the paper's: W in R^{p x q} (weights x), Q in R^{p x r} (projection,
orthonormal columns), g = Q^T G in R^{r x q} (low-rank gradient), u, v in
R^{r x q} (first and second moment), E in R^{p x q} (error buffer), t (count of
local steps taken so far), Delta (pseudo-gradient), b (outer momentum).

Readings of points the paper leaves open (each is stated again at its use):
  * bias correction (omitted "for ease of notation" in Alg. 1 and 2 but present
    in Sec. 2 and in the second-moment rotation) is ON by default:
    u_hat = u / (1 - beta1^t), v_hat = v / (1 - beta2^t), t never reset;
  * the squares in the second-moment rotation (Alg. 1, "rotate the second
    moment locally") are elementwise;
  * pseudo-gradient sign follows App. A.1 / A.2: Delta = anchor - x and the
    outer step is x <- anchor - eta_s * step(Delta);
  * Nesterov outer optimizer (App. D.4, D.5 name it, give no formula):
    b <- mu b + Delta ; x <- anchor - eta_s (Delta + mu b);
  * mu(z) of the full-rank QHM term (Sec. 3.2) is the mean over the rank index,
    one scale per column.

Parity pins live in tests/test_oracle_*.py.  Unpinned: nothing (the full-rank
QHM form is pinned by its reductions at omega = 0 and 1 and by the formula of
Sec. 3.2 written out with plain loops at an interior omega).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------
# hyper-parameters (Alg. 1, "Require")
# ----------------------------------------------------------------------------
@dataclass
class Hyper:
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    bias_correction: bool = True
    qhm_mode: str = "none"          # "none" | "low" | "full"   (Alg. 1, three cases of the update)
    omega: float = 1.0
    error_feedback: bool = False    # Alg. 1, error-feedback lines
    uplink_buffer: bool = False     # App. A.5.1: accumulate the low-rank updates of the window
    outer_lr: float = 1.0           # OuterOpt: averaging by default (Alg. 1, Require)
    outer_momentum: float = 0.0
    outer_nesterov: bool = False
    power_iters: int = 2
    rayleigh_ritz: bool = False     # order the basis as singular vectors (Sec. 2: Q = first r columns of U)


@dataclass
class MatrixState:
    """Optimizer state of one weight matrix."""
    Q: np.ndarray                   # p x r
    u: np.ndarray                   # r x q
    v: np.ndarray                   # r x q
    anchor: np.ndarray              # p x q : x_{t-K_x}
    E: np.ndarray | None = None     # p x q
    b: np.ndarray | None = None     # p x q
    A: np.ndarray | None = None     # r x q : up-link time buffer, sum over the window of eta_t N_t
    t: int = 0
    last_g: np.ndarray | None = field(default=None, repr=False)
    last_N: np.ndarray | None = field(default=None, repr=False)


def identity_projection(p: int, r: int) -> np.ndarray:
    """Q_0 = first r columns of the identity (Alg. 2, Require)."""
    Q = np.zeros((p, r), dtype=F64)
    Q[np.arange(r), np.arange(r)] = 1.0
    return Q


def init_state(W0: np.ndarray, r: int, Q0: np.ndarray | None = None) -> MatrixState:
    """u_{-1} = v_{-1} = 0, E_{-1} = 0 (Alg. 1, Require); anchor = x_0; b_0 = 0."""
    W0 = np.asarray(W0, dtype=F64)
    p, q = W0.shape
    Q = identity_projection(p, r) if Q0 is None else np.array(Q0, dtype=F64)
    assert Q.shape == (p, r)
    return MatrixState(Q=Q, u=np.zeros((r, q)), v=np.zeros((r, q)), anchor=W0.copy(),
                       E=np.zeros((p, q)), b=np.zeros((p, q)), A=np.zeros((r, q)), t=0)


# ----------------------------------------------------------------------------
# local step (Sec. 2, low-rank update equations; Alg. 1 inner loop)
# ----------------------------------------------------------------------------
def project_down(Q: np.ndarray, A: np.ndarray) -> np.ndarray:
    """g = Q^T A, r x q (Sec. 2; Alg. 1 low-rank gradient signal)."""
    return Q.T @ A


def update_moments(u, v, g, beta1, beta2):
    """u <- beta1 u + (1-beta1) g ; v <- beta2 v + (1-beta2) g*g (Sec. 2; Alg. 1)."""
    u_new = beta1 * u + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * (g * g)
    return u_new, v_new


def bias_factors(t: int, hp: Hyper):
    """c1 = 1 - beta1^t, c2 = 1 - beta2^t; both 1 when bias correction is off."""
    if not hp.bias_correction:
        return 1.0, 1.0
    return 1.0 - hp.beta1 ** t, 1.0 - hp.beta2 ** t


def low_rank_direction(u, v, g, t: int, hp: Hyper) -> np.ndarray:
    """Bracketed r x q term of the update (Alg. 1, cases "No QHM" and "Low-Rank QHM";
    the full-rank case uses the "No QHM" bracket).  eps sits outside the root (Sec. 2)."""
    c1, c2 = bias_factors(t, hp)
    u_hat = u / c1
    v_hat = v / c2
    denom = np.sqrt(v_hat) + hp.eps
    if hp.qhm_mode == "low":
        return (hp.omega * u_hat + (1.0 - hp.omega) * g) / denom
    return u_hat / denom


def project_up(Q: np.ndarray, N: np.ndarray) -> np.ndarray:
    """Q N, p x q (Sec. 2; Alg. 1 parameter update)."""
    return Q @ N


def local_step(st: MatrixState, W: np.ndarray, G: np.ndarray, lr: float, hp: Hyper,
               grad_scale: float = 1.0) -> np.ndarray:
    """One local step of Alg. 1 for one matrix.  Returns the new W; updates st."""
    W = np.asarray(W, dtype=F64)
    G_hat = grad_scale * np.asarray(G, dtype=F64)      # clipped gradient: caller's scale
    st.t += 1
    A = G_hat + st.E if hp.error_feedback else G_hat
    g = project_down(st.Q, A)
    if hp.error_feedback:
        st.E = A - project_up(st.Q, g)                 # E_t = G + E_{t-1} - Q g
    st.u, st.v = update_moments(st.u, st.v, g, hp.beta1, hp.beta2)
    N = low_rank_direction(st.u, st.v, g, st.t, hp)
    st.last_g, st.last_N = g, N
    if hp.uplink_buffer:                               # App. A.5.1: sum_tau eta_tau alpha_tau, alpha the bracketed term
        assert hp.qhm_mode != "full", "the full-rank QHM update has no low-rank form (App. A.5.1)"
        st.A = st.A + lr * N
    if hp.qhm_mode == "full":
        _, c2 = bias_factors(st.t, hp)
        col_scale = np.mean(np.sqrt(st.v / c2) + hp.eps, axis=0)      # mu(.) over the rank index
        step = (1.0 - hp.omega) * (G_hat / col_scale[None, :]) + hp.omega * project_up(st.Q, N)
    else:
        step = project_up(st.Q, N)
    return W - lr * step


# ----------------------------------------------------------------------------
# weights kept in bf16 (storage option; the paper does not state the precision of its runs, Sec. 5.1)
# ----------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 value (8 significant bits, the exponent range of float32), ties to even, of float64
    numbers, rounded ONCE from float64: x = f * 2^e with 1 <= |f| < 2 is moved to the nearest multiple of
    2^(e-7).  (Values below the smallest normal float32, 2^-126, do not occur in this use and are not handled.)"""
    x = np.asarray(x, dtype=F64)
    out = np.zeros_like(x)
    nz = x != 0
    e = np.floor(np.log2(np.abs(x[nz])))
    quantum = 2.0 ** (e - 7.0)
    out[nz] = np.rint(x[nz] / quantum) * quantum        # numpy's rint rounds halves to even
    return out


def local_step_bf16_weights(st: MatrixState, W: np.ndarray, G: np.ndarray, lr: float, hp: Hyper,
                            grad_scale: float = 1.0) -> np.ndarray:
    """The local step of Alg. 1 for weights that are STORED in bf16: the update is applied to the stored value in
    full precision and the result is rounded to bf16 once.  (Reading: the paper is silent on storage precision;
    moments, projection and every intermediate stay as they are, only x is kept in the short format.)"""
    return round_to_bf16(local_step(st, W, G, lr, hp, grad_scale))


def outer_step_bf16_weights(st: MatrixState, avg_delta: np.ndarray, hp: Hyper) -> np.ndarray:
    """Outer step for bf16-stored weights: OuterOpt in full precision from the anchor, the new model rounded once;
    the anchor of the next window is the model as stored."""
    W_new = round_to_bf16(outer_step(st, avg_delta, hp))
    st.anchor = W_new.copy()
    return W_new


def local_step_bf16_residual(st: MatrixState, W: np.ndarray, G: np.ndarray, lr: float, hp: Hyper,
                             grad_scale: float = 1.0) -> np.ndarray:
    """The local step of Alg. 1 with error feedback when the residual E is STORED in bf16 (same reading as for the
    weights): the step runs in full precision from the stored residual -- projection of G_hat + E, new residual
    G_hat + E - Q g -- and the new residual is rounded to bf16 once.  Nothing else changes."""
    W_new = local_step(st, W, G, lr, hp, grad_scale)
    st.E = round_to_bf16(st.E)
    return W_new


# ----------------------------------------------------------------------------
# projection on the right (Sec. 2 with the roles of rows and columns exchanged)
# ----------------------------------------------------------------------------
def local_step_right(st: MatrixState, W: np.ndarray, G: np.ndarray, lr: float, hp: Hyper,
                     grad_scale: float = 1.0) -> np.ndarray:
    """One local step with the projection on the right, written out on the p x q arrays:
    g = G_hat Q (p x r), Adam moments on g, W <- W - lr N Q^T, with Q of size q x r.  This is Sec. 2's update
    of the transposed matrix; `st` is the state of that transposed problem (Q: q x r; u, v, last_g, last_N: r x p,
    i.e. the transposes of the p x r arrays of this function; E: q x p).  In the "Full-Rank QHM" case (Sec. 3.2) the
    scale mu(.) of the gradient term, a mean over the rank index, belongs to the ROWS of W here: one value per row i,
    s_i = mean_k (sqrt(v_hat_ik) + eps), and the term is diag(1 / s) G_hat."""
    W = np.asarray(W, dtype=F64)
    G_hat = grad_scale * np.asarray(G, dtype=F64)
    st.t += 1
    A = G_hat + st.E.T if hp.error_feedback else G_hat  # st.E is kept in the layout of the transposed problem (q x p)
    g = A @ st.Q                                       # p x r
    if hp.error_feedback:
        st.E = (A - g @ st.Q.T).T                      # E_t = G + E_{t-1} - g Q^T
    u, v = update_moments(st.u.T, st.v.T, g, hp.beta1, hp.beta2)
    N = low_rank_direction(u, v, g, st.t, hp)          # p x r
    st.u, st.v = u.T, v.T
    st.last_g, st.last_N = g.T, N.T
    if hp.uplink_buffer:                               # App. A.5.1, in the layout of the transposed problem (r x p)
        assert hp.qhm_mode != "full", "the full-rank QHM update has no low-rank form (App. A.5.1)"
        st.A = st.A + lr * N.T
    if hp.qhm_mode == "full":
        _, c2 = bias_factors(st.t, hp)
        row_scale = np.mean(np.sqrt(v / c2) + hp.eps, axis=1)      # mu(.) over the rank index: one value per row of W
        return W - lr * ((1.0 - hp.omega) * (G_hat / row_scale[:, None]) + hp.omega * (N @ st.Q.T))
    return W - lr * (N @ st.Q.T)


def refresh_subspace_right(st: MatrixState, A_src: np.ndarray, Omega: np.ndarray, hp: Hyper,
                           Q_forced: np.ndarray | None = None) -> np.ndarray:
    """Refresh for the projection on the right: the right singular subspace of the source is the left one of its
    transpose, so this is ComputeProjection (Sec. 2) on A_src^T, Omega of size p x r, and the same rotation."""
    return refresh_subspace(st, np.asarray(A_src, dtype=F64).T, Omega, hp, Q_forced)


# ----------------------------------------------------------------------------
# subspace refresh (Sec. 2 "ComputeProjection"; Alg. 1 sync branch)
# ----------------------------------------------------------------------------
def svd_projection(A: np.ndarray, r: int) -> np.ndarray:
    """The paper's default: U, S, V = SVD(A); Q = U[:, :r] (Sec. 2)."""
    U, _, _ = np.linalg.svd(np.asarray(A, dtype=F64), full_matrices=False)
    return U[:, :r]


def orth(Y: np.ndarray) -> np.ndarray:
    """Thin QR (Householder), columns signed so that diag(R) > 0."""
    Qf, R = np.linalg.qr(Y)
    s = np.sign(np.diag(R))
    s[s == 0] = 1.0
    return Qf * s[None, :]


def initial_projection(block: np.ndarray) -> np.ndarray:
    """Q_0 of the global variant (Alg. 1, Require: a random initial projection): the orthonormal
    basis of a random p x r block, made unique by the positive diagonal of its triangular factor."""
    return orth(np.asarray(block, dtype=F64))


# ----------------------------------------------------------------------------
# random blocks the method draws (Alg. 1, Require: "random initial projection"; the Gaussian start of the
# range finder): a counter-based generator, so that a second implementation can draw the identical block
# ----------------------------------------------------------------------------
def philox4x32_10(counter: np.ndarray, key: np.ndarray) -> np.ndarray:
    """Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
    SC 2011).  counter: (..., 4) uint32, key: (..., 2) uint32 -> (..., 4) uint32.  One round: with
    (hi0, lo0) = 0xD2511F53 * c0 and (hi1, lo1) = 0xCD9E8D57 * c2 as 64-bit products,
    c <- (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0); the key is bumped by (0x9E3779B9, 0xBB67AE85) between rounds."""
    c = [np.asarray(counter, dtype=np.uint64)[..., i] for i in range(4)]
    k = [np.asarray(key, dtype=np.uint64)[..., i] for i in range(2)]
    mask = np.uint64(0xFFFFFFFF)
    for _ in range(10):
        prod0 = np.uint64(0xD2511F53) * c[0]
        prod1 = np.uint64(0xCD9E8D57) * c[2]
        hi0, lo0 = prod0 >> np.uint64(32), prod0 & mask
        hi1, lo1 = prod1 >> np.uint64(32), prod1 & mask
        c = [hi1 ^ c[1] ^ k[0], lo1, hi0 ^ c[3] ^ k[1], lo0]
        k = [(k[0] + np.uint64(0x9E3779B9)) & mask, (k[1] + np.uint64(0xBB67AE85)) & mask]
    return np.stack(c, axis=-1).astype(np.uint32)


def gaussian_block(seed: int, matrix: int, draw: int, rows: int, cols: int) -> np.ndarray:
    """rows x cols block of standard normals: element e (row-major) is output e % 4 of
    Philox-4x32-10(counter = (e // 4 low word, e // 4 high word, matrix, draw), key = (seed low, seed high)),
    the four outputs turned into normals in pairs by Box-Muller: u = ((x >> 8) + 1/2) 2^-24 lies in (0, 1);
    (z0, z1) = sqrt(-2 ln u0) (cos 2 pi u1, sin 2 pi u1) from outputs 0 and 1, (z2, z3) likewise from 2 and 3."""
    total = rows * cols
    nquads = (total + 3) // 4
    quad = np.arange(nquads, dtype=np.uint64)
    counter = np.stack([quad & np.uint64(0xFFFFFFFF), quad >> np.uint64(32),
                        np.full(nquads, matrix, dtype=np.uint64), np.full(nquads, draw, dtype=np.uint64)], axis=-1)
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint64)
    x = philox4x32_10(counter, np.broadcast_to(key, (nquads, 2)))
    u = ((x >> np.uint32(8)).astype(F64) + 0.5) * 2.0 ** -24
    z = np.empty((nquads, 4), dtype=F64)
    for h in range(2):
        rad = np.sqrt(-2.0 * np.log(u[:, 2 * h]))
        ang = 2.0 * np.pi * u[:, 2 * h + 1]
        z[:, 2 * h] = rad * np.cos(ang)
        z[:, 2 * h + 1] = rad * np.sin(ang)
    return z.reshape(-1)[:total].reshape(rows, cols)


def range_finder(A: np.ndarray, Omega: np.ndarray, power_iters: int) -> np.ndarray:
    """Block power iteration with a Gaussian start, orthonormalised after every product:
    Y = orth(A Omega); repeat: Z = orth(A^T Y); Y = orth(A Z)."""
    A = np.asarray(A, dtype=F64)
    Y = orth(A @ np.asarray(Omega, dtype=F64))
    for _ in range(power_iters):
        Z = orth(A.T @ Y)
        Y = orth(A @ Z)
    return Y


def rayleigh_ritz(Q: np.ndarray, A: np.ndarray):
    """Turn an orthonormal basis Q of (approximately) the leading left singular subspace of A into
    (approximate) singular vectors in the order of Sec. 2's ComputeProjection (Q = U[:, :r] of the SVD,
    largest singular value first): B = Q^T A (r x q) is the matrix restricted to the subspace;
    B = U_B S V^T is a small SVD; Q U_B are the Ritz vectors and S the Ritz values.  The span is unchanged.
    Each column is signed so that its entry of largest magnitude is positive.  Returns (Q U_B, S)."""
    Q = np.asarray(Q, dtype=F64)
    B = Q.T @ np.asarray(A, dtype=F64)
    U_B, S, _ = np.linalg.svd(B, full_matrices=False)
    Qr = Q @ U_B[:, :Q.shape[1]]
    lead = np.argmax(np.abs(Qr), axis=0)
    sign = np.sign(Qr[lead, np.arange(Qr.shape[1])])
    sign[sign == 0] = 1.0
    return Qr * sign[None, :], S[:Q.shape[1]]


def rotate_moments(Q_new, Q_old, u, v, t: int, hp: Hyper):
    """Alg. 1, "rotate the first / second moment locally" (same lines in Alg. 2):
    R = Q_new^T Q_old;  u <- R u;
    v <- (1 - beta2^t) | (R o R)(v_hat - u_hat o u_hat) + (R u_hat) o (R u_hat) |."""
    R = Q_new.T @ Q_old
    c1, c2 = bias_factors(t, hp)
    u_hat = u / c1
    v_hat = v / c2
    u_new = R @ u
    Ru = R @ u_hat
    v_new = c2 * np.abs((R * R) @ (v_hat - u_hat * u_hat) + Ru * Ru)
    return u_new, v_new


def refresh_subspace(st: MatrixState, A_src: np.ndarray, Omega: np.ndarray, hp: Hyper,
                     Q_forced: np.ndarray | None = None) -> np.ndarray:
    """New projection from A_src, then rotation of both moments into it.
    `Q_forced` replaces the computed basis (tests use it to teacher-force the
    basis the other implementation found; the rotation is basis dependent)."""
    if Q_forced is None:
        Q_new = range_finder(A_src, Omega, hp.power_iters)
        if hp.rayleigh_ritz:
            Q_new, _ = rayleigh_ritz(Q_new, A_src)
    else:
        Q_new = np.asarray(Q_forced, dtype=F64)
    if st.t > 0:                                        # before any step both moments are zero
        st.u, st.v = rotate_moments(Q_new, st.Q, st.u, st.v, st.t, hp)
    st.Q = Q_new
    return Q_new


def local_variant_source(st: MatrixState, G: np.ndarray, grad_scale: float = 1.0) -> np.ndarray:
    """Argument of ComputeProjection in the local variant (Alg. 2): the clipped gradient of the
    step plus the error buffer the previous step left, G_hat_t + E_{t-1}."""
    return grad_scale * np.asarray(G, dtype=F64) + st.E


def mssv(Q_new: np.ndarray, Q_old: np.ndarray) -> float:
    """Mean squared singular value of R = Q_new^T Q_old (Sec. 5.1, Metrics):
    (1/r) sum sigma_i^2 = ||R||_F^2 / r."""
    R = Q_new.T @ Q_old
    return float(np.sum(R * R) / R.shape[0])


# ----------------------------------------------------------------------------
# outer step (Alg. 1 sync branch; App. A.1, A.2; App. D.4, D.5)
# ----------------------------------------------------------------------------
def stable_rank(A: np.ndarray) -> float:
    """Stable rank (Sec. 5.1, Metrics): sr(A) = ||A||_F^2 / ||A||_2^2, the spectral norm from the library SVD."""
    A = np.asarray(A, dtype=F64)
    sigma = np.linalg.svd(A, compute_uv=False)
    return float(np.sum(A * A) / sigma[0] ** 2)


def spectral_gap(A: np.ndarray, r: int) -> float:
    """The r-th spectral gap sigma_r - sigma_{r+1} (Sec. 5.1, Metrics), singular values from the library SVD
    (sigma_{r+1} = 0 when the matrix has only r of them)."""
    sigma = np.linalg.svd(np.asarray(A, dtype=F64), compute_uv=False)
    return float(sigma[r - 1] - (sigma[r] if r < len(sigma) else 0.0))


def next_singular_value_estimate(A: np.ndarray, Q: np.ndarray, Omega: np.ndarray, iters: int = 2) -> float:
    """Estimate of sigma_{r+1}(A) given a basis Q of the leading r-dimensional left singular subspace: block power
    iteration (the range finder above) on the deflated matrix (I - Q Q^T) A, then the largest singular value of the
    matrix restricted to the block found.  Never above the spectral norm of the deflated matrix."""
    A = np.asarray(A, dtype=F64)
    Q = np.asarray(Q, dtype=F64)

    def deflate(Y):
        return Y - Q @ (Q.T @ Y)

    Y = orth(deflate(A @ np.asarray(Omega, dtype=F64)))
    for _ in range(iters):
        Z = orth(A.T @ Y)                 # = ((I - Q Q^T) A)^T Y, since Y is orthogonal to Q
        Y = orth(deflate(A @ Z))
    # When the deflated matrix has fewer than r nonzero singular values (2r > min(p, q)), the orthonormalisation
    # completes the block with directions that need not be orthogonal to Q: deflating the block once more keeps
    # the result below the norm of the deflated matrix (it changes nothing for a block orthogonal to Q).
    return float(np.linalg.svd(deflate(Y).T @ A, compute_uv=False)[0])


def pseudo_gradient(st: MatrixState, W: np.ndarray) -> np.ndarray:
    """Delta^m = x_{t-K_x} - x_t  (App. A.1 sign convention)."""
    return st.anchor - np.asarray(W, dtype=F64)


def outer_step_lowrank(st: MatrixState, avg_A: np.ndarray, hp: Hyper) -> np.ndarray:
    """Outer step from the averaged up-link buffers (App. A.5.1): with one projection shared by all
    workers the mean pseudo-gradient is rebuilt as Delta = Q mean_m(A^m), then the ordinary outer
    step; a new window starts with an empty buffer."""
    W_new = outer_step(st, st.Q @ np.asarray(avg_A, dtype=F64), hp)
    return W_new


def outer_step(st: MatrixState, avg_delta: np.ndarray, hp: Hyper) -> np.ndarray:
    """x <- OuterOpt(Delta, x_{t-K_x}).  Plain: x = anchor - eta_s Delta (eta_s = 1 is
    averaging).  With momentum mu: b <- mu b + Delta; step = Delta + mu b (Nesterov)
    or b (heavy ball).  The new x becomes the anchor of the next window."""
    D = np.asarray(avg_delta, dtype=F64)
    st.b = hp.outer_momentum * st.b + D
    step = D + hp.outer_momentum * st.b if hp.outer_nesterov else st.b
    W_new = st.anchor - hp.outer_lr * step
    st.anchor = W_new.copy()
    if st.A is not None:
        st.A = np.zeros_like(st.A)                     # the window's accumulated update has been consumed
    return W_new
