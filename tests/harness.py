"""Side-by-side driver of the float64 oracle and the HIP library on identical seeded inputs.

The two implementations share nothing but the input arrays built here.  The only value that
ever travels from the HIP side to the oracle is a basis handed over on purpose (teacher
forcing, because the second-moment rotation depends on the basis and not only on its span)
and the sign decision of elements whose first-step update is the sign of a number that is
zero to working precision (see `first_step_patch`).
"""
from __future__ import annotations

import numpy as np

from oracle import lordo_oracle as orc
from paper_2602_04396_amd import synth


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def projector_distance(Qa, Qb):
    """|| Qa Qa^T - Qb Qb^T ||_F computed without forming p x p matrices:
    = sqrt(ra + rb - 2 ||Qa^T Qb||_F^2) for orthonormal bases."""
    Qa = np.asarray(Qa, dtype=np.float64)
    Qb = np.asarray(Qb, dtype=np.float64)
    ga = Qa.T @ Qa
    gb = Qb.T @ Qb
    cross = Qa.T @ Qb
    val = np.sum(ga * ga) + np.sum(gb * gb) - 2.0 * np.sum(cross * cross)
    return float(np.sqrt(max(val, 0.0)))


def check_first_step_closed_form(N_lib, g_lib, ohp, where, t=1):
    """First step from the zero state (Alg. 1 moment and update lines at t = 1): u = (1 - beta1) g,
    v = (1 - beta2) g^2, so the bracketed update is a function of g alone,
        N = (w u_hat + (1 - w) g) / (sqrt(v_hat) + eps),   w = omega for the low-rank QHM case, else 1.
    (t > 1: the same after t steps with one constant gradient, u = (1 - beta1^t) g, v = (1 - beta2^t) g^2.)
    Where a test takes the library's N (elements whose g is zero to working precision) that value must be this
    closed form evaluated at the library's OWN g, to fp32 accuracy: |N| <= 1, so 2e-5 absolute covers the
    2^-17 split of N into two bf16 planes and the fp32 arithmetic."""
    g = np.asarray(g_lib, dtype=np.float64)[where]
    N = np.asarray(N_lib, dtype=np.float64)[where]
    c1 = 1.0 - ohp.beta1 ** t if ohp.bias_correction else 1.0
    c2 = 1.0 - ohp.beta2 ** t if ohp.bias_correction else 1.0
    u_hat = (1.0 - ohp.beta1 ** t) * g / c1
    den = np.sqrt((1.0 - ohp.beta2 ** t) * g * g / c2) + ohp.eps
    w = ohp.omega if ohp.qhm_mode == "low" else 1.0
    with np.errstate(invalid="ignore", divide="ignore"):
        closed = np.where(den > 0, (w * u_hat + (1.0 - w) * g) / den, 0.0)
    assert np.all(np.abs(N) <= 1.0 + 1e-6)
    assert np.max(np.abs(N - closed), initial=0.0) <= 2e-5, "library N at a sign-ambiguous element is not g / (|g| + eps) of its own g"


class Pair:
    """Oracle states + one Lordo context over the same matrices."""

    def __init__(self, torch, shapes, W0, oracle_hp: orc.Hyper, gpu_hp, Q0=None):
        from paper_2602_04396_amd import lordo
        self.torch = torch
        self.lordo = lordo
        self.shapes = shapes
        self.ohp = oracle_hp
        self.dev = torch.device("cuda:0")
        self.W_gpu = [torch.tensor(w, dtype=torch.float32, device=self.dev).contiguous() for w in W0]
        self.W_orc = [np.asarray(w, dtype=np.float64).copy() for w in W0]
        self.W0 = [w.copy() for w in self.W_orc]
        self.opt = lordo.Lordo(shapes, gpu_hp, self.W_gpu, torch)
        self.st = []
        # a shape may carry a fourth entry, side: 1 = projection on the right; the oracle state of such a matrix is
        # the state of the transposed problem (as the library's low-rank arrays are)
        self.side = [int(sh[3]) if len(sh) > 3 else 0 for sh in shapes]
        for i, sh in enumerate(shapes):
            r = sh[2]
            q0 = None if Q0 is None else Q0[i]
            self.st.append(orc.init_state(self.W_orc[i].T if self.side[i] else self.W_orc[i], r, q0))
            if q0 is not None:
                self.opt.set_state(i, lordo.STATE_Q, torch.tensor(q0, dtype=torch.float32, device=self.dev).contiguous())
                # the oracle continues from the fp32 value the library was given
                self.st[i].Q = np.asarray(q0, dtype=np.float32).astype(np.float64)

    # ------------------------------------------------------------------------------------------
    def to_dev(self, arrs, bf16):
        t = self.torch
        out = []
        for a in arrs:
            x = t.tensor(np.asarray(a, dtype=np.float32), device=self.dev)
            out.append((x.to(t.bfloat16) if bf16 else x).contiguous())
        return out

    def get(self, i, which):
        return self.opt.get_state(i, which).cpu().numpy().astype(np.float64)

    def local_step(self, G, lr, grad_scale=1.0, bf16=True, first_step_patch=False):
        """G: list of float32 arrays (already bf16-representable when bf16=True)."""
        Gd = getattr(self, "_held_G", None) or self.to_dev(G, bf16)     # the tensors a local-variant refresh was given
        self._held_G = None
        self.opt.local_step(self.W_gpu, Gd, lr, grad_scale)
        self.torch.cuda.synchronize()
        patched = 0
        for i in range(len(self.shapes)):
            step = orc.local_step_right if self.side[i] else orc.local_step
            self.W_orc[i] = step(self.st[i], self.W_orc[i], np.asarray(G[i], dtype=np.float64), lr, self.ohp, grad_scale)
            if first_step_patch:
                patched += self._patch_sign_ambiguous(i, lr)
        return patched

    def _patch_sign_ambiguous(self, i, lr):
        """From a zero state the update is N = g / (|g| + eps): the sign of g.  Where |g| is
        below what fp32 accumulation can resolve, either sign (any value in [-1, 1]) is a correct
        answer; take the library's value there after checking that it is the closed form of the first
        step evaluated at the library's own g, and that only a sliver of the elements is concerned."""
        st = self.st[i]          # (called at t > 1 only by the constant-gradient test, where the same closed form holds)
        g = st.last_g
        tau = 1e-4 * np.sqrt(np.mean(g * g))
        amb = np.abs(g) < tau
        if not amb.any():
            return 0
        assert amb.sum() <= 1e-3 * g.size + 3, f"{int(amb.sum())} of {g.size} elements below the resolution of g"
        N_gpu = self.get(i, self.lordo.STATE_NUPD)
        g_gpu = self.get(i, self.lordo.STATE_GLOW)
        check_first_step_closed_form(N_gpu, g_gpu, self.ohp, amb, st.t)
        N_new = st.last_N.copy()
        N_new[amb] = N_gpu[amb]
        weight = self.ohp.omega if self.ohp.qhm_mode == "full" else 1.0      # share of Q N in the update
        fix = lr * weight * st.Q @ (st.last_N - N_new)
        self.W_orc[i] = self.W_orc[i] + (fix.T if self.side[i] else fix)
        if self.ohp.uplink_buffer:
            st.A = st.A + lr * (N_new - st.last_N)
        st.last_N = N_new
        return int(amb.sum())

    def compare_local(self, tol=1e-4, check_N=True):
        L = self.lordo
        worst = {}
        for i in range(len(self.shapes)):
            st = self.st[i]
            errs = {
                "g": rel_l2(self.get(i, L.STATE_GLOW), st.last_g),
                "u": rel_l2(self.get(i, L.STATE_U), st.u),
                "v": rel_l2(self.get(i, L.STATE_V), st.v),
                "dW": rel_l2(self.W_gpu[i].cpu().numpy().astype(np.float64) - self.W0[i], self.W_orc[i] - self.W0[i]),
            }
            if check_N:
                errs["N"] = rel_l2(self.get(i, L.STATE_NUPD), st.last_N)
            if self.ohp.error_feedback:
                # E = A - Q g is a difference of two matrices of the size of A = G_hat + E_prev: an error
                # of tol * ||g|| in g alone (the bound on g above) moves E by tol * ||A|| when Q holds most
                # of A, however small E itself is.  So E is held to tol relative to ||A||, and
                # ||A||^2 = ||g||^2 + ||E||^2 for orthonormal Q.
                scale = np.sqrt(np.sum(st.last_g * st.last_g) + np.sum(st.E * st.E))
                E_gpu = self.get(i, L.STATE_ERR)             # the caller's layout; the oracle state of a right-projected matrix holds E^T
                errs["E"] = float(np.linalg.norm((E_gpu.T if self.side[i] else E_gpu) - st.E) / max(scale, 1e-300))
            if self.ohp.uplink_buffer:
                errs["A"] = rel_l2(self.get(i, L.STATE_UPLINK), st.A)
            for k, e in errs.items():
                worst[k] = max(worst.get(k, 0.0), e)
                assert e <= tol, f"matrix {i} {self.shapes[i]}: rel L2 error of {k} = {e:.3e} > {tol}"
        return worst

    def refresh(self, Src, Omega, bf16):
        """Library refresh, then the oracle's own refresh for the subspace check, then the oracle
        redoes the rotation with the library's basis.  Returns (projector distances, orthonormality)."""
        L = self.lordo
        Sd = self.to_dev(Src, bf16)
        Od = self.to_dev(Omega, False)
        self.opt.refresh_subspace(Sd, Od)
        self.opt.poll_status()
        dists, orths = [], []
        for i, sh in enumerate(self.shapes):
            r = sh[2]
            Qg = self.get(i, L.STATE_Q)
            orths.append(float(np.linalg.norm(Qg.T @ Qg - np.eye(r))))
            src = np.asarray(Src[i], dtype=np.float64)
            Qo = orc.range_finder(src.T if self.side[i] else src, np.asarray(Omega[i], dtype=np.float64), self.ohp.power_iters)
            dists.append(projector_distance(Qg, Qo))
            orc.refresh_subspace(self.st[i], None, None, self.ohp, Q_forced=Qg)
        return dists, orths

    def refresh_local(self, G, Omega, grad_scale=1.0, bf16=True):
        """Refresh of the local variant (Alg. 2): the library folds the gradient into its error
        buffer and refreshes from the sum; the oracle forms G_hat + E itself.  The following
        `local_step` must be given the same G; the device tensors are kept for it."""
        L = self.lordo
        self._held_G = self.to_dev(G, bf16)
        Od = self.to_dev(Omega, False)
        self.opt.refresh_subspace_local(self._held_G, Od, grad_scale)
        self.opt.poll_status()
        dists, orths = [], []
        for i, sh in enumerate(self.shapes):
            r = sh[2]
            Qg = self.get(i, L.STATE_Q)
            orths.append(float(np.linalg.norm(Qg.T @ Qg - np.eye(r))))
            Gi = np.asarray(G[i], dtype=np.float64)
            src = orc.local_variant_source(self.st[i], Gi.T if self.side[i] else Gi, grad_scale)     # in the layout of the oracle state
            Qo = orc.range_finder(src, np.asarray(Omega[i], dtype=np.float64), self.ohp.power_iters)
            dists.append(projector_distance(Qg, Qo))
            orc.refresh_subspace(self.st[i], None, None, self.ohp, Q_forced=Qg)
        return dists, orths
