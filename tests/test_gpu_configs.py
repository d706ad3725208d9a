"""Parity at the full size and launch configuration of the larger workloads (generated on the device exactly as
bench.py does): c3 (~1B set, 168 matrices, r = 256, Student-t gradients), c4 (~7B set, 224 matrices, r = 512) and
c5 (one 8192 x 28672 matrix, ranks 64 and 1024).  The float64 oracle follows sampled columns of one matrix per
distinct shape -- every formula of the local step, of the moment rotation and of the outer step acts column by
column -- and recomputes the refreshed subspace of those matrices in full with its own range finder.  For the plain
update the second step is also checked on EVERY element of EVERY matrix against lr Q N from the library's own Q and N."""
import numpy as np
import pytest

from oracle import lordo_oracle as orc
from paper_2602_04396_amd import synth
from tests.harness import check_first_step_closed_form, projector_distance, rel_l2

pytestmark = pytest.mark.gpu

TOL = 1e-4
TOL_SUBSPACE = 1e-3
TOL_ORTH = 1e-4


def _f64(t):
    return t.float().cpu().numpy().astype(np.float64)


class Sampled:
    """Oracle states on sampled columns of picked matrices of one library context."""

    def __init__(self, torch, lordo, opt, shapes, W, picked, ohp, seed):
        self.torch, self.lordo, self.opt, self.shapes, self.W, self.ohp = torch, lordo, opt, shapes, W, ohp
        self.picked = picked
        rng = np.random.default_rng(seed)
        self.s = {}
        for i in picked:
            p, q, r = shapes[i]
            Q = _f64(opt.get_state(i, lordo.STATE_Q))
            assert np.linalg.norm(Q.T @ Q - np.eye(r)) <= TOL_ORTH
            cols = np.unique(np.concatenate([[0, 1, q - 1, 127, 128, 255, 256, 257, q - 257], rng.integers(0, q, 10)]))
            st = orc.init_state(_f64(W[i][:, cols]), r, Q)
            self.s[i] = dict(cols=cols, st=st, W=st.anchor.copy())

    def cols_of(self, i, which):
        return _f64(self.opt.get_state(i, which))[:, self.s[i]["cols"]]

    def local_step(self, Wp, Gp, G, lr, tag):
        torch, lordo = self.torch, self.lordo
        before = {i: _f64(self.W[i][:, self.s[i]["cols"]]) for i in self.picked}
        self.opt.local_step(Wp, Gp, lr)
        torch.cuda.synchronize()
        for i in self.picked:
            sm = self.s[i]
            st, cols = sm["st"], sm["cols"]
            first = st.t == 0
            sm["W"] = orc.local_step(st, before[i], _f64(G[i][:, cols]), lr, self.ohp)      # from the weights as the library holds them
            where = f"{tag}, matrix {i} {self.shapes[i]}"
            assert rel_l2(self.cols_of(i, lordo.STATE_GLOW), st.last_g) <= TOL, "g, " + where
            assert rel_l2(self.cols_of(i, lordo.STATE_U), st.u) <= TOL, "u, " + where
            assert rel_l2(self.cols_of(i, lordo.STATE_V), st.v) <= TOL, "v, " + where
            n_gpu = self.cols_of(i, lordo.STATE_NUPD)
            dW_gpu = _f64(self.W[i][:, cols]) - before[i]
            if first:
                # from a zero state N = g / (|g| + eps) is the sign of g: where |g| is below what fp32 resolves the
                # library's value is taken after the closed-form check, and the oracle continues from it
                amb = np.abs(st.last_g) < 1e-4 * np.sqrt(np.mean(st.last_g ** 2))
                assert amb.sum() <= 1e-3 * amb.size + 3
                check_first_step_closed_form(n_gpu, self.cols_of(i, lordo.STATE_GLOW), self.ohp, amb)
                N_new = np.where(amb, n_gpu, st.last_N)
                share = self.ohp.omega if self.ohp.qhm_mode == "full" else 1.0           # weight of Q N in the update
                sm["W"] = sm["W"] + lr * share * st.Q @ (st.last_N - N_new)
                st.last_N = N_new
            assert rel_l2(n_gpu, st.last_N) <= TOL, "N, " + where
            assert rel_l2(dW_gpu, sm["W"] - before[i]) <= TOL, "weight change, " + where
            if self.ohp.error_feedback:     # held relative to the matrix that was projected (||A||^2 = ||g||^2 + ||E||^2)
                scale = np.sqrt(np.sum(st.last_g ** 2) + np.sum(st.E ** 2))
                assert np.linalg.norm(self.cols_of(i, lordo.STATE_ERR) - st.E) <= TOL * scale, "E, " + where

    def outer_step(self, Wp, Dp, D, tag):
        lordo = self.lordo
        self.opt.outer_step(Wp, Dp)
        self.torch.cuda.synchronize()
        for i in self.picked:
            sm = self.s[i]
            st, cols = sm["st"], sm["cols"]
            anchor_before = st.anchor.copy()
            sm["W"] = orc.outer_step(st, _f64(D[i][:, cols]), self.ohp)
            got = _f64(self.W[i][:, cols])
            assert rel_l2(got - anchor_before, sm["W"] - anchor_before) <= TOL, f"outer step, {tag}, matrix {i}"
            assert self.torch.equal(self.opt.get_state(i, lordo.STATE_ANCHOR), self.W[i])
            if self.ohp.outer_momentum != 0:
                assert rel_l2(_f64(self.opt.get_state(i, lordo.STATE_MOM))[:, cols], st.b) <= TOL, f"momentum, {tag}, matrix {i}"

    def refresh(self, Src, Omega, power_iters, tag, full_oracle_for):
        """Library refresh on the whole set; the oracle's own range finder on the matrices in `full_oracle_for`
        (projector distance), and the rotation of the sampled moment columns with the library's basis."""
        lordo, opt = self.lordo, self.opt
        opt.refresh_subspace(Src, Omega)
        opt.poll_status()
        for i in self.picked:
            p, q, r = self.shapes[i]
            Qg = _f64(opt.get_state(i, lordo.STATE_Q))
            assert np.linalg.norm(Qg.T @ Qg - np.eye(r)) <= TOL_ORTH, f"orthonormality, {tag}, matrix {i}"
            if i in full_oracle_for:
                src = Src.tensors[i] if hasattr(Src, "tensors") else Src[i]
                om = Omega.tensors[i] if hasattr(Omega, "tensors") else Omega[i]
                Qo = orc.range_finder(_f64(src), _f64(om), power_iters)
                d = projector_distance(Qg, Qo)
                print(f"{tag}: matrix {i} {self.shapes[i]} projector distance {d:.2e}", flush=True)
                assert d <= TOL_SUBSPACE, f"subspace, {tag}, matrix {i}: {d:.3e}"
            st = self.s[i]["st"]
            orc.refresh_subspace(st, None, None, self.ohp, Q_forced=Qg)      # the rotation acts column by column
            if st.t > 0:
                assert rel_l2(self.cols_of(i, lordo.STATE_U), st.u) <= TOL, f"rotated u, {tag}, matrix {i}"
                assert rel_l2(self.cols_of(i, lordo.STATE_V), st.v) <= TOL, f"rotated v, {tag}, matrix {i}"


def _whole_state_after_first_step(opt, lordo, shapes, G0, ohp, tag):
    """The whole low-rank state after the first step from the zero state, every matrix: g against Q^T G from the library
    GEMM (the residual is zero at this step), and the moments against their closed form, u = (1 - beta1) g,
    v = (1 - beta2) g^2."""
    worst = 0.0
    for i in range(len(shapes)):
        g = opt.get_state(i, lordo.STATE_GLOW)
        ref = opt.get_state(i, lordo.STATE_Q).T @ G0[i].float()
        rms = float(ref.square().mean().sqrt())
        dev = float((g - ref).abs().max())
        worst = max(worst, dev / rms)
        assert dev <= 1e-3 * rms, f"{tag} matrix {i} {shapes[i]}: g deviates from Q^T G by {dev:.3e} somewhere (rms {rms:.3e})"
        u, v = opt.get_state(i, lordo.STATE_U), opt.get_state(i, lordo.STATE_V)
        assert float((u - (1.0 - ohp.beta1) * g).abs().max()) <= 1e-6 * rms, f"{tag} matrix {i}: u after the first step"
        assert float((v - (1.0 - ohp.beta2) * g * g).abs().max()) <= 1e-6 * rms * rms, f"{tag} matrix {i}: v after the first step"
    print(f"{tag}: whole-array check of g, u, v after the first step over {len(shapes)} matrices, largest deviation of g / its rms {worst:.2e}", flush=True)


def _whole_weight_change(opt, lordo, shapes, W_before, W, lr, tag):
    """Every element of every matrix after a step of the plain update: W_before - W = lr Q N, with Q N formed by the library
    GEMM from the library's own Q and N (the sampled columns tie those to the oracle).  A tile written to the wrong place,
    twice or not at all, in any of the matrices, is off by the size of the change; fp32 rounding of W is four orders below
    it.  Consumes W_before."""
    worst = 0.0
    for i in range(len(shapes)):
        ref = opt.get_state(i, lordo.STATE_Q) @ opt.get_state(i, lordo.STATE_NUPD)
        ref *= lr
        rms = float(ref.square().mean().sqrt())
        W_before[i] -= W[i]
        W_before[i] -= ref
        dev = float(W_before[i].abs().max())
        worst = max(worst, dev / rms)
        assert dev <= 2e-2 * rms, f"{tag} matrix {i} {shapes[i]}: the change deviates from lr Q N by {dev:.3e} somewhere (rms of the change {rms:.3e})"
        W_before[i] = None
    print(f"{tag}: whole-array check of the weight change over {len(shapes)} matrices, largest deviation / rms of the change {worst:.2e}", flush=True)


def _whole_residual(opt, lordo, shapes, G_t, E_prev, tag):
    """Every element of every residual after a step (Alg. 1 error-feedback lines): E = G + E_prev - Q g, with Q g formed by
    the library GEMM from the library's own Q and g; E_prev None = the zero residual of the first step."""
    worst = 0.0
    for i in range(len(shapes)):
        ref = G_t[i].float()
        if E_prev is not None:
            ref += E_prev[i]
        scale = float(ref.square().mean().sqrt())
        ref -= opt.get_state(i, lordo.STATE_Q) @ opt.get_state(i, lordo.STATE_GLOW)
        dev = float((opt.get_state(i, lordo.STATE_ERR) - ref).abs().max())
        worst = max(worst, dev / scale)
        assert dev <= 1e-3 * scale, f"{tag} matrix {i} {shapes[i]}: the residual deviates from G + E - Q g by {dev:.3e} somewhere (rms of G + E {scale:.3e})"
    print(f"{tag}: whole-array check of the residual over {len(shapes)} matrices, largest deviation / rms of G + E {worst:.2e}", flush=True)


def _whole_weight_change_full_qhm(opt, lordo, shapes, W_before, W, G_t, lr, ohp, t, tag):
    """Every element of every matrix after step t of the full-rank QHM update (Sec. 3.2; Alg. 1 "Full-Rank QHM"):
    W_before - W = lr [omega Q N + (1 - omega) G diag(1 / s)], s_j = mean over the rank of sqrt(v_hat_kj) + eps, from the
    library's own Q, N and v.  Consumes W_before."""
    worst = 0.0
    c2 = 1.0 - ohp.beta2 ** t if ohp.bias_correction else 1.0
    for i in range(len(shapes)):
        s_col = ((opt.get_state(i, lordo.STATE_V) / c2).sqrt() + ohp.eps).mean(dim=0)
        ref = opt.get_state(i, lordo.STATE_Q) @ opt.get_state(i, lordo.STATE_NUPD)
        ref *= lr * ohp.omega
        ref += (lr * (1.0 - ohp.omega)) * (G_t[i].float() / s_col[None, :])
        rms = float(ref.square().mean().sqrt())
        W_before[i] -= W[i]
        W_before[i] -= ref
        dev = float(W_before[i].abs().max())
        worst = max(worst, dev / rms)
        assert dev <= 2e-2 * rms, f"{tag} matrix {i} {shapes[i]}: the change deviates from the full-rank QHM update by {dev:.3e} somewhere (rms {rms:.3e})"
        W_before[i] = None
    print(f"{tag}: whole-array check of the full-rank QHM weight change over {len(shapes)} matrices, largest deviation / rms {worst:.2e}", flush=True)


def _whole_rotation(opt, lordo, shapes, old, t, ohp, tag):
    """Every element of every moment array after a refresh (Alg. 1, rotation of the moments): with R = Q_new^T Q_old from
    the library's own bases, u = R u_old and v = c2 |(R o R)(v_hat - u_hat^2) + (R u_hat)^2|, evaluated in fp32 by the
    library GEMM; `old` holds (Q, u, v) of every matrix from before the refresh."""
    c1 = 1.0 - ohp.beta1 ** t if ohp.bias_correction else 1.0
    c2 = 1.0 - ohp.beta2 ** t if ohp.bias_correction else 1.0
    worst = 0.0
    for i in range(len(shapes)):
        Q_old, u_old, v_old = old[i]
        R = opt.get_state(i, lordo.STATE_Q).T @ Q_old
        u_hat = u_old / c1
        Ru = R @ u_hat
        v_ref = c2 * ((R * R) @ (v_old / c2 - u_hat * u_hat) + Ru * Ru).abs()
        u_ref = R @ u_old
        du = float((opt.get_state(i, lordo.STATE_U) - u_ref).abs().max()) / float(u_ref.square().mean().sqrt())
        dv = float((opt.get_state(i, lordo.STATE_V) - v_ref).abs().max()) / float(v_ref.square().mean().sqrt())
        worst = max(worst, du, dv)
        assert du <= 1e-3 and dv <= 1e-3, f"{tag} matrix {i} {shapes[i]}: rotated moments deviate by {du:.3e} (u), {dv:.3e} (v) of their rms somewhere"
        old[i] = None
    print(f"{tag}: whole-array check of the rotated moments over {len(shapes)} matrices, largest deviation / rms {worst:.2e}", flush=True)


def _whole_subspace(opt, lordo, shapes, Src, Omega, power_iters, tag):
    """The refreshed subspace of EVERY matrix against the same range finder (Sec. 2 ComputeProjection as block power
    iteration) run in fp32 with the library QR and GEMM of torch on the same source and start block: projector distance."""
    import torch
    worst = 0.0
    for i, (p, q, r) in enumerate(shapes):
        A = Src[i].float()
        Y = torch.linalg.qr(A @ Omega[i]).Q
        for _ in range(power_iters):
            Z = torch.linalg.qr(A.T @ Y).Q
            Y = torch.linalg.qr(A @ Z).Q
        Ql = opt.get_state(i, lordo.STATE_Q)
        # || Y Y^T - Q Q^T ||_F = sqrt(2) || (I - Y Y^T) Q ||_F for two orthonormal bases of equal rank (the form that does
        # not cancel in fp32)
        dist = float(2.0 ** 0.5 * torch.linalg.norm(Ql - Y @ (Y.T @ Ql)))
        worst = max(worst, dist)
        assert dist <= TOL_SUBSPACE, f"{tag} matrix {i} {shapes[i]}: projector distance {dist:.3e} to the fp32 range finder of torch"
    print(f"{tag}: subspace of all {len(shapes)} matrices against torch's fp32 range finder, largest projector distance {worst:.2e}", flush=True)


def _first_of_each_shape(shapes):
    seen, out = set(), []
    for i, s in enumerate(shapes):
        if s not in seen:
            seen.add(s)
            out.append(i)
    return out


def _run_model_config(cfg, power_iters, **update):
    import torch
    import bench
    from paper_2602_04396_amd import lordo
    shapes, W, G, Omega, D, grad_dtype = bench.build_workload(torch, lordo, synth, cfg, None, 2)
    kw = dict(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True, power_iters=power_iters)
    hp = lordo.hparams(seed=synth.seed_for(int(cfg[1:]), 77), **kw, **{k: ({"low": 1, "full": 2}[v] if k == "qhm_mode" else v) for k, v in update.items()})
    ohp = orc.Hyper(**kw, **update)
    opt = lordo.Lordo(shapes, hp, W, torch)
    Wp = opt.ptrs(W)
    Gp = [opt.ptrs(g, grad_dtype) for g in G]
    Dp = opt.ptrs(D)
    Op = opt.ptrs(Omega, torch.float32, "qr")
    opt.init_projection(None)                      # Alg. 1: random initial projection, drawn by the library
    opt.poll_status()
    distinct = _first_of_each_shape(shapes)
    picked = distinct + [len(shapes) // 2, len(shapes) - 1]
    sm = Sampled(torch, lordo, opt, shapes, W, picked, ohp, synth.seed_for(int(cfg[1:]), 4242))
    sm.local_step(Wp, Gp[0], G[0], 1e-3, f"{cfg} step 1")
    _whole_state_after_first_step(opt, lordo, shapes, G[0], ohp, cfg)
    ef, full = bool(update.get("error_feedback")), update.get("qhm_mode") == "full"
    plain = not full                   # (the low-rank QHM bracket is inside N: the weight change is lr Q N as well)
    if ef:
        _whole_residual(opt, lordo, shapes, G[0], None, f"{cfg} step 1")
    E_before = [opt.get_state(i, lordo.STATE_ERR) for i in range(len(shapes))] if ef else None
    W_before = [w.clone() for w in W] if plain or full else None
    sm.local_step(Wp, Gp[1], G[1], 2e-3, f"{cfg} step 2")
    if plain:
        _whole_weight_change(opt, lordo, shapes, W_before, W, 2e-3, cfg)
    if full:
        _whole_weight_change_full_qhm(opt, lordo, shapes, W_before, W, G[1], 2e-3, ohp, 2, f"{cfg} step 2")
    if ef:
        _whole_residual(opt, lordo, shapes, G[1], E_before, f"{cfg} step 2")
    del E_before, W_before
    # synchronisation branch of Alg. 1: outer step on the generated averaged pseudo-gradient, new projection from it
    anchors = [opt.get_state(i, lordo.STATE_ANCHOR) for i in range(len(shapes))]
    sm.outer_step(Wp, Dp, D, cfg)
    # every element of every matrix: from a zero momentum b' = mu 0 + D and W = anchor - eta_s (D + mu b') (Nesterov), in fp32
    for i in range(len(shapes)):
        assert torch.equal(opt.get_state(i, lordo.STATE_MOM), D[i]), f"{cfg} matrix {i}: momentum after the first outer step"
        ref = anchors[i]
        ref -= float(ohp.outer_lr * (1.0 + ohp.outer_momentum)) * D[i]
        dev = float((W[i] - ref).abs().max())
        scale = float(D[i].abs().max()) * ohp.outer_lr
        assert dev <= 1e-5 * scale, f"{cfg} matrix {i} {shapes[i]}: outer step off by {dev:.3e} somewhere (largest step {scale:.3e})"
        assert torch.equal(opt.get_state(i, lordo.STATE_ANCHOR), W[i]), f"{cfg} matrix {i}: anchor after the outer step"
        anchors[i] = None
    print(f"{cfg}: whole-array check of the outer step over {len(shapes)} matrices", flush=True)
    del anchors, ref
    old = [(opt.get_state(i, lordo.STATE_Q), opt.get_state(i, lordo.STATE_U), opt.get_state(i, lordo.STATE_V)) for i in range(len(shapes))]
    sm.refresh(Dp, Op, power_iters, f"{cfg} refresh from the averaged pseudo-gradient (fp32)", set(distinct))
    _whole_rotation(opt, lordo, shapes, old, 2, ohp, cfg)
    _whole_subspace(opt, lordo, shapes, D, Omega, power_iters, cfg)
    del old
    worst = 0.0
    for i, (p_, q_, r_) in enumerate(shapes):          # every refreshed basis, not only the sampled matrices
        Qi = opt.get_state(i, lordo.STATE_Q)
        worst = max(worst, float(torch.linalg.norm(Qi.T @ Qi - torch.eye(r_, device=Qi.device))))
    print(f"{cfg}: orthonormality of all {len(shapes)} refreshed bases, largest ||Q^T Q - I||_F {worst:.2e}", flush=True)
    assert worst <= TOL_ORTH
    sm.local_step(Wp, Gp[0], G[0], 1e-3, f"{cfg} step 3 (after the refresh)")
    for i in picked:
        assert torch.isfinite(W[i]).all()
    opt.poll_status()
    opt.close()
    del opt, W, G, D, Omega
    torch.cuda.empty_cache()


def test_c3_full_size_student_t_sampled_columns():
    """168 matrices, r = 256, heavy-tailed (Student-t, nu = 4) bf16 gradients plus a rank-64 spike: two local steps
    (no split-K: the moment update runs in the epilogue of the down-projection), Nesterov outer step, refresh from
    the fp32 averaged pseudo-gradient with one power iteration, one more step."""
    assert synth.CONFIG_DEFAULTS["c3"]["noise"] == "student"
    _run_model_config("c3", synth.CONFIG_DEFAULTS["c3"]["power_iters"])


def test_c3_low_rank_qhm_in_the_fused_epilogue():
    """The same sequence with the low-rank QHM update (Alg. 1, second update case): at this launch shape its bracket
    (omega u_hat + (1 - omega) g) / (sqrt(v_hat) + eps) is formed in the epilogue of the down-projection."""
    _run_model_config("c3", synth.CONFIG_DEFAULTS["c3"]["power_iters"], qhm_mode="low", omega=0.8)


def test_c3_lordo_global_in_the_fused_epilogue():
    """Full-rank QHM with error feedback (Sec. 3.2, Alg. 1: the paper's LoRDO-Global): at this launch shape the column
    sums of the QHM scale and the operand planes of g for the residual update come out of the down-projection's epilogue."""
    _run_model_config("c3", synth.CONFIG_DEFAULTS["c3"]["power_iters"], qhm_mode="full", omega=0.8, error_feedback=True)


def test_c4_full_size_sampled_columns():
    """224 matrices, r = 512 (up to 4096 x 11008 and 11008 x 4096): the same sequence at the largest set."""
    _run_model_config("c4", synth.CONFIG_DEFAULTS["c4"]["power_iters"])


@pytest.mark.parametrize("rank,power_iters", [(64, 1), (64, 2), (1024, 1), (1024, 2)])
def test_c5_largest_matrix_rank_sweep_ends(rank, power_iters):
    """One 8192 x 28672 bf16 matrix at both ends of the rank sweep: refresh from the gradient with one and two power
    iterations against the oracle's range finder on the same start block, then two local steps on sampled columns."""
    import torch
    import bench
    from paper_2602_04396_amd import lordo
    shapes, W, G, Omega, D, grad_dtype = bench.build_workload(torch, lordo, synth, "c5", rank, 2)
    hp = lordo.hparams(power_iters=power_iters)
    ohp = orc.Hyper(power_iters=power_iters)
    opt = lordo.Lordo(shapes, hp, W, torch)
    Wp = opt.ptrs(W)
    Gp = [opt.ptrs(g, grad_dtype) for g in G]
    Op = opt.ptrs(Omega, torch.float32, "qr")
    sm = Sampled(torch, lordo, opt, shapes, W, [0], ohp, synth.seed_for(5, 4242 + rank))
    sm.refresh(Gp[0], Op, power_iters, f"c5 r={rank} q_it={power_iters}", {0})
    sm.local_step(Wp, Gp[1], G[1], 1e-3, f"c5 r={rank} step 1")
    _whole_state_after_first_step(opt, lordo, shapes, G[1], ohp, f"c5 r={rank}")
    W_before = [W[0].clone()]
    sm.local_step(Wp, Gp[0], G[0], 2e-3, f"c5 r={rank} step 2")
    _whole_weight_change(opt, lordo, shapes, W_before, W, 2e-3, f"c5 r={rank}")
    assert torch.isfinite(W[0]).all()
    opt.poll_status()
    opt.close()
    del opt, W, G, D, Omega
    torch.cuda.empty_cache()


def test_c4_lordo_global_with_bf16_storage_sampled_columns():
    """The paper's LoRDO-Global (full-rank QHM + error feedback; Sec. 3.2, Alg. 1) at the c4 launch shape with the
    weights and the residual stored in bf16, as `bench.py` times it among its variants: three local steps on sampled
    columns of one matrix per distinct shape.  Every step starts from the weights and the residual as the library
    stored them; g, the moments and N within 1e-4, every stored weight and residual element a single rounding of the
    float64 update (the criteria of tests/test_gpu_bf16_weights.py)."""
    import torch
    import bench
    from paper_2602_04396_amd import lordo
    from tests.test_gpu_bf16_weights import _check_rounded_once
    shapes, W, G, Omega, D, grad_dtype = bench.build_workload(torch, lordo, synth, "c4", None, 2, torch.bfloat16)
    kw = dict(omega=0.8, error_feedback=True)
    hp = lordo.hparams(seed=synth.seed_for(4, 78), qhm_mode=2, param_dtype=lordo.BF16, err_dtype=lordo.BF16, **kw)
    ohp = orc.Hyper(qhm_mode="full", **kw)
    opt = lordo.Lordo(shapes, hp, W, torch)
    Wp = opt.ptrs(W, torch.bfloat16)
    Gp = [opt.ptrs(g, grad_dtype) for g in G]
    opt.init_projection(None)
    opt.poll_status()
    picked = _first_of_each_shape(shapes)
    rng = np.random.default_rng(synth.seed_for(4, 4343))
    state = {}
    for i in picked:
        p, q, r = shapes[i]
        Q = _f64(opt.get_state(i, lordo.STATE_Q))
        assert np.linalg.norm(Q.T @ Q - np.eye(r)) <= TOL_ORTH
        cols = np.unique(np.concatenate([[0, 1, q - 1, 127, 128, 255, 256, 257, q - 257], rng.integers(0, q, 10)]))
        state[i] = (cols, orc.init_state(_f64(W[i][:, cols]), r, Q))
    for t, lr in enumerate((1e-3, 2e-3, 1e-3)):
        before, E_prev = {}, {}
        for i in picked:
            cols, st = state[i]
            before[i] = _f64(W[i][:, cols])
            E_prev[i] = _f64(opt.get_state(i, lordo.STATE_ERR))[:, cols]
            assert np.array_equal(orc.round_to_bf16(E_prev[i]), E_prev[i]), "the stored residual is not bf16"
            st.E = E_prev[i].copy()
        W_all = [w.clone() for w in W] if t == 1 else None
        opt.local_step(Wp, Gp[t % 2], lr)
        torch.cuda.synchronize()
        if t == 1:
            # every stored weight of every matrix is the fp32 update of the stored value rounded once: within half a bf16
            # unit of the update formed by the library GEMM from the library's own Q, N and v (plus the fp32 slack of that sum)
            c2 = 1.0 - ohp.beta2 ** 2
            worst = 0.0
            for i in range(len(shapes)):
                s_col = ((opt.get_state(i, lordo.STATE_V) / c2).sqrt() + ohp.eps).mean(dim=0)
                upd = opt.get_state(i, lordo.STATE_Q) @ opt.get_state(i, lordo.STATE_NUPD)
                upd *= lr * ohp.omega
                upd += (lr * (1.0 - ohp.omega)) * (G[t % 2][i].float() / s_col[None, :])
                rms = float(upd.square().mean().sqrt())
                full = W_all[i].float() - upd
                ulp = torch.exp2(torch.frexp(full).exponent.float() - 8.0)        # spacing of bf16 at |full|
                over = (W[i].float() - full).abs() - 0.5 * ulp
                worst = max(worst, float(over.max()) / rms)
                assert float(over.max()) <= 1e-3 * rms, f"c4 bf16 storage matrix {i} {shapes[i]}: a stored weight is {float(over.max()):.3e} beyond half a unit (rms of the update {rms:.3e})"
                W_all[i] = None
            print(f"c4 global bf16 storage: every weight of {len(shapes)} matrices within half a bf16 unit of the fp32 update, largest excess / rms of the update {worst:.2e}", flush=True)
            del W_all, upd, full, ulp, over
        for i in picked:
            cols, st = state[i]
            Gc = _f64(G[t % 2][i][:, cols])
            full_W = orc.local_step(st, before[i], Gc, lr, ohp)          # leaves the unrounded residual in st.E
            where = f"c4 global bf16 storage, step {t + 1}, matrix {i} {shapes[i]}"
            get = lambda which: _f64(opt.get_state(i, which))[:, cols]
            assert rel_l2(get(lordo.STATE_GLOW), st.last_g) <= TOL, "g, " + where
            assert rel_l2(get(lordo.STATE_U), st.u) <= TOL and rel_l2(get(lordo.STATE_V), st.v) <= TOL, "moments, " + where
            _check_rounded_once(get(lordo.STATE_ERR), st.E, Gc + E_prev[i], where + " (residual)", max_mismatch=0.1)
            if t > 0:           # (the first update is the sign of g, decided by rounding where g is zero to working precision)
                assert rel_l2(get(lordo.STATE_NUPD), st.last_N) <= TOL, "N, " + where
                _check_rounded_once(_f64(W[i][:, cols]), full_W, full_W - before[i], where + " (weights)", slack_scale=2.0)
    for i in picked:
        assert torch.isfinite(W[i].float()).all()
    opt.poll_status()
    opt.close()
    del opt, W, G, D, Omega
    torch.cuda.empty_cache()
