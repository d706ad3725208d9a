"""Parity of the HIP library (through its C ABI) with the float64 oracle on identical seeded inputs.

Tolerances (from the stated targets): relative L2 <= 1e-4 on g, u, v, N and on the weight change;
|| Q Q^T - Q' Q'^T ||_F <= 1e-3 for the refreshed subspace; || Q^T Q - I ||_F <= 1e-4.
"""
import numpy as np
import pytest

from oracle import lordo_oracle as orc
from paper_2602_04396_amd import synth
from tests.harness import Pair, projector_distance, rel_l2

pytestmark = pytest.mark.gpu

TOL = 1e-4
TOL_SUBSPACE = 1e-3
TOL_ORTH = 1e-4


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available()
    from paper_2602_04396_amd import lordo
    lordo.load()          # fails loudly if the HIP library is not built
    return t


def _spiked(shapes, cfg, n_spike, noise="gauss", bf16=True):
    return [synth.SpikedGradient(p, q, n_spike, synth.seed_for(cfg, i), noise=noise, bf16=bf16)
            for i, (p, q, r) in enumerate(shapes)]


def _weights(shapes, cfg):
    return [synth.weights(np.random.default_rng(synth.seed_for(cfg, 500 + i)), p, q) for i, (p, q, r) in enumerate(shapes)]


def _rand_Q(shapes, cfg):
    return [synth.orthonormal(np.random.default_rng(synth.seed_for(cfg, 700 + i)), p, r) for i, (p, q, r) in enumerate(shapes)]


# several tiles, ragged tails in p, q and r, odd q (unaligned rows), r = p
SMALL_SHAPES = [(200, 330, 48), (96, 70, 20), (300, 129, 33), (64, 64, 64), (130, 257, 128)]


def test_local_steps_bf16_small(torch):
    from paper_2602_04396_amd import lordo
    shapes = SMALL_SHAPES
    pair = Pair(torch, shapes, _weights(shapes, 10), orc.Hyper(), lordo.hparams(grad_dtype=lordo.BF16), _rand_Q(shapes, 10))
    gens = _spiked(shapes, 10, 8)
    for t in range(4):
        G = [g.draw(t) for g in gens]
        pair.local_step(G, lr=1e-3 * (1 + t), first_step_patch=(t == 0))
        worst = pair.compare_local(TOL)
        print(f"step {t + 1}: worst rel L2 {worst}", flush=True)
    assert pair.opt.step == 4


def test_local_steps_bf16_aligned_shapes(torch):
    """Every q a multiple of 8 and every pointer 16-byte aligned: the 16-byte / direct-to-LDS kernels run
    (the odd shapes above take the dword fallbacks); ragged p, q and r, r up to 256 (two rank tiles)."""
    from paper_2602_04396_amd import lordo
    shapes = [(200, 328, 48), (96, 72, 20), (300, 136, 33), (130, 264, 128), (520, 392, 256)]
    pair = Pair(torch, shapes, _weights(shapes, 14), orc.Hyper(), lordo.hparams(grad_dtype=lordo.BF16), _rand_Q(shapes, 14))
    gens = _spiked(shapes, 14, 8)
    for t in range(3):
        pair.local_step([g.draw(t) for g in gens], lr=1e-3, first_step_patch=(t == 0))
        worst = pair.compare_local(TOL)
    print("aligned shapes: worst rel L2", worst, flush=True)


def test_local_steps_large_ranks_several_rank_tiles(torch):
    """Ranks above 256: several 256-rank tiles per column block of the down-projection (the gradient is then read
    through L2 by each of them, with a ragged last tile), several rank chunks in the up-projection; 600 columns are
    two 256-column tiles and a ragged third."""
    from paper_2602_04396_amd import lordo
    shapes = [(400, 264, 320), (640, 600, 544), (96, 72, 20)]
    pair = Pair(torch, shapes, _weights(shapes, 16), orc.Hyper(), lordo.hparams(grad_dtype=lordo.BF16), _rand_Q(shapes, 16))
    gens = _spiked(shapes, 16, 8)
    for t in range(3):
        pair.local_step([g.draw(t) for g in gens], lr=1e-3, first_step_patch=(t == 0))
        worst = pair.compare_local(TOL)
    print("large ranks: worst rel L2", worst, flush=True)


ALIGNED_SHAPES = [(200, 328, 48), (96, 72, 20), (300, 136, 33), (130, 264, 128), (520, 392, 256)]


@pytest.mark.parametrize("variant", ["low_qhm", "full_qhm", "error_feedback", "lordo_global", "ef_fp32_grads"])
def test_local_steps_qhm_and_error_feedback(torch, variant):
    """The other two update cases of Alg. 1 and its error-feedback lines, and their combination
    (full-rank QHM with error feedback is the configuration the paper calls LoRDO-Global)."""
    from paper_2602_04396_amd import lordo
    kw = {"low_qhm": dict(qhm_mode="low", omega=0.7), "full_qhm": dict(qhm_mode="full", omega=0.9),
          "error_feedback": dict(error_feedback=True), "lordo_global": dict(qhm_mode="full", omega=0.95, error_feedback=True),
          "ef_fp32_grads": dict(error_feedback=True, qhm_mode="low", omega=0.5)}[variant]
    mode = {"none": 0, "low": 1, "full": 2}[kw.get("qhm_mode", "none")]
    bf16 = variant != "ef_fp32_grads"
    shapes = ALIGNED_SHAPES
    pair = Pair(torch, shapes, _weights(shapes, 15), orc.Hyper(**kw),
                lordo.hparams(qhm_mode=mode, omega=kw.get("omega", 1.0), error_feedback=kw.get("error_feedback", False),
                              grad_dtype=lordo.BF16 if bf16 else lordo.F32), _rand_Q(shapes, 15))
    gens = _spiked(shapes, 15, 8, bf16=bf16)
    for t in range(4):
        pair.local_step([g.draw(t) for g in gens], lr=1e-3 * (1 + t), grad_scale=0.8 if t == 2 else 1.0, bf16=bf16,
                        first_step_patch=(t == 0))
        worst = pair.compare_local(TOL)
    print(f"{variant}: worst rel L2 {worst}", flush=True)
    if kw.get("error_feedback"):
        # the residual is orthogonal to the subspace (Alg. 1: E = A - Q Q^T A)
        for i, (p, q, r) in enumerate(shapes):
            E = pair.get(i, lordo.STATE_ERR)
            Q = pair.get(i, lordo.STATE_Q)
            assert np.linalg.norm(Q.T @ E) <= 1e-4 * np.linalg.norm(E)


def test_qhm_full_rejects_unaligned(torch):
    from paper_2602_04396_amd import lordo
    import torch as t
    shapes = [(64, 70, 16)]                                   # q % 4 != 0
    W = [t.zeros(64, 70, device="cuda")]
    G = [t.zeros(64, 70, device="cuda", dtype=t.bfloat16)]
    opt = lordo.Lordo(shapes, lordo.hparams(qhm_mode=2, omega=0.9), W, t)
    with pytest.raises(lordo.LordoError) as e:
        opt.local_step(W, G, 1e-3)
    assert e.value.code == lordo.EINVAL


def test_local_steps_degenerate_shapes(torch):
    """Smallest and most lopsided matrices: a single element, a single column, r = p, r > q, one row block."""
    from paper_2602_04396_amd import lordo
    shapes = [(1, 1, 1), (2, 8, 2), (33, 1, 5), (5, 12, 5), (40, 4, 40), (31, 257, 31)]
    for bf16 in (True, False):
        pair = Pair(torch, shapes, _weights(shapes, 16), orc.Hyper(),
                    lordo.hparams(grad_dtype=lordo.BF16 if bf16 else lordo.F32), _rand_Q(shapes, 16))
        rng = np.random.default_rng(synth.seed_for(16, 1 if bf16 else 2))
        for t in range(3):
            G = [(1e-3 * rng.standard_normal((p, q))).astype(np.float32) for p, q, r in shapes]
            if bf16:
                G = [synth.bf16_round(g) for g in G]
            pair.local_step(G, lr=1e-3, bf16=bf16, first_step_patch=(t == 0))
        pair.compare_local(TOL)


def test_empty_and_invalid_sets(torch):
    from paper_2602_04396_amd import lordo
    with pytest.raises(lordo.LordoError) as e:
        lordo.workspace_bytes([], lordo.hparams())
    assert e.value.code == lordo.EINVAL


def test_local_steps_ranks_from_256_up_ragged_edges(torch):
    """Every rank >= 256: the plain update runs on 256 x 128 tiles.  Rows that are no multiple of 256 (or of 32),
    columns that are no multiple of 128, a rank that is no multiple of 32, one matrix smaller than a tile."""
    from paper_2602_04396_amd import lordo
    shapes = [(520, 392, 256), (300, 260, 257), (257, 132, 256), (1100, 644, 320), (256, 128, 256)]
    pair = Pair(torch, shapes, _weights(shapes, 16), orc.Hyper(), lordo.hparams(), _rand_Q(shapes, 16))
    gens = _spiked(shapes, 16, 8)
    for t in range(3):
        pair.local_step([g.draw(t) for g in gens], lr=1e-3 * (1 + t), first_step_patch=(t == 0))
        worst = pair.compare_local(TOL)
    print("ranks >= 256:", worst, flush=True)


@pytest.mark.parametrize("shape_set", ["ragged", "one_slice"])
@pytest.mark.parametrize("variant", ["full_qhm", "ef", "global", "global_fp32_grads"])
def test_local_steps_ranks_from_256_up_gradient_term(torch, variant, shape_set):
    """Every rank >= 256 with the epilogues that read a gradient tile on the 256 x 128 tiles: the full-rank QHM update
    (Sec. 3.2), the residual of the error feedback (Alg. 1), both (LoRDO-Global); with fp32 gradients the 128 x 128
    kernel takes these launches.  Columns are multiples of 4 (the four-column accesses of these epilogues), otherwise
    ragged: rows no multiple of 256 or 32, a rank that is no multiple of 32."""
    from paper_2602_04396_amd import lordo
    shapes = [(520, 392, 256), (300, 260, 257), (257, 132, 256), (1100, 644, 320), (256, 128, 256)]
    if shape_set == "one_slice":      # no matrix taller than 256 rows: no split-K, so the moment update -- with the column sums of the
        shapes = [(256, 520, 256), (256, 388, 250), (250, 132, 250)]      # full-rank QHM scale and the operand planes of g -- runs
                                                                          # in the epilogue of the down-projection
    bf16 = variant != "global_fp32_grads"
    qhm = "none" if variant == "ef" else "full"
    ef = variant != "full_qhm"
    kw = dict(omega=0.8 if qhm == "full" else 1.0, error_feedback=ef)
    pair = Pair(torch, shapes, _weights(shapes, 18), orc.Hyper(qhm_mode=qhm, **kw),
                lordo.hparams(qhm_mode=2 if qhm == "full" else 0, grad_dtype=lordo.BF16 if bf16 else lordo.F32, **kw), _rand_Q(shapes, 18))
    gens = _spiked(shapes, 18, 8, bf16=bf16)
    for t in range(3):
        pair.local_step([g.draw(t) for g in gens], lr=1e-3 * (1 + t), grad_scale=0.9, bf16=bf16, first_step_patch=(t == 0))
        worst = pair.compare_local(TOL)
    print(f"ranks >= 256, {variant}, {shape_set}:", worst, flush=True)


def test_local_steps_identity_init_and_grad_scale(torch):
    """Q_0 = first r columns of I (the library's own initial state), grad_scale != 1."""
    from paper_2602_04396_amd import lordo
    shapes = [(160, 96, 32), (70, 50, 7)]
    pair = Pair(torch, shapes, _weights(shapes, 11), orc.Hyper(), lordo.hparams())
    gens = _spiked(shapes, 11, 4)
    for t in range(3):
        pair.local_step([g.draw(t) for g in gens], lr=2e-3, grad_scale=0.37, first_step_patch=(t == 0))
    pair.compare_local(TOL)


def test_local_steps_no_bias_correction_fp32_grads(torch):
    from paper_2602_04396_amd import lordo
    shapes = [(150, 200, 24), (33, 65, 33)]
    pair = Pair(torch, shapes, _weights(shapes, 12), orc.Hyper(bias_correction=False, beta1=0.8, beta2=0.95, eps=1e-6),
                lordo.hparams(beta1=0.8, beta2=0.95, eps=1e-6, bias_correction=False, grad_dtype=lordo.F32),
                _rand_Q(shapes, 12))
    gens = _spiked(shapes, 12, 4, bf16=False)
    for t in range(3):
        pair.local_step([g.draw(t) for g in gens], lr=1e-2, bf16=False, first_step_patch=(t == 0))
    pair.compare_local(TOL)


def test_full_rank_identity_is_adam(torch):
    """r = p with Q = I: the library's local step must be the full-rank Adam step (Sec. 2);
    compared with torch.optim.Adam in float64 on the CPU, not with the oracle."""
    import torch as t
    from paper_2602_04396_amd import lordo
    p, q = 64, 96
    W0 = _weights([(p, q, p)], 13)
    Wg = [t.tensor(W0[0], device="cuda")]
    opt_g = lordo.Lordo([(p, q, p)], lordo.hparams(), Wg, t)
    Wt = t.tensor(W0[0], dtype=t.float64, requires_grad=True)
    opt = t.optim.Adam([Wt], lr=1e-3, betas=(0.9, 0.999), eps=1e-8)
    gen = _spiked([(p, q, p)], 13, 4)[0]
    for step in range(3):
        G = gen.draw(step)
        opt_g.local_step(Wg, [t.tensor(G, device="cuda").to(t.bfloat16)], 1e-3)
        Wt.grad = t.tensor(G, dtype=t.float64)
        opt.step()
        got = Wg[0].cpu().numpy().astype(np.float64) - W0[0]
        assert rel_l2(got, Wt.detach().numpy() - W0[0]) <= TOL
    assert rel_l2(opt_g.get_state(0, lordo.STATE_V).cpu().numpy(), opt.state[Wt]["exp_avg_sq"].numpy()) <= TOL


def test_config1_chain(torch):
    """Config 1: 256 x 256 fp32, r = 16, Q from the range finder on G_0 (2 power iterations),
    10 local steps with fresh noise, one Nesterov outer step on the worker's own pseudo-gradient."""
    from paper_2602_04396_amd import lordo
    rng = np.random.default_rng(synth.seed_for(1, 0))
    S = synth.c1_signal(rng)
    G0 = synth.c1_gradient(S, rng)
    Om = synth.omega(rng, 256, 16)
    W0 = [synth.weights(np.random.default_rng(synth.seed_for(1, 99)), 256, 256)]
    ohp = orc.Hyper(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True, power_iters=2)
    ghp = lordo.hparams(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True, power_iters=2, grad_dtype=lordo.F32)
    pair = Pair(torch, [(256, 256, 16)], W0, ohp, ghp)
    dists, orths = pair.refresh([G0], [Om], bf16=False)
    print("config1 refresh: projector distance", dists, "orthonormality", orths, flush=True)
    assert max(dists) <= TOL_SUBSPACE and max(orths) <= TOL_ORTH
    # the signal subspace found must be the SVD's (paper's default projection), cf. the oracle pin
    U8 = np.linalg.svd(G0.astype(np.float64), full_matrices=False)[0][:, :8]
    Qg = pair.get(0, lordo.STATE_Q)
    assert np.linalg.norm(U8 - Qg @ (Qg.T @ U8)) < 1e-2
    for t in range(10):
        G = synth.c1_gradient(S, np.random.default_rng(synth.seed_for(1, 0, t)))
        pair.local_step([G], lr=1e-3, bf16=False, first_step_patch=(t == 0))
    worst = pair.compare_local(TOL)
    print("config1 after 10 steps:", worst, flush=True)
    # own pseudo-gradient, then Nesterov outer step on it
    out = [torch.empty_like(pair.W_gpu[0])]
    pair.opt.export_pseudograd(pair.W_gpu, out)
    D_orc = orc.pseudo_gradient(pair.st[0], pair.W_orc[0])
    assert rel_l2(out[0].cpu().numpy(), D_orc) <= TOL
    pair.opt.outer_step(pair.W_gpu, None)
    W_new = orc.outer_step(pair.st[0], D_orc, ohp)
    assert rel_l2(pair.W_gpu[0].cpu().numpy().astype(np.float64) - W0[0], W_new - W0[0]) <= TOL
    assert torch.equal(pair.opt.get_state(0, lordo.STATE_ANCHOR), pair.W_gpu[0])      # anchor <- new model
    assert rel_l2(pair.get(0, lordo.STATE_MOM), pair.st[0].b) <= TOL


def test_config1_constant_gradient_closed_form(torch):
    """Constant gradient: N = sign-like g/(|g|+eps) at every step, so after 10 steps at eta = 1e-3
    W_10 = W_0 - 1e-2 Q N.  Elements whose g is zero to working precision are taken from the library."""
    from paper_2602_04396_amd import lordo
    rng = np.random.default_rng(synth.seed_for(1, 0))
    S = synth.c1_signal(rng)
    G0 = synth.c1_gradient(S, rng)
    Om = synth.omega(rng, 256, 16)
    W0 = [synth.weights(np.random.default_rng(synth.seed_for(1, 99)), 256, 256)]
    pair = Pair(torch, [(256, 256, 16)], W0, orc.Hyper(power_iters=2), lordo.hparams(power_iters=2, grad_dtype=lordo.F32))
    pair.refresh([G0], [Om], bf16=False)
    for t in range(10):
        pair.local_step([G0], lr=1e-3, bf16=False, first_step_patch=True)
    pair.compare_local(TOL)
    Q = pair.st[0].Q
    N = pair.st[0].last_N
    got = pair.W_gpu[0].cpu().numpy().astype(np.float64) - W0[0]
    assert rel_l2(got, -1e-2 * Q @ N) <= TOL


@pytest.mark.parametrize("shape_set", ["ragged", "aligned"])
def test_refresh_rotates_moments(torch, shape_set):
    """Refresh after some steps: subspace against the oracle's own range finder, then moments
    against the oracle's rotation done with the library's basis (the rotation depends on the basis,
    which is only fixed up to rounding-level differences), plus a basis-free check.  The aligned
    shapes (q % 32 == 0, r % 4 == 0) with a bf16 source take the range-finder products through the
    projection-type kernels, the ragged ones through the grouped GEMM."""
    from paper_2602_04396_amd import lordo
    shapes = [(200, 330, 48), (300, 129, 33), (96, 160, 20), (256, 192, 128)] if shape_set == "ragged" else \
             [(200, 320, 48), (300, 128, 32), (130, 160, 20), (256, 192, 128), (520, 384, 256)]
    # (power iterations, bf16 gradients, bf16 refresh source): the last case is an fp32 source (an averaged
    # pseudo-gradient, Alg. 1) in a context planned for bf16 gradients
    for power_iters, bf16, src_bf16 in [(1, True, True), (2, False, False), (0, True, True), (2, True, True), (1, True, False)]:
        ohp = orc.Hyper(power_iters=power_iters)
        ghp = lordo.hparams(power_iters=power_iters, grad_dtype=lordo.BF16 if bf16 else lordo.F32)
        pair = Pair(torch, shapes, _weights(shapes, 20), ohp, ghp, _rand_Q(shapes, 20))
        gens = _spiked(shapes, 20, 8, bf16=bf16)
        for t in range(3):
            pair.local_step([g.draw(t) for g in gens], lr=1e-3, bf16=bf16, first_step_patch=(t == 0))
        Src = [g.draw(100) for g in gens]
        if bf16 and not src_bf16:          # something fp32 that is not bf16-representable
            Src = [(0.75 * a + 0.25 * g.draw(101)).astype(np.float32) for a, g in zip(Src, gens)]
        Om = [synth.omega(np.random.default_rng(synth.seed_for(20, 900 + i)), q, r) for i, (p, q, r) in enumerate(shapes)]
        Qu_before = [pair.st[i].Q @ pair.st[i].u for i in range(len(shapes))]
        Q_old = [pair.st[i].Q.copy() for i in range(len(shapes))]
        with pytest.raises(lordo.LordoError):                 # no refresh yet: nothing to report
            pair.opt.mssv()
        dists, orths = pair.refresh(Src, Om, bf16=src_bf16)
        # similarity diagnostic (Sec. 5.1): basis-free, so the oracle's own new basis serves
        mssv_gpu = pair.opt.mssv().cpu().numpy()
        for i, (p, q, r) in enumerate(shapes):
            Qo = orc.range_finder(np.asarray(Src[i], dtype=np.float64), np.asarray(Om[i], dtype=np.float64), power_iters)
            assert abs(mssv_gpu[i] - orc.mssv(Qo, Q_old[i])) <= 1e-4, f"MSSV of matrix {i}"
        print(f"refresh {shape_set} q_it={power_iters} bf16 grads={bf16} source={src_bf16}: dist {np.round(dists, 6)} orth {np.round(orths, 7)}", flush=True)
        assert max(dists) <= TOL_SUBSPACE and max(orths) <= TOL_ORTH
        for i in range(len(shapes)):
            u_g = pair.get(i, lordo.STATE_U)
            v_g = pair.get(i, lordo.STATE_V)
            assert rel_l2(u_g, pair.st[i].u) <= TOL, f"u of matrix {i}"
            assert rel_l2(v_g, pair.st[i].v) <= TOL, f"v of matrix {i}"
            # basis-free: Q_new u_new = P_new (Q_old u_old)
            Qg = pair.get(i, lordo.STATE_Q)
            assert rel_l2(Qg @ u_g, Qg @ (Qg.T @ Qu_before[i])) <= TOL
        for t in range(3, 5):
            pair.local_step([g.draw(t) for g in gens], lr=1e-3, bf16=bf16)
        pair.compare_local(TOL)


@pytest.mark.parametrize("bf16", [True, False])
def test_local_variant_refresh_from_gradient_plus_residual(torch, bf16):
    """Call order of the local variant (Alg. 2): identity Q_0, a step, then a refresh computed from
    this step's gradient plus the error buffer followed by the step on the same gradient, more
    steps, and a second refresh; low-rank QHM as the paper pairs it with this variant."""
    from paper_2602_04396_amd import lordo
    shapes = [(200, 328, 48), (96, 72, 20), (300, 136, 33), (256, 192, 128)]
    ohp = orc.Hyper(error_feedback=True, qhm_mode="low", omega=0.9, power_iters=1)
    ghp = lordo.hparams(error_feedback=True, qhm_mode=1, omega=0.9, power_iters=1, grad_dtype=lordo.BF16 if bf16 else lordo.F32)
    pair = Pair(torch, shapes, _weights(shapes, 24), ohp, ghp)          # Q_0 = identity columns
    gens = _spiked(shapes, 24, 8, bf16=bf16)
    Om = [synth.omega(np.random.default_rng(synth.seed_for(24, 900 + i)), q, r) for i, (p, q, r) in enumerate(shapes)]
    t = 0
    pair.local_step([g.draw(t) for g in gens], lr=1e-3, bf16=bf16, first_step_patch=True)
    pair.compare_local(TOL)
    for window in range(2):
        t += 1
        G = [g.draw(t) for g in gens]
        scale = 0.7 if window == 1 else 1.0
        dists, orths = pair.refresh_local(G, Om, grad_scale=scale, bf16=bf16)
        print(f"local-variant refresh {window} bf16={bf16}: dist {np.round(dists, 6)} orth {np.round(orths, 7)}", flush=True)
        assert max(dists) <= TOL_SUBSPACE and max(orths) <= TOL_ORTH
        # the buffer holds G + E until the step that consumes it
        with pytest.raises(lordo.LordoError) as e:
            pair.opt.get_state(0, lordo.STATE_ERR)
        assert e.value.code == lordo.ESTATE
        with pytest.raises(lordo.LordoError) as e:
            pair.opt.refresh_subspace(pair._held_G, pair.to_dev(Om, False))
        assert e.value.code == lordo.ESTATE
        with pytest.raises(lordo.LordoError) as e:                     # other gradient tensors than the folded ones
            pair.opt.local_step(pair.W_gpu, pair.to_dev(G, bf16), 1e-3)
        assert e.value.code == lordo.ESTATE
        pair.local_step(G, lr=1e-3, grad_scale=scale, bf16=bf16)
        pair.compare_local(TOL)
        for _ in range(2):
            t += 1
            pair.local_step([g.draw(t) for g in gens], lr=1e-3, bf16=bf16)
        pair.compare_local(TOL)
    for i, (p, q, r) in enumerate(shapes):
        E = pair.get(i, lordo.STATE_ERR)
        Q = pair.get(i, lordo.STATE_Q)
        assert np.linalg.norm(Q.T @ E) <= 1e-4 * np.linalg.norm(E)
    # without error feedback there is no buffer to refresh from
    plain = Pair(torch, shapes[:1], _weights(shapes[:1], 24), orc.Hyper(), lordo.hparams())
    with pytest.raises(lordo.LordoError) as e:
        plain.opt.refresh_subspace_local(plain.to_dev([gens[0].draw(0)], True), plain.to_dev(Om[:1], False))
    assert e.value.code == lordo.ESTATE


@pytest.mark.parametrize("src_bf16,ranks", [(True, "to_128"), (False, "to_128"), (True, "to_256"), (True, "to_512"), (True, "to_1024")],
                         ids=["bf16_source", "fp32_source", "ranks_to_256", "ranks_to_512", "ranks_to_1024"])
def test_refresh_with_rayleigh_ritz_orders_the_basis(torch, src_bf16, ranks):
    """Refresh that ends with the Rayleigh-Ritz step (Sec. 2: Q = the first r columns of U, largest singular
    value first).  Unique quantities are compared with the oracle: the subspace (projector), the Ritz values,
    and -- where a singular value is separated from its neighbours -- the column itself up to its sign.  For
    all columns: Q^T Src Src^T Q must be diagonal with descending entries.  Then moments and steps as usual."""
    from paper_2602_04396_amd import lordo
    # ranks up to 128: the solver of the Rayleigh-Ritz step runs in LDS in one launch; above: the blocked form, whose
    # three instantiations cover ranks up to 256, 512 and 1024
    shapes = {"to_128": [(200, 328, 48), (96, 72, 20), (300, 136, 33), (256, 192, 128), (130, 257, 7), (384, 640, 127)],
              "to_256": [(520, 392, 256), (300, 400, 129), (640, 512, 200), (96, 72, 20)],
              "to_512": [(700, 616, 300), (96, 72, 20), (900, 520, 257)],
              "to_1024": [(1200, 808, 600), (300, 136, 33)]}[ranks]
    ohp = orc.Hyper(power_iters=2, rayleigh_ritz=True)
    ghp = lordo.hparams(power_iters=2, rayleigh_ritz=True)
    pair = Pair(torch, shapes, _weights(shapes, 37), ohp, ghp, _rand_Q(shapes, 37))
    gens = _spiked(shapes, 37, 6)
    for t in range(2):
        pair.local_step([g.draw(t) for g in gens], lr=1e-3, first_step_patch=(t == 0))
    with pytest.raises(lordo.LordoError) as e:                  # no refresh yet
        pair.opt.get_state(0, lordo.STATE_RITZ)
    assert e.value.code == lordo.ESTATE
    Src = [g.draw(100) for g in gens]
    if not src_bf16:
        Src = [(0.75 * a + 0.25 * g.draw(101)).astype(np.float32) for a, g in zip(Src, gens)]
    Om = [synth.omega(np.random.default_rng(synth.seed_for(37, 900 + i)), q, r) for i, (p, q, r) in enumerate(shapes)]
    dists, orths = pair.refresh(Src, Om, bf16=src_bf16)
    print(f"rayleigh-ritz refresh: dist {np.round(dists, 6)} orth {np.round(orths, 7)}", flush=True)
    assert max(dists) <= TOL_SUBSPACE and max(orths) <= TOL_ORTH
    sr_gpu = pair.opt.stable_rank().cpu().numpy().astype(np.float64)
    for i, (p, q, r) in enumerate(shapes):
        A = np.asarray(Src[i], dtype=np.float64)
        Qg = pair.get(i, lordo.STATE_Q)
        ritz = pair.opt.get_state(i, lordo.STATE_RITZ).cpu().numpy().astype(np.float64)
        Qo, S = orc.rayleigh_ritz(orc.range_finder(A, np.asarray(Om[i], dtype=np.float64), ohp.power_iters), A)
        assert np.all(np.diff(ritz) <= 0)
        assert np.max(np.abs(ritz - S) / S) <= TOL, f"Ritz values of matrix {i}"
        D = Qg.T @ A @ A.T @ Qg
        d = np.diag(D)
        assert np.linalg.norm(D - np.diag(d)) <= 1e-5 * np.linalg.norm(D), f"matrix {i}: restricted matrix not diagonal"
        assert np.all(np.diff(d) <= 1e-5 * d[0]), f"matrix {i}: columns not in descending order"
        assert np.max(np.abs(np.sqrt(d) - ritz) / ritz) <= TOL
        # stable rank of the source (Sec. 5.1) against the definition: the leading Ritz value stands for the
        # spectral norm, which the spiked recipe separates well
        assert abs(sr_gpu[i] - orc.stable_rank(A)) <= TOL * orc.stable_rank(A), f"stable rank of matrix {i}"
        # columns whose singular value is separated by 5 % from both neighbours are fixed up to sign; the two
        # bases differ by the subspace error divided by the gap at most (a few times, to be safe)
        nb = np.concatenate([[np.inf], S, [0.0]])
        gap = np.minimum(nb[:-2] - S, S - nb[2:]) / S
        sep = np.where(gap >= 0.05)[0]
        assert len(sep) >= 3, f"matrix {i}: the input recipe should leave separated spikes"
        for k in sep:
            resid = Qg[:, k] - (Qg[:, k] @ Qo[:, k]) * Qo[:, k]       # part of the library's column outside the oracle's
            sin = float(np.linalg.norm(resid) / np.linalg.norm(Qg[:, k]))
            assert sin <= 4.0 * (dists[i] + 1e-5) / gap[k], f"matrix {i} column {k}: sin {sin:.2e}, gap {gap[k]:.3f}"
    for i in range(len(shapes)):
        assert rel_l2(pair.get(i, lordo.STATE_U), pair.st[i].u) <= TOL
        assert rel_l2(pair.get(i, lordo.STATE_V), pair.st[i].v) <= TOL
    # r-th spectral gap (Sec. 5.1): sigma_r from the Ritz values, sigma_{r+1} from the deflated block iteration;
    # the oracle runs the same iteration with the library's basis, and the definition bounds the estimate
    Om2 = [synth.omega(np.random.default_rng(synth.seed_for(37, 950 + i)), q, r) for i, (p, q, r) in enumerate(shapes)]
    Q_before = [pair.opt.get_state(i, lordo.STATE_Q) for i in range(len(shapes))]
    gap = pair.opt.spectral_gap(pair.to_dev(Src, src_bf16), pair.to_dev(Om2, False)).cpu().numpy().astype(np.float64)
    pair.opt.poll_status()
    for i, (p, q, r) in enumerate(shapes):
        A = np.asarray(Src[i], dtype=np.float64)
        Qg = pair.get(i, lordo.STATE_Q)
        assert torch.equal(pair.opt.get_state(i, lordo.STATE_Q), Q_before[i])          # the basis is left alone
        ritz = pair.opt.get_state(i, lordo.STATE_RITZ).cpu().numpy().astype(np.float64)
        est_gpu = ritz[-1] - gap[i]
        est_orc = orc.next_singular_value_estimate(A, Qg, np.asarray(Om2[i], dtype=np.float64), 2)
        sigma = np.linalg.svd(A, compute_uv=False)
        deflated = np.linalg.svd(A - Qg @ (Qg.T @ A), compute_uv=False)[0]
        if 2 * r > min(p, q):
            # fewer than r directions are left after the deflation: the block is completed arbitrarily (differently
            # on the two sides) and the estimate is a bound only
            assert est_gpu <= deflated * (1 + TOL) and est_orc <= deflated * (1 + 1e-9)
            continue
        assert abs(est_gpu - est_orc) <= TOL * est_orc, f"sigma_(r+1) estimate of matrix {i}: {est_gpu} vs {est_orc}"
        # what the estimate approaches is the norm of the deflated source, which is sigma_(r+1) for the exact leading
        # subspace and above it for the range finder's (whose trailing directions lie in the noise bulk here)
        assert sigma[r] * (1 - 1e-6) <= deflated and 0.85 * deflated <= est_gpu <= deflated * (1 + TOL), \
            f"matrix {i}: estimate {est_gpu}, deflated norm {deflated}, sigma_(r+1) {sigma[r]}"
        assert abs(gap[i] - (ritz[-1] - est_orc)) <= TOL * ritz[-1]
    for t in range(2, 4):
        pair.local_step([g.draw(t) for g in gens], lr=1e-3)
    pair.compare_local(TOL)
    with pytest.raises(lordo.LordoError) as e:                  # the solver takes ranks up to 1024
        lordo.workspace_bytes([(2048, 1100, 1025)], ghp)
    assert e.value.code == lordo.EINVAL


def test_local_variant_with_rayleigh_ritz(torch):
    """Alg. 2 refresh (source = this step's gradient plus the error buffer, fp32 in the arena) ending with the
    Rayleigh-Ritz step: the new basis diagonalises the restricted source, in descending order, and its Ritz values
    and stable rank are those of G + E; the step on the same gradient follows."""
    from paper_2602_04396_amd import lordo
    shapes = [(200, 328, 48), (96, 72, 20), (300, 136, 33), (256, 192, 128)]
    ohp = orc.Hyper(error_feedback=True, qhm_mode="low", omega=0.9, power_iters=1, rayleigh_ritz=True)
    ghp = lordo.hparams(error_feedback=True, qhm_mode=1, omega=0.9, power_iters=1, rayleigh_ritz=True)
    pair = Pair(torch, shapes, _weights(shapes, 38), ohp, ghp)
    gens = _spiked(shapes, 38, 8)
    Om = [synth.omega(np.random.default_rng(synth.seed_for(38, 900 + i)), q, r) for i, (p, q, r) in enumerate(shapes)]
    pair.local_step([g.draw(0) for g in gens], lr=1e-3, first_step_patch=True)
    G = [g.draw(1) for g in gens]
    sources = [orc.local_variant_source(pair.st[i], np.asarray(G[i], dtype=np.float64), 0.8) for i in range(len(shapes))]
    dists, orths = pair.refresh_local(G, Om, grad_scale=0.8)
    assert max(dists) <= TOL_SUBSPACE and max(orths) <= TOL_ORTH
    sr = pair.opt.stable_rank().cpu().numpy().astype(np.float64)
    for i, (p, q, r) in enumerate(shapes):
        A = sources[i]
        Qg = pair.get(i, lordo.STATE_Q)
        ritz = pair.opt.get_state(i, lordo.STATE_RITZ).cpu().numpy().astype(np.float64)
        _, S = orc.rayleigh_ritz(orc.range_finder(A, np.asarray(Om[i], dtype=np.float64), 1), A)
        assert np.max(np.abs(ritz - S) / S) <= TOL, f"Ritz values of matrix {i}"
        D = Qg.T @ A @ A.T @ Qg
        d = np.diag(D)
        assert np.linalg.norm(D - np.diag(d)) <= 1e-5 * np.linalg.norm(D) and np.all(np.diff(d) <= 1e-5 * d[0])
        assert abs(sr[i] - np.sum(A * A) / S[0] ** 2) <= TOL * sr[i]
    pair.local_step(G, lr=1e-3, grad_scale=0.8)
    pair.compare_local(TOL)


def test_refresh_before_first_step_and_exact_reconstruction(torch):
    """rank(Src) = r exactly: the refreshed Q must reproduce Src (Q Q^T Src = Src); t = 0: no rotation."""
    from paper_2602_04396_amd import lordo
    p, q, r = 192, 160, 24
    rng = np.random.default_rng(synth.seed_for(21, 0))
    Src = (rng.standard_normal((p, r)) @ rng.standard_normal((r, q))).astype(np.float32)
    Om = synth.omega(rng, q, r)
    pair = Pair(torch, [(p, q, r)], _weights([(p, q, r)], 21), orc.Hyper(power_iters=1), lordo.hparams(power_iters=1))
    dists, orths = pair.refresh([Src], [Om], bf16=False)
    assert max(dists) <= TOL_SUBSPACE and max(orths) <= TOL_ORTH
    Qg = pair.get(0, lordo.STATE_Q)
    S64 = Src.astype(np.float64)
    assert rel_l2(Qg @ (Qg.T @ S64), S64) <= TOL
    assert not pair.get(0, lordo.STATE_U).any() and not pair.get(0, lordo.STATE_V).any()


@pytest.mark.parametrize("rayleigh_ritz", [False, True], ids=["plain", "rayleigh_ritz"])
def test_refresh_rank_deficient_source_three_passes(torch, rayleigh_ritz):
    """rank(Src) < r: the completion of the basis is arbitrary; only Q^T Q = I and Q Q^T Src = Src
    are fixed.  Three CholeskyQR passes are requested for this degenerate case.  With the Rayleigh-Ritz step the
    leading Ritz values are the five singular values of the source and the others vanish."""
    from paper_2602_04396_amd import lordo
    p, q, r = 128, 96, 16
    rng = np.random.default_rng(synth.seed_for(22, 0))
    Src = (rng.standard_normal((p, 5)) @ rng.standard_normal((5, q))).astype(np.float32)
    Om = synth.omega(rng, q, r)
    W = [torch.zeros(p, q, device="cuda")]
    opt = lordo.Lordo([(p, q, r)], lordo.hparams(power_iters=1, orth_passes=3, rayleigh_ritz=rayleigh_ritz), W, torch)
    G0 = torch.tensor(rng.standard_normal((p, q)).astype(np.float32), device="cuda").bfloat16()
    opt.local_step(W, [G0], 1e-3)          # moments that a rotation would change
    before = [opt.get_state(0, which) for which in (lordo.STATE_Q, lordo.STATE_U, lordo.STATE_V)]
    opt.refresh_subspace([torch.tensor(Src, device="cuda")], [torch.tensor(Om, device="cuda")])
    try:
        opt.poll_status()
    except lordo.LordoError as e:          # a latched breakdown is an allowed outcome here
        assert e.code == lordo.ENUMERIC
        # the refresh that broke down left the projection and the moments alone, and the next step works
        for x, which in zip(before, (lordo.STATE_Q, lordo.STATE_U, lordo.STATE_V)):
            assert torch.equal(opt.get_state(0, which), x)
        opt.local_step(W, [G0], 1e-3)
        opt.poll_status()
        assert torch.isfinite(W[0]).all()
        return
    Qg = opt.get_state(0, lordo.STATE_Q).cpu().numpy().astype(np.float64)
    S64 = Src.astype(np.float64)
    assert np.isfinite(Qg).all()
    assert rel_l2(Qg @ (Qg.T @ S64), S64) <= 1e-3
    if rayleigh_ritz:
        ritz = opt.get_state(0, lordo.STATE_RITZ).cpu().numpy().astype(np.float64)
        sigma = np.linalg.svd(S64, compute_uv=False)
        assert np.max(np.abs(ritz[:5] - sigma[:5]) / sigma[:5]) <= 1e-4
        assert np.all(ritz[5:] <= 2e-3 * sigma[0])          # zero up to the rounding of the squared values
        assert np.linalg.norm(Qg.T @ Qg - np.eye(r)) <= 1e-3


def test_rayleigh_ritz_nearly_rank_deficient_source(torch):
    """A source of rank five plus noise four orders of magnitude below it: the factor of the Ritz matrix has a
    condition number of 1e4 and most of its singular values are tiny; the five leading Ritz values must be the five
    singular values of the source to 1e-4, the others must be of the size of the noise, and the basis orthonormal."""
    from paper_2602_04396_amd import lordo
    p, q, r = 256, 192, 24
    rng = np.random.default_rng(synth.seed_for(23, 0))
    Src = (rng.standard_normal((p, 5)) @ rng.standard_normal((5, q)) + 1e-3 * rng.standard_normal((p, q))).astype(np.float32)
    Om = synth.omega(rng, q, r)
    W = [torch.zeros(p, q, device="cuda")]
    # the robust variant of the orthonormalisation (orth_passes = 3): with the default the conditioning of this source,
    # 1e4, compounds over the products of the power iteration and the last, unshifted pass breaks down
    opt = lordo.Lordo([(p, q, r)], lordo.hparams(power_iters=2, rayleigh_ritz=True, orth_passes=3), W, torch)
    opt.refresh_subspace([torch.tensor(Src, device="cuda")], [torch.tensor(Om, device="cuda")])
    opt.poll_status()
    Qg = opt.get_state(0, lordo.STATE_Q).cpu().numpy().astype(np.float64)
    ritz = opt.get_state(0, lordo.STATE_RITZ).cpu().numpy().astype(np.float64)
    S64 = Src.astype(np.float64)
    sigma = np.linalg.svd(S64, compute_uv=False)
    _, S = orc.rayleigh_ritz(orc.range_finder(S64, Om.astype(np.float64), 2), S64)
    assert np.linalg.norm(Qg.T @ Qg - np.eye(r)) <= TOL_ORTH
    assert np.max(np.abs(ritz[:5] - sigma[:5]) / sigma[:5]) <= TOL
    assert np.all(np.diff(ritz) <= 0)
    assert np.max(np.abs(ritz - S)) <= TOL * sigma[0]           # the small ones in absolute terms
    assert np.all(ritz[5:] <= 2.0 * sigma[5])


@pytest.mark.parametrize("mode", ["average", "nesterov", "heavy_ball", "own_delta"])
def test_outer_step(torch, mode):
    from paper_2602_04396_amd import lordo
    shapes = [(100, 77, 8), (64, 128, 16), (33, 2049, 4)]
    kw = dict(average=dict(outer_lr=1.0), nesterov=dict(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True),
              heavy_ball=dict(outer_lr=0.5, outer_momentum=0.8), own_delta=dict(outer_lr=0.9, outer_momentum=0.5, outer_nesterov=True))[mode]
    ohp = orc.Hyper(**kw)
    pair = Pair(torch, shapes, _weights(shapes, 30), ohp, lordo.hparams(**kw), _rand_Q(shapes, 30))
    gens = _spiked(shapes, 30, 2)
    step = 0
    for rnd in range(2):
        for _ in range(2):
            pair.local_step([g.draw(step) for g in gens], lr=1e-2, first_step_patch=(step == 0))
            step += 1
        own = [orc.pseudo_gradient(pair.st[i], pair.W_orc[i]) for i in range(len(shapes))]
        out = [torch.empty_like(w) for w in pair.W_gpu]
        pair.opt.export_pseudograd(pair.W_gpu, out)
        for i in range(len(shapes)):
            assert rel_l2(out[i].cpu().numpy(), own[i]) <= TOL
        if mode == "own_delta":
            avg = own
            pair.opt.outer_step(pair.W_gpu, None)
        else:
            other = [synth.SpikedGradient(p, q, 2, synth.seed_for(31, i), bf16=False).draw(rnd) * 1e-2 * 2
                     for i, (p, q, r) in enumerate(shapes)]
            avg = [synth.avg_pseudograd(out[i].cpu().numpy(), other[i]) for i in range(len(shapes))]
            pair.opt.outer_step(pair.W_gpu, pair.to_dev(avg, False))
        for i in range(len(shapes)):
            Wn = orc.outer_step(pair.st[i], np.asarray(avg[i], dtype=np.float64), ohp)
            pair.W_orc[i] = Wn
            got = pair.W_gpu[i].cpu().numpy().astype(np.float64)
            assert rel_l2(got - pair.W0[i], Wn - pair.W0[i]) <= TOL, f"{mode} round {rnd} matrix {i}"
            assert torch.equal(pair.opt.get_state(i, lordo.STATE_ANCHOR), pair.W_gpu[i])  # anchor <- new model
            if ohp.outer_momentum != 0:
                assert rel_l2(pair.get(i, lordo.STATE_MOM), pair.st[i].b) <= TOL
    if mode == "average":
        # eta_s = 1, no momentum: the new model is the mean of the workers' models (Alg. 1 default)
        pass


@pytest.mark.parametrize("mode", ["average", "nesterov", "heavy_ball_lowqhm", "own_buffer_unaligned"])
def test_uplink_buffer_and_lowrank_outer_step(torch, mode):
    """Up-link time buffer (App. A.5.1): A accumulates eta_t N_t over the window, Q A is the dense
    pseudo-gradient, and the outer step fed the mean of the workers' buffers matches the oracle's."""
    from paper_2602_04396_amd import lordo
    kw = dict(average=dict(outer_lr=1.0), nesterov=dict(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True),
              heavy_ball_lowqhm=dict(outer_lr=0.5, outer_momentum=0.8, qhm_mode="low", omega=0.8),
              own_buffer_unaligned=dict(outer_lr=0.9, outer_momentum=0.5, outer_nesterov=True))[mode]
    shapes = [(100, 77, 8), (33, 2049, 4), (130, 67, 33)] if mode == "own_buffer_unaligned" else \
             [(200, 328, 48), (96, 72, 20), (300, 136, 33), (256, 192, 128)]
    ohp = orc.Hyper(uplink_buffer=True, **kw)
    gkw = {k: v for k, v in kw.items() if k != "qhm_mode"}
    ghp = lordo.hparams(uplink_buffer=True, qhm_mode=1 if kw.get("qhm_mode") == "low" else 0, **gkw)
    pair = Pair(torch, shapes, _weights(shapes, 33), ohp, ghp, _rand_Q(shapes, 33))
    gens = _spiked(shapes, 33, 4)
    n = len(shapes)
    step = 0
    for window in range(2):
        for k in range(3):
            pair.local_step([g.draw(step) for g in gens], lr=1e-3 * (1 + k), first_step_patch=(step == 0))
            step += 1
        pair.compare_local(TOL)                                   # includes the buffer A against the oracle's
        out = [torch.empty(r, q, dtype=torch.float32, device="cuda") for p, q, r in shapes]
        pair.opt.export_uplink(out)
        dense = [torch.empty_like(w) for w in pair.W_gpu]
        pair.opt.export_pseudograd(pair.W_gpu, dense)
        for i in range(n):
            assert torch.equal(out[i], pair.opt.get_state(i, lordo.STATE_UPLINK))
            Qg = pair.get(i, lordo.STATE_Q)
            assert rel_l2(Qg @ out[i].cpu().numpy().astype(np.float64), dense[i].cpu().numpy()) <= TOL   # anchor - W = Q A
        with pytest.raises(lordo.LordoError) as e:                # the buffer is in coordinates of the current Q
            pair.opt.refresh_subspace(pair.to_dev([g.draw(0) for g in gens], True),
                                      pair.to_dev([np.zeros((q, r), np.float32) for p, q, r in shapes], False))
        assert e.value.code == lordo.ESTATE
        if mode == "own_buffer_unaligned":
            avg = [o.cpu().numpy() for o in out]
            pair.opt.outer_step_lowrank(pair.W_gpu, None)
        else:
            rng = np.random.default_rng(synth.seed_for(33, 700 + window))
            other = [(rng.standard_normal((r, q)) * 3e-3).astype(np.float32) for p, q, r in shapes]   # another worker's buffer
            avg = [(0.5 * (out[i].cpu().numpy().astype(np.float64) + other[i])).astype(np.float32) for i in range(n)]
            pair.opt.outer_step_lowrank(pair.W_gpu, pair.to_dev(avg, False))
        pair.opt.poll_status()
        for i in range(n):
            Wn = orc.outer_step_lowrank(pair.st[i], np.asarray(avg[i], dtype=np.float64), ohp)
            pair.W_orc[i] = Wn
            got = pair.W_gpu[i].cpu().numpy().astype(np.float64)
            assert rel_l2(got - pair.W0[i], Wn - pair.W0[i]) <= TOL, f"{mode} window {window} matrix {i}"
            assert torch.equal(pair.opt.get_state(i, lordo.STATE_ANCHOR), pair.W_gpu[i])
            if ohp.outer_momentum != 0:
                assert rel_l2(pair.get(i, lordo.STATE_MOM), pair.st[i].b) <= TOL
            assert not pair.opt.get_state(i, lordo.STATE_UPLINK).any()      # a new window starts empty
    # the dense outer step ends a window too
    pair.local_step([g.draw(step) for g in gens], lr=1e-3)
    pair.opt.outer_step(pair.W_gpu, None)
    assert not pair.opt.get_state(0, lordo.STATE_UPLINK).any()
    # no buffer configured: the calls say so
    plain = Pair(torch, shapes[:1], _weights(shapes[:1], 33), orc.Hyper(), lordo.hparams())
    for call in (lambda: plain.opt.outer_step_lowrank(plain.W_gpu, None),
                 lambda: plain.opt.export_uplink([torch.empty(shapes[0][2], shapes[0][1], device="cuda")]),
                 lambda: plain.opt.get_state(0, lordo.STATE_UPLINK)):
        with pytest.raises(lordo.LordoError) as e:
            call()
        assert e.value.code == lordo.ESTATE


def test_packed_sync_payload_two_workers(torch):
    """Synchronisation through the packed payload (Alg. 1 synchronisation of the optimizer states; App. A.5.1): two
    workers with the same Q and different gradients average the contiguous region [u | v | A] in place -- what a single
    all-reduce(mean) would do -- and take the low-rank outer step from the averaged buffer where it lies.  Every tensor
    must equal the mean of the two oracle workers' tensors, and both workers must end with identical weights."""
    from paper_2602_04396_amd import lordo
    shapes = [(200, 328, 48), (96, 72, 20), (300, 136, 33), (256, 192, 128)]
    kw = dict(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True)
    ohp, ghp = orc.Hyper(uplink_buffer=True, **kw), lordo.hparams(uplink_buffer=True, **kw)
    n = len(shapes)
    W0, Q0 = _weights(shapes, 35), _rand_Q(shapes, 35)
    workers = [Pair(torch, shapes, W0, ohp, ghp, Q0) for _ in range(2)]
    gens = [_spiked(shapes, 35 + 40 * w, 4) for w in range(2)]
    step = 0
    for window in range(2):
        for k in range(3):
            for w, pair in enumerate(workers):
                pair.local_step([g.draw(step) for g in gens[w]], lr=1e-3 * (1 + k), first_step_patch=(step == 0))
            step += 1
        for pair in workers:
            pair.compare_local(TOL)
        views = [pair.opt.sync_payload() for pair in workers]
        lr_total = views[0][1] // 2
        assert views[0][0].numel() == 3 * lr_total and views[0][1] == views[1][1]
        assert lr_total >= sum(r * q for p, q, r in shapes)
        mean = (views[0][0] + views[1][0]) * 0.5                   # the collective, stood in for by one elementwise mean
        for v, _ in views:
            v.copy_(mean)
        # oracle: the same means, tensor by tensor
        for i in range(n):
            u = 0.5 * (workers[0].st[i].u + workers[1].st[i].u)
            v = 0.5 * (workers[0].st[i].v + workers[1].st[i].v)
            A = 0.5 * (workers[0].st[i].A + workers[1].st[i].A)
            for pair in workers:
                pair.st[i].u, pair.st[i].v = u.copy(), v.copy()
                assert rel_l2(pair.get(i, lordo.STATE_U), u) <= TOL
                assert rel_l2(pair.get(i, lordo.STATE_V), v) <= TOL
                assert rel_l2(pair.get(i, lordo.STATE_UPLINK), A) <= TOL
                pair.W_orc[i] = orc.outer_step_lowrank(pair.st[i], A, ohp)
        for pair in workers:
            pair.opt.outer_step_lowrank(pair.W_gpu, None)
            pair.opt.poll_status()
        for i in range(n):
            for pair in workers:
                got = pair.W_gpu[i].cpu().numpy().astype(np.float64)
                assert rel_l2(got - pair.W0[i], pair.W_orc[i] - pair.W0[i]) <= TOL, f"window {window} matrix {i}"
                assert rel_l2(pair.get(i, lordo.STATE_MOM), pair.st[i].b) <= TOL
                assert not pair.opt.get_state(i, lordo.STATE_UPLINK).any()
            assert torch.equal(workers[0].W_gpu[i], workers[1].W_gpu[i])       # same inputs, deterministic kernels
    # without the up-link buffer the payload is the moments alone
    plain = Pair(torch, shapes[:2], _weights(shapes[:2], 35), orc.Hyper(), lordo.hparams())
    view, moments = plain.opt.sync_payload()
    assert view.numel() == moments


def test_random_initial_projection(torch):
    """Alg. 1 starts from a random projection: Q_0 = orth(Gaussian block) on the device against the oracle's
    (the factorisation with positive diagonal is unique, so the bases agree element by element), then steps."""
    from paper_2602_04396_amd import lordo
    shapes = [(200, 330, 48), (300, 129, 33), (96, 160, 20), (256, 192, 128), (520, 392, 256)]
    ohp, ghp = orc.Hyper(), lordo.hparams()
    pair = Pair(torch, shapes, _weights(shapes, 26), ohp, ghp)
    blocks = [np.random.default_rng(synth.seed_for(26, 300 + i)).standard_normal((p, r)).astype(np.float32)
              for i, (p, q, r) in enumerate(shapes)]
    pair.opt.init_projection(pair.to_dev(blocks, False))
    pair.opt.poll_status()
    for i, (p, q, r) in enumerate(shapes):
        Qg = pair.get(i, lordo.STATE_Q)
        Qo = orc.initial_projection(blocks[i])
        assert np.linalg.norm(Qg.T @ Qg - np.eye(r)) <= TOL_ORTH
        assert rel_l2(Qg, Qo) <= TOL, f"Q_0 of matrix {i}"
        pair.st[i].Q = Qg                      # the oracle continues from the fp32 basis the library holds
    gens = _spiked(shapes, 26, 8)
    for t in range(2):
        pair.local_step([g.draw(t) for g in gens], lr=1e-3, first_step_patch=(t == 0))
    pair.compare_local(TOL)
    with pytest.raises(lordo.LordoError) as e:     # moments are running: only a refresh may change the basis now
        pair.opt.init_projection(pair.to_dev(blocks, False))
    assert e.value.code == lordo.ESTATE


def test_state_roundtrip_and_errors(torch):
    from paper_2602_04396_amd import lordo
    p, q, r = 70, 45, 9
    W = [torch.randn(p, q, device="cuda")]
    opt = lordo.Lordo([(p, q, r)], lordo.hparams(outer_momentum=0.5), W, torch)
    assert torch.equal(opt.get_state(0, lordo.STATE_ANCHOR), W[0])
    Q0 = opt.get_state(0, lordo.STATE_Q).cpu().numpy()
    assert np.array_equal(Q0, np.eye(p, r, dtype=np.float32))
    for which in (lordo.STATE_U, lordo.STATE_V):
        x = torch.rand(r, q, device="cuda")
        opt.set_state(0, which, x)
        assert torch.equal(opt.get_state(0, which), x)
    opt.step = 17
    assert opt.step == 17
    with pytest.raises(lordo.LordoError) as e:
        opt.set_state(0, lordo.STATE_GLOW, torch.rand(r, q, device="cuda"))
    assert e.value.code == lordo.EINVAL
    with pytest.raises(lordo.LordoError) as e:
        lordo.Lordo([(8, 8, 9)], lordo.hparams(), [torch.zeros(8, 8, device="cuda")], torch)
    assert e.value.code == lordo.EINVAL
    with pytest.raises(lordo.LordoError) as e:
        lordo.Lordo([(8, 8, 4)], lordo.hparams(qhm_mode=3), [torch.zeros(8, 8, device="cuda")], torch)
    assert e.value.code == lordo.EINVAL
    with pytest.raises(lordo.LordoError) as e:                # no residual without error feedback
        opt.get_state(0, lordo.STATE_ERR)
    assert e.value.code == lordo.ESTATE
    opt.poll_status()


@pytest.mark.parametrize("rayleigh_ritz,top_rank,short_side", [(False, 128, False), (True, 128, False), (True, 200, False), (True, 128, True)],
                         ids=["plain_refresh", "rayleigh_ritz", "rayleigh_ritz_blocked_solver", "tall_matrix_projected_on_the_right"])
def test_two_contexts_with_the_same_inputs_agree_bit_for_bit(torch, rayleigh_ritz, top_rank, short_side):
    """Workers that see the same averaged source recompute the same projection instead of receiving it (Alg. 1): that
    needs run-to-run identical results.  Two contexts, identical inputs, steps (split-K down-projection), a refresh
    (grouped GEMMs with split-K, factorisations, with or without the Rayleigh-Ritz solver), more steps and an outer
    step: every state tensor must agree bit for bit."""
    from paper_2602_04396_amd import lordo
    shapes = [(520, 392, top_rank), (300, 640, 64), (200, 328, 48), (1024, 256, 100)]
    kw = dict(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True, power_iters=2, rayleigh_ritz=rayleigh_ritz)
    gens = _spiked(shapes, 39, 6)
    W0 = _weights(shapes, 39)
    Om = [torch.tensor(synth.omega(np.random.default_rng(synth.seed_for(39, 900 + i)), q, r), device="cuda")
          for i, (p, q, r) in enumerate(shapes)]
    if short_side:          # the tall matrix projected on its columns: generic products in the refresh, shadow launches in the step
        Om[3] = torch.tensor(synth.omega(np.random.default_rng(synth.seed_for(39, 903)), 1024, 100), device="cuda")
        shapes = shapes[:3] + [(1024, 256, 100, 1)]
    G = [[torch.tensor(g.draw(t), device="cuda").bfloat16() for g in gens] for t in range(5)]
    runs = []
    for _ in range(2):
        W = [torch.tensor(w, dtype=torch.float32, device="cuda") for w in W0]
        opt = lordo.Lordo(shapes, lordo.hparams(**kw), W, torch)
        opt.local_step(W, G[0], 1e-3)
        opt.local_step(W, G[1], 2e-3)
        opt.refresh_subspace(G[2], Om)
        opt.local_step(W, G[3], 1e-3)
        opt.outer_step(W, None)
        opt.local_step(W, G[4], 1e-3)
        opt.poll_status()
        runs.append((W, opt))
    (Wa, a), (Wb, b) = runs
    for i in range(len(shapes)):
        assert torch.equal(Wa[i], Wb[i]), f"W of matrix {i}"
        for which in (lordo.STATE_Q, lordo.STATE_U, lordo.STATE_V, lordo.STATE_ANCHOR, lordo.STATE_MOM, lordo.STATE_NUPD):
            assert torch.equal(a.get_state(i, which), b.get_state(i, which)), f"state {which} of matrix {i}"
    assert torch.equal(a.mssv(), b.mssv())
    if rayleigh_ritz:
        assert torch.equal(a.stable_rank(), b.stable_rank())
        assert torch.equal(a.spectral_gap(G[2], Om), b.spectral_gap(G[2], Om))


def test_calls_follow_the_callers_stream(torch):
    """Every call only enqueues on the stream it is given: the same sequence on a side stream, with its inputs
    produced on that stream right before each call and no synchronisation in between, gives the same bits as on the
    default stream."""
    from paper_2602_04396_amd import lordo
    shapes = [(520, 392, 128), (300, 640, 64), (200, 328, 48)]
    kw = dict(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True, power_iters=1)
    W0 = [torch.tensor(w, dtype=torch.float32, device="cuda") for w in _weights(shapes, 40)]
    base = [torch.tensor(g.draw(0), device="cuda") for g in _spiked(shapes, 40, 6)]
    Om = [torch.tensor(synth.omega(np.random.default_rng(synth.seed_for(40, 900 + i)), q, r), device="cuda")
          for i, (p, q, r) in enumerate(shapes)]
    torch.cuda.synchronize()

    def run():
        W = [w.clone() for w in W0]
        opt = lordo.Lordo(shapes, lordo.hparams(**kw), W, torch)
        for t in range(4):
            G = [(b * (1.0 + 0.25 * t)).bfloat16() for b in base]       # produced on the current stream, consumed at once
            if t == 2:
                opt.refresh_subspace(G, Om)
            opt.local_step(W, G, 1e-3)
        opt.outer_step(W, None)
        return W, opt

    Wa, a = run()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        Wb, b = run()
    side.synchronize()
    torch.cuda.synchronize()
    a.poll_status()
    b.poll_status()
    for i in range(len(shapes)):
        assert torch.equal(Wa[i], Wb[i])
        for which in (lordo.STATE_Q, lordo.STATE_U, lordo.STATE_V, lordo.STATE_MOM):
            assert torch.equal(a.get_state(i, which), b.get_state(i, which))
