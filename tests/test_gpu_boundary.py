"""Boundary semantics of the C ABI that need a GPU: blocks drawn by the library's own generator (Alg. 1 "Require":
random initial projection; Gaussian start of the range finder) against the oracle's implementation of the same
counter-based generator, matrices left out of a refresh, the state check of the outer step, eps = 0."""
import ctypes as C

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
    lordo.load()
    return t


def _weights(shapes, cfg):
    return [synth.weights(np.random.default_rng(synth.seed_for(cfg, 500 + i)), sh[0], sh[1]) for i, sh in enumerate(shapes)]


def _spiked(shapes, cfg, n_spike, bf16=True):
    return [synth.SpikedGradient(sh[0], sh[1], n_spike, synth.seed_for(cfg, i), bf16=bf16) for i, sh in enumerate(shapes)]


def test_library_drawn_blocks_match_the_oracle_generator(torch):
    """No block from the caller: Q_0 = orth(Gaussian block) and the start blocks of two refreshes come from the
    library's generator (seed, matrix, draw number, element).  The oracle draws the same blocks with its own
    implementation of that generator; the initial basis then agrees element by element (unique factorisation), the
    refreshed subspaces as projectors."""
    from paper_2602_04396_amd import lordo
    seed = 0x9E3779B97F4A7C15
    shapes = [(200, 330, 48), (300, 129, 33), (96, 160, 20), (256, 192, 128), (520, 392, 256)]
    ohp, ghp = orc.Hyper(power_iters=1), lordo.hparams(power_iters=1, seed=seed)
    pair = Pair(torch, shapes, _weights(shapes, 71), ohp, ghp)
    pair.opt.init_projection(None)                               # draw 0
    pair.opt.poll_status()
    for i, (p, q, r) in enumerate(shapes):
        Qg = pair.get(i, lordo.STATE_Q)
        Qo = orc.initial_projection(orc.gaussian_block(seed, i, 0, p, r))
        assert np.linalg.norm(Qg.T @ Qg - np.eye(r)) <= TOL_ORTH
        assert rel_l2(Qg, Qo) <= TOL, f"Q_0 of matrix {i}"
        pair.st[i].Q = Qg
    gens = _spiked(shapes, 71, 8)
    for t in range(2):
        pair.local_step([g.draw(t) for g in gens], lr=1e-3, first_step_patch=(t == 0))
    pair.compare_local(TOL)
    for draw in (1, 2):                                          # two refreshes: draws 1 and 2, bf16 then fp32 source
        bf16 = draw == 1
        Src = [g.draw(10 + draw) for g in gens]
        Sd = pair.to_dev(Src, bf16)
        pair.opt.refresh_subspace(Sd, None)
        pair.opt.poll_status()
        for i, (p, q, r) in enumerate(shapes):
            Qg = pair.get(i, lordo.STATE_Q)
            Om = orc.gaussian_block(seed, i, draw, q, r)
            Qo = orc.range_finder(np.asarray(Src[i], dtype=np.float64), Om, 1)
            assert np.linalg.norm(Qg.T @ Qg - np.eye(r)) <= TOL_ORTH
            assert projector_distance(Qg, Qo) <= TOL_SUBSPACE, f"refresh {draw}, matrix {i}"
            orc.refresh_subspace(pair.st[i], None, None, ohp, Q_forced=Qg)
        pair.local_step([g.draw(20 + draw) for g in gens], lr=1e-3)
        pair.compare_local(TOL)
    # the same seed in a second context gives the same blocks, bit for bit; another seed does not
    W2 = [torch.tensor(w, device="cuda") for w in _weights(shapes, 71)]
    a = lordo.Lordo(shapes, lordo.hparams(power_iters=1, seed=seed), W2, torch)
    b = lordo.Lordo(shapes, lordo.hparams(power_iters=1, seed=seed + 1), W2, torch)
    a.init_projection(None)
    b.init_projection(None)
    pair2 = Pair(torch, shapes, _weights(shapes, 71), ohp, ghp)
    pair2.opt.init_projection(None)
    for i in range(len(shapes)):
        assert torch.equal(a.get_state(i, lordo.STATE_Q), pair2.opt.get_state(i, lordo.STATE_Q))
        assert not torch.equal(a.get_state(i, lordo.STATE_Q), b.get_state(i, lordo.STATE_Q))


@pytest.mark.parametrize("aligned", [True, False])
def test_refresh_leaves_out_matrices_with_a_null_source(torch, aligned):
    """A NULL entry in the source table: that matrix keeps Q, u, v (and its similarity value) bit for bit while
    the others are refreshed as usual -- on the specialised refresh kernels (aligned shapes) and on the grouped GEMM."""
    from paper_2602_04396_amd import lordo
    shapes = [(256, 384, 64), (512, 256, 128), (384, 256, 64), (256, 256, 32)] if aligned else \
             [(200, 330, 48), (300, 129, 33), (96, 160, 20), (130, 257, 64)]
    ohp, ghp = orc.Hyper(power_iters=2), lordo.hparams(power_iters=2)
    pair = Pair(torch, shapes, _weights(shapes, 72), ohp, ghp)
    gens = _spiked(shapes, 72, 8)
    Om = [synth.omega(np.random.default_rng(synth.seed_for(72, 900 + i)), q, r) for i, (p, q, r) in enumerate(shapes)]
    dists, orths = pair.refresh([g.draw(0) for g in gens], Om, bf16=True)
    assert max(dists) <= TOL_SUBSPACE and max(orths) <= TOL_ORTH
    for t in range(2):
        pair.local_step([g.draw(1 + t) for g in gens], lr=1e-3, first_step_patch=(t == 0))
    pair.compare_local(TOL)
    mssv_before = pair.opt.mssv().clone()
    left_out = (1, 3)
    before = {i: [pair.opt.get_state(i, w).clone() for w in (lordo.STATE_Q, lordo.STATE_U, lordo.STATE_V)] for i in left_out}
    Src = [g.draw(5) for g in gens]
    Sd = pair.to_dev(Src, True)
    Od = pair.to_dev(Om, False)
    pair.opt.refresh_subspace([None if i in left_out else Sd[i] for i in range(len(shapes))],
                              [None if i in left_out else Od[i] for i in range(len(shapes))])
    pair.opt.poll_status()
    mssv_after = pair.opt.mssv()
    for i, (p, q, r) in enumerate(shapes):
        if i in left_out:
            for old, which in zip(before[i], (lordo.STATE_Q, lordo.STATE_U, lordo.STATE_V)):
                assert torch.equal(old, pair.opt.get_state(i, which)), f"matrix {i} was to be left alone"
            assert mssv_after[i] == mssv_before[i]
            continue
        Qg = pair.get(i, lordo.STATE_Q)
        Qo = orc.range_finder(np.asarray(Src[i], dtype=np.float64), np.asarray(Om[i], dtype=np.float64), 2)
        assert np.linalg.norm(Qg.T @ Qg - np.eye(r)) <= TOL_ORTH
        assert projector_distance(Qg, Qo) <= TOL_SUBSPACE, f"matrix {i}"
        orc.refresh_subspace(pair.st[i], None, None, ohp, Q_forced=Qg)
        assert rel_l2(pair.get(i, lordo.STATE_U), pair.st[i].u) <= TOL and rel_l2(pair.get(i, lordo.STATE_V), pair.st[i].v) <= TOL
    # the optimizer goes on with the mixed set of bases
    pair.local_step([g.draw(6) for g in gens], lr=1e-3)
    pair.compare_local(TOL)
    # a start block is needed for every matrix that takes part
    with pytest.raises(lordo.LordoError) as e:
        pair.opt.refresh_subspace(Sd, [None] + Od[1:])
    assert e.value.code == lordo.EINVAL
    # nothing to do is not an error
    none = (C.c_void_p * len(shapes))()
    assert pair.opt.lib.lordo_refresh_subspace(pair.opt.ctx, none, lordo.BF16, none, None) == lordo.OK


def test_outer_step_needs_local_steps_for_its_own_pseudo_gradient(torch):
    """Through the raw C symbol: with no averaged pseudo-gradient the outer step uses anchor - W, which exists only
    after a local step of the current window; before that the call is a state error and touches nothing."""
    from paper_2602_04396_amd import lordo
    p, q, r = 96, 128, 16
    W = [torch.randn(p, q, device="cuda") * 0.02]
    opt = lordo.Lordo([(p, q, r)], lordo.hparams(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True), W, torch)
    Wp = (C.c_void_p * 1)(W[0].data_ptr())
    W0 = W[0].clone()
    assert opt.lib.lordo_outer_step(opt.ctx, Wp, None, None) == lordo.ESTATE
    torch.cuda.synchronize()
    assert torch.equal(W[0], W0) and not opt.get_state(0, lordo.STATE_MOM).any()
    G = [(torch.randn(p, q, device="cuda") * 1e-3).bfloat16()]
    opt.local_step(W, G, 1e-3)
    assert opt.lib.lordo_outer_step(opt.ctx, Wp, None, None) == lordo.OK
    assert opt.lib.lordo_outer_step(opt.ctx, Wp, None, None) == lordo.ESTATE        # the window is empty again
    D = [torch.randn(p, q, device="cuda") * 1e-3]
    Dp = (C.c_void_p * 1)(D[0].data_ptr())
    assert opt.lib.lordo_outer_step(opt.ctx, Wp, Dp, None) == lordo.OK               # a given mean needs no own steps
    bad = (C.c_void_p * 1)()
    assert opt.lib.lordo_outer_step(opt.ctx, bad, Dp, None) == lordo.EINVAL
    assert opt.lib.lordo_outer_step(opt.ctx, Wp, bad, None) == lordo.EINVAL
    opt.poll_status()


@pytest.mark.parametrize("variant", ["plain", "uplink", "fused"])
def test_eps_zero_with_ragged_ranks_stays_finite_and_matches(torch, variant):
    """eps = 0 (Sec. 2 puts eps outside the root, so the update is then u_hat / sqrt(v_hat)): the zero padding of the
    low-rank arrays has a zero second moment, and the update there must be zero, not 0 / 0 -- ranks that are not a
    multiple of 32 (config 1 has r = 16) would otherwise turn the whole weight matrix into NaN.  `fused`: a launch
    without split-K, where the update runs in the epilogue of the down-projection."""
    from paper_2602_04396_amd import lordo
    if variant == "fused":
        shapes = [(160, 8192 + 64, 40)]             # a short matrix: no split-K, the update rides in the down-projection
    else:
        shapes = [(256, 256, 16), (200, 330, 48), (96, 70, 20), (300, 129, 33)]
    uplink = variant == "uplink"
    ohp = orc.Hyper(eps=0.0, uplink_buffer=uplink)
    ghp = lordo.hparams(eps=0.0, uplink_buffer=uplink)
    Q0 = [synth.orthonormal(np.random.default_rng(synth.seed_for(73, 700 + i)), p, r) for i, (p, q, r) in enumerate(shapes)]
    pair = Pair(torch, shapes, _weights(shapes, 73), ohp, ghp, Q0)
    gens = _spiked(shapes, 73, 8)
    for t in range(3):
        pair.local_step([g.draw(t) for g in gens], lr=1e-3, first_step_patch=(t == 0))
        for i in range(len(shapes)):
            assert torch.isfinite(pair.W_gpu[i]).all(), f"step {t}, matrix {i}"
    pair.compare_local(TOL)
    view, moments = pair.opt.sync_payload()
    assert torch.isfinite(view).all()                # the padding of the packed payload stays zero
    if uplink:
        pair.opt.outer_step_lowrank(pair.W_gpu, None)
        for i in range(len(shapes)):
            Wn = orc.outer_step_lowrank(pair.st[i], pair.st[i].A.copy(), ohp)
            got = pair.W_gpu[i].cpu().numpy().astype(np.float64)
            assert rel_l2(got - pair.W0[i], Wn - pair.W0[i]) <= TOL
    pair.opt.poll_status()


@pytest.mark.parametrize("shape_set,update", [("split_k", "plain"), ("fused_128_rank_tiles", "plain"), ("fused_256_rank_tiles", "plain"),
                                              ("split_k", "global"), ("fused_256_rank_tiles", "global")])
def test_recorded_local_step_counts_its_replays(torch, shape_set, update):
    """A local step recorded into a HIP graph: the step count and the bias corrections 1 - beta^t (Sec. 2) live in device
    memory and advance per REPLAY, so replaying the recording k times on new gradients is k local steps.  Two contexts
    from the same start: one issues the steps one by one, the other replays one recording; weights and state must be
    equal bit for bit after every replay (eager work and synchronisation between the replays), and the oracle agrees.
    Then a refresh on the replayed context rotates the moments with the bias corrections of the replayed count.
    `global`: the same with error feedback and the full-rank QHM update (the paper's LoRDO-Global), whose step holds the
    residual launch and the gradient-term epilogue as well; the residual is compared too."""
    from paper_2602_04396_amd import lordo
    shapes = {"split_k": [(256, 384, 64), (130, 260, 128), (520, 392, 96)],
              "fused_128_rank_tiles": [(256, 520, 192), (250, 388, 120)],          # no matrix taller than 256 rows: no split-K,
              "fused_256_rank_tiles": [(256, 520, 256), (250, 388, 250)]}[shape_set]  # the moment update is in the epilogue
    n = len(shapes)
    W0 = _weights(shapes, 73)
    Q0 = [synth.orthonormal(np.random.default_rng(synth.seed_for(73, 700 + i)), p, r).astype(np.float32) for i, (p, q, r) in enumerate(shapes)]
    kw = dict(error_feedback=True, omega=0.8) if update == "global" else {}
    ohp, ghp = orc.Hyper(qhm_mode="full" if kw else "none", **kw), lordo.hparams(qhm_mode=2 if kw else 0, **kw)
    eager = Pair(torch, shapes, W0, ohp, ghp, Q0)
    Wr = [torch.tensor(w, device="cuda") for w in W0]
    rec = lordo.Lordo(shapes, ghp, Wr, torch)
    for i in range(n):
        rec.set_state(i, lordo.STATE_Q, torch.tensor(Q0[i], device="cuda").contiguous())
    gens = _spiked(shapes, 73, 6)
    Gbuf = [torch.zeros(p, q, device="cuda", dtype=torch.bfloat16) for p, q, r in shapes]
    lr = 2e-3

    def load(t):
        G = [g.draw(t) for g in gens]
        for buf, g in zip(Gbuf, G):
            buf.copy_(torch.tensor(g, device="cuda").bfloat16())
        return G

    # first step issued on both (also lets every kernel of the step set itself up outside the recording)
    G = load(0)
    rec.local_step(Wr, Gbuf, lr)
    eager.local_step(G, lr=lr, first_step_patch=True)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rec.local_step(Wr, Gbuf, lr)             # recorded, not run
    for t in range(1, 5):
        G = load(t)
        graph.replay()
        eager.local_step(G, lr=lr)
        torch.cuda.synchronize()
        for i in range(n):
            assert torch.equal(Wr[i], eager.W_gpu[i]), f"weights after replay {t}, matrix {i}"
            for which in (lordo.STATE_U, lordo.STATE_V, lordo.STATE_NUPD) + ((lordo.STATE_ERR,) if kw else ()):
                assert torch.equal(rec.get_state(i, which), eager.opt.get_state(i, which)), f"state {which} after replay {t}, matrix {i}"
    worst = eager.compare_local(TOL)                              # and the eager chain is the oracle's chain
    print(f"recorded step, {shape_set} {update}: 4 replays bit-equal to 4 issued steps; against the oracle {worst}", flush=True)
    assert rec.step == 2 and eager.opt.step == 5                 # issued calls: the recording counts once
    if shape_set == "fused_256_rank_tiles":
        return                      # (r = p: a square start block, not a case for the range finder)
    # a refresh after the replays: tell the context how many steps ran, then both rotate alike
    rec.step = 5
    Src = [g.draw(50) for g in gens]
    Om = [synth.omega(np.random.default_rng(synth.seed_for(73, 900 + i)), q, r) for i, (p, q, r) in enumerate(shapes)]
    Sd = [torch.tensor(a, device="cuda").bfloat16() for a in Src]
    Od = [torch.tensor(o, device="cuda", dtype=torch.float32) for o in Om]
    rec.refresh_subspace(Sd, Od)
    eager.opt.refresh_subspace(Sd, Od)
    rec.poll_status(); eager.opt.poll_status()
    for i in range(n):
        for which in (lordo.STATE_Q, lordo.STATE_U, lordo.STATE_V):
            assert torch.equal(rec.get_state(i, which), eager.opt.get_state(i, which)), f"state {which} after the refresh, matrix {i}"
