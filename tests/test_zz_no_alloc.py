"""lordo_init_static: the context whose workspace is the library's own fixed device array (for callers that
cannot allocate device memory) against the context of lordo_init on a torch-allocated arena -- same inputs, same
calls, results compared bit for bit (the kernels are deterministic and both contexts use the same layout), on two
contexts in a row, the second over smaller matrices in the array the first one left behind."""
import ctypes as C

import numpy as np
import pytest

from paper_2602_04396_amd import synth

pytestmark = pytest.mark.gpu


def _run(torch, lordo, shapes, static, seed):
    """init, library-drawn Q_0, two steps, refresh with library-drawn start blocks, a step, outer step, a step."""
    dev = torch.device("cuda:0")
    W = [torch.tensor(synth.weights(np.random.default_rng(synth.seed_for(81, i)), p, q), device=dev) for i, (p, q, r) in enumerate(shapes)]
    gens = [synth.SpikedGradient(p, q, 4, synth.seed_for(81, 100 + i)) for i, (p, q, r) in enumerate(shapes)]
    G = [[torch.tensor(g.draw(t), device=dev).bfloat16() for g in gens] for t in range(5)]
    hp = lordo.hparams(outer_lr=0.7, outer_momentum=0.9, outer_nesterov=True, power_iters=1, seed=seed)
    opt = lordo.Lordo(shapes, hp, W, torch, static_workspace=static)
    opt.init_projection(None)
    opt.local_step(W, G[0], 1e-3)
    opt.local_step(W, G[1], 2e-3)
    opt.refresh_subspace(G[2], None)
    opt.local_step(W, G[3], 1e-3)
    opt.outer_step(W, None)
    opt.local_step(W, G[4], 1e-3)
    opt.poll_status()
    state = {}
    for i in range(len(shapes)):
        for which in (lordo.STATE_Q, lordo.STATE_U, lordo.STATE_V, lordo.STATE_ANCHOR, lordo.STATE_MOM, lordo.STATE_GLOW, lordo.STATE_NUPD):
            state[(i, which)] = opt.get_state(i, which).clone()
    mssv = opt.mssv().clone()
    return opt, W, state, mssv


def test_static_workspace_context_matches_the_arena_context_twice_in_a_row():
    import torch
    from paper_2602_04396_amd import lordo
    lib = lordo.load()
    first = [(256, 384, 64), (192, 128, 32), (130, 257, 48)]
    second = [(128, 96, 16)]                                      # smaller: runs inside what the first context left
    assert lordo.workspace_bytes(second, lordo.hparams(outer_momentum=0.9)) < lordo.workspace_bytes(first, lordo.hparams(outer_momentum=0.9))
    for shapes in (first, second):
        assert lordo.workspace_bytes(shapes, lordo.hparams(outer_momentum=0.9)) <= lordo.STATIC_WORKSPACE_BYTES
        ref, W_ref, st_ref, mssv_ref = _run(torch, lordo, shapes, False, 17)
        opt, W, st, mssv = _run(torch, lordo, shapes, True, 17)
        for i in range(len(shapes)):
            assert torch.equal(W[i], W_ref[i]), f"weights of matrix {i} {shapes[i]}"
            assert torch.isfinite(W[i]).all()
        for key in st_ref:
            assert torch.equal(st[key], st_ref[key]), f"state {key}"
        assert torch.equal(mssv, mssv_ref)
        # one context per GPU at a time: a second one would share the array
        other = C.c_void_p()
        hp = lordo.hparams()
        Wp = (C.c_void_p * len(shapes))(*[w.data_ptr() for w in W])
        shp = (lordo.Shape * len(shapes))(*[lordo.Shape(p, q, r, 0) for p, q, r in shapes])
        assert lib.lordo_init_static(C.byref(other), shp, len(shapes), C.byref(hp), Wp, None) == lordo.ESTATE and not other.value
        opt.close()
        ref.close()
    # beyond the fixed size: refused with a clear error, nothing allocated
    big = [(4096, 4096, 128)]
    assert lordo.workspace_bytes(big, lordo.hparams()) > lordo.STATIC_WORKSPACE_BYTES
    ctx = C.c_void_p()
    hp = lordo.hparams()
    Wbig = [torch.zeros(4096, 4096, device="cuda")]
    Wp = (C.c_void_p * 1)(Wbig[0].data_ptr())
    shp = (lordo.Shape * 1)(lordo.Shape(4096, 4096, 128, 0))
    assert lib.lordo_init_static(C.byref(ctx), shp, 1, C.byref(hp), Wp, None) == lordo.ENOMEM and not ctx.value
    # after the refusal and the releases above the array is free again
    opt = lordo.Lordo(second, lordo.hparams(), [torch.zeros(128, 96, device="cuda")], torch, static_workspace=True)
    opt.close()
