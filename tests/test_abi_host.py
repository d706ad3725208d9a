"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes its arena sensibly and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_2602_04396_amd import lordo, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(lordo.LIB_PATH):
        from paper_2602_04396_amd import build
        build.build(verbose=False)
    return lordo.load()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "lordo.h")).read()
    declared = set(re.findall(r"\b(lordo_[a-z_]+)\s*\(", header))
    assert declared == set(lordo.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layout_matches_header():
    assert C.sizeof(lordo.Shape) == 24
    assert C.sizeof(lordo.HParams) == 104 and lordo.HParams.seed.offset == 96 and lordo.HParams.err_dtype.offset == 88
    assert lordo.HParams.rayleigh_ritz.offset == 80
    assert lordo.HParams.omega.offset == 32 and lordo.HParams.outer_lr.offset == 48
    assert lordo.HParams.power_iters.offset == 64 and lordo.HParams.grad_dtype.offset == 72


def test_workspace_bytes_scales_and_validates(lib):
    hp = lordo.hparams()
    small = lordo.workspace_bytes([(256, 256, 16)], hp)
    c2 = lordo.workspace_bytes(synth.config_shapes("c2"), hp)
    assert 0 < small < c2
    # state alone (u, v, anchor) is a lower bound; scratch keeps the total within a small multiple
    shapes = synth.config_shapes("c2")
    lower = sum(4 * (p * q + 2 * r * q) for p, q, r in shapes)
    assert lower < c2 < 8 * lower
    with_mom = lordo.workspace_bytes(shapes, lordo.hparams(outer_momentum=0.9))
    assert with_mom - c2 >= sum(4 * p * q for p, q, r in shapes)
    for bad in ([(8, 8, 9)], [(0, 8, 1)], [(8, 8, 0)],
                [(32768, 32768, 64)],          # p * q * 4 bytes reach 4 GiB
                [(32512, 33024, 64)],          # the array fits below 4 GiB, the array plus a tile of 256 rows does not
                [(32000, 33000, 64)],          # above 2 GiB the sides must be multiples of 256 ...
                [(33024, 32256, 64, 1)],       # ... and the projection on the left
                [(23040, 23300, 64)],          # (23040 + 256) * 23300 * 4 bytes reach 2 GiB and 23300 is ragged
                [(1 << 19, 700, 1100)]):       # a low-rank array p x r of 2 GiB
        with pytest.raises(lordo.LordoError) as e:
            lordo.workspace_bytes(bad, hp)
        assert e.value.code == lordo.EINVAL, bad
    for good in ([(32256, 33024, 64)],         # 3.97 GiB, aligned
                 [(22900, 23100, 64)],         # 1.97 GiB, ragged
                 [(23100, 22900, 64, 1)],
                 [(1 << 19, 700, 1000)]):
        assert lordo.workspace_bytes(good, hp) > 0, good
    with_ef = lordo.workspace_bytes(shapes, lordo.hparams(error_feedback=True))
    assert with_ef - c2 >= sum(4 * p * q for p, q, r in shapes)          # the residual E
    assert lordo.workspace_bytes(shapes, lordo.hparams(qhm_mode=2, omega=0.9)) > c2   # column sums
    assert lordo.workspace_bytes(shapes, lordo.hparams(uplink_buffer=True)) - c2 >= sum(4 * r * q for p, q, r in shapes)
    assert lordo.workspace_bytes(shapes, lordo.hparams(rayleigh_ritz=True)) - c2 >= sum(4 * r for p, q, r in shapes)   # Ritz values
    with pytest.raises(lordo.LordoError) as e:                   # the solver of the Rayleigh-Ritz step takes ranks up to 1024
        lordo.workspace_bytes([(2048, 2048, 1025)], lordo.hparams(rayleigh_ritz=True))
    assert e.value.code == lordo.EINVAL
    for bad_hp in (lordo.hparams(qhm_mode=3), lordo.hparams(qhm_mode=2, omega=0.9, uplink_buffer=True), lordo.hparams(qhm_mode=1, omega=1.5), lordo.hparams(beta1=1.0),
                   lordo.hparams(power_iters=9), lordo.hparams(orth_passes=5), lordo.hparams(grad_dtype=7)):
        with pytest.raises(lordo.LordoError) as e:
            lordo.workspace_bytes([(8, 8, 4)], bad_hp)
        assert e.value.code == lordo.EINVAL


def test_right_projection_validation(lib):
    hp = lordo.hparams()
    tall = lordo.workspace_bytes([(3072, 768, 128, 1)], hp)       # projection on the short side: Q 768 x 128, moments 128 x 3072
    assert 0 < tall
    with pytest.raises(lordo.LordoError) as e:                     # rank is bounded by the projected side: the columns
        lordo.workspace_bytes([(64, 32, 33, 1)], hp)
    assert e.value.code == lordo.EINVAL
    assert lordo.workspace_bytes([(32, 64, 33, 1)], hp) > 0        # ... and not by the rows
    with pytest.raises(lordo.LordoError):
        lordo.workspace_bytes([(64, 32, 8, 2)], hp)
    # every update case, error feedback and the up-link buffer (the last not with full-rank QHM, as on the left)
    assert lordo.workspace_bytes([(64, 32, 8, 1)], lordo.hparams(qhm_mode=1, omega=0.9)) > 0
    assert lordo.workspace_bytes([(64, 32, 8, 1)], lordo.hparams(uplink_buffer=True)) > 0
    assert lordo.workspace_bytes([(64, 32, 8, 1)], lordo.hparams(error_feedback=True)) > 0
    assert lordo.workspace_bytes([(64, 32, 8, 1)], lordo.hparams(qhm_mode=2, omega=0.9)) > 0
    assert lordo.workspace_bytes([(64, 32, 8, 1)], lordo.hparams(qhm_mode=2, omega=0.9, error_feedback=True)) > 0
    with pytest.raises(lordo.LordoError) as e:
        lordo.workspace_bytes([(64, 32, 8, 1)], lordo.hparams(qhm_mode=2, omega=0.9, uplink_buffer=True))
    assert e.value.code == lordo.EINVAL


def test_strerror_and_null_handling(lib):
    assert lib.lordo_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert len(lib.lordo_strerror(code)) > 3
    lib.lordo_destroy(None)
    assert lib.lordo_local_step(None, None, None, 1e-3, 1.0, None) == lordo.EINVAL
    assert lib.lordo_outer_step(None, None, None, None) == lordo.EINVAL
    assert lib.lordo_poll_status(None, None) == lordo.EINVAL
    assert lib.lordo_refresh_subspace(None, None, lordo.BF16, None, None) == lordo.EINVAL
    assert lib.lordo_refresh_subspace_local(None, None, 1.0, None, None) == lordo.EINVAL
    assert lib.lordo_init_projection(None, None, None) == lordo.EINVAL
    assert lib.lordo_export_uplink(None, None, None) == lordo.EINVAL
    assert lib.lordo_outer_step_lowrank(None, None, None, None) == lordo.EINVAL
    assert lib.lordo_sync_payload(None, None, None, None) == lordo.EINVAL
    assert lib.lordo_get_mssv(None, None, None) == lordo.EINVAL
    assert lib.lordo_get_stable_rank(None, None, None) == lordo.EINVAL
    assert lib.lordo_spectral_gap(None, None, lordo.BF16, None, None, None) == lordo.EINVAL
    assert lib.lordo_get_state(None, 0, 0, None, None) == lordo.EINVAL


def test_init_without_gpu_fails_loudly(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    shapes = (lordo.Shape * 1)(lordo.Shape(8, 8, 4, 0))
    hp = lordo.hparams()
    ctx = C.c_void_p()
    w = (C.c_void_p * 1)(0x1000)
    rc = lib.lordo_init(C.byref(ctx), shapes, 1, C.byref(hp), C.c_void_p(0x100000), 1 << 30, w, None)
    assert rc == lordo.EHIP and not ctx.value
