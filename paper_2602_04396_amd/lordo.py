"""Thin ctypes binding of liblordo.so (see include/lordo.h for the contract of every call).

Only argument marshalling happens here: torch tensors supply device memory and the
current stream; every step of the path runs in the library's kernels.  There is no
fallback: if the library has not been built, importing `load()` raises.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "lib", "liblordo.so")

OK, EINVAL, ENOMEM, EHIP, ESTATE, ENUMERIC = 0, -1, -2, -3, -4, -5
F32, BF16 = 0, 1
STATE_Q, STATE_U, STATE_V, STATE_ANCHOR, STATE_MOM, STATE_GLOW, STATE_NUPD, STATE_ERR, STATE_UPLINK, STATE_RITZ = range(10)

EXPORTS = [
    "lordo_workspace_bytes", "lordo_init", "lordo_local_step", "lordo_refresh_subspace",
    "lordo_export_pseudograd", "lordo_outer_step", "lordo_get_state", "lordo_set_state",
    "lordo_get_step", "lordo_set_step", "lordo_poll_status", "lordo_strerror", "lordo_destroy",
    "lordo_profile_enable", "lordo_profile_read", "lordo_get_mssv", "lordo_refresh_subspace_local",
    "lordo_export_uplink", "lordo_outer_step_lowrank", "lordo_init_projection", "lordo_sync_payload",
    "lordo_get_stable_rank", "lordo_spectral_gap", "lordo_init_static",
]
STATIC_WORKSPACE_BYTES = 64 << 20
K_DOWN, K_ADAM, K_UP, K_OUTER, K_EXPORT, K_REFRESH = range(6)


class Shape(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("rank", C.c_int32), ("side", C.c_int32)]


class HParams(C.Structure):
    _fields_ = [
        ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
        ("bias_correction", C.c_int32), ("qhm_mode", C.c_int32),
        ("omega", C.c_double),
        ("error_feedback", C.c_int32), ("outer_nesterov", C.c_int32),
        ("outer_lr", C.c_double), ("outer_momentum", C.c_double),
        ("power_iters", C.c_int32), ("orth_passes", C.c_int32),
        ("grad_dtype", C.c_int32), ("uplink_buffer", C.c_int32),
        ("rayleigh_ritz", C.c_int32), ("param_dtype", C.c_int32),
        ("err_dtype", C.c_int32), ("reserved", C.c_int32),
        ("seed", C.c_uint64),
    ]


def hparams(beta1=0.9, beta2=0.999, eps=1e-8, bias_correction=True, outer_lr=1.0, outer_momentum=0.0,
            outer_nesterov=False, power_iters=2, orth_passes=2, grad_dtype=BF16, qhm_mode=0, omega=1.0,
            error_feedback=False, uplink_buffer=False, rayleigh_ritz=False, seed=0, param_dtype=F32, err_dtype=F32) -> HParams:
    return HParams(beta1, beta2, eps, int(bias_correction), qhm_mode, omega, int(error_feedback),
                   int(outer_nesterov), outer_lr, outer_momentum, power_iters, orth_passes, grad_dtype, int(uplink_buffer),
                   int(rayleigh_ritz), int(param_dtype), int(err_dtype), 0, int(seed))


class LordoError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"lordo error {code}: {msg}")
        self.code = code


_lib = None


def load() -> C.CDLL:
    """Load the built library; raise if it is missing (no CPU or eager fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not built: run `python -m paper_2602_04396_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, vpp = C.c_void_p, C.POINTER(C.c_void_p)
    lib.lordo_workspace_bytes.argtypes = [C.POINTER(Shape), C.c_int32, C.POINTER(HParams), C.POINTER(C.c_size_t)]
    lib.lordo_init.argtypes = [C.POINTER(vp), C.POINTER(Shape), C.c_int32, C.POINTER(HParams), vp, C.c_size_t, vpp, vp]
    lib.lordo_init_static.argtypes = [C.POINTER(vp), C.POINTER(Shape), C.c_int32, C.POINTER(HParams), vpp, vp]
    lib.lordo_local_step.argtypes = [vp, vpp, vpp, C.c_double, C.c_double, vp]
    lib.lordo_refresh_subspace.argtypes = [vp, vpp, C.c_int32, vpp, vp]
    lib.lordo_refresh_subspace_local.argtypes = [vp, vpp, C.c_double, vpp, vp]
    lib.lordo_export_pseudograd.argtypes = [vp, vpp, vpp, vp]
    lib.lordo_outer_step.argtypes = [vp, vpp, vpp, vp]
    lib.lordo_init_projection.argtypes = [vp, vpp, vp]
    lib.lordo_export_uplink.argtypes = [vp, vpp, vp]
    lib.lordo_outer_step_lowrank.argtypes = [vp, vpp, vpp, vp]
    lib.lordo_sync_payload.argtypes = [vp, vpp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    lib.lordo_get_state.argtypes = [vp, C.c_int32, C.c_int32, vp, vp]
    lib.lordo_set_state.argtypes = [vp, C.c_int32, C.c_int32, vp, vp]
    lib.lordo_get_mssv.argtypes = [vp, vp, vp]
    lib.lordo_get_stable_rank.argtypes = [vp, vp, vp]
    lib.lordo_spectral_gap.argtypes = [vp, vpp, C.c_int32, vpp, vp, vp]
    lib.lordo_get_step.argtypes = [vp, C.POINTER(C.c_int64)]
    lib.lordo_set_step.argtypes = [vp, C.c_int64]
    lib.lordo_poll_status.argtypes = [vp, vp]
    lib.lordo_profile_enable.argtypes = [vp, C.c_int32]
    lib.lordo_profile_read.argtypes = [vp, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64), vp]
    lib.lordo_strerror.argtypes = [C.c_int]
    lib.lordo_strerror.restype = C.c_char_p
    lib.lordo_destroy.argtypes = [vp]
    lib.lordo_destroy.restype = None
    for name in EXPORTS:
        if name not in ("lordo_strerror", "lordo_destroy"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(code):
    if code != OK:
        raise LordoError(code, load().lordo_strerror(code).decode())


class PtrList:
    """Pointer array of an already validated tensor list, reusable across calls (keeps the
    tensors alive).  Built by Lordo.ptrs(); lets a tight loop skip per-call validation."""

    def __init__(self, tensors, arr):
        self.tensors = tensors
        self.arr = arr


def _ptr_array(tensors):
    if isinstance(tensors, PtrList):
        return tensors.arr
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else t.data_ptr()
    return arr


def _shape_array(shapes):
    arr = (Shape * len(shapes))()
    for i, sh in enumerate(shapes):      # (p, q, r) or (p, q, r, side); side 1 = projection on the right
        arr[i] = Shape(sh[0], sh[1], sh[2], sh[3] if len(sh) > 3 else 0)
    return arr


def workspace_bytes(shapes, hp: HParams) -> int:
    out = C.c_size_t(0)
    _check(load().lordo_workspace_bytes(_shape_array(shapes), len(shapes), C.byref(hp), C.byref(out)))
    return out.value


class Lordo:
    """One optimizer context over a list of (p, q, r) matrices.  `W` and every other
    argument is a list of torch CUDA tensors, contiguous, in the order of `shapes`."""

    def __init__(self, shapes, hp: HParams, W, torch, static_workspace=False):
        self.lib = load()
        self.torch = torch
        self.shapes = [tuple(s) for s in shapes]
        self.hp = hp
        self.n = len(shapes)
        self._check_tensors(W, torch.bfloat16 if hp.param_dtype == BF16 else torch.float32, "pq")
        self.device = W[0].device
        self.ctx = C.c_void_p()
        if static_workspace:         # lordo_init_static: the workspace is the library's own fixed array, nothing is allocated
            self.arena = None
            _check(self.lib.lordo_init_static(C.byref(self.ctx), _shape_array(self.shapes), self.n, C.byref(hp),
                                              _ptr_array(W), self._stream()))
            return
        nbytes = workspace_bytes(self.shapes, hp)
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=W[0].device)
        base = self.arena.data_ptr()
        self.arena_ptr = (base + 255) // 256 * 256
        self.arena_bytes = nbytes
        _check(self.lib.lordo_init(C.byref(self.ctx), _shape_array(self.shapes), self.n, C.byref(hp),
                                   C.c_void_p(self.arena_ptr), nbytes, _ptr_array(W), self._stream()))

    # -- helpers ----------------------------------------------------------------------------
    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream().cuda_stream)

    def ptrs(self, tensors, dtype=None, kind="pq") -> PtrList:
        """Validate a tensor list once and freeze its device pointers for repeated calls."""
        self._check_tensors(tensors, dtype or self.torch.float32, kind)
        return PtrList(list(tensors), _ptr_array(tensors))

    def _check_tensors(self, ts, dtype, kind, allow_none=False):
        if isinstance(ts, PtrList):
            return
        if len(ts) != self.n:
            raise ValueError("one tensor per matrix expected")
        for t, sh in zip(ts, self.shapes):
            if t is None and allow_none:
                continue
            p, q, r = sh[:3]
            # low-rank arrays of a right-projected matrix are those of the transposed problem
            tp, tq = (q, p) if len(sh) > 3 and sh[3] else (p, q)
            want = {"pq": (p, q), "qr": (tq, r), "rq": (r, tq), "pr": (tp, r)}[kind]
            if tuple(t.shape) != want or t.dtype != dtype or not t.is_contiguous() or not t.is_cuda:
                raise ValueError(f"expected contiguous CUDA {dtype} tensor of shape {want}, got {t.dtype} {tuple(t.shape)}")

    def _w_dtype(self):
        return self.torch.bfloat16 if self.hp.param_dtype == BF16 else self.torch.float32

    def _grad_dtype(self):
        return self.torch.bfloat16 if self.hp.grad_dtype == BF16 else self.torch.float32

    # -- the four calls -----------------------------------------------------------------------
    def local_step(self, W, G, lr, grad_scale=1.0):
        self._check_tensors(W, self._w_dtype(), "pq")
        self._check_tensors(G, self._grad_dtype(), "pq")
        _check(self.lib.lordo_local_step(self.ctx, _ptr_array(W), _ptr_array(G), float(lr), float(grad_scale), self._stream()))

    def init_projection(self, block=None):
        """Q_0 = orthonormal basis of the p x r blocks given (Alg. 1: random initial projection); None: blocks
        drawn by the library from hp.seed."""
        if block is None:
            _check(self.lib.lordo_init_projection(self.ctx, None, self._stream()))
            return
        self._check_tensors(block, self.torch.float32, "pr")
        _check(self.lib.lordo_init_projection(self.ctx, _ptr_array(block), self._stream()))

    def refresh_subspace(self, Src, Omega=None):
        """Src: one tensor per matrix (None entries leave that matrix out); Omega None: start blocks from hp.seed."""
        src_list = Src.tensors if isinstance(Src, PtrList) else Src
        live = [t for t in src_list if t is not None]
        if not live:
            return
        dt = live[0].dtype
        if dt not in (self.torch.bfloat16, self.torch.float32):
            raise ValueError("refresh source must be bf16 or fp32")
        self._check_tensors(Src, dt, "pq", allow_none=True)
        if Omega is not None:
            self._check_tensors(Omega, self.torch.float32, "qr", allow_none=True)
        code = BF16 if dt == self.torch.bfloat16 else F32
        _check(self.lib.lordo_refresh_subspace(self.ctx, _ptr_array(Src), code, None if Omega is None else _ptr_array(Omega),
                                               self._stream()))

    def spectral_gap(self, Src, Omega):
        """Per matrix: estimate of sigma_r - sigma_{r+1} of Src (the source of the last refresh; needs rayleigh_ritz)."""
        dt = (Src.tensors if isinstance(Src, PtrList) else Src)[0].dtype
        if dt not in (self.torch.bfloat16, self.torch.float32):
            raise ValueError("source must be bf16 or fp32")
        self._check_tensors(Src, dt, "pq")
        self._check_tensors(Omega, self.torch.float32, "qr")
        out = self.torch.empty(len(self.shapes), dtype=self.torch.float32, device=self.device)
        _check(self.lib.lordo_spectral_gap(self.ctx, _ptr_array(Src), BF16 if dt == self.torch.bfloat16 else F32,
                                           _ptr_array(Omega), C.c_void_p(out.data_ptr()), self._stream()))
        return out

    def refresh_subspace_local(self, G, Omega, grad_scale=1.0):
        """Alg. 2 refresh from grad_scale * G + E; the next call must be local_step with the same G."""
        self._check_tensors(G, self._grad_dtype(), "pq")
        if Omega is not None:
            self._check_tensors(Omega, self.torch.float32, "qr")
        _check(self.lib.lordo_refresh_subspace_local(self.ctx, _ptr_array(G), float(grad_scale),
                                                     None if Omega is None else _ptr_array(Omega), self._stream()))

    def export_pseudograd(self, W, out):
        self._check_tensors(W, self._w_dtype(), "pq")
        self._check_tensors(out, self.torch.float32, "pq")
        _check(self.lib.lordo_export_pseudograd(self.ctx, _ptr_array(W), _ptr_array(out), self._stream()))

    def outer_step(self, W, avg_delta=None):
        self._check_tensors(W, self._w_dtype(), "pq")
        if avg_delta is not None:
            self._check_tensors(avg_delta, self.torch.float32, "pq")
            _check(self.lib.lordo_outer_step(self.ctx, _ptr_array(W), _ptr_array(avg_delta), self._stream()))
        else:
            _check(self.lib.lordo_outer_step(self.ctx, _ptr_array(W), None, self._stream()))

    def export_uplink(self, out):
        """out_i <- the r x q up-link buffer of matrix i (App. A.5.1)."""
        self._check_tensors(out, self.torch.float32, "rq")
        _check(self.lib.lordo_export_uplink(self.ctx, _ptr_array(out), self._stream()))

    def outer_step_lowrank(self, W, avg_acc=None):
        """Outer step with Delta = Q avg_acc (avg_acc: mean of the workers' exported buffers; None: own buffer)."""
        self._check_tensors(W, self._w_dtype(), "pq")
        if avg_acc is not None:
            self._check_tensors(avg_acc, self.torch.float32, "rq")
            _check(self.lib.lordo_outer_step_lowrank(self.ctx, _ptr_array(W), _ptr_array(avg_acc), self._stream()))
        else:
            _check(self.lib.lordo_outer_step_lowrank(self.ctx, _ptr_array(W), None, self._stream()))

    def sync_payload(self):
        """(payload, moments_count): the contiguous fp32 region [u | v | A] of the workspace as a tensor view
        (Alg. 1 synchronisation; App. A.5.1) and the number of leading elements that are moments."""
        if self.arena is None:
            raise ValueError("the payload view needs a torch-owned arena (context created with static_workspace)")
        ptr, count, moments = C.c_void_p(), C.c_size_t(), C.c_size_t()
        _check(self.lib.lordo_sync_payload(self.ctx, C.byref(ptr), C.byref(count), C.byref(moments)))
        off = ptr.value - self.arena.data_ptr()
        assert 0 <= off and off + 4 * count.value <= self.arena.numel()
        return self.arena[off:off + 4 * count.value].view(self.torch.float32), moments.value

    # -- state ------------------------------------------------------------------------------------
    def _state_shape(self, mat, which):
        sh = self.shapes[mat]
        p, q, r = sh[:3]
        tp, tq = (q, p) if len(sh) > 3 and sh[3] else (p, q)
        return {STATE_Q: (tp, r), STATE_ANCHOR: (p, q), STATE_MOM: (p, q), STATE_ERR: (p, q), STATE_RITZ: (r,)}.get(which, (r, tq))

    def get_state(self, mat, which):
        out = self.torch.empty(self._state_shape(mat, which), dtype=self.torch.float32, device=self.device)
        _check(self.lib.lordo_get_state(self.ctx, mat, which, C.c_void_p(out.data_ptr()), self._stream()))
        return out

    def set_state(self, mat, which, src):
        want = self._state_shape(mat, which)
        if tuple(src.shape) != want or src.dtype != self.torch.float32 or not src.is_contiguous() or not src.is_cuda:
            raise ValueError(f"expected contiguous CUDA float32 tensor of shape {want}")
        _check(self.lib.lordo_set_state(self.ctx, mat, which, C.c_void_p(src.data_ptr()), self._stream()))

    def mssv(self):
        """Per matrix: mean squared singular value of Q_new^T Q_old of the last refresh (tensor of n floats)."""
        out = self.torch.empty(len(self.shapes), dtype=self.torch.float32, device=self.device)
        _check(self.lib.lordo_get_mssv(self.ctx, C.c_void_p(out.data_ptr()), self._stream()))
        return out

    def stable_rank(self):
        """Per matrix: ||Src||_F^2 / ||Src||_2^2 of the source of the last refresh (needs rayleigh_ritz)."""
        out = self.torch.empty(len(self.shapes), dtype=self.torch.float32, device=self.device)
        _check(self.lib.lordo_get_stable_rank(self.ctx, C.c_void_p(out.data_ptr()), self._stream()))
        return out

    @property
    def step(self):
        t = C.c_int64(0)
        _check(self.lib.lordo_get_step(self.ctx, C.byref(t)))
        return t.value

    @step.setter
    def step(self, t):
        _check(self.lib.lordo_set_step(self.ctx, int(t)))

    def poll_status(self):
        _check(self.lib.lordo_poll_status(self.ctx, self._stream()))

    def profile_enable(self, on=True):
        _check(self.lib.lordo_profile_enable(self.ctx, int(on)))

    def profile_read(self, kernel_class):
        """(total milliseconds, number of spans) of one kernel class since profiling was enabled."""
        ms, cnt = C.c_double(0), C.c_int64(0)
        _check(self.lib.lordo_profile_read(self.ctx, kernel_class, C.byref(ms), C.byref(cnt), self._stream()))
        return ms.value, cnt.value

    def close(self):
        if self.ctx:
            self.lib.lordo_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
