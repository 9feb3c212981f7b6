"""ctypes binding of libsignmuon.so: argument marshalling only.

Each function has the name of the C entry point it calls (see
include/signmuon.h); tensors are torch CUDA tensors used as device buffers,
and the context is bound to torch's current HIP stream.  There is no CPU or
PyTorch fallback: if the library is missing, import of this module fails.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsignmuon.so")

# constants of signmuon.h
SM_OK, SM_EINVAL, SM_EUNSUPPORTED, SM_ENOMEM, SM_EHIP = 0, -1, -2, -3, -4
SM_F32, SM_BF16 = 0, 1
SM_SCALE_FRO, SM_SCALE_SPECTRAL, SM_SCALE_NONE = 0, 1, 2
SM_SIGN_1BIT, SM_SIGN_INT8 = 0, 1
SM_VOTE_BITS, SM_VOTE_INT8, SM_VOTE_BF16, SM_VOTE_F32 = 0, 1, 2, 3
(SM_K_MOMENTUM, SM_K_NS_GRAM, SM_K_NS_APPLY, SM_K_SIGN_PACK, SM_K_VOTE,
 SM_K_UPDATE, SM_K_OTHER, SM_K_NS_SMALL, SM_K_POWER_ITER, SM_K_COUNT) = range(10)

SCALES = {"fro": SM_SCALE_FRO, "spectral": SM_SCALE_SPECTRAL, "none": SM_SCALE_NONE}
SIGN_FMTS = {"1bit": SM_SIGN_1BIT, "int8": SM_SIGN_INT8}
VOTE_FMTS = {"bits": SM_VOTE_BITS, "int8": SM_VOTE_INT8, "bf16": SM_VOTE_BF16, "f32": SM_VOTE_F32}

SM_OPT_GEMM_TILE, SM_OPT_NS_PATH, SM_OPT_NS_STORE, SM_OPT_POWER_ITER = 0, 1, 2, 3
POWER_ITERS = {"auto": 0, "fused": 1, "separate": 2}
NS_PATHS = {"pairs": 0, "single": 1, "stepwise": 2}
NS_STORES = {"upper": 0, "full": 1}
SM_NOALLOC_SCRATCH_BYTES = 4 << 20

EXPORTS = [
    "signmuon_create", "signmuon_destroy", "signmuon_set_option", "signmuon_get_option",
    "signmuon_strerror", "signmuon_last_error",
    "signmuon_workspace_bytes", "signmuon_momentum", "signmuon_momentum_noalloc", "signmuon_polar_ns",
    "signmuon_sign_pack",
    "signmuon_majority_vote", "signmuon_step", "signmuon_profile_enable", "signmuon_profile_reset",
    "signmuon_profile_read", "signmuon_profile_work", "signmuon_kernel_name",
]


class StepArgs(C.Structure):
    _fields_ = [
        ("n_mats", C.c_int32), ("M", C.c_int32),
        ("rows", C.POINTER(C.c_int32)), ("cols", C.POINTER(C.c_int32)),
        ("w", C.POINTER(C.c_void_p)), ("mom", C.POINTER(C.c_void_p)), ("grad", C.POINTER(C.c_void_p)),
        ("beta", C.c_float), ("weight_decay", C.c_float), ("lr", C.c_float), ("eps", C.c_float),
        ("coeffs", C.c_float * 3),
        ("ns_steps", C.c_int32), ("scale", C.c_int32), ("power_iters", C.c_int32),
        ("v0", C.POINTER(C.c_void_p)),
        ("sign_fmt", C.c_int32), ("local_polar_steps", C.c_int32),
        ("update_rsqrt_mn", C.c_int32), ("reserved", C.c_int32),
        ("signs_out", C.POINTER(C.c_void_p)), ("counts_out", C.POINTER(C.c_void_p)),
        ("u_out", C.POINTER(C.c_void_p)), ("d_out", C.POINTER(C.c_void_p)),
    ]


def load_library(path: str = LIB_PATH) -> C.CDLL:
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(path)
    vp, i32, i64, f32 = C.c_void_p, C.c_int, C.c_int64, C.c_float
    lib.signmuon_create.argtypes = [C.POINTER(vp), vp, C.c_size_t]
    lib.signmuon_destroy.argtypes = [vp]
    lib.signmuon_set_option.argtypes = [vp, i32, i32]
    lib.signmuon_get_option.argtypes = [vp, i32, C.POINTER(i32)]
    lib.signmuon_strerror.argtypes = [i32]
    lib.signmuon_strerror.restype = C.c_char_p
    lib.signmuon_last_error.argtypes = [vp]
    lib.signmuon_last_error.restype = C.c_char_p
    lib.signmuon_workspace_bytes.argtypes = [vp]
    lib.signmuon_workspace_bytes.restype = C.c_size_t
    lib.signmuon_momentum.argtypes = [vp, vp, vp, vp, i32, i32, i32, f32, f32, vp, vp]
    lib.signmuon_momentum_noalloc.argtypes = [vp, vp, vp, vp, i32, i32, i32, f32, f32, vp, vp]
    lib.signmuon_polar_ns.argtypes = [vp, vp, i32, i32, i32, i32, C.POINTER(f32), i32, i32, i32, f32, vp]
    lib.signmuon_sign_pack.argtypes = [vp, vp, i32, i32, i64, i32, vp, i64]
    lib.signmuon_majority_vote.argtypes = [vp, vp, i32, i32, i64, i64, vp, i32, vp, vp, f32]
    lib.signmuon_step.argtypes = [vp, C.POINTER(StepArgs)]
    lib.signmuon_profile_enable.argtypes = [vp, C.c_uint]
    lib.signmuon_profile_reset.argtypes = [vp]
    lib.signmuon_profile_read.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(C.c_double)]
    lib.signmuon_profile_work.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                          C.POINTER(C.c_double)]
    lib.signmuon_kernel_name.argtypes = [i32]
    lib.signmuon_kernel_name.restype = C.c_char_p
    return lib


_lib = load_library()


class SignMuonError(RuntimeError):
    pass


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return C.c_void_p(t.data_ptr())


def _dtype_code(t):
    if t.dtype == torch.float32:
        return SM_F32
    if t.dtype == torch.bfloat16:
        return SM_BF16
    raise ValueError(f"unsupported dtype {t.dtype}")


class Context:
    """signmuon_ctx bound to torch's current stream on the current device."""

    def __init__(self, stream: "torch.cuda.Stream | None" = None, workspace_bytes_hint: int = 0, *,
                 gemm_tile: int = 0, ns_path: str = "pairs", ns_store: str = "upper", power_iter: str = "auto"):
        if not torch.cuda.is_available():
            raise SignMuonError("no HIP device: libsignmuon has no CPU path")
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        rc = _lib.signmuon_create(C.byref(h), C.c_void_p(self.stream.cuda_stream), int(workspace_bytes_hint))
        if rc != SM_OK:
            raise SignMuonError(f"signmuon_create: {_lib.signmuon_strerror(rc).decode()}")
        self._h = h
        self.set_option(SM_OPT_GEMM_TILE, gemm_tile)
        self.set_option(SM_OPT_NS_PATH, NS_PATHS[ns_path])
        self.set_option(SM_OPT_NS_STORE, NS_STORES[ns_store])
        self.set_option(SM_OPT_POWER_ITER, POWER_ITERS[power_iter])

    def set_option(self, option: int, value: int):
        self._check(_lib.signmuon_set_option(self._h, int(option), int(value)), "signmuon_set_option")

    def get_option(self, option: int) -> int:
        v = C.c_int()
        self._check(_lib.signmuon_get_option(self._h, int(option), C.byref(v)), "signmuon_get_option")
        return v.value

    def close(self):
        if getattr(self, "_h", None):
            _lib.signmuon_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc, what):
        if rc != SM_OK:
            msg = _lib.signmuon_last_error(self._h).decode()
            raise SignMuonError(f"{what}: {_lib.signmuon_strerror(rc).decode()} ({rc}): {msg}")

    @property
    def workspace_bytes(self):
        return _lib.signmuon_workspace_bytes(self._h)

    # -- timing taps
    def profile_enable(self, class_mask=(1 << SM_K_COUNT) - 1):
        self._check(_lib.signmuon_profile_enable(self._h, int(class_mask)), "profile_enable")

    def profile_reset(self):
        self._check(_lib.signmuon_profile_reset(self._h), "profile_reset")

    def profile_read(self, kernel_class):
        n, ms = C.c_int64(), C.c_double()
        self._check(_lib.signmuon_profile_read(self._h, kernel_class, C.byref(n), C.byref(ms)), "profile_read")
        return n.value, ms.value

    def profile_work(self, kernel_class):
        """(executed flop, dense flop, bytes) booked by the timed launches of a GEMM class."""
        fl, fd, by = C.c_double(), C.c_double(), C.c_double()
        self._check(_lib.signmuon_profile_work(self._h, kernel_class, C.byref(fl), C.byref(fd), C.byref(by)),
                    "profile_work")
        return fl.value, fd.value, by.value


def kernel_name(kernel_class):
    return _lib.signmuon_kernel_name(kernel_class).decode()


def signmuon_momentum(ctx, mom, grad, w, beta, weight_decay=0.0, x_bf16=None, sumsq=None):
    """mom[M,r,c] (in place), grad[M,r,c], w[r,c] or None."""
    M, r, c = grad.shape
    assert mom.shape == grad.shape and mom.dtype == grad.dtype == torch.float32
    ctx._check(_lib.signmuon_momentum(ctx._h, _ptr(mom), _ptr(grad), _ptr(w), M, r, c, beta, weight_decay,
                                      _ptr(x_bf16), _ptr(sumsq)), "signmuon_momentum")


def signmuon_momentum_noalloc(ctx, mom, grad, w, beta, weight_decay=0.0, x_bf16=None, sumsq=None):
    """signmuon_momentum without any device allocation (static scratch inside the library)."""
    M, r, c = grad.shape
    assert mom.shape == grad.shape and mom.dtype == grad.dtype == torch.float32
    ctx._check(_lib.signmuon_momentum_noalloc(ctx._h, _ptr(mom), _ptr(grad), _ptr(w), M, r, c, beta, weight_decay,
                                              _ptr(x_bf16), _ptr(sumsq)), "signmuon_momentum_noalloc")


def signmuon_polar_ns(ctx, x, steps, coeffs=(1.5, -0.5, 0.0), scale="fro", power_iters=2, eps=1e-12, v0=None):
    """In place on x[batch,r,c] (float32 or bfloat16)."""
    batch, r, c = x.shape
    cf = (C.c_float * 3)(*coeffs)
    ctx._check(_lib.signmuon_polar_ns(ctx._h, _ptr(x), _dtype_code(x), batch, r, c, cf, steps, SCALES[scale],
                                      power_iters, eps, _ptr(v0)), "signmuon_polar_ns")


def signmuon_sign_pack(ctx, u, fmt, out, out_stride_bytes=None):
    """u[batch,n] -> out (uint8 tensor [batch, stride])."""
    batch, n = u.shape
    if out_stride_bytes is None:
        out_stride_bytes = out.stride(0) * out.element_size() if out.dim() == 2 else out.numel() * out.element_size()
    ctx._check(_lib.signmuon_sign_pack(ctx._h, _ptr(u), _dtype_code(u), batch, n, SIGN_FMTS[fmt], _ptr(out),
                                       out_stride_bytes), "signmuon_sign_pack")


def signmuon_majority_vote(ctx, signs, fmt, M, n, stride_bytes, voted=None, vfmt="bits", counts=None, w=None,
                           lr_scaled=0.0):
    ctx._check(_lib.signmuon_majority_vote(ctx._h, _ptr(signs), SIGN_FMTS[fmt], M, n, stride_bytes, _ptr(voted),
                                           VOTE_FMTS[vfmt], _ptr(counts), _ptr(w), lr_scaled),
               "signmuon_majority_vote")


class StepPlan:
    """Marshalled signmuon_step_args for a fixed set of tensors (reusable across steps)."""

    def __init__(self, w, mom, grad, *, beta, lr, ns_steps, weight_decay=0.0, eps=1e-12,
                 coeffs=(1.5, -0.5, 0.0), scale="fro", power_iters=2, v0=None, sign_fmt="1bit",
                 local_polar_steps=0, update_rsqrt_mn=False, signs_out=None, counts_out=None,
                 u_out=None, d_out=None):
        n = len(w)
        assert len(mom) == n and len(grad) == n
        self._keep = (w, mom, grad, v0, signs_out, counts_out, u_out, d_out)
        M = grad[0].shape[0]
        a = StepArgs()
        a.n_mats, a.M = n, M
        self._rows = (C.c_int32 * n)(*[t.shape[0] for t in w])
        self._cols = (C.c_int32 * n)(*[t.shape[1] for t in w])
        a.rows, a.cols = self._rows, self._cols

        def ptr_array(ts):
            if ts is None:
                return None
            arr = (C.c_void_p * n)(*[None if t is None else _ptr(t).value for t in ts])
            return arr

        for t_w, t_m, t_g in zip(w, mom, grad):
            assert t_w.dtype == t_m.dtype == t_g.dtype == torch.float32
            assert tuple(t_m.shape) == (M,) + tuple(t_w.shape) == tuple(t_g.shape)
        self._arrs = [ptr_array(x) for x in (w, mom, grad, v0, signs_out, counts_out, u_out, d_out)]
        a.w, a.mom, a.grad, a.v0, a.signs_out, a.counts_out, a.u_out, a.d_out = [
            C.cast(x, C.POINTER(C.c_void_p)) if x is not None else None for x in self._arrs]
        a.beta, a.weight_decay, a.lr, a.eps = beta, weight_decay, lr, eps
        a.coeffs = (C.c_float * 3)(*coeffs)
        a.ns_steps, a.scale, a.power_iters = ns_steps, SCALES[scale], power_iters
        a.sign_fmt, a.local_polar_steps = SIGN_FMTS[sign_fmt], local_polar_steps
        # 0 / False: kappa = 1; 1 / True: 1 / sqrt(rows * cols); 2 or "op_norm": 1 / PowerIter(voted sign)
        a.update_rsqrt_mn, a.reserved = (2 if update_rsqrt_mn == "op_norm" else int(update_rsqrt_mn)), 0
        self.args = a


def signmuon_step(ctx, plan: StepPlan):
    ctx._check(_lib.signmuon_step(ctx._h, C.byref(plan.args)), "signmuon_step")
