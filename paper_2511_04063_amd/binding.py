"""ctypes binding of libdartqr.so: argument marshalling only.

Every method of :class:`Context` has the name of the C entry point it calls (see
``include/dartqr.h``) and passes raw device pointers of torch tensors plus the current HIP
stream.  Nothing is computed here; if the HIP library is missing this module raises.
"""

from __future__ import annotations

import ctypes
import os

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libdartqr.so")

DQ_OK = 0
DQ_ERR_NULL, DQ_ERR_SHAPE, DQ_ERR_DTYPE, DQ_ERR_ALIGN, DQ_ERR_WORKSPACE, DQ_ERR_HIP, DQ_ERR_UNSUPPORTED = range(1, 8)
DQ_F32, DQ_BF16 = 0, 1
DQ_REDUCE_TOKEN_MEAN, DQ_REDUCE_SUM = 0, 1
DQ_OBJ_WHIP, DQ_OBJ_VARIANCE, DQ_OBJ_KURTOSIS, DQ_OBJ_QUANT = 0, 1, 2, 3
DQ_FLAG_SINGULAR, DQ_FLAG_NONFINITE, DQ_FLAG_ILLCOND_PANEL, DQ_FLAG_BAD_INDEX, DQ_FLAG_SYNC_TIMEOUT = 1, 2, 4, 8, 16
DQ_K_GEMM_F32, DQ_K_GEMM_BF16, DQ_K_WHIP, DQ_K_PANEL, DQ_K_SMALL, DQ_K_COUNT = range(6)
DQ_OPT_ACCUM_PANELS, DQ_OPT_TALL_PANEL_MIN_ROWS, DQ_OPT_SINGLE_STREAM, DQ_OPT_FUSED_WHIP, DQ_OPT_HEADS_BATCHED, DQ_OPT_DEVICE_SYNC, DQ_OPT_SPLIT_GEMM, DQ_OPT_FUSED_PANEL, DQ_OPT_TWO_LEVEL_ROWS = range(9)
DQ_MAX_N = 8192

_c = ctypes
_vp, _i, _l, _f, _sz = _c.c_void_p, _c.c_int, _c.c_long, _c.c_float, _c.c_size_t

# name -> (restype, argtypes); mirrors include/dartqr.h
SIGNATURES = {
    "dq_create": (_i, [_c.POINTER(_vp), _vp]),
    "dq_destroy": (_i, [_vp]),
    "dq_workspace_bytes": (_i, [_i, _i, _i, _i, _c.POINTER(_sz)]),
    "dq_set_workspace": (_i, [_vp, _vp, _sz]),
    "dq_status_string": (_c.c_char_p, [_i]),
    "dq_device_flags": (_i, [_vp, _c.POINTER(_c.c_uint)]),
    "dq_set_option": (_i, [_vp, _i, _i]),
    "dq_stream_handover_probe": (_i, [_vp, _vp, _vp, _c.POINTER(_i)]),
    "dq_qr_orth": (_i, [_vp, _i, _i, _vp, _l, _vp, _l, _vp, _l]),
    "dq_rotate_loss_grad": (_i, [_vp, _i, _i, _i, _vp, _i, _l, _vp, _l, _i, _vp, _vp, _l, _vp, _l, _vp, _l]),
    "dq_calib_step": (_i, [_vp, _i, _i, _i, _vp, _i, _l, _vp, _l, _f, _i, _vp, _vp, _l]),
    "dq_whip_loss_grad": (_i, [_vp, _i, _i, _i, _vp, _l, _i, _vp, _vp, _i, _l]),
    "dq_whip_loss_grad_noalloc": (_i, [_vp, _i, _i, _i, _vp, _l, _i, _vp, _vp, _i, _l]),
    "dq_qr_backward": (_i, [_vp, _i, _i, _vp, _l, _vp, _l, _vp, _l, _vp, _l]),
    "dq_sgd_update": (_i, [_vp, _i, _i, _vp, _l, _vp, _l, _f]),
    "dq_hadamard_init": (_i, [_vp, _i, _i, _vp, _vp, _l]),
    "dq_objective_loss_grad": (_i, [_vp, _i, _i, _i, _i, _i, _vp, _l, _i, _vp, _vp, _i, _l]),
    "dq_set_objective": (_i, [_vp, _i, _i]),
    "dq_calib_run_host_batches": (_i, [_vp, _i, _i, _vp, _i, _i, _l, _vp, _vp, _l, _f, _i, _i, _vp]),
    "dq_outlier_count": (_i, [_vp, _i, _i, _i, _vp, _l, _f, _vp]),
    "dq_gather_rows": (_i, [_vp, _i, _i, _i, _i, _vp, _i, _l, _vp, _vp, _l]),
    "dq_adam_update": (_i, [_vp, _i, _i, _vp, _l, _vp, _l, _vp, _l, _vp, _l, _i, _f, _f, _f, _f]),
    "dq_sgd_momentum_update": (_i, [_vp, _i, _i, _vp, _l, _vp, _l, _vp, _l, _f, _f]),
    "dq_calib_step_adam": (_i, [_vp, _i, _i, _i, _vp, _i, _l, _vp, _l, _vp, _l, _vp, _l, _i, _f, _f, _f, _f, _i, _vp,
                                _vp, _l]),
    "dq_cayley_update": (_i, [_vp, _i, _i, _vp, _l, _vp, _l, _vp, _l, _f, _f, _f, _i, _f, _vp]),
    "dq_cayley_step": (_i, [_vp, _i, _i, _i, _vp, _i, _l, _vp, _l, _vp, _l, _f, _f, _f, _i, _f, _i, _vp]),
    "dq_gemm_f32": (_i, [_vp, _i, _i, _i, _f, _vp, _l, _i, _vp, _l, _i, _f, _vp, _l]),
    "dq_gemm_bf16": (_i, [_vp, _i, _i, _i, _vp, _l, _i, _vp, _l, _i, _vp, _l]),
    "dq_profile_enable": (_i, [_vp, _c.c_uint]),
    "dq_profile_read": (_i, [_vp, _i, _c.POINTER(_c.c_double), _c.POINTER(_l), _c.POINTER(_c.c_double),
                             _c.POINTER(_c.c_double)]),
}

_lib = None


class DartQRError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = status_string(status) if _lib is not None else str(status)
        super().__init__(f"{where}: {msg} (status {status})")


def load_library(path: str | None = None):
    """Load libdartqr.so and set the prototypes.  Raises if it has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    # PyTorch first: it ships its own HIP runtime, and a process must not end up with two of them (the library would
    # otherwise pull in the system-wide runtime when it is loaded before torch, and that copy then sees no device)
    import torch  # noqa: F401
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError(
            f"{p} is missing: build it first with `python -m paper_2511_04063_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(p)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)          # AttributeError if the symbol is not exported
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().dq_status_string(int(status)).decode()


def workspace_bytes(b: int, n: int, T: int, x_dtype: int) -> int:
    out = _sz(0)
    st = load_library().dq_workspace_bytes(b, n, T, x_dtype, ctypes.byref(out))
    if st != DQ_OK:
        raise DartQRError(st, "dq_workspace_bytes")
    return int(out.value)


def _ptr(t):
    return 0 if t is None else int(t.data_ptr())


def dq_whip_loss_grad_noalloc(stream, Y, reduce, loss, dY, dy_dtype):
    """The entry point that allocates nothing: no context, the raw stream handle (or None) first."""
    b = Y.shape[0] if Y.dim() == 3 else 1
    T, n = Y.shape[-2], Y.shape[-1]
    handle = 0 if stream is None else int(stream.cuda_stream)
    st = load_library().dq_whip_loss_grad_noalloc(_vp(handle), b, T, n, _ptr(Y), _ld(Y), reduce, _ptr(loss), _ptr(dY),
                                                  dy_dtype, _ld(dY))
    if st != DQ_OK:
        raise DartQRError(st, "dq_whip_loss_grad_noalloc")


def _ld(t):
    """Leading dimension (elements) of the last two dims of a row-major tensor."""
    if t is None:
        return 0
    assert t.stride(-1) == 1, "matrices must be row-major with unit column stride"
    return int(t.stride(-2))


class Context:
    """One dq_ctx bound to the current torch HIP stream (or the one given)."""

    def __init__(self, stream=None):
        import torch
        self._torch = torch
        self.lib = load_library()
        if stream is None:
            stream = torch.cuda.current_stream()
        self.stream = stream
        h = _vp(0)
        st = self.lib.dq_create(ctypes.byref(h), _vp(stream.cuda_stream))
        if st != DQ_OK:
            raise DartQRError(st, "dq_create")
        self.h = h
        self._ws = None

    def close(self):
        if getattr(self, "h", None) is not None:
            self.lib.dq_destroy(self.h)
            self.h = None

    def __del__(self):  # pragma: no cover
        try:
            self.close()
        except Exception:
            pass

    # ---- workspace (device memory comes from torch)
    def dq_set_workspace(self, tensor):
        st = self.lib.dq_set_workspace(self.h, _vp(_ptr(tensor)), tensor.numel() * tensor.element_size())
        if st != DQ_OK:
            raise DartQRError(st, "dq_set_workspace")
        self._ws = tensor

    def ensure_workspace(self, b, n, T, x_dtype):
        need = workspace_bytes(b, n, T, x_dtype)
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            ws = self._torch.empty(need, dtype=self._torch.uint8, device="cuda")
            self.dq_set_workspace(ws)
        return need

    def _check(self, st, where):
        if st != DQ_OK:
            raise DartQRError(st, where)

    def dq_set_option(self, option, value):
        self._check(self.lib.dq_set_option(self.h, option, value), "dq_set_option")

    def dq_stream_handover_probe(self, consumer_stream, producer_stream) -> bool:
        """Streams are raw hipStream_t handles (ints; 0 = the default stream)."""
        out = ctypes.c_int(-1)
        self._check(self.lib.dq_stream_handover_probe(self.h, ctypes.c_void_p(consumer_stream),
                                                      ctypes.c_void_p(producer_stream), ctypes.byref(out)),
                    "dq_stream_handover_probe")
        return bool(out.value)

    def dq_device_flags(self) -> int:
        out = ctypes.c_uint(0)
        self._check(self.lib.dq_device_flags(self.h, ctypes.byref(out)), "dq_device_flags")
        return int(out.value)

    # ---- hot path
    def dq_qr_orth(self, Z, R, U=None):
        b, n = (Z.shape[0], Z.shape[-1]) if Z.dim() == 3 else (1, Z.shape[-1])
        self._check(self.lib.dq_qr_orth(self.h, b, n, _ptr(Z), _ld(Z), _ptr(R), _ld(R), _ptr(U), _ld(U)),
                    "dq_qr_orth")

    def dq_rotate_loss_grad(self, X, x_dtype, R, reduce, loss, G, Y=None, dY=None):
        b = X.shape[0] if X.dim() == 3 else 1
        T, n = X.shape[-2], X.shape[-1]
        self._check(self.lib.dq_rotate_loss_grad(self.h, b, T, n, _ptr(X), x_dtype, _ld(X), _ptr(R), _ld(R), reduce,
                                                 _ptr(loss), _ptr(G), _ld(G), _ptr(Y), _ld(Y), _ptr(dY), _ld(dY)),
                    "dq_rotate_loss_grad")

    def dq_calib_step(self, X, x_dtype, Z, lr, reduce, loss, R=None):
        b = X.shape[0] if X.dim() == 3 else 1
        T, n = X.shape[-2], X.shape[-1]
        self._check(self.lib.dq_calib_step(self.h, b, T, n, _ptr(X), x_dtype, _ld(X), _ptr(Z), _ld(Z), float(lr),
                                           reduce, _ptr(loss), _ptr(R), _ld(R)), "dq_calib_step")

    def dq_calib_run_host_batches(self, X_host_batches, x_dtype, staging, Z, lr, reduce, steps, losses):
        """X_host_batches: list of host tensors (T x n, ideally pinned); staging: device tensor (2, T, n)."""
        T, n = X_host_batches[0].shape
        for x in X_host_batches:
            assert not x.is_cuda and tuple(x.shape) == (T, n) and _ld(x) == _ld(X_host_batches[0])
        ptrs = (_c.c_void_p * len(X_host_batches))(*[int(x.data_ptr()) for x in X_host_batches])
        assert staging.is_cuda and staging.numel() >= 2 * T * _ld(X_host_batches[0])
        self._check(self.lib.dq_calib_run_host_batches(self.h, T, n, ptrs, len(X_host_batches), x_dtype,
                                                       _ld(X_host_batches[0]), _ptr(staging), _ptr(Z), _ld(Z),
                                                       float(lr), reduce, int(steps), _ptr(losses)),
                    "dq_calib_run_host_batches")

    # ---- stages
    def dq_whip_loss_grad(self, Y, reduce, loss, dY, dy_dtype):
        b = Y.shape[0] if Y.dim() == 3 else 1
        T, n = Y.shape[-2], Y.shape[-1]
        self._check(self.lib.dq_whip_loss_grad(self.h, b, T, n, _ptr(Y), _ld(Y), reduce, _ptr(loss), _ptr(dY),
                                               dy_dtype, _ld(dY)), "dq_whip_loss_grad")

    def dq_objective_loss_grad(self, objective, quant_bits, Y, reduce, loss, dY, dy_dtype):
        b = Y.shape[0] if Y.dim() == 3 else 1
        T, n = Y.shape[-2], Y.shape[-1]
        self._check(self.lib.dq_objective_loss_grad(self.h, objective, quant_bits, b, T, n, _ptr(Y), _ld(Y), reduce,
                                                    _ptr(loss), _ptr(dY), dy_dtype, _ld(dY)), "dq_objective_loss_grad")

    def dq_set_objective(self, objective, quant_bits=4):
        self._check(self.lib.dq_set_objective(self.h, objective, quant_bits), "dq_set_objective")

    def dq_qr_backward(self, R, U, G, dZ):
        b, n = (R.shape[0], R.shape[-1]) if R.dim() == 3 else (1, R.shape[-1])
        self._check(self.lib.dq_qr_backward(self.h, b, n, _ptr(R), _ld(R), _ptr(U), _ld(U), _ptr(G), _ld(G),
                                            _ptr(dZ), _ld(dZ)), "dq_qr_backward")

    def dq_adam_update(self, Z, dZ, m, v, step, lr, beta1=0.9, beta2=0.999, eps=1e-8):
        b, n = (Z.shape[0], Z.shape[-1]) if Z.dim() == 3 else (1, Z.shape[-1])
        self._check(self.lib.dq_adam_update(self.h, b, n, _ptr(Z), _ld(Z), _ptr(dZ), _ld(dZ), _ptr(m), _ld(m), _ptr(v),
                                            _ld(v), int(step), float(lr), float(beta1), float(beta2), float(eps)),
                    "dq_adam_update")

    def dq_sgd_momentum_update(self, Z, dZ, buf, lr, mu):
        b, n = (Z.shape[0], Z.shape[-1]) if Z.dim() == 3 else (1, Z.shape[-1])
        self._check(self.lib.dq_sgd_momentum_update(self.h, b, n, _ptr(Z), _ld(Z), _ptr(dZ), _ld(dZ), _ptr(buf),
                                                    _ld(buf), float(lr), float(mu)), "dq_sgd_momentum_update")

    def dq_calib_step_adam(self, X, x_dtype, Z, m, v, step, lr, reduce, loss, beta1=0.9, beta2=0.999, eps=1e-8,
                           R=None):
        b = X.shape[0] if X.dim() == 3 else 1
        T, n = X.shape[-2], X.shape[-1]
        self._check(self.lib.dq_calib_step_adam(self.h, b, T, n, _ptr(X), x_dtype, _ld(X), _ptr(Z), _ld(Z), _ptr(m),
                                                _ld(m), _ptr(v), _ld(v), int(step), float(lr), float(beta1),
                                                float(beta2), float(eps), reduce, _ptr(loss), _ptr(R), _ld(R)),
                    "dq_calib_step_adam")

    def dq_hadamard_init(self, signs, Z):
        b, n = (Z.shape[0], Z.shape[-1]) if Z.dim() == 3 else (1, Z.shape[-1])
        self._check(self.lib.dq_hadamard_init(self.h, b, n, _ptr(signs), _ptr(Z), _ld(Z)), "dq_hadamard_init")

    def dq_outlier_count(self, Y, tau, counts):
        b = Y.shape[0] if Y.dim() == 3 else 1
        T, n = Y.shape[-2], Y.shape[-1]
        self._check(self.lib.dq_outlier_count(self.h, b, T, n, _ptr(Y), _ld(Y), float(tau), _ptr(counts)),
                    "dq_outlier_count")

    def dq_gather_rows(self, X_all, dtype, idx, X_out):
        b = X_all.shape[0] if X_all.dim() == 3 else 1
        T_all, n = X_all.shape[-2], X_all.shape[-1]
        T_out = X_out.shape[-2]
        self._check(self.lib.dq_gather_rows(self.h, b, T_all, T_out, n, _ptr(X_all), dtype, _ld(X_all), _ptr(idx),
                                            _ptr(X_out), _ld(X_out)), "dq_gather_rows")

    def dq_sgd_update(self, Z, dZ, lr):
        b, n = (Z.shape[0], Z.shape[-1]) if Z.dim() == 3 else (1, Z.shape[-1])
        self._check(self.lib.dq_sgd_update(self.h, b, n, _ptr(Z), _ld(Z), _ptr(dZ), _ld(dZ), float(lr)),
                    "dq_sgd_update")

    def dq_cayley_update(self, R, G, M, lr, beta=0.9, q=0.5, iters=2, eps=1e-8, alpha=None):
        b, n = (R.shape[0], R.shape[-1]) if R.dim() == 3 else (1, R.shape[-1])
        self._check(self.lib.dq_cayley_update(self.h, b, n, _ptr(R), _ld(R), _ptr(G), _ld(G), _ptr(M), _ld(M), lr, beta, q,
                                              iters, eps, _ptr(alpha)), "dq_cayley_update")

    def dq_cayley_step(self, X, x_dtype, R, M, lr, reduce, loss, beta=0.9, q=0.5, iters=2, eps=1e-8):
        b = X.shape[0] if X.dim() == 3 else 1
        T, n = X.shape[-2], X.shape[-1]
        self._check(self.lib.dq_cayley_step(self.h, b, T, n, _ptr(X), x_dtype, _ld(X), _ptr(R), _ld(R), _ptr(M), _ld(M),
                                            lr, beta, q, iters, eps, reduce, _ptr(loss)), "dq_cayley_step")

    def dq_gemm_f32(self, M, N, K, alpha, A, ta, B, tb, beta, C):
        self._check(self.lib.dq_gemm_f32(self.h, M, N, K, float(alpha), _ptr(A), _ld(A), int(ta), _ptr(B), _ld(B),
                                         int(tb), float(beta), _ptr(C), _ld(C)), "dq_gemm_f32")

    def dq_gemm_bf16(self, M, N, K, A, ta, B, tb, C):
        self._check(self.lib.dq_gemm_bf16(self.h, M, N, K, _ptr(A), _ld(A), int(ta), _ptr(B), _ld(B), int(tb),
                                          _ptr(C), _ld(C)), "dq_gemm_bf16")

    # ---- measurement
    def dq_profile_enable(self, mask: int):
        self._check(self.lib.dq_profile_enable(self.h, mask), "dq_profile_enable")

    def dq_profile_read(self, klass: int):
        ms, cnt, fl, by = _c.c_double(0), _l(0), _c.c_double(0), _c.c_double(0)
        self._check(self.lib.dq_profile_read(self.h, klass, ctypes.byref(ms), ctypes.byref(cnt), ctypes.byref(fl),
                                             ctypes.byref(by)), "dq_profile_read")
        return {"ms": ms.value, "launches": int(cnt.value), "flops": fl.value, "bytes": by.value}
