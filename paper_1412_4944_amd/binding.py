"""ctypes binding of libsbo: same names as the C entry points, argument
marshalling only.  Tensors are torch CUDA tensors used as device memory; torch
does no arithmetic here.  Fails loudly when the HIP library is missing."""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libsbo.so")

SBO_OK, SBO_EINVAL, SBO_ENOMEM, SBO_EHIP, SBO_ELIMIT = 0, -1, -2, -3, -4
SBO_GROUP_STATIC_MAX_K, SBO_GROUP_STATIC_MAX_M = 128, 1 << 20
STAGES = ("energy", "group", "select", "accum", "svd")

EXPORTS = ("sbo_create", "sbo_destroy", "sbo_workspace_bytes", "sbo_code", "sbo_group", "sbo_group_static",
           "sbo_accumulate", "sbo_polar", "sbo_update", "sbo_train_rounds", "sbo_iterate", "sbo_sqerr",
           "sbo_worst", "sbo_init_base", "sbo_new_base", "sbo_set_blocks", "sbo_learn", "sbo_svd_sweeps", "sbo_set_option", "sbo_set_timing", "sbo_stage_ms", "sbo_strerror")

_lib = None


class SboError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libsbo error {code}: {text}")
        self.code = code


def lib() -> ctypes.CDLL:
    """Load libsbo.so (built by paper_1412_4944_amd.build); no fallback exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1412_4944_amd.build` "
                           "(there is no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    L.sbo_create.argtypes = [ctypes.POINTER(vp), i32, i32, i32, i64, vp]
    L.sbo_destroy.argtypes = [vp]
    L.sbo_workspace_bytes.argtypes = [i32, i32, i32, i64]
    L.sbo_workspace_bytes.restype = ctypes.c_size_t
    L.sbo_code.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp]
    L.sbo_group.argtypes = [vp, vp, i64, vp, vp, vp]
    L.sbo_group_static.argtypes = [vp, i64, i32, vp, vp, vp, vp]
    L.sbo_accumulate.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    L.sbo_polar.argtypes = [vp, vp, vp, vp]
    L.sbo_update.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp]
    L.sbo_train_rounds.argtypes = [vp, vp, i64, vp, vp, i32, vp, vp, vp]
    L.sbo_iterate.argtypes = [vp, vp, i64, vp, i32, vp, vp, vp, vp, vp]
    L.sbo_sqerr.argtypes = [vp, vp, i64, vp]
    L.sbo_worst.argtypes = [vp, vp, i64, i64, vp]
    L.sbo_init_base.argtypes = [vp, vp, i64, vp, i64, vp, vp]
    L.sbo_new_base.argtypes = [vp, vp, i64, vp, i64, i32, i32, vp, vp, vp, vp, vp]
    L.sbo_set_blocks.argtypes = [vp, i32]
    L.sbo_learn.argtypes = [vp, vp, i64, vp, vp, i32, i64, i32, i64, i32, ctypes.c_double, vp, vp, vp, vp,
                            ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    L.sbo_svd_sweeps.argtypes = [vp, ctypes.POINTER(ctypes.c_int32)]
    L.sbo_set_option.argtypes = [vp, i32, i32]
    L.sbo_set_timing.argtypes = [vp, i32]
    L.sbo_stage_ms.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
    L.sbo_strerror.argtypes = [i32]
    L.sbo_strerror.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("sbo_workspace_bytes", "sbo_strerror"):
            getattr(L, name).restype = i32
    _lib = L
    return L


def sbo_strerror(code: int) -> str:
    return lib().sbo_strerror(code).decode()


def _check(rc: int) -> None:
    if rc != SBO_OK:
        raise SboError(rc, sbo_strerror(rc))


def _ptr(t, dtype=None, optional=False):
    if t is None:
        if optional:
            return None
        raise ValueError("required tensor is None")
    import torch
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libsbo takes contiguous device tensors")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def sbo_workspace_bytes(p: int, K: int, s0: int, m_max: int) -> int:
    return int(lib().sbo_workspace_bytes(p, K, s0, m_max))


def sbo_create(p: int, K: int, s0: int, m_max: int, stream: int | None = None) -> ctypes.c_void_p:
    """Returns an opaque context handle.  stream: a raw hipStream_t value; default =
    torch's current stream."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    h = ctypes.c_void_p()
    _check(lib().sbo_create(ctypes.byref(h), p, K, s0, m_max, ctypes.c_void_p(stream)))
    return h


def sbo_destroy(ctx) -> None:
    _check(lib().sbo_destroy(ctx))


def sbo_code(ctx, Y, D, blk, supp, coef, err) -> None:
    import torch
    _check(lib().sbo_code(ctx, _ptr(Y, torch.float32), Y.shape[0], _ptr(D, torch.float32),
                          _ptr(blk, torch.int32), _ptr(supp, torch.int32),
                          _ptr(coef, torch.float32), _ptr(err, torch.float32)))


def sbo_group(ctx, blk, counts=None, offsets=None, perm=None) -> None:
    import torch
    _check(lib().sbo_group(ctx, _ptr(blk, torch.int32), blk.shape[0],
                           _ptr(counts, torch.int32, True), _ptr(offsets, torch.int32, True),
                           _ptr(perm, torch.int32, True)))


def sbo_group_static(blk, K: int, counts, offsets, perm, stream: int | None = None) -> None:
    """sbo_group without a context and without any allocation (static device scratch)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().sbo_group_static(_ptr(blk, torch.int32), blk.shape[0], int(K), _ptr(counts, torch.int32),
                                  _ptr(offsets, torch.int32), _ptr(perm, torch.int32),
                                  ctypes.c_void_p(stream)))


def sbo_accumulate(ctx, Y, blk, supp, coef, M) -> None:
    import torch
    _check(lib().sbo_accumulate(ctx, _ptr(Y, torch.float32), Y.shape[0], _ptr(blk, torch.int32),
                                _ptr(supp, torch.int32), _ptr(coef, torch.float32),
                                _ptr(M, torch.float32)))


def sbo_polar(ctx, M, counts, D) -> None:
    import torch
    _check(lib().sbo_polar(ctx, _ptr(M, torch.float32), _ptr(counts, torch.int32, True),
                           _ptr(D, torch.float32)))


def sbo_update(ctx, Y, blk, supp, coef, D, counts=None) -> None:
    import torch
    _check(lib().sbo_update(ctx, _ptr(Y, torch.float32), Y.shape[0], _ptr(blk, torch.int32),
                            _ptr(supp, torch.int32), _ptr(coef, torch.float32),
                            _ptr(D, torch.float32), _ptr(counts, torch.int32, True)))


def sbo_train_rounds(ctx, Y, blk, D, R, supp, coef, err) -> None:
    import torch
    _check(lib().sbo_train_rounds(ctx, _ptr(Y, torch.float32), Y.shape[0], _ptr(blk, torch.int32),
                                  _ptr(D, torch.float32), int(R), _ptr(supp, torch.int32),
                                  _ptr(coef, torch.float32), _ptr(err, torch.float32)))


def sbo_iterate(ctx, Y, D, n_iter, blk, supp, coef, err, sqerr_per_iter=None) -> None:
    import torch
    _check(lib().sbo_iterate(ctx, _ptr(Y, torch.float32), Y.shape[0], _ptr(D, torch.float32),
                             int(n_iter), _ptr(blk, torch.int32), _ptr(supp, torch.int32),
                             _ptr(coef, torch.float32), _ptr(err, torch.float32),
                             _ptr(sqerr_per_iter, torch.float64, True)))


def sbo_sqerr(ctx, err, out) -> None:
    import torch
    _check(lib().sbo_sqerr(ctx, _ptr(err, torch.float32), err.shape[0], _ptr(out, torch.float64)))


def sbo_worst(ctx, err, W, ids) -> None:
    import torch
    _check(lib().sbo_worst(ctx, _ptr(err, torch.float32), err.shape[0], int(W), _ptr(ids, torch.int32)))


def sbo_init_base(ctx, Y, ids, Q, sv=None) -> None:
    import torch
    _check(lib().sbo_init_base(ctx, _ptr(Y, torch.float32), Y.shape[0], _ptr(ids, torch.int32),
                               ids.shape[0], _ptr(Q, torch.float32), _ptr(sv, torch.float32, True)))


def sbo_new_base(ctx, Y, ids, R, have_q0, Q, supp, coef, err, sqerr_per_round=None) -> None:
    import torch
    _check(lib().sbo_new_base(ctx, _ptr(Y, torch.float32), Y.shape[0], _ptr(ids, torch.int32),
                              ids.shape[0], int(R), 1 if have_q0 else 0, _ptr(Q, torch.float32),
                              _ptr(supp, torch.int32), _ptr(coef, torch.float32),
                              _ptr(err, torch.float32), _ptr(sqerr_per_round, torch.float64, True)))


def sbo_set_blocks(ctx, K: int) -> None:
    _check(lib().sbo_set_blocks(ctx, int(K)))


def sbo_learn(ctx, Y, D, init_ids, R, W, K_max, target_rmse, blk, supp, coef, err):
    """Returns (K_final, rmse_history); D must have room for K_max orthobases."""
    import torch
    K0, P0 = init_ids.shape
    kf, nh = ctypes.c_int(0), ctypes.c_int(0)
    hist = (ctypes.c_double * (K_max - K0 + 1))()
    _check(lib().sbo_learn(ctx, _ptr(Y, torch.float32), Y.shape[0], _ptr(D, torch.float32),
                           _ptr(init_ids, torch.int32), int(K0), int(P0), int(R), int(W), int(K_max),
                           float(target_rmse), _ptr(blk, torch.int32), _ptr(supp, torch.int32),
                           _ptr(coef, torch.float32), _ptr(err, torch.float32), ctypes.byref(kf),
                           hist, ctypes.byref(nh)))
    return kf.value, [hist[i] for i in range(nh.value)]


def sbo_svd_sweeps(ctx, K: int) -> list:
    """Per orthobase, for the most recent SVD stage (K = blocks in use): Jacobi sweeps (> 0) or
    minus the Newton-Schulz steps (< 0); 0 = kept its basis."""
    buf = (ctypes.c_int32 * K)()
    _check(lib().sbo_svd_sweeps(ctx, buf))
    return list(buf)


SBO_OPT_SVD_METHOD, SBO_OPT_CODING_ARITH = 0, 1
SBO_SVD_AUTO, SBO_SVD_JACOBI = 0, 1
SBO_ARITH_F32, SBO_ARITH_BF16X3, SBO_ARITH_BF16X3_SCREEN, SBO_ARITH_F16X2 = 0, 1, 2, 3


def sbo_set_option(ctx, option: int, value: int) -> None:
    _check(lib().sbo_set_option(ctx, int(option), int(value)))


def sbo_set_timing(ctx, enable) -> None:
    """enable: False/0 off, True/1 every stage, 2 the energy kernel only."""
    _check(lib().sbo_set_timing(ctx, int(enable)))


def sbo_stage_ms(ctx) -> dict:
    buf = (ctypes.c_float * len(STAGES))()
    _check(lib().sbo_stage_ms(ctx, buf))
    return {name: float(buf[i]) for i, name in enumerate(STAGES)}
