"""Thin ctypes binding of libbb.so: argument marshalling only.

Functions mirror include/bb.h.  Tensor arguments are torch tensors on the GPU
(bf16, contiguous); torch is used for device memory and the current stream,
every step of the computation runs inside the library's HIP kernels.  There is
no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libbb.so")

BB_OK = 0
BB_ERR_WORKSPACE = -7
BB_ERR_VARIANT = -9
BB_ERR_TIMEOUT = -10
BB_ERR_INIT = -11
STATIC_SCRATCH_BYTES = 32 << 20
VARIANT_AUTO, VARIANT_STREAM, VARIANT_SNAPSHOT1, VARIANT_UNFUSED, VARIANT_PRESCALE, VARIANT_NEST = 0, 1, 2, 3, 4, 5
OP_FFN, OP_LN, OP_FFN_UNFUSED, OP_LN_UNFUSED = 0, 1, 2, 3

EXPORTS = [
    "bb_rmsnorm_swiglu_ffn", "bb_layernorm_matmul",
    "bb_rmsnorm_swiglu_ffn_unfused", "bb_layernorm_matmul_unfused",
    "bb_rmsnorm_swiglu_ffn_t", "bb_layernorm_matmul_t", "bb_attention", "bb_attention_workspace_bytes",
    "bb_rmsnorm_swiglu_ffn_residual", "bb_rmsnorm_swiglu_ffn_residual_t",
    "bb_rmsnorm_swiglu_ffn_tune", "bb_layernorm_matmul_tune", "bb_tuned_variant", "bb_tune_clear",
    "bb_workspace_bytes", "bb_set_workspace", "bb_set_variant", "bb_get_variant",
    "bb_shutdown", "bb_status_string", "bb_version", "bb_last_hip_error",
    "bb_calib_copy", "bb_calib_read", "bb_calib_mfma", "bb_calib_mfma_data",
    "bb_profile_enable", "bb_profile_count", "bb_profile_get", "bb_profile_calls", "bb_profile_count_of",
    "bb_profile_get_of", "bb_check_fault", "bb_debug_inject_fault", "bb_debug_set_spin_limit",
    "bb_init", "bb_rmsnorm_swiglu_ffn_static",
]

_lib = None


class BBError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} (status {status})")


def load() -> ctypes.CDLL:
    """Loads libbb.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2505_07829_amd.build`")
    # torch first: libbb.so must bind to the HIP runtime torch has loaded (same soname), so that
    # both work in one device context; loaded the other way round the process ends up with two
    # runtimes and this library's sees no device.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, f32, sz, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t, ctypes.c_int
    lib.bb_rmsnorm_swiglu_ffn.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, f32, vp]
    lib.bb_rmsnorm_swiglu_ffn_unfused.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, f32, vp]
    lib.bb_rmsnorm_swiglu_ffn_static.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, f32, vp]
    lib.bb_rmsnorm_swiglu_ffn_t.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, f32, vp]
    lib.bb_layernorm_matmul_t.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, f32, vp]
    lib.bb_layernorm_matmul.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, f32, vp]
    lib.bb_layernorm_matmul_unfused.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, f32, vp]
    pi, pf = ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float)
    lib.bb_rmsnorm_swiglu_ffn_tune.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, f32, vp, ci, pi, pf]
    lib.bb_layernorm_matmul_tune.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, f32, vp, ci, pi, pf]
    lib.bb_tuned_variant.argtypes = [ci, i64, i64, i64]
    lib.bb_rmsnorm_swiglu_ffn_residual.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, f32, vp]
    lib.bb_rmsnorm_swiglu_ffn_residual_t.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, f32, vp]
    lib.bb_attention.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, vp]
    lib.bb_attention_workspace_bytes.argtypes = [i64, i64, i64, i64, i64]
    lib.bb_attention_workspace_bytes.restype = sz
    lib.bb_workspace_bytes.argtypes = [ci, i64, i64, i64]
    lib.bb_workspace_bytes.restype = sz
    lib.bb_set_workspace.argtypes = [vp, sz]
    lib.bb_set_variant.argtypes = [ci]
    lib.bb_status_string.argtypes = [ci]
    lib.bb_status_string.restype = ctypes.c_char_p
    lib.bb_calib_copy.argtypes = [vp, vp, sz, vp]
    lib.bb_calib_read.argtypes = [vp, sz, vp, vp]
    lib.bb_calib_mfma.argtypes = [ci, ci, vp, vp]
    lib.bb_calib_mfma_data.argtypes = [vp, ci, ci, vp, vp]
    lib.bb_profile_enable.argtypes = [ci]
    lib.bb_profile_get.argtypes = [ci, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_char_p)]
    lib.bb_profile_count_of.argtypes = [ci]
    lib.bb_profile_get_of.argtypes = [ci, ci, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_char_p)]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if name not in ("bb_workspace_bytes", "bb_status_string", "bb_attention_workspace_bytes"):
            fn.restype = ci
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().bb_status_string(int(status)).decode()


def _check(rc: int, what: str) -> None:
    if rc != BB_OK:
        raise BBError(rc, what)


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream() -> int:
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


def _require(t, shape, name):
    import torch
    if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous CUDA bfloat16 tensor")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")


def bb_rmsnorm_swiglu_ffn(X, g, W1, W3, W2, eps: float, Y=None, unfused: bool = False):
    """Y = (SiLU(Xh W1) * (Xh W3)) W2 with Xh = g * X / sqrt(mean(X^2) + eps).  Returns Y."""
    import torch
    lib = load()
    M, D = X.shape
    F = W1.shape[1]
    _require(X, (M, D), "X"); _require(g, (D,), "g")
    _require(W1, (D, F), "W1"); _require(W3, (D, F), "W3"); _require(W2, (F, D), "W2")
    if Y is None:
        Y = torch.empty((M, D), dtype=torch.bfloat16, device=X.device)
    _require(Y, (M, D), "Y")
    fn = lib.bb_rmsnorm_swiglu_ffn_unfused if unfused else lib.bb_rmsnorm_swiglu_ffn
    _check(fn(_ptr(X), _ptr(g), _ptr(W1), _ptr(W3), _ptr(W2), _ptr(Y), M, D, F, float(eps), _stream()),
           "bb_rmsnorm_swiglu_ffn" + ("_unfused" if unfused else ""))
    return Y


def bb_init() -> None:
    """Sets the current device up (the one call of the no-allocation path that may allocate)."""
    _check(load().bb_init(), "bb_init")


def bb_rmsnorm_swiglu_ffn_static(X, g, W1, W3, W2, eps: float, Y):
    """bb_rmsnorm_swiglu_ffn with the library's static scratch array; allocates nothing, so Y is required."""
    lib = load()
    M, D = X.shape
    F = W1.shape[1]
    _require(X, (M, D), "X"); _require(g, (D,), "g")
    _require(W1, (D, F), "W1"); _require(W3, (D, F), "W3"); _require(W2, (F, D), "W2")
    _require(Y, (M, D), "Y")
    _check(lib.bb_rmsnorm_swiglu_ffn_static(_ptr(X), _ptr(g), _ptr(W1), _ptr(W3), _ptr(W2), _ptr(Y), M, D, F,
                                            float(eps), _stream()), "bb_rmsnorm_swiglu_ffn_static")
    return Y


def bb_rmsnorm_swiglu_ffn_t(X, g, W1t, W3t, W2t, eps: float, Y=None):
    """The same operator with transposed weights W1t [F,D], W3t [F,D], W2t [D,F].  Returns Y."""
    import torch
    lib = load()
    M, D = X.shape
    F = W1t.shape[0]
    _require(X, (M, D), "X"); _require(g, (D,), "g")
    _require(W1t, (F, D), "W1t"); _require(W3t, (F, D), "W3t"); _require(W2t, (D, F), "W2t")
    if Y is None:
        Y = torch.empty((M, D), dtype=torch.bfloat16, device=X.device)
    _require(Y, (M, D), "Y")
    _check(lib.bb_rmsnorm_swiglu_ffn_t(_ptr(X), _ptr(g), _ptr(W1t), _ptr(W3t), _ptr(W2t), _ptr(Y), M, D, F,
                                       float(eps), _stream()), "bb_rmsnorm_swiglu_ffn_t")
    return Y


def bb_rmsnorm_swiglu_ffn_residual(X, g, W1, W3, W2, R, eps: float, Y=None, transposed: bool = False):
    """Y = R + FFN(RMSNorm(X)); weights [D,F],[D,F],[F,D], or transposed [F,D],[F,D],[D,F].
    Y may be R (in place).  Returns Y."""
    import torch
    lib = load()
    M, D = X.shape
    F = W1.shape[0] if transposed else W1.shape[1]
    _require(X, (M, D), "X"); _require(g, (D,), "g"); _require(R, (M, D), "R")
    wshape, w2shape = ((F, D), (D, F)) if transposed else ((D, F), (F, D))
    _require(W1, wshape, "W1"); _require(W3, wshape, "W3"); _require(W2, w2shape, "W2")
    if Y is None:
        Y = torch.empty((M, D), dtype=torch.bfloat16, device=X.device)
    _require(Y, (M, D), "Y")
    fn = lib.bb_rmsnorm_swiglu_ffn_residual_t if transposed else lib.bb_rmsnorm_swiglu_ffn_residual
    _check(fn(_ptr(X), _ptr(g), _ptr(W1), _ptr(W3), _ptr(W2), _ptr(R), _ptr(Y), M, D, F, float(eps), _stream()),
           "bb_rmsnorm_swiglu_ffn_residual")
    return Y


def bb_rmsnorm_swiglu_ffn_tune(X, g, W1, W3, W2, eps: float, reps: int = 5, Y=None):
    """Times the candidate programs of the FFN operator on these operands and records the fastest
    for this shape.  Returns (variant, {variant: ms})."""
    import torch
    lib = load()
    M, D = X.shape
    F = W1.shape[1]
    _require(X, (M, D), "X"); _require(g, (D,), "g")
    _require(W1, (D, F), "W1"); _require(W3, (D, F), "W3"); _require(W2, (F, D), "W2")
    if Y is None:
        Y = torch.empty((M, D), dtype=torch.bfloat16, device=X.device)
    _require(Y, (M, D), "Y")
    chosen, ms = ctypes.c_int(0), (ctypes.c_float * 6)()
    _check(lib.bb_rmsnorm_swiglu_ffn_tune(_ptr(X), _ptr(g), _ptr(W1), _ptr(W3), _ptr(W2), _ptr(Y), M, D, F,
                                          float(eps), _stream(), int(reps), ctypes.byref(chosen), ms),
           "bb_rmsnorm_swiglu_ffn_tune")
    return chosen.value, {v: float(ms[v]) for v in (1, 2, 3, 4, 5) if ms[v] >= 0}


def bb_layernorm_matmul_tune(X, gamma, beta, W, eps: float, reps: int = 5, Y=None):
    """Times the candidate programs of LN->matmul on these operands and records the fastest for this
    shape.  Returns (variant, {variant: ms})."""
    import torch
    lib = load()
    M, D = X.shape
    N = W.shape[1]
    _require(X, (M, D), "X"); _require(gamma, (D,), "gamma"); _require(beta, (D,), "beta")
    _require(W, (D, N), "W")
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
    _require(Y, (M, N), "Y")
    chosen, ms = ctypes.c_int(0), (ctypes.c_float * 6)()
    _check(lib.bb_layernorm_matmul_tune(_ptr(X), _ptr(gamma), _ptr(beta), _ptr(W), _ptr(Y), M, D, N, float(eps),
                                        _stream(), int(reps), ctypes.byref(chosen), ms),
           "bb_layernorm_matmul_tune")
    return chosen.value, {v: float(ms[v]) for v in (1, 2, 3, 4, 5) if ms[v] >= 0}


def bb_tuned_variant(op: int, M: int, D: int, F_or_N: int) -> int:
    return int(load().bb_tuned_variant(op, M, D, F_or_N))


def bb_tune_clear() -> None:
    _check(load().bb_tune_clear(), "bb_tune_clear")


def bb_attention(Q, K, V, O=None):
    """O = softmax(Q K^T / sqrt(d)) V per problem; Q [B,M,d], K [B,N,d], V [B,N,dv].  Returns O [B,M,dv]."""
    import torch
    lib = load()
    B, M, d = Q.shape
    N, dv = V.shape[1], V.shape[2]
    _require(Q, (B, M, d), "Q"); _require(K, (B, N, d), "K"); _require(V, (B, N, dv), "V")
    if O is None:
        O = torch.empty((B, M, dv), dtype=torch.bfloat16, device=Q.device)
    _require(O, (B, M, dv), "O")
    _check(lib.bb_attention(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), B, M, N, d, dv, _stream()), "bb_attention")
    return O


def bb_attention_workspace_bytes(B: int, M: int, N: int, d: int, dv: int) -> int:
    return int(load().bb_attention_workspace_bytes(B, M, N, d, dv))


def bb_layernorm_matmul_t(X, gamma, beta, Wt, eps: float, Y=None):
    """Y = LN(X; gamma, beta, eps) W with W given transposed, Wt [N,D].  Returns Y."""
    import torch
    lib = load()
    M, D = X.shape
    N = Wt.shape[0]
    _require(X, (M, D), "X"); _require(gamma, (D,), "gamma"); _require(beta, (D,), "beta")
    _require(Wt, (N, D), "Wt")
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
    _require(Y, (M, N), "Y")
    _check(lib.bb_layernorm_matmul_t(_ptr(X), _ptr(gamma), _ptr(beta), _ptr(Wt), _ptr(Y), M, D, N, float(eps),
                                     _stream()), "bb_layernorm_matmul_t")
    return Y


def bb_layernorm_matmul(X, gamma, beta, W, eps: float, Y=None, unfused: bool = False):
    """Y = LN(X; gamma, beta, eps) W.  Returns Y."""
    import torch
    lib = load()
    M, D = X.shape
    N = W.shape[1]
    _require(X, (M, D), "X"); _require(gamma, (D,), "gamma"); _require(beta, (D,), "beta")
    _require(W, (D, N), "W")
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
    _require(Y, (M, N), "Y")
    fn = lib.bb_layernorm_matmul_unfused if unfused else lib.bb_layernorm_matmul
    _check(fn(_ptr(X), _ptr(gamma), _ptr(beta), _ptr(W), _ptr(Y), M, D, N, float(eps), _stream()),
           "bb_layernorm_matmul" + ("_unfused" if unfused else ""))
    return Y


def bb_workspace_bytes(op: int, M: int, D: int, F_or_N: int) -> int:
    return int(load().bb_workspace_bytes(op, M, D, F_or_N))


def bb_set_workspace(t) -> None:
    """t: zero-filled CUDA tensor (any dtype) or None to return to the internal buffer."""
    if t is None:
        _check(load().bb_set_workspace(None, 0), "bb_set_workspace")
    else:
        _check(load().bb_set_workspace(_ptr(t), t.numel() * t.element_size()), "bb_set_workspace")


def bb_set_variant(v: int) -> None:
    _check(load().bb_set_variant(int(v)), "bb_set_variant")


def bb_get_variant() -> int:
    return int(load().bb_get_variant())


def bb_shutdown() -> None:
    _check(load().bb_shutdown(), "bb_shutdown")


def bb_version() -> int:
    return int(load().bb_version())


def bb_last_hip_error() -> int:
    return int(load().bb_last_hip_error())


def bb_calib_copy(src, dst) -> None:
    _check(load().bb_calib_copy(_ptr(src), _ptr(dst), src.numel() * src.element_size(), _stream()), "bb_calib_copy")


def bb_calib_read(src, sink) -> None:
    _check(load().bb_calib_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream()), "bb_calib_read")


def bb_calib_mfma(workgroups: int, iters: int, sink) -> None:
    _check(load().bb_calib_mfma(int(workgroups), int(iters), _ptr(sink), _stream()), "bb_calib_mfma")


def bb_calib_mfma_data(operands, workgroups: int, iters: int, sink) -> None:
    _check(load().bb_calib_mfma_data(_ptr(operands), int(workgroups), int(iters), _ptr(sink), _stream()),
           "bb_calib_mfma_data")


def bb_check_fault() -> None:
    """Raises BBError(BB_ERR_TIMEOUT) once if a streaming kernel of an earlier launch gave up a wait."""
    _check(load().bb_check_fault(), "bb_check_fault")


def bb_debug_inject_fault() -> None:
    _check(load().bb_debug_inject_fault(), "bb_debug_inject_fault")


def bb_debug_set_spin_limit(polls: int) -> None:
    _check(load().bb_debug_set_spin_limit(ctypes.c_uint(int(polls))), "bb_debug_set_spin_limit")


def bb_profile_enable(on: bool) -> None:
    _check(load().bb_profile_enable(1 if on else 0), "bb_profile_enable")


def bb_profile_last(back: int = 0):
    """[(kernel name, milliseconds)] of the operator call `back` calls before the most recent one (waits for it)."""
    lib = load()
    out = []
    for i in range(int(lib.bb_profile_count_of(int(back)))):
        ms, name = ctypes.c_float(), ctypes.c_char_p()
        _check(lib.bb_profile_get_of(int(back), i, ctypes.byref(ms), ctypes.byref(name)), "bb_profile_get_of")
        out.append((name.value.decode(), float(ms.value)))
    return out


def bb_profile_history():
    """[[(kernel name, milliseconds)]] of the calls kept since profiling was switched on, oldest first."""
    n = int(load().bb_profile_calls())
    return [bb_profile_last(back) for back in range(n - 1, -1, -1)]
