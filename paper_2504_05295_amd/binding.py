"""ctypes binding of libdion.so: the same entry points as include/dion.h, argument marshalling only.

PyTorch tensors are used as handles to device memory (``data_ptr()``) and for the current HIP
stream; every step of the Dion update runs in the library's HIP kernels.  There is no CPU
fallback: if the library has not been built, importing works but every call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdion.so")

DION_OK = 0
DION_EINVAL = -1
DION_EWORKSPACE = -2
DION_ELAUNCH = -3
DION_ENOMEM = -4
DION_NUM_BREAKDOWN = 1
DION_WAIT_TIMEOUT = 2
DION_G_F32, DION_G_BF16 = 0, 1
DION_MATH_F32, DION_MATH_BF16 = 0, 1
STAGES = ("k1_BQ", "orth", "k2_BtP", "colnorm", "k5_update")
DEBUG_Z, DEBUG_P, DEBUG_R, DEBUG_S, DEBUG_STATUS, DEBUG_P1, DEBUG_C, DEBUG_L, DEBUG_W, DEBUG_D, DEBUG_NULL = range(11)

DION_ORTH_CHOLQR2, DION_ORTH_SHIFTED_CHOLQR3, DION_ORTH_CHOLQR2_FALLBACK = 0, 1, 2
DION_FORM_STANDARD, DION_FORM_TRANSPOSED = 0, 1

EXPORTS = ("dion_workspace_bytes", "dion_init_state", "dion_init_state_ex", "dion_step", "dion_step_batched", "dion_lazy_step", "dion_lazy_step_batched",
           "dion_double_step", "dion_step_static", "dion_last_status",
           "dion_set_orth_mode", "dion_retry_breakdowns", "dion_set_wait_limit", "dion_cholesky_grid", "dion_set_stage_timing", "dion_stage_times", "dion_measure_ceilings", "dion_debug_buffer", "dion_destroy_state", "dion_strerror")

_lib = None


class DionError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, strerror(code), code))


def lib() -> C.CDLL:
    """Loads libdion.so (built by ``python -m paper_2504_05295_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libdion.so is not built: run `python -m paper_2504_05295_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        i64p, vpp = C.POINTER(C.c_int64), C.POINTER(C.c_void_p)
        L.dion_workspace_bytes.argtypes = [C.c_int, i64p, i64p, i64p, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
        L.dion_init_state.argtypes = [C.POINTER(C.c_void_p), C.c_int, i64p, i64p, i64p, C.c_int, C.c_int, C.c_void_p,
                                      C.c_size_t, vpp, vpp, C.c_int, C.c_uint64, C.c_void_p]
        L.dion_init_state_ex.argtypes = [C.POINTER(C.c_void_p), C.c_int, i64p, i64p, i64p, C.POINTER(C.c_int), C.c_int, C.c_int,
                                         C.c_void_p, C.c_size_t, vpp, vpp, C.c_int, C.c_uint64, C.c_void_p]
        L.dion_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                C.c_int64, C.c_float, C.c_float, C.c_void_p]
        L.dion_step_batched.argtypes = [C.c_void_p, C.c_int, vpp, vpp, vpp, vpp, i64p, i64p, i64p, C.c_float,
                                        C.c_float, C.c_void_p]
        L.dion_retry_breakdowns.argtypes = [C.c_void_p, C.c_int, vpp, vpp, vpp, vpp, i64p, i64p, i64p, C.c_float,
                                            C.c_float, C.c_void_p, C.POINTER(C.c_int)]
        L.dion_lazy_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                     C.c_int64, C.c_float, C.c_float, C.c_int, C.c_void_p]
        L.dion_lazy_step_batched.argtypes = [C.c_void_p, C.c_int, vpp, vpp, vpp, vpp, i64p, i64p, i64p, C.c_float,
                                             C.c_float, C.c_int, C.c_void_p]
        L.dion_double_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int, vpp, vpp, vpp, vpp, vpp, vpp, vpp, i64p, i64p, i64p, i64p,
                                       C.c_float, C.c_float, C.c_float, C.c_void_p]
        L.dion_step_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int,
                                       C.c_int, C.c_float, C.c_float, C.c_void_p, C.c_void_p]
        L.dion_last_status.argtypes = [C.c_void_p, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.dion_set_stage_timing.argtypes = [C.c_void_p, C.c_int]
        L.dion_set_orth_mode.argtypes = [C.c_void_p, C.c_int]
        L.dion_set_wait_limit.argtypes = [C.c_void_p, C.c_uint]
        L.dion_cholesky_grid.argtypes = [C.c_int, C.c_int, C.c_int64, C.POINTER(C.c_int)]
        L.dion_stage_times.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
        L.dion_measure_ceilings.argtypes = [C.c_void_p, C.c_size_t, C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p]
        L.dion_debug_buffer.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_void_p), i64p]
        L.dion_destroy_state.argtypes = [C.c_void_p]
        L.dion_strerror.argtypes = [C.c_int]
        L.dion_strerror.restype = C.c_char_p
        for name in EXPORTS:
            if name != "dion_strerror":
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().dion_strerror(int(code)).decode()


def _check(code: int, where: str):
    if code < 0:
        raise DionError(code, where)
    return code


def _i64(vals: Sequence[int]):
    return (C.c_int64 * len(vals))(*[int(v) for v in vals])


def _ptrs(tensors) -> "C.Array":
    return (C.c_void_p * len(tensors))(*[C.c_void_p(_ptr(t)) for t in tensors])


def _ptr(t) -> int:
    return int(t) if isinstance(t, int) else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    return C.c_void_p(int(stream))


def _check_tensor(t, dtype, shape, name):
    import torch
    if not isinstance(t, torch.Tensor):
        raise TypeError("%s must be a torch tensor" % name)
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise ValueError("%s must be a contiguous device tensor of dtype %s and shape %s (got %s %s)"
                         % (name, dtype, tuple(shape), t.dtype, tuple(t.shape)))


class DionState:
    """Owner of a dion_state_t* (and of the references that keep its workspace alive)."""

    def __init__(self, handle, shapes, g_dtype, math, workspace):
        self.handle = handle
        self.shapes = list(shapes)
        self.g_dtype = g_dtype
        self.math = math
        self.workspace = workspace

    def close(self):
        if self.handle:
            lib().dion_destroy_state(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def dion_workspace_bytes(shapes: Sequence[Tuple[int, int, int]], g_dtype: int, math: int) -> int:
    m, n, r = _i64([s[0] for s in shapes]), _i64([s[1] for s in shapes]), _i64([s[2] for s in shapes])
    out = C.c_size_t(0)
    _check(lib().dion_workspace_bytes(len(shapes), m, n, r, g_dtype, math, C.byref(out)), "dion_workspace_bytes")
    return int(out.value)


def dion_init_state(shapes, g_dtype, math, M: List, Q: List, q_is_filled: bool = True, seed: int = 0,
                    workspace=None, stream=None, forms=None) -> DionState:
    """Creates the state for matrices of `shapes` = [(m, n, r), ...]; zero-fills M, column-normalises Q
    (drawing it first when q_is_filled is False).  `workspace`: a uint8 device tensor, allocated here if None.
    `forms`: per-matrix DION_FORM_* (dion_init_state_ex); a transposed-form matrix has an m x r factor."""
    import torch
    need = dion_workspace_bytes(shapes, g_dtype, math)
    if workspace is None:
        workspace = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    base = workspace.data_ptr()
    aligned = (base + 255) // 256 * 256
    avail = workspace.numel() - (aligned - base)
    for i, (m, n, r) in enumerate(shapes):
        _check_tensor(M[i], torch.float32, (m, n), "M[%d]" % i)
        frows = m if (forms is not None and forms[i] == DION_FORM_TRANSPOSED) else n
        _check_tensor(Q[i], torch.float32, (frows, r), "Q[%d]" % i)
    handle = C.c_void_p(None)
    m, n, r = _i64([s[0] for s in shapes]), _i64([s[1] for s in shapes]), _i64([s[2] for s in shapes])
    if forms is None:
        _check(lib().dion_init_state(C.byref(handle), len(shapes), m, n, r, g_dtype, math, C.c_void_p(aligned), avail,
                                     _ptrs(M), _ptrs(Q), 1 if q_is_filled else 0, int(seed), _stream(stream)),
               "dion_init_state")
    else:
        farr = (C.c_int * len(shapes))(*[int(f) for f in forms])
        _check(lib().dion_init_state_ex(C.byref(handle), len(shapes), m, n, r, farr, g_dtype, math, C.c_void_p(aligned),
                                        avail, _ptrs(M), _ptrs(Q), 1 if q_is_filled else 0, int(seed), _stream(stream)),
               "dion_init_state_ex")
    st = DionState(handle, shapes, g_dtype, math, workspace)
    st.forms = list(forms) if forms is not None else [DION_FORM_STANDARD] * len(shapes)
    return st


def _g_dtype(state):
    import torch
    return torch.bfloat16 if state.g_dtype == DION_G_BF16 else torch.float32


def dion_step(state: DionState, X, G, M, Q, mu: float, eta: float, stream=None) -> None:
    import torch
    m, n = X.shape
    r = Q.shape[1]
    _check_tensor(X, torch.float32, (m, n), "X")
    _check_tensor(G, _g_dtype(state), (m, n), "G")
    _check_tensor(M, torch.float32, (m, n), "M")
    if tuple(Q.shape) != (n, r) and tuple(Q.shape) != (m, r):
        raise ValueError("Q must be n x r (standard form) or m x r (transposed form)")
    _check_tensor(Q, torch.float32, tuple(Q.shape), "Q")
    _check(lib().dion_step(state.handle, _ptr(X), _ptr(G), _ptr(M), _ptr(Q), m, n, r, mu, eta, _stream(stream)), "dion_step")


def dion_step_batched(state: DionState, X: List, G: List, M: List, Q: List, mu: float, eta: float, stream=None) -> None:
    import torch
    count = len(X)
    for i in range(count):
        m, n, r = state.shapes[i]
        _check_tensor(X[i], torch.float32, (m, n), "X[%d]" % i)
        _check_tensor(G[i], _g_dtype(state), (m, n), "G[%d]" % i)
        _check_tensor(M[i], torch.float32, (m, n), "M[%d]" % i)
        frows = m if getattr(state, "forms", None) and state.forms[i] == DION_FORM_TRANSPOSED else n
        _check_tensor(Q[i], torch.float32, (frows, r), "Q[%d]" % i)
    sh = state.shapes[:count]
    _check(lib().dion_step_batched(state.handle, count, _ptrs(X), _ptrs(G), _ptrs(M), _ptrs(Q), _i64([s[0] for s in sh]),
                                   _i64([s[1] for s in sh]), _i64([s[2] for s in sh]), mu, eta, _stream(stream)),
           "dion_step_batched")


def dion_lazy_step(state: DionState, X, G, M, V, mu: float, eta: float, refresh: bool, stream=None) -> None:
    import torch
    m, n = X.shape
    r = V.shape[1]
    _check_tensor(X, torch.float32, (m, n), "X")
    _check_tensor(G, _g_dtype(state), (m, n), "G")
    _check_tensor(M, torch.float32, (m, n), "M")
    _check_tensor(V, torch.float32, (n, r), "V")
    _check(lib().dion_lazy_step(state.handle, _ptr(X), _ptr(G), _ptr(M), _ptr(V), m, n, r, mu, eta, 1 if refresh else 0,
                                _stream(stream)), "dion_lazy_step")


def dion_lazy_step_batched(state: DionState, X: List, G: List, M: List, V: List, mu: float, eta: float, refresh: bool,
                           stream=None) -> None:
    import torch
    count = len(X)
    for i in range(count):
        m, n, r = state.shapes[i]
        _check_tensor(X[i], torch.float32, (m, n), "X[%d]" % i)
        _check_tensor(G[i], _g_dtype(state), (m, n), "G[%d]" % i)
        _check_tensor(M[i], torch.float32, (m, n), "M[%d]" % i)
        _check_tensor(V[i], torch.float32, (n, r), "V[%d]" % i)
    sh = state.shapes[:count]
    _check(lib().dion_lazy_step_batched(state.handle, count, _ptrs(X), _ptrs(G), _ptrs(M), _ptrs(V),
                                        _i64([s[0] for s in sh]), _i64([s[1] for s in sh]), _i64([s[2] for s in sh]),
                                        mu, eta, 1 if refresh else 0, _stream(stream)), "dion_lazy_step_batched")


def dion_double_step(state1: DionState, state2: DionState, X: List, G: List, M1: List, V1: List, M2: List, V2: List, D: List,
                     mu1: float, mu2: float, eta: float, stream=None) -> None:
    """One Double Dion step: state1 holds the rank-r1 stage (M1, V1), state2 the rank-r2 stage (M2, V2);
    D are m x n fp32 scratch tensors for the stage-1 sketch."""
    import torch
    count = len(X)
    for i in range(count):
        m, n, r1 = state1.shapes[i]
        r2 = state2.shapes[i][2]
        _check_tensor(X[i], torch.float32, (m, n), "X[%d]" % i)
        _check_tensor(G[i], _g_dtype(state1), (m, n), "G[%d]" % i)
        _check_tensor(D[i], torch.float32, (m, n), "D[%d]" % i)
        _check_tensor(M1[i], torch.float32, (m, n), "M1[%d]" % i)
        _check_tensor(M2[i], torch.float32, (m, n), "M2[%d]" % i)
        _check_tensor(V1[i], torch.float32, (n, r1), "V1[%d]" % i)
        _check_tensor(V2[i], torch.float32, (n, r2), "V2[%d]" % i)
    sh1, sh2 = state1.shapes[:count], state2.shapes[:count]
    _check(lib().dion_double_step(state1.handle, state2.handle, count, _ptrs(X), _ptrs(G), _ptrs(M1), _ptrs(V1), _ptrs(M2),
                                  _ptrs(V2), _ptrs(D), _i64([s[0] for s in sh1]), _i64([s[1] for s in sh1]),
                                  _i64([s[2] for s in sh1]), _i64([s[2] for s in sh2]), mu1, mu2, eta, _stream(stream)),
           "dion_double_step")


DION_STATIC_SCRATCH_BYTES = 32 << 20


def dion_step_static(X, G, M, Q, g_dtype: int, math: int, mu: float, eta: float, status=None, stream=None) -> None:
    """One Dion step on the library's static workspace (no state object, nothing allocated); `status`: an int32
    device tensor of one element that receives the status word, or None."""
    import torch
    m, n = X.shape
    r = Q.shape[1]
    _check_tensor(X, torch.float32, (m, n), "X")
    _check_tensor(G, torch.bfloat16 if g_dtype == DION_G_BF16 else torch.float32, (m, n), "G")
    _check_tensor(M, torch.float32, (m, n), "M")
    _check_tensor(Q, torch.float32, (n, r), "Q")
    if status is not None:
        _check_tensor(status, torch.int32, (1,), "status")
    _check(lib().dion_step_static(_ptr(X), _ptr(G), _ptr(M), _ptr(Q), m, n, r, g_dtype, math, mu, eta,
                                  C.c_void_p(_ptr(status)) if status is not None else None, _stream(stream)), "dion_step_static")


def dion_retry_breakdowns(state: DionState, X: List, G: List, M: List, Q: List, mu: float, eta: float, stream=None) -> int:
    """Repeats the last batched step, with the robust orthonormalisation, for the matrices that broke down."""
    sh = state.shapes[:len(X)]
    n_retried = C.c_int(0)
    _check(lib().dion_retry_breakdowns(state.handle, len(X), _ptrs(X), _ptrs(G), _ptrs(M), _ptrs(Q),
                                       _i64([s[0] for s in sh]), _i64([s[1] for s in sh]), _i64([s[2] for s in sh]),
                                       mu, eta, _stream(stream), C.byref(n_retried)), "dion_retry_breakdowns")
    return int(n_retried.value)


def dion_last_status(state: DionState) -> Tuple[int, int]:
    """Synchronises the last step's stream; returns (status, first_bad_index)."""
    st, bad = C.c_int(0), C.c_int(-1)
    _check(lib().dion_last_status(state.handle, C.byref(st), C.byref(bad)), "dion_last_status")
    return int(st.value), int(bad.value)


def dion_set_orth_mode(state: DionState, mode: int) -> None:
    _check(lib().dion_set_orth_mode(state.handle, int(mode)), "dion_set_orth_mode")


def dion_set_wait_limit(state: DionState, polls: int) -> None:
    _check(lib().dion_set_wait_limit(state.handle, int(polls)), "dion_set_wait_limit")


def dion_cholesky_grid(compute_units: int, batch: int, r: int) -> int:
    """Workgroups per matrix of the single-launch factorisation, or 0 for a launch per panel.  Host only."""
    w = C.c_int(0)
    _check(lib().dion_cholesky_grid(int(compute_units), int(batch), int(r), C.byref(w)), "dion_cholesky_grid")
    return int(w.value)


def dion_set_stage_timing(state: DionState, enable: bool) -> None:
    _check(lib().dion_set_stage_timing(state.handle, 1 if enable else 0), "dion_set_stage_timing")


def dion_stage_times(state: DionState) -> dict:
    arr = (C.c_float * len(STAGES))()
    _check(lib().dion_stage_times(state.handle, arr), "dion_stage_times")
    return {k: float(arr[i]) for i, k in enumerate(STAGES)}


def dion_measure_ceilings(scratch, stream=None) -> dict:
    """Measured bf16 MFMA issue rate (TFLOP/s) and 18-byte-per-element streaming rate (GB/s) of the current GPU.
    `scratch`: a uint8 device tensor (overwritten), 1 GiB or so."""
    import torch
    mf, st = C.c_double(0.0), C.c_double(0.0)
    s = stream if stream is not None else torch.cuda.current_stream()
    _check(lib().dion_measure_ceilings(C.c_void_p(scratch.data_ptr()), scratch.numel() * scratch.element_size(), C.byref(mf),
                                       C.byref(st), C.c_void_p(s.cuda_stream)), "dion_measure_ceilings")
    return {"mfma_tflops": float(mf.value), "stream_gbps": float(st.value)}


def dion_debug_buffer(state: DionState, index: int, which: int):
    """Returns a torch view (no copy) of an intermediate left in the workspace by the last step."""
    import torch
    p, ld = C.c_void_p(None), C.c_int64(0)
    _check(lib().dion_debug_buffer(state.handle, index, which, C.byref(p), C.byref(ld)), "dion_debug_buffer")
    m, n, r = state.shapes[index]
    rows = {DEBUG_Z: m, DEBUG_P: m, DEBUG_P1: m, DEBUG_R: n, DEBUG_S: r, DEBUG_D: r, DEBUG_STATUS: 1, DEBUG_NULL: (r + 63) // 64 * 64,
            DEBUG_C: int(ld.value), DEBUG_L: int(ld.value), DEBUG_W: int(ld.value)}[which]
    cols = int(ld.value)
    dtype = torch.int32 if which in (DEBUG_STATUS, DEBUG_NULL) else torch.float32
    nbytes = rows * cols * 4
    ws = state.workspace
    off = int(p.value) - ws.data_ptr()
    assert 0 <= off and off + nbytes <= ws.numel()
    return ws[off:off + nbytes].view(dtype).view(rows, cols)


def dion_destroy_state(state: DionState) -> None:
    state.close()
