"""paper_2510_00236_amd -- thin Python binding of libpex (HIP, gfx950).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch supplies
device memory and streams.  There is no CPU fallback: if ``libpex.so`` is missing or a tensor is not on
the GPU the call raises.

Functions mirror the C ABI in ``include/pex.h``:
``pex_stat``, ``pex_stat_multi``, ``pex_token_sq``, ``pex_adam_update``, ``pex_signsgd_update`` and the
workspace queries.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpex.so")

PEX_OK = 0
PEX_F32, PEX_BF16 = 0, 1
PEX_PHI_IDENTITY, PEX_PHI_SQUARE, PEX_PHI_SIGN = 0, 1, 2
PEX_ADAM, PEX_MICROADAM, PEX_MICROADAM_VAR, PEX_MICROADAM_MSQ = 0, 1, 2, 3
PHI = {"identity": PEX_PHI_IDENTITY, "square": PEX_PHI_SQUARE, "sign": PEX_PHI_SIGN}
PEX_MICROSIGNSGD, PEX_SIGNSGD, PEX_SIGNEMA = 0, 1, 2
SIGN_VARIANT = {"microsignsgd": PEX_MICROSIGNSGD, "signsgd": PEX_SIGNSGD, "signema": PEX_SIGNEMA}
VARIANT = {"adam": PEX_ADAM, "microadam": PEX_MICROADAM, "microadam_var": PEX_MICROADAM_VAR,
           "microadam_msq": PEX_MICROADAM_MSQ}

PEX_WANT_IDENTITY, PEX_WANT_SQUARE, PEX_WANT_SIGN = 1, 2, 4
WANT = {"identity": PEX_WANT_IDENTITY, "square": PEX_WANT_SQUARE, "sign": PEX_WANT_SIGN}

EXPORTS = ("pex_status_string", "pex_version", "pex_stat_workspace_bytes", "pex_stat",
           "pex_stat_multi_workspace_bytes", "pex_stat_multi", "pex_vec_stat_workspace_bytes", "pex_vec_stat",
           "pex_example_norms_workspace_bytes", "pex_example_norms", "pex_weighted_sum_workspace_bytes",
           "pex_weighted_sum", "pex_token_norms", "pex_sign_update",
           "pex_stat_power_workspace_bytes", "pex_stat_power",
           "pex_token_sq_workspace_bytes", "pex_token_sq", "pex_adam_update", "pex_signsgd_update",
           "pex_moment_track_workspace_bytes", "pex_moment_track", "pex_embed_stat_workspace_bytes", "pex_embed_stat",
           "pex_mfma_probe_operand_bytes", "pex_mfma_probe_sink_floats", "pex_mfma_probe",
           "pex_sum_squares_workspace_bytes", "pex_sum_squares", "pex_adam_update_clipped", "pex_stat_noalloc", "pex_set_option", "pex_get_option", "pex_clip_weights")


class PexError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libpex: {msg} (status {code})")
        self.code = code


class AdamParams(ctypes.Structure):
    """Mirror of ``pex_adam_params``."""
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("eps_root", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("grad_scale", ctypes.c_float), ("sq_scale", ctypes.c_float),
                ("step", ctypes.c_int64), ("B", ctypes.c_int32)]


class MomentParams(ctypes.Structure):
    """Mirror of ``pex_moment_params``."""
    _fields_ = [("beta2", ctypes.c_float), ("grad_scale", ctypes.c_float), ("sq_scale", ctypes.c_float),
                ("B", ctypes.c_int32), ("debias", ctypes.c_int32), ("step", ctypes.c_int64)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libpex.so (built by ``python -m paper_2510_00236_amd.build``); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2510_00236_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        i64, i32, p, sz, f = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
        L.pex_status_string.argtypes = [ctypes.c_int]
        L.pex_status_string.restype = ctypes.c_char_p
        L.pex_version.restype = ctypes.c_int
        L.pex_stat_workspace_bytes.argtypes = [i64, i64, i64, i64, ctypes.c_int, ctypes.c_int]
        L.pex_stat_workspace_bytes.restype = sz
        L.pex_stat.argtypes = [p, p, i64, i64, i64, i64, ctypes.c_int, ctypes.c_int, p, p, sz, p]
        L.pex_stat.restype = ctypes.c_int
        L.pex_clip_weights.argtypes = [p, i64, i32, f, p, p]
        L.pex_clip_weights.restype = ctypes.c_int
        L.pex_set_option.argtypes = [ctypes.c_int, i32]
        L.pex_set_option.restype = ctypes.c_int
        L.pex_get_option.argtypes = [ctypes.c_int]
        L.pex_get_option.restype = i32
        L.pex_stat_noalloc.argtypes = [p, p, i64, i64, i64, i64, ctypes.c_int, ctypes.c_int, p, p]
        L.pex_stat_noalloc.restype = ctypes.c_int
        L.pex_stat_multi_workspace_bytes.argtypes = [i64, i64, i64, i64, ctypes.c_int, ctypes.c_uint32]
        L.pex_stat_multi_workspace_bytes.restype = sz
        L.pex_stat_multi.argtypes = [p, p, i64, i64, i64, i64, ctypes.c_int, ctypes.c_uint32, p, p, p, p, sz, p]
        L.pex_stat_multi.restype = ctypes.c_int
        L.pex_vec_stat_workspace_bytes.argtypes = [i64, i64, i64, ctypes.c_int]
        L.pex_vec_stat_workspace_bytes.restype = sz
        L.pex_vec_stat.argtypes = [p, p, i64, i64, i64, ctypes.c_int, ctypes.c_uint32, p, p, p, p, sz, p]
        L.pex_vec_stat.restype = ctypes.c_int
        for fn in (L.pex_example_norms_workspace_bytes, L.pex_weighted_sum_workspace_bytes):
            fn.argtypes = [i64, i64, i64, i64, ctypes.c_int]
            fn.restype = sz
        L.pex_example_norms.argtypes = [p, p, i64, i64, i64, i64, ctypes.c_int, p, p, sz, p]
        L.pex_example_norms.restype = ctypes.c_int
        L.pex_weighted_sum.argtypes = [p, p, p, i64, i64, i64, i64, ctypes.c_int, p, p, sz, p]
        L.pex_weighted_sum.restype = ctypes.c_int
        L.pex_stat_power_workspace_bytes.argtypes = [i64, i64, i64, i64, ctypes.c_int]
        L.pex_stat_power_workspace_bytes.restype = sz
        L.pex_stat_power.argtypes = [p, p, i64, i64, i64, i64, ctypes.c_int, f, p, p, sz, p]
        L.pex_stat_power.restype = ctypes.c_int
        L.pex_token_norms.argtypes = [p, p, i64, i64, i64, i64, ctypes.c_int, p, p]
        L.pex_token_norms.restype = ctypes.c_int
        L.pex_token_sq_workspace_bytes.argtypes = [i64, i64, i64, i64, ctypes.c_int]
        L.pex_token_sq_workspace_bytes.restype = sz
        L.pex_token_sq.argtypes = [p, p, i64, i64, i64, i64, ctypes.c_int, p, p, sz, p]
        L.pex_token_sq.restype = ctypes.c_int
        L.pex_adam_update.argtypes = [p, p, p, p, p, i64, ctypes.c_int, ctypes.POINTER(AdamParams), p]
        L.pex_adam_update.restype = ctypes.c_int
        L.pex_signsgd_update.argtypes = [p, p, p, i64, f, f, f, i32, i32, i64, p]
        L.pex_signsgd_update.restype = ctypes.c_int
        L.pex_sign_update.argtypes = [p, p, p, i64, ctypes.c_int, f, f, f, i32, i32, i64, p]
        L.pex_sign_update.restype = ctypes.c_int
        L.pex_moment_track_workspace_bytes.argtypes = [i64]
        L.pex_moment_track_workspace_bytes.restype = sz
        L.pex_moment_track.argtypes = [p, p, p, p, i64, ctypes.POINTER(MomentParams), p, p, sz, p]
        L.pex_moment_track.restype = ctypes.c_int
        L.pex_embed_stat_workspace_bytes.argtypes = [i64, i64, i64, i64]
        L.pex_embed_stat_workspace_bytes.restype = sz
        L.pex_embed_stat.argtypes = [p, i32, p, i64, i64, i64, i64, ctypes.c_int, ctypes.c_uint32, p, p, p, p, sz, p]
        L.pex_embed_stat.restype = ctypes.c_int
        L.pex_mfma_probe_operand_bytes.restype = sz
        L.pex_mfma_probe_sink_floats.argtypes = [i32]
        L.pex_mfma_probe_sink_floats.restype = sz
        L.pex_mfma_probe.argtypes = [p, i32, i32, p, ctypes.POINTER(ctypes.c_double), p]
        L.pex_mfma_probe.restype = ctypes.c_int
        L.pex_sum_squares_workspace_bytes.argtypes = [i64]
        L.pex_sum_squares_workspace_bytes.restype = sz
        L.pex_sum_squares.argtypes = [p, i64, p, i32, p, sz, p]
        L.pex_sum_squares.restype = ctypes.c_int
        L.pex_adam_update_clipped.argtypes = [p, p, p, p, p, i64, ctypes.c_int, ctypes.POINTER(AdamParams), p, f, p]
        L.pex_adam_update_clipped.restype = ctypes.c_int
        _lib = L
    return _lib


PEX_OPT_MAX_SPLIT, PEX_OPT_TOKEN_PRESQUARE, PEX_OPT_WIDE_BLOCKS, PEX_OPT_GRAM_NORMS, PEX_OPT_MEMORY_FOLD = 0, 1, 2, 3, 4
OPTION = {"max_split": PEX_OPT_MAX_SPLIT, "token_presquare": PEX_OPT_TOKEN_PRESQUARE, "wide_blocks": PEX_OPT_WIDE_BLOCKS,
          "gram_norms": PEX_OPT_GRAM_NORMS, "memory_fold": PEX_OPT_MEMORY_FOLD}


def pex_set_option(opt, value) -> None:
    """Set a planner option ('max_split' 1..32, 'token_presquare' 0|1|2, 'wide_blocks' 0|1|2, 'gram_norms' 0|1|2|3, 'memory_fold' 0|1|2, or the code)."""
    _check(lib().pex_set_option(OPTION.get(opt, opt), int(value)))


def pex_get_option(opt) -> int:
    return int(lib().pex_get_option(OPTION.get(opt, opt)))


def status_string(code: int) -> str:
    return lib().pex_status_string(int(code)).decode()


def _check(code: int):
    if code != PEX_OK:
        raise PexError(code, status_string(code))


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return PEX_F32
    if t.dtype == torch.bfloat16:
        return PEX_BF16
    raise TypeError(f"X and G must be float32 or bfloat16, got {t.dtype}")


class _Buf:
    """A tensor whose type and size have been checked, on its way to becoming a raw device pointer."""
    __slots__ = ("t", "name")

    def __init__(self, t, name):
        self.t, self.name = t, name


def _invoke(fn, *args):
    """Call a library function: every checked tensor must live on the GPU (all type and size checks of the call
    have passed by now), then goes in as its address; a status other than PEX_OK raises."""
    for a in args:
        if isinstance(a, _Buf) and not a.t.is_cuda:
            raise ValueError(f"{a.name} must live in GPU memory (libpex has no CPU path)")
    _check(fn(*[a.t.data_ptr() if isinstance(a, _Buf) else a.handle() if isinstance(a, _Stream) else a for a in args]))


def _dev(t, name, dtype=None, numel=None, shape=None):
    """``t`` as an argument for _invoke after checking what the library cannot check through a raw pointer: where the tensor
    lives, that it is dense, and -- when given -- its element type and its size (a buffer of another type or size
    would make a kernel read or write past its end)."""
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"{name} must have {numel} elements, got {t.numel()}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return _Buf(t, name)


def _f32(t, name, numel=None, shape=None):
    import torch
    return _dev(t, name, torch.float32, numel, shape)


def _f64(t, name, numel=None):
    import torch
    return _dev(t, name, torch.float64, numel)


class _Stream:
    """The stream argument of a call, turned into a hipStream_t by _invoke (None = torch's current stream)."""
    __slots__ = ("stream",)

    def __init__(self, stream):
        self.stream = stream

    def handle(self):
        import torch
        s = torch.cuda.current_stream() if self.stream is None else self.stream
        return ctypes.c_void_p(s.cuda_stream)


def _stream(stream):
    return _Stream(stream)


def _shapes(X, G):
    if X.dim() != 3 or G.dim() != 3 or X.shape[:2] != G.shape[:2]:
        raise ValueError(f"expected X[B,T,din] and G[B,T,dout], got {tuple(X.shape)} and {tuple(G.shape)}")
    if X.dtype != G.dtype:
        raise TypeError("X and G must share a dtype")
    B, T, din = X.shape
    return int(B), int(T), int(din), int(G.shape[2])


def pex_stat_workspace_bytes(B, T, din, dout, dtype_code, phi) -> int:
    return int(lib().pex_stat_workspace_bytes(B, T, din, dout, dtype_code, PHI.get(phi, phi)))


def _want_mask(want) -> int:
    if isinstance(want, int):
        return want
    mask = 0
    for w in want:
        mask |= WANT[w]
    return mask


def pex_stat_multi_workspace_bytes(B, T, din, dout, dtype_code, want) -> int:
    return int(lib().pex_stat_multi_workspace_bytes(B, T, din, dout, dtype_code, _want_mask(want)))


def pex_token_sq_workspace_bytes(B, T, din, dout, dtype_code) -> int:
    return int(lib().pex_token_sq_workspace_bytes(B, T, din, dout, dtype_code))


def _workspace(nbytes, like, workspace, stream=None):
    """The caller's workspace (uint8, at least ``nbytes``) or a temporary one.  A temporary is allocated under the
    stream the kernels run on, so the caching allocator does not hand its memory out again before they finish."""
    import torch
    if workspace is None:
        if nbytes == 0:
            return None, None, 0
        if stream is None:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=like.device)
        else:
            with torch.cuda.stream(stream):
                workspace = torch.empty(nbytes, dtype=torch.uint8, device=like.device)
    else:
        if workspace.dtype != torch.uint8:
            raise TypeError(f"workspace must be uint8, got {workspace.dtype}")
        if workspace.numel() < nbytes:
            raise ValueError(f"workspace holds {workspace.numel()} bytes, the call needs {nbytes}")
    return workspace, _dev(workspace, "workspace"), workspace.numel()


def pex_stat(X, G, phi, S=None, workspace=None, stream=None):
    """S[din,dout] = sum_b phi(X_b^T G_b), fp32.  ``phi`` is 'identity' | 'square' | 'sign' (or its code)."""
    import torch
    B, T, din, dout = _shapes(X, G)
    dt = _dtype_code(X)
    code = PHI.get(phi, phi)
    if S is None:
        S = torch.empty(din, dout, dtype=torch.float32, device=X.device)
    ws, wptr, wbytes = _workspace(pex_stat_workspace_bytes(B, T, din, dout, dt, code), X, workspace, stream)
    _invoke(lib().pex_stat, _dev(X, "X"), _dev(G, "G"), B, T, din, dout, dt, code, _f32(S, "S", shape=(din, dout)), wptr, wbytes,
                          _stream(stream))
    return S


NOALLOC_SCRATCH_BYTES = 32 << 20


def pex_stat_noalloc(X, G, phi, S, stream=None):
    """pex_stat into the caller's ``S`` with the library's own static scratch: nothing is allocated, here or in the
    library.  Raises PexError (PEX_ERR_TOO_LARGE) when the call needs more than NOALLOC_SCRATCH_BYTES."""
    B, T, din, dout = _shapes(X, G)
    _invoke(lib().pex_stat_noalloc, _dev(X, "X"), _dev(G, "G"), B, T, din, dout, _dtype_code(X), PHI.get(phi, phi),
                                  _f32(S, "S", shape=(din, dout)), _stream(stream))
    return S


def pex_stat_multi(X, G, want, out=None, workspace=None, stream=None):
    """Several statistics from one pass.  ``want`` is an iterable of 'identity' | 'square' | 'sign' (or the bit
    set); returns a dict name -> S[din,dout] fp32.  ``out`` may supply the output tensors by name."""
    import torch
    B, T, din, dout = _shapes(X, G)
    dt = _dtype_code(X)
    mask = _want_mask(want)
    res = {}
    ptrs = []
    for name, bit in WANT.items():
        if mask & bit:
            S = (out or {}).get(name)
            if S is None:
                S = torch.empty(din, dout, dtype=torch.float32, device=X.device)
            res[name] = S
            ptrs.append(_f32(S, name, shape=(din, dout)))
        else:
            ptrs.append(None)
    ws, wptr, wbytes = _workspace(pex_stat_multi_workspace_bytes(B, T, din, dout, dt, mask), X, workspace, stream)
    _invoke(lib().pex_stat_multi, _dev(X, "X"), _dev(G, "G"), B, T, din, dout, dt, mask, ptrs[0], ptrs[1], ptrs[2],
                                wptr, wbytes, _stream(stream))
    return res


def pex_vec_stat_workspace_bytes(B, T, d, dtype_code) -> int:
    return int(lib().pex_vec_stat_workspace_bytes(B, T, d, dtype_code))


def pex_vec_stat(A, C=None, want=("identity", "square", "sign"), out=None, workspace=None, stream=None):
    """Statistics of a vector parameter: s[d] = sum_b phi(sum_t A[b,t,:] * C[b,t,:]); ``C=None`` is an offset.
    Returns a dict name -> s[d] fp32."""
    import torch
    if A.dim() != 3 or (C is not None and C.shape != A.shape):
        raise ValueError("expected A[B,T,d] and C of the same shape (or None)")
    if C is not None and C.dtype != A.dtype:
        raise TypeError("A and C must share a dtype")
    B, T, d = (int(x) for x in A.shape)
    dt = _dtype_code(A)
    mask = _want_mask(want)
    res, ptrs = {}, []
    for name, bit in WANT.items():
        if mask & bit:
            s = (out or {}).get(name)
            if s is None:
                s = torch.empty(d, dtype=torch.float32, device=A.device)
            res[name] = s
            ptrs.append(_f32(s, name, numel=d))
        else:
            ptrs.append(None)
    ws, wptr, wbytes = _workspace(pex_vec_stat_workspace_bytes(B, T, d, dt), A, workspace, stream)
    _invoke(lib().pex_vec_stat, _dev(A, "A"), _dev(C, "C") if C is not None else None, B, T, d, dt, mask,
                              ptrs[0], ptrs[1], ptrs[2], wptr, wbytes, _stream(stream))
    return res


def pex_example_norms_workspace_bytes(B, T, din, dout, dtype_code) -> int:
    return int(lib().pex_example_norms_workspace_bytes(B, T, din, dout, dtype_code))


def pex_weighted_sum_workspace_bytes(B, T, din, dout, dtype_code) -> int:
    return int(lib().pex_weighted_sum_workspace_bytes(B, T, din, dout, dtype_code))


def pex_stat_power_workspace_bytes(B, T, din, dout, dtype_code) -> int:
    return int(lib().pex_stat_power_workspace_bytes(B, T, din, dout, dtype_code))


def pex_example_norms(X, G, N=None, workspace=None, stream=None):
    """N[B] = ||X_b^T G_b||_F^2, fp32."""
    import torch
    B, T, din, dout = _shapes(X, G)
    dt = _dtype_code(X)
    if N is None:
        N = torch.empty(B, dtype=torch.float32, device=X.device)
    ws, wptr, wbytes = _workspace(pex_example_norms_workspace_bytes(B, T, din, dout, dt), X, workspace, stream)
    _invoke(lib().pex_example_norms, _dev(X, "X"), _dev(G, "G"), B, T, din, dout, dt, _f32(N, "N", numel=B), wptr, wbytes,
                                   _stream(stream))
    return N


def pex_weighted_sum(X, G, w, S=None, workspace=None, stream=None):
    """S[din,dout] = sum_b w[b] X_b^T G_b, fp32 (``w`` fp32 [B] on the GPU)."""
    import torch
    B, T, din, dout = _shapes(X, G)
    dt = _dtype_code(X)
    if S is None:
        S = torch.empty(din, dout, dtype=torch.float32, device=X.device)
    ws, wptr, wbytes = _workspace(pex_weighted_sum_workspace_bytes(B, T, din, dout, dt), X, workspace, stream)
    _invoke(lib().pex_weighted_sum, _dev(X, "X"), _dev(G, "G"), _f32(w, "w", numel=B), B, T, din, dout, dt, _f32(S, "S", shape=(din, dout)), wptr,
                                  wbytes, _stream(stream))
    return S


def pex_clip_weights(N, max_norm, w=None, stream=None):
    """w[B] = min(1, max_norm / sqrt(sum over layers of N)), ``N`` fp32 [layers, B] (or [B]) of per-layer squared
    per-example gradient norms on the GPU."""
    import torch
    if N.dim() not in (1, 2):
        raise ValueError("N must be [layers, B] or [B]")
    nlayers, B = (1, N.shape[0]) if N.dim() == 1 else (int(N.shape[0]), int(N.shape[1]))
    if w is None:
        w = torch.empty(B, dtype=torch.float32, device=N.device)
    _invoke(lib().pex_clip_weights, _f32(N, "N"), B, nlayers, float(max_norm), _f32(w, "w", numel=B), _stream(stream))
    return w


def pex_stat_power(X, G, alpha, S=None, workspace=None, stream=None):
    """S[din,dout] = sum_b |X_b^T G_b|^alpha, fp32."""
    import torch
    B, T, din, dout = _shapes(X, G)
    dt = _dtype_code(X)
    if S is None:
        S = torch.empty(din, dout, dtype=torch.float32, device=X.device)
    ws, wptr, wbytes = _workspace(pex_stat_power_workspace_bytes(B, T, din, dout, dt), X, workspace, stream)
    _invoke(lib().pex_stat_power, _dev(X, "X"), _dev(G, "G"), B, T, din, dout, dt, float(alpha), _f32(S, "S", shape=(din, dout)), wptr,
                                wbytes, _stream(stream))
    return S


def pex_token_norms(X, G, N_tok=None, stream=None):
    """N_tok[B,T] = ||x_bt||^2 ||g_bt||^2, fp32."""
    import torch
    B, T, din, dout = _shapes(X, G)
    dt = _dtype_code(X)
    if N_tok is None:
        N_tok = torch.empty(B, T, dtype=torch.float32, device=X.device)
    _invoke(lib().pex_token_norms, _dev(X, "X"), _dev(G, "G"), B, T, din, dout, dt, _f32(N_tok, "N_tok", numel=B * T), _stream(stream))
    return N_tok


def pex_token_sq(X, G, S=None, workspace=None, stream=None):
    """S_tok[din,dout] = (X o X)^T (G o G), fp32."""
    import torch
    B, T, din, dout = _shapes(X, G)
    dt = _dtype_code(X)
    if S is None:
        S = torch.empty(din, dout, dtype=torch.float32, device=X.device)
    ws, wptr, wbytes = _workspace(pex_token_sq_workspace_bytes(B, T, din, dout, dt), X, workspace, stream)
    _invoke(lib().pex_token_sq, _dev(X, "X"), _dev(G, "G"), B, T, din, dout, dt, _f32(S, "S", shape=(din, dout)), wptr, wbytes,
                              _stream(stream))
    return S


def pex_adam_update(theta, m, v, S_id, S_sq, variant, params: AdamParams, stream=None):
    """One in-place step of the Adam family (Algorithm 1).  ``S_sq`` may be None for plain Adam."""
    code = VARIANT.get(variant, variant)
    n = theta.numel()
    _invoke(lib().pex_adam_update, _f32(theta, "theta"), _f32(m, "m", n), _f32(v, "v", n), _f32(S_id, "S_id", n),
                                 _f32(S_sq, "S_sq", n) if S_sq is not None else None, n, code,
                                 ctypes.byref(params), _stream(stream))


def pex_signsgd_update(theta, m, S_sign, lr, beta, weight_decay, B, debias=False, step=1, stream=None):
    """One in-place MicroSignSGD step (EMA o avg o sign)."""
    n = theta.numel()
    _invoke(lib().pex_signsgd_update, _f32(theta, "theta"), _f32(m, "m", n), _f32(S_sign, "S_sign", n), n, lr, beta,
                                    weight_decay, int(B), int(bool(debias)), int(step), _stream(stream))


def pex_sign_update(theta, m, S, variant, lr, beta, weight_decay, B, debias=False, step=1, stream=None):
    """One in-place step of 'microsignsgd' | 'signsgd' | 'signema' (Sec. 3.1); S is the sum of per-example signs for
    the first and the sum of gradients for the other two."""
    n = theta.numel()
    _invoke(lib().pex_sign_update, _f32(theta, "theta"), _f32(m, "m", n), _f32(S, "S", n), n, SIGN_VARIANT.get(variant, variant),
                                 lr, beta, weight_decay, int(B), int(bool(debias)), int(step), _stream(stream))


def pex_moment_track_workspace_bytes(n) -> int:
    return int(lib().pex_moment_track_workspace_bytes(n))


def pex_moment_track(ema_adam, ema_micro, S_id, S_sq, params: MomentParams, sums=None, workspace=None, stream=None):
    """One step of the on-line mu^2 / sigma^2 measurement (Sec. 3.2.2): updates the two EMAs in place and returns a
    float64 tensor [2] = (sum of mu^2-hat, sum of sigma^2-hat) over the parameters."""
    import torch
    n = ema_adam.numel()
    if sums is None:
        sums = torch.empty(2, dtype=torch.float64, device=ema_adam.device)
    ws, wptr, wbytes = _workspace(pex_moment_track_workspace_bytes(n), ema_adam, workspace, stream)
    _invoke(lib().pex_moment_track, _f32(ema_adam, "ema_adam"), _f32(ema_micro, "ema_micro", n), _f32(S_id, "S_id", n),
                                  _f32(S_sq, "S_sq", n), n, ctypes.byref(params), _f64(sums, "sums", 2), wptr, wbytes,
                                  _stream(stream))
    return sums


def pex_embed_stat_workspace_bytes(B, T, V, d) -> int:
    return int(lib().pex_embed_stat_workspace_bytes(B, T, V, d))


def pex_embed_stat(ids, G, V, want, out=None, workspace=None, stream=None):
    """Per-example gradient statistics of an embedding table: ``ids`` [B,T] int32/int64, ``G`` [B,T,d] cotangents of
    the looked-up vectors; returns a dict name -> S[V,d] fp32 for the names in ``want``.  Ids outside [0,V) are padding."""
    import torch
    if ids.dim() != 2 or G.dim() != 3 or tuple(G.shape[:2]) != tuple(ids.shape):
        raise ValueError("ids must be [B,T] and G [B,T,d]")
    if ids.dtype not in (torch.int32, torch.int64):
        raise TypeError(f"ids must be int32 or int64, got {ids.dtype}")
    B, T, d = G.shape
    mask = _want_mask(want)
    res, ptrs = {}, []
    for name, bit in WANT.items():
        if mask & bit:
            S = (out or {}).get(name)
            if S is None:
                S = torch.empty(V, d, dtype=torch.float32, device=G.device)
            res[name] = S
            ptrs.append(_f32(S, name, shape=(V, d)))
        else:
            ptrs.append(None)
    ws, wptr, wbytes = _workspace(pex_embed_stat_workspace_bytes(B, T, V, d), G, workspace, stream)
    _invoke(lib().pex_embed_stat, _dev(ids, "ids"), ids.element_size(), _dev(G, "G"), B, T, V, d, _dtype_code(G), mask,
                                ptrs[0], ptrs[1], ptrs[2], wptr, wbytes, _stream(stream))
    return res


def pex_mfma_probe_operand_bytes() -> int:
    return int(lib().pex_mfma_probe_operand_bytes())


def pex_mfma_probe_sink_floats(workgroups) -> int:
    return int(lib().pex_mfma_probe_sink_floats(int(workgroups)))


def pex_version() -> int:
    return int(lib().pex_version())


def pex_status_string(code: int) -> str:
    return status_string(code)


def pex_mfma_probe(operands, workgroups, iters, sink=None, stream=None):
    """Measurement aid: one launch of nothing but bf16 MFMAs (see ``pex_mfma_probe`` in the header).  ``operands`` is a
    bf16 tensor of at least ``pex_mfma_probe_operand_bytes()`` bytes.  Returns (FLOP of the launch, sink tensor)."""
    import torch
    need = pex_mfma_probe_operand_bytes()
    if operands.numel() * operands.element_size() < need:
        raise ValueError(f"operands must hold at least {need} bytes")
    if sink is None:
        sink = torch.empty(pex_mfma_probe_sink_floats(workgroups), dtype=torch.float32, device=operands.device)
    flop = ctypes.c_double(0.0)
    _invoke(lib().pex_mfma_probe, _dev(operands, "operands"), int(workgroups), int(iters), _f32(sink, "sink"), ctypes.byref(flop),
                                _stream(stream))
    return flop.value, sink


def pex_sum_squares_workspace_bytes(n) -> int:
    return int(lib().pex_sum_squares_workspace_bytes(n))


def pex_sum_squares(x, acc=None, accumulate=False, workspace=None, stream=None):
    """acc[0] (+)= sum of x^2 in fp64 (one double on the GPU): the squared global gradient norm, layer by layer."""
    import torch
    n = x.numel()
    if acc is None:
        acc = torch.zeros(1, dtype=torch.float64, device=x.device)
    ws, wptr, wbytes = _workspace(pex_sum_squares_workspace_bytes(n), x, workspace, stream)
    _invoke(lib().pex_sum_squares, _f32(x, "x"), n, _f64(acc, "acc", 1), int(bool(accumulate)), wptr, wbytes, _stream(stream))
    return acc


def pex_adam_update_clipped(theta, m, v, S_id, S_sq, variant, params: AdamParams, sum_sq, max_norm, stream=None):
    """pex_adam_update with every per-example gradient multiplied by kappa = min(1, max_norm / ||mean gradient||);
    ``sum_sq`` is the double on the GPU that pex_sum_squares accumulated over the S_id of all layers."""
    code = VARIANT.get(variant, variant)
    n = theta.numel()
    _invoke(lib().pex_adam_update_clipped, _f32(theta, "theta"), _f32(m, "m", n), _f32(v, "v", n), _f32(S_id, "S_id", n),
                                         _f32(S_sq, "S_sq", n) if S_sq is not None else None, n, code, ctypes.byref(params),
                                         _f64(sum_sq, "sum_sq", 1), float(max_norm), _stream(stream))
