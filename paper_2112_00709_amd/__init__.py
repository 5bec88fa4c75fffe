"""Python binding of libfb_amd.so (include/fb.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch is used for
device memory and the current stream, nothing else.  There is no CPU fallback:
if the shared library is missing or a call fails, an exception is raised.

The functions carry the names of the C entry points:
``fb_graph_create``, ``fb_graph_layout``, ``fb_alpha``, ``fb_beta``,
``fb_posteriors``, ``lfmmi_loss_grad``.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfb_amd.so")

FB_OK, FB_EINVAL, FB_ENOMEM, FB_EHIP, FB_EUNSUPPORTED = 0, -1, -2, -3, -4
FB_GRAPH_HOST_ONLY, FB_GRAPH_WIDE_STATE, FB_GRAPH_NARROW_STATE = 1, 2, 4
LAYOUT = {"in_ptr": 0, "in_src": 1, "in_w": 2, "in_perm": 3, "out_ptr": 4, "out_dst": 5, "out_w": 6,
          "out_perm": 7, "pdf_ptr": 8, "pdf_states": 9}

# every symbol include/fb.h declares
SYMBOLS = ["fb_graph_create", "fb_graph_destroy", "fb_graph_layout_size", "fb_graph_layout", "fb_check_lengths",
           "fb_alpha", "fb_beta", "fb_posteriors", "fb_lfmmi_workspace_bytes", "lfmmi_loss_grad", "lfmmi_loss_grad_ragged",
           "fb_limits_max_states", "fb_strerror", "fb_last_error", "fb_graph_schedule_apply_host",
           "fb_profile_enable", "fb_profile_read", "fb_viterbi_workspace_bytes", "fb_viterbi", "fb_graph_linear_weights",
           "fb_debug_linear_restarts", "fb_graph_plan_cycles", "lfmmi_loss_grad_static", "fb_static_scratch_bytes",
           "fb_leaky_workspace_bytes", "fb_leaky_posteriors"]


class FBError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libfb_amd error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """Load the built library (fails loudly when it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        # PyTorch first: it ships its own HIP runtime, and the library must bind to that copy (loading the
        # system's runtime before it leaves PyTorch without a GPU)
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_size_t
        L.fb_graph_create.argtypes = [ctypes.POINTER(vp), i32, i64, vp, vp, vp, vp, vp, vp, i32, i32, vp, u32]
        L.fb_graph_create.restype = ctypes.c_int
        L.fb_graph_destroy.argtypes = [vp]
        L.fb_graph_destroy.restype = ctypes.c_int
        L.fb_graph_layout_size.argtypes = [vp, ctypes.c_int]
        L.fb_graph_layout_size.restype = i64
        L.fb_graph_layout.argtypes = [vp, ctypes.c_int, vp, sz]
        L.fb_graph_layout.restype = ctypes.c_int
        L.fb_graph_schedule_apply_host.argtypes = [vp, ctypes.c_int, i32, vp, vp]
        L.fb_graph_schedule_apply_host.restype = ctypes.c_int
        L.fb_check_lengths.argtypes = [vp, i32, i32]
        L.fb_check_lengths.restype = ctypes.c_int
        L.fb_alpha.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp]
        L.fb_alpha.restype = ctypes.c_int
        L.fb_beta.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp]
        L.fb_beta.restype = ctypes.c_int
        L.fb_posteriors.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, vp]
        L.fb_posteriors.restype = ctypes.c_int
        L.fb_lfmmi_workspace_bytes.argtypes = [vp, vp, i32, i32, i32]
        L.fb_lfmmi_workspace_bytes.restype = sz
        L.lfmmi_loss_grad_static.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp]
        L.lfmmi_loss_grad_static.restype = ctypes.c_int
        L.fb_static_scratch_bytes.argtypes = []
        L.fb_static_scratch_bytes.restype = sz
        L.lfmmi_loss_grad.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.lfmmi_loss_grad.restype = ctypes.c_int
        L.lfmmi_loss_grad_ragged.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp]
        L.lfmmi_loss_grad_ragged.restype = ctypes.c_int
        L.fb_graph_linear_weights.argtypes = [vp]
        L.fb_graph_linear_weights.restype = ctypes.c_int
        L.fb_graph_plan_cycles.argtypes = [vp, ctypes.c_int, vp, vp]
        L.fb_graph_plan_cycles.restype = ctypes.c_int
        L.fb_debug_linear_restarts.argtypes = []
        L.fb_debug_linear_restarts.restype = i64
        L.fb_limits_max_states.argtypes = [i32, ctypes.c_int]
        L.fb_limits_max_states.restype = i32
        L.fb_viterbi_workspace_bytes.argtypes = [vp, i32, i32]
        L.fb_viterbi_workspace_bytes.restype = sz
        L.fb_viterbi.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
        L.fb_viterbi.restype = ctypes.c_int
        L.fb_leaky_workspace_bytes.argtypes = [vp, i32, i32]
        L.fb_leaky_workspace_bytes.restype = sz
        L.fb_leaky_posteriors.argtypes = [vp, vp, vp, i32, i32, i32, ctypes.c_float, vp, vp, vp, sz, vp]
        L.fb_leaky_posteriors.restype = ctypes.c_int
        L.fb_profile_enable.argtypes = [ctypes.c_int]
        L.fb_profile_enable.restype = ctypes.c_int
        L.fb_profile_read.argtypes = [vp]
        L.fb_profile_read.restype = ctypes.c_int
        L.fb_strerror.argtypes = [ctypes.c_int]
        L.fb_strerror.restype = ctypes.c_char_p
        L.fb_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != FB_OK:
        raise FBError(rc, (lib().fb_last_error() or b"").decode() or lib().fb_strerror(rc).decode())


def _np(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _hp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


class Graph:
    """Owner of an ``fb_graph*``."""

    def __init__(self, handle, K, E, D, n_seq, host_only):
        self._h, self.K, self.E, self.D, self.n_seq, self.host_only = handle, K, E, D, n_seq, host_only

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("graph already destroyed")
        return self._h

    @property
    def shared(self) -> bool:
        return self.n_seq == 0

    def destroy(self) -> None:
        if self._h is not None:
            h, self._h = self._h, None
            _check(lib().fb_graph_destroy(h))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def fb_graph_create(K, src, dst, logw, pdf, init, final, D, state_off=None, host_only=False, state="auto") -> Graph:
    """state: 'auto', 'wide' (double carriers) or 'narrow' (single carriers)."""
    flags = (FB_GRAPH_HOST_ONLY if host_only else 0) | {"auto": 0, "wide": FB_GRAPH_WIDE_STATE, "narrow": FB_GRAPH_NARROW_STATE}[state]
    src, dst, logw = _np(src, np.int32), _np(dst, np.int32), _np(logw, np.float32)
    pdf, init, final = _np(pdf, np.int32), _np(init, np.float32), _np(final, np.float32)
    state_off = _np(state_off, np.int32)
    E = 0 if src is None else int(src.shape[0])
    n_seq = 0 if state_off is None else int(state_off.shape[0]) - 1
    h = ctypes.c_void_p()
    _check(lib().fb_graph_create(ctypes.byref(h), int(K), E, _hp(src), _hp(dst), _hp(logw), _hp(pdf), _hp(init),
                                 _hp(final), int(D), n_seq, _hp(state_off), flags))
    return Graph(h, int(K), E, int(D), n_seq, host_only)


def graph_from(g, D: int, host_only: bool = False, state: str = "auto") -> Graph:
    """Build from an object with fields K, src, dst, logw, pdf, init, final, state_off."""
    return fb_graph_create(g.K, g.src, g.dst, g.logw, g.pdf, g.init, g.final, D, g.state_off, host_only, state)


def fb_graph_layout(g: Graph, name: str) -> np.ndarray:
    which = LAYOUT[name]
    n = lib().fb_graph_layout_size(g.handle, which)
    if n < 0:
        _check(int(n))
    out = np.empty(int(n), dtype=np.float32 if name.endswith("_w") else np.int32)
    _check(lib().fb_graph_layout(g.handle, which, _hp(out), out.nbytes))
    return out


def fb_graph_schedule_apply_host(g: Graph, which: int, sub: int, x: np.ndarray, y: np.ndarray) -> np.ndarray:
    x = _np(x, np.float64)
    assert y.dtype == np.float64 and y.flags.c_contiguous
    _check(lib().fb_graph_schedule_apply_host(g.handle, which, sub, _hp(x), _hp(y)))
    return y


def fb_check_lengths(lengths, N: int) -> None:
    lengths = _np(lengths, np.int32)
    _check(lib().fb_check_lengths(_hp(lengths), int(lengths.shape[0]), int(N)))


def fb_profile_enable(on: bool) -> None:
    _check(lib().fb_profile_enable(1 if on else 0))


def fb_profile_read() -> dict:
    """Milliseconds of the stages of the latest lfmmi_loss_grad call (waits for it)."""
    ms = (ctypes.c_float * 4)()
    _check(lib().fb_profile_read(ctypes.cast(ms, ctypes.c_void_p)))
    return {"num_recursion": ms[0], "den_recursion": ms[1], "posteriors_grad": ms[2], "loss": ms[3]}


def fb_graph_linear_weights(g: Graph) -> int:
    """Diagnostic: 0 the graph's recursions add weights in the exponent, 1 they multiply by 2^w, 2 they run in the
    probability domain (and fall back to form 0 where a sequence leaves its range)."""
    return int(lib().fb_graph_linear_weights(g.handle))


def fb_graph_plan_cycles(g: Graph, backward: bool):
    """Diagnostic: (modelled on-chip memory cycles of one time step's gathers, the floor of two per gather)."""
    c, f = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().fb_graph_plan_cycles(g.handle, 1 if backward else 0, ctypes.byref(c), ctypes.byref(f)))
    return int(c.value), int(f.value)


def fb_debug_linear_restarts() -> int:
    """Diagnostic: runs the probability-domain kernel has redone in the log form so far (synchronises)."""
    return int(lib().fb_debug_linear_restarts())


def fb_limits_max_states(D: int, shared: bool) -> int:
    return int(lib().fb_limits_max_states(int(D), 1 if shared else 0))


# ----------------------------------------------------------------- device calls

def _torch():
    import torch
    return torch


def _dp(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


# Tests set this to have every buffer the binding allocates for an output or a workspace start out as NaN
# (all bits set) instead of whatever the allocator hands back: a kernel that leaves part of an output unwritten,
# or reads workspace it has not written in the same call, then cannot pass by luck.
POISON_NEW_BUFFERS = False


def _new(shape, dtype, device):
    torch = _torch()
    t = torch.empty(shape, dtype=dtype, device=device)
    if POISON_NEW_BUFFERS:
        t.view(torch.uint8).fill_(255)
    return t


def _stream():
    return ctypes.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _dev_inputs(emis, lengths):
    torch = _torch()
    if not (emis.is_cuda and emis.dtype == torch.float32 and emis.is_contiguous() and emis.dim() == 3):
        raise ValueError("emis must be a contiguous float32 CUDA tensor [B, N, D]")
    if not (lengths.is_cuda and lengths.dtype == torch.int32 and lengths.is_contiguous()
            and lengths.shape == (emis.shape[0],)):
        raise ValueError("lengths must be a contiguous int32 CUDA tensor [B]")
    return tuple(int(s) for s in emis.shape)


def _vec_shape(g: Graph, B: int, N: int):
    return (B, N, g.K) if g.shared else (N, g.K)


def _recursion(fn, g: Graph, emis, lengths, want_vectors: bool):
    torch = _torch()
    B, N, D = _dev_inputs(emis, lengths)
    vec = _new(_vec_shape(g, B, N), torch.float32, emis.device) if want_vectors else None
    off = _new((B, N), torch.float64, emis.device)
    logz = _new((B,), torch.float64, emis.device)
    _check(fn(g.handle, _dp(emis), _dp(lengths), B, N, D, _dp(vec), _dp(off), _dp(logz), _stream()))
    return vec, off, logz


def fb_alpha(g: Graph, emis, lengths, want_vectors: bool = True):
    """-> (alpha, alpha_cum [B,N] float64, logz [B]); alpha is [B,N,K] (shared) or [N,K] (packed); the true row of
    frame n is alpha[.., n, :] + alpha_cum[b, n]."""
    return _recursion(lib().fb_alpha, g, emis, lengths, want_vectors)


def fb_beta(g: Graph, emis, lengths, want_vectors: bool = True):
    """-> (beta, beta_cum [B,N] float64, logz [B])."""
    return _recursion(lib().fb_beta, g, emis, lengths, want_vectors)


def fb_posteriors(g: Graph, alpha, beta, lengths, B: int, N: int, want_state: bool = True, want_pdf: bool = True):
    """-> (state_post like alpha, pdf_post [B,N,D])."""
    torch = _torch()
    state = _new(tuple(alpha.shape), torch.float32, alpha.device) if want_state else None
    pdfp = _new((B, N, g.D), torch.float32, alpha.device) if want_pdf else None
    _check(lib().fb_posteriors(g.handle, _dp(alpha), _dp(beta), _dp(lengths), B, N, g.D, _dp(state), _dp(pdfp), _stream()))
    return state, pdfp


def fb_lfmmi_workspace_bytes(den: Graph, num: Graph, B: int, N: int, D: int) -> int:
    return int(lib().fb_lfmmi_workspace_bytes(den.handle, num.handle, B, N, D))


def fb_leaky_workspace_bytes(g: Graph, B: int, N: int) -> int:
    return int(lib().fb_leaky_workspace_bytes(g.handle, B, N))


def fb_leaky_posteriors(g: Graph, emis, lengths, leak: float, ws=None):
    """Leaky-HMM comparison mode -> (logz [B] float64, pdf_post [B,N,D]), on the device."""
    torch = _torch()
    B, N, D = _dev_inputs(emis, lengths)
    need = int(lib().fb_leaky_workspace_bytes(g.handle, B, N))
    if ws is None:
        ws = _new((need,), torch.uint8, emis.device)
    logz = _new((B,), torch.float64, emis.device)
    post = _new((B, N, D), torch.float32, emis.device)
    _check(lib().fb_leaky_posteriors(g.handle, _dp(emis), _dp(lengths), B, N, D, float(leak), _dp(logz), _dp(post), _dp(ws),
                                     int(ws.numel()), _stream()))
    return logz, post


def fb_viterbi(g: Graph, emis, lengths, ws=None):
    """-> (score [B] float64, path [B,N] int32), on the device."""
    torch = _torch()
    B, N, D = _dev_inputs(emis, lengths)
    need = int(lib().fb_viterbi_workspace_bytes(g.handle, B, N))
    if ws is None:
        ws = _new((need,), torch.uint8, emis.device)
    score = _new((B,), torch.float64, emis.device)
    path = _new((B, N), torch.int32, emis.device)
    _check(lib().fb_viterbi(g.handle, _dp(emis), _dp(lengths), B, N, D, _dp(score), _dp(path), _dp(ws), int(ws.numel()),
                            _stream()))
    return score, path


def fb_static_scratch_bytes() -> int:
    """Bytes of the scratch memory built into the library (what lfmmi_loss_grad_static can use as workspace)."""
    return int(lib().fb_static_scratch_bytes())


def lfmmi_loss_grad_static(den: Graph, num: Graph, emis, lengths, loss, logz_num, logz_den, grad):
    """lfmmi_loss_grad for callers that cannot allocate: the workspace is the library's built-in scratch memory and
    every output is the caller's (loss [1] float64, logz_num / logz_den [B] float64, grad [B,N,D] float32, all on
    the device).  Raises FBError(FB_EUNSUPPORTED) when the sizes need more than fb_static_scratch_bytes()."""
    B, N, D = _dev_inputs(emis, lengths)
    _check(lib().lfmmi_loss_grad_static(den.handle, num.handle, _dp(emis), _dp(lengths), B, N, D, _dp(loss), _dp(logz_num),
                                        _dp(logz_den), _dp(grad), _stream()))
    return loss, logz_num, logz_den, grad


def lfmmi_loss_grad(den: Graph, num: Graph, emis, lengths, ws=None, grad=None, lengths_host=None):
    """-> (loss [1] float64, logz_num [B], logz_den [B], grad [B,N,D]), all on the device.
    ``ws`` (uint8 CUDA tensor of fb_lfmmi_workspace_bytes) and ``grad`` may be passed in for reuse.
    ``lengths_host``: a host copy of ``lengths`` (numpy int32 or a sequence); with it the call goes to
    lfmmi_loss_grad_ragged, which picks the schedule of the call's launches from them (same results to rounding)."""
    torch = _torch()
    B, N, D = _dev_inputs(emis, lengths)
    need = fb_lfmmi_workspace_bytes(den, num, B, N, D)
    if ws is None:
        ws = _new((need,), torch.uint8, emis.device)
    if grad is None:
        grad = _new((B, N, D), torch.float32, emis.device)
    loss = _new((1,), torch.float64, emis.device)
    zn = _new((B,), torch.float64, emis.device)
    zd = _new((B,), torch.float64, emis.device)
    if lengths_host is not None:
        lh = np.ascontiguousarray(np.asarray(lengths_host), dtype=np.int32)
        if lh.shape != (B,):
            raise ValueError("lengths_host must hold one length per sequence")
        _check(lib().lfmmi_loss_grad_ragged(den.handle, num.handle, _dp(emis), _dp(lengths), lh.ctypes.data_as(ctypes.c_void_p),
                                            B, N, D, _dp(loss), _dp(zn), _dp(zd), _dp(grad), _dp(ws), int(ws.numel()),
                                            _stream()))
    else:
        _check(lib().lfmmi_loss_grad(den.handle, num.handle, _dp(emis), _dp(lengths), B, N, D, _dp(loss), _dp(zn), _dp(zd),
                                     _dp(grad), _dp(ws), int(ws.numel()), _stream()))
    return loss, zn, zd, grad
