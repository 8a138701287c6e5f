"""Thin ctypes binding of the C ABI in include/ws_synapse.h.

Same names as the C entry points; argument marshalling only.  PyTorch supplies device
memory (inputs, outputs, workspace) and the current HIP stream; every step of the path runs
in the library's kernels.  There is no CPU fallback: if the library has not been built the
import of a symbol fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import torch

WS_OK, WS_ERR_INVALID_ARG, WS_ERR_UNSUPPORTED, WS_ERR_WORKSPACE, WS_ERR_HIP, WS_ERR_TOO_LARGE = range(6)
WS_F32, WS_BF16 = 0, 1
WS_OP_DENSITY, WS_OP_SELECT, WS_OP_GATHER, WS_OP_ATTEND = range(4)
WS_OP_ATTENTION_MASS, WS_OP_DENSITY_APPEND, WS_OP_INJECT = 4, 5, 6
WS_SELECT_AUTO, WS_SELECT_STREAMING, WS_SELECT_RESIDENT = 0, 1, 2
_SELECT_KERNELS = {"auto": WS_SELECT_AUTO, "stream": WS_SELECT_STREAMING, "resident": WS_SELECT_RESIDENT}

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libws_synapse.so")
_lib = None


class SelectPlan(ctypes.Structure):
    """Mirror of ws_select_plan."""
    _fields_ = [(n, ctypes.c_int) for n in ("resident", "heads_in_flight", "workgroups_per_head", "threads",
                                            "rows_in_registers", "rows_in_lds", "compute_units")]


class WsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2601_01298_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, ci, cf = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float
        L.ws_synapse_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci, ci, ci]
        L.ws_synapse_workspace_bytes.restype = sz
        L.ws_synapse_density.argtypes = [vp, ci, ci, ci, ci, ctypes.POINTER(cf), vp, vp, sz, vp]
        L.ws_synapse_density.restype = ci
        L.ws_synapse_select.argtypes = [vp, ci, ci, ci, ci, vp, ci, cf, vp, vp, vp, sz, vp]
        L.ws_synapse_select.restype = ci
        L.ws_synapse_density_check.argtypes = [vp, ci, vp, ctypes.POINTER(ci), ctypes.POINTER(cf)]
        L.ws_synapse_density_check.restype = ci
        L.ws_synapse_density_is_symmetric.argtypes = [ci, ci, ci]
        L.ws_synapse_density_is_symmetric.restype = ci
        L.ws_synapse_select_with.argtypes = [ci, vp, ci, ci, ci, ci, vp, ci, cf, vp, vp, vp, sz, vp]
        L.ws_synapse_select_with.restype = ci
        L.ws_synapse_select_static.argtypes = [vp, ci, ci, ci, ci, vp, ci, cf, vp, vp, vp]
        L.ws_synapse_select_static.restype = ci
        L.ws_synapse_select_failed.argtypes = [vp, vp, ctypes.POINTER(ci)]
        L.ws_synapse_select_failed.restype = ci
        L.ws_synapse_select_plan.argtypes = [ci, ci, ci, ci, ci, ci, ci, ctypes.POINTER(SelectPlan)]
        L.ws_synapse_select_plan.restype = ci
        L.ws_synapse_gather.argtypes = [vp, vp, ci, ci, ci, ci, vp, ci, vp, vp, vp]
        L.ws_synapse_gather.restype = ci
        L.ws_synapse_attend.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, vp, vp, sz, vp]
        L.ws_synapse_attend.restype = ci
        L.ws_synapse_attend_indexed.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, vp, vp, sz, vp]
        L.ws_synapse_attend_indexed.restype = ci
        L.ws_synapse_attention_mass.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, cf, ci, vp, vp, sz, vp]
        L.ws_synapse_attention_mass.restype = ci
        L.ws_synapse_density_append.argtypes = [vp, ci, ci, ci, ci, ci, ctypes.POINTER(cf), vp, vp, vp, sz, vp]
        L.ws_synapse_density_append.restype = ci
        L.ws_synapse_gate.argtypes = [vp, vp, ci, ci, ci, cf, vp, vp, vp]
        L.ws_synapse_gate.restype = ci
        L.ws_synapse_inject.argtypes = [vp, vp, ci, ci, ci, ci, ci, vp, vp, ci, vp, cf, vp, sz, vp]
        L.ws_synapse_inject.restype = ci
        L.ws_synapse_select_is_resident.argtypes = [ci, ci, ci, ci]
        L.ws_synapse_select_is_resident.restype = ci
        L.ws_status_string.argtypes = [ci]
        L.ws_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().ws_status_string(int(status)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return WS_F32
    if t.dtype == torch.bfloat16:
        return WS_BF16
    raise TypeError(f"unsupported element type {t.dtype}")


def _dev(t: torch.Tensor, name: str) -> torch.Tensor:
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    return t


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _on_stream(stream):
    """Context in which torch allocates for the stream the kernels will run on, so that the caching
    allocator never hands a temporary or an output to other work while those kernels still use it."""
    if stream is None or not hasattr(stream, "cuda_stream"):
        import contextlib
        return contextlib.nullcontext()
    return torch.cuda.stream(stream)


def _workspace(nbytes: int, device, workspace, stream=None):
    if workspace is None:
        with _on_stream(stream):
            workspace = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    elif not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous device tensor")
    return workspace


def _new(shape, dtype, device, stream):
    with _on_stream(stream):
        return torch.empty(shape, dtype=dtype, device=device)


def _want(t: torch.Tensor, name: str, shape, dtype) -> torch.Tensor:
    """Shape, element type, placement and layout of an argument, checked before any pointer is taken."""
    _dev(t, name)
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return t


def _check(status: int, where: str):
    if status != WS_OK:
        raise WsError(status, where)


def ws_synapse_workspace_bytes(op: int, dt: int, H: int, L: int, d: int, k: int = 1, N: int = 1, Hq: int = 1) -> int:
    n = lib().ws_synapse_workspace_bytes(op, dt, H, L, d, k, N, Hq)
    if n == ctypes.c_size_t(-1).value:
        raise WsError(WS_ERR_UNSUPPORTED, "ws_synapse_workspace_bytes")
    return int(n)


def ws_synapse_select_is_resident(dt: int, H: int, L: int, d: int) -> bool:
    return bool(lib().ws_synapse_select_is_resident(dt, H, L, d))


def ws_synapse_density(K: torch.Tensor, sigma, rho: torch.Tensor | None = None, workspace=None, stream=None):
    """K [H,L,d] device; sigma: H host floats -> rho [H,L] fp32 device."""
    _dev(K, "K")
    H, L, d = K.shape
    dt = _dtype_code(K)
    if len(sigma) != H:
        raise ValueError("one bandwidth per head")
    sig = (ctypes.c_float * H)(*[float(s) for s in sigma])
    if rho is None:
        rho = _new((H, L), torch.float32, K.device, stream)
    _want(rho, "rho", (H, L), torch.float32)
    need = ws_synapse_workspace_bytes(WS_OP_DENSITY, dt, H, L, d)
    workspace = _workspace(need, K.device, workspace, stream)
    _check(lib().ws_synapse_density(K.data_ptr(), dt, H, L, d, sig, rho.data_ptr(),
                                    workspace.data_ptr(), workspace.numel(), _stream(stream)), "ws_synapse_density")
    return rho


def ws_synapse_density_check(workspace: torch.Tensor, H: int, stream=None):
    """Waits for the stream; returns (flagged, estimates): whether some head's estimated relative error per kernel
    term exceeded the library's bound in the last density call on this workspace, and the H estimates."""
    flag = ctypes.c_int(0)
    est = (ctypes.c_float * H)()
    _check(lib().ws_synapse_density_check(_dev(workspace, "workspace").data_ptr(), int(H), _stream(stream),
                                          ctypes.byref(flag), est), "ws_synapse_density_check")
    return bool(flag.value), list(est)


def ws_synapse_density_is_symmetric(dt: int, L: int, d: int) -> bool:
    return bool(lib().ws_synapse_density_is_symmetric(dt, L, d))


def ws_synapse_select(K: torch.Tensor, rho: torch.Tensor, k: int, alpha: float, idx: torch.Tensor | None = None,
                      score_out: torch.Tensor | None = None, workspace=None, stream=None, want_score: bool = False,
                      kernel: str = "auto", check: bool = True):
    """K [H,L,d], rho [H,L] fp32 -> idx [H,k] int32 (and the winning scores [H,k] when asked).

    kernel: "auto" (the library picks), "stream" or "resident" (ws_synapse_select_with).
    check:  read the selection's failure flag back afterwards (this waits for the stream) and raise if
            the kernel gave up; pass False inside graph capture or when the host must not wait, and call
            ws_synapse_select_failed on the workspace later."""
    _dev(K, "K")
    H, L, d = K.shape
    dt = _dtype_code(K)
    _want(rho, "rho", (H, L), torch.float32)
    if idx is None:
        idx = _new((H, k), torch.int32, K.device, stream)
    _want(idx, "idx", (H, k), torch.int32)
    if score_out is None and want_score:
        score_out = _new((H, k), torch.float32, K.device, stream)
    if score_out is not None:
        _want(score_out, "score_out", (H, k), torch.float32)
    need = ws_synapse_workspace_bytes(WS_OP_SELECT, dt, H, L, d, k)
    workspace = _workspace(need, K.device, workspace, stream)
    _check(lib().ws_synapse_select_with(_SELECT_KERNELS[kernel], K.data_ptr(), dt, H, L, d, rho.data_ptr(), int(k),
                                        float(alpha), idx.data_ptr(),
                                        score_out.data_ptr() if score_out is not None else None,
                                        workspace.data_ptr(), workspace.numel(), _stream(stream)), "ws_synapse_select")
    if check and ws_synapse_select_failed(workspace, stream):
        raise WsError(WS_ERR_HIP, "ws_synapse_select: a wait between workgroups expired (the grid was not "
                                  "co-resident); idx holds -1 entries")
    return (idx, score_out) if (want_score or score_out is not None) else idx


def ws_synapse_select_with(kernel: str, K, rho, k, alpha, **kw):
    """ws_synapse_select with the kernel named: "stream" or "resident"."""
    return ws_synapse_select(K, rho, k, alpha, kernel=kernel, **kw)


def ws_synapse_select_static(K: torch.Tensor, rho: torch.Tensor, k: int, alpha: float, idx: torch.Tensor,
                             score_out: torch.Tensor | None = None, stream=None):
    """ws_synapse_select on the library's own fixed scratch: nothing is allocated here or in the library, so
    the caller supplies idx [H,k] int32 (and score_out [H,k] fp32 if wanted)."""
    _dev(K, "K")
    H, L, d = K.shape
    dt = _dtype_code(K)
    _want(rho, "rho", (H, L), torch.float32)
    _want(idx, "idx", (H, k), torch.int32)
    if score_out is not None:
        _want(score_out, "score_out", (H, k), torch.float32)
    _check(lib().ws_synapse_select_static(K.data_ptr(), dt, H, L, d, rho.data_ptr(), int(k), float(alpha), idx.data_ptr(),
                                          score_out.data_ptr() if score_out is not None else None, _stream(stream)),
           "ws_synapse_select_static")
    return idx


def ws_synapse_select_failed(workspace: torch.Tensor | None, stream=None) -> bool:
    """Waits for the stream, then reports whether the last selection on this workspace gave up
    (workspace None: the fixed scratch of ws_synapse_select_static)."""
    out = ctypes.c_int(0)
    ptr = _dev(workspace, "workspace").data_ptr() if workspace is not None else None
    _check(lib().ws_synapse_select_failed(ptr, _stream(stream), ctypes.byref(out)), "ws_synapse_select_failed")
    return bool(out.value)


def ws_synapse_select_plan(kernel: str, dt: int, H: int, L: int, d: int, compute_units: int = 0,
                           workgroups_per_cu: int = 0) -> SelectPlan:
    """How a selection of these sizes would be launched (0 = ask the current device)."""
    plan = SelectPlan()
    _check(lib().ws_synapse_select_plan(_SELECT_KERNELS[kernel], dt, H, L, d, compute_units, workgroups_per_cu,
                                        ctypes.byref(plan)), "ws_synapse_select_plan")
    return plan


def ws_synapse_gather(K: torch.Tensor, V: torch.Tensor, idx: torch.Tensor, Ks: torch.Tensor | None = None,
                      Vs: torch.Tensor | None = None, stream=None):
    """K,V [H,L,d], idx [H,k] -> Ks,Vs [H,k,d] (bit copies in pick order)."""
    _dev(K, "K")
    H, L, d = K.shape
    dt = _dtype_code(K)
    _want(V, "V", (H, L, d), K.dtype)
    if idx.dim() != 2:
        raise ValueError("idx must be [H,k]")
    k = idx.shape[1]
    _want(idx, "idx", (H, k), torch.int32)
    if Ks is None:
        Ks = _new((H, k, d), K.dtype, K.device, stream)
    if Vs is None:
        Vs = _new((H, k, d), K.dtype, K.device, stream)
    _want(Ks, "Ks", (H, k, d), K.dtype)
    _want(Vs, "Vs", (H, k, d), K.dtype)
    _check(lib().ws_synapse_gather(K.data_ptr(), V.data_ptr(), dt, H, L, d, idx.data_ptr(), k,
                                   Ks.data_ptr(), Vs.data_ptr(), _stream(stream)),
           "ws_synapse_gather")
    return Ks, Vs


def ws_synapse_attend(Q: torch.Tensor, Ks: torch.Tensor, Vs: torch.Tensor, scale: float = 0.0,
                      O: torch.Tensor | None = None, workspace=None, stream=None):
    """Q [N,Hq,d], Ks,Vs [Hkv,k,d] -> O [N,Hq,d] fp32.  scale <= 0 means 1/sqrt(d)."""
    _dev(Q, "Q")
    _dev(Ks, "Ks")
    if Q.dim() != 3 or Ks.dim() != 3:
        raise ValueError("Q must be [N,Hq,d] and Ks [Hkv,k,d]")
    N, Hq, d = Q.shape
    Hkv, k, dk = Ks.shape
    dt = _dtype_code(Q)
    if dk != d:
        raise ValueError(f"Q has head dimension {d}, Ks {dk}")
    _want(Ks, "Ks", (Hkv, k, d), Q.dtype)
    _want(Vs, "Vs", (Hkv, k, d), Q.dtype)
    if O is None:
        O = _new((N, Hq, d), torch.float32, Q.device, stream)
    _want(O, "O", (N, Hq, d), torch.float32)
    need = ws_synapse_workspace_bytes(WS_OP_ATTEND, dt, Hkv, k, d, k, N, Hq)
    if need or workspace is not None:
        workspace = _workspace(need, Q.device, workspace, stream)
    wptr, wlen = (workspace.data_ptr(), workspace.numel()) if workspace is not None else (None, 0)
    _check(lib().ws_synapse_attend(Q.data_ptr(), Ks.data_ptr(), Vs.data_ptr(), dt, N, Hq, Hkv, k, d, float(scale),
                                   O.data_ptr(), wptr, wlen, _stream(stream)), "ws_synapse_attend")
    return O


def ws_synapse_attend_indexed(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, idx: torch.Tensor, scale: float = 0.0,
                              O: torch.Tensor | None = None, workspace=None, stream=None):
    """Q [N,Hq,d], K,V [Hkv,L,d], idx [Hkv,k] int32 -> O [N,Hq,d] fp32: gather and attend in one pass."""
    _dev(Q, "Q")
    _dev(K, "K")
    if Q.dim() != 3 or K.dim() != 3 or idx.dim() != 2:
        raise ValueError("Q must be [N,Hq,d], K [Hkv,L,d] and idx [Hkv,k]")
    N, Hq, d = Q.shape
    Hkv, L, dk = K.shape
    k = idx.shape[1]
    dt = _dtype_code(Q)
    if dk != d:
        raise ValueError(f"Q has head dimension {d}, K {dk}")
    _want(K, "K", (Hkv, L, d), Q.dtype)
    _want(V, "V", (Hkv, L, d), Q.dtype)
    _want(idx, "idx", (Hkv, k), torch.int32)
    if O is None:
        O = _new((N, Hq, d), torch.float32, Q.device, stream)
    _want(O, "O", (N, Hq, d), torch.float32)
    need = ws_synapse_workspace_bytes(WS_OP_ATTEND, dt, Hkv, k, d, k, N, Hq)
    if need or workspace is not None:
        workspace = _workspace(need, Q.device, workspace, stream)
    wptr, wlen = (workspace.data_ptr(), workspace.numel()) if workspace is not None else (None, 0)
    _check(lib().ws_synapse_attend_indexed(Q.data_ptr(), K.data_ptr(), V.data_ptr(), idx.data_ptr(), dt, N, Hq, Hkv, L,
                                           k, d, float(scale), O.data_ptr(), wptr, wlen, _stream(stream)),
           "ws_synapse_attend_indexed")
    return O


def ws_synapse_attention_mass(K: torch.Tensor, Q: torch.Tensor, G: int, scale: float = 0.0, as_density: bool = True,
                              out: torch.Tensor | None = None, workspace=None, stream=None):
    """K [G*Hkv,L,d], Q [G*Hq,d] -> out [G*Hkv,L] fp32 (1/A when as_density, else A)."""
    _dev(K, "K")
    GHkv, L, d = K.shape
    GHq = Q.shape[0]
    _want(Q, "Q", (GHq, d), K.dtype)
    if GHkv % G or GHq % G:
        raise ValueError("head counts must be multiples of the number of groups")
    dt = _dtype_code(K)
    if out is None:
        out = _new((GHkv, L), torch.float32, K.device, stream)
    _want(out, "out", (GHkv, L), torch.float32)
    need = ws_synapse_workspace_bytes(WS_OP_ATTENTION_MASS, dt, GHkv, L, d, Hq=GHq)
    workspace = _workspace(need, K.device, workspace, stream)
    _check(lib().ws_synapse_attention_mass(K.data_ptr(), Q.data_ptr(), dt, G, GHkv // G, GHq // G, L, d, float(scale),
                                           int(bool(as_density)), _dev(out, "out").data_ptr(), workspace.data_ptr(),
                                           workspace.numel(), _stream(stream)), "ws_synapse_attention_mass")
    return out


def ws_synapse_density_append(K: torch.Tensor, m: int, sigma, rho_old: torch.Tensor, rho_new: torch.Tensor | None = None,
                              workspace=None, stream=None):
    """K [H,L,d] with the m new rows last, rho_old [H,L-m] -> rho_new [H,L]."""
    _dev(K, "K")
    _dev(rho_old, "rho_old")
    H, L, d = K.shape
    dt = _dtype_code(K)
    _want(rho_old, "rho_old", (H, L - m), torch.float32)
    if len(sigma) != H:
        raise ValueError("one bandwidth per head")
    sig = (ctypes.c_float * H)(*[float(s) for s in sigma])
    if rho_new is None:
        rho_new = _new((H, L), torch.float32, K.device, stream)
    _want(rho_new, "rho_new", (H, L), torch.float32)
    need = ws_synapse_workspace_bytes(WS_OP_DENSITY_APPEND, dt, H, L, d)
    workspace = _workspace(need, K.device, workspace, stream)
    _check(lib().ws_synapse_density_append(K.data_ptr(), dt, H, L, d, int(m), sig, rho_old.data_ptr(),
                                           _dev(rho_new, "rho_new").data_ptr(), workspace.data_ptr(), workspace.numel(),
                                           _stream(stream)), "ws_synapse_density_append")
    return rho_new


def ws_synapse_gate(h_main: torch.Tensor, T: torch.Tensor, theta: float, score: torch.Tensor | None = None,
                    accept: torch.Tensor | None = None, stream=None):
    """h_main [dm], T [N,dm] -> (score [N] fp32, accept [N] int32)."""
    _dev(h_main, "h_main")
    _dev(T, "T")
    N, dm = T.shape
    dt = _dtype_code(T)
    if h_main.dtype != T.dtype or h_main.numel() != dm:
        raise ValueError("h_main must have T's element type and dm elements")
    if score is None:
        score = _new((N,), torch.float32, T.device, stream)
    if accept is None:
        accept = _new((N,), torch.int32, T.device, stream)
    _want(score, "score", (N,), torch.float32)
    _want(accept, "accept", (N,), torch.int32)
    _check(lib().ws_synapse_gate(h_main.data_ptr(), T.data_ptr(), dt, N, dm, float(theta), score.data_ptr(),
                                 accept.data_ptr(), _stream(stream)), "ws_synapse_gate")
    return score, accept


def ws_synapse_inject(Kc: torch.Tensor, Vc: torch.Tensor, L: int, Knew: torch.Tensor, Vnew: torch.Tensor,
                      pos: torch.Tensor, base: float, workspace=None, stream=None):
    """Kc,Vc [H,Lcap,d] caches with L rows in use; Knew,Vnew [H,m,d]; pos [m] int32.  Writes rows L..L+m-1."""
    for t, name in ((Kc, "Kc"), (Vc, "Vc"), (Knew, "Knew"), (Vnew, "Vnew"), (pos, "pos")):
        _dev(t, name)
    H, Lcap, d = Kc.shape
    m = Knew.shape[1]
    dt = _dtype_code(Kc)
    _want(Vc, "Vc", (H, Lcap, d), Kc.dtype)
    _want(Knew, "Knew", (H, m, d), Kc.dtype)
    _want(Vnew, "Vnew", (H, m, d), Kc.dtype)
    _want(pos, "pos", (m,), torch.int32)
    need = ws_synapse_workspace_bytes(WS_OP_INJECT, dt, H, Lcap, d, k=m)
    workspace = _workspace(need, Kc.device, workspace, stream)
    _check(lib().ws_synapse_inject(Kc.data_ptr(), Vc.data_ptr(), dt, H, Lcap, d, int(L), Knew.data_ptr(), Vnew.data_ptr(),
                                   m, pos.data_ptr(), float(base), workspace.data_ptr(), workspace.numel(),
                                   _stream(stream)), "ws_synapse_inject")
    return L + m
