"""Thin ctypes binding of the lnpegn C ABI (include/lnpegn.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
Tensors are torch tensors on the GPU (torch is used for device memory and streams and for
nothing else); results are returned in freshly allocated torch tensors unless the caller
passes output buffers.  A missing or unloadable library raises -- there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

from . import build as _build

F32, BF16 = 0, 1
STATUS = {0: "LNPEGN_OK", 1: "LNPEGN_EINVAL", 2: "LNPEGN_EUNSUPPORTED", 3: "LNPEGN_EWORKSPACE",
          4: "LNPEGN_EHIP"}
STATIC_SCRATCH_BYTES = 64 << 20     # LNPEGN_STATIC_SCRATCH_BYTES of the header
EXPORTS = ("lnpegn_workspace_bytes", "lnpegn_status_string", "lnpegn_last_hip_error", "ln_fwd_stats", "ln_bwd",
           "ln_bwd_pegn", "ln_bwd_pegn_static", "gns_estimate", "lnpegn_set_tuning", "lnpegn_plan_query",
           "lnpegn_set_profile_events", "lnpegn_stream_probe", "ln_bwd_deferred", "ln_bwd_pegn_deferred", "lnpegn_reduce_deferred",
           "ln_fwd", "ln_bwd_ex", "rms_fwd", "rms_bwd_ex",
           "gns_ema_update", "gns_offline", "gns_linear_accum_steps",
           "linear_pegn_workspace_bytes", "linear_pegn", "embedding_pegn_workspace_bytes", "embedding_pegn",
           "embedding_sort_ids", "embedding_pegn_presorted")
PER_EXAMPLE, DEFER, ACCUMULATE = 1, 2, 4

_lib = None


class LnpegnError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        detail = ""
        if status == 4 and _lib is not None:          # LNPEGN_EHIP: say which HIP error, if the library kept it
            try:
                detail = f" (hipError_t {_lib.lnpegn_last_hip_error()})"
            except AttributeError:
                pass
        super().__init__(f"{fn} returned {STATUS.get(status, status)}{detail}")


def lib_path() -> str:
    return _build.LIB


def load() -> ctypes.CDLL:
    """Load liblnpegn.so (building it only when no library exists yet)."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.ensure_built()
    # torch ships a HIP runtime of its own; it must be in the process before this library is loaded, so that
    # both bind to that one copy (loaded first, this library would pull in the system's copy beside torch's,
    # and kernel launches then fail with hipErrorNoDevice)
    import torch  # noqa: F401
    lib = ctypes.CDLL(path)
    vp, fp, i, f, sz = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.lnpegn_workspace_bytes.argtypes = [i, i, i, i]
    lib.lnpegn_workspace_bytes.restype = sz
    lib.lnpegn_status_string.argtypes = [i]
    lib.lnpegn_status_string.restype = ctypes.c_char_p
    lib.ln_fwd_stats.argtypes = [vp, fp, fp, i, i, i, i, f, vp]
    lib.ln_bwd.argtypes = [vp, vp, vp, fp, fp, vp, fp, fp, i, i, i, i, i, f, vp, sz, vp]
    lib.ln_bwd_pegn.argtypes = [vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, i, i, i, i, i, f, vp, sz, vp]
    lib.ln_bwd_pegn_static.argtypes = [vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, i, i, i, i, i, f, vp]
    lib.ln_bwd_deferred.argtypes = lib.ln_bwd.argtypes
    lib.ln_bwd_pegn_deferred.argtypes = lib.ln_bwd_pegn.argtypes
    lib.lnpegn_reduce_deferred.argtypes = [ctypes.POINTER(ctypes.c_void_p), i, i, i, i, i, vp]
    lib.ln_fwd.argtypes = [vp, vp, vp, vp, fp, fp, i, i, i, i, i, f, vp]
    lib.ln_bwd_ex.argtypes = [vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, i, i, i, i, i, f, vp, sz,
                              ctypes.c_uint, vp]
    lib.gns_ema_update.argtypes = [vp, fp, i, ctypes.c_double, fp, vp]
    lib.gns_offline.argtypes = [fp, ctypes.c_int64, fp, vp]
    lib.gns_linear_accum_steps.argtypes = [ctypes.c_int64, ctypes.c_int64, i]
    lib.linear_pegn_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.linear_pegn_workspace_bytes.restype = sz
    lib.linear_pegn.argtypes = [vp, vp, fp, fp, fp, i, i, i, i, i, vp, sz, ctypes.c_uint, vp]
    lib.embedding_pegn_workspace_bytes.argtypes = [i, i, i, i]
    lib.embedding_pegn_workspace_bytes.restype = sz
    lib.embedding_pegn.argtypes = [vp, i, vp, fp, fp, fp, i, i, i, i, i, vp, sz, ctypes.c_uint, vp]
    lib.embedding_sort_ids.argtypes = [vp, i, i, i, i, vp, vp, vp, sz, vp]
    lib.embedding_pegn_presorted.argtypes = [vp, vp, vp, fp, fp, fp, i, i, i, i, i, vp, sz, ctypes.c_uint, vp]
    lib.rms_fwd.argtypes = [vp, vp, vp, fp, i, i, i, i, i, f, vp]
    lib.rms_bwd_ex.argtypes = [vp, vp, vp, fp, vp, fp, fp, fp, i, i, i, i, i, f, vp, sz, ctypes.c_uint, vp]
    lib.gns_estimate.argtypes = [fp, fp, i, i, f, fp, vp]
    lib.lnpegn_set_tuning.argtypes = [i, i]
    lib.lnpegn_plan_query.argtypes = [i, i, i, i, i, i, ctypes.POINTER(ctypes.c_int64), i]
    lib.lnpegn_set_profile_events.argtypes = [vp, vp]
    lib.lnpegn_stream_probe.argtypes = [vp, vp, vp, sz, i, vp]
    for name in ("ln_fwd_stats", "ln_bwd", "ln_bwd_pegn", "ln_bwd_pegn_static", "gns_estimate", "lnpegn_set_tuning",
                 "lnpegn_plan_query",
                 "lnpegn_set_profile_events", "lnpegn_stream_probe", "ln_bwd_deferred",
                 "ln_bwd_pegn_deferred", "lnpegn_reduce_deferred", "ln_fwd", "ln_bwd_ex",
                 "rms_fwd", "rms_bwd_ex", "gns_ema_update", "gns_offline", "gns_linear_accum_steps",
                 "linear_pegn", "embedding_pegn", "embedding_sort_ids", "embedding_pegn_presorted"):
        getattr(lib, name).restype = i
    _lib = lib
    return lib


def _torch():
    import torch
    return torch


def _dt(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _check3(x):
    if x.dim() != 3 or not x.is_contiguous() or not x.is_cuda:
        raise ValueError("expected a contiguous CUDA tensor [B,T,D]")
    return x.shape


def workspace_bytes(B: int, T: int, D: int, dtype: int) -> int:
    return int(load().lnpegn_workspace_bytes(B, T, D, dtype))


def alloc_workspace(B: int, T: int, D: int, dtype: int, device="cuda"):
    torch = _torch()
    return torch.empty(workspace_bytes(B, T, D, dtype), dtype=torch.uint8, device=device)


def gns_ema_update(state, records, alpha: float, smoothed=None, stream=None):
    """state [n,3] fp64 (updated in place), records [n,5] fp32 -> smoothed [n,3] fp32."""
    torch = _torch()
    n = state.shape[0]
    if state.dtype != torch.float64 or tuple(state.shape) != (n, 3) or not state.is_contiguous():
        raise ValueError("state must be a contiguous [n,3] float64 tensor")
    if records.dtype != torch.float32 or tuple(records.shape) != (n, 5) or not records.is_contiguous():
        raise ValueError("records must be a contiguous [n,5] float32 tensor")
    smoothed = torch.empty((n, 3), dtype=torch.float32, device=state.device) if smoothed is None else smoothed
    rc = load().gns_ema_update(_ptr(state), _ptr(records), n,
                               float(alpha), _ptr(smoothed), _stream(stream))
    if rc:
        raise LnpegnError("gns_ema_update", rc)
    return smoothed


def gns_offline(records, out=None, stream=None):
    """records [n,5] fp32 history of one group -> out[5] = mean_G2, mean_S, B_simple, stderr, B_simple_jack."""
    torch = _torch()
    if records.dtype != torch.float32 or records.dim() != 2 or records.shape[1] != 5 or not records.is_contiguous():
        raise ValueError("records must be a contiguous [n,5] float32 tensor")
    out = torch.empty(5, dtype=torch.float32, device=records.device) if out is None else out
    rc = load().gns_offline(_ptr(records), records.shape[0], _ptr(out), _stream(stream))
    if rc:
        raise LnpegnError("gns_offline", rc)
    return out


def gns_linear_accum_steps(tokens_seen: int, ramp_tokens: int, accum_final: int) -> int:
    rc = load().gns_linear_accum_steps(tokens_seen, ramp_tokens, accum_final)
    if rc < 0:
        raise LnpegnError("gns_linear_accum_steps", -rc)
    return rc


def linear_pegn(x, g, w=None, accumulate=False, s=None, big_sq=None, workspace=None, stream=None):
    """x [B,T,K], g [B,T,L] -> (w [K,L] fp32, s [B] fp32, big_sq [1] fp32)."""
    torch = _torch()
    B, T, K = _check3(x)
    B2, T2, L = _check3(g)
    if (B2, T2) != (B, T) or g.dtype != x.dtype:
        raise ValueError("x and g must agree in B, T and dtype")
    f32 = dict(dtype=torch.float32, device=x.device)
    if w is None:
        if accumulate:
            raise ValueError("accumulate needs the buffer to add to")
        w = torch.empty((K, L), **f32)
    if w.dtype != torch.float32 or tuple(w.shape) != (K, L) or not w.is_contiguous():
        raise ValueError("w must be a contiguous [K,L] float32 tensor")
    s = torch.empty(B, **f32) if s is None else s
    big_sq = torch.empty(1, **f32) if big_sq is None else big_sq
    if workspace is None:
        nbytes = load().linear_pegn_workspace_bytes(B, T, K, L, _dt(x))
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=x.device)
    rc = load().linear_pegn(_ptr(x), _ptr(g), _ptr(w), _ptr(s), _ptr(big_sq), B, T, K, L, _dt(x),
                            _ptr(workspace), workspace.numel(), ACCUMULATE if accumulate else 0, _stream(stream))
    if rc:
        raise LnpegnError("linear_pegn", rc)
    return w, s, big_sq


def embedding_pegn(ids, g, V: int, w=None, accumulate=False, s=None, big_sq=None, workspace=None, stream=None):
    """ids [B,T] int32/int64, g [B,T,D] -> (w [V,D] fp32, s [B] fp32, big_sq [1] fp32)."""
    torch = _torch()
    B, T, D = _check3(g)
    if tuple(ids.shape) != (B, T) or not ids.is_contiguous() or ids.dtype not in (torch.int32, torch.int64):
        raise ValueError("ids must be a contiguous [B,T] int32 or int64 tensor")
    f32 = dict(dtype=torch.float32, device=g.device)
    if w is None:
        if accumulate:
            raise ValueError("accumulate needs the buffer to add to")
        w = torch.empty((V, D), **f32)
    if w.dtype != torch.float32 or tuple(w.shape) != (V, D) or not w.is_contiguous():
        raise ValueError("w must be a contiguous [V,D] float32 tensor")
    s = torch.empty(B, **f32) if s is None else s
    big_sq = torch.empty(1, **f32) if big_sq is None else big_sq
    if workspace is None:
        nbytes = load().embedding_pegn_workspace_bytes(B, T, D, V)
        if nbytes == 0:
            raise LnpegnError("embedding_pegn_workspace_bytes", 1)
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=g.device)
    rc = load().embedding_pegn(_ptr(ids), 1 if ids.dtype == torch.int64 else 0, _ptr(g), _ptr(w), _ptr(s), _ptr(big_sq),
                               B, T, D, V, _dt(g), _ptr(workspace), workspace.numel(),
                               ACCUMULATE if accumulate else 0, _stream(stream))
    if rc:
        raise LnpegnError("embedding_pegn", rc)
    return w, s, big_sq


def embedding_sort_ids(ids, V: int, workspace=None, stream=None):
    """ids [B,T] int32/int64 -> (sorted_ids [B*T] int32 bit patterns of uint32, sorted_pos [B*T]): what
    embedding_pegn_presorted takes in place of ids (sort once at forward time)."""
    torch = _torch()
    if ids.dim() != 2 or not ids.is_contiguous() or ids.dtype not in (torch.int32, torch.int64):
        raise ValueError("ids must be a contiguous [B,T] int32 or int64 tensor")
    B, T = ids.shape
    n = B * T
    sorted_ids = torch.empty(n, dtype=torch.int32, device=ids.device)
    sorted_pos = torch.empty(n, dtype=torch.int32, device=ids.device)
    if workspace is None:
        workspace = torch.empty(load().embedding_pegn_workspace_bytes(B, T, 1, V), dtype=torch.uint8, device=ids.device)
    rc = load().embedding_sort_ids(_ptr(ids), 1 if ids.dtype == torch.int64 else 0, B, T, V, _ptr(sorted_ids),
                                   _ptr(sorted_pos), _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise LnpegnError("embedding_sort_ids", rc)
    return sorted_ids, sorted_pos


def embedding_pegn_presorted(sorted_ids, sorted_pos, g, V: int, w=None, accumulate=False, s=None, big_sq=None,
                             workspace=None, stream=None):
    """embedding_pegn with the ids sorted beforehand by embedding_sort_ids -> (w [V,D], s [B], big_sq [1])."""
    torch = _torch()
    B, T, D = _check3(g)
    if sorted_ids.numel() != B * T or sorted_pos.numel() != B * T:
        raise ValueError("sorted_ids and sorted_pos must hold B*T entries")
    f32 = dict(dtype=torch.float32, device=g.device)
    if w is None:
        if accumulate:
            raise ValueError("accumulate needs the buffer to add to")
        w = torch.empty((V, D), **f32)
    s = torch.empty(B, **f32) if s is None else s
    big_sq = torch.empty(1, **f32) if big_sq is None else big_sq
    if workspace is None:
        workspace = torch.empty(load().embedding_pegn_workspace_bytes(B, T, D, V), dtype=torch.uint8, device=g.device)
    rc = load().embedding_pegn_presorted(_ptr(sorted_ids), _ptr(sorted_pos), _ptr(g), _ptr(w), _ptr(s), _ptr(big_sq),
                                         B, T, D, V, _dt(g), _ptr(workspace), workspace.numel(),
                                         ACCUMULATE if accumulate else 0, _stream(stream))
    if rc:
        raise LnpegnError("embedding_pegn_presorted", rc)
    return w, s, big_sq


def set_tuning(key: int, value: int) -> None:
    rc = load().lnpegn_set_tuning(key, value)
    if rc:
        raise LnpegnError("lnpegn_set_tuning", rc)


PLAN_FIELDS = ("vector_kernel", "waves_per_row", "row_groups", "vectors_per_lane", "chunks_per_example", "chunks",
               "rows_per_block", "stagger", "chunks_per_xcd", "lds_bytes", "row_kernel_emits_norms", "examples_in_reduction",
               "groups", "chunks_per_group", "workspace_bytes", "rows_per_example")


def plan_query(B: int, T: int, D: int, dt: int, per_example: bool = True, aligned: bool = True) -> dict:
    """The launch plan of ln_bwd_pegn (or ln_bwd) for a shape, by field name (host only, no device needed)."""
    out = (ctypes.c_int64 * len(PLAN_FIELDS))()
    rc = load().lnpegn_plan_query(B, T, D, dt, 1 if per_example else 0, 1 if aligned else 0, out, len(PLAN_FIELDS))
    if rc:
        raise LnpegnError("lnpegn_plan_query", rc)
    return dict(zip(PLAN_FIELDS, (int(v) for v in out)))


def set_profile_events(start_event, stop_event) -> None:
    """Arm (or with two Nones disarm) the one-shot hipEvent pair around the next row kernel.
    Events are raw hipEvent_t handles (integers or ctypes void pointers)."""
    rc = load().lnpegn_set_profile_events(start_event, stop_event)
    if rc:
        raise LnpegnError("lnpegn_set_profile_events", rc)


def stream_probe(a, b, out, mode: int, stream=None) -> None:
    """Streaming yardstick kernel: out = a (mode 0) or a XOR b (modes 1, 2: 2 = one-shot workgroups, streaming
    loads and stores) over equal-sized buffers."""
    nbytes = out.numel() * out.element_size()
    rc = load().lnpegn_stream_probe(_ptr(a), _ptr(b), _ptr(out), nbytes, mode, _stream(stream))
    if rc:
        raise LnpegnError("lnpegn_stream_probe", rc)


def ln_fwd_stats(x, eps: float, mean=None, rstd=None, stream=None):
    """mean[B,T], rstd[B,T] (fp32) of x[B,T,D]."""
    torch = _torch()
    B, T, D = _check3(x)
    mean = torch.empty((B, T), dtype=torch.float32, device=x.device) if mean is None else mean
    rstd = torch.empty((B, T), dtype=torch.float32, device=x.device) if rstd is None else rstd
    rc = load().ln_fwd_stats(_ptr(x), _ptr(mean), _ptr(rstd), B, T, D, _dt(x), eps, _stream(stream))
    if rc:
        raise LnpegnError("ln_fwd_stats", rc)
    return mean, rstd


def ln_fwd(x, gamma, beta, eps: float, y=None, mean=None, rstd=None, want_stats=True, stream=None):
    """LayerNorm forward -> (y, mean[B,T], rstd[B,T]); the statistics are None if not wanted."""
    torch = _torch()
    B, T, D = _check3(x)
    y = torch.empty_like(x) if y is None else y
    if want_stats:
        mean = torch.empty((B, T), dtype=torch.float32, device=x.device) if mean is None else mean
        rstd = torch.empty((B, T), dtype=torch.float32, device=x.device) if rstd is None else rstd
    rc = load().ln_fwd(_ptr(x), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(mean), _ptr(rstd), B, T, D,
                       _dt(x), _dt(gamma), eps, _stream(stream))
    if rc:
        raise LnpegnError("ln_fwd", rc)
    return y, mean, rstd


def ln_bwd_ex(x, dy, gamma, eps: float, flags: int, dgamma, dbeta, mean=None, rstd=None, dx=None,
              pe_gamma_sq=None, pe_beta_sq=None, big_sq=None, workspace=None, stream=None):
    """General backward (flags: PER_EXAMPLE | DEFER | ACCUMULATE); the caller passes dgamma and
    dbeta, which ACCUMULATE adds to.  Returns dx."""
    torch = _torch()
    B, T, D = _check3(x)
    _check3(dy)
    dx = torch.empty_like(x) if dx is None else dx
    workspace = alloc_workspace(B, T, D, _dt(x), x.device) if workspace is None else workspace
    rc = load().ln_bwd_ex(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(mean), _ptr(rstd), _ptr(dx), _ptr(dgamma),
                          _ptr(dbeta), _ptr(pe_gamma_sq), _ptr(pe_beta_sq), _ptr(big_sq), B, T, D, _dt(x),
                          _dt(gamma), eps, _ptr(workspace), workspace.numel(), flags, _stream(stream))
    if rc:
        raise LnpegnError("ln_bwd_ex", rc)
    return dx


def rms_fwd(x, gamma, eps: float, y=None, rstd=None, want_rstd=True, stream=None):
    """RMSNorm forward -> (y, rstd[B,T] or None)."""
    torch = _torch()
    B, T, D = _check3(x)
    y = torch.empty_like(x) if y is None else y
    if want_rstd and rstd is None:
        rstd = torch.empty((B, T), dtype=torch.float32, device=x.device)
    rc = load().rms_fwd(_ptr(x), _ptr(gamma), _ptr(y), _ptr(rstd), B, T, D, _dt(x), _dt(gamma), eps,
                        _stream(stream))
    if rc:
        raise LnpegnError("rms_fwd", rc)
    return y, rstd


def rms_bwd_ex(x, dy, gamma, eps: float, flags: int, dgamma=None, rstd=None, dx=None, pe_gamma_sq=None,
               big_sq=None, workspace=None, stream=None):
    """RMSNorm backward (flags as ln_bwd_ex) -> (dx, dgamma, pe_gamma_sq[B] or None, big_sq[1] or None)."""
    torch = _torch()
    B, T, D = _check3(x)
    _check3(dy)
    f32 = dict(dtype=torch.float32, device=x.device)
    dx = torch.empty_like(x) if dx is None else dx
    dgamma = torch.zeros(D, **f32) if dgamma is None else dgamma
    if flags & PER_EXAMPLE:
        pe_gamma_sq = torch.empty(B, **f32) if pe_gamma_sq is None else pe_gamma_sq
        big_sq = torch.empty(1, **f32) if big_sq is None else big_sq
    workspace = alloc_workspace(B, T, D, _dt(x), x.device) if workspace is None else workspace
    rc = load().rms_bwd_ex(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(rstd), _ptr(dx), _ptr(dgamma),
                           _ptr(pe_gamma_sq), _ptr(big_sq), B, T, D, _dt(x), _dt(gamma), eps,
                           _ptr(workspace), workspace.numel(), flags, _stream(stream))
    if rc:
        raise LnpegnError("rms_bwd_ex", rc)
    return dx, dgamma, pe_gamma_sq, big_sq


def ln_bwd(x, dy, gamma, eps: float, mean=None, rstd=None, dx=None, dgamma=None, dbeta=None,
           workspace=None, stream=None, deferred=False):
    """Plain LayerNorm backward -> (dx, dgamma, dbeta).  deferred=True runs only the pass over x
    and dy; dgamma/dbeta appear after reduce_deferred() on this call's own workspace."""
    torch = _torch()
    B, T, D = _check3(x)
    _check3(dy)
    dx = torch.empty_like(x) if dx is None else dx
    dgamma = torch.empty(D, dtype=torch.float32, device=x.device) if dgamma is None else dgamma
    dbeta = torch.empty(D, dtype=torch.float32, device=x.device) if dbeta is None else dbeta
    workspace = alloc_workspace(B, T, D, _dt(x), x.device) if workspace is None else workspace
    fn = load().ln_bwd_deferred if deferred else load().ln_bwd
    rc = fn(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(mean), _ptr(rstd), _ptr(dx),
            _ptr(dgamma), _ptr(dbeta), B, T, D, _dt(x), _dt(gamma), eps,
            _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise LnpegnError("ln_bwd", rc)
    return dx, dgamma, dbeta


def ln_bwd_pegn(x, dy, gamma, eps: float, mean=None, rstd=None, dx=None, dgamma=None, dbeta=None,
                pe_gamma_sq=None, pe_beta_sq=None, big_sq=None, workspace=None, stream=None,
                deferred=False):
    """Fused backward -> (dx, dgamma, dbeta, pe_gamma_sq[B], pe_beta_sq[B], big_sq[2]).
    deferred=True runs only the pass over x and dy; everything but dx appears after
    reduce_deferred() on this call's own workspace."""
    torch = _torch()
    B, T, D = _check3(x)
    _check3(dy)
    f32 = dict(dtype=torch.float32, device=x.device)
    dx = torch.empty_like(x) if dx is None else dx
    dgamma = torch.empty(D, **f32) if dgamma is None else dgamma
    dbeta = torch.empty(D, **f32) if dbeta is None else dbeta
    pe_gamma_sq = torch.empty(B, **f32) if pe_gamma_sq is None else pe_gamma_sq
    pe_beta_sq = torch.empty(B, **f32) if pe_beta_sq is None else pe_beta_sq
    big_sq = torch.empty(2, **f32) if big_sq is None else big_sq
    workspace = alloc_workspace(B, T, D, _dt(x), x.device) if workspace is None else workspace
    fn = load().ln_bwd_pegn_deferred if deferred else load().ln_bwd_pegn
    rc = fn(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(mean), _ptr(rstd), _ptr(dx),
            _ptr(dgamma), _ptr(dbeta), _ptr(pe_gamma_sq), _ptr(pe_beta_sq),
            _ptr(big_sq), B, T, D, _dt(x), _dt(gamma), eps, _ptr(workspace),
            workspace.numel(), _stream(stream))
    if rc:
        raise LnpegnError("ln_bwd_pegn", rc)
    return dx, dgamma, dbeta, pe_gamma_sq, pe_beta_sq, big_sq


def ln_bwd_pegn_static(x, dy, gamma, eps: float, dx, dgamma, dbeta, pe_gamma_sq, pe_beta_sq, big_sq=None,
                       mean=None, rstd=None, stream=None):
    """ln_bwd_pegn without a workspace: the library's own fixed scratch is used and nothing is
    allocated, here or in the library -- every output buffer is the caller's.  Shapes whose workspace
    would exceed STATIC_SCRATCH_BYTES raise LnpegnError(LNPEGN_EWORKSPACE)."""
    B, T, D = _check3(x)
    _check3(dy)
    rc = load().ln_bwd_pegn_static(_ptr(x), _ptr(dy), _ptr(gamma), _ptr(mean), _ptr(rstd), _ptr(dx), _ptr(dgamma),
                                   _ptr(dbeta), _ptr(pe_gamma_sq), _ptr(pe_beta_sq), _ptr(big_sq), B, T, D,
                                   _dt(x), _dt(gamma), eps, _stream(stream))
    if rc:
        raise LnpegnError("ln_bwd_pegn_static", rc)
    return dx, dgamma, dbeta, pe_gamma_sq, pe_beta_sq, big_sq


def reduce_deferred(workspaces, B: int, T: int, D: int, dtype: int, stream=None) -> None:
    """Finish every deferred backward call whose workspace is listed (all of one shape)."""
    n = len(workspaces)
    arr = (ctypes.c_void_p * n)(*[w.data_ptr() for w in workspaces])
    rc = load().lnpegn_reduce_deferred(arr, n, B, T, D, dtype, _stream(stream))
    if rc:
        raise LnpegnError("lnpegn_reduce_deferred", rc)


def gns_estimate(pe_sq, big_sq, pe_scale: float, out=None, stream=None):
    """pe_sq [n_groups,B] fp32, big_sq [n_groups] fp32 -> out[5] fp32 on the device:
    |G_small|^2, |G_big|^2, G2, S, B_simple."""
    torch = _torch()
    if pe_sq.dim() == 1:
        pe_sq = pe_sq[None]
    if pe_sq.dtype != torch.float32 or big_sq.dtype != torch.float32:
        raise TypeError("gns_estimate takes fp32 norms")
    if not pe_sq.is_contiguous() or not big_sq.is_contiguous():
        raise ValueError("gns_estimate takes contiguous tensors")
    n_groups, B = pe_sq.shape
    if big_sq.numel() != n_groups:
        raise ValueError("big_sq must hold one value per group")
    out = torch.empty(5, dtype=torch.float32, device=pe_sq.device) if out is None else out
    rc = load().gns_estimate(_ptr(pe_sq), _ptr(big_sq), n_groups, B, pe_scale, _ptr(out),
                             _stream(stream))
    if rc:
        raise LnpegnError("gns_estimate", rc)
    return out
