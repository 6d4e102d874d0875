"""ctypes binding of libulorl: argument marshalling only.

Every function here has the name of the C entry point it wraps (minus the ``ulorl_`` prefix)
and does nothing but check tensors (device, dtype, contiguity), allocate outputs with torch
and pass raw pointers plus the current HIP stream.  All arithmetic runs in the HIP kernels.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

F32, BF16 = 0, 1
IS_SAIS, IS_POIS = 0, 1
GATE_PER_RESPONSE, GATE_GLOBAL, GATE_ALWAYS, GATE_NEVER = 0, 1, 2, 3
STATUS_BAD_TOKEN, STATUS_NONFINITE, STATUS_BAD_CU, STATUS_SYNC = 1, 2, 4, 8
LAUNCH_PER_ROW = 1
LAUNCH_DENSE_ROWS = 2

_HERE = os.path.dirname(os.path.abspath(__file__))


class UlorlError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


class _CParams(ctypes.Structure):
    _fields_ = [("eps_low", ctypes.c_float), ("eps_high", ctypes.c_float),
                ("tau", ctypes.c_float), ("sigma", ctypes.c_float),
                ("is_mode", ctypes.c_int32), ("gate_mode", ctypes.c_int32),
                ("seg_len", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("denominator", ctypes.c_double)]


class _CLaunch(ctypes.Structure):
    _fields_ = [("flags", ctypes.c_uint32), ("sync_spins", ctypes.c_int32), ("gemm_tile", ctypes.c_int32),
                ("gemm_group_m", ctypes.c_int32), ("reserved", ctypes.c_int32 * 4)]


class _CSegStats(ctypes.Structure):
    _fields_ = [("K", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("count", ctypes.c_void_p), ("ratio_sum", ctypes.c_void_p), ("ratio_max", ctypes.c_void_p),
                ("clipped", ctypes.c_void_p), ("kl_sum", ctypes.c_void_p), ("ent_sum", ctypes.c_void_p),
                ("masked", ctypes.c_void_p), ("out_of_range", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


@dataclass
class Launch:
    """Per-call launch options (ulorl_launch); the defaults are the library's."""
    per_row: bool = False
    dense_rows: bool = False
    sync_spins: int = 0
    gemm_tile: int = 0
    gemm_group_m: int = 0

    def to_c(self) -> _CLaunch:
        return _CLaunch((LAUNCH_PER_ROW if self.per_row else 0) | (LAUNCH_DENSE_ROWS if self.dense_rows else 0), self.sync_spins, self.gemm_tile, self.gemm_group_m,
                        (ctypes.c_int32 * 4)(0, 0, 0, 0))


def _launch_ref(launch: Optional["Launch"]):
    """(pointer argument, object to keep alive) for an optional Launch."""
    if launch is None:
        return None, None
    c = launch.to_c()
    return ctypes.byref(c), c


@dataclass
class Params:
    """Scalar parameters; defaults are the paper's (tau = 0.99, sigma = 0.2, Sec. 4.1)."""
    eps_low: float = 0.2
    eps_high: float = 0.2
    tau: float = 0.99
    sigma: float = 0.2
    is_mode: int = IS_SAIS
    gate_mode: int = GATE_PER_RESPONSE
    seg_len: int = 0
    denominator: float = 0.0

    def to_c(self) -> _CParams:
        return _CParams(self.eps_low, self.eps_high, self.tau, self.sigma, self.is_mode,
                        self.gate_mode, self.seg_len, 0, self.denominator)


def lib_path() -> str:
    return os.path.join(_HERE, "lib", "libulorl.so")


_lib = None


def load_library(build_if_missing: bool = True):
    """Load lib/libulorl.so (building it once if it is absent)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        if not build_if_missing:
            raise FileNotFoundError(path)
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(path)
    c = ctypes
    lib.ulorl_version.restype = c.c_int32
    lib.ulorl_status_string.restype = c.c_char_p
    lib.ulorl_status_string.argtypes = [c.c_int32]
    lib.ulorl_token_loss_workspace_bytes.restype = c.c_size_t
    lib.ulorl_token_loss_workspace_bytes.argtypes = [c.c_int64, c.c_int64, c.c_int32]
    vp = c.c_void_p
    lib.ulorl_token_loss_fwd.restype = c.c_int32
    lib.ulorl_token_loss_fwd.argtypes = [
        vp, c.c_int32, c.c_int64, c.c_int64, c.c_int64,      # logits, dt, N, V, stride
        vp, vp, c.c_int32,                                   # token_ids, cu_seqlens, R
        vp, vp, vp,                                          # segment_ids, old_logp, advantages
        c.POINTER(_CParams),
        vp, vp, vp, vp, vp,                                  # loss, logp, entropy, lse, gcoef
        vp, vp, vp,                                          # mpt_mask, ratio, segment_out
        vp, vp, vp,                                          # resp_entropy, resp_gate, counters
        vp,                                                  # seg_stats
        vp, c.c_size_t, vp, vp]                              # workspace, bytes, launch, stream
    lib.ulorl_token_loss_fwd_bwd.restype = c.c_int32
    lib.ulorl_token_loss_fwd_bwd.argtypes = [
        vp, c.c_int32, c.c_int64, c.c_int64, c.c_int64,      # logits, dt, N, V, stride
        vp, vp, c.c_int32,                                   # token_ids, cu_seqlens, R
        vp, vp, vp,                                          # segment_ids, old_logp, advantages
        c.POINTER(_CParams), c.c_float,                      # params, grad_out
        vp, vp, vp, vp, vp,                                  # loss, logp, entropy, lse, gcoef
        vp, vp, vp,                                          # mpt_mask, ratio, segment_out
        vp, vp, vp,                                          # resp_entropy, resp_gate, counters
        vp,                                                  # seg_stats
        vp, vp, c.c_size_t, vp, vp]                          # dlogits, workspace, bytes, launch, stream
    lib.ulorl_init.restype = c.c_int32
    lib.ulorl_init.argtypes = []
    lib.ulorl_static_scratch_bytes.restype = c.c_size_t
    lib.ulorl_static_scratch_bytes.argtypes = []
    lib.ulorl_token_loss_fwd_bwd_static.restype = c.c_int32
    lib.ulorl_token_loss_fwd_bwd_static.argtypes = lib.ulorl_token_loss_fwd_bwd.argtypes[:-4] + [vp, vp]
    lib.ulorl_lmhead_workspace_bytes.restype = c.c_size_t
    lib.ulorl_lmhead_workspace_bytes.argtypes = [c.c_int64, c.c_int64, c.c_int64, c.c_int32, c.c_int32]
    lib.ulorl_lmhead_token_loss_fwd.restype = c.c_int32
    lib.ulorl_lmhead_token_loss_fwd.argtypes = [
        vp, vp, c.c_int64, c.c_int64, c.c_int64, c.c_int32,  # hidden, W, N, Hd, V, chunk
        vp, vp, c.c_int32, vp, vp, vp, c.POINTER(_CParams),
        vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
        vp, vp, c.c_size_t, vp, vp]                          # seg_stats, workspace, bytes, launch, stream
    lib.ulorl_lmhead_token_loss_bwd.restype = c.c_int32
    lib.ulorl_lmhead_token_loss_bwd.argtypes = [
        vp, vp, c.c_int64, c.c_int64, c.c_int64, c.c_int32, vp, vp, vp, c.c_float, vp, vp, vp, c.c_size_t, vp, vp]
    lib.ulorl_gemm_tn_bf16.restype = c.c_int32
    lib.ulorl_gemm_tn_bf16.argtypes = [vp, c.c_int64, vp, c.c_int64, c.c_int64, c.c_int64, c.c_int64, vp, c.c_int64, vp, vp]
    lib.ulorl_advantage_prep.restype = c.c_int32
    lib.ulorl_advantage_prep.argtypes = [vp, vp, vp, c.c_int32, c.c_int32, c.c_int64, c.c_float, c.c_int32,
                                         vp, vp, vp, vp, vp]
    lib.ulorl_segment_diagnostics_workspace_bytes.restype = c.c_size_t
    lib.ulorl_segment_diagnostics_workspace_bytes.argtypes = [c.c_int64, c.c_int32]
    lib.ulorl_segment_diagnostics.restype = c.c_int32
    lib.ulorl_segment_diagnostics.argtypes = [c.c_int64, c.c_int32, vp, vp, vp, vp, vp, vp, vp, c.c_float, c.c_float,
                                              vp, vp, vp, vp, vp, vp, vp, vp, vp, c.c_size_t, vp]
    lib.ulorl_segment_pool_step.restype = c.c_int32
    lib.ulorl_segment_pool_step.argtypes = [c.c_int32, vp, vp, vp, c.c_int32, c.c_int32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.ulorl_token_loss_bwd.restype = c.c_int32
    lib.ulorl_token_loss_bwd.argtypes = [
        vp, c.c_int32, c.c_int64, c.c_int64, c.c_int64, vp, vp, vp, c.c_float, vp, vp]
    _lib = lib
    return lib


def version() -> int:
    return int(load_library().ulorl_version())


def status_string(status: int) -> str:
    return load_library().ulorl_status_string(status).decode()


def token_loss_workspace_bytes(N: int, V: int, R: int) -> int:
    return int(load_library().ulorl_token_loss_workspace_bytes(N, V, R))


# ------------------------------------------------------------------------------------ helpers

def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("logits must be float32 or bfloat16, got %s" % t.dtype)


def _check_logits(logits: torch.Tensor):
    if not logits.is_cuda:
        raise RuntimeError("libulorl runs on the GPU only: logits must be a device tensor")
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be [N, V] with unit stride along V")
    return _dtype_code(logits), logits.shape[0], logits.shape[1], logits.stride(0)


def _vec(t: Optional[torch.Tensor], dtype, n: int, name: str, dev):
    if t is None:
        return None
    if t.device != dev or t.dtype != dtype or t.dim() != 1 or t.shape[0] != n or not t.is_contiguous():
        raise ValueError("%s must be a contiguous %s[%d] tensor on %s" % (name, dtype, n, dev))
    return t


def _p(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(dev) -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream)


@dataclass
class FwdResult:
    loss: Optional[torch.Tensor]
    logp: torch.Tensor
    entropy: torch.Tensor
    lse: torch.Tensor
    gcoef: Optional[torch.Tensor] = None
    mpt_mask: Optional[torch.Tensor] = None
    ratio: Optional[torch.Tensor] = None
    segment_out: Optional[torch.Tensor] = None
    resp_entropy: Optional[torch.Tensor] = None
    resp_gate: Optional[torch.Tensor] = None
    counters: Optional[torch.Tensor] = None
    segment_stats: Optional[dict] = None      # per-segment diagnostics, when asked for (segments=K)


def _segment_stats_buffers(K: int, N: int, dev):
    """Output tensors and workspace of the per-segment diagnostics -> (dict, ulorl_segment_stats)."""
    i64 = dict(dtype=torch.int64, device=dev)
    f64 = dict(dtype=torch.float64, device=dev)
    out = {"count": torch.empty(K, **i64), "ratio_sum": torch.empty(K, **f64),
           "ratio_max": torch.empty(K, dtype=torch.float32, device=dev), "clipped": torch.empty(K, **i64),
           "kl_sum": torch.empty(K, **f64), "ent_sum": torch.empty(K, **f64), "masked": torch.empty(K, **i64),
           "out_of_range": torch.empty(1, **i64)}
    need = int(load_library().ulorl_segment_diagnostics_workspace_bytes(N, K))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    out["_workspace"] = ws
    c = _CSegStats(K, 0, out["count"].data_ptr(), out["ratio_sum"].data_ptr(), out["ratio_max"].data_ptr(),
                   out["clipped"].data_ptr(), out["kl_sum"].data_ptr(), out["ent_sum"].data_ptr(),
                   out["masked"].data_ptr(), out["out_of_range"].data_ptr(), ws.data_ptr(), ws.numel())
    return out, c


def _prepare_objective(logits, token_ids, cu_seqlens, advantages, old_logp, params, segment_ids, out, workspace):
    """Shared marshalling of the objective's inputs/outputs for the fwd and fwd_bwd calls."""
    dt, N, V, stride = _check_logits(logits)
    dev = logits.device
    f32 = dict(dtype=torch.float32, device=dev)
    token_ids = _vec(token_ids, torch.int32, N, "token_ids", dev)
    if out is None:
        out = FwdResult(None, torch.empty(N, **f32), torch.empty(N, **f32), torch.empty(N, **f32))
    params = params or Params()
    if cu_seqlens.device != dev or cu_seqlens.dtype != torch.int32 or not cu_seqlens.is_contiguous():
        raise ValueError("cu_seqlens must be a contiguous int32 device tensor")
    R = cu_seqlens.shape[0] - 1
    advantages = _vec(advantages, torch.float32, N, "advantages", dev)
    old_logp = _vec(old_logp, torch.float32, N, "old_logp", dev)
    segment_ids = _vec(segment_ids, torch.int32, N, "segment_ids", dev)
    if out.loss is None:
        out.loss = torch.empty(1, **f32)
        out.gcoef = torch.empty(N, **f32)
        out.mpt_mask = torch.empty(N, dtype=torch.uint8, device=dev)
        out.ratio = torch.empty(N, **f32)
        out.segment_out = torch.empty(N, dtype=torch.int32, device=dev)
        out.resp_entropy = torch.empty(max(R, 1), **f32)[:R]
        out.resp_gate = torch.empty(max(R, 1), dtype=torch.uint8, device=dev)[:R]
        out.counters = torch.empty(4, dtype=torch.int64, device=dev)
    if workspace is None:
        workspace = torch.empty(max(token_loss_workspace_bytes(N, V, R), 256), dtype=torch.uint8, device=dev)
    ws_bytes = workspace.numel() * workspace.element_size()
    return (dt, N, V, stride, dev, token_ids, R, advantages, old_logp, segment_ids, params.to_c(), out,
            workspace, ws_bytes)


def token_loss_fwd(logits, token_ids, cu_seqlens, advantages, old_logp=None, params: Params = None,
                   segment_ids=None, out: Optional[FwdResult] = None,
                   workspace: Optional[torch.Tensor] = None, launch: Optional[Launch] = None,
                   segments: int = 0) -> FwdResult:
    """ulorl_token_loss_fwd.  ``advantages=None`` selects the stats-only pass.
    ``out``/``workspace`` let a caller reuse buffers (nothing is allocated then).
    ``segments=K`` asks for the per-segment diagnostics of ids 0..K-1 (``out.segment_stats``)."""
    lib = load_library()
    lref, _keep = _launch_ref(launch)
    if advantages is None:                       # stats-only: lse, logp, entropy
        dt, N, V, stride = _check_logits(logits)
        dev = logits.device
        token_ids = _vec(token_ids, torch.int32, N, "token_ids", dev)
        f32 = dict(dtype=torch.float32, device=dev)
        if out is None:
            out = FwdResult(None, torch.empty(N, **f32), torch.empty(N, **f32), torch.empty(N, **f32))
        if workspace is None:                    # optional here; with it the statistics are formed by pieces
            workspace = torch.empty(token_loss_workspace_bytes(N, V, 1), dtype=torch.uint8, device=dev)
        ws_bytes = workspace.numel() * workspace.element_size()
        rc = lib.ulorl_token_loss_fwd(
            _p(logits), dt, N, V, stride, _p(token_ids), None, 0, None, None, None, None,
            None, _p(out.logp), _p(out.entropy), _p(out.lse), None, None, None, None, None, None, None, None,
            _p(workspace), ws_bytes, lref, _stream(dev))
        if rc != 0:
            raise UlorlError(rc, "ulorl_token_loss_fwd")
        return out
    (dt, N, V, stride, dev, token_ids, R, advantages, old_logp, segment_ids, cparams, out, workspace,
     ws_bytes) = _prepare_objective(logits, token_ids, cu_seqlens, advantages, old_logp, params,
                                    segment_ids, out, workspace)
    sref = None
    if segments > 0:
        out.segment_stats, cseg = _segment_stats_buffers(segments, N, dev)
        sref = ctypes.byref(cseg)
    rc = lib.ulorl_token_loss_fwd(
        _p(logits), dt, N, V, stride, _p(token_ids), _p(cu_seqlens), R, _p(segment_ids), _p(old_logp),
        _p(advantages), ctypes.byref(cparams),
        _p(out.loss), _p(out.logp), _p(out.entropy), _p(out.lse), _p(out.gcoef),
        _p(out.mpt_mask), _p(out.ratio), _p(out.segment_out), _p(out.resp_entropy),
        _p(out.resp_gate), _p(out.counters), sref, _p(workspace), ws_bytes, lref, _stream(dev))
    if rc != 0:
        raise UlorlError(rc, "ulorl_token_loss_fwd")
    return out


def token_loss_fwd_bwd(logits, token_ids, cu_seqlens, advantages, old_logp=None, params: Params = None,
                       segment_ids=None, grad_out: float = 1.0, dlogits: Optional[torch.Tensor] = None,
                       inplace: bool = False, out: Optional[FwdResult] = None,
                       workspace: Optional[torch.Tensor] = None, launch: Optional[Launch] = None,
                       segments: int = 0):
    """ulorl_token_loss_fwd_bwd -> (FwdResult, dlogits).  ``inplace=True`` overwrites ``logits``."""
    lib = load_library()
    lref, _keep = _launch_ref(launch)
    (dt, N, V, stride, dev, token_ids, R, advantages, old_logp, segment_ids, cparams, out, workspace,
     ws_bytes) = _prepare_objective(logits, token_ids, cu_seqlens, advantages, old_logp, params,
                                    segment_ids, out, workspace)
    if advantages is None:
        raise ValueError("token_loss_fwd_bwd needs advantages")
    if inplace:
        dlogits = logits
    elif dlogits is None:
        dlogits = torch.empty_strided((N, V), (stride, 1), dtype=logits.dtype, device=dev)
    if (dlogits.shape != logits.shape or dlogits.dtype != logits.dtype or dlogits.device != dev
            or dlogits.stride() != logits.stride()):
        raise ValueError("dlogits must match logits in shape, dtype, strides and device")
    sref = None
    if segments > 0:
        out.segment_stats, cseg = _segment_stats_buffers(segments, N, dev)
        sref = ctypes.byref(cseg)
    rc = lib.ulorl_token_loss_fwd_bwd(
        _p(logits), dt, N, V, stride, _p(token_ids), _p(cu_seqlens), R, _p(segment_ids), _p(old_logp),
        _p(advantages), ctypes.byref(cparams), float(grad_out),
        _p(out.loss), _p(out.logp), _p(out.entropy), _p(out.lse), _p(out.gcoef),
        _p(out.mpt_mask), _p(out.ratio), _p(out.segment_out), _p(out.resp_entropy),
        _p(out.resp_gate), _p(out.counters), sref, _p(dlogits), _p(workspace), ws_bytes, lref, _stream(dev))
    if rc != 0:
        raise UlorlError(rc, "ulorl_token_loss_fwd_bwd")
    return out, dlogits


def init() -> None:
    """ulorl_init: resolve the static scratch array of the current device (set-up time)."""
    rc = load_library().ulorl_init()
    if rc != 0:
        raise UlorlError(rc, "ulorl_init")


def static_scratch_bytes() -> int:
    return int(load_library().ulorl_static_scratch_bytes())


def token_loss_fwd_bwd_static(logits, token_ids, cu_seqlens, advantages, old_logp=None, params: Params = None,
                              segment_ids=None, grad_out: float = 1.0, dlogits: Optional[torch.Tensor] = None,
                              inplace: bool = False, out: Optional[FwdResult] = None,
                              launch: Optional[Launch] = None):
    """ulorl_token_loss_fwd_bwd_static -> (FwdResult, dlogits): the one-call path on the library's
    static scratch array (the C call allocates nothing; pass ``out`` and ``dlogits`` to keep this
    wrapper from allocating outputs either)."""
    lib = load_library()
    dt, N, V, stride = _check_logits(logits)
    dev = logits.device
    f32 = dict(dtype=torch.float32, device=dev)
    token_ids = _vec(token_ids, torch.int32, N, "token_ids", dev)
    if cu_seqlens.device != dev or cu_seqlens.dtype != torch.int32 or not cu_seqlens.is_contiguous():
        raise ValueError("cu_seqlens must be a contiguous int32 device tensor")
    R = cu_seqlens.shape[0] - 1
    advantages = _vec(advantages, torch.float32, N, "advantages", dev)
    old_logp = _vec(old_logp, torch.float32, N, "old_logp", dev)
    segment_ids = _vec(segment_ids, torch.int32, N, "segment_ids", dev)
    if advantages is None:
        raise ValueError("token_loss_fwd_bwd_static needs advantages")
    lref, _keep = _launch_ref(launch)
    cparams = (params or Params()).to_c()
    if out is None:
        out = FwdResult(torch.empty(1, **f32), torch.empty(N, **f32), torch.empty(N, **f32), torch.empty(N, **f32),
                        torch.empty(N, **f32), torch.empty(N, dtype=torch.uint8, device=dev), torch.empty(N, **f32),
                        torch.empty(N, dtype=torch.int32, device=dev), torch.empty(max(R, 1), **f32)[:R],
                        torch.empty(max(R, 1), dtype=torch.uint8, device=dev)[:R],
                        torch.empty(4, dtype=torch.int64, device=dev))
    if inplace:
        dlogits = logits
    elif dlogits is None:
        dlogits = torch.empty_strided((N, V), (stride, 1), dtype=logits.dtype, device=dev)
    if (dlogits.shape != logits.shape or dlogits.dtype != logits.dtype or dlogits.device != dev
            or dlogits.stride() != logits.stride()):
        raise ValueError("dlogits must match logits in shape, dtype, strides and device")
    rc = lib.ulorl_token_loss_fwd_bwd_static(
        _p(logits), dt, N, V, stride, _p(token_ids), _p(cu_seqlens), R, _p(segment_ids), _p(old_logp),
        _p(advantages), ctypes.byref(cparams), float(grad_out),
        _p(out.loss), _p(out.logp), _p(out.entropy), _p(out.lse), _p(out.gcoef),
        _p(out.mpt_mask), _p(out.ratio), _p(out.segment_out), _p(out.resp_entropy),
        _p(out.resp_gate), _p(out.counters), None, _p(dlogits), lref, _stream(dev))
    if rc != 0:
        raise UlorlError(rc, "ulorl_token_loss_fwd_bwd_static")
    return out, dlogits


def row_stats(logits, token_ids, out: Optional[FwdResult] = None, launch: Optional[Launch] = None) -> FwdResult:
    """Stats-only forward: lse, chosen-token log-prob and entropy per row."""
    return token_loss_fwd(logits, token_ids, None, None, out=out, launch=launch)


def token_loss_bwd(logits, token_ids, lse, gcoef, grad_out: float = 1.0,
                   dlogits: Optional[torch.Tensor] = None, inplace: bool = False) -> torch.Tensor:
    """ulorl_token_loss_bwd.  ``inplace=True`` overwrites ``logits`` with the gradient."""
    lib = load_library()
    dt, N, V, stride = _check_logits(logits)
    dev = logits.device
    token_ids = _vec(token_ids, torch.int32, N, "token_ids", dev)
    lse = _vec(lse, torch.float32, N, "lse", dev)
    gcoef = _vec(gcoef, torch.float32, N, "gcoef", dev)
    if inplace:
        dlogits = logits
    elif dlogits is None:
        dlogits = torch.empty_strided((N, V), (stride, 1), dtype=logits.dtype, device=dev)
    if (dlogits.shape != logits.shape or dlogits.dtype != logits.dtype or dlogits.device != dev
            or dlogits.stride() != logits.stride()):
        raise ValueError("dlogits must match logits in shape, dtype, strides and device")
    rc = lib.ulorl_token_loss_bwd(_p(logits), dt, N, V, stride, _p(token_ids), _p(lse), _p(gcoef),
                                  float(grad_out), _p(dlogits), _stream(dev))
    if rc != 0:
        raise UlorlError(rc, "ulorl_token_loss_bwd")
    return dlogits


# ------------------------------------------------------------------------------------ lm_head variant

def lmhead_workspace_bytes(N: int, Hd: int, V: int, R: int, vocab_chunk: int) -> int:
    return int(load_library().ulorl_lmhead_workspace_bytes(N, Hd, V, R, vocab_chunk))


def _check_lmhead(hidden, weight):
    if not hidden.is_cuda or not weight.is_cuda:
        raise RuntimeError("libulorl runs on the GPU only")
    if hidden.dtype != torch.bfloat16 or weight.dtype != torch.bfloat16:
        raise TypeError("hidden and weight must be bfloat16")
    if hidden.dim() != 2 or weight.dim() != 2 or not hidden.is_contiguous() or not weight.is_contiguous():
        raise ValueError("hidden [N, Hd] and weight [Hd, V] must be contiguous")
    if hidden.shape[1] != weight.shape[0]:
        raise ValueError("hidden is [N, Hd], weight is [Hd, V]")
    return hidden.shape[0], hidden.shape[1], weight.shape[1]


def lmhead_token_loss_fwd(hidden, weight, token_ids, cu_seqlens, advantages, old_logp=None,
                          params: Params = None, segment_ids=None, vocab_chunk: int = 8192,
                          out: Optional[FwdResult] = None, workspace: Optional[torch.Tensor] = None,
                          launch: Optional[Launch] = None, segments: int = 0) -> FwdResult:
    """ulorl_lmhead_token_loss_fwd."""
    lib = load_library()
    lref, _keep = _launch_ref(launch)
    N, Hd, V = _check_lmhead(hidden, weight)
    dev = hidden.device
    f32 = dict(dtype=torch.float32, device=dev)
    token_ids = _vec(token_ids, torch.int32, N, "token_ids", dev)
    params = params or Params()
    cparams = params.to_c()
    R = cu_seqlens.shape[0] - 1 if cu_seqlens is not None else 1
    advantages = _vec(advantages, torch.float32, N, "advantages", dev)
    old_logp = _vec(old_logp, torch.float32, N, "old_logp", dev)
    segment_ids = _vec(segment_ids, torch.int32, N, "segment_ids", dev)
    if advantages is None:          # stats-only pass
        if out is None:
            out = FwdResult(None, torch.empty(N, **f32), torch.empty(N, **f32), torch.empty(N, **f32),
                            None, None, None, None, None, None, None)
        if workspace is None:
            workspace = torch.empty(max(lmhead_workspace_bytes(N, Hd, V, R, vocab_chunk), 256), dtype=torch.uint8,
                                    device=dev)
        rc = lib.ulorl_lmhead_token_loss_fwd(
            _p(hidden), _p(weight), N, Hd, V, vocab_chunk, _p(token_ids), _p(cu_seqlens), R, None, None, None,
            ctypes.byref(cparams), None, _p(out.logp), _p(out.entropy), _p(out.lse), None, None, None, None, None,
            None, None, None, _p(workspace), workspace.numel(), lref, _stream(dev))
        if rc != 0:
            raise UlorlError(rc, "ulorl_lmhead_token_loss_fwd")
        return out
    if out is None:
        out = FwdResult(torch.empty(1, **f32), torch.empty(N, **f32), torch.empty(N, **f32), torch.empty(N, **f32),
                        torch.empty(N, **f32), torch.empty(N, dtype=torch.uint8, device=dev), torch.empty(N, **f32),
                        torch.empty(N, dtype=torch.int32, device=dev), torch.empty(max(R, 1), **f32)[:R],
                        torch.empty(max(R, 1), dtype=torch.uint8, device=dev)[:R],
                        torch.empty(4, dtype=torch.int64, device=dev))
    if workspace is None:
        workspace = torch.empty(max(lmhead_workspace_bytes(N, Hd, V, R, vocab_chunk), 256), dtype=torch.uint8, device=dev)
    sref = None
    if segments > 0:
        out.segment_stats, cseg = _segment_stats_buffers(segments, N, dev)
        sref = ctypes.byref(cseg)
    rc = lib.ulorl_lmhead_token_loss_fwd(
        _p(hidden), _p(weight), N, Hd, V, vocab_chunk, _p(token_ids), _p(cu_seqlens), R, _p(segment_ids),
        _p(old_logp), _p(advantages), ctypes.byref(cparams),
        _p(out.loss), _p(out.logp), _p(out.entropy), _p(out.lse), _p(out.gcoef), _p(out.mpt_mask), _p(out.ratio),
        _p(out.segment_out), _p(out.resp_entropy), _p(out.resp_gate), _p(out.counters), sref,
        _p(workspace), workspace.numel(), lref, _stream(dev))
    if rc != 0:
        raise UlorlError(rc, "ulorl_lmhead_token_loss_fwd")
    return out


def lmhead_token_loss_bwd(hidden, weight, token_ids, lse, gcoef, grad_out: float = 1.0, vocab_chunk: int = 8192,
                          d_hidden: Optional[torch.Tensor] = None, d_weight: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None, launch: Optional[Launch] = None):
    """ulorl_lmhead_token_loss_bwd -> (d_hidden [N, Hd] bf16, d_weight [Hd, V] bf16)."""
    lib = load_library()
    N, Hd, V = _check_lmhead(hidden, weight)
    dev = hidden.device
    token_ids = _vec(token_ids, torch.int32, N, "token_ids", dev)
    lse = _vec(lse, torch.float32, N, "lse", dev)
    gcoef = _vec(gcoef, torch.float32, N, "gcoef", dev)
    if d_hidden is None:
        d_hidden = torch.empty_like(hidden)
    if d_weight is None:
        d_weight = torch.empty_like(weight)
    if workspace is None:
        workspace = torch.empty(max(lmhead_workspace_bytes(N, Hd, V, 1, vocab_chunk), 256), dtype=torch.uint8, device=dev)
    lref, _keep = _launch_ref(launch)
    rc = lib.ulorl_lmhead_token_loss_bwd(
        _p(hidden), _p(weight), N, Hd, V, vocab_chunk, _p(token_ids), _p(lse), _p(gcoef), float(grad_out),
        _p(d_hidden), _p(d_weight), _p(workspace), workspace.numel(), lref, _stream(dev))
    if rc != 0:
        raise UlorlError(rc, "ulorl_lmhead_token_loss_bwd")
    return d_hidden, d_weight


def gemm_tn_bf16(a: torch.Tensor, b: torch.Tensor, out: Optional[torch.Tensor] = None,
                 launch: Optional[Launch] = None) -> torch.Tensor:
    """ulorl_gemm_tn_bf16: a [M, K] . b [N, K]^T -> fp32 [M, N]."""
    lib = load_library()
    if not (a.is_cuda and b.is_cuda) or a.dtype != torch.bfloat16 or b.dtype != torch.bfloat16:
        raise TypeError("a and b must be bfloat16 device tensors")
    if a.dim() != 2 or b.dim() != 2 or a.stride(1) != 1 or b.stride(1) != 1 or a.shape[1] != b.shape[1]:
        raise ValueError("a is [M, K], b is [N, K], unit stride along K")
    M, K = a.shape
    N = b.shape[0]
    if out is None:
        out = torch.empty(M, N, dtype=torch.float32, device=a.device)
    lref, _keep = _launch_ref(launch)
    rc = lib.ulorl_gemm_tn_bf16(_p(a), a.stride(0), _p(b), b.stride(0), M, N, K, _p(out), out.stride(0), lref,
                                _stream(a.device))
    if rc != 0:
        raise UlorlError(rc, "ulorl_gemm_tn_bf16")
    return out


# ------------------------------------------------------------------------------------ neighbours of the hot path

def advantage_prep(rewards, cu_seqlens, group_size: int, truncated=None, eps: float = 1e-6, unbiased: bool = False):
    """ulorl_advantage_prep -> (resp_adv [R], group_keep [R/G], token_adv [N], kept_tokens [1] int64)."""
    lib = load_library()
    dev = rewards.device
    if not rewards.is_cuda:
        raise RuntimeError("libulorl runs on the GPU only")
    R = rewards.shape[0]
    rewards = _vec(rewards, torch.float32, R, "rewards", dev)
    truncated = _vec(truncated, torch.uint8, R, "truncated", dev)
    if cu_seqlens.device != dev or cu_seqlens.dtype != torch.int32 or cu_seqlens.shape[0] != R + 1:
        raise ValueError("cu_seqlens must be int32 [R+1] on the same device")
    N = int(cu_seqlens[-1].item())
    resp = torch.empty(R, dtype=torch.float32, device=dev)
    keep = torch.empty(max(R // max(group_size, 1), 1), dtype=torch.uint8, device=dev)
    tok = torch.empty(N, dtype=torch.float32, device=dev)
    kept = torch.empty(1, dtype=torch.int64, device=dev)
    rc = lib.ulorl_advantage_prep(_p(rewards), _p(truncated), _p(cu_seqlens), R, group_size, N, float(eps),
                                  1 if unbiased else 0, _p(resp), _p(keep), _p(tok), _p(kept), _stream(dev))
    if rc != 0:
        raise UlorlError(rc, "ulorl_advantage_prep")
    return resp, keep[:R // group_size], tok, kept


def segment_diagnostics(res: FwdResult, advantages, old_logp, K: int, eps_low: float = 0.2, eps_high: float = 0.2,
                        segment_ids=None):
    """ulorl_segment_diagnostics on the outputs of a forward call -> dict of per-segment tensors."""
    lib = load_library()
    seg = res.segment_out if segment_ids is None else segment_ids
    dev = seg.device
    N = seg.shape[0]
    i64 = dict(dtype=torch.int64, device=dev)
    f64 = dict(dtype=torch.float64, device=dev)
    out = {"count": torch.empty(K, **i64), "ratio_sum": torch.empty(K, **f64),
           "ratio_max": torch.empty(K, dtype=torch.float32, device=dev), "clipped": torch.empty(K, **i64),
           "kl_sum": torch.empty(K, **f64), "ent_sum": torch.empty(K, **f64), "masked": torch.empty(K, **i64),
           "out_of_range": torch.empty(1, **i64)}
    ws = torch.empty(max(int(lib.ulorl_segment_diagnostics_workspace_bytes(N, K)), 256), dtype=torch.uint8, device=dev)
    rc = lib.ulorl_segment_diagnostics(
        N, K, _p(seg), _p(res.ratio), _p(res.logp), _p(old_logp), _p(res.entropy), _p(res.mpt_mask), _p(advantages),
        float(eps_low), float(eps_high), _p(out["count"]), _p(out["ratio_sum"]), _p(out["ratio_max"]),
        _p(out["clipped"]), _p(out["kl_sum"]), _p(out["ent_sum"]), _p(out["masked"]), _p(out["out_of_range"]),
        _p(ws), ws.numel(), _stream(dev))
    if rc != 0:
        raise UlorlError(rc, "ulorl_segment_diagnostics")
    return out


def segment_pool_step(prev_len, new_len, hit_eos, seg_len: int, max_len: int):
    """ulorl_segment_pool_step -> dict of device tensors: state, total_len, segments [B];
    unfinished_idx, experience_idx, exp_truncated [B] and exp_cu_seqlens [B+1] (only the leading
    counts[0] / counts[1] (+1) entries are meaningful); counts [5] int64."""
    lib = load_library()
    if not prev_len.is_cuda:
        raise RuntimeError("libulorl runs on the GPU only")
    dev = prev_len.device
    B = prev_len.shape[0]
    prev_len = _vec(prev_len, torch.int32, B, "prev_len", dev)
    new_len = _vec(new_len, torch.int32, B, "new_len", dev)
    hit_eos = _vec(hit_eos, torch.uint8, B, "hit_eos", dev)
    i32 = dict(dtype=torch.int32, device=dev)
    u8 = dict(dtype=torch.uint8, device=dev)
    out = {"state": torch.empty(B, **u8), "total_len": torch.empty(B, **i32), "segments": torch.empty(B, **i32),
           "unfinished_idx": torch.empty(B, **i32), "experience_idx": torch.empty(B, **i32),
           "exp_cu_seqlens": torch.empty(B + 1, **i32), "exp_truncated": torch.empty(B, **u8),
           "counts": torch.empty(5, dtype=torch.int64, device=dev)}
    rc = lib.ulorl_segment_pool_step(
        B, _p(prev_len), _p(new_len), _p(hit_eos), int(seg_len), int(max_len), _p(out["state"]), _p(out["total_len"]),
        _p(out["segments"]), _p(out["unfinished_idx"]), _p(out["experience_idx"]), _p(out["exp_cu_seqlens"]),
        _p(out["exp_truncated"]), _p(out["counts"]), _stream(dev))
    if rc != 0:
        raise UlorlError(rc, "ulorl_segment_pool_step")
    return out
