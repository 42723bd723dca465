"""Python binding of the MI355X KLA library (libkla.so, C ABI in include/kla.h).

Argument marshalling only: every step of the path runs in the HIP kernels.  PyTorch supplies
device memory and the current stream.  There is no CPU fallback: if the compiled library is
missing, or a tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os
import threading

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# KLA_LIBRARY names another build of the same library (the host-sanitizer run of tests/host_sanitizers.py uses it)
LIB_PATH = os.environ.get("KLA_LIBRARY") or os.path.join(_HERE, "libkla.so")
HEADER_PATH = os.path.join(os.path.dirname(_HERE), "include", "kla.h")

KLA_F32, KLA_BF16 = 0, 1
KLA_OPT_NORMALIZE_Q, KLA_OPT_GDN_BETA = 1, 2
_lock = threading.Lock()
_lib = None

_vp, _fp, _ip = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
_SIGNATURES = {
    "kla_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "kla_chunk_fwd_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int] * 6 + [ctypes.c_int, _ip, ctypes.c_int]),
    "kla_chunk_fwd_workspace_bytes_opts": (ctypes.c_size_t, [ctypes.c_int] * 6 + [ctypes.c_int, _ip, ctypes.c_int, ctypes.c_uint]),
    "kla_chunk_bwd_workspace_bytes_opts": (ctypes.c_size_t, [ctypes.c_int] * 6 + [ctypes.c_int, _ip, ctypes.c_int, ctypes.c_uint]),
    "kla_chunk_fwd": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp, _fp, _ip, _ip, ctypes.c_int]
                      + [ctypes.c_int] * 6 + [ctypes.c_int, _vp, ctypes.c_size_t, _vp]),
    "kla_chunk_fwd_static": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp, _fp, _ip, _ip, ctypes.c_int]
                             + [ctypes.c_int] * 6 + [ctypes.c_int, _vp]),
    "kla_chunk_fwd_opts": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp, _fp, _ip, _ip, ctypes.c_int]
                           + [ctypes.c_int] * 6 + [ctypes.c_int, _vp, ctypes.c_size_t, _vp, ctypes.c_uint]),
    "kla_chunk_fwd_diag_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int] * 6 + [ctypes.c_int, _ip, ctypes.c_int]),
    "kla_chunk_fwd_diag": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp, _fp, _ip, _ip, ctypes.c_int]
                           + [ctypes.c_int] * 6 + [ctypes.c_int, _vp, ctypes.c_size_t, _vp]),
    "kla_decode_step_diag": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp]
                             + [ctypes.c_int] * 4 + [ctypes.c_int, _vp]),
    "kla_chunk_fwd_diag_opts": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp, _fp, _ip, _ip, ctypes.c_int]
                                + [ctypes.c_int] * 6 + [ctypes.c_int, _vp, ctypes.c_size_t, _vp, ctypes.c_uint]),
    "kla_decode_step_diag_opts": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp]
                                  + [ctypes.c_int] * 4 + [ctypes.c_int, _vp, ctypes.c_uint]),
    "kla_chunk_bwd_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int] * 6 + [ctypes.c_int, _ip, ctypes.c_int]),
    "kla_chunk_bwd": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp, _fp, _vp, _vp, _vp, _fp, _fp, _fp,
                                     _ip, _ip, ctypes.c_int] + [ctypes.c_int] * 6 + [ctypes.c_int, _vp, ctypes.c_size_t, _vp]),
    "kla_chunk_bwd_opts": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp, _fp, _vp, _vp, _vp, _fp, _fp, _fp,
                                          _ip, _ip, ctypes.c_int] + [ctypes.c_int] * 6
                           + [ctypes.c_int, _vp, ctypes.c_size_t, _vp, ctypes.c_uint]),
    "kla_debug_chunk_stage": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp, _fp, _ip, _ip, ctypes.c_int]
                              + [ctypes.c_int] * 6 + [ctypes.c_int, _vp, ctypes.c_size_t, _vp, ctypes.c_int]),
    "kla_decode_step": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp]
                        + [ctypes.c_int] * 4 + [ctypes.c_int, _vp]),
    "kla_decode_step_opts": (ctypes.c_int, [_vp, _vp, _vp, _fp, _fp, ctypes.c_float, _fp, _vp]
                             + [ctypes.c_int] * 4 + [ctypes.c_int, _vp, ctypes.c_uint]),
    "kla_beta": (ctypes.c_int, [_vp, _fp, ctypes.c_float, _fp, ctypes.c_long, ctypes.c_int, ctypes.c_int, _vp]),
    "kla_debug_peak_probe": (ctypes.c_int, [ctypes.c_int, _vp, _vp, ctypes.c_size_t, ctypes.c_int, _vp]),
    "kla_debug_intra_chunk": (ctypes.c_int, [_vp, _vp, _fp, _fp, ctypes.c_float, _fp, _fp, _fp, _ip, _ip, ctypes.c_int]
                              + [ctypes.c_int] * 5 + [ctypes.c_int, _vp, ctypes.c_size_t, _vp]),
}


class KlaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %s" % (where, lib().kla_status_string(code).decode()))


def lib():
    """The loaded C library; raises if it has not been built (python -m paper_2605_08587_amd.build)."""
    global _lib
    with _lock:
        if _lib is None:
            if not os.path.exists(LIB_PATH):
                raise RuntimeError("libkla.so is not built: run `python -m paper_2605_08587_amd.build` "
                                   "(there is no CPU fallback)")
            l = ctypes.CDLL(LIB_PATH)
            for name, (res, args) in _SIGNATURES.items():
                fn = getattr(l, name)
                fn.restype, fn.argtypes = res, args
            _lib = l
    return _lib


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return KLA_BF16
    if t.dtype == torch.float32:
        return KLA_F32
    raise TypeError("q, k, v must be bfloat16 or float32, got %s" % t.dtype)


def _dev(*ts):
    for t in ts:
        if t is not None:
            if not t.is_cuda:
                raise RuntimeError("KLA kernels need GPU tensors (no CPU fallback)")
            if not t.is_contiguous():
                raise ValueError("tensors must be contiguous")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


# Tuning fields of the `opts` argument (KLA_TUNE_* of include/kla.h): for tests and A/B measurements.  DEFAULT_TUNE is
# what a call uses when it is given no `tune` of its own (binding-side convenience; the library keeps no such state).
KLA_TUNE_GENERIC_SCAN, KLA_TUNE_GENERIC_INTRA, KLA_TUNE_GENERIC_BWD, KLA_TUNE_UNFUSED, KLA_TUNE_FUSED = 1 << 15, 1 << 16, 1 << 17, 1 << 24, 1 << 25
DEFAULT_TUNE = 0


def tune(scan_waves=0, segments=0, generic_scan=False, generic_intra=False, generic_bwd=False, unfused=False, fused=False,
         decode_slice=0, decode_nt=None) -> int:
    """The tuning fields as one integer for the `tune` argument of the calls below (0 = the library's own choice)."""
    if scan_waves not in (0, 1, 2, 4) or not 0 <= segments <= 16 or decode_slice not in (0, 32, 64, 128, 256) \
            or decode_nt not in (None, 0, 1, 2, 3):
        raise ValueError("tuning value out of range")
    bits = ((3 if scan_waves == 4 else scan_waves) << 8) | (segments << 10)
    bits |= (KLA_TUNE_GENERIC_SCAN if generic_scan else 0) | (KLA_TUNE_GENERIC_INTRA if generic_intra else 0)
    bits |= (KLA_TUNE_GENERIC_BWD if generic_bwd else 0) | (KLA_TUNE_UNFUSED if unfused else 0) | (KLA_TUNE_FUSED if fused else 0)
    bits |= {0: 0, 32: 1, 64: 2, 128: 3, 256: 4}[decode_slice] << 18
    bits |= 0 if decode_nt is None else (decode_nt + 1) << 21
    return bits


def _tune(t):
    return DEFAULT_TUNE if t is None else int(t)


def _check(name, t, shape, dtype):
    """The C ABI sees raw pointers only: extents and element types are checked here, before anything is launched."""
    if t is None:
        return
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    if t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))


def _check_chunk(q, k, v, log_alpha, eta, h0, n_states, la_shape=None, **others):
    """q defines N, T, H, dk and the element type; everything else must fit it.  others: name -> (tensor, shape, dtype)."""
    if q.dim() != 4 or v.dim() != 4:
        raise ValueError("q, k must be [N, T, H, dk] and v [N, T, H, dv]")
    N, T, H, dk = q.shape
    dv = v.shape[-1]
    _dt(q)
    _check("k", k, (N, T, H, dk), q.dtype)
    _check("v", v, (N, T, H, dv), q.dtype)
    _check("log_alpha", log_alpha, la_shape or (N, T, H), torch.float32)
    _check("eta", eta, (N, T, H), torch.float32)
    _check("h0", h0, (n_states, H, dk, dv), torch.float32)
    for name, (t, shape, dtype) in others.items():
        _check(name, t, shape, dtype)
    return N, T, H, dk, dv


def _check_decode(q, k, v, log_alpha, eta, S, out, la_shape=None):
    if q.dim() != 3 or v.dim() != 3:
        raise ValueError("q, k must be [B, H, dk] and v [B, H, dv]")
    B, H, dk = q.shape
    dv = v.shape[-1]
    _dt(q)
    _check("k", k, (B, H, dk), q.dtype)
    _check("v", v, (B, H, dv), q.dtype)
    _check("log_alpha", log_alpha, la_shape or (B, H), torch.float32)
    _check("eta", eta, (B, H), torch.float32)
    _check("S", S, (B, H, dk, dv), torch.float32)
    _check("out", out, (B, H, dv), q.dtype)
    return B, H, dk, dv


def _host_cu(cu_seqlens, cu_seqlens_host=None):
    """Host copy of the sequence offsets.  Copying a device tensor synchronises: callers that must not (inside a
    stream capture, in a serving loop) pass the host copy they already have as cu_seqlens_host."""
    if cu_seqlens is None:
        return None, None, 0
    if cu_seqlens.dtype != torch.int32 or cu_seqlens.dim() != 1 or cu_seqlens.numel() < 1:
        raise TypeError("cu_seqlens must be a 1-d int32 tensor of n_seq + 1 offsets")
    src = cu_seqlens if cu_seqlens_host is None else cu_seqlens_host
    cu_host = src.detach().to("cpu", torch.int32).contiguous()
    if cu_host.numel() != cu_seqlens.numel():
        raise ValueError("cu_seqlens_host must hold the same offsets as cu_seqlens")
    return cu_host, ctypes.c_void_p(cu_host.data_ptr()), cu_host.numel() - 1


def kla_chunk_fwd_workspace_bytes(N, T, H, dk, dv, dtype, cu_seqlens=None, chunk=64, tune=None) -> int:
    cu_host, cu_hp, n_seq = _host_cu(cu_seqlens)
    dt = KLA_BF16 if dtype == torch.bfloat16 else KLA_F32
    return int(lib().kla_chunk_fwd_workspace_bytes_opts(N, T, H, dk, dv, chunk, dt, cu_hp, n_seq, _tune(tune)))


def _opts(normalize_q, gdn_beta) -> int:
    return (KLA_OPT_NORMALIZE_Q if normalize_q else 0) | (KLA_OPT_GDN_BETA if gdn_beta else 0)


def _ws_bytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def kla_chunk_fwd(q, k, v, log_alpha, eta, eps, h0=None, cu_seqlens=None, want_hT=True, workspace=None,
                  out=None, hT=None, chunk=64, _stage=None, normalize_q=False, gdn_beta=False, cu_seqlens_host=None,
                  tune=None):
    """Chunkwise forward.  q,k [N,T,H,dk], v [N,T,H,dv], gates [N,T,H] fp32; returns (o, hT).

    cu_seqlens: int32 device tensor [n_seq+1] for a packed batch (then N == 1); cu_seqlens_host: the same offsets
    as a CPU tensor, if the caller has them (saves the device-to-host copy, which synchronises).
    workspace / out / hT may be passed in to avoid allocations (e.g. inside a timed loop or a stream capture).
    normalize_q: o_t = S_t^T q_t / ||q_t||;  gdn_beta: beta_t = eta_t (kla_chunk_fwd_opts of the C ABI).
    tune: tuning fields (see tune()); None = DEFAULT_TUNE.
    """
    cu_host, cu_hp, n_seq = _host_cu(cu_seqlens, cu_seqlens_host)
    n_states = n_seq if n_seq > 0 else q.shape[0]
    N, T, H, dk, dv = _check_chunk(q, k, v, log_alpha, eta, h0, n_states,
                                   out=(out, (q.shape[0], q.shape[1], q.shape[2], v.shape[-1]), q.dtype),
                                   hT=(hT, (n_states, q.shape[2], q.shape[3], v.shape[-1]), torch.float32))
    _dev(q, k, v, log_alpha, eta, h0, cu_seqlens, workspace, out, hT)
    dt = _dt(q)
    bits = _opts(normalize_q, gdn_beta) | _tune(tune)
    if _stage is not None:
        if normalize_q or gdn_beta:
            raise ValueError("the single-stage hook takes no options")
        bits = KLA_TUNE_UNFUSED
    if workspace is None:
        need = int(lib().kla_chunk_fwd_workspace_bytes_opts(N, T, H, dk, dv, chunk, dt, cu_hp, n_seq, bits & ~3))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    if out is None:
        out = torch.empty((N, T, H, dv), dtype=q.dtype, device=q.device)
    if hT is None and want_hT:
        hT = torch.empty((n_states, H, dk, dv), dtype=torch.float32, device=q.device)
    args = (_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(eta), float(eps), _ptr(h0), _ptr(out),
            _ptr(hT), _ptr(cu_seqlens), cu_hp, n_seq, N, T, H, dk, dv, chunk, dt,
            _ptr(workspace), _ws_bytes(workspace), _stream())
    if _stage is not None:
        rc = lib().kla_debug_chunk_stage(*args, int(_stage))
    elif bits:
        rc = lib().kla_chunk_fwd_opts(*args, bits)
    else:
        rc = lib().kla_chunk_fwd(*args)
    if rc != 0:
        raise KlaError(rc, "kla_chunk_fwd")
    return out, hT


KLA_STATIC_SCRATCH_BYTES = 32 << 20


def kla_chunk_fwd_static(q, k, v, log_alpha, eta, eps, out, hT=None, h0=None, cu_seqlens=None, cu_seqlens_host=None,
                         chunk=64):
    """kla_chunk_fwd without a workspace and without any allocation (kla_chunk_fwd_static of the C ABI): the caller
    passes `out` (and `hT` if wanted); the per-chunk objects go to the library's fixed scratch array, so the problem
    must need at most KLA_STATIC_SCRATCH_BYTES of workspace.  For a packed batch pass cu_seqlens_host as well if the
    call must not synchronise.  Returns (out, hT)."""
    cu_host, cu_hp, n_seq = _host_cu(cu_seqlens, cu_seqlens_host)
    n_states = n_seq if n_seq > 0 else q.shape[0]
    N, T, H, dk, dv = _check_chunk(q, k, v, log_alpha, eta, h0, n_states,
                                   out=(out, (q.shape[0], q.shape[1], q.shape[2], v.shape[-1]), q.dtype),
                                   hT=(hT, (n_states, q.shape[2], q.shape[3], v.shape[-1]), torch.float32))
    _dev(q, k, v, log_alpha, eta, h0, cu_seqlens, out, hT)
    if out is None:
        raise ValueError("kla_chunk_fwd_static allocates nothing: pass `out`")
    rc = lib().kla_chunk_fwd_static(_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(eta), float(eps), _ptr(h0), _ptr(out),
                                    _ptr(hT), _ptr(cu_seqlens), cu_hp, n_seq, N, T, H, dk, dv, chunk, _dt(q), _stream())
    if rc != 0:
        raise KlaError(rc, "kla_chunk_fwd_static")
    return out, hT


def kla_chunk_fwd_diag(q, k, v, log_alpha, eta, eps, h0=None, cu_seqlens=None, want_hT=True, workspace=None,
                       out=None, hT=None, chunk=64, cu_seqlens_host=None, normalize_q=False, gdn_beta=False, tune=None):
    """Chunkwise forward with diagonal gating: log_alpha is [N,T,H,dk] fp32 (one decay per key channel).
    Everything else, the options included, as kla_chunk_fwd; returns (o, hT)."""
    cu_host, cu_hp, n_seq = _host_cu(cu_seqlens, cu_seqlens_host)
    n_states = n_seq if n_seq > 0 else q.shape[0]
    N, T, H, dk, dv = _check_chunk(q, k, v, log_alpha, eta, h0, n_states, la_shape=tuple(q.shape),
                                   out=(out, (q.shape[0], q.shape[1], q.shape[2], v.shape[-1]), q.dtype),
                                   hT=(hT, (n_states, q.shape[2], q.shape[3], v.shape[-1]), torch.float32))
    _dev(q, k, v, log_alpha, eta, h0, cu_seqlens, workspace, out, hT)
    dt = _dt(q)
    need = int(lib().kla_chunk_fwd_diag_workspace_bytes(N, T, H, dk, dv, chunk, dt, cu_hp, n_seq))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    if out is None:
        out = torch.empty((N, T, H, dv), dtype=q.dtype, device=q.device)
    if hT is None and want_hT:
        hT = torch.empty((n_states, H, dk, dv), dtype=torch.float32, device=q.device)
    args = (_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(eta), float(eps), _ptr(h0), _ptr(out),
            _ptr(hT), _ptr(cu_seqlens), cu_hp, n_seq, N, T, H, dk, dv, chunk, dt,
            _ptr(workspace), _ws_bytes(workspace), _stream())
    bits = _opts(normalize_q, gdn_beta) | _tune(tune)
    rc = lib().kla_chunk_fwd_diag_opts(*args, bits) if bits else lib().kla_chunk_fwd_diag(*args)
    if rc != 0:
        raise KlaError(rc, "kla_chunk_fwd_diag")
    return out, hT


def kla_decode_step_diag(q, k, v, log_alpha, eta, eps, S, out=None, normalize_q=False, gdn_beta=False, tune=None):
    """One decode step with diagonal gating: log_alpha is [B,H,dk]; S [B,H,dk,dv] fp32 is updated in place."""
    B, H, dk, dv = _check_decode(q, k, v, log_alpha, eta, S, out, la_shape=tuple(q.shape))
    _dev(q, k, v, log_alpha, eta, S, out)
    if out is None:
        out = torch.empty((B, H, dv), dtype=q.dtype, device=q.device)
    args = (_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(eta), float(eps), _ptr(S), _ptr(out), B, H, dk, dv, _dt(q),
            _stream())
    bits = _opts(normalize_q, gdn_beta) | _tune(tune)
    rc = lib().kla_decode_step_diag_opts(*args, bits) if bits else lib().kla_decode_step_diag(*args)
    if rc != 0:
        raise KlaError(rc, "kla_decode_step_diag")
    return out


def kla_chunk_bwd_workspace_bytes(N, T, H, dk, dv, dtype, cu_seqlens=None, chunk=64, tune=None) -> int:
    cu_host, cu_hp, n_seq = _host_cu(cu_seqlens)
    dt = KLA_BF16 if dtype == torch.bfloat16 else KLA_F32
    return int(lib().kla_chunk_bwd_workspace_bytes_opts(N, T, H, dk, dv, chunk, dt, cu_hp, n_seq, _tune(tune)))


def kla_chunk_bwd(q, k, v, log_alpha, eta, eps, d_o, h0=None, d_hT=None, cu_seqlens=None, want_dh0=True,
                  workspace=None, out=None, chunk=64, gdn_beta=False, normalize_q=False, cu_seqlens_host=None, tune=None):
    """Backward of kla_chunk_fwd: gradients of sum <d_o, o> + sum <d_hT, hT>.  gdn_beta, normalize_q: of the forward
    with the same options (kla_chunk_bwd_opts of the C ABI).

    d_o [N,T,H,dv] in the dtype of q; d_hT [n_states,H,dk,dv] fp32 or None (zeros).
    Returns a dict: dq, dk, dv (dtype of q), dlog_alpha, deta (fp32 [N,T,H]), dh0 (fp32, or None).
    `out` may hold preallocated tensors under the same names; `workspace` a uint8 buffer.
    """
    cu_host, cu_hp, n_seq = _host_cu(cu_seqlens, cu_seqlens_host)
    n_states = n_seq if n_seq > 0 else q.shape[0]
    out = dict(out or {})
    sq, sv, sg, ss = tuple(q.shape), tuple(q.shape[:3]) + (v.shape[-1],), tuple(q.shape[:3]), (n_states, q.shape[2], q.shape[3], v.shape[-1])
    N, T, H, dk, dv = _check_chunk(q, k, v, log_alpha, eta, h0, n_states, d_o=(d_o, sv, q.dtype), d_hT=(d_hT, ss, torch.float32),
                                   dq=(out.get("dq"), sq, q.dtype), dk=(out.get("dk"), sq, q.dtype),
                                   dv=(out.get("dv"), sv, q.dtype), dlog_alpha=(out.get("dlog_alpha"), sg, torch.float32),
                                   deta=(out.get("deta"), sg, torch.float32), dh0=(out.get("dh0"), ss, torch.float32))
    if d_o is None:
        raise ValueError("d_o is required")
    _dev(q, k, v, log_alpha, eta, d_o, h0, d_hT, cu_seqlens, workspace, *out.values())
    dt = _dt(q)
    bits = _opts(normalize_q, gdn_beta) | _tune(tune)
    if workspace is None:
        need = int(lib().kla_chunk_bwd_workspace_bytes_opts(N, T, H, dk, dv, chunk, dt, cu_hp, n_seq, bits & ~3))
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    for name, like in (("dq", q), ("dk", k), ("dv", v)):
        if name not in out:
            out[name] = torch.empty_like(like)
    for name in ("dlog_alpha", "deta"):
        if name not in out:
            out[name] = torch.empty((N, T, H), dtype=torch.float32, device=q.device)
    if "dh0" not in out:
        out["dh0"] = torch.empty((n_states, H, dk, dv), dtype=torch.float32, device=q.device) if want_dh0 else None
    args = (_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(eta), float(eps), _ptr(h0), _ptr(d_o),
            _ptr(d_hT), _ptr(out["dq"]), _ptr(out["dk"]), _ptr(out["dv"]), _ptr(out["dlog_alpha"]),
            _ptr(out["deta"]), _ptr(out["dh0"]), _ptr(cu_seqlens), cu_hp, n_seq, N, T, H, dk, dv, chunk,
            dt, _ptr(workspace), _ws_bytes(workspace), _stream())
    rc = lib().kla_chunk_bwd_opts(*args, bits) if bits else lib().kla_chunk_bwd(*args)
    if rc != 0:
        raise KlaError(rc, "kla_chunk_bwd")
    return out


def kla_debug_chunk_stage(stage, q, k, v, log_alpha, eta, eps, workspace, out, hT=None, h0=None, cu_seqlens=None):
    """Profiling hook: stage 1 (intra-chunk) or stage 2 (scan) of the two-kernel form of kla_chunk_fwd alone, on
    preallocated buffers; the workspace is that of kla_chunk_fwd_workspace_bytes(..., tune=tune(unfused=True))."""
    return kla_chunk_fwd(q, k, v, log_alpha, eta, eps, h0=h0, cu_seqlens=cu_seqlens, want_hT=hT is not None,
                         workspace=workspace, out=out, hT=hT, _stage=stage)


def kla_decode_step(q, k, v, log_alpha, eta, eps, S, out=None, normalize_q=False, gdn_beta=False, tune=None):
    """One decode step; S [B,H,dk,dv] fp32 is updated in place; returns o [B,H,dv].  Options as in kla_chunk_fwd."""
    B, H, dk, dv = _check_decode(q, k, v, log_alpha, eta, S, out)
    _dev(q, k, v, log_alpha, eta, S, out)
    if out is None:
        out = torch.empty((B, H, dv), dtype=q.dtype, device=q.device)
    args = (_ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(eta), float(eps), _ptr(S), _ptr(out),
            B, H, dk, dv, _dt(q), _stream())
    bits = _opts(normalize_q, gdn_beta) | _tune(tune)
    rc = lib().kla_decode_step_opts(*args, bits) if bits else lib().kla_decode_step(*args)
    if rc != 0:
        raise KlaError(rc, "kla_decode_step")
    return out


def kla_beta(k, eta, eps, out=None):
    """beta = eta / (||k||^2 + eps) for k [..., dk], eta [...]; returns fp32 [...]."""
    _dt(k)
    dk = k.shape[-1]
    n = k.numel() // dk
    _check("eta", eta, tuple(k.shape[:-1]), torch.float32)
    _check("out", out, tuple(k.shape[:-1]), torch.float32)
    _dev(k, eta, out)
    if out is None:
        out = torch.empty(k.shape[:-1], dtype=torch.float32, device=k.device)
    rc = lib().kla_beta(_ptr(k), _ptr(eta), float(eps), _ptr(out), n, dk, _dt(k), _stream())
    if rc != 0:
        raise KlaError(rc, "kla_beta")
    return out


def kla_debug_intra_chunk(q, k, log_alpha, eta, eps, cu_seqlens=None, chunk=64):
    """Test hook: (Tb, P, g) of every chunk as fp32 [n_chunks, H, 64, 64] / [n_chunks, H, 64]."""
    if q.dim() != 4:
        raise ValueError("q, k must be [N, T, H, dk]")
    N, T, H, dk = q.shape
    dt = _dt(q)
    _check("k", k, (N, T, H, dk), q.dtype)
    _check("log_alpha", log_alpha, (N, T, H), torch.float32)
    _check("eta", eta, (N, T, H), torch.float32)
    _dev(q, k, log_alpha, eta, cu_seqlens)
    cu_host, cu_hp, n_seq = _host_cu(cu_seqlens)
    if n_seq > 0:
        n_chunks = int(((cu_host[1:] - cu_host[:-1] + 63) // 64).sum())
    else:
        n_chunks = N * ((T + 63) // 64)
    need = int(lib().kla_chunk_fwd_workspace_bytes_opts(N, T, H, dk, 64, chunk, dt, cu_hp, n_seq, KLA_TUNE_UNFUSED))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    Tb = torch.zeros((n_chunks, H, 64, 64), dtype=torch.float32, device=q.device)
    P = torch.zeros_like(Tb)
    g = torch.zeros((n_chunks, H, 64), dtype=torch.float32, device=q.device)
    rc = lib().kla_debug_intra_chunk(_ptr(q), _ptr(k), _ptr(log_alpha), _ptr(eta), float(eps), _ptr(Tb), _ptr(P),
                                     _ptr(g), _ptr(cu_seqlens), cu_hp, n_seq, N, T, H, dk, chunk, dt, _ptr(ws),
                                     ws.numel(), _stream())
    if rc != 0:
        raise KlaError(rc, "kla_debug_intra_chunk")
    return Tb, P, g


def kla_debug_peak_probe(kind, buf=None, aux=None, n=0, iters=0):
    """Measurement hook (kla_debug_peak_probe of the C ABI): kind 0 in-place streaming over the fp32 tensor `buf`
    (iters != 0: non-temporal), kind 1 read-only streaming of `buf` (aux: fp32, buf bytes / 16384 elements), kind 2 dense
    bf16 matrix pipe on `n` workgroups x `iters` rounds (aux: fp32, 256 n elements), kind 3 the chunk kernels' copy wave
    alone reading `buf` (iters = copies of 1 KiB per step + 256 (ring depth - 1))."""
    _dev(buf, aux)
    size = n if kind == 2 else buf.numel() * buf.element_size()
    if kind == 1 and (aux is None or aux.numel() * aux.element_size() < size // 4096):
        raise ValueError("aux too small")
    if kind == 2 and (aux is None or aux.numel() < 256 * n):
        raise ValueError("aux too small")
    rc = lib().kla_debug_peak_probe(int(kind), _ptr(buf), _ptr(aux), size, int(iters), _stream())
    if rc != 0:
        raise KlaError(rc, "kla_debug_peak_probe")


class _KlaChunk(torch.autograd.Function):
    """kla_chunk_fwd / kla_chunk_bwd as one differentiable call (marshalling only: every step runs in the library)."""

    @staticmethod
    def forward(ctx, q, k, v, log_alpha, eta, h0, eps, cu_seqlens, cu_seqlens_host, normalize_q, gdn_beta):
        o, hT = kla_chunk_fwd(q, k, v, log_alpha, eta, eps, h0=h0, cu_seqlens=cu_seqlens, cu_seqlens_host=cu_seqlens_host,
                              normalize_q=normalize_q, gdn_beta=gdn_beta)
        ctx.save_for_backward(q, k, v, log_alpha, eta, h0 if h0 is not None else q.new_empty(0))
        ctx.misc = (eps, cu_seqlens, cu_seqlens_host, normalize_q, gdn_beta, h0 is not None)
        return o, hT

    @staticmethod
    def backward(ctx, d_o, d_hT):
        q, k, v, log_alpha, eta, h0 = ctx.saved_tensors
        eps, cu_seqlens, cu_seqlens_host, normalize_q, gdn_beta, has_h0 = ctx.misc
        g = kla_chunk_bwd(q, k, v, log_alpha, eta, eps, d_o.contiguous(), h0=h0 if has_h0 else None,
                          d_hT=None if d_hT is None else d_hT.contiguous(), cu_seqlens=cu_seqlens,
                          cu_seqlens_host=cu_seqlens_host, want_dh0=has_h0 and ctx.needs_input_grad[5],
                          normalize_q=normalize_q, gdn_beta=gdn_beta)
        return (g["dq"], g["dk"], g["dv"], g["dlog_alpha"], g["deta"], g["dh0"], None, None, None, None, None)


def kla_chunk(q, k, v, log_alpha, eta, eps, h0=None, cu_seqlens=None, cu_seqlens_host=None, normalize_q=False,
              gdn_beta=False):
    """Differentiable chunkwise forward for training loops: returns (o, hT) like kla_chunk_fwd; gradients with respect to
    q, k, v, log_alpha, eta and h0 come from kla_chunk_bwd (the forward is recomputed there, nothing else is saved)."""
    return _KlaChunk.apply(q, k, v, log_alpha, eta, h0, eps, cu_seqlens, cu_seqlens_host, normalize_q, gdn_beta)
