"""ctypes front end of the fp64 token-by-token oracle (oracle/kla_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
CPU-baseline leg of the benchmark.  Nothing here touches the GPU library and
the GPU library never imports this.

The arithmetic lives in the C file (Algorithm 1, left panel, with the
coefficient of eq. (3)); this module only marshals numpy arrays and spreads the
independent (sequence, head) units over host threads (ctypes drops the GIL
during the call).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kla_oracle.c")
_LIB = os.path.join(_HERE, "libkla_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math: summation order is kept).  KLA_ORACLE_LIBRARY names another build
    of the same source (the host-sanitizer run of tests/host_sanitizers.py uses it)."""
    if os.environ.get("KLA_ORACLE_LIBRARY"):
        return os.environ["KLA_ORACLE_LIBRARY"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            fp = ctypes.POINTER(ctypes.c_float)
            dp = ctypes.POINTER(ctypes.c_double)
            lib.kla_oracle_sequence.restype = ctypes.c_int
            lib.kla_oracle_sequence.argtypes = [fp, fp, fp, dp, dp, ctypes.c_double, dp, dp, dp,
                                                ctypes.c_long, ctypes.c_long, ctypes.c_int,
                                                ctypes.c_int, ctypes.c_int, ctypes.c_int]
            lib.kla_oracle_sequence_opts.restype = ctypes.c_int
            lib.kla_oracle_sequence_opts.argtypes = lib.kla_oracle_sequence.argtypes + [ctypes.c_int, ctypes.c_int]
            lib.kla_oracle_decode_unit.restype = ctypes.c_int
            lib.kla_oracle_decode_unit.argtypes = [fp, fp, fp, ctypes.c_double, ctypes.c_double,
                                                   ctypes.c_double, dp, dp, ctypes.c_int, ctypes.c_int]
            lib.kla_oracle_decode_unit_opts.restype = ctypes.c_int
            lib.kla_oracle_decode_unit_opts.argtypes = lib.kla_oracle_decode_unit.argtypes + [ctypes.c_int, ctypes.c_int]
            lib.kla_oracle_sequence_diag_opts.restype = ctypes.c_int
            lib.kla_oracle_sequence_diag_opts.argtypes = lib.kla_oracle_sequence.argtypes + [ctypes.c_int, ctypes.c_int]
            lib.kla_oracle_decode_unit_diag_opts.restype = ctypes.c_int
            lib.kla_oracle_decode_unit_diag_opts.argtypes = [fp, fp, fp, dp, ctypes.c_double, ctypes.c_double, dp, dp,
                                                             ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
            lib.kla_oracle_sequence_bwd_opts.restype = ctypes.c_int
            lib.kla_oracle_sequence_bwd_opts.argtypes = [fp, fp, fp, dp, dp, ctypes.c_double, dp, dp, dp,
                                                    dp, dp, dp, dp, dp, dp,
                                                    ctypes.c_long, ctypes.c_long, ctypes.c_int,
                                                    ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                    ctypes.c_int]
            _lib = lib
    return _lib


def _f32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _fp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _dp(a, offset_elems=0):
    return ctypes.cast(a.ctypes.data + 8 * offset_elems, ctypes.POINTER(ctypes.c_double))


def default_threads() -> int:
    return len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)


def kla_recurrent(q, k, v, log_alpha, eta, eps, h0=None, cu_seqlens=None, threads=None, units=None,
                  normalize_q=False, gdn_beta=False):
    """Whole-batch recurrence.

    q, k: [N, T, H, dk]; v: [N, T, H, dv]; log_alpha, eta: [N, T, H];
    h0: [n_seq, H, dk, dv] or None.  With cu_seqlens (n_seq+1 offsets into the
    token axis) N must be 1 and the sequences are packed along T.
    `units`, if given, restricts the work to those (sequence, head) pairs; the
    other rows of the outputs stay zero.
    normalize_q: readout divided by ||q_t|| (Sec. 3.3); gdn_beta: beta_t = eta_t (no key-norm denominator).
    Returns (o [N, T, H, dv] float64, hT [n_seq, H, dk, dv] float64, threads_used).
    """
    lib = _load()
    q, k, v = _f32(q), _f32(k), _f32(v)
    la, et = _f64(log_alpha), _f64(eta)
    N, T, H, dk = q.shape
    dv = v.shape[-1]
    if cu_seqlens is None:
        starts = [n * T for n in range(N)]
        lens = [T] * N
    else:
        assert N == 1
        cu = [int(x) for x in cu_seqlens]
        starts = cu[:-1]
        lens = [cu[i + 1] - cu[i] for i in range(len(cu) - 1)]
    n_seq = len(starts)
    h0d = None if h0 is None else _f64(h0)
    o = np.zeros((N, T, H, dv), dtype=np.float64)
    hT = np.zeros((n_seq, H, dk, dv), dtype=np.float64)
    todo = [(s, h) for s in range(n_seq) for h in range(H)] if units is None else list(units)

    def run(unit):
        s, h = unit
        off = (s * H + h) * dk * dv
        rc = lib.kla_oracle_sequence_opts(_fp(q), _fp(k), _fp(v), _dp(la), _dp(et), float(eps),
                                          None if h0d is None else _dp(h0d, off), _dp(o), _dp(hT, off),
                                          starts[s], lens[s], h, H, dk, dv, int(normalize_q), int(gdn_beta))
        if rc != 0:
            raise MemoryError("oracle scratch allocation failed")

    nthr = max(1, min(threads or default_threads(), len(todo))) if todo else 1
    if nthr == 1:
        for u in todo:
            run(u)
    else:
        with ThreadPoolExecutor(nthr) as ex:
            list(ex.map(run, todo))
    return o, hT, nthr


def kla_recurrent_diag(q, k, v, log_alpha, eta, eps, h0=None, cu_seqlens=None, threads=None, units=None,
                       normalize_q=False, gdn_beta=False):
    """kla_recurrent with diagonal gating (App. B): log_alpha is [N, T, H, dk], one decay per key channel.
    normalize_q, gdn_beta: as in kla_recurrent."""
    lib = _load()
    q, k, v = _f32(q), _f32(k), _f32(v)
    la, et = _f64(log_alpha), _f64(eta)
    N, T, H, dk = q.shape
    dv = v.shape[-1]
    assert la.shape == (N, T, H, dk)
    if cu_seqlens is None:
        starts = [n * T for n in range(N)]
        lens = [T] * N
    else:
        assert N == 1
        cu = [int(x) for x in cu_seqlens]
        starts = cu[:-1]
        lens = [cu[i + 1] - cu[i] for i in range(len(cu) - 1)]
    n_seq = len(starts)
    h0d = None if h0 is None else _f64(h0)
    o = np.zeros((N, T, H, dv), dtype=np.float64)
    hT = np.zeros((n_seq, H, dk, dv), dtype=np.float64)
    todo = [(s, h) for s in range(n_seq) for h in range(H)] if units is None else list(units)

    def run(unit):
        s, h = unit
        off = (s * H + h) * dk * dv
        rc = lib.kla_oracle_sequence_diag_opts(_fp(q), _fp(k), _fp(v), _dp(la), _dp(et), float(eps),
                                               None if h0d is None else _dp(h0d, off), _dp(o), _dp(hT, off),
                                               starts[s], lens[s], h, H, dk, dv, int(normalize_q), int(gdn_beta))
        if rc != 0:
            raise MemoryError("oracle scratch allocation failed")

    nthr = max(1, min(threads or default_threads(), len(todo))) if todo else 1
    if nthr == 1:
        for u in todo:
            run(u)
    else:
        with ThreadPoolExecutor(nthr) as ex:
            list(ex.map(run, todo))
    return o, hT, nthr


def kla_decode_diag(q, k, v, log_alpha, eta, eps, S, threads=None, normalize_q=False, gdn_beta=False):
    """kla_decode with diagonal gating: log_alpha is [B, H, dk].  Returns (o, S_new); S is not modified."""
    lib = _load()
    q, k, v = _f32(q), _f32(k), _f32(v)
    la, et = _f64(log_alpha), _f64(eta)
    S = np.array(S, dtype=np.float64, order="C", copy=True)
    B, H, dk = q.shape
    dv = v.shape[-1]
    o = np.zeros((B, H, dv), dtype=np.float64)
    for u in range(B * H):
        rc = lib.kla_oracle_decode_unit_diag_opts(
            ctypes.cast(q.ctypes.data + 4 * u * dk, ctypes.POINTER(ctypes.c_float)),
            ctypes.cast(k.ctypes.data + 4 * u * dk, ctypes.POINTER(ctypes.c_float)),
            ctypes.cast(v.ctypes.data + 4 * u * dv, ctypes.POINTER(ctypes.c_float)),
            _dp(la, u * dk), float(et.reshape(-1)[u]), float(eps), _dp(S, u * dk * dv), _dp(o, u * dv), dk, dv,
            int(normalize_q), int(gdn_beta))
        if rc != 0:
            raise MemoryError("oracle scratch allocation failed")
    return o, S


def kla_recurrent_bwd(q, k, v, log_alpha, eta, eps, d_o, h0=None, d_hT=None, cu_seqlens=None, threads=None,
                      units=None, gdn_beta=False, normalize_q=False):
    """Gradient of L = sum <d_o, o> + sum <d_hT, hT> of kla_recurrent with respect to its inputs.

    Shapes as in kla_recurrent; d_o: [N, T, H, dv]; d_hT: [n_seq, H, dk, dv] or None (zeros).
    `units`, if given, restricts the work to those (sequence, head) pairs; other rows stay zero.
    gdn_beta: gradient of the recurrence with beta_t = eta_t; normalize_q: of the read-out divided by ||q_t||.
    Returns a dict with dq, dk, dv, dlog_alpha, deta, dh0 (float64, shapes of the corresponding inputs).
    """
    lib = _load()
    q, k, v = _f32(q), _f32(k), _f32(v)
    la, et, go = _f64(log_alpha), _f64(eta), _f64(d_o)
    N, T, H, dk = q.shape
    dv = v.shape[-1]
    if cu_seqlens is None:
        starts = [n * T for n in range(N)]
        lens = [T] * N
    else:
        assert N == 1
        cu = [int(x) for x in cu_seqlens]
        starts = cu[:-1]
        lens = [cu[i + 1] - cu[i] for i in range(len(cu) - 1)]
    n_seq = len(starts)
    h0d = None if h0 is None else _f64(h0)
    ghT = None if d_hT is None else _f64(d_hT)
    out = {"dq": np.zeros((N, T, H, dk)), "dk": np.zeros((N, T, H, dk)), "dv": np.zeros((N, T, H, dv)),
           "dlog_alpha": np.zeros((N, T, H)), "deta": np.zeros((N, T, H)), "dh0": np.zeros((n_seq, H, dk, dv))}
    todo = [(s, h) for s in range(n_seq) for h in range(H)] if units is None else list(units)

    def run(unit):
        s, h = unit
        off = (s * H + h) * dk * dv
        rc = lib.kla_oracle_sequence_bwd_opts(_fp(q), _fp(k), _fp(v), _dp(la), _dp(et), float(eps),
                                         None if h0d is None else _dp(h0d, off), _dp(go),
                                         None if ghT is None else _dp(ghT, off),
                                         _dp(out["dq"]), _dp(out["dk"]), _dp(out["dv"]), _dp(out["dlog_alpha"]),
                                         _dp(out["deta"]), _dp(out["dh0"], off),
                                         starts[s], lens[s], h, H, dk, dv, int(normalize_q), int(gdn_beta))
        if rc != 0:
            raise MemoryError("oracle scratch allocation failed")

    nthr = max(1, min(threads or default_threads(), len(todo))) if todo else 1
    if nthr == 1:
        for u in todo:
            run(u)
    else:
        with ThreadPoolExecutor(nthr) as ex:
            list(ex.map(run, todo))
    return out


def kla_decode(q, k, v, log_alpha, eta, eps, S, threads=None, normalize_q=False, gdn_beta=False):
    """One decode step for every (batch, head).

    q, k: [B, H, dk]; v: [B, H, dv]; log_alpha, eta: [B, H]; S: [B, H, dk, dv].
    Returns (o [B, H, dv] float64, S_new [B, H, dk, dv] float64); S is not modified.
    """
    lib = _load()
    q, k, v = _f32(q), _f32(k), _f32(v)
    la, et = _f64(log_alpha), _f64(eta)
    S = np.array(S, dtype=np.float64, order="C", copy=True)
    B, H, dk = q.shape
    dv = v.shape[-1]
    o = np.zeros((B, H, dv), dtype=np.float64)

    def run(u):
        rc = lib.kla_oracle_decode_unit_opts(
            ctypes.cast(q.ctypes.data + 4 * u * dk, ctypes.POINTER(ctypes.c_float)),
            ctypes.cast(k.ctypes.data + 4 * u * dk, ctypes.POINTER(ctypes.c_float)),
            ctypes.cast(v.ctypes.data + 4 * u * dv, ctypes.POINTER(ctypes.c_float)),
            float(la.reshape(-1)[u]), float(et.reshape(-1)[u]), float(eps),
            _dp(S, u * dk * dv), _dp(o, u * dv), dk, dv, int(normalize_q), int(gdn_beta))
        if rc != 0:
            raise MemoryError("oracle scratch allocation failed")

    n = B * H
    nthr = max(1, min(threads or default_threads(), n))
    if nthr == 1:
        for u in range(n):
            run(u)
    else:
        with ThreadPoolExecutor(nthr) as ex:
            list(ex.map(run, range(n)))
    return o, S


def rel_err(x, ref) -> float:
    """max|x - ref| / max|ref| over the whole tensor (the parity metric)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = float(np.max(np.abs(ref))) if ref.size else 0.0
    num = float(np.max(np.abs(x - ref))) if ref.size else 0.0
    if den == 0.0:
        return num
    return num / den
