"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/kla.h declares, and every validation error is reported before anything is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2605_08587_amd as kla

pytestmark = pytest.mark.skipif(not os.path.exists(kla.LIB_PATH),
                                reason="libkla.so not built (python -m paper_2605_08587_amd.build)")

OK, E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_WS, E_SEQ, E_HIP = 0, -1, -2, -3, -4, -5, -6, -7


def _declared_functions():
    src = open(kla.HEADER_PATH).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(kla_[a-z_0-9]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"kla_chunk_fwd", "kla_decode_step", "kla_beta", "kla_chunk_fwd_workspace_bytes", "kla_status_string",
            "kla_debug_intra_chunk", "kla_chunk_fwd_opts", "kla_decode_step_opts"} <= set(names)
    lib = ctypes.CDLL(kla.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings():
    lib = kla.lib()
    for code in range(0, -8, -1):
        s = lib.kla_status_string(code).decode()
        assert s.startswith("KLA_")
    assert "unknown" in lib.kla_status_string(-99).decode()


UNFUSED = kla.tune(unfused=True)


def test_workspace_bytes():
    lib = kla.lib()
    f = lambda *a: lib.kla_chunk_fwd_workspace_bytes_opts(*a, UNFUSED)
    # two-kernel form, 4096 chunk-heads, bf16: a record of 2 x 6 KiB operand areas + 3 x 256 B of per-token factors, and
    # 512 B of g and 1/|q| each, plus the (empty) offsets table
    n = f(8, 4096, 8, 128, 128, 64, kla.KLA_BF16, None, 0)
    assert n >= 4096 * (2 * 6144 + 768 + 512) and n <= 4096 * (2 * 6144 + 768 + 512) + 4 * 256
    assert f(8, 4096, 8, 128, 128, 64, kla.KLA_F32, None, 0) > n
    assert f(8, 4096, 8, 128, 128, 32, kla.KLA_BF16, None, 0) == 0        # chunk != 64
    assert f(8, 4096, 8, 96, 128, 64, kla.KLA_BF16, None, 0) == 0         # bad dk
    cu = np.array([0, 10, 10, 200], dtype=np.int32)                       # 1 + 0 + 3 chunks
    n2 = f(1, 200, 2, 64, 64, 64, kla.KLA_BF16, cu.ctypes.data, 3)
    assert n2 >= 4 * 2 * (2 * 6144 + 768 + 512)
    bad = np.array([0, 10, 5, 200], dtype=np.int32)
    assert f(1, 200, 2, 64, 64, 64, kla.KLA_BF16, bad.ctypes.data, 3) == 0
    # the plain query is the one with opts = 0; where the fused bf16 kernel runs nothing of the workspace is used and
    # a token 256 bytes are reported; fp32 and wide value heads (four compute waves per workgroup) keep the two kernels
    g = lib.kla_chunk_fwd_workspace_bytes
    assert g(8, 4096, 8, 128, 128, 64, kla.KLA_BF16, None, 0) == 256
    assert g(8, 4096, 8, 128, 128, 64, kla.KLA_BF16, None, 0) == lib.kla_chunk_fwd_workspace_bytes_opts(
        8, 4096, 8, 128, 128, 64, kla.KLA_BF16, None, 0, 0)
    assert g(8, 4096, 8, 128, 128, 64, kla.KLA_F32, None, 0) == f(8, 4096, 8, 128, 128, 64, kla.KLA_F32, None, 0)
    assert g(64, 4096, 16, 128, 256, 64, kla.KLA_BF16, None, 0) == f(64, 4096, 16, 128, 256, 64, kla.KLA_BF16, None, 0)
    assert g(2, 2048, 8, 128, 128, 64, kla.KLA_BF16, None, 0) == f(2, 2048, 8, 128, 128, 64, kla.KLA_BF16, None, 0)    # few chains
    assert lib.kla_chunk_fwd_workspace_bytes_opts(2, 2048, 8, 128, 128, 64, kla.KLA_BF16, None, 0, kla.tune(fused=True)) == 256
    assert g(1, 200, 2, 64, 64, 64, kla.KLA_BF16, bad.ctypes.data, 3) == 0
    # tuning fields out of range are refused (0 from the queries, KLA_ERR_SHAPE from the calls)
    assert lib.kla_chunk_fwd_workspace_bytes_opts(8, 4096, 8, 128, 128, 64, kla.KLA_BF16, None, 0, 17 << 10) == 0
    assert lib.kla_chunk_fwd_workspace_bytes_opts(8, 4096, 8, 128, 128, 64, kla.KLA_BF16, None, 0, 1 << 26) == 0
    assert lib.kla_chunk_fwd_workspace_bytes_opts(8, 4096, 8, 128, 128, 64, kla.KLA_BF16, None, 0, 3 << 24) == 0   # fused and unfused
    assert lib.kla_chunk_fwd_workspace_bytes_opts(8, 4096, 8, 128, 128, 64, kla.KLA_BF16, None, 0, 4) == 0


def test_tune_bits_match_the_header():
    """The binding's tune() builds the KLA_TUNE_* fields of include/kla.h."""
    hdr = open(kla.HEADER_PATH).read()
    for name, val in (("KLA_TUNE_GENERIC_SCAN", 15), ("KLA_TUNE_GENERIC_INTRA", 16), ("KLA_TUNE_GENERIC_BWD", 17),
                      ("KLA_TUNE_UNFUSED", 24), ("KLA_TUNE_FUSED", 25)):
        assert re.search(r"#define %s\s+\(1u << %d\)" % (name, val), hdr), name
        assert getattr(kla, name) == 1 << val
    assert kla.tune(scan_waves=4) == 3 << 8 and kla.tune(scan_waves=2) == 2 << 8
    assert kla.tune(segments=16) == 16 << 10
    assert kla.tune(decode_slice=256) == 4 << 18 and kla.tune(decode_slice=32) == 1 << 18
    assert kla.tune(decode_nt=0) == 1 << 21 and kla.tune(decode_nt=3) == 4 << 21
    assert kla.tune(generic_scan=True, generic_intra=True, generic_bwd=True, unfused=True) == (7 << 15) | (1 << 24)
    with pytest.raises(ValueError):
        kla.tune(scan_waves=3)


def _chunk_call(**over):
    """kla_chunk_fwd with fake but well-aligned non-NULL device pointers; only validation can run."""
    a = dict(q=0x1000, k=0x2000, v=0x3000, la=0x4000, eta=0x5000, eps=1e-6, h0=None, o=0x6000, hT=None,
             cu_dev=None, cu_host=None, n_seq=0, N=1, T=64, H=1, dk=64, dv=64, chunk=64, dt=kla.KLA_BF16,
             ws=0x100000, ws_bytes=1 << 30, stream=None)
    a.update(over)
    return kla.lib().kla_chunk_fwd(a["q"], a["k"], a["v"], a["la"], a["eta"], a["eps"], a["h0"], a["o"], a["hT"],
                                   a["cu_dev"], a["cu_host"], a["n_seq"], a["N"], a["T"], a["H"], a["dk"], a["dv"],
                                   a["chunk"], a["dt"], a["ws"], a["ws_bytes"], a["stream"])


def test_chunk_fwd_validation_errors():
    assert _chunk_call(q=None) == E_NULL
    assert _chunk_call(o=None) == E_NULL
    assert _chunk_call(eta=None) == E_NULL
    assert _chunk_call(dk=96) == E_SHAPE
    assert _chunk_call(dv=32) == E_SHAPE
    assert _chunk_call(chunk=128) == E_SHAPE
    assert _chunk_call(H=0) == E_SHAPE
    assert _chunk_call(eps=-1.0) == E_SHAPE
    assert _chunk_call(eps=float("nan")) == E_SHAPE
    assert _chunk_call(dt=7) == E_DTYPE
    assert _chunk_call(q=0x1004) == E_ALIGN
    assert _chunk_call(h0=0x7008) == E_ALIGN
    assert _chunk_call(ws=None) == E_WS
    assert _chunk_call(ws=0x100010) == E_WS
    assert _chunk_call(ws_bytes=100) == E_WS
    cu = np.array([0, 30, 64], dtype=np.int32)
    assert _chunk_call(n_seq=2, cu_host=cu.ctypes.data, cu_dev=None) == E_NULL
    assert _chunk_call(n_seq=2, cu_host=None, cu_dev=0x8000) == E_NULL
    assert _chunk_call(n_seq=2, cu_host=cu.ctypes.data, cu_dev=0x8000, N=2) == E_SHAPE
    assert _chunk_call(n_seq=0, cu_host=cu.ctypes.data) == E_SHAPE
    bad = np.array([0, 40, 30], dtype=np.int32)
    assert _chunk_call(n_seq=2, cu_host=bad.ctypes.data, cu_dev=0x8000) == E_SEQ
    bad = np.array([1, 40, 64], dtype=np.int32)
    assert _chunk_call(n_seq=2, cu_host=bad.ctypes.data, cu_dev=0x8000) == E_SEQ
    bad = np.array([0, 40, 63], dtype=np.int32)
    assert _chunk_call(n_seq=2, cu_host=bad.ctypes.data, cu_dev=0x8000) == E_SEQ
    # nothing to do: no sequences at all
    assert _chunk_call(N=0) == OK


def test_decode_and_beta_validation_errors():
    lib = kla.lib()
    d = lambda **o: lib.kla_decode_step(*[{**dict(q=0x1000, k=0x2000, v=0x3000, la=0x4000, eta=0x5000, eps=1e-6,
                                                  S=0x6000, o=0x7000, B=2, H=2, dk=128, dv=128, dt=kla.KLA_BF16,
                                                  st=None), **o}[n]
                                          for n in ("q", "k", "v", "la", "eta", "eps", "S", "o", "B", "H", "dk", "dv",
                                                    "dt", "st")])
    assert d(S=None) == E_NULL
    assert d(k=None) == E_NULL
    assert d(dk=100) == E_SHAPE
    assert d(dv=512) == E_SHAPE
    assert d(eps=-1e-3) == E_SHAPE
    assert d(dt=2) == E_DTYPE
    assert d(S=0x6004) == E_ALIGN
    assert d(eta=0x5002) == E_ALIGN                 # the gates are fp32: 4-byte aligned, as in the chunk entry points
    assert d(la=0x4001) == E_ALIGN
    assert d(B=0) == OK
    b = lambda **o: lib.kla_beta(*[{**dict(k=0x1000, eta=0x2000, eps=1e-6, beta=0x3000, n=10, dk=128,
                                           dt=kla.KLA_F32, st=None), **o}[n]
                                   for n in ("k", "eta", "eps", "beta", "n", "dk", "dt", "st")])
    assert b(k=None) == E_NULL
    assert b(beta=None) == E_NULL
    assert b(dk=32) == E_SHAPE
    assert b(n=-1) == E_SHAPE
    assert b(dt=-1) == E_DTYPE
    assert b(k=0x1002) == E_ALIGN
    assert b(n=0) == OK


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros((1, 64, 1, 64))
    g = torch.zeros((1, 64, 1))
    with pytest.raises(RuntimeError):
        kla.kla_chunk_fwd(x, x, x, g, g, 1e-6)
    with pytest.raises(RuntimeError):
        kla.kla_beta(x, g, 1e-6)


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    """No HIP library, no result: the product path has no CPU fallback to slip into."""
    monkeypatch.setattr(kla, "LIB_PATH", str(tmp_path / "libkla.so"))
    monkeypatch.setattr(kla, "_lib", None)
    with pytest.raises(RuntimeError, match="not built"):
        kla.lib()
    with pytest.raises(RuntimeError, match="not built"):
        kla.kla_chunk_fwd_workspace_bytes(1, 64, 1, 64, 64, None)


def test_option_entry_points_validate_like_the_plain_ones():
    lib = kla.lib()
    chunk = lambda opts, **o: lib.kla_chunk_fwd_opts(
        *[{**dict(q=0x1000, k=0x2000, v=0x3000, la=0x4000, eta=0x5000, eps=1e-6, h0=None, o=0x6000, hT=None,
                  cu_dev=None, cu_host=None, n_seq=0, N=1, T=64, H=1, dk=64, dv=64, chunk=64, dt=kla.KLA_BF16,
                  ws=0x100000, ws_bytes=1 << 30, stream=None), **o}[n]
          for n in ("q", "k", "v", "la", "eta", "eps", "h0", "o", "hT", "cu_dev", "cu_host", "n_seq", "N", "T", "H",
                    "dk", "dv", "chunk", "dt", "ws", "ws_bytes", "stream")], opts)
    assert chunk(4) == E_SHAPE                      # unknown option bit
    assert chunk(8 | kla.KLA_OPT_GDN_BETA) == E_SHAPE
    assert chunk(kla.KLA_OPT_NORMALIZE_Q, q=None) == E_NULL
    assert chunk(kla.KLA_OPT_NORMALIZE_Q | kla.KLA_OPT_GDN_BETA, N=0) == OK
    dec = lambda opts, **o: lib.kla_decode_step_opts(
        *[{**dict(q=0x1000, k=0x2000, v=0x3000, la=0x4000, eta=0x5000, eps=1e-6, S=0x6000, o=0x7000, B=2, H=2,
                  dk=128, dv=128, dt=kla.KLA_BF16, st=None), **o}[n]
          for n in ("q", "k", "v", "la", "eta", "eps", "S", "o", "B", "H", "dk", "dv", "dt", "st")], opts)
    assert dec(16) == E_SHAPE
    assert dec(kla.KLA_OPT_GDN_BETA, S=None) == E_NULL
    assert dec(3, B=0) == OK


def test_workspace_bytes_of_the_segmented_scan():
    """A long sequence in a small bf16 batch is scanned in segments: the workspace then also holds, per
    (sequence, head), G-1 maps [N | M] and G incoming states in fp32."""
    f = lambda *a, **kw: kla.lib().kla_chunk_fwd_workspace_bytes_opts(*a, kla.tune(**kw))
    base = f(1, 65536, 8, 128, 128, 64, kla.KLA_BF16, None, 0, segments=1, unfused=True)
    extra = 8 * 128 * (3 * (128 + 128) + 4 * 128) * 4
    assert base + extra <= f(1, 65536, 8, 128, 128, 64, kla.KLA_BF16, None, 0, segments=4) <= base + extra + 512
    assert f(1, 65536, 8, 128, 128, 64, kla.KLA_F32, None, 0, segments=4) == \
        f(1, 65536, 8, 128, 128, 64, kla.KLA_F32, None, 0, segments=1)                      # bf16 only
    assert f(1, 65536, 8, 128, 128, 64, kla.KLA_BF16, None, 0) > base          # chosen automatically here
    # a large batch is never segmented: same size with and without the field at 1
    assert f(8, 4096, 8, 128, 128, 64, kla.KLA_BF16, None, 0, unfused=True) == \
        f(8, 4096, 8, 128, 128, 64, kla.KLA_BF16, None, 0, unfused=True, segments=1)


def test_chunk_bwd_validation_and_workspace():
    """kla_chunk_bwd validates like kla_chunk_fwd (before any launch), and its workspace is the documented sum:
    per chunk-head a record [T' | M^T | P^T | 4 vectors], two state checkpoints in the element type, and the
    [tokens, H, dv] arrays X, Y (and U, which only the element-type-generic kernels keep) in the element type."""
    lib = kla.lib()
    names = ("q", "k", "v", "la", "eta", "eps", "h0", "d_o", "d_hT", "dq", "dk_", "dv_", "dla", "deta", "dh0", "cu_dev",
             "cu_host", "n_seq", "N", "T", "H", "dk", "dv", "chunk", "dt", "ws", "ws_bytes", "stream")
    base = dict(q=0x1000, k=0x2000, v=0x3000, la=0x4000, eta=0x5000, eps=1e-6, h0=None, d_o=0x6000, d_hT=None,
                dq=0x7000, dk_=0x8000, dv_=0x9000, dla=0xa000, deta=0xb000, dh0=None, cu_dev=None, cu_host=None, n_seq=0,
                N=1, T=64, H=1, dk=64, dv=64, chunk=64, dt=kla.KLA_BF16, ws=0x100000, ws_bytes=1 << 30, stream=None)
    call = lambda **o: lib.kla_chunk_bwd(*[{**base, **o}[n] for n in names])
    assert call(q=None) == E_NULL
    assert call(d_o=None) == E_NULL
    assert call(dk_=None) == E_NULL
    assert call(deta=None) == E_NULL
    assert call(dk=96) == E_SHAPE
    assert call(chunk=32) == E_SHAPE
    assert call(eps=-1.0) == E_SHAPE
    assert call(dt=5) == E_DTYPE
    assert call(d_o=0x6008) == E_ALIGN
    assert call(dh0=0xc004) == E_ALIGN
    assert call(ws=None) == E_WS
    assert call(ws_bytes=1000) == E_WS
    cu = np.array([0, 30, 64], dtype=np.int32)
    assert call(n_seq=2, cu_host=cu.ctypes.data, cu_dev=None) == E_NULL
    assert call(N=0) == OK
    r256 = lambda x: (x + 255) // 256 * 256
    for dt, eb in ((kla.KLA_BF16, 2), (kla.KLA_F32, 4)):
        N, T, H, dk, dv = 3, 200, 2, 128, 256
        n_ch = N * 4 * H
        expect = r256(n_ch * (3 * 384 * 8 * eb + 1280))
        expect = r256(expect + 4)                              # chunk offsets of a packed batch (n_seq + 1 ints)
        expect += 2 * r256(n_ch * dk * dv * eb)                # S_c and dS'_c
        rows = r256(N * T * H * dv * eb)
        assert lib.kla_chunk_bwd_workspace_bytes_opts(N, T, H, dk, dv, 64, dt, None, 0, kla.tune(generic_bwd=True)) == expect + 3 * rows   # X, U, Y
        expect += (2 if dt == kla.KLA_BF16 else 3) * rows      # the bf16 kernels form U again instead of keeping it
        assert lib.kla_chunk_bwd_workspace_bytes(N, T, H, dk, dv, 64, dt, None, 0) == expect
    assert lib.kla_chunk_bwd_workspace_bytes(1, 64, 1, 100, 64, 64, kla.KLA_BF16, None, 0) == 0
    # one long bf16 sequence on few heads: the sweeps run in segments (here 8 of 16 chunks), and the workspace also holds
    # 7 maps [N | M] and 3 x 8 states per (sequence, head) in fp32; fp32 inputs never segment
    N, T, H, dk, dv = 1, 8192, 2, 128, 128
    plain = {}
    for dt, eb in ((kla.KLA_BF16, 2), (kla.KLA_F32, 4)):
        n_ch = N * (T // 64) * H
        x = r256(r256(n_ch * (3 * 384 * 8 * eb + 1280)) + 4) + 2 * r256(n_ch * dk * dv * eb) + (2 if dt == kla.KLA_BF16 else 3) * r256(N * T * H * dv * eb)
        plain[dt] = x
    seg = plain[kla.KLA_BF16] + r256(N * 7 * H * dk * (dv + dk) * 4) + 3 * r256(N * 8 * H * dk * dv * 4)
    assert lib.kla_chunk_bwd_workspace_bytes(N, T, H, dk, dv, 64, kla.KLA_BF16, None, 0) == seg
    assert lib.kla_chunk_bwd_workspace_bytes_opts(N, T, H, dk, dv, 64, kla.KLA_BF16, None, 0, kla.tune(segments=1)) == plain[kla.KLA_BF16]
    assert lib.kla_chunk_bwd_workspace_bytes(N, T, H, dk, dv, 64, kla.KLA_F32, None, 0) == plain[kla.KLA_F32]
    opt = lambda opts, **o: lib.kla_chunk_bwd_opts(*[{**base, **o}[n] for n in names], opts)
    assert opt(8) == E_SHAPE
    assert opt(kla.KLA_OPT_GDN_BETA, q=None) == E_NULL
    assert opt(kla.KLA_OPT_GDN_BETA, N=0) == OK
    assert opt(kla.KLA_OPT_GDN_BETA | kla.KLA_OPT_NORMALIZE_Q, N=0) == OK


def test_diag_entry_points_validate():
    lib = kla.lib()
    names = ("q", "k", "v", "la", "eta", "eps", "h0", "o", "hT", "cu_dev", "cu_host", "n_seq", "N", "T", "H", "dk", "dv",
             "chunk", "dt", "ws", "ws_bytes", "stream")
    base = dict(q=0x1000, k=0x2000, v=0x3000, la=0x4000, eta=0x5000, eps=1e-6, h0=None, o=0x6000, hT=None, cu_dev=None,
                cu_host=None, n_seq=0, N=1, T=64, H=1, dk=64, dv=64, chunk=64, dt=kla.KLA_BF16, ws=0x100000,
                ws_bytes=1 << 30, stream=None)
    call = lambda **o: lib.kla_chunk_fwd_diag(*[{**base, **o}[n] for n in names])
    assert call(la=None) == E_NULL
    assert call(dk=32) == E_SHAPE
    assert call(dt=9) == E_DTYPE
    assert call(v=0x3002) == E_ALIGN
    assert call(ws_bytes=10) == E_WS
    assert call(N=0) == OK
    # workspace: the forward's records and vectors, then K+, Q+, K~ in the element type and gamma_C per channel
    r256 = lambda x: (x + 255) // 256 * 256
    N, T, H, dk, dv = 2, 130, 3, 128, 64
    n_ch = N * 3 * H
    expect = r256(n_ch * (2 * 6144 + 768))
    expect = r256(expect + n_ch * 512)
    expect = r256(expect + 4)
    expect += 3 * (r256(N * T * H * dk * 2) + 256) + r256(n_ch * dk * 4)   # the three arrays are 256 bytes out of step
    assert lib.kla_chunk_fwd_diag_workspace_bytes(N, T, H, dk, dv, 64, kla.KLA_BF16, None, 0) == expect
    dec = lambda **o: lib.kla_decode_step_diag(*[{**dict(q=0x1000, k=0x2000, v=0x3000, la=0x4000, eta=0x5000, eps=1e-6,
                                                        S=0x6000, o=0x7000, B=2, H=2, dk=128, dv=128, dt=kla.KLA_BF16,
                                                        st=None), **o}[n]
                                                 for n in ("q", "k", "v", "la", "eta", "eps", "S", "o", "B", "H", "dk", "dv",
                                                           "dt", "st")])
    assert dec(la=None) == E_NULL
    assert dec(dv=100) == E_SHAPE
    assert dec(S=0x6008) == E_ALIGN
    assert dec(eta=0x5002) == E_ALIGN
    assert dec(la=0x4002) == E_ALIGN
    assert dec(B=0) == OK
    # the option variants validate the same way, and refuse unknown bits
    copt = lambda opts, **o: lib.kla_chunk_fwd_diag_opts(*[{**base, **o}[n] for n in names], opts)
    assert copt(4) == E_SHAPE
    assert copt(kla.KLA_OPT_NORMALIZE_Q, la=None) == E_NULL
    assert copt(kla.KLA_OPT_NORMALIZE_Q | kla.KLA_OPT_GDN_BETA, N=0) == OK
    dopt = lambda opts, **o: lib.kla_decode_step_diag_opts(
        *[{**dict(q=0x1000, k=0x2000, v=0x3000, la=0x4000, eta=0x5000, eps=1e-6, S=0x6000, o=0x7000, B=2, H=2, dk=128,
                  dv=128, dt=kla.KLA_BF16, st=None), **o}[n]
          for n in ("q", "k", "v", "la", "eta", "eps", "S", "o", "B", "H", "dk", "dv", "dt", "st")], opts)
    assert dopt(16) == E_SHAPE
    assert dopt(kla.KLA_OPT_GDN_BETA, S=None) == E_NULL
    assert dopt(kla.KLA_OPT_NORMALIZE_Q, B=0) == OK


def test_binding_refuses_wrong_shapes_and_dtypes():
    """The C ABI sees raw pointers, so the binding checks extents and element types of every tensor before it calls
    (a mismatch would otherwise be an out-of-bounds access on the GPU).  CPU tensors suffice: the checks come first,
    and tensors that pass them are then refused for not being on the GPU (there is no CPU fallback)."""
    import torch
    N, T, H, dk, dv = 2, 70, 3, 64, 128
    mk = lambda *shape, dtype=torch.bfloat16: torch.zeros(shape, dtype=dtype)
    good = dict(q=mk(N, T, H, dk), k=mk(N, T, H, dk), v=mk(N, T, H, dv), log_alpha=mk(N, T, H, dtype=torch.float32),
                eta=mk(N, T, H, dtype=torch.float32), eps=1e-6)
    call = lambda f, **o: f(**{**good, **o})
    with pytest.raises(RuntimeError, match="GPU"):
        call(kla.kla_chunk_fwd)
    bad = [dict(k=mk(N, T, H + 1, dk)), dict(k=mk(N, T, H, dk, dtype=torch.float32)), dict(v=mk(N, T + 1, H, dv)),
           dict(log_alpha=mk(N, T, H, dtype=torch.float64)), dict(log_alpha=mk(N, T, H, dtype=torch.bfloat16)),
           dict(eta=mk(N, T)), dict(eta=mk(N * T * H, dtype=torch.float32)), dict(h0=mk(N, H, dk, dv)),
           dict(h0=mk(N + 1, H, dk, dv, dtype=torch.float32)), dict(out=mk(N, T, H, dk)),
           dict(hT=mk(N, H, dv, dk, dtype=torch.float32)), dict(q=mk(N, T, H, dk, dtype=torch.float16)),
           dict(cu_seqlens=torch.tensor([0, 70, 140], dtype=torch.int64))]
    for o in bad:
        with pytest.raises((ValueError, TypeError)):
            call(kla.kla_chunk_fwd, **o)
    for o in (dict(log_alpha=mk(N, T, H, dtype=torch.float32)), dict(log_alpha=mk(N, T, H, dk)), dict(k=mk(N, T, H, dv))):
        with pytest.raises((ValueError, TypeError)):
            call(kla.kla_chunk_fwd_diag, **o)
    d_o = mk(N, T, H, dv)
    for o in (dict(d_o=mk(N, T, H, dk)), dict(d_o=d_o.float()), dict(d_o=d_o, d_hT=mk(N, H, dk, dv)),
              dict(d_o=d_o, out=dict(dq=mk(N, T, H, dv))), dict(d_o=d_o, out=dict(deta=mk(N, T, H))),
              dict(d_o=d_o, out=dict(dlog_alpha=mk(N, T, dtype=torch.float32))), dict(d_o=d_o, eta=mk(N, T, H))):
        with pytest.raises((ValueError, TypeError)):
            call(kla.kla_chunk_bwd, **o)
    with pytest.raises(RuntimeError, match="GPU"):
        call(kla.kla_chunk_bwd, d_o=d_o)
    B = 4
    dgood = dict(q=mk(B, H, dk), k=mk(B, H, dk), v=mk(B, H, dv), log_alpha=mk(B, H, dtype=torch.float32),
                 eta=mk(B, H, dtype=torch.float32), eps=1e-6, S=mk(B, H, dk, dv, dtype=torch.float32))
    dcall = lambda f, **o: f(**{**dgood, **o})
    with pytest.raises(RuntimeError, match="GPU"):
        dcall(kla.kla_decode_step)
    for o in (dict(S=mk(B, H, dk, dv)), dict(S=mk(B, H, dv, dk, dtype=torch.float32)), dict(eta=mk(B, H + 1, dtype=torch.float32)),
              dict(log_alpha=mk(B, H)), dict(k=mk(B, H, dv)), dict(out=mk(B, H, dk)), dict(v=mk(B, H, dv, dtype=torch.float32))):
        with pytest.raises((ValueError, TypeError)):
            dcall(kla.kla_decode_step, **o)
    for o in (dict(), dict(log_alpha=mk(B, H, dk))):                     # diagonal gating wants fp32 [B, H, dk]
        with pytest.raises((ValueError, TypeError)):
            dcall(kla.kla_decode_step_diag, **o)
    with pytest.raises((ValueError, TypeError)):
        kla.kla_beta(mk(5, dk), mk(5, dtype=torch.bfloat16), 1e-6)
    with pytest.raises((ValueError, TypeError)):
        kla.kla_beta(mk(5, dk), mk(6, dtype=torch.float32), 1e-6)
    with pytest.raises(RuntimeError, match="GPU"):
        kla.kla_beta(mk(5, dk), mk(5, dtype=torch.float32), 1e-6)


def test_peak_probe_validates():
    """The measurement hook checks its arguments before it launches anything (no GPU needed for the error paths)."""
    lib = kla.lib()
    call = lambda kind, buf, aux, size, iters: lib.kla_debug_peak_probe(kind, buf, aux, size, iters, None)
    assert call(4, 0x1000, None, 65536, 0) == E_SHAPE
    assert call(0, None, None, 65536, 0) == E_NULL
    assert call(0, 0x1000, None, 1000, 0) == E_SHAPE
    assert call(1, 0x1000, None, 65536, 0) == E_NULL
    assert call(2, None, None, 16, 4) == E_NULL
    # kind 3: copies per step one of 16 / 32 / 48 / 60, ring depth 1 or 2, buffer of at least n x 4 MiB
    assert call(3, 0x1000, None, 1 << 30, 17) == E_SHAPE
    assert call(3, 0x1000, None, 1 << 30, 16 + 512) == E_SHAPE
    assert call(3, None, None, 1 << 30, 16) == E_NULL
    assert call(3, 0x1008, None, 1 << 30, 16) == E_ALIGN
    assert call(3, 0x1000, None, (16 << 22) - 1, 16) == E_WS
