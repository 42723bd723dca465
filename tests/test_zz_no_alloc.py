"""The entry point that allocates nothing (kla_chunk_fwd_static): same kernels as kla_chunk_fwd, with the per-chunk
objects in the library's fixed scratch array.  Its output must equal kla_chunk_fwd's bit for bit (and meet the bar
against the fp64 oracle) on two calls in a row, the second on a smaller problem that leaves stale records of the
first in the array; sizes beyond the array are refused before anything runs."""
import os

import numpy as np
import pytest
import torch

import kla_inputs
import paper_2605_08587_amd as kla
from oracle import token_oracle

TOL_BF16, TOL_F32 = 2e-2, 1e-4      # max|x - ref| / max|ref| for bf16 / fp32 inputs (the bar of every parity test)

needs_lib = pytest.mark.skipif(not os.path.exists(kla.LIB_PATH), reason="libkla.so not built")


@needs_lib
def test_static_refuses_what_does_not_fit():
    """Config 2's sizes with fp32 inputs need 107 MB of per-chunk objects: KLA_ERR_WORKSPACE, decided on the host
    before any HIP call (the pointers are fakes; nothing may be launched).  Argument errors come out as from
    kla_chunk_fwd.  (With bf16 inputs the same sizes run the fused kernel, which needs no scratch at all.)"""
    f = kla.lib().kla_chunk_fwd_static
    args = lambda N, T, H, q=0x1000, dt=kla.KLA_F32: (q, 0x2000, 0x3000, 0x4000, 0x5000, 1e-6, None, 0x6000, None, None,
                                                      None, 0, N, T, H, 128, 128, 64, dt, None)
    assert kla.lib().kla_chunk_fwd_workspace_bytes(8, 4096, 8, 128, 128, 64, kla.KLA_F32, None, 0) > kla.KLA_STATIC_SCRATCH_BYTES
    assert f(*args(8, 4096, 8)) == -5
    # a small bf16 batch of one long sequence runs the segment-parallel scan, whose maps and records live in the scratch
    assert kla.lib().kla_chunk_fwd_workspace_bytes(1, 65536, 8, 128, 128, 64, kla.KLA_BF16, None, 0) > kla.KLA_STATIC_SCRATCH_BYTES
    assert f(*args(1, 65536, 8, dt=kla.KLA_BF16)) == -5
    assert f(*args(1, 64, 1, q=None)) == -1
    assert f(*args(1, 64, 1, q=0x1004)) == -4
    assert f(*args(0, 64, 1)) == 0
    import re
    hdr = open(kla.HEADER_PATH).read()
    assert int(re.search(r"KLA_STATIC_SCRATCH_BYTES \((\d+)u << 20\)", hdr).group(1)) << 20 == kla.KLA_STATIC_SCRATCH_BYTES


def _case(N, T, H, dk, dv, dtype, seed, packed=False):
    if packed:
        lens = [T, 1, 3 * T // 4 + 5]
        d = kla_inputs.chunk_inputs(1, sum(lens), H, dk, dv, dtype=dtype, seed=seed, h0_std=0.1, n_h0=len(lens))
        d["cu"] = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32)
    else:
        d = kla_inputs.chunk_inputs(N, T, H, dk, dv, dtype=dtype, seed=seed, h0_std=0.1)
        d["cu"] = None
    return d


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_static_matches_workspace_entry_point(dtype):
    tol = TOL_BF16 if dtype == torch.bfloat16 else TOL_F32
    # first a larger problem (ragged tail, several chunks; the packed one also has a one-token sequence), then a
    # smaller one on the same GPU: the array still holds the first call's records.  All of these go through the scratch
    # (fp32 always does; bf16 batches this small run the two-kernel form, the 4100-token one the segment-parallel scan
    # with records, maps and states); only large bf16 batches run the fused kernel, which leaves the array alone.
    for (N, T, H, dk, dv, seed, packed) in ((1, 4100, 2, 128, 128, 30, False), (2, 1000, 4, 128, 128, 31, False), (1, 200, 2, 128, 128, 32, False),
                                            (1, 333, 3, 64, 256, 33, True), (1, 70, 2, 64, 64, 34, False)):
        d = _case(N, T, H, dk, dv, dtype, seed, packed)
        dev = {n: d[n].cuda() for n in ("q", "k", "v", "log_alpha", "eta", "h0")}
        cu = None if d["cu"] is None else d["cu"].cuda()
        o_ws, h_ws = kla.kla_chunk_fwd(dev["q"], dev["k"], dev["v"], dev["log_alpha"], dev["eta"], d["eps"], h0=dev["h0"],
                                       cu_seqlens=cu)
        out = torch.full_like(o_ws, float("nan"))
        hT = torch.full_like(h_ws, float("nan"))
        print("static: N=%d T=%d H=%d dk=%d dv=%d %s packed=%s" % (N, d["q"].shape[1], H, dk, dv, dtype, packed), flush=True)
        kla.kla_chunk_fwd_static(dev["q"], dev["k"], dev["v"], dev["log_alpha"], dev["eta"], d["eps"], out, hT=hT,
                                 h0=dev["h0"], cu_seqlens=cu, cu_seqlens_host=d["cu"])
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                           o_ws.view(torch.int16 if dtype == torch.bfloat16 else torch.int32))
        assert torch.equal(hT.view(torch.int32), h_ws.view(torch.int32))
        ro, rh, _ = token_oracle.kla_recurrent(*(kla_inputs.to_numpy_f32(d[x]) for x in "qkv"), d["log_alpha"].numpy(),
                                               d["eta"].numpy(), d["eps"], h0=d["h0"].numpy(),
                                               cu_seqlens=None if d["cu"] is None else d["cu"].numpy())
        assert token_oracle.rel_err(out.float().cpu().numpy(), ro) <= tol
        assert token_oracle.rel_err(hT.cpu().numpy(), rh) <= tol
