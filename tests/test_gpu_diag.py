"""GPU parity of diagonal (per-channel) gating: kla_chunk_fwd_diag and kla_decode_step_diag, called through the C ABI,
against the fp64 token-loop oracle with D_t = diag(alpha_t) (App. B, "Extension to diagonal gating").

Metric and bars as for the scalar path: max|x_gpu - x_ref| / max|x_ref|, <= 1e-4 for fp32 inputs, <= 2e-2 for bf16.
"""
import numpy as np
import pytest
import torch

import kla_inputs
from oracle import token_oracle

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}


@pytest.fixture(scope="module")
def kla():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_08587_amd as m
    m.lib()          # raises if the HIP library is not built: there is no fallback to test instead
    return m


def _cuda(t):
    return None if t is None else t.cuda()


def _check(kla, d, seed, scale=1.0):
    lad = kla_inputs.diag_gates(d, seed, scale)
    print("case N=%d T=%d H=%d dk=%d dv=%d %s varlen=%s decay x%g" % (d["N"], d["T"], d["H"], d["dk"], d["dv"], d["dtype"],
                                                                     d["cu_seqlens"] is not None, scale), flush=True)
    o, hT = kla.kla_chunk_fwd_diag(_cuda(d["q"]), _cuda(d["k"]), _cuda(d["v"]), _cuda(lad), _cuda(d["eta"]), d["eps"],
                                   h0=_cuda(d["h0"]), cu_seqlens=_cuda(d["cu_seqlens"]))
    torch.cuda.synchronize()
    o, hT = o.float().cpu().numpy(), hT.cpu().numpy()
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(hT))
    q, k, v = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    ro, rh, _ = token_oracle.kla_recurrent_diag(q, k, v, lad.numpy(), d["eta"].numpy(), d["eps"],
                                                h0=None if d["h0"] is None else d["h0"].numpy(),
                                                cu_seqlens=None if d["cu_seqlens"] is None else d["cu_seqlens"].numpy())
    eo, eh = token_oracle.rel_err(o, ro), token_oracle.rel_err(hT, rh)
    print("   rel err o=%.3e hT=%.3e (bar %.0e)" % (eo, eh, TOL[d["dtype"]]), flush=True)
    assert eo <= TOL[d["dtype"]] and eh <= TOL[d["dtype"]]


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (128, 256), (64, 128)])
@pytest.mark.parametrize("T", [1, 63, 65, 200])
def test_diag_chunk_small_shapes(kla, dt, dk, dv, T):
    _check(kla, kla_inputs.chunk_inputs(2, T, 3, dk, dv, dtype=dt, seed=400 + T + dk + dv, h0_std=0.5), seed=T)


@pytest.mark.parametrize("T", [1, 64, 65, 130, 200])
def test_diag_chunk_two_wave_scan_short_sequences(kla, T):
    """Enough (sequence, head) pairs for the scan with two compute waves per workgroup, whose two-stage ring at d_k = 128
    is filled in two parts per chunk: sequences of one, two, three and four chunks walk through its start and its end."""
    _check(kla, kla_inputs.chunk_inputs(8, T, 8, 128, 128, dtype=torch.bfloat16, seed=470 + T, h0_std=0.3), seed=T)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_diag_chunk_varlen(kla, dt):
    d = kla_inputs.varlen_inputs(6, 1, 300, 2, 128, 128, dtype=dt, seed=420, h0_std=0.3)
    cu = d["cu_seqlens"].clone()
    cu[3] = cu[2]                              # one empty sequence
    d["cu_seqlens"] = cu
    _check(kla, d, seed=2)


@pytest.mark.parametrize("dt,scale", [(torch.float32, 8.0), (torch.bfloat16, 4.0), (torch.bfloat16, 0.02)])
def test_diag_chunk_decay_range(kla, dt, scale):
    """Strong decay (gamma underflows inside a chunk: every ratio must still be formed without overflow) and slow
    decay (long carry)."""
    _check(kla, kla_inputs.chunk_inputs(1, 700, 2, 128, 128, dtype=dt, seed=430, h0_std=0.3), seed=3, scale=scale)


def test_diag_generic_scan_on_bf16(kla, monkeypatch):
    """The element-type-generic scan kernel (the fp32 path's) on bf16 inputs."""
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(generic_scan=True))
    _check(kla, kla_inputs.chunk_inputs(2, 200, 2, 128, 128, dtype=torch.bfloat16, seed=435, h0_std=0.3), seed=4)


def test_diag_equal_channels_repeat_the_scalar_path(kla):
    """All channels equal: the diagonal kernels must agree with the scalar-gate kernels (different code, same map)."""
    d = kla_inputs.chunk_inputs(2, 300, 2, 128, 128, dtype=torch.float32, seed=440, h0_std=0.3)
    q, k, v, la, eta, h0 = (_cuda(d[n]) for n in ("q", "k", "v", "log_alpha", "eta", "h0"))
    o1, h1 = kla.kla_chunk_fwd(q, k, v, la, eta, d["eps"], h0=h0)
    lad = la[..., None].expand(-1, -1, -1, d["dk"]).contiguous()
    o2, h2 = kla.kla_chunk_fwd_diag(q, k, v, lad, eta, d["eps"], h0=h0)
    assert token_oracle.rel_err(o2.cpu().numpy(), o1.cpu().numpy()) <= 1e-5
    assert token_oracle.rel_err(h2.cpu().numpy(), h1.cpu().numpy()) <= 1e-5


def test_diag_chunk_config2_shape_full(kla):
    """The benchmark's secondary workload: config 2's tensors with per-channel gates; every (sequence, head) compared."""
    _check(kla, kla_inputs.config(2), seed=5)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (128, 256)])
def test_diag_decode(kla, dt, dk, dv):
    dd = kla_inputs.decode_inputs(4, 5, 3, dk, dv, dtype=dt, seed=450)
    gen = torch.Generator().manual_seed(451)
    lad = -torch.nn.functional.softplus(torch.randn((4, 5, 3, dk), generator=gen))
    S = dd["S"].cuda().clone()
    Sr = dd["S"].numpy().astype(np.float64)
    for t in range(4):
        o = kla.kla_decode_step_diag(*(dd[n][t].contiguous().cuda() for n in ("q", "k", "v")), lad[t].contiguous().cuda(),
                                     dd["eta"][t].contiguous().cuda(), dd["eps"], S)
        ro, Sr = token_oracle.kla_decode_diag(*(kla_inputs.to_numpy_f32(dd[x][t]) for x in "qkv"), lad[t].numpy(),
                                              dd["eta"][t].numpy(), dd["eps"], Sr)
        assert token_oracle.rel_err(o.float().cpu().numpy(), ro) <= TOL[dt]
        assert token_oracle.rel_err(S.cpu().numpy(), Sr) <= 1e-4          # the state is fp32 in both cases


def test_diag_prefill_then_decode(kla):
    """chunk forward on T tokens, then one decode step, equals the chunk forward on T + 1 tokens."""
    d = kla_inputs.chunk_inputs(2, 130, 2, 128, 128, dtype=torch.bfloat16, seed=460)
    lad = kla_inputs.diag_gates(d, 6, 0.1).cuda()
    q, k, v, eta = (_cuda(d[n]) for n in ("q", "k", "v", "eta"))
    o, hT = kla.kla_chunk_fwd_diag(q, k, v, lad, eta, d["eps"])
    T = d["T"]
    cut = lambda x: x[:, :T - 1].contiguous()
    o1, h1 = kla.kla_chunk_fwd_diag(cut(q), cut(k), cut(v), cut(lad), cut(eta), d["eps"])
    od = kla.kla_decode_step_diag(q[:, T - 1].contiguous(), k[:, T - 1].contiguous(), v[:, T - 1].contiguous(),
                                  lad[:, T - 1].contiguous(), eta[:, T - 1].contiguous(), d["eps"], h1)
    assert token_oracle.rel_err(od.float().cpu().numpy(), o[:, T - 1].float().cpu().numpy()) <= 2e-2
    assert token_oracle.rel_err(h1.cpu().numpy(), hT.cpu().numpy()) <= 1e-2


def test_diag_no_tokens(kla):
    """A batch without tokens: the final state is the initial state."""
    H, dk, dv = 2, 64, 128
    z = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device="cuda")
    h0 = torch.randn((2, H, dk, dv), generator=torch.Generator().manual_seed(2)).cuda()
    o, hT = kla.kla_chunk_fwd_diag(z(2, 0, H, dk), z(2, 0, H, dk), z(2, 0, H, dv), torch.zeros((2, 0, H, dk), device="cuda"),
                                   torch.zeros((2, 0, H), device="cuda"), 1e-6, h0=h0)
    torch.cuda.synchronize()
    assert o.shape[1] == 0 and torch.equal(hT, h0)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("nq,gdn", [(True, False), (False, True), (True, True)])
@pytest.mark.parametrize("T,dk,dv,varlen", [(200, 128, 128, False), (130, 64, 256, False), (300, 128, 64, True)])
def test_diag_chunk_options(kla, dt, nq, gdn, T, dk, dv, varlen):
    """The option bits on the diagonal-gating forward: normalised read-out (with one zero query and queries of very
    different lengths) and beta_t = eta_t, alone and together; fixed and packed batches."""
    if varlen:
        d = kla_inputs.varlen_inputs(4, 1, T, 2, dk, dv, dtype=dt, seed=460, h0_std=0.3)
    else:
        d = kla_inputs.chunk_inputs(2, T, 3, dk, dv, dtype=dt, seed=461 + T, h0_std=0.3)
    if gdn:
        d["k"] = (d["k"].float() / d["k"].float().norm(dim=-1, keepdim=True)).to(dt)      # keeps the plain delta rule stable
    scale = torch.logspace(-1.5, 1.5, d["T"]).reshape(1, d["T"], 1, 1)
    d["q"] = (d["q"].float() * scale).to(dt)
    d["q"][0, 7, 1] = 0
    lad = kla_inputs.diag_gates(d, 6, 1.0)
    o, hT = kla.kla_chunk_fwd_diag(_cuda(d["q"]), _cuda(d["k"]), _cuda(d["v"]), _cuda(lad), _cuda(d["eta"]), d["eps"],
                                   h0=_cuda(d["h0"]), cu_seqlens=_cuda(d["cu_seqlens"]), normalize_q=nq, gdn_beta=gdn)
    torch.cuda.synchronize()
    q, k, v = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    ro, rh, _ = token_oracle.kla_recurrent_diag(q, k, v, lad.numpy(), d["eta"].numpy(), d["eps"], h0=d["h0"].numpy(),
                                                cu_seqlens=None if d["cu_seqlens"] is None else d["cu_seqlens"].numpy(),
                                                normalize_q=nq, gdn_beta=gdn)
    o = o.float().cpu().numpy()
    if nq:
        assert np.all(o[0, 7, 1] == 0.0)
    else:                                          # without the normalisation o scales with ||q||: compare row by row in those units
        qn = np.linalg.norm(q.astype(np.float64), axis=-1, keepdims=True)
        qn = np.where(qn == 0.0, 1.0, qn)
        o, ro = o / qn, ro / qn
    eo, eh = token_oracle.rel_err(o, ro), token_oracle.rel_err(hT.cpu().numpy(), rh)
    print("   rel err o=%.3e hT=%.3e" % (eo, eh), flush=True)
    assert eo <= TOL[dt] and eh <= TOL[dt]


def test_diag_options_generic_scan_on_bf16(kla, monkeypatch):
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(generic_scan=True))
    d = kla_inputs.chunk_inputs(2, 200, 2, 128, 128, dtype=torch.bfloat16, seed=465, h0_std=0.3)
    lad = kla_inputs.diag_gates(d, 7, 1.0)
    o, hT = kla.kla_chunk_fwd_diag(_cuda(d["q"]), _cuda(d["k"]), _cuda(d["v"]), _cuda(lad), _cuda(d["eta"]), d["eps"],
                                   h0=_cuda(d["h0"]), normalize_q=True)
    torch.cuda.synchronize()
    q, k, v = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    ro, rh, _ = token_oracle.kla_recurrent_diag(q, k, v, lad.numpy(), d["eta"].numpy(), d["eps"], h0=d["h0"].numpy(),
                                                normalize_q=True)
    assert token_oracle.rel_err(o.float().cpu().numpy(), ro) <= TOL[torch.bfloat16]
    assert token_oracle.rel_err(hT.cpu().numpy(), rh) <= TOL[torch.bfloat16]


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("nq,gdn", [(True, False), (False, True), (True, True)])
def test_diag_decode_options(kla, dt, nq, gdn):
    d = kla_inputs.decode_inputs(3, 5, 4, 128, 128, dtype=dt, seed=470, state_std=1.0)
    gen = torch.Generator().manual_seed(471)
    lad = -torch.nn.functional.softplus(torch.randn((3, 5, 4, 128), generator=gen))
    kk = d["k"]
    if gdn:
        kk = (kk.float() / kk.float().norm(dim=-1, keepdim=True)).to(dt)
    qq = d["q"].clone()
    qq[0, 2, 1] = 0
    S = d["S"].cuda().clone()
    Sref = d["S"].double().numpy()
    for t in range(3):
        o = kla.kla_decode_step_diag(_cuda(qq[t].contiguous()), _cuda(kk[t].contiguous()), _cuda(d["v"][t].contiguous()),
                                     _cuda(lad[t].contiguous()), _cuda(d["eta"][t].contiguous()), d["eps"], S,
                                     normalize_q=nq, gdn_beta=gdn)
        ro, Sref = token_oracle.kla_decode_diag(kla_inputs.to_numpy_f32(qq[t]), kla_inputs.to_numpy_f32(kk[t]),
                                                kla_inputs.to_numpy_f32(d["v"][t]), lad[t].numpy(), d["eta"][t].numpy(),
                                                d["eps"], Sref, normalize_q=nq, gdn_beta=gdn)
        assert token_oracle.rel_err(o.float().cpu().numpy(), ro) <= (1e-5 if dt == torch.float32 else 1e-2)
        assert token_oracle.rel_err(S.cpu().numpy(), Sref) <= 1e-5
        if nq and t == 0:
            assert np.all(o[2, 1].float().cpu().numpy() == 0.0)
