"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the same
seeded inputs, element by element.

Metric and bars (the ones the task fixes): max|x_gpu - x_ref| / max|x_ref| over the whole tensor,
<= 1e-4 for fp32 inputs and <= 2e-2 for bf16 inputs, separately for the outputs and for the
final states.  Integer-free path: nothing here is bit-exact except run-to-run determinism.
"""
import numpy as np
import pytest
import torch

import kla_inputs
from oracle import chunk_oracle, token_oracle

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}


@pytest.fixture(scope="module")
def kla():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_08587_amd as m
    m.lib()          # raises if the HIP library is not built: there is no fallback to test instead
    return m


def _gpu(d, *names):
    return [None if d[n] is None else d[n].cuda() for n in names]


def _oracle_chunk(d):
    q, k, v = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    h0 = None if d["h0"] is None else d["h0"].numpy()
    cu = None if d["cu_seqlens"] is None else d["cu_seqlens"].numpy()
    return token_oracle.kla_recurrent(q, k, v, d["log_alpha"].numpy(), d["eta"].numpy(), d["eps"], h0=h0,
                                      cu_seqlens=cu)


def _run_chunk(kla, d):
    q, k, v, la, eta, h0, cu = _gpu(d, "q", "k", "v", "log_alpha", "eta", "h0", "cu_seqlens")
    o, hT = kla.kla_chunk_fwd(q, k, v, la, eta, d["eps"], h0=h0, cu_seqlens=cu)
    torch.cuda.synchronize()
    return o.float().cpu().numpy(), hT.cpu().numpy()


def _check_chunk(kla, d, tol=None):
    tol = tol or TOL[d["dtype"]]
    print("case N=%d T=%d H=%d dk=%d dv=%d %s varlen=%s" % (d["N"], d["T"], d["H"], d["dk"], d["dv"], d["dtype"],
                                                           d["cu_seqlens"] is not None), flush=True)
    o, hT = _run_chunk(kla, d)
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(hT))
    ro, rh, _ = _oracle_chunk(d)
    eo, eh = token_oracle.rel_err(o, ro), token_oracle.rel_err(hT, rh)
    print("   rel err o=%.3e hT=%.3e (bar %.0e)" % (eo, eh, tol), flush=True)
    assert eo <= tol and eh <= tol
    return eo, eh


# ---------------------------------------------------------------------------------------------
def test_beta(kla):
    gen = torch.Generator().manual_seed(11)
    for dt in (torch.float32, torch.bfloat16):
        for dk in (64, 128):
            k = (torch.randn((3, 77, 5, dk), generator=gen) * 1.7).to(dt)
            eta = torch.rand((3, 77, 5), generator=gen)
            k[1, 3, 2] = 0
            for eps in (1e-6, 0.0):
                b = kla.kla_beta(k.cuda(), eta.cuda(), eps).cpu().double().numpy()
                kk = k.double().numpy()
                den = (kk * kk).sum(-1) + eps
                ref = np.where(den == 0, 0.0, eta.double().numpy() / np.where(den == 0, 1, den))
                assert np.max(np.abs(b - ref) / np.maximum(np.abs(ref), 1e-30)) < 1e-5


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (128, 256), (64, 256)])
def test_decode_small(kla, dt, dk, dv):
    d = kla_inputs.decode_inputs(5, 3, 4, dk, dv, dtype=dt, seed=21, state_std=1.0)
    S = d["S"].cuda().clone()
    Sref = d["S"].double().numpy()
    for t in range(d["steps"]):
        q, k, v, la, eta = (d[n][t].contiguous().cuda() for n in ("q", "k", "v", "log_alpha", "eta"))
        o = kla.kla_decode_step(q, k, v, la, eta, d["eps"], S)
        ro, Sref = token_oracle.kla_decode(*(kla_inputs.to_numpy_f32(d[n][t]) for n in "qkv"),
                                           d["log_alpha"][t].numpy(), d["eta"][t].numpy(), d["eps"], Sref)
        assert token_oracle.rel_err(o.float().cpu().numpy(), ro) <= (1e-5 if dt == torch.float32 else 1e-2)
        assert token_oracle.rel_err(S.cpu().numpy(), Sref) <= 1e-5


@pytest.mark.parametrize("B", [1, 16, 40])
@pytest.mark.parametrize("sl", [None, "32", "64", "128", "256"])
def test_decode_slice_widths(kla, B, sl, monkeypatch):
    """Every width of the state slice a workgroup takes (the library picks 32 .. 128 columns by batch size; the
    tuning field forces one), on a batch of 1, 16 and 40 x 8 heads: same results."""
    monkeypatch.setattr(kla, "DEFAULT_TUNE", 0 if sl is None else kla.tune(decode_slice=int(sl)))
    d = kla_inputs.decode_inputs(2, B, 8, 128, 256, dtype=torch.bfloat16, seed=23, state_std=1.0)
    S = d["S"].cuda().clone()
    Sref = d["S"].double().numpy()
    for t in range(d["steps"]):
        q, k, v, la, eta = (d[n][t].contiguous().cuda() for n in ("q", "k", "v", "log_alpha", "eta"))
        o = kla.kla_decode_step(q, k, v, la, eta, d["eps"], S)
        ro, Sref = token_oracle.kla_decode(*(kla_inputs.to_numpy_f32(d[n][t]) for n in "qkv"),
                                           d["log_alpha"][t].numpy(), d["eta"][t].numpy(), d["eps"], Sref)
        assert token_oracle.rel_err(o.float().cpu().numpy(), ro) <= 1e-2
        assert token_oracle.rel_err(S.cpu().numpy(), Sref) <= 1e-5


def test_decode_config4_full(kla):
    """Config 4 as benchmarked: B=64, H=8, d=128, 256 consecutive steps, state updated in place."""
    d = kla_inputs.config(4)
    S = d["S"].cuda().clone()
    dev = {n: d[n].cuda() for n in ("q", "k", "v", "log_alpha", "eta")}
    outs = []
    for t in range(d["steps"]):
        outs.append(kla.kla_decode_step(dev["q"][t], dev["k"][t], dev["v"][t], dev["log_alpha"][t], dev["eta"][t],
                                        d["eps"], S))
    torch.cuda.synchronize()
    o = torch.stack(outs).float().cpu().numpy()
    Sref = d["S"].double().numpy()
    ro = np.zeros(o.shape)
    qn, kn, vn = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    for t in range(d["steps"]):
        ro[t], Sref = token_oracle.kla_decode(qn[t], kn[t], vn[t], d["log_alpha"][t].numpy(), d["eta"][t].numpy(),
                                              d["eps"], Sref)
    eo, es = token_oracle.rel_err(o, ro), token_oracle.rel_err(S.cpu().numpy(), Sref)
    print("decode cfg4: rel err o=%.3e S=%.3e" % (eo, es), flush=True)
    assert eo <= 2e-2 and es <= 2e-2


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dk", [64, 128])
def test_intra_chunk_objects(kla, dt, dk):
    """Stage 1 alone against eqs. (6)-(7): T' = (I+L)^-1 B, P = A o QK^T, g, incl. a ragged last chunk."""
    d = kla_inputs.chunk_inputs(2, 150, 3, dk, 64, dtype=dt, seed=31)
    q, k, la, eta = _gpu(d, "q", "k", "log_alpha", "eta")
    Tb, P, g = (x.cpu().double().numpy() for x in kla.kla_debug_intra_chunk(q, k, la, eta, d["eps"]))
    qn, kn = kla_inputs.to_numpy_f32(d["q"]), kla_inputs.to_numpy_f32(d["k"])
    tol = 1e-5 if dt == torch.float32 else 8e-3
    NT = 3
    for n in range(2):
        for h in range(3):
            for c in range(NT):
                a, b = 64 * c, min(150, 64 * c + 64)
                beta, gg, A, L = chunk_oracle.chunk_objects(kn[n, a:b, h], d["log_alpha"][n, a:b, h].numpy(),
                                                            d["eta"][n, a:b, h].numpy(), d["eps"])
                m = b - a
                Tref = np.linalg.solve(np.eye(m) + L, np.diag(beta))
                Pref = A * (qn[n, a:b, h].astype(np.float64) @ kn[n, a:b, h].astype(np.float64).T)
                ch = n * NT + c
                assert token_oracle.rel_err(Tb[ch, h, :m, :m], Tref) <= tol
                assert token_oracle.rel_err(P[ch, h, :m, :m], Pref) <= tol
                assert np.max(np.abs(g[ch, h, :m] - gg)) <= 1e-5 * max(1.0, np.max(np.abs(gg)))
                assert np.all(Tb[ch, h, m:, :] == 0) and np.all(Tb[ch, h, :, m:] == 0)
                assert np.all(P[ch, h, m:, :] == 0) and np.all(P[ch, h, :, m:] == 0)


def test_chunk_config1_fp32(kla):
    _check_chunk(kla, kla_inputs.config(1))


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (128, 256), (64, 128)])
@pytest.mark.parametrize("T", [1, 63, 64, 65, 200])
def test_chunk_small_shapes(kla, dt, dk, dv, T):
    d = kla_inputs.chunk_inputs(2, T, 3, dk, dv, dtype=dt, seed=41 + T, h0_std=0.5)
    _check_chunk(kla, d)


@pytest.mark.parametrize("form", ["fused", "unfused"])
@pytest.mark.parametrize("waves", ["1", "2", "4"])
def test_chunk_wave_shapes(kla, waves, form, monkeypatch):
    """Same result for every workgroup shape of the scan stage (also an LDS hazard check), as one fused kernel (one or
    two compute waves; with four the field changes nothing) and as the two-kernel form."""
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(scan_waves=int(waves), fused=form == "fused", unfused=form == "unfused"))
    d = kla_inputs.chunk_inputs(2, 300, 2, 128, 128, dtype=torch.bfloat16, seed=51, h0_std=0.1)
    _check_chunk(kla, d)
    d = kla_inputs.chunk_inputs(1, 200, 3, 64, 256, dtype=torch.bfloat16, seed=52, h0_std=0.1)
    _check_chunk(kla, d)


@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (128, 256), (64, 128)])
@pytest.mark.parametrize("T", [1, 63, 64, 65, 129, 200])
def test_chunk_small_shapes_fused(kla, dk, dv, T, monkeypatch):
    """test_chunk_small_shapes runs these few-chain bf16 shapes through the two-kernel form (the library's choice for
    them); here the fused kernel on the same shapes, and the two forms against each other."""
    d = kla_inputs.chunk_inputs(2, T, 3, dk, dv, dtype=torch.bfloat16, seed=41 + T, h0_std=0.5)
    o1, h1 = _run_chunk(kla, d)
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(fused=True))
    _check_chunk(kla, d)
    o2, h2 = _run_chunk(kla, d)
    assert token_oracle.rel_err(o2, o1) <= TOL[torch.bfloat16] and token_oracle.rel_err(h2, h1) <= TOL[torch.bfloat16]


@pytest.mark.parametrize("case", ["options", "packed", "extreme_decay", "zero_keys_and_eta", "long_carry", "no_h0_ragged"])
def test_chunk_fused_edge_cases(kla, case, monkeypatch):
    """The fused kernel (what large bf16 batches run) forced on the cases the other tests send through the two-kernel
    form: both option bits, packed batches with one-token and exactly-one-chunk sequences, decay that wipes the state
    within a token, zero keys and eta = 0 tokens, a state carried over ~60 chunks, and ragged tails without h0."""
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(fused=True))
    bf = torch.bfloat16
    if case == "options":
        for nq, gdn, (T, dk, dv) in ((True, False, (200, 128, 128)), (False, True, (65, 64, 128)), (True, True, (130, 128, 64))):
            d = kla_inputs.chunk_inputs(2, T, 3, dk, dv, dtype=bf, seed=191 + T, h0_std=0.5)
            if gdn:
                d["k"] = (d["k"].float() * 0.08).to(bf)
            if nq:
                d["q"][1, min(7, T - 1), 2] = 0
            q, k, v, la, eta, h0 = _gpu(d, "q", "k", "v", "log_alpha", "eta", "h0")
            o, hT = kla.kla_chunk_fwd(q, k, v, la, eta, d["eps"], h0=h0, normalize_q=nq, gdn_beta=gdn)
            torch.cuda.synchronize()
            o, hT = o.float().cpu().numpy(), hT.cpu().numpy()
            qn, kn, vn = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
            ro, rh, _ = token_oracle.kla_recurrent(qn, kn, vn, d["log_alpha"].numpy(), d["eta"].numpy(), d["eps"],
                                                   h0=d["h0"].numpy(), normalize_q=nq, gdn_beta=gdn)
            eo, eh = token_oracle.rel_err(o, ro), token_oracle.rel_err(hT, rh)
            print("fused, options nq=%s gdn=%s T=%d: rel err o=%.3e hT=%.3e" % (nq, gdn, T, eo, eh), flush=True)
            assert eo <= TOL[bf] and eh <= TOL[bf]
            if nq:
                assert np.all(o[1, min(7, T - 1), 2] == 0.0)
        return
    if case == "packed":
        d = kla_inputs.varlen_inputs(6, 1, 300, 3, 128, 128, dtype=bf, seed=161, h0_std=0.3)
        _check_chunk(kla, d)
        d = kla_inputs.varlen_inputs(5, 1, 130, 2, 64, 64, dtype=bf, seed=162, h0_std=0.3)
        _check_chunk(kla, d)
        # hand-made lengths: a one-token sequence, exactly one chunk, one chunk + 1, an empty sequence
        lens = [1, 64, 65, 0, 200]
        d = kla_inputs.chunk_inputs(1, sum(lens), 2, 128, 64, dtype=bf, seed=163)
        d["cu_seqlens"] = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32)
        d["h0"] = torch.randn(len(lens), 2, 128, 64, generator=torch.Generator().manual_seed(164)) * 0.3
        _check_chunk(kla, d)
        return
    if case == "extreme_decay":
        d = kla_inputs.chunk_inputs(2, 300, 2, 128, 128, dtype=bf, seed=171, h0_std=0.5, log_alpha_scale=50.0)
        _check_chunk(kla, d)
        return
    if case == "zero_keys_and_eta":
        d = kla_inputs.chunk_inputs(2, 200, 2, 128, 128, dtype=bf, seed=181, h0_std=0.5)
        d["k"][0, 5:9] = 0                      # zero keys: beta = 0 for eps = 0, no write
        d["k"][1, 64:128] = 0                   # a whole chunk of them
        d["eta"][0, 20:40] = 0                  # pure decay steps
        d["eta"][1, :, 1] = 0                   # a head that never writes
        d["eps"] = 0.0
        _check_chunk(kla, d)
        return
    if case == "long_carry":
        d = kla_inputs.chunk_inputs(1, 4000, 2, 128, 128, dtype=bf, seed=175, log_alpha_scale=0.01, h0_std=0.2)
        _check_chunk(kla, d)
        return
    for T in (3, 127, 191, 1000):
        _check_chunk(kla, kla_inputs.chunk_inputs(3, T, 2, 64, 128, dtype=bf, seed=201 + T))


def test_chunk_config2_two_kernel_form(kla, monkeypatch):
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(unfused=True))
    _check_chunk(kla, kla_inputs.config(2))


def test_chunk_varlen_small(kla):
    d = kla_inputs.varlen_inputs(5, 1, 300, 3, 128, 256, seed=61, h0_std=0.3)
    _check_chunk(kla, d)
    d = kla_inputs.varlen_inputs(4, 0, 130, 2, 64, 64, dtype=torch.float32, seed=62, h0_std=0.3)
    _check_chunk(kla, d)


def test_chunk_slow_decay_long_carry(kla):
    """log_alpha scaled by 0.01: the state carries across ~100 chunks, so inter-chunk error would show."""
    d = kla_inputs.chunk_inputs(1, 4096, 2, 128, 128, dtype=torch.bfloat16, seed=71, log_alpha_scale=0.01)
    _check_chunk(kla, d)
    d = kla_inputs.chunk_inputs(1, 2048, 2, 64, 64, dtype=torch.float32, seed=72, log_alpha_scale=0.01)
    _check_chunk(kla, d)


def test_chunk_config2_full(kla):
    """Config 2 at full size, in the launch configuration the benchmark times; every (n, h) compared."""
    _check_chunk(kla, kla_inputs.config(2))


def test_chunk_config3_full(kla):
    _check_chunk(kla, kla_inputs.config(3))


def test_chunk_config5_full(kla):
    """Config 5 at full size (16 packed sequences, 16 heads, d_v = 256, per-sequence h0); every (sequence, head) compared."""
    _check_chunk(kla, kla_inputs.config(5))


def test_split_and_handoff(kla):
    """Resume = pass h_T as h0: chunk_fwd(T1) then chunk_fwd(T2, h0=h_T) equals chunk_fwd(T1+T2), and
    chunk_fwd on T tokens followed by decode_step on token T+1 equals chunk_fwd on T+1 tokens."""
    d = kla_inputs.chunk_inputs(2, 321, 4, 128, 128, dtype=torch.bfloat16, seed=81, log_alpha_scale=0.05)
    q, k, v, la, eta = _gpu(d, "q", "k", "v", "log_alpha", "eta")
    o, hT = kla.kla_chunk_fwd(q, k, v, la, eta, d["eps"])
    a = 192
    o1, h1 = kla.kla_chunk_fwd(q[:, :a].contiguous(), k[:, :a].contiguous(), v[:, :a].contiguous(),
                               la[:, :a].contiguous(), eta[:, :a].contiguous(), d["eps"])
    o2, h2 = kla.kla_chunk_fwd(q[:, a:].contiguous(), k[:, a:].contiguous(), v[:, a:].contiguous(),
                               la[:, a:].contiguous(), eta[:, a:].contiguous(), d["eps"], h0=h1)
    ocat = torch.cat([o1, o2], dim=1).float().cpu().numpy()
    assert token_oracle.rel_err(ocat, o.float().cpu().numpy()) <= 1e-2
    assert token_oracle.rel_err(h2.cpu().numpy(), hT.cpu().numpy()) <= 1e-2
    # prefill T-1 tokens, decode the last one
    T = d["T"]
    o3, h3 = kla.kla_chunk_fwd(q[:, :T - 1].contiguous(), k[:, :T - 1].contiguous(), v[:, :T - 1].contiguous(),
                               la[:, :T - 1].contiguous(), eta[:, :T - 1].contiguous(), d["eps"])
    od = kla.kla_decode_step(q[:, T - 1].contiguous(), k[:, T - 1].contiguous(), v[:, T - 1].contiguous(),
                             la[:, T - 1].contiguous(), eta[:, T - 1].contiguous(), d["eps"], h3)
    assert token_oracle.rel_err(od.float().cpu().numpy(), o[:, T - 1].float().cpu().numpy()) <= 2e-2
    assert token_oracle.rel_err(h3.cpu().numpy(), hT.cpu().numpy()) <= 1e-2


def test_determinism_and_aliasing(kla):
    """No atomics anywhere: two runs are bitwise equal; hT may alias h0."""
    d = kla_inputs.chunk_inputs(2, 500, 4, 128, 128, dtype=torch.bfloat16, seed=91, h0_std=0.2)
    q, k, v, la, eta, h0 = _gpu(d, "q", "k", "v", "log_alpha", "eta", "h0")
    o1, h1 = kla.kla_chunk_fwd(q, k, v, la, eta, d["eps"], h0=h0)
    o2, h2 = kla.kla_chunk_fwd(q, k, v, la, eta, d["eps"], h0=h0)
    assert torch.equal(o1, o2) and torch.equal(h1, h2)
    h_alias = h0.clone()
    o3, h3 = kla.kla_chunk_fwd(q, k, v, la, eta, d["eps"], h0=h_alias, hT=h_alias)
    assert torch.equal(o3, o1) and torch.equal(h_alias, h1)


def test_projection_property_on_gpu(kla):
    """Theorem 1 on the GPU decode path: alpha=1, eta=1, eps=0 => S^T k = v after the write (fp32)."""
    gen = torch.Generator().manual_seed(101)
    B, H, dk, dv = 2, 2, 128, 128
    S = torch.randn((B, H, dk, dv), generator=gen).cuda()
    k = torch.randn((B, H, dk), generator=gen).cuda()
    v = torch.randn((B, H, dv), generator=gen).cuda()
    q = torch.randn((B, H, dk), generator=gen).cuda()
    kla.kla_decode_step(q, k, v, torch.zeros((B, H)).cuda(), torch.ones((B, H)).cuda(), 0.0, S)
    res = torch.einsum("bhkv,bhk->bhv", S.double(), k.double()) - v.double()
    assert float(res.abs().max()) <= 1e-4 * float(v.abs().max())


# ---------------------------------------------------------------------------------------------
# options of the *_opts entry points: normalised read-out (Sec. 3.3) and beta = eta (Table 2)
@pytest.mark.gpu
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("nq,gdn", [(True, False), (False, True), (True, True)])
@pytest.mark.parametrize("T,dk,dv", [(200, 128, 128), (65, 64, 256)])
def test_chunk_options(kla, dt, nq, gdn, T, dk, dv):
    # keys scaled down in the beta = eta mode: without the Kaczmarz denominator I - eta k k^T must stay a contraction
    d = kla_inputs.chunk_inputs(2, T, 3, dk, dv, dtype=dt, seed=91 + T, h0_std=0.5)
    if gdn:
        d["k"] = (d["k"].float() * 0.08).to(dt)
    if nq:                                            # one zero query: its output must be exactly 0
        d["q"][1, min(7, T - 1), 2] = 0
    q, k, v, la, eta, h0 = _gpu(d, "q", "k", "v", "log_alpha", "eta", "h0")
    o, hT = kla.kla_chunk_fwd(q, k, v, la, eta, d["eps"], h0=h0, normalize_q=nq, gdn_beta=gdn)
    torch.cuda.synchronize()
    o, hT = o.float().cpu().numpy(), hT.cpu().numpy()
    qn, kn, vn = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    ro, rh, _ = token_oracle.kla_recurrent(qn, kn, vn, d["log_alpha"].numpy(), d["eta"].numpy(), d["eps"],
                                           h0=d["h0"].numpy(), normalize_q=nq, gdn_beta=gdn)
    eo, eh = token_oracle.rel_err(o, ro), token_oracle.rel_err(hT, rh)
    print("options nq=%s gdn=%s %s T=%d dk=%d dv=%d: rel err o=%.3e hT=%.3e" % (nq, gdn, dt, T, dk, dv, eo, eh), flush=True)
    assert eo <= TOL[dt] and eh <= TOL[dt]
    if nq:
        assert np.all(o[1, min(7, T - 1), 2] == 0.0)
    # the options change the result (the comparison above is not vacuous)
    po, ph = kla.kla_chunk_fwd(q, k, v, la, eta, d["eps"], h0=h0)
    assert token_oracle.rel_err(po.float().cpu().numpy(), ro) > 10 * TOL[dt]


@pytest.mark.gpu
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("nq,gdn", [(True, False), (False, True), (True, True)])
def test_decode_options(kla, dt, nq, gdn):
    d = kla_inputs.decode_inputs(4, 5, 3, 128, 256, dtype=dt, seed=93)
    S = d["S"].cuda()
    Sref = d["S"].numpy().astype(np.float64)
    for t in range(4):
        qt, kt, vt = d["q"][t], (d["k"][t].float() * (0.08 if gdn else 1.0)).to(dt), d["v"][t]
        if nq and t == 1:
            qt = qt.clone(); qt[2, 1] = 0
        o = kla.kla_decode_step(qt.cuda(), kt.cuda(), vt.cuda(), d["log_alpha"][t].cuda(), d["eta"][t].cuda(), d["eps"], S,
                                normalize_q=nq, gdn_beta=gdn)
        ro, Sref = token_oracle.kla_decode(kla_inputs.to_numpy_f32(qt), kla_inputs.to_numpy_f32(kt),
                                           kla_inputs.to_numpy_f32(vt), d["log_alpha"][t].numpy(), d["eta"][t].numpy(),
                                           d["eps"], Sref, normalize_q=nq, gdn_beta=gdn)
        torch.cuda.synchronize()
        assert token_oracle.rel_err(o.float().cpu().numpy(), ro) <= TOL[dt]
        if nq and t == 1:
            assert np.all(o[2, 1].float().cpu().numpy() == 0.0)
    assert token_oracle.rel_err(S.cpu().numpy(), Sref) <= TOL[dt]


# ---------------------------------------------------------------------------------------------
# segment-parallel scan (long sequences in small batches): forced on small shapes, automatic on config 3
@pytest.mark.gpu
@pytest.mark.parametrize("segs", ["2", "3", "5"])
@pytest.mark.parametrize("N,T,H,dk,dv,h0", [(2, 1000, 2, 128, 128, None), (1, 777, 3, 64, 256, 0.3), (1, 130, 1, 128, 64, 0.3)])
def test_chunk_segmented(kla, segs, N, T, H, dk, dv, h0, monkeypatch):
    d = kla_inputs.chunk_inputs(N, T, H, dk, dv, dtype=torch.bfloat16, seed=97 + T, h0_std=h0)
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(segments=1))
    o1, h1 = _run_chunk(kla, d)
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(segments=int(segs)))
    eo, eh = _check_chunk(kla, d)
    o2, h2 = _run_chunk(kla, d)
    # the two routes round differently but agree far inside the bar
    assert token_oracle.rel_err(o2, o1) <= TOL[torch.bfloat16] and token_oracle.rel_err(h2, h1) <= TOL[torch.bfloat16]
    # the segmented route really ran: its workspace holds the maps and the per-segment states
    w1 = kla.kla_chunk_fwd_workspace_bytes(N, T, H, dk, dv, torch.bfloat16, tune=kla.tune(segments=1, unfused=True))
    assert kla.kla_chunk_fwd_workspace_bytes(N, T, H, dk, dv, torch.bfloat16) > w1


@pytest.mark.gpu
@pytest.mark.parametrize("segs", ["3", "5"])
def test_chunk_segmented_slow_decay(kla, segs, monkeypatch):
    """With the usual gates a state is forgotten within a chunk or two, and the maps of a segment are numerically zero;
    here log_alpha is scaled by 0.01, so the state entering a segment carries a thousand tokens of history through the
    composed maps.  The segmented route then rounds differently from the plain one (checked: they differ) and both
    stay inside the bar."""
    d = kla_inputs.chunk_inputs(1, 2000, 2, 128, 128, dtype=torch.bfloat16, seed=98, h0_std=0.3, log_alpha_scale=0.01)
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(segments=1))
    o1, h1 = _run_chunk(kla, d)
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(segments=int(segs)))
    _check_chunk(kla, d)
    o2, h2 = _run_chunk(kla, d)
    assert np.any(h2 != h1)
    assert token_oracle.rel_err(o2, o1) <= TOL[torch.bfloat16] and token_oracle.rel_err(h2, h1) <= TOL[torch.bfloat16]


@pytest.mark.gpu
def test_chunk_segmented_with_options(kla, monkeypatch):
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(segments=4))
    d = kla_inputs.chunk_inputs(1, 900, 2, 128, 128, dtype=torch.bfloat16, seed=99, h0_std=0.2)
    q, k, v, la, eta, h0 = _gpu(d, "q", "k", "v", "log_alpha", "eta", "h0")
    o, hT = kla.kla_chunk_fwd(q, k, v, la, eta, d["eps"], h0=h0, normalize_q=True)
    torch.cuda.synchronize()
    qn, kn, vn = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    ro, rh, _ = token_oracle.kla_recurrent(qn, kn, vn, d["log_alpha"].numpy(), d["eta"].numpy(), d["eps"],
                                           h0=d["h0"].numpy(), normalize_q=True)
    assert token_oracle.rel_err(o.float().cpu().numpy(), ro) <= TOL[torch.bfloat16]
    assert token_oracle.rel_err(hT.cpu().numpy(), rh) <= TOL[torch.bfloat16]
