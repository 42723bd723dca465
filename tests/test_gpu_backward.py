"""GPU parity of the backward pass: kla_chunk_bwd, called through the C ABI, against the fp64 reverse-accumulation
oracle on the same seeded inputs, element by element.

Metric and bars as for the forward: max|x_gpu - x_ref| / max|x_ref| over the whole tensor, <= 1e-4 for fp32
inputs and <= 2e-2 for bf16 inputs, separately for each of dq, dk, dv, dlog_alpha, deta and dh0.
"""
import numpy as np
import pytest
import torch

import bwd_bounds
import kla_inputs
from oracle import token_oracle

pytestmark = pytest.mark.gpu

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}
NAMES = ("dq", "dk", "dv", "dlog_alpha", "deta", "dh0")


@pytest.fixture(scope="module")
def kla():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_08587_amd as m
    m.lib()          # raises if the HIP library is not built: there is no fallback to test instead
    return m


def _cuda(t):
    return None if t is None else t.cuda()


def _run(kla, d, d_o, d_hT, **kw):
    out = kla.kla_chunk_bwd(_cuda(d["q"]), _cuda(d["k"]), _cuda(d["v"]), _cuda(d["log_alpha"]), _cuda(d["eta"]), d["eps"],
                            _cuda(d_o), h0=_cuda(d["h0"]), d_hT=_cuda(d_hT), cu_seqlens=_cuda(d["cu_seqlens"]), **kw)
    torch.cuda.synchronize()
    return {n: (None if out[n] is None else out[n].float().cpu().numpy()) for n in NAMES}


def _oracle(d, d_o, d_hT):
    q, k, v = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    return token_oracle.kla_recurrent_bwd(
        q, k, v, d["log_alpha"].numpy(), d["eta"].numpy(), d["eps"], kla_inputs.to_numpy_f32(d_o),
        h0=None if d["h0"] is None else d["h0"].numpy(), d_hT=None if d_hT is None else d_hT.numpy(),
        cu_seqlens=None if d["cu_seqlens"] is None else d["cu_seqlens"].numpy())


def _check(kla, d, seed, d_hT=True, tol=None):
    tol = tol or TOL[d["dtype"]]
    print("case N=%d T=%d H=%d dk=%d dv=%d %s varlen=%s" % (d["N"], d["T"], d["H"], d["dk"], d["dv"], d["dtype"],
                                                           d["cu_seqlens"] is not None), flush=True)
    d_o, g = kla_inputs.grad_inputs(d, seed, d_hT=d_hT)
    got = _run(kla, d, d_o, g)
    ref = _oracle(d, d_o, g)
    errs = {}
    for n in NAMES:
        x, r = got[n], ref[n]
        assert np.all(np.isfinite(x)), n
        errs[n] = token_oracle.rel_err(x, r)
    print("   rel err " + " ".join("%s=%.2e" % kv for kv in errs.items()) + " (bar %.0e)" % tol, flush=True)
    for n in NAMES:
        assert errs[n] <= tol, (n, errs[n])
    return errs


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dk,dv", [(64, 64), (128, 128), (128, 256), (64, 128)])
@pytest.mark.parametrize("T", [1, 63, 65, 200])
def test_bwd_small_shapes(kla, dt, dk, dv, T):
    """Single chunks, a ragged tail, several chunks; non-zero h0 and d_hT; both state widths per workgroup."""
    _check(kla, kla_inputs.chunk_inputs(2, T, 3, dk, dv, dtype=dt, seed=300 + T + dk + dv, h0_std=0.5), seed=T)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_bwd_without_states(kla, dt):
    """h0 = NULL, d_hT = NULL and dh0 unwanted."""
    d = kla_inputs.chunk_inputs(1, 150, 2, 128, 128, dtype=dt, seed=311)
    d_o, _ = kla_inputs.grad_inputs(d, 1, d_hT=False)
    got = _run(kla, d, d_o, None, want_dh0=False)
    ref = _oracle(d, d_o, None)
    assert got["dh0"] is None
    for n in NAMES[:-1]:
        assert token_oracle.rel_err(got[n], ref[n]) <= TOL[dt], n


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_bwd_varlen(kla, dt):
    """Packed batch with per-sequence h0 and d_hT, lengths from 1 token to several chunks, one empty sequence."""
    d = kla_inputs.varlen_inputs(6, 1, 300, 2, 128, 256 if dt == torch.bfloat16 else 128, dtype=dt, seed=320, h0_std=0.3)
    cu = d["cu_seqlens"].clone()
    cu[3] = cu[2]                              # sequence 2 is empty: its dh0 is d_hT itself
    d["cu_seqlens"] = cu
    _check(kla, d, seed=2)


@pytest.mark.parametrize("dk,dv,T", [(128, 128, 200), (64, 256, 130)])
def test_bwd_generic_kernels_on_bf16(kla, dk, dv, T, monkeypatch):
    """The element-type-generic kernels (the fp32 path's) on bf16 inputs."""
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(generic_bwd=True))
    _check(kla, kla_inputs.chunk_inputs(2, T, 2, dk, dv, dtype=torch.bfloat16, seed=325, h0_std=0.3), seed=9)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_bwd_gdn_beta_option(kla, dt):
    """beta_t = eta_t (Table 2's delta rule): d eta = d beta, and dk has no term through the coefficient."""
    d = kla_inputs.chunk_inputs(2, 200, 2, 128, 128, dtype=dt, seed=370, h0_std=0.3)
    d["k"] = (d["k"].float() / d["k"].float().norm(dim=-1, keepdim=True)).to(dt)       # unit keys: the plain delta rule is stable
    d_o, g = kla_inputs.grad_inputs(d, 10)
    got = _run(kla, d, d_o, g, gdn_beta=True)
    q, k, v = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    ref = token_oracle.kla_recurrent_bwd(q, k, v, d["log_alpha"].numpy(), d["eta"].numpy(), d["eps"],
                                         kla_inputs.to_numpy_f32(d_o), h0=d["h0"].numpy(), d_hT=g.numpy(), gdn_beta=True)
    for n in NAMES:
        assert token_oracle.rel_err(got[n], ref[n]) <= TOL[dt], n


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("dk,dv,T,varlen", [(128, 128, 200, False), (64, 256, 130, False), (128, 256, 300, True)])
def test_bwd_normalize_q_option(kla, dt, dk, dv, T, varlen):
    """o_t = S_t^T q_t / ||q_t|| (Sec. 3.3): gradients of that read-out, with one zero query (dq = 0 there) and queries
    of very different lengths; dq is orthogonal to q."""
    if varlen:
        d = kla_inputs.varlen_inputs(4, 1, T, 2, dk, dv, dtype=dt, seed=380, h0_std=0.3)
    else:
        d = kla_inputs.chunk_inputs(2, T, 2, dk, dv, dtype=dt, seed=381, h0_std=0.3)
    scale = torch.logspace(-1.5, 1.5, d["T"]).reshape(1, d["T"], 1, 1)
    d["q"] = (d["q"].float() * scale).to(dt)
    d["q"][0, 7, 1] = 0
    d_o, g = kla_inputs.grad_inputs(d, 11)
    got = _run(kla, d, d_o, g, normalize_q=True)
    q, k, v = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    ref = token_oracle.kla_recurrent_bwd(q, k, v, d["log_alpha"].numpy(), d["eta"].numpy(), d["eps"],
                                         kla_inputs.to_numpy_f32(d_o), h0=d["h0"].numpy(), d_hT=g.numpy(),
                                         cu_seqlens=None if d["cu_seqlens"] is None else d["cu_seqlens"].numpy(),
                                         normalize_q=True)
    assert np.all(got["dq"][0, 7, 1] == 0.0)
    # dq spans three decades with the query lengths: compare it in units of 1/||q|| (row by row), the rest as usual
    nq = np.linalg.norm(q.astype(np.float64), axis=-1, keepdims=True)
    errs = {n: token_oracle.rel_err(got[n], ref[n]) for n in NAMES if n != "dq"}
    errs["dq"] = token_oracle.rel_err(got["dq"] * nq, ref["dq"] * nq)
    print("   rel err " + " ".join("%s=%.2e" % kv for kv in errs.items()), flush=True)
    for n in NAMES:
        assert errs[n] <= TOL[dt], (n, errs[n])
    if dt == torch.float32:
        cosq = np.sum(got["dq"] * q, -1) / (np.linalg.norm(got["dq"], axis=-1) * nq[..., 0] + 1e-30)
        assert np.max(np.abs(cosq)) <= 1e-3


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_bwd_both_options(kla, dt):
    """Normalised read-out and beta_t = eta_t together."""
    d = kla_inputs.chunk_inputs(2, 150, 2, 128, 128, dtype=dt, seed=385, h0_std=0.3)
    d["k"] = (d["k"].float() / d["k"].float().norm(dim=-1, keepdim=True)).to(dt)
    d_o, g = kla_inputs.grad_inputs(d, 12)
    got = _run(kla, d, d_o, g, normalize_q=True, gdn_beta=True)
    q, k, v = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    ref = token_oracle.kla_recurrent_bwd(q, k, v, d["log_alpha"].numpy(), d["eta"].numpy(), d["eps"],
                                         kla_inputs.to_numpy_f32(d_o), h0=d["h0"].numpy(), d_hT=g.numpy(),
                                         normalize_q=True, gdn_beta=True)
    for n in NAMES:
        assert token_oracle.rel_err(got[n], ref[n]) <= TOL[dt], n


def test_bwd_normalize_q_generic_kernels_on_bf16(kla, monkeypatch):
    """The element-type-generic backward kernels with the normalised read-out, on bf16 inputs."""
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(generic_bwd=True))
    d = kla_inputs.chunk_inputs(2, 130, 2, 128, 128, dtype=torch.bfloat16, seed=386, h0_std=0.3)
    d_o, g = kla_inputs.grad_inputs(d, 13)
    got = _run(kla, d, d_o, g, normalize_q=True)
    q, k, v = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    ref = token_oracle.kla_recurrent_bwd(q, k, v, d["log_alpha"].numpy(), d["eta"].numpy(), d["eps"],
                                         kla_inputs.to_numpy_f32(d_o), h0=d["h0"].numpy(), d_hT=g.numpy(), normalize_q=True)
    for n in NAMES:
        assert token_oracle.rel_err(got[n], ref[n]) <= TOL[torch.bfloat16], n


def test_bwd_two_waves_per_workgroup(kla):
    """Enough (sequence, head) pairs for the 32-column workgroups the benchmark shape uses."""
    _check(kla, kla_inputs.chunk_inputs(16, 192, 4, 128, 128, dtype=torch.bfloat16, seed=330, h0_std=0.1), seed=3)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_bwd_eta_zero_and_zero_keys(kla, dt):
    """Tokens with eta = 0 (beta = 0 but d eta != 0) and zero keys (the coefficient's denominator is eps alone)."""
    d = kla_inputs.chunk_inputs(1, 200, 2, 64, 64, dtype=dt, seed=340, h0_std=0.5)
    d["eta"][:, ::5] = 0.0
    d["k"][:, 7::11] = 0.0
    d["eps"] = 0.5
    _check(kla, d, seed=4)


def test_bwd_slow_decay_long_carry(kla):
    """Slow decay: gradients travel over a thousand tokens, so errors of the state sweeps would add up."""
    d = kla_inputs.chunk_inputs(1, 1500, 2, 128, 128, dtype=torch.bfloat16, seed=350, log_alpha_scale=0.02, h0_std=0.2)
    _check(kla, d, seed=5)
    d = kla_inputs.chunk_inputs(1, 700, 2, 64, 64, dtype=torch.float32, seed=351, log_alpha_scale=0.02, h0_std=0.2)
    _check(kla, d, seed=6)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_bwd_extreme_decay(kla, dt):
    """log_alpha scaled by 50 (down to -150 per token): nothing overflows and every gradient but one keeps the usual bar.
    d log_alpha is formed chunkwise as a running sum of three inner products per token (see bwd_bounds.py); where the
    decay wipes the state out almost completely they cancel to a thousandth of their size (here: parts up to 44, result
    up to 0.015), so fp32 inputs are held to 1e-4 of the result or 1e-5 of the parts that were summed, whichever is
    larger; bf16 inputs keep their plain bar."""
    d = kla_inputs.chunk_inputs(2, 200, 2, 128, 128, dtype=dt, seed=353, h0_std=0.3, log_alpha_scale=50.0)
    d_o, g = kla_inputs.grad_inputs(d, 25)
    got = _run(kla, d, d_o, g)
    ref = _oracle(d, d_o, g)
    errs = {n: token_oracle.rel_err(got[n], ref[n]) for n in NAMES}
    print("   rel err " + " ".join("%s=%.2e" % kv for kv in errs.items()), flush=True)
    for n in NAMES:
        assert np.all(np.isfinite(got[n])), n
        if n == "dlog_alpha" and dt == torch.float32:
            _, parts = bwd_bounds.bounds(d, d_o, g, lambda t: kla_inputs.to_numpy_f32(t).astype(np.float64))
            bar_abs = max(TOL[dt] * np.abs(ref[n]).max(), 1e-5 * parts.max())
            print("   dlog_alpha: max|ref| %.3e, parts up to %.3e, max abs err %.3e (bar %.3e)" % (
                np.abs(ref[n]).max(), parts.max(), np.abs(got[n] - ref[n]).max(), bar_abs), flush=True)
            assert parts.max() > 100 * np.abs(ref[n]).max()          # the case is what it claims to be
            assert np.abs(got[n] - ref[n]).max() <= bar_abs
        else:
            assert errs[n] <= TOL[dt], (n, errs[n])


def test_bwd_config2_full(kla):
    """Config 2 at full size, in the launch configuration the benchmark times; every (sequence, head) compared."""
    _check(kla, kla_inputs.config(2), seed=7, d_hT=True)


def test_bwd_config3_full(kla):
    """Config 3 at full size (one 65 536-token sequence, 8 heads), in the launch configuration the benchmark times:
    segment-parallel sweeps, eight segments chosen by the library; every head compared."""
    d = kla_inputs.config(3)
    assert kla.kla_chunk_bwd_workspace_bytes(d["N"], d["T"], d["H"], d["dk"], d["dv"], torch.bfloat16) > \
        kla.kla_chunk_bwd_workspace_bytes(d["N"], d["T"], d["H"], d["dk"], d["dv"], torch.bfloat16, tune=kla.tune(segments=1))
    _check(kla, d, seed=9, d_hT=True)


def test_bwd_determinism(kla):
    """No atomics: two runs are bitwise equal."""
    d = kla_inputs.chunk_inputs(2, 300, 4, 128, 128, dtype=torch.bfloat16, seed=360, h0_std=0.2)
    d_o, g = kla_inputs.grad_inputs(d, 8)
    a = _run(kla, d, d_o, g)
    b = _run(kla, d, d_o, g)
    for n in NAMES:
        assert np.array_equal(a[n], b[n]), n


def test_bwd_no_tokens(kla):
    """Sequences without tokens: the state passes through, so dh0 = d_hT and nothing else is written."""
    H, dk, dv = 2, 128, 128
    z = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device="cuda")
    g = torch.randn((3, H, dk, dv), generator=torch.Generator().manual_seed(1)).cuda()
    cu = torch.zeros(4, dtype=torch.int32, device="cuda")
    out = kla.kla_chunk_bwd(z(1, 0, H, dk), z(1, 0, H, dk), z(1, 0, H, dv), torch.zeros((1, 0, H), device="cuda"),
                            torch.zeros((1, 0, H), device="cuda"), 1e-6, z(1, 0, H, dv), h0=torch.zeros_like(g), d_hT=g,
                            cu_seqlens=cu)
    torch.cuda.synchronize()
    assert torch.equal(out["dh0"], g)


def test_bwd_config5_full(kla):
    """Config 5 at full size (16 packed sequences, H = 16, d_v = 256, per-sequence h0); every (sequence, head) compared."""
    _check(kla, kla_inputs.config(5), seed=11)


# ---------------------------------------------------------------------------------------------
# segment-parallel sweeps (long sequences in small batches): forced on small shapes, automatic on long ones
@pytest.mark.parametrize("segs", ["2", "3", "5"])
@pytest.mark.parametrize("N,T,H,dk,dv,h0,ghT", [(2, 1000, 2, 128, 128, None, True), (1, 777, 3, 64, 256, 0.3, True),
                                               (1, 130, 1, 128, 64, 0.3, False)])
def test_bwd_segmented(kla, segs, N, T, H, dk, dv, h0, ghT, monkeypatch):
    """The tuning field forces the segmented sweeps; ragged last segments, two segments (no reverse composition
    step), with and without h0 and d_hT.  The two routes agree far inside the bar, and the segmented one really ran
    (its workspace holds the maps and the per-segment states)."""
    d = kla_inputs.chunk_inputs(N, T, H, dk, dv, dtype=torch.bfloat16, seed=197 + T, h0_std=h0)
    d_o, g = kla_inputs.grad_inputs(d, 21, d_hT=ghT)
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(segments=1))
    w1 = kla.kla_chunk_bwd_workspace_bytes(N, T, H, dk, dv, torch.bfloat16)
    one = _run(kla, d, d_o, g)
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(segments=int(segs)))
    assert kla.kla_chunk_bwd_workspace_bytes(N, T, H, dk, dv, torch.bfloat16) > w1
    got = _run(kla, d, d_o, g)
    ref = _oracle(d, d_o, g)
    errs = {n: token_oracle.rel_err(got[n], ref[n]) for n in NAMES}
    print("   rel err " + " ".join("%s=%.2e" % kv for kv in errs.items()), flush=True)
    for n in NAMES:
        assert errs[n] <= TOL[torch.bfloat16], (n, errs[n])
        assert token_oracle.rel_err(got[n], one[n]) <= TOL[torch.bfloat16], n


@pytest.mark.parametrize("segs", ["2", "3", "5"])
def test_bwd_segmented_slow_decay(kla, segs, monkeypatch):
    """log_alpha scaled by 0.02: states and their gradients carry over a thousand tokens, so the composed maps (forward)
    and their transposes (reverse) matter - with the usual gates they are numerically zero.  The segmented route rounds
    differently from the plain one (checked: they differ) and both stay inside the bar."""
    d = kla_inputs.chunk_inputs(1, 1500, 2, 128, 128, dtype=torch.bfloat16, seed=352, log_alpha_scale=0.02, h0_std=0.2)
    d_o, g = kla_inputs.grad_inputs(d, 24)
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(segments=1))
    one = _run(kla, d, d_o, g)
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(segments=int(segs)))
    got = _run(kla, d, d_o, g)
    ref = _oracle(d, d_o, g)
    errs = {n: token_oracle.rel_err(got[n], ref[n]) for n in NAMES}
    print("   rel err " + " ".join("%s=%.2e" % kv for kv in errs.items()), flush=True)
    print("   vs plain " + " ".join("%s=%.2e" % (n, token_oracle.rel_err(got[n], one[n])) for n in NAMES), flush=True)
    # dq sees the forward states; dh0 only the reverse sweep, which with two segments is the plain computation
    assert np.any(got["dq"] != one["dq"]) and (segs == "2" or np.any(got["dh0"] != one["dh0"]))
    for n in NAMES:
        assert errs[n] <= TOL[torch.bfloat16], (n, errs[n])
        assert token_oracle.rel_err(got[n], one[n]) <= TOL[torch.bfloat16], n


def test_bwd_segmented_with_options(kla, monkeypatch):
    monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(segments=4))
    d = kla_inputs.chunk_inputs(1, 900, 2, 128, 128, dtype=torch.bfloat16, seed=199, h0_std=0.2)
    d["k"] = (d["k"].float() / d["k"].float().norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    d_o, g = kla_inputs.grad_inputs(d, 22)
    got = _run(kla, d, d_o, g, normalize_q=True, gdn_beta=True)
    q, k, v = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
    ref = token_oracle.kla_recurrent_bwd(q, k, v, d["log_alpha"].numpy(), d["eta"].numpy(), d["eps"],
                                         kla_inputs.to_numpy_f32(d_o), h0=d["h0"].numpy(), d_hT=g.numpy(),
                                         normalize_q=True, gdn_beta=True)
    for n in NAMES:
        assert token_oracle.rel_err(got[n], ref[n]) <= TOL[torch.bfloat16], n


def test_bwd_segmented_automatic_long_sequence(kla):
    """One sequence of 8192 tokens on two heads: few chains, many chunks - the sweeps are cut into segments by the
    library's own rule (the workspace says so); all gradients against the oracle."""
    N, T, H, dk, dv = 1, 8192, 2, 128, 128
    d = kla_inputs.chunk_inputs(N, T, H, dk, dv, dtype=torch.bfloat16, seed=198, h0_std=0.2)
    eb = 2
    plain = 3 * N * T * H * dv * eb + 2 * (N * (T // 64) * H) * dk * dv * eb + (N * (T // 64) * H) * (3 * 6144 + 1280)
    assert kla.kla_chunk_bwd_workspace_bytes(N, T, H, dk, dv, torch.bfloat16) > plain + 4 * dk * dv * 4 * H
    _check(kla, d, seed=23)


def test_autograd_wrapper_matches_the_entry_points(kla):
    """kla.kla_chunk: torch autograd through the two entry points gives exactly what calling them by hand gives."""
    d = kla_inputs.chunk_inputs(2, 150, 2, 128, 128, dtype=torch.bfloat16, seed=390, h0_std=0.3)
    d_o, g = kla_inputs.grad_inputs(d, 26)
    leaves = {n: d[n].cuda().requires_grad_(True) for n in ("q", "k", "v", "log_alpha", "eta", "h0")}
    o, hT = kla.kla_chunk(leaves["q"], leaves["k"], leaves["v"], leaves["log_alpha"], leaves["eta"], d["eps"], h0=leaves["h0"],
                          normalize_q=True)
    torch.autograd.backward([o, hT], [d_o.cuda(), g.cuda()])
    torch.cuda.synchronize()
    ref = _run(kla, d, d_o, g, normalize_q=True)
    o2, h2 = kla.kla_chunk_fwd(*(leaves[n].detach() for n in ("q", "k", "v", "log_alpha", "eta")), d["eps"],
                               h0=leaves["h0"].detach(), normalize_q=True)
    assert torch.equal(o, o2) and torch.equal(hT, h2)
    for n, leaf in (("dq", "q"), ("dk", "k"), ("dv", "v"), ("dlog_alpha", "log_alpha"), ("deta", "eta"), ("dh0", "h0")):
        assert np.array_equal(leaves[leaf].grad.float().cpu().numpy(), ref[n]), n
