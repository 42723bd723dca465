"""Maximum sizes: tensors of more than 2^31 elements and 2^32 bytes, so that every offset the kernels form has to
be 64-bit.  The inputs are drawn on the GPU (kla_inputs.device_randn); the oracle gets the slices of the sampled
(sequence, head) units copied back to the host - the first unit, the last one (largest offsets) and one in the
middle - and the comparison is element by element on those units, to the usual bars."""
import numpy as np
import pytest
import torch

import kla_inputs
from oracle import token_oracle

pytestmark = pytest.mark.gpu
TOL = 2e-2          # bf16 inputs


@pytest.fixture(scope="module")
def kla():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    if torch.cuda.get_device_properties(0).total_memory < 160 * 2 ** 30:
        pytest.skip("needs about 100 GB of device memory")
    import paper_2605_08587_amd as m
    m.lib()
    return m


N, T, H, DK, DV = 66, 16384, 16, 128, 128           # 66 * 16384 * 16 * 128 = 2.2e9 elements per tensor
UNITS = ((0, 0), (N // 2, 5), (N - 1, H - 1))


@pytest.fixture(scope="module")
def big(kla):
    assert N * T * H * DK > 2 ** 31 and N * T * H * DK * 2 > 2 ** 32
    q = kla_inputs.device_randn((N, T, H, DK), torch.bfloat16, 901)
    k = kla_inputs.device_randn((N, T, H, DK), torch.bfloat16, 902)
    v = kla_inputs.device_randn((N, T, H, DV), torch.bfloat16, 903)
    la, eta = kla_inputs.device_gates((N, T, H), 904)
    h0 = kla_inputs.device_randn((N, H, DK, DV), torch.float32, 906, std=0.1)
    torch.cuda.synchronize()
    yield dict(q=q, k=k, v=v, log_alpha=la, eta=eta, h0=h0)
    del q, k, v, la, eta, h0
    torch.cuda.empty_cache()


def _unit(d, n, h):
    """Host copies of one (sequence, head) unit, shaped [1, T, 1, *] like a batch of its own."""
    f = lambda t: t[n:n + 1, :, h:h + 1].float().cpu().numpy()
    return (f(d["q"]), f(d["k"]), f(d["v"]), d["log_alpha"][n:n + 1, :, h:h + 1].cpu().numpy().astype(np.float64),
            d["eta"][n:n + 1, :, h:h + 1].cpu().numpy().astype(np.float64), d["h0"][n:n + 1, h:h + 1].cpu().numpy())


def test_chunk_fwd_beyond_2G_elements(kla, big):
    o, hT = kla.kla_chunk_fwd(big["q"], big["k"], big["v"], big["log_alpha"], big["eta"], kla_inputs.EPS, h0=big["h0"])
    torch.cuda.synchronize()
    for n, h in UNITS:
        q, k, v, la, eta, h0 = _unit(big, n, h)
        ro, rh, _ = token_oracle.kla_recurrent(q, k, v, la, eta, kla_inputs.EPS, h0=h0)
        eo = token_oracle.rel_err(o[n, :, h].float().cpu().numpy(), ro[0, :, 0])
        eh = token_oracle.rel_err(hT[n, h].cpu().numpy(), rh[0, 0])
        print("unit (%d, %d): rel err o=%.3e hT=%.3e" % (n, h, eo, eh), flush=True)
        assert eo <= TOL and eh <= TOL
    del o, hT


def test_chunk_fwd_packed_beyond_2G_elements(kla, big):
    """The same memory as one packed batch [1, N*T, H, *] of 700 sequences with seeded lengths; the last sequence
    sits at the largest offsets."""
    total = N * T
    gen = torch.Generator().manual_seed(77)
    cuts = torch.sort(torch.randperm(total - 1, generator=gen)[:699] + 1).values
    cu = torch.cat([torch.zeros(1, dtype=torch.long), cuts, torch.tensor([total])]).to(torch.int32)
    n_seq = cu.numel() - 1
    pk = {x: big[x].view(1, total, H, -1) for x in "qkv"}
    la, eta = big["log_alpha"].view(1, total, H), big["eta"].view(1, total, H)
    h0 = kla_inputs.device_randn((n_seq, H, DK, DV), torch.float32, 907, std=0.1)
    o, hT = kla.kla_chunk_fwd(pk["q"], pk["k"], pk["v"], la, eta, kla_inputs.EPS, h0=h0, cu_seqlens=cu.cuda(), cu_seqlens_host=cu)
    torch.cuda.synchronize()
    for s, h in ((0, 0), (n_seq // 2, 7), (n_seq - 1, H - 1)):
        a, b = int(cu[s]), int(cu[s + 1])
        f = lambda t: t[:, a:b, h:h + 1].float().cpu().numpy()
        ro, rh, _ = token_oracle.kla_recurrent(f(pk["q"]), f(pk["k"]), f(pk["v"]), la[:, a:b, h:h + 1].cpu().numpy().astype(np.float64),
                                               eta[:, a:b, h:h + 1].cpu().numpy().astype(np.float64), kla_inputs.EPS,
                                               h0=h0[s:s + 1, h:h + 1].cpu().numpy())
        eo = token_oracle.rel_err(o[0, a:b, h].float().cpu().numpy(), ro[0, :, 0])
        eh = token_oracle.rel_err(hT[s, h].cpu().numpy(), rh[0, 0])
        print("sequence %d (tokens %d..%d), head %d: rel err o=%.3e hT=%.3e" % (s, a, b, h, eo, eh), flush=True)
        assert eo <= TOL and eh <= TOL
    del o, hT, h0


def test_chunk_fwd_diag_beyond_2G_elements(kla, big):
    xa = kla_inputs.device_randn((N, T, H, DK), torch.float32, 908)
    lad = -torch.nn.functional.softplus(xa)
    del xa
    o, hT = kla.kla_chunk_fwd_diag(big["q"], big["k"], big["v"], lad, big["eta"], kla_inputs.EPS, h0=big["h0"])
    torch.cuda.synchronize()
    for n, h in (UNITS[0], UNITS[2]):
        q, k, v, _, eta, h0 = _unit(big, n, h)
        ro, rh, _ = token_oracle.kla_recurrent_diag(q, k, v, lad[n:n + 1, :, h:h + 1].cpu().numpy().astype(np.float64), eta,
                                                    kla_inputs.EPS, h0=h0)
        eo = token_oracle.rel_err(o[n, :, h].float().cpu().numpy(), ro[0, :, 0])
        eh = token_oracle.rel_err(hT[n, h].cpu().numpy(), rh[0, 0])
        print("unit (%d, %d): rel err o=%.3e hT=%.3e" % (n, h, eo, eh), flush=True)
        assert eo <= TOL and eh <= TOL
    del o, hT, lad


def test_chunk_bwd_beyond_2G_elements(kla, big):
    d_o = kla_inputs.device_randn((N, T, H, DV), torch.bfloat16, 909)
    d_hT = kla_inputs.device_randn((N, H, DK, DV), torch.float32, 910)
    g = kla.kla_chunk_bwd(big["q"], big["k"], big["v"], big["log_alpha"], big["eta"], kla_inputs.EPS, d_o, h0=big["h0"], d_hT=d_hT)
    torch.cuda.synchronize()
    for n, h in (UNITS[0], UNITS[2]):
        q, k, v, la, eta, h0 = _unit(big, n, h)
        ref = token_oracle.kla_recurrent_bwd(q, k, v, la, eta, kla_inputs.EPS, d_o[n:n + 1, :, h:h + 1].float().cpu().numpy(),
                                             h0=h0, d_hT=d_hT[n:n + 1, h:h + 1].cpu().numpy())
        errs = {}
        for name in ("dq", "dk", "dv", "dlog_alpha", "deta"):
            errs[name] = token_oracle.rel_err(g[name][n, :, h].float().cpu().numpy(), ref[name][0, :, 0])
        errs["dh0"] = token_oracle.rel_err(g["dh0"][n, h].cpu().numpy(), ref["dh0"][0, 0])
        print("unit (%d, %d): rel err " % (n, h) + " ".join("%s=%.2e" % kv for kv in errs.items()), flush=True)
        assert max(errs.values()) <= TOL, errs
    del g, d_o, d_hT


def test_decode_beyond_2G_elements(kla):
    """131 200 (batch, head) states of 128 x 128 fp32: 2.15e9 elements, 8.6 GB."""
    B, Hd = 8200, 16
    assert B * Hd * DK * DV > 2 ** 31
    S = kla_inputs.device_randn((B, Hd, DK, DV), torch.float32, 920, std=0.02)
    q = kla_inputs.device_randn((B, Hd, DK), torch.bfloat16, 921)
    k = kla_inputs.device_randn((B, Hd, DK), torch.bfloat16, 922)
    v = kla_inputs.device_randn((B, Hd, DV), torch.bfloat16, 923)
    la, eta = kla_inputs.device_gates((B, Hd), 924)
    rows = [0, B // 2, B - 1]
    S0 = {b: S[b].cpu().numpy() for b in rows}
    o = kla.kla_decode_step(q, k, v, la, eta, kla_inputs.EPS, S)
    torch.cuda.synchronize()
    for b in rows:
        f = lambda t: t[b:b + 1].float().cpu().numpy()
        ro, rS = token_oracle.kla_decode(f(q), f(k), f(v), la[b:b + 1].cpu().numpy().astype(np.float64),
                                         eta[b:b + 1].cpu().numpy().astype(np.float64), kla_inputs.EPS, S0[b][None])
        eo = token_oracle.rel_err(o[b].float().cpu().numpy(), ro[0])
        es = token_oracle.rel_err(S[b].cpu().numpy(), rS[0])
        print("batch row %d: rel err o=%.3e S=%.3e" % (b, eo, es), flush=True)
        assert eo <= TOL and es <= TOL
