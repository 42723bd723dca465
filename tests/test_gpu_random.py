"""Seeded random sweep over shapes, dtypes, packing, initial states, gate ranges, options and launch knobs: every case is
one call of an entry point compared element by element with the oracle, to the usual bars.  The cases are drawn from
one numpy generator, so the sweep is the same on every run; it is meant to reach combinations the hand-written cases
do not name."""
import numpy as np
import pytest
import torch

import bwd_bounds
import kla_inputs
from oracle import token_oracle

pytestmark = pytest.mark.gpu
TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}
f32 = kla_inputs.to_numpy_f32


@pytest.fixture(scope="module")
def kla():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_08587_amd as m
    m.lib()
    return m


def _c(t):
    return None if t is None else t.cuda()


def _draw(rng):
    dt = torch.bfloat16 if rng.random() < 0.6 else torch.float32
    dk, dv = int(rng.choice([64, 128])), int(rng.choice([64, 128, 256]))
    H = int(rng.choice([1, 2, 3, 5, 8]))
    seed = int(rng.integers(1 << 30))
    h0 = 0.3 if rng.random() < 0.7 else None
    if rng.random() < 0.4:
        d = kla_inputs.varlen_inputs(int(rng.integers(1, 7)), 1, int(rng.choice([5, 70, 200, 400])), H, dk, dv, dtype=dt, seed=seed,
                                     h0_std=h0)
    else:
        d = kla_inputs.chunk_inputs(int(rng.integers(1, 5)), int(rng.choice([1, 2, 17, 64, 65, 127, 128, 129, 300, 513])), H, dk, dv,
                                    dtype=dt, seed=seed, h0_std=h0, log_alpha_scale=float(rng.choice([1.0, 0.1, 3.0, 0.02])))
    return d, seed


@pytest.mark.parametrize("block", range(4))
def test_random_cases(kla, block, monkeypatch):
    rng = np.random.default_rng(1000 + block)
    for case in range(12):
        d, seed = _draw(rng)
        dt = d["dtype"]
        kind = str(rng.choice(["fwd", "bwd", "diag"]))
        nq, gdn = bool(rng.random() < 0.3), bool(rng.random() < 0.2)
        segs, waves = str(rng.choice(["", "2", "3", "7"])), str(rng.choice(["", "1", "2", "4"]))
        form = str(rng.choice(["auto", "fused", "unfused"]))
        monkeypatch.setattr(kla, "DEFAULT_TUNE", kla.tune(segments=int(segs or 0), scan_waves=int(waves or 0), fused=form == "fused",
                                                        unfused=form == "unfused"))
        if gdn:                                    # the plain delta rule is only stable for short keys
            d["k"] = (d["k"].float() / d["k"].float().norm(dim=-1, keepdim=True).clamp_min(1e-6)).to(dt)
        print("block %d case %d: %s %s N=%d T=%d H=%d dk=%d dv=%d packed=%s h0=%s nq=%s gdn=%s segments=%s waves=%s form=%s" % (
            block, case, kind, str(dt)[6:], d["N"], d["T"], d["H"], d["dk"], d["dv"], d["cu_seqlens"] is not None,
            d["h0"] is not None, nq, gdn, segs or "-", waves or "-", form), flush=True)
        a = [_c(d[x]) for x in ("q", "k", "v", "log_alpha", "eta")]
        n = [f32(d[x]) for x in "qkv"] + [d["log_alpha"].numpy(), d["eta"].numpy()]
        cu = None if d["cu_seqlens"] is None else d["cu_seqlens"].numpy()
        h0n = None if d["h0"] is None else d["h0"].numpy()
        if kind == "fwd":
            o, hT = kla.kla_chunk_fwd(*a, d["eps"], h0=_c(d["h0"]), cu_seqlens=_c(d["cu_seqlens"]), normalize_q=nq, gdn_beta=gdn)
            ro, rh, _ = token_oracle.kla_recurrent(*n, d["eps"], h0=h0n, cu_seqlens=cu, normalize_q=nq, gdn_beta=gdn)
            errs = {"o": token_oracle.rel_err(o.float().cpu().numpy(), ro), "hT": token_oracle.rel_err(hT.cpu().numpy(), rh)}
        elif kind == "bwd":
            d_o, g = kla_inputs.grad_inputs(d, seed % 1000, d_hT=bool(rng.random() < 0.7))
            out = kla.kla_chunk_bwd(*a, d["eps"], _c(d_o), h0=_c(d["h0"]), d_hT=_c(g), cu_seqlens=_c(d["cu_seqlens"]),
                                    normalize_q=nq, gdn_beta=gdn)
            ref = token_oracle.kla_recurrent_bwd(*n, d["eps"], f32(d_o), h0=h0n, d_hT=None if g is None else g.numpy(),
                                                 cu_seqlens=cu, normalize_q=nq, gdn_beta=gdn)
            errs = {k: token_oracle.rel_err(out[k].float().cpu().numpy(), ref[k]) for k in ref}
            if nq:                                 # dq scales with 1/||q||: compare it row by row in those units
                qn = np.linalg.norm(n[0].astype(np.float64), axis=-1, keepdims=True)
                errs["dq"] = token_oracle.rel_err(out["dq"].float().cpu().numpy() * qn, ref["dq"] * qn)
            if d["T"] * d["H"] < 64 and dt == torch.bfloat16:
                # a handful of entries, each a sum over d_v products of bf16-rounded rows that mostly cancel: d eta is
                # held to the first-order bound of that rounding where it exceeds the plain bar (see bwd_bounds.py)
                be, _ = bwd_bounds.bounds(d, d_o, g, lambda t: f32(t).astype(np.float64))
                bound = float(be.max() / max(np.abs(ref["deta"]).max(), 1e-300))
                print("    deta: first-order bound of the bf16 intermediates %.2e" % bound, flush=True)
                assert errs["deta"] <= max(TOL[dt], bound), errs["deta"]
                errs.pop("deta")
        else:
            lad = kla_inputs.diag_gates(d, seed % 1000, float(rng.choice([1.0, 0.1, 5.0])))
            o, hT = kla.kla_chunk_fwd_diag(a[0], a[1], a[2], _c(lad), a[4], d["eps"], h0=_c(d["h0"]), cu_seqlens=_c(d["cu_seqlens"]),
                                           normalize_q=nq, gdn_beta=gdn)
            ro, rh, _ = token_oracle.kla_recurrent_diag(n[0], n[1], n[2], lad.numpy(), n[4], d["eps"], h0=h0n, cu_seqlens=cu,
                                                        normalize_q=nq, gdn_beta=gdn)
            errs = {"o": token_oracle.rel_err(o.float().cpu().numpy(), ro), "hT": token_oracle.rel_err(hT.cpu().numpy(), rh)}
        print("    " + " ".join("%s=%.2e" % kv for kv in errs.items()), flush=True)
        for k, e in errs.items():
            assert np.isfinite(e) and e <= TOL[dt], (k, e)
