"""Seeded synthetic inputs for the KLA hot path.

Shared by the tests, the smoke check and the benchmark; used by both the CPU
oracle and the GPU library, and therefore holds none of the method's
arithmetic: it only draws tensors.  The workloads stand in for the paper's
(text through a trained 0.4B model, which is not available): they copy its
shapes -- 8 heads of dimension 128 (App. C), 4K training context (Sec. 5.1),
65K evaluation context (Table 3), 32K decode context (Sec. 5.4), eps = 1e-6
(App. C), value expansion 2 (Sec. 5.5) -- with Gaussian q, k, v and gates
log_alpha = -softplus(x), eta = sigmoid(x), x ~ N(0,1).

Draw order from one CPU torch.Generator seeded with `seed`:
q, k, v, [per-token key scale], x_alpha, x_eta, [h0 or S].  Everything is drawn
in fp32 on the CPU and then cast, so the same seed gives the same tensors on
every machine.
"""
from __future__ import annotations

import torch

EPS = 1e-6


def _gates(gen, shape):
    xa = torch.randn(shape, generator=gen, dtype=torch.float32)
    xe = torch.randn(shape, generator=gen, dtype=torch.float32)
    return -torch.nn.functional.softplus(xa), torch.sigmoid(xe)


def chunk_inputs(N, T, H, dk, dv, dtype=torch.bfloat16, seed=0, k_scale=False, h0_std=None,
                 n_h0=None, log_alpha_scale=1.0):
    """Fixed-length batch: q,k [N,T,H,dk], v [N,T,H,dv] in `dtype`; fp32 gates [N,T,H]."""
    gen = torch.Generator().manual_seed(seed)
    q = torch.randn((N, T, H, dk), generator=gen, dtype=torch.float32)
    k = torch.randn((N, T, H, dk), generator=gen, dtype=torch.float32)
    v = torch.randn((N, T, H, dv), generator=gen, dtype=torch.float32)
    if k_scale:
        c = torch.rand((N, T, H, 1), generator=gen, dtype=torch.float32) * 1.5 + 0.5
        k = k * c
    log_alpha, eta = _gates(gen, (N, T, H))
    h0 = None
    if h0_std is not None:
        h0 = torch.randn((n_h0 or N, H, dk, dv), generator=gen, dtype=torch.float32) * h0_std
    return dict(q=q.to(dtype), k=k.to(dtype), v=v.to(dtype), log_alpha=log_alpha * log_alpha_scale,
                eta=eta, h0=h0, eps=EPS, cu_seqlens=None, N=N, T=T, H=H, dk=dk, dv=dv, dtype=dtype)


def varlen_inputs(n_seq, lo, hi, H, dk, dv, dtype=torch.bfloat16, seed=4, h0_std=0.02):
    """Packed variable-length batch [1, sum(len), H, *] with int32 cu_seqlens [n_seq+1]."""
    gen = torch.Generator().manual_seed(seed)
    lens = torch.randint(lo, hi + 1, (n_seq,), generator=gen)
    cu = torch.zeros(n_seq + 1, dtype=torch.int32)
    cu[1:] = torch.cumsum(lens, 0).to(torch.int32)
    total = int(cu[-1])
    d = chunk_inputs(1, total, H, dk, dv, dtype=dtype, seed=seed + 1000, h0_std=h0_std, n_h0=n_seq)
    d["cu_seqlens"] = cu
    return d


def decode_inputs(steps, B, H, dk, dv, dtype=torch.bfloat16, seed=3, state_std=0.02):
    """`steps` decode tokens: q,k [steps,B,H,dk], v [steps,B,H,dv], gates [steps,B,H], S [B,H,dk,dv]."""
    gen = torch.Generator().manual_seed(seed)
    q = torch.randn((steps, B, H, dk), generator=gen, dtype=torch.float32)
    k = torch.randn((steps, B, H, dk), generator=gen, dtype=torch.float32)
    v = torch.randn((steps, B, H, dv), generator=gen, dtype=torch.float32)
    log_alpha, eta = _gates(gen, (steps, B, H))
    S = torch.randn((B, H, dk, dv), generator=gen, dtype=torch.float32) * state_std
    return dict(q=q.to(dtype), k=k.to(dtype), v=v.to(dtype), log_alpha=log_alpha, eta=eta, S=S,
                eps=EPS, steps=steps, B=B, H=H, dk=dk, dv=dv, dtype=dtype)


def config(i: int):
    """The five benchmark configurations, numbered 1..5."""
    if i == 1:   # tiny fp32 chunk forward
        return chunk_inputs(1, 256, 2, 64, 64, dtype=torch.float32, seed=0)
    if i == 2:   # 0.4B-scale training shape; keys scaled per token by U(0.5, 2)
        return chunk_inputs(8, 4096, 8, 128, 128, seed=1, k_scale=True)
    if i == 3:   # long-context prefill
        return chunk_inputs(1, 65536, 8, 128, 128, seed=2)
    if i == 4:   # decode at 32K context, 256 consecutive steps
        return decode_inputs(256, 64, 8, 128, 128, seed=3)
    if i == 5:   # packed variable-length batch, d_v = 2 d_k, non-zero initial states
        return varlen_inputs(16, 512, 4096, 16, 128, 256, seed=4)
    raise ValueError("config index must be 1..5")


def to_numpy_f32(t):
    """Exact widening of a bf16/fp32 torch tensor to a float32 numpy array."""
    return t.detach().to("cpu").to(torch.float32).contiguous().numpy()


def grad_inputs(d, seed=0, d_hT=True):
    """Upstream gradients for a chunk-forward input set d: d_o ~ N(0,1) in the dtype of v, d_hT ~ N(0,1) fp32."""
    gen = torch.Generator().manual_seed(10_000 + seed)
    d_o = torch.randn(tuple(d["v"].shape), generator=gen, dtype=torch.float32).to(d["dtype"])
    n_states = d["N"] if d["cu_seqlens"] is None else d["cu_seqlens"].numel() - 1
    g = torch.randn((n_states, d["H"], d["dk"], d["dv"]), generator=gen, dtype=torch.float32) if d_hT else None
    return d_o, g


def diag_gates(d, seed=0, scale=1.0):
    """Per-channel decay gates for diagonal gating: log_alpha [.., dk] = -softplus(x) * scale, x ~ N(0,1), shaped like
    d["k"] (chunk inputs) in fp32."""
    gen = torch.Generator().manual_seed(20_000 + seed)
    x = torch.randn(tuple(d["k"].shape), generator=gen, dtype=torch.float32)
    return -torch.nn.functional.softplus(x) * scale


def device_randn(shape, dtype, seed, device="cuda", std=1.0):
    """A large N(0, std^2) tensor drawn on `device`, one leading index at a time (bounded temporaries), each slice
    from its own seed.  For the tests whose tensors exceed 2^31 elements: the values are compared with the oracle on
    slices copied back to the host, so only reproducibility on one device matters."""
    out = torch.empty(shape, dtype=dtype, device=device)
    gen = torch.Generator(device=device)
    for i in range(shape[0]):
        gen.manual_seed(seed * 100_003 + i)
        out[i] = (torch.randn(shape[1:], generator=gen, dtype=torch.float32, device=device) * std).to(dtype)
    return out


def device_gates(shape, seed, device="cuda"):
    """log_alpha = -softplus(x), eta = sigmoid(x), x ~ N(0,1), drawn on `device` (see device_randn)."""
    xa = device_randn(shape, torch.float32, seed, device)
    xe = device_randn(shape, torch.float32, seed + 1, device)
    return -torch.nn.functional.softplus(xa), torch.sigmoid(xe)
