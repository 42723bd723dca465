#!/usr/bin/env python3
"""Benchmark of the KLA hot path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W

A "step" is one kla_chunk_fwd call (everything from the key norms to the outputs and the final state) on the
0.4B-scale training shape: N=8, H=8, T=4096, d_k=d_v=128, chunk 64, bf16 q/k/v, fp32 gates and state, inputs
resident in HBM.  The same JSON line also carries: the roofline of the dominant kernel (its launches timed one group
at a time with events, median of the groups), the matrix-pipe fraction, what this GPU delivers for plain streaming
and for back-to-back MFMA (measured in the same run, as second denominators beside the published peaks), the two
other chunk workloads (configs 3 and 5) with their own roofline figures, the backward pass, the diagonal-gating
variant, the decode step on the 32K-context decode shape (B=64, H=8, d=128, 256 consecutive steps) with the
in-place-streaming ceiling of the same launch shape, and the CPU oracle timed on the host cores.
Synthetic seeded inputs (kla_inputs.py).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
C = 64


def chunk_bytes_per_token_head(dk, dv):
    """q, k, v read and o written in bf16, two fp32 gates."""
    return 2 * (2 * dk + 2 * dv) + 8


def chunk_flop_per_token_head(dk, dv, dense=False):
    """Algorithmic flops of eqs. (6)-(8) per token and head: the three d_k x d_v products (K S, Q S, the state update)
    and the five chunk-local products (K K^T, the solve, Q K^T, P U), triangular ones at half cost unless `dense`
    (what a tiled kernel issues if it does not skip the masked tiles)."""
    return 6 * dk * dv + C * ((6 if dense else 3) * dk + (4 if dense else 2) * dv)


DECODE_BYTES_PER_TOKEN_HEAD = 2 * 4 * 128 * 128 + 2 * (2 * 128 + 128) + 8 + 2 * 128   # state r+w, q,k,v, gates, o


def _warm(torch, fn, ms=50.0):
    """Untimed: keeps the GPU busy with fn() for about `ms` milliseconds.  After an idle spell the first ~25 ms of work
    run 10-20 % slower (clocks ramp up), so every timed region below starts from a busy GPU, as a training or serving
    loop would."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ms:
        for _ in range(4):
            fn()
        torch.cuda.synchronize()


MAX_GROUPS = 1 << 30   # --max-groups: a counter run needs only a few launches of each kernel


def _events(torch, fn, reps, warm_ms=50.0, groups=1):
    """Milliseconds per fn() by events on the current stream (the stream the binding launches on), after an untimed
    warm-up: `groups` groups of `reps` launches, each group between its own pair of events; returns the median group."""
    _warm(torch, fn, warm_ms)
    groups = max(1, min(groups, MAX_GROUPS))
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(groups)]
    torch.cuda.synchronize()
    for e0, e1 in ev:
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
    torch.cuda.synchronize()
    return statistics.median(e0.elapsed_time(e1) / reps for e0, e1 in ev)


def _traffic(key):
    """Memory-side bytes per launch (read + written past L2) from the committed rocprofv3 --pmc summary
    (profiles/hbm_traffic_per_launch.txt), or None.  Not measured in this run."""
    p = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
    try:
        for line in open(p):
            f = line.split()
            if len(f) >= 2 and f[0] == key:
                return int(f[1])
    except OSError:
        pass
    return None


def _clocks():
    """Shader and memory clock as rocm-smi shows them (MHz), or None where the tool is not allowed."""
    try:
        out = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=20).stdout
        got = {}
        for name in ("sclk", "mclk"):
            m = re.search(r"%s clock level:?\s*\d+:?\s*\((\d+)Mhz\)" % name, out)
            if m:
                got[name + "_MHz"] = int(m.group(1))
        return got or None
    except Exception:  # noqa: BLE001
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--skip-decode", action="store_true")
    ap.add_argument("--skip-rotating", action="store_true",
                    help="skip the config-2 step on three rotating copies of its tensors")
    ap.add_argument("--skip-extra", action="store_true",
                    help="skip everything but the headline step and its roofline (so that a kernel trace or a counter run "
                         "of this command holds the benchmarked launches only)")
    ap.add_argument("--sections", default="all",
                    help="comma-separated secondary measurements to run beside the headline step: two_kernel, rotating, "
                         "peaks, fp32, config3, config5, backward, backward_config3, diag, decode (default: all)")
    ap.add_argument("--max-groups", type=int, default=0,
                    help="cap on the event groups per measurement (for rocprofv3 --pmc runs, which serialise every dispatch)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run a plain device copy of 1 GiB five times (reference for the rocprofv3 byte counters)")
    args = ap.parse_args()
    sections = set(args.sections.split(","))

    def want(name):
        if args.skip_extra or (name == "decode" and args.skip_decode) or (name == "rotating" and args.skip_rotating):
            return False
        return "all" in sections or name in sections

    if args.max_groups > 0:
        global MAX_GROUPS
        MAX_GROUPS = args.max_groups
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by design (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import kla_inputs
    import paper_2605_08587_amd as kla

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    kla.lib()   # fails loudly if the HIP library is not built

    if args.copy_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": 1 << 30, "copy_probe_bytes_written": 1 << 30, "launches": 5}))
        return

    clocks_start = _clocks()

    # ------------------------------------------------------------------ chunk forward, config 2
    d = kla_inputs.config(2)
    N, T, H, dk, dv = d["N"], d["T"], d["H"], d["dk"], d["dv"]
    dev = {n: d[n].cuda() for n in ("q", "k", "v", "log_alpha", "eta")}
    unfused = kla.tune(unfused=True)
    # the default call runs the fused kernel and uses no workspace; the two-kernel form (timed beside it) does
    ws = torch.empty(kla.kla_chunk_fwd_workspace_bytes(N, T, H, dk, dv, torch.bfloat16, tune=unfused), dtype=torch.uint8, device="cuda")
    out = torch.empty((N, T, H, dv), dtype=torch.bfloat16, device="cuda")
    hT = torch.empty((N, H, dk, dv), dtype=torch.float32, device="cuda")

    def step():
        kla.kla_chunk_fwd(dev["q"], dev["k"], dev["v"], dev["log_alpha"], dev["eta"], d["eps"], workspace=ws, out=out, hT=hT)

    def step_two_kernels():
        kla.kla_chunk_fwd(dev["q"], dev["k"], dev["v"], dev["log_alpha"], dev["eta"], d["eps"], workspace=ws, out=out, hT=hT,
                          tune=unfused)

    def stage(i):
        kla.kla_debug_chunk_stage(i, dev["q"], dev["k"], dev["v"], dev["log_alpha"], dev["eta"], d["eps"], ws, out, hT=hT)

    _warm(torch, step)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    tokens = N * T
    token_heads = N * T * H
    value = tokens / (ms_per_step * 1e-3)

    # The step is ONE kernel (the fused scan): its launches timed by events on the launch stream, 20 groups of 10
    ms_kernel = _events(torch, step, 10, groups=20)
    alg_bytes = chunk_bytes_per_token_head(dk, dv) * token_heads
    achieved = alg_bytes / (ms_kernel * 1e-3) / 1e9
    fused_ran = kla.kla_chunk_fwd_workspace_bytes(N, T, H, dk, dv, torch.bfloat16) == 256
    roofline = {"bound": "hbm", "kernel": "scan_bf16_kernel<128, 2, fused>" if fused_ran else "scan_bf16_kernel",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": _traffic("chunk_fused_scan_bf16_kernel_config2"),
                "traffic_source": "profiles/hbm_traffic_per_launch.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run "
                                  "of this command; not measured in this run)",
                "algorithmic_bytes_per_launch": alg_bytes, "ms_per_launch": round(ms_kernel, 4),
                "timing": "events on the launch stream, median of 20 groups of 10 launches"}
    f_alg = chunk_flop_per_token_head(dk, dv) * token_heads
    f_dense = chunk_flop_per_token_head(dk, dv, dense=True) * token_heads
    tflops = f_alg / (ms_per_step * 1e-3) / 1e12
    mfma = {"achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4), "flop_per_token_head": chunk_flop_per_token_head(dk, dv),
            "frac_on_dense_tiles": round(f_dense / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "flop_per_token_head_dense_tiles": chunk_flop_per_token_head(dk, dv, dense=True),
            "whole_path_hbm_frac": round(alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "ms_per_chunk_step": round(ms_kernel / (T // C + 2), 6)}

    # The same step as two kernels (intra-chunk stage, then scan), the form that runs for fp32, wide value heads and
    # segmented scans
    two = None
    rotating = None
    if want("two_kernel"):
        ms_two = _events(torch, step_two_kernels, 10, groups=20)
        ms_intra = _events(torch, lambda: stage(1), 10, groups=20)
        ms_scan = _events(torch, lambda: stage(2), 10, groups=20)
        two = {"ms_per_step": round(ms_two, 4), "ms_intra_kernel": round(ms_intra, 4), "ms_scan_kernel": round(ms_scan, 4),
               "traffic": (_traffic("chunk_intra_bf16_kernel_config2") or 0) + (_traffic("chunk_scan_bf16_kernel_config2") or 0) or None,
               "note": "kla_chunk_fwd with KLA_TUNE_UNFUSED on the same tensors"}
    # The same step over three copies of the inputs and outputs in turn (1 GB in all): nothing of a step's tensors is
    # still in the 256 MB memory-side cache when the step comes round again.
    if want("rotating"):
        rot = [{n: t.clone() for n, t in dev.items()} for _ in range(3)]
        rot_out = [torch.empty_like(out) for _ in range(3)]
        rot_i = [0]

        def step_rot():
            i = rot_i[0] = (rot_i[0] + 1) % 3
            g = rot[i]
            kla.kla_chunk_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["eta"], d["eps"], workspace=ws, out=rot_out[i], hT=hT)
        for _ in range(6):
            step_rot()
        ms_rot = _events(torch, step_rot, 12, groups=20)
        rotating = {"sets": 3, "ms_per_step": round(ms_rot, 4), "tokens_per_s": round(tokens / (ms_rot * 1e-3), 1),
                    "note": "same step cycling over three copies of the inputs and outputs, so no tensor of a step is left "
                            "in the memory-side cache from its previous turn"}
        del rot, rot_out

    # ------------------------------------------------------------------ what this GPU delivers (second denominators)
    measured = None
    if want("peaks"):
        big = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1e-30)     # 1 GiB
        aux = torch.empty(max(big.numel() * 4 // 16384, 256 * 2048), dtype=torch.float32, device="cuda")
        ms_rw = _events(torch, lambda: kla.kla_debug_peak_probe(0, big, aux, iters=1), 5, groups=5)
        ms_ro = _events(torch, lambda: kla.kla_debug_peak_probe(1, big, aux), 5, groups=5)
        n_wg, iters = 2048, 4096
        ms_mm = _events(torch, lambda: kla.kla_debug_peak_probe(2, None, aux, n=n_wg, iters=iters), 3, groups=5)
        measured = {"stream_read_GBps": round(big.numel() * 4 / (ms_ro * 1e-3) / 1e9, 1),
                    "stream_inplace_GBps": round(2 * big.numel() * 4 / (ms_rw * 1e-3) / 1e9, 1),
                    "mfma_bf16_TFLOPs": round(n_wg * 4 * iters * 8 * 16384 / (ms_mm * 1e-3) / 1e12, 1),
                    "note": "kla_debug_peak_probe: 1 GiB read once; 1 GiB read and written in place (non-temporal); "
                            "2048 workgroups of back-to-back 16x16x32 bf16 MFMA from registers"}
        # the copy wave of the chunk kernels alone: 256 workgroups x 64 steps of n KiB per step (one LDS-DMA copy per KiB)
        ring = {}
        for n_kib, depth in ((16, 2), (32, 2), (48, 2), (60, 2), (16, 1), (32, 1), (48, 1), (60, 1)):
            ms_rc = _events(torch, lambda: kla.kla_debug_peak_probe(3, big, None, iters=n_kib + 256 * (depth - 1)), 5, groups=5)
            ring["%dKiB_depth%d" % (n_kib, depth)] = round(ms_rc * 1e3 / 64, 3)
        measured["ring_copy_us_per_step"] = ring
        measured["ring_copy_note"] = ("kla_debug_peak_probe kind 3: one workgroup per CU, one wave issuing n LDS-DMA copies of 1 KiB "
                                      "per step (256-byte rows 2 KiB apart, shared by the four workgroups of a head) through a ring "
                                      "one or two steps deep, a barrier per step; us per step")
        roofline["frac_of_measured_stream_read"] = round(achieved / measured["stream_read_GBps"], 4)
        mfma["frac_of_measured_mfma"] = round(tflops / measured["mfma_bf16_TFLOPs"], 4)
        del big, aux

    # ------------------------------------------------------------------ fp32 inputs: the element-type-generic kernels
    fp32_path = None
    if want("fp32"):
        fp32_path = {"note": "fp32 q/k/v run the element-type-generic kernels (two-kernel form, fp32 MFMA and vector sums): "
                             "the path that carries the 1e-4 parity bar, not tuned for speed"}
        for name, cfg, shape in (("config1", kla_inputs.config(1), None), ("config2_shape", d, "fp32 copies of config 2's tensors")):
            f = {n: cfg[n].float().cuda() for n in ("q", "k", "v")}
            g = {n: cfg[n].cuda() for n in ("log_alpha", "eta")}
            n1, t1, h1, k1, v1 = cfg["N"], cfg["T"], cfg["H"], cfg["dk"], cfg["dv"]
            w32 = torch.empty(kla.kla_chunk_fwd_workspace_bytes(n1, t1, h1, k1, v1, torch.float32), dtype=torch.uint8, device="cuda")
            o32 = torch.empty((n1, t1, h1, v1), dtype=torch.float32, device="cuda")
            h32 = torch.empty((n1, h1, k1, v1), dtype=torch.float32, device="cuda")
            fn32 = lambda: kla.kla_chunk_fwd(f["q"], f["k"], f["v"], g["log_alpha"], g["eta"], cfg["eps"], workspace=w32, out=o32, hT=h32)
            ms32 = _events(torch, fn32, 5, groups=10)
            fp32_path[name] = {"ms_per_call": round(ms32, 4), "tokens_per_s": round(n1 * t1 / (ms32 * 1e-3), 1),
                               "workload": shape or "N=%d,H=%d,T=%d,dk=%d,dv=%d" % (n1, h1, t1, k1, v1)}
            del f, w32, o32, h32

    # ------------------------------------------------------------------ secondary chunk workloads (not the headline)
    extra = None
    if want("config3") or want("config5"):
        extra = {}
        for ci, name, chain in ((3, "config3: N=1,H=8,T=65536,d=128 (one long sequence; segment-parallel scan)", None),
                                (5, "config5: 16 packed sequences of 512..4096 tokens,H=16,dk=128,dv=256,h0", None)):
            if not want("config%d" % ci):
                continue
            e = kla_inputs.config(ci)
            g = {n: e[n].cuda() for n in ("q", "k", "v", "log_alpha", "eta")}
            cu = None if e["cu_seqlens"] is None else e["cu_seqlens"].cuda()
            h0 = None if e["h0"] is None else e["h0"].cuda()
            n_states = e["N"] if cu is None else cu.numel() - 1
            w2 = torch.empty(kla.kla_chunk_fwd_workspace_bytes(e["N"], e["T"], e["H"], e["dk"], e["dv"], torch.bfloat16,
                                                               cu_seqlens=cu), dtype=torch.uint8, device="cuda")
            o2 = torch.empty((e["N"], e["T"], e["H"], e["dv"]), dtype=torch.bfloat16, device="cuda")
            h2 = torch.empty((n_states, e["H"], e["dk"], e["dv"]), dtype=torch.float32, device="cuda")
            fn = lambda: kla.kla_chunk_fwd(g["q"], g["k"], g["v"], g["log_alpha"], g["eta"], e["eps"], h0=h0,
                                           cu_seqlens=cu, cu_seqlens_host=e["cu_seqlens"], workspace=w2, out=o2, hT=h2)
            for _ in range(3):
                fn()
            ms = _events(torch, fn, 5, groups=20)
            th = e["N"] * e["T"] * e["H"]
            ab = chunk_bytes_per_token_head(e["dk"], e["dv"]) * th
            fl = chunk_flop_per_token_head(e["dk"], e["dv"]) * th
            if cu is None:
                longest = e["T"]
            else:
                longest = int((e["cu_seqlens"][1:] - e["cu_seqlens"][:-1]).max())
            extra["config%d" % ci] = {
                "workload": name, "ms_per_call": round(ms, 4), "tokens_per_s": round(e["N"] * e["T"] / (ms * 1e-3), 1),
                "algorithmic_bytes": ab, "hbm_frac": round(ab / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                "algorithmic_flop": fl, "mfma_frac": round(fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                "chunks_of_longest_sequence": (longest + C - 1) // C,
                "us_per_chunk_of_longest_sequence": round(ms * 1e3 / ((longest + C - 1) // C), 4),
                "workspace_MB": round(w2.numel() / 1e6, 1)}
            del g, w2, o2, h2

    # ------------------------------------------------------------------ backward of the chunk path, config 2 (secondary)
    backward = None
    if want("backward"):
        d_o, d_hT = kla_inputs.grad_inputs(d, 1)
        d_o, d_hT = d_o.cuda(), d_hT.cuda()
        wb = torch.empty(kla.kla_chunk_bwd_workspace_bytes(N, T, H, dk, dv, torch.bfloat16), dtype=torch.uint8, device="cuda")
        grads = kla.kla_chunk_bwd(dev["q"], dev["k"], dev["v"], dev["log_alpha"], dev["eta"], d["eps"], d_o, d_hT=d_hT,
                                  workspace=wb)
        fnb = lambda: kla.kla_chunk_bwd(dev["q"], dev["k"], dev["v"], dev["log_alpha"], dev["eta"], d["eps"], d_o,
                                        d_hT=d_hT, workspace=wb, out=grads)
        for _ in range(3):
            fnb()
        msb = _events(torch, fnb, 5, groups=10)
        backward = {"workload": "config2, gradients of q,k,v,log_alpha,eta,h0 (forward quantities recomputed)",
                    "ms_per_call": round(msb, 4), "tokens_per_s": round(tokens / (msb * 1e-3), 1),
                    "times_forward": round(msb / ms_per_step, 2), "workspace_MB": round(wb.numel() / 1e6, 1),
                    "traffic": _traffic("chunk_bwd_config2")}
        del wb, grads, d_o, d_hT
    if backward is not None and want("backward_config3"):
        # the same on config 3 (one 65K-token sequence): segment-parallel sweeps
        e3 = kla_inputs.config(3)
        g3 = {n: e3[n].cuda() for n in ("q", "k", "v", "log_alpha", "eta")}
        do3, dh3 = kla_inputs.grad_inputs(e3, 2)
        do3, dh3 = do3.cuda(), dh3.cuda()
        w3 = torch.empty(kla.kla_chunk_bwd_workspace_bytes(e3["N"], e3["T"], e3["H"], e3["dk"], e3["dv"], torch.bfloat16),
                         dtype=torch.uint8, device="cuda")
        gr3 = kla.kla_chunk_bwd(g3["q"], g3["k"], g3["v"], g3["log_alpha"], g3["eta"], e3["eps"], do3, d_hT=dh3, workspace=w3)
        fn3 = lambda: kla.kla_chunk_bwd(g3["q"], g3["k"], g3["v"], g3["log_alpha"], g3["eta"], e3["eps"], do3, d_hT=dh3,
                                        workspace=w3, out=gr3)
        for _ in range(2):
            fn3()
        ms3 = _events(torch, fn3, 3, groups=5)
        backward["config3"] = {"workload": "config3 (N=1,H=8,T=65536): segment-parallel sweeps", "ms_per_call": round(ms3, 4),
                               "tokens_per_s": round(e3["N"] * e3["T"] / (ms3 * 1e-3), 1)}
        del w3, gr3, do3, dh3, g3

    # ------------------------------------------------------------------ diagonal gating on config 2's tensors (secondary)
    diag = None
    if want("diag"):
        lad = kla_inputs.diag_gates(d, 1).cuda()
        wd = torch.empty(int(kla.lib().kla_chunk_fwd_diag_workspace_bytes(N, T, H, dk, dv, 64, kla.KLA_BF16, None, 0)),
                         dtype=torch.uint8, device="cuda")
        fnd = lambda: kla.kla_chunk_fwd_diag(dev["q"], dev["k"], dev["v"], lad, dev["eta"], d["eps"], workspace=wd, out=out, hT=hT)
        for _ in range(3):
            fnd()
        msd = _events(torch, fnd, 5, groups=10)
        diag = {"workload": "config2 tensors with per-channel decay gates log_alpha [N,T,H,dk] (kla_chunk_fwd_diag)",
                "ms_per_call": round(msd, 4), "tokens_per_s": round(tokens / (msd * 1e-3), 1),
                "times_scalar_gate_forward": round(msd / ms_per_step, 2), "traffic": _traffic("chunk_diag_config2")}
        del wd, lad

    # ------------------------------------------------------------------ decode, config 4
    decode = None
    if want("decode"):
        dd = kla_inputs.config(4)
        B, Hd, steps = dd["B"], dd["H"], dd["steps"]
        g = {n: dd[n].cuda() for n in ("q", "k", "v", "log_alpha", "eta")}
        S0 = dd["S"].cuda()
        od = torch.empty((B, Hd, dd["dv"]), dtype=torch.bfloat16, device="cuda")

        def run256(states):
            ns = len(states)
            for t in range(steps):
                kla.kla_decode_step(g["q"][t], g["k"][t], g["v"][t], g["log_alpha"][t], g["eta"][t], dd["eps"],
                                    states[t % ns], out=od)

        def graph_of(fn):
            """fn() captured once and replayed as one graph launch: no per-step launch cost on the host."""
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                fn()
            torch.cuda.current_stream().wait_stream(side)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                fn()
            graph.replay()
            return graph

        S = S0.clone()
        run256([S])
        ms256 = _events(torch, lambda: run256([S]), 3, groups=3)
        # 24 state sets take turns, as the 24 layers of the paper's 0.4B model (App. C) would: 805 MB, so a
        # set is never found in the 256 MB Infinity Cache when its turn comes again
        many = [S0.clone() for _ in range(24)]
        run256(many)
        ms256_cold = _events(torch, lambda: run256(many), 3, groups=3)
        bytes256 = DECODE_BYTES_PER_TOKEN_HEAD * B * Hd * steps
        # Back-to-back eager launches are bound by the host's launch path (about 13 us per call through the
        # Python binding), so the kernel's own rate is taken from graph replays; the eager figures stay beside it.
        try:
            gs = S0.clone()
            ms_graph = _events(torch, graph_of(lambda: run256([gs])).replay, 2, groups=20)
            ms_graph_cold = _events(torch, graph_of(lambda: run256(many)).replay, 2, groups=20)
            # the ceiling of this launch shape on this GPU: the same graph with every step replaced by a plain in-place
            # x <- 2 x over the same state set (same bytes read and written, same workgroups, none of the arithmetic)
            def probe256():
                for t in range(steps):
                    kla.kla_debug_peak_probe(0, many[t % 24], iters=1)
            ms_probe = _events(torch, graph_of(probe256).replay, 2, groups=20)
            graph_error = None
        except Exception as e:  # noqa: BLE001
            ms_graph, ms_graph_cold, ms_probe, graph_error = ms256, ms256_cold, None, str(e)[:120]
        gbs = bytes256 / (ms_graph_cold * 1e-3) / 1e9
        decode = {"metric": "decode_tokens_per_s", "workload": "config4: B=64,H=8,dk=dv=128,bf16 q/k/v,fp32 state,256 steps",
                  "value": round(B * steps / (ms_graph * 1e-3), 1), "unit": "tokens/s",
                  "us_per_step": round(ms_graph * 1e3 / steps, 3),
                  "launch": "one graph of 256 steps, state updated in place; median of 20 groups of 2 replays",
                  "eager_tokens_per_s": round(B * steps / (ms256 * 1e-3), 1),
                  "eager_us_per_step": round(ms256 * 1e3 / steps, 3),
                  "roofline": {"bound": "hbm", "kernel": "decode_kernel", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                               "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                               "traffic": _traffic("decode_kernel_config4"),
                               "traffic_source": "profiles/hbm_traffic_per_launch.txt; not measured in this run",
                               "note": "one graph of 256 steps rotating over 24 state sets (805 MB, one per layer of the "
                                       "0.4B model): a set is never resident in the Infinity Cache when its turn comes",
                               "us_per_step": round(ms_graph_cold * 1e3 / steps, 3),
                               "eager_us_per_step": round(ms256_cold * 1e3 / steps, 3)},
                  "same_state_GBps": round(bytes256 / (ms_graph * 1e-3) / 1e9, 1)}
        if ms_probe:
            us_probe = ms_probe * 1e3 / steps
            pb = 2 * S0.numel() * 4
            decode["roofline"]["inplace_stream_ceiling"] = {
                "us_per_launch": round(us_probe, 3), "GBps": round(pb / us_probe / 1e3, 1),
                "frac_of_peak": round(pb / us_probe / 1e3 / HBM_PEAK_GBS, 4),
                "decode_frac_of_ceiling": round(us_probe / (ms_graph_cold * 1e3 / steps), 4),
                "note": "x <- 2 x in place over the same 33.5 MB state sets, same graph of 256 launches, same workgroup shape, "
                        "non-temporal accesses: what this GPU delivers for the step's traffic without its arithmetic"}
        if graph_error:
            decode["graph_error"] = graph_error
        else:
            # the same steps with per-channel decay gates (kla_decode_step_diag), rotating over the 24 state sets
            gen = torch.Generator().manual_seed(4)
            lad = (-torch.nn.functional.softplus(torch.randn((steps, B, Hd, dd["dk"]), generator=gen))).cuda()

            def run256_diag():
                for t in range(steps):
                    kla.kla_decode_step_diag(g["q"][t], g["k"][t], g["v"][t], lad[t], g["eta"][t], dd["eps"], many[t % 24], out=od)

            ms_diag = _events(torch, graph_of(run256_diag).replay, 2, groups=5)
            decode["diagonal_gating_us_per_step"] = round(ms_diag * 1e3 / steps, 3)
            del lad

    # ------------------------------------------------------------------ CPU oracle beside it
    cpu = None
    parity = None
    if not args.skip_cpu_baseline:
        from oracle import token_oracle
        qn, kn, vn = (kla_inputs.to_numpy_f32(d[x]) for x in "qkv")
        la, et = d["log_alpha"].numpy(), d["eta"].numpy()
        # the whole of config 2, three times over (about 25 s of CPU work on 16 threads); the rate is that of the best pass
        dt = float("inf")
        for _ in range(3):
            t0 = time.perf_counter()
            ro, rh, nthr = token_oracle.kla_recurrent(qn, kn, vn, la, et, d["eps"])
            dt = min(dt, time.perf_counter() - t0)
        # one thread on a 1/8 slice: the first sequence of the batch (8 of the 64 sequence-heads)
        t0 = time.perf_counter()
        token_oracle.kla_recurrent(qn[:1], kn[:1], vn[:1], la[:1], et[:1], d["eps"], threads=1)
        dt1 = time.perf_counter() - t0
        cpu = {"value": round(tokens / dt, 1), "unit": "tokens/s", "cores": nthr, "kind": "oracle",
               "sample": "all of config 2 (64 sequence-heads x 4096 tokens), fp64 token loop, best of 3 passes, %.1f s wall each" % dt,
               "single_thread": {"value": round(T / dt1, 1), "unit": "tokens/s (of 8 heads)", "cores": 1,
                                 "sample": "1/8 slice: the first sequence (8 sequence-heads x 4096 tokens), %.1f s wall" % dt1}}
        step()
        torch.cuda.synchronize()
        parity = {"o": float("%.3e" % token_oracle.rel_err(out.float().cpu().numpy(), ro)),
                  "hT": float("%.3e" % token_oracle.rel_err(hT.cpu().numpy(), rh)), "bar": 2e-2}

    line = {"metric": "chunk_fwd_tokens_per_s", "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "config2: N=8,H=8,T=4096,dk=dv=128,chunk=64,bf16 q/k/v,fp32 gates+state",
                       "global_batch": N, "seq_len": T, "heads": H},
            "roofline": roofline, "mfma": mfma, "measured_peaks": measured, "two_kernel_form": two, "fp32_path": fp32_path, "rotating_inputs": rotating,
            "other_chunk_workloads": extra, "backward": backward, "diagonal_gating": diag, "decode": decode,
            "cpu_baseline": cpu, "parity": parity, "clocks": {"start": clocks_start, "end": _clocks()}}
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
