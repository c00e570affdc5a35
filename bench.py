"""Benchmark of the PSA forward hot path on one MI355X.

One step = psa_build_pyramid + psa_allocate_levels + psa_attention_fwd over one synthetic batch that
is already resident in HBM.  Prints ONE JSON line: whole-path dense-equivalent TFLOP/s (dense FLOPs of
the same attention problem divided by the PSA step time), ms per step, the roofline of the dominant
kernel (the MFMA attention kernel, on EXECUTED FLOPs), the HBM roofline of the pyramid pass, and the
CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="dit1p3b", help="key of synth_inputs.CONFIGS")
    ap.add_argument("--budget", type=float, default=None, help="compute budget rho-bar (default: the workload's)")
    ap.add_argument("--levels", type=int, default=None, help="pyramid depth override (1 = binary block-sparse)")
    ap.add_argument("--seq", type=int, default=None, help="sequence length override (shorter variant of the workload)")
    ap.add_argument("--heads", type=int, default=None, help="query-head count override (KV heads scale along)")
    ap.add_argument("--copy-probe-mb", type=int, default=0,
                    help="also run one plain device copy of this many MiB (calibrates rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--no-attainable", action="store_true", help="skip the copy / MFMA-only microbenchmarks")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--check-dense", action="store_true", help="also report rel-L2 of PSA vs dense attention")
    return ap.parse_args()


def dense_flops(w) -> float:
    if w.causal:
        return 2.0 * w.N * (w.N + 1) * w.d * w.B * w.Hq
    return 4.0 * float(w.N) ** 2 * w.d * w.B * w.Hq


def executed_flops(M: np.ndarray, w, levels: int) -> float:
    """Token-exact FLOPs of the attention kernel for level map M: 4 d sum rows_i * pooled tokens."""
    nq, nk = M.shape[2], M.shape[3]
    rows = np.minimum(w.bq, w.N - np.arange(nq) * w.bq).astype(np.float64)
    total = 0.0
    for h in range(1, levels + 1):
        span = 1 << (h - 1)
        th = w.bk >> (h - 1)
        first = (np.arange(nk * th) * span).reshape(nk, th)
        valid = (first < w.N).sum(axis=1).astype(np.float64)
        sel = (M == h)
        total += float(np.einsum("bhij,i,j->", sel.astype(np.float64), rows, valid))
    return 4.0 * w.d * total


def pyramid_bytes(w, levels: int) -> float:
    e = 2 if w.dtype == "bf16" else 4
    frac = 1.0 + sum(2.0 ** -(h - 1) for h in range(2, levels + 1))
    return 2.0 * w.B * w.Hkv * w.N * w.d * e * frac


def measured_traffic(w, budget, kernel_prefix: str):
    """HBM-side bytes per launch of a kernel from the committed rocprofv3 counter summary for this exact
    workload and budget (FETCH_SIZE / WRITE_SIZE scaled by the copy-kernel calibration); None otherwise."""
    path = os.path.join(ROOT, "profiles", f"psa_fwd_{w.name}_budget{budget}_traffic.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path))
    for name, v in rec["kernels"].items():
        if name.startswith(kernel_prefix):
            return v["read_bytes"] + v["write_bytes"]
    return None


def attainable_peaks(torch, psa):
    """What this GPU sustains on two trivial kernels of the library: a streaming copy (read + write
    bytes per second) and a loop of nothing but bf16 32x32x16 MFMAs on register operands, once with
    few-valued operands and once with random signs and mantissas (the clock follows the power the
    multipliers draw, so the second is the ceiling for real activations)."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    sink = torch.empty(2048 * 256, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    psa.psa_probe_copy(src, dst, n)
    e0.record()
    for _ in range(5):
        psa.psa_probe_copy(src, dst, n)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2.0 * n / (e0.elapsed_time(e1) * 1e-3) / 1e9
    rates = {}
    for random_operands in (False, True):
        for _ in range(3):     # long enough for the clock to settle
            psa.psa_probe_mfma(sink, 2048, 2000, random_operands)
        e0.record()
        flops = 0.0
        for _ in range(5):
            flops += psa.psa_probe_mfma(sink, 2048, 2000, random_operands)
        e1.record()
        torch.cuda.synchronize()
        rates[random_operands] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    return {"hbm_copy_gbs": copy_gbs, "mfma_bf16_tflops": rates[False], "mfma_bf16_tflops_random_operands": rates[True],
            "note": "measured on this GPU by psa_probe_copy (1 GiB) and psa_probe_mfma (2048 workgroups x 2000 x 16 MFMAs "
                    "per wavefront; few-valued operands, then random signs and mantissas)"}


def cpu_baseline(w, budget, Q, K, V, n_heads: int = 3):
    """The oracle as it stands on this host: pyramid, importance, allocation and attention (every query
    block) of the first `n_heads` heads, extrapolated to the whole workload."""
    import dataclasses

    import synth_inputs as si
    from oracle import psa_oracle as orc
    from tests.psa_testlib import oracle_params
    op = oracle_params(w, budget=budget)
    op1 = dataclasses.replace(op, B=1, Hq=1, Hkv=1)
    group = w.Hq // w.Hkv
    n_heads = min(n_heads, w.Hq)
    t_pyr = t_alloc = t_attn = 0.0
    for hq in range(n_heads):
        hk = hq // group
        Q1 = si.to_f64(Q[:1, hq:hq + 1], w.dtype)
        K1 = si.to_f64(K[:1, hk:hk + 1], w.dtype)
        V1 = si.to_f64(V[:1, hk:hk + 1], w.dtype)
        t0 = time.perf_counter()
        Kp, Vp = orc.build_pyramid(K1, op1), orc.build_pyramid(V1, op1)
        t1 = time.perf_counter()
        M = orc.allocate_levels(orc.importance(Q1, K1, op1), op1)
        t2 = time.perf_counter()
        orc.psa_attention(Q1, Kp, Vp, M, op1)
        t3 = time.perf_counter()
        t_pyr += t1 - t0
        t_alloc += t2 - t1
        t_attn += t3 - t2
    full = (t_pyr * w.Hkv + (t_alloc + t_attn) * w.Hq) * w.B / n_heads
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {
        "value": dense_flops(w) / full / 1e12, "unit": "TFLOP/s (dense-equivalent, extrapolated)",
        "cores": int(cores), "kind": "oracle",
        "sample": f"{n_heads} of {w.B * w.Hq} heads, every query block: pyramid {t_pyr:.2f}s, "
                  f"importance+allocation {t_alloc:.2f}s, attention {t_attn:.2f}s; "
                  f"extrapolated whole-workload time {full:.1f}s",
        "ms_per_step_extrapolated": full * 1e3,
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1).", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2512_04025_amd as psa
    import synth_inputs as si
    from paper_2512_04025_amd.plumbing import Buffers, from_dev, to_dev

    w = si.CONFIGS[args.workload]
    # the importance estimator of the workload (8 pooled representatives per block) stays the same when
    # the pyramid depth is overridden, so --levels 1 is block-sparse attention on the SAME scores
    sq, sk = 8, w.bk >> (w.levels - 1)
    if args.levels:
        w = w.with_(levels=args.levels)
    if args.seq or args.heads:
        hq = args.heads or w.Hq
        w = si.small_variant(w, args.seq or w.N, Hq=hq, Hkv=max(1, hq * w.Hkv // w.Hq))
    budget = args.budget if args.budget is not None else w.budget
    gp = psa.make_params(w.B, w.Hq, w.Hkv, w.N, w.d, w.bq, w.bk, w.levels,
                         dtype=psa.PSA_BF16 if w.dtype == "bf16" else psa.PSA_F32, causal=w.causal,
                         sq=sq, sk=sk, rep_mode=psa.PSA_REP_POOLED, est_pool=psa.PSA_EST_MAX,
                         alloc_mode=psa.PSA_ALLOC_BUDGET, budget=budget)
    torch.cuda.set_device(0)
    Q, K, V = si.generate_qkv(w)
    Qd, Kd, Vd = (to_dev(x, w.dtype) for x in (Q, K, V))
    buf = Buffers(gp)

    def step():
        psa.psa_build_pyramid(gp, Kd, Vd, buf.Kpyr, buf.Vpyr)
        psa.psa_allocate_levels(gp, Qd, Kd, buf.Kpyr, buf.M, buf.scratch, rho_out=buf.rho)
        psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.copy_probe_mb:
        src = torch.empty(args.copy_probe_mb << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        ev[k][0].record()
        psa.psa_build_pyramid(gp, Kd, Vd, buf.Kpyr, buf.Vpyr)
        ev[k][1].record()
        psa.psa_allocate_levels(gp, Qd, Kd, buf.Kpyr, buf.M, buf.scratch, rho_out=buf.rho)
        ev[k][2].record()
        psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch)
        ev[k][3].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / args.steps
    ms_pyr = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    ms_alloc = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))
    ms_attn = float(np.mean([e[2].elapsed_time(e[3]) for e in ev]))

    M = buf.M.cpu().numpy()
    rho = float(buf.rho.mean().item())
    coverage = float((M > 0).mean()) if not w.causal else None
    fl_exec = executed_flops(M, w, w.levels)
    fl_dense = dense_flops(w)
    attn_tflops = fl_exec / (ms_attn * 1e-3) / 1e12
    pyr_gbs = pyramid_bytes(w, w.levels) / (ms_pyr * 1e-3) / 1e9 if w.levels > 1 else None

    out = {
        "metric": "psa_fwd_dense_equivalent_tflops", "value": fl_dense / (ms_step * 1e-3) / 1e12,
        "unit": "TFLOP/s (dense-equivalent: dense attention FLOPs / PSA forward time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} N={w.N} d={w.d} bq={w.bq} bk={w.bk} "
                               f"levels={w.levels} causal={int(w.causal)} budget={budget}",
                   "alloc_mode": "budget", "rep_mode": "pooled", "est_pool": "max"},
        "phases_ms": {"build_pyramid": ms_pyr, "allocate_levels": ms_alloc, "attention_fwd": ms_attn},
        "achieved_rho": rho, "kv_coverage": coverage,
        "executed_tflop": fl_exec / 1e12, "dense_tflop": fl_dense / 1e12,
        "roofline": {"kernel": "attn_mfma_kernel", "bound": "mfma", "achieved": attn_tflops, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": attn_tflops / PEAK_BF16_TFLOPS,
                     "traffic": measured_traffic(w, budget, "psa::attn_mfma_kernel"),
                     "note": "executed FLOPs / mean HIP-event time of psa_attention_fwd (includes its block-list and tile-descriptor kernels)"},
        "roofline_pyramid": None if pyr_gbs is None else {
            "kernel": "pyramid_kernel", "bound": "hbm", "achieved": pyr_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": pyr_gbs / PEAK_HBM_GBS, "traffic": measured_traffic(w, budget, "psa::pyramid_kernel"),
            "algorithmic_bytes": pyramid_bytes(w, w.levels)},
    }
    if not args.no_attainable:
        att = attainable_peaks(torch, psa)
        out["attainable"] = att
        out["roofline"]["frac_of_attainable"] = attn_tflops / att["mfma_bf16_tflops"]
        out["roofline"]["frac_of_attainable_random_operands"] = attn_tflops / att["mfma_bf16_tflops_random_operands"]
        if pyr_gbs is not None:
            out["roofline_pyramid"]["frac_of_attainable"] = pyr_gbs / att["hbm_copy_gbs"]
    if w.dtype != "bf16":
        out["roofline"]["note"] += "; fp32 mode runs on the VALU (correctness mode), bf16 MFMA peak shown for scale only"
    if args.check_dense:
        dense = torch.empty_like(buf.O)
        psa.psa_dense_ref(gp, Qd, Kd, Vd, dense)
        torch.cuda.synchronize()
        a, b = from_dev(buf.O, w.dtype), from_dev(dense, w.dtype)
        out["rel_l2_vs_dense"] = float(np.linalg.norm(a - b) / np.linalg.norm(b))
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, budget, Q, K, V)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
