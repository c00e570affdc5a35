"""Benchmark of the PSA forward hot path on one MI355X.

One step = psa_build_pyramid + psa_allocate_levels + psa_attention_fwd over one synthetic batch that
is already resident in HBM.  Prints ONE JSON line: whole-path dense-equivalent TFLOP/s (dense FLOPs of
the same attention problem divided by the PSA step time), ms per step, the roofline of the dominant
kernel (the MFMA attention kernel, on EXECUTED FLOPs), the HBM rooflines of the pyramid pass and of
the whole pre-pass (pyramid + importance + allocation), the error against dense attention, a parity
check of the timed configuration against the CPU oracle (outside the timed region), a second point
with the threshold rule of Alg. 2, and the CPU oracle timed on a bounded sample of the same workload.
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
    ap.add_argument("--bq", type=int, default=None, help="query block size override (block-size ablation, App. C)")
    ap.add_argument("--bk", type=int, default=None, help="key block size override (a power of two)")
    ap.add_argument("--copy-probe-mb", type=int, default=0,
                    help="also run one plain device copy of this many MiB (calibrates rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--no-attainable", action="store_true", help="skip the copy / MFMA-only microbenchmarks")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check-dense", action="store_true", help="skip rel-L2 of PSA vs dense attention")
    ap.add_argument("--no-parity", action="store_true", help="skip the oracle check of sampled query blocks")
    ap.add_argument("--hilbert", action="store_true",
                    help="reorder Q, K, V along the Hilbert curve of the workload's token grid before the path and "
                         "restore the order of O after it (Sec. 3.3.1); the four row permutations are timed as "
                         "part of the step")
    ap.add_argument("--sim-cap", action="store_true",
                    help="build the cosine-similarity level cap of App. B.1 in the pyramid pass (psa_build_pyramid_cap, "
                         "thresholds 0.70, 0.65, 0.60 as printed for video generation) and feed it to the allocation")
    ap.add_argument("--backward", action="store_true",
                    help="also time psa_attention_bwd on the run's level map (outside the forward's timed region)")
    ap.add_argument("--no-threshold-point", action="store_true",
                    help="skip the second point with Alg. 2's threshold rule (tau = 0.5, 0.7, 0.8, 0.9)")
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


def prepass_bytes(w, levels: int, nq: int, nk: int) -> float:
    """Algorithmic HBM bytes of pyramid + importance + allocation: K and V read once and the pooled
    levels written once; Q read once (its 8 pooled representatives per block are formed on the fly);
    the level-H keys read once per head as representative keys; S written and read once (fp32) and M
    written once (uint8)."""
    e = 2 if w.dtype == "bf16" else 4
    q_bytes = float(w.B) * w.Hq * w.N * w.d * e
    krep_bytes = float(w.B) * w.Hkv * nk * (w.bk >> (levels - 1)) * w.d * e if levels > 1 else 0.0
    sm_bytes = float(w.B) * w.Hq * nq * nk * (4 + 4 + 1)
    return pyramid_bytes(w, levels) + q_bytes + krep_bytes + sm_bytes


def measured_traffic(w, budget, kernel_prefix: str):
    """(bytes, source): HBM-side bytes per launch of a kernel from the committed rocprofv3 counter summary
    for this exact workload and budget (FETCH_SIZE / WRITE_SIZE scaled by the copy-kernel calibration).
    The counters cannot be read from inside this process, so the figure is the one of the committed
    profile, named in `source`; (None, None) when there is no profile for the workload."""
    rel = os.path.join("profiles", f"psa_fwd_{w.name}_budget{budget}_traffic.json")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    rec = json.load(open(path))
    for name, v in rec["kernels"].items():
        if name.startswith(kernel_prefix):
            return v["read_bytes"] + v["write_bytes"], rel
    return None, None


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


def parity_leg(w, gp, budget, Q, K, V, buf, torch):
    """A few query blocks of the LAST (batch, head) of the timed configuration against the oracle, under
    the level map the timed run itself produced: a timed run can never be a wrong run unnoticed."""
    import synth_inputs as si
    from oracle import psa_oracle as orc
    from paper_2512_04025_amd.plumbing import from_dev
    from tests.psa_testlib import oracle_params
    b, hq = w.B - 1, w.Hq - 1
    hk = hq // (w.Hq // w.Hkv)
    op1 = oracle_params(w, budget=budget, B=1, Hq=1, Hkv=1)
    Q1 = si.to_f64(Q[b:b + 1, hq:hq + 1], w.dtype)
    K1 = si.to_f64(K[b:b + 1, hk:hk + 1], w.dtype)
    V1 = si.to_f64(V[b:b + 1, hk:hk + 1], w.dtype)
    M1 = buf.M[b:b + 1, hq:hq + 1].cpu().numpy()
    qblocks = sorted({0, op1.nq // 2, op1.nq - 1})
    O1, _ = orc.psa_attention(Q1, orc.build_pyramid(K1, op1), orc.build_pyramid(V1, op1), M1, op1, q_blocks=qblocks)
    max_abs, num, den = 0.0, 0.0, 0.0
    for i in qblocks:
        rows = slice(i * w.bq, min((i + 1) * w.bq, w.N))
        got, ref = from_dev(buf.O[b, hq, rows], w.dtype), O1[0, 0][rows]
        max_abs = max(max_abs, float(np.abs(got - ref).max()))
        num += float(((got - ref) ** 2).sum())
        den += float((ref ** 2).sum())
    return {"parity_max_abs": max_abs, "parity_rel_l2": float(np.sqrt(num / den)),
            "parity_sample": f"batch {b} head {hq}, query blocks {qblocks} vs the CPU oracle under the run's own level map"}


def timed_phases(torch, fns, steps):
    """HIP events around each call of `fns` on the current stream, `steps` times; returns
    (wall ms per step, [mean ms per call], [median ms per call])."""
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(fns) + 1)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        ev[k][0].record()
        for c, fn in enumerate(fns):
            fn()
            ev[k][c + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per = np.array([[e[c].elapsed_time(e[c + 1]) for c in range(len(fns))] for e in ev])
    return (t1 - t0) * 1e3 / steps, per.mean(axis=0).tolist(), np.median(per, axis=0).tolist()


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
    if args.bq or args.bk:
        w = w.with_(bq=args.bq or w.bq, bk=args.bk or w.bk)
    sq, sk = 8, (w.bk >> (w.levels - 1) if not (args.bq or args.bk) else min(8, w.bk))
    if args.levels:
        w = w.with_(levels=args.levels)
    if args.seq or args.heads:
        hq = args.heads or w.Hq
        w = si.small_variant(w, args.seq or w.N, Hq=hq, Hkv=max(1, hq * w.Hkv // w.Hq))
    budget = args.budget if args.budget is not None else w.budget

    def params(**kw):
        base = dict(dtype=psa.PSA_BF16 if w.dtype == "bf16" else psa.PSA_F32, causal=w.causal, sq=sq, sk=sk,
                    rep_mode=psa.PSA_REP_POOLED, est_pool=psa.PSA_EST_MAX, alloc_mode=psa.PSA_ALLOC_BUDGET, budget=budget)
        base.update(kw)
        return psa.make_params(w.B, w.Hq, w.Hkv, w.N, w.d, w.bq, w.bk, w.levels, **base)

    gp = params()
    torch.cuda.set_device(0)
    Q, K, V = si.generate_qkv(w)
    Qd, Kd, Vd = (to_dev(x, w.dtype) for x in (Q, K, V))
    buf = Buffers(gp)

    # the two microbenchmarks run first: they also bring the clock to its sustained state
    att = None if args.no_attainable else attainable_peaks(torch, psa)

    hil = None
    if args.hilbert:
        T, Hg, W = w.grid
        if w.text_tokens or T * Hg * W != w.N:
            print("--hilbert needs a workload whose tokens are exactly its T x Hg x W grid", file=sys.stderr)
            sys.exit(2)
        perm_host = psa.psa_hilbert_order(T, Hg, W)
        hil = {"perm": torch.from_numpy(perm_host).cuda(), "raster": (Qd, Kd, Vd), "O": torch.empty_like(buf.O)}
        Qd, Kd, Vd = (torch.empty_like(x) for x in hil["raster"])    # the path works on the reordered copies

    def permute_in():
        for src, dst in zip(hil["raster"], (Qd, Kd, Vd)):
            psa.psa_permute_tokens(gp, src, hil["perm"], dst)

    cap = None
    if args.sim_cap and w.levels > 1:
        tau_s = ((0.70, 0.65, 0.60) + (0.60,) * 8)[:w.levels - 1]
        cap = {"tau_s": tau_s, "sim": torch.empty((w.B, w.Hkv, gp.nk, w.levels - 1), dtype=torch.float32, device="cuda"),
               "L": torch.empty((w.B, w.Hkv, gp.nk), dtype=torch.uint8, device="cuda")}

    def pyramid_call():
        if cap:
            psa.psa_build_pyramid_cap(gp, Kd, Vd, buf.Kpyr, buf.Vpyr, cap["tau_s"], cap["sim"], cap["L"])
        else:
            psa.psa_build_pyramid(gp, Kd, Vd, buf.Kpyr, buf.Vpyr)

    calls = [pyramid_call,
             lambda: psa.psa_allocate_levels(gp, Qd, Kd, buf.Kpyr, buf.M, buf.scratch, rho_out=buf.rho,
                                             level_cap=cap["L"] if cap else None),
             lambda: psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch)]
    if hil:
        calls = [permute_in] + calls + [lambda: psa.psa_permute_tokens(gp, buf.O, hil["perm"], hil["O"], inverse=True)]
    for _ in range(args.warmup):
        for fn in calls:
            fn()
    torch.cuda.synchronize()
    if args.copy_probe_mb:
        src = torch.empty(args.copy_probe_mb << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ms_step, mean_ms, median_ms = timed_phases(torch, calls, args.steps)
    ms_perm = None
    if hil:
        ms_perm = mean_ms[0] + mean_ms[-1]
        mean_ms, median_ms = mean_ms[1:-1], median_ms[1:-1]
    ms_pyr, ms_alloc, ms_attn = mean_ms

    M = buf.M.cpu().numpy()
    rho = float(buf.rho.mean().item())
    coverage = float((M > 0).mean()) if not w.causal else None
    fl_exec = executed_flops(M, w, w.levels)
    fl_dense = dense_flops(w)
    attn_tflops = fl_exec / (ms_attn * 1e-3) / 1e12
    pyr_gbs = pyramid_bytes(w, w.levels) / (ms_pyr * 1e-3) / 1e9 if w.levels > 1 else None
    pre_bytes = prepass_bytes(w, w.levels, gp.nq, gp.nk)
    pre_gbs = pre_bytes / ((ms_pyr + ms_alloc) * 1e-3) / 1e9
    attn_traffic, attn_src = measured_traffic(w, budget, "psa::attn_mfma_kernel")
    pyr_traffic, pyr_src = measured_traffic(w, budget, "psa::pyramid_kernel")

    out = {
        "metric": "psa_fwd_dense_equivalent_tflops", "value": fl_dense / (ms_step * 1e-3) / 1e12,
        "unit": "TFLOP/s (dense-equivalent: dense attention FLOPs / PSA forward time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: B={w.B} Hq={w.Hq} Hkv={w.Hkv} N={w.N} d={w.d} bq={w.bq} bk={w.bk} "
                               f"levels={w.levels} causal={int(w.causal)} budget={budget}",
                   "alloc_mode": "budget", "rep_mode": "pooled", "est_pool": "max"},
        "phases_ms": {"build_pyramid": ms_pyr, "allocate_levels": ms_alloc, "attention_fwd": ms_attn},
        "phases_ms_median": dict(zip(("build_pyramid", "allocate_levels", "attention_fwd"), median_ms)),
        "achieved_rho": rho, "kv_coverage": coverage,
        "executed_tflop": fl_exec / 1e12, "dense_tflop": fl_dense / 1e12,
        "roofline": {"kernel": "attn_mfma_kernel", "bound": "mfma", "achieved": attn_tflops, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": attn_tflops / PEAK_BF16_TFLOPS,
                     "traffic": attn_traffic, "traffic_source": attn_src,
                     "note": "executed FLOPs / mean HIP-event time of psa_attention_fwd (includes its block-list and tile-descriptor kernel)"},
        "roofline_pyramid": None if pyr_gbs is None else {
            "kernel": "pyramid_kernel", "bound": "hbm", "achieved": pyr_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": pyr_gbs / PEAK_HBM_GBS, "traffic": pyr_traffic, "traffic_source": pyr_src,
            "algorithmic_bytes": pyramid_bytes(w, w.levels)},
        "roofline_prepass": {
            "kernels": "psa_build_pyramid + psa_allocate_levels (pyramid, representatives, importance, allocation)",
            "bound": "hbm", "achieved": pre_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": pre_gbs / PEAK_HBM_GBS,
            "algorithmic_bytes": pre_bytes,
            "note": "K, V read + pooled levels written + Q read + level-H keys read + S written and read + M written, "
                    "over the mean HIP-event time of the two calls"},
    }
    if cap:
        Lh = cap["L"].cpu().numpy()
        out["config"]["similarity_cap"] = {"tau_s": list(cap["tau_s"]), "reduce": "per_head",
                                           "level_cap_histogram": [int((Lh == h).sum()) for h in range(1, w.levels + 1)]}
        out["roofline_pyramid"]["kernel"] = "pyramid_kernel with the similarities of Alg. 3 + cap_kernel"
    if hil:
        e = 2 if w.dtype == "bf16" else 4
        perm_bytes = 2.0 * e * w.N * w.d * w.B * (2 * w.Hq + 2 * w.Hkv)     # Q, K, V in and O out, each read and written once
        out["config"]["reorder"] = "hilbert"
        out["phases_ms"]["permute_qkv_and_o"] = ms_perm
        out["roofline_permute"] = {"kernel": "permute_kernel (4 launches)", "bound": "hbm", "achieved": perm_bytes / (ms_perm * 1e-3) / 1e9,
                                   "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": perm_bytes / (ms_perm * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                   "algorithmic_bytes": perm_bytes}
    if att is not None:
        out["attainable"] = att
        out["roofline"]["frac_of_attainable"] = attn_tflops / att["mfma_bf16_tflops"]
        out["roofline"]["frac_of_attainable_random_operands"] = attn_tflops / att["mfma_bf16_tflops_random_operands"]
        if pyr_gbs is not None:
            out["roofline_pyramid"]["frac_of_attainable"] = pyr_gbs / att["hbm_copy_gbs"]
        out["roofline_prepass"]["frac_of_attainable"] = pre_gbs / att["hbm_copy_gbs"]
    if w.dtype != "bf16":
        out["roofline"]["note"] += "; fp32 mode runs on the VALU (correctness mode), bf16 MFMA peak shown for scale only"
    if not args.no_parity:
        if hil:      # the path saw the reordered tensors: give the oracle the same
            from oracle import psa_oracle as orc
            Q, K, V = (orc.permute_tokens(x, perm_host) for x in (Q, K, V))
        out.update(parity_leg(w, gp, budget, Q, K, V, buf, torch))
    if not args.no_check_dense:
        # dense attention = the same call with every block at level 1 (that equality is a parity test)
        dense = torch.empty_like(buf.O)
        ones = torch.ones_like(buf.M)
        psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, ones, dense, buf.scratch)
        torch.cuda.synchronize()
        num = den = 0.0
        for b in range(w.B):            # head by head: the fp64 copies stay small
            for h in range(w.Hq):
                x, y = from_dev(buf.O[b, h], w.dtype), from_dev(dense[b, h], w.dtype)
                num += float(((x - y) ** 2).sum())
                den += float((y ** 2).sum())
        out["rel_l2_vs_dense"] = float(np.sqrt(num / den))
        del dense, ones
    if not args.no_threshold_point and w.levels == 4:
        # Alg. 2 with the thresholds the paper prints for its ablation; the compute ratio is whatever results
        tau = (0.5, 0.7, 0.8, 0.9)
        gt = params(alloc_mode=psa.PSA_ALLOC_THRESHOLD, tau=tau)
        tcalls = [lambda: psa.psa_allocate_levels(gt, Qd, Kd, buf.Kpyr, buf.M, buf.scratch, rho_out=buf.rho),
                  lambda: psa.psa_attention_fwd(gt, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch)]
        for _ in range(5):
            for fn in tcalls:
                fn()
        _, tmean, _ = timed_phases(torch, tcalls, 20)
        Mt = buf.M.cpu().numpy()
        fl_t = executed_flops(Mt, w, w.levels)
        rows_len = (Mt > 0).sum(axis=-1)
        out["threshold_point"] = {
            "rule": "Alg. 2", "tau": list(tau), "achieved_rho": float(buf.rho.mean().item()),
            "kv_coverage": float((Mt > 0).mean()) if not w.causal else None,
            "kept_blocks_per_row_min_max": [int(rows_len.min()), int(rows_len.max())],
            "allocate_levels_ms": tmean[0], "attention_fwd_ms": tmean[1], "executed_tflop": fl_t / 1e12,
            "attention_frac_of_peak": fl_t / (tmean[1] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "dense_equivalent_tflops": fl_dense / ((ms_pyr + tmean[0] + tmean[1]) * 1e-3) / 1e12,
        }
    if args.backward:
        # gradients under the budget rule's level map (the threshold point above has overwritten buf.M)
        psa.psa_allocate_levels(gp, Qd, Kd, buf.Kpyr, buf.M, buf.scratch)
        psa.psa_attention_fwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.scratch, lse=buf.lse)
        bscr = torch.empty(psa.psa_query_bwd_sizes(gp), dtype=torch.uint8, device="cuda")
        dO = torch.randn_like(buf.O)
        grads = [torch.empty_like(x) for x in (Qd, Kd, Vd)]
        bcall = [lambda: psa.psa_attention_bwd(gp, Qd, Kd, Vd, buf.Kpyr, buf.Vpyr, buf.M, buf.O, buf.lse, dO, *grads, bscr)]
        bcall[0]()
        _, bmean, _ = timed_phases(torch, bcall, 3)
        out["backward"] = {"attention_bwd_ms": bmean[0], "executed_tflop": 2.5 * fl_exec / 1e12,
                           "achieved_tflops": 2.5 * fl_exec / (bmean[0] * 1e-3) / 1e12,
                           "frac_of_bf16_mfma_peak": 2.5 * fl_exec / (bmean[0] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                           "note": "bf16: matrix-core kernels for dQ and the pooled dK, dV; FLOPs = 2.5 x the forward's executed FLOPs "
                                   "(five products per kept pair instead of two)"}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, budget, Q, K, V)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
