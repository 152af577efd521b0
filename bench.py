#!/usr/bin/env python3
"""Benchmark of the SALE prefill attention path on one MI355X.

One step = one pass of the whole hot path over one synthetic Llama-3.1-8B
attention layer: sale_quantize_qk -> sale_select -> sale_sparse_attn, inputs
resident in HBM.  The dense causal kernel (the speed-up denominator) is timed
in the same run.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--tau T]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_INT8_TOPS = 5000.0       # MI355X dense int8 MFMA
PEAK_FP8_TFLOPS = 5000.0      # MI355X dense fp8 MFMA
PEAK_FP6_TFLOPS = 10100.0     # MI355X dense fp6 MFMA
PEAK_HBM_GBS = 8000.0


def _oracle_threads() -> int:
    """Threads the oracle's numpy work really runs on: the thread count of numpy's BLAS (its matrix products are
    where the time goes; the element-wise parts are single-threaded), capped by the cores this process may use."""
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:
        avail = os.cpu_count() or 1
    try:
        from threadpoolctl import threadpool_info
        blas = [i["num_threads"] for i in threadpool_info() if i.get("user_api") == "blas"]
        return min(max(blas), avail) if blas else 1
    except Exception:
        return 1


def cpu_baseline(w, q, k, v, budget_units: int, seed: int = 1234, block_k: int = 64, segment: int = 0):
    """Times the CPU oracle (as it stands) on a seeded sample of (head, query
    block) units of the same workload and extrapolates to the whole layer."""
    import numpy as np
    import torch
    from oracle import sale_oracle as so

    geo = so.Geometry(w.seq_len, w.head_dim, 64, block_k, 1, 4, segment=segment)
    rng = np.random.default_rng(seed)
    units = [(int(rng.integers(0, w.n_q_heads)), int(rng.integers(0, geo.n_q))) for _ in range(budget_units)]
    t0 = time.perf_counter()
    cache = {}
    for h, i in units:
        g = h // w.group
        if g not in cache:           # quantizing K of the group is part of the oracle's work
            kf = k[g].float().numpy()
            kc, ks = so.quantize_blocks(kf[None], block_k)
            cache = {g: (kf, kc[0], ks[0], v[g].float().numpy())}
        kf, kc, ks, vf = cache[g]
        rs = slice(i * 64, (i + 1) * 64)
        qf = q[h, rs].float().numpy()
        qc, qs = so.quantize_blocks(qf[None], 64)
        row, *_ = so.select_row(geo, i, qf, kf, qc[0], kc, float(qs[0, 0]), ks, w.tau)
        so.attention_block(geo, i, qf, kf, vf, row)
    dt = time.perf_counter() - t0
    total_units = w.n_q_heads * geo.n_q
    return {
        "value": dt / len(units) * total_units * 1e3,
        "unit": "ms",
        "cores": _oracle_threads(),
        "kind": "oracle",
        "sample": f"{len(units)} of {total_units} (head, 64-row query block) units drawn uniformly (seed {seed}) from the "
                  f"same workload, measured {dt:.1f} s; value = sample mean x {total_units} units (extrapolated); "
                  f"host reports {os.cpu_count()} CPUs, numpy BLAS threads as in `cores`",
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--dense-steps", type=int, default=2)
    ap.add_argument("--workload", default="llama31-8b-layer-128k")
    ap.add_argument("--tau", type=float, default=None)
    ap.add_argument("--block-k", type=int, default=64, choices=(64, 32),
                    help="key block size b_k (64: the headline configuration; 32: the paper's shape)")
    ap.add_argument("--segment-local", action="store_true", help="segment rule for the local area (Appendix C)")
    ap.add_argument("--attn-int8-qk", action="store_true",
                    help="quantized Computation-Pass (Sec. 3.4): 8-bit Q, K in the first product of sparse AND dense attention")
    ap.add_argument("--attn-fp8-pv", action="store_true",
                    help="fully quantized Computation-Pass: --attn-int8-qk plus the FP8 second product (64x64 blocks)")
    ap.add_argument("--cpu-units", type=int, default=96, help="oracle sample size (0 = skip the CPU baseline)")
    ap.add_argument("--no-lengths", dest="lengths", action="store_false",
                    help="skip the 32K and 64K legs that the default 128K run adds (object `lengths`)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path shards by KV head without communication, "
              "but no multi-GPU run is part of it); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2505_24179_amd import inputs, sale

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    if args.attn_fp8_pv:
        args.attn_int8_qk = True
    flags = (sale.FLAG_SEGMENT_LOCAL if args.segment_local else 0) | (sale.FLAG_ATTN_INT8_QK if args.attn_int8_qk else 0) | \
            (sale.FLAG_ATTN_FP8_PV if args.attn_fp8_pv else 0)

    def measure(w, steps, warmup, dense_steps):
        """One workload: K timed steps of quantize -> select -> sparse attention (HIP events around every stage on
        the launch stream), then the dense kernel.  -> (figures, host tensors q, k, v)"""
        t_gen = time.perf_counter()
        q, k, v = inputs.make_inputs(w)
        t_gen = time.perf_counter() - t_gen
        p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, block_k=args.block_k, flags=flags)
        qd, kd, vd = (t.unsqueeze(0).to(dev) for t in (q, k, v))
        tau = torch.tensor([w.tau], dtype=torch.float32, device=dev)
        # all outputs and the workspaces are allocated once, outside the timed region
        q4 = torch.empty(1, w.n_q_heads, w.seq_len, 64, dtype=torch.uint8, device=dev)
        k4 = torch.empty(1, w.n_kv_heads, w.seq_len, 64, dtype=torch.uint8, device=dev)
        qs = torch.empty(1, w.n_q_heads, p.n_q, dtype=torch.float32, device=dev)
        ks = torch.empty(1, w.n_kv_heads, p.n_k, dtype=torch.float32, device=dev)
        mask = torch.empty(1, w.n_q_heads, p.n_q, p.words, dtype=torch.int64, device=dev)
        counts = torch.empty(1, w.n_q_heads, p.n_q, dtype=torch.int32, device=dev)
        o = torch.empty_like(qd)
        ws_sel = torch.empty(max(1, sale.workspace_bytes(p, sale.WS_SELECT)), dtype=torch.uint8, device=dev)
        # The attention workspace holds one parking slot per LONG row (rows keeping more than 192 x 64 keys are swept
        # window by window): their number is read once from a first Selection-Pass, outside the timed region.
        sale.quantize_qk(p, qd, kd, out=(q4, k4, qs, ks))
        sale.select(p, qd, kd, q4, k4, qs, ks, tau, out=(mask, counts), ws=ws_sel)
        n_long = int((counts > 192 * (64 // args.block_k)).sum().item())
        ws_bytes = {"select": int(ws_sel.numel()),
                    "sparse_attn": sale.workspace_bytes(p, sale.WS_SPARSE_ATTN_MIN) + n_long * sale.PARKED_ROW_BYTES,
                    "dense_attn": sale.workspace_bytes(p, sale.WS_DENSE_ATTN), "long_rows": n_long}
        ws_att = torch.empty(max(1, ws_bytes["sparse_attn"], ws_bytes["dense_attn"]), dtype=torch.uint8, device=dev)

        def step(ev=None):
            if ev: ev[0].record()
            sale.quantize_qk(p, qd, kd, out=(q4, k4, qs, ks))
            if ev: ev[1].record()
            sale.select(p, qd, kd, q4, k4, qs, ks, tau, out=(mask, counts), ws=ws_sel)
            if ev: ev[2].record()
            sale.sparse_attn(p, qd, kd, vd, mask, counts, out=o, ws=ws_att)
            if ev: ev[3].record()

        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        t0 = time.perf_counter()
        for s in range(steps):
            step(evs[s])
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        quant_ms = sum(e[0].elapsed_time(e[1]) for e in evs) / steps
        select_ms = sum(e[1].elapsed_time(e[2]) for e in evs) / steps
        sparse_ms = sum(e[2].elapsed_time(e[3]) for e in evs) / steps
        dense_ms = None
        if dense_steps > 0:      # the denominator
            sale.dense_attn(p, qd, kd, vd, out=o, ws=ws_att)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(dense_steps):
                sale.dense_attn(p, qd, kd, vd, out=o, ws=ws_att)
            b.record()
            torch.cuda.synchronize()
            dense_ms = a.elapsed_time(b) / dense_steps

        # a "pair" is one (query block, key block) tile: 64 x b_k logits
        n_q, kpq = p.n_q, 64 // args.block_k
        causal_pairs = w.n_q_heads * sum((i + 1) * kpq for i in range(n_q))
        kept_pairs = int(counts.sum().item())
        flop_pair = 4.0 * 64 * args.block_k * 128
        # (the segment rule moves at most 3 blocks per row from the middle to the local area: not subtracted)
        middle_pairs = sum(max(0, (i + 1) * kpq - p.sink_blocks - p.local_blocks) for i in range(n_q)) * w.n_q_heads
        quant_bytes = (w.n_q_heads + w.n_kv_heads) * w.seq_len * (256 + 64) + (w.n_q_heads + w.n_kv_heads) * n_q * 4
        bf16_peak = PEAK_BF16_TFLOPS
        if args.attn_int8_qk:       # the first product runs at the int8 MFMA rate, the second at the bf16 (or FP8) rate
            bf16_peak = 2.0 / (1.0 / (PEAK_FP8_TFLOPS if args.attn_fp8_pv else PEAK_BF16_TFLOPS) + 1.0 / PEAK_INT8_TOPS)
        kernels = {
            "quantize": {"bound": "hbm", "achieved": quant_bytes / (quant_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                         "unit": "GB/s", "ms": quant_ms},
            "select": {"bound": "mfma", "achieved": middle_pairs * 2.0 * 64 * args.block_k * 128 / (select_ms * 1e-3) / 1e12,
                       "peak": PEAK_FP6_TFLOPS, "unit": "TFLOP/s", "ms": select_ms},
            "sparse_attn": {"bound": "mfma", "achieved": kept_pairs * flop_pair / (sparse_ms * 1e-3) / 1e12,
                            "peak": bf16_peak, "unit": "TFLOP/s", "ms": sparse_ms},
        }
        if dense_ms:
            kernels["dense_attn"] = {"bound": "mfma", "achieved": causal_pairs * flop_pair / (dense_ms * 1e-3) / 1e12,
                                     "peak": bf16_peak, "unit": "TFLOP/s", "ms": dense_ms}
        for kv in kernels.values():
            kv["frac"] = kv["achieved"] / kv["peak"]
        sale_ms = quant_ms + select_ms + sparse_ms
        # the dense time of a kernel AT the 60 % target: the overhead bound must not lean on a slow denominator
        dense60_ms = causal_pairs * flop_pair / (0.6 * bf16_peak * 1e12) * 1e3
        fig = {
            "sale_ms": sale_ms, "wall_ms": wall_ms, "input_gen_s": t_gen,
            "stages_ms": {"quantize": quant_ms, "select": select_ms, "sparse_attn": sparse_ms, "dense_attn": dense_ms},
            "density": kept_pairs / causal_pairs, "workspace_bytes": ws_bytes,
            "select_overhead_pct": None if not dense_ms else 100.0 * (quant_ms + select_ms) / dense_ms,
            "select_overhead_pct_of_dense_at_60pct_peak": 100.0 * (quant_ms + select_ms) / dense60_ms,
            "computation_pass_speedup": None if not dense_ms else dense_ms / sparse_ms,
            "end_to_end_speedup": None if not dense_ms else dense_ms / sale_ms,
            "effective_tflops": causal_pairs * flop_pair / (sale_ms * 1e-3) / 1e12,
            "tokens_per_s": w.seq_len / (sale_ms * 1e-3),
            "kernels": kernels,
        }
        return fig, (q, k, v)

    w = inputs.WORKLOADS[args.workload]
    if args.tau is not None:
        from dataclasses import replace
        w = replace(w, tau=args.tau)
    fig, (q, k, v) = measure(w, args.steps, args.warmup, args.dense_steps)
    kernels = fig["kernels"]
    dominant = max(("quantize", "select", "sparse_attn"), key=lambda n: kernels[n]["ms"])
    roof = dict(kernels[dominant])
    roof.pop("ms")
    roof.update({"kernel": dominant, "traffic": None})
    # HBM-side bytes per call measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (committed summary)
    tfile = os.path.join(ROOT, "profiles", f"traffic_{w.name}.json")
    if os.path.exists(tfile) and args.tau is None and args.block_k == 64 and not args.attn_int8_qk:
        with open(tfile) as f:
            t = json.load(f).get(dominant)
        if t:
            roof["traffic"] = {"read_bytes": t["fetch_bytes"], "write_bytes": t["write_bytes"],
                               "source": os.path.relpath(tfile, ROOT)}

    # the other lengths of the metric (32K and 64K of the same layer), a few steps each
    lengths = {}
    if args.lengths and args.workload == "llama31-8b-layer-128k" and args.tau is None:
        for name in ("llama31-8b-layer-32k", "llama31-8b-layer-64k"):
            f2, _ = measure(inputs.WORKLOADS[name], 5, 2, 2)
            lengths[name] = {key: f2[key] for key in ("sale_ms", "stages_ms", "density", "select_overhead_pct",
                                                       "select_overhead_pct_of_dense_at_60pct_peak",
                                                       "computation_pass_speedup", "end_to_end_speedup", "effective_tflops")}
            lengths[name]["frac"] = {n: kv["frac"] for n, kv in f2["kernels"].items()}
            lengths[name]["achieved"] = {n: kv["achieved"] for n, kv in f2["kernels"].items()}

    out = {
        "metric": "sparse prefill attn ms + speedup vs own dense kernel at 128K; select overhead %",
        "value": fig["sale_ms"],
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": fig["wall_ms"],
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "seq_len": w.seq_len, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "block": f"64x{args.block_k}", "segment_local": bool(args.segment_local),
                   "attn_int8_qk": bool(args.attn_int8_qk), "attn_fp8_pv": bool(args.attn_fp8_pv), "tau": w.tau, "rho": w.rho, "n_heavy": w.n_heavy,
                   "seed": w.seed},
        "stages_ms": fig["stages_ms"],
        "density": fig["density"],
        "workspace_bytes": fig["workspace_bytes"],
        "select_overhead_pct": fig["select_overhead_pct"],
        "select_overhead_pct_of_dense_at_60pct_peak": fig["select_overhead_pct_of_dense_at_60pct_peak"],
        "computation_pass_speedup": fig["computation_pass_speedup"],
        "end_to_end_speedup": fig["end_to_end_speedup"],
        "effective_tflops": fig["effective_tflops"],
        "tokens_per_s": fig["tokens_per_s"],
        "roofline": roof,
        "kernels": kernels,
        "lengths": lengths,
        "input_gen_s": fig["input_gen_s"],
    }
    if args.cpu_units > 0 and not args.attn_int8_qk:      # (the CPU leg times the unquantized oracle path)
        out["cpu_baseline"] = cpu_baseline(w, q, k, v, args.cpu_units, block_k=args.block_k,
                                           segment=4 if args.segment_local else 0)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
