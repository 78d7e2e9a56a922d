#!/usr/bin/env python3
"""Benchmark of the SEA attention forward pass on one MI355X.

A step is one sea_forward call (feature maps, key-side state, estimate contraction, per-row
top-k^ + mask expansion, sparse attention) over one batch of synthetic Q, K, V already resident
in HBM.  Prints ONE JSON line: tokens/s per attention layer, the roofline figure of the dominant
kernel (sparse attention, timed with HIP events on the launch stream inside the timed region),
and the CPU oracle timed on this machine's host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM bytes per launch of the sparse-attention kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (scaled by the copy-kernel factors 2.0 / 1.0); see profiles/sea_forward_<workload>.md
MEASURED_TRAFFIC_BYTES = {"c2": 39.5e6 + 12.6e6, "c3": 262.4e6 + 67.1e6, "c4_T32768": 189.7e6 + 134.2e6,
                          "c6_T131072": 265.8e6 + 201.5e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)   # c2: about 20 ms of timed work
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2",
                    help="c1..c5 or c4_T<len>; c2 is the configuration the metric is quoted on")
    ap.add_argument("--grouping", choices=["per_query", "causal_per_batch"], default="per_query",
                    help="top-k^ grouping (Sec. 3.1); the headline metric uses per_query")
    ap.add_argument("--geometry", choices=["fixed", "row_width"], default="fixed",
                    help="how the K columns map to keys: the same key buckets for every row (headline), or "
                         "each causal row resized to its own t + 1 keys (App. A.4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="CPU-work budget of the oracle sample")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="only run a plain device copy of this many MiB three times (calibrates the "
                         "FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc) and exit")
    return ap.parse_args()


def cpu_baseline(wl, x, budget_s):
    """Oracle forward on a bounded sample of heads, all host threads; tokens/s scaled to the layer."""
    import numpy as np
    import torch
    import oracle

    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
    f64 = lambda t: t.to(torch.float64).numpy()
    nheads = wl.B * wl.H
    p = oracle.Params(B=wl.B, H=wl.H, T=wl.T, d=wl.d, m=wl.m, K=wl.K, k_hat=wl.k_hat,
                      k_budget=wl.k_budget, causal=wl.causal, scale=wl.scale,
                      round8=wl.dtype == "bf16" and wl.geometry == 0, grouping=wl.grouping, geometry=wl.geometry)
    Q, K, V, W = f64(x["Q"]), f64(x["K"]), f64(x["V"]), f64(x["W"])
    sl = None if x["seq_len"] is None else x["seq_len"].numpy()
    t0 = time.perf_counter()
    oracle.forward(p, Q, K, V, W, seq_len=sl, heads=(0, wl.H if wl.grouping else 1), n_threads=1, want_aux=False)
    one_heads = wl.H if wl.grouping else 1
    one = time.perf_counter() - t0
    one /= one_heads
    n = int(max(1, min(nheads, budget_s / max(one, 1e-6))))
    n = max(min(nheads, cores), (n // cores) * cores) if n >= cores else n
    n = min(n, nheads)
    if wl.grouping:                       # whole batch elements only
        n = max(wl.H, (n // wl.H) * wl.H)
    t0 = time.perf_counter()
    out = oracle.forward(p, Q, K, V, W, seq_len=sl, heads=(0, n), n_threads=cores, want_aux=False)
    wall = time.perf_counter() - t0
    tokens = wl.B * wl.T * (n / nheads)
    return {"value": tokens / wall, "unit": "tokens/s", "cores": int(out["threads"]), "kind": "oracle",
            "sample": f"first {n} of {nheads} heads of {wl.name} (full T={wl.T}), fp64 C oracle, "
                      f"{wall:.2f} s wall; one head on one thread {one:.2f} s"}


def issued_tile_flops(wl, seq_len):
    """Flops of the 32-key x 32-query tiles the tiled attention visits (launch geometry only):
    each wave of 32 rows walks the compact key list up to the last key its rows may see."""
    w = wl.T // wl.K
    r = w if wl.k_budget == 0 else min(w, max(1, wl.k_budget // wl.k_hat))
    if wl.k_hat == 1 and not wl.grouping:
        # bucket form: every active row against the r keys of its one column (32-key granules;
        # partly filled 32-row tiles at bucket ends not counted)
        rows = sum((wl.T if seq_len is None else int(seq_len[b])) for b in range(wl.B)) * wl.H
        return float(rows) * (-(-r // 32) * 32) * wl.d * 4
    total = 0
    for b in range(wl.B):
        ln = wl.T if seq_len is None else int(seq_len[b])
        for q0 in range(0, wl.T, 32):
            jmax = min(q0 + 31, wl.T - 1, ln - 1) if wl.causal else ln - 1
            if jmax < 0 or q0 >= wl.T:
                continue
            col, delta = divmod(jmax, w)
            u_end = col * r + min(r, -(-(delta + 1) * r // w))
            total += -(-u_end // 32)
    return float(total) * wl.H * 32 * 32 * wl.d * 4


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the B*H heads are independent, so more GPUs "
              "would each take a share of them with no exchange); rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2310_01777_amd import binding as sea
    from paper_2310_01777_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    if args.copy_probe > 0:
        src = torch.ones(args.copy_probe << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes": args.copy_probe << 20, "copies": 3}))
        return
    wl = synth.get_workload(args.workload)
    if args.grouping == "causal_per_batch":
        import dataclasses
        wl = dataclasses.replace(wl, name=wl.name + "+causal_per_batch", grouping=1)
    if args.geometry == "row_width":
        import dataclasses
        wl = dataclasses.replace(wl, name=wl.name + "+row_width", geometry=1)
    x = synth.make_inputs(wl)
    d = {k: x[k].to(dev) for k in "QKVW"}
    sl = None if x["seq_len"] is None else x["seq_len"].to(dev)
    p = sea.SeaParams(B=wl.B, H=wl.H, T=wl.T, d=wl.d, m=wl.m, K=wl.K, k_hat=wl.k_hat,
                      k_budget=wl.k_budget, causal=wl.causal, scale=wl.scale, dtype=wl.dtype, seq_len=sl,
                      grouping=wl.grouping, geometry=wl.geometry)
    ws = sea.alloc_workspace(p, dev)
    O = torch.empty_like(d["Q"])
    L = sea.sea_row_stride(p)

    # one untimed call with cnt kept, to count the (query, key) pairs the sparse stage processes
    cnt = torch.empty(wl.B, wl.H, wl.T, dtype=torch.int32, device=dev)
    sea.sea_forward(p, d["Q"], d["K"], d["V"], d["W"], O, None, None, None, cnt, ws)
    torch.cuda.synchronize()
    pairs = int(cnt.sum().item())
    active_rows = int((cnt > 0).sum().item())
    del cnt

    step = lambda: sea.sea_forward(p, d["Q"], d["K"], d["V"], d["W"], O, None, None, None, None, ws)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: only the dominant kernel (the sparse-attention stage) is bracketed by events,
    # and only on every fourth step, since every event pair costs a few microseconds of stream time
    sea.sea_profile_enable(False)
    sea.sea_profile_collect()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % 4 == 0:
            sea.sea_profile_enable(["sparse"])
        elif i % 4 == 1:
            sea.sea_profile_enable(False)
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stages = sea.sea_profile_collect()
    # per-stage table from a separate, untimed pass with every stage bracketed
    sea.sea_profile_enable(True)
    for _ in range(max(3, args.steps // 4)):
        step()
    torch.cuda.synchronize()
    all_stages = sea.sea_profile_collect()
    sea.sea_profile_enable(False)
    all_stages["sparse"] = stages["sparse"]

    tokens = wl.B * wl.T
    ms_per_step = elapsed / args.steps * 1e3
    value = tokens * args.steps / elapsed
    avg = {k: (v[0] / v[1]) for k, v in all_stages.items() if v[1] > 0}   # ms per launch

    # ---- roofline of the dominant kernel: the sparse attention stage ----
    # Per (query, key) pair the stage does 4 d flops and, in the per-row gather accounting, moves
    # one K row + one V row + one index; per query row q in and o out.
    es = 2 if wl.dtype == "bf16" else 4
    nrows = wl.B * wl.H * wl.T
    sparse_ms = avg.get("sparse", 0.0)
    algo_flops = 4.0 * wl.d * pairs
    algo_bytes = pairs * (2 * wl.d * es + 4) + nrows * (2 * wl.d * es + 4)
    tiled = sea.sea_attention_path(p) == 1   # the tiled matrix-core kernel ran (bf16, column-structured mask)
    if tiled:
        issued = issued_tile_flops(wl, x["seq_len"])
        ach = algo_flops / (sparse_ms * 1e-3) / 1e12
        roofline = {"kernel": "tile_attn_kernel", "bound": "mfma", "achieved": ach,
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name), "avg_kernel_ms": sparse_ms,
                    "timed_launches": int(stages["sparse"][1]),
                    "algorithmic_flops": algo_flops,
                    "issued_flops": issued, "issued_tflops": issued / (sparse_ms * 1e-3) / 1e12,
                    "pairs": pairs,
                    "note": "achieved counts only the selected (query, key) pairs (4 d flops each); issued "
                            "counts every pair of the 32x32 tiles the kernel visits"}
    else:
        # per-row list kernel: the bytes that must cross HBM once are Q, K, V, O and the lists; the
        # repeated K / V row gathers of the pairs are served by the caches (see gather_equivalent)
        once_bytes = 4 * nrows * wl.d * es + pairs * 4 + nrows * 4
        ach = once_bytes / (sparse_ms * 1e-3) / 1e9
        roofline = {"kernel": "sparse_attn_kernel", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": None, "avg_kernel_ms": sparse_ms,
                    "algorithmic_bytes": once_bytes, "pairs": pairs}
    # the same stage in the per-row gather accounting (bytes a row-by-row gather would move)
    gather_equiv = {"algorithmic_bytes": algo_bytes,
                    "GBps": algo_bytes / (sparse_ms * 1e-3) / 1e9 if sparse_ms > 0 else 0.0,
                    "frac_of_hbm_peak": algo_bytes / (sparse_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if sparse_ms > 0 else 0.0}
    # estimator (features + state + contraction [+ in-register top-k]): dense matrix-core flop count
    est_ms = sum(avg.get(k, 0.0) for k in ("features", "state", "contract"))
    est_flops = wl.B * wl.H * (4.0 * wl.T * wl.d * wl.m + 2.0 * wl.T * wl.m * wl.K)
    est = {"ms": est_ms, "dense_flops": est_flops,
           "tflops": est_flops / (est_ms * 1e-3) / 1e12 if est_ms > 0 else 0.0,
           "frac_of_bf16_mfma_peak": (est_flops / (est_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS)
           if est_ms > 0 and wl.dtype == "bf16" else None,
           "includes_topk": "topk_mask" not in avg}
    if wl.geometry == 1:
        # per-row width geometry: the contraction is K + 1 gathered fp64 prefix rows of m features per
        # query row, served by the caches
        gbytes = float(nrows) * (wl.K + 1) * wl.m * 8
        cms = avg.get("contract", 0.0)
        est.update({"frac_of_bf16_mfma_peak": None, "rows_kernel_ms": cms, "gathered_bytes": gbytes,
                    "gather_TBps": gbytes / (cms * 1e-3) / 1e12 if cms > 0 else 0.0})

    # ---- dense (quadratic) attention on the same shape, same dtype, for comparison ----
    dense = None
    if wl.dtype == "bf16":
        dws = torch.empty(sea.sea_dense_workspace_bytes(p), dtype=torch.uint8, device=dev)
        Od = torch.empty_like(d["Q"])
        for _ in range(3):
            sea.sea_dense_attn(p, d["Q"], d["K"], d["V"], Od, dws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        nd = max(3, args.steps // 2)
        for _ in range(nd):
            sea.sea_dense_attn(p, d["Q"], d["K"], d["V"], Od, dws)
        torch.cuda.synchronize()
        dms = (time.perf_counter() - t0) / nd * 1e3
        dflops = wl.B * wl.H * 4.0 * wl.d * wl.T * wl.T * (0.5 if wl.causal else 1.0)
        dense = {"ms_per_call": dms, "tokens_per_s": tokens / (dms * 1e-3),
                 "tflops": dflops / (dms * 1e-3) / 1e12, "kernel": "tile_attn_kernel<dense>"}

    # ---- output mixing epilogue (Sec. 3.1.1), timed on its own: not part of the headline step ----
    mix_ms = None
    if wl.causal:   # the bidirectional form also needs A_hat, which the headline step does not keep
        mws = torch.empty(sea.sea_output_mix_workspace_bytes(p), dtype=torch.uint8, device=dev)
        s_mix = torch.rand(wl.B, wl.H, wl.T, device=dev)
        Om = torch.empty_like(O)
        for _ in range(3):
            sea.sea_output_mix(p, O, d["V"], s_mix, Om, mws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            sea.sea_output_mix(p, O, d["V"], s_mix, Om, mws)
        torch.cuda.synchronize()
        mix_ms = (time.perf_counter() - t0) / 10 * 1e3

    out = {
        "metric": "SEA attn fwd tokens/s per layer + % HBM/MFMA roofline, T=1k..32k",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.B} H={wl.H} T={wl.T} d={wl.d} m={wl.m} K={wl.K} "
                               f"k_hat={wl.k_hat} k_budget={wl.k_budget} causal={int(wl.causal)} "
                               f"pad_frac={wl.pad_frac} clustered Q/K ({wl.centroids} centroids), seed {wl.seed}",
                   "row_stride": L, "mean_keys_per_active_row": pairs / max(active_rows, 1)},
        "roofline": roofline,
        "gather_equivalent": gather_equiv,
        "stage_ms": avg,
        "estimator": est,
        "dense_attention": dense,
        "output_mix_ms": mix_ms,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, x, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
