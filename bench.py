#!/usr/bin/env python3
"""Benchmark of the SEA attention forward pass on one MI355X.

A step is one sea_forward call (feature maps, key-side state, estimate contraction, per-row
top-k^ + mask expansion, sparse attention) over one batch of synthetic Q, K, V already resident
in HBM.  Prints ONE JSON line: tokens/s per attention layer on the largest configuration of the
metric (c4 at T = 32768 unless --workload says otherwise), the roofline figure of the kernel that
takes the largest share of the step (timed with HIP events on the launch stream), a sweep over the
other configurations, and the CPU oracle timed on this machine's host cores on a bounded sample
of the same workload.
"""
import argparse
import dataclasses
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0   # dense bf16 matrix cores
FP64_PEAK_TFLOPS = 78.6          # fp64 vector / matrix
DEFAULT_WORKLOAD = "c4_T32768"
SWEEP = ("c1", "c2", "c3", "c4_T4096", "c4_T8192", "c4_T16384", "c5")
# HBM bytes per launch (fetched, written) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script, scaled by the copy-kernel factors; they cannot be read inside this process, so they are
# quoted from the committed summary and only for the workload and kernel that summary covers.
TRAFFIC_FROM_PROFILES = {("c4_T32768", "sparse"): (190.8e6, 134.2e6), ("c4_T32768", "contract"): (361.7e6, 33.6e6),
                         ("c4_T32768", "state"): (135.1e6, 92.3e6)}
TRAFFIC_SOURCE = "profiles/sea_forward_c4_T32768.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, not measured in this run)"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)   # c4_T32768: about 0.2 s of timed work
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD,
                    help="c1..c5, c4_T<len>, c6_T<len>, c6c_T<len>, c7_T<len>; the default is the largest "
                         "single-GPU configuration of the metric (T = 32768)")
    ap.add_argument("--grouping", choices=["per_query", "causal_per_batch"], default="per_query",
                    help="top-k^ grouping (Sec. 3.1); the headline metric uses per_query")
    ap.add_argument("--geometry", choices=["fixed", "row_width"], default="fixed",
                    help="how the K columns map to keys: the same key buckets for every row (headline), or "
                         "each causal row resized to its own t + 1 keys (App. A.4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the short runs of the other configurations")
    ap.add_argument("--no-decoder", action="store_true", help="skip the decoder-shaped layer (c2 and c5 shapes)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="CPU-work budget of the oracle sample")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="only run a plain device copy of this many MiB three times (calibrates the "
                         "FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc) and exit")
    return ap.parse_args()


def cpu_baseline(wl, x, budget_s):
    """Oracle forward on a bounded sample of whole heads, one host thread per head.  Two one-thread
    probes (every 16th and every 8th query row of the first head) split a head's cost into its
    key-side part and its per-row part; the sample then takes as many whole heads as fit about
    `budget_s` seconds of CPU work, but at least one per thread.  Only when a single head would run
    longer than 20 s are its query rows thinned (every s-th row; the key-side work is still done
    in full, so the figure then understates the oracle a little).  tokens/s is scaled to the layer by
    the sampled share of (head, row) pairs."""
    import numpy as np
    import torch
    import oracle

    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
    f64 = lambda t: t.to(torch.float64).numpy()
    nheads = wl.B * wl.H
    p = oracle.Params(B=wl.B, H=wl.H, T=wl.T, d=wl.d, m=wl.m, K=wl.K, k_hat=wl.k_hat,
                      k_budget=wl.k_budget, causal=wl.causal, scale=wl.scale,
                      round8=wl.dtype == "bf16", grouping=wl.grouping, geometry=wl.geometry)
    Q, K, V, W = f64(x["Q"]), f64(x["K"]), f64(x["V"]), f64(x["W"])
    sl = None if x["seq_len"] is None else x["seq_len"].numpy()
    unit = wl.H if wl.grouping else 1          # heads that must be computed together

    def probe(stride):
        rows = np.arange(0, wl.T, stride, dtype=np.int32)
        t0 = time.perf_counter()
        oracle.forward(p, Q, K, V, W, seq_len=sl, rows=rows, heads=(0, unit), n_threads=1, want_aux=False)
        return (time.perf_counter() - t0) / unit

    t16, t8 = probe(16), probe(8)
    row_part = max(16.0 * (t8 - t16), 0.0)             # all rows of one head
    key_part = max(t16 - row_part / 16.0, 0.0)         # phi(K) and the state of one head
    head = key_part + row_part
    per_thread = max(cores // unit, 1) * unit          # heads that keep every thread busy
    stride = 1
    if head <= 20.0:
        n = int(budget_s / max(head, 1e-6))
        n = min(nheads, max(per_thread, (n // per_thread) * per_thread))
    else:
        n = min(nheads, per_thread)
        stride = int(min(256, max(2, -(-row_part // max(20.0 - key_part, 1.0)))))
    n = max(unit, (n // unit) * unit)
    rows = None if stride == 1 else np.arange(0, wl.T, stride, dtype=np.int32)
    t0 = time.perf_counter()
    out = oracle.forward(p, Q, K, V, W, seq_len=sl, rows=rows, heads=(0, n), n_threads=cores, want_aux=False)
    wall = time.perf_counter() - t0
    share = (n / nheads) * (1.0 if rows is None else len(rows) / wl.T)
    tokens = wl.B * wl.T * share
    return {"value": tokens / wall, "unit": "tokens/s", "cores": int(min(out["threads"], n // unit)), "kind": "oracle",
            "sample": f"first {n} of {nheads} heads of {wl.name} (T={wl.T}), "
                      f"{'every query row' if rows is None else f'every {stride}th query row'}, fp64 C oracle, "
                      f"{wall:.2f} s wall; one head on one thread: {head:.2f} s ({key_part:.2f} s key side)"}


def bucket_form(wl):
    """The attention stage groups (row, selected column) entries by column instead of walking tiles."""
    return wl.grouping == 0 and (wl.k_hat == 1 or (wl.k_hat <= 8 and 8 * wl.k_hat <= wl.K))


def issued_tile_flops(wl, seq_len, selected_columns):
    """Flops of the 32-key x 32-query tiles the tiled attention visits (launch geometry only).
    Tile walk: each wave of 32 rows walks the compact key list up to the last key its rows may
    see.  Bucket form: every (row, selected column) entry meets the r keys of its column, in
    32-key granules (partly filled 32-row tiles at bucket ends not counted)."""
    w = wl.T // wl.K
    r = w if wl.k_budget == 0 else min(w, max(1, wl.k_budget // wl.k_hat))
    if bucket_form(wl):
        return float(selected_columns) * (-(-r // 32) * 32) * wl.d * 4
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


def attention_mass_recall(torch, wl, d, sl, idx, cnt, n_heads=4, n_rows=256):
    """Share of the exact softmax attention mass (over the admissible keys of a row) that falls on
    the keys the sparse stage attends, averaged over sampled rows of sampled heads.  A diagnostic of
    the estimate + selection, computed with library ops on the device; not part of the path."""
    g = torch.Generator().manual_seed(0)
    N = wl.B * wl.H
    heads = torch.randperm(N, generator=g)[:n_heads].tolist()
    tot, n = 0.0, 0
    for bh in heads:
        b, h = divmod(bh, wl.H)
        ln = wl.T if sl is None else int(sl[b])
        if ln <= 0:
            continue
        rows = torch.randint(0, ln, (n_rows,), generator=g).to(d["Q"].device)
        q = d["Q"][b, h].index_select(0, rows).float()
        logits = (q @ d["K"][b, h, :ln].float().t()) * wl.scale
        keys = torch.arange(ln, device=logits.device)
        if wl.causal:
            logits = logits.masked_fill(keys[None, :] > rows[:, None], float("-inf"))
        prob = torch.softmax(logits, -1)
        ii = idx[b, h].index_select(0, rows).long()
        valid = ii >= 0
        got = torch.gather(prob, 1, ii.clamp(min=0, max=ln - 1)) * valid
        tot += float(got.sum())
        n += int(rows.numel())
    return tot / max(n, 1)


def measure(torch, sea, synth, wl, steps, warmup, detail):
    """Times sea_forward on one workload.  Returns (record, inputs)."""
    dev = "cuda:0"
    x = synth.make_inputs(wl)
    d = {k: x[k].to(dev) for k in "QKVW"}
    sl = None if x["seq_len"] is None else x["seq_len"].to(dev)
    p = sea.SeaParams(B=wl.B, H=wl.H, T=wl.T, d=wl.d, m=wl.m, K=wl.K, k_hat=wl.k_hat,
                      k_budget=wl.k_budget, causal=wl.causal, scale=wl.scale, dtype=wl.dtype, seq_len=sl,
                      grouping=wl.grouping, geometry=wl.geometry)
    ws = sea.alloc_workspace(p, dev)
    O = torch.empty_like(d["Q"])
    L = sea.sea_row_stride(p)

    # one untimed call that keeps the lists, to count the (query, key) pairs of the sparse stage
    cnt = torch.empty(wl.B, wl.H, wl.T, dtype=torch.int32, device=dev)
    idx = torch.empty(wl.B, wl.H, wl.T, L, dtype=torch.int32, device=dev) if detail else None
    sel = torch.empty(wl.B, wl.H, wl.T, sea.sea_sel_stride(p), dtype=torch.int32, device=dev)
    sea.sea_forward(p, d["Q"], d["K"], d["V"], d["W"], O, None, sel, idx, cnt, ws)
    torch.cuda.synchronize()
    pairs = int(cnt.sum().item())
    active_rows = int((cnt > 0).sum().item())
    selected_columns = int((sel >= 0).sum().item())
    recall = attention_mass_recall(torch, wl, d, x["seq_len"], idx, cnt) if detail else None
    del cnt, idx, sel

    step = lambda: sea.sea_forward(p, d["Q"], d["K"], d["V"], d["W"], O, None, None, None, None, ws)
    sea.sea_profile_enable(False)
    sea.sea_profile_collect()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # ---- the timed region: exactly `steps` calls, nothing else on the stream ----
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # ---- per-step spread: the same calls, each between two events of the launch stream ----
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    per_step = [a.elapsed_time(b) for a, b in ev]
    # ---- per-kernel durations: the same calls with every stage bracketed by HIP events ----
    sea.sea_profile_enable(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    stages = sea.sea_profile_collect()
    sea.sea_profile_enable(False)

    tokens = wl.B * wl.T
    ms_per_step = elapsed / steps * 1e3
    avg = {k: (v[0] / v[1]) for k, v in stages.items() if v[1] > 0}   # ms per launch
    launches = {k: int(v[1]) for k, v in stages.items() if v[1] > 0}

    es = 2 if wl.dtype == "bf16" else 4
    nrows = wl.B * wl.H * wl.T
    N = wl.B * wl.H
    tiled = sea.sea_attention_path(p) == 1
    wcol = wl.T // wl.K
    fused = tiled and wl.m in (64, 128, 256) and wl.K <= 256 and (wcol & (wcol - 1)) == 0
    kernels = {}
    # sparse attention: 4 d flops per selected (query, key) pair
    sparse_ms = avg.get("sparse", 0.0)
    algo_flops = 4.0 * wl.d * pairs
    if sparse_ms > 0 and tiled:
        ach = algo_flops / (sparse_ms * 1e-3) / 1e12
        issued = issued_tile_flops(wl, x["seq_len"], selected_columns)
        kernels["sparse"] = {"kernel": "tile_attn_kernel" + (" (bucket form, with its grouping kernels)" if bucket_form(wl) else ""),
                             "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": ach / MFMA_BF16_PEAK_TFLOPS, "avg_kernel_ms": sparse_ms,
                             "algorithmic_flops": algo_flops, "issued_flops": issued,
                             "issued_tflops": issued / (sparse_ms * 1e-3) / 1e12, "pairs": pairs,
                             "note": "achieved counts the selected (query, key) pairs only, 4 d flops each; issued "
                                     "counts every pair of the 32 x 32 tiles the kernel visits"}
    elif sparse_ms > 0 and sea.sea_attention_path(p) == 2:
        # fp32 tensors: q.k on the fp64 matrix cores (2 d flops per pair), P V on the fp32 ones (2 d)
        ach = 2.0 * wl.d * pairs / (sparse_ms * 1e-3) / 1e12
        kernels["sparse"] = {"kernel": "tile_attn_f32_kernel", "bound": "mfma", "achieved": ach, "peak": FP64_PEAK_TFLOPS,
                             "unit": "TFLOP/s", "frac": ach / FP64_PEAK_TFLOPS, "avg_kernel_ms": sparse_ms,
                             "algorithmic_flops": 2.0 * wl.d * pairs, "pairs": pairs,
                             "note": "fp64 products of the selected (query, key) pairs only, against the fp64 matrix "
                                     "peak; the fp32 products of P V (as many again) run beside them"}
    elif sparse_ms > 0 and sea.sea_attention_path(p) == 3:
        # the tiled kernel on one mask bit per (row, key) (per-row width geometry): the walk of the dense
        # causal kernel, every 32 x 32 tile at or below the diagonal issued
        fp32 = wl.dtype != "bf16"
        peak3 = FP64_PEAK_TFLOPS if fp32 else MFMA_BF16_PEAK_TFLOPS
        fl3 = (2.0 if fp32 else 4.0) * wl.d * pairs
        tiles_row = (wl.T + 31) // 32
        issued_pairs = float(N) * 1024.0 * tiles_row * (tiles_row + 1) / 2
        ach = fl3 / (sparse_ms * 1e-3) / 1e12
        kernels["sparse"] = {"kernel": ("tile_attn_f32_kernel" if fp32 else "tile_attn_kernel") + " (one mask bit per (row, key))",
                             "bound": "mfma", "achieved": ach, "peak": peak3, "unit": "TFLOP/s", "frac": ach / peak3,
                             "avg_kernel_ms": sparse_ms, "algorithmic_flops": fl3, "pairs": pairs,
                             "issued_flops_upper_bound": (2.0 if fp32 else 4.0) * wl.d * issued_pairs,
                             "note": "achieved counts the selected (query, key) pairs only; the upper bound of the issued "
                                     "flops counts every 32 x 32 tile at or below the diagonal (padding ignored)"}
    elif sparse_ms > 0:
        # per-row list kernel: the bytes that must cross HBM once are Q, K, V, O and the lists; the
        # repeated K / V row gathers of the pairs are served by the caches
        once_bytes = 4 * nrows * wl.d * es + pairs * 4 + nrows * 4
        ach = once_bytes / (sparse_ms * 1e-3) / 1e9
        kernels["sparse"] = {"kernel": "sparse_attn_kernel", "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS,
                             "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "avg_kernel_ms": sparse_ms,
                             "algorithmic_bytes": once_bytes, "pairs": pairs}
    # estimator: dense flop counts of the contractions (2 T d m per projection, 2 T m K)
    proj = 2.0 * wl.T * wl.d * wl.m * N
    contr = 2.0 * wl.T * wl.m * wl.K * N
    if fused:
        for name, kern, fl in (("state", "key_state_kernel", proj), ("contract", "estimate_rows_kernel", proj + contr)):
            ms = avg.get(name, 0.0)
            if ms > 0:
                ach = fl / (ms * 1e-3) / 1e12
                kernels[name] = {"kernel": kern, "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
                                 "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS, "avg_kernel_ms": ms,
                                 "algorithmic_flops": fl,
                                 "note": "dense count; about half of a causal contraction lies above the diagonal "
                                         "and is skipped" if name == "contract" and wl.causal else "dense count"}
    if wl.grouping == 1 and wl.geometry == 0 and avg.get("topk_mask", 0.0) > 0:
        # causal-per-batch selection: every time step's H x K slab of fp32 scores is read once, mask bits written
        gms = avg["topk_mask"]
        gbytes = float(nrows) * wl.K * 4 + float(nrows) * ((wl.K + 31) // 32) * 4
        kernels["topk_mask"] = {"kernel": "topk_group_kernel", "bound": "hbm", "achieved": gbytes / (gms * 1e-3) / 1e9,
                                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbytes / (gms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                "avg_kernel_ms": gms, "algorithmic_bytes": gbytes,
                                "note": "reads A_hat (fp32) once and writes the mask bits"}
    est_ms = sum(avg.get(k, 0.0) for k in ("features", "state", "contract"))
    est_flops = 2.0 * proj + contr
    peak = MFMA_BF16_PEAK_TFLOPS if wl.dtype == "bf16" else FP64_PEAK_TFLOPS
    est = {"ms": est_ms, "dense_flops": est_flops,
           "tflops": est_flops / (est_ms * 1e-3) / 1e12 if est_ms > 0 else 0.0,
           "peak_tflops": peak if wl.geometry == 0 else None,
           "frac_of_peak": (est_flops / (est_ms * 1e-3) / 1e12 / peak) if est_ms > 0 and wl.geometry == 0 else None,
           "useful_flops": est_flops - (0.5 * contr * (1.0 - 1.0 / wl.K) if wl.causal else 0.0),
           "includes_topk": "topk_mask" not in avg}
    if wl.geometry == 1:
        cms = avg.get("contract", 0.0)
        if wl.dtype == "bf16":
            # phi~(K) phi~(Q)^T below the diagonal on the bf16 matrix cores, 2 m flops per (row, key) pair,
            # every product then binned in LDS (the time includes the binning)
            fl = float(N) * wl.T * (wl.T + 1) / 2 * 2 * wl.m
            est.update({"tiles_kernel_ms": cms, "pair_flops": fl,
                        "pair_tflops": fl / (cms * 1e-3) / 1e12 if cms > 0 else 0.0,
                        "frac_of_bf16_mfma_peak": fl / (cms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS if cms > 0 else 0.0,
                        "binned_pairs_per_s": float(N) * wl.T * (wl.T + 1) / 2 / (cms * 1e-3) if cms > 0 else 0.0})
            if cms > 0:
                kernels["contract"] = {"kernel": "rw_tiles_mfma_kernel", "bound": "mfma", "achieved": fl / (cms * 1e-3) / 1e12,
                                       "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                       "frac": fl / (cms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "avg_kernel_ms": cms,
                                       "algorithmic_flops": fl,
                                       "note": "2 m flops per (row, key) pair at or below the diagonal; the time includes "
                                               "binning every product into its column in LDS"}
        elif wl.m <= 128:
            # tile form: phi(K) phi(Q)^T below the diagonal on the fp64 matrix cores, 2 m flops per (row, key) pair
            fl = float(N) * wl.T * (wl.T + 1) / 2 * 2 * wl.m
            est.update({"rows_kernel_ms": cms, "fp64_flops": fl,
                        "fp64_tflops": fl / (cms * 1e-3) / 1e12 if cms > 0 else 0.0,
                        "frac_of_fp64_matrix_peak": fl / (cms * 1e-3) / 1e12 / FP64_PEAK_TFLOPS if cms > 0 else 0.0})
            if cms > 0:
                kernels["contract"] = {"kernel": "rw_tiles_kernel", "bound": "mfma", "achieved": fl / (cms * 1e-3) / 1e12,
                                       "peak": FP64_PEAK_TFLOPS, "unit": "TFLOP/s",
                                       "frac": fl / (cms * 1e-3) / 1e12 / FP64_PEAK_TFLOPS, "avg_kernel_ms": cms,
                                       "algorithmic_flops": fl,
                                       "note": "2 m flops per (row, key) pair at or below the diagonal on the fp64 matrix "
                                               "cores; the time includes binning every product into its column in LDS"}
        else:
            gbytes = float(nrows) * (wl.K + 1) * wl.m * 8
            est.update({"rows_kernel_ms": cms, "gathered_bytes": gbytes,
                        "gather_TBps": gbytes / (cms * 1e-3) / 1e12 if cms > 0 else 0.0})
    dominant = max(kernels, key=lambda k: kernels[k]["avg_kernel_ms"]) if kernels else None
    if dominant is None and avg:
        # correctness paths (general shapes, fp32): report the estimator against its arithmetic peak
        dominant = "estimator"
        ach = est["tflops"]
        kernels["estimator"] = {"kernel": "estimate (features + state + contraction)", "bound": "alu" if wl.dtype == "f32" else "mfma",
                                "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak,
                                "avg_kernel_ms": est_ms, "algorithmic_flops": est_flops}
    rec = {"workload": wl.name, "ms_per_step": ms_per_step, "tokens_per_s": tokens * steps / elapsed,
           "median_ms": statistics.median(per_step), "min_ms": min(per_step), "steps": steps,
           "stage_ms": avg, "stage_launches_timed": launches, "pairs": pairs,
           "mean_keys_per_active_row": pairs / max(active_rows, 1), "row_stride": L,
           "dominant": dominant, "kernels": kernels, "estimator": est, "attention_mass_recall": recall,
           "gather_equivalent": None}
    if sparse_ms > 0:
        # the sparse stage in the per-row gather accounting (bytes a row-by-row gather would move):
        # K row + V row + index per pair, q in and o out per row.  With 128 rows sharing each staged
        # key tile the kernel is not bound by it; kept because the metric names an HBM fraction.
        gb = pairs * (2 * wl.d * es + 4) + nrows * (2 * wl.d * es + 4)
        rec["gather_equivalent"] = {"algorithmic_bytes": gb, "GBps": gb / (sparse_ms * 1e-3) / 1e9,
                                    "frac_of_hbm_peak": gb / (sparse_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    ctx = dict(x=x, d=d, p=p, O=O, ws=ws, step=step)
    return rec, ctx


def decoder_leg(torch, sea, synth, name, steps):
    """The paper's whole layer with its learned decoder (Sec. 3.1 "CNN Decoder", App. A.5.1) on random
    stand-in weights: sea_decoder_forward = Performer output on [V_I; V], MLPs, three-layer CNN, softmax,
    top-k^, sparse attention, output mixing.  A throughput workload: no quality claim.  Reports the
    dense / sparse split the paper's Fig. "complexity" gives for its own implementation."""
    dev = "cuda:0"
    wl = synth.get_workload(name)
    x = synth.make_inputs(wl)
    d = {k: x[k].to(dev) for k in "QKVW"}
    sl = None if x["seq_len"] is None else x["seq_len"].to(dev)
    p = sea.SeaParams(B=wl.B, H=wl.H, T=wl.T, d=wl.d, m=wl.m, K=wl.K, k_hat=wl.k_hat, k_budget=wl.k_budget,
                      causal=wl.causal, scale=wl.scale, dtype=wl.dtype, seq_len=sl)
    nbytes = sea.sea_decoder_workspace_bytes(p)
    if nbytes == 0:
        return None
    wd = {k: v.to(dev) for k, v in synth.decoder_weights(wl.H, wl.d, wl.K).items()}
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    O = torch.empty_like(d["Q"])
    step = lambda: sea.sea_decoder_forward(p, wd, d["Q"], d["K"], d["V"], d["W"], O, ws)
    for _ in range(3):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    sea.sea_profile_enable(True)
    sea.sea_profile_collect()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    st = sea.sea_profile_collect()
    sea.sea_profile_enable(False)
    avg = {k: v[0] / v[1] for k, v in st.items() if v[1] > 0}
    dense_ms = sum(avg.get(k, 0.0) for k in ("features", "state", "contract"))
    sparse_ms = avg.get("topk_mask", 0.0) + avg.get("sparse", 0.0)
    C, Wd, N = 4 * wl.H, wl.K // 2, wl.B * wl.H
    T1 = wl.T if wl.causal else -(-wl.T // 2)
    conv_flops = 2.0 * wl.B * 9 * C * (C * T1 * Wd * 2 + wl.H * wl.T * wl.K)
    mlp_flops = 2.0 * N * wl.T * 128 * (192 + 128 + 4 * Wd)
    lin_flops = 2.0 * N * wl.T * wl.m * (2 * 144 + (32 if wl.causal else 0)) + 4.0 * N * wl.T * wl.d * wl.m
    cms = avg.get("contract", 0.0)
    return {"workload": wl.name, "ms_per_step": ms, "tokens_per_s": wl.B * wl.T / (ms * 1e-3), "stage_ms": avg,
            "dense_ms": dense_ms, "sparse_ms": sparse_ms,
            "dense_share": dense_ms / max(dense_ms + sparse_ms, 1e-12),
            "mlp_cnn_tflops": (conv_flops + mlp_flops) / (cms * 1e-3) / 1e12 if cms > 0 else None,
            "mlp_cnn_frac_of_bf16_mfma_peak": (conv_flops + mlp_flops) / (cms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS if cms > 0 else None,
            "performer_flops": lin_flops, "weights": "random (Gaussian, fan-in scaled), seed 7",
            "note": "stages: features = phi(Q), phi(K); state = linear attention on [V_I; V]; contract = mu, nu, "
                    "CNN, softmax; topk_mask + sparse = selection and sparse attention"}


def copy_rate(torch, mib=1024, reps=10):
    """GB/s (read + written bytes) of a plain device-to-device copy: the achievable HBM figure."""
    src = torch.ones(mib << 20, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(reps):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    return 2.0 * (mib << 20) * reps / (a.elapsed_time(b) * 1e-3) / 1e9


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
        wl = dataclasses.replace(wl, name=wl.name + "+causal_per_batch", grouping=1)
    if args.geometry == "row_width":
        wl = dataclasses.replace(wl, name=wl.name + "+row_width", geometry=1)
    rec, ctx = measure(torch, sea, synth, wl, args.steps, args.warmup, detail=True)
    x, d, p, O = ctx["x"], ctx["d"], ctx["p"], ctx["O"]
    tokens = wl.B * wl.T

    roofline = dict(rec["kernels"][rec["dominant"]]) if rec["dominant"] else None
    if roofline is not None:
        t = TRAFFIC_FROM_PROFILES.get((wl.name, rec["dominant"]))
        roofline["traffic"] = None if t is None else t[0] + t[1]
        roofline["traffic_source"] = None if t is None else TRAFFIC_SOURCE
        roofline["timed_launches"] = rec["stage_launches_timed"].get(rec["dominant"])

    # ---- dense (quadratic) attention on the same shape, same dtype, for comparison ----
    dense = None
    if wl.dtype == "bf16":
        dws = torch.empty(sea.sea_dense_workspace_bytes(p), dtype=torch.uint8, device=dev)
        Od = torch.empty_like(d["Q"])
        for _ in range(3):
            sea.sea_dense_attn(p, d["Q"], d["K"], d["V"], Od, dws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        nd = max(3, min(args.steps // 2, 50))
        for _ in range(nd):
            sea.sea_dense_attn(p, d["Q"], d["K"], d["V"], Od, dws)
        torch.cuda.synchronize()
        dms = (time.perf_counter() - t0) / nd * 1e3
        dflops = wl.B * wl.H * 4.0 * wl.d * wl.T * wl.T * (0.5 if wl.causal else 1.0)
        dense = {"ms_per_call": dms, "tokens_per_s": tokens / (dms * 1e-3),
                 "tflops": dflops / (dms * 1e-3) / 1e12,
                 "frac_of_bf16_mfma_peak": dflops / (dms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                 "kernel": "tile_attn_kernel<dense>",
                 "note": "this library's own quadratic kernel, itself well below the matrix-core peak: any "
                         "sparse/dense crossover read from these numbers is relative to it"}
        del Od

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
        del Om, mws, s_mix

    out = {
        "metric": "SEA attn fwd tokens/s per layer + % HBM/MFMA roofline, T=1k..32k",
        "value": rec["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rec["ms_per_step"], "median_ms": rec["median_ms"], "min_ms": rec["min_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: B={wl.B} H={wl.H} T={wl.T} d={wl.d} m={wl.m} K={wl.K} "
                               f"k_hat={wl.k_hat} k_budget={wl.k_budget} causal={int(wl.causal)} "
                               f"pad_frac={wl.pad_frac} clustered Q/K ({wl.centroids} centroids), seed {wl.seed}",
                   "row_stride": rec["row_stride"], "mean_keys_per_active_row": rec["mean_keys_per_active_row"]},
        "roofline": roofline,
        "kernels": rec["kernels"],
        "gather_equivalent": rec["gather_equivalent"],
        "stage_ms": rec["stage_ms"],
        "estimator": rec["estimator"],
        "attention_mass_recall": rec["attention_mass_recall"],
        "dense_attention": dense,
        "output_mix_ms": mix_ms,
        "copy_GBps": copy_rate(torch),
    }
    del ctx, d, O
    torch.cuda.empty_cache()
    if not args.no_sweep:
        sweep = {}
        for name in SWEEP:
            if name == wl.name:
                continue
            w2 = synth.get_workload(name)
            r2, c2 = measure(torch, sea, synth, w2, max(20, args.steps // 4), max(5, args.warmup // 2), detail=False)
            dom = r2["kernels"].get(r2["dominant"]) if r2["dominant"] else None
            entry = {"ms_per_step": r2["ms_per_step"], "median_ms": r2["median_ms"], "min_ms": r2["min_ms"],
                     "tokens_per_s": r2["tokens_per_s"], "stage_ms": r2["stage_ms"],
                     "dominant_kernel": None if dom is None else dom["kernel"],
                     "roofline_bound": None if dom is None else dom["bound"],
                     "roofline_frac": None if dom is None else dom["frac"],
                     "kernel_fracs": {k: v["frac"] for k, v in r2["kernels"].items()}}
            if name == "c1":
                # launch-latency-free time of the small configuration: replay of a captured graph
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    c2["step"]()
                torch.cuda.current_stream().wait_stream(side)
                torch.cuda.synchronize()
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    c2["step"]()
                for _ in range(5):
                    graph.replay()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(50):
                    graph.replay()
                torch.cuda.synchronize()
                entry["graph_replay_ms"] = (time.perf_counter() - t0) / 50 * 1e3
                del graph
            sweep[name] = entry
            del c2
            torch.cuda.empty_cache()
        out["sweep"] = sweep
    if not args.no_decoder:
        out["decoder"] = {name: decoder_leg(torch, sea, synth, name, max(5, args.steps // 20)) for name in ("c2", "c5")}
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, x, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
