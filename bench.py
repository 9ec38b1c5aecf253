#!/usr/bin/env python3
"""Benchmark of the Dense-and-Sparse LUT matvec on one MI355X.

Workload (default): the LLaMA-65B-shaped MLP pair at 3 bits — layers 22016x8192 and 8192x22016, the largest
single-GPU configuration of the benchmark list: 8 fp16 centroids per output row, 0.45 % fp16 CSR outliers with
heavy row skew (1 % of the rows hold 30 % of the nonzeros), batch 1, synthetic seeded weights (Student-t(4) * 0.02)
and N(0,1) activations.

A "step" is one pass of the hot path over that pair: two calls of sqllm_dense_sparse_matvec, back to back on
one stream.  To measure HBM and not the 256 MB last-level cache, the steps rotate over enough copies of the
two layers (at distinct addresses) for the working set to exceed 1 GB.  All inputs are resident in HBM
before the timed region starts.  The K steps are captured in one HIP graph that is replayed several times; the
median replay is the reported time (minimum and maximum are printed beside it).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
SEED = 20230613
WORKLOADS = {
    # name: (list of (M, N), bits, frac, skew, B)
    "llama7b_mlp_pair_3bit": ([(11008, 4096), (4096, 11008)], 3, 0.0045, (0.10, 0.50), 1),
    "llama7b_mlp_pair_4bit": ([(11008, 4096), (4096, 11008)], 4, 0.0045, (0.10, 0.50), 1),
    "llama7b_mlp_pair_2bit": ([(11008, 4096), (4096, 11008)], 2, 0.0045, (0.10, 0.50), 1),
    "llama7b_mlp_pair_2bit_sparse0.1": ([(11008, 4096), (4096, 11008)], 2, 0.001, (0.10, 0.50), 1),
    "single_4096_4bit": ([(4096, 4096)], 4, 0.0045, None, 1),
    "llama13b_attn_3bit": ([(5120, 5120)], 3, 0.0045, None, 1),
    "llama13b_attn_4bit": ([(5120, 5120)], 4, 0.0045, None, 1),
    "llama13b_mlp_pair_3bit": ([(13824, 5120), (5120, 13824)], 3, 0.0045, None, 1),
    "llama13b_mlp_pair_4bit": ([(13824, 5120), (5120, 13824)], 4, 0.0045, None, 1),
    "llama13b_up_3bit_sparse0.05": ([(13824, 5120)], 3, 0.0005, None, 1),
    "llama13b_up_3bit_sparse1.0": ([(13824, 5120)], 3, 0.01, None, 1),
    "llama7b_block_3bit": ([(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)], 3, 0.0045, (0.10, 0.50), 1),
    # the same block with the projections that share an input stacked row-wise (q,k,v -> 12288 rows; gate,up ->
    # 22016 rows): exact, because every output row has its own table; 4 launches per block instead of 7
    "llama7b_block_3bit_stacked": ([(12288, 4096), (4096, 4096), (22016, 4096), (4096, 11008)], 3, 0.0045, (0.10, 0.50), 1),
    "llama65b_attn_3bit": ([(8192, 8192)], 3, 0.0045, (0.01, 0.30), 1),
    "llama65b_mlp_pair_3bit": ([(22016, 8192), (8192, 22016)], 3, 0.0045, (0.01, 0.30), 1),
    "llama65b_attn_3bit_batch2": ([(8192, 8192)], 3, 0.0045, (0.01, 0.30), 2),
    "llama65b_attn_3bit_batch4": ([(8192, 8192)], 3, 0.0045, (0.01, 0.30), 4),
    "llama65b_attn_3bit_batch8": ([(8192, 8192)], 3, 0.0045, (0.01, 0.30), 8),
    "llama65b_attn_3bit_batch16": ([(8192, 8192)], 3, 0.0045, (0.01, 0.30), 16),
    "llama7b_mlp_pair_3bit_batch16": ([(11008, 4096), (4096, 11008)], 3, 0.0045, (0.10, 0.50), 16),
}


# offline side: one step = one whole sqllm_quantize_layer call (split + weighted k-means) on one matrix
QUANT_WORKLOADS = {
    # name: (M, N, bits, outlier share, sensitive share, max centroid updates)
    "quantize_llama7b_attn_3bit": (4096, 4096, 3, 0.004, 0.0005, 32),
    "quantize_llama7b_up_3bit": (11008, 4096, 3, 0.004, 0.0005, 32),
    "quantize_llama7b_down_4bit": (4096, 11008, 4, 0.004, 0.0005, 32),
}
ALU_PEAK_TOPS = 39.3   # 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz: one integer / compare lane operation per lane and clock


def bench_quantize(args):
    import numpy as np
    import torch
    import gen
    import paper_2306_07629_amd as sq
    from oracle import quant_oracle as qo   # parity gate and cpu_baseline leg only

    M, N, bits, of, sf, max_iter = QUANT_WORKLOADS[args.workload]
    K = 1 << bits
    w = gen.make_weights(M, N, gen.layer_seed(SEED, 6, 0))
    s = gen.make_sens(M, N, gen.layer_seed(SEED, 6, 0))
    n_lo, n_hi, n_sens = sq.sqllm_extraction_counts(M, N, of, sf)
    wd = torch.from_numpy(w.view(np.int16)).cuda()
    sd = torch.from_numpy(s.view(np.int16)).cuda()
    q = sq.quantize_layer(wd, sd, bits, n_lo, n_hi, n_sens, max_iter)
    torch.cuda.synchronize()

    # ---- parity gate: the split in full, tables / indices / iteration counts on a sample of rows
    rows = np.unique(np.random.default_rng(1).integers(0, M, 24))
    t0 = time.perf_counter()
    thr = qo.thresholds(w, s, n_lo, n_hi, n_sens)
    mask = qo.split_mask(w, s, thr)
    rowptr, cols, vals = qo.csr_from_mask(w, mask)
    t_split = time.perf_counter() - t0
    t0 = time.perf_counter()
    ref = qo.quantize_layer(w, s, bits, n_lo, n_hi, n_sens, max_iter, rows=rows)
    t_rows = time.perf_counter() - t0 - t_split           # quantize_layer repeats the split
    import oracle
    nnz = q.nnz()
    idx = oracle.unpack(M, N, bits, q.qidx.cpu().numpy())
    ok = (np.array_equal(q.rowptr.cpu().numpy(), rowptr) and np.array_equal(q.cols.cpu().numpy()[:nnz], cols)
          and np.array_equal(q.vals.cpu().numpy().view(np.uint16)[:nnz], vals)
          and np.array_equal(q.lut.cpu().numpy().view(np.uint16)[rows], ref["lut"][rows]) and np.array_equal(idx[rows], ref["idx"][rows])
          and np.array_equal(q.iters.cpu().numpy()[rows], ref["iters"][rows]))
    if not ok:
        print("bench.py: parity FAILED for the quantised layer", file=sys.stderr)
        sys.exit(4)

    def step(_):
        sq.quantize_layer(wd, sd, bits, n_lo, n_hi, n_sens, max_iter)

    sec, wall = time_steps(torch, step, args.steps, args.warmup, use_graph=False)
    ms = sec / args.steps * 1e3
    iters = q.iters.float()
    mean_it = float(iters.mean().item())
    # lane operations the method itself needs: per weight and assignment pass K - 1 compare-and-count pairs plus the
    # exact product and three accumulations; 16 search steps of K compares for the equal-count start; one final pass
    passes = mean_it + 1
    ops = M * N * (passes * (2 * (K - 1) + 10) + 16 * 2 * K + 2 * (K - 1) + 10)
    tops = ops / (sec / args.steps) / 1e12
    cpu = None
    if not args.no_cpu_baseline:
        cpu = {"value": (t_split + max(t_rows, 0.0) * M / len(rows)) * 1e3, "unit": "ms per layer", "cores": 1, "kind": "oracle",
               "sample": f"split of the whole matrix ({t_split:.2f} s) + Lloyd iterations on {len(rows)} of {M} rows ({t_rows:.2f} s), scaled to all rows; numpy, one thread"}
    out = {
        "metric": "ms per weight matrix quantised (Dense-and-Sparse split + sensitivity-weighted k-means)", "value": ms, "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "i64", "data": "synthetic",
        "config": {"workload": args.workload, "shape": f"{M}x{N}", "bits": bits, "outlier_share": of, "sensitive_share": sf,
                   "n_lo": n_lo, "n_hi": n_hi, "n_sens": n_sens, "max_updates": max_iter, "seed": SEED},
        "mean_updates_per_row": mean_it, "max_updates_seen": int(iters.max().item()), "extracted": nnz,
        "weights_per_second": M * N / (sec / args.steps), "parity": "bit-exact on the split and on sampled rows",
        "host_wall_s_timed_region": wall,
        "roofline": {"bound": "alu", "achieved": tops, "peak": ALU_PEAK_TOPS, "unit": "TOP/s", "frac": tops / ALU_PEAK_TOPS, "traffic": None,
                     "kernel": f"sqllm::quant_kmeans_kernel<{bits},*> (80-90 % of the call; the 7 split kernels are timed with it)",
                     "note": "operations of the plain method (a pass over all weights per update); the kernel sorts the row and moves boundaries instead",
                     "algorithmic_lane_ops_per_launch": ops},
        "cpu_baseline": cpu,
    }
    if args.workload == "llama65b_mlp_pair_3bit" and not args.no_extras:
        # the two other headline figures, measured by the same process after the line's own figures are final; a failure here
        # is reported in place and leaves the line as it is
        del ring, dev
        torch.cuda.empty_cache()
        extras = {}
        try:
            extras["llama7b_mlp_pair_3bit"] = extra_matvec_workload(args, "llama7b_mlp_pair_3bit")
            a2 = argparse.Namespace(**vars(args))
            a2.workload, a2.steps, a2.warmup, a2.no_cpu_baseline = "llama7b_decode_step_3bit_multi_step", 20, 3, True
            d = bench_decode_step(a2, emit=False, fp16=False)
            extras["llama7b_decode_step_3bit_multi_step"] = {"workload": a2.workload, "us_per_token_equivalent": d["value"], "us_per_matvec": d["us_per_matvec"],
                                                             "effective_gbs": d["effective_gbs"], "roofline_frac": d["roofline"]["frac"],
                                                             "entry_point": d["config"]["entry_point"], "replay_stats_ms_for_K_steps": d["replay_stats_ms_for_K_steps"]}
        except (Exception, SystemExit) as e:   # the default line must not depend on the extras
            extras["error"] = repr(e)
        out["extras"] = extras
    print(json.dumps(out))


# App. C ablation: the balanced CSR kernel against the standard one-thread-per-row kernel, under row skew
CSR_ABLATION = {
    # name: (M, N, bits, sparse share)
    "csr_ablation_llama7b_up": (11008, 4096, 3, 0.0045),
    "csr_ablation_llama65b_attn": (8192, 8192, 3, 0.0045),
}


# Full batch-1 decode step of a 7B-shaped model (the linear layers only): 32 blocks x (q, k, v, o 4096x4096; gate, up
# 11008x4096; down 4096x11008), every one of the 224 layers with its own seeded weights resident in HBM (2.6 GB), one
# step = the 224 matvecs back to back on one stream.
DECODE_STEP = {
    # name: (blocks, layer shapes of one block, bits, frac, skew)
    "llama7b_decode_step_3bit": (32, [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)], 3, 0.0045, (0.10, 0.50)),
    "llama7b_decode_step_4bit": (32, [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)], 4, 0.0045, (0.10, 0.50)),
    # projections that share an input stacked row-wise (q,k,v -> 12288 rows; gate,up -> 22016 rows): 128 launches
    "llama7b_decode_step_3bit_stacked": (32, [(12288, 4096), (4096, 4096), (22016, 4096), (4096, 11008)], 3, 0.0045, (0.10, 0.50)),
    # the same 224 layers through sqllm_dense_sparse_matvec_multi: one call per decoder block (two launches: the six 4096-wide
    # layers, the 11008-wide one), or one call for the whole step (14 launches of 16 layers).  The matvecs of the synthetic step
    # do not depend on each other.
    "llama7b_decode_step_3bit_multi_block": (32, [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)], 3, 0.0045, (0.10, 0.50)),
    "llama7b_decode_step_3bit_multi_step": (32, [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)], 3, 0.0045, (0.10, 0.50)),
    # one call per group of projections that are independent in a real decoder block too: (q, k, v), (o), (gate, up), (down)
    "llama7b_decode_step_3bit_multi_groups": (32, [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)], 3, 0.0045, (0.10, 0.50)),
    "llama7b_decode_step_4bit_multi_step": (32, [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)], 4, 0.0045, (0.10, 0.50)),
}
MULTI_GROUPS = [3, 1, 2, 1]


def committed_traffic(workload, no_plan):
    """HBM bytes per matvec from the rocprofv3 counter summary committed for this workload, or None"""
    tpath = os.path.join(ROOT, "profiles", "traffic_" + workload + ".json")
    if not os.path.exists(tpath):
        return None
    try:
        return json.load(open(tpath)).get("hbm_bytes_per_launch_no_plan" if no_plan else "hbm_bytes_per_launch")
    except Exception:
        return None


def bench_decode_step(args, emit=True, fp16=True):
    import numpy as np
    import torch
    import gen
    import oracle   # parity gate and cpu_baseline leg only
    import paper_2306_07629_amd as sq

    blocks, shapes, bits, frac, skew = DECODE_STEP[args.workload]
    checked = sorted({0, blocks // 2 - 1, blocks - 1})          # blocks whose layers are compared with the oracle
    dev, step_bytes, worst, kept = [], 0, 0.0, []
    t_gen = time.perf_counter()
    for b in range(blocks):
        for li, (M, N) in enumerate(shapes):
            L = gen.make_layer(M, N, bits, frac=frac, skew=skew, B=1, seed=gen.layer_seed(SEED, 4, b * len(shapes) + li))
            D = sq.DeviceLayer(L)
            if not args.no_plan:
                D.build_plan()
            step_bytes += sq.sqllm_algorithmic_bytes(L.M, L.N, L.bits, L.nnz, 1)
            if b in checked:
                y = D.matvec().cpu().numpy().view(np.float16).astype(np.float64)
                y_ref, absdot = oracle.layer_matvec(L)
                ratio = float(np.max(np.abs(y - y_ref) / (2e-3 * absdot)))
                if not (ratio <= 1.0):
                    print(f"bench.py: parity FAILED for block {b} layer {li} ({M}x{N}): worst err/bound {ratio}", file=sys.stderr)
                    sys.exit(4)
                worst = max(worst, ratio)
                if b == 0:
                    kept.append(L)                             # the cpu_baseline sample
            dev.append(D)
            del L
        print(f"bench.py: block {b + 1}/{blocks} generated and uploaded ({time.perf_counter() - t_gen:.0f} s)", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    n_layers = len(dev)

    multi = next((m for m in ("multi_block", "multi_step", "multi_groups") if args.workload.endswith("_" + m)), None)
    if multi:
        sizes = {"multi_block": [len(shapes)], "multi_step": [n_layers], "multi_groups": MULTI_GROUPS}[multi]
        calls, i = [], 0
        while i < n_layers:
            for n in sizes:
                calls.append(sq.layer_descriptors([D.descriptor() for D in dev[i:i + n]]))
                i += n
        # the multi-layer call must reproduce the bits of the single-layer entry point (itself checked against the oracle above)
        for D in dev:
            D.matvec()
        torch.cuda.synchronize()
        want = [D.y.clone() for D in dev]
        for D in dev:
            D.y.zero_()
        for c in calls:
            sq.sqllm_dense_sparse_matvec_multi(c)
        torch.cuda.synchronize()
        if not all(torch.equal(D.y, w) for D, w in zip(dev, want)):
            print("bench.py: the multi-layer call does not reproduce the single-layer results", file=sys.stderr)
            sys.exit(4)
        del want

        def step(_s):
            for c in calls:
                sq.sqllm_dense_sparse_matvec_multi(c)
    else:
        def step(_s):
            for D in dev:
                D.matvec()

    G = not args.no_graph
    sec, wall = time_steps(torch, step, args.steps, args.warmup, G, args.replays, tag="cold")
    us_step = sec / args.steps * 1e6
    gbs = step_bytes * args.steps / sec / 1e9

    # fp16 baseline: the same 224 shapes as fp16 matrices (13 GB), library GEMV and the own kernel
    us_torch = us_own = None
    if fp16:
        ws = [(torch.randn(M, N, device="cuda", dtype=torch.float16) * 0.02) for _ in range(blocks) for M, N in shapes]
        xs = {N: torch.randn(N, device="cuda", dtype=torch.float16) for _, N in shapes}
        ys = {M: torch.zeros(M, device="cuda", dtype=torch.float16) for M, _ in shapes}

        def step_torch(_s):
            for w in ws:
                torch.mv(w, xs[w.shape[1]], out=ys[w.shape[0]])

        def step_own(_s):
            for w in ws:
                sq.sqllm_fp16_gemv(w.shape[0], w.shape[1], 1, w, xs[w.shape[1]], ys[w.shape[0]])

        fsteps = max(3, args.steps // 4)
        us_torch = time_steps(torch, step_torch, fsteps, 1, G)[0] / fsteps * 1e6
        us_own = time_steps(torch, step_own, fsteps, 1, G)[0] / fsteps * 1e6
        del ws

    cpu = None
    if not args.no_cpu_baseline:
        times = []
        for _ in range(3):
            t0 = time.perf_counter()
            for L in kept:
                oracle.layer_matvec(L)
            times.append(time.perf_counter() - t0)
        med = sorted(times)[1]
        cpu = {"value": med * blocks * 1e6, "unit": "us per token-equivalent", "cores": oracle.threads(), "kind": "oracle",
               "sample": f"the {len(kept)} layers of block 0, median of 3 passes, scaled by {blocks} blocks; fp64, OpenMP over rows"}

    out = {
        "metric": f"us per token-equivalent: the {n_layers} dense+sparse matvecs ({bits}-bit LUT + {100 * frac:g}% CSR) of the linear layers of a 7B-shaped decode step, back to back on one stream",
        "value": us_step, "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": us_step * 1e-3,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "blocks": blocks, "layers_per_block": [f"{M}x{N}" for M, N in shapes], "bits": bits, "sparse_frac": frac,
                   "skew": skew, "batch": 1, "seed": SEED, "distinct_layers_resident": n_layers, "resident_gb": step_bytes / 1e9,
                   "parity_checked_blocks": checked, "matvecs_per_step": n_layers, "sparse_term": "CSR arrays" if args.no_plan else "plan built once per matrix",
                   "entry_point": "sqllm_dense_sparse_matvec_multi, one call per " + {"multi_block": "decoder block", "multi_step": "step", "multi_groups": "group of independent projections (q,k,v | o | gate,up | down)"}[multi] if multi else "sqllm_dense_sparse_matvec, one call per layer"},
        "replay_stats_ms_for_K_steps": REPLAY_STATS.get("cold"),
        "us_per_matvec": us_step / n_layers, "effective_gbs": gbs, "pct_of_hbm_roofline": 100.0 * gbs / HBM_PEAK_GBS,
        "fp16_step_us": {"own_kernel": us_own, "torch_mv": us_torch}, "speedup_vs_fp16": min(us_own, us_torch) / us_step if fp16 else None,
        "parity_worst_err_over_bound": worst, "launch_mode": "hip_graph_replay" if G else "python_ctypes", "host_wall_s_timed_region": wall,
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                     "traffic": committed_traffic(args.workload, args.no_plan),      # per matvec, like algorithmic_bytes_per_launch
                     "kernel": f"sqllm::matvec{'_planned' if not args.no_plan else ''}{'_multi' if multi else ''}_kernel<{bits},*>",
                     "algorithmic_bytes_per_launch": step_bytes / n_layers},
        "cpu_baseline": cpu,
    }
    del dev
    torch.cuda.empty_cache()
    if emit:
        print(json.dumps(out))
    return out


def bench_csr_ablation(args):
    import numpy as np
    import torch
    import gen
    import oracle   # parity gate only
    import paper_2306_07629_amd as sq

    M, N, bits, frac = CSR_ABLATION[args.workload]
    rows = []
    for label, skew in (("uniform", None), ("10% of rows hold 50%", (0.10, 0.50)), ("1% of rows hold 30%", (0.01, 0.30)), ("0.1% of rows hold 10%", (0.001, 0.10))):
        L = gen.make_layer(M, N, bits, frac=frac, skew=skew, B=1, seed=gen.layer_seed(SEED, 7, 0))
        D = sq.DeviceLayer(L)
        y_ref, absdot = oracle.layer_matvec(L)
        y_ref_s, absdot_s = oracle.layer_matvec(L, dense=False)
        for fn, ref, ad in ((lambda: D.matvec(), y_ref, absdot), (lambda: D.csr_spmv(), y_ref_s, absdot_s), (lambda: D.csr_spmv(rowwise=True), y_ref_s, absdot_s),
                            (lambda: (D.lut_gemv(), D.csr_spmv(accumulate=1, rowwise=True))[1], y_ref, 2 * absdot)):
            y = fn().cpu().numpy().view(np.float16).astype(np.float64)
            if not (np.abs(y - ref) <= 2e-3 * ad).all():
                print(f"bench.py: parity FAILED in the CSR ablation ({label})", file=sys.stderr)
                sys.exit(4)
        nbytes = sq.sqllm_algorithmic_bytes(M, N, bits, L.nnz, 1)
        copies = max(2, int(np.ceil(args.footprint_gb * 1e9 / nbytes)))
        ring = [D] + [D.clone_weights() for _ in range(copies - 1)]
        t = {}
        for name, fn in (("dense_only", lambda s: ring[s % copies].lut_gemv()),
                         ("fused_balanced", lambda s: ring[s % copies].matvec()),
                         ("dense_then_standard", lambda s: (ring[s % copies].lut_gemv(), ring[s % copies].csr_spmv(accumulate=1, rowwise=True))),
                         ("sparse_balanced", lambda s: ring[s % copies].csr_spmv()),
                         ("sparse_standard", lambda s: ring[s % copies].csr_spmv(rowwise=True))):
            sec, _ = time_steps(torch, fn, args.steps, args.warmup, not args.no_graph)
            t[name] = sec / args.steps * 1e6
        # the same fused call with the one-time plan of the sparse term (sqllm_csr_plan_build) in place of the CSR arrays
        for r in ring:
            r.build_plan()
        y = D.matvec().cpu().numpy().view(np.float16).astype(np.float64)
        if not (np.abs(y - y_ref) <= 2e-3 * absdot).all():
            print(f"bench.py: parity FAILED in the CSR ablation with a plan ({label})", file=sys.stderr)
            sys.exit(4)
        sec, _ = time_steps(torch, lambda s: ring[s % copies].matvec(), args.steps, args.warmup, not args.no_graph)
        t["fused_planned"] = sec / args.steps * 1e6
        counts = np.diff(L.rowptr)
        rows.append({"skew": label, "max_row_nnz": int(counts.max()), "mean_row_nnz": float(counts.mean()), **{k: round(v, 2) for k, v in t.items()},
                     "sparse_overhead_balanced_pct": round(100 * (t["fused_balanced"] / t["dense_only"] - 1), 1),
                     "sparse_overhead_planned_pct": round(100 * (t["fused_planned"] / t["dense_only"] - 1), 1),
                     "sparse_overhead_standard_pct": round(100 * (t["dense_then_standard"] / t["dense_only"] - 1), 1)})
        del ring, D
        torch.cuda.empty_cache()
    worst = rows[-1]
    print(json.dumps({"metric": "us per matvec: balanced (fused) against standard one-thread-per-row CSR kernel", "value": worst["fused_balanced"], "unit": "us",
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": worst["fused_balanced"] * 1e-3, "higher_is_better": False,
                      "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": args.workload, "shape": f"{M}x{N}", "bits": bits, "sparse_frac": frac, "seed": SEED}, "rows": rows}))


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--replays", type=int, default=11, help="timed replays of the captured K steps; the median is reported")
    ap.add_argument("--workload", default="llama65b_mlp_pair_3bit", choices=sorted(WORKLOADS) + sorted(QUANT_WORKLOADS) + sorted(CSR_ABLATION) + sorted(DECODE_STEP))
    ap.add_argument("--footprint-gb", type=float, default=1.1, help="bytes of distinct weight copies to rotate over")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="issue every launch from Python instead of replaying a HIP graph")
    ap.add_argument("--no-extras", action="store_true", help="default workload only: do not add the 7B MLP pair and the 7B decode step as extra keys")
    ap.add_argument("--no-plan", action="store_true", help="sparse term straight from the CSR arrays instead of from the one-time plan (sqllm_csr_plan_build)")
    return ap.parse_args()


def device_info(torch):
    """what the runtime reports about the GPU the figures come from (clocks cannot be pinned by an ordinary user)"""
    p = torch.cuda.get_device_properties(0)
    info = {"name": p.name, "compute_units": p.multi_processor_count, "memory_gb": round(p.total_memory / 1e9, 1)}
    for k in ("clock_rate", "memory_clock_rate", "gcnArchName", "L2_cache_size"):
        if hasattr(p, k):
            info[k] = getattr(p, k)
    return info


REPLAY_STATS = {}


def time_steps(torch, fn, steps, warmup, use_graph=True, replays=11, tag=None):
    """W untimed + exactly K timed calls of fn(step), bracketed by device synchronisation, timed with HIP
    events on the launch stream.  With use_graph the K launches are first captured into one HIP graph
    (still K separate kernel launches, executed in order on one stream) so that the Python/ctypes cost of
    issuing a launch (about 10 us, more than the kernel itself) is not what is measured; the graph is replayed
    `replays` times, each replay timed by its own event pair, and the MEDIAN replay is returned (seconds for the
    K steps) with the host wall time of that many steps.  Minimum and maximum go to REPLAY_STATS[tag]."""
    for s in range(warmup):
        fn(s)
    torch.cuda.synchronize()
    if use_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for s in range(steps):
                    fn(warmup + s)
            torch.cuda.synchronize()
            for _ in range(3):                   # untimed replays: the first uploads the graph, the others let the clocks settle
                graph.replay()
            torch.cuda.synchronize()
            secs, walls = [], []
            for _ in range(max(1, replays)):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                t0 = time.perf_counter()
                e0.record()
                graph.replay()
                e1.record()
                torch.cuda.synchronize()
                walls.append(time.perf_counter() - t0)
                secs.append(e0.elapsed_time(e1) * 1e-3)
        order = sorted(range(len(secs)), key=lambda i: secs[i])
        mid = order[len(order) // 2]
        if tag:
            REPLAY_STATS[tag] = {"replays": len(secs), "median_ms": secs[mid] * 1e3, "min_ms": min(secs) * 1e3, "max_ms": max(secs) * 1e3}
        return secs[mid], walls[mid]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for s in range(steps):
        fn(warmup + s)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if tag:
        REPLAY_STATS[tag] = {"replays": 1, "median_ms": e0.elapsed_time(e1), "min_ms": e0.elapsed_time(e1), "max_ms": e0.elapsed_time(e1)}
    return e0.elapsed_time(e1) * 1e-3, wall


def extra_matvec_workload(args, name):
    """cold, graph-replayed us per matvec of another workload of WORKLOADS (parity gate included), for the extras of the default line"""
    import numpy as np
    import torch
    import gen
    import oracle   # parity gate only
    import paper_2306_07629_amd as sq
    shapes, bits, frac, skew, B = WORKLOADS[name]
    dev, step_bytes = [], 0
    for li, (M, N) in enumerate(shapes):
        L = gen.make_layer(M, N, bits, frac=frac, skew=skew, B=B, seed=gen.layer_seed(SEED, 2, li))
        D = sq.DeviceLayer(L)
        if not args.no_plan:
            D.build_plan()
        y = D.matvec().cpu().numpy().view(np.float16).astype(np.float64)
        y_ref, absdot = oracle.layer_matvec(L)
        if not (np.abs(y - y_ref) <= 2e-3 * absdot).all():
            raise RuntimeError(f"parity failed for {name} layer {M}x{N}")
        step_bytes += sq.sqllm_algorithmic_bytes(L.M, L.N, L.bits, L.nnz, L.B)
        dev.append(D)
    copies = max(2, int(np.ceil(args.footprint_gb * 1e9 / step_bytes)))
    ring = [[D] + [D.clone_weights() for _ in range(copies - 1)] for D in dev]

    def step(s):
        for r in ring:
            r[s % copies].matvec()

    sec, _ = time_steps(torch, step, args.steps, args.warmup, not args.no_graph, args.replays)
    us = sec / (args.steps * len(shapes)) * 1e6
    gbs = step_bytes * args.steps / sec / 1e9
    del ring, dev
    torch.cuda.empty_cache()
    return {"workload": name, "us_per_matvec": us, "effective_gbs": gbs, "roofline_frac": gbs / HBM_PEAK_GBS}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path is a single-GPU matvec); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import gen
    import paper_2306_07629_amd as sq

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.workload in CSR_ABLATION:
        if args.steps == 256 and args.warmup == 32:
            args.steps, args.warmup = 200, 20
        return bench_csr_ablation(args)
    if args.workload in DECODE_STEP:
        if args.steps == 256 and args.warmup == 32:
            args.steps, args.warmup = 20, 3
        return bench_decode_step(args)
    if args.workload in QUANT_WORKLOADS:
        if args.steps == 256 and args.warmup == 32:     # the defaults are sized for the microsecond matvecs
            args.steps, args.warmup = 20, 3
        return bench_quantize(args)
    shapes, bits, frac, skew, B = WORKLOADS[args.workload]

    # ---- generate, upload, check parity against the oracle before any timing
    import oracle  # only for the parity gate and the cpu_baseline leg
    layers, dev, worst = [], [], 0.0
    for li, (M, N) in enumerate(shapes):
        L = gen.make_layer(M, N, bits, frac=frac, skew=skew, B=B, seed=gen.layer_seed(SEED, 2, li))
        D = sq.DeviceLayer(L)
        if not args.no_plan:
            D.build_plan()                                       # once per (static) weight matrix, outside every timed region
        y = D.matvec().cpu().numpy().view(np.float16).astype(np.float64)
        y_ref, absdot = oracle.layer_matvec(L)
        ratio = float(np.max(np.abs(y - y_ref) / (2e-3 * absdot)))
        if not (ratio <= 1.0):
            print(f"bench.py: parity FAILED for layer {M}x{N}: worst err/bound {ratio}", file=sys.stderr)
            sys.exit(4)
        worst = max(worst, ratio)
        layers.append(L); dev.append(D)

    alg_bytes = [sq.sqllm_algorithmic_bytes(L.M, L.N, L.bits, L.nnz, L.B) for L in layers]
    step_bytes = sum(alg_bytes)
    copies = max(2, int(np.ceil(args.footprint_gb * 1e9 / step_bytes)))
    ring = [[D] + [D.clone_weights() for _ in range(copies - 1)] for D in dev]
    torch.cuda.synchronize()

    def step_cold(s):
        c = s % copies
        for r in ring:
            r[c].matvec()

    def step_warm(s):
        for D in dev:
            D.matvec()

    G = not args.no_graph
    sec_cold, wall_cold = time_steps(torch, step_cold, args.steps, args.warmup, G, args.replays, tag="cold")
    sec_warm, _ = time_steps(torch, step_warm, args.steps, args.warmup, G, 3)
    launches = args.steps * len(shapes)
    touched = len({(args.warmup + st) % copies for st in range(args.steps)})
    us_per_matvec = sec_cold / launches * 1e6
    gbs = step_bytes * args.steps / sec_cold / 1e9

    # ---- single-launch latency: an event pair around ONE launch of the first layer after the device went idle
    # (cold copy each time), median of 15; contains what a back-to-back stream hides: launch ramp, first data, drain
    singles = []
    for i in range(15):
        torch.cuda.synchronize()
        time.sleep(0.002)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ring[0][(i + 1) % copies].matvec()
        e1.record()
        torch.cuda.synchronize()
        singles.append(e0.elapsed_time(e1) * 1e3)
    single_launch_us = sorted(singles)[len(singles) // 2]

    # ---- fp16 baselines on the same shapes (own kernel and the vendor library through torch), cold as well
    fp16_bytes = sum(M * N * 2 + (M + N) * 2 for M, N in shapes)
    fcopies = max(2, int(np.ceil(args.footprint_gb * 1e9 / fp16_bytes)))
    wring = [[(torch.randn(M, N, device="cuda", dtype=torch.float16) * 0.02) for _ in range(fcopies)] for M, N in shapes]
    # the baselines see the same batch: x[N][B] -> y[M][B] (torch.mv for one column, torch.mm for more)
    xs = [torch.randn(N, B, device="cuda", dtype=torch.float16) for M, N in shapes]
    ys = [torch.zeros(M, B, device="cuda", dtype=torch.float16) for M, N in shapes]
    xv = [x[:, 0].contiguous() for x in xs]
    yv = [y[:, 0].contiguous() for y in ys]

    def step_fp16_own(s):
        c = s % fcopies
        for k, (M, N) in enumerate(shapes):
            sq.sqllm_fp16_gemv(M, N, B, wring[k][c], xs[k], ys[k])

    def step_fp16_torch(s):
        c = s % fcopies
        for k in range(len(shapes)):
            if B == 1:
                torch.mv(wring[k][c], xv[k], out=yv[k])
            else:
                torch.mm(wring[k][c], xs[k], out=ys[k])

    fsteps = max(20, args.steps // 4)
    sec_f_torch, _ = time_steps(torch, step_fp16_torch, fsteps, 10, G)
    us_f_torch = sec_f_torch / (fsteps * len(shapes)) * 1e6
    if B == 1:
        sec_f_own, _ = time_steps(torch, step_fp16_own, fsteps, 10, G)
        us_f_own = sec_f_own / (fsteps * len(shapes)) * 1e6
        us_f = min(us_f_own, us_f_torch)
    else:
        # the library's fp16 kernel is a one-column streaming design (parity baseline); at wider batches the vendor
        # GEMM is the fp16 baseline
        us_f_own, us_f = None, us_f_torch
    del wring

    # ---- HBM traffic per launch measured with rocprofv3 counters, if a summary is committed
    traffic = committed_traffic(args.workload, args.no_plan)

    # ---- CPU baseline: the oracle as it stands, on this machine's host cores, bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        times = []
        t_begin = time.perf_counter()
        reps = 0
        while reps < 3 or (time.perf_counter() - t_begin < 10.0 and reps < 200):   # about 10 s of CPU work
            t0 = time.perf_counter()
            for L in layers:
                oracle.layer_matvec(L)
            times.append(time.perf_counter() - t0)
            reps += 1
        med = sorted(times)[len(times) // 2]
        cpu = {"value": med / len(shapes) * 1e6, "unit": "us per matvec", "cores": oracle.threads(), "kind": "oracle",
               "sample": f"{reps} full passes over the same {len(shapes)} layers (median), fp64, OpenMP over rows",
               "gbs": step_bytes / med / 1e9}

    # ---- context: what a plain device-to-device copy of 1 GiB reaches on this machine (bytes read + bytes written per second)
    big = [torch.ones(1 << 28, dtype=torch.int32, device="cuda") for _ in range(3)]
    sec_cp, _ = time_steps(torch, lambda s_: big[2].copy_(big[s_ % 2]), 8, 2, G, 3)
    copy_gbs = 8 * 2 * (1 << 30) / sec_cp / 1e9
    del big

    out = {
        "metric": f"us per dense+sparse matvec ({bits}-bit LUT + {100 * frac:g}% CSR), effective HBM GB/s in roofline",
        "value": us_per_matvec, "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec_cold / args.steps * 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "layers": [f"{M}x{N}" for M, N in shapes], "bits": bits, "sparse_frac": frac,
                   "skew": skew, "batch": B, "seed": SEED, "storage": "fp16 tables / CSR values / x / y, fp32 accumulation",
                   "sparse_term": "CSR arrays" if (args.no_plan or B > 1) else "plan built once per matrix by sqllm_csr_plan_build", "weight_copies_allocated": copies,
                   "weight_copies_touched_in_timed_region": touched, "working_set_gb": step_bytes * touched / 1e9, "matvecs_per_step": len(shapes)},
        "replay_stats_ms_for_K_steps": REPLAY_STATS.get("cold"),
        "effective_gbs": gbs, "pct_of_hbm_roofline": 100.0 * gbs / HBM_PEAK_GBS, "us_per_step": sec_cold / args.steps * 1e6,
        "single_launch_after_idle_us": single_launch_us,
        "warm_us_per_matvec": sec_warm / launches * 1e6, "warm_effective_gbs": step_bytes * args.steps / sec_warm / 1e9,
        "fp16_gemv_us": {"own_kernel": us_f_own, "torch_mv" if B == 1 else "torch_mm": us_f_torch}, "speedup_vs_fp16": us_f / us_per_matvec,
        "parity_worst_err_over_bound": worst, "launch_mode": "hip_graph_replay" if G else "python_ctypes", "host_wall_s_timed_region": wall_cold,
        "device": device_info(torch), "context_device_copy_1gib_gbs_read_plus_write": copy_gbs,
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                     "traffic": traffic,
                     "kernel": (f"sqllm::matvec_kernel<{bits},*>" if args.no_plan else f"sqllm::matvec_planned_kernel<{bits},*>") if B == 1 else f"sqllm::matvec_b16_kernel<{bits},*>",
                     "algorithmic_bytes_per_launch": step_bytes / len(shapes)},
        "cpu_baseline": cpu,
    }
    if args.workload == "llama65b_mlp_pair_3bit" and not args.no_extras:
        # the two other headline figures, measured by the same process after the line's own figures are final; a failure here
        # is reported in place and leaves the line as it is
        del ring, dev
        torch.cuda.empty_cache()
        extras = {}
        try:
            extras["llama7b_mlp_pair_3bit"] = extra_matvec_workload(args, "llama7b_mlp_pair_3bit")
            a2 = argparse.Namespace(**vars(args))
            a2.workload, a2.steps, a2.warmup, a2.no_cpu_baseline = "llama7b_decode_step_3bit_multi_step", 20, 3, True
            d = bench_decode_step(a2, emit=False, fp16=False)
            extras["llama7b_decode_step_3bit_multi_step"] = {"workload": a2.workload, "us_per_token_equivalent": d["value"], "us_per_matvec": d["us_per_matvec"],
                                                             "effective_gbs": d["effective_gbs"], "roofline_frac": d["roofline"]["frac"],
                                                             "entry_point": d["config"]["entry_point"], "replay_stats_ms_for_K_steps": d["replay_stats_ms_for_K_steps"]}
        except (Exception, SystemExit) as e:   # the default line must not depend on the extras
            extras["error"] = repr(e)
        out["extras"] = extras
    print(json.dumps(out))


if __name__ == "__main__":
    main()
