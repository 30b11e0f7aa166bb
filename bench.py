#!/usr/bin/env python3
"""Benchmark of the SLIDE training step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config i]

A step is one pass of the whole hot path (hidden layer, hashing, bucket lookup + union, forward over
the active set, sparse backward, row-sparse Adam) over one fresh synthetic batch already resident in
HBM.  Prints one JSON line: whole-job samples/s, the HBM roofline of the dominant kernel (row
gradient + Adam on the touched output rows, timed with HIP events inside the library on the step's
own stream, on the K steps that follow the timed ones), and the CPU oracle timed on the host cores on
a bounded sample of the same workload.  `value` charges every step its share of the periodic table
rebuild; the rebuild-free figure is reported beside it.
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

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak

# HBM bytes per launch from rocprofv3 --pmc runs (FETCH_SIZE + WRITE_SIZE, scaled by the same counters
# on the library's plain copy kernel).  They are profile results, not measurements of this run: each
# entry names the summary under profiles/ it was copied from, and is dropped (None) when a kernel it
# covers has changed since that profile was taken.
PROFILED_TRAFFIC = {
    "cfg2-670k": {"update_kernel": 777.6e6, "forward_kernel": 209.9e6,
                  "source": "profiles/cfg2-670k_step_kernels.md (FETCH_SIZE x 2048 + WRITE_SIZE x 1024 bytes per "
                            "dispatch, mean of 45 dispatches, both factors from the copy kernel in the same runs)"},
    "cfg1-shard167k": {"update_kernel": 212.2e6, "forward_kernel": 51.7e6,
                       "source": "profiles/cfg1-shard167k_step_kernels.md (mean of 45 dispatches)"},
    "cfg4-825m": {"update_kernel": 587.0e6, "forward_kernel": 39.0e6,
                  "source": "profiles/cfg4-825m_step_kernels.md (mean of 45 dispatches)"},
    "cfg3-wide325k": {"update_kernel": 424.7e6, "forward_kernel": 109.4e6,
                      "source": "profiles/cfg3-wide325k_step_kernels.md (update_sliced_kernel; mean of 45 dispatches "
                                "of a workload whose touched rows shrink step by step)"},
    "cfg5-text8-shape": {"update_kernel": 2056.5e6, "forward_kernel": 1072.7e6,
                         "source": "profiles/cfg5-text8-shape_step_kernels.md (mean of 45 dispatches)"},
}


def algorithmic_bytes_update(U: float, A: float, U1: float, nnz: float, B: int, H: int) -> float:
    """Bytes the update launch (gradient + Adam on every touched row) must move: each touched row of
    W2 / W1 and of its momentum and velocity read once and written once (6 rows of H floats), for W2
    also the bias (6 floats); per row its list header (16 bytes); per (sample, row) pair its sample
    index, coefficient index and coefficient (12 bytes); the hidden activations and their gradient
    (B*H floats each) read once from HBM."""
    row = H * 4.0
    return U * (6 * row + 24 + 16) + U1 * (6 * row + 16) + 12.0 * (A + nnz) + 2.0 * B * row


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="0..8; 2 = the 670K-class model the metric is quoted on")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-steps", type=int, default=20, help="oracle steps timed for cpu_baseline (0 = skip)")
    ap.add_argument("--cpu-steps-1thread", type=int, default=2,
                    help="oracle steps timed on a single thread after those (0 = skip)")
    ap.add_argument("--breakdown", action="store_true", help="bracket every stage (not only the two row-gather launches) in the roofline pass")
    ap.add_argument("--sample-budget", type=int, default=0,
                    help="retrieved neurons kept per sample (0 = all, the configuration the metric is quoted on)")
    ap.add_argument("--sample-fill", action="store_true", help="fill an unmet budget with uniformly drawn neurons")
    ap.add_argument("--rebuild-every", type=int, default=None, help="override the workload's rebuild schedule")
    ap.add_argument("--incremental-rebuild", action="store_true",
                    help="scheduled rebuilds hash only the rows updated since the last build")
    ap.add_argument("--predict-topk", type=int, default=0, metavar="K",
                    help="only time slide_predict (retrieved neurons, then all neurons) on one batch of the "
                         "workload and print its own JSON line")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="only run the library's plain copy kernel on MIB mebibytes (10 launches) and print "
                         "its bandwidth: the yardstick for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2201_12667_amd import slide, synth

    if args.calibrate_copy:
        n = args.calibrate_copy << 20
        src = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        st = torch.cuda.current_stream().cuda_stream
        for _ in range(3):
            slide.debug_copy(dst, src, st)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            slide.debug_copy(dst, src, st)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        print(json.dumps({"kernel": "copy_kernel", "bytes_read": n, "bytes_written": n, "avg_launch_ms": ms,
                          "GBs": 2 * n / (ms * 1e-3) / 1e9}))
        return 0

    wl = synth.config(args.config)
    if args.sample_budget:
        import dataclasses
        wl = dataclasses.replace(wl, sample_budget=args.sample_budget, sample_fill=args.sample_fill)
    if args.rebuild_every is not None or args.incremental_rebuild:
        import dataclasses
        wl = dataclasses.replace(wl, incremental_rebuild=args.incremental_rebuild,
                                 rebuild_every=wl.rebuild_every if args.rebuild_every is None else args.rebuild_every)
    gen = synth.Generator(wl, args.seed)
    weights, hp = gen.weights(), gen.hash_params()
    model = slide.Slide(slide.config_from_workload(wl), weights, hp)
    if args.predict_topk:
        model.build_tables()
        db = model.to_device(gen.batch(0))
        res = {"kernel": "slide_predict", "workload": wl.name, "batch": wl.batch, "topk": args.predict_topk}
        for mode, name in ((0, "retrieved_neurons_ms"), (1, "all_neurons_ms")):
            for _ in range(2):
                model.predict(db, args.predict_topk, mode)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(10):
                model.predict(db, args.predict_topk, mode)
            torch.cuda.synchronize()
            res[name] = (time.perf_counter() - t0) / 10 * 1e3
        flop = 2.0 * wl.batch * wl.num_classes * wl.hidden_dim
        res["all_neurons_TFLOPs"] = flop / (res["all_neurons_ms"] * 1e-3) / 1e12
        res["fp32_matrix_peak_TFLOPs"] = 157.3
        if args.cpu_steps > 0:                       # the oracle beside it, on a bounded sample of the batch
            from oracle import slide_oracle as so
            orc = so.SlideOracle(input_dim=wl.input_dim, hidden_dim=wl.hidden_dim, num_classes=wl.num_classes,
                                 hash_kind=wl.hash_kind, K=wl.K, L=wl.L, bucket_cap=wl.bucket_cap, rebuild_every=0,
                                 lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, dwta_bin=wl.dwta_bin,
                                 overflow_policy=wl.overflow_policy, weights=weights, hash_params=hp)
            orc.build_tables()
            hb = gen.batch(0)
            ns = min(wl.batch, 32)
            xe, ye = int(hb["x_indptr"][ns]) if wl.input_dim else 0, int(hb["y_indptr"][ns])
            sub = {"x_indptr": hb["x_indptr"][:ns + 1], "x_indices": hb["x_indices"][:xe], "x_values": hb["x_values"][:xe],
                   "y_indptr": hb["y_indptr"][:ns + 1], "y_indices": hb["y_indices"][:ye]} if wl.input_dim else \
                  {"hidden": hb["hidden"][:ns], "y_indptr": hb["y_indptr"][:ns + 1], "y_indices": hb["y_indices"][:ye]}
            cpu = {}
            for mode, name in ((0, "retrieved_neurons"), (1, "all_neurons")):
                c0 = time.perf_counter()
                orc.predict(sub, args.predict_topk, mode)
                cpu[name + "_samples_per_s"] = ns / (time.perf_counter() - c0)
            res["cpu_baseline"] = dict(cpu, cores=so.num_threads(), kind="oracle",
                                       sample="the first %d samples of the same batch" % ns)
            res["retrieved_neurons_samples_per_s"] = wl.batch / (res["retrieved_neurons_ms"] * 1e-3)
            res["all_neurons_samples_per_s"] = wl.batch / (res["all_neurons_ms"] * 1e-3)
        print(json.dumps(res))
        return 0

    W, K = args.warmup, args.steps
    # W warm-up steps, K timed steps (the headline), then K more steps with HIP events around the
    # forward and update launches (the roofline figures): the event records stay out of the headline.
    host_batches = [gen.batch(s) for s in range(W + 2 * K)]
    batches = [model.to_device(b) for b in host_batches]
    R = wl.rebuild_every
    i_fwd, i_upd, i_reb = (slide.STAGES.index(n) for n in ("forward", "update", "rebuild"))

    model.build_tables()
    for s in range(W):
        model.train_step(batches[s])
    torch.cuda.synchronize()
    assert model.status() == 0, "device flagged bad batch data"
    model.reset_stats()
    model.profile(1 << i_reb)                            # (only brackets a rebuild, if the schedule fires one)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(W, W + K):
        model.train_step(batches[s])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms, n = model.profile_read()
    rebuilds_in_region = int(n[i_reb])
    rebuild_in_region_ms = float(ms[i_reb]) / max(rebuilds_in_region, 1)
    assert rebuilds_in_region == sum(1 for t in range(W + 1, W + K + 1) if R and t % R == 0)
    st_timed = model.stats()
    loss = float(model.d_loss.item())
    assert np.isfinite(loss), "loss is not finite"

    # roofline pass: the next K batches, events on the caller's stream around the two row-gather launches
    model.reset_stats()
    model.profile(((1 << slide.NUM_STAGES) - 1) if args.breakdown else ((1 << i_fwd) | (1 << i_upd)))
    for s in range(W + K, W + 2 * K):
        model.train_step(batches[s])
    ms, n = model.profile_read()
    model.profile(0)
    stage_ms = {slide.STAGES[i]: float(ms[i]) / int(n[i]) for i in range(slide.NUM_STAGES) if n[i]} if args.breakdown else None
    st = model.stats()
    steps_done = max(st["sum_steps"], 1)
    A, U, U1 = (st[k] / steps_done for k in ("sum_active_pairs", "sum_unique_out_rows", "sum_unique_in_rows"))
    upd_ms = float(ms[i_upd]) / max(int(n[i_upd]), 1)
    fwd_ms = float(ms[i_fwd]) / max(int(n[i_fwd]), 1)
    nnz_mean = float(np.mean([b["nnz"] for b in batches[W + K:W + 2 * K]]))
    row = wl.hidden_dim * 4.0
    upd_bytes = algorithmic_bytes_update(U, A, U1, nnz_mean, wl.batch, wl.hidden_dim)
    achieved = upd_bytes / (upd_ms * 1e-3) / 1e9

    # a scheduled rebuild of the trained weights, timed on its own (what every R-th step pays)
    torch.cuda.synchronize()
    b0 = time.perf_counter()
    model.build_tables()
    torch.cuda.synchronize()
    build_ms = (time.perf_counter() - b0) * 1e3

    # the practical ceiling: the library's plain copy kernel, 1 GiB read + 1 GiB written, same run
    src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(2):
        slide.debug_copy(dst, src, stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        slide.debug_copy(dst, src, stream)
    e1.record()
    torch.cuda.synchronize()
    copy_GBs = 2.0 * (1 << 30) * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst

    # Headline: the whole hot path including its periodic rebuild.  When the schedule fires inside the
    # timed region the measured time already holds it; otherwise every step is charged 1/R of a rebuild.
    raw_s = t1 - t0
    amort_s = raw_s + (0.0 if (rebuilds_in_region or not R) else K * build_ms * 1e-3 / R)
    step_ms = amort_s * 1e3 / K
    value = wl.batch * K / amort_s
    prof = PROFILED_TRAFFIC.get(wl.name)
    compulsory = 7.0 * row * (U + U1) + 40.0 * A

    out = {
        "metric": "train samples/s (fwd+bwd+Adam), 670K-class SLIDE step",
        "value": value, "unit": "samples/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": step_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "config_index": args.config, "batch": wl.batch,
                   "input_dim": wl.input_dim, "hidden_dim": wl.hidden_dim, "num_classes": wl.num_classes,
                   "hash": "dwta" if wl.hash_kind == synth.HASH_DWTA else "simhash", "K": wl.K, "L": wl.L,
                   "bucket_cap": wl.bucket_cap, "rebuild_every": R,
                   "rebuilds_in_timed_region": rebuilds_in_region,
                   "incremental_rebuild": bool(wl.incremental_rebuild), "seed": args.seed,
                   "sample_budget": wl.sample_budget, "sample_fill": bool(wl.sample_fill)},
        "value_includes": ("the K timed steps" + (" with the %d scheduled rebuild(s) that fell among them" % rebuilds_in_region
                                                  if rebuilds_in_region else
                                                  (" plus K/R of one table rebuild (%.3f ms, measured in this run on the trained "
                                                   "weights; the schedule fires every %d steps, none of the timed ones)" % (build_ms, R)
                                                   if R else " (no rebuild schedule in this workload)"))),
        "ms_per_step_without_rebuild": raw_s * 1e3 / K if not rebuilds_in_region else None,
        "value_without_rebuild": wl.batch * K / raw_s if not rebuilds_in_region else None,
        "table_build_ms": build_ms,
        "roofline": {"bound": "hbm",
                     "kernel": "update_kernel (gradient + Adam on the touched rows of W2 and W1)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": prof["update_kernel"] if prof else None,
                     "traffic_source": prof["source"] if prof else None,
                     "algorithmic_bytes_per_launch": upd_bytes, "avg_launch_ms": upd_ms, "launches": int(n[i_upd]),
                     "timed_on": "the %d steps after the timed region (HIP events on the step's stream)" % K,
                     "copy_ceiling_GBs": copy_GBs, "frac_of_copy_ceiling": achieved / copy_GBs},
        "roofline_forward": {"bound": "hbm",
                             "kernel": "forward_kernel (logits + running soft-max over the gathered rows of W2; "
                                       "the launch also builds the row lists)",
                             "avg_launch_ms": fwd_ms, "launches": int(n[i_fwd]),
                             "gathered_bytes_per_launch": A * row + 16.0 * A,
                             "gathered_GBs": (A * row + 16.0 * A) / (fwd_ms * 1e-3) / 1e9,
                             "distinct_row_bytes_per_launch": U * row,
                             "achieved": U * row / (fwd_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": U * row / (fwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             "traffic": prof["forward_kernel"] if prof else None,
                             "traffic_source": prof["source"] if prof else None},
        "workload_stats": {"active_pairs_per_step": A, "unique_out_rows_per_step": U,
                           "unique_in_rows_per_step": U1,
                           "candidates_per_step": st["sum_candidates"] / steps_done,
                           "overflowed_buckets_at_build": st["overflowed_buckets"], "last_loss": loss},
        "step_bytes": {"compulsory": compulsory,
                       "compulsory_GBs_without_rebuild": compulsory / (raw_s / K) / 1e9,
                       "frac_of_peak_without_rebuild": compulsory / (raw_s / K) / 1e9 / HBM_PEAK_GBS},
    }
    if stage_ms:
        out["stage_ms"] = stage_ms
    if rebuilds_in_region:
        out["rebuild_in_region"] = {"avg_ms": rebuild_in_region_ms, "count": rebuilds_in_region,
                                    "incremental": bool(wl.incremental_rebuild),
                                    "rows_hashed_by_last": st_timed["rehashed_rows"]}

    if args.cpu_steps > 0:
        from oracle import slide_oracle as so
        orc = so.SlideOracle(input_dim=wl.input_dim, hidden_dim=wl.hidden_dim, num_classes=wl.num_classes,
                             hash_kind=wl.hash_kind, K=wl.K, L=wl.L, bucket_cap=wl.bucket_cap, rebuild_every=0,
                             lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, dwta_bin=wl.dwta_bin,
                             overflow_policy=wl.overflow_policy, weights=weights, hash_params=hp,
                             sample_budget=wl.sample_budget, sample_fill=wl.sample_fill, sample_seed=wl.sample_seed)
        cores = so.num_threads()
        tb0 = time.perf_counter()
        orc.build_tables()
        tb1 = time.perf_counter()
        ncpu = min(args.cpu_steps, len(host_batches))
        c0 = time.perf_counter()
        for s in range(ncpu):
            orc.train_step(host_batches[s])
        c1 = time.perf_counter()
        out["cpu_baseline"] = {"value": wl.batch * ncpu / (c1 - c0), "unit": "samples/s",
                               "cores": cores, "kind": "oracle",
                               "sample": "%d full steps (batch %d) of the same workload, tables prebuilt "
                                         "(table build took %.1f s and is not in the timed sample)"
                                         % (ncpu, wl.batch, tb1 - tb0)}
        if args.cpu_steps_1thread > 0:                   # the same oracle on one core, fewer steps
            so.set_num_threads(1)
            n1 = min(args.cpu_steps_1thread, len(host_batches) - ncpu)
            c0 = time.perf_counter()
            for s in range(ncpu, ncpu + n1):
                orc.train_step(host_batches[s])
            c1 = time.perf_counter()
            so.set_num_threads(cores)
            out["cpu_baseline_1thread"] = {"value": wl.batch * n1 / (c1 - c0), "unit": "samples/s", "cores": 1,
                                           "kind": "oracle",
                                           "sample": "the next %d full steps (batch %d), same tables" % (n1, wl.batch)}
    print(json.dumps(out))
    model.destroy()
    return 0


if __name__ == "__main__":
    sys.exit(main())
