#!/usr/bin/env python3
"""Benchmark of the sparse global attention path on one MI355X.

A "step" is one pass of the whole path (pool -> compressed attention with the TopK bounds ->
TopK filter sweep + candidate TopK -> selection attention + merge) over one batch of synthetic Q/K/V that is already resident in HBM.
Default workload: config 4, 1000 views x 1374 tokens, 16 heads, head_dim 64, bf16, block 64,
top-64.  Prints ONE JSON line: the metric (tokens/s of the whole path), the roofline of the selection
kernel (executed FLOP/s against the bf16 MFMA peak, plus its memory side and a second, measured bound:
the same kernel with its arithmetic taken out), a roofline fraction per stage, per-stage times from HIP
events (taken in a second, instrumented pass: the headline time is measured with the events switched
off), the dense denominator and the CPU baseline.  The in-house dense attention on the
same inputs is timed once for the speed-up ratio, and the fp64 CPU oracle is timed on a bounded
sample of the same workload as a reported baseline (cpu_baseline)."""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
CONFIG4 = None   # set in main(): the workload the stored counter figures belong to
PAPER_CONTEXT = {"speedup_end_to_end_model": 12.4, "views": 1024, "hardware": "1x NVIDIA H100",
                 "note": "whole-model inference latency, pi3 backbone (Fig. 4); context, not a target"}


def e_bytes(wl):
    return 2 if wl.dtype == "bf16" else 4


def say(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def valid_pairs(idx: torch.Tensor, n_tok: int, block: int) -> int:
    """Number of (query token, key token) pairs the selection stage evaluates: executed work only."""
    heads, n_blk, kk = idx.shape
    lens = torch.full((n_blk,), block, dtype=torch.int64, device=idx.device)
    lens[-1] = n_tok - (n_blk - 1) * block
    keys = lens[idx.long()].sum(dim=-1)                      # [heads, n_blk] valid keys per query block
    return int((keys * lens[None, :]).sum().item())


TRAFFIC_FILE = "profiles/hbm_traffic_config4.md"


def measured_traffic(wl):
    """HBM bytes per launch of the selection kernel from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE runs, scaled by a known-size copy).  A stored figure, not one measured in
    this run: only quoted for exactly the workload it was measured on (config 4 as BASELINE states it)."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    ref = CONFIG4
    if ((wl.name, wl.views, wl.block, wl.topk, wl.dtype) != (ref.name, ref.views, ref.block, ref.topk, ref.dtype)
            or not os.path.exists(path)):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch_select_kernel:"):
            return float(line.split(":")[1])
    return None


def dense_launch_edge(n_tok, heads):
    """First query row of the dense kernel's second launch (it runs in launches of about 2e14 FLOP over
    groups of 128 query rows), or None when one launch covers the problem."""
    per_launch = max(int(2e14 / (4.0 * 64.0 * 128 * n_tok * heads)), 1)
    return per_launch * 128 if per_launch * 128 < n_tok else None


def cpu_baseline(wl, q, k, v, idx_dev, budget_s: float, dense_out=None):
    """Times the fp64 oracle on the host: pooling in full, then scores / compressed attention /
    TopK / selection / merge on as many sampled query blocks as fit the time budget; the per-block
    time is extrapolated linearly to all blocks.  With `dense_out` (the dense kernel's result on the
    same inputs) a few of its rows -- both ends and either side of its launch boundary -- are compared
    with the oracle's dense attention as well."""
    from oracle import gsa_oracle
    gsa_oracle.build()
    say("cpu_baseline: copying inputs to the host")
    qf, kf, vf = (t.cpu().to(torch.float32).numpy() for t in (q, k, v))
    scale = 1.0 / math.sqrt(wl.head_dim)
    dense_check = None
    if dense_out is not None:
        edge = dense_launch_edge(wl.n_tok, wl.heads)
        rows = [0, 1, wl.n_tok // 2, wl.n_tok - 2, wl.n_tok - 1] + ([edge - 1, edge, edge + 1] if edge else [])
        rows = np.unique(np.asarray(rows, dtype=np.int64))
        ref = gsa_oracle.dense_attn(qf, kf, vf, scale, q_tok=rows)
        got = dense_out.index_select(0, torch.from_numpy(rows).to(dense_out.device)).cpu().to(torch.float32).numpy()
        rms = math.sqrt(float(np.mean(ref * ref)))
        err = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rms)))
        dense_check = {"rows": [int(r) for r in rows], "max_rel_err_vs_oracle": err, "tolerance": 2e-2, "ok": bool(err <= 2e-2)}
        say(f"dense rows vs oracle: {dense_check}")
    t0 = time.perf_counter()
    qc, kc, vc = gsa_oracle.pool(qf, wl.block), gsa_oracle.pool(kf, wl.block), gsa_oracle.pool(vf, wl.block)
    t_pool = time.perf_counter() - t0
    say(f"cpu_baseline: pooling (full) {t_pool:.2f} s")
    rng = np.random.default_rng(0)
    n_rows, t_rows, batch = 0, 0.0, 4
    kk = min(wl.topk, wl.n_blk)
    while t_rows + t_pool < budget_s and n_rows < wl.n_blk:
        rows = np.sort(rng.choice(wl.n_blk, size=min(batch, wl.n_blk - n_rows), replace=False)).astype(np.int64)
        t0 = time.perf_counter()
        s = gsa_oracle.scores(qc, kc, rows)
        oc = gsa_oracle.compressed_attn(s, vc, scale)
        idx = gsa_oracle.topk(s, kk)
        o_sel, _ = gsa_oracle.select_attn(qf, kf, vf, wl.block, idx, scale, rows)
        gsa_oracle.merge(oc, o_sel, None, wl.n_tok, wl.block, rows)
        dt = time.perf_counter() - t0
        t_rows += dt
        n_rows += rows.size
        if dt < 2.0:
            batch *= 2
    est_total = t_pool + t_rows / max(n_rows, 1) * wl.n_blk
    say(f"cpu_baseline: {n_rows} query blocks in {t_rows:.2f} s -> estimated full job {est_total:.1f} s")
    return {"value": wl.n_tok / est_total, "unit": "tokens/s", "cores": gsa_oracle.threads(),
            "kind": "oracle",
            "sample": (f"pooling of all {wl.n_blk} blocks ({t_pool:.2f} s) + scores, compressed attention, "
                       f"TopK, selection and merge on {n_rows} random query blocks x {wl.heads} heads "
                       f"({t_rows:.2f} s), extrapolated linearly to all {wl.n_blk} query blocks"),
            "estimated_full_job_s": est_total}, dense_check


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="workload (1..5); the metric is quoted on 4")
    ap.add_argument("--views", type=int, default=None, help="override the number of views")
    ap.add_argument("--topk", type=int, default=None)
    ap.add_argument("--block", type=int, default=None, help="override the pooling block (16, 32, 64, 128)")
    ap.add_argument("--dtype", choices=("bf16", "f32"), default=None,
                    help="override the I/O type of the workload (f32: the matrix-core kernels on bf16 operand parts)")
    ap.add_argument("--kernel-choice", type=int, default=0, choices=(0, 1, 2),
                    help="speed3r_set_kernel_choice: 0 automatic, 1 the generic one-thread-per-row attention kernel, "
                         "2 TopK always from stored scores; not the headline metric unless 0")
    ap.add_argument("--special", type=int, default=0,
                    help="treat the first N tokens of every view as special tokens (dense rows); not the headline metric")
    ap.add_argument("--forced-vggt", action="store_true",
                    help="force the blocks of the reference view and of every 100th view; not the headline metric")
    ap.add_argument("--compress-queries", action="store_true",
                    help="compression branch with every token's own query against the pooled keys; not the headline metric")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense denominator run")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true",
                    help="skip the load-only run of the selection kernel (the measured data-movement bound)")
    ap.add_argument("--probe-sweep", action="store_true",
                    help="also time the load-only kernel with deeper LDS rings and fewer workgroups per CU "
                         "(how the stage's data movement depends on the number of query blocks in progress)")
    ap.add_argument("--cpu-budget-s", type=float, default=20.0)
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel (a known-size reference "
                         "for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1")

    from paper_2603_08055_amd import speed3r as s3r
    from paper_2603_08055_amd import workloads
    s3r.load()
    over = {}
    if args.views is not None:
        over["views"] = args.views
    if args.topk is not None:
        over["topk"] = args.topk
    if args.block is not None:
        over["block"] = args.block
    if args.dtype is not None:
        over["dtype"] = args.dtype
    s3r.speed3r_set_kernel_choice(args.kernel_choice)
    global CONFIG4
    CONFIG4 = workloads.config(4)
    wl = workloads.config(args.config, **over)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    say(f"workload {wl.name}: n_tok={wl.n_tok} heads={wl.heads} block={wl.block} topk={wl.topk} {wl.dtype}")
    q, k, v = workloads.make_inputs(wl, device=dev)
    out = torch.empty_like(q)
    # the sequence the sparse path works on: every token, or the image tokens when --special is given
    seq = workloads.Workload(wl.name, wl.views, wl.tokens_per_view - args.special, wl.heads, wl.head_dim, wl.dtype,
                             wl.block, wl.topk, wl.seed, wl.kind)
    forced = None
    if args.forced_vggt:
        forced = torch.from_numpy(workloads.vggt_forced_blocks(seq)).to(dev)
    n_forced = 0 if forced is None else forced.numel()
    kk = s3r.speed3r_selected_per_row(seq.n_tok, wl.block, wl.topk, n_forced)
    idx = torch.empty((wl.heads, seq.n_blk, kk), dtype=torch.int32, device=dev)
    dt_code = s3r.S3R_BF16 if wl.dtype == "bf16" else s3r.S3R_F32
    tpv = wl.tokens_per_view if args.special else 0
    ws_bytes = s3r.speed3r_workspace_bytes_ex(wl.n_tok, wl.heads, wl.head_dim, wl.block, wl.topk, dt_code,
                                              n_forced, tpv, args.special, compress_queries=int(args.compress_queries))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    say(f"workspace {ws_bytes / 2**30:.2f} GiB")

    def step():
        s3r.speed3r_sparse_global_attn_ex(q, k, v, out, wl.block, wl.topk, topk_idx=idx, workspace=ws,
                                          forced_blocks=forced, tokens_per_view=tpv, special_per_view=args.special,
                                          compress_queries=int(args.compress_queries))

    if args.pmc_calibration:
        src = torch.ones(2 ** 29, dtype=torch.bfloat16, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    # the headline: K steps with the library's per-launch events switched off
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    # the same K steps once more with HIP events around every launch, on the call's stream: per-stage times
    s3r.speed3r_set_profiling(True)
    s3r.speed3r_get_stage_ms()                       # clear anything recorded so far
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_instrumented = (time.perf_counter() - t0) * 1e3 / args.steps
    stage_ms, stage_n = s3r.speed3r_get_stage_ms()
    s3r.speed3r_set_profiling(False)
    say(f"{ms_per_step:.3f} ms/step ({ms_instrumented:.3f} with per-launch events); per-stage ms/step: "
        + ", ".join(f"{s}={stage_ms[s] / args.steps:.3f}" for s in ("pool", "split", "compress", "topk", "select")))

    # roofline of the dominant kernel (selection attention, bf16 MFMA): executed FLOPs only
    pairs = valid_pairs(idx, seq.n_tok, wl.block)
    sel_flops = 4.0 * wl.head_dim * pairs
    sel_ms = stage_ms["select"] / max(stage_n["select"], 1)
    achieved = sel_flops / (sel_ms * 1e-3) / 1e12
    traffic = None if (args.special or n_forced or args.compress_queries or args.kernel_choice) else measured_traffic(wl)
    pipe = (args.kernel_choice != 1 and wl.dtype == "bf16" and wl.block == 64 and kk <= 128 and not args.special
            and not args.compress_queries and not (kk > 96 and 2 * n_forced >= kk))
    roofline = {"kernel": ("select_generic_kernel" if args.kernel_choice == 1 else
                           "select_pipe_kernel" if pipe else "select_mfma_kernel"),
                "bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                "traffic": traffic,
                "traffic_source": (None if traffic is None else
                                   f"{TRAFFIC_FILE}: rocprofv3 FETCH_SIZE + WRITE_SIZE of this workload, scaled by a copy "
                                   "of known size; a stored figure, not re-measured in this run"),
                "kernel_ms": sel_ms, "flops_per_launch": sel_flops}
    # the same kernel seen from the memory side: K/V tiles of the selected blocks + Q read + out written, against what a bare gather of such pieces reaches
    kv_bytes = float(wl.heads) * seq.n_blk * kk * 2 * wl.block * wl.head_dim * e_bytes(wl)
    qo_bytes = 2.0 * seq.n_tok * wl.heads * wl.head_dim * e_bytes(wl)
    roofline["memory_side"] = {"algorithmic_bytes_per_launch": kv_bytes + qo_bytes,
                               "achieved_GBps": (kv_bytes + qo_bytes) / (sel_ms * 1e-3) / 1e9,
                               "hbm_peak_GBps": 8000.0,
                               "measured_traffic_GBps": (None if roofline["traffic"] is None
                                                         else roofline["traffic"] / (sel_ms * 1e-3) / 1e9),
                               "note": "scattered 16 KiB K/V units; see data_movement_bound for what moving them costs by itself"}
    # second bound, measured here: the same kernel on the same index lists with its arithmetic taken out
    if not args.no_probe and wl.dtype == "bf16" and wl.block in (64, 128) and not args.special and not n_forced:
        probe_out = torch.empty_like(q)

        def time_probe(stages, wg_per_cu, n=5):
            for _ in range(2):
                s3r.speed3r_probe_select_loads(q, k, v, idx, probe_out, wl.block, stages, wg_per_cu)
            torch.cuda.synchronize()
            s3r.speed3r_set_profiling(True)
            s3r.speed3r_get_stage_ms()
            for _ in range(n):
                s3r.speed3r_probe_select_loads(q, k, v, idx, probe_out, wl.block, stages, wg_per_cu)
            torch.cuda.synchronize()
            p_ms, p_n = s3r.speed3r_get_stage_ms()
            s3r.speed3r_set_profiling(False)
            return p_ms["select"] / max(p_n["select"], 1)

        # the probe at the occupancy of the kernel that ran: long rows on long sequences run two workgroups per
        # CU (64 query blocks in progress per XCD), everything else as many as fit
        probe_wg = 2 if (wl.block == 64 and kk >= 40 and seq.n_blk >= 3000) else 0
        probe_ms = time_probe(0, probe_wg)
        assert torch.equal(probe_out, q), "the load probe must leave a copy of q in its output"
        sweep = None
        if args.probe_sweep:
            sweep = []
            for stages, wg in ((2, 5), (2, 4), (2, 3), (2, 2), (3, 3), (3, 2), (3, 1), (4, 2), (4, 1)):
                ms = time_probe(stages, wg)
                sweep.append({"ring_stages": stages, "wg_per_cu": wg, "query_blocks_in_progress_per_xcd": 32 * wg,
                              "units_requested_ahead_per_cu": (stages - 1) * wg, "loads_only_ms": ms})
                say(f"load probe, {stages} stages, {wg} workgroups per CU: {ms:.3f} ms")
        del probe_out
        s3r.speed3r_release_scratch()
        roofline["data_movement_bound"] = {
            "bound": "fabric", "what": "select_mfma_kernel<PROBE>: the same index lists walked with the same work mapping, "
                                       "K/V units moved into LDS through a two-stage ring, Q read and out written, "
                                       "no MFMA / softmax; " + (f"{probe_wg} workgroups per CU like the kernel that ran"
                                                                if probe_wg else "as many workgroups per CU as fit"),
            "loads_only_ms": probe_ms, "kernel_ms": sel_ms, "frac": probe_ms / sel_ms,
            "loads_only_GBps": (kv_bytes + qo_bytes) / (probe_ms * 1e-3) / 1e9,
            "mfma_frac_if_arithmetic_were_free": sel_flops / (probe_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
        if sweep is not None:
            roofline["data_movement_bound"]["sweep"] = sweep
        say(f"selection kernel {sel_ms:.3f} ms, its loads alone {probe_ms:.3f} ms")
    # HBM-side figures of the two bandwidth-bound stages (algorithmic bytes / measured time)
    e = 2 if wl.dtype == "bf16" else 4
    pool_bytes = 3.0 * wl.n_tok * wl.heads * wl.head_dim * e + 3.0 * seq.n_blk * wl.heads * wl.head_dim * 4
    topk_bytes = 4.0 * seq.n_blk * seq.n_blk * wl.heads + 4.0 * seq.n_blk * kk * wl.heads
    hbm = {"pool_GBps": pool_bytes / (stage_ms["pool"] / args.steps * 1e-3) / 1e9, "peak_GBps": 8000.0}
    # one roofline fraction per stage: algorithmic bytes (HBM-bound stages) or executed matrix FLOPs over the stage's time
    def stage_s(name):
        return stage_ms[name] / args.steps * 1e-3
    # K and V tiles in operand order: one bf16 copy each (fp32 problems: K in three bf16 parts, V in two)
    tiles_bytes = (2.0 if wl.dtype == "bf16" else 5.0) * seq.n_blk * wl.block * wl.heads * wl.head_dim * 2
    if args.kernel_choice == 1:
        tiles_bytes = 0.0   # the generic kernel reads K and V in place

    def device_copy_gbps(moved):
        """What a plain device-to-device copy (torch's copy kernel) moving the same number of bytes, half read and
        half written, sustains on this GPU: the practical reference beside the 8 TB/s of the data sheet."""
        n = int(moved // 2) // 16 * 16
        src = torch.empty(n, dtype=torch.uint8, device="cuda")
        src.zero_()
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        return 2.0 * n / (e0.elapsed_time(e1) / 5 * 1e-3) / 1e9
    sweep_flops = 2.0 * wl.head_dim * float(seq.n_blk) * float(seq.n_blk) * wl.heads     # one N_b x N_b x d product
    in_sweep = kk - n_forced <= 64
    stages = {
        "pool": {"bound": "hbm", "unit": "GB/s", "peak": 8000.0, "achieved": pool_bytes / stage_s("pool") / 1e9,
                 "frac": pool_bytes / stage_s("pool") / 1e9 / 8000.0, "algorithmic_bytes": pool_bytes,
                 "moved_bytes": pool_bytes + tiles_bytes,
                 "moved_GBps": (pool_bytes + tiles_bytes) / stage_s("pool") / 1e9,
                 "note": "moved = algorithmic + the K/V operand-order tiles this design writes for the selection kernel"},
        "compress": {"bound": "mfma", "unit": "TFLOP/s", "peak": MFMA_BF16_PEAK_TFLOPS,
                     "achieved": 2.0 * sweep_flops / stage_s("compress") / 1e12,
                     "frac": 2.0 * sweep_flops / stage_s("compress") / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                     "flops": 2.0 * sweep_flops, "note": "Qc Kc^T and P Vc, 4 d N_b^2 H FLOP (eqs. 3-4), counted once each"},
    }
    if not args.no_probe:
        copy_gbps = device_copy_gbps(pool_bytes + tiles_bytes)
        stages["pool"]["device_copy_GBps"] = copy_gbps
        stages["pool"]["moved_over_device_copy"] = stages["pool"]["moved_GBps"] / copy_gbps
        say(f"pool stage moves {stages['pool']['moved_GBps']:.0f} GB/s; a plain device copy of as many bytes {copy_gbps:.0f} GB/s")
    if in_sweep:
        stages["topk"] = {"bound": "mfma", "unit": "TFLOP/s", "peak": MFMA_BF16_PEAK_TFLOPS,
                          "achieved": sweep_flops / stage_s("topk") / 1e12,
                          "frac": sweep_flops / stage_s("topk") / 1e12 / MFMA_BF16_PEAK_TFLOPS, "flops": sweep_flops,
                          "note": "filter sweep recomputes Qc Kc^T (2 d N_b^2 H FLOP); the time also holds the candidate TopK"}
    else:
        stages["topk"] = {"bound": "hbm", "unit": "GB/s", "peak": 8000.0, "achieved": topk_bytes / stage_s("topk") / 1e9,
                          "frac": topk_bytes / stage_s("topk") / 1e9 / 8000.0, "algorithmic_bytes": topk_bytes}
        stages["compress"]["note"] += "; this route also writes S_guide (4 N_b^2 H bytes)"
    if kk - n_forced > 64:   # TopK from S_guide in memory (k > 64); otherwise TopK runs inside the compression sweep
        hbm["topk_GBps"] = topk_bytes / (stage_ms["topk"] / args.steps * 1e-3) / 1e9
    else:
        hbm["topk_route"] = "inside the compression sweep (S_guide not written to memory)"

    result = {
        "metric": ("sparse global-attn tokens/s at 1000 views" if wl.views == 1000 else "sparse global-attn tokens/s")
                  + (" (VGGT-variant layer: " + ", ".join(x for x in (f"{args.special} special tokens per view" if args.special else "",
                                                                       f"{n_forced} forced blocks" if n_forced else "") if x) + ")"
                     if args.special or n_forced else "")
                  + (" (compression branch with unpooled queries)" if args.compress_queries else ""),
        "value": wl.n_tok / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_with_launch_events": ms_instrumented,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "views": wl.views, "tokens_per_view": wl.tokens_per_view,
                   "n_tok": wl.n_tok, "heads": wl.heads, "head_dim": wl.head_dim, "block": wl.block,
                   "topk": wl.topk, "kind": wl.kind, "seed": wl.seed, "kernel_choice": args.kernel_choice,
                   "generator": "torch.Generator(device='cuda'), one view at a time (the tests' small cases draw on the CPU generator)"},
        "roofline": roofline,
        "stages": stages,
        "stage_ms_per_step": {s: stage_ms[s] / args.steps for s in ("pool", "split", "compress", "topk", "select")},
        "stage_launches_per_step": {s: stage_n[s] / args.steps for s in ("pool", "split", "compress", "topk", "select")},
        "hbm_stages": hbm,
        "paper_context": PAPER_CONTEXT,
    }
    if args.compress_queries:
        result["config"]["compress_queries"] = 1
        result["compress_queries_flops_per_step"] = 4.0 * wl.head_dim * float(seq.n_tok) * float(seq.n_blk) * wl.heads
    if args.special:
        result["stage_ms_per_step"]["dense_special_rows"] = stage_ms["dense"] / args.steps
        result["config"]["special_per_view"] = args.special
        spec_flops = 4.0 * wl.head_dim * float(wl.views * args.special) * float(wl.n_tok) * wl.heads
        result["special_rows"] = {"rows": wl.views * args.special,
                                  "tflops": spec_flops / (stage_ms["dense"] / args.steps * 1e-3) / 1e12}
    if n_forced:
        result["config"]["forced_blocks"] = n_forced
        result["config"]["blocks_per_query_block"] = kk

    dense_out = None
    if not args.no_dense:
        dense_out = torch.empty_like(q)
        # a cheap call that uses the same library-held scratch (the K/V tiles) first, so that its allocation
        # and the device synchronisation that goes with it stay outside the timed run
        s3r.speed3r_select_attn(q, k, v, idx[:, :, :1].contiguous(), dense_out, wl.block)
        torch.cuda.synchronize()
        say("dense attention (same inputs), one timed run")
        s3r.speed3r_set_profiling(True)
        s3r.speed3r_get_stage_ms()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        s3r.speed3r_dense_attn(q, k, v, dense_out)
        torch.cuda.synchronize()
        dense_s = time.perf_counter() - t0
        d_ms, _ = s3r.speed3r_get_stage_ms()
        s3r.speed3r_set_profiling(False)
        dense_flops = 4.0 * wl.head_dim * float(wl.n_tok) * float(wl.n_tok) * wl.heads
        result["dense"] = {"ms": dense_s * 1e3, "kernel_ms": d_ms["dense"], "relayout_ms": d_ms["pool"],
                           "tflops": dense_flops / (d_ms["dense"] * 1e-3) / 1e12,
                           "mfma_frac": dense_flops / (d_ms["dense"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
        result["speedup_vs_dense"] = (d_ms["dense"] + d_ms["pool"]) / ms_per_step
        say(f"dense {dense_s * 1e3:.1f} ms wall, {d_ms['dense'] + d_ms['pool']:.1f} ms of kernels -> speed-up "
            f"{result['speedup_vs_dense']:.1f}x")
        s3r.speed3r_release_scratch()

    if not args.no_cpu_baseline and not args.special and not n_forced:
        result["cpu_baseline"], dense_check = cpu_baseline(wl, q, k, v, idx, args.cpu_budget_s, dense_out)
        if dense_check is not None:
            result["dense"]["check"] = dense_check

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
