#!/usr/bin/env python3
"""Benchmark of the vote step (Algorithm 1, error compensation .. error update)
on one MI355X.

One "step" is one mv_vote_step() call: the whole hot path over one batch of
synthetic gradients (N x d), inputs resident in HBM.  The error buffer is
carried from step to step as in training; the gradients cycle over a few
distinct pre-generated matrices.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E peak


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def measured_traffic(workload):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3
    counters (FETCH_SIZE, WRITE_SIZE scaled by a plain copy of known size); the
    committed summary under profiles/ carries the figure.  None if no summary
    covers this workload."""
    path = os.path.join(ROOT, "profiles", "vote_step_%s_hbm_counters.txt" % workload)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split("=")[1])
    except OSError:
        pass
    return None


def comm_load_context(w):
    """The paper's closed-form communication load for this (d, phi), q = 32, H = 1
    (Sec. 2.1): context printed beside the measurement."""
    import math
    bits = math.ceil(math.log2(w.d / w.K) - 1e-12) + 2
    q_loc = w.K * bits
    q_val = 32 * w.K
    return {"bits_per_position": bits, "Q_loc_bits": q_loc, "Q_val_bits": q_val,
            "compression": round(32.0 * w.d / (q_loc + q_val), 1)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--grad-sets", type=int, default=2, help="distinct gradient matrices cycled over")
    ap.add_argument("--k", type=int, default=0,
                    help="override the workload's K (e.g. 111740 = the paper's phi = 1e-2 on ResNet-18's size); "
                         "the headline figure is the workload's own K")
    ap.add_argument("--scheme", default="mv", choices=["mv", "ad", "rs"],
                    help="mv: majority voting (Algorithm 1); ad: majority voting with add-drop (Algorithm 2), "
                         "a full first vote untimed, then K_ad = K/10 per step; rs: majority voting with "
                         "random selection (Algorithm 1, S_rand-weighted), seeded Exp(1) numbers resident in HBM")
    ap.add_argument("--codec", action="store_true",
                    help="also time the sparse position code (Sec. 4.3.1) on the workers' vote lists "
                         "of the last step (untimed extra; needs worker_idx, scheme mv)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step per gradient set into a HIP graph and time replays "
                         "(needs --profile-level 0: no events inside a captured step)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-worker-idx", action="store_true",
                    help="do not request the per-worker sorted vote lists (optional output)")
    ap.add_argument("--profile-level", type=int, default=1, choices=[0, 1, 2],
                    help="HIP events inside the timed region: 1 = dominant kernel only, 2 = every kernel")
    ap.add_argument("--breakdown", action="store_true",
                    help="after the timed region, run extra untimed steps with events around every kernel")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2011_06495_amd import binding as B
    from paper_2011_06495_amd import build as mv_build
    from paper_2011_06495_amd import workloads as W

    if not os.path.exists(B.LIB_PATH):
        mv_build.build_lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    w = W.WORKLOADS[args.workload]
    if args.k > 0:
        w = w.with_size(w.d, K=args.k)
    bf16 = w.grad_dtype == "bf16"
    N, d, K = w.N, w.d, w.K
    ld_g = (d + (7 if bf16 else 3)) // (8 if bf16 else 4) * (8 if bf16 else 4)
    ld_e = (d + 3) // 4 * 4

    # ---- inputs: generated on the host from seeds, then resident in HBM
    t0 = time.time()
    gen_threads = min(16, os.cpu_count() or 1)
    g_host0 = None
    g_dev = []
    for s in range(max(1, args.grad_sets)):
        gh = W.gradients(w, s, threads=gen_threads)
        if s == 0:
            g_host0 = gh
        t = torch.zeros((N, ld_g), dtype=torch.int16 if bf16 else torch.float32, device=dev)
        t[:, :d].copy_(torch.from_numpy(gh.view(np.int16) if bf16 else gh))
        g_dev.append(t)
    log("generated %d gradient sets of %s (N=%d d=%d K=%d) in %.1f s" % (len(g_dev), w.name, N, d, K, time.time() - t0))

    e_dev = torch.zeros((N, ld_e), dtype=torch.float32, device=dev)
    widx = None if args.no_worker_idx else torch.zeros((N, K), dtype=torch.int32, device=dev)
    votes = torch.zeros(d, dtype=torch.uint8, device=dev)
    mask = torch.zeros(K, dtype=torch.int32, device=dev)
    agg = torch.zeros(K, dtype=torch.float32, device=dev)
    ad = args.scheme == "ad"
    rs = args.scheme == "rs"
    r_dev, r_host0 = [], None
    if rs:
        for s in range(max(1, args.grad_sets)):
            rh = W.selection_clocks(w, s)
            if s == 0:
                r_host0 = rh
            r_dev.append(torch.from_numpy(rh).to(dev))
    ctx = B.mv_begin(B.make_config(N, d, K, B.MV_BF16 if bf16 else B.MV_F32,
                                   flags=B.MV_FLAG_ADD_DROP if ad else 0))
    stream = torch.cuda.current_stream(dev)
    k_ad = max(1, K // 10)
    if ad:
        ld_bits = ((d + 31) // 32 + 3) // 4 * 4
        vote_bits = torch.zeros((N, ld_bits), dtype=torch.int32, device=dev)
        msum = torch.zeros((d + 15) // 16 * 16, dtype=torch.uint8, device=dev)
        add_idx = torch.zeros((N, K), dtype=torch.int32, device=dev)
        drop_idx = torch.zeros((N, K), dtype=torch.int32, device=dev)
        counts = torch.zeros(2 * N, dtype=torch.int32, device=dev)

    def step(i):
        if ad:   # step 0 is a full vote from the empty state, every later step changes at most K/10 votes
            B.mv_ad_vote_step(ctx, g_dev[i % len(g_dev)], e_dev, K if i == 0 else k_ad, vote_bits, msum,
                              add_idx, drop_idx, counts, mask, agg, stream=stream, ld_g=ld_g, ld_e=ld_e)
        elif rs:
            B.mv_rs_vote_step(ctx, g_dev[i % len(g_dev)], e_dev, r_dev[i % len(r_dev)], widx, votes, mask, agg,
                              stream=stream, ld_g=ld_g, ld_e=ld_e)
        else:
            B.mv_vote_step(ctx, g_dev[i % len(g_dev)], e_dev, widx, votes, mask, agg, stream=stream,
                           ld_g=ld_g, ld_e=ld_e)

    # ---- step 0 result kept for the check against the oracle
    step(0)
    torch.cuda.synchronize()
    mask0 = mask.cpu().numpy().view(np.uint32).copy()
    agg0 = agg.cpu().numpy().copy()
    cand, tau, slow = B.mv_last_step_row_stats(ctx, N)
    log("step 0: candidates per row min/max %d/%d, select path per row %s" % (min(cand), max(cand), slow))

    # ---- warmup, then the timed region
    if args.graph:
        assert args.profile_level == 0, "--graph needs --profile-level 0"
        n_sets = max(len(g_dev), len(r_dev), 1)
        side = torch.cuda.Stream(device=dev)
        graphs = []
        eager_stream = stream
        for s_i in range(n_sets):
            gph = torch.cuda.CUDAGraph()
            torch.cuda.synchronize()
            with torch.cuda.graph(gph, stream=side):
                stream = torch.cuda.current_stream(dev)
                step(1 + s_i)                       # any step index after 0 with this gradient set
            graphs.append(gph)
        stream = eager_stream
        torch.cuda.synchronize()
        eager_step = step

        def step(i):                                # noqa: F811
            graphs[(i - 1) % n_sets].replay() if i >= 1 else eager_step(i)
    B.mv_set_profiling(ctx, args.profile_level)
    for i in range(args.warmup):
        step(1 + i)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(1 + args.warmup + i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start

    names = B.kernel_names()
    dom = names.index("mv_stream_collect")
    dom_ms = []
    per_kernel = {}
    if args.profile_level > 0:
        for back in range(min(args.steps, 64)):
            ms = B.mv_step_kernel_ms(ctx, back)
            dom_ms.append(ms[dom])
            if args.profile_level == 2:
                for nme, v in zip(names, ms):
                    per_kernel.setdefault(nme, []).append(v)
    cand_last, _, slow_last = B.mv_last_step_row_stats(ctx, N)
    log("last timed step: candidates per row min/max %d/%d, select path per row %s" %
        (min(cand_last), max(cand_last), slow_last))

    breakdown = None
    if args.breakdown:
        B.mv_set_profiling(ctx, 2)
        acc = {n: [] for n in names}
        for i in range(10):
            step(1000 + i)
            torch.cuda.synchronize()
            for nme, v in zip(names, B.mv_step_kernel_ms(ctx, 0)):
                acc[nme].append(v)
        breakdown = {n: round(float(np.median(v)) * 1e3, 2) for n, v in acc.items()}   # microseconds
    B.mv_set_profiling(ctx, 0)

    # ---- optional: the position code on the vote lists of the last step
    codec = None
    if args.codec and not ad and widx is not None:
        block_len = int(round(d / K))
        max_bits = B.mv_codec_stream_bits(K, d, block_len)
        ld_words = (max_bits + 31) // 32
        streams = torch.zeros((N, ld_words), dtype=torch.int32, device=dev)
        nbits = torch.zeros(N, dtype=torch.int64, device=dev)
        dec = torch.zeros((N, K), dtype=torch.int32, device=dev)
        dcnt = torch.zeros(N, dtype=torch.int32, device=dev)
        scratch = torch.empty(B.mv_codec_scratch_bytes(max_bits, N), dtype=torch.uint8, device=dev)
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        reps = 20
        for it in range(2):                       # first round warms up
            evs[0].record(stream)
            for _ in range(reps):
                B.mv_codec_encode(widx, K, d, block_len, streams, nbits, stream=stream)
            evs[1].record(stream)
            for _ in range(reps):
                B.mv_codec_decode(streams, nbits, max_bits, d, block_len, dec, K, dcnt, scratch, stream=stream)
            evs[2].record(stream)
            torch.cuda.synchronize()
        codec = {"rows": N, "positions_per_row": K, "block_len": block_len,
                 "bits_per_position": round(float(nbits.cpu().numpy().mean()) / K, 3),
                 "paper_bits_per_position": comm_load_context(w)["bits_per_position"],
                 "encode_us": round(evs[0].elapsed_time(evs[1]) * 1e3 / reps, 2),
                 "decode_us": round(evs[1].elapsed_time(evs[2]) * 1e3 / reps, 2),
                 "round_trip_ok": bool(torch.equal(dec, widx) and int(dcnt.min()) == K and int(dcnt.max()) == K)}
        # the fractional quantiser (Sec. 4.3.2, q = 4) on N x K values: the gradients at the mask's coordinates
        q = 4
        sent = g_dev[0][:, :d].float()[:, mask.long()].contiguous() if not bf16 else None
        if sent is not None:
            qs = torch.zeros((N, (K * q + 31) // 32), dtype=torch.int32, device=dev)
            qm = torch.zeros((N, 1 << (q - 1)), dtype=torch.float32, device=dev)
            qo = torch.zeros((N, K), dtype=torch.float32, device=dev)
            qscr = torch.empty(B.mv_quant_scratch_bytes(K, N, q), dtype=torch.uint8, device=dev)
            for it in range(2):
                evs[0].record(stream)
                for _ in range(reps):
                    B.mv_quant_encode(sent, q, qs, qm, qscr, stream=stream)
                evs[1].record(stream)
                for _ in range(reps):
                    B.mv_quant_decode(qs, K, q, qm, qo, stream=stream)
                evs[2].record(stream)
                torch.cuda.synchronize()
            rel = float(((qo - sent).abs().sum() / sent.abs().sum()).item())
            codec["quantiser"] = {"q_bits": q, "rows": N, "values_per_row": K,
                                  "encode_us": round(evs[0].elapsed_time(evs[1]) * 1e3 / reps, 2),
                                  "decode_us": round(evs[1].elapsed_time(evs[2]) * 1e3 / reps, 2),
                                  "relative_l1_error": round(rel, 4)}

    # ---- yardstick: a plain streaming copy of the same footprint (read n, write n bytes)
    src = torch.empty(N * ld_e, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        B.mv_probe_copy(dst, src, stream)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(10):
        B.mv_probe_copy(dst, src, stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    copy_gbs = 2.0 * src.numel() * 4 * 10 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del src, dst

    coords = float(N) * float(d)
    ms_per_step = elapsed / args.steps * 1e3
    value = coords * args.steps / elapsed
    bytes_per_coord = 10.0 if bf16 else 12.0      # read g, read e, write e
    roofline = None
    if dom_ms:
        avg_ms = float(np.mean(dom_ms))
        achieved = bytes_per_coord * coords / (avg_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "mv_stream_collect", "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": measured_traffic(w.name), "avg_kernel_ms": round(avg_ms, 4),
                    "algorithmic_bytes_per_launch": bytes_per_coord * coords}
    step_frac = bytes_per_coord * coords / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS

    # ---- the oracle on the host, same inputs as step 0 (one full step)
    cpu_baseline = None
    oracle_agrees = None
    if not args.no_cpu_baseline:
        from oracle import mv_oracle
        threads = max(1, min(N, mv_oracle.max_threads(), 16))
        e0 = np.zeros((N, d), np.float32)
        log("timing the oracle on one step of %s with %d threads ..." % (w.name, threads))
        t1 = time.perf_counter()
        if ad:
            ref = mv_oracle.ad_vote_step(g_host0, e0, K, K, np.zeros((N, d), np.uint8), np.zeros(d, np.uint8),
                                         threads=threads)
        elif rs:
            ref = mv_oracle.rs_vote_step(g_host0, e0, K, r_host0, threads=threads)
        else:
            ref = mv_oracle.vote_step(g_host0, e0, K, threads=threads)
        t_or = time.perf_counter() - t1
        oracle_agrees = bool(np.array_equal(ref.mask_idx, mask0) and
                             np.array_equal(ref.agg.view(np.uint32), agg0.view(np.uint32)))
        # one thread, on a bounded sample: the plain vote step of the first two workers' rows
        n1 = min(N, 2)
        t1 = time.perf_counter()
        mv_oracle.vote_step(g_host0[:n1], e0[:n1], K, threads=1)
        t_one = time.perf_counter() - t1
        cpu_baseline = {"value": round(coords / t_or, 1), "unit": "coords/s", "cores": threads,
                        "kind": "oracle", "seconds": round(t_or, 2),
                        "single_thread": {"value": round(n1 * d / t_one, 1), "unit": "coords/s", "cores": 1,
                                          "seconds": round(t_one, 2),
                                          "sample": "plain vote step of rows 0..%d only" % (n1 - 1)},
                        "sample": "one full %s of %s (all %d rows, d=%d), step-0 inputs" %
                                  ("add-drop step (first, full vote)" if ad else
                                   "vote step with random selection" if rs else "vote step", w.name, N, d)}

    B.mv_end(ctx)
    B.mv_release(ctx)

    out = {
        "metric": "vote-step throughput (N*d coords/sec), 1 GPU" +
                  (", add-drop voting" if ad else ", random selection" if rs else ""),
        "value": round(value, 1),
        "unit": "coords/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: N=%d d=%d K=%d grads=%s, %s, error feedback carried" %
                               (w.name, N, d, K, w.grad_dtype, w.kind),
                   "N": N, "d": d, "K": K, "grad_sets_cycled": len(g_dev),
                   "scheme": "majority voting with add-drop, K_ad=%d" % k_ad if ad else
                             "majority voting with random selection" if rs else "majority voting",
                   "outputs": "mask_idx, agg_vals, add/drop lists, standing votes, vote sum" if ad else
                              "mask_idx, agg_vals, votes" + ("" if args.no_worker_idx else ", worker_idx")},
        "step_hbm_frac_algorithmic": round(step_frac, 4),
        "copy_probe_GBs": round(copy_gbs, 1),
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "oracle_agrees_on_step0": oracle_agrees,
        "launch": "hip graph replay" if args.graph else "eager",
        "slow_path_rows_last_step": int(sum(1 for x in slow_last if x == 1)),
        "paper_comm_load": comm_load_context(w),
    }
    if per_kernel:
        out["kernel_us_in_timed_region"] = {n: round(float(np.mean(v)) * 1e3, 2) for n, v in per_kernel.items()}
    if breakdown:
        out["kernel_us_breakdown"] = breakdown
    if codec:
        out["position_codec"] = codec
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
