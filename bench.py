#!/usr/bin/env python3
"""Benchmark of the vote step (Algorithm 1, error compensation .. error update)
on one MI355X.

One "step" is one mv_vote_step() call: the whole hot path over one batch of
synthetic gradients (N x d), inputs resident in HBM.  A workload is a SEQUENCE
of steps (C4: 5, C3: 20, ...) with fresh seeded gradients every step and the
error buffer carried from step to step, starting from zero.  The timed region
is made of repeats of that sequence: before each repeat the error buffer is
put back to zero outside the timed region, so every repeat does identical
work.  Every step is bracketed by a pair of HIP events on the stream; the
headline is the wall clock over exactly --steps steps, the median of the
per-step event times is reported beside it.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C4] [--no-all-configs]
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


def measured_traffic(tag):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3
    counters (FETCH_SIZE, WRITE_SIZE scaled by a plain copy of known size); the
    committed summary under profiles/ carries the figure.  None if no summary
    covers this workload."""
    path = os.path.join(ROOT, "profiles", "vote_step_%s_hbm_counters.txt" % tag)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split("=")[1]), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def comm_load_context(w):
    """The paper's closed-form communication load for this (d, phi), q = 32, H = 1
    (Sec. 2.1): context printed beside the measurement."""
    import math
    bits = math.ceil(math.log2(w.d / w.K) - 1e-12) + 2
    q_loc = w.K * bits
    q_val = 32 * w.K
    return {"bits_per_position": bits, "Q_loc_bits": q_loc, "Q_val_bits": q_val,
            "compression": round(32.0 * w.d / (q_loc + q_val), 1)}


class Problem:
    """Device buffers, context and gradient sets of one workload and scheme."""

    def __init__(self, w, scheme, want_worker_idx, keep_host_sets, mods):
        np, torch, B, W = mods
        self.mods, self.w, self.scheme = mods, w, scheme
        self.ad, self.rs = scheme == "ad", scheme == "rs"
        dev = torch.device("cuda:0")
        self.dev = dev
        bf16 = w.grad_dtype == "bf16"
        self.bf16 = bf16
        N, d, K = w.N, w.d, w.K
        self.ld_g = (d + (7 if bf16 else 3)) // (8 if bf16 else 4) * (8 if bf16 else 4)
        self.ld_e = (d + 3) // 4 * 4
        self.L = max(1, w.steps)                       # steps of the workload's own sequence
        gen_threads = min(16, os.cpu_count() or 1)
        t0 = time.time()
        self.g_dev, self.g_host, self.r_dev, self.r_host = [], [], [], []
        for s in range(self.L):
            gh = W.gradients(w, s, threads=gen_threads)
            t = torch.zeros((N, self.ld_g), dtype=torch.int16 if bf16 else torch.float32, device=dev)
            t[:, :d].copy_(torch.from_numpy(gh.view(np.int16) if bf16 else gh))
            self.g_dev.append(t)
            self.g_host.append(gh if s < keep_host_sets else None)
            if self.rs:
                rh = W.selection_clocks(w, s)
                self.r_dev.append(torch.from_numpy(rh).to(dev))
                self.r_host.append(rh if s < keep_host_sets else None)
        log("%s: generated %d gradient sets (N=%d d=%d K=%d) in %.1f s" % (w.name, self.L, N, d, K, time.time() - t0))
        self.e = torch.zeros((N, self.ld_e), dtype=torch.float32, device=dev)
        self.widx = torch.zeros((N, K), dtype=torch.int32, device=dev) if want_worker_idx and not self.ad else None
        self.votes = torch.zeros(d, dtype=torch.uint8, device=dev)
        self.mask = torch.zeros(K, dtype=torch.int32, device=dev)
        self.agg = torch.zeros(K, dtype=torch.float32, device=dev)
        self.k_ad = max(1, K // 10)
        if self.ad:
            ld_bits = ((d + 31) // 32 + 3) // 4 * 4
            self.vote_bits = torch.zeros((N, ld_bits), dtype=torch.int32, device=dev)
            self.msum = torch.zeros((d + 15) // 16 * 16, dtype=torch.uint8, device=dev)
            self.add_idx = torch.zeros((N, K), dtype=torch.int32, device=dev)
            self.drop_idx = torch.zeros((N, K), dtype=torch.int32, device=dev)
            self.counts = torch.zeros(2 * N, dtype=torch.int32, device=dev)
        self.ctx = B.mv_begin(B.make_config(N, d, K, B.MV_BF16 if bf16 else B.MV_F32,
                                            flags=B.MV_FLAG_ADD_DROP if self.ad else 0))
        self.stream = torch.cuda.current_stream(dev)

    def reset(self):
        """Back to the start of the sequence: zero error buffers (and standing votes)."""
        self.e.zero_()
        if self.ad:
            self.vote_bits.zero_()
            self.msum.zero_()

    def step(self, i):
        """Step i of the sequence (i < L)."""
        np, torch, B, W = self.mods
        g = self.g_dev[i]
        if self.ad:    # step 0 is a full vote from the empty state, every later step changes at most K/10 votes
            B.mv_ad_vote_step(self.ctx, g, self.e, self.w.K if i == 0 else self.k_ad, self.vote_bits, self.msum,
                              self.add_idx, self.drop_idx, self.counts, self.mask, self.agg, stream=self.stream,
                              ld_g=self.ld_g, ld_e=self.ld_e)
        elif self.rs:
            B.mv_rs_vote_step(self.ctx, g, self.e, self.r_dev[i], self.widx, self.votes, self.mask, self.agg,
                              stream=self.stream, ld_g=self.ld_g, ld_e=self.ld_e)
        else:
            B.mv_vote_step(self.ctx, g, self.e, self.widx, self.votes, self.mask, self.agg, stream=self.stream,
                           ld_g=self.ld_g, ld_e=self.ld_e)

    def close(self):
        np, torch, B, W = self.mods
        B.mv_end(self.ctx)
        B.mv_release(self.ctx)
        self.g_dev = self.r_dev = None


def time_sequence_repeats(p, n_steps, warmup, profile_level):
    """Times exactly n_steps steps: repeats of the workload's sequence, each from a zeroed
    error buffer (restored outside the timed region).  Returns the wall seconds of the
    timed regions, the per-step event times (ms), the host time spent enqueueing (s),
    and the dominant kernel's durations (ms) when the library recorded them."""
    np, torch, B, W = p.mods
    L = p.L
    B.mv_set_profiling(p.ctx, 0)
    done = 0
    while done < warmup:                              # warm-up: the sequence from its start, untimed
        p.reset()
        for i in range(min(L, warmup - done)):
            p.step(i)
        done += min(L, warmup - done)
    torch.cuda.synchronize()
    B.mv_set_profiling(p.ctx, profile_level)
    names = B.kernel_names()
    dom = names.index("mv_stream_collect")
    wall, enqueue, step_ms, dom_ms = 0.0, 0.0, [], []
    left = n_steps
    while left > 0:
        n = min(L, left)
        p.reset()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev[0].record(p.stream)
        for i in range(n):
            ta = time.perf_counter()
            p.step(i)
            enqueue += time.perf_counter() - ta
            ev[i + 1].record(p.stream)
        torch.cuda.synchronize()
        wall += time.perf_counter() - t0
        step_ms += [ev[i].elapsed_time(ev[i + 1]) for i in range(n)]
        if profile_level > 0:
            for back in range(min(n, 64)):
                dom_ms.append(B.mv_step_kernel_ms(p.ctx, back)[dom])
        left -= n
    B.mv_set_profiling(p.ctx, 0)
    return wall, step_ms, enqueue, dom_ms


def check_against_oracle(p, n_chk):
    """Runs the sequence's first n_chk steps once more (untimed) and compares the mask and the
    aggregate of step n_chk - 1 with the oracle's, which takes the same steps on the host."""
    np, torch, B, W = p.mods
    from oracle import mv_oracle
    w = p.w
    p.reset()
    for i in range(n_chk):
        p.step(i)
    torch.cuda.synchronize()
    mask = p.mask.cpu().numpy().view(np.uint32).copy()
    agg = p.agg.cpu().numpy().copy()
    threads = max(1, min(w.N, mv_oracle.max_threads(), 16))
    e = np.zeros((w.N, w.d), np.float32)
    vote = np.zeros((w.N, w.d), np.uint8) if p.ad else None
    msum = np.zeros(w.d, np.uint8) if p.ad else None
    ref = None
    for i in range(n_chk):
        if p.ad:
            ref = mv_oracle.ad_vote_step(p.g_host[i], e, w.K, w.K if i == 0 else p.k_ad, vote, msum, threads=threads)
            vote, msum = ref.vote, ref.msum
        elif p.rs:
            ref = mv_oracle.rs_vote_step(p.g_host[i], e, w.K, p.r_host[i], threads=threads)
        else:
            ref = mv_oracle.vote_step(p.g_host[i], e, w.K, threads=threads)
        e = ref.err
    return bool(np.array_equal(ref.mask_idx, mask) and np.array_equal(ref.agg.view(np.uint32), agg.view(np.uint32)))


def summarize(p, wall, step_ms, dom_ms, n_steps):
    np = p.mods[0]
    w = p.w
    coords = float(w.N) * float(w.d)
    bpc = 10.0 if p.bf16 else 12.0                     # read g, read e, write e
    ms = wall / n_steps * 1e3
    med = float(np.median(step_ms))
    out = {"ms_per_step": round(ms, 4), "ms_per_step_median_of_events": round(med, 4),
           "ms_per_step_mean_of_events": round(float(np.mean(step_ms)), 4),
           "coords_per_s": round(coords * n_steps / wall, 1),
           "step_hbm_frac_algorithmic": round(bpc * coords / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
           "step_hbm_frac_algorithmic_median": round(bpc * coords / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    if dom_ms:
        avg = float(np.mean(dom_ms))
        out["dominant_kernel_ms"] = round(avg, 4)
        out["dominant_kernel_frac"] = round(bpc * coords / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100,
                    help="timed steps: repeats of the workload's own sequence (C4: 5 steps), the last one cut short")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C4", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--k", type=int, default=0,
                    help="override the workload's K (e.g. 111740 = the paper's phi = 1e-2 on ResNet-18's size); "
                         "the headline figure is the workload's own K")
    ap.add_argument("--seq", type=int, default=0, help="override the length of the workload's sequence of steps")
    ap.add_argument("--scheme", default="mv", choices=["mv", "ad", "rs"],
                    help="mv: majority voting (Algorithm 1); ad: majority voting with add-drop (Algorithm 2), "
                         "a full first vote, then K_ad = K/10 per step; rs: majority voting with "
                         "random selection (Algorithm 1, S_rand-weighted), seeded Exp(1) numbers resident in HBM")
    ap.add_argument("--codec", action="store_true",
                    help="also time the sparse position code (Sec. 4.3.1) and the quantiser (Sec. 4.3.2) on the "
                         "workers' vote lists of the last step (untimed extra; scheme mv with worker_idx)")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="skip the extra key all_configs (the other workloads, each timed the same way)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle: no cpu_baseline, no agreement check")
    ap.add_argument("--oracle-steps", type=int, default=3,
                    help="steps of a sequence that the oracle re-computes for the agreement check of the "
                         "workloads under all_configs (the headline workload is checked over its whole sequence)")
    ap.add_argument("--no-worker-idx", action="store_true",
                    help="do not request the per-worker sorted vote lists (optional output)")
    ap.add_argument("--profile-level", type=int, default=1, choices=[0, 1, 2],
                    help="HIP events inside the library in the timed region: 1 = dominant kernel only, 2 = every kernel")
    ap.add_argument("--breakdown", action="store_true",
                    help="after the timed region, run the sequence once more with events around every kernel")
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
    mods = (np, torch, B, W)
    w = W.WORKLOADS[args.workload]
    if args.k > 0 or args.seq > 0:
        w = w.with_size(w.d, K=args.k if args.k > 0 else w.K, steps=args.seq if args.seq > 0 else w.steps)
    oracle_on = not args.no_cpu_baseline
    ad, rs = args.scheme == "ad", args.scheme == "rs"

    # ---- the headline workload
    p = Problem(w, args.scheme, not args.no_worker_idx, w.steps if oracle_on else 0, mods)
    N, d, K = w.N, w.d, w.K
    wall, step_ms, enqueue, dom_ms = time_sequence_repeats(p, args.steps, args.warmup, args.profile_level)
    head = summarize(p, wall, step_ms, dom_ms, args.steps)
    cand_last, _, slow_last = B.mv_last_step_row_stats(p.ctx, N)
    log("%s: %.4f ms per step (wall over %d steps), median of the steps' event times %.4f ms; last step: candidates "
        "per row min/max %d/%d, select path per row %s" % (w.name, head["ms_per_step"], args.steps,
                                                         head["ms_per_step_median_of_events"],
                                                         min(cand_last) & 0x7FFFFFFF, max(cand_last) & 0x7FFFFFFF,
                                                         slow_last))
    per_kernel = None
    if args.breakdown:
        names = B.kernel_names()
        B.mv_set_profiling(p.ctx, 2)
        acc = {n: [] for n in names}
        for rep in range(3):
            p.reset()
            for i in range(p.L):
                p.step(i)
                torch.cuda.synchronize()
                for nme, v in zip(names, B.mv_step_kernel_ms(p.ctx, 0)):
                    if v >= 0:
                        acc[nme].append(v)
        B.mv_set_profiling(p.ctx, 0)
        per_kernel = {n: round(float(np.median(v)) * 1e3, 2) for n, v in acc.items() if v}   # microseconds

    # ---- optional: the position code and the quantiser on the vote lists of the last step
    codec = None
    if args.codec and not ad and p.widx is not None:
        dev, stream, widx, mask = p.dev, p.stream, p.widx, p.mask
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
        q = 4   # the fractional quantiser (Sec. 4.3.2) on N x K values: the gradients at the mask's coordinates
        sent = p.g_dev[0][:, :d].float()[:, mask.long()].contiguous() if not p.bf16 else None
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
    src = torch.empty(N * p.ld_e, dtype=torch.float32, device=p.dev).normal_()
    dst = torch.empty_like(src)
    for _ in range(3):
        B.mv_probe_copy(dst, src, p.stream)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(p.stream)
    for _ in range(10):
        B.mv_probe_copy(dst, src, p.stream)
    ev1.record(p.stream)
    torch.cuda.synchronize()
    copy_gbs = 2.0 * src.numel() * 4 * 10 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    copy_bytes_each_way = src.numel() * 4
    del src, dst

    coords = float(N) * float(d)
    bytes_per_coord = 10.0 if p.bf16 else 12.0
    roofline = None
    if dom_ms:
        avg_ms = float(np.mean(dom_ms))
        achieved = bytes_per_coord * coords / (avg_ms * 1e-3) / 1e9
        tag = w.name if args.k == 0 else "%s_k%d" % (w.name, K)
        traffic, traffic_src = measured_traffic(tag) if not (ad or rs) else (None, None)
        roofline = {"bound": "hbm", "kernel": "mv_stream_collect", "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": traffic, "traffic_source": traffic_src,
                    "avg_kernel_ms": round(avg_ms, 4), "kernel_launches_timed": len(dom_ms),
                    "algorithmic_bytes_per_launch": bytes_per_coord * coords,
                    "algorithmic_bytes_rule": "%d B x %d x %s" % (bytes_per_coord, N, format(d, ",")),
                    "note": "the kernel also holds the threshold estimate (sampling workgroups at the head of its grid)"}

    # ---- the oracle on the host: agreement over the whole sequence, then its speed on one step
    cpu_baseline, oracle_agrees = None, None
    if oracle_on:
        from oracle import mv_oracle
        log("%s: the oracle re-computes the sequence's %d steps ..." % (w.name, p.L))
        oracle_agrees = check_against_oracle(p, p.L)
        threads = max(1, min(N, mv_oracle.max_threads(), 16))
        e0 = np.zeros((N, d), np.float32)
        log("%s: timing the oracle on step 0 with %d threads, then with one ..." % (w.name, threads))
        t1 = time.perf_counter()
        mv_oracle.vote_step(p.g_host[0], e0, K, threads=threads)
        t_or = time.perf_counter() - t1
        t1 = time.perf_counter()
        mv_oracle.vote_step(p.g_host[0], e0, K, threads=1)
        t_one = time.perf_counter() - t1
        cpu_baseline = {"value": round(coords / t_or, 1), "unit": "coords/s", "cores": threads,
                        "kind": "oracle", "seconds": round(t_or, 2),
                        "sample": "one full plain vote step of %s (all %d rows, d=%d), step-0 inputs" % (w.name, N, d),
                        "single_thread": {"value": round(coords / t_one, 1), "unit": "coords/s", "cores": 1,
                                          "seconds": round(t_one, 2), "sample": "the same full step"}}
    p.close()
    del p

    # ---- the other workloads, each timed the same way (extra key; the headline stays the workload above)
    all_configs = None
    if not args.no_all_configs and args.scheme == "mv" and args.workload == "C4" and args.k == 0:
        all_configs = {}
        extra = [W.C1, W.C2, W.C3, W.C5, W.C2.with_size(W.C2.d, K=111740)]
        for wx in extra:
            tag = wx.name if wx.K == W.WORKLOADS[wx.name].K else "%s_k%d" % (wx.name, wx.K)
            n_chk = min(wx.steps, max(1, args.oracle_steps)) if oracle_on else 0
            px = Problem(wx, "mv", not args.no_worker_idx, n_chk, mods)
            n_steps = 20 * px.L
            wl, sm, enq, dm = time_sequence_repeats(px, n_steps, min(px.L, 5), 1)
            rec = summarize(px, wl, sm, dm, n_steps)
            rec.update({"N": wx.N, "d": wx.d, "K": wx.K, "grads": wx.grad_dtype, "sequence_steps": px.L,
                        "steps_timed": n_steps, "host_enqueue_us_per_step": round(enq / n_steps * 1e6, 1)})
            if wx.name == "C1":
                rec["note"] = "working set fits the last-level cache: not an HBM measurement"
            if oracle_on:
                rec["oracle_agrees"] = check_against_oracle(px, n_chk)
                rec["oracle_steps_checked"] = n_chk
            log("%s: %.4f ms per step, median %.4f, whole-step frac %.3f%s" %
                (tag, rec["ms_per_step"], rec["ms_per_step_median_of_events"], rec["step_hbm_frac_algorithmic"],
                 ", oracle agrees: %s" % rec.get("oracle_agrees") if oracle_on else ""))
            all_configs[tag] = rec
            px.close()
            del px

    out = {
        "metric": "vote-step throughput (N*d coords/sec), 1 GPU" +
                  (", add-drop voting" if ad else ", random selection" if rs else ""),
        "value": head["coords_per_s"],
        "unit": "coords/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: N=%d d=%d K=%d grads=%s, %s; its %d-step sequence from a zero error buffer, "
                               "fresh seeded gradients every step, repeated" % (w.name, N, d, K, w.grad_dtype, w.kind,
                                                                                w.steps),
                   "N": N, "d": d, "K": K, "sequence_steps": w.steps,
                   "scheme": "majority voting with add-drop, K_ad=%d" % max(1, K // 10) if ad else
                             "majority voting with random selection" if rs else "majority voting",
                   "outputs": "mask_idx, agg_vals, add/drop lists, standing votes, vote sum" if ad else
                              "mask_idx, agg_vals, votes" + ("" if args.no_worker_idx else ", worker_idx")},
        "timing": "wall clock over the timed steps (error buffer zeroed outside the timed region before each repeat "
                  "of the sequence); every step also bracketed by HIP events on the stream",
        "ms_per_step_median_of_events": head["ms_per_step_median_of_events"],
        "ms_per_step_mean_of_events": head["ms_per_step_mean_of_events"],
        "host_enqueue_us_per_step": round(enqueue / args.steps * 1e6, 1),
        "step_hbm_frac_algorithmic": head["step_hbm_frac_algorithmic"],
        "step_hbm_frac_algorithmic_median": head["step_hbm_frac_algorithmic_median"],
        "copy_probe_GBs": round(copy_gbs, 1),
        "copy_probe_bytes_each_way": copy_bytes_each_way,
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "oracle_agrees_on_sequence": oracle_agrees,
        "launch": "eager",
        "slow_path_rows_last_step": int(sum(1 for x in slow_last if x == 1)),
        "paper_comm_load": comm_load_context(w),
    }
    if per_kernel:
        out["kernel_us_breakdown"] = per_kernel
    if codec:
        out["position_codec"] = codec
    if all_configs is not None:
        out["all_configs"] = all_configs
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
