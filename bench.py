#!/usr/bin/env python3
"""Benchmark of the SpecInF hot path on one MI355X.

Workload (BASELINE.json configs[1], "Data-parallel rank share"): a GPT-style decoder training step (12 layers,
d=768, 12 heads, seq 1024, micro-batch 8, bf16, vocab 50257) whose gradient all-reduce is modelled as one
4.98 ms bubble per step (248.9 MB at 50 GB/s), filled with offline inference of a BERT-base-shaped encoder
(12 layers, d=768, seq 128, batch 32, bf16).  One "step" = one collocated training step: all training kernels,
the bubble, the monitor / Algorithm 1 / barrier decisions and every inference kernel released into the bubble.

Prints ONE JSON line.  `value` = inference samples completed per second of wall time over the K timed steps,
with all inputs resident in HBM.  Also reported: training slowdown versus the solo run of the same K steps,
the fraction of bubble time covered by inference kernels, the roofline of the dominant kernel (the bf16 MFMA
GEMM, timed with HIP events on the stream it runs on), and the CPU oracle's throughput on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
# Kernel arguments in device memory: the command processor then fetches them from HBM instead of over PCIe, which
# takes about 1 us off each of the 5 us gaps between dependent kernels of a stream.  The HIP runtime reads the
# variable when it starts, so it is set before anything loads it; a value the caller has set is left alone.
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

MFMA_BF16_PEAK_TFLOPS = 2500.0
# Average HBM bytes per dispatch of gemm_bf16_kernel<0,0> in this workload, from the FETCH_SIZE / WRITE_SIZE counter
# runs summarised in profiles/bench_cfg2_hbm_traffic.md (counters cannot be read from inside a timed run).
GEMM00_HBM_BYTES_PER_LAUNCH = 368.1e6


def cpu_baseline(sample_batch):
    """The oracle's encoder forward (fp64 numpy, as it stands) on `sample_batch` samples of the fill workload."""
    import numpy as np
    import synth_inputs as Y
    from oracle import encoder as OE
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    cfg = Y.FILL_ENCODER
    w = OE.working_copy(Y.encoder_params(11, cfg), "bf16")
    ids = Y.token_ids(12, sample_batch, cfg["seq"], cfg["vocab"])
    t0 = time.time()
    OE.encoder_forward(w, ids, cfg, "bf16")
    dt = time.time() - t0
    return {"value": sample_batch / dt, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{sample_batch} samples of the fill encoder (12 layers, d=768, seq 128), one forward pass, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--coalesce", type=int, default=16, help="queued offline requests of equal shape released as one kernel sequence (1 = off)")
    ap.add_argument("--online-coalesce", type=int, default=8, help="online requests waiting together run as one kernel sequence (1 = one at a time)")
    ap.add_argument("--kernel-us-max", type=int, default=600, help="longest kernel the planner emits, us (the 4.98 ms bubble of this workload takes long kernels; the library's default of 300 is for shorter bubbles)")
    ap.add_argument("--period-us", type=int, default=0, help="monitor period P, us (0 = the library's default, 5)")
    ap.add_argument("--skip-concurrent", action="store_true", help="leave out the extra phase with concurrent filling (profiles of the headline phase: it is then the last thing the process does)")
    ap.add_argument("--feedback", action="store_true", help="offline phase with concurrent filling as well (kernels beside training within the allowance)")
    ap.add_argument("--feedback-eps-ppm", type=int, default=30000, help="online run with concurrent filling: step time allowed above its running minimum, ppm")
    ap.add_argument("--online-feedback-eps-ppm", type=int, default=40000, help="the same allowance for the online run with concurrent filling")
    ap.add_argument("--feedback-add-ppm", type=int, default=50000, help="online run with concurrent filling: share of busy time added per step while within the allowance, ppm")
    ap.add_argument("--cpu-sample", type=int, default=128, help="samples for the CPU oracle baseline (0 = skip)")
    ap.add_argument("--online-requests", type=int, default=2000, help="online phase (configs[4]): Poisson requests at 200/s; 0 = skip")
    ap.add_argument("--dp-bucket-mb", type=float, default=0.0,
                    help="offline phase only: exchange the gradients in buckets of at least this many MiB beside backward, so that only "
                         "the tail of the exchange is a bubble (0 = the configuration's single exposed all-reduce)")
    ap.add_argument("--allow-serial-streams", action="store_true", help="for runs under a counter-collecting profiler, which serialises all kernels")
    ap.add_argument("--small", action="store_true", help="reduced shapes (development only; not a valid measurement)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no second GPU); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth_inputs as Y
    import paper_2503_02550_amd as S
    from paper_2503_02550_amd import params as P
    from paper_2503_02550_amd.session import Session, decoder_shape, encoder_shape

    dev = "cuda:0"
    dec, enc = dict(Y.DP_DECODER), dict(Y.FILL_ENCODER)
    if args.small:
        dec.update(n_layers=2, vocab=4096, batch=2)
        enc.update(n_layers=2, vocab=4096)
    K, W = args.steps, args.warmup
    dshape, eshape = decoder_shape(dec), encoder_shape(enc)
    to = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(dt)

    dec_master = P.pack(dshape, Y.decoder_params(1, dec))
    enc_master = P.pack(eshape, Y.encoder_params(2, enc))
    ids_np, tg_np = Y.token_ids(3, dec["batch"], dec["seq"], dec["vocab"]), Y.token_ids(4, dec["batch"], dec["seq"], dec["vocab"])

    # ================= offline phase (configs[1]): the headline measurement =====================================
    cfg = S.sif_default_config()
    cfg.allow_serial_streams = 1 if args.allow_serial_streams else 0
    if args.kernel_us_max:
        cfg.kernel_us_max = args.kernel_us_max
    if args.period_us:
        cfg.period_us = args.period_us
    if args.feedback:
        cfg.feedback, cfg.feedback_eps_ppm, cfg.feedback_add_ppm = 1, args.feedback_eps_ppm, args.feedback_add_ppm
    with Session(cfg) as s:
        s.register_training(dshape, dec_master, par_mode=S.SIF_PAR_DP, lr=dec["lr"], bw_bytes_per_s=dec["bw_bytes_per_s"],
                            dp_bucket_bytes=int(args.dp_bucket_mb * 2 ** 20))
        m = s.register_inference(eshape, enc_master, coalesce=args.coalesce)
        ids, tg = to(ids_np, torch.int32), to(tg_np, torch.int32)
        eids = to(Y.token_ids(5, enc["batch"], enc["seq"], enc["vocab"]), torch.int32)
        outs = [torch.zeros((enc["batch"], enc["seq"], enc["d_model"]), device=dev, dtype=torch.bfloat16) for _ in range(4)]
        torch.cuda.synchronize()
        S.sif_calibrate(s.ctx, 3)

        def run_steps(n):
            for _ in range(n):
                s.step(ids, tg)

        # solo training: the barrier releases nothing.  Both timed regions carry the same event records around the
        # launches of the roofline kernel, so that the slowdown compares like with like.
        S.sif_set_collocate(s.ctx, 0)
        run_steps(W)
        s.sync()
        S.sif_profile_gemm(s.ctx, 2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(K)
        s.sync()
        solo_s = time.perf_counter() - t0
        S.sif_profile_gemm(s.ctx, 0)

        # collocation switched on with nothing to run: what the monitor and barrier threads cost the training step
        S.sif_set_collocate(s.ctx, 1)
        run_steps(W)
        s.sync()
        S.sif_profile_gemm(s.ctx, 2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(K)
        s.sync()
        idle_s = time.perf_counter() - t0
        S.sif_profile_gemm(s.ctx, 0)

        # collocated: offline batches queued ahead, released into the bubbles
        S.sif_reset_stats(s.ctx)
        S.sif_set_collocate(s.ctx, 1)
        per_step = 16
        for i in range(min(4000, (K + W + 1) * per_step)):
            s.submit_offline(m, eids, outs[i % 4], enc["batch"], enc["seq"])
        run_steps(W)
        s.sync()
        st0 = s.stats()
        S.sif_profile_gemm(s.ctx, 2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(K)
        s.sync()
        col_s = time.perf_counter() - t0
        st1 = s.stats()
        S.sif_profile_gemm(s.ctx, 0)
        prof = S.sif_profile_read(s.ctx)
        # scheduler latencies from the device trace of the timed steps: bubble start -> first inference kernel start,
        # bubble end -> end of the last inference kernel that began inside it (how far it runs into training time)
        tr_t, tr_i = S.sif_read_trace(s.ctx, 0), S.sif_read_trace(s.ctx, 1)
        bub = [(a, b) for kind, _, _, _, a, b in tr_t if kind == 3][-K:]
        ran = sorted((a, b) for kind, _, dec_, _, a, b in tr_i if kind == 2 and dec_ == 1)
        first_us, over_us = [], []
        import bisect
        starts = [a for a, _ in ran]
        for b0, b1 in bub:
            lo, hi = bisect.bisect_left(starts, b0), bisect.bisect_right(starts, b1)
            if hi > lo:
                first_us.append((ran[lo][0] - b0) / 1e3)
                over_us.append(max(0.0, (max(e for _, e in ran[lo:hi]) - b1) / 1e3))
        sched = {"bubbles": len(bub), "bubbles_with_inference": len(first_us),
                 "first_kernel_after_bubble_start_us_p50": float(np.median(first_us)) if first_us else None,
                 "overrun_past_bubble_end_us_p50": float(np.median(over_us)) if over_us else None,
                 "overrun_past_bubble_end_us_max": float(max(over_us)) if over_us else None}
        # all four GEMM variants, over a few more (untimed) collocated steps
        S.sif_profile_gemm(s.ctx, 1)
        run_steps(3)
        s.sync()
        S.sif_profile_gemm(s.ctx, 0)
        prof_all = S.sif_profile_read(s.ctx)

    # ================= the same offline load with concurrent filling (row N4: kernels also beside training) ==========
    # Not the headline: `value` is the paper's method, bubbles only.  Here the barrier also releases offline kernels
    # beside training, paced by the share of busy time that the feedback controller allows.
    concurrent = None
    if not args.feedback and not args.allow_serial_streams and not args.skip_concurrent:
        fcfg = S.sif_default_config()
        fcfg.kernel_us_max, fcfg.period_us, fcfg.feedback = cfg.kernel_us_max, cfg.period_us, 1
        fcfg.feedback_eps_ppm, fcfg.feedback_add_ppm = args.feedback_eps_ppm, args.feedback_add_ppm
        with Session(fcfg) as s:
            s.register_training(dshape, dec_master, par_mode=S.SIF_PAR_DP, lr=dec["lr"], bw_bytes_per_s=dec["bw_bytes_per_s"],
                                dp_bucket_bytes=int(args.dp_bucket_mb * 2 ** 20))
            m = s.register_inference(eshape, enc_master, coalesce=args.coalesce)
            ids, tg = to(ids_np, torch.int32), to(tg_np, torch.int32)
            torch.cuda.synchronize()
            S.sif_calibrate(s.ctx, 3)
            settle = 20                                        # steps over which the share finds its level
            for i in range(min(4000, (K + W + settle + 1) * 24)):
                s.submit_offline(m, eids, outs[i % 4], enc["batch"], enc["seq"])
            for _ in range(W + settle):
                s.step(ids, tg)
            s.sync()
            c0 = s.stats()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(K):
                s.step(ids, tg)
            s.sync()
            con_s = time.perf_counter() - t0
            c1 = s.stats()
            concurrent = {"value": (c1.offline_samples - c0.offline_samples) / con_s, "unit": "samples/s", "ms_per_step": 1e3 * con_s / K,
                          "training_slowdown": (con_s - solo_s) / solo_s, "slowdown_within_5pct": bool((con_s - solo_s) / solo_s <= 0.05),
                          "allowance_ppm": int(args.feedback_eps_ppm), "share_ppm_at_end": int(c1.concurrent_share_ppm)}

    # ================= online phase (configs[4]): same training step, Poisson requests, batch 1 ==================
    # Run at the configured 200 req/s and at a quarter of it: one 4.98 ms bubble per ~34 ms step holds only a few
    # batch-1 requests (each is ~110 launch-bound kernels), so the configured rate can exceed what the bubbles of one
    # GPU can serve; the second rate shows the latency of a load the bubbles do hold.
    online = None
    if args.online_requests > 0:
        import threading
        onl = dict(enc, batch=1, seq=Y.ONLINE["seq_max"])
        oshape = encoder_shape(onl)
        online = {}
        def online_phase(ocfg, runs, suffix):
            with Session(ocfg) as s:
                s.register_training(dshape, dec_master, par_mode=S.SIF_PAR_DP, lr=dec["lr"], bw_bytes_per_s=dec["bw_bytes_per_s"])
                mo = s.register_inference(oshape, enc_master, online=True, coalesce=args.online_coalesce)
                ids, tg = to(ids_np, torch.int32), to(tg_np, torch.int32)
                oids = to(Y.token_ids(7, 1, Y.ONLINE["seq_max"], enc["vocab"]), torch.int32)
                oouts = [torch.zeros((1, Y.ONLINE["seq_max"], enc["d_model"]), device=dev, dtype=torch.bfloat16) for _ in range(64)]
                torch.cuda.synchronize()
                slo = S.sif_calibrate(s.ctx, 3)
                for _ in range(W + (20 if ocfg.feedback else 0)):      # the share of concurrent filling settles over some steps
                    s.step(ids, tg)
                s.sync()
                for rate, n_req in runs:
                    t_arr, seqs = Y.poisson_arrivals(6, rate, n_req, Y.ONLINE["seq_min"], Y.ONLINE["seq_max"])
                    S.sif_reset_stats(s.ctx)
                    t_start = S.sif_now_ns()

                    def submitter():
                        for i in range(n_req):
                            while S.sif_now_ns() - t_start < int(t_arr[i]):
                                time.sleep(0.0002)
                            s.submit_online(mo, oids, oouts[i % 64], int(seqs[i]), t_start + int(t_arr[i]))

                    th = threading.Thread(target=submitter)
                    th.start()
                    n_steps, t0 = 0, time.perf_counter()
                    while th.is_alive():
                        s.step(ids, tg)
                        s.sync()
                        n_steps += 1
                    on_s = time.perf_counter() - t0
                    th.join()
                    drain = 0
                    while s.stats().online_done < n_req and drain < 400:      # bubbles for what is still queued
                        s.step(ids, tg)
                        s.sync()
                        drain += 1
                    so = s.stats()
                    online[f"{rate:g}_req_per_s{suffix}"] = {
                        "requests": n_req, "served_during_arrivals_plus_drain": int(so.online_done), "drain_steps": drain,
                        "p50_ms": so.online_p50_ns / 1e6, "p95_ms": so.online_p95_ns / 1e6,
                        "ms_per_step": 1e3 * on_s / max(1, n_steps),
                        "training_slowdown": (on_s / max(1, n_steps)) / (solo_s / K) - 1.0}
                    if ocfg.feedback:
                        online[f"{rate:g}_req_per_s{suffix}"]["concurrent_share_ppm"] = int(so.concurrent_share_ppm)
                return slo

        slo = online_phase(cfg, ((Y.ONLINE["rate_per_s"], args.online_requests), (Y.ONLINE["rate_per_s"] / 4, max(1, args.online_requests // 4))), "")
        # The same load with concurrent filling (this build's reading of the paper's outlook): a request need not wait
        # for the next bubble, its kernels run beside training, paced by the share of busy time that the feedback
        # controller allows (training step at most 4 % longer than its running minimum).
        fcfg = S.sif_default_config()
        fcfg.allow_serial_streams, fcfg.kernel_us_max, fcfg.period_us, fcfg.feedback = cfg.allow_serial_streams, cfg.kernel_us_max, cfg.period_us, 1
        fcfg.feedback_eps_ppm, fcfg.feedback_add_ppm = args.online_feedback_eps_ppm, args.feedback_add_ppm
        online_phase(fcfg, ((Y.ONLINE["rate_per_s"], args.online_requests),), "_beside_training")
        online["principle_2_ok"] = bool(slo == S.SIF_OK)

    samples = st1.offline_samples - st0.offline_samples
    bubble_ns = st1.bubble_ns - st0.bubble_ns
    filled_ns = st1.filled_ns - st0.filled_ns
    slowdown = (col_s - solo_s) / solo_s
    n00, f00, t00 = prof[0]              # A [M][K], B [N][K]: every forward product of both models
    all_f, all_t = sum(p[1] for p in prof_all), sum(p[2] for p in prof_all)      # every variant, from the extra untimed steps
    achieved = (f00 / t00 / 1e12) if t00 > 0 else 0.0
    out = {
        "metric": "filled inference samples/s at <=5% training slowdown",
        "value": samples / col_s,
        "unit": "samples/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": 1e3 * col_s / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1] data-parallel rank share: GPT decoder 12L d768 h12 seq1024 mb8 vocab50257 training step "
                               "+ 4.98 ms modelled all-reduce bubble, filled with BERT-base-shaped encoder inference 12L d768 seq128 batch32"
                               + (" [REDUCED --small]" if args.small else ""),
                   "bubble_model": "gradient bytes / 50 GB/s, host-timed" if args.dp_bucket_mb == 0 else
                                   f"[NOT the configuration's bubble] gradients exchanged in buckets of >= {args.dp_bucket_mb:g} MiB at 50 GB/s beside "
                                   "backward, only the tail exposed, host-timed",
                   "period_us": int(cfg.period_us)},
        "training_slowdown": slowdown,
        "slowdown_within_5pct": bool(slowdown <= 0.05),
        "solo_ms_per_step": 1e3 * solo_s / K,
        "bubble_fill_fraction": (filled_ns / bubble_ns) if bubble_ns else 0.0,
        "bubble_ms_per_step": bubble_ns / 1e6 / K,
        "inference_batches": int(st1.offline_batches - st0.offline_batches),
        "kernels_run": int(st1.kernels_run - st0.kernels_run), "kernels_skipped": int(st1.kernels_skipped - st0.kernels_skipped),
        "gate_violations": int(st1.gate_violations),
        "collocated_idle_overhead": (idle_s - solo_s) / solo_s,      # collocation on, nothing queued, against solo
        "scheduler_latency": sched,
        "with_concurrent_filling": concurrent,
        "online_p95_ms": online[f"{Y.ONLINE['rate_per_s']:g}_req_per_s"]["p95_ms"] if online else None,
        "online": online,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": GEMM00_HBM_BYTES_PER_LAUNCH,
                     "algorithmic_flops_per_launch": (f00 / n00) if n00 else None,
                     "kernel": "gemm_bf16_kernel<0,0>", "launches": int(n00), "avg_us": (1e6 * t00 / n00) if n00 else None,
                     "all_gemm_variants_tflops": (all_f / all_t / 1e12) if all_t > 0 else None},
        "paper_context": "paper (4x A100-40GB): up to 14x offline throughput over TGS, 67% lower online p95 than MPS; not comparable",
    }
    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(args.cpu_sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
