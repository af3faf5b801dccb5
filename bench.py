#!/usr/bin/env python3
"""Benchmark of the SpecInF hot path on one MI355X.

Headline workload (BASELINE.json configs[1], "Data-parallel rank share"): a GPT-style decoder training step (12
layers, d=768, 12 heads, seq 1024, micro-batch 8, bf16, vocab 50257) whose gradient all-reduce is modelled as one
4.98 ms bubble per step (248.9 MB at 50 GB/s), filled with offline inference of a BERT-base-shaped encoder (12
layers, d=768, seq 128, batch 32, bf16).  One "step" = one collocated training step: all training kernels, the
bubble, the monitor / Algorithm 1 / barrier decisions and every inference kernel released into the bubble.

Prints ONE JSON line.  `value` = inference samples completed per second of wall time over the K timed steps, with
all inputs resident in HBM.  Also reported: training slowdown versus the solo run of the same K steps (timed before
and after the collocated phase; the shorter of the two counts), the fraction of bubble time covered by inference
kernels, the roofline of the dominant kernel (the bf16 MFMA GEMM, timed with HIP events on the stream it runs on),
the CPU oracle's throughput on a bounded sample, and under `per_config` the same figures for the other
configurations (configs[0] Tiny, configs[2] pipeline stage, configs[3] tensor shard, configs[4] online).

`--kernel NAME --shape ...` instead times one kernel through the C ABI and prints one JSON line for it (the program
to put behind `rocprofv3 ... --` when a kernel's counters are wanted).
"""
import argparse
import bisect
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
HBM_PEAK_TBPS = 8.0
# Average bytes per dispatch of gemm_bf16_kernel<0,0> that pass between the L2s and the memory side in the headline
# workload, from the FETCH_SIZE / WRITE_SIZE counter runs summarised in the file named beside it (counters cannot be
# read from inside a timed run).
GEMM00_HBM_BYTES_PER_LAUNCH = 754.7e6
GEMM00_HBM_BYTES_SOURCE = "constant from profiles/bench_cfg2_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command)"
PROF_SAMPLED = 3     # sif_profile_gemm: event pairs around every third launch of the a_layout = b_layout = 0 variant per stream
N_RING = 64          # distinct input / output buffers the queued requests cycle through (a coalesced group is 32)


def oracle_cores():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline(sample_batch):
    """The oracle as it stands (fp64 numpy) on bounded samples of the headline workload: the fill encoder's forward
    pass on `sample_batch` samples (the figure comparable with `value`), and for the training side one decoder layer
    forward + backward at the full configs[1] shape (the whole step is that times 12 plus the vocabulary part:
    reported as a labelled extrapolation) and configs[0] in full."""
    import numpy as np
    import synth_inputs as Y
    from oracle import decoder as OD
    from oracle import encoder as OE
    from oracle import mlp as OM
    from oracle.numerics import Prec, bf16_round
    cores = oracle_cores()
    cfg = Y.FILL_ENCODER
    w = OE.working_copy(Y.encoder_params(11, cfg), "bf16")
    ids = Y.token_ids(12, sample_batch, cfg["seq"], cfg["vocab"])
    t0 = time.time()
    OE.encoder_forward(w, ids, cfg, "bf16")
    dt = time.time() - t0
    out = {"value": sample_batch / dt, "unit": "samples/s", "cores": cores, "kind": "oracle",
           "sample": f"{sample_batch} samples of the fill encoder (12 layers, d=768, seq 128), one forward pass, {dt:.1f} s"}
    # training side, configs[1]: one layer forward + backward at full shape
    dcfg = dict(Y.DP_DECODER, n_layers=1, vocab=0, max_pos=0)
    prec = Prec("bf16")
    wl = OD.working_copy(Y.decoder_params(13, dcfg), prec)["layers"]
    x = bf16_round(Y.activations(14, dcfg["batch"], dcfg["seq"], dcfg["d_model"]))
    dy = bf16_round(Y.activations(15, dcfg["batch"], dcfg["seq"], dcfg["d_model"], scale=0.01))
    t0 = time.time()
    OD.stack_fwd_bwd(wl, x, dy, dcfg, prec)
    dl = time.time() - t0
    # configs[0] in full: 20 training steps and 20 inference batches of 8
    c = Y.TINY_MLP
    p = {k: v.astype(np.float64) for k, v in Y.mlp_params(0, c["d_in"], c["d_hidden"], c["d_out"]).items()}
    t0 = time.time()
    for st in range(c["steps"]):
        xb, tb = Y.mlp_batch(0, st, c["train_batch"], c["d_in"], c["d_out"])
        _, p, _ = OM.mlp_train_step(p, xb, tb, c["lr"])
        OM.mlp_forward(p, xb[:c["infer_batch"]])
    dtiny = time.time() - t0
    out["training"] = {
        "configs[1]_one_decoder_layer_fwd_bwd_s": dl,
        "configs[1]_step_s_extrapolated": dl * Y.DP_DECODER["n_layers"],
        "extrapolation": "one layer forward + backward at full shape (8 x 1024 tokens, d 768) x 12 layers; embedding, LM head and loss not included",
        "configs[0]_20_steps_and_20_inference_batches_s": dtiny,
        "configs[0]_inference_samples_per_s": c["steps"] * c["infer_batch"] / dtiny,
    }
    return out


def kernel_mode(args):
    """One kernel through the C ABI: GEMM (M N K), fused attention forward (BATCH SEQ HEADS D_HEAD), LayerNorm forward
    (ROWS D), cross entropy (TOKENS VOCAB), SGD update (N).  Prints one JSON line with its time and rate."""
    import torch
    import paper_2503_02550_amd as S
    dev = "cuda:0"
    sh = args.shape
    rec = {"kernel": args.kernel, "shape": sh, "iters": args.iters}
    if args.kernel == "gemm":
        m, n, k = sh
        A = torch.randn((m, k) if args.a_layout == 0 else (k, m), device=dev).to(torch.bfloat16)
        B = torch.randn((n, k) if args.b_layout == 0 else (k, n), device=dev).to(torch.bfloat16)
        Cm = torch.zeros((m, n), device=dev, dtype=torch.bfloat16)
        bias = torch.zeros(n, device=dev, dtype=torch.bfloat16)
        res = torch.zeros((m, n), device=dev, dtype=torch.bfloat16) if args.epilogue & 4 else None

        def run():
            S.sif_k_gemm_bf16(A, B, Cm, m, n, k, A.shape[1], B.shape[1], n, a_layout=args.a_layout, b_layout=args.b_layout,
                              epilogue=args.epilogue, bias=bias, res=res, tile=args.tile)
        flops, nbytes = 2.0 * m * n * k, 2.0 * (m * k + n * k + m * n)
    elif args.kernel == "attn":
        b, sq, h, dh = sh
        da = h * dh
        qkv = torch.randn((b * sq, 3 * da), device=dev).to(torch.bfloat16)
        o = torch.zeros((b * sq, da), device=dev, dtype=torch.bfloat16)

        def run():
            S.sif_k_attn_fwd(qkv, o, b, sq, h, dh, 3 * da, da, 1 if args.causal else 0)
        flops, nbytes = 4.0 * b * h * sq * sq * dh * (0.5 if args.causal else 1.0), 8.0 * b * sq * da
    elif args.kernel == "layernorm":
        rows, d = sh
        x = torch.randn((rows, d), device=dev).to(torch.bfloat16)
        g, be = torch.ones(d, device=dev, dtype=torch.bfloat16), torch.zeros(d, device=dev, dtype=torch.bfloat16)
        y = torch.zeros_like(x)

        def run():
            S.sif_k_layernorm_fwd(x, g, be, y, None, None, rows, d)
        flops, nbytes = 0.0, 4.0 * rows * d
    elif args.kernel == "xent":
        tokens, vocab = sh
        ld = (vocab + 7) // 8 * 8
        logits = torch.randn((tokens, ld), device=dev).to(torch.bfloat16)
        tg = torch.randint(0, vocab, (tokens,), device=dev, dtype=torch.int32)
        loss = torch.zeros(tokens, device=dev)

        def run():
            S.sif_k_xent_fwd_bwd(logits, tg, loss, tokens, vocab, ld)
        flops, nbytes = 0.0, 4.0 * tokens * ld
    elif args.kernel == "sgd":
        # a streaming kernel of known traffic (6 B read and 6 B written per parameter): the reference that HBM byte
        # counters are scaled by
        n, = sh
        master = torch.randn(n, device=dev)
        grad = torch.randn(n, device=dev).to(torch.bfloat16)
        work = torch.zeros(n, device=dev, dtype=torch.bfloat16)

        def run():
            S.sif_k_sgd_bf16(master, grad, work, n, 1e-6)
        flops, nbytes = 0.0, 12.0 * n
    else:
        print(f"bench.py: unknown --kernel {args.kernel}", file=sys.stderr)
        sys.exit(2)
    for _ in range(3):
        run()
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(args.iters):
        run()
    t1.record()
    torch.cuda.synchronize()
    us = t0.elapsed_time(t1) * 1e3 / args.iters
    rec.update({"us": us, "algorithmic_bytes": nbytes, "TB_per_s": nbytes / us / 1e6, "frac_of_hbm_peak": nbytes / us / 1e6 / HBM_PEAK_TBPS})
    if flops:
        rec.update({"algorithmic_flops": flops, "TFLOP_per_s": flops / us / 1e6, "frac_of_mfma_peak": flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS})
    print(json.dumps(rec))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--configs", default="0,1,2,3,4", help="which configurations to run besides the headline configs[1] (comma-separated indices into BASELINE.json configs; 1 always runs)")
    ap.add_argument("--coalesce", type=int, default=32, help="queued offline requests of equal shape released as one kernel sequence (1 = off)")
    ap.add_argument("--pp-coalesce", type=int, default=8, help="configs[2]: queued requests released as one kernel sequence")
    ap.add_argument("--pp-kernel-us-max", type=int, default=1200, help="configs[2]: longest kernel the planner emits, us")
    ap.add_argument("--tp-coalesce", type=int, default=21, help="configs[3]: queued requests released as one kernel sequence")
    ap.add_argument("--tp-kernel-us-max", type=int, default=200, help="configs[3]: longest kernel the planner emits, us")
    ap.add_argument("--online-coalesce", type=int, default=8, help="online requests waiting together run as one kernel sequence (1 = one at a time, the paper's rule; it is always reported beside this)")
    ap.add_argument("--kernel-us-max", type=int, default=1200, help="longest kernel the planner emits for the headline workload, us (its 4.98 ms bubble takes long kernels; configs[3] always uses 200)")
    ap.add_argument("--period-us", type=int, default=0, help="monitor period P, us (0 = the library's default, 5)")
    ap.add_argument("--skip-concurrent", action="store_true", help="leave out the extra phases with concurrent filling and with binding tokens (profiles of the headline phase)")
    ap.add_argument("--timed-region-last", action="store_true", help="end the headline phase with its timed collocated steps (no further steps with all GEMM variants timed, no second solo phase): in a kernel trace of the process the last dispatches are then those of the timed region")
    ap.add_argument("--feedback", action="store_true", help="headline phase with concurrent filling as well (kernels beside training within the allowance)")
    ap.add_argument("--feedback-eps-ppm", type=int, default=30000, help="concurrent filling: step time allowed above its running minimum, ppm")
    ap.add_argument("--online-feedback-eps-ppm", type=int, default=40000, help="the same allowance for the online run with concurrent filling")
    ap.add_argument("--feedback-add-ppm", type=int, default=50000, help="concurrent filling: share of busy time added per step while within the allowance, ppm")
    ap.add_argument("--cpu-sample", type=int, default=64, help="samples for the CPU oracle baseline (0 = skip)")
    ap.add_argument("--online-requests", type=int, default=2000, help="configs[4]: Poisson requests at 200/s; 0 = skip")
    ap.add_argument("--dp-bucket-mb", type=float, default=0.0,
                    help="headline phase only: exchange the gradients in buckets of at least this many MiB beside backward, so that only "
                         "the tail of the exchange is a bubble (0 = the configuration's single exposed all-reduce)")
    ap.add_argument("--allow-serial-streams", action="store_true", help="for runs under a counter-collecting profiler, which serialises all kernels")
    ap.add_argument("--small", action="store_true", help="reduced shapes (development only; not a valid measurement)")
    ap.add_argument("--kernel", default="", help="single-kernel mode: gemm | attn | layernorm | xent | sgd")
    ap.add_argument("--shape", type=int, nargs="+", default=[], help="single-kernel mode: gemm M N K; attn BATCH SEQ HEADS D_HEAD; layernorm ROWS D; xent TOKENS VOCAB; sgd N")
    ap.add_argument("--tile", type=int, default=0)
    ap.add_argument("--a-layout", type=int, default=0, help="gemm: 0 A stored [M][K], 1 [K][M]")
    ap.add_argument("--b-layout", type=int, default=0, help="gemm: 0 B stored [N][K], 1 [K][N]")
    ap.add_argument("--epilogue", type=int, default=0, help="gemm: SIF_EPI_* bits (1 bias, 2 GELU, 4 residual)")
    ap.add_argument("--causal", action="store_true")
    ap.add_argument("--iters", type=int, default=10)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no second GPU); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.kernel:
        return kernel_mode(args)
    legs = {int(v) for v in args.configs.split(",") if v.strip() != ""}

    import numpy as np
    import torch
    import synth_inputs as Y
    import paper_2503_02550_amd as S
    from paper_2503_02550_amd import params as P
    from paper_2503_02550_amd.session import Session, decoder_shape, encoder_shape, mlp_shape

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

    def fill_buffers(e):
        """N_RING distinct token-id tensors and output buffers: every request of a coalesced group (and of the groups in
        flight beside it) reads its own ids and writes its own rows."""
        ids = [to(Y.token_ids(1000 + i, e["batch"], e["seq"], e["vocab"]), torch.int32) for i in range(N_RING)]
        outs = [torch.zeros((e["batch"], e["seq"], e["d_model"]), device=dev, dtype=torch.bfloat16) for _ in range(N_RING)]
        return ids, outs

    def timed_steps(s, n, step):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            step()
        s.sync()
        return time.perf_counter() - t0

    def trace_summary(s, n_bubbles):
        """Scheduler latencies from the device trace: bubble start -> first inference kernel start, bubble end -> end of
        the last inference kernel that began inside it; and the longest inference kernel that ran."""
        tr_t, tr_i = S.sif_read_trace(s.ctx, 0), S.sif_read_trace(s.ctx, 1)
        bub = [(a, b) for kind, _, _, _, a, b in tr_t if kind == 3][-n_bubbles:]
        ran = sorted((a, b) for kind, _, dec_, _, a, b in tr_i if kind == 2 and dec_ == 1)
        first_us, over_us, longest = [], [], 0.0
        starts = [a for a, _ in ran]
        for b0, b1 in bub:
            lo, hi = bisect.bisect_left(starts, b0), bisect.bisect_right(starts, b1)
            if hi > lo:
                first_us.append((ran[lo][0] - b0) / 1e3)
                over_us.append(max(0.0, (max(e for _, e in ran[lo:hi]) - b1) / 1e3))
                longest = max(longest, max((e - a) / 1e3 for a, e in ran[lo:hi]))
        return {"bubbles": len(bub), "bubbles_with_inference": len(first_us),
                "first_kernel_after_bubble_start_us_p50": float(np.median(first_us)) if first_us else None,
                "overrun_past_bubble_end_us_p50": float(np.median(over_us)) if over_us else None,
                "overrun_past_bubble_end_us_max": float(max(over_us)) if over_us else None,
                "longest_inference_kernel_us": longest}

    def offline_leg(cfg, register, step_inputs, e, emaster, coalesce, k, w, queue_per_step, bubbles_per_step, calibrate_with_inputs=True):
        """Solo steps, collocated steps with offline batches queued ahead, solo steps again; the shorter solo time counts."""
        with Session(cfg) as s:
            register(s)
            m = s.register_inference(encoder_shape(e) if "d_model" in e else e["shape"], emaster, coalesce=coalesce)
            ids, outs = e["buffers"]() if "buffers" in e else fill_buffers(e)
            a, b = step_inputs
            torch.cuda.synchronize()
            if calibrate_with_inputs:
                S.sif_calibrate(s.ctx, 3, a, b)
            else:
                S.sif_calibrate(s.ctx, 3)
            step = lambda: s.step(a, b)
            S.sif_set_collocate(s.ctx, 0)
            for _ in range(w):
                step()
            s.sync()
            solo_a = timed_steps(s, k, step)
            S.sif_reset_stats(s.ctx)
            n_sub = min(3900, (k + w + 1) * queue_per_step)
            for i in range(n_sub):
                s.submit_offline(m, ids[i % N_RING], outs[i % N_RING], e["batch"], e.get("seq", 1))
            S.sif_set_collocate(s.ctx, 1)
            for _ in range(w):
                step()
            s.sync()
            st0 = s.stats()
            col = timed_steps(s, k, step)
            st1 = s.stats()
            sched = trace_summary(s, k * bubbles_per_step)
            S.sif_set_collocate(s.ctx, 0)              # what is still queued stays queued; destroy cancels it
            for _ in range(w):
                step()
            s.sync()
            solo_b = timed_steps(s, k, step)
            fin = s.stats()
        solo = min(solo_a, solo_b)
        bubble_ns, filled_ns = st1.bubble_ns - st0.bubble_ns, st1.filled_ns - st0.filled_ns
        samples = st1.offline_samples - st0.offline_samples
        return {"samples_per_s": samples / col, "steps": k, "ms_per_step": 1e3 * col / k, "solo_ms_per_step": 1e3 * solo / k,
                "solo_ms_per_step_before_and_after": [1e3 * solo_a / k, 1e3 * solo_b / k],
                "training_slowdown": (col - solo) / solo, "slowdown_within_5pct": bool((col - solo) / solo <= 0.05),
                "bubble_fill_fraction": (filled_ns / bubble_ns) if bubble_ns else 0.0, "bubble_ms_per_step": bubble_ns / 1e6 / k,
                "queue_ran_dry": bool(st1.offline_batches + max(1, coalesce) > n_sub),
                "kernels_run": int(st1.kernels_run - st0.kernels_run), "kernels_skipped": int(st1.kernels_skipped - st0.kernels_skipped),
                "gate_violations": int(fin.gate_violations), "gate_checked": int(fin.gate_checked), "gate_unchecked": int(fin.gate_unchecked),
                "scheduler_latency": sched}

    per_config = {}

    # ================= configs[0] Tiny: fp32 MLP training, fixed 2 ms bubble, MLP inference batches of 8 ============
    if 0 in legs:
        c = Y.TINY_MLP
        tshape, ishape = mlp_shape(c["d_in"], c["d_hidden"], c["d_out"], c["train_batch"]), mlp_shape(c["d_in"], c["d_hidden"], c["d_out"], c["infer_batch"])
        xb, tb = (to(a, torch.float32) for a in Y.mlp_batch(0, 0, c["train_batch"], c["d_in"], c["d_out"]))

        def tiny_buffers():
            ids = [to(Y.activations(100 + i, c["infer_batch"], c["d_in"]), torch.float32) for i in range(N_RING)]
            outs = [torch.zeros((c["infer_batch"], c["d_out"]), device=dev) for _ in range(N_RING)]
            return ids, outs
        tcfg = S.sif_default_config()
        r = offline_leg(tcfg, lambda s: s.register_training(tshape, P.pack(tshape, Y.mlp_params(0, c["d_in"], c["d_hidden"], c["d_out"])),
                                                            par_mode=S.SIF_PAR_FIXED, lr=c["lr"], fixed_bubble_ns=c["bubble_ns"]),
                        (xb, tb), dict(shape=ishape, batch=c["infer_batch"], buffers=tiny_buffers), P.pack(ishape, Y.mlp_params(1, c["d_in"], c["d_hidden"], c["d_out"])),
                        0, c["steps"], 2, 190, 1, calibrate_with_inputs=False)
        r["workload"] = "configs[0] Tiny: 2-layer fp32 MLP training step (hidden 256, batch 32) + fixed 2 ms bubble, 20 steps; fill: 2-layer fp32 MLP inference, batch 8"
        r["dtype"] = "f32"
        per_config["configs[0]"] = r

    # ================= configs[1]: the headline measurement =========================================================
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
        eids, outs = fill_buffers(enc)
        torch.cuda.synchronize()
        S.sif_calibrate(s.ctx, 3)
        step = lambda: s.step(ids, tg)

        def run_steps(n):
            for _ in range(n):
                step()

        # solo training: the barrier releases nothing.  All timed regions carry the same event records around every
        # third launch of the roofline kernel on each stream (an event pair takes about 2 us of its stream's time: around
        # every launch the pairs cost the inference stream 2.5 % of a bubble; a layer's launches come in fours, so every
        # shape is sampled alike), so that the slowdown compares like with like.
        S.sif_set_collocate(s.ctx, 0)
        run_steps(W)
        s.sync()
        S.sif_profile_gemm(s.ctx, PROF_SAMPLED)
        solo_a = timed_steps(s, K, step)
        S.sif_profile_gemm(s.ctx, 0)

        # collocation switched on with nothing to run: what the monitor and barrier threads cost the training step
        S.sif_set_collocate(s.ctx, 1)
        run_steps(W)
        s.sync()
        S.sif_profile_gemm(s.ctx, PROF_SAMPLED)
        idle_s = timed_steps(s, K, step)
        S.sif_profile_gemm(s.ctx, 0)

        # collocated: offline batches queued ahead, released into the bubbles
        S.sif_reset_stats(s.ctx)
        S.sif_set_collocate(s.ctx, 1)
        per_step = 16
        n_sub = min(3900, (K + W + 1) * per_step)
        for i in range(n_sub):
            s.submit_offline(m, eids[i % N_RING], outs[i % N_RING], enc["batch"], enc["seq"])
        run_steps(W)
        s.sync()
        st0 = s.stats()
        S.sif_profile_gemm(s.ctx, PROF_SAMPLED)
        col_s = timed_steps(s, K, step)
        st1 = s.stats()
        S.sif_profile_gemm(s.ctx, 0)
        prof = S.sif_profile_read(s.ctx)
        sched = trace_summary(s, K)
        prof_all, solo_b = prof, solo_a
        if not args.timed_region_last:
            # all four GEMM variants, over a few more (untimed) collocated steps
            S.sif_profile_gemm(s.ctx, 1)
            run_steps(3)
            s.sync()
            S.sif_profile_gemm(s.ctx, 0)
            prof_all = S.sif_profile_read(s.ctx)
            # solo once more, after the collocated phase (whatever is still queued stays queued)
            S.sif_set_collocate(s.ctx, 0)
            run_steps(W)
            s.sync()
            S.sif_profile_gemm(s.ctx, PROF_SAMPLED)
            solo_b = timed_steps(s, K, step)
            S.sif_profile_gemm(s.ctx, 0)
        fin = s.stats()
    solo_s = min(solo_a, solo_b)

    # ================= the same offline load in other regimes (not the headline) ====================================
    concurrent, binding = None, None
    if not args.feedback and not args.allow_serial_streams and not args.skip_concurrent:
        # (a) concurrent filling (this build's reading of the paper's outlook for PP): the barrier also releases offline
        # kernels beside training, paced by the share of busy time that the feedback controller allows.
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
            for i in range(min(3900, (K + W + settle + 1) * 24)):
                s.submit_offline(m, eids[i % N_RING], outs[i % N_RING], enc["batch"], enc["seq"])
            for _ in range(W + settle):
                s.step(ids, tg)
            s.sync()
            c0 = s.stats()
            con_s = timed_steps(s, K, lambda: s.step(ids, tg))
            c1 = s.stats()
            concurrent = {"value": (c1.offline_samples - c0.offline_samples) / con_s, "unit": "samples/s", "ms_per_step": 1e3 * con_s / K,
                          "training_slowdown": (con_s - solo_s) / solo_s, "slowdown_within_5pct": bool((con_s - solo_s) / solo_s <= 0.05),
                          "allowance_ppm": int(args.feedback_eps_ppm), "share_ppm_at_end": int(c1.concurrent_share_ppm)}
        # (b) constants of Algorithm 1 with which the tokens limit what is forwarded: period 100 us, grants of at most
        # 100 tokens (= 100 us of predicted kernel time) per period.  With the defaults the grant never binds.
        bcfg = S.sif_default_config()
        bcfg.kernel_us_max, bcfg.period_us = 100, 100
        bcfg.alg1.t0, bcfg.alg1.ll, bcfg.alg1.ul = 25, 50, 100
        kb = max(10, K // 5)
        with Session(bcfg) as s:
            s.register_training(dshape, dec_master, par_mode=S.SIF_PAR_DP, lr=dec["lr"], bw_bytes_per_s=dec["bw_bytes_per_s"])
            m = s.register_inference(eshape, enc_master, coalesce=args.coalesce)
            ids, tg = to(ids_np, torch.int32), to(tg_np, torch.int32)
            torch.cuda.synchronize()
            S.sif_calibrate(s.ctx, 3)
            for i in range(min(3900, (kb + W + 1) * per_step)):
                s.submit_offline(m, eids[i % N_RING], outs[i % N_RING], enc["batch"], enc["seq"])
            for _ in range(W):
                s.step(ids, tg)
            s.sync()
            b0 = s.stats()
            bin_s = timed_steps(s, kb, lambda: s.step(ids, tg))
            b1 = s.stats()
            log = S.sif_read_release_log(s.ctx)
            spent = {}
            for period, grant, _, charge, _, kind in log:
                if kind == 0:
                    spent[period] = (spent.get(period, (0, grant))[0] + charge, grant)
            binding = {"period_us": 100, "t0": 25, "LL": 50, "UL": 100, "kernel_us_max": 100, "steps": kb,
                       "value": (b1.offline_samples - b0.offline_samples) / bin_s, "unit": "samples/s", "ms_per_step": 1e3 * bin_s / kb,
                       "training_slowdown": (bin_s / kb) / (solo_s / K) - 1.0,
                       "bubble_fill_fraction": (b1.filled_ns - b0.filled_ns) / max(1, b1.bubble_ns - b0.bubble_ns),
                       "periods_with_releases": len(spent), "tokens_spent_over_grant_max": max([t / g for t, g in spent.values() if g] + [0.0]),
                       "periods_where_the_grant_ran_out": sum(1 for t, g in spent.values() if t + 100 > g)}

    # ================= configs[2] pipeline stage, configs[3] tensor shard ===========================================
    def stack_master(shape, seed):
        """Parameters of a layer stack: weights N(0, 0.02), LayerNorm gains 1, offsets and biases 0, drawn straight into
        the flat layout (the nested generator of the tests takes several times longer at these sizes)."""
        rng = np.random.default_rng(seed)
        flat = np.empty(S.sif_model_n_params(shape), dtype=np.float32)
        off = 0
        for path, shp in P.layout(shape):
            n = int(np.prod(shp))
            key = path if isinstance(path, str) else path[2]
            if len(shp) == 2:
                flat[off:off + n] = rng.standard_normal(n, dtype=np.float32) * np.float32(0.02)
            else:
                flat[off:off + n] = 1.0 if key.endswith("_g") else 0.0
            off += n
        return flat

    def stack_leg(name, dcfg, ecfg, coalesce, kernel_us_max, k, par):
        shp = decoder_shape(dcfg)
        master = stack_master(shp, 31)
        micro = dcfg["n_micro"] if par == "pp" else 1
        dims = (micro, dcfg["batch"], dcfg["seq"], dcfg["d_model"]) if micro > 1 else (dcfg["batch"], dcfg["seq"], dcfg["d_model"])
        x = to(Y.activations(32, *dims), torch.bfloat16)
        # upstream gradient N(0, 1) / sqrt(batch * seq * d): the SGD steps of this linear objective then stay small
        dy = to(Y.activations(33, *dims, scale=1.0 / np.sqrt(dcfg["batch"] * dcfg["seq"] * dcfg["d_model"])), torch.bfloat16)
        lcfg = S.sif_default_config()
        lcfg.kernel_us_max = kernel_us_max

        def register(s):
            if par == "pp":
                s.register_training(shp, master, par_mode=S.SIF_PAR_PP, lr=dcfg["lr"], pp_stages=dcfg["n_stages"], pp_micro=micro, pp_stage=dcfg["stage"])
            else:
                s.register_training(shp, master, par_mode=S.SIF_PAR_TP, lr=dcfg["lr"], bw_bytes_per_s=dcfg["bw_bytes_per_s"])
        bubbles = 5 if par == "pp" else 4 * dcfg["n_layers"]
        emaster = P.pack(encoder_shape(ecfg), Y.encoder_params(2, ecfg))
        # enough queued work for every bubble of every step: ~16 k (pp) / ~17 k (tp) samples/s times the step time, and half as much again
        per_step = 56 if par == "pp" else 150
        r = offline_leg(lcfg, register, (x, dy), ecfg, emaster, coalesce, k, 2, per_step, bubbles)
        r["workload"] = name
        r["dtype"] = "bf16"
        r["kernel_us_max"] = kernel_us_max
        return r

    if 2 in legs and not args.small:
        per_config["configs[2]"] = stack_leg(
            "configs[2] pipeline stage: 1F1B, stage 1 of 4, 8 micro-batches, 6 decoder layers d2048 h16x128 seq2048 mb2; idle intervals of the "
            "schedule sized from the measured pass times; fill: 6-layer d512 encoder seq256 batch64", Y.PP_DECODER, Y.PP_FILL_ENCODER, args.pp_coalesce, args.pp_kernel_us_max, 12, "pp")
    if 3 in legs and not args.small:
        per_config["configs[3]"] = stack_leg(
            "configs[3] tensor shard: 24 decoder layers, d4096 split 1/8 (4 local heads of 128, d_ffn 2048), batch 4 x seq2048; 96 bubbles of 1.34 ms "
            "per step (2 activation all-reduces per layer and pass at 50 GB/s); fill: 12-layer d768 encoder seq128 batch32 in kernels <= 200 us",
            Y.TP_DECODER, Y.FILL_ENCODER, args.tp_coalesce, args.tp_kernel_us_max, 8, "tp")

    # ================= configs[4] online: same training step, Poisson requests, batch 1 ==============================
    # At the configured 200 req/s, with the requests that wait together run as one kernel sequence (this build's
    # coalescing) and pulled strictly one by one (the paper's rule); one by one at a quarter of the rate as well: one
    # 4.98 ms bubble per 19 ms step holds about three batch-1 requests run one at a time (each is 86 launch-bound
    # kernels), so one by one the configured rate exceeds what the bubbles can serve and the latency is queueing.
    online = None
    if args.online_requests > 0 and 4 in legs:
        import threading
        onl = dict(enc, batch=1, seq=Y.ONLINE["seq_max"])
        oshape = encoder_shape(onl)
        online = {}
        n_slots = 256

        def online_phase(ocfg, coalesce, runs, suffix, label):
            with Session(ocfg) as s:
                s.register_training(dshape, dec_master, par_mode=S.SIF_PAR_DP, lr=dec["lr"], bw_bytes_per_s=dec["bw_bytes_per_s"])
                mo = s.register_inference(oshape, enc_master, online=True, coalesce=coalesce)
                ids, tg = to(ids_np, torch.int32), to(tg_np, torch.int32)
                oids = [to(Y.token_ids(2000 + i, 1, Y.ONLINE["seq_max"], enc["vocab"]), torch.int32) for i in range(n_slots)]
                oouts = [torch.zeros((1, Y.ONLINE["seq_max"], enc["d_model"]), device=dev, dtype=torch.bfloat16) for _ in range(n_slots)]
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
                            s.submit_online(mo, oids[i % n_slots], oouts[i % n_slots], int(seqs[i]), t_start + int(t_arr[i]))

                    th = threading.Thread(target=submitter)
                    th.start()
                    n_steps, t0 = 0, time.perf_counter()
                    while th.is_alive():
                        s.step(ids, tg)
                        s.sync()
                        n_steps += 1
                    on_s = time.perf_counter() - t0
                    th.join()
                    served_in_time = int(s.stats().online_done)
                    drain = 0
                    while s.stats().online_done < n_req and drain < 600:      # bubbles for what is still queued
                        s.step(ids, tg)
                        s.sync()
                        drain += 1
                    so = s.stats()
                    online[f"{rate:g}_req_per_s{suffix}"] = {
                        "rule": label, "requests": n_req, "served_while_requests_arrived": served_in_time, "served_after_drain": int(so.online_done),
                        "drain_steps": drain, "p50_ms": so.online_p50_ns / 1e6, "p95_ms": so.online_p95_ns / 1e6,
                        "ms_per_step": 1e3 * on_s / max(1, n_steps),
                        "training_slowdown": (on_s / max(1, n_steps)) / (solo_s / K) - 1.0,
                        "gate_violations": int(so.gate_violations)}
                    if ocfg.feedback:
                        online[f"{rate:g}_req_per_s{suffix}"]["concurrent_share_ppm"] = int(so.concurrent_share_ppm)
                return slo

        rate, n_on = Y.ONLINE["rate_per_s"], args.online_requests
        slo = online_phase(cfg, args.online_coalesce, ((rate, n_on),), "", f"requests that wait together run as one kernel sequence (up to {args.online_coalesce}; this build's addition)")
        if args.online_coalesce != 1:
            online_phase(cfg, 1, ((rate, n_on), (rate / 4, max(1, n_on // 4))), "_one_by_one", "requests pulled and run strictly one by one (the paper's pull-and-execute rule)")
        if not args.skip_concurrent and not args.allow_serial_streams:
            # The same load with concurrent filling (this build's reading of the paper's outlook): a request need not wait
            # for the next bubble, its kernels run beside training, paced by the share of busy time the controller allows.
            fcfg = S.sif_default_config()
            fcfg.allow_serial_streams, fcfg.kernel_us_max, fcfg.period_us, fcfg.feedback = cfg.allow_serial_streams, cfg.kernel_us_max, cfg.period_us, 1
            fcfg.feedback_eps_ppm, fcfg.feedback_add_ppm = args.online_feedback_eps_ppm, args.feedback_add_ppm
            online_phase(fcfg, args.online_coalesce, ((rate, n_on),), "_beside_training", "concurrent filling with feedback (this build's reading of the paper's outlook), coalesced")
        online["principle_2_ok"] = bool(slo == S.SIF_OK)
        head = online[f"{rate:g}_req_per_s"]
        per_config["configs[4]"] = {"workload": "configs[4] online: the configs[1] training step + Poisson arrivals at 200 req/s, 12-layer d768 encoder, seq uniform in [32,256], batch 1",
                                    "p50_ms": head["p50_ms"], "p95_ms": head["p95_ms"], "training_slowdown": head["training_slowdown"],
                                    "p50_ms_one_by_one": online.get(f"{rate:g}_req_per_s_one_by_one", {}).get("p50_ms"),
                                    "p95_ms_one_by_one": online.get(f"{rate:g}_req_per_s_one_by_one", {}).get("p95_ms"), "dtype": "bf16"}

    samples = st1.offline_samples - st0.offline_samples
    bubble_ns = st1.bubble_ns - st0.bubble_ns
    filled_ns = st1.filled_ns - st0.filled_ns
    slowdown = (col_s - solo_s) / solo_s
    n00, f00, t00 = prof[0]              # A [M][K], B [N][K]: every forward product of both models
    all_f, all_t = sum(p[1] for p in prof_all), sum(p[2] for p in prof_all)      # every variant, from the extra untimed steps
    achieved = (f00 / t00 / 1e12) if t00 > 0 else 0.0
    per_config["configs[1]"] = {"workload": "headline (see config.workload)", "samples_per_s": samples / col_s, "training_slowdown": slowdown,
                                "bubble_fill_fraction": (filled_ns / bubble_ns) if bubble_ns else 0.0,
                                "kernels_skipped": int(st1.kernels_skipped - st0.kernels_skipped), "dtype": "bf16"}
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
                   "period_us": int(cfg.period_us), "offline_coalesce": int(args.coalesce), "kernel_us_max": int(cfg.kernel_us_max),
                   "queued_requests": f"every queued request has its own token ids and output buffer out of {N_RING} distinct ones"},
        "training_slowdown": slowdown,
        "slowdown_within_5pct": bool(slowdown <= 0.05),
        "solo_ms_per_step": 1e3 * solo_s / K,
        "solo_ms_per_step_before_and_after": [1e3 * solo_a / K, 1e3 * solo_b / K],
        "bubble_fill_fraction": (filled_ns / bubble_ns) if bubble_ns else 0.0,
        "bubble_ms_per_step": bubble_ns / 1e6 / K,
        "inference_batches": int(st1.offline_batches - st0.offline_batches),
        "queue_ran_dry": bool(st1.offline_batches + max(1, args.coalesce) > n_sub),
        "kernels_run": int(st1.kernels_run - st0.kernels_run), "kernels_skipped": int(st1.kernels_skipped - st0.kernels_skipped),
        "gate_violations": int(fin.gate_violations), "gate_checked": int(fin.gate_checked), "gate_unchecked": int(fin.gate_unchecked),
        "collocated_idle_overhead": (idle_s - solo_s) / solo_s,      # collocation on, nothing queued, against solo
        "scheduler_latency": sched,
        "with_concurrent_filling": concurrent,
        "with_binding_tokens": binding,
        "per_config": per_config,
        "online_p95_ms": online[f"{Y.ONLINE['rate_per_s']:g}_req_per_s"]["p95_ms"] if online else None,
        "online": online,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": GEMM00_HBM_BYTES_PER_LAUNCH, "traffic_source": GEMM00_HBM_BYTES_SOURCE,
                     "algorithmic_flops_per_launch": (f00 / n00) if n00 else None,
                     "kernel": "gemm_bf16_kernel<0,0>", "launches": int(n00), "launches_are": "every third launch of the kernel on each stream in the timed region (HIP event pairs)",
                     "avg_us": (1e6 * t00 / n00) if n00 else None,
                     "all_gemm_variants_tflops": (all_f / all_t / 1e12) if all_t > 0 else None},
        "paper_context": "paper (4x A100-40GB): up to 14x offline throughput over TGS, 67% lower online p95 than MPS; not comparable",
    }
    if args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(args.cpu_sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
