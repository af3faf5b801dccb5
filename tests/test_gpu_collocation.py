"""Scheduling invariants on the GPU (Sec. 2.2: training throughput is to be kept while inference is served beside
it): training results are bit-identical with and without collocation, inference
outputs are bit-identical to a solo run and match the oracle, and no inference kernel starts outside a bubble."""
import numpy as np
import pytest
import torch

import synth_inputs as Y
from oracle import encoder as OE
from oracle import mlp as OM

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2503_02550_amd as S
    from paper_2503_02550_amd import params as P
    from paper_2503_02550_amd.session import Session, decoder_shape, encoder_shape, mlp_shape
    from gpu_util import DEV, bf, f32, i32, up, q, assert_bf16_close, assert_f32_close


def bubbles_and_kernels(s, after_launch=0):
    """Bubble intervals of the training stream and the inference kernels launched after launch number
    `after_launch` (the calibration run comes before it and is ungated by design)."""
    tr = S.sif_read_trace(s.ctx, 0)
    inf = [r for r in S.sif_read_trace(s.ctx, 1) if r[3] > after_launch]
    bubbles = [(t0, t1) for kind, _, _, _, t0, t1 in tr if kind == 3]
    ran = [(t0, t1) for kind, _, dec, _, t0, t1 in inf if kind == 2 and dec == 1]
    skipped = sum(1 for kind, _, dec, _, _, _ in inf if kind == 2 and dec == 2)
    return bubbles, ran, skipped


def last_launch(s):
    tr = S.sif_read_trace(s.ctx, 1)
    return tr[-1][3] if tr else 0


def settled_stats(s, n_gated):
    """Statistics once the barrier thread has judged the start of every gated kernel that ran (it does so when it sees
    the kernel complete and its bubble end, a few microseconds after the streams are idle)."""
    import time
    t_end = time.time() + 2.0
    st = s.stats()
    while st.gate_checked + st.gate_unchecked < n_gated and time.time() < t_end:
        time.sleep(0.001)
        st = s.stats()
    return st


def assert_library_checked_every_start(s, ran):
    """The library's own check of the invariant (sif_stats.gate_violations) covered every kernel that ran."""
    st = settled_stats(s, len(ran))
    assert st.gate_checked == len(ran) and st.gate_unchecked == 0 and st.gate_violations == 0 and st.gate_timeouts == 0, \
        (st.gate_checked, st.gate_unchecked, st.gate_violations, st.gate_timeouts, len(ran))


def assert_starts_inside_bubbles(bubbles, ran):
    b0 = np.array([b[0] for b in bubbles]); b1 = np.array([b[1] for b in bubbles])
    for t0, _ in ran:
        i = np.searchsorted(b0, t0, side="right") - 1
        assert i >= 0 and b0[i] <= t0 <= b1[i], ("inference kernel started outside a bubble", t0)


def run_tiny(collocate, n_batches, steps=20):
    """Tiny configuration: fp32 MLP training with a fixed 2 ms bubble per step, MLP inference batches of 8."""
    c = Y.TINY_MLP
    shape, ishape = mlp_shape(c["d_in"], c["d_hidden"], c["d_out"], c["train_batch"]), mlp_shape(c["d_in"], c["d_hidden"], c["d_out"], c["infer_batch"])
    p_tr, p_inf = Y.mlp_params(0, c["d_in"], c["d_hidden"], c["d_out"]), Y.mlp_params(1, c["d_in"], c["d_hidden"], c["d_out"])
    cfg = S.sif_default_config()
    cfg.collocate = 1 if collocate else 0
    with Session(cfg) as s:
        s.register_training(shape, P.pack(shape, p_tr), par_mode=S.SIF_PAR_FIXED, lr=c["lr"], fixed_bubble_ns=c["bubble_ns"])
        m = s.register_inference(ishape, P.pack(ishape, p_inf))
        S.sif_calibrate(s.ctx, 2)
        n_cal = last_launch(s)
        xs = [f32(Y.activations(100 + i, c["infer_batch"], c["d_in"])) for i in range(n_batches)]
        outs = [torch.zeros((c["infer_batch"], c["d_out"]), device=DEV) for _ in range(n_batches)]
        batches = [tuple(f32(a) for a in Y.mlp_batch(0, st, c["train_batch"], c["d_in"], c["d_out"])) for st in range(steps)]
        losses = torch.zeros(steps, device=DEV)
        torch.cuda.synchronize()          # buffers are filled on torch's stream; the library uses its own two
        tickets = [s.submit_offline(m, xs[i], outs[i], c["infer_batch"]) for i in range(n_batches)]
        for st in range(steps):
            s.step(batches[st][0], batches[st][1], losses[st:st + 1])
        s.sync()
        if collocate:
            for t in tickets:
                s.wait(t, 20.0)
        stats = s.stats()
        trace = bubbles_and_kernels(s, n_cal)
        return up(s.train["master"]), up(losses), [up(o) for o in outs], stats, trace


def test_tiny_configuration_invariants():
    c = Y.TINY_MLP
    w_solo, l_solo, _, st_solo, _ = run_tiny(False, 0)
    w_col, l_col, outs, st, (bubbles, ran, skipped) = run_tiny(True, 64)
    assert np.array_equal(w_solo, w_col) and np.array_equal(l_solo, l_col)          # training untouched by collocation
    assert st.steps == 20 and len(bubbles) == 20
    assert all(b1 - b0 >= c["bubble_ns"] for b0, b1 in bubbles)                     # modelled wait is at least its length
    assert st.offline_batches == 64 and st.offline_samples == 64 * c["infer_batch"]
    assert len(ran) == 128 and st.kernels_run == 128 + 6                            # two kernels per batch, each ran once (+ calibration)
    assert_starts_inside_bubbles(bubbles, ran)
    # oracle and solo run
    p_inf = {k: v.astype(np.float64) for k, v in Y.mlp_params(1, c["d_in"], c["d_hidden"], c["d_out"]).items()}
    ishape = mlp_shape(c["d_in"], c["d_hidden"], c["d_out"], c["infer_batch"])
    with Session() as s:                                                            # no training instance: solo inference
        m = s.register_inference(ishape, P.pack(ishape, Y.mlp_params(1, c["d_in"], c["d_hidden"], c["d_out"])))
        for i in (0, 17, 63):
            x = Y.activations(100 + i, c["infer_batch"], c["d_in"])
            X, out = f32(x), torch.zeros((c["infer_batch"], c["d_out"]), device=DEV)
            torch.cuda.synchronize()
            s.wait(s.submit_offline(m, X, out, c["infer_batch"]))
            assert np.array_equal(up(out), outs[i])                                 # bit-identical to the solo run
            assert_f32_close(outs[i], OM.mlp_forward(p_inf, x)[0], "tiny inference")
    # training against the oracle: 20 SGD steps
    ref = {k: v.astype(np.float64) for k, v in Y.mlp_params(0, c["d_in"], c["d_hidden"], c["d_out"]).items()}
    for stp in range(20):
        x, t = Y.mlp_batch(0, stp, c["train_batch"], c["d_in"], c["d_out"])
        rl, ref, _ = OM.mlp_train_step(ref, x, t, c["lr"])
        assert abs(l_col[stp] - rl) <= 1e-4 * abs(rl)
    shape = mlp_shape(c["d_in"], c["d_hidden"], c["d_out"], c["train_batch"])
    got = P.unpack(shape, w_col)
    for k in ref:
        assert_f32_close(got[k], ref[k], k)


DEC = dict(n_layers=2, d_model=256, n_heads=4, d_head=64, d_ffn=1024, vocab=1000, max_pos=128, batch=4, seq=128, causal=True)
ENC = dict(n_layers=2, d_model=256, n_heads=4, d_head=64, d_ffn=1024, vocab=500, max_pos=64, batch=8, seq=64)


def run_transformer(collocate, n_batches, steps=6, bubble_ns=1_500_000, coalesce=0, tweak=None, extras=None):
    shape, ishape = decoder_shape(DEC), encoder_shape(ENC)
    cfg = S.sif_default_config()
    cfg.collocate = 1 if (collocate and not coalesce) else 0
    if tweak:
        tweak(cfg)
    with Session(cfg) as s:
        s.register_training(shape, P.pack(shape, Y.decoder_params(1, DEC)), par_mode=S.SIF_PAR_FIXED, lr=0.01, fixed_bubble_ns=bubble_ns)
        m = s.register_inference(ishape, P.pack(ishape, Y.encoder_params(2, ENC, perturb=True)), coalesce=coalesce)
        S.sif_calibrate(s.ctx, 2)
        n_cal = last_launch(s)
        ids = [i32(Y.token_ids(50 + i, ENC["batch"], ENC["seq"], ENC["vocab"])) for i in range(n_batches)]
        outs = [torch.zeros((ENC["batch"], ENC["seq"], ENC["d_model"]), device=DEV, dtype=torch.bfloat16) for _ in range(n_batches)]
        x, t = i32(Y.token_ids(3, DEC["batch"], DEC["seq"], DEC["vocab"])), i32(Y.token_ids(4, DEC["batch"], DEC["seq"], DEC["vocab"]))
        losses = torch.zeros(steps, device=DEV)
        torch.cuda.synchronize()
        tickets = [s.submit_offline(m, ids[i], outs[i], ENC["batch"], ENC["seq"]) for i in range(n_batches)]
        if collocate and coalesce:
            S.sif_set_collocate(s.ctx, 1)      # all requests are queued before the barrier admits the first
        for st in range(steps):
            s.step(x, t, losses[st:st + 1])
        s.sync()
        w, l = up(s.train["master"]), up(losses)
        if collocate:
            extra = 0                     # a slow host may need more bubbles than the steps compared with the solo run offer
            while s.stats().offline_batches < n_batches and extra < 40:
                s.step(x, t)
                s.sync()
                extra += 1
            for tk in tickets:
                s.wait(tk, 20.0)
        trace = bubbles_and_kernels(s, n_cal)
        if extras is not None:
            extras["release_log"] = S.sif_read_release_log(s.ctx)
            extras["stats"] = settled_stats(s, len(trace[1]))
            extras["n_cal"] = n_cal
        return w, l, outs, s.stats(), trace


def test_transformer_collocation_invariants():
    w_solo, l_solo, _, _, _ = run_transformer(False, 0)
    ex = {}
    w_col, l_col, outs, st, (bubbles, ran, skipped) = run_transformer(True, 6, extras=ex)
    assert np.array_equal(w_solo, w_col) and np.array_equal(l_solo, l_col)
    assert st.offline_batches == 6
    assert_starts_inside_bubbles(bubbles, ran)
    assert len(ran) + skipped == st.kernels_launched
    # the library's own check of the same invariant judged every kernel that ran, and found nothing
    sx = ex["stats"]
    assert sx.gate_checked == len(ran) and sx.gate_unchecked == 0 and sx.gate_violations == 0 and sx.gate_timeouts == 0
    assert st.filled_ns <= st.infer_busy_ns
    ishape = encoder_shape(ENC)
    master = Y.encoder_params(2, ENC, perturb=True)
    w = OE.working_copy(master, "bf16")
    with Session() as s:
        m = s.register_inference(ishape, P.pack(ishape, master))
        for i in (0, 5):
            ids = Y.token_ids(50 + i, ENC["batch"], ENC["seq"], ENC["vocab"])
            I, out = i32(ids), torch.zeros_like(outs[i])
            torch.cuda.synchronize()
            s.wait(s.submit_offline(m, I, out, ENC["batch"], ENC["seq"]))
            assert torch.equal(out, outs[i])                                       # same bits as the solo run
            assert_bf16_close(up(outs[i]), OE.encoder_forward(w, ids, ENC, "bf16"), "collocated encoder", elem_slack=1.5e-2)


def solo_encoder_outputs(indices, like):
    ishape = encoder_shape(ENC)
    master = Y.encoder_params(2, ENC, perturb=True)
    got = {}
    with Session() as s:
        m = s.register_inference(ishape, P.pack(ishape, master))
        for i in indices:
            I, out = i32(Y.token_ids(50 + i, ENC["batch"], ENC["seq"], ENC["vocab"])), torch.zeros_like(like)
            torch.cuda.synchronize()
            s.wait(s.submit_offline(m, I, out, ENC["batch"], ENC["seq"]))
            got[i] = out
    return got


def test_tokens_limit_what_is_forwarded_per_period_when_the_grant_is_small():
    """The offline token mechanism (Sec. 3.3 "Kernel Barrier") in a regime where it binds: period 100 us, grants of at
    most 100 tokens = 100 us of predicted kernel time per period.  From the barrier's own log of what it forwarded:
    the tokens taken within one period never exceed that period's grant, the grants are those Algorithm 1 can hand
    out, and the limit was reached in some periods (the next kernel had to wait for the next grant)."""
    def binding(cfg):
        cfg.period_us = 100
        cfg.alg1.alpha, cfg.alg1.beta, cfg.alg1.gamma_num, cfg.alg1.gamma_den, cfg.alg1.m = 1, 3, 2, 1, 1
        cfg.alg1.t0, cfg.alg1.ll, cfg.alg1.ul = 25, 50, 100
    ex = {}
    w_solo, l_solo, _, _, _ = run_transformer(False, 0)
    w_col, l_col, outs, st, (bubbles, ran, skipped) = run_transformer(True, 6, bubble_ns=3_000_000, tweak=binding, extras=ex)
    assert np.array_equal(w_solo, w_col) and np.array_equal(l_solo, l_col)
    assert st.offline_batches == 6
    assert_starts_inside_bubbles(bubbles, ran)
    log = [r for r in ex["release_log"] if r[4] > ex["n_cal"]]
    assert len(log) == st.kernels_launched and all(kind == 0 for *_, kind in log)
    per_period = {}
    for period, grant, model, charge, launch, kind in log:
        assert grant in (50, 100) and 1 <= charge <= 100, (grant, charge)          # incremental phase: LL; stable phase: UL
        tot, g = per_period.get(period, (0, grant))
        assert g == grant
        per_period[period] = (tot + charge, grant)
    assert all(tot <= g for tot, g in per_period.values()), [v for v in per_period.values() if v[0] > v[1]]
    biggest = max(c for _, _, _, c, _, _ in log)
    assert sum(1 for tot, g in per_period.values() if tot + biggest > g) >= 3      # the grant did run out
    assert len(per_period) >= sum(c for _, _, _, c, _, _ in log) / 100             # so the work needed that many periods
    for i, out in solo_encoder_outputs((0, 5), outs[0]).items():
        assert torch.equal(out, outs[i])


def test_launch_given_back_by_blocks_that_stop_waiting_for_the_gate_is_run_again():
    """A block of a speculatively launched kernel waits a bounded time for the decision of the launch's first block and
    then gives the launch back to the host.  Forced from the host here (every fifth launch waits for two polls only);
    every kernel exits normally, the launches are run again and every output keeps the bits of a run by itself."""
    def impatient(cfg):
        cfg.gate_spin_log2, cfg.gate_spin_every = 1, 5
    ex = {}
    w_solo, l_solo, _, _, _ = run_transformer(False, 0)
    w_col, l_col, outs, st, (bubbles, ran, skipped) = run_transformer(True, 6, steps=6, tweak=impatient, extras=ex)
    assert np.array_equal(w_solo, w_col) and np.array_equal(l_solo, l_col)
    assert st.offline_batches == 6
    assert ex["stats"].gate_timeouts != 0 and ex["stats"].gate_violations == 0
    assert_starts_inside_bubbles(bubbles, ran)
    for i, out in solo_encoder_outputs(range(6), outs[0]).items():
        assert torch.equal(out, outs[i]), i


def test_event_timing_of_gemm_launches_all_one_variant_or_every_third():
    """sif_profile_gemm: mode 1 times every GEMM launch, mode 2 the variant with both operands K-contiguous, mode 3 every
    third launch of that variant per stream; the flops of the timed launches follow, and the timing changes no result."""
    shape = decoder_shape(DEC)
    with Session() as s:
        s.register_training(shape, P.pack(shape, Y.decoder_params(1, DEC)), par_mode=S.SIF_PAR_NONE, lr=0.01)
        x, t = i32(Y.token_ids(3, DEC["batch"], DEC["seq"], DEC["vocab"])), i32(Y.token_ids(4, DEC["batch"], DEC["seq"], DEC["vocab"]))
        torch.cuda.synchronize()
        got = {}
        for mode in (1, 2, 3):
            S.sif_profile_gemm(s.ctx, mode)
            for _ in range(3):
                s.step(x, t)
            s.sync()
            S.sif_profile_gemm(s.ctx, 0)
            got[mode] = S.sif_profile_read(s.ctx)
        per_step = 4 * DEC["n_layers"] + 1                       # qkv, attention output, two MLP products per layer, LM head
        assert got[2][0][0] == 3 * per_step and all(got[2][v][0] == 0 for v in (1, 2, 3))
        assert got[1][0][0] == 3 * per_step and all(got[1][v][0] > 0 for v in (1, 3))
        assert got[3][0][0] == (3 * per_step + 2) // 3 and all(got[3][v][0] == 0 for v in (1, 2, 3))
        assert got[1][0][1] == got[2][0][1] and 0 < got[3][0][1] < got[2][0][1]
        assert all(g[0][2] > 0 for g in got.values())


def test_coalesced_offline_requests_give_the_same_bits_as_single_ones():
    """Queued requests of equal shape run as one kernel sequence over their concatenated rows; every request's
    output must be what a run by itself gives, and the scheduling invariants hold as before."""
    w_solo, l_solo, _, _, _ = run_transformer(False, 0)
    w_col, l_col, outs, st, (bubbles, ran, skipped) = run_transformer(True, 6, coalesce=3)
    assert np.array_equal(w_solo, w_col) and np.array_equal(l_solo, l_col)
    assert st.offline_batches == 6 and st.offline_samples == 6 * ENC["batch"]
    assert_starts_inside_bubbles(bubbles, ran)
    assert len(ran) + skipped == st.kernels_launched
    # two groups of three: one embedding launch for all three + its LayerNorm + 2 layers x 7 kernels (the last
    # LayerNorm writes every request's own output buffer)
    assert len(ran) == 2 * (1 + 1 + 2 * 7)
    ishape = encoder_shape(ENC)
    master = Y.encoder_params(2, ENC, perturb=True)
    with Session() as s:
        m = s.register_inference(ishape, P.pack(ishape, master))
        for i in range(6):
            I, out = i32(Y.token_ids(50 + i, ENC["batch"], ENC["seq"], ENC["vocab"])), torch.zeros_like(outs[i])
            torch.cuda.synchronize()
            s.wait(s.submit_offline(m, I, out, ENC["batch"], ENC["seq"]))
            assert torch.equal(out, outs[i]), i


def test_training_that_never_idles_starves_inference_without_deadlock():
    c = Y.TINY_MLP
    shape, ishape = mlp_shape(c["d_in"], c["d_hidden"], c["d_out"], c["train_batch"]), mlp_shape(c["d_in"], c["d_hidden"], c["d_out"], c["infer_batch"])
    with Session() as s:
        s.register_training(shape, P.pack(shape, Y.mlp_params(0, 256, 256, 256)), par_mode=S.SIF_PAR_NONE, lr=0.01)   # no bubbles
        m = s.register_inference(ishape, P.pack(ishape, Y.mlp_params(1, 256, 256, 256)))
        x, out = f32(Y.activations(1, 8, 256)), torch.zeros((8, 256), device=DEV)
        xb, tb = (f32(a) for a in Y.mlp_batch(0, 0, 32, 256, 256))
        torch.cuda.synchronize()
        tk = s.submit_offline(m, x, out, 8)
        for _ in range(200):
            s.step(xb, tb)
        s.sync()
        st = s.stats()
        assert st.kernels_run == 0 or st.offline_batches <= 1       # nothing may run while the training stream is busy
        with pytest.raises(S.SifError) as e:
            s.wait(tk, 0.05) if st.offline_batches == 0 else (_ for _ in ()).throw(S.SifError(S.SIF_E_TIMEOUT, "done"))
        assert e.value.status == S.SIF_E_TIMEOUT
    # destroy cancelled the pending ticket and returned


def test_online_requests_are_pulled_one_at_a_time_inside_bubbles():
    """Online fill (Sec. 3.3 "Kernel Barrier", pull-and-execute): Poisson arrivals, batch 1, ragged lengths."""
    import threading
    import time
    enc = dict(ENC, batch=1, seq=64)
    shape, ishape = decoder_shape(DEC), encoder_shape(enc)
    master = Y.encoder_params(2, enc, perturb=True)
    n_req = 40
    t_arr, seqs = Y.poisson_arrivals(7, 2000.0, n_req, 5, 64)          # 2000 req/s so that the test is short
    with Session() as s:
        s.register_training(shape, P.pack(shape, Y.decoder_params(1, DEC)), par_mode=S.SIF_PAR_FIXED, lr=0.01, fixed_bubble_ns=2_000_000)
        m = s.register_inference(ishape, P.pack(ishape, master), online=True)
        assert S.sif_calibrate(s.ctx, 2) == S.SIF_OK                     # Principle-II holds: a request is shorter than a bubble
        n_cal = last_launch(s)
        ids = [i32(Y.token_ids(200 + i, 1, int(seqs[i]), enc["vocab"])) for i in range(n_req)]
        outs = [torch.zeros((1, int(seqs[i]), enc["d_model"]), device=DEV, dtype=torch.bfloat16) for i in range(n_req)]
        x, t = i32(Y.token_ids(3, DEC["batch"], DEC["seq"], DEC["vocab"])), i32(Y.token_ids(4, DEC["batch"], DEC["seq"], DEC["vocab"]))
        torch.cuda.synchronize()
        tickets = [None] * n_req
        t0 = S.sif_now_ns()

        def submitter():
            for i in range(n_req):
                while S.sif_now_ns() - t0 < int(t_arr[i]):
                    time.sleep(0.0002)
                tickets[i] = s.submit_online(m, ids[i], outs[i], int(seqs[i]), t0 + int(t_arr[i]))

        th = threading.Thread(target=submitter)
        th.start()
        steps = 0
        while th.is_alive() or steps < 12:
            s.step(x, t)
            s.sync()
            steps += 1
        th.join()
        extra = 0
        while (s.stats().online_done < n_req and extra < 60) or extra < 6:       # a few more bubbles for the stragglers
            s.step(x, t)
            s.sync()
            extra += 1
        for tk in tickets:
            s.wait(tk, 20.0)
        st = s.stats()
        bubbles, ran, skipped = bubbles_and_kernels(s, n_cal)
        assert st.online_done == n_req and st.offline_batches == 0
        assert 0 < st.online_p50_ns <= st.online_p95_ns
        assert_starts_inside_bubbles(bubbles, ran)
    w = OE.working_copy(master, "bf16")
    with Session() as s:
        m = s.register_inference(ishape, P.pack(ishape, master), online=True)
        for i in (0, 11, 39):
            idn = Y.token_ids(200 + i, 1, int(seqs[i]), enc["vocab"])
            I, out = i32(idn), torch.zeros_like(outs[i])
            torch.cuda.synchronize()
            s.wait(s.submit_online(m, I, out, int(seqs[i])))
            assert torch.equal(out, outs[i])
            assert_bf16_close(up(outs[i]), OE.encoder_forward(w, idn, enc, "bf16"), "online request", elem_slack=1.5e-2)


def test_online_requests_take_priority_and_offline_batches_fill_the_rest():
    """Both kinds of inference instance on one GPU: queued online requests are served before the offline backlog, the
    offline batches use what the online load leaves of the bubbles, and every output has the bits of a solo run."""
    enc_on = dict(ENC, batch=1, seq=64)
    shape, off_shape, on_shape = decoder_shape(DEC), encoder_shape(ENC), encoder_shape(enc_on)
    m_off, m_on = Y.encoder_params(2, ENC, perturb=True), Y.encoder_params(8, enc_on, perturb=True)
    n_off, n_on = 16, 6
    cfg = S.sif_default_config()
    cfg.collocate = 0
    with Session(cfg) as s:
        s.register_training(shape, P.pack(shape, Y.decoder_params(1, DEC)), par_mode=S.SIF_PAR_FIXED, lr=0.01, fixed_bubble_ns=1_500_000)
        h_off = s.register_inference(off_shape, P.pack(off_shape, m_off))
        h_on = s.register_inference(on_shape, P.pack(on_shape, m_on), online=True)
        S.sif_calibrate(s.ctx, 2)
        n_cal = last_launch(s)
        ids_off = [i32(Y.token_ids(300 + i, ENC["batch"], ENC["seq"], ENC["vocab"])) for i in range(n_off)]
        out_off = [torch.zeros((ENC["batch"], ENC["seq"], ENC["d_model"]), device=DEV, dtype=torch.bfloat16) for _ in range(n_off)]
        seqs = [64, 17, 40, 64, 5, 33]
        ids_on = [i32(Y.token_ids(400 + i, 1, seqs[i], ENC["vocab"])) for i in range(n_on)]
        out_on = [torch.zeros((1, seqs[i], ENC["d_model"]), device=DEV, dtype=torch.bfloat16) for i in range(n_on)]
        x, t = i32(Y.token_ids(3, DEC["batch"], DEC["seq"], DEC["vocab"])), i32(Y.token_ids(4, DEC["batch"], DEC["seq"], DEC["vocab"]))
        torch.cuda.synchronize()
        tk = [s.submit_offline(h_off, ids_off[i], out_off[i], ENC["batch"], ENC["seq"]) for i in range(n_off)]     # the backlog comes first
        tk += [s.submit_online(h_on, ids_on[i], out_on[i], seqs[i]) for i in range(n_on)]
        S.sif_set_collocate(s.ctx, 1)
        online_done_at, offline_done_at = None, None
        for step in range(60):
            s.step(x, t)
            s.sync()
            st = s.stats()
            if online_done_at is None and st.online_done == n_on:
                online_done_at = (step, st.offline_batches)
            if offline_done_at is None and st.offline_batches == n_off:
                offline_done_at = step
            if online_done_at is not None and offline_done_at is not None:
                break
        for k in tk:
            s.wait(k, 20.0)
        assert online_done_at is not None and offline_done_at is not None
        assert online_done_at[1] < n_off, "the online requests waited for the whole offline backlog"
        bubbles, ran, skipped = bubbles_and_kernels(s, n_cal)
        assert_starts_inside_bubbles(bubbles, ran)
        assert s.stats().gate_violations == 0
    with Session() as s:
        h_off = s.register_inference(off_shape, P.pack(off_shape, m_off))
        h_on = s.register_inference(on_shape, P.pack(on_shape, m_on), online=True)
        for i in (0, n_off - 1):
            out = torch.zeros_like(out_off[i])
            torch.cuda.synchronize()
            s.wait(s.submit_offline(h_off, ids_off[i], out, ENC["batch"], ENC["seq"]))
            assert torch.equal(out, out_off[i])
        for i in range(n_on):
            out = torch.zeros_like(out_on[i])
            torch.cuda.synchronize()
            s.wait(s.submit_online(h_on, ids_on[i], out, seqs[i]))
            assert torch.equal(out, out_on[i])


def test_two_offline_instances_share_the_grant_and_neither_starves():
    """m = 2 inference instances (Algorithm 1 divides the pool by m; Fig. 7's setting): each spends its own share of
    every grant, so an instance with a short queue is not kept waiting by the other's backlog."""
    shape, ishape = decoder_shape(DEC), encoder_shape(ENC)
    masters = [Y.encoder_params(2, ENC, perturb=True), Y.encoder_params(9, ENC, perturb=True)]
    n_a, n_b = 14, 3
    cfg = S.sif_default_config()
    cfg.collocate = 0
    cfg.alg1.m = 2
    with Session(cfg) as s:
        s.register_training(shape, P.pack(shape, Y.decoder_params(1, DEC)), par_mode=S.SIF_PAR_FIXED, lr=0.01, fixed_bubble_ns=1_500_000)
        h = [s.register_inference(ishape, P.pack(ishape, m)) for m in masters]
        S.sif_calibrate(s.ctx, 2)
        n_cal = last_launch(s)
        ids = [i32(Y.token_ids(500 + i, ENC["batch"], ENC["seq"], ENC["vocab"])) for i in range(n_a + n_b)]
        outs = [torch.zeros((ENC["batch"], ENC["seq"], ENC["d_model"]), device=DEV, dtype=torch.bfloat16) for _ in range(n_a + n_b)]
        x, t = i32(Y.token_ids(3, DEC["batch"], DEC["seq"], DEC["vocab"])), i32(Y.token_ids(4, DEC["batch"], DEC["seq"], DEC["vocab"]))
        torch.cuda.synchronize()
        tk_a = [s.submit_offline(h[0], ids[i], outs[i], ENC["batch"], ENC["seq"]) for i in range(n_a)]
        tk_b = [s.submit_offline(h[1], ids[n_a + i], outs[n_a + i], ENC["batch"], ENC["seq"]) for i in range(n_b)]
        S.sif_set_collocate(s.ctx, 1)
        b_done_with = None
        for step in range(80):
            s.step(x, t)
            s.sync()
            while tk_b:                                   # an instance finishes its requests in order
                try:
                    s.wait(tk_b[0], 0.0)
                    tk_b.pop(0)
                except S.SifError:
                    break
            if not tk_b and b_done_with is None:
                b_done_with = int(s.stats().offline_batches)
            if s.stats().offline_batches == n_a + n_b:
                break
        for k in tk_a:
            s.wait(k, 20.0)
        assert b_done_with is not None and b_done_with < n_a + n_b - 2, "the short queue waited for the long one"
        bubbles, ran, skipped = bubbles_and_kernels(s, n_cal)
        assert_starts_inside_bubbles(bubbles, ran)
    for which, rng in ((0, (0, n_a - 1)), (1, (n_a, n_a + n_b - 1))):
        with Session() as s:
            hm = s.register_inference(ishape, P.pack(ishape, masters[which]))
            for i in rng:
                I, out = i32(Y.token_ids(500 + i, ENC["batch"], ENC["seq"], ENC["vocab"])), torch.zeros_like(outs[i])
                torch.cuda.synchronize()
                s.wait(s.submit_offline(hm, I, out, ENC["batch"], ENC["seq"]))
                assert torch.equal(out, outs[i]), (which, i)


# ---- bucketed gradient exchange beside backward (data parallel, overlapped): only the tail of it is a bubble
DEC4 = dict(n_layers=4, d_model=256, n_heads=4, d_head=64, d_ffn=1024, vocab=1000, max_pos=128, batch=4, seq=128, causal=True)


def dec4_groups():
    """Gradient bytes in the order backward finalizes them: layers last to first (the final LayerNorm with the last
    layer), then the embeddings."""
    d, f = DEC4["d_model"], DEC4["d_ffn"]
    layer = 2 * d + 3 * d * d + 3 * d + d * d + d + 2 * d + f * d + f + d * f + d
    return [2 * (layer + (2 * d if l == 0 else 0)) for l in range(DEC4["n_layers"])] + [2 * (DEC4["vocab"] + DEC4["max_pos"]) * d]


def run_overlapped(bucket_bytes, bw, device_timed, steps=3, n_batches=0, calibrate=False, all_steps=False):
    from oracle import bubbles as OB
    shape, ishape = decoder_shape(DEC4), encoder_shape(ENC)
    cfg = S.sif_default_config()
    cfg.device_timed_bubbles = 1 if device_timed else 0
    with Session(cfg) as s:
        h = s.register_training(shape, P.pack(shape, Y.decoder_params(1, DEC4)), par_mode=S.SIF_PAR_DP, lr=0.01, bw_bytes_per_s=bw,
                                dp_bucket_bytes=bucket_bytes)
        x, t = i32(Y.token_ids(3, DEC4["batch"], DEC4["seq"], DEC4["vocab"])), i32(Y.token_ids(4, DEC4["batch"], DEC4["seq"], DEC4["vocab"]))
        outs, ids, tickets, n_cal = [], [], [], 0
        if n_batches:
            m = s.register_inference(ishape, P.pack(ishape, Y.encoder_params(2, ENC, perturb=True)))
        if calibrate:                     # three training steps of its own, then the inference model's kernels
            torch.cuda.synchronize()
            S.sif_calibrate(s.ctx, 2, x, t)
            n_cal = last_launch(s)
        if n_batches:
            ids = [i32(Y.token_ids(50 + i, ENC["batch"], ENC["seq"], ENC["vocab"])) for i in range(n_batches)]
            outs = [torch.zeros((ENC["batch"], ENC["seq"], ENC["d_model"]), device=DEV, dtype=torch.bfloat16) for _ in range(n_batches)]
        torch.cuda.synchronize()
        tickets = [s.submit_offline(m, ids[i], outs[i], ENC["batch"], ENC["seq"]) for i in range(n_batches)]
        for _ in range(steps):
            s.step(x, t)
        s.sync()
        w = up(s.train["master"])
        buckets = S.sif_train_dp_buckets(s.ctx, h) if bucket_bytes else []
        tr = S.sif_read_trace(s.ctx, 0)
        marks = [i for i, r in enumerate(tr) if r[0] == 4]
        last = tr[marks[-2] + 1:marks[-1]] if len(marks) >= 2 else tr      # the last step: between its two markers
        # every step of this run: the records in front of each of its `steps` end markers (a step's begin marker leaves
        # no record of its own, so a step's records lie between the previous step's end marker and its own)
        per_step = [tr[(marks[i - 1] + 1 if i > 0 else 0):marks[i]] for i in range(len(marks) - steps, len(marks))] if all_steps else None
        extra = 0                         # a slow host may need more bubbles than the steps that are compared
        while s.stats().offline_batches < n_batches and extra < 60:
            s.step(x, t)
            s.sync()
            extra += 1
        for tk in tickets:
            s.wait(tk, 20.0)
        res = (w, buckets, last, s.stats(), (bubbles_and_kernels(s, n_cal) if n_batches else None), outs)
        return res + (per_step,) if all_steps else res


def test_overlapped_gradient_exchange_exposes_only_its_tail():
    from oracle import bubbles as OB
    cap, bw = 3_000_000, 10_000_000_000
    groups = dec4_groups()
    want_buckets = OB.dp_gradient_buckets(groups, cap)
    assert len(want_buckets) == 3
    _, _, last_plain, _, _, _ = run_overlapped(0, bw, True)
    for device_timed in (True, False):
        # Every step of the run is judged (the wait of each step against the oracle's value from that step's own
        # stamps).  Device-timed, every wait ends within 6 us of that value.  Host-timed, the monitor thread releases
        # it and may lose its core for a scheduling quantum now and then: the lower bound holds for every step, the
        # median step ends within 300 us, and none later than the device's own deadline would show (100 ms).
        steps = 3 if device_timed else 9
        w, buckets, _, st, _, _, per_step = run_overlapped(cap, bw, device_timed, steps=steps, all_steps=True)
        assert np.array_equal(w, run_overlapped(0, bw, True, steps=steps)[0])      # finalizing per bucket changes no gradient bit
        assert [b for b, _ in buckets] == [sum(groups[g] for g in grp) for grp in want_buckets]
        whole, = [t1 - t0 for kind, _, _, _, t0, t1 in last_plain if kind == 3]
        late = []
        for last in per_step:
            end_of = {rid: t1 for kind, rid, _, _, _, t1 in last if kind == 1}
            (b0, b1), = [(t0, t1) for kind, _, _, _, t0, t1 in last if kind == 3]
            ready = [end_of[r] for _, r in buckets]
            assert ready == sorted(ready) and ready[-1] <= b0
            dur = [OB.collective_ns(b, bw) for b, _ in buckets]
            want = OB.dp_overlapped_wait(ready, dur, b0)
            assert 0 < want < whole                                         # part of the exchange hid behind backward
            got = b1 - b0
            assert want - 500 <= got, (got, want, device_timed)
            late.append(got - want)
        assert len(late) == steps
        if device_timed:
            assert max(late) <= 6_000, late
        else:
            assert float(np.median(late)) <= 300_000 and max(late) <= 100_000_000, late
    # a link so fast that the exchange is over when backward ends: no bubble at all, the stream never goes idle
    _, _, last, st, _, _ = run_overlapped(cap, 10 ** 15, True)
    (b0, b1), = [(t0, t1) for kind, _, _, _, t0, t1 in last if kind == 3]
    assert b1 == b0 and st.bubble_ns == 0


def test_inference_fills_the_tail_of_an_overlapped_exchange():
    cap, bw = 3_000_000, 2_000_000_000          # ~1.6 ms per two-layer bucket: a tail long enough for the encoder's kernels
    w_solo, _, _, _, _, _ = run_overlapped(cap, bw, False)
    w_col, _, _, st, (bubbles, ran, skipped), outs = run_overlapped(cap, bw, False, steps=8, n_batches=4, calibrate=True)
    w_ref, _, _, _, _, _ = run_overlapped(cap, bw, False, steps=8, calibrate=True)
    assert np.array_equal(w_col, w_ref) and not np.array_equal(w_col, w_solo)
    assert st.offline_batches == 4 and st.gate_violations == 0
    assert_starts_inside_bubbles(bubbles, ran)
    ishape = encoder_shape(ENC)
    with Session() as s:
        m = s.register_inference(ishape, P.pack(ishape, Y.encoder_params(2, ENC, perturb=True)))
        for i in range(4):
            I, out = i32(Y.token_ids(50 + i, ENC["batch"], ENC["seq"], ENC["vocab"])), torch.zeros_like(outs[i])
            torch.cuda.synchronize()
            s.wait(s.submit_offline(m, I, out, ENC["batch"], ENC["seq"]))
            assert torch.equal(out, outs[i])


# ---- concurrent filling with feedback: offline kernels run beside training, paced by a share of busy time
def run_feedback(feedback, n_batches, steps=12):
    shape, ishape = decoder_shape(DEC), encoder_shape(ENC)
    cfg = S.sif_default_config()
    cfg.feedback, cfg.feedback_add_ppm, cfg.feedback_eps_ppm, cfg.feedback_cap_ppm = (1 if feedback else 0), 250_000, 100_000, 750_000
    with Session(cfg) as s:
        s.register_training(shape, P.pack(shape, Y.decoder_params(1, DEC)), par_mode=S.SIF_PAR_FIXED, lr=0.01, fixed_bubble_ns=300_000)
        m = s.register_inference(ishape, P.pack(ishape, Y.encoder_params(2, ENC, perturb=True)))
        x, t = i32(Y.token_ids(3, DEC["batch"], DEC["seq"], DEC["vocab"])), i32(Y.token_ids(4, DEC["batch"], DEC["seq"], DEC["vocab"]))
        torch.cuda.synchronize()
        S.sif_calibrate(s.ctx, 2, x, t)
        n_cal = last_launch(s)
        ids = [i32(Y.token_ids(50 + i, ENC["batch"], ENC["seq"], ENC["vocab"])) for i in range(n_batches)]
        outs = [torch.zeros((ENC["batch"], ENC["seq"], ENC["d_model"]), device=DEV, dtype=torch.bfloat16) for _ in range(n_batches)]
        torch.cuda.synchronize()
        tickets = [s.submit_offline(m, ids[i], outs[i], ENC["batch"], ENC["seq"]) for i in range(n_batches)]
        shares = []
        for _ in range(steps):
            s.step(x, t)
            s.sync()
            shares.append(s.stats().concurrent_share_ppm)
        w = up(s.train["master"])
        extra = 0
        while s.stats().offline_batches < n_batches and extra < 60:
            s.step(x, t)
            s.sync()
            extra += 1
        for tk in tickets:
            s.wait(tk, 20.0)
        return w, outs, s.stats(), bubbles_and_kernels(s, n_cal), shares


def test_concurrent_filling_with_feedback_keeps_every_result_bit():
    w_ref, _, _, _, _ = run_feedback(False, 0)
    w_fb, outs, st, (bubbles, ran, skipped), shares = run_feedback(True, 24)
    assert np.array_equal(w_ref, w_fb)                         # training does not see what runs beside it
    assert st.offline_batches == 24
    assert all(0 <= v <= 750_000 for v in shares) and max(shares) > 0
    b0 = np.array([b[0] for b in bubbles]); b1 = np.array([b[1] for b in bubbles])
    outside = 0
    for t0, _ in ran:
        i = np.searchsorted(b0, t0, side="right") - 1
        outside += not (i >= 0 and b0[i] <= t0 <= b1[i])
    assert outside > 0                                          # kernels did start while training was busy
    assert st.filled_ns < st.infer_busy_ns
    ishape = encoder_shape(ENC)
    with Session() as s:
        m = s.register_inference(ishape, P.pack(ishape, Y.encoder_params(2, ENC, perturb=True)))
        for i in (0, 11, 23):
            I, out = i32(Y.token_ids(50 + i, ENC["batch"], ENC["seq"], ENC["vocab"])), torch.zeros_like(outs[i])
            torch.cuda.synchronize()
            s.wait(s.submit_offline(m, I, out, ENC["batch"], ENC["seq"]))
            assert torch.equal(out, outs[i])
    # without the option the same load stays inside the bubbles
    _, _, st0, (bubbles0, ran0, _), shares0 = run_feedback(False, 2)
    assert_starts_inside_bubbles(bubbles0, ran0)
    assert max(shares0) == 0


def test_online_requests_that_wait_together_run_as_one_sequence():
    """Online requests of different lengths that are queued when one is pulled run as one kernel sequence over their
    rows laid back to back; each output has the bits of a run by itself, every kernel still starts inside a bubble,
    and far fewer kernels are launched than one sequence per request would take."""
    enc = dict(ENC, batch=1, seq=64)
    shape, ishape = decoder_shape(DEC), encoder_shape(enc)
    master = Y.encoder_params(2, enc, perturb=True)
    lens = [64, 5, 33, 17, 64, 48, 1, 29, 60, 12, 7, 40]
    n_req = len(lens)
    per_request = 2 + 7 * enc["n_layers"]                    # embed, its LayerNorm, seven kernels per layer
    cfg = S.sif_default_config()
    cfg.collocate = 0
    with Session(cfg) as s:
        s.register_training(shape, P.pack(shape, Y.decoder_params(1, DEC)), par_mode=S.SIF_PAR_FIXED, lr=0.01, fixed_bubble_ns=2_000_000)
        m = s.register_inference(ishape, P.pack(ishape, master), online=True, coalesce=8)
        assert S.sif_calibrate(s.ctx, 2) == S.SIF_OK
        n_cal = last_launch(s)
        ids = [i32(Y.token_ids(300 + i, 1, lens[i], enc["vocab"])) for i in range(n_req)]
        outs = [torch.zeros((1, lens[i], enc["d_model"]), device=DEV, dtype=torch.bfloat16) for i in range(n_req)]
        x, t = i32(Y.token_ids(3, DEC["batch"], DEC["seq"], DEC["vocab"])), i32(Y.token_ids(4, DEC["batch"], DEC["seq"], DEC["vocab"]))
        torch.cuda.synchronize()
        tickets = [s.submit_online(m, ids[i], outs[i], lens[i]) for i in range(n_req)]      # all wait before the first bubble
        S.sif_reset_stats(s.ctx)
        S.sif_set_collocate(s.ctx, 1)
        steps = 0
        while steps < 8 or (s.stats().online_done < n_req and steps < 60):
            s.step(x, t)
            s.sync()
            steps += 1
        for tk in tickets:
            s.wait(tk, 20.0)
        st = s.stats()
        bubbles, ran, skipped = bubbles_and_kernels(s, n_cal)
        assert st.online_done == n_req
        assert_starts_inside_bubbles(bubbles, ran)
        assert len(ran) < n_req * per_request // 2, (len(ran), n_req * per_request)
    w = OE.working_copy(master, "bf16")
    with Session() as s:
        m = s.register_inference(ishape, P.pack(ishape, master), online=True)
        for i in range(n_req):
            idn = Y.token_ids(300 + i, 1, lens[i], enc["vocab"])
            I, out = i32(idn), torch.zeros_like(outs[i])
            torch.cuda.synchronize()
            s.wait(s.submit_online(m, I, out, lens[i]))
            assert torch.equal(out, outs[i]), i
            if i in (0, 6, 9):
                assert_bf16_close(up(outs[i]), OE.encoder_forward(w, idn, enc, "bf16"), "coalesced online request", elem_slack=1.5e-2)


def test_online_requests_run_beside_training_with_concurrent_filling():
    """With concurrent filling on, an online request does not wait for the next bubble: its kernels are released
    beside training against the time account.  The training result keeps its bits, every output has the bits of a run
    by itself, kernels did start outside the bubbles, and without the option the same requests start inside bubbles
    only."""
    enc = dict(ENC, batch=1, seq=64)
    shape, ishape = decoder_shape(DEC), encoder_shape(enc)
    master = Y.encoder_params(2, enc, perturb=True)
    lens = [64, 5, 33, 17, 64, 48, 1, 29]
    n_req = len(lens)
    res = {}
    for feedback in (0, 1):
        cfg = S.sif_default_config()
        cfg.collocate = 0
        cfg.feedback, cfg.feedback_add_ppm, cfg.feedback_eps_ppm, cfg.feedback_cap_ppm = feedback, 250_000, 100_000, 750_000
        with Session(cfg) as s:
            s.register_training(shape, P.pack(shape, Y.decoder_params(1, DEC)), par_mode=S.SIF_PAR_FIXED, lr=0.01, fixed_bubble_ns=300_000)
            m = s.register_inference(ishape, P.pack(ishape, master), online=True, coalesce=4)
            x, t = i32(Y.token_ids(3, DEC["batch"], DEC["seq"], DEC["vocab"])), i32(Y.token_ids(4, DEC["batch"], DEC["seq"], DEC["vocab"]))
            S.sif_calibrate(s.ctx, 2, x, t)
            n_cal = last_launch(s)
            ids = [i32(Y.token_ids(300 + i, 1, lens[i], enc["vocab"])) for i in range(n_req)]
            outs = [torch.zeros((1, lens[i], enc["d_model"]), device=DEV, dtype=torch.bfloat16) for i in range(n_req)]
            torch.cuda.synchronize()
            S.sif_reset_stats(s.ctx)
            S.sif_set_collocate(s.ctx, 1)
            tickets = []
            for step in range(12):
                if step >= 2 and len(tickets) < n_req:         # the account is in credit after the first steps
                    tickets.append(s.submit_online(m, ids[len(tickets)], outs[len(tickets)], lens[len(tickets)]))
                s.step(x, t)
                s.sync()
            w = up(s.train["master"])
            extra = 0
            while s.stats().online_done < n_req and extra < 60:
                s.step(x, t)
                s.sync()
                extra += 1
            for tk in tickets:
                s.wait(tk, 20.0)
            st = s.stats()
            assert st.online_done == n_req
            res[feedback] = (w, [o.cpu() for o in outs], bubbles_and_kernels(s, n_cal), st)
    assert np.array_equal(res[0][0], res[1][0])                # training does not see what runs beside it
    bubbles0, ran0, _ = res[0][2]
    assert_starts_inside_bubbles(bubbles0, ran0)
    bubbles, ran, _ = res[1][2]
    b0 = np.array([b[0] for b in bubbles]); b1 = np.array([b[1] for b in bubbles])
    outside = 0
    for t0, _ in ran:
        i = np.searchsorted(b0, t0, side="right") - 1
        outside += not (i >= 0 and b0[i] <= t0 <= b1[i])
    assert outside > 0
    for i in range(n_req):
        assert torch.equal(res[0][1][i], res[1][1][i]), i     # and both are what a run by itself gives (tested above for the bubbles' path)
    with Session() as s:
        m = s.register_inference(ishape, P.pack(ishape, master), online=True)
        for i in (0, 6):
            I, out = i32(Y.token_ids(300 + i, 1, lens[i], enc["vocab"])), torch.zeros_like(res[1][1][i], device=DEV)
            torch.cuda.synchronize()
            s.wait(s.submit_online(m, I, out, lens[i]))
            assert torch.equal(out.cpu(), res[1][1][i]), i
