"""The pipeline-stage and tensor-shard configurations at their stated shapes (Sec. 5.2, the MP and PP experiments:
short, numerous bubbles).

  * one layer of each training model at full shape, forward and backward, against the oracle: 2 x 2048 tokens,
    d 2048, 16 heads of 128, d_ffn 8192 (pipeline stage) and 4 x 2048 tokens, d 4096, 4 local heads of 128, local
    d_ffn 2048 (tensor shard) - the fused d_head-128 attention path and the tile configurations those shapes select;
  * each configuration as a whole (6 layers, 1F1B with 4 stages x 8 micro-batches, its 6-layer d 512 fill encoder;
    24 layers with 96 bubbles of 1.34 ms per step, fills in kernels of at most 200 us): training keeps its bits
    with and without collocation, inference outputs have the bits of a run alone and match the oracle on sampled
    rows, every inference kernel starts inside a bubble, and for the tensor shard no inference kernel that ran
    lasted longer than the limit.
The whole-model oracle cannot run these sizes in seconds; per-layer parity plus the properties above stand in."""
import numpy as np
import pytest
import torch

import synth_inputs as Y
from oracle import decoder as OD
from oracle import encoder as OE
from oracle.numerics import Prec

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2503_02550_amd as S
    from paper_2503_02550_amd import params as P
    from paper_2503_02550_amd.session import Session, decoder_shape, encoder_shape
    from gpu_util import assert_deep_bf16_close, DEV, bf, i32, up, q, rel_err, assert_bf16_close


@pytest.mark.parametrize("which", ["pipeline-stage-layer", "tensor-shard-layer"])
def test_one_layer_at_full_shape_forward_and_backward_matches_oracle(which):
    base = Y.PP_DECODER if which == "pipeline-stage-layer" else Y.TP_DECODER
    cfg = dict(base, n_layers=1)
    shape = decoder_shape(cfg)
    master = Y.decoder_params(4, cfg, perturb=True)
    b, sq, d = cfg["batch"], cfg["seq"], cfg["d_model"]
    x, dy = Y.activations(5, b, sq, d), Y.activations(6, b, sq, d, scale=0.01)
    with Session() as s:
        s.register_training(shape, P.pack(shape, master), par_mode=S.SIF_PAR_NONE, lr=0.0)
        X, DY = bf(x), bf(dy)
        torch.cuda.synchronize()
        s.step(X, DY)
        s.sync()
        got = {name: up(s.train_tensor(name, 0)) for name in ("ln1", "qkv", "o", "x_mid", "ln2", "z", "a", "x_out")}
        got_dx = up(s.train_tensor("dx_in"))
        got_g = P.unpack(shape, up(s.train_tensor("grads")))
    prec = Prec("bf16")
    w = OD.working_copy(master, prec)
    ry, rdx, rgr, caches = OD.stack_fwd_bwd(w["layers"], q(x), q(dy), cfg, prec)
    c = caches[0]
    for name in ("ln1", "qkv", "o", "x_mid", "ln2", "z", "a"):
        assert_bf16_close(got[name].reshape(c[name].shape), c[name], f"{which} {name}", elem_slack=8e-3)
    assert_bf16_close(got["x_out"].reshape(ry.shape), ry, f"{which} output", elem_slack=8e-3)
    assert_bf16_close(got_dx.reshape(rdx.shape), rdx, f"{which} input gradient", elem_slack=2e-2)
    for k in OD.LAYER_KEYS:
        assert_bf16_close(got_g["layers"][0][k], rgr[0][k], f"{which} gradient of {k}", elem_slack=2e-2)


def _trace(s, n_cal):
    tr = S.sif_read_trace(s.ctx, 0)
    inf = [r for r in S.sif_read_trace(s.ctx, 1) if r[3] > n_cal]
    bubbles = [(t0, t1) for kind, _, _, _, t0, t1 in tr if kind == 3]
    ran = [(t0, t1) for kind, _, dec, _, t0, t1 in inf if kind == 2 and dec == 1]
    return bubbles, ran


def _assert_inside(bubbles, ran):
    b0 = np.array([b[0] for b in bubbles]); b1 = np.array([b[1] for b in bubbles])
    for t0, _ in ran:
        i = np.searchsorted(b0, t0, side="right") - 1
        assert i >= 0 and b0[i] <= t0 <= b1[i], ("inference kernel started outside a bubble", t0)


def _run_config(dec, enc, n_batches, steps, coalesce, kernel_us_max, register):
    """Solo steps, then the same steps collocated with `n_batches` queued fill batches.  Returns the master parameters
    after each phase, the fill outputs, statistics and the trace of the collocated phase."""
    dshape, eshape = decoder_shape(dec), encoder_shape(enc)
    dmaster = P.pack(dshape, Y.decoder_params(21, dec))
    emaster_np = Y.encoder_params(22, enc, perturb=True)
    emaster = P.pack(eshape, emaster_np)
    micro = dec.get("n_micro", 1) if "n_stages" in dec else 1
    shape_x = (micro, dec["batch"], dec["seq"], dec["d_model"]) if micro > 1 else (dec["batch"], dec["seq"], dec["d_model"])
    # upstream gradient N(0, 1) / sqrt(batch * seq * d): with it the SGD steps of this linear objective stay small
    x, dy = Y.activations(23, *shape_x), Y.activations(24, *shape_x, scale=1.0 / np.sqrt(dec["batch"] * dec["seq"] * dec["d_model"]))
    eids = [Y.token_ids(300 + i, enc["batch"], enc["seq"], enc["vocab"]) for i in range(n_batches)]
    res = {}
    for collocate in (0, 1):
        cfg = S.sif_default_config()
        cfg.collocate = 0
        cfg.kernel_us_max = kernel_us_max
        with Session(cfg) as s:
            register(s, dshape, dmaster)
            m = s.register_inference(eshape, emaster, coalesce=coalesce)
            X, DY = bf(x), bf(dy)
            torch.cuda.synchronize()
            S.sif_calibrate(s.ctx, 2, X, DY)
            n_cal = (S.sif_read_trace(s.ctx, 1) or [(0, 0, 0, 0)])[-1][3]
            E = [i32(e) for e in eids]
            outs = [torch.zeros((enc["batch"], enc["seq"], enc["d_model"]), device=DEV, dtype=torch.bfloat16) for _ in range(n_batches)]
            torch.cuda.synchronize()
            S.sif_reset_stats(s.ctx)
            tickets = [s.submit_offline(m, E[i], outs[i], enc["batch"], enc["seq"]) for i in range(n_batches)] if collocate else []
            S.sif_set_collocate(s.ctx, collocate)
            for _ in range(steps):
                s.step(X, DY)
            s.sync()
            st = s.stats()
            res[collocate] = dict(master=s.train["master"].clone().cpu().view(torch.int32), stats=st)      # compared as bits
            if not collocate:
                continue
            extra = 0
            while s.stats().offline_batches < n_batches and extra < 30:
                s.step(X, DY)
                s.sync()
                extra += 1
            for tk in tickets:
                s.wait(tk, 30.0)
            bubbles, ran = _trace(s, n_cal)
            res["outs"], res["bubbles"], res["ran"] = [o.cpu() for o in outs], bubbles, ran
            import time
            t_end = time.time() + 2.0
            fin = s.stats()
            while fin.gate_checked + fin.gate_unchecked < len(ran) and time.time() < t_end:
                time.sleep(0.001)
                fin = s.stats()
            res["final_stats"] = fin
    # the fill outputs against a run by itself and, on sampled rows, against the oracle
    w = OE.working_copy(emaster_np, "bf16")
    with Session() as s:
        m = s.register_inference(eshape, emaster)
        for i in sorted({0, n_batches // 2, n_batches - 1}):
            I, out = i32(eids[i]), torch.zeros((enc["batch"], enc["seq"], enc["d_model"]), device=DEV, dtype=torch.bfloat16)
            torch.cuda.synchronize()
            s.wait(s.submit_offline(m, I, out, enc["batch"], enc["seq"]))
            assert torch.equal(out.cpu(), res["outs"][i]), i
        for i, b in ((0, 1), (n_batches - 1, enc["batch"] - 1)):
            ref = OE.encoder_forward(w, eids[i][b:b + 1], enc, "bf16")
            if enc["n_layers"] >= 12:
                assert_deep_bf16_close(res["outs"][i][b:b + 1].float().numpy(), ref, OE.encoder_forward(w, eids[i][b:b + 1], enc, "f32"), f"fill batch {i} sample {b}")
            else:
                assert_bf16_close(res["outs"][i][b:b + 1].float().numpy(), ref, f"fill batch {i} sample {b}", elem_slack=2e-2)
    return res


def test_pipeline_stage_configuration_at_full_size():
    """configs[2]: stage 1 of 4, 8 micro-batches in 1F1B order, 6 layers of d 2048; offline fill with the 6-layer d 512
    encoder, seq 256, batch 64."""
    dec, enc = dict(Y.PP_DECODER), dict(Y.PP_FILL_ENCODER)

    def register(s, dshape, dmaster):
        s.register_training(dshape, dmaster, par_mode=S.SIF_PAR_PP, lr=dec["lr"], pp_stages=dec["n_stages"], pp_micro=dec["n_micro"], pp_stage=dec["stage"])
    res = _run_config(dec, enc, n_batches=12, steps=2, coalesce=8, kernel_us_max=1200, register=register)      # as bench.py runs it
    assert torch.equal(res[0]["master"], res[1]["master"])                     # collocation leaves training untouched, bit for bit
    assert bool(torch.isfinite(res[0]["master"].view(torch.float32)).all())
    fin = res["final_stats"]
    assert fin.offline_batches == 12 and fin.offline_samples == 12 * enc["batch"]
    _assert_inside(res["bubbles"], res["ran"])
    assert fin.gate_violations == 0 and fin.gate_unchecked == 0 and fin.gate_checked == len(res["ran"])
    # the step's bubbles are the 1F1B idle intervals of stage 1: before the first forward, before the first backward,
    # two cool-down gaps, the wait at the end
    st = res[1]["stats"]
    assert st.steps == 2 and st.bubble_ns > 0
    per_step = [b for b in res["bubbles"]][-5:]
    assert len(res["bubbles"]) >= 10 and all(b1 > b0 for b0, b1 in per_step)


def test_tensor_shard_configuration_at_full_size_keeps_kernels_within_200_us():
    """configs[3]: 24 layers of the 1/8 shard of d 4096, batch 4 x seq 2048, four bubbles of 1.34 ms per layer and
    step (96 per step); the fill runs in kernels planned for at most 200 us."""
    dec, enc = dict(Y.TP_DECODER), dict(Y.FILL_ENCODER)
    limit_us = 200

    def register(s, dshape, dmaster):
        s.register_training(dshape, dmaster, par_mode=S.SIF_PAR_TP, lr=dec["lr"], bw_bytes_per_s=dec["bw_bytes_per_s"])
    res = _run_config(dec, enc, n_batches=21, steps=1, coalesce=21, kernel_us_max=limit_us, register=register)      # as bench.py runs it
    assert torch.equal(res[0]["master"], res[1]["master"])
    assert bool(torch.isfinite(res[0]["master"].view(torch.float32)).all())
    fin = res["final_stats"]
    assert fin.offline_batches == 21
    _assert_inside(res["bubbles"], res["ran"])
    assert fin.gate_violations == 0 and fin.gate_unchecked == 0 and fin.gate_checked == len(res["ran"])
    want_ns = S.sif_collective_ns(dec["batch"] * dec["seq"] * dec["d_model"] * 2, dec["bw_bytes_per_s"])
    assert want_ns == 1_342_177
    assert len(res["bubbles"]) % 96 == 0 and all(b1 - b0 >= want_ns for b0, b1 in res["bubbles"])
    # No inference kernel that ran lasted longer than the limit.  The planner cuts products by predicted time; the
    # slack covers what a kernel measured alone can differ by from its prediction (clock, a partly filled last round).
    dur_us = np.array([(t1 - t0) / 1e3 for t0, t1 in res["ran"]])
    print("inference kernels:", len(dur_us), "longest", dur_us.max(), "us, p99", np.percentile(dur_us, 99))
    assert dur_us.max() <= limit_us * 1.1, dur_us.max()
    # and none ran past the end of its bubble by more than a small fraction of it (the device gate admits a kernel only
    # if its predicted time fits the predicted rest of the bubble)
    b0 = np.array([b[0] for b in res["bubbles"]]); b1 = np.array([b[1] for b in res["bubbles"]])
    over = [max(0, t1 - b1[np.searchsorted(b0, t0, side="right") - 1]) for t0, t1 in res["ran"]]
    assert max(over) <= 0.1 * want_ns, max(over)
