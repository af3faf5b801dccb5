"""Pins for oracle/mlp.py, decoder.py, encoder.py: finite differences, torch fp64 autograd as an independent
library implementation, brute force on tiny shapes, closed forms and structural invariants."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as S
from oracle import decoder as D
from oracle import encoder as E
from oracle import mlp as M
from oracle.numerics import Prec, bf16_round

TINY = dict(n_layers=2, d_model=16, n_heads=2, d_head=8, d_ffn=24, vocab=37, max_pos=8, causal=True)
SHARD = dict(n_layers=2, d_model=16, n_heads=2, d_head=4, d_ffn=12, vocab=0, max_pos=0, causal=True)  # da != d


def to64(p):
    return {k: ([to64(l) for l in v] if k == "layers" else np.asarray(v, np.float64)) for k, v in p.items()}


def tt(a, grad=True):
    return torch.tensor(np.asarray(a, np.float64), requires_grad=grad)


# ---------------------------------------------------------------- MLP
def test_mlp_matches_torch_autograd_and_sgd_closed_form():
    p = to64(S.mlp_params(0, 12, 10, 7))
    p["b1"] += 0.3; p["b2"] -= 0.2
    x, t = S.mlp_batch(0, 0, 5, 12, 7)
    loss, new, g = M.mlp_train_step(p, x, t, 0.01)
    tp = {k: tt(v) for k, v in p.items()}
    y = F.gelu(tt(x, False) @ tp["w1"].T + tp["b1"]) @ tp["w2"].T + tp["b2"]
    lt = 0.5 * ((y - tt(t, False)) ** 2).mean()
    lt.backward()
    assert abs(loss - lt.item()) < 1e-14
    for k in p:
        assert np.allclose(g[k], tp[k].grad.numpy(), atol=1e-14), k
        assert np.array_equal(new[k], p[k] - 0.01 * g[k])


def test_mlp_finite_differences():
    p = to64(S.mlp_params(1, 6, 5, 4))
    x, t = S.mlp_batch(1, 0, 3, 6, 4)
    _, g = M.mlp_loss_and_grads(p, x, t)
    for k, idx in (("w1", (2, 3)), ("b1", (1,)), ("w2", (0, 4)), ("b2", (3,))):
        q = {kk: v.copy() for kk, v in p.items()}
        q[k][idx] += 1e-6
        lp, _ = M.mlp_loss_and_grads(q, x, t)
        q[k][idx] -= 2e-6
        lm, _ = M.mlp_loss_and_grads(q, x, t)
        assert abs((lp - lm) / 2e-6 - g[k][idx]) < 1e-8, k


# ---------------------------------------------------------------- decoder
def torch_layer(p, x, cfg):
    h, dh = cfg["n_heads"], cfg["d_head"]
    da = h * dh
    b, s, d = x.shape
    y = F.layer_norm(x, (d,), p["ln1_g"], p["ln1_b"], 1e-5)
    qkv = y @ p["w_qkv"].T + p["b_qkv"]
    q, k, v = (qkv[..., i * da:(i + 1) * da].reshape(b, s, h, dh).transpose(1, 2) for i in range(3))
    o = F.scaled_dot_product_attention(q, k, v, is_causal=cfg.get("causal", True))
    x = x + o.transpose(1, 2).reshape(b, s, da) @ p["w_o"].T + p["b_o"]
    y = F.layer_norm(x, (d,), p["ln2_g"], p["ln2_b"], 1e-5)
    return x + F.gelu(y @ p["w_fc"].T + p["b_fc"]) @ p["w_proj"].T + p["b_proj"]


def torch_gpt_loss(tp, ids, targets, cfg):
    s = ids.shape[1]
    x = tp["wte"][torch.from_numpy(ids).long()] + tp["wpe"][:s][None]
    for p in tp["layers"]:
        x = torch_layer(p, x, cfg)
    x = F.layer_norm(x, (cfg["d_model"],), tp["lnf_g"], tp["lnf_b"], 1e-5)
    logits = x.reshape(-1, cfg["d_model"]) @ tp["wte"].T
    return F.cross_entropy(logits, torch.from_numpy(targets.reshape(-1)).long()), logits


def to_torch(p):
    return {k: ([to_torch(l) for l in v] if k == "layers" else tt(v)) for k, v in p.items()}


def test_gpt_matches_torch_autograd_fp64():
    cfg = TINY
    w = to64(S.decoder_params(3, cfg, perturb=True))
    ids, tg = S.token_ids(4, 2, 6, cfg["vocab"]), S.token_ids(5, 2, 6, cfg["vocab"])
    ids[0, 3] = ids[0, 1] = ids[1, 2]                       # repeated tokens exercise the scatter-add
    loss, g, cache = D.gpt_loss_and_grads(w, ids, tg, cfg, Prec("f32"))
    tp = to_torch(w)
    lt, logits = torch_gpt_loss(tp, ids, tg, cfg)
    lt.backward()
    assert abs(loss - lt.item()) < 1e-12
    assert np.allclose(cache["logits"], logits.detach().numpy(), atol=1e-12)
    for k in ("wte", "wpe", "lnf_g", "lnf_b"):
        assert np.allclose(g[k][:tp[k].shape[0]], tp[k].grad.numpy(), atol=1e-12), k
    for l in range(cfg["n_layers"]):
        for k in D.LAYER_KEYS:
            assert np.allclose(g["layers"][l][k], tp["layers"][l][k].grad.numpy(), atol=1e-12), (l, k)


def test_gpt_finite_differences():
    cfg = TINY
    w = to64(S.decoder_params(6, cfg, perturb=True))
    ids, tg = S.token_ids(7, 2, 5, cfg["vocab"]), S.token_ids(8, 2, 5, cfg["vocab"])
    _, g, _ = D.gpt_loss_and_grads(w, ids, tg, cfg, Prec("f32"))
    f = lambda: D.gpt_loss_and_grads(w, ids, tg, cfg, Prec("f32"))[0]
    probes = [(w["wte"], g["wte"], (int(ids[0, 0]), 3)), (w["wpe"], g["wpe"], (2, 5)), (w["lnf_g"], g["lnf_g"], (4,))]
    for l in range(2):
        for k, idx in (("w_qkv", (5, 2)), ("w_qkv", (20, 7)), ("w_qkv", (40, 1)), ("b_qkv", (17,)), ("w_o", (3, 9)),
                       ("b_o", (1,)), ("ln1_g", (2,)), ("ln1_b", (6,)), ("w_fc", (11, 4)), ("b_fc", (13,)),
                       ("w_proj", (7, 19)), ("b_proj", (0,)), ("ln2_g", (9,)), ("ln2_b", (15,))):
            probes.append((w["layers"][l][k], g["layers"][l][k], idx))
    for arr, grad, idx in probes:
        old = arr[idx]
        arr[idx] = old + 1e-6; lp = f()
        arr[idx] = old - 1e-6; lm = f()
        arr[idx] = old
        fd = (lp - lm) / 2e-6
        assert abs(fd - grad[idx]) <= 1e-6 * max(1.0, abs(fd)) + 2e-9, (idx, fd, grad[idx])


def test_stack_matches_torch_with_local_heads():
    cfg = SHARD
    layers = to64(S.decoder_params(9, cfg, perturb=True))["layers"]
    x, dy = S.activations(10, 2, 5, 16), S.activations(11, 2, 5, 16)
    y, dx, grads, _ = D.stack_fwd_bwd(layers, x, dy, cfg, Prec("f32"))
    tl = [to_torch(l) for l in layers]
    xt = tt(x)
    yt = xt
    for p in tl:
        yt = torch_layer(p, yt, cfg)
    (yt * tt(dy, False)).sum().backward()
    assert np.allclose(y, yt.detach().numpy(), atol=1e-12)
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-12)
    for l in range(2):
        for k in D.LAYER_KEYS:
            assert np.allclose(grads[l][k], tl[l][k].grad.numpy(), atol=1e-12), (l, k)


def test_attention_brute_force_loops():
    rng = np.random.default_rng(12)
    b, s, h, dh = 2, 5, 2, 3
    qkv = rng.standard_normal((b, s, 3 * h * dh))
    for causal in (True, False):
        o, p = D.attention_fwd(qkv, h, dh, causal, Prec("f32"))
        for bi in range(b):
            for hi in range(h):
                for i in range(s):
                    q = qkv[bi, i, hi * dh:(hi + 1) * dh]
                    js = range(i + 1) if causal else range(s)
                    e = [math.exp(sum(q[c] * qkv[bi, j, h * dh + hi * dh + c] for c in range(dh)) / math.sqrt(dh)) for j in js]
                    z = sum(e)
                    for c in range(dh):
                        want = sum(e[n] / z * qkv[bi, j, 2 * h * dh + hi * dh + c] for n, j in enumerate(js))
                        assert abs(o[bi, i, hi * dh + c] - want) < 1e-12
                    assert abs(p[bi, hi, i, :len(e)].sum() - 1) < 1e-12 and np.all(p[bi, hi, i, len(e):] == 0)


def test_gpt_closed_forms_and_causality():
    cfg = TINY
    w = to64(S.decoder_params(13, cfg))
    ids, tg = S.token_ids(14, 2, 6, cfg["vocab"]), S.token_ids(15, 2, 6, cfg["vocab"])
    zero = {k: ([{kk: vv * 0 for kk, vv in l.items()} for l in v] if k == "layers" else v * 0) for k, v in w.items()}
    loss, _, _ = D.gpt_loss_and_grads(zero, ids, tg, cfg, Prec("f32"))
    assert abs(loss - math.log(cfg["vocab"])) < 1e-12                 # uniform prediction
    logits, _ = D.gpt_forward(w, ids, cfg, Prec("f32"))
    ids2 = ids.copy(); ids2[:, 4:] = (ids2[:, 4:] + 1) % cfg["vocab"]
    logits2, _ = D.gpt_forward(w, ids2, cfg, Prec("f32"))
    l1, l2 = logits.reshape(2, 6, -1), logits2.reshape(2, 6, -1)
    assert np.array_equal(l1[:, :4], l2[:, :4]) and not np.allclose(l1[:, 4:], l2[:, 4:])
    assert D.n_params(S.DP_DECODER) == 124_439_808


def test_gpt_bf16_mode_rounds_every_stored_tensor_and_stays_close():
    cfg = TINY
    m = S.decoder_params(16, cfg, perturb=True)
    ids, tg = S.token_ids(17, 2, 6, cfg["vocab"]), S.token_ids(18, 2, 6, cfg["vocab"])
    loss_b, new_b, g_b, c_b = D.gpt_train_step(m, ids, tg, cfg, 0.01, "bf16")
    loss_f, new_f, g_f, c_f = D.gpt_train_step(m, ids, tg, cfg, 0.01, "f32")
    assert abs(loss_b - loss_f) < 2e-2 * abs(loss_f)
    for k in ("wte", "wpe", "lnf_g"):
        assert np.array_equal(bf16_round(g_b[k]), g_b[k])
        assert np.max(np.abs(g_b[k] - g_f[k])) <= 3e-2 * np.max(np.abs(g_f[k])), k
    for k in D.LAYER_KEYS:
        assert np.array_equal(bf16_round(g_b["layers"][0][k]), g_b["layers"][0][k])
        assert np.max(np.abs(g_b["layers"][0][k] - g_f["layers"][0][k])) <= 3e-2 * np.max(np.abs(g_f["layers"][0][k])), k
    for k in ("ln1", "qkv", "prob", "o", "x_mid", "ln2", "z", "a"):
        assert np.array_equal(bf16_round(c_b["layers"][1][k]), c_b["layers"][1][k]), k
    # SGD closed form on the fp32 masters
    assert np.array_equal(new_b["lnf_g"], m["lnf_g"].astype(np.float64) - 0.01 * g_b["lnf_g"])


# ---------------------------------------------------------------- encoder
ENC = dict(n_layers=2, d_model=16, n_heads=2, d_head=8, d_ffn=24, vocab=29, max_pos=8)


def torch_encoder(w, ids, cfg):
    h, dh, d = cfg["n_heads"], cfg["d_head"], cfg["d_model"]
    b, s = ids.shape
    x = tt(w["wte"], False)[torch.from_numpy(ids).long()] + tt(w["wpe"], False)[:s][None]
    x = F.layer_norm(x, (d,), tt(w["emb_ln_g"], False), tt(w["emb_ln_b"], False), 1e-5)
    for p in w["layers"]:
        p = {k: tt(v, False) for k, v in p.items()}
        qkv = x @ p["w_qkv"].T + p["b_qkv"]
        q, k, v = (qkv[..., i * h * dh:(i + 1) * h * dh].reshape(b, s, h, dh).transpose(1, 2) for i in range(3))
        o = F.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(b, s, h * dh)
        x = F.layer_norm(x + o @ p["w_o"].T + p["b_o"], (d,), p["ln1_g"], p["ln1_b"], 1e-5)
        y = F.gelu(x @ p["w_fc"].T + p["b_fc"]) @ p["w_proj"].T + p["b_proj"]
        x = F.layer_norm(x + y, (d,), p["ln2_g"], p["ln2_b"], 1e-5)
    return x.numpy()


def test_encoder_matches_torch_fp64():
    w = to64(S.encoder_params(20, ENC, perturb=True))
    ids = S.token_ids(21, 3, 7, ENC["vocab"])
    assert np.allclose(E.encoder_forward(w, ids, ENC, "f32"), torch_encoder(w, ids, ENC), atol=1e-12)


def test_encoder_invariants():
    w = to64(S.encoder_params(22, ENC, perturb=True))
    ids = S.token_ids(23, 3, 7, ENC["vocab"])
    out = E.encoder_forward(w, ids, ENC, "f32")
    # batch independence: a sample's output does not depend on the other samples (row chunking is safe)
    assert np.array_equal(E.encoder_forward(w, ids[1:2], ENC, "f32"), out[1:2])
    # no mask: permuting tokens together with their position rows permutes the outputs
    perm = np.array([3, 0, 6, 1, 5, 2, 4])
    w2 = dict(w); w2["wpe"] = w["wpe"].copy(); w2["wpe"][:7] = w["wpe"][:7][perm]
    assert np.allclose(E.encoder_forward(w2, ids[:, perm], ENC, "f32"), out[:, perm], atol=1e-12)
    # bf16 mode: outputs representable and close
    wb = E.working_copy(S.encoder_params(22, ENC, perturb=True), "bf16")
    ob = E.encoder_forward(wb, ids, ENC, "bf16")
    assert np.array_equal(bf16_round(ob), ob)
    assert np.max(np.abs(ob - out)) < 3e-2 * np.max(np.abs(out))


def test_microbatched_stack_accumulates_like_one_big_batch():
    # without rounding, accumulating parameter gradients over micro-batches equals the gradient of the
    # concatenated batch (the loss is a sum over samples), and outputs / input gradients are per sample
    cfg = SHARD
    master = S.decoder_params(30, cfg, perturb=True)["layers"]
    xs, dys = S.activations(31, 3, 2, 5, 16), S.activations(32, 3, 2, 5, 16)
    ys, dxs, new, grads = D.stack_train_step_microbatched(master, xs, dys, cfg, 0.05, "f32")
    layers = to64({"layers": master})["layers"]
    y, dx, g_big, _ = D.stack_fwd_bwd(layers, xs.reshape(6, 5, 16), dys.reshape(6, 5, 16), cfg, Prec("f32"))
    assert np.allclose(ys.reshape(6, 5, 16), y, atol=1e-12) and np.allclose(dxs.reshape(6, 5, 16), dx, atol=1e-12)
    for l in range(2):
        for k in D.LAYER_KEYS:
            assert np.allclose(grads[l][k], g_big[l][k], atol=1e-12), (l, k)
            assert np.allclose(new[l][k], layers[l][k] - 0.05 * g_big[l][k], atol=1e-12)
    # bf16: every stored accumulated gradient is representable and close to the unrounded one
    _, _, _, gb = D.stack_train_step_microbatched(master, xs, dys, cfg, 0.05, "bf16")
    for k in D.LAYER_KEYS:
        assert np.array_equal(bf16_round(gb[0][k]), gb[0][k])
        assert np.max(np.abs(gb[0][k] - grads[0][k])) <= 3e-2 * np.max(np.abs(grads[0][k])), k
