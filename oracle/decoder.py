"""Pre-LN GPT-style decoder: the training instance of the data-, pipeline- and tensor-parallel configurations.

The paper trains named transformer models (Sec. 5.1 "Workloads") and defines no numerics; this is the textbook
block those models are made of, with the shapes of the benchmark configurations:

  x <- x + Attn(LN1(x)),   x <- x + MLP(LN2(x))
  Attn: [q|k|v] = h Wqkv^T + b;  per head P = softmax(q k^T / sqrt(dh) + causal mask);  o = P v;  o Wo^T + bo
  MLP : GELU(h Wfc^T + bfc) Wproj^T + bproj

Full model (data-parallel share): token + learned position embedding, L blocks, final LN, LM head tied to the
token embedding, mean token cross entropy, plain SGD.  Stack only (pipeline stage / tensor shard): activations
in, upstream gradient in.  A tensor shard is the same block with n_heads local heads (d_attn = n_heads * d_head
columns of Wqkv per q/k/v, d_attn rows of Wo^T) and a local d_ffn; the row-parallel outputs stay local partial
sums because the all-reduce is modelled as time only.

Weights are [out_features, in_features].  `prec.store` marks every tensor the GPU keeps in memory.
"""
import numpy as np
from .numerics import (Prec, gelu, gelu_grad, layernorm_fwd, layernorm_bwd, softmax_rows,
                       cross_entropy_mean)

LAYER_KEYS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
              "ln2_g", "ln2_b", "w_fc", "b_fc", "w_proj", "b_proj")


def _split_heads(t, n_heads, d_head):
    b, s, _ = t.shape
    return t.reshape(b, s, n_heads, d_head).transpose(0, 2, 1, 3)


def _merge_heads(t):
    b, h, s, dh = t.shape
    return t.transpose(0, 2, 1, 3).reshape(b, s, h * dh)


def attention_fwd(qkv, n_heads, d_head, causal, prec):
    """qkv [B,S,3*da] -> o [B,S,da]; returns (o, P) with P the stored attention probabilities [B,H,S,S]."""
    da = n_heads * d_head
    q = _split_heads(qkv[..., 0:da], n_heads, d_head)
    k = _split_heads(qkv[..., da:2 * da], n_heads, d_head)
    v = _split_heads(qkv[..., 2 * da:3 * da], n_heads, d_head)
    s = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(d_head)
    if causal:
        n = s.shape[-1]
        s = np.where(np.tril(np.ones((n, n), dtype=bool)), s, -np.inf)
    p = prec.store(softmax_rows(s))
    o = prec.store(_merge_heads(p @ v))
    return o, p


def attention_bwd(do, qkv, p, n_heads, d_head, prec):
    """Gradient of attention_fwd w.r.t. qkv given do [B,S,da] and the stored probabilities."""
    da = n_heads * d_head
    q = _split_heads(qkv[..., 0:da], n_heads, d_head)
    k = _split_heads(qkv[..., da:2 * da], n_heads, d_head)
    v = _split_heads(qkv[..., 2 * da:3 * da], n_heads, d_head)
    doh = _split_heads(do, n_heads, d_head)
    dv = p.transpose(0, 1, 3, 2) @ doh
    dp = doh @ v.transpose(0, 1, 3, 2)
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True)) / np.sqrt(d_head)
    ds = prec.store(ds)
    dq = ds @ k
    dk = ds.transpose(0, 1, 3, 2) @ q
    return prec.store(np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=-1))


def layer_fwd(p, x, cfg, prec):
    h, dh = cfg["n_heads"], cfg["d_head"]
    ln1, m1, r1 = layernorm_fwd(x, p["ln1_g"], p["ln1_b"])
    ln1 = prec.store(ln1)
    qkv = prec.store(ln1 @ p["w_qkv"].T + p["b_qkv"])
    o, prob = attention_fwd(qkv, h, dh, cfg.get("causal", True), prec)
    x_mid = prec.store(x + o @ p["w_o"].T + p["b_o"])
    ln2, m2, r2 = layernorm_fwd(x_mid, p["ln2_g"], p["ln2_b"])
    ln2 = prec.store(ln2)
    zf = ln2 @ p["w_fc"].T + p["b_fc"]
    z = prec.store(zf)
    a = prec.store(gelu(zf))
    x_out = prec.store(x_mid + a @ p["w_proj"].T + p["b_proj"])
    cache = dict(x=x, ln1=ln1, m1=m1, r1=r1, qkv=qkv, prob=prob, o=o, x_mid=x_mid,
                 ln2=ln2, m2=m2, r2=r2, z=z, a=a)
    return x_out, cache


def _flat(t):
    return t.reshape(-1, t.shape[-1])


def layer_bwd(p, dx_out, c, cfg, prec, acc=None):
    """Returns (dx_in, grads of this layer's parameters); every stored gradient is rounded by prec.
    With `acc` (the gradients stored so far, micro-batch accumulation) each new gradient is added to the stored
    one before it is rounded and stored again."""
    h, dh = cfg["n_heads"], cfg["d_head"]
    g = {}

    def put(k, raw):
        g[k] = prec.store(raw if acc is None else acc[k] + raw)

    dxo = _flat(dx_out)
    put("b_proj", dxo.sum(axis=0))
    put("w_proj", dxo.T @ _flat(c["a"]))
    dz = prec.store((dx_out @ p["w_proj"]) * gelu_grad(c["z"]))
    put("b_fc", _flat(dz).sum(axis=0))
    put("w_fc", _flat(dz).T @ _flat(c["ln2"]))
    dln2 = prec.store(dz @ p["w_fc"])
    dxl, dg, db = layernorm_bwd(dln2, c["x_mid"], p["ln2_g"], c["m2"], c["r2"])
    put("ln2_g", dg)
    put("ln2_b", db)
    dx_mid = prec.store(dx_out + dxl)

    dxm = _flat(dx_mid)
    put("b_o", dxm.sum(axis=0))
    put("w_o", dxm.T @ _flat(c["o"]))
    do = prec.store(dx_mid @ p["w_o"])
    dqkv = attention_bwd(do, c["qkv"], c["prob"], h, dh, prec)
    put("b_qkv", _flat(dqkv).sum(axis=0))
    put("w_qkv", _flat(dqkv).T @ _flat(c["ln1"]))
    dln1 = prec.store(dqkv @ p["w_qkv"])
    dxl, dg, db = layernorm_bwd(dln1, c["x"], p["ln1_g"], c["m1"], c["r1"])
    put("ln1_g", dg)
    put("ln1_b", db)
    dx_in = prec.store(dx_mid + dxl)
    return dx_in, g


def working_copy(master, prec):
    """The copy of the parameters the kernels read: fp32 masters rounded to the storage precision."""
    out = {}
    for k, v in master.items():
        out[k] = [working_copy(l, prec) for l in v] if k == "layers" else prec.store(v)
    return out


def stack_fwd_bwd(layers, x, dy, cfg, prec):
    """Pipeline-stage / tensor-shard share: L blocks forward on x, backward from the upstream gradient dy."""
    x = prec.store(x)
    caches = []
    for p in layers:
        x, c = layer_fwd(p, x, cfg, prec)
        caches.append(c)
    y = x
    dx = prec.store(dy)
    grads = [None] * len(layers)
    for i in reversed(range(len(layers))):
        dx, grads[i] = layer_bwd(layers[i], dx, caches[i], cfg, prec)
    return y, dx, grads, caches


def stack_train_step_microbatched(master_layers, xs, dys, cfg, lr, prec_kind="bf16"):
    """Pipeline-stage share of one training step: n_micro micro-batches (xs, dys: [n_micro, B, S, d]) go forward
    and backward through the stage's blocks, parameter gradients accumulate over the micro-batches in the order
    their backward passes run (0, 1, ...), then one SGD update.  The order in which forward and backward passes
    interleave (1F1B) does not change any value: the parameters are constant within the step.
    Returns (ys, dxs, new master layers, accumulated grads)."""
    prec = Prec(prec_kind)
    layers = working_copy({"layers": master_layers}, prec)["layers"]
    ys, dxs, grads = [], [], [None] * len(layers)
    for k in range(len(xs)):
        x = prec.store(xs[k])
        caches = []
        for p in layers:
            x, c = layer_fwd(p, x, cfg, prec)
            caches.append(c)
        ys.append(x)
        dx = prec.store(dys[k])
        for i in reversed(range(len(layers))):
            dx, grads[i] = layer_bwd(layers[i], dx, caches[i], cfg, prec, grads[i])
        dxs.append(dx)
    new = sgd_update({"layers": master_layers}, {"layers": grads}, lr)["layers"]
    return np.stack(ys), np.stack(dxs), new, grads


def gpt_forward(w, ids, cfg, prec):
    """ids [B,S] ints -> (logits [B*S,V] stored, cache)."""
    b, s = ids.shape
    x = prec.store(w["wte"][ids] + w["wpe"][np.arange(s)][None, :, :])
    caches = []
    for p in w["layers"]:
        x, c = layer_fwd(p, x, cfg, prec)
        caches.append(c)
    lnf, mf, rf = layernorm_fwd(x, w["lnf_g"], w["lnf_b"])
    lnf = prec.store(lnf)
    logits = prec.store(_flat(lnf) @ w["wte"].T)
    return logits, dict(layers=caches, x_last=x, lnf=lnf, mf=mf, rf=rf)


def gpt_loss_and_grads(w, ids, targets, cfg, prec):
    """Returns (loss, grads with the same nesting as w, cache).  targets [B,S] ints."""
    b, s = ids.shape
    logits, cache = gpt_forward(w, ids, cfg, prec)
    loss, dlogits = cross_entropy_mean(logits, targets.reshape(-1))
    dlogits = prec.store(dlogits)
    cache["logits"], cache["dlogits"] = logits, dlogits
    g = {"layers": [None] * len(w["layers"])}
    d = cfg["d_model"]
    dwte_head = prec.store(dlogits.T @ _flat(cache["lnf"]))
    dlnf = prec.store(dlogits @ w["wte"]).reshape(b, s, d)
    dx, dg, db = layernorm_bwd(dlnf, cache["x_last"], w["lnf_g"], cache["mf"], cache["rf"])
    g["lnf_g"], g["lnf_b"] = prec.store(dg), prec.store(db)
    dx = prec.store(dx)
    for i in reversed(range(len(w["layers"]))):
        dx, g["layers"][i] = layer_bwd(w["layers"][i], dx, cache["layers"][i], cfg, prec)
    # embedding backward: rows of wte receive the head gradient plus the sum over the tokens that used them
    scat = np.zeros_like(dwte_head)
    np.add.at(scat, ids.reshape(-1), _flat(dx))
    g["wte"] = prec.store(dwte_head + scat)
    dwpe = np.zeros_like(np.asarray(w["wpe"], dtype=np.float64))
    dwpe[:s] = dx.sum(axis=0)
    g["wpe"] = prec.store(dwpe)
    cache["dx0"] = dx
    return loss, g, cache


def sgd_update(master, grads, lr):
    """theta <- theta - lr * grad on the fp32 masters (same nesting as master)."""
    out = {}
    for k, v in master.items():
        if k == "layers":
            out[k] = [sgd_update(l, gl, lr) for l, gl in zip(v, grads[k])]
        else:
            out[k] = np.asarray(v, dtype=np.float64) - lr * grads[k]
    return out


def gpt_train_step(master, ids, targets, cfg, lr, prec_kind="bf16"):
    """One training step from fp32 masters.  Returns (loss, new masters, grads, cache)."""
    prec = Prec(prec_kind)
    w = working_copy(master, prec)
    loss, g, cache = gpt_loss_and_grads(w, ids, targets, cfg, prec)
    return loss, sgd_update(master, g, lr), g, cache


def n_params(cfg):
    d, da, f = cfg["d_model"], cfg["n_heads"] * cfg["d_head"], cfg["d_ffn"]
    per_layer = 2 * d + 3 * da * d + 3 * da + d * da + d + 2 * d + f * d + f + d * f + d
    n = cfg["n_layers"] * per_layer
    if cfg.get("vocab"):
        n += cfg["vocab"] * d + cfg["max_pos"] * d + 2 * d
    return n
