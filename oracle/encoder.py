"""Post-LN BERT-shaped encoder forward: the inference instance that fills the bubbles (Sec. 5.1 "Workloads"
names BERT-base among the inference models; the numerics are the textbook block).

  x0 = LN(wte[id] + wpe[pos])
  x  <- LN1(x + Attn(x)),  x <- LN2(x + MLP(x))        bidirectional attention, all tokens valid
  output = final hidden states [B,S,d]

Weights are [out_features, in_features]; `prec.store` marks every tensor the GPU keeps in memory.
"""
import numpy as np
from .numerics import Prec, gelu, layernorm_fwd
from .decoder import attention_fwd

LAYER_KEYS = ("w_qkv", "b_qkv", "w_o", "b_o", "ln1_g", "ln1_b",
              "w_fc", "b_fc", "w_proj", "b_proj", "ln2_g", "ln2_b")


def layer_fwd(p, x, cfg, prec):
    qkv = prec.store(x @ p["w_qkv"].T + p["b_qkv"])
    o, _ = attention_fwd(qkv, cfg["n_heads"], cfg["d_head"], False, prec)
    t = prec.store(x + o @ p["w_o"].T + p["b_o"])
    x1 = prec.store(layernorm_fwd(t, p["ln1_g"], p["ln1_b"])[0])
    a = prec.store(gelu(x1 @ p["w_fc"].T + p["b_fc"]))
    t = prec.store(x1 + a @ p["w_proj"].T + p["b_proj"])
    return prec.store(layernorm_fwd(t, p["ln2_g"], p["ln2_b"])[0])


def encoder_forward(w, ids, cfg, prec_kind="bf16", return_layers=False):
    """w: weights already in storage precision (see working_copy); ids [B,S] ints -> hidden [B,S,d]."""
    prec = Prec(prec_kind)
    b, s = ids.shape
    e = prec.store(w["wte"][ids] + w["wpe"][np.arange(s)][None, :, :])
    x = prec.store(layernorm_fwd(e, w["emb_ln_g"], w["emb_ln_b"])[0])
    outs = [x]
    for p in w["layers"]:
        x = layer_fwd(p, x, cfg, prec)
        outs.append(x)
    return (x, outs) if return_layers else x


def working_copy(master, prec_kind="bf16"):
    prec = Prec(prec_kind)
    out = {}
    for k, v in master.items():
        out[k] = [{kk: prec.store(vv) for kk, vv in l.items()} for l in v] if k == "layers" else prec.store(v)
    return out
