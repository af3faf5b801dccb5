"""Flat parameter layout of the registered models (the order documented beside sif_model_n_params in
include/specinf.h) and packing of nested dicts of arrays into it.  Data movement only."""
import numpy as np

from . import binding as B

DEC_LAYER = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_fc", "b_fc", "w_proj", "b_proj")
ENC_LAYER = ("w_qkv", "b_qkv", "w_o", "b_o", "ln1_g", "ln1_b", "w_fc", "b_fc", "w_proj", "b_proj", "ln2_g", "ln2_b")


def make_shape(kind, dtype, **kw):
    s = B.sif_model_shape()
    s.kind, s.dtype = kind, dtype
    for k, v in kw.items():
        setattr(s, k, v)
    return s


def layout(shape):
    """List of (path, shape) in flat order; path is a key or ("layers", l, key)."""
    d, da, f = shape.d_model, shape.n_heads * shape.d_head, shape.d_ffn
    lay = dict(ln1_g=(d,), ln1_b=(d,), w_qkv=(3 * da, d), b_qkv=(3 * da,), w_o=(d, da), b_o=(d,), ln2_g=(d,), ln2_b=(d,),
               w_fc=(f, d), b_fc=(f,), w_proj=(d, f), b_proj=(d,))
    out = []
    if shape.kind == B.SIF_MODEL_MLP:
        return [("w1", (shape.d_hidden, shape.d_in)), ("b1", (shape.d_hidden,)), ("w2", (shape.d_out, shape.d_hidden)),
                ("b2", (shape.d_out,))]
    if shape.kind == B.SIF_MODEL_DECODER:
        if shape.vocab:
            out += [("wte", (shape.vocab, d)), ("wpe", (shape.max_pos, d))]
        for l in range(shape.n_layers):
            out += [(("layers", l, k), lay[k]) for k in DEC_LAYER]
        if shape.vocab:
            out += [("lnf_g", (d,)), ("lnf_b", (d,))]
        return out
    out += [("wte", (shape.vocab, d)), ("wpe", (shape.max_pos, d)), ("emb_ln_g", (d,)), ("emb_ln_b", (d,))]
    for l in range(shape.n_layers):
        out += [(("layers", l, k), lay[k]) for k in ENC_LAYER]
    return out


def _get(p, path):
    return p[path] if isinstance(path, str) else p[path[0]][path[1]][path[2]]


def pack(shape, params, dtype=np.float32):
    """Nested dict -> flat array in layout order."""
    parts = []
    for path, shp in layout(shape):
        a = np.asarray(_get(params, path), dtype=dtype)
        assert a.shape == tuple(shp), (path, a.shape, shp)
        parts.append(a.reshape(-1))
    flat = np.concatenate(parts)
    assert flat.size == B.sif_model_n_params(shape)
    return flat


def unpack(shape, flat):
    """Flat array -> nested dict of views."""
    out, off = {}, 0
    if shape.kind != B.SIF_MODEL_MLP:
        out["layers"] = [dict() for _ in range(shape.n_layers)]
    for path, shp in layout(shape):
        n = int(np.prod(shp))
        a = flat[off:off + n].reshape(shp)
        off += n
        if isinstance(path, str):
            out[path] = a
        else:
            out["layers"][path[1]][path[2]] = a
    return out
