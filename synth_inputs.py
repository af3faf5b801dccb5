"""Seeded synthetic inputs shared by the oracle-side tests and the GPU-side tests/benchmark.

Holds shapes and random draws only, none of the method's arithmetic.  All tensors are fp32 numpy arrays drawn
from numpy's PCG64 `default_rng(seed)`: weight matrices and embeddings N(0, 0.02), LayerNorm gains 1 and
offsets 0, biases 0, float inputs N(0, 1), token ids uniform over the vocabulary, Poisson arrivals as
exponential gaps.  They stand in for the paper's BERT / RoBERTa / LLaMA2 / ChatGLM / GPT2 workloads and their
datasets (Sec. 5.1), none of which exist here; the shapes are those of the benchmark configurations.
"""
import numpy as np

# ---- shapes ---------------------------------------------------------------------------------------------
TINY_MLP = dict(d_in=256, d_hidden=256, d_out=256, train_batch=32, infer_batch=8, lr=0.01, bubble_ns=2_000_000,
                steps=20)

# data-parallel rank share: GPT-2-small-shaped decoder
DP_DECODER = dict(n_layers=12, d_model=768, n_heads=12, d_head=64, d_ffn=3072, vocab=50257, max_pos=1024,
                  batch=8, seq=1024, causal=True, lr=0.01, bw_bytes_per_s=50_000_000_000)
# offline fill: BERT-base-shaped encoder
FILL_ENCODER = dict(n_layers=12, d_model=768, n_heads=12, d_head=64, d_ffn=3072, vocab=30522, max_pos=512,
                    batch=32, seq=128)
# pipeline-parallel stage share
PP_DECODER = dict(n_layers=6, d_model=2048, n_heads=16, d_head=128, d_ffn=8192, vocab=0, max_pos=0,
                  batch=2, seq=2048, causal=True, lr=0.01, n_stages=4, n_micro=8, stage=1)
PP_FILL_ENCODER = dict(n_layers=6, d_model=512, n_heads=8, d_head=64, d_ffn=2048, vocab=30522, max_pos=512,
                       batch=64, seq=256)
# tensor-parallel shard share: d=4096 split 1/8 -> 4 of 32 heads, 2048 of 16384 ffn columns
TP_DECODER = dict(n_layers=24, d_model=4096, n_heads=4, d_head=128, d_ffn=2048, vocab=0, max_pos=0,
                  batch=4, seq=2048, causal=True, lr=0.01, bw_bytes_per_s=50_000_000_000)
ONLINE = dict(rate_per_s=200.0, seq_min=32, seq_max=256, n_requests=2000)


def small(cfg, **over):
    """A reduced copy of a configuration (tests): same structure, smaller sizes."""
    c = dict(cfg)
    c.update(over)
    return c


# ---- draws ----------------------------------------------------------------------------------------------
def _w(rng, *shape):
    return (rng.standard_normal(shape) * 0.02).astype(np.float32)


def mlp_params(seed, d_in, d_hidden, d_out):
    rng = np.random.default_rng(seed)
    return dict(w1=_w(rng, d_hidden, d_in), b1=np.zeros(d_hidden, np.float32),
                w2=_w(rng, d_out, d_hidden), b2=np.zeros(d_out, np.float32))


def mlp_batch(seed, step, batch, d_in, d_out):
    """Batch `step` of the seeded stream: inputs and regression targets, both N(0,1)."""
    rng = np.random.default_rng([seed, 1000 + step])
    return (rng.standard_normal((batch, d_in)).astype(np.float32),
            rng.standard_normal((batch, d_out)).astype(np.float32))


def decoder_layer_params(rng, d, da, f, perturb=False):
    """perturb=True draws gains/offsets/biases away from their 1/0 initial values (tests use it so that a
    dropped bias or gain changes the result)."""
    def vec(n, base):
        v = np.full(n, base, np.float32)
        return v + _w(rng, n) * 5 if perturb else v
    return dict(ln1_g=vec(d, 1.0), ln1_b=vec(d, 0.0), w_qkv=_w(rng, 3 * da, d), b_qkv=vec(3 * da, 0.0),
                w_o=_w(rng, d, da), b_o=vec(d, 0.0), ln2_g=vec(d, 1.0), ln2_b=vec(d, 0.0),
                w_fc=_w(rng, f, d), b_fc=vec(f, 0.0), w_proj=_w(rng, d, f), b_proj=vec(d, 0.0))


def decoder_params(seed, cfg, perturb=False):
    rng = np.random.default_rng(seed)
    d, da, f = cfg["d_model"], cfg["n_heads"] * cfg["d_head"], cfg["d_ffn"]
    p = {}
    if cfg.get("vocab"):
        p["wte"] = _w(rng, cfg["vocab"], d)
        p["wpe"] = _w(rng, cfg["max_pos"], d)
    p["layers"] = [decoder_layer_params(rng, d, da, f, perturb) for _ in range(cfg["n_layers"])]
    if cfg.get("vocab"):
        one, zero = np.ones(d, np.float32), np.zeros(d, np.float32)
        p["lnf_g"] = one + _w(rng, d) * 5 if perturb else one
        p["lnf_b"] = zero + _w(rng, d) * 5 if perturb else zero
    return p


def encoder_params(seed, cfg, perturb=False):
    rng = np.random.default_rng(seed)
    d, da, f = cfg["d_model"], cfg["n_heads"] * cfg["d_head"], cfg["d_ffn"]

    def vec(n, base):
        v = np.full(n, base, np.float32)
        return v + _w(rng, n) * 5 if perturb else v
    p = dict(wte=_w(rng, cfg["vocab"], d), wpe=_w(rng, cfg["max_pos"], d),
             emb_ln_g=vec(d, 1.0), emb_ln_b=vec(d, 0.0), layers=[])
    for _ in range(cfg["n_layers"]):
        p["layers"].append(dict(w_qkv=_w(rng, 3 * da, d), b_qkv=vec(3 * da, 0.0), w_o=_w(rng, d, da),
                                b_o=vec(d, 0.0), ln1_g=vec(d, 1.0), ln1_b=vec(d, 0.0),
                                w_fc=_w(rng, f, d), b_fc=vec(f, 0.0), w_proj=_w(rng, d, f),
                                b_proj=vec(d, 0.0), ln2_g=vec(d, 1.0), ln2_b=vec(d, 0.0)))
    return p


def token_ids(seed, batch, seq, vocab):
    rng = np.random.default_rng(seed)
    return rng.integers(0, vocab, size=(batch, seq), dtype=np.int64).astype(np.int32)


def activations(seed, *shape, scale=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(shape) * scale).astype(np.float32)


def poisson_arrivals(seed, rate_per_s, n, seq_min, seq_max):
    """Arrival times (ns, ascending) with exponential gaps of mean 1/rate, and a sequence length per request
    uniform in [seq_min, seq_max]."""
    rng = np.random.default_rng(seed)
    gaps = rng.exponential(1.0 / rate_per_s, size=n)
    t_ns = np.round(np.cumsum(gaps) * 1e9).astype(np.int64)
    seqs = rng.integers(seq_min, seq_max + 1, size=n).astype(np.int32)
    return t_ns, seqs
