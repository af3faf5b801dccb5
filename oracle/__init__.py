"""CPU oracle for the SpecInF hot path (arxiv 2503.02550).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, fp64 numpy / pure-Python statement of what the
GPU library computes.  Only tests, the smoke check and the benchmark's cpu_baseline leg may import it; the
product (the HIP library and its Python binding) never does, and nothing here imports the product.

Contents
  numerics.py   bf16 rounding model, exact-erf GELU, LayerNorm, softmax, cross entropy
  mlp.py        two-Linear fp32 MLP: training step (SGD) and forward   (Tiny configuration)
  decoder.py    pre-LN GPT-style decoder: forward, loss, backward, SGD (training instance)
  encoder.py    post-LN BERT-shaped encoder: forward                   (inference instance)
  bubbles.py    bubble model: DP / 1F1B-PP / TP idle intervals from bytes, bandwidth and phase times
  scheduler.py  Bubble Monitor zero-count (Sec. 3.3 "Bubble Monitor"), Algorithm 1, Kernel Barrier
                token accounting and the online pull rule (Sec. 3.3 "Kernel Barrier")

Pin status (see tests/test_oracle_*.py): every function is pinned by finite differences, closed forms,
brute force or a library cross-check, except the *choice* of the Algorithm 1 constants
(alpha, beta, gamma, LL, UL, seed tokens): the paper prints none, so the values are "parity unpinned".
"""
