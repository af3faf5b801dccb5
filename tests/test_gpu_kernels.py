"""GPU parity of the single kernels against the oracle's definitions (fp64 numpy), through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import numerics as N

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2503_02550_amd as S
    from gpu_util import DEV, bf, f32, i32, up, q, assert_bf16_close, assert_f32_close, rel_err, lse_reference


def rnd(seed, *shape, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float32)


# ------------------------------------------------------------------------------------------------ bf16 GEMM
@pytest.mark.parametrize("al,bl", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("m,n,k", [(200, 264, 136), (128, 128, 64), (1, 8, 8), (300, 72, 520)])
def test_gemm_bf16_layouts(al, bl, m, n, k):
    if al == 1 and m % 8:
        m = (m + 7) // 8 * 8
    a, b = rnd(1, m, k), rnd(2, k, n)
    ref = q(a) @ q(b)
    A = bf(a if al == 0 else a.T)
    B = bf(b.T if bl == 0 else b)
    c = torch.full((m, n), 7.0, device=DEV, dtype=torch.bfloat16)
    S.sif_k_gemm_bf16(A, B, c, m, n, k, A.shape[1], B.shape[1], n, a_layout=al, b_layout=bl)
    torch.cuda.synchronize()
    assert_bf16_close(up(c), ref, f"gemm {al}{bl} {m}x{n}x{k}")


def test_gemm_bf16_epilogues_and_f32_out():
    m, n, k = 136, 200, 72
    a, b, bias, res = rnd(3, m, k), rnd(4, n, k), rnd(5, n), rnd(6, m, n)
    acc = q(a) @ q(b).T
    A, B, BI, R = bf(a), bf(b), bf(bias), bf(res)
    c = torch.zeros((m, n), device=DEV, dtype=torch.bfloat16)
    S.sif_k_gemm_bf16(A, B, c, m, n, k, k, k, n, epilogue=S.SIF_EPI_BIAS | S.SIF_EPI_RESIDUAL, bias=BI, res=R, alpha=0.5)
    assert_bf16_close(up(c), 0.5 * acc + q(bias) + q(res), "bias+res")
    z = torch.zeros_like(c)
    S.sif_k_gemm_bf16(A, B, c, m, n, k, k, k, n, epilogue=S.SIF_EPI_GELU, bias=BI, aux=z)
    assert_bf16_close(up(z), acc + q(bias), "gelu pre-activation")
    assert_bf16_close(up(c), N.gelu(acc + q(bias)), "gelu")
    S.sif_k_gemm_bf16(A, B, c, m, n, k, k, k, n, epilogue=S.SIF_EPI_GELU_GRAD, aux=z)
    assert_bf16_close(up(c), acc * N.gelu_grad(up(z)), "gelu grad")
    cf = torch.zeros((m, n), device=DEV, dtype=torch.float32)
    S.sif_k_gemm_bf16(A, B, cf, m, n, k, k, k, n, epilogue=S.SIF_EPI_OUT_F32, alpha=0.125)
    assert_f32_close(up(cf), 0.125 * acc, "f32 out", tol=1e-5)


def test_gemm_bf16_batched_heads_and_causal():
    # attention-shaped: qkv [B,S,3*H*dh]; scores = q k^T per (b,h); P V with a lower-triangular P
    bsz, s, h, dh = 2, 200, 3, 64
    da = h * dh
    qkv = rnd(7, bsz, s, 3 * da)
    Q = bf(qkv)
    sc = torch.zeros((bsz * h, s, s), device=DEV, dtype=torch.float32)
    S.sif_k_gemm_bf16(Q, Q[:, :, da:], sc, s, s, dh, 3 * da, 3 * da, s, epilogue=S.SIF_EPI_OUT_F32 | S.SIF_EPI_CAUSAL_SKIP,
                      alpha=0.125, batch_outer=bsz, batch_inner=h, a_strides=(s * 3 * da, dh), b_strides=(s * 3 * da, dh),
                      c_strides=(h * s * s, s * s))
    x = q(qkv).reshape(bsz, s, 3, h, dh)
    ref = 0.125 * np.einsum("bihd,bjhd->bhij", x[:, :, 0], x[:, :, 1]).reshape(bsz * h, s, s)
    got = up(sc)
    tile_lower = (np.arange(s)[None, :] // 128) <= (np.arange(s)[:, None] // 128)
    assert_f32_close(got[:, tile_lower], ref[:, tile_lower], "scores", tol=1e-5)
    assert np.all(got[:, ~tile_lower] == 0)                      # skipped tiles untouched
    p = np.tril(np.abs(rnd(8, bsz * h, s, s)))
    P = bf(p)
    o = torch.zeros((bsz, s, da), device=DEV, dtype=torch.bfloat16)
    S.sif_k_gemm_bf16(P, Q[:, :, 2 * da:], o, s, dh, s, s, 3 * da, da, b_layout=S.SIF_B_ROW_N, batch_outer=bsz, batch_inner=h,
                      a_strides=(h * s * s, s * s), b_strides=(s * 3 * da, dh), c_strides=(s * da, dh), k_causal=1)
    ref = np.einsum("bhij,bjhd->bihd", q(p).reshape(bsz, h, s, s), x[:, :, 2]).reshape(bsz, s, da)
    assert_bf16_close(up(o), ref, "P V causal")
    # dV = P^T dO: A stored [K=i][M=j], contraction only over i >= j
    do = rnd(9, bsz, s, da)
    DO = bf(do)
    dv = torch.zeros((bsz, s, da), device=DEV, dtype=torch.bfloat16)
    S.sif_k_gemm_bf16(P, DO, dv, s, dh, s, s, da, da, a_layout=S.SIF_A_ROW_M, b_layout=S.SIF_B_ROW_N, batch_outer=bsz,
                      batch_inner=h, a_strides=(h * s * s, s * s), b_strides=(s * da, dh), c_strides=(s * da, dh), k_causal=2)
    ref = np.einsum("bhij,bihd->bjhd", q(p).reshape(bsz, h, s, s), q(do).reshape(bsz, s, h, dh)).reshape(bsz, s, da)
    assert_bf16_close(up(dv), ref, "P^T dO causal")


def test_gemm_bf16_row_range_is_bit_identical():
    m, n, k = 512, 256, 192
    A, B = bf(rnd(10, m, k)), bf(rnd(11, n, k))
    full = torch.zeros((m, n), device=DEV, dtype=torch.bfloat16)
    part = torch.zeros_like(full)
    S.sif_k_gemm_bf16(A, B, full, m, n, k, k, k, n)
    for r0, r1 in ((0, 128), (128, 384), (384, 512)):
        S.sif_k_gemm_bf16(A[r0:], B, part[r0:], r1 - r0, n, k, k, k, n)
    torch.cuda.synchronize()
    assert torch.equal(full, part)


@pytest.mark.parametrize("al,bl", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("m,n,k", [(256, 256, 64), (520, 776, 192), (1024, 512, 448)])
def test_gemm_bf16_large_tiles_give_the_same_bits(al, bl, m, n, k):
    """The 256x256 configuration (chosen automatically only for large products) against the 128x128 one and the
    definition, ragged M and N included."""
    a, b = rnd(30, m, k), rnd(31, n, k)
    A = bf(a if al == 0 else a.T.copy())
    B = bf(b if bl == 0 else b.T.copy())
    bias = bf(rnd(32, n))
    c128, c256 = (torch.zeros((m, n), device=DEV, dtype=torch.bfloat16) for _ in range(2))
    for tile, c in ((128, c128), (256, c256)):
        S.sif_k_gemm_bf16(A, B, c, m, n, k, A.shape[1], B.shape[1], n, a_layout=al, b_layout=bl, epilogue=S.SIF_EPI_BIAS, bias=bias, tile=tile)
    assert torch.equal(c128, c256)
    assert_bf16_close(up(c256), q(a) @ q(b).T + q(rnd(32, n)), f"gemm 256 tiles {al}{bl}")
    with pytest.raises(S.SifError):
        S.sif_k_gemm_bf16(A, B, c256, m, n, k - 8, A.shape[1], B.shape[1], n, a_layout=al, b_layout=bl, tile=256)


@pytest.mark.parametrize("k", [520, 1024])
def test_gemm_bf16_several_products_in_one_launch_give_the_bits_of_launches_of_their_own(k):
    """Weight-gradient-shaped products (A stored [K][M], B stored [K][N]) as one launch: a large one, a ragged one, one
    that adds to what its output holds, and a one-row product whose left operand is a column of ones (a bias gradient:
    the column sums of B); K ragged (the register path) and whole K steps (the direct fetches)."""
    shapes = [(256, 384, False), (72, 136, False), (200, 128, True), (1, 208, False)]
    prods, singles, outs, refs = [], [], [], []
    for i, (m, n, acc) in enumerate(shapes):
        mp = (m + 7) // 8 * 8
        a = np.zeros((k, mp), dtype=np.float32)
        a[:, :m] = 1.0 if m == 1 else rnd(60 + i, k, m)
        b = rnd(70 + i, k, n)
        A, B = bf(a), bf(b)
        c0 = bf(rnd(80 + i, m, n)) if acc else torch.zeros((m, n), device=DEV, dtype=torch.bfloat16)
        c1 = c0.clone()
        kw = dict(a_layout=S.SIF_A_ROW_M, b_layout=S.SIF_B_ROW_N, epilogue=S.SIF_EPI_RESIDUAL if acc else 0)
        prods.append(S.gemm_args(A, B, c0, m, n, k, mp, n, n, res=c0 if acc else None, **kw))
        singles.append((A, B, c1, m, n, k, mp, n, n, dict(res=c1 if acc else None, tile=128, **kw)))
        outs.append((c0, c1))
        refs.append(q(a[:, :m]).T @ q(b) + (q(rnd(80 + i, m, n)) if acc else 0.0))
    records = torch.zeros(S.sif_k_gemm_bf16_group_bytes(len(prods)) + 16, device=DEV, dtype=torch.uint8)
    torch.cuda.synchronize()
    S.sif_k_gemm_bf16_group(prods, records)
    for A, B, c1, m, n, kk, lda, ldb, ldc, kw in singles:
        S.sif_k_gemm_bf16(A, B, c1, m, n, kk, lda, ldb, ldc, **kw)
    torch.cuda.synchronize()
    for i, (c0, c1) in enumerate(outs):
        assert torch.equal(c0, c1), shapes[i]
        assert_bf16_close(up(c0), refs[i], f"grouped product {shapes[i]}", elem_slack=1e-2)
    with pytest.raises(S.SifError):
        S.sif_k_gemm_bf16_group([], records)
    with pytest.raises(S.SifError):
        S.sif_k_gemm_bf16_group(prods * 5, records)
    other = S.gemm_args(prods[0].a_dev, prods[0].b_dev, prods[0].c_dev, 8, 8, 64, 64, 64, 8)      # both operands K-contiguous
    with pytest.raises(S.SifError):
        S.sif_k_gemm_bf16_group([other], records)


@pytest.mark.parametrize("bl", [0, 1])
def test_gemm_bf16_slices_of_one_long_k(bl):
    """batch_inner cuts K into slices whose results go to separate fp32 outputs; with k_limit the last slice is
    shorter than the others (and here not a multiple of 8).  The slices add up to the whole product."""
    m, n, kper, slices, k_total = 200, 136, 192, 4, 3 * 192 + 77
    ld = (k_total + 7) // 8 * 8
    a = np.zeros((m, ld), np.float32); a[:, :k_total] = rnd(33, m, k_total)
    b = rnd(34, n, ld) if bl == 0 else rnd(34, ld, n)
    A, B = bf(a), bf(b)
    part = torch.full((slices, m, n), 9.0, device=DEV)
    S.sif_k_gemm_bf16(A, B, part, m, n, kper, ld, B.shape[1], n, b_layout=bl, epilogue=S.SIF_EPI_OUT_F32, batch_inner=slices,
                      a_strides=(0, kper), b_strides=(0, kper if bl == 0 else kper * n), c_strides=(0, m * n), k_limit=k_total)
    got = up(part)
    bq = q(b)[:, :k_total] if bl == 0 else q(b)[:k_total].T
    for i in range(slices):
        lo, hi = i * kper, min(k_total, (i + 1) * kper)
        assert_f32_close(got[i], q(a)[:, lo:hi] @ bq[:, lo:hi].T, f"slice {i}", tol=1e-4)
    assert_f32_close(got.sum(0), q(a)[:, :k_total] @ bq.T, "sum of the slices", tol=1e-4)
    with pytest.raises(S.SifError):                      # k_limit must lie in the last slice
        S.sif_k_gemm_bf16(A, B, part, m, n, kper, ld, B.shape[1], n, b_layout=bl, epilogue=S.SIF_EPI_OUT_F32, batch_inner=slices,
                          a_strides=(0, kper), b_strides=(0, kper), c_strides=(0, m * n), k_limit=2 * kper)


@pytest.mark.parametrize("bl", [0, 1])
def test_gemm_bf16_slices_of_one_long_k_on_large_tiles(bl):
    """The 256x256 configuration takes a K cut into slices when every slice, the shorter last one too, is a whole number
    of 64-wide K steps (the LM head's data gradient over the padded vocabulary): same bits as the 128x128 one, ragged M
    and N included; a last slice that is not a whole number of steps is refused for these tiles."""
    m, n, kper, slices, k_total = 520, 264, 192, 3, 2 * 192 + 128
    a = rnd(43, m, k_total)
    b = rnd(44, n, k_total) if bl == 0 else rnd(44, k_total, n)
    A, B = bf(a), bf(b)
    parts = []
    for tile in (128, 256):
        part = torch.full((slices, m, n), 9.0, device=DEV)
        S.sif_k_gemm_bf16(A, B, part, m, n, kper, k_total, B.shape[1], n, b_layout=bl, epilogue=S.SIF_EPI_OUT_F32, batch_inner=slices,
                          a_strides=(0, kper), b_strides=(0, kper if bl == 0 else kper * n), c_strides=(0, m * n), k_limit=k_total, tile=tile)
        parts.append(part)
    torch.cuda.synchronize()
    assert torch.equal(parts[0], parts[1])
    bq = q(b) if bl == 0 else q(b).T
    assert_f32_close(up(parts[1]).sum(0), q(a) @ bq.T, "sum of the slices, large tiles", tol=1e-4)
    with pytest.raises(S.SifError):
        S.sif_k_gemm_bf16(A, B, parts[1], m, n, kper, k_total, B.shape[1], n, b_layout=bl, epilogue=S.SIF_EPI_OUT_F32, batch_inner=slices,
                          a_strides=(0, kper), b_strides=(0, kper if bl == 0 else kper * n), c_strides=(0, m * n), k_limit=k_total - 8, tile=256)


def test_gemm_bf16_rejects_bad_arguments():
    A = bf(rnd(12, 16, 16))
    c = torch.zeros((16, 16), device=DEV, dtype=torch.bfloat16)
    with pytest.raises(S.SifError):
        S.sif_k_gemm_bf16(A, A, c, 16, 16, 16, 12, 16, 16)          # lda not a multiple of 8
    with pytest.raises(S.SifError):
        S.sif_k_gemm_bf16(A, A, c, 0, 16, 16, 16, 16, 16)           # empty
    with pytest.raises(S.SifError):
        S.sif_k_gemm_bf16(A, A, None, 16, 16, 16, 16, 16, 16)       # null output
    with pytest.raises(S.SifError):
        S.sif_k_gemm_bf16(A, A, c, 16, 16, 16, 16, 16, 16, epilogue=S.SIF_EPI_RESIDUAL)


# ------------------------------------------------------------------------------------------------ fp32 GEMM
def test_gemm_f32_strided_and_epilogues():
    m, n, k = 37, 70, 45
    a, b, bias = rnd(13, m, k), rnd(14, n, k), rnd(15, n)
    A, B, BI = f32(a), f32(b), f32(bias)
    c, z = torch.zeros((m, n), device=DEV), torch.zeros((m, n), device=DEV)
    S.sif_k_gemm_f32(A, k, 1, B, 1, k, c, n, m, n, k, epilogue=S.SIF_EPI_GELU, bias=BI, aux=z)       # x W^T + b
    pre = a.astype(np.float64) @ b.astype(np.float64).T + bias
    assert_f32_close(up(z), pre, "pre", 1e-5)
    assert_f32_close(up(c), N.gelu(pre), "gelu", 1e-5)
    dy = rnd(16, m, n)
    DY, dx = f32(dy), torch.zeros((m, k), device=DEV)
    S.sif_k_gemm_f32(DY, n, 1, B, k, 1, dx, k, m, k, n)                                             # dy W
    assert_f32_close(up(dx), dy.astype(np.float64) @ b.astype(np.float64), "dgrad", 1e-5)
    dw = torch.zeros((n, k), device=DEV)
    S.sif_k_gemm_f32(DY, 1, n, A, k, 1, dw, k, n, k, m)                                             # dy^T x
    assert_f32_close(up(dw), dy.astype(np.float64).T @ a.astype(np.float64), "wgrad", 1e-5)
    S.sif_k_gemm_f32(DY, n, 1, B, k, 1, dx, k, m, k, n, epilogue=S.SIF_EPI_GELU_GRAD, aux=f32(a))
    assert_f32_close(up(dx), (dy.astype(np.float64) @ b.astype(np.float64)) * N.gelu_grad(a), "gelu grad", 1e-5)


# ------------------------------------------------------------------------------------------------ row kernels
@pytest.mark.parametrize("rows,d", [(1, 8), (37, 768), (130, 2048), (5, 4096)])
def test_layernorm_fwd_bwd(rows, d):
    x, g, b, dy, res = rnd(20, rows, d, scale=2.0) + 0.5, rnd(21, d) + 1, rnd(22, d), rnd(23, rows, d), rnd(24, rows, d)
    X, G, B_, DY, R = bf(x), bf(g), bf(b), bf(dy), bf(res)
    y = torch.zeros_like(X)
    mean, rstd = torch.zeros(rows, device=DEV), torch.zeros(rows, device=DEV)
    S.sif_k_layernorm_fwd(X, G, B_, y, mean, rstd, rows, d)
    ry, rm, rr = N.layernorm_fwd(q(x), q(g), q(b))
    assert_bf16_close(up(y), ry, "ln y")
    assert_f32_close(up(mean), rm[:, 0], "mean", 1e-5)
    assert_f32_close(up(rstd), rr[:, 0], "rstd", 1e-5)
    dx, dg, db = torch.zeros_like(X), torch.zeros(d, device=DEV, dtype=torch.bfloat16), torch.zeros(d, device=DEV, dtype=torch.bfloat16)
    part = torch.zeros(3 * S.sif_colsum_parts(rows) * d, device=DEV)
    dsum = torch.full((d,), 9.0, device=DEV, dtype=torch.bfloat16)
    S.sif_k_layernorm_bwd(DY, X, G, mean, rstd, R, dx, dg, db, part, rows, d, dsum=dsum)
    rdx, rdg, rdb = N.layernorm_bwd(q(dy), q(x), q(g), rm, rr)
    assert_bf16_close(up(dx), q(res) + rdx, "ln dx")
    assert_bf16_close(up(dg), rdg, "ln dg")
    assert_bf16_close(up(db), rdb, "ln db")
    # column sums of the stored dx (the gradient of a bias added upstream of the residual sum)
    assert_bf16_close(up(dsum), up(dx).sum(axis=0), "ln column sums of dx")
    assert_bf16_close(up(dsum), q(q(res) + rdx).sum(axis=0), "ln column sums of dx vs oracle", elem_slack=8e-3)
    S.sif_k_layernorm_bwd(DY, X, G, mean, rstd, None, dx, dg, db, part, rows, d)
    assert_bf16_close(up(dx), rdx, "ln dx no residual")


@pytest.mark.parametrize("rows,n,ld", [(1, 8, 8), (333, 776, 784), (4100, 2304, 2304)])
def test_colsum(rows, n, ld):
    x = rnd(25, rows, ld)
    X = bf(x)
    out = torch.zeros(n, device=DEV, dtype=torch.bfloat16)
    part = torch.zeros(S.sif_colsum_parts(rows) * n, device=DEV)
    S.sif_k_colsum(X, ld, out, part, rows, n)
    assert_bf16_close(up(out), q(x)[:, :n].sum(axis=0), "colsum")


@pytest.mark.parametrize("causal", [0, 1])
@pytest.mark.parametrize("batch,rows,cols", [(3, 37, 37), (2, 200, 200), (1, 5, 2048), (2, 128, 128)])
def test_softmax_fwd_bwd(batch, rows, cols, causal):
    if causal and rows != cols:
        pytest.skip("causal needs a square problem")
    ld = (cols + 7) // 8 * 8
    s = np.zeros((batch, rows, ld), np.float32)
    s[:, :, :cols] = rnd(26, batch, rows, cols, scale=3.0)
    Sd = f32(s)
    p = torch.full((batch, rows, ld), 9.0, device=DEV, dtype=torch.bfloat16)
    S.sif_k_softmax_fwd(Sd, p, batch, rows, cols, ld, ld, causal)
    sm = s[:, :, :cols].astype(np.float64)
    if causal:
        sm = np.where(np.tril(np.ones((rows, cols), bool)), sm, -np.inf)
    ref = N.softmax_rows(sm)
    got = up(p)
    # causal rows are written up to the end of their 128-column tile only; beyond it the buffer keeps its old value
    written = np.ones((rows, ld), bool) if not causal else (np.arange(ld)[None, :] < ((np.arange(rows)[:, None] // 128 + 1) * 128))
    ref_full = np.zeros((batch, rows, ld))
    ref_full[:, :, :cols] = ref
    assert_bf16_close(np.where(written, got, 0.0), np.where(written, ref_full, 0.0), "softmax")
    assert np.all(got[:, ~written] == 9.0)
    dp = np.zeros((batch, rows, ld), np.float32)
    dp[:, :, :cols] = rnd(27, batch, rows, cols)
    ds = torch.full((batch, rows, ld), 9.0, device=DEV, dtype=torch.bfloat16)
    S.sif_k_softmax_bwd(f32(dp), p, ds, batch, rows, cols, ld, 0.125, causal)
    pq = got[:, :, :cols]
    d = dp[:, :, :cols].astype(np.float64)
    if causal:
        d = np.where(np.tril(np.ones((rows, cols), bool)), d, 0.0)
    ref = 0.125 * pq * (d - (d * pq).sum(-1, keepdims=True))
    ref_full = np.zeros((batch, rows, ld))
    ref_full[:, :, :cols] = ref
    assert_bf16_close(np.where(written, up(ds), 0.0), np.where(written, ref_full, 0.0), "softmax bwd")


@pytest.mark.parametrize("tokens,seq,d,vocab", [(8192, 1024, 768, 50257), (1000, 8, 64, 40000), (16416, 16, 32, 3000)])
def test_embedding_gradient_at_training_size_keeps_the_order_of_the_sums(tokens, seq, d, vocab):
    """Token-embedding gradient where most ids occur once and a few several times (8192 draws from 50257 ids: a few
    hundred pairs), with a ragged last group of 32 tokens, and with more tokens than the LDS variant takes (the other
    kernel): rows with the same id are added in ascending token order on top of what the table already holds."""
    ids = np.random.default_rng(40).integers(0, vocab, tokens).astype(np.int32)
    dx, head = rnd(41, tokens, d), rnd(42, vocab, d) * 0.1
    dwte, dwpe = bf(head), torch.zeros((seq, d), device=DEV, dtype=torch.bfloat16)
    S.sif_k_embed_bwd(i32(ids), bf(dx), dwte, dwpe, vocab, tokens, seq, d)
    torch.cuda.synchronize()
    # the kernel's arithmetic written out: fp32 sum of the rows in ascending token order, added to the table's value in fp32
    order = np.argsort(ids, kind="stable")
    acc = np.zeros((vocab, d), np.float32)
    dq = q(dx).astype(np.float32)
    for t in order: acc[ids[t]] += dq[t]
    want = N.bf16_round((q(head).astype(np.float32) + acc).astype(np.float64))
    touched = np.unique(ids)
    assert np.array_equal(up(dwte)[touched], want[touched])             # same order of additions, same bits
    untouched = np.setdiff1d(np.arange(vocab), touched)
    assert np.array_equal(up(dwte)[untouched], q(head)[untouched])


def test_embedding_fwd_bwd():
    tokens, seq, d, vocab = 96, 24, 64, 17          # small vocabulary: many repeated ids
    ids = np.random.default_rng(28).integers(0, vocab, tokens).astype(np.int32)
    wte, wpe, dx = rnd(29, vocab, d), rnd(30, seq, d), rnd(31, tokens, d)
    I, WTE, WPE, DX = i32(ids), bf(wte), bf(wpe), bf(dx)
    x = torch.zeros((tokens, d), device=DEV, dtype=torch.bfloat16)
    S.sif_k_embed_fwd(I, WTE, WPE, x, vocab, tokens, seq, d)
    assert_bf16_close(up(x), q(wte)[ids] + q(wpe)[np.arange(tokens) % seq], "embed")
    head = rnd(32, vocab, d)
    dwte, dwpe = bf(head), torch.zeros((seq, d), device=DEV, dtype=torch.bfloat16)
    S.sif_k_embed_bwd(I, DX, dwte, dwpe, vocab, tokens, seq, d)
    scat = np.zeros((vocab, d))
    np.add.at(scat, ids, q(dx))
    assert_bf16_close(up(dwte), q(head) + scat, "dwte")
    assert_bf16_close(up(dwpe), q(dx).reshape(-1, seq, d).sum(0), "dwpe")
    again = bf(head)
    S.sif_k_embed_bwd(I, DX, again, dwpe, vocab, tokens, seq, d)
    assert torch.equal(again, dwte)                 # fixed summation order
    # ids outside the vocabulary are taken as the nearest valid id: nothing outside the table is touched
    wild = ids.copy()
    wild[3], wild[40], wild[41] = -5, vocab, 2 ** 31 - 1
    near = np.clip(wild.astype(np.int64), 0, vocab - 1)
    S.sif_k_embed_fwd(i32(wild), WTE, WPE, x, vocab, tokens, seq, d)
    assert_bf16_close(up(x), q(wte)[near] + q(wpe)[np.arange(tokens) % seq], "embed, wild ids")
    guard = torch.full(((vocab + 4) * d,), 3.0, device=DEV, dtype=torch.bfloat16)
    tab = guard[2 * d:(2 + vocab) * d].view(vocab, d)
    tab.copy_(bf(head))
    S.sif_k_embed_bwd(i32(wild), DX, tab, dwpe, vocab, tokens, seq, d)
    scat = np.zeros((vocab, d))
    np.add.at(scat, near, q(dx))
    assert_bf16_close(up(tab), q(head) + scat, "dwte, wild ids")
    assert bool((guard[:2 * d] == 3.0).all()) and bool((guard[(2 + vocab) * d:] == 3.0).all())


@pytest.mark.parametrize("tokens,vocab", [(5, 37), (64, 50257), (3, 8), (4, 60001), (2, 70003)])
def test_cross_entropy(tokens, vocab):
    ld = (vocab + 7) // 8 * 8
    lg = np.zeros((tokens, ld), np.float32)
    lg[:, :vocab] = rnd(33, tokens, vocab, scale=2.0)
    lg[:, vocab:] = 50.0                            # padding must be ignored
    tg = np.random.default_rng(34).integers(0, vocab, tokens).astype(np.int32)
    L = bf(lg)
    loss = torch.zeros(tokens, device=DEV)
    S.sif_k_xent_fwd_bwd(L, i32(tg), loss, tokens, vocab, ld)
    rl, rd = N.cross_entropy_mean(q(lg)[:, :vocab], tg)
    out = torch.zeros(1, device=DEV)
    S.sif_k_reduce_sum(loss, out, tokens, 1.0 / tokens)
    assert abs(out.item() - rl) <= 1e-4 * abs(rl)
    got = up(L)
    assert_bf16_close(got[:, :vocab], rd, "dlogits", elem_slack=1e-3)
    assert np.all(got[:, vocab:] == 0)
    # a target outside the vocabulary is taken as the nearest valid one
    wild = tg.copy()
    wild[0], wild[-1] = -3, vocab + 5
    L2 = bf(lg)
    S.sif_k_xent_fwd_bwd(L2, i32(wild), loss, tokens, vocab, ld)
    _, rd2 = N.cross_entropy_mean(q(lg)[:, :vocab], np.clip(wild, 0, vocab - 1))
    assert_bf16_close(up(L2)[:, :vocab], rd2, "dlogits, wild targets", elem_slack=1e-3)


def test_sgd_and_mse_and_colsum_f32():
    n = 8 * 1000 + 5
    m, g = rnd(35, n), rnd(36, n)
    M, G = f32(m), bf(g)
    W = torch.zeros(n, device=DEV, dtype=torch.bfloat16)
    S.sif_k_sgd_bf16(M, None, W, n, 0.0)
    assert np.array_equal(up(W), q(m)) and np.array_equal(up(M), m.astype(np.float64))
    S.sif_k_sgd_bf16(M, G, W, n, 0.01)
    ref = m.astype(np.float64) - 0.01 * q(g)
    assert_f32_close(up(M), ref, "sgd master", 1e-6)
    assert np.array_equal(up(W), q(up(M)))
    P_, G2 = f32(m), f32(g)
    S.sif_k_sgd_f32(P_, G2, n, 0.01)
    assert_f32_close(up(P_), m.astype(np.float64) - 0.01 * g.astype(np.float64), "sgd f32", 1e-6)
    y, t = rnd(37, 32, 256), rnd(38, 32, 256)
    d, loss = torch.zeros(32 * 256, device=DEV), torch.zeros(1, device=DEV)
    S.sif_k_mse_fwd_bwd(f32(y), f32(t), d, loss, 32 * 256)
    e = y.astype(np.float64) - t
    assert abs(loss.item() - 0.5 * (e ** 2).mean()) < 1e-5
    assert_f32_close(up(d).reshape(32, 256), e / e.size, "mse grad", 1e-6)
    cs = torch.zeros(256, device=DEV)
    S.sif_k_colsum_f32(f32(y), 256, cs, 32, 256)
    assert_f32_close(up(cs), y.astype(np.float64).sum(0), "colsum f32", 1e-5)


# ------------------------------------------------------------------------------------------------ fused attention
@pytest.mark.parametrize("causal", [0, 1])
@pytest.mark.parametrize("bsz,s,h,dh", [(2, 5, 2, 64), (3, 37, 2, 64), (2, 128, 3, 64), (2, 200, 2, 64), (1, 300, 2, 128), (2, 64, 1, 128)])
def test_fused_attention_forward(bsz, s, h, dh, causal):
    from oracle.decoder import attention_fwd
    from oracle.numerics import Prec
    da = h * dh
    qkv = rnd(40, bsz, s, 3 * da)
    Q = bf(qkv)
    o = torch.full((bsz, s, da), 3.0, device=DEV, dtype=torch.bfloat16)
    S.sif_k_attn_fwd(Q, o, bsz, s, h, dh, 3 * da, da, causal)
    ref, _ = attention_fwd(q(qkv), h, dh, bool(causal), Prec("bf16"))
    assert_bf16_close(up(o), ref, f"fused attention s={s} dh={dh} causal={causal}", elem_slack=4e-3)


@pytest.mark.parametrize("causal", [0, 1])
@pytest.mark.parametrize("lens,h,dh", [([5, 130, 1, 64], 2, 64), ([256, 33, 129, 128, 7, 200, 32, 255], 3, 64), ([40], 2, 128), ([300, 17], 1, 128)])
def test_fused_attention_forward_sequences_of_unequal_length(lens, h, dh, causal):
    """Sequences stored back to back: each one's result is the oracle's for that sequence alone, and has the very bits
    of a launch that holds only that sequence; rows of the output that belong to no sequence are not written."""
    from oracle.decoder import attention_fwd
    from oracle.numerics import Prec
    da, total = h * dh, sum(lens)
    qkv = rnd(43, total + 3, 3 * da)                       # three rows after the last sequence
    Q = bf(qkv)
    o = torch.full((total + 3, da), 3.0, device=DEV, dtype=torch.bfloat16)
    starts = [0]
    for n in lens:
        starts.append(starts[-1] + n)
    S.sif_k_attn_fwd_varlen(Q, o, starts, h, dh, 3 * da, da, causal)
    got = up(o)
    assert np.all(got[total:] == 3.0)
    for i, n in enumerate(lens):
        rows = slice(starts[i], starts[i + 1])
        ref, _ = attention_fwd(q(qkv[rows])[None], h, dh, bool(causal), Prec("bf16"))
        assert_bf16_close(got[rows], ref[0], f"sequence {i} of {lens}, dh={dh} causal={causal}", elem_slack=4e-3)
        alone = torch.zeros((n, da), device=DEV, dtype=torch.bfloat16)
        S.sif_k_attn_fwd(Q[rows].contiguous(), alone, 1, n, h, dh, 3 * da, da, causal)
        assert np.array_equal(got[rows], up(alone))
    with pytest.raises(S.SifError):
        S.sif_k_attn_fwd_varlen(Q, o, [0, 5, 5], h, dh, 3 * da, da, causal)          # an empty sequence


@pytest.mark.parametrize("causal", [0, 1])
@pytest.mark.parametrize("bsz,s,h,dh", [(2, 5, 2, 64), (3, 37, 2, 64), (2, 128, 3, 64), (2, 200, 2, 64), (1, 300, 2, 128), (2, 64, 1, 128),
                                        (1, 520, 1, 64)])
def test_fused_attention_backward(bsz, s, h, dh, causal):
    from oracle.decoder import attention_bwd, attention_fwd
    from oracle.numerics import Prec
    da = h * dh
    qkv, do = rnd(41, bsz, s, 3 * da), rnd(42, bsz, s, da)
    Q, DO = bf(qkv), bf(do)
    o = torch.zeros((bsz, s, da), device=DEV, dtype=torch.bfloat16)
    lse = torch.full((bsz * h, s), 7.0, device=DEV)
    delta = torch.zeros((bsz * h, s), device=DEV)
    dqkv = torch.full((bsz, s, 3 * da), 5.0, device=DEV, dtype=torch.bfloat16)
    S.sif_k_attn_fwd(Q, o, bsz, s, h, dh, 3 * da, da, causal, lse=lse)
    S.sif_k_attn_bwd(Q, o, DO, lse, delta, dqkv, bsz, s, h, dh, 3 * da, da, 3 * da, causal)
    prec = Prec("bf16")
    ref_o, p = attention_fwd(q(qkv), h, dh, bool(causal), prec)
    ref = attention_bwd(q(do), q(qkv), p, h, dh, prec)
    assert_f32_close(up(lse), lse_reference(q(qkv), h, dh, bool(causal)), "lse", tol=1e-5)
    ref_delta = (q(do) * ref_o).reshape(bsz, s, h, dh).sum(-1).transpose(0, 2, 1).reshape(bsz * h, s)
    assert rel_err(up(delta), ref_delta) <= 2e-2
    got = up(dqkv)
    for name, lo in (("dq", 0), ("dk", da), ("dv", 2 * da)):
        assert_bf16_close(got[..., lo:lo + da], ref[..., lo:lo + da], f"fused attention {name} s={s} dh={dh} causal={causal}", elem_slack=6e-3)


def test_tiles_fetched_into_lds_give_the_same_bits_beside_other_kernels():
    """The attention kernels and the GEMM fetch their tiles global -> LDS in parts, one part per wavefront, and a
    barrier publishes the tile: every wavefront has to wait for its own part in front of that barrier.  When it did
    not, the results were right on a quiet device and changed now and then once other kernels kept the memory system
    busy.  Here the kernels run many times on one stream while copies run on another; every result must have the bits
    of the quiet run."""
    bsz, s, h, dh = 16, 512, 12, 64
    da = h * dh
    Q, DO = bf(rnd(51, bsz, s, 3 * da)), bf(rnd(52, bsz, s, da))
    m, n, k = 2048, 2304, 768
    A, B = bf(rnd(53, m, k)), bf(rnd(54, n, k))

    def run(stream):
        o = torch.zeros((bsz, s, da), device=DEV, dtype=torch.bfloat16)
        lse, delta = torch.zeros((bsz * h, s), device=DEV), torch.zeros((bsz * h, s), device=DEV)
        dqkv = torch.zeros((bsz, s, 3 * da), device=DEV, dtype=torch.bfloat16)
        c = torch.zeros((m, n), device=DEV, dtype=torch.bfloat16)
        torch.cuda.synchronize()
        S.sif_k_attn_fwd(Q, o, bsz, s, h, dh, 3 * da, da, 1, lse=lse, stream=stream)
        S.sif_k_attn_bwd(Q, o, DO, lse, delta, dqkv, bsz, s, h, dh, 3 * da, da, 3 * da, 1, stream=stream)
        S.sif_k_gemm_bf16(A, B, c, m, n, k, k, k, n, stream=stream)
        return o, lse, dqkv, c

    quiet = [t.cpu() for t in run(None)]
    torch.cuda.synchronize()
    side, main = torch.cuda.Stream(), torch.cuda.Stream()
    big = torch.zeros(64 * 2 ** 20, device=DEV)
    for rep in range(12):
        with torch.cuda.stream(side):
            for _ in range(4):
                big.add_(1.0)                      # 256 MB read and written per pass, beside the kernels under test
        got = run(main)
        torch.cuda.synchronize()
        for name, a, b in zip(("o", "lse", "dqkv", "c"), quiet, got):
            assert torch.equal(a, b.cpu()), f"{name} differs from the quiet run in repetition {rep}"


@pytest.mark.parametrize("tile", [128, 256])
def test_gemm_bf16_packed_and_fp32_staged_epilogues_give_the_same_bits(tile):
    """Epilogues that read only the bias are finished in the accumulator layout and staged as bf16; with the
    pre-activation output requested the same product takes the fp32-staged path.  Both must give the same bits."""
    m, n, k = 520, 776, 192
    a, b, bias = rnd(61, m, k), rnd(62, n, k), rnd(63, n)
    A, B, BI = bf(a), bf(b), bf(bias)
    c0 = torch.zeros((m, n), device=DEV, dtype=torch.bfloat16)
    c1, z = torch.zeros_like(c0), torch.zeros_like(c0)
    S.sif_k_gemm_bf16(A, B, c0, m, n, k, k, k, n, epilogue=S.SIF_EPI_GELU, bias=BI, tile=tile)
    S.sif_k_gemm_bf16(A, B, c1, m, n, k, k, k, n, epilogue=S.SIF_EPI_GELU, bias=BI, aux=z, tile=tile)
    torch.cuda.synchronize()
    assert torch.equal(c0, c1)
    acc = q(a) @ q(b).T + q(bias)
    assert_bf16_close(up(z), acc, "pre-activation")
    assert_bf16_close(up(c0), N.gelu(acc), "gelu epilogue", elem_slack=1e-2)
