"""The column sum that allocates nothing (sif_k_colsum_static): its partial sums live in a device array inside
the library.  Checked through the C ABI against sif_k_colsum (same bits: the kernels are the same) and against the
sum written out in fp64, on two calls in a row, the second with a smaller input that leaves most of the array as
the first call left it.  Collected last: it must pass alone in a fresh process and after all other tests."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import paper_2503_02550_amd as S
    from gpu_util import DEV, bf, up, q, assert_bf16_close


def _draw(seed, rows, ld):
    return np.random.default_rng(seed).standard_normal((rows, ld)).astype(np.float32)


def test_static_scratch_column_sum_matches_the_allocating_entry_point_twice_in_a_row():
    for seed, rows, n, ld in ((31, 4100, 2048, 2056), (32, 333, 776, 784)):          # 512 x 2048 floats = the whole array; then a small one
        x = _draw(seed, rows, ld)
        X = bf(x)
        want = torch.zeros(n, device=DEV, dtype=torch.bfloat16)
        part = torch.zeros(S.sif_colsum_parts(rows) * n, device=DEV)
        got = torch.full((n,), 7.0, device=DEV, dtype=torch.bfloat16)
        torch.cuda.synchronize()
        S.sif_k_colsum(X, ld, want, part, rows, n)
        S.sif_k_colsum_static(X, ld, got, rows, n)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (rows, n)
        assert_bf16_close(up(got), q(x)[:, :n].sum(axis=0), f"static colsum {rows}x{n}")


def test_static_scratch_column_sum_refuses_what_does_not_fit():
    rows, n = 8192, 2056                                                            # 512 parts x 2056 columns > 2^20 floats
    assert S.sif_colsum_parts(rows) * n > S.sif_colsum_static_max_floats()
    X = torch.zeros((rows, n), device=DEV, dtype=torch.bfloat16)
    out = torch.full((n,), 3.0, device=DEV, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    with pytest.raises(S.SifError) as e:
        S.sif_k_colsum_static(X, n, out, rows, n)
    assert e.value.status == S.SIF_E_NOMEM and "static buffer" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())                                                 # nothing was launched
    with pytest.raises(S.SifError):
        S.sif_k_colsum_static(X, n, None, 16, 8)
