"""The prefill encode kernel trusts a matrix-core score only when it beats the runner-up by more
than an error bound.  That bound assumes a rounding model for the fp16 MFMA instructions (exact
products; a sum that loses at most 2^-23 of the largest magnitude in flight per term and for the
final rounding; fp16 subnormal inputs honoured).  These tests pin the model to the hardware
through cq_probe_mfma, against exact fp64 sums of the same fp16 operands."""
import numpy as np
import pytest
import torch

import paper_2405_03917_amd as cq

pytestmark = pytest.mark.gpu


def _mfma(a16: np.ndarray, b16: np.ndarray) -> np.ndarray:
    d = cq.cq_probe_mfma(torch.from_numpy(a16).cuda(), torch.from_numpy(b16).cuda())
    torch.cuda.synchronize()
    return d.cpu().numpy().astype(np.float64)


def _record(cb: np.ndarray, kdim: int) -> np.ndarray:
    """Rows [channels | three fp16 pieces of -|c|^2 / 2 | zeros], as the kernel stages them."""
    n, c = cb.shape
    a = np.zeros((n, kdim), dtype=np.float16)
    a[:, :c] = cb
    v = (-0.5 * (cb.astype(np.float32) ** 2).sum(-1, dtype=np.float32)).astype(np.float32)
    h1 = v.astype(np.float16)
    r1 = (v - h1.astype(np.float32)).astype(np.float32)
    h2 = r1.astype(np.float16)
    h3 = (r1 - h2.astype(np.float32)).astype(np.float16)
    a[:, c], a[:, c + 1], a[:, c + 2] = h1, h2, h3
    return a


@pytest.mark.parametrize("kdim,c", [(16, 8), (8, 4), (8, 2)])
def test_mfma_error_stays_inside_the_model(kdim, c):
    rng = np.random.default_rng(5 + c)
    worst = 0.0
    for trial in range(64):
        cs, xs = 8.0 * (1 + trial % 5), 8.0 * (1 + trial % 3)
        cb = (cs * rng.standard_normal((32, c))).astype(np.float16)
        a = _record(cb, kdim)
        b = np.zeros((kdim, 32), dtype=np.float16)
        b[:c] = (xs * rng.standard_normal((c, 32))).astype(np.float16)
        b[c:c + 3] = 1.0
        d = _mfma(a, b)
        terms = a.astype(np.float64)[:, :, None] * b.astype(np.float64)[None, :, :]     # [32, kdim, 32]
        exact, mag = terms.sum(1), np.abs(terms).sum(1)
        worst = max(worst, float((np.abs(d - exact) / mag).max()))
    # the kernel's budget for this part is 12 * 2^-23 of the magnitude sum; the hardware stays far below
    assert worst <= 12 * 2.0 ** -23, worst
    assert worst <= 4 * 2.0 ** -24, worst      # what this chip has been seen to do (worst about 2.9)


@pytest.mark.parametrize("kdim", [16, 8])
def test_mfma_honours_fp16_subnormals_and_keeps_exact_products(kdim):
    a = np.zeros((32, kdim), dtype=np.float16)
    b = np.zeros((kdim, 32), dtype=np.float16)
    a[:, 0] = np.float16(2.0 ** -20)            # fp16 subnormal
    b[0, :] = np.float16(1024.0)
    assert np.all(_mfma(a, b) == 2.0 ** -10)
    a[:, 0] = np.float16(1.0 + 2.0 ** -10)      # product needs 21 significant bits
    b[0, :] = np.float16(1.0 + 2.0 ** -10)
    assert np.all(_mfma(a, b) == (1.0 + 2.0 ** -10) ** 2)


@pytest.mark.parametrize("kdim", [16, 8])
def test_mfma_output_layout_matches_the_kernels_decoding(kdim):
    """d[i][j] = sum_k a[i][k] b[k][j] with a = one-hot rows and b = one-hot columns scaled by
    distinct values: checks the lane/register -> (row, column) map the encode kernel decodes."""
    rng = np.random.default_rng(1)
    a = rng.integers(-8, 9, size=(32, kdim)).astype(np.float16)
    b = rng.integers(-8, 9, size=(kdim, 32)).astype(np.float16)
    want = a.astype(np.float64) @ b.astype(np.float64)        # small integers: exact
    assert np.array_equal(_mfma(a, b), want)
