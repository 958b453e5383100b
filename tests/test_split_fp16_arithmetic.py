"""The arithmetic of the opt-in split-fp16 products, emulated in NumPy on the CPU (no GPU, no library call).

The library's header states the scheme: every fp32 operand is scaled by the power of two that brings the matrix's
largest entry into [2^14, 2^15), split into hi = fp16(s x) and lo = fp16(s x - hi), and the product is accumulated
as hiA hiB + hiA loB + loA hiB.  These tests pin what that statement promises: no overflow for any input range,
22 bits kept for every entry within 2^-17 of the largest, each of the three partial products exact in fp32, and a
product error around 3e-7 of a term - below what fp32 accumulation of a 4096-long sum costs anyway."""
import numpy as np
import pytest


def split(x):
    """(hi, lo, s) of a float32 array by the stated rule."""
    x = np.asarray(x, dtype=np.float32)
    amax = float(np.max(np.abs(x))) if x.size else 0.0
    s = 1.0
    if amax > 0 and np.isfinite(amax):
        s = 2.0 ** (14 - int(np.floor(np.log2(amax))))
    y = (x * np.float32(s)).astype(np.float32)                 # exact: a power of two
    hi = y.astype(np.float16)
    lo = (y - hi.astype(np.float32)).astype(np.float16)
    return hi, lo, s


@pytest.mark.parametrize("amax", [1.0, 0.999, 3.7e-5, 8191.5, 65504.0, 1e20, 2.0 ** -100, 1.0000001])
def test_scaling_brings_the_largest_entry_under_the_fp16_range(amax):
    rng = np.random.default_rng(0)
    x = (rng.uniform(-1, 1, 1000) * amax).astype(np.float32)
    x[17] = amax
    hi, lo, s = split(x)
    top = float(np.max(np.abs(x))) * s
    assert 2.0 ** 14 <= top < 2.0 ** 15
    assert np.all(np.isfinite(hi.astype(np.float32))) and np.all(np.isfinite(lo.astype(np.float32)))


def test_zero_matrix_and_single_entries():
    hi, lo, s = split(np.zeros(10, np.float32))
    assert s == 1.0 and not hi.any() and not lo.any()
    hi, lo, s = split(np.array([0.0, -3.0], np.float32))
    assert float(hi[1]) / s == -3.0 and float(lo[1]) == 0.0


def test_pair_keeps_22_bits_of_entries_within_2_to_minus_17_of_the_largest():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(200000) * np.exp(3 * rng.standard_normal(200000))).astype(np.float32)
    hi, lo, s = split(x)
    back = (hi.astype(np.float64) + lo.astype(np.float64)) / s
    amax = np.max(np.abs(x))
    big = np.abs(x) >= amax * 2.0 ** -17
    rel = np.abs(back[big] - x[big].astype(np.float64)) / np.abs(x[big])
    assert rel.max() <= 2.0 ** -22
    # smaller entries lose bits gracefully (their lo parts become fp16 subnormals): the absolute error of any entry
    # stays below 2^-39 of the LARGEST entry, or 2^-22 of its own size, whichever is larger
    err = np.abs(back - x.astype(np.float64))
    assert np.all(err <= np.maximum(np.abs(x).astype(np.float64) * 2.0 ** -22, float(amax) * 2.0 ** -39))


def test_each_partial_product_is_exact_in_fp32():
    rng = np.random.default_rng(2)
    a = rng.standard_normal(50000).astype(np.float32)
    b = (rng.standard_normal(50000) * 7).astype(np.float32)
    ah, al, _ = split(a)
    bh, bl, _ = split(b)
    for u, v in ((ah, bh), (ah, bl), (al, bh)):
        exact = u.astype(np.float64) * v.astype(np.float64)
        assert np.array_equal((u.astype(np.float32) * v.astype(np.float32)).astype(np.float64), exact)


@pytest.mark.parametrize("k,outlier", [(4096, 1.0), (4096, 50.0), (512, 1.0)])
def test_three_term_product_against_the_exact_product(k, outlier):
    """A^T B with k-long sums, the three terms added exactly (float64) so that only the scheme's own error shows:
    dropped lo*lo term and the operands' bits 23-24."""
    rng = np.random.default_rng(k)
    A = (rng.standard_normal((k, 48)) / np.sqrt(k)).astype(np.float32)          # like the rows of an orthogonal Q
    B = (rng.standard_normal((k, 40)) * 0.02).astype(np.float32)
    B[:5] *= outlier                                                              # a few heavy input channels
    Ah, Al, sa = split(A)
    Bh, Bl, sb = split(B)
    f = lambda m: m.astype(np.float64)
    got = (f(Ah).T @ f(Bh) + f(Ah).T @ f(Bl) + f(Al).T @ f(Bh)) / (sa * sb)
    ref = f(A).T @ f(B)
    err = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert err < 6e-7
    # for comparison: the same sum accumulated in plain fp32, k terms one after the other per output
    acc = np.zeros((48, 40), np.float32)
    for r in range(0, k, 8):                                    # eight terms per step keep the loop short
        acc += (A[r:r + 8].T @ B[r:r + 8]).astype(np.float32)
    err32 = np.linalg.norm(acc.astype(np.float64) - ref) / np.linalg.norm(ref)
    assert err < 4 * max(err32, 1e-7)
