"""The arithmetic behind LP_FP32_PRODUCTS_BF16X6, checked with NumPy (no GPU, no library code):

* an fp32 value is the exact sum of three bfloat16 terms taken by repeated round-to-nearest of what is left over
  (for magnitudes up to the largest bfloat16, 3.39e38: above it the first term rounds to infinity);
* the six term products the kernels keep reproduce the fp64 product of two fp32 values to within 2^-24 relative
  (the three left out are each below 2^-25 of it), i.e. within half an fp32 rounding;
* accumulated in fp32 over a row, the split product is as close to fp64 as a plain fp32 accumulation.
"""
import numpy as np


def to_bf16(x):
    """Round fp32 to the nearest bfloat16 (ties to even), returned as fp32."""
    u = np.asarray(x, np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32)


def split3(x):
    x = np.asarray(x, np.float32)
    t0 = to_bf16(x)
    r1 = (x - t0).astype(np.float32)
    t1 = to_bf16(r1)
    r2 = (r1 - t1).astype(np.float32)
    t2 = to_bf16(r2)
    return t0, t1, t2


KEPT = [(2, 0), (0, 2), (1, 1), (1, 0), (0, 1), (0, 0)]   # (term of x, term of y), smallest products first


def test_three_terms_add_up_exactly():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32),
                        (rng.standard_normal(50000) * 1e-6).astype(np.float32),
                        (rng.standard_normal(50000) * 1e6).astype(np.float32),
                        np.float32([0.0, 1.0, -1.0, 1.0 + 2.0 ** -23, 2.0 ** -100, 3.0e38, 255.99998])])
    t0, t1, t2 = split3(x)
    total = t0.astype(np.float64) + t1.astype(np.float64) + t2.astype(np.float64)
    assert np.array_equal(total, x.astype(np.float64))
    nz = x != 0
    assert np.all(np.abs(t1[nz]) <= 2.0 ** -8 * np.abs(x[nz])) and np.all(np.abs(t2[nz]) <= 2.0 ** -16 * np.abs(x[nz]))


def test_six_kept_products_are_within_half_an_fp32_rounding():
    rng = np.random.default_rng(2)
    x = rng.standard_normal(300000).astype(np.float32)
    y = rng.standard_normal(300000).astype(np.float32)
    tx, ty = split3(x), split3(y)
    kept = sum(tx[i].astype(np.float64) * ty[j].astype(np.float64) for i, j in KEPT)
    exact = x.astype(np.float64) * y.astype(np.float64)
    assert np.all(np.abs(kept - exact) <= 2.0 ** -24 * np.abs(exact))
    # every single term product fits in fp32 (two 8-bit significands), so the matrix cores add exact products
    for i, j in KEPT:
        p = tx[i].astype(np.float64) * ty[j].astype(np.float64)
        assert np.array_equal(p.astype(np.float32).astype(np.float64), p)


def test_accumulated_rows_are_as_close_to_fp64_as_fp32_accumulation():
    rng = np.random.default_rng(3)
    M, K, N = 96, 512, 64
    A = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32)
    ref = A.astype(np.float64) @ W.astype(np.float64)
    ta, tw = split3(A), split3(W)
    split = np.zeros((M, N), np.float32)
    plain = np.zeros((M, N), np.float32)
    for k in range(0, K, 16):     # sixteen values per matrix instruction, rounded into the fp32 accumulator
        for i, j in KEPT:
            split = (split.astype(np.float64) + ta[i][:, k:k + 16].astype(np.float64) @ tw[j][k:k + 16].astype(np.float64)).astype(np.float32)
        for kk in range(k, k + 16, 2):
            plain = (plain.astype(np.float64) + A[:, kk:kk + 2].astype(np.float64) @ W[kk:kk + 2].astype(np.float64)).astype(np.float32)
    err = lambda C: np.linalg.norm(C - ref) / np.linalg.norm(ref)
    assert err(split) <= 1.25 * err(plain) and err(split) < 1e-6
