"""The arithmetic behind the stage-1 inner products, checked on the CPU with numpy alone.

The coarse kernels scale a row by a power of two, split it into hi = fp16(x) and lo = fp16(x - hi)
and accumulate lo*hi + hi*lo + hi*hi in fp32.  These tests pin the claims that design rests on
(they do not touch the library): the split keeps 22 bits, every fp16 product is exact in fp32,
and the resulting inner product is as accurate as an fp32 one.
"""
import numpy as np


def split(x, rowwise):
    m = np.abs(x).max(axis=1, keepdims=True) if rowwise else np.abs(x).max()
    e = np.floor(np.log2(m))
    s = np.exp2(14 - e).astype(np.float32)
    xs = (x * s).astype(np.float32)
    hi = xs.astype(np.float16)
    lo = (xs - hi.astype(np.float32)).astype(np.float16)
    return hi, lo, (1.0 / s).astype(np.float32), xs


def test_scaled_values_fit_fp16_and_the_split_keeps_22_bits():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((200, 96)) * np.exp2(rng.integers(-20, 20, size=(200, 1)))).astype(np.float32)
    hi, lo, inv, xs = split(x, rowwise=True)
    assert np.isfinite(hi.astype(np.float32)).all() and np.abs(hi.astype(np.float32)).max() < 65504
    assert (np.abs(xs).max(axis=1) >= 2.0 ** 14).all() and (np.abs(xs).max(axis=1) < 2.0 ** 15).all()
    # xs - hi is exact in fp32, and hi + lo reproduces xs to 2^-22 of the row's largest entry
    err = np.abs(xs.astype(np.float64) - hi.astype(np.float64) - lo.astype(np.float64))
    assert (err <= 2.0 ** -22 * np.abs(xs).max(axis=1, keepdims=True)).all()
    # elements not far below the largest keep their full 22 bits
    big = np.abs(xs) >= 2.0 ** -2
    assert (err[big] <= 2.0 ** -23 * np.abs(xs[big])).all()
    # the scale is a power of two: undoing it is exact
    assert (np.log2(inv) == np.round(np.log2(inv))).all()


def test_fp16_products_are_exact_in_fp32():
    rng = np.random.default_rng(4)
    a = rng.standard_normal(100000).astype(np.float16)
    b = (rng.standard_normal(100000) * 300).astype(np.float16)
    p32 = a.astype(np.float32) * b.astype(np.float32)
    assert (p32.astype(np.float64) == a.astype(np.float64) * b.astype(np.float64)).all()


def test_three_product_inner_product_is_as_accurate_as_fp32():
    rng = np.random.default_rng(5)
    D, nq, K = 96, 64, 1500
    Q = rng.standard_normal((nq, D)).astype(np.float32)
    Q /= np.linalg.norm(Q, axis=1, keepdims=True)
    C = (rng.standard_normal((K, D)) * 0.5 + Q[rng.integers(0, nq, K)]).astype(np.float32)
    C[:10] *= 2.0 ** -5                                   # some rows far below the table's scale
    exact = Q.astype(np.float64) @ C.astype(np.float64).T
    qh, ql, qs, _ = split(Q, rowwise=True)
    ch, cl, cs, _ = split(C, rowwise=False)
    f64 = lambda v: v.astype(np.float64)
    acc = np.zeros((nq, K), np.float32)
    for k0 in range(0, D, 16):                            # one matrix instruction = 16 dims, fp32 accumulate
        sl = slice(k0, k0 + 16)
        for a, b in ((ql, ch), (qh, cl), (qh, ch)):
            acc = (f64(acc) + f64(a[:, sl]) @ f64(b[:, sl]).T).astype(np.float32)
    dot = f64(acc) * f64(qs) * float(cs)
    seq = np.zeros((nq, K), np.float32)                   # the fp32 dot product it stands in for
    for k in range(D):
        seq = seq + Q[:, k:k + 1] * C[:, k][None, :]
    u = 2.0 ** -24
    scale = np.linalg.norm(Q, axis=1)[:, None] * np.linalg.norm(C, axis=1).max()
    e_split = np.abs(dot - exact) / (u * scale)
    e_seq = np.abs(f64(seq) - exact) / (u * scale)
    assert e_split.max() <= 4.0, e_split.max()            # a few units of fp32 rounding of |q||c|
    assert e_split.max() <= e_seq.max() * 1.5 + 1.0       # no worse than sequential fp32
