"""The arithmetic fact the encoders' matrix path rests on, checked on the CPU with numpy: an fp32
value is the exact sum of three bf16 pieces (each the nearest bf16 of what is left), a product of
two pieces is exact in fp32, and leaving out the three piece products of order > 2 changes a
product by less than 2^-22 of its magnitude.  (The GPU parity tests check the kernels themselves; their rounding
bands assume exactly this.)"""
import numpy as np


def _bf16(v):
    """Round fp32 to bf16 (nearest, ties to even), returned as fp32."""
    b = v.view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return b.astype(np.uint32).view(np.float32)


def _split3(v):
    p0 = _bf16(v)
    r = v - p0
    p1 = _bf16(r)
    s = r - p1
    p2 = _bf16(s)
    return p0, p1, p2, s - p2


def _values(n, seed):
    rng = np.random.default_rng(seed)
    v = (rng.standard_normal(n) * np.exp(rng.uniform(-20, 20, n))).astype(np.float32)
    v[:8] = np.float32([0.0, 1.0, -1.0, 3.0, 1.0 + 2.0 ** -23, -(2.0 - 2.0 ** -23), 2.0 ** -100, 65504.0])
    return v


def test_three_pieces_leave_nothing():
    v = _values(200000, 1)
    p0, p1, p2, rest = _split3(v)
    assert np.all(rest == 0.0)
    assert np.all(p0.astype(np.float64) + p1.astype(np.float64) + p2.astype(np.float64) == v.astype(np.float64))
    for p in (p0, p1, p2):                                        # each piece is a bf16 number
        assert np.all((p.view(np.uint32) & np.uint32(0xFFFF)) == 0)
    nz = v != 0
    assert np.all(np.abs(p1[nz]) <= np.abs(v[nz]) * 2.0 ** -8 * (1 + 2.0 ** -7))
    assert np.all(np.abs(p2[nz]) <= np.abs(v[nz]) * 2.0 ** -16 * (1 + 2.0 ** -7))


def test_piece_products_are_exact_in_fp32_and_the_omitted_ones_are_negligible():
    x, c = _values(100000, 2), _values(100000, 3)
    x = np.clip(x, -1e15, 1e15)
    c = np.clip(c, -1e15, 1e15)
    xs, cs = _split3(x)[:3], _split3(c)[:3]
    exact = x.astype(np.float64) * c.astype(np.float64)
    kept = np.zeros_like(exact)
    for i in range(3):
        for j in range(3):
            prod32 = xs[i] * cs[j]                                # fp32 product
            prod64 = xs[i].astype(np.float64) * cs[j].astype(np.float64)
            ok = (prod64 == 0) | (np.abs(prod64) > 1e-30)         # leave fp32 underflow aside
            assert np.all(prod32.astype(np.float64)[ok] == prod64[ok])
            if i + j <= 2:
                kept += prod64
    nz = exact != 0
    assert np.all(np.abs(kept - exact)[nz] <= np.abs(exact[nz]) * 2.0 ** -22)
