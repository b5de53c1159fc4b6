"""Host-side pins of the arithmetic identity behind the kernels that run fp32 contractions
on the bf16 matrix cores: an fp32 number is the exact sum of three bfloat16 numbers taken by
truncation, and the six piece products that are kept reproduce a dot product to fp32's own
rounding level.  Plain numpy on bit patterns; no GPU."""
import numpy as np


def split3(x):
    """h, m, l (each a float32 whose low 16 bits are zero, i.e. a bfloat16 value) with
    h + m + l == x: masks and exact subtractions, as in the kernels."""
    x = np.asarray(x, dtype=np.float32)
    h = (x.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    r1 = x - h
    m = (r1.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    r2 = r1 - m
    l = (r2.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    return h, m, l, r2


def samples(n, seed):
    rng = np.random.default_rng(seed)
    bits = rng.integers(0, 2 ** 32, size=n, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    x = x[np.isfinite(x) & (np.abs(x) > 1e-30) & (np.abs(x) < 1e30)]
    special = np.array([0.0, -0.0, 1.0, -1.0, 1.0 + 2.0 ** -23, 1.0 - 2.0 ** -24, 3.1415927, -65504.0, 2.0 ** -100,
                        np.float32(1e-5), np.float32(0.1), 255.0, 16777215.0], dtype=np.float32)
    return np.concatenate([x, special, rng.standard_normal(n).astype(np.float32) * 0.1])


def test_three_truncated_pieces_reproduce_the_number_exactly():
    x = samples(1_000_000, 0)
    h, m, l, r2 = split3(x)
    assert np.array_equal(r2.view(np.uint32) & np.uint32(0xFFFF), np.zeros(x.size, np.uint32)), \
        "the last remainder already fits bfloat16: nothing is lost by keeping its upper half"
    total = h.astype(np.float64) + m.astype(np.float64) + l.astype(np.float64)
    assert np.array_equal(total, x.astype(np.float64))
    # the subtractions are exact and the pieces shrink by 2^-8 each
    nz = x != 0
    assert np.all(np.abs(m[nz]) <= np.abs(x[nz]) * 2.0 ** -7) and np.all(np.abs(l[nz]) <= np.abs(x[nz]) * 2.0 ** -15)


def test_six_piece_products_match_the_dot_product_to_fp32_rounding():
    rng = np.random.default_rng(1)
    K = 64
    for scale in (1.0, 1e-3, 300.0):
        w = (rng.standard_normal((512, K)) * scale / 8).astype(np.float32)
        e = (rng.standard_normal((512, K)) * 0.1 + 0.3).astype(np.float32)
        exact = (w.astype(np.float64) * e.astype(np.float64)).sum(axis=1)
        wh, wm, wl, _ = split3(w)
        eh, em, el, _ = split3(e)
        f = lambda a, b: (a.astype(np.float64) * b.astype(np.float64)).sum(axis=1)
        kept = f(wh, eh) + f(wh, em) + f(wm, eh) + f(wm, em) + f(wh, el) + f(wl, eh)
        bound = 2.0 ** -22 * (np.abs(w).astype(np.float64) * np.abs(e).astype(np.float64)).sum(axis=1)
        assert np.all(np.abs(kept - exact) <= bound)
        # every piece product is exact in fp32 (8 x 8 significant bits), so the matrix core adds exact terms
        p = wh.astype(np.float32) * eh.astype(np.float32)
        assert np.array_equal(p.astype(np.float64), wh.astype(np.float64) * eh.astype(np.float64))


def test_small_integer_codes_are_exact_bfloat16_values():
    # (the codes of Eq. 3 are at most 255: one piece, no splitting)
    c = np.arange(256, dtype=np.float32)
    assert np.array_equal(c.view(np.uint32) & np.uint32(0xFFFF), np.zeros(256, np.uint32))
