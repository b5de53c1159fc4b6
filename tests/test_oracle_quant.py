"""Pins for the CPU oracle's quantizer (no GPU).

Each test checks the oracle against something fixed outside of it: published
Philox known answers, the closed forms of Proposition 1 and its appendix proof
(unbiasedness, Var = p(1-p) per element, the d R^2 / (4 B^2) bound), the
endpoint and grid-point behaviour Eq. (3) implies, numpy's own bit packing, and
brute-force enumeration on tiny inputs.
"""
import os

import numpy as np
import pytest

from oracle import ref
from workloads import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ALL_BITS = [1, 2, 4, 8]


# ----------------------------------------------------------------- Philox ----
def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = ref.philox4x32_10(ctr, key)
        assert [int(x) for x in got] == want


def _philox_py(ctr, key):
    """Independent big-integer Philox4x32-10 (Python ints), used to pin the
    element -> (counter, word, half) mapping of noise16."""
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r:
            k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
    return c


def test_philox_py_matches_known_answers():
    for ctr, key, want in _kat_rows():
        assert _philox_py(ctr, key) == want


def test_noise16_mapping():
    rng = np.random.default_rng(5)
    cases = [(0, 0), (1, 7), (1, 8), (0xDEADBEEFCAFEF00D, (1 << 35) + 13), (2**64 - 1, 2**40 + 5)]
    cases += [(int(rng.integers(0, 2**63)), int(rng.integers(0, 2**45))) for _ in range(200)]
    for seed, i in cases:
        q = i >> 3
        o = _philox_py([q & 0xFFFFFFFF, q >> 32, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        w = o[(i >> 1) & 3]
        want = (w >> 16) if (i & 1) else (w & 0xFFFF)
        assert ref.noise16(seed, i) == want


def test_noise16_is_uniform():
    # 2^18 draws: mean of h/2^16 within 5 sigma of 1/2, chi-square over 64 bins
    n = 1 << 18
    h = np.array([ref.noise16(12345, i) for i in range(0, n)], dtype=np.float64)
    u = h / 65536.0
    assert abs(u.mean() - 0.5 + 0.5 / 65536) < 5 * np.sqrt(1 / 12 / n)
    counts = np.bincount((h // 1024).astype(int), minlength=64)
    chi2 = ((counts - n / 64) ** 2 / (n / 64)).sum()
    assert chi2 < 63 + 6 * np.sqrt(2 * 63)
    # neighbouring elements are not correlated
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 5 / np.sqrt(n)


# ------------------------------------------------------------ bit packing ----
@pytest.mark.parametrize("bits", ALL_BITS)
def test_pack_matches_numpy_packbits(bits):
    rng = np.random.default_rng(bits)
    n = 8 * 37
    codes = rng.integers(0, 1 << bits, size=n, dtype=np.uint8)
    # LSB-first stream of the b bits of each code, element order = memory order
    bitmat = ((codes[:, None] >> np.arange(bits)) & 1).astype(np.uint8)
    want = np.packbits(bitmat.ravel(), bitorder="little")
    got = ref.pack(codes, bits)
    assert got.size == n * bits // 8
    assert np.array_equal(got, want)
    assert np.array_equal(ref.unpack(got, n, bits), codes)


@pytest.mark.parametrize("bits", ALL_BITS)
def test_pack_every_code_at_every_position(bits):
    per_byte = 8 // bits
    for pos in range(per_byte):
        for code in range(1 << bits):
            codes = np.zeros(per_byte * 3, dtype=np.uint8)
            codes[per_byte + pos] = code
            packed = ref.pack(codes, bits)
            assert packed[0] == 0 and packed[2] == 0
            assert packed[1] == code << (pos * bits)
            assert np.array_equal(ref.unpack(packed, codes.size, bits), codes)


def test_pack_rejects_wide_code():
    with pytest.raises(ValueError):
        ref.pack(np.array([0, 4, 0, 0], dtype=np.uint8), 2)


# -------------------------------------------------- Eq. (3): deterministic ----
@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("group", [32, 64, 128, 256])
def test_endpoints_and_range(bits, group):
    B = (1 << bits) - 1
    x = gen.student_t_activations(64, 64, seed=3)
    for seed in range(20):
        codes, gmin, gscale = ref.quantize_codes(x, bits, group, seed)
        xg = x.reshape(-1, group)
        cg = codes.reshape(-1, group)
        assert cg.max() <= B
        assert np.array_equal(gmin, xg.min(axis=1))
        is_min = xg == xg.min(axis=1, keepdims=True)
        is_max = xg == xg.max(axis=1, keepdims=True)
        assert np.all(cg[is_min] == 0)
        assert np.all(cg[is_max] == B)
        rng_ = xg.max(axis=1) - xg.min(axis=1)
        assert np.array_equal(gscale, (rng_ / np.float32(B)).astype(np.float32))


@pytest.mark.parametrize("bits", ALL_BITS)
def test_dyadic_grid_round_trips_for_every_seed(bits):
    # groups on an exactly representable grid: min integer, range = B * 2^k
    B = (1 << bits) - 1
    rng = np.random.default_rng(11)
    group = 64
    rows = []
    want = []
    for k in (-3, 0, 5):
        step = np.float32(2.0 ** k)
        for mn in (-7.0, 0.0, 12.0):
            j = rng.integers(0, B + 1, size=group)
            j[0], j[1] = 0, B  # make sure both ends are present
            rows.append(np.float32(mn) + j.astype(np.float32) * step)
            want.append(j)
    x = np.stack(rows).astype(np.float32)
    want = np.concatenate(want).astype(np.uint8)
    for seed in range(50):
        codes, gmin, gscale = ref.quantize_codes(x, bits, group, seed)
        assert np.array_equal(codes, want)
        packed, gmin2, gscale2 = ref.quantize(x, bits, group, seed)
        assert np.array_equal(gmin, gmin2) and np.array_equal(gscale, gscale2)
        xh = ref.dequantize(packed, gmin, gscale, x.shape[0], x.shape[1], bits, group)
        assert np.array_equal(xh.view(np.uint32), x.view(np.uint32))


@pytest.mark.parametrize("bits", ALL_BITS)
def test_codes_are_floor_or_ceil_of_exact_value(bits):
    # whatever the random draw, code is one of the two integers around the exact
    # (e - Z) / R * B (computed in float64), up to one float32 rounding of slack
    B = (1 << bits) - 1
    x = gen.normal_activations(128, 64, seed=7)
    codes, gmin, gscale = ref.quantize_codes(x, bits, 64, seed=9)
    xg = x.reshape(-1, 64).astype(np.float64)
    mn = xg.min(axis=1, keepdims=True)
    R = xg.max(axis=1, keepdims=True) - mn
    exact = (xg - mn) / R * B
    c = codes.reshape(-1, 64).astype(np.float64)
    assert np.all(c >= np.floor(exact - 1e-4))
    assert np.all(c <= np.ceil(exact + 1e-4))
    # and dequantisation error is below one step (Eq. 4)
    xh = ref.dequantize(ref.pack(codes, bits), gmin, gscale, 128, 64, bits, 64).astype(np.float64)
    step = gscale.astype(np.float64)[:, None]
    assert np.all(np.abs(xh.reshape(-1, 64) - xg) <= step * (1 + 2.0 ** -20))


def test_dequantize_is_eq4():
    # Eq. (4) with exact rational arithmetic on a case where R*code/B + Z is
    # representable: scale 0.25, min -3 -> values -3 + 0.25*code
    for bits in ALL_BITS:
        B = (1 << bits) - 1
        codes = (np.arange(64) % (B + 1)).astype(np.uint8)
        gmin = np.array([-3.0], dtype=np.float32)
        gscale = np.array([0.25], dtype=np.float32)
        out = ref.dequantize(ref.pack(codes, bits), gmin, gscale, 1, 64, bits, 64)
        assert np.array_equal(out.ravel(), (-3.0 + 0.25 * codes).astype(np.float32))


def test_constant_negzero_and_tiny_groups():
    x = np.zeros((5, 64), dtype=np.float32)
    x[4, :] = np.float32(1e-36) * np.arange(64, dtype=np.float32) / 63   # tiny normal range
    x[0, :] = 2.5                       # constant group
    x[1, :] = -0.0                      # all negative zero
    x[2, :] = np.float32(1e-40) * np.arange(64, dtype=np.float32)   # denormal range
    x[3, :] = np.linspace(-1, 1, 64, dtype=np.float32)
    x[3, 5] = -0.0
    for bits in ALL_BITS:
        B = (1 << bits) - 1
        for seed in range(5):
            codes, gmin, gscale = ref.quantize_codes(x, bits, 64, seed)
            c = codes.reshape(5, 64)
            assert np.all(c[0] == 0) and gmin[0] == np.float32(2.5) and gscale[0] == 0
            assert np.all(c[1] == 0) and gmin[1].view(np.uint32) == 0  # stored as +0
            assert gscale[1].view(np.uint32) == 0                      # R/B is +0 too
            assert c[2, 0] == 0 and c[2, 63] == B and np.all(c[2] <= B)
            assert np.all(np.diff(c[2].astype(int)) >= -1)
            xh = ref.dequantize(ref.pack(codes, bits), gmin, gscale, 5, 64, bits, 64)
            assert np.array_equal(xh[0], x[0])
            assert np.all(xh[1] == 0)
            # B/R overflows for this row: the factor is clamped, codes lean low,
            # but every value still decodes inside the group's range
            assert np.all(np.abs(xh[2] - x[2]) <= (x[2, 63] - x[2, 0]) * 1.01)
            # a tiny but normal range quantizes as usual: error below one step
            assert c[4, 0] == 0 and c[4, 63] == B
            assert np.all(np.abs(xh[4].astype(np.float64) - x[4]) <= float(gscale[4]) * 1.001 + 1e-44)


def test_slice_with_first_index_equals_full_run():
    x = gen.normal_activations(256, 64, seed=1)
    for bits, group in [(2, 64), (4, 128), (8, 32), (2, 256)]:
        full_p, full_mn, full_sc = ref.quantize(x, bits, group, seed=77)
        r0, r1 = 96, 160
        part_p, part_mn, part_sc = ref.quantize(x[r0:r1], bits, group, seed=77, first_index=r0 * 64)
        b0, b1 = r0 * 64 * bits // 8, r1 * 64 * bits // 8
        assert np.array_equal(part_p, full_p[b0:b1])
        assert np.array_equal(part_mn, full_mn[r0 * 64 // group:r1 * 64 // group])
        assert np.array_equal(part_sc, full_sc[r0 * 64 // group:r1 * 64 // group])
        # a different seed changes the codes, the same seed does not
        again, _, _ = ref.quantize(x, bits, group, seed=77)
        other, _, _ = ref.quantize(x, bits, group, seed=78)
        assert np.array_equal(again, full_p) and not np.array_equal(other, full_p)


def test_shape_errors():
    x = np.zeros((3, 50), dtype=np.float32)
    with pytest.raises(ValueError):
        ref.quantize(x, 2, 64, 0)
    with pytest.raises(ValueError):
        ref.quantize(np.zeros((2, 64), np.float32), 3, 64, 0)


@pytest.mark.parametrize("bits,group", [(2, 64), (4, 128), (8, 64), (2, 32), (1, 256)])
def test_bytes_per_activation(bits, group):
    # codes + fp32 min + fp32 scale per group  ->  b/8 + 8/G bytes per element
    x = gen.normal_activations(64, 64, seed=0)
    packed, gmin, gscale = ref.quantize(x, bits, group, 0)
    total = packed.nbytes + gmin.nbytes + gscale.nbytes
    assert total / x.size == bits / 8 + 8 / group


# ----------------------------------------- nearest rounding (Table 6 switch) --
@pytest.mark.parametrize("bits", ALL_BITS)
def test_nearest_rounding(bits):
    B = (1 << bits) - 1
    x = gen.normal_activations(64, 64, seed=21)
    codes, gmin, gscale = ref.quantize_codes(x, bits, 64, seed=0, rounding=1)
    xg = x.reshape(-1, 64).astype(np.float64)
    mn = xg.min(axis=1, keepdims=True)
    R = xg.max(axis=1, keepdims=True) - mn
    exact = (xg - mn) / R * B
    c = codes.reshape(-1, 64).astype(np.float64)
    near_tie = np.abs(exact - np.floor(exact) - 0.5) < 1e-4
    assert np.all((c == np.floor(exact + 0.5)) | near_tie)
    # independent of the seed
    codes2, _, _ = ref.quantize_codes(x, bits, 64, seed=99, rounding=1)
    assert np.array_equal(codes, codes2)


# ---------------------------------------- Proposition 1: bias and variance ----
def _moments(x, bits, group, n_seeds):
    """Per-element mean and variance of Dequant(Quant(x)) over seeds."""
    s1 = np.zeros(x.shape, dtype=np.float64)
    s2 = np.zeros(x.shape, dtype=np.float64)
    for seed in range(n_seeds):
        p, mn, sc = ref.quantize(x, bits, group, seed)
        xh = ref.dequantize(p, mn, sc, x.shape[0], x.shape[1], bits, group).astype(np.float64)
        s1 += xh
        s2 += xh * xh
    mean = s1 / n_seeds
    var = s2 / n_seeds - mean * mean
    return mean, var


def _frac_and_scale(x, bits, group):
    B = (1 << bits) - 1
    xg = x.reshape(-1, group).astype(np.float64)
    mn = xg.min(axis=1, keepdims=True)
    R = xg.max(axis=1, keepdims=True) - mn
    xb = (xg - mn) / R * B
    p = xb - np.floor(xb)
    return p.reshape(x.shape), np.broadcast_to(R / B, xg.shape).reshape(x.shape)


@pytest.mark.parametrize("bits,group", [(2, 64), (4, 64), (8, 64), (1, 64), (2, 32), (4, 128)])
def test_unbiased_with_exact_variance(bits, group):
    S = 10000
    x = gen.normal_activations(64, 64, seed=2)
    mean, var = _moments(x, bits, group, S)
    p, scale = _frac_and_scale(x, bits, group)
    var_exact = scale ** 2 * p * (1 - p)          # appendix: Var[SR(x)] = p - p^2
    inner = (p > 1e-3) & (p < 1 - 1e-3)
    z = (mean - x.astype(np.float64))[inner] / np.sqrt(var_exact[inner] / S)
    # E[Dequant(Quant(e))] = e  (Eq. 5): standardised errors behave like N(0,1)
    assert np.abs(z).max() < 6.0
    frac3 = np.mean(np.abs(z) > 3.0)
    assert 0.0003 < frac3 < 0.008
    assert 0.9 < np.mean(z * z) < 1.1
    assert abs(z.mean()) < 5.0 / np.sqrt(z.size) + 0.02
    # Var per element equals scale^2 p (1-p) and never exceeds scale^2 / 4
    rel = var[inner] / var_exact[inner]
    assert 0.97 < rel.mean() < 1.03
    assert np.all(var <= scale ** 2 / 4 * (1 + 1e-4) + 1e-30)   # slack: fp32 rounding of scale and of e_hat
    # vector bound of Proposition 1: sum_i Var <= d R^2 / (4 B^2) per group
    vg = var.reshape(-1, group).sum(axis=1)
    bound = group * scale.reshape(-1, group)[:, 0] ** 2 / 4
    assert np.all(vg <= bound * (1 + 1e-4))
    # elements where the draw cannot matter (p = 0) are reproduced exactly
    assert np.all(np.abs(var[p == 0]) < 1e-9)      # up to cancellation in s2/S - mean^2


def test_probability_of_rounding_up_by_enumeration():
    # brute force on one element: over many seeds the up-frequency at a known
    # fractional part p matches p; built on a dyadic group so p is exact.
    bits, B = 2, 3
    group = 64
    x = np.zeros((1, group), dtype=np.float32)
    x[0, 1] = 3.0                                    # min 0, max 3 -> scale 1, inv 1
    fracs = [0.125, 0.25, 0.5, 0.75, 0.9375]
    for j, f in enumerate(fracs):
        x[0, 2 + j] = 1.0 + f
    S = 20000
    ups = np.zeros(len(fracs))
    for seed in range(S):
        codes, _, _ = ref.quantize_codes(x, bits, group, seed)
        c = codes[2:2 + len(fracs)].astype(int)
        assert np.all((c == 1) | (c == 2))
        ups += (c == 2)
    for f, u in zip(fracs, ups):
        assert abs(u / S - f) < 5 * np.sqrt(f * (1 - f) / S)


def test_bf16_widening_matches_the_library_conversion():
    # the oracle's bfloat16 path = fp32 quantizer on exactly widened values; the widening is
    # pinned against torch's own bfloat16 -> float32 conversion on every finite bit pattern
    torch = pytest.importorskip("torch")
    bits16 = np.arange(65536, dtype=np.uint16)
    wide = ref.widen_bf16(bits16)
    t = torch.from_numpy(bits16.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    finite = np.isfinite(t)
    assert np.array_equal(wide[finite].view(np.uint32), t[finite].view(np.uint32))
    x = wide[finite][::15][:4096].reshape(64, 64)
    x = np.clip(x, -1e30, 1e30).astype(np.float32)
    xb = (x.view(np.uint32) >> 16).astype(np.uint16)
    a = ref.quantize_bf16(xb, 2, 64, 5)
    b = ref.quantize(ref.widen_bf16(xb), 2, 64, 5)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
