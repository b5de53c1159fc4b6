"""GPU parity: the HIP quantizer / dequantizer against the CPU oracle, through
the C ABI.  Packed codes, per-group min and scale must be bit-exact; dequantised
values are a single fma of exact inputs, so they are compared bit-exactly too
(the bar is 1e-5 relative)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ref
from workloads import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tk():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2212_04540_amd as tk
    tk.lib()
    return tk


def gpu_quant(tk, x, bits, group, seed, **kw):
    xt = torch.from_numpy(x).cuda()
    p, mn, sc = tk.tinykg_quantize(xt, bits, group, seed, **kw)
    torch.cuda.synchronize()
    return p.cpu().numpy(), mn.cpu().numpy(), sc.cpu().numpy()


def assert_same(got, want, what):
    gp, gm, gs = got
    wp, wm, ws = want
    assert np.array_equal(gm.view(np.uint32), wm.view(np.uint32)), f"{what}: gmin differs"
    assert np.array_equal(gs.view(np.uint32), ws.view(np.uint32)), f"{what}: gscale differs"
    if not np.array_equal(gp, wp):
        bad = np.nonzero(gp != wp)[0]
        raise AssertionError(f"{what}: {bad.size} packed bytes differ, first at {bad[0]}: "
                             f"{gp[bad[0]]:#x} vs {wp[bad[0]]:#x}")


def test_config0_standalone_compressor(tk):
    # 4096 x 64 fp32 N(0,1) seed 0, one row per group, INT2, Philox seed 1
    x = gen.normal_activations(4096, 64, seed=0)
    got = gpu_quant(tk, x, 2, 64, 1)
    want = ref.quantize(x, 2, 64, 1)
    assert got[0].size == 4096 * 16
    assert_same(got, want, "config0")
    out = tk.tinykg_dequantize(*[torch.from_numpy(a).cuda() for a in got], 4096, 64, 2, 64)
    torch.cuda.synchronize()
    want_x = ref.dequantize(*want, 4096, 64, 2, 64)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), want_x.view(np.uint32))
    # compression ratio of this configuration: 0.375 B per activation
    assert (got[0].nbytes + got[1].nbytes + got[2].nbytes) / x.size == 0.375


@pytest.mark.parametrize("bits", [1, 2, 4, 8])
@pytest.mark.parametrize("group", [32, 64, 128, 256])
def test_all_bits_and_groups_ragged(tk, bits, group):
    # several tiles (1024 elements each) plus a ragged tail; heavy-tailed values
    rows = 16 * 37 + 4            # 596 rows x 64 = 38144 elements: 37 tiles + 256
    x = gen.student_t_activations(rows, 64, seed=bits * 10 + group)
    seed = 0x1234_5678_9ABC_DEF0 + bits
    got = gpu_quant(tk, x, bits, group, seed)
    want = ref.quantize(x, bits, group, seed)
    assert_same(got, want, f"b{bits} g{group}")
    out = tk.tinykg_dequantize(*[torch.from_numpy(a).cuda() for a in got], rows, 64, bits, group)
    want_x = ref.dequantize(*want, rows, 64, bits, group)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), want_x.view(np.uint32))
    err = np.abs(out.cpu().numpy().astype(np.float64) - x).reshape(-1, group)
    assert np.all(err <= want[2].astype(np.float64)[:, None] * (1 + 2.0 ** -20))


@pytest.mark.parametrize("shape", [(1, 32), (1, 64), (2, 64), (3, 32), (5, 256), (17, 64), (1, 1024),
                                   (1, 1056), (33, 32), (1000, 16)])
def test_tiny_and_odd_shapes(tk, shape):
    rows, dim = shape
    x = gen.normal_activations(rows, dim, seed=rows * 1000 + dim)
    for bits, group in [(2, 32), (4, 32), (8, 32), (1, 32)]:
        if (rows * dim) % group:
            continue
        assert_same(gpu_quant(tk, x, bits, group, 7), ref.quantize(x, bits, group, 7), str(shape))


def test_empty_input_is_ok(tk):
    x = torch.empty((0, 64), dtype=torch.float32, device="cuda")
    p, mn, sc = tk.tinykg_quantize(x, 2, 64, 0)
    assert p.numel() == 0 and mn.numel() == 0
    out = tk.tinykg_dequantize(p, mn, sc, 0, 64, 2, 64)
    assert out.numel() == 0


def test_shape_error_raises(tk):
    x = torch.zeros((3, 50), dtype=torch.float32, device="cuda")
    with pytest.raises(tk.TinyKGError) as e:
        tk.tinykg_quantize(x, 2, 64, 0, out=tk.alloc_quantized(4, 64, 2, 64))
    assert e.value.status == 2


def test_special_groups(tk):
    # constant, all -0, mixed zeros, denormal range, tiny normal range, huge values,
    # exact dyadic grid, and a group whose max*inv falls below B
    x = np.zeros((8, 64), dtype=np.float32)
    x[0] = 2.5
    x[1] = -0.0
    x[2, ::2] = -0.0
    x[3] = np.float32(1e-40) * np.arange(64, dtype=np.float32)
    x[4] = np.float32(1e-36) * np.arange(64, dtype=np.float32) / 63
    x[5] = np.linspace(-8e37, 8e37, 64, dtype=np.float32)
    x[6] = -7.0 + (np.arange(64) % 4).astype(np.float32) * 0.5
    x[7] = np.linspace(0.1, 0.7, 64, dtype=np.float32)
    for bits in (1, 2, 4, 8):
        for seed in range(3):
            got = gpu_quant(tk, x, bits, 64, seed)
            want = ref.quantize(x, bits, 64, seed)
            assert_same(got, want, f"special b{bits}")
            out = tk.tinykg_dequantize(*[torch.from_numpy(a).cuda() for a in got], 8, 64, bits, 64)
            want_x = ref.dequantize(*want, 8, 64, bits, 64)
            assert np.array_equal(out.cpu().numpy().view(np.uint32), want_x.view(np.uint32))


def test_correctly_rounded_divides(tk):
    # R/B and B/R must be IEEE-correct on the GPU: many random ranges, one group each,
    # min 0 so that range == max exactly; scale is compared bit for bit and the codes
    # of mid-range elements depend on every bit of B/R.
    rng = np.random.default_rng(3)
    rows = 1 << 14
    x = np.zeros((rows, 32), dtype=np.float32)
    mx = np.exp(rng.uniform(np.log(1e-30), np.log(1e30), size=rows)).astype(np.float32)
    x[:, 1] = mx
    x[:, 2:] = (rng.random((rows, 30)) * mx[:, None]).astype(np.float32)
    for bits in (2, 4, 8):
        assert_same(gpu_quant(tk, x, bits, 32, 5), ref.quantize(x, bits, 32, 5), f"divide b{bits}")


def test_first_index_and_nearest_rounding(tk):
    x = gen.normal_activations(512, 64, seed=4)
    full = ref.quantize(x, 4, 128, 99)
    r0, r1 = 128, 384
    got = gpu_quant(tk, x[r0:r1], 4, 128, 99, first_index=r0 * 64)
    assert np.array_equal(got[0], full[0][r0 * 64 // 2:r1 * 64 // 2])
    # huge offsets: the 64-bit counter carries into its high word
    off = (1 << 35) + 1024
    assert_same(gpu_quant(tk, x, 2, 64, 3, first_index=off), ref.quantize(x, 2, 64, 3, first_index=off),
                "offset")
    for bits in (1, 2, 4, 8):
        assert_same(gpu_quant(tk, x, bits, 64, 0, rounding=1), ref.quantize(x, bits, 64, 0, rounding=1),
                    f"nearest b{bits}")


def test_deterministic_across_launches(tk):
    x = torch.from_numpy(gen.student_t_activations(3000, 64, seed=8)).cuda()
    a = tk.tinykg_quantize(x, 2, 64, 42)
    b = tk.tinykg_quantize(x, 2, 64, 42)
    c = tk.tinykg_quantize(x, 2, 64, 43)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])
    assert not torch.equal(a[0], c[0])


def test_gpu_unbiased_with_closed_form_variance(tk):
    # Proposition 1 measured on the GPU path itself: 2000 seeds, INT2, group 64
    x = gen.normal_activations(64, 64, seed=2)
    xt = torch.from_numpy(x).cuda()
    S = 2000
    s1 = torch.zeros_like(xt, dtype=torch.float64)
    s2 = torch.zeros_like(xt, dtype=torch.float64)
    buf = tk.alloc_quantized(64, 64, 2, 64)
    out = torch.empty_like(xt)
    for seed in range(S):
        tk.tinykg_quantize(xt, 2, 64, seed, out=buf)
        tk.tinykg_dequantize(*buf, 64, 64, 2, 64, out=out)
        s1 += out
        s2 += out.double() ** 2
    mean = (s1 / S).cpu().numpy()
    var = (s2 / S).cpu().numpy() - mean ** 2
    xg = x.astype(np.float64)
    mn = xg.min(axis=1, keepdims=True)
    R = xg.max(axis=1, keepdims=True) - mn
    xb = (xg - mn) / R * 3
    p = xb - np.floor(xb)
    var_exact = (R / 3) ** 2 * p * (1 - p)
    inner = (p > 1e-3) & (p < 1 - 1e-3)
    z = (mean - xg)[inner] / np.sqrt(var_exact[inner] / S)
    assert np.abs(z).max() < 6 and 0.85 < np.mean(z * z) < 1.15
    assert 0.95 < (var[inner] / var_exact[inner]).mean() < 1.05
    assert np.all(var <= (R / 3) ** 2 / 4 * (1 + 1e-4))


def test_large_tensor_sampled_rows(tk):
    # a size that needs the grid-stride loop (more tiles than resident waves):
    # 2^20 rows x 64 (256 MiB); the oracle checks sampled slices via first_index
    rows, dim = 1 << 20, 64
    g = torch.Generator(device="cuda"); g.manual_seed(0)
    z = torch.randn((rows, dim), generator=g, device="cuda")
    chi = torch.randn((rows, dim, 3), generator=g, device="cuda").square_().sum(-1)
    x = (z / (chi / 3).sqrt_()).contiguous()           # Student-t, nu = 3 (inputs only)
    del z, chi
    for bits, group in [(2, 64), (4, 128), (8, 256), (2, 32)]:
        p, mn, sc = tk.tinykg_quantize(x, bits, group, 1)
        torch.cuda.synchronize()
        for r0 in (0, 4096 * 3, rows // 2 + 16, rows - 64):
            r1 = r0 + 64
            xs = x[r0:r1].cpu().numpy()
            wp, wm, ws = ref.quantize(xs, bits, group, 1, first_index=r0 * dim)
            b0, b1 = r0 * dim * bits // 8, r1 * dim * bits // 8
            g0, g1 = r0 * dim // group, r1 * dim // group
            assert np.array_equal(p[b0:b1].cpu().numpy(), wp)
            assert np.array_equal(mn[g0:g1].cpu().numpy().view(np.uint32), wm.view(np.uint32))
            assert np.array_equal(sc[g0:g1].cpu().numpy().view(np.uint32), ws.view(np.uint32))
        out = tk.tinykg_dequantize(p, mn, sc, rows, dim, bits, group)
        r0 = rows - 128
        want = ref.dequantize(p[r0 * dim * bits // 8:].cpu().numpy(), mn[r0 * dim // group:].cpu().numpy(),
                              sc[r0 * dim // group:].cpu().numpy(), 128, dim, bits, group)
        assert np.array_equal(out[r0:].cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_config2_full_size_sweep(tk):
    # configs[2] at its full size (2^23 x 64 fp32, 2 GiB, Student-t nu = 3) in the launch
    # configuration bench.py times, all nine cells bits x group: the oracle checks sampled
    # row slices (quantizer bit-exact via first_index, dequantizer bit-exact on the GPU's own
    # bytes); per-element variance over 64 seeds on the first 4096 rows against Proposition 1
    # (closed form scale^2 p (1 - p) evaluated from the ORACLE's min / scale, bound scale^2 / 4).
    rows, dim = 1 << 23, 64
    g = torch.Generator(device="cuda"); g.manual_seed(0)
    x = torch.empty((rows, dim), dtype=torch.float32, device="cuda")
    step = 1 << 20
    for r0 in range(0, rows, step):
        z = torch.randn((step, dim), generator=g, device="cuda")
        chi = torch.randn((step, dim, 3), generator=g, device="cuda").square_().sum(-1)
        x[r0:r0 + step] = z / (chi / 3).sqrt_()
    del z, chi
    out = torch.empty_like(x)
    sub_rows = 4096
    xs_sub = x[:sub_rows].cpu().numpy()
    for bits in (2, 4, 8):
        B = (1 << bits) - 1
        for group in (32, 64, 256):
            p, mn, sc = tk.tinykg_quantize(x, bits, group, 1)
            tk.tinykg_dequantize(p, mn, sc, rows, dim, bits, group, out=out)
            torch.cuda.synchronize()
            for r0 in (0, 12345 * 4, rows // 2 + 8, rows - 64):
                r1 = r0 + 64
                xs = x[r0:r1].cpu().numpy()
                wp, wm, ws = ref.quantize(xs, bits, group, 1, first_index=r0 * dim)
                b0, b1 = r0 * dim * bits // 8, r1 * dim * bits // 8
                g0, g1 = r0 * dim // group, r1 * dim // group
                assert np.array_equal(p[b0:b1].cpu().numpy(), wp), (bits, group, r0)
                assert np.array_equal(mn[g0:g1].cpu().numpy().view(np.uint32), wm.view(np.uint32))
                assert np.array_equal(sc[g0:g1].cpu().numpy().view(np.uint32), ws.view(np.uint32))
                want = ref.dequantize(wp, wm, ws, 64, dim, bits, group)
                assert np.array_equal(out[r0:r1].cpu().numpy().view(np.uint32), want.view(np.uint32))
            del p, mn, sc
            # variance over 64 seeds on the subsample
            xt = x[:sub_rows].contiguous()
            S = 64
            s1 = torch.zeros((sub_rows, dim), dtype=torch.float64, device="cuda")
            s2 = torch.zeros_like(s1)
            buf = tk.alloc_quantized(sub_rows, dim, bits, group)
            o = torch.empty_like(xt)
            for seed in range(S):
                tk.tinykg_quantize(xt, bits, group, 100 + seed, out=buf)
                tk.tinykg_dequantize(*buf, sub_rows, dim, bits, group, out=o)
                s1 += o
                s2 += o.double() ** 2
            var = (s2 / S - (s1 / S) ** 2).cpu().numpy()
            _, wm, ws = ref.quantize(xs_sub, bits, group, 100)
            gmn = np.repeat(wm.astype(np.float64), group).reshape(sub_rows, dim)
            gsc = np.repeat(ws.astype(np.float64), group).reshape(sub_rows, dim)
            xb = np.clip((xs_sub.astype(np.float64) - gmn) / np.where(gsc > 0, gsc, 1.0), 0, B)
            pf = xb - np.floor(xb)
            closed = gsc ** 2 * pf * (1 - pf)
            # a two-point variable's population variance never exceeds a quarter of its step
            assert np.all(var <= gsc ** 2 / 4 * (1 + 1e-4) + 1e-30), (bits, group)
            ratio = var.sum() / closed.sum()
            assert 0.97 < ratio < 1.03, (bits, group, ratio)


def test_bf16_inputs_give_the_codes_of_the_widened_tensor(tk):
    # Sec. 4.1.4: half-precision activations.  The kernel widens bfloat16 exactly, so its
    # output must be byte for byte the oracle's on the widened values.
    g = torch.Generator(device="cuda"); g.manual_seed(3)
    for rows, dim, bits, group in [(4096, 64, 2, 64), (1000, 32, 4, 32), (333, 256, 8, 256), (7, 128, 1, 128),
                                   (5000, 64, 2, 256)]:
        xb = (torch.randn((rows, dim), generator=g, device="cuda") * 3).to(torch.bfloat16)
        got = tk.tinykg_quantize_bf16(xb, bits, group, 11)
        torch.cuda.synchronize()
        bits16 = xb.view(torch.int16).cpu().numpy().view(np.uint16)
        want = ref.quantize_bf16(bits16, bits, group, 11)
        assert_same(tuple(a.cpu().numpy() for a in got), want, f"bf16 {rows}x{dim} b{bits} g{group}")
        same = tk.tinykg_quantize(xb.float(), bits, group, 11)     # and of the fp32 kernel on the widened tensor
        assert all(torch.equal(a, b) for a, b in zip(got, same))
    # a slice of a long tensor: first_index, nearest rounding
    xb = torch.randn((1 << 16, 64), generator=g, device="cuda").to(torch.bfloat16)
    r0 = 4096 * 5
    got = tk.tinykg_quantize_bf16(xb[r0:r0 + 128].contiguous(), 2, 64, 3, first_index=r0 * 64, rounding=tk.ROUND_NEAREST)
    full = tk.tinykg_quantize_bf16(xb, 2, 64, 3, rounding=tk.ROUND_NEAREST)
    torch.cuda.synchronize()
    assert torch.equal(got[0], full[0][r0 * 16:(r0 + 128) * 16]) and torch.equal(got[1], full[1][r0:r0 + 128])
