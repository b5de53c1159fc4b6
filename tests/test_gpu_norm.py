"""GPU parity of batch normalisation with a compressed input (Sec. 4.1.4 operator list)
against oracle/ref.py, through the C ABI.

Protocol: (1) y, mean, rstd against the float64 oracle (1e-5, tolerance of test_gpu_agg.py);
(2) Q(x) byte for byte the oracle quantizer's output on the same x; (3) backward: the oracle
starts from the bytes, means and inverse deviations the GPU saved, so both sides evaluate the
same formulas at identical inputs (1e-5)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ref
from parity import close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tk():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2212_04540_amd as tk
    tk.lib()
    return tk


def problem(rows, dim, seed=0, shift=1.0):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((rows, dim)) * rng.uniform(0.2, 3.0, dim) + shift * rng.standard_normal(dim)).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, dim).astype(np.float32)
    beta = rng.standard_normal(dim).astype(np.float32)
    g = rng.standard_normal((rows, dim)).astype(np.float32)
    return x, gamma, beta, g


def run_case(tk, x, gamma, beta, g, bits, group, eps=1e-5, seed=7):
    rows, dim = x.shape
    dev = "cuda"
    tx, tga, tbe, tg = (torch.from_numpy(a).to(dev) for a in (x, gamma, beta, g))
    ctx = tk.NormContext(rows, dim, bits, group)
    y = tk.tinykg_batchnorm_fwd(tx, tga, tbe, eps, bits, group, seed, ctx)
    torch.cuda.synchronize()
    wy, wmu, wrs = ref.batchnorm_fwd(x, gamma, beta, eps)
    close(y, wy, "y")
    mu, rs = ctx.mean.cpu().numpy(), ctx.rstd.cpu().numpy()
    assert np.allclose(mu, wmu, rtol=1e-6, atol=1e-6 * np.sqrt(np.mean(x.astype(np.float64) ** 2)))
    assert np.allclose(rs, wrs, rtol=2e-6)
    if bits == 32:
        xh = ctx.packed.cpu().numpy().view(np.float32).reshape(rows, dim)
        assert np.array_equal(xh.view(np.uint32), x.view(np.uint32))
    else:
        wp, wmn, wsc = ref.quantize(x, bits, group, seed)
        assert np.array_equal(ctx.packed.cpu().numpy(), wp), "Q(x) differs"
        assert np.array_equal(ctx.gmin.cpu().numpy().view(np.uint32), wmn.view(np.uint32))
        assert np.array_equal(ctx.gscale.cpu().numpy().view(np.uint32), wsc.view(np.uint32))
        xh = ref.dequantize(wp, wmn, wsc, rows, dim, bits, group)
    gx, gg, gb = tk.tinykg_batchnorm_bwd(ctx, tga, tg)
    torch.cuda.synchronize()
    wgx, wgg, wgb = ref.batchnorm_bwd(xh, mu, rs, gamma, g)
    close(gx, wgx, "grad_x")
    # the column sums have rows terms of size ~|g|: tolerance relative to their root-sum-square
    rss_b = np.sqrt((g.astype(np.float64) ** 2).sum(axis=0))
    xbar = (xh.astype(np.float64) - mu) * rs
    rss_g = np.sqrt(((g * xbar) ** 2).sum(axis=0))
    assert np.all(np.abs(gb.cpu().numpy() - wgb) <= 1e-5 * np.maximum(np.abs(wgb), rss_b))
    assert np.all(np.abs(gg.cpu().numpy() - wgg) <= 1e-5 * np.maximum(np.abs(wgg), rss_g))
    # determinism: a second call gives the same bytes
    gx2, gg2, gb2 = tk.tinykg_batchnorm_bwd(ctx, tga, tg)
    assert torch.equal(gx, gx2) and torch.equal(gg, gg2) and torch.equal(gb, gb2)
    return ctx


@pytest.mark.parametrize("rows,dim,bits,group", [
    (1000, 64, 2, 64), (4096, 64, 4, 128), (333 * 8, 48, 2, 32), (2048, 128, 8, 256), (64, 1024, 2, 64),
    (999 * 8, 4, 1, 32), (1600, 20, 2, 32), (5000, 64, 32, 64), (513, 256, 4, 32)])
def test_shapes_and_widths(tk, rows, dim, bits, group):
    run_case(tk, *problem(rows, dim, seed=rows + dim), bits, group)


def test_large_means_constant_column_and_single_row(tk):
    x, gamma, beta, g = problem(4096, 64, seed=3, shift=1000.0)     # |mean| >> std
    x[:, 5] = -2.5                                                  # constant column: var = 0
    run_case(tk, x, gamma, beta, g, 2, 64, eps=1e-3)
    x, gamma, beta, g = problem(1, 64, seed=4)                      # one row: var = 0 everywhere
    run_case(tk, x, gamma, beta, g, 2, 64, eps=1e-2)


def test_half_million_rows(tk):
    # 2^19 x 64 (several workgroups per column slab, partial sums across 2048 workgroups)
    run_case(tk, *problem(1 << 19, 64, seed=9), 2, 64)


def test_empty_and_error_paths(tk):
    assert tk.lib().tinykg_batchnorm_workspace_bytes(100, 6) == 0                      # dim % 4
    assert tk.lib().tinykg_batchnorm_workspace_bytes(100, 2048) == 0                   # dim > 1024
    ctx = tk.NormContext(64, 64, 2, 64)
    x = torch.zeros((64, 64), device="cuda"); ga = torch.ones(64, device="cuda"); be = torch.zeros(64, device="cuda")
    with pytest.raises(tk.TinyKGError) as e:
        tk.tinykg_batchnorm_fwd(x, ga, be, 1e-5, 3, 64, 0, ctx)
    assert e.value.status == 1                                                          # bits = 3
    small = tk.NormContext(64, 64, 2, 64)
    small.ws = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(tk.TinyKGError) as e:
        tk.tinykg_batchnorm_fwd(x, ga, be, 1e-5, 2, 64, 0, small)
    assert e.value.status == 4                                                          # workspace
    odd = tk.NormContext(3, 20, 2, 32)                                                  # 60 % 32 != 0
    with pytest.raises(tk.TinyKGError) as e:
        tk.tinykg_batchnorm_fwd(torch.zeros((3, 20), device="cuda"), torch.ones(20, device="cuda"),
                                torch.zeros(20, device="cuda"), 1e-5, 2, 32, 0, odd)
    assert e.value.status == 2                                                          # shape
    # rows == 0: nothing to do forward, zero parameter gradients backward
    empty = tk.NormContext(0, 64, 2, 64)
    tk.tinykg_batchnorm_fwd(torch.zeros((0, 64), device="cuda"), ga, be, 1e-5, 2, 64, 0, empty)
    gx, gg, gb = tk.tinykg_batchnorm_bwd(empty, ga, torch.zeros((0, 64), device="cuda"),
                                         out=(torch.zeros((0, 64), device="cuda"), torch.ones(64, device="cuda"),
                                              torch.ones(64, device="cuda")))
    torch.cuda.synchronize()
    assert not gg.any() and not gb.any()
