"""Pins of the BatchNorm and max-pooling (SPMM_MAX) oracles in oracle/ref.py -- the two
other operators Sec. 4.1.4 names as carrying a compressed context -- against things other
than themselves: torch's own routines, plain loops, closed forms, finite differences and
Proposition 1."""
import numpy as np
import pytest

from oracle import ref

torch = pytest.importorskip("torch")


# ------------------------------------------------------------------ BatchNorm
def bn_problem(n=37, d=8, seed=0, shift=3.0):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((n, d)) * rng.uniform(0.5, 2.0, d) + shift * rng.standard_normal(d)).astype(np.float32)
    gamma = rng.uniform(0.5, 1.5, d).astype(np.float32)
    beta = rng.standard_normal(d).astype(np.float32)
    g = rng.standard_normal((n, d)).astype(np.float32)
    return x, gamma, beta, g


def test_batchnorm_matches_torch_forward_and_autograd():
    x, gamma, beta, g = bn_problem()
    eps = 1e-5
    y, mu, rstd = ref.batchnorm_fwd(x, gamma, beta, eps)
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tg = torch.tensor(gamma, dtype=torch.float64, requires_grad=True)
    tb = torch.tensor(beta, dtype=torch.float64, requires_grad=True)
    ty = torch.nn.functional.batch_norm(tx, None, None, tg, tb, training=True, eps=eps)
    assert np.allclose(y, ty.detach().numpy(), rtol=1e-6, atol=1e-6)
    ty.backward(torch.tensor(g, dtype=torch.float64))
    gx, gg, gb = ref.batchnorm_bwd(x, mu.astype(np.float64), rstd.astype(np.float64), gamma, g)
    # (mu, rstd were rounded to fp32 on the way out: 1e-6 relative)
    assert np.allclose(gx, tx.grad.numpy(), rtol=2e-5, atol=2e-6)
    assert np.allclose(gg, tg.grad.numpy(), rtol=2e-5, atol=2e-5)
    assert np.allclose(gb, tb.grad.numpy(), rtol=1e-6, atol=1e-6)


def test_batchnorm_closed_forms():
    x, gamma, beta, g = bn_problem(n=64, seed=1)
    eps = 1e-3
    y, mu, rstd = ref.batchnorm_fwd(x, gamma, beta, eps)
    x64 = x.astype(np.float64)
    var = x64.var(axis=0)
    assert np.allclose(mu, x64.mean(axis=0), rtol=1e-6)
    assert np.allclose(y.astype(np.float64).mean(axis=0), beta, atol=1e-6)
    assert np.allclose(y.astype(np.float64).std(axis=0), gamma * np.sqrt(var / (var + eps)), rtol=1e-5)
    # a constant column: y = beta, rstd = eps^-1/2
    x[:, 2] = 1.25
    y, mu, rstd = ref.batchnorm_fwd(x, gamma, beta, eps)
    assert np.array_equal(y[:, 2], np.full(64, beta[2], np.float32)) and mu[2] == 1.25
    assert np.isclose(rstd[2], eps ** -0.5, rtol=1e-6)


def test_batchnorm_backward_by_finite_differences_and_loops():
    x, gamma, beta, g = bn_problem(n=11, d=3, seed=2)
    eps = 1e-2
    x64 = x.astype(np.float64)

    def loss(xx, ga, be):
        mu = xx.mean(axis=0); var = xx.var(axis=0)
        return float(np.sum(g * (ga * (xx - mu) / np.sqrt(var + eps) + be)))

    y, mu, rstd = ref.batchnorm_fwd(x, gamma, beta, eps)
    mu64 = x64.mean(axis=0); rstd64 = 1 / np.sqrt(x64.var(axis=0) + eps)
    gx, gg, gb = ref.batchnorm_bwd(x, mu64, rstd64, gamma, g)
    h = 1e-6
    for idx in [(0, 0), (5, 1), (10, 2)]:
        up = x64.copy(); up[idx] += h
        dn = x64.copy(); dn[idx] -= h
        fd = (loss(up, gamma, beta) - loss(dn, gamma, beta)) / (2 * h)
        assert abs(fd - gx[idx]) <= 1e-6 * max(1.0, abs(fd))
    for c in range(3):
        e = np.zeros(3); e[c] = h
        assert abs((loss(x64, gamma + e, beta) - loss(x64, gamma - e, beta)) / (2 * h) - gg[c]) <= 1e-6 * max(1, abs(gg[c]))
        assert abs((loss(x64, gamma, beta + e) - loss(x64, gamma, beta - e)) / (2 * h) - gb[c]) <= 1e-6 * max(1, abs(gb[c]))
    # the saved tensors are what is used: arbitrary x_hat, mu, rstd, explicit loops
    rng = np.random.default_rng(3)
    xh = x64 + 0.1 * rng.standard_normal(x.shape)
    m2 = rng.standard_normal(3); r2 = rng.uniform(0.5, 2, 3)
    gx, gg, gb = ref.batchnorm_bwd(xh, m2, r2, gamma, g)
    n = x.shape[0]
    for c in range(3):
        sb = sum(float(g[i, c]) for i in range(n))
        sg = sum(float(g[i, c]) * (xh[i, c] - m2[c]) * r2[c] for i in range(n))
        assert np.isclose(gb[c], sb, rtol=1e-6) and np.isclose(gg[c], sg, rtol=1e-6, atol=1e-6)
        for i in range(n):
            xb = (xh[i, c] - m2[c]) * r2[c]
            want = float(gamma[c]) * r2[c] * (float(g[i, c]) - sb / n - xb * sg / n)
            assert np.isclose(gx[i, c], want, rtol=1e-5, atol=1e-6)


def test_batchnorm_gamma_gradient_is_unbiased_under_the_compressed_context():
    # grad_gamma is linear in x_hat, so Proposition 1 carries over: its mean over seeds is the
    # exact value and its variance is at most sum_n (g rstd)^2 scale^2 / 4
    n, d, bits, group = 64, 32, 2, 64
    x, gamma, beta, g = bn_problem(n=n, d=d, seed=4, shift=0.5)
    y, mu, rstd = ref.batchnorm_fwd(x, gamma, beta, 1e-5)
    exact = ref.batchnorm_bwd(x, mu, rstd, gamma, g)[1].astype(np.float64)
    S = 400
    acc = np.zeros(d); acc2 = np.zeros(d)
    for s in range(S):
        p, mn, sc = ref.quantize(x, bits, group, seed=1000 + s)
        xh = ref.dequantize(p, mn, sc, n, d, bits, group)
        gg = ref.batchnorm_bwd(xh, mu, rstd, gamma, g)[1].astype(np.float64)
        acc += gg; acc2 += gg * gg
    mean = acc / S
    _, _, sc = ref.quantize(x, bits, group, seed=0)
    scale_el = np.repeat(sc, group).reshape(n, d).astype(np.float64)
    bound = ((g.astype(np.float64) * rstd) ** 2 * scale_el ** 2 / 4).sum(axis=0)
    z = (mean - exact) / np.sqrt(bound / S)
    assert np.max(np.abs(z)) < 5.0
    var = acc2 / S - mean ** 2
    assert np.all(var <= bound * 1.25)


# ------------------------------------------------------------------ SPMM_MAX
def max_problem(n=12, r=3, t=40, d=6, seed=0):
    rng = np.random.default_rng(seed)
    head = rng.integers(0, n - 2, t).astype(np.int32)       # the last two nodes have no out-edges
    rel = rng.integers(0, r, t).astype(np.int32)
    tail = rng.integers(0, n, t).astype(np.int32)
    tail[0] = head[0]                                       # self-loop
    head[2], rel[2], tail[2] = head[1], rel[1], tail[1]     # repeated triplet (an exact tie)
    E = rng.standard_normal((n, d)).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    return head, rel, tail, E, G


def test_spmm_max_by_loops_with_ties():
    n, d = 12, 6
    head, rel, tail, E, G = max_problem(n=n, d=d)
    E[3, :] = E[7, :]                                       # two different tails with equal rows
    E[:, 4] = 0.5                                           # a whole column of ties
    M, arg = ref.spmm_max_fwd(n, head, rel, tail, E)
    # the head's out-edges in (relation, tail, input position) order, by plain sorting
    want_M = np.zeros((n, d), np.float32); want_arg = np.zeros((n, d), np.int64)
    gE = np.zeros((n, d))
    for h in range(n):
        edges = sorted((int(rel[i]), int(tail[i]), i) for i in range(head.size) if head[i] == h)
        for c in range(d):
            best = None
            for j, (_, t, _) in enumerate(edges):
                if best is None or E[t, c] > E[edges[best][1], c]:
                    best = j
            if best is not None:
                want_M[h, c] = E[edges[best][1], c]; want_arg[h, c] = best
                gE[edges[best][1], c] += float(G[h, c])
    assert np.array_equal(M.view(np.uint32), want_M.view(np.uint32))
    assert np.array_equal(arg, want_arg)
    got = ref.spmm_max_bwd(n, head, rel, tail, arg, G)
    assert np.allclose(got, gE, rtol=1e-6, atol=1e-7)
    assert np.all(M[n - 2:] == 0) and np.all(arg[n - 2:] == 0)


def test_spmm_max_matches_torch_scatter_amax_and_its_gradient():
    n, d = 50, 8
    head, rel, tail, E, G = max_problem(n=n, r=4, t=300, d=d, seed=1)
    keep = np.ones(head.size, bool); keep[2] = False        # no exact ties: torch splits them evenly
    head, rel, tail = head[keep], rel[keep], tail[keep]
    tE = torch.tensor(E, dtype=torch.float64, requires_grad=True)
    idx = torch.tensor(head.astype(np.int64))[:, None].expand(-1, d)
    out = torch.zeros((n, d), dtype=torch.float64).scatter_reduce(0, idx, tE[torch.tensor(tail.astype(np.int64))],
                                                                  reduce="amax", include_self=False)
    M, arg = ref.spmm_max_fwd(n, head, rel, tail, E)
    assert np.array_equal(M.astype(np.float64), out.detach().numpy())
    out.backward(torch.tensor(G, dtype=torch.float64))
    got = ref.spmm_max_bwd(n, head, rel, tail, arg, G)
    assert np.allclose(got, tE.grad.numpy(), rtol=1e-6, atol=1e-7)


def test_spmm_max_ring_graph_and_conservation():
    n, d = 9, 4
    rng = np.random.default_rng(2)
    E = rng.standard_normal((n, d)).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    head = np.arange(n, dtype=np.int32); tail = ((head + 1) % n).astype(np.int32); rel = np.zeros(n, np.int32)
    M, arg = ref.spmm_max_fwd(n, head, rel, tail, E)
    assert np.array_equal(M, np.roll(E, -1, axis=0)) and not arg.any()
    assert np.array_equal(ref.spmm_max_bwd(n, head, rel, tail, arg, G), np.roll(G, 1, axis=0))
    # every head with an out-edge passes each of its gradient entries to exactly one tail
    head, rel, tail, E, G = max_problem(seed=5)
    M, arg = ref.spmm_max_fwd(12, head, rel, tail, E)
    gE = ref.spmm_max_bwd(12, head, rel, tail, arg, G)
    has = np.bincount(head, minlength=12) > 0
    assert np.allclose(gE.sum(axis=0), G[has].astype(np.float64).sum(axis=0), atol=1e-5)
