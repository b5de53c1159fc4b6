"""Pins of the uniform-attention oracle (oracle/ref.py: uniform_fwd / uniform_bwd),
Eq. (2) with the row-normalised adjacency: checked against things other than itself."""
import numpy as np

from oracle import ref
from workloads import gen

SLOPE = np.float32(0.2)


def small_graph(n=10, r=3, t=37, seed=0):
    rng = np.random.default_rng(seed)
    head = rng.integers(0, n - 2, t).astype(np.int32)      # the last two nodes have no out-edges
    rel = rng.integers(0, r, t).astype(np.int32)
    tail = rng.integers(0, n, t).astype(np.int32)
    tail[:3] = head[:3]                                     # self-loops
    head[5], rel[5], tail[5] = head[4], rel[4], tail[4]     # a repeated triplet
    return head, rel, tail


def test_brute_force_dense_loops():
    # plain loops over a dense N x N count matrix, written separately from the CSR oracle
    n, d, dout = 10, 8, 6
    head, rel, tail = small_graph(n)
    rng = np.random.default_rng(1)
    E = rng.normal(size=(n, d)).astype(np.float32)
    W = rng.normal(size=(dout, d)).astype(np.float32)
    G = rng.normal(size=(n, dout)).astype(np.float32)
    cnt = np.zeros((n, n))
    for h, t in zip(head, tail):
        cnt[h, t] += 1
    H = np.zeros((n, d))
    for h in range(n):
        deg = cnt[h].sum()
        for k in range(d):
            acc = float(E[h, k])
            for t in range(n):
                if cnt[h, t]:
                    acc += cnt[h, t] / deg * float(E[t, k])
            H[h, k] = acc
    J = np.zeros((n, dout))
    for h in range(n):
        for o in range(dout):
            J[h, o] = sum(H[h, k] * float(W[o, k]) for k in range(d))
    want = np.where(J > 0, J, float(SLOPE) * J)
    Eo, Hh, mask = ref.uniform_fwd(n, head, tail, E, W, SLOPE)
    assert np.allclose(Eo, want, rtol=1e-6, atol=1e-7) and np.allclose(Hh, H, rtol=1e-6, atol=1e-7)
    assert np.array_equal(mask != 0, J > 0)
    # backward by loops, at the exact context
    gJ = G.astype(np.float64) * np.where(J > 0, 1.0, float(SLOPE))
    gH = np.zeros((n, d)); gW = np.zeros((dout, d))
    for h in range(n):
        for k in range(d):
            gH[h, k] = sum(gJ[h, o] * float(W[o, k]) for o in range(dout))
    for o in range(dout):
        for k in range(d):
            gW[o, k] = sum(gJ[h, o] * H[h, k] for h in range(n))
    gE = gH.copy()
    for h in range(n):
        deg = cnt[h].sum()
        for t in range(n):
            if cnt[h, t]:
                gE[t] += cnt[h, t] / deg * gH[h]
    got_gE, got_gW = ref.uniform_bwd(n, head, tail, H, mask, W, SLOPE, G)
    assert np.allclose(got_gE, gE, rtol=1e-6, atol=1e-6) and np.allclose(got_gW, gW, rtol=1e-6, atol=1e-6)


def test_equals_attentive_oracle_with_zero_projections():
    # W_r = 0, e_r = 0 makes every score 0 and the softmax uniform: the attentive oracle (C++,
    # a separate implementation) must give the same layer, forward and backward
    n, r, t, d, dout = 300, 4, 2500, 32, 16
    head, rel, tail = gen.kg_triplets(n, r, t, seed=3, tail_zipf=1.1)
    E = gen.entity_embeddings(n, d, seed=4)
    _, _, W = gen.layer_params(r, d, d, dout, seed=5)
    Wr0 = np.zeros((r, d, d), np.float32); er0 = np.zeros((r, d), np.float32)
    G = gen.upstream_grad(n, dout, seed=6)
    Eo, H, mask = ref.uniform_fwd(n, head, tail, E, W, SLOPE)
    aEo, aH, amask = ref.aggregate_fwd(n, head, rel, tail, E, Wr0, er0, W, float(SLOPE))
    assert np.allclose(Eo, aEo, rtol=2e-6, atol=1e-7) and np.allclose(H, aH, rtol=2e-6, atol=1e-7)
    assert np.array_equal(mask != 0, amask != 0)
    gE, gW = ref.uniform_bwd(n, head, tail, H, mask, W, SLOPE, G)
    aE, aWr, aer, aW = ref.aggregate_bwd(n, head, rel, tail, E, H, mask, Wr0, er0, W, float(SLOPE), G)
    assert np.allclose(gE, aE, rtol=2e-6, atol=1e-6) and np.allclose(gW, aW, rtol=2e-6, atol=1e-6)
    assert not aWr.any() or np.abs(aWr).max() < 1e-30      # nothing flows into W_r when a = 0, tanh(b) = 0


def test_backward_is_the_gradient_by_finite_differences():
    n, d, dout = 12, 6, 5
    head, rel, tail = small_graph(n, seed=7)
    rng = np.random.default_rng(8)
    E = rng.normal(size=(n, d)); W = rng.normal(size=(dout, d)); G = rng.normal(size=(n, dout))
    A = ref._uniform_adjacency(n, head, tail).toarray()

    def loss(E_, W_):
        J = (E_ + A @ E_) @ W_.T
        return float(np.sum(G * np.where(J > 0, J, 0.2 * J)))

    J0 = (E + A @ E) @ W.T
    gE, gW = ref.uniform_bwd(n, head, tail, E + A @ E, (J0 > 0), W, 0.2, G)
    eps = 1e-6
    for (i, k) in [(0, 0), (3, 2), (11, 5), (7, 1)]:
        Ep = E.copy(); Ep[i, k] += eps; Em = E.copy(); Em[i, k] -= eps
        assert abs((loss(Ep, W) - loss(Em, W)) / (2 * eps) - gE[i, k]) < 2e-4 * max(1, abs(gE[i, k]))
    for (o, k) in [(0, 0), (4, 5), (2, 3)]:
        Wp = W.copy(); Wp[o, k] += eps; Wm = W.copy(); Wm[o, k] -= eps
        assert abs((loss(E, Wp) - loss(E, Wm)) / (2 * eps) - gW[o, k]) < 2e-4 * max(1, abs(gW[o, k]))


def test_closed_forms():
    # a ring i -> i+1: H_i = e_i + e_{i+1}; grad_E_i = grad_H_i + grad_H_{i-1}
    n, d = 7, 4
    head = np.arange(n, dtype=np.int32); tail = ((head + 1) % n).astype(np.int32)
    rng = np.random.default_rng(9)
    E = rng.normal(size=(n, d)).astype(np.float32)
    W = np.eye(d, dtype=np.float32)
    _, H, mask = ref.uniform_fwd(n, head, tail, E, W, 1.0)           # slope 1: the activation is the identity
    assert np.allclose(H, E + np.roll(E, -1, axis=0), rtol=1e-6, atol=1e-7)
    G = rng.normal(size=(n, d)).astype(np.float32)
    gE, gW = ref.uniform_bwd(n, head, tail, H, mask, W, 1.0, G)
    assert np.allclose(gE, G + np.roll(G, 1, axis=0), rtol=1e-6, atol=1e-6)
    assert np.allclose(gW, G.astype(np.float64).T @ H.astype(np.float64), rtol=1e-6, atol=1e-6)
    # no edges at all: H = E, grad_E = grad_H
    none = np.zeros(0, np.int32)
    _, H0, m0 = ref.uniform_fwd(n, none, none, E, W, 1.0)
    assert np.array_equal(H0, E)
    g0, _ = ref.uniform_bwd(n, none, none, H0, m0, W, 1.0, G)
    assert np.allclose(g0, G)
