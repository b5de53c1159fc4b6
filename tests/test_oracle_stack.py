"""Pins for the oracle's readout / ranking loss and its layer chaining (no GPU)."""
import numpy as np

from oracle import ref
from workloads import gen


def test_bpr_closed_forms():
    # all-zero embeddings: every score is 0, loss = log 2, coefficient = 1/(2 batch)
    layers = [np.zeros((6, 4)), np.zeros((6, 8))]
    u = np.array([0, 1, 2]); p = np.array([3, 4, 5]); n = np.array([5, 3, 4])
    loss, coef, grads = ref.bpr_loss_grad(layers, u, p, n)
    assert abs(loss - np.log(2.0)) < 1e-15 and np.allclose(coef, 1 / 6)
    assert all(np.all(g == 0) for g in grads)
    # one sample, hand-computed: z_u = (1, 2), z_pos = (3, 0), z_neg = (0, 1): y+ = 3, y- = 2
    layers = [np.array([[1.0], [3.0], [0.0]]), np.array([[2.0], [0.0], [1.0]])]
    loss, coef, grads = ref.bpr_loss_grad(layers, [0], [1], [2])
    assert abs(loss - np.log1p(np.exp(-1.0))) < 1e-15
    s = 1 / (1 + np.exp(1.0))
    assert abs(coef[0] - s) < 1e-15
    gZ = np.concatenate(grads, axis=1)
    assert np.allclose(gZ[0], s * (np.array([0, 1]) - np.array([3, 0])))
    assert np.allclose(gZ[1], -s * np.array([1, 2])) and np.allclose(gZ[2], s * np.array([1, 2]))


def test_bpr_gradient_matches_finite_differences():
    rng = np.random.default_rng(0)
    layers = [rng.standard_normal((20, 8)), rng.standard_normal((20, 4)), rng.standard_normal((20, 12))]
    u = rng.integers(0, 20, 30); p = rng.integers(0, 20, 30); n = rng.integers(0, 20, 30)
    u[1] = u[0]; p[3] = n[4]            # repeated ids, an item that is positive and negative
    loss, coef, grads = ref.bpr_loss_grad(layers, u, p, n)
    eps = 1e-6
    for l in range(3):
        for _ in range(25):
            i, j = rng.integers(0, 20), rng.integers(0, layers[l].shape[1])
            up = [a.copy() for a in layers]; up[l][i, j] += eps
            dn = [a.copy() for a in layers]; dn[l][i, j] -= eps
            fd = (ref.bpr_loss_grad(up, u, p, n)[0] - ref.bpr_loss_grad(dn, u, p, n)[0]) / (2 * eps)
            assert abs(fd - grads[l][i, j]) < 1e-8


def test_stack_step_is_the_chain_rule_of_its_parts():
    # with an uncompressed context (bits = 32) the step's gradient of the loss with respect
    # to E0 and to the first layer's W must match finite differences of the whole chain
    N, R, T = 24, 3, 80
    head, rel, tail = gen.kg_triplets(N, R, T, seed=1)
    dims = [32, 32, 16]
    rng = np.random.default_rng(2)
    E0 = (rng.standard_normal((N, 32)) * 0.5).astype(np.float32)
    params = [gen.layer_params(R, dims[l], dims[l], dims[l + 1], seed=10 + l) for l in range(2)]
    u = rng.integers(0, N, 16); p = rng.integers(0, N, 16); n = rng.integers(0, N, 16)
    out = ref.stack_step(N, head, rel, tail, E0, params, 0.2, 32, 64, 0, u, p, n)

    def loss_of(E0v, W0v):
        a = [E0v.astype(np.float64)]
        for l, (Wr, er, W) in enumerate(params):
            Wl = W0v if l == 0 else W
            a.append(ref.aggregate_fwd_f64(N, head, rel, tail, a[-1], Wr, er, Wl, float(np.float32(0.2)))[0])
        return ref.bpr_loss_grad(a, u, p, n)[0]

    eps = 1e-6
    W0 = params[0][2].astype(np.float64)
    for _ in range(12):
        i, j = rng.integers(0, N), rng.integers(0, 32)
        up = E0.astype(np.float64).copy(); up[i, j] += eps
        dn = E0.astype(np.float64).copy(); dn[i, j] -= eps
        fd = (loss_of(up, W0) - loss_of(dn, W0)) / (2 * eps)
        assert abs(fd - out["layer_grads"][0][i, j]) < 2e-5 * max(1.0, abs(fd)) + 2e-6
        i, j = rng.integers(0, 32), rng.integers(0, 32)
        up = W0.copy(); up[i, j] += eps
        dn = W0.copy(); dn[i, j] -= eps
        fd = (loss_of(E0.astype(np.float64), up) - loss_of(E0.astype(np.float64), dn)) / (2 * eps)
        assert abs(fd - out["param_grads"][0][2][i, j]) < 2e-5 * max(1.0, abs(fd)) + 2e-6
    # seeds: layer l saves Q(E; seed + 2l), Q(H; seed + 2l + 1)
    out2 = ref.stack_step(N, head, rel, tail, E0, params, 0.2, 2, 64, 7, u, p, n)
    pE, _, _ = ref.quantize(out2["acts"][1], 2, 64, 9)
    assert np.array_equal(out2["ctxs"][1]["packed_E"], pE)
