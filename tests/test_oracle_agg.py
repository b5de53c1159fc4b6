"""Pins for the CPU oracle's attentive aggregation layer (no GPU).

The oracle is checked against things fixed outside of it: a dense brute-force
evaluation of the layer written here with N x R x N loops, central finite
differences of that forward pass (for the backward formulas), the uniform
special case that reduces to the normalised-adjacency spmm of Eq. (2) (scipy),
and the layer identities grad_Theta = H^T grad_J, grad_E = A^T grad_H.
"""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import ref
from workloads import gen


def small_problem(N=10, R=3, T=24, d=8, k=8, dout=6, seed=0, scale=0.7):
    rng = np.random.default_rng(seed)
    head = rng.integers(0, N - 1, size=T).astype(np.int32)     # node N-1 has no out-edge
    rel = rng.integers(0, R, size=T).astype(np.int32)
    tail = rng.integers(0, N, size=T).astype(np.int32)
    head[1], rel[1], tail[1] = head[0], rel[0], tail[0]         # a repeated triplet
    tail[2] = head[2]                                           # a self-loop
    E = rng.standard_normal((N, d)) * scale
    Wr = rng.standard_normal((R, k, d)) * scale / np.sqrt(d)
    er = rng.standard_normal((R, k)) * 0.3
    W = rng.standard_normal((dout, d)) / np.sqrt(d)
    G = rng.standard_normal((N, dout))
    return dict(N=N, R=R, T=T, d=d, k=k, dout=dout, head=head, rel=rel, tail=tail, E=E, Wr=Wr,
                er=er, W=W, G=G, slope=0.2)


def dense_forward(P, E=None, Wr=None, er=None, W=None):
    """Brute force: multiplicity tensor M[h, r, t], loops over every (h, r, t)."""
    E = P["E"] if E is None else E
    Wr = P["Wr"] if Wr is None else Wr
    er = P["er"] if er is None else er
    W = P["W"] if W is None else W
    N, R = P["N"], P["R"]
    M = np.zeros((N, R, N), dtype=int)
    for h, r, t in zip(P["head"], P["rel"], P["tail"]):
        M[h, r, t] += 1
    H = np.zeros_like(E)
    PI = np.zeros((N, R, N))
    for h in range(N):
        scores = {}
        for r in range(R):
            for t in range(N):
                if M[h, r, t]:
                    a = Wr[r] @ E[t]
                    b = Wr[r] @ E[h] + er[r]
                    scores[(r, t)] = float(a @ np.tanh(b))
        H[h] = E[h]
        if not scores:
            continue
        mx = max(scores.values())
        Z = sum(M[h, r, t] * np.exp(s - mx) for (r, t), s in scores.items())
        for (r, t), s in scores.items():
            PI[h, r, t] = np.exp(s - mx) / Z                    # weight of ONE copy
            H[h] = H[h] + M[h, r, t] * PI[h, r, t] * E[t]
    J = H @ W.T
    Eout = np.where(J > 0, J, P["slope"] * J)
    return Eout, H, J, PI


def oracle_fwd(P, threads=1, **over):
    a = dict(E=P["E"], Wr=P["Wr"], er=P["er"], W=P["W"])
    a.update(over)
    return ref.aggregate_fwd_f64(P["N"], P["head"], P["rel"], P["tail"], a["E"], a["Wr"], a["er"],
                                 a["W"], P["slope"], threads)


def test_forward_matches_dense_brute_force():
    for seed in range(4):
        P = small_problem(seed=seed)
        Eout, H, J, pi = oracle_fwd(P)
        Eb, Hb, Jb, PIb = dense_forward(P)
        assert np.allclose(H, Hb, rtol=1e-12, atol=1e-13)
        assert np.allclose(J, Jb, rtol=1e-12, atol=1e-13)
        assert np.allclose(Eout, Eb, rtol=1e-12, atol=1e-13)
        want_pi = PIb[P["head"], P["rel"], P["tail"]]
        assert np.allclose(pi, want_pi, rtol=1e-12, atol=1e-15)
        # attention sums to one over each head's out-edges; isolated head keeps e_h
        sums = np.zeros(P["N"])
        np.add.at(sums, P["head"], pi)
        has = np.bincount(P["head"], minlength=P["N"]) > 0
        assert np.allclose(sums[has], 1.0, atol=1e-13)
        assert np.array_equal(H[~has], P["E"][~has])


def _loss(P, **over):
    Eout, _, _, _ = dense_forward(P, **over)
    return float((Eout * P["G"]).sum())


@pytest.mark.parametrize("seed", [0, 1])
def test_backward_matches_finite_differences_of_brute_force(seed):
    P = small_problem(seed=seed)
    _, H, J, _ = oracle_fwd(P)
    assert np.abs(J).min() > 1e-4          # no element sits on the LeakyReLU kink
    gE, gWr, ger, gW = ref.aggregate_bwd_f64(P["N"], P["head"], P["rel"], P["tail"], P["E"], H,
                                             J > 0, P["Wr"], P["er"], P["W"], P["slope"], P["G"])
    eps = 1e-6
    rng = np.random.default_rng(100 + seed)
    for name, grad in (("E", gE), ("Wr", gWr), ("er", ger), ("W", gW)):
        base = P[name]
        flat_idx = rng.choice(base.size, size=min(base.size, 40), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, base.shape)
            up = base.copy(); up[idx] += eps
            dn = base.copy(); dn[idx] -= eps
            fd = (_loss(P, **{name: up}) - _loss(P, **{name: dn})) / (2 * eps)
            assert abs(fd - grad[idx]) <= 2e-7 * max(1.0, abs(fd)), (name, idx, fd, grad[idx])


def test_zero_relation_maps_reduce_to_normalised_adjacency_spmm():
    # W_r = 0  =>  every score is 0  =>  pi = 1/deg  =>  H = E + D^-1 A E  (Eq. 2's spmm)
    P = small_problem(N=30, T=120, seed=3)
    Wr0 = np.zeros_like(P["Wr"])
    Wid = np.eye(P["d"])                       # Theta = I and slope 1: E' = J = H
    A = sp.coo_matrix((np.ones(P["T"]), (P["head"], P["tail"])), shape=(P["N"], P["N"])).tocsr()
    deg = np.asarray(A.sum(axis=1)).ravel()
    Dinv = sp.diags(np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0))
    Ahat = Dinv @ A
    Eout, H, J, pi = ref.aggregate_fwd_f64(P["N"], P["head"], P["rel"], P["tail"], P["E"], Wr0,
                                           P["er"], Wid, 1.0)
    assert np.allclose(H, P["E"] + Ahat @ P["E"], rtol=1e-12, atol=1e-13)
    assert np.allclose(Eout, H) and np.allclose(pi, 1.0 / deg[P["head"]])
    # backward of the same special case: grad_E = grad_H + A_hat^T grad_H, no grad to W_r, e_r
    G = np.random.default_rng(1).standard_normal((P["N"], P["d"]))
    gE, gWr, ger, gW = ref.aggregate_bwd_f64(P["N"], P["head"], P["rel"], P["tail"], P["E"], H,
                                             np.ones_like(H), Wr0, P["er"], Wid, 1.0, G)
    assert np.allclose(gE, G + Ahat.T @ G, rtol=1e-12, atol=1e-13)
    assert np.allclose(gW, G.T @ H, rtol=1e-12, atol=1e-12)          # grad_Theta = grad_J^T H
    assert np.all(ger == 0)
    # grad_Wr is not zero here: d s / d W_r = e_t tanh(e_r)^T does not vanish at W_r = 0
    # but it must be orthogonal to the softmax shift: sum_j grad_s_j = 0 per head
    Eb = P["E"]
    gs_total = 0.0
    for h in range(P["N"]):
        js = np.nonzero(P["head"] == h)[0]
        if js.size == 0:
            continue
        g = (G[h] @ Eb[P["tail"][js]].T)
        p = pi[js]
        gs = p * (g - (p * g).sum())
        gs_total += abs(gs.sum())
    assert gs_total < 1e-12


def test_single_neighbour_heads_get_no_attention_gradient():
    # one out-edge per head => pi = 1, grad_s = 0 => grad_Wr = grad_er = 0
    N, d = 12, 8
    P = small_problem(N=N, d=d, k=d, seed=5)
    P["head"] = np.arange(N - 1, dtype=np.int32)
    P["tail"] = np.roll(np.arange(N - 1), 3).astype(np.int32)
    P["rel"] = (np.arange(N - 1) % P["R"]).astype(np.int32)
    P["T"] = N - 1
    Eout, H, J, pi = oracle_fwd(P)
    assert np.allclose(pi, 1.0)
    assert np.allclose(H[:N - 1], P["E"][:N - 1] + P["E"][P["tail"]])
    gE, gWr, ger, gW = ref.aggregate_bwd_f64(N, P["head"], P["rel"], P["tail"], P["E"], H, J > 0,
                                             P["Wr"], P["er"], P["W"], P["slope"], P["G"])
    assert np.abs(gWr).max() < 1e-14 and np.abs(ger).max() < 1e-14
    gJ = P["G"] * np.where(J > 0, 1.0, P["slope"])
    gH = gJ @ P["W"]
    want = gH.copy()
    np.add.at(want, P["tail"], gH[P["head"]])
    assert np.allclose(gE, want, rtol=1e-12, atol=1e-13)


def test_backward_uses_the_saved_tensors():
    # grad_W is grad_J^T H_hat with whatever H_hat and mask were saved (Eq. 2);
    # the attention part is evaluated at E_hat, not at the exact E.
    P = small_problem(seed=7)
    rng = np.random.default_rng(8)
    Hhat = rng.standard_normal((P["N"], P["d"]))
    mask = rng.integers(0, 2, size=(P["N"], P["dout"]))
    Ehat = P["E"] + 0.05 * rng.standard_normal(P["E"].shape)
    gE, gWr, ger, gW = ref.aggregate_bwd_f64(P["N"], P["head"], P["rel"], P["tail"], Ehat, Hhat,
                                             mask, P["Wr"], P["er"], P["W"], P["slope"], P["G"])
    gJ = P["G"] * np.where(mask != 0, 1.0, P["slope"])
    want_gW = np.zeros_like(P["W"])
    for n in range(P["N"]):
        for o in range(P["dout"]):
            for i in range(P["d"]):
                want_gW[o, i] += gJ[n, o] * Hhat[n, i]
    assert np.allclose(gW, want_gW, rtol=1e-12, atol=1e-13)
    # with the mask and H_hat a forward pass at E_hat would have produced, the
    # result is the exact gradient of the layer at E_hat
    Q = dict(P); Q["E"] = Ehat
    _, H2, J2, _ = oracle_fwd(Q)
    g2 = ref.aggregate_bwd_f64(P["N"], P["head"], P["rel"], P["tail"], Ehat, H2, J2 > 0, P["Wr"],
                               P["er"], P["W"], P["slope"], P["G"])
    eps = 1e-6
    for idx in [(0, 0), (3, 5), (9, 2)]:
        up = Ehat.copy(); up[idx] += eps
        dn = Ehat.copy(); dn[idx] -= eps
        fd = (_loss(P, E=up) - _loss(P, E=dn)) / (2 * eps)
        assert abs(fd - g2[0][idx]) <= 2e-7 * max(1.0, abs(fd))


def test_threads_and_float_entry_points_agree_with_serial_double():
    P = small_problem(N=50, T=400, d=16, k=16, dout=8, seed=9)
    E1 = oracle_fwd(P, threads=1)
    E4 = oracle_fwd(P, threads=4)
    for a, b in zip(E1, E4):
        assert np.array_equal(a, b)
    mask = E1[2] > 0
    b1 = ref.aggregate_bwd_f64(P["N"], P["head"], P["rel"], P["tail"], P["E"], E1[1], mask,
                               P["Wr"], P["er"], P["W"], P["slope"], P["G"], threads=1)
    b4 = ref.aggregate_bwd_f64(P["N"], P["head"], P["rel"], P["tail"], P["E"], E1[1], mask,
                               P["Wr"], P["er"], P["W"], P["slope"], P["G"], threads=4)
    for a, b in zip(b1, b4):
        assert np.allclose(a, b, rtol=1e-13, atol=1e-14)
    # float entry points: same numbers from float inputs, rounded once
    f = {n: P[n].astype(np.float32) for n in ("E", "Wr", "er", "W", "G")}
    s32 = float(np.float32(P["slope"]))      # the float entry points take the slope as fp32
    Eo32, H32, m32 = ref.aggregate_fwd(P["N"], P["head"], P["rel"], P["tail"], f["E"], f["Wr"],
                                       f["er"], f["W"], P["slope"], threads=2)
    Eo64, H64, J64, _ = ref.aggregate_fwd_f64(P["N"], P["head"], P["rel"], P["tail"], f["E"],
                                              f["Wr"], f["er"], f["W"], s32)
    assert np.array_equal(Eo32, Eo64.astype(np.float32)) and np.array_equal(H32, H64.astype(np.float32))
    assert np.array_equal(m32 != 0, J64 > 0)
    g32 = ref.aggregate_bwd(P["N"], P["head"], P["rel"], P["tail"], f["E"], H32, m32, f["Wr"],
                            f["er"], f["W"], P["slope"], f["G"], threads=2)
    g64 = ref.aggregate_bwd_f64(P["N"], P["head"], P["rel"], P["tail"], f["E"], H32, m32, f["Wr"],
                                f["er"], f["W"], s32, f["G"])
    for a, b in zip(g32, g64):
        assert np.allclose(a, b.astype(np.float32), rtol=1e-6, atol=1e-7)


def test_rejects_bad_indices():
    P = small_problem()
    bad = P["tail"].copy(); bad[0] = P["N"]
    with pytest.raises(ValueError):
        ref.aggregate_fwd_f64(P["N"], P["head"], P["rel"], bad, P["E"], P["Wr"], P["er"], P["W"], 0.2)


def test_compressed_context_gives_unbiased_linear_gradient():
    # Proposition 1 carried through the layer: grad_W = grad_J^T H_hat is linear in
    # the saved H, so its mean over quantisation seeds tends to the bits=32 value.
    P = small_problem(N=64, T=300, d=16, k=16, dout=8, seed=11)
    f = {n: P[n].astype(np.float32) for n in ("E", "Wr", "er", "W", "G")}
    Eo, H, mask = ref.aggregate_fwd(P["N"], P["head"], P["rel"], P["tail"], f["E"], f["Wr"],
                                    f["er"], f["W"], P["slope"])
    exact_ctx = ref.save_context(f["E"], H, mask, 32, 64, 0)
    Eh, Hh, mk = ref.restore_context(exact_ctx, P["N"], P["d"], P["dout"])
    assert np.array_equal(Eh, f["E"]) and np.array_equal(Hh, H) and np.array_equal(mk, mask)
    gW_exact = ref.aggregate_bwd(P["N"], P["head"], P["rel"], P["tail"], Eh, Hh, mk, f["Wr"],
                                 f["er"], f["W"], P["slope"], f["G"])[3].astype(np.float64)
    S = 300
    acc = np.zeros_like(gW_exact); acc2 = np.zeros_like(gW_exact)
    for seed in range(S):
        ctx = ref.save_context(f["E"], H, mask, 2, 64, seed * 2)
        Eh, Hh, mk = ref.restore_context(ctx, P["N"], P["d"], P["dout"])
        assert np.array_equal(mk, mask)
        gW = ref.aggregate_bwd(P["N"], P["head"], P["rel"], P["tail"], Eh, Hh, mk, f["Wr"],
                               f["er"], f["W"], P["slope"], f["G"])[3].astype(np.float64)
        acc += gW; acc2 += gW * gW
    mean = acc / S
    sd = np.sqrt(np.maximum(acc2 / S - mean ** 2, 1e-30) / S)
    z = (mean - gW_exact) / sd
    assert np.abs(z).max() < 5.0 and 0.7 < np.mean(z * z) < 1.4


def test_context_without_H_rebuilds_it_from_E_hat():
    # the variant that saves Q(E) and the mask only: H~ is the brute-force second stage of
    # Eq. 2 at E_hat (not at E, and not the dequantised Q(H)); with an uncompressed context
    # it is the forward pass's own H, so both variants give the same gradients there
    P = small_problem(N=16, seed=11)
    N, d, dout = P["N"], P["d"], P["dout"]
    a = (N, P["head"], P["rel"], P["tail"])
    E32 = P["E"].astype(np.float32)
    Wr, er, W = (P[k].astype(np.float32) for k in ("Wr", "er", "W"))
    Eo, H, mask = ref.aggregate_fwd(*a, E32, Wr, er, W, P["slope"])
    ctx = ref.save_context(E32, H, mask, 2, 32, seed=3, keep_H=False)
    assert "packed_H" not in ctx
    full = ref.save_context(E32, H, mask, 2, 32, seed=3)
    assert np.array_equal(ctx["packed_E"], full["packed_E"]) and np.array_equal(ctx["mask"], full["mask"])
    Eh, Hh, mk = ref.restore_context(ctx, N, d, dout)
    assert Hh is None and np.array_equal(mk, mask != 0)
    Ht = ref.rebuild_H(*a, Eh, Wr, er, W, P["slope"])
    Q = dict(P)
    _, H_brute, _, _ = dense_forward(Q, E=Eh.astype(np.float64), Wr=Wr.astype(np.float64),
                                     er=er.astype(np.float64), W=W.astype(np.float64))
    assert np.allclose(Ht, H_brute, rtol=2e-6, atol=1e-7)
    assert not np.allclose(Ht, H, atol=1e-3)                      # 2-bit E_hat is far from E
    _, Hq, _ = ref.restore_context(full, N, d, dout)
    assert not np.allclose(Ht, Hq, atol=1e-3)
    # uncompressed: identical
    c32 = ref.save_context(E32, H, mask, 32, 32, seed=3, keep_H=False)
    E0, H0, m0 = ref.restore_context(c32, N, d, dout)
    assert H0 is None
    assert np.array_equal(ref.rebuild_H(*a, E0, Wr, er, W, P["slope"]), H)
