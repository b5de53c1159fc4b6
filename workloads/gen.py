"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module only draws random inputs (numpy's PCG64 streams); it holds none of
the compressor's or the aggregation's arithmetic.  Both the GPU library and the
CPU oracle are fed the arrays made here.

The paper trains on Amazon-book, MovieLens-20M and Yelp2018 (Table 1); those
datasets are not available, so every workload is a synthetic stand-in with the
same shapes and degree skew.
"""
import numpy as np


def normal_activations(rows, dim, seed=0, std=1.0):
    """fp32 [rows, dim], N(0, std^2): the standalone-compressor workload."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((rows, dim), dtype=np.float32) * np.float32(std)).astype(np.float32)


def student_t_activations(rows, dim, seed=0, nu=3, chunk_rows=1 << 18):
    """fp32 [rows, dim], Student-t(nu): heavy-tailed activations (large range,
    most codes in the lowest bins).  Drawn chunk-wise so peak host memory stays
    near the size of the result."""
    rng = np.random.default_rng(seed)
    out = np.empty((rows, dim), dtype=np.float32)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        out[r0:r1] = rng.standard_t(nu, size=(r1 - r0, dim)).astype(np.float32)
    return out


def zipf_indices(n_items, count, exponent, rng):
    """`count` draws from {0..n_items-1} with P(rank k) ~ (k+1)^-exponent (exact
    finite table, inverse CDF); rank -> id through a seeded random permutation."""
    w = (np.arange(1, n_items + 1, dtype=np.float64)) ** (-float(exponent))
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    ranks = np.searchsorted(cdf, rng.random(count), side="left")
    ranks = np.minimum(ranks, n_items - 1)
    perm = rng.permutation(n_items)
    return perm[ranks].astype(np.int32)


def kg_triplets(n_nodes, n_rel, n_edges, seed=0, tail_zipf=1.1, head_zipf=None):
    """(head, rel, tail) int32 arrays in random order.  Heads uniform (or Zipf),
    relations uniform, tails Zipf(tail_zipf).  Duplicates and self-loops are kept
    (the graph is a multigraph)."""
    rng = np.random.default_rng(seed)
    if head_zipf is None:
        head = rng.integers(0, n_nodes, size=n_edges, dtype=np.int32)
    else:
        head = zipf_indices(n_nodes, n_edges, head_zipf, rng)
    rel = rng.integers(0, n_rel, size=n_edges, dtype=np.int32)
    tail = zipf_indices(n_nodes, n_edges, tail_zipf, rng)
    return head, rel, tail


def layer_params(n_rel, d_in, d_rel, d_out, seed=0, er_std=0.1):
    """W_r[R, d_rel, d_in], e_r[R, d_rel], W[d_out, d_in]: N(0, 1/d_in) weights,
    N(0, er_std^2) relation embeddings (0.1 in every workload)."""
    rng = np.random.default_rng(seed)
    s = np.float32(1.0 / np.sqrt(d_in))
    Wr = rng.standard_normal((n_rel, d_rel, d_in), dtype=np.float32) * s
    er = rng.standard_normal((n_rel, d_rel), dtype=np.float32) * np.float32(er_std)
    W = rng.standard_normal((d_out, d_in), dtype=np.float32) * s
    return Wr.astype(np.float32), er.astype(np.float32), W.astype(np.float32)


def entity_embeddings(n_nodes, dim, seed=0, std=0.1):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n_nodes, dim), dtype=np.float32) * np.float32(std)).astype(np.float32)


def upstream_grad(n_nodes, dim, seed=0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n_nodes, dim), dtype=np.float32)


def user_item_entity_graph(n_users, n_items, n_attr, n_kg_rel, n_kg_edges, n_interactions,
                           seed=0, zipf=1.2):
    """Amazon-book-shaped stand-in (Table 1): node ids are users, then items,
    then attribute entities.  KG triplets join items and attributes with Zipf
    endpoints and relation ids 0..n_kg_rel-1; each user-item pair is inserted in
    both directions with relation ids n_kg_rel (user->item) and n_kg_rel+1."""
    rng = np.random.default_rng(seed)
    n_ent = n_items + n_attr
    kh = zipf_indices(n_ent, n_kg_edges, zipf, rng) + n_users
    kt = zipf_indices(n_ent, n_kg_edges, zipf, rng) + n_users
    kr = rng.integers(0, n_kg_rel, size=n_kg_edges, dtype=np.int32)
    u = rng.integers(0, n_users, size=n_interactions, dtype=np.int32)
    it = zipf_indices(n_items, n_interactions, zipf, rng) + n_users
    head = np.concatenate([kh, u, it]).astype(np.int32)
    tail = np.concatenate([kt, it, u]).astype(np.int32)
    rel = np.concatenate([kr, np.full(n_interactions, n_kg_rel, np.int32),
                          np.full(n_interactions, n_kg_rel + 1, np.int32)]).astype(np.int32)
    return head, rel, tail
