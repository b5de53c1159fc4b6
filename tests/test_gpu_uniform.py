"""GPU parity: the uniform-attention layer (Eq. (2) with the row-normalised adjacency)
against the CPU oracle, through the C ABI.  Same protocol and tolerance as the attentive
layer (tests/test_gpu_agg.py): exact forward checked at 1e-5, Q(H) and the mask bit-exact
against the oracle run on the GPU's own H, backward started from the bytes the GPU saved."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ref
from parity import close
from workloads import gen

pytestmark = pytest.mark.gpu
SLOPE = 0.2


@pytest.fixture(scope="module")
def tk():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2212_04540_amd as tk
    tk.lib()
    return tk


def run_uniform(tk, N, R, head, rel, tail, d, dout, bits, group, seed=9, data_seed=0):
    E = gen.entity_embeddings(N, d, seed=data_seed + 1)
    _, _, W = gen.layer_params(max(R, 1), d, d, dout, seed=data_seed + 2)
    G = gen.upstream_grad(N, dout, seed=data_seed + 3)
    dev = "cuda"
    graph = tk.Graph(N, R, *(torch.from_numpy(np.ascontiguousarray(a)).to(dev) for a in (head, rel, tail)))
    tE, tW, tG = (torch.from_numpy(a).to(dev) for a in (E, W, G))
    nb = max(tk.tinykg_kg_aggregate_workspace_bytes(graph, d, d, dout, False),
             tk.tinykg_kg_aggregate_workspace_bytes(graph, d, d, dout, True), 16)
    ws = torch.empty(nb, dtype=torch.uint8, device=dev)

    sv32 = tk.SavedContext(N, d, dout, 32, group, with_E=False)
    Eo32 = tk.tinykg_kg_uniform_fwd(graph, tE, tW, SLOPE, 32, group, seed, sv32, ws)
    torch.cuda.synchronize()
    H_gpu = sv32.packed_H.cpu().numpy().view(np.float32).reshape(N, d)
    wEo, wH, wmask = ref.uniform_fwd(N, head, tail, E, W, SLOPE)
    close(Eo32, wEo, "E_out")
    close(H_gpu, wH, "H")
    gmask = ref.unpack(sv32.mask_J.cpu().numpy(), N * dout, 1).reshape(N, dout)
    assert np.array_equal(gmask != 0, Eo32.cpu().numpy() > 0), "mask is not the sign of the GPU's own J"

    sv = tk.SavedContext(N, d, dout, bits, group, with_E=False)
    Eo = tk.tinykg_kg_uniform_fwd(graph, tE, tW, SLOPE, bits, group, seed, sv, ws)
    torch.cuda.synchronize()
    assert torch.equal(Eo, Eo32), "compression changed the forward output"
    assert np.array_equal(sv.mask_J.cpu().numpy(), sv32.mask_J.cpu().numpy())
    hp, hmn, hsc = ref.quantize(H_gpu, bits, group, (seed + 1) & (2 ** 64 - 1))
    assert np.array_equal(sv.packed_H.cpu().numpy(), hp)
    assert np.array_equal(sv.gmin_H.cpu().numpy().view(np.uint32), hmn.view(np.uint32))
    assert np.array_equal(sv.gscale_H.cpu().numpy().view(np.uint32), hsc.view(np.uint32))

    for b, s, Hh in ((32, sv32, H_gpu), (bits, sv, ref.dequantize(hp, hmn, hsc, N, d, bits, group))):
        gE, gW = tk.tinykg_kg_uniform_bwd(graph, s, tW, SLOPE, b, group, tG, ws)
        torch.cuda.synchronize()
        wgE, wgW = ref.uniform_bwd(N, head, tail, Hh, gmask, W, SLOPE, G)
        close(gE, wgE, f"grad_E (bits={b})")
        close(gW, wgW, f"grad_W (bits={b})")
    graph.close()


@pytest.mark.parametrize("d,dout,bits,group", [(64, 64, 2, 64), (32, 16, 2, 64), (128, 128, 4, 128),
                                               (64, 32, 8, 32), (128, 48, 2, 256), (128, 128, 1, 128),
                                               (128, 128, 8, 256), (128, 128, 2, 128)])
def test_small_graphs(tk, d, dout, bits, group):
    N, R, T = 1000, 5, 9000
    head, rel, tail = gen.kg_triplets(N, R, T, seed=11, tail_zipf=1.1)
    run_uniform(tk, N, R, head, rel, tail, d, dout, bits, group)


def test_hot_head_hot_tail_and_isolated_nodes(tk):
    # one head with 5000 out-edges (the segment path), one tail with 60 % of all in-edges
    # (the double-precision rows), nodes without any edge
    N, R = 4096, 3
    rng = np.random.default_rng(0)
    T = 40000
    head = rng.integers(0, N - 500, T).astype(np.int32)
    tail = rng.integers(0, N - 500, T).astype(np.int32)
    rel = rng.integers(0, R, T).astype(np.int32)
    head[:5000] = 17
    tail[rng.random(T) < 0.6] = 123
    run_uniform(tk, N, R, head, rel, tail, 64, 64, 2, 64)


def test_no_edges(tk):
    none = np.zeros(0, np.int32)
    run_uniform(tk, 256, 0, none, none, none, 64, 32, 2, 64)
    run_uniform(tk, 192, 0, none, none, none, 128, 128, 4, 128)


def test_fewer_nodes_than_a_tile_at_width_128(tk):
    # the dense stage works on 64-node tiles: 8 nodes, 20 edges, saved codes with one pair per row
    rng = np.random.default_rng(4)
    head, tail = rng.integers(0, 8, 20).astype(np.int32), rng.integers(0, 8, 20).astype(np.int32)
    rel = rng.integers(0, 2, 20).astype(np.int32)
    run_uniform(tk, 8, 2, head, rel, tail, 128, 128, 4, 128)
    run_uniform(tk, 65, 2, head, rel, tail, 128, 128, 2, 128)


def test_config1_graph_full_size(tk):
    # the 100k-entity / 1M-triplet graph of configs[1] with the uniform layer, INT2 group 64
    N, R, T = 100_000, 16, 1_000_000
    head, rel, tail = gen.kg_triplets(N, R, T, seed=0, tail_zipf=1.1)
    run_uniform(tk, N, R, head, rel, tail, 64, 64, 2, 64)
