"""The attentive layer's forward + backward captured into a HIP graph: the entry points
allocate nothing, synchronise nothing and clear their scratch memory with kernels, so a
captured step can be replayed.  Every replay (with eager work of the same entry points in
between) must reproduce the eager result: E_out and the saved bytes exactly, the gradients
up to the order of their atomics."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from workloads import gen

pytestmark = pytest.mark.gpu


def test_captured_step_replays_the_eager_result():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2212_04540_amd as tk
    tk.lib()
    N, R, T, d = 4096, 6, 40_000, 64
    head, rel, tail = gen.kg_triplets(N, R, T, seed=3, tail_zipf=1.1)
    dev = "cuda"
    graph = tk.Graph(N, R, *(torch.from_numpy(a).to(dev) for a in (head, rel, tail)))
    E = torch.from_numpy(gen.entity_embeddings(N, d, seed=1, std=0.1)).to(dev)
    Wr, er, W = (torch.from_numpy(a).to(dev) for a in gen.layer_params(R, d, d, d, seed=2))
    G = torch.from_numpy(gen.upstream_grad(N, d, seed=3)).to(dev)
    saved = tk.SavedContext(N, d, d, 2, 64)
    ws = torch.empty(max(tk.tinykg_kg_aggregate_workspace_bytes(graph, d, d, d, False),
                         tk.tinykg_kg_aggregate_workspace_bytes(graph, d, d, d, True)), dtype=torch.uint8, device=dev)
    E_out = torch.empty((N, d), device=dev)
    grads = (torch.empty((N, d), device=dev), torch.empty_like(Wr), torch.empty_like(er), torch.empty_like(W))

    def step(seed):
        tk.tinykg_kg_aggregate_fwd(graph, E, Wr, er, W, 0.2, 2, 64, seed, saved, ws, E_out=E_out)
        tk.tinykg_kg_aggregate_bwd(graph, saved, Wr, er, W, 0.2, 2, 64, G, ws, out=grads)

    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        step(7)
    torch.cuda.synchronize()
    want = [x.clone() for x in grads]
    want_out, want_codes = E_out.clone(), saved.packed_E.clone()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step(7)
    torch.cuda.synchronize()
    for k in range(3):
        step(100 + k)                       # eager work with another seed between the replays
        for x in grads:
            x.fill_(float("nan"))
        E_out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(E_out, want_out) and torch.equal(saved.packed_E, want_codes), f"replay {k}"
        for a, b, nm in zip(grads, want, ("grad_E", "grad_Wr", "grad_er", "grad_W")):
            scale = float(b.abs().max())
            assert float((a - b).abs().max()) <= 1e-5 * scale, f"replay {k}: {nm}"
    graph.close()
