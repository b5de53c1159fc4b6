"""The measurement hooks: per-kernel device times, all launches or the launches of one name."""
import pytest

from workloads import gen

pytestmark = pytest.mark.gpu
SLOPE = 0.2


@pytest.fixture(scope="module")
def tk():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2212_04540_amd as tk
    tk.lib()
    return tk


def test_report_covers_all_launches_or_the_selected_name(tk):
    import torch
    N, R, T, d = 336, 5, 3000, 64
    head, rel, tail = gen.kg_triplets(N, R, T, seed=3)
    dev = "cuda"
    graph = tk.Graph(N, R, *(torch.from_numpy(a).to(dev) for a in (head, rel, tail)))
    E = torch.from_numpy(gen.entity_embeddings(N, d, seed=1)).to(dev)
    Wr, er, W = (torch.from_numpy(a).to(dev) for a in gen.layer_params(R, d, d, d, seed=2))
    G = torch.from_numpy(gen.upstream_grad(N, d, seed=3)).to(dev)
    saved = tk.SavedContext(N, d, d, 2, 64)
    ws = torch.empty(max(tk.tinykg_kg_aggregate_workspace_bytes(graph, d, d, d, False),
                         tk.tinykg_kg_aggregate_workspace_bytes(graph, d, d, d, True)), dtype=torch.uint8, device=dev)

    def step():
        tk.tinykg_kg_aggregate_fwd(graph, E, Wr, er, W, SLOPE, 2, 64, 7, saved, ws)
        tk.tinykg_kg_aggregate_bwd(graph, saved, Wr, er, W, SLOPE, 2, 64, G, ws)

    try:
        tk.tinykg_profile_select(None)
        tk.tinykg_profile_enable(True)
        for _ in range(3):
            step()
        torch.cuda.synchronize()
        full = tk.tinykg_profile_report()
        tk.tinykg_profile_enable(False)
        assert full["edge_bwd_kernel"][0] == 3 and full["score_kernel"][0] == 6
        assert {"attend_fwd_kernel", "attend_bwd_kernel", "dense_fwd_kernel", "dense_bwd_kernel",
                "quantize_kernel", "epilogue_kernel"} <= set(full)
        assert all(ms > 0 for _, ms in full.values())

        tk.tinykg_profile_select("edge_bwd_kernel")
        tk.tinykg_profile_enable(True)          # also drops the earlier records
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        only = tk.tinykg_profile_report()
        tk.tinykg_profile_enable(False)
        assert set(only) == {"edge_bwd_kernel"} and only["edge_bwd_kernel"][0] == 2

        step()                                   # disabled: nothing is recorded
        assert tk.tinykg_profile_report() == only
    finally:
        tk.tinykg_profile_select(None)
        tk.tinykg_profile_enable(False)
        graph.close()
