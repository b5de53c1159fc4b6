#!/usr/bin/env python3
"""Benchmark of the TinyKG hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
the attentive aggregation layer's forward pass (which quantises and bit-packs the
saved activations E and H and keeps a 1-bit mask of J) followed by its backward
pass (which unpacks and dequantises them inside its gathers), on the 100k-entity /
1M-triplet configuration (configs[1]).  Inputs are resident in HBM before the timed
region.

Prints ONE JSON line.  `value` is algorithmic bytes per step / step time of the
configs[1] step; `roofline` prices its dominant kernel against its own bound.  The same
line carries the other configurations as extra objects: `sweep` (configs[2]: the nine
bits x group cells of the compressor on the 2 GiB heavy-tailed activation), `config3`
(three-layer step on the user-item-entity graph), `config4` (20M entities x 128, 150M
triplets, two layers, INT4/G128), `uniform_large` (the uniform-attention layer of Eq. 2
on the configs[4] graph: the dequantize-fused backward aggregation at a size that leaves
the 256 MB Infinity Cache, priced against the HBM roofline) and `cpu_baseline` (the CPU
oracle on the configs[1] step).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_FP32_PEAK_TFLOPS = 157.3
MFMA_BF16_PEAK_TFLOPS = 2500.0
METRIC = "quantize+pack and dequant+agg-bwd HBM GB/s (fraction of peak); bytes/activation"

# configs[1]
N, D, R, T = 100_000, 64, 16, 1_000_000
BITS, GROUP, SLOPE = 2, 64, 0.2
# configs[2]
C2_ROWS, C2_DIM = 1 << 23, 64
# configs[4]
C4_N, C4_R, C4_T, C4_D, C4_BITS, C4_GROUP = 20_000_000, 60, 150_000_000, 128, 4, 128


def bytes_per_activation(bits, group):
    return 4.0 if bits == 32 else bits / 8 + 8 / group


def step_algorithmic_bytes(saved_H=True):
    """Compulsory bytes of one forward+backward step (per-edge and per-node terms).
    saved_H=False: Q(H) is neither written nor read; the packed e_t rows are gathered twice."""
    bpa = bytes_per_activation(BITS, GROUP)
    nq = 2 if saved_H else 1
    fwd_edge = 4 * D + 4 + 4 + 4            # e_t row, tail id, relation id, score
    fwd_node = 4 * D + 4 * D + nq * D * bpa + D / 8  # E in, E' out, Q(E) (+Q(H)) saved, mask
    bwd_edge = (3 - nq) * D * bpa + 12      # packed e_t row, ids + score gradient
    bwd_node = 4 * D + D * bpa + D / 8 + 4 * D       # grad_E' in, H_hat (or E_hat), mask, grad_E out
    return T * (fwd_edge + bwd_edge) + N * (fwd_node + bwd_node)


def edge_bwd_flops(n_edges=T, d=D):
    """ALGORITHMIC contractions of the edge-level backward kernel: per triplet six k x d
    products (recompute W_r e_t and W_r e_h, W_r^T grad_a, W_r^T grad_b, two outer products)."""
    return n_edges * 6 * 2 * d * d


def tile_stats(rel, tail):
    """32-edge tiles of the relation order (edges sorted by relation, then tail; tiles counted
    from each relation's first edge): how many there are and how many hold ONE tail (those take
    the edge kernel's run form).  Host arithmetic on the benchmark's own input, for the
    executed-flops account only."""
    import numpy as np
    order = np.lexsort((tail, rel))
    r, t = rel[order], tail[order]
    first = np.searchsorted(r, np.arange(int(r.max()) + 2 if r.size else 1))
    tiles = one = 0
    for k in range(first.size - 1):
        seg = t[first[k]:first[k + 1]]
        if seg.size == 0:
            continue
        n_t = (seg.size + 31) // 32
        pad = np.full(n_t * 32, -1, dtype=seg.dtype)
        pad[:seg.size] = seg
        pad = pad.reshape(n_t, 32)
        same = ((pad == pad[:, :1]) | (pad < 0)).all(axis=1)
        tiles += n_t
        one += int(same.sum())
    return tiles, one


def edge_executed(tiles, d=D):
    """What the d <= 64 edge kernel executes on the matrix cores for a compressed context (its code
    form, whole 32-row tiles), all of it bfloat16 piece products: a and b as three products each
    (codes are exact bfloat16 values), the two outer products for grad_W_r likewise three each,
    W_r^T grad_a and W_r^T grad_b six each."""
    prod = 2 * 32 * d * d
    return 0, tiles * (2 * 3 + 2 * 3 + 2 * 6) * prod


def parse_profile_rows(path, kernel_prefix):
    """Rows of a committed rocprofv3 summary whose kernel name starts with `kernel_prefix`: token lists."""
    try:
        n = len(kernel_prefix)
        return [l.split() for l in open(path) if l.startswith(kernel_prefix) and l[n:n + 1] in ("<", " ", ",", ">")]
    except OSError:
        return []


PROFILE_STEP = os.path.join(ROOT, "profiles", "aggregation_step_configs1.txt")
PROFILE_ALL = os.path.join(ROOT, "profiles", "default_bench_all_configs.txt")
PROFILE_SQ = os.path.join(ROOT, "profiles", "sq_counters_configs1_step.txt")


def profiled_traffic(kernel, summary=None):
    """HBM bytes per launch of `kernel` from a committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by what the counter reads for a copy of known
    size): measured OFFLINE with the commands that file lists, not in this run."""
    rows = [r for r in parse_profile_rows(summary or PROFILE_STEP, kernel) if len(r) >= 6]
    tot = []
    for r in rows:
        try:
            f, w = float(r[-2]), float(r[-1])
        except ValueError:
            continue
        if f == f and w == w:
            tot.append((f + w) * 1e6)
    return round(max(tot)) if tot else None


def profiled_sq(kernel):
    """(mfma_util, wait) of `kernel` from the committed SQ counter summary (offline run)."""
    for r in parse_profile_rows(PROFILE_SQ, kernel):
        try:
            return float(r[-3]), float(r[-1])
        except (ValueError, IndexError):
            continue
    return None, None


def make_inputs():
    from workloads import gen
    head, rel, tail = gen.kg_triplets(N, R, T, seed=0, tail_zipf=1.1)
    E = gen.entity_embeddings(N, D, seed=1)
    Wr, er, W = gen.layer_params(R, D, D, D, seed=2)
    G = gen.upstream_grad(N, D, seed=3)
    return dict(head=head, rel=rel, tail=tail, E=E, Wr=Wr, er=er, W=W, G=G)


def cpu_baseline(inp, seed):
    """The oracle as it stands, on this host's cores, on the full configs[1] step."""
    from oracle import ref
    threads = ref.default_threads()
    t0 = time.perf_counter()
    Eo, H, mask = ref.aggregate_fwd(N, inp["head"], inp["rel"], inp["tail"], inp["E"], inp["Wr"],
                                    inp["er"], inp["W"], SLOPE, threads=threads)
    ctx = ref.save_context(inp["E"], H, mask, BITS, GROUP, seed)
    Eh, Hh, mk = ref.restore_context(ctx, N, D, D)
    ref.aggregate_bwd(N, inp["head"], inp["rel"], inp["tail"], Eh, Hh, mk, inp["Wr"], inp["er"],
                      inp["W"], SLOPE, inp["G"], threads=threads)
    dt = time.perf_counter() - t0
    return {"value": round(step_algorithmic_bytes() / dt / 1e9, 4), "unit": "GB/s", "cores": threads,
            "kind": "oracle", "seconds": round(dt, 3),
            "sample": "one full configs[1] step (forward, INT2/G64 save, restore, backward); "
                      "aggregation loops threaded over heads, quantizer single-threaded"}


def student_t_matrix(torch, rows, dim, seed=0):
    """Student-t(3) = z / sqrt(chi2_3 / 3), drawn on the device in slabs."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    x = torch.empty((rows, dim), dtype=torch.float32, device="cuda")
    step = min(rows, 1 << 20)
    for r0 in range(0, rows, step):
        z = torch.randn((step, dim), generator=g, device="cuda")
        chi = torch.randn((step, dim, 3), generator=g, device="cuda").square_().sum(-1)
        x[r0:r0 + step] = z / (chi / 3).sqrt_()
    return x


def variance_stats(tk, torch, x, bits, group, seeds=64):
    """Per-element variance of dequantize(quantize(x; seed)) over `seeds` seeds against
    Proposition 1's closed form scale^2 p (1 - p) and its bound scale^2 / 4 (statistics of
    the kernels' outputs, accumulated with torch on the device)."""
    rows, dim = x.shape
    s1 = torch.zeros((rows, dim), dtype=torch.float64, device="cuda")
    s2 = torch.zeros_like(s1)
    buf = tk.alloc_quantized(rows, dim, bits, group)
    out = torch.empty_like(x)
    for seed in range(seeds):
        tk.tinykg_quantize(x, bits, group, 1000 + seed, out=buf)
        tk.tinykg_dequantize(*buf, rows, dim, bits, group, out=out)
        s1 += out
        s2 += out.double() ** 2
    var = s2 / seeds - (s1 / seeds) ** 2                     # population variance over the seeds
    mn = buf[1].double().repeat_interleave(group).reshape(rows, dim)
    sc = buf[2].double().repeat_interleave(group).reshape(rows, dim)
    xb = torch.where(sc > 0, (x.double() - mn) / sc, torch.zeros_like(sc)).clamp_(0, (1 << bits) - 1)
    pfrac = xb - xb.floor()
    closed = sc * sc * pfrac * (1 - pfrac)
    bound = sc * sc / 4
    live = bound > 0
    return {"seeds": seeds, "rows": rows,
            "mean_var_over_closed_form": round(float(var.sum() / closed.sum()), 4),
            "max_var_over_quarter_scale2": round(float((var[live] / bound[live]).max()), 4),
            "mean_var_over_quarter_scale2": round(float((var[live] / bound[live]).mean()), 4)}


def sweep_cells(tk, torch, steps, with_variance):
    """configs[2]: the 9 cells bits x group on the 2 GiB heavy-tailed activation, plus the
    plain copy of the same size as the practical ceiling.  Pack and unpack are fused into
    quantize / dequantize and are not separately observable."""
    x = student_t_matrix(torch, C2_ROWS, C2_DIM)
    n = x.numel()
    out = torch.empty_like(x)
    sub = x[:4096].contiguous()
    cells = []
    for bits in (2, 4, 8):
        for group in (32, 64, 256):
            buf = tk.alloc_quantized(C2_ROWS, C2_DIM, bits, group)
            for _ in range(2):
                tk.tinykg_quantize(x, bits, group, 1, out=buf)
                tk.tinykg_dequantize(*buf, C2_ROWS, C2_DIM, bits, group, out=out)
            torch.cuda.synchronize()
            tk.tinykg_profile_enable(True)
            for i in range(steps):
                tk.tinykg_quantize(x, bits, group, 1 + i, out=buf)
                tk.tinykg_dequantize(*buf, C2_ROWS, C2_DIM, bits, group, out=out)
            torch.cuda.synchronize()
            rep = tk.tinykg_profile_report()
            tk.tinykg_profile_enable(False)
            bpe = 4 + bytes_per_activation(bits, group)
            cell = {"bits": bits, "group": group, "bytes_per_activation": bytes_per_activation(bits, group),
                    "compression_ratio": round(4 / bytes_per_activation(bits, group), 3)}
            for key, name in (("quantize_pack", "quantize_kernel"), ("unpack_dequantize", "dequantize_kernel")):
                cnt, ms = rep[name]
                gbs = n * bpe / (ms / cnt) / 1e6
                cell[key] = {"ms": round(ms / cnt, 4), "GB/s": round(gbs, 1),
                             "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
            pair_ms = cell["quantize_pack"]["ms"] + cell["unpack_dequantize"]["ms"]
            cell["pair_frac_of_hbm_peak"] = round(2 * n * bpe / pair_ms / 1e6 / HBM_PEAK_GBS, 4)
            # the dequantizer launched back to back: it then does not inherit the write-back of the dirty
            # lines that the quantizer's launch left in the 256 MB last-level cache (about 40 us when full)
            tk.tinykg_profile_enable(True)
            for i in range(steps):
                tk.tinykg_dequantize(*buf, C2_ROWS, C2_DIM, bits, group, out=out)
            torch.cuda.synchronize()
            cnt, ms = tk.tinykg_profile_report()["dequantize_kernel"]
            tk.tinykg_profile_enable(False)
            gbs = n * bpe / (ms / cnt) / 1e6
            cell["unpack_dequantize_back_to_back"] = {"ms": round(ms / cnt, 4), "GB/s": round(gbs, 1),
                                                      "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
            if with_variance:
                cell["variance"] = variance_stats(tk, torch, sub, bits, group)
            cells.append(cell)
            del buf
    tk.tinykg_profile_enable(True)
    for _ in range(5):
        tk.tinykg_profile_copy(out, x)      # plain copy of known size: practical HBM ceiling
    torch.cuda.synchronize()
    cnt, ms = tk.tinykg_profile_report()["calibration_copy_kernel"]
    tk.tinykg_profile_enable(False)
    gbs = 2 * n * 4 / (ms / cnt) / 1e6
    copy = {"ms": round(ms / cnt, 4), "GB/s": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    del x, out, sub
    torch.cuda.empty_cache()
    return cells, copy


def sweep_object(cells, copy, steps):
    fq = [c["quantize_pack"]["frac_of_hbm_peak"] for c in cells]
    fd = [c["unpack_dequantize"]["frac_of_hbm_peak"] for c in cells]
    fp = [c["pair_frac_of_hbm_peak"] for c in cells]
    fb = [c["unpack_dequantize_back_to_back"]["frac_of_hbm_peak"] for c in cells]
    return {"workload": f"configs[2]: {C2_ROWS}x{C2_DIM} fp32 Student-t(3) (2 GiB), bits in {{2,4,8}} x group in "
                        "{32,64,256}; HIP-event averages per launch, GB/s = (4 + b/8 + 8/G) B x 2^29 / time",
            "schedule": "quantize and dequantize launches alternate (each dequantize launch inherits the write-back of "
                        "the dirty lines its quantize launch left in the last-level cache); unpack_dequantize_back_to_back "
                        "times the dequantizer's launches in a row; pair = both kernels' bytes over both kernels' time",
            "launches_per_cell": steps, "min_frac_quantize_pack": min(fq), "min_frac_unpack_dequantize": min(fd),
            "min_frac_pair": min(fp), "min_frac_unpack_dequantize_back_to_back": min(fb),
            "plain_copy": copy, "cells": cells}


def compressor_sweep(a):
    import torch
    import paper_2212_04540_amd as tk
    cells, copy = sweep_cells(tk, torch, a.steps, with_variance=True)
    ref = next(c for c in cells if c["bits"] == BITS and c["group"] == GROUP)
    print(json.dumps({
        "metric": METRIC,
        "value": ref["quantize_pack"]["GB/s"], "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": 2,
        "ms_per_step": ref["quantize_pack"]["ms"] + ref["unpack_dequantize"]["ms"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[2]: compressor sweep on {C2_ROWS}x{C2_DIM} fp32 Student-t(3) (2 GiB), "
                               "bits in {2,4,8} x group in {32,64,256}; value = quantize+pack of INT2/G64"},
        "roofline": {"kernel": "quantize_kernel", "bound": "hbm", "achieved": ref["quantize_pack"]["GB/s"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ref["quantize_pack"]["frac_of_hbm_peak"],
                     "traffic": profiled_traffic("quantize_kernel<float, 2, 64", PROFILE_ALL),
                     "traffic_source": "offline rocprofv3 counters, profiles/" + os.path.basename(PROFILE_ALL)},
        "plain_copy": copy, "cells": cells}))


# ------------------------------------------------------------------ uniform layer ----
def uniform_result(tk, torch, graph, n_nodes, n_edges, n_tails, d, bits, group, steps, warmup, label, E=None, G=None):
    """The uniform-attention layer (Eq. 2 as printed, row-normalised adjacency), forward +
    backward: no projections, so every kernel is a gather or a stream and HBM bounds the step
    once the tensors leave the cache.  Per kernel: HIP-event time, algorithmic bytes, GB/s."""
    dev = "cuda"
    g = torch.Generator(device=dev)
    g.manual_seed(11)
    if E is None:
        E = torch.randn((n_nodes, d), generator=g, device=dev) * 0.1
    if G is None:
        G = torch.randn((n_nodes, d), generator=g, device=dev)
    W = torch.randn((d, d), generator=g, device=dev) / d ** 0.5
    saved = tk.SavedContext(n_nodes, d, d, bits, group, with_E=False)
    ws = torch.empty(max(tk.tinykg_kg_aggregate_workspace_bytes(graph, d, d, d, False),
                         tk.tinykg_kg_aggregate_workspace_bytes(graph, d, d, d, True)),
                     dtype=torch.uint8, device=dev)
    E_out = torch.empty((n_nodes, d), dtype=torch.float32, device=dev)
    grads = (torch.empty((n_nodes, d), dtype=torch.float32, device=dev), torch.empty_like(W))

    def step(i):
        tk.tinykg_kg_uniform_fwd(graph, E, W, SLOPE, bits, group, 1 + 2 * i, saved, ws, E_out=E_out)
        tk.tinykg_kg_uniform_bwd(graph, saved, W, SLOPE, bits, group, G, ws, out=grads)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    # per-kernel times: a second pass with every launch bracketed by HIP events
    k_steps = min(steps, 5)
    tk.tinykg_profile_enable(True)
    for i in range(k_steps):
        step(warmup + steps + i)
    torch.cuda.synchronize()
    rep = tk.tinykg_profile_report()
    tk.tinykg_profile_enable(False)
    bpa = bytes_per_activation(bits, group)
    Tn, Nn = n_edges, n_nodes
    alg_k = {
        # forward gather: e_t row + tail id per edge; E in, H out per node
        "attend_fwd_kernel": Tn * (4 * d + 4) + Nn * (8 * d + 4),
        "quantize_kernel": Nn * d * (4 + bpa),
        "dense_fwd_kernel": Nn * (4 * d + 4 * d + d / 8),
        # dense backward with H_hat dequantised on load: grad_E' in, packed H_hat + mask in, grad_H and grad_E out
        "dense_bwd_kernel": Nn * (4 * d + d * bpa + d / 8 + 8 * d),
        # backward gather (the transposed sparse product): the head's row of grad_H / deg + head id + tail id per
        # edge; per node that has in-edges (n_tails of them) its own grad_H row read and its grad_E row written
        "uniform_bwd_kernel": Tn * (4 * d + 8) + n_tails * 8 * d,
    }
    kernels = {}
    for k, v in rep.items():
        ms = v[1] / k_steps
        kernels[k] = {"launches_per_step": v[0] / k_steps, "ms_per_step": round(ms, 4)}
        if k in alg_k:
            gbs = alg_k[k] / (ms * 1e-3) / 1e9
            kernels[k].update({"algorithmic_bytes": int(alg_k[k]), "algorithmic_GBps": round(gbs, 1),
                               "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)})
    alg = sum(alg_k.values())
    gat = kernels.get("uniform_bwd_kernel", {})
    bwd_ms = sum(kernels[k]["ms_per_step"] for k in ("dense_bwd_kernel", "uniform_bwd_kernel") if k in kernels)
    bwd_bytes = alg_k["dense_bwd_kernel"] + alg_k["uniform_bwd_kernel"]
    res = {"workload": label, "bits": bits, "group": group, "nodes_with_in_edges": n_tails,
           "ms_per_step": round(dt * 1e3, 4), "steps": steps,
           "algorithmic_bytes_per_step": int(alg), "GB/s": round(alg / dt / 1e9, 1),
           "frac_of_hbm_peak": round(alg / dt / 1e9 / HBM_PEAK_GBS, 4),
           "saved_context_bytes": saved.nbytes(), "fp32_context_bytes": n_nodes * d * 4 + n_nodes * d // 8,
           "launch_gap_share": round(max(0.0, 1.0 - sum(k["ms_per_step"] for k in kernels.values()) / (dt * 1e3)), 4),
           "dequant_fused_backward": {"kernels": ["dense_bwd_kernel", "uniform_bwd_kernel"], "ms": round(bwd_ms, 4),
                                      "algorithmic_GBps": round(bwd_bytes / (bwd_ms * 1e-3) / 1e9, 1) if bwd_ms else None,
                                      "frac_of_hbm_peak": round(bwd_bytes / (bwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if bwd_ms else None},
           "roofline": {"kernel": "uniform_bwd_kernel", "bound": "hbm", "achieved": gat.get("algorithmic_GBps"),
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gat.get("frac_of_hbm_peak"),
                        "rocprof_name": f"uniform_tail_kernel<{d}>",
                        "traffic": profiled_traffic(f"uniform_tail_kernel<{d}>", PROFILE_ALL) if n_nodes == C4_N else None,
                        "traffic_source": "offline rocprofv3 counters (not this run), profiles/" + os.path.basename(PROFILE_ALL),
                        "avg_launch_ms": gat.get("ms_per_step")},
           "kernels": kernels}
    del saved, ws, E_out, grads
    return res


def uniform_workload(a):
    """The uniform-attention layer on the configs[1] graph (cache-resident) or, with --large,
    on the configs[4] graph (20M x 128: every tensor is 10 GB)."""
    import torch
    import paper_2212_04540_amd as tk
    if a.large:
        head, rel, tail = device_kg_triplets(torch, C4_N, C4_R, C4_T, 1.05, seed=0)
        graph = tk.Graph(C4_N, C4_R, head, rel, tail)
        n_tails = int(torch.unique(tail).numel())
        del head, rel, tail
        res = uniform_result(tk, torch, graph, C4_N, C4_T, n_tails, C4_D, C4_BITS, C4_GROUP, a.steps, a.warmup,
                             "uniform-attention layer (Eq. 2), forward+backward, on the configs[4] graph: 20M entities, "
                             "dim 128, 150M triplets (Zipf 1.05 tails), saved Q(H) INT4 group 128")
    else:
        inp = make_inputs()
        t = {k: torch.from_numpy(v).cuda() for k, v in inp.items()}
        graph = tk.Graph(N, R, t["head"], t["rel"], t["tail"])
        import numpy as np
        res = uniform_result(tk, torch, graph, N, T, int(np.unique(inp["tail"]).size), D, BITS, GROUP, a.steps, a.warmup,
                             "uniform-attention layer (Eq. 2, row-normalised adjacency), forward+backward, on the "
                             "configs[1] graph: 100k entities, dim 64, 1M triplets, saved Q(H) INT2 group 64",
                             E=t["E"], G=t["G"])
    graph.close()
    print(json.dumps({
        "metric": METRIC, "value": res["GB/s"], "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": res["workload"], "bits": res["bits"], "group": res["group"],
                   "algorithmic_bytes_per_step": res["algorithmic_bytes_per_step"],
                   "saved_context_bytes": res["saved_context_bytes"]},
        "frac_of_hbm_peak": res["frac_of_hbm_peak"], "roofline": res["roofline"],
        "dequant_fused_backward": res["dequant_fused_backward"], "launch_gap_share": res["launch_gap_share"],
        "kernels": res["kernels"]}))


def maxpool_workload(a):
    """Max-pooling aggregation (SPMM_MAX, Sec. 4.1.4 operator list) on the configs[1] graph:
    a gather and a scatter, no arithmetic to speak of."""
    import torch
    import paper_2212_04540_amd as tk
    dev = "cuda"
    inp = make_inputs()
    t = {k: torch.from_numpy(v).to(dev) for k, v in inp.items()}
    graph = tk.Graph(N, R, t["head"], t["rel"], t["tail"])
    nb = int(tk.lib().tinykg_kg_max_arg_bytes(graph.handle))
    G = t["G"]
    M, arg = tk.tinykg_kg_max_fwd(graph, t["E"])
    ws = torch.empty(int(tk.lib().tinykg_kg_max_workspace_bytes(graph.handle, D)), dtype=torch.uint8, device=dev)
    gE = torch.empty_like(G)

    def step(i):
        tk.tinykg_kg_max_fwd(graph, t["E"], out=(M, arg))
        tk.tinykg_kg_max_bwd(graph, arg, G, workspace=ws, out=gE)

    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    tk.tinykg_profile_enable(True)
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(a.warmup + i)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / a.steps
    rep = tk.tinykg_profile_report()
    tk.tinykg_profile_enable(False)
    fwd_bytes = T * (4 * D + 4) + N * (4 * D + D * nb + 4)          # e_t row + tail id; M, numbers, row pointer
    bwd_bytes = T * (4 * D + D * nb + 13) + N * 4 * D                # per edge: grad_M row, numbers of the head's row,
    #                                                                  head / tail / position / flags; grad_E cleared
    alg = fwd_bytes + bwd_bytes
    kernels = {k: {"launches_per_step": v[0] / a.steps, "ms_per_step": round(v[1] / a.steps, 4)} for k, v in rep.items()}
    f_ms = rep["max_fwd_kernel"][1] / rep["max_fwd_kernel"][0]
    print(json.dumps({
        "metric": METRIC,
        "value": round(alg / dt / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(dt * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "max-pooling aggregation (SPMM_MAX), forward+backward, on the configs[1] graph: "
                               "100k entities, dim 64, 1M triplets",
                   "context_bytes_per_element": nb, "algorithmic_bytes_per_step": alg,
                   "saved_context_bytes": N * D * nb, "int64_argmax_context_bytes": N * D * 8},
        "frac_of_hbm_peak": round(alg / dt / 1e9 / HBM_PEAK_GBS, 5),
        "roofline": {"kernel": "max_fwd_kernel", "bound": "hbm", "achieved": round(fwd_bytes / (f_ms * 1e-3) / 1e9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(fwd_bytes / (f_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": None, "avg_launch_ms": round(f_ms, 4)},
        "kernels": kernels}))
    graph.close()


def batchnorm_workload(a):
    """Batch normalisation with a compressed input (Sec. 4.1.4 operator list) on the
    configs[2] tensor shape: every kernel is a stream, so HBM bounds the whole step."""
    import torch
    import paper_2212_04540_amd as tk
    dev = "cuda"
    rows, dim = C2_ROWS, C2_DIM
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    x = torch.randn((rows, dim), generator=g, device=dev) * 1.5 + 0.3
    gy = torch.randn((rows, dim), generator=g, device=dev)
    gamma = torch.rand(dim, generator=g, device=dev) + 0.5
    beta = torch.randn(dim, generator=g, device=dev)
    ctx = tk.NormContext(rows, dim, BITS, GROUP)
    y = torch.empty_like(x)
    out = (torch.empty_like(x), torch.empty_like(gamma), torch.empty_like(gamma))

    def step(i):
        tk.tinykg_batchnorm_fwd(x, gamma, beta, 1e-5, BITS, GROUP, 1 + i, ctx, y=y)
        tk.tinykg_batchnorm_bwd(ctx, gamma, gy, out=out)

    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    tk.tinykg_profile_enable(True)
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(a.warmup + i)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / a.steps
    rep = tk.tinykg_profile_report()
    tk.tinykg_profile_enable(False)
    bpa = bytes_per_activation(BITS, GROUP)
    n = rows * dim
    per_kernel = {"bn_stats_kernel<fwd>": 4.0, "quantize_kernel": 8.0 + bpa, "bn_stats_kernel<bwd>": 4.0 + bpa,
                  "bn_apply_bwd_kernel": 8.0 + bpa}
    alg = n * sum(per_kernel.values())
    kernels = {}
    for k, v in rep.items():
        ms = v[1] / v[0]
        kernels[k] = {"launches_per_step": v[0] / a.steps, "ms_per_launch": round(ms, 4)}
        if k in per_kernel:
            kernels[k]["algorithmic_GBps"] = round(n * per_kernel[k] / (ms * 1e-3) / 1e9, 1)
            kernels[k]["frac_of_hbm_peak"] = round(n * per_kernel[k] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    dom = max(per_kernel, key=lambda k: rep[k][1])
    dom_ms = rep[dom][1] / rep[dom][0]
    bn_summary = os.path.join(ROOT, "profiles", "batchnorm_2p23x64_int2_g64.txt")
    print(json.dumps({
        "metric": METRIC,
        "value": round(alg / dt / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(dt * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"batch normalisation with a compressed input, forward+backward, {rows}x{dim} fp32 "
                               f"(2 GiB per tensor), INT{BITS} group {GROUP}",
                   "bits": BITS, "group": GROUP, "bytes_per_activation": bpa, "algorithmic_bytes_per_step": alg,
                   "saved_context_bytes": ctx.nbytes(), "fp32_context_bytes": n * 4 + 8 * dim},
        "frac_of_hbm_peak": round(alg / dt / 1e9 / HBM_PEAK_GBS, 5),
        "roofline": {"kernel": dom, "bound": "hbm", "achieved": round(n * per_kernel[dom] / (dom_ms * 1e-3) / 1e9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(n * per_kernel[dom] / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": profiled_traffic(dom, bn_summary),
                     "traffic_source": "offline rocprofv3 counters, profiles/" + os.path.basename(bn_summary),
                     "avg_launch_ms": round(dom_ms, 4)},
        "kernels": kernels}))


# ------------------------------------------------------------- configs[3] / [4] ----
def device_kg_triplets(torch, n_nodes, n_rel, n_edges, tail_zipf, seed=0):
    """(head, rel, tail) int32 on the device: heads and relations uniform, tails Zipf by inverse
    CDF on the exact finite table, rank -> id through a seeded random permutation -- the recipe
    of workloads/gen.py's kg_triplets, drawn with torch's device generator (no host pass over
    150M triplets)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    head = torch.randint(0, n_nodes, (n_edges,), generator=g, device="cuda", dtype=torch.int32)
    rel = torch.randint(0, n_rel, (n_edges,), generator=g, device="cuda", dtype=torch.int32)
    w = torch.arange(1, n_nodes + 1, device="cuda", dtype=torch.float64).pow_(-float(tail_zipf))
    cdf = torch.cumsum(w, 0)
    cdf /= cdf[-1].clone()
    del w
    perm = torch.randperm(n_nodes, generator=g, device="cuda").to(torch.int32)
    tail = torch.empty(n_edges, dtype=torch.int32, device="cuda")
    slab = 1 << 24
    for e0 in range(0, n_edges, slab):
        u = torch.rand(min(slab, n_edges - e0), generator=g, device="cuda", dtype=torch.float64)
        ranks = torch.searchsorted(cdf, u).clamp_(max=n_nodes - 1)
        tail[e0:e0 + u.numel()] = perm[ranks]
    del cdf, perm
    return head, rel, tail


def stack_result(a, which, steps, warmup, bits=None, keep_graph=False):
    """configs[3] / configs[4]: a stack of layers, forward + ranking loss + backward: step time,
    saved-activation footprint, and the dominant kernel against its roofline."""
    import numpy as np
    import torch
    import paper_2212_04540_amd as tk
    from workloads import gen
    dev = "cuda"
    t_prep = time.perf_counter()
    if which == "config3":
        nu, ni, na = 70_000, 25_000, 90_000
        head, rel, tail = gen.user_item_entity_graph(nu, ni, na, 40, 3_000_000, 850_000, seed=0, zipf=1.2)
        n_nodes, n_rel, dims, bits, group, sample_hi = nu + ni + na, 42, [64, 64, 32, 16], 2, 64, nu + ni
        name = ("configs[3]: 3-layer KG GNN step on a 185k-node user-item-entity graph (3M KG triplets + "
                "2 x 850k interaction edges, Zipf 1.2), dims 64-64-32-16, INT2 group 64, BPR on 4096 triples")
        head, rel, tail = (torch.from_numpy(x).to(dev) for x in (head, rel, tail))
    else:
        n_nodes, n_rel, n_edges = C4_N, C4_R, C4_T
        head, rel, tail = device_kg_triplets(torch, n_nodes, n_rel, n_edges, 1.05, seed=0)
        dims, bits, group, sample_hi = [C4_D] * 3, bits or C4_BITS, C4_GROUP, n_nodes
        name = ("configs[4]: 20M entities x dim 128, 60 relations, 150M triplets (Zipf 1.05 tails), "
                f"two layers, saved activations {'fp32' if bits == 32 else 'INT%d group 128' % bits}")
    n_edges = head.numel()
    torch.cuda.synchronize()
    t_graph = time.perf_counter()
    graph = tk.Graph(n_nodes, n_rel, head, rel, tail)
    torch.cuda.synchronize()
    graph_s = time.perf_counter() - t_graph
    n_tails = int(torch.unique(tail).numel()) if keep_graph else 0
    del head, rel, tail
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    E0 = torch.randn((n_nodes, dims[0]), generator=g, device=dev) * 0.1
    params = [tuple(torch.from_numpy(x).to(dev) for x in gen.layer_params(n_rel, dims[l], dims[l], dims[l + 1], seed=20 + l))
              for l in range(len(dims) - 1)]
    rng = np.random.default_rng(5)
    u, p, n = (torch.from_numpy(rng.integers(0, sample_hi, 4096).astype(np.int32)).to(dev) for _ in range(3))
    stack = tk.KGStack(graph, dims, bits, group, SLOPE, save_H=not a.rebuild_H)
    if a.rebuild_H:
        name += "; contexts without Q(H) (H rebuilt in the backward pass)"
    prep_s = time.perf_counter() - t_prep
    torch.cuda.reset_peak_memory_stats()
    for i in range(warmup):
        stack.forward(E0, params, i, u, p, n)
        stack.backward(params)
    torch.cuda.synchronize()
    # timed region: events round the dominant kernel only; the per-kernel table comes from a
    # second, untimed pass with every launch bracketed (as in the configs[1] workload)
    tk.tinykg_profile_select("edge_bwd_kernel")
    tk.tinykg_profile_enable(True)
    t0 = time.perf_counter()
    for i in range(steps):
        stack.forward(E0, params, warmup + i, u, p, n)
        stack.backward(params)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    dom = tk.tinykg_profile_report()["edge_bwd_kernel"]
    tk.tinykg_profile_enable(False)
    breakdown_steps = min(steps, 3)
    tk.tinykg_profile_select(None)
    tk.tinykg_profile_enable(True)
    for i in range(breakdown_steps):
        stack.forward(E0, params, warmup + steps + i, u, p, n)
        stack.backward(params)
    torch.cuda.synchronize()
    rep = tk.tinykg_profile_report()
    tk.tinykg_profile_enable(False)
    bpa = bytes_per_activation(bits, group)
    alg = 0.0
    flops = 0.0
    for l in range(len(dims) - 1):
        d, do = dims[l], dims[l + 1]
        alg += n_edges * (4 * d + 12 + d * bpa + 12) + n_nodes * (4 * d + 4 * do + 2 * d * bpa + do / 8 + 4 * do + d * bpa + do / 8 + 4 * d)
        flops += edge_bwd_flops(n_edges, d)
    dom_ms = dom[1] / steps                      # all edge-backward launches of a step
    achieved = flops / (dom_ms * 1e-3) / 1e12
    res = {"workload": name, "steps": steps, "warmup": warmup, "ms_per_step": round(dt * 1e3, 3),
           "GB/s": round(alg / dt / 1e9, 2), "bits": bits, "group": group, "bytes_per_activation": bpa,
           "saved_context_bytes": stack.saved_context_bytes(), "fp32_context_bytes": stack.fp32_context_bytes(),
           "context_ratio": round(stack.fp32_context_bytes() / max(1, stack.saved_context_bytes()), 3),
           "readout_rows_bytes": stack.readout_rows_bytes(),
           "peak_device_bytes_torch": torch.cuda.max_memory_allocated(),
           "preparation_s": round(prep_s, 1), "graph_create_s": round(graph_s, 2),
           "roofline": {"kernel": "edge_bwd_kernel", "bound": "mfma", "achieved": round(achieved, 2),
                        "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / MFMA_FP32_PEAK_TFLOPS, 4),
                        "ms_per_step": round(dom_ms, 4), "launches_per_step": dom[0] / steps,
                        "note": "algorithmic fp32 flops (six k x d products per triplet and layer) over the "
                                "launches' HIP-event time inside the timed region"},
           "kernels": {k: {"launches_per_step": v[0] / breakdown_steps, "ms_per_step": round(v[1] / breakdown_steps, 4)}
                       for k, v in rep.items()},
           "kernels_note": f"per-kernel device times from a separate pass of {breakdown_steps} steps after the timed region"}
    del stack, E0, params
    torch.cuda.empty_cache()
    if keep_graph:
        return res, graph, n_tails
    graph.close()
    return res


def stack_workload(a, which):
    res = stack_result(a, which, a.steps, a.warmup, bits=a.bits or None)
    out = {"metric": METRIC, "value": res["GB/s"], "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
           "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {k: res[k] for k in ("workload", "bits", "group", "bytes_per_activation", "saved_context_bytes",
                                          "fp32_context_bytes", "context_ratio", "readout_rows_bytes",
                                          "peak_device_bytes_torch", "preparation_s", "graph_create_s")},
           "roofline": res["roofline"], "kernels": res["kernels"], "kernels_note": res["kernels_note"]}
    print(json.dumps(out))


# ------------------------------------------------------------------ configs[1] ----
def config1_result(a, tk, torch, inp):
    dev = "cuda"
    t = {k: torch.from_numpy(v).to(dev) for k, v in inp.items()}
    graph = tk.Graph(N, R, t["head"], t["rel"], t["tail"])
    saved = tk.SavedContext(N, D, D, BITS, GROUP, with_H=not a.rebuild_H)
    ws = torch.empty(max(tk.tinykg_kg_aggregate_workspace_bytes(graph, D, D, D, False),
                         tk.tinykg_kg_aggregate_workspace_bytes(graph, D, D, D, True)),
                     dtype=torch.uint8, device=dev)
    E_out = torch.empty((N, D), dtype=torch.float32, device=dev)
    grads = (torch.empty((N, D), dtype=torch.float32, device=dev), torch.empty_like(t["Wr"]),
             torch.empty_like(t["er"]), torch.empty_like(t["W"]))

    def step(i):
        tk.tinykg_kg_aggregate_fwd(graph, t["E"], t["Wr"], t["er"], t["W"], SLOPE, BITS, GROUP, 1 + 2 * i,
                                   saved, ws, E_out=E_out)
        tk.tinykg_kg_aggregate_bwd(graph, saved, t["Wr"], t["er"], t["W"], SLOPE, BITS, GROUP, t["G"], ws,
                                   out=grads)

    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    # HIP events around the dominant kernel's launches inside the timed region (events around
    # all launches of a step would cost about 4 % of it)
    tk.tinykg_profile_select("edge_bwd_kernel")
    tk.tinykg_profile_enable(True)
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(a.warmup + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    dom = tk.tinykg_profile_report()["edge_bwd_kernel"]
    tk.tinykg_profile_enable(False)
    # the other kernels: a second, untimed pass with every launch bracketed
    breakdown_steps = min(a.steps, 20)
    tk.tinykg_profile_select(None)
    tk.tinykg_profile_enable(True)
    for i in range(breakdown_steps):
        step(a.warmup + a.steps + i)
    torch.cuda.synchronize()
    rep = tk.tinykg_profile_report()
    tk.tinykg_profile_enable(False)
    # the same step captured once into a HIP graph and replayed (no launch gaps)
    graph_ms = None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        cg = torch.cuda.CUDAGraph()
        with torch.cuda.graph(cg):
            step(0)
        for _ in range(5):
            cg.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(a.steps):
            cg.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t1) / a.steps * 1e3
        del cg
    except Exception as e:   # capture is a measurement extra: report its absence, never fail the line
        graph_ms = f"not measured: {type(e).__name__}"

    ms_per_step = dt / a.steps * 1e3
    alg = step_algorithmic_bytes(saved_H=not a.rebuild_H)
    kernels = {k: {"launches_per_step": v[0] / breakdown_steps, "ms_per_step": round(v[1] / breakdown_steps, 4)}
               for k, v in rep.items()}
    assert dom[0] == a.steps
    dom_ms = dom[1] / dom[0]
    achieved = edge_bwd_flops() / (dom_ms * 1e-3) / 1e12
    tiles, one_tail = tile_stats(inp["rel"], inp["tail"])
    ex32, ex16 = edge_executed(tiles)
    pipe_floor_ms = (ex32 / (MFMA_FP32_PEAK_TFLOPS * 1e12) + ex16 / (MFMA_BF16_PEAK_TFLOPS * 1e12)) * 1e3
    traffic = profiled_traffic("edge_code_kernel")
    mfma_busy, wait = profiled_sq("edge_code_kernel")
    bpa = bytes_per_activation(BITS, GROUP)
    # the kernel's own compulsory bytes: two packed rows + ids, weights, flag byte and the head's grad_H row per
    # edge; one grad_E row per node; W_r once per relation
    kernel_alg = T * (2 * D * bpa + 3 * 4 + 2 * 4 + 1 + 4 * D) + N * 4 * D + R * D * D * 4
    out = {
        "metric": METRIC,
        "value": round(alg / (ms_per_step * 1e-3) / 1e9, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "dtype_note": "fp32 in, fp32 out, fp32 accumulation; the contractions (attention projections, dense "
                      "forward stage, and the backward products on saved codes) are evaluated as exact three-way "
                      "bfloat16 splits of their fp32 operands on the bf16 matrix cores (fp32 accuracy; integer "
                      "codes are exact bfloat16 values)",
        "data": "synthetic",
        "config": {"workload": "configs[1]: one KGAT-style attentive aggregation layer, forward+backward, "
                               "100k entities, dim 64, 16 relations, 1M triplets (Zipf 1.1 tails), "
                               "saved inputs INT2 group 64"
                               + ("; context without Q(H) (H rebuilt in the backward pass)" if a.rebuild_H else ""),
                   "bits": BITS, "group": GROUP, "bytes_per_activation": bpa,
                   "compression_ratio": round(4 / bpa, 3),
                   "algorithmic_bytes_per_step": alg,
                   "saved_context_bytes": saved.nbytes(), "fp32_context_bytes": 2 * N * D * 4 + N * D * 4},
        "frac_of_hbm_peak": round(alg / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 5),
        "ms_per_step_as_hip_graph": round(graph_ms, 4) if isinstance(graph_ms, float) else graph_ms,
        "launches_per_step": sum(k["launches_per_step"] for k in kernels.values()),
        "roofline": {"kernel": "edge_bwd_kernel", "rocprof_name": "edge_code_kernel<64, 2>", "bound": "mfma",
                     "achieved": round(achieved, 3), "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / MFMA_FP32_PEAK_TFLOPS, 4),
                     "avg_launch_ms": round(dom_ms, 4),
                     "algorithmic_flops": edge_bwd_flops(),
                     "executed": {"tiles": tiles, "one_tail_tiles": one_tail,
                                  "fp32_pipe_flops": ex32, "bf16_pipe_flops": ex16,
                                  "bf16_pipe_TFLOPs": round(ex16 / (dom_ms * 1e-3) / 1e12, 2),
                                  "matrix_pipe_floor_ms": round(pipe_floor_ms, 4),
                                  "frac_of_matrix_pipe_floor": round(pipe_floor_ms / dom_ms, 4)},
                     "mfma_busy": mfma_busy, "wait": wait,
                     "counters_source": "offline rocprofv3 --pmc run, profiles/" + os.path.basename(PROFILE_SQ),
                     "traffic": traffic,
                     "traffic_unit": "HBM-side bytes per launch (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, scaled by "
                                     "the calibration copy)",
                     "traffic_source": "offline rocprofv3 counters (not this run), profiles/" + os.path.basename(PROFILE_STEP),
                     "kernel_algorithmic_bytes": int(kernel_alg),
                     "traffic_over_algorithmic": round(traffic / kernel_alg, 2) if traffic else None,
                     "note": "frac prices the ALGORITHMIC fp32 flops (six k x d products for every triplet) over the "
                             "launch time against the fp32 matrix peak (157.3 TFLOP/s).  `executed` is what the kernel "
                             "runs: every product on the bf16 matrix cores (dense peak 2500 TFLOP/s) as exact bfloat16 "
                             "piece products -- three per product where one operand is a matrix of integer codes, six "
                             "otherwise -- at fp32 accuracy; frac_of_matrix_pipe_floor is the time that pipe needs at "
                             "its peak over the launch time (the kernel is bound by its vector work and LDS round "
                             "trips, not by the matrix pipe: see mfma_busy)"},
        "kernels": kernels,
        "kernels_note": f"per-kernel device times from a separate pass of {breakdown_steps} steps after the timed "
                        "region (every launch bracketed by HIP events); roofline.avg_launch_ms is measured "
                        "inside the timed region",
    }
    sc = rep["score_kernel"]
    out["score_kernels"] = {"launches_per_step": sc[0] / breakdown_steps, "avg_launch_ms": round(sc[1] / sc[0], 4),
                            "fp32_equivalent_TFLOPs": round(T * 2 * 2 * D * D / (sc[1] / sc[0] * 1e-3) / 1e12, 1),
                            "note": "two k x d projections per triplet on the bf16 matrix cores: six bfloat16 piece "
                                    "products each in the forward launch (fp32 rows), three in the backward launch "
                                    "(integer codes are exact bfloat16 values)"}
    graph.close()
    del saved, ws, E_out, grads, t
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="config1 only: leave out the sweep, config3, config4 and uniform_large objects")
    ap.add_argument("--workload", choices=["config1", "config2", "config3", "config4", "uniform", "batchnorm", "maxpool"], default="config1",
                    help="config1 (default: the headline step, with every other configuration as an extra object); "
                         "config2: the 9-cell compressor sweep with variance statistics; config3 / config4: the "
                         "multi-layer steps alone; uniform: the uniform-attention layer (--large: on the config4 graph)")
    ap.add_argument("--rebuild-H", action="store_true",
                    help="config1/3/4: save Q(E) and the mask only; the backward pass rebuilds H from E_hat")
    ap.add_argument("--bits", type=int, default=0, help="config4 only: 4 (default) or 32 for the fp32 run")
    ap.add_argument("--large", action="store_true", help="uniform only: run on the configs[4] graph")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the paper's method is single-GPU); "
                 "run with --gpus 1")

    import torch
    import paper_2212_04540_amd as tk
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    tk.lib()
    if a.workload == "config2":
        return compressor_sweep(a)
    if a.workload == "uniform":
        return uniform_workload(a)
    if a.workload == "batchnorm":
        return batchnorm_workload(a)
    if a.workload == "maxpool":
        return maxpool_workload(a)
    if a.workload != "config1":
        return stack_workload(a, a.workload)
    inp = make_inputs()
    out = config1_result(a, tk, torch, inp)
    if not a.no_extras:
        print("bench: configs[1] done, sweep next", file=sys.stderr, flush=True)
        cells, copy = sweep_cells(tk, torch, 10, with_variance=False)
        out["sweep"] = sweep_object(cells, copy, 10)
        ref = next(c for c in cells if c["bits"] == BITS and c["group"] == GROUP)
        out["compressor"] = {"workload": f"configs[2] cell: {C2_ROWS}x{C2_DIM} fp32 Student-t(3), INT{BITS}, group {GROUP}",
                             "bytes_per_element": 4 + bytes_per_activation(BITS, GROUP),
                             "quantize": ref["quantize_pack"], "dequantize": ref["unpack_dequantize"], "plain_copy": copy}
        print("bench: sweep done, configs[3] next", file=sys.stderr, flush=True)
        out["config3"] = stack_result(a, "config3", 20, 3)
        print("bench: configs[3] done, configs[4] next", file=sys.stderr, flush=True)
        c4, graph4, n_tails4 = stack_result(a, "config4", 3, 1, keep_graph=True)
        out["config4"] = c4
        print("bench: configs[4] done, uniform layer on its graph next", file=sys.stderr, flush=True)
        out["uniform_large"] = uniform_result(
            tk, torch, graph4, C4_N, C4_T, n_tails4, C4_D, C4_BITS, C4_GROUP, 5, 1,
            "uniform-attention layer (Eq. 2), forward+backward, on the configs[4] graph: 20M entities, dim 128, "
            "150M triplets (Zipf 1.05 tails), saved Q(H) INT4 group 128 (every tensor is 10 GB: nothing stays in "
            "the 256 MB Infinity Cache)")
        graph4.close()
        torch.cuda.empty_cache()
    if not a.no_cpu_baseline:
        print("bench: CPU oracle baseline next", file=sys.stderr, flush=True)
        out["cpu_baseline"] = cpu_baseline(inp, 1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
