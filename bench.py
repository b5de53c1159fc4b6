#!/usr/bin/env python3
"""Benchmark of the TinyKG hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input:
the attentive aggregation layer's forward pass (which quantises and bit-packs the
saved activations E and H and keeps a 1-bit mask of J) followed by its backward
pass (which unpacks and dequantises them inside its gathers), on the 100k-entity /
1M-triplet configuration.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is algorithmic bytes per step / step time; the
`roofline` object prices the dominant kernel of the step against its own bound;
`compressor` reports the standalone quantize+pack / unpack+dequantize kernels on
the 2 GiB heavy-tailed activation (HBM-bound, the streaming roofline of the
method); `cpu_baseline` times the CPU oracle on the same workload.
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

# configs[1]
N, D, R, T = 100_000, 64, 16, 1_000_000
BITS, GROUP, SLOPE = 2, 64, 0.2
# configs[2] (one cell of the sweep is timed by default: INT2, group 64)
C2_ROWS, C2_DIM = 1 << 23, 64


def bytes_per_activation(bits, group):
    return bits / 8 + 8 / group


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


def edge_bwd_flops():
    """Contractions of the edge-level backward kernel: per triplet six k x d products
    (recompute W_r e_t and W_r e_h, W_r^T grad_a, W_r^T grad_b, two outer products)."""
    return T * 6 * 2 * D * D


PROFILE_SUMMARY = os.path.join(ROOT, "profiles", "aggregation_step_configs1_and_compressor_configs2.txt")


def profiled_traffic(kernel, summary=None):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by what the counter reads for a copy of known
    size): measured offline with the commands that file lists, not in this run."""
    try:
        rows = [l.split() for l in open(summary or PROFILE_SUMMARY) if l.startswith(kernel + "<") and len(l.split()) >= 6]
        tot = [(float(r[-2]) + float(r[-1])) * 1e6 for r in rows if r[-1] != "nan" and r[-2] != "nan"]
        return round(max(tot)) if tot else None
    except (OSError, ValueError):
        return None


def make_inputs(torch):
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


def compressor_line(tk, torch, iters=20):
    """quantize+pack and unpack+dequantize on the 2 GiB Student-t activation."""
    x = student_t_matrix(torch, C2_ROWS, C2_DIM)
    n = x.numel()
    buf = tk.alloc_quantized(C2_ROWS, C2_DIM, BITS, GROUP)
    out = torch.empty_like(x)
    for _ in range(3):
        tk.tinykg_quantize(x, BITS, GROUP, 1, out=buf)
        tk.tinykg_dequantize(*buf, C2_ROWS, C2_DIM, BITS, GROUP, out=out)
    torch.cuda.synchronize()
    tk.tinykg_profile_enable(True)
    for _ in range(5):
        tk.tinykg_profile_copy(out, x)      # plain copy of known size: practical HBM ceiling
    for _ in range(iters):
        tk.tinykg_quantize(x, BITS, GROUP, 1, out=buf)
        tk.tinykg_dequantize(*buf, C2_ROWS, C2_DIM, BITS, GROUP, out=out)
    torch.cuda.synchronize()
    rep = tk.tinykg_profile_report()
    tk.tinykg_profile_enable(False)
    bpe = 4 + bytes_per_activation(BITS, GROUP)
    res = {"workload": f"configs[2] cell: {C2_ROWS}x{C2_DIM} fp32 Student-t(3), INT{BITS}, group {GROUP}",
           "bytes_per_element": bpe}
    for key, name in (("quantize", "quantize_kernel"), ("dequantize", "dequantize_kernel")):
        cnt, ms = rep[name]
        gbs = n * bpe / (ms / cnt) / 1e6
        res[key] = {"ms": round(ms / cnt, 4), "GB/s": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    cnt, ms = rep["calibration_copy_kernel"]
    gbs = 2 * n * 4 / (ms / cnt) / 1e6
    res["plain_copy"] = {"ms": round(ms / cnt, 4), "GB/s": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)}
    del x, out, buf
    torch.cuda.empty_cache()
    return res


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


def compressor_sweep(a):
    """configs[2]: the 9 cells bits x group on the 2 GiB heavy-tailed activation.  Pack and
    unpack are fused into quantize / dequantize and are not separately observable."""
    import torch
    import paper_2212_04540_amd as tk
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
            for i in range(a.steps):
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
            cell["variance"] = variance_stats(tk, torch, sub, bits, group)
            cells.append(cell)
            del buf
    ref = next(c for c in cells if c["bits"] == BITS and c["group"] == GROUP)
    print(json.dumps({
        "metric": "quantize+pack and dequant+agg-bwd HBM GB/s (fraction of peak); bytes/activation",
        "value": ref["quantize_pack"]["GB/s"], "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": 2,
        "ms_per_step": ref["quantize_pack"]["ms"] + ref["unpack_dequantize"]["ms"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[2]: compressor sweep on {C2_ROWS}x{C2_DIM} fp32 Student-t(3) (2 GiB), "
                               "bits in {2,4,8} x group in {32,64,256}; value = quantize+pack of INT2/G64"},
        "roofline": {"kernel": "quantize_kernel", "bound": "hbm", "achieved": ref["quantize_pack"]["GB/s"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ref["quantize_pack"]["frac_of_hbm_peak"],
                     "traffic": profiled_traffic("quantize_kernel")},
        "cells": cells}))


def uniform_workload(a):
    """The uniform-attention layer (Eq. 2 as printed, row-normalised adjacency) on the
    configs[1] graph: no projections, so the step is bound by gathers and streams."""
    import torch
    import paper_2212_04540_amd as tk
    dev = "cuda"
    inp = make_inputs(torch)
    t = {k: torch.from_numpy(v).to(dev) for k, v in inp.items()}
    graph = tk.Graph(N, R, t["head"], t["rel"], t["tail"])
    saved = tk.SavedContext(N, D, D, BITS, GROUP, with_E=False)
    ws = torch.empty(max(tk.tinykg_kg_aggregate_workspace_bytes(graph, D, D, D, False),
                         tk.tinykg_kg_aggregate_workspace_bytes(graph, D, D, D, True)),
                     dtype=torch.uint8, device=dev)
    E_out = torch.empty((N, D), dtype=torch.float32, device=dev)
    grads = (torch.empty((N, D), dtype=torch.float32, device=dev), torch.empty_like(t["W"]))

    def step(i):
        tk.tinykg_kg_uniform_fwd(graph, t["E"], t["W"], SLOPE, BITS, GROUP, 1 + 2 * i, saved, ws, E_out=E_out)
        tk.tinykg_kg_uniform_bwd(graph, saved, t["W"], SLOPE, BITS, GROUP, t["G"], ws, out=grads)

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
    fwd_edge, fwd_node = 4 * D + 4, 4 * D + 4 * D + D * bpa + D / 8       # e_t row + tail id; E, E', Q(H), mask
    bwd_edge, bwd_node = 4 * D + 8, 4 * D + D * bpa + D / 8 + 4 * D       # grad_H row + ids; grad_E', H_hat, mask, grad_E
    alg = T * (fwd_edge + bwd_edge) + N * (fwd_node + bwd_node)
    kernels = {k: {"launches_per_step": v[0] / a.steps, "ms_per_step": round(v[1] / a.steps, 4)}
               for k, v in rep.items()}
    gather_ms = rep["uniform_bwd_kernel"][1] / rep["uniform_bwd_kernel"][0]
    gather_bytes = T * bwd_edge + N * 4 * D
    print(json.dumps({
        "metric": "quantize+pack and dequant+agg-bwd HBM GB/s (fraction of peak); bytes/activation",
        "value": round(alg / dt / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(dt * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "uniform-attention layer (Eq. 2, row-normalised adjacency), forward+backward, on "
                               "the configs[1] graph: 100k entities, dim 64, 1M triplets, saved Q(H) INT2 group 64",
                   "bits": BITS, "group": GROUP, "bytes_per_activation": bpa,
                   "algorithmic_bytes_per_step": alg, "saved_context_bytes": saved.nbytes()},
        "frac_of_hbm_peak": round(alg / dt / 1e9 / HBM_PEAK_GBS, 5),
        "roofline": {"kernel": "uniform_bwd_kernel", "bound": "hbm",
                     "achieved": round(gather_bytes / (gather_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(gather_bytes / (gather_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "traffic": None, "avg_launch_ms": round(gather_ms, 4)},
        "kernels": kernels}))
    graph.close()


def maxpool_workload(a):
    """Max-pooling aggregation (SPMM_MAX, Sec. 4.1.4 operator list) on the configs[1] graph:
    a gather and a scatter, no arithmetic to speak of."""
    import torch
    import paper_2212_04540_amd as tk
    dev = "cuda"
    inp = make_inputs(torch)
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
        "metric": "quantize+pack and dequant+agg-bwd HBM GB/s (fraction of peak); bytes/activation",
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
    print(json.dumps({
        "metric": "quantize+pack and dequant+agg-bwd HBM GB/s (fraction of peak); bytes/activation",
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
                     "traffic": profiled_traffic(dom, os.path.join(ROOT, "profiles", "batchnorm_2p23x64_int2_g64.txt")),
                     "avg_launch_ms": round(dom_ms, 4)},
        "kernels": kernels}))


def stack_workload(a, which):
    """configs[3] / configs[4]: a stack of layers, forward + ranking loss + backward.
    Reported for the step time and the saved-activation footprint; not the default."""
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
    else:
        n_nodes, n_rel, n_edges = 20_000_000, 60, 150_000_000
        head, rel, tail = gen.kg_triplets(n_nodes, n_rel, n_edges, seed=0, tail_zipf=1.05)
        dims, bits, group, sample_hi = [128, 128, 128], a.bits or 4, 128, n_nodes
        name = ("configs[4]: 20M entities x dim 128, 60 relations, 150M triplets (Zipf 1.05 tails), "
                f"two layers, saved activations {'fp32' if bits == 32 else 'INT%d group 128' % bits}")
    T = head.size
    graph = tk.Graph(n_nodes, n_rel, *(torch.from_numpy(x).to(dev) for x in (head, rel, tail)))
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
    for i in range(a.warmup):
        stack.forward(E0, params, i, u, p, n)
        stack.backward(params)
    torch.cuda.synchronize()
    # timed region: events round the dominant kernel only; the per-kernel table comes from a
    # second, untimed pass with every launch bracketed (as in the configs[1] workload)
    tk.tinykg_profile_select("edge_bwd_kernel")
    tk.tinykg_profile_enable(True)
    t0 = time.perf_counter()
    for i in range(a.steps):
        stack.forward(E0, params, a.warmup + i, u, p, n)
        stack.backward(params)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / a.steps
    dom = tk.tinykg_profile_report()["edge_bwd_kernel"]
    tk.tinykg_profile_enable(False)
    breakdown_steps = min(a.steps, 3)
    tk.tinykg_profile_select(None)
    tk.tinykg_profile_enable(True)
    for i in range(breakdown_steps):
        stack.forward(E0, params, a.warmup + a.steps + i, u, p, n)
        stack.backward(params)
    torch.cuda.synchronize()
    rep = tk.tinykg_profile_report()
    tk.tinykg_profile_enable(False)
    bpa = 4.0 if bits == 32 else bytes_per_activation(bits, group)
    alg = 0.0
    for l in range(len(dims) - 1):
        d, do = dims[l], dims[l + 1]
        alg += T * (4 * d + 12 + d * bpa + 12) + n_nodes * (4 * d + 4 * do + 2 * d * bpa + do / 8 + 4 * do + d * bpa + do / 8 + 4 * d)
    out = {"metric": "quantize+pack and dequant+agg-bwd HBM GB/s (fraction of peak); bytes/activation",
           "value": round(alg / dt / 1e9, 2), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
           "ms_per_step": round(dt * 1e3, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": name, "bits": bits, "group": group, "bytes_per_activation": bpa,
                      "saved_context_bytes": stack.saved_context_bytes(),
                      "fp32_context_bytes": stack.fp32_context_bytes(),
                      "readout_rows_bytes": stack.readout_rows_bytes(),
                      "peak_device_bytes_torch": torch.cuda.max_memory_allocated(),
                      "host_preparation_s": round(prep_s, 1)},
           "edge_bwd_kernel_ms_per_step_in_timed_region": round(dom[1] / a.steps, 4),
           "kernels": {k: {"launches_per_step": v[0] / breakdown_steps, "ms_per_step": round(v[1] / breakdown_steps, 4)}
                       for k, v in rep.items()},
           "kernels_note": f"per-kernel device times from a separate pass of {breakdown_steps} steps after the timed region"}
    graph.close()
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-compressor", action="store_true")
    ap.add_argument("--workload", choices=["config1", "config2", "config3", "config4", "uniform", "batchnorm", "maxpool"], default="config1",
                    help="config1 (default, the headline step); config2: the 9-cell compressor sweep; "
                         "config3 / config4: multi-layer steps; uniform: the uniform-attention "
                         "layer on the config1 graph")
    ap.add_argument("--rebuild-H", action="store_true",
                    help="config1/3/4: save Q(E) and the mask only; the backward pass rebuilds H from E_hat")
    ap.add_argument("--bits", type=int, default=0, help="config4 only: 4 (default) or 32 for the fp32 run")
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
    dev = "cuda"
    inp = make_inputs(torch)
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
    # all ten launches of a step would cost about 4 % of it)
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

    ms_per_step = dt / a.steps * 1e3
    alg = step_algorithmic_bytes(saved_H=not a.rebuild_H)
    kernels = {k: {"launches_per_step": v[0] / breakdown_steps, "ms_per_step": round(v[1] / breakdown_steps, 4)}
               for k, v in rep.items()}
    assert dom[0] == a.steps
    dom_ms = dom[1] / dom[0]
    achieved = edge_bwd_flops() / (dom_ms * 1e-3) / 1e12
    out = {
        "metric": "quantize+pack and dequant+agg-bwd HBM GB/s (fraction of peak); bytes/activation",
        "value": round(alg / (ms_per_step * 1e-3) / 1e9, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "dtype_note": "fp32 in, fp32 out, fp32 accumulation; the attention projections are evaluated as exact "
                      "three-way bfloat16 splits of their fp32 operands on the bf16 matrix cores (fp32 accuracy)",
        "data": "synthetic",
        "config": {"workload": "configs[1]: one KGAT-style attentive aggregation layer, forward+backward, "
                               "100k entities, dim 64, 16 relations, 1M triplets (Zipf 1.1 tails), "
                               "saved inputs INT2 group 64"
                               + ("; context without Q(H) (H rebuilt in the backward pass)" if a.rebuild_H else ""),
                   "bits": BITS, "group": GROUP, "bytes_per_activation": bytes_per_activation(BITS, GROUP),
                   "compression_ratio": round(4 / bytes_per_activation(BITS, GROUP), 3),
                   "algorithmic_bytes_per_step": alg,
                   "saved_context_bytes": saved.nbytes(), "fp32_context_bytes": 2 * N * D * 4 + N * D * 4},
        "frac_of_hbm_peak": round(alg / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 5),
        "roofline": {"kernel": "edge_bwd_kernel", "bound": "mfma", "achieved": round(achieved, 3),
                     "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / MFMA_FP32_PEAK_TFLOPS, 4),
                     "note": "fp32 flops of the kernel's six k x d contractions per triplet over its launch time, "
                             "against the fp32 matrix peak; four of the six run on the fp32 matrix cores, two (the "
                             "recomputation of a and b) as six bfloat16 piece products each on the bf16 matrix "
                             "cores (dense peak 2500 TFLOP/s), fp32 accumulation, fp32 accuracy.  These are the "
                             "ALGORITHMIC flops (six products for every triplet); for a 32-edge tile whose "
                             "edges share one tail (54 % of the tiles of this graph) the kernel forms the "
                             "two tail-side products W_r^T grad_a and grad_a e_t^T once per tile from the "
                             "sum of grad_a over the tile, so it executes fewer",
                     "traffic": profiled_traffic("edge_wave_kernel"),
                     "traffic_unit": "HBM bytes per launch (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; "
                                     "summary under profiles/)",
                     "avg_launch_ms": round(dom_ms, 4)},
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
    if not a.no_compressor:
        out["compressor"] = compressor_line(tk, torch)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, 1)
    graph.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
