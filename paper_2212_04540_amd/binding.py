"""Thin ctypes binding of libtinykg.so (the C ABI declared in include/tinykg.h).

Argument marshalling only: every step of the path runs inside the HIP library.
torch is used for device memory and for the current stream; tensors are never
touched by torch arithmetic here.  There is no CPU fallback: if the library is
missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtinykg.so")
_lib = None

ROUND_STOCHASTIC = 0
ROUND_NEAREST = 1

EXPORTS = [
    "tinykg_status_string", "tinykg_packed_bytes", "tinykg_num_groups", "tinykg_quantize",
    "tinykg_quantize_ex", "tinykg_quantize_bf16", "tinykg_dequantize", "tinykg_graph_create", "tinykg_graph_destroy",
    "tinykg_graph_num_nodes", "tinykg_graph_num_edges", "tinykg_kg_aggregate_workspace_bytes",
    "tinykg_kg_aggregate_fwd", "tinykg_kg_aggregate_bwd", "tinykg_kg_uniform_fwd",
    "tinykg_kg_uniform_bwd", "tinykg_profile_enable", "tinykg_profile_select",
    "tinykg_profile_report", "tinykg_profile_copy", "tinykg_bpr_loss", "tinykg_bpr_grad",
    "tinykg_gather_rows", "tinykg_scatter_add_rows", "tinykg_fill_zero", "tinykg_readout_ids",
    "tinykg_batchnorm_workspace_bytes", "tinykg_batchnorm_fwd", "tinykg_batchnorm_bwd", "tinykg_batchnorm_bwd_static",
    "tinykg_kg_max_arg_bytes", "tinykg_kg_max_workspace_bytes", "tinykg_kg_max_fwd", "tinykg_kg_max_bwd",
]


class TinyKGError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        msg = lib().tinykg_status_string(int(status)).decode()
        super().__init__(f"{what}: {msg} (status {int(status)})")


class Saved(C.Structure):
    """tinykg_saved: device pointers of one layer's saved context."""
    _fields_ = [("packed_E", C.c_void_p), ("gmin_E", C.c_void_p), ("gscale_E", C.c_void_p),
                ("packed_H", C.c_void_p), ("gmin_H", C.c_void_p), ("gscale_H", C.c_void_p),
                ("mask_J", C.c_void_p)]


def lib():
    """Load libtinykg.so (built in-tree by paper_2212_04540_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with "
                               "`python -m paper_2212_04540_amd.build` (hipcc, gfx950)")
        L = C.CDLL(_LIB_PATH)
        vp, i64, u64, i32, f32, sz = C.c_void_p, C.c_int64, C.c_uint64, C.c_int, C.c_float, C.c_size_t
        L.tinykg_status_string.argtypes = [C.c_int]
        L.tinykg_status_string.restype = C.c_char_p
        L.tinykg_packed_bytes.argtypes = [i64, i64, i32]
        L.tinykg_packed_bytes.restype = sz
        L.tinykg_num_groups.argtypes = [i64, i64, i32]
        L.tinykg_num_groups.restype = i64
        L.tinykg_quantize.argtypes = [vp, i64, i64, i32, i32, u64, vp, vp, vp, vp]
        L.tinykg_quantize_ex.argtypes = [vp, i64, i64, i32, i32, u64, u64, i32, vp, vp, vp, vp]
        L.tinykg_quantize_bf16.argtypes = [vp, i64, i64, i32, i32, u64, u64, i32, vp, vp, vp, vp]
        L.tinykg_dequantize.argtypes = [vp, vp, vp, i64, i64, i32, i32, vp, vp]
        if hasattr(L, "tinykg_graph_create"):
            L.tinykg_graph_create.argtypes = [i64, C.c_int32, i64, vp, vp, vp, vp, C.POINTER(vp)]
            L.tinykg_graph_destroy.argtypes = [vp]
            L.tinykg_graph_destroy.restype = None
            L.tinykg_graph_num_nodes.argtypes = [vp]
            L.tinykg_graph_num_nodes.restype = i64
            L.tinykg_graph_num_edges.argtypes = [vp]
            L.tinykg_graph_num_edges.restype = i64
            L.tinykg_kg_aggregate_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
            L.tinykg_kg_aggregate_workspace_bytes.restype = sz
            L.tinykg_kg_aggregate_fwd.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, f32, i32, i32,
                                                  u64, vp, C.POINTER(Saved), vp, sz, vp]
            L.tinykg_kg_aggregate_bwd.argtypes = [vp, C.POINTER(Saved), vp, vp, vp, i32, i32, i32,
                                                  f32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
            L.tinykg_kg_uniform_fwd.argtypes = [vp, vp, vp, i32, i32, f32, i32, i32, u64, vp,
                                                C.POINTER(Saved), vp, sz, vp]
            L.tinykg_kg_uniform_bwd.argtypes = [vp, C.POINTER(Saved), vp, i32, i32, f32, i32, i32,
                                                vp, vp, vp, vp, sz, vp]
        L.tinykg_profile_enable.argtypes = [i32]
        L.tinykg_profile_enable.restype = None
        L.tinykg_profile_select.argtypes = [C.c_char_p]
        L.tinykg_profile_select.restype = None
        L.tinykg_profile_report.argtypes = [C.c_char_p, sz]
        L.tinykg_profile_report.restype = sz
        L.tinykg_profile_copy.argtypes = [vp, vp, sz, vp]
        L.tinykg_bpr_loss.argtypes = [C.POINTER(vp), C.POINTER(i32), i32, i64, vp, vp, vp, i64, vp, vp, vp]
        L.tinykg_bpr_grad.argtypes = [vp, i32, i64, vp, vp, vp, vp, i64, i32, vp, vp]
        L.tinykg_gather_rows.argtypes = [vp, i32, vp, i64, vp, vp]
        L.tinykg_scatter_add_rows.argtypes = [vp, i32, vp, i64, vp, vp]
        L.tinykg_fill_zero.argtypes = [vp, i64, vp]
        L.tinykg_readout_ids.argtypes = [vp, vp, vp, i64, vp, vp, vp]
        L.tinykg_kg_max_arg_bytes.argtypes = [vp]
        L.tinykg_kg_max_workspace_bytes.argtypes = [vp, i32]
        L.tinykg_kg_max_workspace_bytes.restype = sz
        L.tinykg_kg_max_fwd.argtypes = [vp, vp, i32, vp, vp, vp]
        L.tinykg_kg_max_bwd.argtypes = [vp, vp, i32, vp, vp, vp, sz, vp]
        L.tinykg_batchnorm_workspace_bytes.argtypes = [i64, i32]
        L.tinykg_batchnorm_workspace_bytes.restype = sz
        L.tinykg_batchnorm_fwd.argtypes = [vp, i64, i32, vp, vp, f32, i32, i32, u64, vp, vp, vp, vp, vp, vp,
                                           vp, sz, vp]
        L.tinykg_batchnorm_bwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, vp, vp, vp, vp, vp, sz,
                                           vp]
        L.tinykg_batchnorm_bwd_static.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _dev(t, dtype, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{what}: expected a contiguous {dtype} CUDA tensor")
    return t


def _ok(status, what):
    if status != 0:
        raise TinyKGError(status, what)


def tinykg_packed_bytes(rows, dim, bits):
    return int(lib().tinykg_packed_bytes(rows, dim, bits))


def tinykg_num_groups(rows, dim, group):
    return int(lib().tinykg_num_groups(rows, dim, group))


def alloc_quantized(rows, dim, bits, group, device="cuda"):
    """Device buffers in tinykg_quantize's output layout: packed, gmin, gscale."""
    ng = max(tinykg_num_groups(rows, dim, group), 0)
    return (torch.empty(tinykg_packed_bytes(rows, dim, bits), dtype=torch.uint8, device=device),
            torch.empty(ng, dtype=torch.float32, device=device),
            torch.empty(ng, dtype=torch.float32, device=device))


def tinykg_quantize(act, bits, group, seed, out=None, first_index=0, rounding=ROUND_STOCHASTIC):
    """act: [rows, dim] fp32 CUDA tensor -> (packed uint8, gmin fp32, gscale fp32)."""
    _dev(act, torch.float32, "act")
    if act.dim() != 2:
        raise TypeError("act must be 2-D [rows, dim]")
    rows, dim = act.shape
    packed, gmin, gscale = out if out is not None else alloc_quantized(rows, dim, bits, group, act.device)
    st = lib().tinykg_quantize_ex(_ptr(act), rows, dim, bits, group, C.c_uint64(seed),
                                  C.c_uint64(first_index), rounding, _ptr(packed), _ptr(gmin),
                                  _ptr(gscale), _stream())
    _ok(st, "tinykg_quantize")
    return packed, gmin, gscale


def tinykg_dequantize(packed, gmin, gscale, rows, dim, bits, group, out=None):
    _dev(packed, torch.uint8, "packed")
    _dev(gmin, torch.float32, "gmin")
    _dev(gscale, torch.float32, "gscale")
    if out is None:
        out = torch.empty((rows, dim), dtype=torch.float32, device=packed.device)
    st = lib().tinykg_dequantize(_ptr(packed), _ptr(gmin), _ptr(gscale), rows, dim, bits, group,
                                 _ptr(out), _stream())
    _ok(st, "tinykg_dequantize")
    return out


def tinykg_profile_enable(on):
    lib().tinykg_profile_enable(1 if on else 0)


def tinykg_profile_select(name=None):
    """Record only the launches reported under `name` (None: every launch)."""
    lib().tinykg_profile_select(name.encode() if name else None)


def tinykg_profile_report():
    """{kernel name: (launches, total device ms)} over the launches recorded since enable(1)."""
    need = lib().tinykg_profile_report(None, 0)
    buf = C.create_string_buffer(need + 1)
    lib().tinykg_profile_report(buf, need + 1)
    out = {}
    for line in buf.value.decode().splitlines():
        name, n, ms = line.split()
        out[name] = (int(n), float(ms))
    return out


def tinykg_profile_copy(dst, src):
    """Plain copy kernel of known size (dst, src: same-size CUDA tensors)."""
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _ok(lib().tinykg_profile_copy(_ptr(dst), _ptr(src), nbytes, _stream()), "tinykg_profile_copy")


def tinykg_bpr_loss(layers, users, pos, neg, loss=None, coef=None):
    """layers: list of [n_nodes, d_l] fp32 CUDA tensors.  Returns (loss[1], coef[2*batch])."""
    n_nodes, batch = layers[0].shape[0], users.numel()
    for t in layers:
        _dev(t, torch.float32, "layer")
    for t, nm in ((users, "users"), (pos, "pos"), (neg, "neg")):
        _dev(t, torch.int32, nm)
    if loss is None:
        loss = torch.empty(1, dtype=torch.float32, device=users.device)
    if coef is None:
        coef = torch.empty(2 * batch, dtype=torch.float32, device=users.device)
    ptrs = (C.c_void_p * len(layers))(*[t.data_ptr() for t in layers])
    dims = (C.c_int * len(layers))(*[t.shape[1] for t in layers])
    _ok(lib().tinykg_bpr_loss(ptrs, dims, len(layers), n_nodes, _ptr(users), _ptr(pos), _ptr(neg), batch,
                              _ptr(loss), _ptr(coef), _stream()), "tinykg_bpr_loss")
    return loss, coef


def tinykg_bpr_grad(E_l, users, pos, neg, coef, grad, accumulate):
    _dev(E_l, torch.float32, "E_l")
    _dev(grad, torch.float32, "grad")
    _ok(lib().tinykg_bpr_grad(_ptr(E_l), E_l.shape[1], E_l.shape[0], _ptr(users), _ptr(pos), _ptr(neg),
                              _ptr(coef), users.numel(), 1 if accumulate else 0, _ptr(grad), _stream()),
        "tinykg_bpr_grad")
    return grad


def tinykg_gather_rows(E, idx, out=None):
    _dev(E, torch.float32, "E")
    _dev(idx, torch.int32, "idx")
    if out is None:
        out = torch.empty((idx.numel(), E.shape[1]), dtype=torch.float32, device=E.device)
    _ok(lib().tinykg_gather_rows(_ptr(E), E.shape[1], _ptr(idx), idx.numel(), _ptr(out), _stream()),
        "tinykg_gather_rows")
    return out


def tinykg_readout_ids(users, pos, neg):
    """ids = users | pos | neg and slot = 0 .. 3*batch - 1, both int32 [3*batch]."""
    for t, nm in ((users, "users"), (pos, "pos"), (neg, "neg")):
        _dev(t, torch.int32, nm)
    batch = users.numel()
    if pos.numel() != batch or neg.numel() != batch:
        raise ValueError("users, pos, neg must have the same length")
    ids = torch.empty(3 * batch, dtype=torch.int32, device=users.device)
    slot = torch.empty(3 * batch, dtype=torch.int32, device=users.device)
    _ok(lib().tinykg_readout_ids(_ptr(users), _ptr(pos), _ptr(neg), batch, _ptr(ids), _ptr(slot), _stream()),
        "tinykg_readout_ids")
    return ids, slot


def tinykg_fill_zero(dst):
    _dev(dst, torch.float32, "dst")
    _ok(lib().tinykg_fill_zero(_ptr(dst), dst.numel(), _stream()), "tinykg_fill_zero")
    return dst


def tinykg_scatter_add_rows(src, idx, dst):
    _dev(src, torch.float32, "src")
    _dev(dst, torch.float32, "dst")
    _dev(idx, torch.int32, "idx")
    _ok(lib().tinykg_scatter_add_rows(_ptr(src), src.shape[1], _ptr(idx), idx.numel(), _ptr(dst), _stream()),
        "tinykg_scatter_add_rows")
    return dst


class Graph:
    """Owner of a tinykg_graph handle."""

    def __init__(self, n_nodes, n_rel, head, rel, tail):
        for t, nm in ((head, "head"), (rel, "rel"), (tail, "tail")):
            _dev(t, torch.int32, nm)
        self.n_nodes, self.n_rel, self.n_edges = int(n_nodes), int(n_rel), int(head.numel())
        h = C.c_void_p()
        st = lib().tinykg_graph_create(self.n_nodes, self.n_rel, self.n_edges, _ptr(head), _ptr(rel),
                                       _ptr(tail), _stream(), C.byref(h))
        _ok(st, "tinykg_graph_create")
        self.handle = h

    def close(self):
        if getattr(self, "handle", None) is not None and self.handle:
            lib().tinykg_graph_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class SavedContext:
    """Device buffers of one layer's saved context + the tinykg_saved struct."""

    def __init__(self, n_nodes, d_in, d_out, bits, group, device="cuda", with_E=True, with_H=True):
        """with_E=False: the context of the uniform-attention layer (Q(H) and the mask only).
        with_H=False: Q(E) and the mask only; the attentive layer's backward pass rebuilds H."""
        self.n_nodes, self.d_in, self.d_out, self.bits, self.group = n_nodes, d_in, d_out, bits, group
        self.packed_E = self.gmin_E = self.gscale_E = None
        self.packed_H = self.gmin_H = self.gscale_H = None
        if not (with_E or with_H):
            raise ValueError("a saved context holds Q(E), Q(H) or both")
        if bits == 32:
            if with_E:
                self.packed_E = torch.empty(n_nodes * d_in * 4, dtype=torch.uint8, device=device)
            if with_H:
                self.packed_H = torch.empty(n_nodes * d_in * 4, dtype=torch.uint8, device=device)
        else:
            if with_E:
                self.packed_E, self.gmin_E, self.gscale_E = alloc_quantized(n_nodes, d_in, bits, group, device)
            if with_H:
                self.packed_H, self.gmin_H, self.gscale_H = alloc_quantized(n_nodes, d_in, bits, group, device)
        self.mask_J = torch.empty((n_nodes * d_out + 7) // 8, dtype=torch.uint8, device=device)
        self.struct = Saved(_ptr(self.packed_E), _ptr(self.gmin_E), _ptr(self.gscale_E),
                            _ptr(self.packed_H), _ptr(self.gmin_H), _ptr(self.gscale_H),
                            _ptr(self.mask_J))

    def nbytes(self):
        ts = [self.packed_E, self.gmin_E, self.gscale_E, self.packed_H, self.gmin_H, self.gscale_H,
              self.mask_J]
        return sum(t.numel() * t.element_size() for t in ts if t is not None)


def tinykg_kg_aggregate_workspace_bytes(graph, d_in, d_rel, d_out, is_bwd):
    return int(lib().tinykg_kg_aggregate_workspace_bytes(graph.handle, d_in, d_rel, d_out,
                                                         1 if is_bwd else 0))


def tinykg_kg_aggregate_fwd(graph, E, Wr, er, W, leaky_slope, bits, group, seed, saved, workspace,
                            E_out=None):
    for t, nm in ((E, "E"), (Wr, "Wr"), (er, "er"), (W, "W")):
        _dev(t, torch.float32, nm)
    d_in, d_rel, d_out = E.shape[1], Wr.shape[1], W.shape[0]
    if E_out is None:
        E_out = torch.empty((graph.n_nodes, d_out), dtype=torch.float32, device=E.device)
    st = lib().tinykg_kg_aggregate_fwd(graph.handle, _ptr(E), _ptr(Wr), _ptr(er), _ptr(W), d_in,
                                       d_rel, d_out, float(leaky_slope), bits, group,
                                       C.c_uint64(seed), _ptr(E_out), C.byref(saved.struct),
                                       _ptr(workspace), workspace.numel(), _stream())
    _ok(st, "tinykg_kg_aggregate_fwd")
    return E_out


def tinykg_kg_aggregate_bwd(graph, saved, Wr, er, W, leaky_slope, bits, group, grad_E_out,
                            workspace, out=None):
    for t, nm in ((Wr, "Wr"), (er, "er"), (W, "W"), (grad_E_out, "grad_E_out")):
        _dev(t, torch.float32, nm)
    d_in, d_rel, d_out = Wr.shape[2], Wr.shape[1], W.shape[0]
    if out is None:
        dev = Wr.device
        out = (torch.empty((graph.n_nodes, d_in), dtype=torch.float32, device=dev),
               torch.empty_like(Wr), torch.empty_like(er), torch.empty_like(W))
    gE, gWr, ger, gW = out
    st = lib().tinykg_kg_aggregate_bwd(graph.handle, C.byref(saved.struct), _ptr(Wr), _ptr(er),
                                       _ptr(W), d_in, d_rel, d_out, float(leaky_slope), bits, group,
                                       _ptr(grad_E_out), _ptr(gE), _ptr(gWr), _ptr(ger), _ptr(gW),
                                       _ptr(workspace), workspace.numel(), _stream())
    _ok(st, "tinykg_kg_aggregate_bwd")
    return gE, gWr, ger, gW


def tinykg_kg_uniform_fwd(graph, E, W, leaky_slope, bits, group, seed, saved, workspace, E_out=None):
    for t, nm in ((E, "E"), (W, "W")):
        _dev(t, torch.float32, nm)
    d_in, d_out = E.shape[1], W.shape[0]
    if E_out is None:
        E_out = torch.empty((graph.n_nodes, d_out), dtype=torch.float32, device=E.device)
    st = lib().tinykg_kg_uniform_fwd(graph.handle, _ptr(E), _ptr(W), d_in, d_out, float(leaky_slope),
                                     bits, group, C.c_uint64(seed), _ptr(E_out), C.byref(saved.struct),
                                     _ptr(workspace), workspace.numel(), _stream())
    _ok(st, "tinykg_kg_uniform_fwd")
    return E_out


def tinykg_kg_uniform_bwd(graph, saved, W, leaky_slope, bits, group, grad_E_out, workspace, out=None):
    for t, nm in ((W, "W"), (grad_E_out, "grad_E_out")):
        _dev(t, torch.float32, nm)
    d_in, d_out = W.shape[1], W.shape[0]
    if out is None:
        out = (torch.empty((graph.n_nodes, d_in), dtype=torch.float32, device=W.device),
               torch.empty_like(W))
    gE, gW = out
    st = lib().tinykg_kg_uniform_bwd(graph.handle, C.byref(saved.struct), _ptr(W), d_in, d_out,
                                     float(leaky_slope), bits, group, _ptr(grad_E_out), _ptr(gE),
                                     _ptr(gW), _ptr(workspace), workspace.numel(), _stream())
    _ok(st, "tinykg_kg_uniform_bwd")
    return gE, gW


def tinykg_quantize_bf16(act, bits, group, seed, out=None, first_index=0, rounding=ROUND_STOCHASTIC):
    """act: [rows, dim] torch.bfloat16 on the device."""
    _dev(act, torch.bfloat16, "act")
    rows, dim = act.shape
    if out is None:
        out = alloc_quantized(rows, dim, bits, group, act.device)
    packed, gmin, gscale = out
    st = lib().tinykg_quantize_bf16(_ptr(act), rows, dim, bits, group, C.c_uint64(seed),
                                    C.c_uint64(first_index), rounding, _ptr(packed), _ptr(gmin),
                                    _ptr(gscale), _stream())
    _ok(st, "tinykg_quantize_bf16")
    return packed, gmin, gscale


class NormContext:
    """Device buffers of a batch-norm layer's saved context: Q(x) (or an fp32 copy with
    bits == 32), the column means and inverse standard deviations, and the workspace."""

    def __init__(self, rows, dim, bits, group, device="cuda"):
        self.rows, self.dim, self.bits, self.group = rows, dim, bits, group
        self.gmin = self.gscale = None
        if bits == 32:
            self.packed = torch.empty(rows * dim * 4, dtype=torch.uint8, device=device)
        else:
            self.packed, self.gmin, self.gscale = alloc_quantized(rows, dim, bits, group, device)
        self.mean = torch.empty(dim, dtype=torch.float32, device=device)
        self.rstd = torch.empty(dim, dtype=torch.float32, device=device)
        nb = int(lib().tinykg_batchnorm_workspace_bytes(rows, dim))
        if nb == 0:
            raise TinyKGError(3, "tinykg_batchnorm_workspace_bytes")
        self.ws = torch.empty(nb, dtype=torch.uint8, device=device)

    def nbytes(self):
        ts = [self.packed, self.gmin, self.gscale, self.mean, self.rstd]
        return sum(t.numel() * t.element_size() for t in ts if t is not None)


def tinykg_batchnorm_fwd(x, gamma, beta, eps, bits, group, seed, ctx, y=None):
    for t, nm in ((x, "x"), (gamma, "gamma"), (beta, "beta")):
        _dev(t, torch.float32, nm)
    rows, dim = x.shape
    if y is None:
        y = torch.empty_like(x)
    st = lib().tinykg_batchnorm_fwd(_ptr(x), rows, dim, _ptr(gamma), _ptr(beta), float(eps), bits, group,
                                    C.c_uint64(seed), _ptr(y), _ptr(ctx.packed), _ptr(ctx.gmin),
                                    _ptr(ctx.gscale), _ptr(ctx.mean), _ptr(ctx.rstd), _ptr(ctx.ws),
                                    ctx.ws.numel(), _stream())
    _ok(st, "tinykg_batchnorm_fwd")
    return y


def tinykg_batchnorm_bwd(ctx, gamma, grad_y, out=None):
    _dev(gamma, torch.float32, "gamma")
    _dev(grad_y, torch.float32, "grad_y")
    if out is None:
        out = (torch.empty_like(grad_y), torch.empty_like(gamma), torch.empty_like(gamma))
    gx, gg, gb = out
    st = lib().tinykg_batchnorm_bwd(_ptr(ctx.packed), _ptr(ctx.gmin), _ptr(ctx.gscale), _ptr(ctx.mean),
                                    _ptr(ctx.rstd), _ptr(gamma), ctx.rows, ctx.dim, ctx.bits, ctx.group,
                                    _ptr(grad_y), _ptr(gx), _ptr(gg), _ptr(gb), _ptr(ctx.ws), ctx.ws.numel(),
                                    _stream())
    _ok(st, "tinykg_batchnorm_bwd")
    return gx, gg, gb


def tinykg_batchnorm_bwd_static(ctx, gamma, grad_y, out):
    """tinykg_batchnorm_bwd without a workspace (the library's fixed scratch array; dim <= 128).
    `out` = (grad_x, grad_gamma, grad_beta), allocated by the caller: nothing is allocated here."""
    _dev(gamma, torch.float32, "gamma")
    _dev(grad_y, torch.float32, "grad_y")
    gx, gg, gb = out
    for t, nm in ((gx, "grad_x"), (gg, "grad_gamma"), (gb, "grad_beta")):
        _dev(t, torch.float32, nm)
    st = lib().tinykg_batchnorm_bwd_static(_ptr(ctx.packed), _ptr(ctx.gmin), _ptr(ctx.gscale), _ptr(ctx.mean),
                                           _ptr(ctx.rstd), _ptr(gamma), ctx.rows, ctx.dim, ctx.bits, ctx.group,
                                           _ptr(grad_y), _ptr(gx), _ptr(gg), _ptr(gb), _stream())
    _ok(st, "tinykg_batchnorm_bwd_static")
    return gx, gg, gb


_ARG_DTYPES = {1: torch.uint8, 2: torch.int16, 4: torch.int32}


def tinykg_kg_max_fwd(graph, E, out=None):
    """M [n, d] fp32 and the saved edge numbers `arg` [n, d] (1, 2 or 4 bytes per element;
    torch has no unsigned 16 / 32-bit types: the signed tensors hold the unsigned bits)."""
    _dev(E, torch.float32, "E")
    d = E.shape[1]
    if out is None:
        nb = int(lib().tinykg_kg_max_arg_bytes(graph.handle))
        out = (torch.empty_like(E), torch.empty((graph.n_nodes, d), dtype=_ARG_DTYPES[nb], device=E.device))
    M, arg = out
    _ok(lib().tinykg_kg_max_fwd(graph.handle, _ptr(E), d, _ptr(M), _ptr(arg), _stream()), "tinykg_kg_max_fwd")
    return M, arg


def tinykg_kg_max_bwd(graph, arg, grad_M, workspace=None, out=None):
    _dev(grad_M, torch.float32, "grad_M")
    d = grad_M.shape[1]
    if workspace is None:
        workspace = torch.empty(int(lib().tinykg_kg_max_workspace_bytes(graph.handle, d)), dtype=torch.uint8,
                                device=grad_M.device)
    if out is None:
        out = torch.empty_like(grad_M)
    _ok(lib().tinykg_kg_max_bwd(graph.handle, _ptr(arg), d, _ptr(grad_M), _ptr(out), _ptr(workspace),
                                workspace.numel(), _stream()), "tinykg_kg_max_bwd")
    return out
