"""numpy-facing wrapper of the CPU oracle (oracle/libtinykg_ref.so).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.
All arrays are host numpy arrays; every function returns fresh arrays.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _declare(_lib)
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _declare(L):
    u8p, f32p, u32p = C.POINTER(C.c_uint8), C.POINTER(C.c_float), C.POINTER(C.c_uint32)
    L.tinykg_ref_philox4x32_10.argtypes = [u32p, u32p, u32p]
    L.tinykg_ref_philox4x32_10.restype = None
    L.tinykg_ref_noise16.argtypes = [C.c_uint64, C.c_uint64]
    L.tinykg_ref_noise16.restype = C.c_uint32
    L.tinykg_ref_pack.argtypes = [u8p, C.c_int64, C.c_int, u8p]
    L.tinykg_ref_unpack.argtypes = [u8p, C.c_int64, C.c_int, u8p]
    L.tinykg_ref_quantize_codes.argtypes = [f32p, C.c_int64, C.c_int, C.c_int, C.c_uint64,
                                            C.c_uint64, C.c_int, u8p, f32p, f32p]
    L.tinykg_ref_quantize.argtypes = [f32p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_uint64,
                                      C.c_uint64, C.c_int, u8p, f32p, f32p]
    L.tinykg_ref_dequantize.argtypes = [u8p, f32p, f32p, C.c_int64, C.c_int64, C.c_int, C.c_int,
                                        f32p]


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid arguments")


def philox4x32_10(ctr, key):
    ctr = np.ascontiguousarray(ctr, dtype=np.uint32)
    key = np.ascontiguousarray(key, dtype=np.uint32)
    assert ctr.shape == (4,) and key.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    lib().tinykg_ref_philox4x32_10(_p(ctr, C.c_uint32), _p(key, C.c_uint32), _p(out, C.c_uint32))
    return out


def noise16(seed, index):
    return int(lib().tinykg_ref_noise16(C.c_uint64(seed), C.c_uint64(index)))


def pack(codes, bits):
    codes = np.ascontiguousarray(codes, dtype=np.uint8).ravel()
    out = np.empty(codes.size * bits // 8, dtype=np.uint8)
    _check(lib().tinykg_ref_pack(_p(codes, C.c_uint8), codes.size, bits, _p(out, C.c_uint8)), "pack")
    return out


def unpack(packed, n, bits):
    packed = np.ascontiguousarray(packed, dtype=np.uint8).ravel()
    assert packed.size * 8 >= n * bits
    out = np.empty(n, dtype=np.uint8)
    _check(lib().tinykg_ref_unpack(_p(packed, C.c_uint8), n, bits, _p(out, C.c_uint8)), "unpack")
    return out


def quantize_codes(act, bits, group, seed, first_index=0, rounding=0):
    """Unpacked codes (uint8, one per element), gmin, gscale."""
    act = np.ascontiguousarray(act, dtype=np.float32)
    n = act.size
    if group <= 0 or n % group:
        raise ValueError("oracle quantize: size not a multiple of the group")
    codes = np.empty(n, dtype=np.uint8)
    gmin = np.empty(n // group, dtype=np.float32)
    gscale = np.empty(n // group, dtype=np.float32)
    _check(lib().tinykg_ref_quantize_codes(_p(act, C.c_float), n, bits, group, C.c_uint64(seed),
                                           C.c_uint64(first_index), rounding, _p(codes, C.c_uint8),
                                           _p(gmin, C.c_float), _p(gscale, C.c_float)),
           "quantize_codes")
    return codes, gmin, gscale


def quantize(act, bits, group, seed, first_index=0, rounding=0):
    """Packed bit-stream (uint8), gmin, gscale for a 2-D (or flat) fp32 array."""
    act = np.ascontiguousarray(act, dtype=np.float32)
    rows, dim = (act.shape if act.ndim == 2 else (1, act.size))
    n = act.size
    if group <= 0 or n % group:
        raise ValueError("oracle quantize: size not a multiple of the group")
    packed = np.empty(n * bits // 8, dtype=np.uint8)
    gmin = np.empty(n // group, dtype=np.float32)
    gscale = np.empty(n // group, dtype=np.float32)
    _check(lib().tinykg_ref_quantize(_p(act, C.c_float), rows, dim, bits, group, C.c_uint64(seed),
                                     C.c_uint64(first_index), rounding, _p(packed, C.c_uint8),
                                     _p(gmin, C.c_float), _p(gscale, C.c_float)), "quantize")
    return packed, gmin, gscale


def dequantize(packed, gmin, gscale, rows, dim, bits, group):
    packed = np.ascontiguousarray(packed, dtype=np.uint8).ravel()
    gmin = np.ascontiguousarray(gmin, dtype=np.float32)
    gscale = np.ascontiguousarray(gscale, dtype=np.float32)
    n = rows * dim
    assert packed.size == n * bits // 8 and gmin.size == n // group == gscale.size
    out = np.empty((rows, dim), dtype=np.float32)
    _check(lib().tinykg_ref_dequantize(_p(packed, C.c_uint8), _p(gmin, C.c_float),
                                       _p(gscale, C.c_float), rows, dim, bits, group,
                                       _p(out, C.c_float)), "dequantize")
    return out


# ------------------------------------------------ attentive aggregation ------
def _declare_agg(L):
    i32p, f32p, f64p, u8p = (C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_double),
                             C.POINTER(C.c_uint8))
    L.tinykg_ref_kg_aggregate_fwd_f64.argtypes = [
        C.c_int64, C.c_int, C.c_int64, i32p, i32p, i32p, f64p, f64p, f64p, f64p, C.c_int, C.c_int,
        C.c_int, C.c_double, C.c_int, f64p, f64p, f64p, f64p]
    L.tinykg_ref_kg_aggregate_bwd_f64.argtypes = [
        C.c_int64, C.c_int, C.c_int64, i32p, i32p, i32p, f64p, f64p, u8p, f64p, f64p, f64p,
        C.c_int, C.c_int, C.c_int, C.c_double, f64p, C.c_int, f64p, f64p, f64p, f64p]
    L.tinykg_ref_kg_aggregate_fwd.argtypes = [
        C.c_int64, C.c_int, C.c_int64, i32p, i32p, i32p, f32p, f32p, f32p, f32p, C.c_int, C.c_int,
        C.c_int, C.c_float, C.c_int, f32p, f32p, u8p]
    L.tinykg_ref_kg_aggregate_bwd.argtypes = [
        C.c_int64, C.c_int, C.c_int64, i32p, i32p, i32p, f32p, f32p, u8p, f32p, f32p, f32p,
        C.c_int, C.c_int, C.c_int, C.c_float, f32p, C.c_int, f32p, f32p, f32p, f32p]


_agg_declared = False


def _agg():
    global _agg_declared
    L = lib()
    if not _agg_declared:
        _declare_agg(L)
        _agg_declared = True
    return L


def _coo(head, rel, tail):
    head = np.ascontiguousarray(head, dtype=np.int32)
    rel = np.ascontiguousarray(rel, dtype=np.int32)
    tail = np.ascontiguousarray(tail, dtype=np.int32)
    assert head.shape == rel.shape == tail.shape and head.ndim == 1
    return head, rel, tail


def default_threads():
    return max(1, min(16, os.cpu_count() or 1))


def aggregate_fwd_f64(n_nodes, head, rel, tail, E, Wr, er, W, slope, threads=1):
    """Double-precision layer forward.  Returns E_out, H, J, pi (per triplet)."""
    head, rel, tail = _coo(head, rel, tail)
    E, Wr, er, W = (np.ascontiguousarray(a, dtype=np.float64) for a in (E, Wr, er, W))
    R, k, d = Wr.shape
    dout = W.shape[0]
    assert E.shape == (n_nodes, d) and er.shape == (R, k) and W.shape == (dout, d)
    Eout = np.empty((n_nodes, dout)); H = np.empty((n_nodes, d)); J = np.empty((n_nodes, dout))
    pi = np.empty(head.size)
    D = C.c_double
    _check(_agg().tinykg_ref_kg_aggregate_fwd_f64(
        n_nodes, R, head.size, _p(head, C.c_int32), _p(rel, C.c_int32), _p(tail, C.c_int32),
        _p(E, D), _p(Wr, D), _p(er, D), _p(W, D), d, k, dout, float(slope), threads,
        _p(Eout, D), _p(H, D), _p(J, D), _p(pi, D)), "aggregate_fwd_f64")
    return Eout, H, J, pi


def aggregate_bwd_f64(n_nodes, head, rel, tail, Ehat, Hhat, mask, Wr, er, W, slope, gEout,
                      threads=1):
    """Double-precision layer backward at the given saved tensors.
    mask: [n_nodes, d_out] array, nonzero where J > 0.  Returns gE, gWr, ger, gW."""
    head, rel, tail = _coo(head, rel, tail)
    Ehat, Hhat, Wr, er, W, gEout = (np.ascontiguousarray(a, dtype=np.float64)
                                    for a in (Ehat, Hhat, Wr, er, W, gEout))
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    R, k, d = Wr.shape
    dout = W.shape[0]
    assert Ehat.shape == (n_nodes, d) == Hhat.shape and mask.shape == (n_nodes, dout) == gEout.shape
    gE = np.empty((n_nodes, d)); gWr = np.empty((R, k, d)); ger = np.empty((R, k))
    gW = np.empty((dout, d))
    D = C.c_double
    _check(_agg().tinykg_ref_kg_aggregate_bwd_f64(
        n_nodes, R, head.size, _p(head, C.c_int32), _p(rel, C.c_int32), _p(tail, C.c_int32),
        _p(Ehat, D), _p(Hhat, D), _p(mask, C.c_uint8), _p(Wr, D), _p(er, D), _p(W, D), d, k, dout,
        float(slope), _p(gEout, D), threads, _p(gE, D), _p(gWr, D), _p(ger, D), _p(gW, D)),
        "aggregate_bwd_f64")
    return gE, gWr, ger, gW


def aggregate_fwd(n_nodes, head, rel, tail, E, Wr, er, W, slope, threads=1):
    """fp32-in / fp32-out layer forward.  Returns E_out, H (fp32) and the boolean
    mask J > 0 as uint8 [n_nodes, d_out]."""
    head, rel, tail = _coo(head, rel, tail)
    E, Wr, er, W = (np.ascontiguousarray(a, dtype=np.float32) for a in (E, Wr, er, W))
    R, k, d = Wr.shape
    dout = W.shape[0]
    assert E.shape == (n_nodes, d) and er.shape == (R, k) and W.shape == (dout, d)
    Eout = np.empty((n_nodes, dout), np.float32); H = np.empty((n_nodes, d), np.float32)
    mask = np.empty((n_nodes, dout), np.uint8)
    F = C.c_float
    _check(_agg().tinykg_ref_kg_aggregate_fwd(
        n_nodes, R, head.size, _p(head, C.c_int32), _p(rel, C.c_int32), _p(tail, C.c_int32),
        _p(E, F), _p(Wr, F), _p(er, F), _p(W, F), d, k, dout, float(slope), threads,
        _p(Eout, F), _p(H, F), _p(mask, C.c_uint8)), "aggregate_fwd")
    return Eout, H, mask


def aggregate_bwd(n_nodes, head, rel, tail, Ehat, Hhat, mask, Wr, er, W, slope, gEout, threads=1):
    """fp32-in / fp32-out layer backward at the given saved tensors."""
    head, rel, tail = _coo(head, rel, tail)
    Ehat, Hhat, Wr, er, W, gEout = (np.ascontiguousarray(a, dtype=np.float32)
                                    for a in (Ehat, Hhat, Wr, er, W, gEout))
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    R, k, d = Wr.shape
    dout = W.shape[0]
    assert Ehat.shape == (n_nodes, d) == Hhat.shape and mask.shape == (n_nodes, dout) == gEout.shape
    gE = np.empty((n_nodes, d), np.float32); gWr = np.empty((R, k, d), np.float32)
    ger = np.empty((R, k), np.float32); gW = np.empty((dout, d), np.float32)
    F = C.c_float
    _check(_agg().tinykg_ref_kg_aggregate_bwd(
        n_nodes, R, head.size, _p(head, C.c_int32), _p(rel, C.c_int32), _p(tail, C.c_int32),
        _p(Ehat, F), _p(Hhat, F), _p(mask, C.c_uint8), _p(Wr, F), _p(er, F), _p(W, F), d, k, dout,
        float(slope), _p(gEout, F), threads, _p(gE, F), _p(gWr, F), _p(ger, F), _p(gW, F)),
        "aggregate_bwd")
    return gE, gWr, ger, gW


# ---- the saved context of one layer (Fig. 1): Q(E; seed), Q(H; seed+1), 1-bit mask
def save_context(E, H, mask, bits, group, seed, keep_H=True):
    """Compress what the backward pass needs.  bits == 32 keeps fp32 copies.
    keep_H=False: H is left out (the backward pass rebuilds it from E_hat, see rebuild_H)."""
    E = np.ascontiguousarray(E, dtype=np.float32)
    H = np.ascontiguousarray(H, dtype=np.float32)
    mask_bits = pack((np.ascontiguousarray(mask) != 0).astype(np.uint8), 1)
    if bits == 32:
        ctx = {"bits": 32, "E": E.copy(), "mask": mask_bits}
        if keep_H:
            ctx["H"] = H.copy()
        return ctx
    pE, mnE, scE = quantize(E, bits, group, seed)
    ctx = {"bits": bits, "group": group, "packed_E": pE, "gmin_E": mnE, "gscale_E": scE,
           "mask": mask_bits}
    if keep_H:
        pH, mnH, scH = quantize(H, bits, group, (seed + 1) & (2 ** 64 - 1))
        ctx.update(packed_H=pH, gmin_H=mnH, gscale_H=scH)
    return ctx


def restore_context(ctx, n_nodes, d_in, d_out):
    """E_hat, H_hat (fp32; None when H was not saved) and the unpacked mask [n_nodes, d_out]."""
    mask = unpack(ctx["mask"], n_nodes * d_out, 1).reshape(n_nodes, d_out)
    if ctx["bits"] == 32:
        return ctx["E"], ctx.get("H"), mask
    b, g = ctx["bits"], ctx["group"]
    Eh = dequantize(ctx["packed_E"], ctx["gmin_E"], ctx["gscale_E"], n_nodes, d_in, b, g)
    Hh = None
    if "packed_H" in ctx:
        Hh = dequantize(ctx["packed_H"], ctx["gmin_H"], ctx["gscale_H"], n_nodes, d_in, b, g)
    return Eh, Hh, mask


def rebuild_H(n_nodes, head, rel, tail, Ehat, Wr, er, W, slope, threads=1):
    """The variant that saves Q(E) and the mask only: the second stage of Eq. 2 is run
    again on E_hat, H~ = e^_h + sum_j pi_j(E_hat) e^_t, and stands where H_hat stood in the
    backward pass (the mask stays the forward pass's own)."""
    return aggregate_fwd(n_nodes, head, rel, tail, Ehat, Wr, er, W, slope, threads)[1]


# ------------------------------------------------ readout + ranking loss ------
def bpr_loss_grad(layers, users, pos, neg):
    """Readout = concatenation of the layer tensors (Sec. 3.2, layer-aggregation);
    y(u, i) = <z_u, z_i>; loss = mean_b softplus(y(u_b, neg_b) - y(u_b, pos_b)).
    Plain numpy, float64.  layers: list of [n, d_l] arrays.  Returns the loss, the
    per-sample coefficient sigmoid(y_neg - y_pos) / batch, and one gradient array per
    layer (same shapes as `layers`)."""
    Z = np.concatenate([np.asarray(a, dtype=np.float64) for a in layers], axis=1)
    users, pos, neg = (np.asarray(a, dtype=np.int64) for a in (users, pos, neg))
    batch = users.size
    diff = np.einsum("bd,bd->b", Z[users], Z[neg] - Z[pos])
    loss = np.mean(np.logaddexp(0.0, diff))
    coef = 1.0 / (1.0 + np.exp(-diff)) / batch
    gZ = np.zeros_like(Z)
    np.add.at(gZ, users, coef[:, None] * (Z[neg] - Z[pos]))
    np.add.at(gZ, pos, -coef[:, None] * Z[users])
    np.add.at(gZ, neg, coef[:, None] * Z[users])
    grads, o = [], 0
    for a in layers:
        d = np.asarray(a).shape[1]
        grads.append(gZ[:, o:o + d])
        o += d
    return loss, coef, grads


def stack_step(n_nodes, head, rel, tail, E0, params, slope, bits, group, seed, users, pos, neg,
               threads=1):
    """One training step of a stack of layers, every stage from the oracle's own
    values: forward through the layers (saving compressed contexts: layer l uses
    seeds seed+2l and seed+2l+1), readout + loss, backward.  Returns a dict."""
    acts = [np.ascontiguousarray(E0, dtype=np.float32)]
    ctxs = []
    for l, (Wr, er, W) in enumerate(params):
        Eo, H, mask = aggregate_fwd(n_nodes, head, rel, tail, acts[-1], Wr, er, W, slope, threads)
        ctxs.append(save_context(acts[-1], H, mask, bits, group, seed + 2 * l))
        acts.append(Eo)
    loss, coef, rgrads = bpr_loss_grad(acts, users, pos, neg)
    g = rgrads[-1].astype(np.float32)
    layer_grads = [None] * len(acts)
    layer_grads[-1] = g
    pgrads = [None] * len(params)
    for l in range(len(params) - 1, -1, -1):
        Wr, er, W = params[l]
        d_in, d_out = acts[l].shape[1], acts[l + 1].shape[1]
        Eh, Hh, mk = restore_context(ctxs[l], n_nodes, d_in, d_out)
        gE, gWr, ger, gW = aggregate_bwd(n_nodes, head, rel, tail, Eh, Hh, mk, Wr, er, W, slope, g, threads)
        g = (gE.astype(np.float64) + rgrads[l]).astype(np.float32)
        layer_grads[l] = g
        pgrads[l] = (gWr, ger, gW)
    return {"acts": acts, "ctxs": ctxs, "loss": loss, "coef": coef, "layer_grads": layer_grads,
            "param_grads": pgrads}


# ------------------------------------------------ uniform-attention layer ------
def _uniform_adjacency(n_nodes, head, tail):
    """Row-normalised adjacency A_hat[h, t] = (number of edges h -> t) / deg(h) as a scipy
    CSR matrix (float64); rows of nodes without out-edges are empty."""
    import scipy.sparse as sp
    head = np.asarray(head, dtype=np.int64)
    tail = np.asarray(tail, dtype=np.int64)
    deg = np.bincount(head, minlength=n_nodes).astype(np.float64)
    w = 1.0 / deg[head] if head.size else np.zeros(0)
    return sp.csr_matrix((w, (head, tail)), shape=(n_nodes, n_nodes))


def uniform_fwd(n_nodes, head, tail, E, W, slope):
    """E' = LeakyReLU((E + A_hat E) W^T) -- Eq. (2) as printed (spmm, mm, activation) with
    the row-normalised adjacency plus self term; every step in float64, outputs rounded
    to fp32 once.  Returns E' [n, d_out], H = E + A_hat E [n, d_in] and the mask [J > 0]."""
    A = _uniform_adjacency(n_nodes, head, tail)
    E64 = np.asarray(E, dtype=np.float64)
    H = E64 + A @ E64
    J = H @ np.asarray(W, dtype=np.float64).T
    out = np.where(J > 0, J, np.float64(slope) * J)
    return out.astype(np.float32), H.astype(np.float32), (J > 0).astype(np.uint8)


def uniform_bwd(n_nodes, head, tail, Hhat, mask, W, slope, gEout):
    """Backward of Eq. (2) at the saved context (H_hat, mask): grad_J = grad_E' * (mask ? 1 :
    slope); grad_W = grad_J^T H_hat; grad_H = grad_J W; grad_E = grad_H + A_hat^T grad_H.
    float64 throughout, outputs rounded to fp32 once."""
    A = _uniform_adjacency(n_nodes, head, tail)
    gJ = np.asarray(gEout, dtype=np.float64) * np.where(np.asarray(mask) != 0, 1.0, np.float64(slope))
    gW = gJ.T @ np.asarray(Hhat, dtype=np.float64)
    gH = gJ @ np.asarray(W, dtype=np.float64)
    gE = gH + A.T @ gH
    return gE.astype(np.float32), gW.astype(np.float32)


# ------------------------------------------------ bfloat16 activations ------
def widen_bf16(act_u16):
    """bfloat16 bit patterns (uint16) -> the fp32 values they denote (exact: bfloat16 is
    the upper half of an fp32)."""
    a = np.ascontiguousarray(act_u16, dtype=np.uint16)
    return (a.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize_bf16(act_u16, bits, group, seed, first_index=0, rounding=0):
    """Quant of Eq. (3) for half-precision inputs (Sec. 4.1.4): the fp32 quantizer applied to
    the exactly widened values."""
    return quantize(widen_bf16(act_u16), bits, group, seed, first_index, rounding)


# ------------------------------------------------ BatchNorm with a compressed context ------
def batchnorm_fwd(x, gamma, beta, eps):
    """Batch normalisation over the rows, training mode (one of the operators whose saved
    input is compressed, Sec. 4.1.4): mu_c = mean_n x[n, c], var_c = mean_n (x[n, c] - mu_c)^2,
    rstd_c = 1 / sqrt(var_c + eps), y = gamma (x - mu) rstd + beta.  float64 throughout,
    outputs rounded to fp32 once.  Returns y, mu, rstd.  The context is Q(x; seed) plus mu and
    rstd themselves (2 * dim numbers, kept exact)."""
    x64 = np.asarray(x, dtype=np.float64)
    n = x64.shape[0]
    mu = x64.sum(axis=0) / n
    var = ((x64 - mu) ** 2).sum(axis=0) / n
    rstd = 1.0 / np.sqrt(var + np.float64(eps))
    y = np.asarray(gamma, np.float64) * (x64 - mu) * rstd + np.asarray(beta, np.float64)
    return y.astype(np.float32), mu.astype(np.float32), rstd.astype(np.float32)


def batchnorm_bwd(xhat, mu, rstd, gamma, grad_y):
    """Backward of batchnorm_fwd at the saved context (x_hat, mu, rstd):
    xbar = (x_hat - mu) rstd; grad_beta = sum_n g; grad_gamma = sum_n g xbar;
    grad_x = gamma rstd (g - grad_beta / n - xbar grad_gamma / n).  float64, rounded once."""
    xh = np.asarray(xhat, dtype=np.float64)
    g = np.asarray(grad_y, dtype=np.float64)
    n = xh.shape[0]
    mu, rstd, gamma = (np.asarray(a, dtype=np.float64) for a in (mu, rstd, gamma))
    xbar = (xh - mu) * rstd
    gbeta = g.sum(axis=0)
    ggamma = (g * xbar).sum(axis=0)
    gx = gamma * rstd * (g - gbeta / n - xbar * ggamma / n)
    return gx.astype(np.float32), ggamma.astype(np.float32), gbeta.astype(np.float32)


# ------------------------------------------------ max-pooling aggregation (SPMM_MAX) ------
def head_order(head, rel, tail):
    """The order in which a head's out-edges are numbered: by (relation, tail, input
    position).  Returns the permutation of the input triplets sorted by (head, relation,
    tail, position)."""
    head, rel, tail = _coo(head, rel, tail)
    order = np.lexsort((np.arange(head.size), tail, rel, head))
    return order


def spmm_max_fwd(n_nodes, head, rel, tail, E):
    """M[h, c] = max over the out-edges (h, r, t) of E[t, c]; 0 for a head without
    out-edges.  The context is, per output element, the LOCAL number (in head_order) of the
    first out-edge that attains the maximum -- a narrow integer instead of the activation
    (Sec. 4.1.4 lists SPMM_MAX among the compressed operators); 0 where there is no edge.
    Returns M (fp32, exact: a maximum has no rounding) and arg (int64 [n, d])."""
    head, rel, tail = _coo(head, rel, tail)
    E = np.ascontiguousarray(E, dtype=np.float32)
    d = E.shape[1]
    order = head_order(head, rel, tail)
    hs, ts = head[order], tail[order]
    M = np.zeros((n_nodes, d), np.float32)
    arg = np.zeros((n_nodes, d), np.int64)
    start = np.searchsorted(hs, np.arange(n_nodes), side="left")
    end = np.searchsorted(hs, np.arange(n_nodes), side="right")
    for h in range(n_nodes):
        if end[h] > start[h]:
            rows = E[ts[start[h]:end[h]]]                 # [deg, d]
            arg[h] = np.argmax(rows, axis=0)              # first occurrence of the maximum
            M[h] = rows[arg[h], np.arange(d)]
    return M, arg


def spmm_max_bwd(n_nodes, head, rel, tail, arg, grad_M):
    """grad_E[t, c] = sum of grad_M[h, c] over the heads h whose saved out-edge number
    arg[h, c] leads to t; heads without out-edges pass nothing on.  float64 sums, rounded once."""
    head, rel, tail = _coo(head, rel, tail)
    g = np.asarray(grad_M, dtype=np.float64)
    d = g.shape[1]
    order = head_order(head, rel, tail)
    hs, ts = head[order], tail[order]
    start = np.searchsorted(hs, np.arange(n_nodes), side="left")
    end = np.searchsorted(hs, np.arange(n_nodes), side="right")
    gE = np.zeros((n_nodes, d), np.float64)
    cols = np.arange(d)
    for h in range(n_nodes):
        if end[h] > start[h]:
            t = ts[start[h] + np.asarray(arg[h], dtype=np.int64)]
            np.add.at(gE, (t, cols), g[h])
    return gE.astype(np.float32)
