"""Thin glue that chains aggregation layers into one training step (forward,
readout + ranking loss, backward): a fixed sequence of C-ABI calls, no arithmetic
of its own.  The exact fp32 activation of a layer is dropped as soon as the next
layer has consumed it and the readout has gathered its sampled rows (Sec. 3.3:
exact activations are discarded layer by layer); only the compressed contexts and
the gathered rows survive until the backward pass.
"""
import torch

from . import binding as B


class KGStack:
    def __init__(self, graph, dims, bits, group, slope=0.2, device="cuda", keep_activations=False,
                 save_H=True):
        """dims = [d_0, d_1, ..., d_L]; layer l maps [N, d_l] -> [N, d_{l+1}].
        save_H=False: the contexts hold Q(E) and the mask only (the backward pass rebuilds H)."""
        self.graph, self.dims, self.bits, self.group, self.slope = graph, list(dims), bits, group, slope
        self.L = len(dims) - 1
        self.N = graph.n_nodes
        self.device = device
        self.save_H = save_H
        self.saved = [B.SavedContext(self.N, dims[l], dims[l + 1], bits, group, device, with_H=save_H)
                      for l in range(self.L)]
        nb = 16
        for l in range(self.L):
            for bwd in (False, True):
                nb = max(nb, B.tinykg_kg_aggregate_workspace_bytes(graph, dims[l], dims[l], dims[l + 1], bwd))
        self.ws = torch.empty(nb, dtype=torch.uint8, device=device)
        self.keep_activations = keep_activations   # debugging / tests: keep every exact E^(l)
        self.acts = None
        self.rows = None          # gathered readout rows per layer: [3 * batch, d_l]
        self.sample_ids = None

    # ---- accounting (bytes alive between forward and backward) -------------------
    def saved_context_bytes(self):
        return sum(s.nbytes() for s in self.saved)

    def fp32_context_bytes(self):
        return sum(2 * self.N * self.dims[l] * 4 + (self.N * self.dims[l + 1] + 7) // 8 for l in range(self.L))

    def readout_rows_bytes(self):
        return 0 if self.rows is None else sum(r.numel() * 4 for r in self.rows)

    # ---- one step ------------------------------------------------------------------
    def forward(self, E0, params, seed, users, pos, neg):
        """params: list of (Wr, er, W) per layer.  Returns the loss tensor [1]."""
        batch = users.numel()
        ids, slot = B.tinykg_readout_ids(users, pos, neg)
        self.sample_ids, self.batch = ids, batch
        self.rows = []
        self.acts = [E0] if self.keep_activations else None
        E = E0
        for l in range(self.L):
            self.rows.append(B.tinykg_gather_rows(E, ids))
            Wr, er, W = params[l]
            E_next = B.tinykg_kg_aggregate_fwd(self.graph, E, Wr, er, W, self.slope, self.bits, self.group,
                                               seed + 2 * l, self.saved[l], self.ws)
            E = E_next          # the previous exact activation is no longer referenced here
            if self.keep_activations:
                self.acts.append(E)
        self.rows.append(B.tinykg_gather_rows(E, ids))
        self._u, self._p, self._n = slot[:batch], slot[batch:2 * batch], slot[2 * batch:]
        self.loss, self.coef = B.tinykg_bpr_loss(self.rows, self._u, self._p, self._n)
        return self.loss

    def backward(self, params):
        """Returns the gradients of the loss with respect to every layer tensor
        ([grad_E^(0), ..., grad_E^(L)]) and a list of (grad_Wr, grad_er, grad_W) per layer."""
        dev = self.device
        g_next = None
        layer_grads = [None] * (self.L + 1)
        pgrads = [None] * self.L
        for l in range(self.L, -1, -1):
            d = self.dims[l]
            if l == self.L:
                g = torch.empty((self.N, d), dtype=torch.float32, device=dev)
            else:
                Wr, er, W = params[l]
                out = B.tinykg_kg_aggregate_bwd(self.graph, self.saved[l], Wr, er, W, self.slope, self.bits,
                                                self.group, g_next, self.ws)
                g, pgrads[l] = out[0], out[1:]
            if l == self.L:
                B.tinykg_fill_zero(g)
            # readout rows of this layer: gradient of the compact rows, scattered back
            gr = torch.empty_like(self.rows[l])
            B.tinykg_bpr_grad(self.rows[l], self._u, self._p, self._n, self.coef, gr, accumulate=False)
            B.tinykg_scatter_add_rows(gr, self.sample_ids, g)
            g_next = g
            layer_grads[l] = g
        return layer_grads, pgrads
