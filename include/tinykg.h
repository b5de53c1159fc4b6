/*
 * tinykg.h -- C ABI of the MI355X (gfx950) implementation of TinyKG's activation
 * compressor and of the attentive knowledge-graph aggregation layer whose saved
 * activations it compresses.
 *
 * General conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, 16-byte
 *     aligned, dense, row-major, unless a parameter says "host".
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return without synchronising; the caller
 *     keeps inputs, outputs and workspace alive until the stream has drained.
 *   - Outputs are fully overwritten (gradients are assigned, not accumulated).
 *   - No entry point allocates or frees device memory except
 *     tinykg_graph_create / tinykg_graph_destroy.
 *   - Errors are returned as tinykg_status; nothing is written when a call
 *     returns TINYKG_ERR_INVALID_ARG / _SHAPE / _UNSUPPORTED / _WORKSPACE.
 *     TINYKG_ERR_DEVICE reports a failed HIP call (launch, copy, allocation).
 *   - Inputs must be finite; behaviour for NaN/Inf activations is unspecified.
 */
#ifndef TINYKG_H
#define TINYKG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TINYKG_OK = 0,
  TINYKG_ERR_INVALID_ARG = 1, /* null pointer, misaligned pointer, bad bits/group/rounding */
  TINYKG_ERR_SHAPE = 2,       /* negative size, rows*dim not a multiple of group, ... */
  TINYKG_ERR_UNSUPPORTED = 3, /* a size the kernels are not built for */
  TINYKG_ERR_WORKSPACE = 4,   /* workspace missing or too small */
  TINYKG_ERR_DEVICE = 5       /* a HIP runtime call failed */
} tinykg_status;

typedef enum { TINYKG_ROUND_STOCHASTIC = 0, TINYKG_ROUND_NEAREST = 1 } tinykg_rounding;

const char* tinykg_status_string(tinykg_status s);

/* Size helpers (host arithmetic only).  Sec. 3.2 "Memory Analysis": an N x d
 * activation map costs rows*dim*bits/8 bytes of codes plus one (min, scale)
 * fp32 pair per group, i.e. bits/8 + 8/group bytes per element. */
size_t  tinykg_packed_bytes(int64_t rows, int64_t dim, int bits); /* rows*dim*bits/8 */
int64_t tinykg_num_groups(int64_t rows, int64_t dim, int group);  /* rows*dim/group  */

/* Quant of Sec. 3.3, Eq. (3), fused with the bit-stream conversion of Sec. 4.1.4.
 *
 * The row-major flattening of act[rows, dim] is cut into groups of `group`
 * consecutive elements.  Per group: Z = min, R = max - Z, B = 2^bits - 1;
 * gmin = Z (a minimum of -0 is stored as +0), gscale = R / B.  Per element
 * code = SR((e - Z) * (B / R)) clamped to [0, B], where SR rounds up with
 * probability equal to the fractional part; the group maximum always gets code
 * B and a constant group gets all-zero codes and gscale = 0.  The rounding
 * noise is 16 bits per element from Philox4x32-10 with key = seed and counter =
 * (flat element index) / 8: element i uses the low (i even) or high (i odd) half
 * of output word (i / 2) mod 4, so the result depends only on (act, seed) and
 * never on the launch geometry.  Codes are packed LSB-first: element i occupies
 * bits [(i*bits) mod 8, +bits) of byte (i*bits) / 8.
 *
 *   act    in   [rows, dim] fp32
 *   bits        1, 2, 4 or 8
 *   group       32, 64, 128 or 256; rows*dim must be a multiple (else ERR_SHAPE)
 *   packed out  tinykg_packed_bytes(rows, dim, bits) bytes
 *   gmin   out  tinykg_num_groups(...) fp32
 *   gscale out  tinykg_num_groups(...) fp32
 * rows*dim == 0 returns TINYKG_OK and writes nothing. */
tinykg_status tinykg_quantize(const float* act, int64_t rows, int64_t dim, int bits, int group,
                              uint64_t seed, uint8_t* packed, float* gmin, float* gscale,
                              void* stream);

/* As tinykg_quantize, with two more controls:
 *   first_index  flat index of act[0] inside a larger tensor (multiple of
 *                `group`); the noise counter starts there, so quantising a slice
 *                yields the bytes the whole tensor's run would produce for it.
 *   rounding     TINYKG_ROUND_STOCHASTIC, or TINYKG_ROUND_NEAREST (the ablation
 *                of Sec. 4.4, Table 6: code = floor(x + 1/2), seed unused). */
tinykg_status tinykg_quantize_ex(const float* act, int64_t rows, int64_t dim, int bits, int group,
                                 uint64_t seed, uint64_t first_index, int rounding,
                                 uint8_t* packed, float* gmin, float* gscale, void* stream);

/* The same quantizer for bfloat16 activations (Sec. 4.1.4: half-precision inputs are
 * supported, for mixed-precision training).  act: [rows, dim] bfloat16 (the upper 16 bits
 * of an fp32 value), DEVICE.  Every value is widened to fp32 exactly and then quantized
 * as above, so packed / gmin / gscale are byte for byte those of tinykg_quantize_ex on the
 * widened fp32 tensor.  Other arguments, limits and errors as tinykg_quantize_ex. */
tinykg_status tinykg_quantize_bf16(const uint16_t* act, int64_t rows, int64_t dim, int bits,
                                   int group, uint64_t seed, uint64_t first_index, int rounding,
                                   uint8_t* packed, float* gmin, float* gscale, void* stream);

/* Dequant of Sec. 3.3, Eq. (4): out[i] = fma(code_i, gscale[i/group], gmin[i/group])
 * (R * code / B + Z with scale = R / B, one rounding).  Arguments as above;
 * out is [rows, dim] fp32. */
tinykg_status tinykg_dequantize(const uint8_t* packed, const float* gmin, const float* gscale,
                                int64_t rows, int64_t dim, int bits, int group, float* out,
                                void* stream);

/* ------------------------------------------------------------------------- *
 * Attentive aggregation layer (the KG-Layer of Sec. 3.2, Eq. (1), in the
 * three-stage form of Eq. (2), with KGAT's attention as the sparse operator):
 *   a_j = W_r e_t,  b_j = W_r e_h + e_r,  s_j = a_j . tanh(b_j)      per triplet j = (h, r, t)
 *   pi_j = softmax of s_j over the triplets that share the head h
 *   H_h = e_h + sum_j pi_j e_t ;  J_h = W H_h ;  E'_h = J_h > 0 ? J_h : slope * J_h
 * A head without triplets has H_h = e_h.  Repeated triplets and self-loops are
 * separate edges.
 * ------------------------------------------------------------------------- */

/* Opaque, immutable graph: triplets grouped by head (CSR), plus the orderings
 * the kernels need.  Built once, shared by every layer and step (Sec. 3.2: the
 * adjacency is kept once for all layers). */
typedef struct tinykg_graph tinykg_graph;

/* head/rel/tail: DEVICE int32 arrays of n_edges entries, any order; ids must lie
 * in [0, n_nodes) and [0, n_rel) (else ERR_INVALID_ARG).  Limits: n_nodes < 2^30,
 * n_edges < 2^31, n_rel <= 65535 (else ERR_UNSUPPORTED).  Synchronises `stream`,
 * allocates device memory owned by the graph.  *out is set only on TINYKG_OK. */
tinykg_status tinykg_graph_create(int64_t n_nodes, int32_t n_rel, int64_t n_edges,
                                  const int32_t* head, const int32_t* rel, const int32_t* tail,
                                  void* stream, tinykg_graph** out);
void tinykg_graph_destroy(tinykg_graph* g);
int64_t tinykg_graph_num_nodes(const tinykg_graph* g);
int64_t tinykg_graph_num_edges(const tinykg_graph* g);

/* The saved context of one layer (Fig. 1; Sec. 3.2: the inputs of the spmm and mm
 * stages, and one bit per element for the ReLU-type stage, Sec. 4.1.4).
 * Caller-allocated device buffers in exactly tinykg_quantize's output layout.
 * With bits == 32 nothing is compressed: packed_E / packed_H hold the fp32
 * tensors themselves (n_nodes*d_in*4 bytes each) and gmin / gscale are unused
 * (may be NULL).
 * packed_H == NULL (attentive layer only) leaves H out of the context: the forward
 * call then saves Q(E) and the mask alone, and the backward call runs the second
 * stage of Eq. 2 again on E_hat and uses that H~ = e^_h + sum_j pi_j(E_hat) e^_t
 * where H_hat would stand (half the saved bytes, one more pass over the edges).
 * Pass the same struct to the forward and the backward call. */
typedef struct {
  uint8_t* packed_E; float* gmin_E; float* gscale_E; /* Q(E; seed),     n = n_nodes*d_in */
  uint8_t* packed_H; float* gmin_H; float* gscale_H; /* Q(H; seed + 1), n = n_nodes*d_in */
  uint8_t* mask_J; /* [J > 0], n_nodes*d_out bits, LSB-first, ceil(n_nodes*d_out/8) bytes */
} tinykg_saved;

/* Scratch bytes the forward (is_bwd == 0) or backward (is_bwd != 0) call needs. */
size_t tinykg_kg_aggregate_workspace_bytes(const tinykg_graph* g, int d_in, int d_rel, int d_out,
                                           int is_bwd);

/* Forward pass; exact (compression never changes E_out -- Fig. 1), and saves the
 * context compressed: Q(E; seed), Q(H; seed+1) with `bits`/`group` as in
 * tinykg_quantize (or fp32 copies when bits == 32), and the sign mask of J.
 *   E [n_nodes, d_in], Wr [n_rel, d_rel, d_in], er [n_rel, d_rel], W [d_out, d_in]
 *   E_out [n_nodes, d_out]
 * Wr / er may be NULL only for a graph without edges (Q(E) is saved all the same).
 * d_in == d_rel in {32, 64, 128} (the relation space has the embedding's width: a d_rel
 * other than d_in is ERR_UNSUPPORTED); d_out a multiple of 16 up to 128; n_nodes*d_in
 * a multiple of `group` (else ERR_UNSUPPORTED / ERR_SHAPE).
 * Arithmetic: fp32 in, fp32 out, fp32 (or wider) accumulation.  The projections W_r e are
 * formed on the matrix cores from exact three-way bfloat16 splits of their fp32 operands
 * (all piece products down to 2^-23 of a term are kept), so they agree with an fp32
 * evaluation to fp32's own rounding level; sums over many edges are reproducible to
 * rounding, not bitwise (atomic order), everything else is deterministic. */
tinykg_status tinykg_kg_aggregate_fwd(const tinykg_graph* g, const float* E, const float* Wr,
                                      const float* er, const float* W, int d_in, int d_rel,
                                      int d_out, float leaky_slope, int bits, int group,
                                      uint64_t seed, float* E_out, const tinykg_saved* saved,
                                      void* workspace, size_t workspace_bytes, void* stream);

/* Backward pass: the vector-Jacobian product of the layer evaluated at the saved
 * context (Sec. 3.3: gradients are computed from the dequantised activations;
 * Eq. (2): grad_J = ctx(J, grad_E'), (grad_H, grad_W) = ctx(H, W, grad_J),
 * grad_E = ctx(A, grad_H)).  Projections, scores and attention are recomputed
 * from E_hat = Dequant(Q(E)); dequantisation is fused into the gathers.
 *   grad_E_out [n_nodes, d_out]  ->  grad_E [n_nodes, d_in], grad_Wr [n_rel, d_rel, d_in],
 *   grad_er [n_rel, d_rel], grad_W [d_out, d_in] */
tinykg_status tinykg_kg_aggregate_bwd(const tinykg_graph* g, const tinykg_saved* saved,
                                      const float* Wr, const float* er, const float* W, int d_in,
                                      int d_rel, int d_out, float leaky_slope, int bits, int group,
                                      const float* grad_E_out, float* grad_E, float* grad_Wr,
                                      float* grad_er, float* grad_W, void* workspace,
                                      size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------- *
 * Uniform-attention layer: Eq. (2) exactly as printed, E' = sigma(A_hat E Theta), with the
 * row-normalised adjacency plus self term of the KGCN / KGNN-LS family (Sec. 3.1):
 *   H_h = e_h + (1 / deg(h)) sum over the out-edges (h, r, t) of e_t ;  J = H W^T ;
 *   E' = LeakyReLU(J).
 * It is the attentive layer with every attention weight pi = 1 / deg(h) (relations are
 * ignored).  Context (Sec. 3.2): the spmm stage needs only A_hat, which the graph holds;
 * the mm stage needs H; the activation needs one bit per element.  So `saved` carries
 * Q(H; seed + 1) and mask_J only -- packed_E / gmin_E / gscale_E are not touched and may be
 * NULL.  Backward (Eq. (2)): grad_J from the mask, grad_W = grad_J^T H_hat,
 * grad_H = grad_J W, grad_E = grad_H + A_hat^T grad_H (row t receives grad_H_h / deg(h)
 * from every in-edge).  Shapes, limits, workspace (use
 * tinykg_kg_aggregate_workspace_bytes with d_rel = d_in) and error behaviour as for the
 * attentive layer.
 * ------------------------------------------------------------------------- */
tinykg_status tinykg_kg_uniform_fwd(const tinykg_graph* g, const float* E, const float* W, int d_in,
                                    int d_out, float leaky_slope, int bits, int group, uint64_t seed,
                                    float* E_out, const tinykg_saved* saved, void* workspace,
                                    size_t workspace_bytes, void* stream);
tinykg_status tinykg_kg_uniform_bwd(const tinykg_graph* g, const tinykg_saved* saved, const float* W,
                                    int d_in, int d_out, float leaky_slope, int bits, int group,
                                    const float* grad_E_out, float* grad_E, float* grad_W,
                                    void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------- *
 * Readout and loss for a stack of layers (Sec. 3.2: after L layers a readout forms
 * the final embedding -- here the concatenation of E^(0..L), "layer-aggregation" --
 * and a downstream loss is optimised).  Score y(u, i) = <concat_l e_u^(l), concat_l
 * e_i^(l)>; pairwise ranking (BPR) loss = mean over the batch of
 * softplus(y(u, i-) - y(u, i+)).
 * ------------------------------------------------------------------------- */

/* layers: HOST array of n_layers DEVICE pointers, layer l being [n_nodes, dims[l]]
 * fp32 (dims: HOST array, each a multiple of 4, at most 128).  users/pos/neg:
 * DEVICE int32 [batch], ids in [0, n_nodes) (not checked).  Writes loss[0] (DEVICE,
 * the mean loss) and coef (DEVICE, 2*batch floats): coef[b] = sigmoid(y_neg - y_pos) /
 * batch, the derivative of the loss with respect to (y_neg - y_pos) of sample b; the
 * second half coef[batch + b] holds the per-sample loss terms (summed in fixed order). */
tinykg_status tinykg_bpr_loss(const float* const* layers, const int* dims, int n_layers,
                              int64_t n_nodes, const int32_t* users, const int32_t* pos,
                              const int32_t* neg, int64_t batch, float* loss, float* coef,
                              void* stream);

/* Gradient of that loss with respect to ONE layer tensor E_l [n_nodes, dim]:
 * row u += coef (e_neg - e_pos), row pos -= coef e_u, row neg += coef e_u, summed
 * over the batch.  accumulate == 0: grad is cleared first; != 0: the rows are
 * added to what grad holds (the gradient arriving from the layer above). */
tinykg_status tinykg_bpr_grad(const float* E_l, int dim, int64_t n_nodes, const int32_t* users,
                              const int32_t* pos, const int32_t* neg, const float* coef,
                              int64_t batch, int accumulate, float* grad, void* stream);

/* Row gather / scatter-add used by the readout so that the full fp32 layer tensors
 * need not outlive the next layer's forward pass (Sec. 3.3: exact activations are
 * discarded layer by layer): out[r, :] = E[idx[r], :] and dst[idx[r], :] += src[r, :].
 * E/dst are [*, dim] fp32 (dim a multiple of 4 for the gather), idx DEVICE int32
 * [n_rows] (ids not checked), out/src [n_rows, dim]. */
tinykg_status tinykg_gather_rows(const float* E, int dim, const int32_t* idx, int64_t n_rows,
                                 float* out, void* stream);
tinykg_status tinykg_scatter_add_rows(const float* src, int dim, const int32_t* idx, int64_t n_rows,
                                      float* dst, void* stream);
/* The id list of one readout batch: ids[0..3*batch) = users | pos | neg (what
 * tinykg_gather_rows takes), and slot[i] = i, so that slot, slot + batch and
 * slot + 2*batch address the three parts inside the gathered rows (what
 * tinykg_bpr_loss / tinykg_bpr_grad take when they run on gathered rows).  All DEVICE
 * int32; ids and slot hold 3*batch entries each; 3*batch < 2^31 (else ERR_SHAPE). */
tinykg_status tinykg_readout_ids(const int32_t* users, const int32_t* pos, const int32_t* neg,
                                 int64_t batch, int32_t* ids, int32_t* slot, void* stream);
/* dst[0..n) = 0 with a fill kernel (n a multiple of 4, dst DEVICE, 16-byte aligned). */
tinykg_status tinykg_fill_zero(float* dst, int64_t n, void* stream);

/* ------------------------------------------------------------------------- *
 * Max-pooling aggregation over the out-edges (the SPMM_MAX operator of the list in
 * Sec. 4.1.4):  M[h,c] = max over the out-edges (h,r,t) of E[t,c];  0 for a head
 * without out-edges.  The backward pass needs no activation, only WHICH out-edge
 * won each output element; the context is that edge's number inside the head's
 * neighbourhood -- out-edges numbered from 0 in the order (relation, tail, position
 * in the arrays given to tinykg_graph_create); the first one on equal values; 0
 * without out-edges -- stored in tinykg_kg_max_arg_bytes(g) bytes per element
 * (1 if the graph's largest out-degree is at most 256, 2 up to 65536, else 4;
 * little-endian unsigned), as `arg` [n_nodes, d].  Backward:
 *   grad_E[t,c] = sum of grad_M[h,c] over the heads h whose saved edge number leads to t.
 * E, M, grad_M, grad_E [n_nodes, d] fp32, d in {32, 64, 128} (else ERR_UNSUPPORTED);
 * all pointers DEVICE and 16-byte aligned; outputs are overwritten.  M and arg are
 * exact and deterministic; grad_E is accumulated with atomics (fp32, double for the
 * nodes with more than 1024 incident edges), so it is reproducible to rounding.
 * An edge number in `arg` beyond its head's degree (a corrupted context) matches no
 * out-edge: that gradient entry is dropped.
 * `workspace` (backward only): tinykg_kg_max_workspace_bytes(g, d) bytes.
 * ------------------------------------------------------------------------- */
int tinykg_kg_max_arg_bytes(const tinykg_graph* g);
size_t tinykg_kg_max_workspace_bytes(const tinykg_graph* g, int d);
tinykg_status tinykg_kg_max_fwd(const tinykg_graph* g, const float* E, int d, float* M, void* arg,
                                void* stream);
tinykg_status tinykg_kg_max_bwd(const tinykg_graph* g, const void* arg, int d, const float* grad_M,
                                float* grad_E, void* workspace, size_t workspace_bytes,
                                void* stream);

/* ------------------------------------------------------------------------- *
 * Batch normalisation over the rows (training mode) with its input saved
 * compressed.  Sec. 4.1.4 names BatchNorm among the operators whose context is
 * compressed; the operator's input takes the place of the activation in Eq. 3 / 4:
 *   mu_c = mean_n x[n,c]   var_c = mean_n (x[n,c] - mu_c)^2   rstd_c = 1/sqrt(var_c + eps)
 *   y[n,c] = gamma_c (x[n,c] - mu_c) rstd_c + beta_c                     (exact)
 * Saved: Q(x; seed) in tinykg_quantize's layout (with bits == 32: an fp32 copy of
 * x in `packed`, rows*dim*4 bytes, gmin / gscale unused), and mean[dim], rstd[dim]
 * themselves.  Backward, at x_hat = the dequantised Q(x), xbar = (x_hat - mu) rstd:
 *   grad_beta_c = sum_n g[n,c]        grad_gamma_c = sum_n g[n,c] xbar[n,c]
 *   grad_x = gamma rstd (g - grad_beta/rows - xbar grad_gamma/rows)
 * All pointers DEVICE, 16-byte aligned, row-major; x, y, grad_y, grad_x [rows, dim]
 * fp32; gamma, beta, mean, rstd, grad_gamma, grad_beta [dim].  dim a multiple of 4
 * in [4, 1024] and rows*dim < 2^34 (else ERR_UNSUPPORTED); rows*dim a multiple of
 * `group` (ERR_SHAPE); eps >= 0.  rows == 0: OK; the forward call writes nothing,
 * the backward call zeroes grad_gamma / grad_beta.  Outputs are overwritten, and
 * every one of them is deterministic.  `workspace`: at least
 * tinykg_batchnorm_workspace_bytes(rows, dim) bytes (0 = unsupported shape);
 * ERR_WORKSPACE if missing or too small.  Calls enqueue on `stream` and return.
 * ------------------------------------------------------------------------- */
size_t tinykg_batchnorm_workspace_bytes(int64_t rows, int dim);
tinykg_status tinykg_batchnorm_fwd(const float* x, int64_t rows, int dim, const float* gamma,
                                   const float* beta, float eps, int bits, int group, uint64_t seed,
                                   float* y, uint8_t* packed, float* gmin, float* gscale,
                                   float* mean, float* rstd, void* workspace,
                                   size_t workspace_bytes, void* stream);
tinykg_status tinykg_batchnorm_bwd(const uint8_t* packed, const float* gmin, const float* gscale,
                                   const float* mean, const float* rstd, const float* gamma,
                                   int64_t rows, int dim, int bits, int group, const float* grad_y,
                                   float* grad_x, float* grad_gamma, float* grad_beta,
                                   void* workspace, size_t workspace_bytes, void* stream);

/* tinykg_batchnorm_bwd for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments (without the workspace pair), same kernels, same results bit
 * for bit.  The partial column sums and the coefficient table live in a fixed array of
 * 4 MiB + 2 KiB of device memory inside the library's code object (each GPU the library
 * runs on holds its own copy until the process ends), so dim is limited to 128: a larger
 * dim returns TINYKG_ERR_UNSUPPORTED and writes nothing.  The call allocates and frees
 * nothing, creates no event (the measurement hooks below ignore it) and clears nothing: every
 * scratch word it reads was written earlier in the same call.  All calls on one GPU share that
 * array: calls that may overlap on one GPU (different streams, or threads) race and must be
 * serialised by the caller; calls on one stream are ordered by the stream. */
tinykg_status tinykg_batchnorm_bwd_static(const uint8_t* packed, const float* gmin, const float* gscale,
                                          const float* mean, const float* rstd, const float* gamma,
                                          int64_t rows, int dim, int bits, int group, const float* grad_y,
                                          float* grad_x, float* grad_gamma, float* grad_beta, void* stream);

/* ------------------------------------------------------------------------- *
 * Measurement hooks (not part of the method): when enabled, every kernel launch
 * made by the entry points above is bracketed by a pair of HIP events recorded
 * on the caller's stream, so a benchmark can read each kernel's device time over
 * exactly the launches it timed.  One global recorder per process, not
 * thread-safe; at most 8192 launches are kept between two resets (later ones are
 * not recorded).
 * ------------------------------------------------------------------------- */
/* on != 0: drop earlier records and start recording; on == 0: stop recording. */
void tinykg_profile_enable(int on);
/* Restricts recording to the launches reported under `name` (one of the names
 * tinykg_profile_report prints, e.g. "edge_bwd_kernel"); NULL or "": every launch again.
 * Bracketing one kernel instead of all keeps the events' own cost (about 4 % of a
 * one-millisecond step when every launch is bracketed) out of a timed region. */
void tinykg_profile_select(const char* name);
/* Waits for the recorded events, then writes one line per kernel name,
 * "<name> <launches> <total_ms>\n", into buf (NUL-terminated, truncated to cap).
 * Returns the number of bytes the full text needs (excluding the NUL). */
size_t tinykg_profile_report(char* buf, size_t cap);
/* A plain 128-bit-per-lane copy kernel (calibration_copy_kernel) of `bytes` bytes
 * (multiple of 16; dst/src device, 16-byte aligned): reads `bytes`, writes `bytes`.
 * Its known traffic calibrates the profiler's HBM byte counters. */
tinykg_status tinykg_profile_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TINYKG_H */
