// Readout (concatenation of the layer tensors) + pairwise ranking loss for a
// stack of aggregation layers, and its gradient with respect to each layer tensor.
// Sec. 3.2: a readout follows the L layers and a downstream loss is optimised; the
// concatenation over layers is the "layer-aggregation" that makes every E^(l) a
// saved activation.  Tiny next to the layers themselves: one wave per sample.
#include "tinykg_common.h"

namespace tinykg {

namespace {

constexpr int kMaxLayers = 8;

struct LayerSet {
  const float* ptr[kMaxLayers];
  int dim[kMaxLayers];
  int n;
};

__device__ __forceinline__ float wave_sum64(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// One wave per (user, positive, negative) sample.  per_sample[b] = softplus(y- - y+)/batch.
__global__ __launch_bounds__(256) void bpr_loss_kernel(LayerSet L, const int32_t* __restrict__ users,
                                                       const int32_t* __restrict__ pos,
                                                       const int32_t* __restrict__ neg, int64_t batch,
                                                       float* __restrict__ per_sample,
                                                       float* __restrict__ coef) {
  const int lane = threadIdx.x & 63;
  const int64_t b = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= batch) return;
  const int64_t u = users[b], ip = pos[b], in = neg[b];
  float diff = 0.f;   // y_neg - y_pos, partial over this lane's elements
  for (int l = 0; l < L.n; ++l) {
    const int d = L.dim[l];
    const float* E = L.ptr[l];
    for (int i = lane; i < d; i += 64) {
      const float eu = E[u * d + i];
      diff = fmaf(eu, E[in * d + i] - E[ip * d + i], diff);
    }
  }
  diff = wave_sum64(diff);
  if (lane == 0) {
    // softplus(x) = max(x, 0) + log1p(exp(-|x|));  sigmoid(x) = 1 / (1 + exp(-x))
    const float sp = fmaxf(diff, 0.f) + log1pf(expf(-fabsf(diff)));
    const float sg = 1.f / (1.f + expf(-diff));
    per_sample[b] = sp / (float)batch;
    coef[b] = sg / (float)batch;
  }
}

// Fixed-order sum of the per-sample terms (one block).
__global__ __launch_bounds__(256) void bpr_reduce_kernel(const float* __restrict__ per_sample,
                                                         int64_t batch, float* __restrict__ loss) {
  __shared__ double part[256];
  double acc = 0.0;
  for (int64_t i = threadIdx.x; i < batch; i += 256) acc += (double)per_sample[i];
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) loss[0] = (float)part[0];
}

__global__ void zero_f32_kernel(float4* __restrict__ dst, int64_t n4) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride)
    dst[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

__global__ __launch_bounds__(256) void bpr_grad_kernel(const float* __restrict__ E, int d,
                                                       const int32_t* __restrict__ users,
                                                       const int32_t* __restrict__ pos,
                                                       const int32_t* __restrict__ neg,
                                                       const float* __restrict__ coef, int64_t batch,
                                                       float* __restrict__ grad) {
  const int lane = threadIdx.x & 63;
  const int64_t b = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= batch) return;
  const int64_t u = users[b], ip = pos[b], in = neg[b];
  const float c = coef[b];
  for (int i = lane; i < d; i += 64) {
    const float eu = E[u * d + i], epos = E[ip * d + i], eneg = E[in * d + i];
    unsafeAtomicAdd(grad + u * d + i, c * (eneg - epos));
    unsafeAtomicAdd(grad + ip * d + i, -c * eu);
    unsafeAtomicAdd(grad + in * d + i, c * eu);
  }
}

// out[r, :] = E[idx[r], :]  (one thread per 128-bit chunk)
__global__ void gather_rows_kernel(const float4* __restrict__ E, int lpr, const int32_t* __restrict__ idx,
                                   int64_t n_rows, float4* __restrict__ out) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < n_rows * lpr; q += stride)
    out[q] = E[(int64_t)idx[q / lpr] * lpr + q % lpr];
}

// dst[idx[r], :] += src[r, :]
__global__ void scatter_add_rows_kernel(const float* __restrict__ src, int d, const int32_t* __restrict__ idx,
                                        int64_t n_rows, float* __restrict__ dst) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < n_rows * d; q += stride)
    unsafeAtomicAdd(dst + (int64_t)idx[q / d] * d + q % d, src[q]);
}

// ids[0..3b) = users | pos | neg; slot[i] = i: the sampled nodes of a batch as one id list for
// the row gathers, and the positions of its three parts inside the gathered rows.
__global__ __launch_bounds__(256) void readout_ids_kernel(const int32_t* __restrict__ users,
                                                          const int32_t* __restrict__ pos,
                                                          const int32_t* __restrict__ neg, int64_t batch,
                                                          int32_t* __restrict__ ids, int32_t* __restrict__ slot) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < 3 * batch;
       i += (int64_t)gridDim.x * blockDim.x) {
    const int32_t* src = i < batch ? users : (i < 2 * batch ? pos : neg);
    ids[i] = src[i % batch];
    slot[i] = (int32_t)i;
  }
}

}  // namespace
}  // namespace tinykg

extern "C" {

tinykg_status tinykg_gather_rows(const float* E, int dim, const int32_t* idx, int64_t n_rows,
                                 float* out, void* stream) {
  using namespace tinykg;
  if (dim <= 0 || dim % 4 != 0 || n_rows < 0) return TINYKG_ERR_SHAPE;
  if (n_rows == 0) return TINYKG_OK;
  if (!E || !idx || !out || !aligned16(E) || !aligned16(out)) return TINYKG_ERR_INVALID_ARG;
  const int64_t n = n_rows * (dim / 4);
  const int64_t want = (n + 255) / 256, cap = (int64_t)num_cus() * 16;
  ProfileScope prof("gather_rows_kernel", (hipStream_t)stream);
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0,
                     (hipStream_t)stream, reinterpret_cast<const float4*>(E), dim / 4, idx, n_rows,
                     reinterpret_cast<float4*>(out));
  return launch_status();
}

tinykg_status tinykg_fill_zero(float* dst, int64_t n, void* stream) {
  using namespace tinykg;
  if (n < 0 || n % 4 != 0) return TINYKG_ERR_SHAPE;
  if (n == 0) return TINYKG_OK;
  if (!dst || !aligned16(dst)) return TINYKG_ERR_INVALID_ARG;
  const int64_t n4 = n / 4;
  const int64_t want = (n4 + 255) / 256, cap = (int64_t)num_cus() * 16;
  ProfileScope prof("zero_f32_kernel", (hipStream_t)stream);
  hipLaunchKernelGGL(zero_f32_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0,
                     (hipStream_t)stream, reinterpret_cast<float4*>(dst), n4);
  return launch_status();
}

tinykg_status tinykg_scatter_add_rows(const float* src, int dim, const int32_t* idx, int64_t n_rows,
                                      float* dst, void* stream) {
  using namespace tinykg;
  if (dim <= 0 || n_rows < 0) return TINYKG_ERR_SHAPE;
  if (n_rows == 0) return TINYKG_OK;
  if (!src || !idx || !dst) return TINYKG_ERR_INVALID_ARG;
  const int64_t n = n_rows * dim;
  const int64_t want = (n + 255) / 256, cap = (int64_t)num_cus() * 16;
  ProfileScope prof("scatter_add_rows_kernel", (hipStream_t)stream);
  hipLaunchKernelGGL(scatter_add_rows_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0,
                     (hipStream_t)stream, src, dim, idx, n_rows, dst);
  return launch_status();
}

tinykg_status tinykg_bpr_loss(const float* const* layers, const int* dims, int n_layers,
                              int64_t n_nodes, const int32_t* users, const int32_t* pos,
                              const int32_t* neg, int64_t batch, float* loss, float* coef,
                              void* stream) {
  using namespace tinykg;
  if (!layers || !dims || n_layers <= 0 || n_layers > kMaxLayers) return TINYKG_ERR_INVALID_ARG;
  if (n_nodes <= 0 || batch <= 0) return TINYKG_ERR_SHAPE;
  if (!users || !pos || !neg || !loss || !coef) return TINYKG_ERR_INVALID_ARG;
  LayerSet L;
  L.n = n_layers;
  for (int l = 0; l < n_layers; ++l) {
    if (!layers[l] || !aligned16(layers[l])) return TINYKG_ERR_INVALID_ARG;
    if (dims[l] <= 0 || dims[l] > 128 || dims[l] % 4 != 0) return TINYKG_ERR_UNSUPPORTED;
    L.ptr[l] = layers[l];
    L.dim[l] = dims[l];
  }
  hipStream_t st = (hipStream_t)stream;
  float* per_sample = coef + batch;   // second half of coef: per-sample loss terms
  {
    ProfileScope prof("bpr_loss_kernel", st);
    hipLaunchKernelGGL(bpr_loss_kernel, dim3((unsigned)((batch + 3) / 4)), dim3(256), 0, st, L, users,
                       pos, neg, batch, per_sample, coef);
  }
  tinykg_status rc = launch_status();
  if (rc != TINYKG_OK) return rc;
  ProfileScope prof("bpr_reduce_kernel", st);
  hipLaunchKernelGGL(bpr_reduce_kernel, dim3(1), dim3(256), 0, st, per_sample, batch, loss);
  return launch_status();
}

tinykg_status tinykg_bpr_grad(const float* E_l, int dim, int64_t n_nodes, const int32_t* users,
                              const int32_t* pos, const int32_t* neg, const float* coef,
                              int64_t batch, int accumulate, float* grad, void* stream) {
  using namespace tinykg;
  if (dim <= 0 || dim > 128 || dim % 4 != 0) return TINYKG_ERR_UNSUPPORTED;
  if (n_nodes <= 0 || batch <= 0) return TINYKG_ERR_SHAPE;
  if (!E_l || !users || !pos || !neg || !coef || !grad || !aligned16(E_l) || !aligned16(grad))
    return TINYKG_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (!accumulate) {
    const int64_t n4 = n_nodes * dim / 4;
    const int64_t want = (n4 + 255) / 256, cap = (int64_t)num_cus() * 16;
    ProfileScope prof("zero_f32_kernel", st);
    hipLaunchKernelGGL(zero_f32_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0, st,
                       reinterpret_cast<float4*>(grad), n4);
    tinykg_status rc = launch_status();
    if (rc != TINYKG_OK) return rc;
  }
  ProfileScope prof("bpr_grad_kernel", st);
  hipLaunchKernelGGL(bpr_grad_kernel, dim3((unsigned)((batch + 3) / 4)), dim3(256), 0, st, E_l, dim,
                     users, pos, neg, coef, batch, grad);
  return launch_status();
}

tinykg_status tinykg_readout_ids(const int32_t* users, const int32_t* pos, const int32_t* neg,
                                 int64_t batch, int32_t* ids, int32_t* slot, void* stream) {
  using namespace tinykg;
  if (batch < 0 || 3 * batch >= ((int64_t)1 << 31)) return TINYKG_ERR_SHAPE;
  if (batch == 0) return TINYKG_OK;
  if (!users || !pos || !neg || !ids || !slot) return TINYKG_ERR_INVALID_ARG;
  const int64_t want = (3 * batch + 255) / 256, cap = (int64_t)num_cus() * 16;
  ProfileScope prof("readout_ids_kernel", (hipStream_t)stream);
  hipLaunchKernelGGL(readout_ids_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0,
                     (hipStream_t)stream, users, pos, neg, batch, ids, slot);
  return launch_status();
}

}  // extern "C"
