// Batch normalisation over the rows (training mode) whose saved input is compressed, for
// gfx950.  Sec. 4.1.4 names BatchNorm among the operators that keep a compressed context:
// the forward pass is exact and saves Q(x; seed) (Eq. 3) with the column means and inverse
// standard deviations; the backward pass evaluates the operator's vector-Jacobian product
// at x_hat, dequantised (Eq. 4) inside the two passes that read it.
//
// Every kernel here is a stream over [rows, dim] tensors and is bound by HBM:
//   forward   bn_stats_kernel<32, false>   column sums of (x - K), (x - K)^2   reads x
//             bn_finish_fwd_kernel         mu, rstd, the column tables         (tiny)
//             quantizer with the affine hook: Q(x) and y in one pass           reads x, writes y + Q(x)
//   backward  bn_stats_kernel<BITS, true>  column sums of g, g xbar            reads g + Q(x)
//             bn_finish_bwd_kernel         grad_gamma, grad_beta, tables       (tiny)
//             bn_apply_bwd_kernel<BITS>    grad_x                              reads g + Q(x), writes grad_x
// Column sums: fp32 over at most 16 rows per thread, then double; per-workgroup partials are
// combined in a fixed order, so every output is deterministic.
#include "tinykg_common.h"
#include "tinykg_fetch.h"

#include <algorithm>
#include <atomic>

namespace tinykg {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxStatBlocks = 2048;
constexpr int kFinishThreads = 1024;
constexpr int kFlushRows = 16;      // fp32 terms per thread between two flushes to double (tail: < 24)
constexpr int kStatUFwd = 8, kStatUBwd = 4;   // rows a thread has in flight in the column-sum kernel
constexpr int kApplyU = 4;          // chunks per thread in the elementwise kernels

typedef float floatx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream(const float4* p) {
  const floatx4 v = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(float4* p, const float4& v) {
  floatx4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<floatx4*>(p));
}

// Column sums of two per-element quantities over the rows of one workgroup's slab.
//   BWD == false: (x - K_c) and (x - K_c)^2, K_c = x[0, c] (shifted sums: no cancellation
//                 in the variance when |mean| >> std)
//   BWD == true:  g and g * xbar, xbar = (x_hat - mu_c) * rstd_c
// Thread t owns column chunk t % lpr of rows t / lpr, t / lpr + rg, ... of the slab.
// part: [gridDim.x][2][dim] doubles.
template <int BITS, bool BWD>
__global__ __launch_bounds__(kThreads) void bn_stats_kernel(Source src, const float* __restrict__ g,
                                                            const float* __restrict__ mu,
                                                            const float* __restrict__ rstd,
                                                            int64_t rows, int lpr, int64_t rows_per_block,
                                                            double* __restrict__ part) {
  __shared__ double red[kThreads][8];
  const int tid = threadIdx.x;
  const int rg = kThreads / lpr;                       // rows in flight per workgroup step
  const int li = tid % lpr, rin = tid / lpr;
  const bool active = rin < rg;
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
  const int64_t r1 = min(rows, r0 + rows_per_block);
  double d1[4] = {0, 0, 0, 0}, d2[4] = {0, 0, 0, 0};
  if (active) {
    float4 k = make_float4(0.f, 0.f, 0.f, 0.f), rs = k;
    if (BWD) {
      k = reinterpret_cast<const float4*>(mu)[li];
      rs = reinterpret_cast<const float4*>(rstd)[li];
    } else {
      k = fetch_chunk<BITS>(src, li);                  // row 0
    }
    const float rv[4] = {rs.x, rs.y, rs.z, rs.w};
    float s1[4] = {0, 0, 0, 0}, s2[4] = {0, 0, 0, 0};
    auto add = [&](const float4& x, const float4& gg) {
      const float v[4] = {x.x - k.x, x.y - k.y, x.z - k.z, x.w - k.w};
      const float gv[4] = {gg.x, gg.y, gg.z, gg.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (BWD) { s1[j] += gv[j]; s2[j] = fmaf(gv[j], v[j] * rv[j], s2[j]); }
        else { s1[j] += v[j]; s2[j] = fmaf(v[j], v[j], s2[j]); }
      }
    };
    auto flush = [&]() {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        d1[j] += (double)s1[j]; d2[j] += (double)s2[j];
        s1[j] = 0.f; s2[j] = 0.f;
      }
    };
    auto fetch_x = [&](int64_t c) {
      if (BITS == 32) return load_stream(reinterpret_cast<const float4*>(src.data) + c);
      return fetch_chunk<BITS>(src, c);
    };
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    constexpr int kStatU = BWD ? kStatUBwd : kStatUFwd;
    int64_t r = r0 + rin;
    int pending = 0;
    // whole batches of kStatU rows: all loads of a batch are issued before the first use
    while (r + (int64_t)(kStatU - 1) * rg < r1) {
      float4 xs[kStatU], gs[kStatU];
#pragma unroll
      for (int u = 0; u < kStatU; ++u) {
        const int64_t c = (r + (int64_t)u * rg) * lpr + li;
        xs[u] = fetch_x(c);
        gs[u] = BWD ? load_stream(reinterpret_cast<const float4*>(g) + c) : zero4;
      }
#pragma unroll
      for (int u = 0; u < kStatU; ++u) add(xs[u], gs[u]);
      r += (int64_t)kStatU * rg;
      pending += kStatU;
      if (pending >= kFlushRows) { flush(); pending = 0; }
    }
    for (; r < r1; r += rg) {
      const int64_t c = r * lpr + li;
      add(fetch_x(c), BWD ? load_stream(reinterpret_cast<const float4*>(g) + c) : zero4);
    }
    flush();
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) { red[tid][j] = d1[j]; red[tid][4 + j] = d2[j]; }
  __syncthreads();
  if (tid < lpr) {
    double t[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int q = 0; q < rg; ++q)
#pragma unroll
      for (int j = 0; j < 8; ++j) t[j] += red[q * lpr + tid][j];
    const int dim = lpr * 4;
    double* out = part + (size_t)blockIdx.x * 2 * dim;
#pragma unroll
    for (int j = 0; j < 4; ++j) { out[tid * 4 + j] = t[j]; out[dim + tid * 4 + j] = t[4 + j]; }
  }
}

// Sums of the per-workgroup partials in a fixed order.  Workgroup b owns the kFinishCols
// columns from b * kFinishCols on; its threads split the partials of a column into
// kFinishThreads / kFinishCols interleaved subsets, combined in two steps through LDS.
// Returns the column (threads below kFinishCols hold its two sums), -1 elsewhere.
constexpr int kFinishCols = 4;
__device__ __forceinline__ int sum_partials(const double* part, int n_part, int dim, double* lds,
                                            double& t0, double& t1) {
  constexpr int kparts = kFinishThreads / kFinishCols, kStep = 16;
  const int tid = threadIdx.x;
  const int cl = tid % kFinishCols, k = tid / kFinishCols;
  const int c = blockIdx.x * kFinishCols + cl;
  double a0 = 0.0, a1 = 0.0;
  for (int b = k; b < n_part; b += kparts) {
    a0 += part[(size_t)b * 2 * dim + c];
    a1 += part[(size_t)b * 2 * dim + dim + c];
  }
  lds[tid * 2] = a0; lds[tid * 2 + 1] = a1;
  __syncthreads();
  a0 = 0.0; a1 = 0.0;
  if (k < kparts / kStep)
    for (int q = k * kStep; q < (k + 1) * kStep; ++q) { a0 += lds[(q * kFinishCols + cl) * 2]; a1 += lds[(q * kFinishCols + cl) * 2 + 1]; }
  __syncthreads();
  if (k < kparts / kStep) { lds[tid * 2] = a0; lds[tid * 2 + 1] = a1; }
  __syncthreads();
  t0 = 0.0; t1 = 0.0;
  if (tid >= kFinishCols) return -1;
  for (int q = 0; q < kparts / kStep; ++q) { t0 += lds[(q * kFinishCols + cl) * 2]; t1 += lds[(q * kFinishCols + cl) * 2 + 1]; }
  return c;
}

// tab: [3][dim] = fl(mu), a = gamma * rstd, b = beta - (mu - fl(mu)) a (what the normalising pass reads)
__global__ __launch_bounds__(kFinishThreads) void bn_finish_fwd_kernel(
    const double* __restrict__ part, int n_part, const float* __restrict__ x_row0,
    const float* __restrict__ gamma, const float* __restrict__ beta, float eps, int64_t rows, int dim,
    float* __restrict__ mean, float* __restrict__ rstd, float* __restrict__ tab) {
  __shared__ double lds[kFinishThreads * 2];
  double s1, s2;
  const int c = sum_partials(part, n_part, dim, lds, s1, s2);
  if (c >= 0) {
    const double m = s1 / (double)rows;
    const double var = fmax(s2 / (double)rows - m * m, 0.0);
    const double mu_d = (double)x_row0[c] + m, rs_d = 1.0 / sqrt(var + (double)eps);
    const float mu = (float)mu_d;
    mean[c] = mu; rstd[c] = (float)rs_d;
    // y = (x - mu) a + b with the part of the mean that fp32 cannot hold moved into b:
    // x - fl(mu) is exact for x near mu, and (mu - fl(mu)) a is far below beta's own ulp scale
    const double a = (double)gamma[c] * rs_d;
    tab[c] = mu; tab[dim + c] = (float)a; tab[2 * dim + c] = (float)((double)beta[c] - (mu_d - (double)mu) * a);
  }
}

// tab: [4][dim] = mu, A, B, C with grad_x = A g + B + C (x_hat - mu):
// A = gamma rstd, B = -A grad_beta / n, C = -A rstd grad_gamma / n
__global__ __launch_bounds__(kFinishThreads) void bn_finish_bwd_kernel(
    const double* __restrict__ part, int n_part, const float* __restrict__ mean,
    const float* __restrict__ rstd, const float* __restrict__ gamma, int64_t rows, int dim,
    float* __restrict__ grad_gamma, float* __restrict__ grad_beta, float* __restrict__ tab) {
  __shared__ double lds[kFinishThreads * 2];
  double gb, gg;
  const int c = sum_partials(part, n_part, dim, lds, gb, gg);
  if (c >= 0) {
    grad_beta[c] = (float)gb; grad_gamma[c] = (float)gg;
    const double A = (double)gamma[c] * (double)rstd[c];
    tab[c] = mean[c];
    tab[dim + c] = (float)A;
    tab[2 * dim + c] = (float)(-A * gb / (double)rows);
    tab[3 * dim + c] = (float)(-A * (double)rstd[c] * gg / (double)rows);
  }
}

// Column position of chunk c0 and of the chunks kThreads, 2 kThreads, ... after it.
struct ColumnWalk {
  uint32_t col, lpr, step;
  __device__ __forceinline__ ColumnWalk(int64_t c0, int lpr_) : lpr((uint32_t)lpr_) {
    col = (uint32_t)c0 % lpr;
    step = (uint32_t)kThreads % lpr;
  }
  __device__ __forceinline__ void next() { col += step; col = col >= lpr ? col - lpr : col; }
};

template <int BITS>
__global__ __launch_bounds__(kThreads) void bn_apply_bwd_kernel(Source src, const float* __restrict__ g,
                                                                const float* __restrict__ tab,
                                                                int64_t n_chunks, int lpr,
                                                                float* __restrict__ grad_x) {
  const int64_t c0 = (int64_t)blockIdx.x * (kThreads * kApplyU) + threadIdx.x;
  const float4* T = reinterpret_cast<const float4*>(tab);
  float4 xh[kApplyU], gg[kApplyU];
#pragma unroll
  for (int u = 0; u < kApplyU; ++u) {
    const int64_t c = c0 + u * kThreads;
    if (c < n_chunks) {
      xh[u] = fetch_chunk<BITS>(src, c);
      gg[u] = load_stream(reinterpret_cast<const float4*>(g) + c);
    }
  }
  ColumnWalk w(c0, lpr);
#pragma unroll
  for (int u = 0; u < kApplyU; ++u) {
    const int64_t c = c0 + u * kThreads;
    if (c < n_chunks) {
      const float4 m = T[w.col], A = T[lpr + w.col], B = T[2 * lpr + w.col], C = T[3 * lpr + w.col];
      float4 o;
      o.x = fmaf(C.x, xh[u].x - m.x, fmaf(A.x, gg[u].x, B.x));
      o.y = fmaf(C.y, xh[u].y - m.y, fmaf(A.y, gg[u].y, B.y));
      o.z = fmaf(C.z, xh[u].z - m.z, fmaf(A.z, gg[u].z, B.z));
      o.w = fmaf(C.w, xh[u].w - m.w, fmaf(A.w, gg[u].w, B.w));
      store_stream(reinterpret_cast<float4*>(grad_x) + c, o);
    }
    w.next();
  }
}

// bits == 32 forward: y from the tables, and the fp32 copy of x that stands for Q(x)
__global__ __launch_bounds__(kThreads) void bn_apply_fwd_copy_kernel(const float* __restrict__ x,
                                                                     const float* __restrict__ tab,
                                                                     int64_t n_chunks, int lpr,
                                                                     float* __restrict__ y,
                                                                     float* __restrict__ copy) {
  const int64_t c0 = (int64_t)blockIdx.x * (kThreads * kApplyU) + threadIdx.x;
  const float4* T = reinterpret_cast<const float4*>(tab);
  ColumnWalk w(c0, lpr);
#pragma unroll
  for (int u = 0; u < kApplyU; ++u) {
    const int64_t c = c0 + u * kThreads;
    if (c < n_chunks) {
      const float4 v = load_stream(reinterpret_cast<const float4*>(x) + c);
      const float4 m = T[w.col], a = T[lpr + w.col], b = T[2 * lpr + w.col];
      float4 o;
      o.x = fmaf(v.x - m.x, a.x, b.x); o.y = fmaf(v.y - m.y, a.y, b.y);
      o.z = fmaf(v.z - m.z, a.z, b.z); o.w = fmaf(v.w - m.w, a.w, b.w);
      store_stream(reinterpret_cast<float4*>(y) + c, o);
      store_stream(reinterpret_cast<float4*>(copy) + c, v);
    }
    w.next();
  }
}

struct NormWs { size_t part, tab, total; };
NormWs norm_layout(int dim) {
  NormWs w;
  w.part = 0;
  w.tab = (size_t)kMaxStatBlocks * 2 * dim * sizeof(double);
  w.total = w.tab + (size_t)4 * dim * sizeof(float);
  return w;
}

struct StatGrid { int blocks; int64_t rows_per_block; };
StatGrid stat_grid(int64_t rows, int dim) {
  const int lpr = dim / 4, rg = kThreads / lpr;
  const int64_t per = (int64_t)rg * 8;                 // at least 8 rows per thread
  int64_t blocks = std::min<int64_t>(kMaxStatBlocks, (rows + per - 1) / per);
  blocks = std::max<int64_t>(blocks, 1);
  int64_t rpb = (rows + blocks - 1) / blocks;
  rpb = (rpb + rg - 1) / rg * rg;
  blocks = (rows + rpb - 1) / rpb;
  return StatGrid{(int)blocks, rpb};
}

tinykg_status check_norm(int64_t rows, int dim, int bits, int group) {
  if (!(bits == 32 || bits_ok(bits))) return TINYKG_ERR_INVALID_ARG;
  if (bits != 32 && !group_ok(group)) return TINYKG_ERR_INVALID_ARG;
  if (rows < 0) return TINYKG_ERR_SHAPE;
  if (dim < 4 || dim > 1024 || dim % 4 != 0) return TINYKG_ERR_UNSUPPORTED;
  if (rows * dim >= ((int64_t)1 << 34)) return TINYKG_ERR_UNSUPPORTED;
  if (bits != 32 && (rows * dim) % group != 0) return TINYKG_ERR_SHAPE;
  return TINYKG_OK;
}

int ilog2i(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

template <int BITS>
tinykg_status bwd_impl(Source src, const float* mean, const float* rstd, const float* gamma, int64_t rows,
                       int dim, const float* grad_y, float* grad_x, float* grad_gamma, float* grad_beta,
                       uint8_t* ws, hipStream_t st) {
  const NormWs L = norm_layout(dim);
  double* part = reinterpret_cast<double*>(ws + L.part);
  float* tab = reinterpret_cast<float*>(ws + L.tab);
  const int lpr = dim / 4;
  const StatGrid sg = stat_grid(rows, dim);
  {
    ProfileScope prof("bn_stats_kernel<bwd>", st);
    hipLaunchKernelGGL((bn_stats_kernel<BITS, true>), dim3(sg.blocks), dim3(kThreads), 0, st, src, grad_y, mean,
                       rstd, rows, lpr, sg.rows_per_block, part);
  }
  hipLaunchKernelGGL(bn_finish_bwd_kernel, dim3(dim / kFinishCols), dim3(kFinishThreads), 0, st, part, sg.blocks, mean, rstd,
                     gamma, rows, dim, grad_gamma, grad_beta, tab);
  const int64_t n_chunks = rows * lpr;
  const int64_t blocks = (n_chunks + kThreads * kApplyU - 1) / (kThreads * kApplyU);
  {
    ProfileScope prof("bn_apply_bwd_kernel", st);
    hipLaunchKernelGGL((bn_apply_bwd_kernel<BITS>), dim3((unsigned)blocks), dim3(kThreads), 0, st, src, grad_y,
                       tab, n_chunks, lpr, grad_x);
  }
  return launch_status();
}

// Argument checks and dispatch shared by tinykg_batchnorm_bwd and its static-scratch variant
// (shape and bits / group already checked; ws holds norm_layout(dim).total bytes).
tinykg_status batchnorm_bwd_body(const uint8_t* packed, const float* gmin, const float* gscale,
                                 const float* mean, const float* rstd, const float* gamma, int64_t rows,
                                 int dim, int bits, int group, const float* grad_y, float* grad_x,
                                 float* grad_gamma, float* grad_beta, uint8_t* ws, hipStream_t st) {
  tinykg_status rc;
  if (!mean || !rstd || !gamma || !grad_gamma || !grad_beta) return TINYKG_ERR_INVALID_ARG;
  if (!aligned16(mean) || !aligned16(rstd) || !aligned16(gamma) || !aligned16(grad_gamma) ||
      !aligned16(grad_beta))
    return TINYKG_ERR_INVALID_ARG;
  if (rows == 0) {   // empty sums
    if ((rc = tinykg_fill_zero(grad_gamma, dim, st)) != TINYKG_OK) return rc;
    return tinykg_fill_zero(grad_beta, dim, st);
  }
  if (!packed || !grad_y || !grad_x || !aligned16(packed) || !aligned16(grad_y) || !aligned16(grad_x))
    return TINYKG_ERR_INVALID_ARG;
  if (bits != 32 && (!gmin || !gscale || !aligned16(gmin) || !aligned16(gscale))) return TINYKG_ERR_INVALID_ARG;
  const Source src{packed, gmin, gscale, bits == 32 ? 0 : ilog2i(group / 4)};
  switch (bits) {
    case 1: return bwd_impl<1>(src, mean, rstd, gamma, rows, dim, grad_y, grad_x, grad_gamma, grad_beta, ws, st);
    case 2: return bwd_impl<2>(src, mean, rstd, gamma, rows, dim, grad_y, grad_x, grad_gamma, grad_beta, ws, st);
    case 4: return bwd_impl<4>(src, mean, rstd, gamma, rows, dim, grad_y, grad_x, grad_gamma, grad_beta, ws, st);
    case 8: return bwd_impl<8>(src, mean, rstd, gamma, rows, dim, grad_y, grad_x, grad_gamma, grad_beta, ws, st);
    case 32: return bwd_impl<32>(src, mean, rstd, gamma, rows, dim, grad_y, grad_x, grad_gamma, grad_beta, ws, st);
  }
  return TINYKG_ERR_INVALID_ARG;
}

// Scratch of tinykg_batchnorm_bwd_static: the partial sums and the coefficient table of a
// layer of at most kStaticMaxDim columns, in device memory that belongs to the library's code
// object (every GPU that loads the library holds its own copy until the process ends).
constexpr int kStaticMaxDim = 128;
constexpr size_t kStaticScratchBytes =
    (size_t)kMaxStatBlocks * 2 * kStaticMaxDim * sizeof(double) + (size_t)4 * kStaticMaxDim * sizeof(float);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// The array's address on the current device.  In host code the array's name only stands for
// the symbol; its device address is asked for once per device (with that device current) and
// kept.  Two threads racing here store the same value.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

tinykg_status static_scratch(uint8_t** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return TINYKG_ERR_DEVICE; }
  if (dev < 0 || dev >= kMaxDevices) return TINYKG_ERR_UNSUPPORTED;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return TINYKG_ERR_DEVICE;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = static_cast<uint8_t*>(p);
  return TINYKG_OK;
}

}  // namespace

}  // namespace tinykg

using namespace tinykg;

extern "C" {

size_t tinykg_batchnorm_workspace_bytes(int64_t rows, int dim) {
  if (check_norm(rows, dim, 32, 0) != TINYKG_OK) return 0;
  return norm_layout(dim).total;
}

tinykg_status tinykg_batchnorm_fwd(const float* x, int64_t rows, int dim, const float* gamma,
                                   const float* beta, float eps, int bits, int group, uint64_t seed,
                                   float* y, uint8_t* packed, float* gmin, float* gscale, float* mean,
                                   float* rstd, void* workspace, size_t workspace_bytes, void* stream) {
  tinykg_status rc;
  if ((rc = check_norm(rows, dim, bits, group)) != TINYKG_OK) return rc;
  if (!(eps >= 0.f)) return TINYKG_ERR_INVALID_ARG;
  if (rows == 0) return TINYKG_OK;
  if (!x || !gamma || !beta || !y || !packed || !mean || !rstd) return TINYKG_ERR_INVALID_ARG;
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(y) || !aligned16(packed) ||
      !aligned16(mean) || !aligned16(rstd))
    return TINYKG_ERR_INVALID_ARG;
  if (bits != 32 && (!gmin || !gscale || !aligned16(gmin) || !aligned16(gscale))) return TINYKG_ERR_INVALID_ARG;
  const NormWs L = norm_layout(dim);
  if (!workspace || !aligned16(workspace) || workspace_bytes < L.total) return TINYKG_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  double* part = reinterpret_cast<double*>(ws + L.part);
  float* tab = reinterpret_cast<float*>(ws + L.tab);
  const int lpr = dim / 4;
  const StatGrid sg = stat_grid(rows, dim);
  const Source src{reinterpret_cast<const uint8_t*>(x), nullptr, nullptr, 0};
  {
    ProfileScope prof("bn_stats_kernel<fwd>", st);
    hipLaunchKernelGGL((bn_stats_kernel<32, false>), dim3(sg.blocks), dim3(kThreads), 0, st, src,
                       (const float*)nullptr, (const float*)nullptr, (const float*)nullptr, rows, lpr,
                       sg.rows_per_block, part);
  }
  hipLaunchKernelGGL(bn_finish_fwd_kernel, dim3(dim / kFinishCols), dim3(kFinishThreads), 0, st, part, sg.blocks, x, gamma, beta,
                     eps, rows, dim, mean, rstd, tab);
  if ((rc = launch_status()) != TINYKG_OK) return rc;
  if (bits == 32) {
    const int64_t n_chunks = rows * lpr;
    const int64_t blocks = (n_chunks + kThreads * kApplyU - 1) / (kThreads * kApplyU);
    ProfileScope prof("bn_apply_fwd_copy_kernel", st);
    hipLaunchKernelGGL(bn_apply_fwd_copy_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, x, tab, n_chunks,
                       lpr, y, reinterpret_cast<float*>(packed));
    return launch_status();
  }
  return launch_quantize_affine(x, rows * dim, bits, group, seed, packed, gmin, gscale, dim, tab, tab + dim,
                                tab + 2 * dim, y, st);
}

tinykg_status tinykg_batchnorm_bwd(const uint8_t* packed, const float* gmin, const float* gscale,
                                   const float* mean, const float* rstd, const float* gamma, int64_t rows,
                                   int dim, int bits, int group, const float* grad_y, float* grad_x,
                                   float* grad_gamma, float* grad_beta, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  tinykg_status rc;
  if ((rc = check_norm(rows, dim, bits, group)) != TINYKG_OK) return rc;
  const NormWs L = norm_layout(dim);
  if (!workspace || !aligned16(workspace) || workspace_bytes < L.total) return TINYKG_ERR_WORKSPACE;
  return batchnorm_bwd_body(packed, gmin, gscale, mean, rstd, gamma, rows, dim, bits, group, grad_y, grad_x,
                            grad_gamma, grad_beta, static_cast<uint8_t*>(workspace), (hipStream_t)stream);
}

tinykg_status tinykg_batchnorm_bwd_static(const uint8_t* packed, const float* gmin, const float* gscale,
                                          const float* mean, const float* rstd, const float* gamma,
                                          int64_t rows, int dim, int bits, int group, const float* grad_y,
                                          float* grad_x, float* grad_gamma, float* grad_beta, void* stream) {
  tinykg_status rc;
  if ((rc = check_norm(rows, dim, bits, group)) != TINYKG_OK) return rc;
  if (dim > kStaticMaxDim || norm_layout(dim).total > kStaticScratchBytes) return TINYKG_ERR_UNSUPPORTED;
  uint8_t* ws = nullptr;
  if ((rc = static_scratch(&ws)) != TINYKG_OK) return rc;
  ProfileMute mute;   // no event is created or recorded on this path
  return batchnorm_bwd_body(packed, gmin, gscale, mean, rstd, gamma, rows, dim, bits, group, grad_y, grad_x,
                            grad_gamma, grad_beta, ws, (hipStream_t)stream);
}

}  // extern "C"
