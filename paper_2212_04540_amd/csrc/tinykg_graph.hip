// tinykg_graph: the immutable sparse structure shared by every layer and step
// (Sec. 3.2, "Memory Analysis": the adjacency is kept once for all layers).
//
// Built once, off the hot path, from device COO triplets:
//   * head order  -- triplets sorted by (head, relation, tail): CSR row pointers
//     and the tail of every edge.  The softmax / gather kernels walk it.
//   * relation order -- the same edges sorted by (relation, tail, head), cut into
//     chunks that never straddle a relation.  The projection kernels (dense
//     contractions with one W_r) walk it; sorting by tail inside a relation puts
//     the edges of a hot tail next to each other, so their gradient rows are
//     summed before they leave the workgroup.
// Everything that touches every edge runs on the device (stable radix sorts of rocPRIM
// through hipCUB, gathers, degree counts, the per-tile row orders); the host only walks
// per-node and per-tile summaries (degrees, one byte per 32-edge tile) to lay out chunks,
// spans and the lists of heavy nodes.  150 M triplets take a few seconds instead of most
// of a minute on the host.
#include "tinykg_graph.h"

#include <hipcub/hipcub.hpp>

#include <algorithm>
#include <numeric>
#include <vector>

namespace tinykg {

namespace {

// Time of a one-tail tile of the edge-level backward kernel (d <= 64) relative to an ordinary one.
constexpr double kOneTailTileCost = 0.7;
// The same for the code form of that kernel (every product on the bf16 matrix cores: a one-tail
// tile saves nothing there but scatters less; 0.8 .. 1.0 measure alike).
constexpr double kOneTailTileCostCode = 0.9;

template <typename T>
tinykg_status upload(const std::vector<T>& v, T** out) {
  *out = nullptr;
  const size_t bytes = std::max<size_t>(v.size(), 1) * sizeof(T);
  TINYKG_HIP_TRY(hipMalloc(reinterpret_cast<void**>(out), bytes));
  if (!v.empty()) TINYKG_HIP_TRY(hipMemcpy(*out, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return TINYKG_OK;
}

// Device memory that lives only while the graph is being built.
struct Scratch {
  std::vector<void*> ptrs;
  ~Scratch() { for (void* p : ptrs) (void)hipFree(p); }
  template <typename T>
  tinykg_status get(size_t n, T** out) {
    *out = nullptr;
    void* p = nullptr;
    TINYKG_HIP_TRY(hipMalloc(&p, std::max<size_t>(n, 1) * sizeof(T)));
    ptrs.push_back(p);
    *out = static_cast<T*>(p);
    return TINYKG_OK;
  }
};

template <typename T>
tinykg_status device_array(size_t n, T** out) {
  *out = nullptr;
  TINYKG_HIP_TRY(hipMalloc(reinterpret_cast<void**>(out), std::max<size_t>(n, 1) * sizeof(T)));
  return TINYKG_OK;
}

int bits_for(int64_t n_values) {   // bits that hold 0 .. n_values - 1
  int b = 1;
  while (((int64_t)1 << b) < n_values) ++b;
  return b;
}

constexpr int kBuildThreads = 256;
inline unsigned build_grid(size_t n) {
  const size_t want = (n + kBuildThreads - 1) / kBuildThreads;
  return (unsigned)std::max<size_t>(1, std::min<size_t>(want, (size_t)num_cus() * 32));
}

// ids outside [0, n_nodes) / [0, n_rel): *bad becomes nonzero
__global__ __launch_bounds__(kBuildThreads) void validate_kernel(const int32_t* __restrict__ head,
                                                                 const int32_t* __restrict__ rel,
                                                                 const int32_t* __restrict__ tail, size_t T,
                                                                 int32_t n_nodes, int32_t n_rel,
                                                                 int32_t* __restrict__ bad) {
  bool wrong = false;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < T; e += (size_t)gridDim.x * blockDim.x)
    wrong |= head[e] < 0 || head[e] >= n_nodes || tail[e] < 0 || tail[e] >= n_nodes || rel[e] < 0 ||
             rel[e] >= n_rel;
  if (wrong) atomicOr(bad, 1);
}

// key = relation * 2^30 + tail of edge e (node ids are below 2^30), value = e
__global__ __launch_bounds__(kBuildThreads) void rel_tail_keys_kernel(const int32_t* __restrict__ rel,
                                                                      const int32_t* __restrict__ tail, size_t T,
                                                                      uint64_t* __restrict__ key,
                                                                      int32_t* __restrict__ val) {
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < T; e += (size_t)gridDim.x * blockDim.x) {
    key[e] = ((uint64_t)(uint32_t)rel[e] << 30) | (uint32_t)tail[e];
    val[e] = (int32_t)e;
  }
}

__global__ __launch_bounds__(kBuildThreads) void iota_i32_kernel(int32_t* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = (int32_t)i;
}

// the tail order's arrays from the sorted head-order positions; bit 30 of a tail: accumulates in double
__global__ __launch_bounds__(kBuildThreads) void tail_order_kernel(const int32_t* __restrict__ h_head,
                                                                   const int32_t* __restrict__ h_tail,
                                                                   const int32_t* __restrict__ pos, size_t T,
                                                                   const int32_t* __restrict__ acc_slot,
                                                                   int32_t* __restrict__ c_head,
                                                                   int32_t* __restrict__ c_tail) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < T; i += (size_t)gridDim.x * blockDim.x) {
    const int32_t p = pos[i], t = h_tail[p];
    c_head[i] = h_head[p];
    c_tail[i] = t | (acc_slot[t] >= 0 ? 0x40000000 : 0);
  }
}

__global__ __launch_bounds__(kBuildThreads) void gather_i32_kernel(const int32_t* __restrict__ src,
                                                                   const int32_t* __restrict__ idx, size_t T,
                                                                   int32_t* __restrict__ dst) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < T; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[idx[i]];
}

__global__ __launch_bounds__(kBuildThreads) void fill_i32_kernel(int32_t* __restrict__ dst, size_t n, int32_t v) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = v;
}

// out_deg[head] and rows[head], rows[tail] (gradient rows a node receives) of every edge
__global__ __launch_bounds__(kBuildThreads) void degree_kernel(const int32_t* __restrict__ head,
                                                               const int32_t* __restrict__ tail, size_t T,
                                                               int32_t* __restrict__ out_deg,
                                                               int32_t* __restrict__ rows) {
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < T; e += (size_t)gridDim.x * blockDim.x) {
    atomicAdd(out_deg + head[e], 1);
    atomicAdd(rows + head[e], 1);
    atomicAdd(rows + tail[e], 1);
  }
}

// first[r] = first position of relation r in the ascending keys (r = n_rel: T)
__global__ __launch_bounds__(kBuildThreads) void rel_first_kernel(const uint64_t* __restrict__ key, size_t T,
                                                                  int32_t n_rel, int64_t* __restrict__ first) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r > n_rel) return;
  size_t lo = 0, hi = T;                    // first position whose relation is >= r
  while (lo < hi) {
    const size_t mid = (lo + hi) >> 1;
    if ((int64_t)(key[mid] >> 30) < (int64_t)r) lo = mid + 1; else hi = mid;
  }
  first[r] = (int64_t)lo;
}

// Relation-order tiles: 32 consecutive edges counted from the first edge of their relation.
// One 32-lane half wave per tile: whether its edges share one tail (tile_one[t] = 1), and the
// byte of every row -- bits 0-4: the tile-local row indices in stable head order (slot k holds
// the row of rank k); bit 6 / bit 7: the tail / head of THIS row accumulates in double.
__global__ __launch_bounds__(kBuildThreads) void tile_kernel(const int32_t* __restrict__ r_head,
                                                             const int32_t* __restrict__ r_tail,
                                                             const int64_t* __restrict__ rel_first,
                                                             const int64_t* __restrict__ rel_tile_ptr,
                                                             int32_t n_rel, int64_t n_tiles,
                                                             const int32_t* __restrict__ acc_slot,
                                                             uint8_t* __restrict__ tile_one,
                                                             uint8_t* __restrict__ hperm) {
  __shared__ uint8_t order[kBuildThreads];
  const int lane = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int64_t per_block = kBuildThreads / 32;
  for (int64_t t0 = (int64_t)blockIdx.x * per_block; t0 < n_tiles; t0 += (int64_t)gridDim.x * per_block) {
    const int64_t t = t0 + grp;
    const bool live = t < n_tiles;
    int nrow = 0;
    int64_t base = 0;
    if (live) {
      int lo = 0, hi = n_rel;                 // the relation r with tile_ptr[r] <= t < tile_ptr[r + 1]
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (rel_tile_ptr[mid] <= t) lo = mid; else hi = mid;
      }
      base = rel_first[lo] + 32 * (t - rel_tile_ptr[lo]);
      nrow = (int)min((int64_t)32, rel_first[lo + 1] - base);
    }
    const bool row = lane < nrow;
    const int h = row ? r_head[base + lane] : 0x7fffffff;
    const int tl = row ? r_tail[base + lane] : 0;
    const int t_first = __shfl(tl, 0, 32);
    const unsigned long long differ = __ballot(row && tl != t_first);
    const unsigned my_half = (unsigned)(differ >> (32 * ((threadIdx.x >> 5) & 1)));
    int rank = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      const int hj = __shfl(h, j, 32);
      rank += (hj < h || (hj == h && j < lane)) ? 1 : 0;
    }
    if (row) order[grp * 32 + rank] = (uint8_t)lane;
    __syncthreads();
    if (row)
      hperm[base + lane] = (uint8_t)(order[grp * 32 + lane] | (acc_slot[tl] >= 0 ? 0x40 : 0) |
                                     (acc_slot[h] >= 0 ? 0x80 : 0));
    if (live && lane == 0) tile_one[t] = my_half == 0 ? 1 : 0;
    __syncthreads();
  }
}

// keys_a -> sorted keys in *keys_sorted (one of the two buffers), values likewise; stable
tinykg_status sort_pairs_u64(Scratch& sc, uint64_t* ka, uint64_t* kb, int32_t* va, int32_t* vb, size_t T,
                             int end_bit, hipStream_t st, uint64_t** keys_sorted, int32_t** vals_sorted) {
  hipcub::DoubleBuffer<uint64_t> keys(ka, kb);
  hipcub::DoubleBuffer<int32_t> vals(va, vb);
  size_t temp_bytes = 0;
  TINYKG_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(nullptr, temp_bytes, keys, vals, (int)T, 0, end_bit, st));
  uint8_t* temp = nullptr;
  tinykg_status rc = sc.get(temp_bytes, &temp);
  if (rc != TINYKG_OK) return rc;
  TINYKG_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(temp, temp_bytes, keys, vals, (int)T, 0, end_bit, st));
  *keys_sorted = keys.Current();
  *vals_sorted = vals.Current();
  return TINYKG_OK;
}

tinykg_status sort_pairs_i32(Scratch& sc, int32_t* ka, int32_t* kb, int32_t* va, int32_t* vb, size_t T,
                             int end_bit, hipStream_t st, int32_t** vals_sorted) {
  hipcub::DoubleBuffer<int32_t> keys(ka, kb);
  hipcub::DoubleBuffer<int32_t> vals(va, vb);
  size_t temp_bytes = 0;
  TINYKG_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(nullptr, temp_bytes, keys, vals, (int)T, 0, end_bit, st));
  uint8_t* temp = nullptr;
  tinykg_status rc = sc.get(temp_bytes, &temp);
  if (rc != TINYKG_OK) return rc;
  TINYKG_HIP_TRY(hipcub::DeviceRadixSort::SortPairs(temp, temp_bytes, keys, vals, (int)T, 0, end_bit, st));
  *vals_sorted = vals.Current();
  return TINYKG_OK;
}

template <typename T>
tinykg_status download(const T* dev, size_t n, std::vector<T>& host, hipStream_t st) {
  host.resize(n);
  if (n) {
    TINYKG_HIP_TRY(hipMemcpyAsync(host.data(), dev, n * sizeof(T), hipMemcpyDeviceToHost, st));
    TINYKG_HIP_TRY(hipStreamSynchronize(st));
  }
  return TINYKG_OK;
}

void release(tinykg_graph* g) {
  if (!g) return;
  void* ptrs[] = {g->rowptr, g->h_tail, g->r_head, g->r_tail, g->r_eid, g->chunk_rel,
                  g->chunk_start, g->chunk_count, g->rel_chunk_ptr, g->heavy_head, g->heavy_seg_ptr,
                  g->hseg_q, g->hseg_e0, g->hseg_cnt, g->r_hperm32, g->acc_slot, g->acc_node, g->c_head, g->c_tail,
                  g->span_group_ptr, g->span_rel, g->span_start, g->span_count, g->rel_span_ptr,
                  g->espan_group_ptr, g->espan_rel, g->espan_start, g->espan_count, g->rel_espan_ptr};
  for (void* p : ptrs)
    if (p) (void)hipFree(p);
  delete g;
}

}  // namespace

}  // namespace tinykg

extern "C" {

tinykg_status tinykg_graph_create(int64_t n_nodes, int32_t n_rel, int64_t n_edges,
                                  const int32_t* head, const int32_t* rel, const int32_t* tail,
                                  void* stream, tinykg_graph** out) {
  using namespace tinykg;
  if (!out) return TINYKG_ERR_INVALID_ARG;
  if (n_nodes < 0 || n_rel < 0 || n_edges < 0) return TINYKG_ERR_SHAPE;
  if (n_nodes >= (int64_t)1 << 30 || n_edges >= (int64_t)1 << 31 || n_rel > 65535)
    return TINYKG_ERR_UNSUPPORTED;
  if (n_edges > 0 && (!head || !rel || !tail)) return TINYKG_ERR_INVALID_ARG;
  if (n_edges > 0 && n_rel == 0) return TINYKG_ERR_INVALID_ARG;

  const size_t T = (size_t)n_edges, N = (size_t)n_nodes;
  hipStream_t st = (hipStream_t)stream;
  Scratch sc;
  tinykg_status rc;
#define TINYKG_TRY(expr) do { if ((rc = (expr)) != TINYKG_OK) return rc; } while (0)
  // (freed on every early return; handed to the caller at the end)
  struct Guard { tinykg_graph* g = nullptr; ~Guard() { release(g); } } guard;
  tinykg_graph*& g = guard.g;

  // ---- ids in range?
  if (T) {
    int32_t* bad = nullptr;
    TINYKG_TRY(sc.get(1, &bad));
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(kBuildThreads), 0, st, bad, (size_t)1, 0);
    hipLaunchKernelGGL(validate_kernel, dim3(build_grid(T)), dim3(kBuildThreads), 0, st, head, rel, tail, T,
                       (int32_t)n_nodes, n_rel, bad);
    std::vector<int32_t> flag;
    TINYKG_TRY(download(bad, 1, flag, st));
    if (flag[0] != 0) return TINYKG_ERR_INVALID_ARG;
  }

  g = new tinykg_graph();
  g->n_nodes = n_nodes; g->n_edges = n_edges; g->n_rel = n_rel;
  TINYKG_TRY(device_array(N + 1, &g->rowptr));
  TINYKG_TRY(device_array(T, &g->h_tail));
  TINYKG_TRY(device_array(T, &g->r_head));
  TINYKG_TRY(device_array(T, &g->r_tail));
  TINYKG_TRY(device_array(T, &g->r_eid));
  TINYKG_TRY(device_array(T, &g->r_hperm32));
  TINYKG_TRY(device_array(T, &g->c_head));
  TINYKG_TRY(device_array(T, &g->c_tail));

  // ---- degrees; CSR row pointers = exclusive prefix sums of the out-degrees
  int32_t *out_deg = nullptr, *rows = nullptr;
  TINYKG_TRY(sc.get(N + 1, &out_deg));
  TINYKG_TRY(sc.get(N + 1, &rows));
  hipLaunchKernelGGL(fill_i32_kernel, dim3(build_grid(N + 1)), dim3(kBuildThreads), 0, st, out_deg, N + 1, 0);
  hipLaunchKernelGGL(fill_i32_kernel, dim3(build_grid(N + 1)), dim3(kBuildThreads), 0, st, rows, N + 1, 0);
  if (T) hipLaunchKernelGGL(degree_kernel, dim3(build_grid(T)), dim3(kBuildThreads), 0, st, head, tail, T, out_deg, rows);
  {
    size_t temp_bytes = 0;
    if (hipcub::DeviceScan::ExclusiveSum(nullptr, temp_bytes, out_deg, g->rowptr, (int)(N + 1), st) != hipSuccess) return TINYKG_ERR_DEVICE;
    uint8_t* temp = nullptr;
    TINYKG_TRY(sc.get(temp_bytes, &temp));
    if (hipcub::DeviceScan::ExclusiveSum(temp, temp_bytes, out_deg, g->rowptr, (int)(N + 1), st) != hipSuccess) return TINYKG_ERR_DEVICE;
  }
  std::vector<int32_t> h_out_deg, h_rows;
  TINYKG_TRY(download(out_deg, N, h_out_deg, st));
  TINYKG_TRY(download(rows, N, h_rows, st));

  // ---- heavy heads (cut into segments of kHeavyDegree head-order edges) and the nodes whose
  //      gradient rows are accumulated in double
  std::vector<int32_t> heavy_head, heavy_seg_ptr(1, 0), hseg_q, hseg_e0, hseg_cnt;
  std::vector<int32_t> acc_slot(N, -1), acc_node;
  {
    int64_t e0 = 0;
    for (size_t h = 0; h < N; ++h) {
      const int32_t deg = h_out_deg[h];
      g->max_out_degree = std::max(g->max_out_degree, deg);
      if (deg > kHeavyDegree) {
        const int32_t q = (int32_t)heavy_head.size();
        heavy_head.push_back((int32_t)h);
        for (int32_t o = 0; o < deg; o += kHeavyDegree) {
          hseg_q.push_back(q);
          hseg_e0.push_back((int32_t)(e0 + o));
          hseg_cnt.push_back(std::min<int32_t>(kHeavyDegree, deg - o));
        }
        heavy_seg_ptr.push_back((int32_t)hseg_q.size());
      }
      if (h_rows[h] > kAccHeavyDegree) {
        acc_slot[h] = (int32_t)acc_node.size();
        acc_node.push_back((int32_t)h);
      }
      e0 += deg;
    }
  }
  g->n_heavy = (int32_t)heavy_head.size();
  g->n_hseg = (int32_t)hseg_q.size();
  g->n_acc_heavy = (int32_t)acc_node.size();
  TINYKG_TRY(upload(heavy_head, &g->heavy_head));
  TINYKG_TRY(upload(heavy_seg_ptr, &g->heavy_seg_ptr));
  TINYKG_TRY(upload(hseg_q, &g->hseg_q));
  TINYKG_TRY(upload(hseg_e0, &g->hseg_e0));
  TINYKG_TRY(upload(hseg_cnt, &g->hseg_cnt));
  TINYKG_TRY(upload(acc_slot, &g->acc_slot));
  TINYKG_TRY(upload(acc_node, &g->acc_node));

  // ---- the two edge orders (stable radix sorts)
  std::vector<int64_t> rel_first((size_t)n_rel + 1, 0);
  if (T) {
    const int rt_bits = 30 + bits_for(std::max<int64_t>(n_rel, 2));
    uint64_t *ka = nullptr, *kb = nullptr, *ks = nullptr;
    int32_t *va = nullptr, *vb = nullptr, *ord = nullptr, *ha = nullptr, *hb = nullptr;
    TINYKG_TRY(sc.get(T, &ka)); TINYKG_TRY(sc.get(T, &kb));
    TINYKG_TRY(sc.get(T, &va)); TINYKG_TRY(sc.get(T, &vb));
    TINYKG_TRY(sc.get(T, &ha)); TINYKG_TRY(sc.get(T, &hb));
    // head order: by (relation, tail) first, then by head; both passes keep the order of
    // equal keys, so equal triplets stay in input order
    hipLaunchKernelGGL(rel_tail_keys_kernel, dim3(build_grid(T)), dim3(kBuildThreads), 0, st, rel, tail, T, ka, va);
    TINYKG_TRY(sort_pairs_u64(sc, ka, kb, va, vb, T, rt_bits, st, &ks, &ord));
    int32_t* other = ord == va ? vb : va;
    hipLaunchKernelGGL(gather_i32_kernel, dim3(build_grid(T)), dim3(kBuildThreads), 0, st, head, ord, T, ha);
    {
      hipcub::DoubleBuffer<int32_t> keys(ha, hb);
      hipcub::DoubleBuffer<int32_t> vals(ord, other);
      size_t temp_bytes = 0;
      const int hb_bits = bits_for(std::max<int64_t>(n_nodes, 2));
      if (hipcub::DeviceRadixSort::SortPairs(nullptr, temp_bytes, keys, vals, (int)T, 0, hb_bits, st) != hipSuccess) return TINYKG_ERR_DEVICE;
      uint8_t* temp = nullptr;
      TINYKG_TRY(sc.get(temp_bytes, &temp));
      if (hipcub::DeviceRadixSort::SortPairs(temp, temp_bytes, keys, vals, (int)T, 0, hb_bits, st) != hipSuccess) return TINYKG_ERR_DEVICE;
      ord = vals.Current();                 // input position of the edge at each head-order position
      other = ord == va ? vb : va;
      ha = keys.Current();                  // its head
    }
    int32_t *h_rel = nullptr;
    TINYKG_TRY(sc.get(T, &h_rel));
    hipLaunchKernelGGL(gather_i32_kernel, dim3(build_grid(T)), dim3(kBuildThreads), 0, st, rel, ord, T, h_rel);
    hipLaunchKernelGGL(gather_i32_kernel, dim3(build_grid(T)), dim3(kBuildThreads), 0, st, tail, ord, T, g->h_tail);
    // relation order over head-order positions: by (relation, tail); the sequence already
    // ascends in head, which a stable pass keeps
    int32_t* rord = nullptr;
    hipLaunchKernelGGL(rel_tail_keys_kernel, dim3(build_grid(T)), dim3(kBuildThreads), 0, st, h_rel, g->h_tail, T, ka, other);
    {
      int32_t* spare = ord;                 // the head-order permutation is no longer needed
      uint64_t* ks2 = nullptr;
      TINYKG_TRY(sort_pairs_u64(sc, ka, kb, other, spare, T, rt_bits, st, &ks2, &rord));
      ks = ks2;
    }
    hipLaunchKernelGGL(gather_i32_kernel, dim3(build_grid(T)), dim3(kBuildThreads), 0, st, ha, rord, T, g->r_head);
    hipLaunchKernelGGL(gather_i32_kernel, dim3(build_grid(T)), dim3(kBuildThreads), 0, st, g->h_tail, rord, T, g->r_tail);
    TINYKG_HIP_TRY(hipMemcpyAsync(g->r_eid, rord, T * 4, hipMemcpyDeviceToDevice, st));
    int64_t* d_first = nullptr;
    TINYKG_TRY(sc.get((size_t)n_rel + 1, &d_first));
    hipLaunchKernelGGL(rel_first_kernel, dim3((n_rel + 1 + kBuildThreads - 1) / kBuildThreads), dim3(kBuildThreads), 0,
                       st, ks, T, n_rel, d_first);
    TINYKG_TRY(download(d_first, (size_t)n_rel + 1, rel_first, st));

    // tail order over head-order positions: one stable pass by tail; heads ascend inside a tail
    {
      int32_t *ta = nullptr, *tb = nullptr, *cord = nullptr;
      TINYKG_TRY(sc.get(T, &ta)); TINYKG_TRY(sc.get(T, &tb));
      TINYKG_HIP_TRY(hipMemcpyAsync(ta, g->h_tail, T * 4, hipMemcpyDeviceToDevice, st));
      hipLaunchKernelGGL(iota_i32_kernel, dim3(build_grid(T)), dim3(kBuildThreads), 0, st, va, T);
      TINYKG_TRY(sort_pairs_i32(sc, ta, tb, va, vb, T, bits_for(std::max<int64_t>(n_nodes, 2)), st, &cord));
      hipLaunchKernelGGL(tail_order_kernel, dim3(build_grid(T)), dim3(kBuildThreads), 0, st, ha, g->h_tail, cord, T,
                         g->acc_slot, g->c_head, g->c_tail);
    }

    // per-tile summaries and per-row bytes
    std::vector<int64_t> rel_tile_ptr((size_t)n_rel + 1, 0);
    for (int32_t r = 0; r < n_rel; ++r)
      rel_tile_ptr[(size_t)r + 1] = rel_tile_ptr[(size_t)r] + (rel_first[(size_t)r + 1] - rel_first[(size_t)r] + 31) / 32;
    const int64_t n_tiles = rel_tile_ptr[(size_t)n_rel];
    int64_t* d_tile_ptr = nullptr;
    uint8_t* d_tile_one = nullptr;
    TINYKG_TRY(sc.get((size_t)n_rel + 1, &d_tile_ptr));
    TINYKG_TRY(sc.get((size_t)n_tiles, &d_tile_one));
    TINYKG_HIP_TRY(hipMemcpyAsync(d_tile_ptr, rel_tile_ptr.data(), ((size_t)n_rel + 1) * 8, hipMemcpyHostToDevice, st));
    TINYKG_HIP_TRY(hipStreamSynchronize(st));   // rel_tile_ptr is a local: the copy must have read it
    hipLaunchKernelGGL(tile_kernel, dim3(build_grid((size_t)n_tiles * 32)), dim3(kBuildThreads), 0, st, g->r_head,
                       g->r_tail, d_first, d_tile_ptr, n_rel, n_tiles, g->acc_slot, d_tile_one, g->r_hperm32);
    if (hipGetLastError() != hipSuccess) return TINYKG_ERR_DEVICE;
    std::vector<uint8_t> tile_one;
    TINYKG_TRY(download(d_tile_one, (size_t)n_tiles, tile_one, st));

    // chunks: runs of at most chunk_edges consecutive relation-order edges of one
    // relation; about 2048 of them: few enough that the per-chunk partial gradients stay
    // small and a workgroup amortises staging W_r, enough to fill 256 compute units.
    int64_t chunk_edges = ((n_edges / 2048 + 63) / 64) * 64;
    if (chunk_edges < 64) chunk_edges = 64;
    g->chunk_edges = (int32_t)chunk_edges;
    std::vector<int32_t> chunk_rel, chunk_start, chunk_count, rel_chunk_ptr((size_t)n_rel + 1, 0);
    for (int32_t r = 0; r < n_rel; ++r) {
      rel_chunk_ptr[(size_t)r] = (int32_t)chunk_rel.size();
      int64_t pos = rel_first[(size_t)r], left = rel_first[(size_t)r + 1] - pos;
      while (left > 0) {
        const int64_t c = std::min(left, chunk_edges);
        chunk_rel.push_back(r);
        chunk_start.push_back((int32_t)pos);
        chunk_count.push_back((int32_t)c);
        pos += c; left -= c;
      }
    }
    rel_chunk_ptr[(size_t)n_rel] = (int32_t)chunk_rel.size();
    g->n_chunks = (int32_t)chunk_rel.size();

    // spans of the persistent edge-level kernel (one group per compute unit): runs of whole
    // 32-edge tiles of one relation (tiles are counted from the relation's first edge).  The
    // groups get equal shares of the kernel's WORK, not of the edges: a tile whose edges share
    // one tail (popular tails own long runs of the relation order) takes the kernel's run form,
    // which skips a third of the matrix products.
    struct Spans { std::vector<int32_t> group_ptr, rel, start, count, rel_ptr; };
    auto cut_spans = [&](double one_tail_cost) {
      Spans S;
      S.group_ptr.assign(1, 0);
      S.rel_ptr.assign((size_t)n_rel + 1, 0);
      std::vector<int32_t>&span_group_ptr = S.group_ptr, &span_rel = S.rel, &span_start = S.start, &span_count = S.count,
                          &rel_span_ptr = S.rel_ptr;
      const int64_t n_groups = std::max<int64_t>(1, std::min<int64_t>(num_cus(), (int64_t)chunk_rel.size()));
      auto tile_cost = [&](int64_t t) { return tile_one[(size_t)t] ? one_tail_cost : 1.0; };
      double total_cost = 0.0;
      for (int64_t t = 0; t < n_tiles; ++t) total_cost += tile_cost(t);
      int64_t cur_group = 0;
      double cost_before = 0.0;
      for (int32_t r = 0; r < n_rel; ++r) {
        const int64_t first = rel_first[(size_t)r], end = rel_first[(size_t)r + 1];
        bool open = false;      // a span of this relation in the current group is being extended
        int64_t t = rel_tile_ptr[(size_t)r];
        for (int64_t t0 = first; t0 < end; t0 += 32, ++t) {
          const int64_t n = std::min<int64_t>(32, end - t0);
          const double cost = tile_cost(t);
          const int64_t grp = std::min<int64_t>(n_groups - 1, (int64_t)((cost_before + 0.5 * cost) * (double)n_groups /
                                                                        std::max(total_cost, 1.0)));
          cost_before += cost;
          if (grp > cur_group) open = false;
          while (cur_group < grp) { span_group_ptr.push_back((int32_t)span_rel.size()); ++cur_group; }
          if (open) {
            span_count.back() += (int32_t)n;
          } else {
            span_rel.push_back(r);
            span_start.push_back((int32_t)t0);
            span_count.push_back((int32_t)n);
            open = true;
          }
        }
      }
      while ((int64_t)span_group_ptr.size() < n_groups + 1) span_group_ptr.push_back((int32_t)span_rel.size());
      size_t sp = 0;
      for (int32_t r = 0; r < n_rel; ++r) {
        while (sp < span_rel.size() && span_rel[sp] < r) ++sp;
        rel_span_ptr[(size_t)r] = (int32_t)sp;
      }
      rel_span_ptr[(size_t)n_rel] = (int32_t)span_rel.size();
      return S;
    };
    const Spans SA = cut_spans(kOneTailTileCost), SE = cut_spans(kOneTailTileCostCode);
    g->n_span_groups = (int32_t)SA.group_ptr.size() - 1;
    g->n_spans = (int32_t)SA.rel.size();
    g->n_espans = (int32_t)SE.rel.size();
    TINYKG_TRY(upload(chunk_rel, &g->chunk_rel));
    TINYKG_TRY(upload(chunk_start, &g->chunk_start));
    TINYKG_TRY(upload(chunk_count, &g->chunk_count));
    TINYKG_TRY(upload(rel_chunk_ptr, &g->rel_chunk_ptr));
    TINYKG_TRY(upload(SA.group_ptr, &g->span_group_ptr));
    TINYKG_TRY(upload(SA.rel, &g->span_rel));
    TINYKG_TRY(upload(SA.start, &g->span_start));
    TINYKG_TRY(upload(SA.count, &g->span_count));
    TINYKG_TRY(upload(SA.rel_ptr, &g->rel_span_ptr));
    TINYKG_TRY(upload(SE.group_ptr, &g->espan_group_ptr));
    TINYKG_TRY(upload(SE.rel, &g->espan_rel));
    TINYKG_TRY(upload(SE.start, &g->espan_start));
    TINYKG_TRY(upload(SE.count, &g->espan_count));
    TINYKG_TRY(upload(SE.rel_ptr, &g->rel_espan_ptr));
  } else {
    const std::vector<int32_t> none, rel_ptr((size_t)n_rel + 1, 0), group_ptr(2, 0);
    g->chunk_edges = 64;
    g->n_span_groups = 1;
    TINYKG_TRY(upload(none, &g->chunk_rel));
    TINYKG_TRY(upload(none, &g->chunk_start));
    TINYKG_TRY(upload(none, &g->chunk_count));
    TINYKG_TRY(upload(rel_ptr, &g->rel_chunk_ptr));
    TINYKG_TRY(upload(group_ptr, &g->span_group_ptr));
    TINYKG_TRY(upload(none, &g->span_rel));
    TINYKG_TRY(upload(none, &g->span_start));
    TINYKG_TRY(upload(none, &g->span_count));
    TINYKG_TRY(upload(rel_ptr, &g->rel_span_ptr));
    TINYKG_TRY(upload(group_ptr, &g->espan_group_ptr));
    TINYKG_TRY(upload(none, &g->espan_rel));
    TINYKG_TRY(upload(none, &g->espan_start));
    TINYKG_TRY(upload(none, &g->espan_count));
    TINYKG_TRY(upload(rel_ptr, &g->rel_espan_ptr));
  }
  if (hipStreamSynchronize(st) != hipSuccess || hipGetLastError() != hipSuccess) return TINYKG_ERR_DEVICE;
#undef TINYKG_TRY
  *out = g;
  guard.g = nullptr;
  return TINYKG_OK;
}

void tinykg_graph_destroy(tinykg_graph* g) { tinykg::release(g); }
int64_t tinykg_graph_num_nodes(const tinykg_graph* g) { return g ? g->n_nodes : 0; }
int64_t tinykg_graph_num_edges(const tinykg_graph* g) { return g ? g->n_edges : 0; }

}  // extern "C"
