// tinykg_graph: the immutable sparse structure shared by every layer and step
// (Sec. 3.2, "Memory Analysis": the adjacency is kept once for all layers).
//
// Built on the host, off the hot path, from device COO triplets:
//   * head order  -- triplets sorted by (head, relation, tail): CSR row pointers
//     and the tail of every edge.  The softmax / gather kernels walk it.
//   * relation order -- the same edges sorted by (relation, tail, head), cut into
//     chunks that never straddle a relation.  The projection kernels (dense
//     contractions with one W_r) walk it; sorting by tail inside a relation puts
//     the edges of a hot tail next to each other, so their gradient rows are
//     summed before they leave the workgroup.
#include "tinykg_graph.h"

#include <algorithm>
#include <numeric>
#include <vector>

namespace tinykg {

namespace {

// Time of a one-tail tile of the edge-level backward kernel (d <= 64) relative to an ordinary one.
constexpr double kOneTailTileCost = 0.7;

template <typename T>
tinykg_status upload(const std::vector<T>& v, T** out) {
  *out = nullptr;
  const size_t bytes = std::max<size_t>(v.size(), 1) * sizeof(T);
  TINYKG_HIP_TRY(hipMalloc(reinterpret_cast<void**>(out), bytes));
  if (!v.empty()) TINYKG_HIP_TRY(hipMemcpy(*out, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice));
  return TINYKG_OK;
}

// One stable counting-sort pass: reorders `ord` by key[ord[i]] (keys in [0, n_keys)).
void counting_pass(std::vector<int32_t>& ord, const std::vector<int32_t>& key, size_t n_keys) {
  std::vector<int64_t> cnt(n_keys + 1, 0);
  for (int32_t e : ord) cnt[(size_t)key[(size_t)e] + 1]++;
  for (size_t k = 0; k < n_keys; ++k) cnt[k + 1] += cnt[k];
  std::vector<int32_t> out(ord.size());
  for (int32_t e : ord) out[(size_t)cnt[(size_t)key[(size_t)e]]++] = e;
  ord.swap(out);
}

void release(tinykg_graph* g) {
  if (!g) return;
  void* ptrs[] = {g->rowptr, g->h_tail, g->r_head, g->r_tail, g->r_eid, g->chunk_rel,
                  g->chunk_start, g->chunk_count, g->rel_chunk_ptr, g->heavy_head, g->heavy_seg_ptr,
                  g->hseg_q, g->hseg_e0, g->hseg_cnt, g->r_hperm32, g->acc_slot, g->acc_node,
                  g->span_group_ptr, g->span_rel, g->span_start, g->span_count, g->rel_span_ptr};
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

  const size_t T = (size_t)n_edges;
  std::vector<int32_t> hh(T), hr(T), ht(T);
  if (T) {
    hipStream_t st = (hipStream_t)stream;
    TINYKG_HIP_TRY(hipMemcpyAsync(hh.data(), head, T * 4, hipMemcpyDeviceToHost, st));
    TINYKG_HIP_TRY(hipMemcpyAsync(hr.data(), rel, T * 4, hipMemcpyDeviceToHost, st));
    TINYKG_HIP_TRY(hipMemcpyAsync(ht.data(), tail, T * 4, hipMemcpyDeviceToHost, st));
    TINYKG_HIP_TRY(hipStreamSynchronize(st));
  }
  for (size_t e = 0; e < T; ++e) {
    if (hh[e] < 0 || hh[e] >= n_nodes || ht[e] < 0 || ht[e] >= n_nodes) return TINYKG_ERR_INVALID_ARG;
    if (hr[e] < 0 || hr[e] >= n_rel) return TINYKG_ERR_INVALID_ARG;
  }

  // head order: (head, relation, tail, input position) -- three stable counting passes
  std::vector<int32_t> ord(T);
  std::iota(ord.begin(), ord.end(), 0);
  counting_pass(ord, ht, (size_t)n_nodes);
  counting_pass(ord, hr, (size_t)n_rel);
  counting_pass(ord, hh, (size_t)n_nodes);
  std::vector<int32_t> rowptr((size_t)n_nodes + 1, 0), h_tail(T), h_head(T), h_rel(T);
  for (size_t i = 0; i < T; ++i) {
    const int32_t e = ord[i];
    h_head[i] = hh[e]; h_rel[i] = hr[e]; h_tail[i] = ht[e];
    rowptr[(size_t)hh[e] + 1]++;
  }
  for (int64_t i = 0; i < n_nodes; ++i) rowptr[(size_t)i + 1] += rowptr[(size_t)i];

  // relation order over head-order edge ids: (relation, tail, head) -- two stable passes
  // over a sequence that already ascends in head
  std::vector<int32_t> rord(T);
  std::iota(rord.begin(), rord.end(), 0);
  counting_pass(rord, h_tail, (size_t)n_nodes);
  counting_pass(rord, h_rel, (size_t)n_rel);
  std::vector<int32_t> r_head(T), r_tail(T), r_eid(T);
  std::vector<int64_t> rel_count((size_t)n_rel, 0);
  for (size_t i = 0; i < T; ++i) {
    const int32_t e = rord[i];
    r_head[i] = h_head[e]; r_tail[i] = h_tail[e]; r_eid[i] = e;
    rel_count[(size_t)h_rel[e]]++;
  }

  // chunks: runs of at most chunk_edges consecutive relation-order edges of one
  // relation; about 2048 of them: few enough that the per-chunk partial gradients stay
  // small and a workgroup amortises staging W_r, enough to fill 256 compute units.
  int64_t chunk_edges = ((n_edges / 2048 + 63) / 64) * 64;
  if (chunk_edges < 64) chunk_edges = 64;
  std::vector<int32_t> chunk_rel, chunk_start, chunk_count, rel_chunk_ptr((size_t)n_rel + 1, 0);
  int64_t pos = 0;
  for (int32_t r = 0; r < n_rel; ++r) {
    rel_chunk_ptr[(size_t)r] = (int32_t)chunk_rel.size();
    int64_t left = rel_count[(size_t)r];
    while (left > 0) {
      const int64_t c = std::min(left, chunk_edges);
      chunk_rel.push_back(r);
      chunk_start.push_back((int32_t)pos);
      chunk_count.push_back((int32_t)c);
      pos += c; left -= c;
    }
  }
  rel_chunk_ptr[(size_t)n_rel] = (int32_t)chunk_rel.size();

  // spans of the persistent edge-level kernel (one group per compute unit): runs of whole
  // 32-edge tiles of one relation (tiles are counted from the relation's first edge).  The
  // groups get equal shares of the kernel's WORK, not of the edges: a tile whose edges share
  // one tail (popular tails own long runs of the relation order) takes the kernel's run form,
  // which skips a third of the matrix products.
  std::vector<int32_t> span_group_ptr(1, 0), span_rel, span_start, span_count, rel_span_ptr((size_t)n_rel + 1, 0);
  {
    const int64_t n_groups = std::max<int64_t>(1, std::min<int64_t>(num_cus(), (int64_t)chunk_rel.size()));
    auto tile_cost = [&](int64_t first, int64_t n) {
      for (int64_t k = 1; k < n; ++k)
        if (r_tail[(size_t)(first + k)] != r_tail[(size_t)first]) return 1.0;
      return kOneTailTileCost;
    };
    double total_cost = 0.0;
    int64_t first = 0;
    for (int32_t r = 0; r < n_rel; ++r) {
      const int64_t end = first + rel_count[(size_t)r];
      for (int64_t t0 = first; t0 < end; t0 += 32) total_cost += tile_cost(t0, std::min<int64_t>(32, end - t0));
      first = end;
    }
    int64_t cur_group = 0;
    double cost_before = 0.0;
    first = 0;
    for (int32_t r = 0; r < n_rel; ++r) {
      const int64_t end = first + rel_count[(size_t)r];
      bool open = false;      // a span of this relation in the current group is being extended
      for (int64_t t0 = first; t0 < end; t0 += 32) {
        const int64_t n = std::min<int64_t>(32, end - t0);
        const double cost = tile_cost(t0, n);
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
      first = end;
    }
    while ((int64_t)span_group_ptr.size() < n_groups + 1) span_group_ptr.push_back((int32_t)span_rel.size());
    size_t sp = 0;
    for (int32_t r = 0; r < n_rel; ++r) {
      while (sp < span_rel.size() && span_rel[sp] < r) ++sp;
      rel_span_ptr[(size_t)r] = (int32_t)sp;
    }
    rel_span_ptr[(size_t)n_rel] = (int32_t)span_rel.size();
  }

  // heavy heads and their segments
  std::vector<int32_t> heavy_head, heavy_seg_ptr(1, 0), hseg_q, hseg_e0, hseg_cnt;
  for (int64_t h = 0; h < n_nodes; ++h) {
    const int32_t e0 = rowptr[(size_t)h], deg = rowptr[(size_t)h + 1] - e0;
    if (deg <= kHeavyDegree) continue;
    const int32_t q = (int32_t)heavy_head.size();
    heavy_head.push_back((int32_t)h);
    for (int32_t o = 0; o < deg; o += kHeavyDegree) {
      hseg_q.push_back(q);
      hseg_e0.push_back(e0 + o);
      hseg_cnt.push_back(std::min<int32_t>(kHeavyDegree, deg - o));
    }
    heavy_seg_ptr.push_back((int32_t)hseg_q.size());
  }
  // nodes whose gradient rows are accumulated in double
  std::vector<int32_t> acc_slot((size_t)n_nodes, -1), acc_node;
  {
    std::vector<int32_t> rows((size_t)n_nodes, 0);
    for (size_t e = 0; e < T; ++e) { rows[(size_t)hh[e]]++; rows[(size_t)ht[e]]++; }
    for (int64_t v = 0; v < n_nodes; ++v)
      if (rows[(size_t)v] > kAccHeavyDegree) {
        acc_slot[(size_t)v] = (int32_t)acc_node.size();
        acc_node.push_back((int32_t)v);
      }
  }
  // tile-local head-sorted row orders (tiles are counted from each chunk's start) and the
  // two accumulation flags of every row
  std::vector<uint8_t> hperm32(T);
  for (size_t c = 0; c < chunk_rel.size(); ++c) {
    for (int32_t t0 = 0; t0 < chunk_count[c]; t0 += 32) {
      const int32_t base = chunk_start[c] + t0, nrow = std::min<int32_t>(32, chunk_count[c] - t0);
      uint8_t idx[32];
      for (int i = 0; i < nrow; ++i) idx[i] = (uint8_t)i;
      std::stable_sort(idx, idx + nrow, [&](uint8_t a, uint8_t b) { return r_head[(size_t)base + a] < r_head[(size_t)base + b]; });
      for (int i = 0; i < nrow; ++i) {
        const size_t pos = (size_t)base + i;
        hperm32[pos] = (uint8_t)(idx[i] | (acc_slot[(size_t)r_tail[pos]] >= 0 ? 0x40 : 0) |
                                 (acc_slot[(size_t)r_head[pos]] >= 0 ? 0x80 : 0));
      }
    }
  }

  tinykg_graph* g = new tinykg_graph();
  g->n_nodes = n_nodes; g->n_edges = n_edges; g->n_rel = n_rel;
  g->n_chunks = (int32_t)chunk_rel.size();
  g->chunk_edges = (int32_t)chunk_edges;
  tinykg_status st = upload(rowptr, &g->rowptr);
  if (st == TINYKG_OK) st = upload(h_tail, &g->h_tail);
  if (st == TINYKG_OK) st = upload(r_head, &g->r_head);
  if (st == TINYKG_OK) st = upload(r_tail, &g->r_tail);
  if (st == TINYKG_OK) st = upload(r_eid, &g->r_eid);
  if (st == TINYKG_OK) st = upload(chunk_rel, &g->chunk_rel);
  if (st == TINYKG_OK) st = upload(chunk_start, &g->chunk_start);
  if (st == TINYKG_OK) st = upload(chunk_count, &g->chunk_count);
  if (st == TINYKG_OK) st = upload(rel_chunk_ptr, &g->rel_chunk_ptr);
  g->n_span_groups = (int32_t)span_group_ptr.size() - 1;
  g->n_spans = (int32_t)span_rel.size();
  if (st == TINYKG_OK) st = upload(span_group_ptr, &g->span_group_ptr);
  if (st == TINYKG_OK) st = upload(span_rel, &g->span_rel);
  if (st == TINYKG_OK) st = upload(span_start, &g->span_start);
  if (st == TINYKG_OK) st = upload(span_count, &g->span_count);
  if (st == TINYKG_OK) st = upload(rel_span_ptr, &g->rel_span_ptr);
  g->n_heavy = (int32_t)heavy_head.size();
  for (int64_t i = 0; i < n_nodes; ++i)
    g->max_out_degree = std::max(g->max_out_degree, rowptr[(size_t)i + 1] - rowptr[(size_t)i]);
  g->n_hseg = (int32_t)hseg_q.size();
  if (st == TINYKG_OK) st = upload(heavy_head, &g->heavy_head);
  if (st == TINYKG_OK) st = upload(heavy_seg_ptr, &g->heavy_seg_ptr);
  if (st == TINYKG_OK) st = upload(hseg_q, &g->hseg_q);
  if (st == TINYKG_OK) st = upload(hseg_e0, &g->hseg_e0);
  if (st == TINYKG_OK) st = upload(hseg_cnt, &g->hseg_cnt);
  if (st == TINYKG_OK) st = upload(hperm32, &g->r_hperm32);
  g->n_acc_heavy = (int32_t)acc_node.size();
  if (st == TINYKG_OK) st = upload(acc_slot, &g->acc_slot);
  if (st == TINYKG_OK) st = upload(acc_node, &g->acc_node);
  if (st != TINYKG_OK) { release(g); return st; }
  *out = g;
  return TINYKG_OK;
}

void tinykg_graph_destroy(tinykg_graph* g) { tinykg::release(g); }
int64_t tinykg_graph_num_nodes(const tinykg_graph* g) { return g ? g->n_nodes : 0; }
int64_t tinykg_graph_num_edges(const tinykg_graph* g) { return g ? g->n_edges : 0; }

}  // extern "C"
