// Definition of the opaque tinykg_graph (internal to the GPU library).
#ifndef TINYKG_GRAPH_H
#define TINYKG_GRAPH_H

#include "tinykg_common.h"

struct tinykg_graph {
  int64_t n_nodes = 0, n_edges = 0;
  int32_t n_rel = 0;
  // head order (edges sorted by head, relation, tail)
  int32_t* rowptr = nullptr;   // [n_nodes + 1]
  int32_t* h_tail = nullptr;   // [n_edges]
  int32_t max_out_degree = 0;
  // relation order (edges sorted by relation, tail, head)
  int32_t* r_head = nullptr;   // [n_edges]
  int32_t* r_tail = nullptr;   // [n_edges]
  int32_t* r_eid = nullptr;    // [n_edges] position of the edge in head order
  // chunks of the relation order: one relation each, at most chunk_edges edges
  int32_t n_chunks = 0, chunk_edges = 64;
  int32_t* chunk_rel = nullptr;      // [n_chunks]
  int32_t* chunk_start = nullptr;    // [n_chunks] first relation-order position
  int32_t* chunk_count = nullptr;    // [n_chunks]
  int32_t* rel_chunk_ptr = nullptr;  // [n_rel + 1] chunks of relation r: [ptr[r], ptr[r+1])
  // spans: the relation order cut at 32-edge tile boundaries (tiles counted from a relation's
  // first edge) into one piece of about equal WORK per compute unit -- a tile whose edges
  // share one tail is cheaper for the edge-level backward kernel -- each piece cut again
  // where the relation changes: what one persistent workgroup of that kernel walks
  int32_t n_span_groups = 0, n_spans = 0;
  int32_t* span_group_ptr = nullptr; // [n_span_groups + 1] spans of workgroup w: [ptr[w], ptr[w+1])
  int32_t* span_rel = nullptr;       // [n_spans]
  int32_t* span_start = nullptr;     // [n_spans] first relation-order position
  int32_t* span_count = nullptr;     // [n_spans]
  int32_t* rel_span_ptr = nullptr;   // [n_rel + 1] spans of relation r: [ptr[r], ptr[r+1])
  // the same cut with a one-tail tile counted almost like any other (for the code form of the
  // edge-level kernel, whose products all run on the bf16 matrix cores)
  int32_t n_espans = 0;
  int32_t* espan_group_ptr = nullptr;
  int32_t* espan_rel = nullptr;
  int32_t* espan_start = nullptr;
  int32_t* espan_count = nullptr;
  int32_t* rel_espan_ptr = nullptr;
  // heads with more than kHeavyDegree out-edges are cut into segments of that many
  // head-order edges, so that one wave never walks a 10^5-edge neighbourhood alone
  int32_t n_heavy = 0, n_hseg = 0;
  int32_t* heavy_head = nullptr;     // [n_heavy] node id
  int32_t* heavy_seg_ptr = nullptr;  // [n_heavy + 1] segments of heavy head q: [ptr[q], ptr[q+1])
  int32_t* hseg_q = nullptr;         // [n_hseg] index of the segment's head in heavy_head
  int32_t* hseg_e0 = nullptr;        // [n_hseg] first head-order edge
  int32_t* hseg_cnt = nullptr;       // [n_hseg] number of edges
  // for every tile of 32 consecutive relation-order edges of a chunk, one byte per edge:
  // bits 0-4 the tile-local row indices sorted by head (equal heads can then be summed
  // before they are scattered), bit 6 / bit 7: the tail / head of THIS row is a node that
  // accumulates its gradient in double
  uint8_t* r_hperm32 = nullptr;      // [n_edges]
  // tail order (edges sorted by tail, then head): what the transposed sparse product of the
  // uniform-attention layer walks -- all in-edges of a tail are adjacent, so their rows are
  // summed before they leave the wave and most tails are written by exactly one wave
  int32_t* c_head = nullptr;   // [n_edges]
  int32_t* c_tail = nullptr;   // [n_edges] bit 30: the tail accumulates its gradient in double
  // nodes that receive more than kAccHeavyDegree gradient rows (in-edges + out-edges)
  // accumulate them in double, in a compact buffer; all others in fp32
  int32_t n_acc_heavy = 0;
  int32_t* acc_slot = nullptr;       // [n_nodes] row of the compact buffer, or -1
  int32_t* acc_node = nullptr;       // [n_acc_heavy] node of each row
};

namespace tinykg {
constexpr int kHeavyDegree = 256;
constexpr int kAccHeavyDegree = 1024;
constexpr int kNodeIdMask = 0x3fffffff;   // bits 30, 31 of a staged node id carry flags
}

#endif
