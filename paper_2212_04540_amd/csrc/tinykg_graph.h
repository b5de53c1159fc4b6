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
};

#endif
