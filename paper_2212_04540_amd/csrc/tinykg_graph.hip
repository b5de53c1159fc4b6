// placeholder entry points until the aggregation kernels land
#include "tinykg_common.h"
extern "C" {
tinykg_status tinykg_graph_create(int64_t, int32_t, int64_t, const int32_t*, const int32_t*,
                                  const int32_t*, void*, tinykg_graph**) { return TINYKG_ERR_UNSUPPORTED; }
void tinykg_graph_destroy(tinykg_graph*) {}
int64_t tinykg_graph_num_nodes(const tinykg_graph*) { return 0; }
int64_t tinykg_graph_num_edges(const tinykg_graph*) { return 0; }
size_t tinykg_kg_aggregate_workspace_bytes(const tinykg_graph*, int, int, int, int) { return 0; }
tinykg_status tinykg_kg_aggregate_fwd(const tinykg_graph*, const float*, const float*, const float*,
                                      const float*, int, int, int, float, int, int, uint64_t, float*,
                                      const tinykg_saved*, void*, size_t, void*) { return TINYKG_ERR_UNSUPPORTED; }
tinykg_status tinykg_kg_aggregate_bwd(const tinykg_graph*, const tinykg_saved*, const float*,
                                      const float*, const float*, int, int, int, float, int, int,
                                      const float*, float*, float*, float*, float*, void*, size_t,
                                      void*) { return TINYKG_ERR_UNSUPPORTED; }
}
