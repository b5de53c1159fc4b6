// Reading a saved activation matrix four elements at a time, dequantised on the fly
// (shared by the kernels whose backward pass gathers compressed rows).
#ifndef TINYKG_FETCH_H
#define TINYKG_FETCH_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tinykg {

// Where a saved (or exact) activation matrix lives.  bits == 32: plain fp32.
struct Source {
  const uint8_t* data;
  const float* gmin;
  const float* gscale;
  int group_chunks_log2;  // log2(group / 4)
};

// Four consecutive elements (chunk c of the flattened matrix), dequantised by
// Eq. (4): fma(code, scale, min).
template <int BITS>
__device__ __forceinline__ float4 fetch_chunk(const Source& src, int64_t c) {
  if (BITS == 32) return reinterpret_cast<const float4*>(src.data)[c];
  constexpr uint32_t B = (BITS == 32) ? 0u : ((1u << (BITS & 31)) - 1u);
  uint32_t w;
  if (BITS == 8) w = reinterpret_cast<const uint32_t*>(src.data)[c];
  else if (BITS == 4) w = reinterpret_cast<const uint16_t*>(src.data)[c];
  else if (BITS == 2) w = src.data[c];
  else w = (src.data[c >> 1] >> ((c & 1) * 4)) & 0xFu;
  const int64_t g = c >> src.group_chunks_log2;
  const float z = src.gmin[g], s = src.gscale[g];
  constexpr int SH = BITS & 31;
  float4 v;
  v.x = fmaf((float)(w & B), s, z);
  v.y = fmaf((float)((w >> SH) & B), s, z);
  v.z = fmaf((float)((w >> (2 * SH)) & B), s, z);
  v.w = fmaf((float)((w >> (3 * SH)) & B), s, z);
  return v;
}

}  // namespace tinykg
#endif
