// Internal helpers shared by the GPU library's translation units (not installed).
#ifndef TINYKG_COMMON_H
#define TINYKG_COMMON_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tinykg.h"

#define TINYKG_HIP_TRY(expr)                         \
  do {                                               \
    if ((expr) != hipSuccess) {                      \
      (void)hipGetLastError();                       \
      return TINYKG_ERR_DEVICE;                      \
    }                                                \
  } while (0)

namespace tinykg {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool bits_ok(int b) { return b == 1 || b == 2 || b == 4 || b == 8; }
inline bool group_ok(int g) { return g == 32 || g == 64 || g == 128 || g == 256; }

// Number of compute units of the current device (cached per process).
int num_cus();

// Launch-status check after a kernel launch.
inline tinykg_status launch_status() {
  return hipGetLastError() == hipSuccess ? TINYKG_OK : TINYKG_ERR_DEVICE;
}

// Argument checks shared by tinykg_quantize_ex and the aggregation's saves.
tinykg_status launch_quantize(const float* act, int64_t n, int bits, int group, uint64_t seed,
                              uint64_t first_index, int rounding, uint8_t* packed, float* gmin,
                              float* gscale, hipStream_t stream);
// The quantizer with y = (x - mu_c) a_c + beta_c (column c of a [*, dim] tensor) written
// in the same pass over x; n / 4 must stay below 2^32.
tinykg_status launch_quantize_affine(const float* act, int64_t n, int bits, int group, uint64_t seed,
                                     uint8_t* packed, float* gmin, float* gscale, int dim,
                                     const float* mu, const float* a, const float* beta, float* y,
                                     hipStream_t stream);
tinykg_status launch_dequantize(const uint8_t* packed, const float* gmin, const float* gscale,
                                int64_t n, int bits, int group, float* out, hipStream_t stream);

// Brackets the kernel launches made while it is alive with two events on `st`
// (only while tinykg_profile_enable(1) is in effect).
class ProfileScope {
 public:
  ProfileScope(const char* name, hipStream_t st);
  ~ProfileScope();
  ProfileScope(const ProfileScope&) = delete;
  ProfileScope& operator=(const ProfileScope&) = delete;

 private:
  int slot_;
  hipStream_t st_;
};

// While one is alive (on this thread's call path: the recorder is not thread-safe) no
// ProfileScope records anything, so the entry points that must not allocate never create an
// event even with tinykg_profile_enable(1) in effect.
class ProfileMute {
 public:
  ProfileMute();
  ~ProfileMute();
  ProfileMute(const ProfileMute&) = delete;
  ProfileMute& operator=(const ProfileMute&) = delete;
};

}  // namespace tinykg
#endif
