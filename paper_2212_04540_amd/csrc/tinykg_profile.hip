// Per-kernel device-time recorder behind tinykg_profile_enable / _report.
#include "tinykg_common.h"

#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <vector>

namespace tinykg {

namespace {
struct Record { const char* name; hipEvent_t start, stop; bool closed; };
bool g_on = false;
int g_mute = 0;                     // > 0: a ProfileMute is alive
std::string g_only;                 // empty: every scope; else only the scopes of this name
std::vector<Record> g_records;
std::vector<hipEvent_t> g_spare;    // events of dropped records, reused (creating one costs microseconds)
constexpr size_t kMaxRecords = 8192;

void drop_records() {
  for (Record& r : g_records) { g_spare.push_back(r.start); g_spare.push_back(r.stop); }
  g_records.clear();
}

bool take_event(hipEvent_t* e) {
  if (!g_spare.empty()) { *e = g_spare.back(); g_spare.pop_back(); return true; }
  return hipEventCreate(e) == hipSuccess;
}
}  // namespace

ProfileScope::ProfileScope(const char* name, hipStream_t st) : slot_(-1), st_(st) {
  if (!g_on || g_mute > 0 || g_records.size() >= kMaxRecords) return;
  if (!g_only.empty() && g_only != name) return;
  Record r{name, nullptr, nullptr, false};
  if (!take_event(&r.start)) return;
  if (!take_event(&r.stop)) { g_spare.push_back(r.start); return; }
  (void)hipEventRecord(r.start, st);
  g_records.push_back(r);
  slot_ = (int)g_records.size() - 1;
}

ProfileScope::~ProfileScope() {
  if (slot_ < 0 || (size_t)slot_ >= g_records.size()) return;
  (void)hipEventRecord(g_records[(size_t)slot_].stop, st_);
  g_records[(size_t)slot_].closed = true;
}

ProfileMute::ProfileMute() { ++g_mute; }
ProfileMute::~ProfileMute() { --g_mute; }

__global__ void calibration_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                        size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace tinykg

extern "C" {

tinykg_status tinykg_profile_copy(void* dst, const void* src, size_t bytes, void* stream) {
  using namespace tinykg;
  if (bytes == 0) return TINYKG_OK;
  if (!dst || !src || !aligned16(dst) || !aligned16(src) || bytes % 16 != 0) return TINYKG_ERR_INVALID_ARG;
  const size_t n16 = bytes / 16;
  const size_t want = (n16 + 255) / 256, cap = (size_t)num_cus() * 32;
  ProfileScope prof("calibration_copy_kernel", (hipStream_t)stream);
  hipLaunchKernelGGL(calibration_copy_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0,
                     (hipStream_t)stream, static_cast<const float4*>(src), static_cast<float4*>(dst), n16);
  return launch_status();
}

void tinykg_profile_enable(int on) {
  using namespace tinykg;
  if (on) drop_records();
  g_on = on != 0;
}

void tinykg_profile_select(const char* name) {
  tinykg::g_only = name ? name : "";
}

size_t tinykg_profile_report(char* buf, size_t cap) {
  using namespace tinykg;
  std::map<std::string, std::pair<long, double>> agg;
  std::vector<std::string> order;
  for (Record& r : g_records) {
    if (!r.closed) continue;
    if (hipEventSynchronize(r.stop) != hipSuccess) continue;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) continue;
    auto it = agg.find(r.name);
    if (it == agg.end()) { order.push_back(r.name); it = agg.emplace(r.name, std::make_pair(0L, 0.0)).first; }
    it->second.first += 1;
    it->second.second += ms;
  }
  std::string text;
  char line[256];
  for (const std::string& n : order) {
    std::snprintf(line, sizeof line, "%s %ld %.6f\n", n.c_str(), agg[n].first, agg[n].second);
    text += line;
  }
  if (buf && cap > 0) {
    const size_t k = text.size() < cap - 1 ? text.size() : cap - 1;
    std::memcpy(buf, text.data(), k);
    buf[k] = '\0';
  }
  return text.size();
}

}  // extern "C"
