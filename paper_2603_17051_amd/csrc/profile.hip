// Optional per-kernel timing with HIP events recorded on the stream each kernel is
// launched on.  Off by default; when off a launch costs one predictable branch.
#include <hip/hip_runtime.h>

#include <cstring>
#include <string>
#include <vector>

#include "../../include/astro.h"
#include "kernels.hpp"

namespace astro {
namespace {
struct Record {
  const char* name;
  hipEvent_t start, stop;
};
bool g_on = false;
std::vector<Record> g_records;
constexpr size_t kMaxRecords = 1 << 16;
}  // namespace

ProfileScope::ProfileScope(const char* name, hipStream_t stream, bool enabled) : stream_(stream), index_(-1) {
  if (!enabled || !g_on || g_records.size() >= kMaxRecords) return;
  Record r{name, nullptr, nullptr};
  if (hipEventCreate(&r.start) != hipSuccess) return;
  if (hipEventCreate(&r.stop) != hipSuccess) {
    (void)hipEventDestroy(r.start);
    return;
  }
  (void)hipEventRecord(r.start, stream);
  index_ = (int)g_records.size();
  g_records.push_back(r);
}
ProfileScope::~ProfileScope() {
  if (index_ >= 0) (void)hipEventRecord(g_records[index_].stop, stream_);
}
}  // namespace astro

using namespace astro;

extern "C" {

int astro_profile_begin(void) {
  if (g_on) return ASTRO_ERR_BAD_STATE;
  g_records.clear();
  g_on = true;
  return ASTRO_OK;
}

int astro_profile_end(astro_kernel_time_t* out, int32_t max_entries, int32_t* n_entries) {
  if (!g_on) return ASTRO_ERR_BAD_STATE;
  if (!n_entries || max_entries < 0 || (max_entries > 0 && !out)) return ASTRO_ERR_INVALID_ARG;
  g_on = false;
  int rc = ASTRO_OK;
  int n = 0;
  for (Record& r : g_records) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) {
      rc = ASTRO_ERR_HIP;
      (void)hipGetLastError();
    } else {
      int i = 0;
      while (i < n && std::strcmp(out[i].name, r.name) != 0) ++i;
      if (i < max_entries) {
        if (i == n) {
          std::memset(&out[i], 0, sizeof(out[i]));
          std::strncpy(out[i].name, r.name, sizeof(out[i].name) - 1);
          ++n;
        }
        out[i].launches += 1;
        out[i].total_ms += ms;
      }
    }
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  g_records.clear();
  *n_entries = n;
  return rc;
}

}  // extern "C"
