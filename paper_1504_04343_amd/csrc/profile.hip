// Optional per-kernel timing with HIP events on the launching stream (measurement aid for
// bench.py; off by default, nothing is recorded and no event is created when off).
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "cct_internal.h"

namespace cct {
namespace {

struct Record {
  std::string name;
  double flops, bytes;
  hipEvent_t start, stop;
};

std::mutex g_mu;
bool g_on = false;
std::vector<Record> g_records;
constexpr size_t kMaxRecords = 1 << 16;

void clear_records() {
  for (auto& r : g_records) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  g_records.clear();
}

}  // namespace

ProfScope::ProfScope(const char* name, double flops, double bytes, hipStream_t st)
    : st_(st), idx_(-1) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_on || g_records.size() >= kMaxRecords) return;
  Record r;
  r.name = name;
  r.flops = flops;
  r.bytes = bytes;
  if (hipEventCreate(&r.start) != hipSuccess) return;
  if (hipEventCreate(&r.stop) != hipSuccess) {
    (void)hipEventDestroy(r.start);
    return;
  }
  (void)hipEventRecord(r.start, st);
  g_records.push_back(r);
  idx_ = (long long)g_records.size() - 1;
}

ProfScope::~ProfScope() {
  if (idx_ < 0) return;
  std::lock_guard<std::mutex> lk(g_mu);
  if ((size_t)idx_ < g_records.size()) (void)hipEventRecord(g_records[idx_].stop, st_);
}

}  // namespace cct

using namespace cct;

namespace {
// One 16-byte load and one 16-byte store per thread: the reference "plain copy of known size"
// against which hardware-counter readings (FETCH_SIZE / WRITE_SIZE) are scaled.
__global__ __launch_bounds__(256) void calibration_copy_kernel(const uint4* __restrict__ src,
                                                               uint4* __restrict__ dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = src[i];
}
}  // namespace

extern "C" {

int cct_calibration_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
  if (!src || !dst || bytes == 0 || bytes % 16) return CCT_EINVAL;
  if (reinterpret_cast<uintptr_t>(src) % 16 || reinterpret_cast<uintptr_t>(dst) % 16)
    return CCT_EINVAL;
  const size_t n = bytes / 16;
  const size_t blocks = (n + 255) / 256;
  if (blocks >= 2147483647ULL) return CCT_EUNSUPPORTED;
  hipLaunchKernelGGL(calibration_copy_kernel, dim3((unsigned)blocks), dim3(256), 0,
                     (hipStream_t)hip_stream, static_cast<const uint4*>(src),
                     static_cast<uint4*>(dst), n);
  CCT_CHECK_LAUNCH();
  return CCT_OK;
}

int cct_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (on) clear_records();
  g_on = on != 0;
  return CCT_OK;
}

int cct_profile_read(cct_profile_entry_t* entries, int32_t max_entries, int32_t* n) {
  if (!entries || !n || max_entries < 1) return CCT_EINVAL;
  std::lock_guard<std::mutex> lk(g_mu);
  std::map<std::string, cct_profile_entry_t> agg;
  std::vector<std::string> order;
  for (auto& r : g_records) {
    if (hipEventSynchronize(r.stop) != hipSuccess) return CCT_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) return CCT_EHIP;
    auto it = agg.find(r.name);
    if (it == agg.end()) {
      cct_profile_entry_t e;
      memset(&e, 0, sizeof(e));
      strncpy(e.name, r.name.c_str(), sizeof(e.name) - 1);
      it = agg.emplace(r.name, e).first;
      order.push_back(r.name);
    }
    it->second.launches += 1;
    it->second.total_ms += ms;
    it->second.flops += r.flops;
    it->second.bytes += r.bytes;
  }
  int32_t k = 0;
  for (auto& nm : order) {
    if (k >= max_entries) break;
    entries[k++] = agg[nm];
  }
  *n = k;
  return CCT_OK;
}

}  // extern "C"
