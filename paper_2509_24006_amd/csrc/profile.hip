// Optional per-kernel timing: when switched on, every launcher brackets its kernel with a
// pair of HIP events on the caller's stream; sla_profile_read waits for them and reports
// count and total milliseconds per kernel name.  Off by default (no events, no cost).
#include <stdio.h>
#include <string.h>

#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/sla.h"
#include "sla_internal.h"

namespace sla {
namespace {
struct Rec {
  const char* name;
  hipEvent_t a, b;
};
std::mutex g_mu;
bool g_on = false;
std::vector<Rec> g_recs;
}  // namespace

hipError_t ensure_dyn_lds(const void* kernel, int bytes) {
  static std::mutex mu;
  static std::map<std::pair<const void*, int>, int> done;   // (kernel, device) -> bytes granted
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lk(mu);
  auto it = done.find({kernel, dev});
  if (it != done.end() && it->second >= bytes) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done[{kernel, dev}] = bytes;
  return e;
}

KernelTimer::KernelTimer(const char* name, hipStream_t st) : st_(st), idx_(-1) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_on) return;
  Rec r{name, nullptr, nullptr};
  if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
  (void)hipEventRecord(r.a, st);
  idx_ = (long)g_recs.size();
  g_recs.push_back(r);
}

KernelTimer::~KernelTimer() {
  if (idx_ < 0) return;
  std::lock_guard<std::mutex> lk(g_mu);
  if ((size_t)idx_ < g_recs.size()) (void)hipEventRecord(g_recs[idx_].b, st_);
}
}  // namespace sla

extern "C" {

int sla_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(sla::g_mu);
  sla::g_on = on != 0;
  return SLA_OK;
}

int sla_profile_read(char* buf, size_t buf_bytes) {
  if (!buf || buf_bytes == 0) return SLA_EINVAL;
  std::lock_guard<std::mutex> lk(sla::g_mu);
  std::map<std::string, std::pair<long, double>> agg;
  std::vector<std::string> order;
  int rc = SLA_OK;
  for (auto& r : sla::g_recs) {
    float ms = 0.0f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess)
      rc = SLA_EHIP;
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
    if (!agg.count(r.name)) order.push_back(r.name);
    auto& e = agg[r.name];
    e.first += 1;
    e.second += ms;
  }
  sla::g_recs.clear();
  size_t off = 0;
  buf[0] = 0;
  for (auto& n : order) {
    char line[256];
    const int len = snprintf(line, sizeof line, "%s %ld %.6f\n", n.c_str(), agg[n].first, agg[n].second);
    if (off + (size_t)len + 1 > buf_bytes) return SLA_ENOSPACE;
    memcpy(buf + off, line, (size_t)len + 1);
    off += (size_t)len;
  }
  return rc;
}
}
