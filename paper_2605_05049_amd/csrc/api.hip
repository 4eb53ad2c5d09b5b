// Host-only entry points of the C ABI: status strings, workspace size, version.
#include "common.h"

#include <mutex>
#include <vector>

namespace moe {
namespace {
struct ProfRecord { const char* name; hipEvent_t start, stop; };
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<ProfRecord> g_prof;
bool g_prof_open = false;
}  // namespace

void prof_begin(const char* name, hipStream_t st) {
  if (!g_prof_on) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  ProfRecord r{name, nullptr, nullptr};
  if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) return;
  (void)hipEventRecord(r.start, st);
  g_prof.push_back(r);
  g_prof_open = true;
}

void prof_end(hipStream_t st) {
  if (!g_prof_on) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (!g_prof_open || g_prof.empty()) return;
  (void)hipEventRecord(g_prof.back().stop, st);
  g_prof_open = false;
}
}  // namespace moe

extern "C" int moe_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(moe::g_prof_mu);
  moe::g_prof_on = on != 0;
  return MOE_OK;
}

extern "C" int moe_profile_count(void) {
  std::lock_guard<std::mutex> lk(moe::g_prof_mu);
  return (int)moe::g_prof.size();
}

extern "C" int moe_profile_get(int i, const char** name, float* ms) {
  std::lock_guard<std::mutex> lk(moe::g_prof_mu);
  if (i < 0 || i >= (int)moe::g_prof.size() || !name || !ms) return MOE_ERR_SHAPE;
  const moe::ProfRecord& r = moe::g_prof[i];
  if (hipEventSynchronize(r.stop) != hipSuccess) return MOE_ERR_RUNTIME;
  if (hipEventElapsedTime(ms, r.start, r.stop) != hipSuccess) return MOE_ERR_RUNTIME;
  *name = r.name;
  return MOE_OK;
}

extern "C" int moe_profile_reset(void) {
  std::lock_guard<std::mutex> lk(moe::g_prof_mu);
  for (auto& r : moe::g_prof) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  moe::g_prof.clear();
  moe::g_prof_open = false;
  return MOE_OK;
}

extern "C" const char* moe_status_str(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_NULL: return "a required pointer is NULL";
    case MOE_ERR_SHAPE: return "shape outside the supported limits";
    case MOE_ERR_ALIGN: return "pointer not sufficiently aligned";
    case MOE_ERR_WORKSPACE: return "workspace too small";
    case MOE_ERR_RUNTIME: return "HIP launch failed";
    default: return "unknown status";
  }
}

extern "C" size_t moe_workspace_bytes(const moe_shape* shape) {
  moe::Dims D;
  if (moe::check_shape(shape, &D) != MOE_OK) return 0;
  return moe::ws_layout(D).total;
}

extern "C" int moe_abi_version(void) { return 1; }
