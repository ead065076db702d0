// Optional per-kernel timing with HIP events recorded on the launch stream (off by default).
#include <hip/hip_runtime.h>
#include <mutex>
#include <vector>
#include "tt_internal.h"
#include "tt_kernels.h"

namespace tt {
namespace {
struct Pending { int id; hipEvent_t start, stop; };
std::mutex g_mu;
bool g_on = false;
std::vector<Pending> g_pending;
double g_ms[TT_N_KERNELS];
int64_t g_launches[TT_N_KERNELS];
}  // namespace

KernelTimer::KernelTimer(int id, hipStream_t st) : id_(id), st_(st), active_(false) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_on) return;
  if (hipEventCreate(&start_) != hipSuccess) return;
  if (hipEventCreate(&stop_) != hipSuccess) { (void)hipEventDestroy(start_); return; }
  active_ = hipEventRecord(start_, st_) == hipSuccess;
  if (!active_) { (void)hipEventDestroy(start_); (void)hipEventDestroy(stop_); }
}

KernelTimer::~KernelTimer() {
  if (!active_) return;
  (void)hipEventRecord(stop_, st_);
  std::lock_guard<std::mutex> lk(g_mu);
  g_pending.push_back({id_, start_, stop_});
}
}  // namespace tt

extern "C" tt_status tt_kernel_timing_enable(int32_t on) {
  tt::clear_error();
  std::lock_guard<std::mutex> lk(tt::g_mu);
  for (auto& p : tt::g_pending) { (void)hipEventSynchronize(p.stop); (void)hipEventDestroy(p.start); (void)hipEventDestroy(p.stop); }
  tt::g_pending.clear();
  for (int i = 0; i < TT_N_KERNELS; i++) { tt::g_ms[i] = 0.0; tt::g_launches[i] = 0; }
  tt::g_on = on != 0;
  return TT_OK;
}

extern "C" tt_status tt_kernel_timing_read(tt_kernel_times* out) {
  tt::clear_error();
  if (!out) return tt::fail(TT_ERR_NULL, "out is NULL");
  std::lock_guard<std::mutex> lk(tt::g_mu);
  for (auto& p : tt::g_pending) {
    float ms = 0.f;
    if (hipEventSynchronize(p.stop) != hipSuccess || hipEventElapsedTime(&ms, p.start, p.stop) != hipSuccess)
      return tt::fail(TT_ERR_HIP, "could not read a timing event");
    tt::g_ms[p.id] += ms;
    tt::g_launches[p.id] += 1;
    (void)hipEventDestroy(p.start);
    (void)hipEventDestroy(p.stop);
  }
  tt::g_pending.clear();
  for (int i = 0; i < TT_N_KERNELS; i++) { out->ms[i] = tt::g_ms[i]; out->launches[i] = tt::g_launches[i]; }
  return TT_OK;
}
