// Per-launch timing, aggregated per kernel family: each launch carries a start and a stop event bound to the kernel
// itself (hipExtLaunchKernel), whose difference is the kernel's execution time.  Off by default: the events cost a few
// microseconds per launch, so timed throughput runs keep it disabled.
#include <mutex>
#include <vector>
#include "kernels.h"

namespace sama {
namespace {
struct Rec { int family; double units; hipEvent_t start, stop; };
std::mutex g_mu;
bool g_on = false;
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;
const char* kNames[F_COUNT] = {"gemm_bf16_nt", "gemm_bf16_nn", "gemm_bf16_tn", "gemm_bf16_nt_hilo", "gemm_bf16_nn_hilo", "gemm_f32", "attention_fwd", "attention_bwd",
                               "layernorm_fwd", "layernorm_bwd", "adam", "adapt_norm", "perturb_lo", "residual_lo",
                               "nudge", "sample_stage", "mlm_softmax", "other"};
hipEvent_t take_event() {
  if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

ProfScope::ProfScope(hipStream_t st, int family, double units) : st_(st), family_(family), units_(units), on_(g_on) {}

void ProfScope::next_events(hipEvent_t* start, hipEvent_t* stop) {
  std::lock_guard<std::mutex> lk(g_mu);
  Rec r{family_, units_, take_event(), take_event()};
  units_ = 0.0;   // a scope's work is credited once
  *start = r.start; *stop = r.stop;
  if (r.start != nullptr && r.stop != nullptr) g_recs.push_back(r);
  else { *start = nullptr; *stop = nullptr; }
}

void prof_enable(bool on) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (on) {
    for (auto& r : g_recs) { g_pool.push_back(r.start); g_pool.push_back(r.stop); }
    g_recs.clear();
  }
  g_on = on;
}

bool prof_read(int family, const char** name, int64_t* launches, double* total_ms, double* units) {
  if (family < 0 || family >= F_COUNT) return false;
  std::lock_guard<std::mutex> lk(g_mu);
  int64_t n = 0; double ms = 0.0, u = 0.0;
  for (auto& r : g_recs) {
    if (r.family != family) continue;
    if (hipEventSynchronize(r.stop) != hipSuccess) continue;
    float t = 0.f;
    if (hipEventElapsedTime(&t, r.start, r.stop) != hipSuccess) continue;
    ms += t; u += r.units; ++n;
  }
  if (name) *name = kNames[family];
  if (launches) *launches = n;
  if (total_ms) *total_ms = ms;
  if (units) *units = u;
  return true;
}

}  // namespace sama
