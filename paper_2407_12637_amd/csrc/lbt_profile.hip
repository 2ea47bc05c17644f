// Optional per-kernel timing with HIP events on the caller's stream.
// When enabled, every kernel launch of the library is bracketed by two events;
// lbt_profile_read waits for them and returns, per kernel class, the number of
// launches, the summed duration and the summed algorithmic work.  The two marker
// packets add a fixed few microseconds to every bracket; callers calibrate that with
// the empty kernel class (k_state_set) measured in the same way.  Disabled by default:
// the hot path then pays one predictable branch per launch.
#include <atomic>
#include <mutex>
#include <vector>

#include "lbt_internal.h"

namespace lbt {
namespace {

struct Record {
  int kid;
  double work;
  hipEvent_t start, stop;
};

std::mutex g_mu;
std::atomic<bool> g_enabled{false};   // read by every launch without the lock
std::atomic<bool> g_skeleton{false};  // products skip their contraction loop (measurement aid)
std::vector<Record> g_records;
std::vector<hipEvent_t> g_pool;

const char* const kNames[KID_COUNT] = {
    "k_absmax3",           "k_quantize_flat(grad)", "k_quantize_flat(operand)",
    "k_quantize_layer",      "k_implicit_gemm(dX)",   "k_implicit_gemm(dW)",
    "k_implicit_gemm(fwd)",
    "k_splitk_reduce",     "k_update_interval",     "k_state_set",
    "k_ste_backward"};

hipEvent_t take_event() {
  if (!g_pool.empty()) {
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

}  // namespace

bool profile_skeleton() { return g_skeleton.load(std::memory_order_relaxed); }

ProfScope::ProfScope(int kid, double work, hipStream_t s) : idx_(-1), s_(s) {
  if (!g_enabled.load(std::memory_order_acquire)) return;
  std::lock_guard<std::mutex> lk(g_mu);
  Record r{kid, work, take_event(), take_event()};
  if (!r.start || !r.stop) return;
  (void)hipEventRecord(r.start, s);
  g_records.push_back(r);
  idx_ = (long long)g_records.size() - 1;
}

ProfScope::~ProfScope() {
  if (idx_ < 0) return;
  std::lock_guard<std::mutex> lk(g_mu);
  if (idx_ < (long long)g_records.size()) (void)hipEventRecord(g_records[idx_].stop, s_);
}

}  // namespace lbt

using namespace lbt;

extern "C" {

int lbt_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& r : g_records) {
    (void)hipEventSynchronize(r.stop);
    g_pool.push_back(r.start);
    g_pool.push_back(r.stop);
  }
  g_records.clear();
  g_enabled.store(on != 0, std::memory_order_release);
  return LBT_OK;
}

int lbt_profile_skeleton(int on) {
  g_skeleton.store(on != 0, std::memory_order_relaxed);
  return LBT_OK;
}

int lbt_profile_kernel_count(void) { return KID_COUNT; }

const char* lbt_profile_kernel_name(int kid) {
  return (kid >= 0 && kid < KID_COUNT) ? kNames[kid] : "?";
}

int lbt_profile_read(int64_t* launches, double* total_ms, double* total_work, int capacity) {
  if (!launches || !total_ms || !total_work) return LBT_ERR_NULL;
  if (capacity < KID_COUNT) return LBT_ERR_SHAPE;
  std::lock_guard<std::mutex> lk(g_mu);
  for (int i = 0; i < KID_COUNT; ++i) {
    launches[i] = 0;
    total_ms[i] = 0.0;
    total_work[i] = 0.0;
  }
  for (auto& r : g_records) {
    // a scope whose launch was skipped (early error return) left its events unrecorded
    float ms = 0.0f;
    if (hipEventSynchronize(r.stop) == hipSuccess &&
        hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
      launches[r.kid] += 1;
      total_ms[r.kid] += (double)ms;
      total_work[r.kid] += r.work;
    }
    (void)hipGetLastError();
    g_pool.push_back(r.start);
    g_pool.push_back(r.stop);
  }
  g_records.clear();
  return LBT_OK;
}

}  // extern "C"
