// Optional per-kernel timing with HIP events on the launch stream (see gcn_profile_* in gcn.h).
#include <atomic>
#include <mutex>
#include <vector>

#include "common.h"

namespace gcn {

namespace {
constexpr int64_t kCapacity = 65536;
struct Slot {
  gcn_profile_rec rec;
  hipEvent_t start = nullptr, stop = nullptr;
  bool closed = false;
};
std::atomic<int> g_enabled{0};
std::atomic<int> g_kind_mask{-1};   // bit k set: launches of kind k are recorded
std::atomic<int> g_only_d{-1};      // >= 0: only launches of this feature width are recorded
std::mutex g_mu;
std::vector<Slot> g_slots;      // events are created once and reused by later recordings
int64_t g_used = 0, g_dropped = 0;
thread_local int t_suppress = 0;
}  // namespace

ProfSuppress::ProfSuppress() { ++t_suppress; }
ProfSuppress::~ProfSuppress() { --t_suppress; }

ProfScope::ProfScope(int kind, hipStream_t s, int d, int dtype, int64_t rows, int64_t inner, double alg_bytes,
                     double touched_bytes, double flops)
    : s_(s) {
  if (!g_enabled.load(std::memory_order_relaxed) || t_suppress > 0) return;
  if (!((g_kind_mask.load(std::memory_order_relaxed) >> kind) & 1)) return;
  const int only_d = g_only_d.load(std::memory_order_relaxed);
  if (only_d >= 0 && d != only_d) return;
  std::lock_guard<std::mutex> lk(g_mu);
  if (g_used >= kCapacity) { ++g_dropped; return; }
  if ((int64_t)g_slots.size() <= g_used) {
    Slot sl;
    if (hipEventCreate(&sl.start) != hipSuccess || hipEventCreate(&sl.stop) != hipSuccess) { ++g_dropped; return; }
    g_slots.push_back(sl);
  }
  Slot& sl = g_slots[g_used];
  sl.rec = gcn_profile_rec{kind, d, dtype, 0, rows, inner, alg_bytes, touched_bytes, flops, 0.0};
  sl.closed = false;
  if (hipEventRecord(sl.start, s) != hipSuccess) { ++g_dropped; return; }
  slot_ = g_used++;
}

ProfScope::~ProfScope() {
  if (slot_ < 0) return;
  std::lock_guard<std::mutex> lk(g_mu);
  if (slot_ >= g_used) return;                    // recording was restarted in between
  Slot& sl = g_slots[slot_];
  sl.closed = hipEventRecord(sl.stop, s_) == hipSuccess;
}

}  // namespace gcn

using namespace gcn;

extern "C" int gcn_profile_enable(int on) {
  clear_error();
  std::lock_guard<std::mutex> lk(g_mu);
  if (on) { g_used = 0; g_dropped = 0; }
  g_enabled.store(on ? 1 : 0, std::memory_order_relaxed);
  return GCN_OK;
}

extern "C" int gcn_profile_filter(int kind_mask, int d) {
  clear_error();
  g_kind_mask.store(kind_mask, std::memory_order_relaxed);
  g_only_d.store(d, std::memory_order_relaxed);
  return GCN_OK;
}

extern "C" int64_t gcn_profile_count(int64_t* dropped) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (dropped) *dropped = g_dropped;
  return g_used;
}

extern "C" int gcn_profile_get(int64_t i, gcn_profile_rec* out) {
  clear_error();
  if (!out) return fail(GCN_EINVAL, "gcn_profile_get: out is NULL");
  std::lock_guard<std::mutex> lk(g_mu);
  if (i < 0 || i >= g_used) return fail(GCN_EINVAL, "gcn_profile_get: no record %lld", (long long)i);
  Slot& sl = g_slots[i];
  if (!sl.closed) return fail(GCN_EHIP, "gcn_profile_get: record %lld has no stop event", (long long)i);
  GCN_HIP(hipEventSynchronize(sl.stop));
  float ms = 0.f;
  GCN_HIP(hipEventElapsedTime(&ms, sl.start, sl.stop));
  *out = sl.rec;
  out->ms = (double)ms;
  return GCN_OK;
}
