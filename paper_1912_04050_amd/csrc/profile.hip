// Measurement aid: HIP event pairs around the product kernels (rtc_profile_enable / _read).
// A fixed ring of event pairs, created lazily and kept for the life of the process; recording
// stops when the ring is full.  One lock serialises every access, so calls from several host
// threads are safe (their kernels share the one record).
#include <hip/hip_runtime.h>

#include <mutex>

#include "rtc_internal.h"

namespace rtc {

thread_local bool t_launch_failed = false;   // see launch_checked
thread_local bool t_dry_run = false;
thread_local bool t_dry_bad = false;

namespace {

constexpr int kRing = 1024;
struct Slot {
  hipEvent_t e0, e1;
  int kind;
  bool made;
};
Slot g_ring[kRing];
int g_count = 0;
bool g_on = false;
bool g_all = false;    // also the launches behind a per-row selector
bool g_open = false;   // a begin without its end
std::mutex g_lock;

}  // namespace

void prof_begin(int kind, hipStream_t stream, bool gated) {
  if (t_dry_run) return;
  std::lock_guard<std::mutex> lock(g_lock);
  if (!g_on || (gated && !g_all) || g_count >= kRing) return;
  Slot& s = g_ring[g_count];
  if (!s.made) {
    if (hipEventCreate(&s.e0) != hipSuccess || hipEventCreate(&s.e1) != hipSuccess) { g_on = false; return; }
    s.made = true;
  }
  s.kind = kind;
  if (hipEventRecord(s.e0, stream) == hipSuccess) g_open = true;
}

void prof_end(hipStream_t stream) {
  if (t_dry_run) return;
  std::lock_guard<std::mutex> lock(g_lock);
  if (!g_on || !g_open) return;
  g_open = false;
  if (hipEventRecord(g_ring[g_count].e1, stream) == hipSuccess) ++g_count;
}

}  // namespace rtc

extern "C" {

int rtc_profile_enable(int on) {
  std::lock_guard<std::mutex> lock(rtc::g_lock);
  rtc::g_on = on != 0;
  rtc::g_all = on >= 2;
  rtc::g_count = 0;
  rtc::g_open = false;
  return RTC_OK;
}

int rtc_profile_read(int max_entries, int* kinds, float* ms) {
  if (kinds == nullptr || ms == nullptr) return RTC_ERR_NULL;
  std::lock_guard<std::mutex> lock(rtc::g_lock);
  int out = 0;
  for (int i = 0; i < rtc::g_count && out < max_entries; ++i) {
    float t = 0.f;
    if (hipEventSynchronize(rtc::g_ring[i].e1) != hipSuccess) return RTC_ERR_HIP;
    if (hipEventElapsedTime(&t, rtc::g_ring[i].e0, rtc::g_ring[i].e1) != hipSuccess) return RTC_ERR_HIP;
    kinds[out] = rtc::g_ring[i].kind;
    ms[out] = t;
    ++out;
  }
  return out;
}

}  // extern "C"
