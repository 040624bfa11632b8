// Error text and version of the C ABI.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "common.h"

namespace rn50 {
static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_err[0] = 0; }

// ------------------------------------------------------------- launch timing
static bool g_prof_on = false;
static char g_prof_tag[64] = "";
static size_t g_prof_max = 0, g_prof_used = 0;
static bool g_prof_paused = false;
static size_t g_prof_ended = 0;  // records of the last rn50_profile_end
static std::vector<hipEvent_t> g_prof_events;  // start/stop pairs, grown on demand, reused
static std::vector<const char*> g_prof_tags;   // the tag (a string literal of the library) of every record

KernelTimer::KernelTimer(const char* tag) {
  if (!g_prof_on || g_prof_paused || g_prof_used >= g_prof_max || strncmp(tag, g_prof_tag, strlen(g_prof_tag)) != 0) return;
  while (g_prof_events.size() < 2 * (g_prof_used + 1)) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return;
    g_prof_events.push_back(e);
  }
  start_ = g_prof_events[2 * g_prof_used];
  stop_ = g_prof_events[2 * g_prof_used + 1];
  if (g_prof_tags.size() <= g_prof_used) g_prof_tags.resize(g_prof_used + 1);
  g_prof_tags[g_prof_used] = tag;
  ++g_prof_used;
}
}  // namespace rn50

extern "C" int rn50_profile_begin(const char* kernel_tag, int max_records) {
  rn50::clear_error();
  if (!kernel_tag || max_records <= 0 || strlen(kernel_tag) >= sizeof(rn50::g_prof_tag))
    return rn50::fail(RN50_ERR_INVALID, "rn50_profile_begin: bad tag or max_records");
  strcpy(rn50::g_prof_tag, kernel_tag);
  rn50::g_prof_max = static_cast<size_t>(max_records);
  rn50::g_prof_used = 0;
  rn50::g_prof_on = true;
  rn50::g_prof_paused = false;
  return RN50_OK;
}
extern "C" void rn50_profile_pause(int paused) { rn50::g_prof_paused = paused != 0; }
static int profile_end_impl(float* ms_out, float* start_ms_out, int capacity);
extern "C" int rn50_profile_end(float* ms_out, int capacity) { return profile_end_impl(ms_out, nullptr, capacity); }
extern "C" int rn50_profile_end_timeline(float* ms_out, float* start_ms_out, int capacity) {
  return profile_end_impl(ms_out, start_ms_out, capacity);
}
static int profile_end_impl(float* ms_out, float* start_ms_out, int capacity) {
  using namespace rn50;
  g_prof_on = false;
  const size_t n = g_prof_used;
  if (n == 0) return 0;
  if (hipEventSynchronize(g_prof_events[2 * n - 1]) != hipSuccess)
    return fail(RN50_ERR_HIP, "rn50_profile_end: event synchronize failed");
  size_t w = 0;
  for (size_t i = 0; i < n && ms_out && w < static_cast<size_t>(capacity); ++i) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_prof_events[2 * i], g_prof_events[2 * i + 1]) != hipSuccess) ms = -1.f;
    if (start_ms_out) {  // begin of this launch after the begin of the first recorded one
      float at = 0.f;
      if (hipEventElapsedTime(&at, g_prof_events[0], g_prof_events[2 * i]) != hipSuccess) at = -1.f;
      start_ms_out[w] = at;
    }
    ms_out[w++] = ms;
  }
  g_prof_used = 0;
  g_prof_ended = n;
  return static_cast<int>(n);
}
extern "C" const char* rn50_profile_tag(int record) {
  using namespace rn50;
  if (record < 0 || static_cast<size_t>(record) >= g_prof_ended || static_cast<size_t>(record) >= g_prof_tags.size()) return "";
  return g_prof_tags[record];
}

extern "C" const char* rn50_last_error(void) { return rn50::g_err; }
extern "C" int rn50_version(void) { return 2; }
