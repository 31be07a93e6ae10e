#include "profile.h"

#include <stdio.h>
#include <string.h>

#include <vector>

#include "common.h"

namespace mdz {

namespace {
struct State {
  bool on = false;
  std::vector<hipEvent_t> ev;  // pairs: 2*i start, 2*i+1 stop
  std::vector<int> tags;
  int n = 0;  // launches recorded
  int cap = 0;
  int dropped = 0;
} g;
const char* kNames[PROF_NUM_TAGS] = {"gemm_portable", "gemm_w64", "gemm_n64", "gemm_w32", "gemm_n32", "gemm_large", "attention", "rmsnorm", "rope", "swiglu",
                                     "embed", "select", "accept", "kv_compact", "misc"};
}  // namespace

const char* prof_tag_name(int tag) { return tag >= 0 && tag < PROF_NUM_TAGS ? kNames[tag] : "?"; }
bool prof_enabled() { return g.on; }

void prof_record(int tag, hipStream_t st, bool start) {
  if (start) {
    if (g.n >= g.cap) {
      ++g.dropped;
      return;
    }
    g.tags[g.n] = tag;
    (void)hipEventRecord(g.ev[2 * g.n], st);
  } else {
    if (g.n >= g.cap) return;
    (void)hipEventRecord(g.ev[2 * g.n + 1], st);
    ++g.n;
  }
}

bool prof_kernel_events(int tag, hipEvent_t* start, hipEvent_t* stop) {
  if (g.n >= g.cap) {
    ++g.dropped;
    return false;
  }
  g.tags[g.n] = tag;
  *start = g.ev[2 * g.n];
  *stop = g.ev[2 * g.n + 1];
  ++g.n;
  return true;
}

}  // namespace mdz

using namespace mdz;

extern "C" {
#pragma GCC visibility push(default)

int medusa_profile_begin(int max_launches) {
  MDZ_REQUIRE(max_launches > 0 && max_launches <= (1 << 20), MDZ_EINVAL, "profile: bad max_launches %d", max_launches);
  MDZ_REQUIRE(!g.on, MDZ_EINVAL, "profile: already recording");
  while ((int)g.ev.size() < 2 * max_launches) {
    hipEvent_t e;
    MDZ_HIP(hipEventCreate(&e));
    g.ev.push_back(e);
  }
  g.tags.assign(max_launches, 0);
  g.n = 0;
  g.cap = max_launches;
  g.dropped = 0;
  g.on = true;
  return MDZ_OK;
}

int medusa_profile_end(char* report, int64_t report_bytes) {
  MDZ_REQUIRE(g.on, MDZ_EINVAL, "profile: not recording");
  g.on = false;
  MDZ_REQUIRE(report && report_bytes > 0, MDZ_EINVAL, "profile: NULL report buffer");
  double total[PROF_NUM_TAGS] = {}, mn[PROF_NUM_TAGS], mx[PROF_NUM_TAGS] = {};
  long cnt[PROF_NUM_TAGS] = {};
  for (int t = 0; t < PROF_NUM_TAGS; ++t) mn[t] = 1e30;
  for (int i = 0; i < g.n; ++i) {
    MDZ_HIP(hipEventSynchronize(g.ev[2 * i + 1]));
    float ms = 0.f;
    MDZ_HIP(hipEventElapsedTime(&ms, g.ev[2 * i], g.ev[2 * i + 1]));
    int t = g.tags[i];
    double us = ms * 1e3;
    total[t] += us;
    cnt[t]++;
    if (us < mn[t]) mn[t] = us;
    if (us > mx[t]) mx[t] = us;
  }
  int64_t off = 0;
  report[0] = 0;
  for (int t = 0; t < PROF_NUM_TAGS; ++t) {
    if (!cnt[t]) continue;
    int w = snprintf(report + off, (size_t)(report_bytes - off), "%s,%ld,%.3f,%.3f,%.3f\n", kNames[t], cnt[t], total[t],
                     mn[t], mx[t]);
    if (w < 0 || off + w >= report_bytes) break;
    off += w;
  }
  if (g.dropped) snprintf(report + off, (size_t)(report_bytes - off), "dropped,%d,0,0,0\n", g.dropped);
  return MDZ_OK;
}

#pragma GCC visibility pop
}
