// Tuning overrides and test hooks, read from the environment ONCE per process (the first library call that needs
// them) instead of on every call; dsbd_reload_knobs() reads them again (tests that change the environment call it).
#include "common.h"
#include <stdlib.h>
#include <atomic>
#include <mutex>

namespace {
DsbdKnobs g_knobs;
std::atomic<int> g_loaded{0};
std::mutex g_mutex;

int env_int(const char* name, int dflt) {
  const char* e = getenv(name);
  return e ? atoi(e) : dflt;
}

void load(DsbdKnobs& k) {
  k.attn_nsplit = env_int("DSBD_ATTN_NSPLIT", 0);
  k.attn_waves8 = getenv("DSBD_ATTN_WAVES8") != nullptr;
  k.attn_staged = getenv("DSBD_ATTN_STAGED") != nullptr;
  k.attn_trace = getenv("DSBD_ATTN_TRACE") != nullptr;
  k.stats_chunk = env_int("DSBD_STATS_CHUNK", 0);
  k.verify_g = env_int("DSBD_VERIFY_G", 0);
  k.verify_trace = getenv("DSBD_VERIFY_TRACE") != nullptr;
  k.verify_trace_wg = 0;
  if (const char* e = getenv("DSBD_VERIFY_TRACE")) { const int v = atoi(e); if (v > 1) k.verify_trace_wg = v - 1; }
  const char* e = getenv("DSBD_VERIFY_SYNC_LIMIT_US");
  k.verify_sync_limit_us = e ? atoll(e) : 0;
  k.verify_mute_wg = env_int("DSBD_VERIFY_TEST_MUTE_WG", -1);
  k.verify_lds_slice = env_int("DSBD_VERIFY_LDS_SLICE", -1);
  k.verify_overlap = env_int("DSBD_VERIFY_OVERLAP", 1);
  k.warp_fast = env_int("DSBD_WARP_FAST", 1);
  k.event_fence = env_int("DSBD_EVENT_FENCE", 0);
  k.stats_side_lds = env_int("DSBD_STATS_SIDE_LDS", -1);
  if (k.stats_side_lds > 65536) k.stats_side_lds = -1;
}
}  // namespace

const DsbdKnobs& dsbd_knobs() {
  if (!g_loaded.load(std::memory_order_acquire)) {
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!g_loaded.load(std::memory_order_relaxed)) {
      load(g_knobs);
      g_loaded.store(1, std::memory_order_release);
    }
  }
  return g_knobs;
}

extern "C" void dsbd_reload_knobs(void) {
  std::lock_guard<std::mutex> lock(g_mutex);
  load(g_knobs);
  g_loaded.store(1, std::memory_order_release);
}
