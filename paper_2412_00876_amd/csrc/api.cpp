// Host-only parts of the C ABI: version, per-thread error text, validation of the cache descriptor.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>

#include "dllava.h"

namespace dllava {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

static std::atomic<int> g_override[DLLAVA_LAUNCH_KNOBS];

int launch_override(int knob) { return g_override[knob].load(std::memory_order_relaxed); }

int check_cache(const dllava_kv_cache* c, const char* who) {
  if (!c) { set_error("%s: cache is NULL", who); return DLLAVA_ENULL; }
  if (!c->pages || !c->block_table || !c->cache_len) {
    set_error("%s: cache pages, block_table and cache_len are required", who);
    return DLLAVA_ENULL;
  }
  if (c->dtype != DLLAVA_F32 && c->dtype != DLLAVA_BF16) {
    set_error("%s: unknown cache dtype %d", who, c->dtype);
    return DLLAVA_EDTYPE;
  }
  if (c->page_size != 16) { set_error("%s: page_size must be 16 (got %d)", who, c->page_size); return DLLAVA_ESHAPE; }
  if (c->Dh != 64 && c->Dh != 128) { set_error("%s: Dh must be 64 or 128 (got %d)", who, c->Dh); return DLLAVA_ESHAPE; }
  if (c->H <= 0 || c->n_pages <= 0 || c->max_pages_per_seq <= 0) {
    set_error("%s: cache H, n_pages and max_pages_per_seq must be positive", who);
    return DLLAVA_ESHAPE;
  }
  if ((reinterpret_cast<uintptr_t>(c->pages) & 15) != 0) { set_error("%s: cache pages must be 16-byte aligned", who); return DLLAVA_EINVAL; }
  return DLLAVA_OK;
}

}  // namespace dllava

extern "C" int dllava_version(void) { return 100; }

extern "C" const char* dllava_last_error(void) { return dllava::g_err; }

extern "C" int dllava_set_launch_override(int knob, int value) {
  if (knob < 0 || knob >= DLLAVA_LAUNCH_KNOBS) {
    dllava::set_error("set_launch_override: unknown knob %d", knob);
    return DLLAVA_EINVAL;
  }
  if (value < 0) {
    dllava::set_error("set_launch_override: value %d < 0", value);
    return DLLAVA_EINVAL;
  }
  dllava::g_override[knob].store(value, std::memory_order_relaxed);
  return DLLAVA_OK;
}
