// Error reporting, descriptor validation and version of the C ABI.
#include <stdarg.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "common.h"

namespace spindle {

static thread_local char g_error[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
}

spindle_status check_desc(const spindle_kv_desc *d) {
  if (!d) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "desc is NULL");
  if (d->batch < 1 || d->n_kv_heads < 1 || d->seq_len < 1)
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "batch, n_kv_heads and seq_len must be >= 1");
  if (d->head_dim != kHeadDim)
    SPINDLE_FAIL(SPINDLE_ERR_UNSUPPORTED, "head_dim must be 128, got %d", d->head_dim);
  if (d->dtype != SPINDLE_F32 && d->dtype != SPINDLE_F16 && d->dtype != SPINDLE_BF16)
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "unknown dtype %d", d->dtype);
  if ((int64_t)d->batch * d->n_kv_heads > 32767)
    SPINDLE_FAIL(SPINDLE_ERR_UNSUPPORTED, "batch * n_kv_heads must be <= 32767");
  return SPINDLE_OK;
}

struct ProfRec {
  char name[32];
  hipEvent_t a, b;
};
static std::mutex g_prof_mu;
static std::vector<ProfRec> g_prof;
static bool g_prof_on = false;

static void prof_clear() {
  for (ProfRec &r : g_prof) {
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  g_prof.clear();
}

ProfScope::ProfScope(const char *name, hipStream_t s) : idx(-1), st(s) {
  if (!g_prof_on) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  ProfRec r;
  strncpy(r.name, name, sizeof(r.name) - 1);
  r.name[sizeof(r.name) - 1] = 0;
  if (hipEventCreate(&r.a) != hipSuccess) return;
  if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return; }
  (void)hipEventRecord(r.a, st);
  idx = (int)g_prof.size();
  g_prof.push_back(r);
}

ProfScope::~ProfScope() {
  if (idx < 0) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (idx < (int)g_prof.size()) (void)hipEventRecord(g_prof[idx].b, st);
}

}  // namespace spindle

extern "C" spindle_status spindle_profile(int32_t enable) {
  std::lock_guard<std::mutex> lk(spindle::g_prof_mu);
  spindle::prof_clear();
  spindle::g_prof_on = enable != 0;
  return SPINDLE_OK;
}

extern "C" int32_t spindle_profile_read(char *names, float *ms, int32_t max) {
  std::lock_guard<std::mutex> lk(spindle::g_prof_mu);
  int32_t n = 0;
  for (spindle::ProfRec &r : spindle::g_prof) {
    if (n >= max || !names || !ms) break;
    if (hipEventSynchronize(r.b) != hipSuccess) return -1;
    float t = 0.f;
    if (hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) return -1;
    memcpy(names + (size_t)n * 32, r.name, 32);
    ms[n] = t;
    ++n;
  }
  spindle::prof_clear();
  return n;
}

extern "C" const char *spindle_last_error(void) { return spindle::g_error; }

extern "C" uint32_t spindle_version(void) { return (0u << 16) | 1u; }
