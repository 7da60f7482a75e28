// Error reporting, descriptor validation and version of the C ABI.
#include <stdarg.h>
#include <string.h>

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

}  // namespace spindle

extern "C" const char *spindle_last_error(void) { return spindle::g_error; }

extern "C" uint32_t spindle_version(void) { return (0u << 16) | 1u; }
