// Error reporting, descriptor validation and version of the C ABI.
#include <math.h>
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

spindle_status kv_layout(const spindle_kv_desc *d, KvLayout *out) {
  const long long elt = dtype_bytes(d->dtype);
  const long long st = d->stride_t ? d->stride_t : d->head_dim;
  const long long sh = d->stride_h ? d->stride_h : (long long)d->seq_len * d->head_dim;
  const long long sb = d->stride_b ? d->stride_b : (long long)d->n_kv_heads * d->seq_len * d->head_dim;
  if (d->stride_b < 0 || d->stride_h < 0 || d->stride_t < 0 || st < d->head_dim)
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "strides must be >= 0 and stride_t >= head_dim");
  if ((st | sh | sb) & 7) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "strides must be multiples of 8 elements");
  out->sb = sb * elt;
  out->sh = sh * elt;
  out->st = st * elt;
  out->H = d->n_kv_heads;
  return SPINDLE_OK;
}

spindle_status allow_lds(LdsLimit &state, const void *kernel, size_t bytes) {
  int dev = 0;
  SPINDLE_HIP(hipGetDevice(&dev));
  const uint64_t bit = 1ull << (dev & 63);
  if (dev < 64 && (state.devices.load(std::memory_order_acquire) & bit)) return SPINDLE_OK;
  SPINDLE_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  if (dev < 64) state.devices.fetch_or(bit, std::memory_order_release);
  return SPINDLE_OK;
}

struct ProfRec {
  char name[32];
  hipEvent_t a, b;
};
static std::mutex g_prof_mu;
static std::vector<ProfRec> g_prof;
static int g_prof_mode = 0;             // 0 off, 1 every kernel, 2 only the similarity kernel

static void prof_clear() {
  for (ProfRec &r : g_prof) {
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  g_prof.clear();
}

ProfScope::ProfScope(const char *name, hipStream_t s) : idx(-1), st(s) {
  if (g_prof_mode == 0) return;
  if (g_prof_mode == 2 && strcmp(name, "shallow_gram") != 0) return;
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
  spindle::g_prof_mode = enable == 2 ? 2 : (enable != 0 ? 1 : 0);
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

// Layer-wise budgets, Eq. 5-6 (Sec. "Attention Weight Based Token Eviction").
extern "C" spindle_status spindle_layer_budgets(double reserve_ratio, int32_t seq_len, int32_t window,
                                                int32_t n_layers, double beta, int32_t *budgets, double *ratios) {
  if (!budgets) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "budgets is NULL");
  if (n_layers < 1 || window < 1 || window > seq_len)
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "need n_layers >= 1 and 1 <= window <= seq_len");
  if (!(beta >= 0.0 && beta <= 1.0) || !(reserve_ratio >= 0.0 && reserve_ratio <= 1.0))
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "beta and reserve_ratio must lie in [0, 1]");
  const int context = seq_len - window;
  double mean = context > 0 ? (reserve_ratio * seq_len - window) / context : 0.0;
  mean = mean < 0.0 ? 0.0 : (mean > 1.0 ? 1.0 : mean);
  const double knee = 0.5 * (1.0 + beta);
  double first = mean, last = mean;                       // at or below the floor: flat
  if (mean > knee) {
    first = 1.0;
    last = 2.0 * mean - 1.0;
  } else if (mean > beta) {
    first = 2.0 * mean - beta;
    last = beta;
  }
  for (int layer = 0; layer < n_layers; ++layer) {
    // Eq. 6 in the printed order of operations (slope per layer, times the layer), so that the
    // integer of Eq. 7 below is the one any evaluation of the printed formulas in doubles gives
    const double share = n_layers > 1 ? first + (last - first) / (double)(n_layers - 1) * layer : mean;
    if (ratios) ratios[layer] = share;
    long kept = (long)floor(share * (double)context);         // Eq. 7: k = floor(r_c(layer) l_c)
    kept = kept < 0 ? 0 : (kept > context ? context : kept);
    budgets[layer] = window + (int32_t)kept;
  }
  return SPINDLE_OK;
}

// Reserve ratio of a layer, Eq. 15 (Sec. "Experiments").
extern "C" spindle_status spindle_reserve_ratio(int64_t kept_tokens, int64_t total_tokens, int64_t codebook_entries,
                                                int32_t head_dim, int32_t index_bits, int32_t elem_bits,
                                                int32_t magnitude_bits, double *out) {
  if (!out) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "out is NULL");
  if (kept_tokens < 1 || total_tokens < 1 || codebook_entries < 1 || head_dim < 1 || index_bits < 1 || elem_bits < 1 ||
      magnitude_bits < 1)
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "counts and widths must be >= 1");
  if (kept_tokens > total_tokens || codebook_entries > kept_tokens)
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "need codebook_entries <= kept_tokens <= total_tokens");
  out[0] = (double)kept_tokens / (double)total_tokens;
  out[1] = (double)codebook_entries / (double)kept_tokens;
  out[2] = ((double)head_dim + (double)index_bits / (double)elem_bits + (double)magnitude_bits / (double)elem_bits) /
           (double)head_dim;
  out[3] = out[0] * out[1] * out[2];
  return SPINDLE_OK;
}

// ---------------------------------------------------------------- measurement aids
namespace spindle {
// (external linkage on purpose: a variable nobody can read would be removed together with
// everything that leads up to the store)
__device__ float g_cal_sink;
namespace {

// Four independent chains of v_mfma_f32_32x32x16_f16 per wave on operands that never leave the
// registers: what the matrix cores sustain with no memory traffic and no other work.  The power
// a matrix instruction draws, and with it the clock the part sustains, depends on how many operand
// bits change from one instruction to the next: pattern 0 = small non-negative values (few bits set,
// little switching), pattern 1 = pseudo-random values with the sign mix and magnitude of the
// similarity kernel's operands (unit vectors of 128 dimensions scaled by 2^10), different for
// every chain on both sides.
__global__ __launch_bounds__(256) void cal_mfma_f16(int iters, int pattern) {
  h8 a[4], b[4];
#pragma unroll
  for (int ch = 0; ch < 4; ++ch)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (pattern == 0) {
        a[ch][i] = (_Float16)(0.001f * (float)((threadIdx.x + i + 5 * ch) & 15));
        b[ch][i] = (_Float16)(0.002f * (float)((threadIdx.x * 3 + i) & 7));
      } else {
        uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 64u + (uint32_t)(ch * 16 + i);
        h = (h ^ 61u) ^ (h >> 16); h *= 9u; h ^= h >> 4; h *= 0x27d4eb2du; h ^= h >> 15;   // integer mix
        // sum of four uniform bytes, centred: roughly normal, standard deviation 90 = 2^10 / sqrt(128)
        const float ga = ((float)(h & 255u) + (float)((h >> 8) & 255u) - 255.f) * 0.864f;
        const float gb = ((float)((h >> 16) & 255u) + (float)(h >> 24) - 255.f) * 0.864f;
        a[ch][i] = (_Float16)ga;
        b[ch][i] = (_Float16)gb;
      }
    }
  f16v c[4];
#pragma unroll
  for (int ch = 0; ch < 4; ++ch)
#pragma unroll
    for (int v = 0; v < 16; ++v) c[ch][v] = (float)ch;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int ch = 0; ch < 4; ++ch) c[ch] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[ch], b[ch], c[ch], 0, 0, 0);
  }
  const float sum = c[0][0] + c[1][5] + c[2][9] + c[3][15];
  if (sum == -1.2345e30f) g_cal_sink = sum;            // never reached with these operands
}

// Plain copy, 16 bytes per thread and trip: the scale reference for the HBM traffic counters
// and the copy rate the memory system sustains.
__global__ __launch_bounds__(256) void cal_copy(const u4 *__restrict__ src, u4 *__restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace
}  // namespace spindle

extern "C" spindle_status spindle_calibrate_copy(const void *src, void *dst, size_t bytes, void *stream, double *gbs) {
  if (!src || !dst || !gbs || bytes < 16 || ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15))
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "src, dst (16-byte aligned device buffers), bytes >= 16 and gbs are required");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t n16 = bytes / 16;
  const int blocks = (int)(n16 / 256 < 16384 ? (n16 + 255) / 256 : 16384);
  hipEvent_t e0, e1;
  SPINDLE_HIP(hipEventCreate(&e0));
  SPINDLE_HIP(hipEventCreate(&e1));
  hipLaunchKernelGGL(spindle::cal_copy, dim3(blocks), dim3(256), 0, st, static_cast<const spindle::u4 *>(src),
                     static_cast<spindle::u4 *>(dst), n16);                                  // warm-up
  SPINDLE_HIP(hipEventRecord(e0, st));
  hipLaunchKernelGGL(spindle::cal_copy, dim3(blocks), dim3(256), 0, st, static_cast<const spindle::u4 *>(src),
                     static_cast<spindle::u4 *>(dst), n16);
  SPINDLE_HIP(hipEventRecord(e1, st));
  SPINDLE_HIP(hipEventSynchronize(e1));
  float ms = 0.f;
  SPINDLE_HIP(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *gbs = 2.0 * (double)(n16 * 16) / ((double)ms * 1e-3) / 1e9;
  return SPINDLE_OK;
}

extern "C" spindle_status spindle_calibrate_mfma(int32_t iters, int32_t pattern, void *stream, double *tflops) {
  if (!tflops || iters < 1 || pattern < 0 || pattern > 1)
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "tflops is required, iters must be >= 1 and pattern 0 or 1");
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipDeviceProp_t prop;
  int dev = 0;
  SPINDLE_HIP(hipGetDevice(&dev));
  SPINDLE_HIP(hipGetDeviceProperties(&prop, dev));
  const int blocks = prop.multiProcessorCount * 2;      // 8 waves per compute unit: two per SIMD
  hipEvent_t e0, e1;
  SPINDLE_HIP(hipEventCreate(&e0));
  SPINDLE_HIP(hipEventCreate(&e1));
  hipLaunchKernelGGL(spindle::cal_mfma_f16, dim3(blocks), dim3(256), 0, st, iters, pattern);     // warm-up
  SPINDLE_HIP(hipEventRecord(e0, st));
  hipLaunchKernelGGL(spindle::cal_mfma_f16, dim3(blocks), dim3(256), 0, st, iters, pattern);
  SPINDLE_HIP(hipEventRecord(e1, st));
  SPINDLE_HIP(hipEventSynchronize(e1));
  float ms = 0.f;
  SPINDLE_HIP(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  const double flop = (double)blocks * 4.0 * (double)iters * 4.0 * 2.0 * 32.0 * 32.0 * 16.0;
  *tflops = flop / ((double)ms * 1e-3) / 1e12;
  return SPINDLE_OK;
}

extern "C" const char *spindle_last_error(void) { return spindle::g_error; }

extern "C" uint32_t spindle_version(void) { return (0u << 16) | 1u; }
