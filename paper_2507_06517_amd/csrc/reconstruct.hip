// Codebook reconstruction, Eq. 14: x~_a = C[r_a] * m_a.
#include "common.h"

namespace spindle {
namespace {

template <int DT>
__global__ __launch_bounds__(256) void reconstruct_kernel(const char *C, const int32_t *ref, const float *mag,
                                                          char *out, int n, int cap, size_t rows) {
  typedef typename Elem<DT>::type T;
  constexpr int per = 16 / sizeof(T);           // elements per 16-byte chunk
  constexpr int tpr = kHeadDim / per;           // threads per row
  const size_t row = (size_t)blockIdx.x * (256 / tpr) + threadIdx.x / tpr;
  if (row >= rows) return;
  const int ch = threadIdx.x % tpr;
  const size_t u = row / n;
  int r = ref[row];
  u4 o = {0, 0, 0, 0};
  if (r >= 0 && r < cap) {
    const float m = mag[row];
    const u4 v = *reinterpret_cast<const u4 *>(C + ((u * cap + r) * kHeadDim) * sizeof(T) + ch * 16);
    const T *e = reinterpret_cast<const T *>(&v);
    T *w = reinterpret_cast<T *>(&o);
#pragma unroll
    for (int i = 0; i < per; ++i) w[i] = Elem<DT>::from_float(Elem<DT>::to_float(e[i]) * m);
  }
  *reinterpret_cast<u4 *>(out + row * kHeadDim * sizeof(T) + ch * 16) = o;
}

}  // namespace
}  // namespace spindle

using namespace spindle;

extern "C" spindle_status spindle_reconstruct(int32_t units, int32_t seq_len, int32_t head_dim, int32_t dtype,
                                              int32_t max_codes, const void *C, const int32_t *ref,
                                              const float *mag, void *out, void *stream) {
  if (units < 1 || seq_len < 1 || max_codes < 1) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "units, seq_len and max_codes must be >= 1");
  if (head_dim != kHeadDim) SPINDLE_FAIL(SPINDLE_ERR_UNSUPPORTED, "head_dim must be 128, got %d", head_dim);
  if (!C || !ref || !mag || !out) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "C, ref, mag and out are required");
  if ((reinterpret_cast<uintptr_t>(C) | reinterpret_cast<uintptr_t>(out)) & 15)
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t rows = (size_t)units * seq_len;
  const char *Cc = static_cast<const char *>(C);
  char *oc = static_cast<char *>(out);
  if (dtype == SPINDLE_F32) {
    hipLaunchKernelGGL(reconstruct_kernel<SPINDLE_F32>, dim3((rows + 7) / 8), dim3(256), 0, st, Cc, ref, mag, oc, seq_len, max_codes, rows);
  } else if (dtype == SPINDLE_F16) {
    hipLaunchKernelGGL(reconstruct_kernel<SPINDLE_F16>, dim3((rows + 15) / 16), dim3(256), 0, st, Cc, ref, mag, oc, seq_len, max_codes, rows);
  } else if (dtype == SPINDLE_BF16) {
    hipLaunchKernelGGL(reconstruct_kernel<SPINDLE_BF16>, dim3((rows + 15) / 16), dim3(256), 0, st, Cc, ref, mag, oc, seq_len, max_codes, rows);
  } else {
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "unknown dtype %d", dtype);
  }
  SPINDLE_HIP(hipGetLastError());
  return SPINDLE_OK;
}
