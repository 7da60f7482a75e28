// Codebook path: workspace layout and the C entry points (kernels: shallow_graph.hip,
// shallow_merge.hip, shallow_codebook.hip; what they share: shallow.h).
#include <vector>

#include "shallow.h"

namespace spindle {
namespace {

// What must hold before the first kernel of a call: counters, list counts and flags zero,
// n_codes = -1 ("not finished"), codebooks zero.  One launch for all of it.
__global__ __launch_bounds__(256) void shallow_init(ShallowParams p, size_t nzero, size_t cwords, int T) {
  const size_t stride = (size_t)gridDim.x * blockDim.x, i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t *z = reinterpret_cast<uint32_t *>(p.counters);
  for (size_t i = i0; i < nzero; i += stride) z[i] = 0u;
  for (int t = 0; t < T; ++t) {
    for (size_t i = i0; i < (size_t)p.U; i += stride) p.n_codes[t][i] = -1;
    u4 *c = reinterpret_cast<u4 *>(p.C[t]);               // 16-byte aligned, a multiple of 16 bytes per row
    for (size_t i = i0; i < cwords / 4; i += stride) c[i] = u4{0, 0, 0, 0};
  }
}

// Copies the rows of G without their padding words.
__global__ void export_adj(const uint32_t *G, uint32_t *out, size_t rows, int Wp, int W) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < rows * W; i += (size_t)gridDim.x * blockDim.x)
    out[i] = G[(i / W) * Wp + (i % W)];
}

// ---------------------------------------------------------------- workspace
// 32-bit words at the end of the workspace that every call clears before use.
size_t zero_words(int UT, int n) {
  const size_t nchunk = (size_t)((n + kChunkCols - 1) / kChunkCols), nI = (size_t)((n + kPanelRows - 1) / kPanelRows);
  return (size_t)UT * kCounters + 4 + 2 * (size_t)UT + (size_t)UT * nchunk + (size_t)UT * nI;
}

size_t carve(ShallowParams &p, void *ws, int UT, int n) {
  Carver cv(ws);
  const size_t N = (size_t)UT * n;
  p.Wp = ((n + 127) / 128) * 4;   // whole 16-byte pieces: shallow_gram writes every word of a row
  p.Xh = cv.take<_Float16>((N + 512) * kHeadDim);   // shallow_gram stages up to 5 tiles past the last token
  p.m64 = cv.take<double>(N);
  p.err = cv.take<float>(N);
  p.G = cv.take<uint32_t>(N * p.Wp);
  p.deg0 = cv.take<int>(N);
  p.alive = cv.take<int>(N);
  p.alive2 = cv.take<int>(N);
  p.gone = cv.take<uint32_t>(N);
  p.n16 = (n + 15) & ~15;
  p.gone8 = cv.take<uint8_t>((size_t)UT * p.n16);
  p.nbr = cv.take<uint16_t>(N * kListCap);
  p.slot = cv.take<int>(N);
  p.cand = cv.take<int>(N);
  p.dying = cv.take<int>(N);
  p.pick_vert = cv.take<int>(N);
  p.rank = cv.take<int>(N);
  p.rank_vert = cv.take<int>(N);
  p.key = cv.take<uint32_t>(N);
  p.m1 = cv.take<uint32_t>(N);
  p.pick_key = cv.take<uint32_t>(N);
  p.ovf = cv.take<uint32_t>(N);
  p.ovf_left = cv.take<uint32_t>(N);
  p.cstat = cv.take<float2>(N * 2);
  p.ccand = cv.take<uint2>(N * 2 * kCandCap);
  p.fix_cap = (unsigned)(32 * (size_t)n > 4096 ? 32 * (size_t)n : 4096);
  p.fix = cv.take<uint32_t>((size_t)UT * p.fix_cap);
  p.fedges = cv.take<uint32_t>((size_t)UT * ((n + kPanelRows - 1) / kPanelRows) * kFixBucket);
  {
    const size_t nI = (size_t)((n + kPanelRows - 1) / kPanelRows), nJc = (size_t)((n + kChunkCols - 1) / kChunkCols);
    p.seg_cap = seg_cap_for(n);
    p.edges = cv.take<uint32_t>((size_t)UT * nJc * nI * 4 * p.seg_cap);
    p.ecount = cv.take<unsigned>((size_t)UT * nJc * nI * 4);
  }
  // everything that must start at zero sits together at the end:
  // counters [UT][kCounters], ovf_count, fix_overflow, need_full + 1 spare, fix_count [UT], ovf_cnt [UT],
  // echunk [UT][chunks], fecount [UT][panels]
  const size_t nchunk = (size_t)((n + kChunkCols - 1) / kChunkCols);
  p.counters = cv.take<int>(zero_words(UT, n));
  int *tail = p.counters ? p.counters + (size_t)UT * kCounters : nullptr;
  p.ovf_count = reinterpret_cast<unsigned *>(tail);
  p.fix_overflow = reinterpret_cast<unsigned *>(tail ? tail + 1 : nullptr);
  p.fix_count = reinterpret_cast<unsigned *>(tail ? tail + 4 : nullptr);
  p.ovf_cnt = reinterpret_cast<unsigned *>(tail ? tail + 4 + UT : nullptr);
  p.echunk = reinterpret_cast<unsigned *>(tail ? tail + 4 + 2 * (size_t)UT : nullptr);
  p.fecount = reinterpret_cast<unsigned *>(tail ? tail + 4 + 2 * (size_t)UT + (size_t)UT * nchunk : nullptr);
  p.need_full = reinterpret_cast<unsigned *>(tail ? tail + 2 : nullptr);
  return cv.total();
}

}  // namespace
}  // namespace spindle

using namespace spindle;

extern "C" spindle_status spindle_shallow_workspace_bytes(const spindle_kv_desc *desc, int32_t n_tensors,
                                                          size_t *bytes) {
  spindle_status s = check_desc(desc);
  if (s != SPINDLE_OK) return s;
  if (!bytes) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "bytes is NULL");
  if (n_tensors < 1 || n_tensors > 2) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "n_tensors must be 1 or 2");
  if (desc->seq_len > 65535) SPINDLE_FAIL(SPINDLE_ERR_UNSUPPORTED, "seq_len must be <= 65535 for the codebook path");
  ShallowParams p;
  *bytes = carve(p, nullptr, desc->batch * desc->n_kv_heads * n_tensors, desc->seq_len);
  return SPINDLE_OK;
}

extern "C" spindle_status spindle_shallow_stats(const spindle_kv_desc *desc, int32_t n_tensors,
                                                const void *workspace, void *stream, int32_t *stats) {
  size_t need = 0;
  spindle_status s = spindle_shallow_workspace_bytes(desc, n_tensors, &need);
  if (s != SPINDLE_OK) return s;
  if (!workspace || !stats) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "workspace and stats are required");
  const int UT = desc->batch * desc->n_kv_heads * n_tensors;
  ShallowParams p;
  memset(&p, 0, sizeof(p));
  carve(p, const_cast<void *>(workspace), UT, desc->seq_len);
  hipStream_t st = static_cast<hipStream_t>(stream);
  std::vector<int> cnt((size_t)UT * kCounters);
  std::vector<unsigned> fixc(UT);
  SPINDLE_HIP(hipStreamSynchronize(st));
  SPINDLE_HIP(hipMemcpy(cnt.data(), p.counters, cnt.size() * sizeof(int), hipMemcpyDeviceToHost));
  SPINDLE_HIP(hipMemcpy(fixc.data(), p.fix_count, fixc.size() * sizeof(unsigned), hipMemcpyDeviceToHost));
  for (int i = 0; i < UT; ++i) {
    stats[16 * i + 0] = cnt[(size_t)i * kCounters + C_ROUNDS];
    stats[16 * i + 1] = cnt[(size_t)i * kCounters + C_PICKS];
    stats[16 * i + 2] = (int32_t)fixc[i];
    stats[16 * i + 3] = 0;
    for (int k = 0; k < 10; ++k) stats[16 * i + 4 + k] = cnt[(size_t)i * kCounters + 6 + k] / 100;
    stats[16 * i + 14] = stats[16 * i + 15] = 0;
  }
  return SPINDLE_OK;
}

namespace {
enum { kPhaseGraph = 1, kPhaseCodebook = 2 };

// The whole call or one of its halves; the arguments are those of spindle_compress_shallow.
spindle_status run_shallow(int phases,
    const spindle_kv_desc *desc, const void *K, const void *V, float theta_k, float theta_v,
    int32_t max_codes, void *Ck, void *Cv, int32_t *n_codes_k, int32_t *n_codes_v, int32_t *n_found_k,
    int32_t *n_found_v, int32_t *ref_k, int32_t *ref_v, float *mag_k, float *mag_v, uint32_t *adj_k,
    uint32_t *adj_v, int32_t *deg_k, int32_t *deg_v, void *workspace, size_t workspace_bytes,
    void *stream) {
  const int T = (K ? 1 : 0) + (V ? 1 : 0);
  if (T == 0) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "at least one of K, V is required");
  size_t need = 0;
  spindle_status s = spindle_shallow_workspace_bytes(desc, T, &need);
  if (s != SPINDLE_OK) return s;
  if (max_codes < 1) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "max_codes must be >= 1");
  if (K && (!Ck || !n_codes_k || !ref_k || !mag_k)) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "K given but one of Ck, n_codes_k, ref_k, mag_k is NULL");
  if (V && (!Cv || !n_codes_v || !ref_v || !mag_v)) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "V given but one of Cv, n_codes_v, ref_v, mag_v is NULL");
  if (!(theta_k == theta_k) || !(theta_v == theta_v)) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "thresholds must not be NaN");
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255))
    SPINDLE_FAIL(SPINDLE_ERR_WORKSPACE, "workspace needs %zu bytes, 256-byte aligned (got %zu)", need, workspace_bytes);
  const uintptr_t al = reinterpret_cast<uintptr_t>(K) | reinterpret_cast<uintptr_t>(V) |
                       reinterpret_cast<uintptr_t>(Ck) | reinterpret_cast<uintptr_t>(Cv);
  if (al & 15) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");

  hipStream_t st = static_cast<hipStream_t>(stream);
  const int U = desc->batch * desc->n_kv_heads, n = desc->seq_len;
  ShallowParams p;
  memset(&p, 0, sizeof(p));
  p.dtype = desc->dtype; p.U = U; p.UT = U * T; p.n = n;
  s = kv_layout(desc, &p.lay);
  if (s != SPINDLE_OK) return s;
  p.cap = max_codes;
  carve(p, workspace, p.UT, n);
  int t = 0;
  uint32_t *adj[2] = {nullptr, nullptr};
  if (K) {
    p.X[t] = static_cast<const char *>(K); p.theta[t] = theta_k; p.C[t] = static_cast<char *>(Ck);
    p.n_codes[t] = n_codes_k; p.n_found[t] = n_found_k; p.ref[t] = ref_k; p.mag[t] = mag_k;
    adj[t] = adj_k; p.deg_out[t] = deg_k; ++t;
  }
  if (V) {
    p.X[t] = static_cast<const char *>(V); p.theta[t] = theta_v; p.C[t] = static_cast<char *>(Cv);
    p.n_codes[t] = n_codes_v; p.n_found[t] = n_found_v; p.ref[t] = ref_v; p.mag[t] = mag_v;
    adj[t] = adj_v; p.deg_out[t] = deg_v; ++t;
  }
  if (phases & kPhaseGraph) {
    // zero: counters, list counts, error flag, barriers; codebooks
    const size_t nzero = zero_words(p.UT, n);
    const size_t cwords = (size_t)U * max_codes * kHeadDim * dtype_bytes(p.dtype) / 4;
    hipLaunchKernelGGL(shallow_init, dim3(1024), dim3(256), 0, st, p, nzero, cwords, T);
    if ((s = launch_graph(p, st, adj[0] || adj[1])) != SPINDLE_OK) return s;
    const int W = (n + 31) / 32;                      // nothing after this point changes G
    for (int i = 0; i < T; ++i) {
      if (adj[i])
        hipLaunchKernelGGL(export_adj, dim3(1024), dim3(256), 0, st, p.G + (size_t)i * U * n * p.Wp, adj[i],
                           (size_t)U * n, p.Wp, W);
    }
  }
  if (phases & kPhaseCodebook) {
    if ((s = launch_merge(p, st)) != SPINDLE_OK) return s;
    if ((s = launch_codebook(p, st)) != SPINDLE_OK) return s;
  }
  SPINDLE_HIP(hipGetLastError());
  return SPINDLE_OK;
}
}  // namespace

#define SHALLOW_ARGS                                                                                    \
  desc, K, V, theta_k, theta_v, max_codes, Ck, Cv, n_codes_k, n_codes_v, n_found_k, n_found_v, ref_k,   \
  ref_v, mag_k, mag_v, adj_k, adj_v, deg_k, deg_v, workspace, workspace_bytes, stream

extern "C" spindle_status spindle_compress_shallow(
    const spindle_kv_desc *desc, const void *K, const void *V, float theta_k, float theta_v,
    int32_t max_codes, void *Ck, void *Cv, int32_t *n_codes_k, int32_t *n_codes_v, int32_t *n_found_k,
    int32_t *n_found_v, int32_t *ref_k, int32_t *ref_v, float *mag_k, float *mag_v, uint32_t *adj_k,
    uint32_t *adj_v, int32_t *deg_k, int32_t *deg_v, void *workspace, size_t workspace_bytes,
    void *stream) {
  return run_shallow(kPhaseGraph | kPhaseCodebook, SHALLOW_ARGS);
}

extern "C" spindle_status spindle_shallow_graph(
    const spindle_kv_desc *desc, const void *K, const void *V, float theta_k, float theta_v,
    int32_t max_codes, void *Ck, void *Cv, int32_t *n_codes_k, int32_t *n_codes_v, int32_t *n_found_k,
    int32_t *n_found_v, int32_t *ref_k, int32_t *ref_v, float *mag_k, float *mag_v, uint32_t *adj_k,
    uint32_t *adj_v, int32_t *deg_k, int32_t *deg_v, void *workspace, size_t workspace_bytes,
    void *stream) {
  return run_shallow(kPhaseGraph, SHALLOW_ARGS);
}

extern "C" spindle_status spindle_shallow_codebook(
    const spindle_kv_desc *desc, const void *K, const void *V, float theta_k, float theta_v,
    int32_t max_codes, void *Ck, void *Cv, int32_t *n_codes_k, int32_t *n_codes_v, int32_t *n_found_k,
    int32_t *n_found_v, int32_t *ref_k, int32_t *ref_v, float *mag_k, float *mag_v, uint32_t *adj_k,
    uint32_t *adj_v, int32_t *deg_k, int32_t *deg_v, void *workspace, size_t workspace_bytes,
    void *stream) {
  return run_shallow(kPhaseCodebook, SHALLOW_ARGS);
}

// ---------------------------------------------------------------- one codebook per layer
namespace {

// The rows of all KV heads of a batch entry as one problem: [B, h_g, l, d] with the heads one
// behind the other in memory is [B, 1, h_g * l, d].
spindle_status layer_desc(const spindle_kv_desc *desc, spindle_kv_desc *one) {
  spindle_status s = check_desc(desc);
  if (s != SPINDLE_OK) return s;
  const int64_t rows = (int64_t)desc->n_kv_heads * desc->seq_len;
  if (rows > 65535)
    SPINDLE_FAIL(SPINDLE_ERR_UNSUPPORTED,
                 "one codebook over all heads of a layer is a problem of n_kv_heads x seq_len = %lld rows; the codebook "
                 "path takes at most 65535 (token indices are 16 bits wide): evict to fewer rows per head first",
                 (long long)rows);
  const int64_t st = desc->stride_t ? desc->stride_t : desc->head_dim;
  const int64_t sh = desc->stride_h ? desc->stride_h : (int64_t)desc->seq_len * desc->head_dim;
  if (sh != (int64_t)desc->seq_len * st)
    SPINDLE_FAIL(SPINDLE_ERR_UNSUPPORTED, "the heads of a batch entry must follow each other in memory "
                 "(stride_h = seq_len * stride_t), as the outputs of spindle_compress_deep do");
  *one = *desc;
  one->n_kv_heads = 1;
  one->seq_len = (int32_t)rows;
  one->stride_h = 0;
  one->stride_b = desc->stride_b ? desc->stride_b : (int64_t)desc->n_kv_heads * sh;
  one->stride_t = desc->stride_t;
  return SPINDLE_OK;
}

}  // namespace

extern "C" spindle_status spindle_shallow_layer_workspace_bytes(const spindle_kv_desc *desc, int32_t n_tensors,
                                                                size_t *bytes) {
  spindle_kv_desc one;
  spindle_status s = layer_desc(desc, &one);
  if (s != SPINDLE_OK) return s;
  return spindle_shallow_workspace_bytes(&one, n_tensors, bytes);
}

extern "C" spindle_status spindle_compress_shallow_layer(
    const spindle_kv_desc *desc, const void *K, const void *V, float theta_k, float theta_v,
    int32_t max_codes, void *Ck, void *Cv, int32_t *n_codes_k, int32_t *n_codes_v, int32_t *n_found_k,
    int32_t *n_found_v, int32_t *ref_k, int32_t *ref_v, float *mag_k, float *mag_v, void *workspace,
    size_t workspace_bytes, void *stream) {
  spindle_kv_desc one;
  spindle_status s = layer_desc(desc, &one);
  if (s != SPINDLE_OK) return s;
  return run_shallow(kPhaseGraph | kPhaseCodebook, &one, K, V, theta_k, theta_v, max_codes, Ck, Cv, n_codes_k, n_codes_v,
                     n_found_k, n_found_v, ref_k, ref_v, mag_k, mag_v, nullptr, nullptr, nullptr, nullptr, workspace,
                     workspace_bytes, stream);
}

// ---------------------------------------------------------------- measurement aid
extern "C" spindle_status spindle_calibrate_similarity(const spindle_kv_desc *desc, int32_t n_tensors, void *workspace,
                                                       size_t workspace_bytes, int32_t mode, void *stream, double *ms_out) {
  size_t need = 0;
  spindle_status s = spindle_shallow_workspace_bytes(desc, n_tensors, &need);
  if (s != SPINDLE_OK) return s;
  if (!ms_out || mode < 0 || mode > 2) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "ms is NULL or mode is not 0, 1 or 2");
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255))
    SPINDLE_FAIL(SPINDLE_ERR_WORKSPACE, "workspace needs %zu bytes, 256-byte aligned (got %zu)", need, workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(stream);
  ShallowParams p;
  memset(&p, 0, sizeof(p));
  p.dtype = desc->dtype; p.U = desc->batch * desc->n_kv_heads; p.UT = p.U * n_tensors; p.n = desc->seq_len;
  if ((s = kv_layout(desc, &p.lay)) != SPINDLE_OK) return s;
  p.theta[0] = p.theta[1] = 0.98f;
  carve(p, workspace, p.UT, p.n);
  hipEvent_t e0, e1;
  SPINDLE_HIP(hipEventCreate(&e0));
  SPINDLE_HIP(hipEventCreate(&e1));
  SPINDLE_HIP(hipEventRecord(e0, st));
  s = launch_bare_similarity(p, st, mode);
  if (s == SPINDLE_OK) {
    SPINDLE_HIP(hipEventRecord(e1, st));
    SPINDLE_HIP(hipEventSynchronize(e1));
    float ms = 0.f;
    SPINDLE_HIP(hipEventElapsedTime(&ms, e0, e1));
    *ms_out = ms;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return s;
}
