// Decode-time merge (Sec. "Similarity Based Token Replacement", the paragraph after Eq. 14):
// tokens generated after the prefill first look for a stored codebook entry within theta;
// those that find none get entries of their own by the construction of Alg. 1, appended to
// the codebook.
//
// Kernels, enqueued on the caller's stream; u indexes one (batch, kv-head) problem of m new tokens:
//   decode_prep    magnitudes (Eq. 8) and the new tokens as doubles
//   decode_match   per new token and slice of 512 stored entries, the entry of highest cosine
//                  (Eq. 4) if it exceeds theta, lowest index on ties; everything in double
//                  precision with the dimension-order sums the adjacency decision is defined by
//   decode_build   one workgroup per problem: the unmatched tokens' adjacency matrix (Eq. 9) in
//                  LDS, the greedy highest-degree loop (Eq. 10-13) as stated, new entries and
//                  references
//   decode_small   all of it in one launch when a call brings at most four tokens per problem
#include <math.h>

#include <mutex>

#include "common.h"

// Scratch memory of spindle_decode_merge_static: lives in the code object, one copy per GPU
// the library is loaded on, for the life of the process.  In host code this name is only a
// handle for hipGetSymbolAddress; the address kernels get is looked up per device below.
constexpr size_t kStaticScratchBytes = (size_t)6 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace spindle {
namespace {

constexpr int kDecodeMax = 1024;     // new tokens per problem and call
constexpr int kMatchTokens = 16;     // new tokens per workgroup of decode_match
constexpr int kMatchThreads = 256;
constexpr int kLaneEntries = 2;      // stored entries per lane of decode_match
constexpr int kSliceEntries = kMatchThreads * kLaneEntries;
constexpr int kBuildThreads = 1024;

struct DecodeParams {
  const char *X;        // [U][m][128] new tokens in `dtype`
  char *C;              // [U][cap][128] codebook in `dtype`, rows < n_codes[u] valid, appended to
  int32_t *n_codes;     // [U] in: stored entries, out: stored entries afterwards
  int32_t *n_found;     // [U] entries needed (stored + new picks), may exceed cap
  int32_t *n_matched;   // [U] optional: tokens merged with an existing entry
  int32_t *ref;         // [U][m]
  float *mag;           // [U][m]
  double *m64;          // workspace [U][m]
  double *Xd;           // workspace [U][tiles][128][16] the new tokens as doubles
  double *part_v;       // workspace [U][tiles][slices][16] best cosine of a token within a slice of entries
  int *part_i;          //           and its entry, -1 if none exceeds theta
  int dtype, U, m, cap;
  int tiles, slices;    // ceil(m / 16), ceil(cap / 512)
  double theta;
};

template <int DT>
__device__ __forceinline__ const char *token_row(const DecodeParams &p, int u, int a) {
  return p.X + ((size_t)u * p.m + a) * (kHeadDim * sizeof(typename Elem<DT>::type));
}

// (value, index) maximum with the lower index winning ties
__device__ __forceinline__ void take_better(double &bv, int &bi, double ov, int oi) {
  if (oi >= 0 && (bi < 0 || ov > bv || (ov == bv && oi < bi))) {
    bv = ov;
    bi = oi;
  }
}

// Double-precision copies of the new tokens, laid out for decode_match: [u][tile of 16 tokens]
// [dimension][token in tile], tokens past m as zeros; magnitudes (Eq. 8, dimension-order sum).
template <int DT>
__global__ __launch_bounds__(kMatchThreads) void decode_prep(DecodeParams p) {
  typedef typename Elem<DT>::type T;
  __shared__ double xs[kHeadDim][kMatchTokens + 1];
  const int u = blockIdx.y, tile = blockIdx.x, a0 = tile * kMatchTokens, tid = threadIdx.x;
  for (int i = tid; i < kMatchTokens * kHeadDim; i += kMatchThreads) {
    const int tok = i / kHeadDim, dim = i % kHeadDim;
    double v = 0.0;
    if (a0 + tok < p.m) v = (double)Elem<DT>::to_float(reinterpret_cast<const T *>(token_row<DT>(p, u, a0 + tok))[dim]);
    xs[dim][tok] = v;
  }
  __syncthreads();
  double *dst = p.Xd + ((size_t)u * p.tiles + tile) * (kHeadDim * kMatchTokens);
  for (int i = tid; i < kMatchTokens * kHeadDim; i += kMatchThreads) dst[i] = xs[i / kMatchTokens][i % kMatchTokens];
  if (tid < kMatchTokens && a0 + tid < p.m) {
    double ss = 0.0;
    for (int dim = 0; dim < kHeadDim; ++dim) ss += xs[dim][tid] * xs[dim][tid];
    const double mg = sqrt(ss);
    p.m64[(size_t)u * p.m + a0 + tid] = mg;
    p.mag[(size_t)u * p.m + a0 + tid] = (float)mg;
  }
}

// One workgroup = 16 new tokens x 512 stored entries, two entries per thread.  The tokens'
// values are the same for every lane, so they are read through uniform loads (scalar
// registers) and each lane streams its own entry row: per dimension 16 fused multiply-adds
// against two conversions and one load per eight dimensions.  Every (token, entry) sum runs
// over the dimensions in order, as the decision is defined.  The best entry of each token
// within the slice goes to the workspace; decode_build combines the slices.
template <int DT>
__global__ __launch_bounds__(kMatchThreads) void decode_match(DecodeParams p, const double *__restrict__ Xd,
                                                             const double *__restrict__ m64) {
  typedef typename Elem<DT>::type T;
  constexpr int per = 16 / sizeof(T);              // elements per 16-byte piece
  constexpr int pieces = kHeadDim / per;
  __shared__ double red_v[kMatchThreads / kWave][kMatchTokens];
  __shared__ int red_i[kMatchThreads / kWave][kMatchTokens];
  const int u = blockIdx.y, tile = blockIdx.x % p.tiles, slice = blockIdx.x / p.tiles, tid = threadIdx.x;
  int nc = p.n_codes[u];
  nc = nc < 0 ? 0 : (nc > p.cap ? p.cap : nc);
  if (slice * kSliceEntries >= nc) return;          // decode_build only reads the slices below nc
  const int a0 = tile * kMatchTokens;
  const double *xt = Xd + ((size_t)u * p.tiles + tile) * (kHeadDim * kMatchTokens);

  double best[kMatchTokens];
  int bidx[kMatchTokens];
  {
    int c[kLaneEntries];
    const u4 *row[kLaneEntries];
    double acc[kLaneEntries][kMatchTokens], css[kLaneEntries];
#pragma unroll
    for (int e = 0; e < kLaneEntries; ++e) {
      c[e] = slice * kSliceEntries + e * kMatchThreads + tid;
      const int cr = c[e] < nc ? c[e] : nc - 1;     // lanes past the last entry recompute it and drop the result
      row[e] = reinterpret_cast<const u4 *>(p.C + ((size_t)u * p.cap + cr) * (kHeadDim * sizeof(T)));
      css[e] = 0.0;
#pragma unroll
      for (int t = 0; t < kMatchTokens; ++t) acc[e][t] = 0.0;
    }
    for (int pc = 0; pc < pieces; ++pc) {
      u4 v[kLaneEntries];
#pragma unroll
      for (int e = 0; e < kLaneEntries; ++e) v[e] = row[e][pc];
#pragma unroll
      for (int j = 0; j < per; ++j) {
        const double *xr = xt + (pc * per + j) * kMatchTokens;
#pragma unroll
        for (int e = 0; e < kLaneEntries; ++e) {
          const double y = (double)Elem<DT>::to_float(reinterpret_cast<const T *>(&v[e])[j]);
          css[e] += y * y;
#pragma unroll
          for (int t = 0; t < kMatchTokens; ++t) acc[e][t] += xr[t] * y;
        }
      }
    }
#pragma unroll
    for (int t = 0; t < kMatchTokens; ++t) {
      best[t] = 0.0;
      bidx[t] = -1;
    }
    // Few (token, entry) pairs come near theta, and a double-precision division costs as much as
    // twenty multiply-adds: the quotient is only formed where the dot product is not already
    // clearly below theta times the norms (for theta >= 0; a quotient that close to theta from
    // below cannot round up past it).
    const double low = p.theta >= 0.0 ? p.theta * (1.0 - 1e-12) : -INFINITY;
#pragma unroll
    for (int e = 0; e < kLaneEntries; ++e) {        // ascending entry index: the first of equal values stays
      const double cn = sqrt(css[e]);
#pragma unroll
      for (int t = 0; t < kMatchTokens; ++t) {
        const double ma = a0 + t < p.m ? m64[(size_t)u * p.m + a0 + t] : 0.0;
        const double den = ma * cn;
        if (c[e] < nc && (!(den > 0.0) || acc[e][t] > low * den)) {
          const double cs = den > 0.0 ? acc[e][t] / den : 0.0;
          if (cs > p.theta) take_better(best[t], bidx[t], cs, c[e]);
        }
      }
    }
  }
  const int lane = lane_id(), wave = tid >> 6;
#pragma unroll
  for (int t = 0; t < kMatchTokens; ++t) {
    double bv = best[t];
    int bi = bidx[t];
    if (__ballot(bi >= 0) != 0) {                    // wave-uniform: most tokens find nothing in most slices
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const double ov = __shfl_xor(bv, o);
        const int oi = __shfl_xor(bi, o);
        take_better(bv, bi, ov, oi);
      }
    }
    if (lane == 0) {
      red_v[wave][t] = bv;
      red_i[wave][t] = bi;
    }
  }
  __syncthreads();
  if (tid < kMatchTokens) {
    double bv = red_v[0][tid];
    int bi = red_i[0][tid];
    for (int w = 1; w < kMatchThreads / kWave; ++w) take_better(bv, bi, red_v[w][tid], red_i[w][tid]);
    const size_t at = (((size_t)u * p.tiles + tile) * p.slices + slice) * kMatchTokens + tid;
    p.part_v[at] = bv;
    p.part_i[at] = bi;
  }
}

// LDS of decode_build, in 32-bit words, for m new tokens: one token as doubles per wave, the
// adjacency rows with an odd pitch (thread i walks row i: consecutive rows must start in
// different banks), two bitmaps, then four 16-bit arrays (position in the input, degree, pick
// number per token; the pick list).  160,000 bytes at m = 1024.
__host__ __device__ inline int build_pitch(int m) { return ((m + 31) / 32) | 1; }
__host__ __device__ inline size_t build_lds_words(int m) {
  return 2 * kHeadDim * (kBuildThreads / kWave) + (size_t)m * build_pitch(m) + 2 * (size_t)((m + 31) / 32) +
         2 * (size_t)((m + 1) & ~1);
}

template <int DT>
__global__ __launch_bounds__(kBuildThreads) void decode_build(DecodeParams p) {
  typedef typename Elem<DT>::type T;
  constexpr int per = 16 / sizeof(T);
  constexpr int pieces = kHeadDim / per;
  constexpr int kWaves = kBuildThreads / kWave;
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  __shared__ int wave_sum[kWaves];
  __shared__ uint32_t wave_key[kWaves];
  __shared__ int sh_r;
  const int u = blockIdx.x, m = p.m, tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
  const int Wd = (m + 31) / 32, pitch = build_pitch(m);
  double *xi = reinterpret_cast<double *>(lds) + (size_t)wave * kHeadDim;   // one token per wave
  uint32_t *adj = lds + 2 * kHeadDim * kWaves;       // [m][pitch]
  uint32_t *alive = adj + (size_t)m * pitch;         // [Wd]
  uint32_t *dying = alive + Wd;                      // [Wd]
  const int m2 = (m + 1) & ~1;
  uint16_t *rest = reinterpret_cast<uint16_t *>(dying + Wd);   // unmatched tokens, input order
  uint16_t *deg = rest + m2;
  uint16_t *rref = deg + m2;                         // pick number of each unmatched token
  uint16_t *picks = rref + m2;                       // unmatched-token index of each pick
  int nc = p.n_codes[u];
  nc = nc < 0 ? 0 : (nc > p.cap ? p.cap : nc);
  int32_t *ref = p.ref + (size_t)u * m;
  const double *m64 = p.m64 + (size_t)u * m;

  // best stored entry of each token over the slices (ascending, so ties stay with the lower
  // index), then the unmatched tokens in input order
  {
    int mine = -1;
    if (tid < m) {
      const int used = (nc + kSliceEntries - 1) / kSliceEntries;
      const size_t at = (((size_t)u * p.tiles + tid / kMatchTokens) * p.slices) * kMatchTokens + tid % kMatchTokens;
      double bv = 0.0;
      for (int sl = 0; sl < used; ++sl) take_better(bv, mine, p.part_v[at + (size_t)sl * kMatchTokens], p.part_i[at + (size_t)sl * kMatchTokens]);
      ref[tid] = mine;
    }
    const bool un = tid < m && mine < 0;
    const unsigned long long mk = __ballot(un);
    if (lane == 0) wave_sum[wave] = __popcll(mk);
    __syncthreads();
    int before = 0, total = 0;
    for (int w = 0; w < kWaves; ++w) {
      before += w < wave ? wave_sum[w] : 0;
      total += wave_sum[w];
    }
    if (un) rest[before + __popcll(mk & ((1ull << lane) - 1ull))] = (uint16_t)tid;
    if (tid == 0) sh_r = total;
  }
  for (int i = tid; i < m * pitch; i += kBuildThreads) adj[i] = 0u;
  __syncthreads();
  const int r = sh_r;
  if (tid == 0 && p.n_matched) p.n_matched[u] = m - r;

  // Eq. 9 among the unmatched tokens: each unordered pair once, both bits set
  for (int i = wave; i < r; i += kWaves) {
    const T *src = reinterpret_cast<const T *>(token_row<DT>(p, u, rest[i]));
    xi[lane] = (double)Elem<DT>::to_float(src[lane]);
    xi[lane + 64] = (double)Elem<DT>::to_float(src[lane + 64]);
    const double mi = m64[rest[i]];
    if (lane == 0) atomicOr(&adj[(size_t)i * pitch + (i >> 5)], 1u << (i & 31));     // G_aa = 1
    __builtin_amdgcn_wave_barrier();
    for (int j0 = i + 1; j0 < r; j0 += kWave) {
      const int j = j0 + lane;
      if (j < r) {
        const u4 *row = reinterpret_cast<const u4 *>(token_row<DT>(p, u, rest[j]));
        double acc = 0.0;
        for (int pc = 0; pc < pieces; ++pc) {
          const u4 v = row[pc];
          const T *e = reinterpret_cast<const T *>(&v);
#pragma unroll
          for (int k = 0; k < per; ++k) acc += xi[pc * per + k] * (double)Elem<DT>::to_float(e[k]);
        }
        const double den = mi * m64[rest[j]];
        const double cs = den > 0.0 ? acc / den : 0.0;
        if (cs > p.theta) {
          atomicOr(&adj[(size_t)i * pitch + (j >> 5)], 1u << (j & 31));
          atomicOr(&adj[(size_t)j * pitch + (i >> 5)], 1u << (i & 31));
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
  for (int w = tid; w < Wd; w += kBuildThreads) {
    const int lo = w * 32;
    alive[w] = r >= lo + 32 ? 0xFFFFFFFFu : (r > lo ? (1u << (r - lo)) - 1u : 0u);
  }
  __syncthreads();
  if (tid < r) {                                     // Eq. 10
    int d = 0;
    for (int w = 0; w < Wd; ++w) d += __popc(adj[(size_t)tid * pitch + w]);
    deg[tid] = (uint16_t)d;
  }
  __syncthreads();

  // Alg. 1: take the remaining token of highest degree (lowest index on ties), give its
  // remaining neighbourhood its entry, remove it, lower the degrees of the others (Eq. 11-13)
  int npicks = 0;
  for (;;) {
    const bool live = tid < r && ((alive[tid >> 5] >> (tid & 31)) & 1u);
    uint32_t key = live ? ((uint32_t)deg[tid] << 16) | (uint32_t)(0xFFFF - tid) : 0u;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const uint32_t ok = __shfl_xor(key, o);
      key = ok > key ? ok : key;
    }
    if (lane == 0) wave_key[wave] = key;
    __syncthreads();
    uint32_t top = 0;
    for (int w = 0; w < kWaves; ++w) top = wave_key[w] > top ? wave_key[w] : top;
    if (top == 0u) break;                            // nobody left
    if ((top >> 16) == 1u) {
      // only isolated tokens are left: each is its own entry, in index order
      if (live) {
        int before = 0;
        for (int w = 0; w < (tid >> 5); ++w) before += __popc(alive[w]);
        before += __popc(alive[tid >> 5] & ((1u << (tid & 31)) - 1u));
        rref[tid] = (uint16_t)(npicks + before);
        picks[npicks + before] = (uint16_t)tid;
      }
      int total = 0;
      for (int w = 0; w < Wd; ++w) total += __popc(alive[w]);
      npicks += total;
      break;
    }
    const int v = 0xFFFF - (int)(top & 0xFFFFu);
    if (tid < Wd) dying[tid] = adj[(size_t)v * pitch + tid] & alive[tid];
    if (tid == 0) picks[npicks] = (uint16_t)v;
    __syncthreads();
    if (live) {
      if ((dying[tid >> 5] >> (tid & 31)) & 1u) {
        rref[tid] = (uint16_t)npicks;                // Eq. 12
      } else {
        int gone = 0;
        for (int w = 0; w < Wd; ++w) {
          const uint32_t dw = dying[w];
          if (dw) gone += __popc(adj[(size_t)tid * pitch + w] & dw);
        }
        deg[tid] = (uint16_t)(deg[tid] - gone);      // Eq. 13, as a degree update
      }
    }
    __syncthreads();
    if (tid < Wd) alive[tid] &= ~dying[tid];
    ++npicks;
    __syncthreads();
  }
  __syncthreads();

  // outputs: references of the unmatched tokens, the new rows, the counts
  const int room = p.cap - nc > 0 ? p.cap - nc : 0;
  const int stored = npicks < room ? npicks : room;
  if (tid < r) ref[rest[tid]] = (int)rref[tid] < room ? nc + (int)rref[tid] : -1;
  T *Cu = reinterpret_cast<T *>(p.C) + (size_t)u * p.cap * kHeadDim;
  for (int j = wave; j < stored; j += kWaves) {
    const int tok = rest[picks[j]];
    const T *src = reinterpret_cast<const T *>(token_row<DT>(p, u, tok));
    const double mg = m64[tok];
    for (int d = lane; d < kHeadDim; d += kWave) {
      const double x = (double)Elem<DT>::to_float(src[d]);
      Cu[(size_t)(nc + j) * kHeadDim + d] = Elem<DT>::from_float(mg > 0.0 ? (float)(x / mg) : 0.f);
    }
  }
  if (tid == 0) {
    p.n_found[u] = nc + npicks;
    p.n_codes[u] = nc + stored;
  }
}

// The usual decode step brings one token per head (a few with speculative decoding): then
// three launches cost more than the work.  One workgroup per problem does it all: the tokens
// as doubles in LDS, every thread a few stored entries (same sums, same decision as
// decode_match), a reduction over the workgroup, and Alg. 1 on the at most MT unmatched
// tokens by the first wave (adjacency in one word per token, the loop as stated).
constexpr int kSmallThreads = 1024;

template <int DT, int MT>
__global__ __launch_bounds__(kSmallThreads) void decode_small(DecodeParams p) {
  typedef typename Elem<DT>::type T;
  constexpr int per = 16 / sizeof(T), pieces = kHeadDim / per, kWaves = kSmallThreads / kWave;
  __shared__ __attribute__((aligned(16))) double xs[kHeadDim][MT];
  __shared__ double ms[MT];
  __shared__ double red_v[kWaves][MT];
  __shared__ int red_i[kWaves][MT];
  __shared__ int ref_s[MT];
  __shared__ uint32_t adjm[MT];
  const int u = blockIdx.x, tid = threadIdx.x, lane = lane_id(), wave = tid >> 6, m = p.m;
  int nc = p.n_codes[u];
  nc = nc < 0 ? 0 : (nc > p.cap ? p.cap : nc);
  for (int i = tid; i < MT * kHeadDim; i += kSmallThreads) {
    const int tok = i / kHeadDim, dim = i % kHeadDim;
    xs[dim][tok] = tok < m ? (double)Elem<DT>::to_float(reinterpret_cast<const T *>(token_row<DT>(p, u, tok))[dim]) : 0.0;
  }
  __syncthreads();
  if (tid < MT) {
    double ss = 0.0;
    for (int dim = 0; dim < kHeadDim; ++dim) ss += xs[dim][tid] * xs[dim][tid];
    const double mg = sqrt(ss);
    ms[tid] = mg;
    if (tid < m) p.mag[(size_t)u * m + tid] = (float)mg;
  }
  __syncthreads();

  double best[MT];
  int bidx[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    best[t] = 0.0;
    bidx[t] = -1;
  }
  const double low = p.theta >= 0.0 ? p.theta * (1.0 - 1e-12) : -INFINITY;   // see decode_match
  for (int c = tid; c < nc; c += kSmallThreads) {   // ascending: the first of equal values stays
    const u4 *row = reinterpret_cast<const u4 *>(p.C + ((size_t)u * p.cap + c) * (kHeadDim * sizeof(T)));
    double acc[MT], css = 0.0;
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = 0.0;
    for (int pc = 0; pc < pieces; ++pc) {
      const u4 v = row[pc];
#pragma unroll
      for (int j = 0; j < per; ++j) {
        const double y = (double)Elem<DT>::to_float(reinterpret_cast<const T *>(&v)[j]);
        css += y * y;
#pragma unroll
        for (int t = 0; t < MT; ++t) acc[t] += xs[pc * per + j][t] * y;
      }
    }
    const double cn = sqrt(css);
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const double den = ms[t] * cn;
      if (t < m && (!(den > 0.0) || acc[t] > low * den)) {
        const double cs = den > 0.0 ? acc[t] / den : 0.0;
        if (cs > p.theta) take_better(best[t], bidx[t], cs, c);
      }
    }
  }
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    double bv = best[t];
    int bi = bidx[t];
    if (__ballot(bi >= 0) != 0) {
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const double ov = __shfl_xor(bv, o);
        const int oi = __shfl_xor(bi, o);
        take_better(bv, bi, ov, oi);
      }
    }
    if (lane == 0) {
      red_v[wave][t] = bv;
      red_i[wave][t] = bi;
    }
  }
  __syncthreads();
  if (tid < MT) {
    double bv = red_v[0][tid];
    int bi = red_i[0][tid];
    for (int w = 1; w < kWaves; ++w) take_better(bv, bi, red_v[w][tid], red_i[w][tid]);
    ref_s[tid] = tid < m ? bi : 0;                   // slots past m count as matched
    adjm[tid] = 0u;
  }
  __syncthreads();
  if (wave != 0) return;

  // the unmatched tokens, in input order, among themselves (Eq. 9-13)
  const bool un = lane < m && ref_s[lane < MT ? lane : 0] < 0;
  const unsigned long long mask = __ballot(un);
  const int r = __popcll(mask);
  int rest[MT];                                      // token of each unmatched position (wave-uniform)
  {
    unsigned long long left = mask;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      rest[i] = left ? __builtin_ctzll(left) : 0;
      left &= left - 1;
    }
  }
  for (int pair = lane; pair < MT * MT; pair += kWave) {
    const int i = pair / MT, j = pair % MT;
    if (i < j && j < r) {
      const int a = rest[i], b = rest[j];
      double acc = 0.0;
      for (int dim = 0; dim < kHeadDim; ++dim) acc += xs[dim][a] * xs[dim][b];
      const double den = ms[a] * ms[b];
      const double cs = den > 0.0 ? acc / den : 0.0;
      if (cs > p.theta) {
        atomicOr(&adjm[i], 1u << j);
        atomicOr(&adjm[j], 1u << i);
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0);
  __builtin_amdgcn_wave_barrier();
  int rref[MT], picks[MT];
  int npicks = 0;
  {
    uint32_t alive = r >= 32 ? 0xFFFFFFFFu : (1u << r) - 1u;
    uint32_t rows[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      rows[i] = adjm[i] | (1u << i);                 // G_aa = 1
      rref[i] = 0;
      picks[i] = 0;
    }
    while (alive) {                                  // every lane runs the same tiny loop
      int pick = 0, top = 0;
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int d = (alive >> i) & 1u ? __popc(rows[i] & alive) : 0;
        if (d > top) { top = d; pick = i; }          // strict: lowest index on ties
      }
      uint32_t leaving = 0;
#pragma unroll
      for (int i = 0; i < MT; ++i)
        if (i == pick) leaving = rows[i] & alive;
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        if ((leaving >> i) & 1u) rref[i] = npicks;
        if (i == npicks) picks[i] = pick;
      }
      alive &= ~leaving;
      ++npicks;
    }
  }
  const int room = p.cap - nc > 0 ? p.cap - nc : 0;
  const int stored = npicks < room ? npicks : room;
  if (lane < m) {
    int out = ref_s[lane < MT ? lane : 0];
    if (out < 0) {
      const int pos = __popcll(mask & ((1ull << lane) - 1ull));
      int rr = 0;
#pragma unroll
      for (int i = 0; i < MT; ++i)
        if (i == pos) rr = rref[i];
      out = rr < room ? nc + rr : -1;
    }
    p.ref[(size_t)u * m + lane] = out;
  }
  T *Cu = reinterpret_cast<T *>(p.C) + (size_t)u * p.cap * kHeadDim;
#pragma unroll
  for (int j = 0; j < MT; ++j) {
    if (j < stored) {
      int tok = 0;
#pragma unroll
      for (int i = 0; i < MT; ++i)
        if (i == picks[j]) tok = rest[i];
      const double mg = ms[tok];
      for (int d = lane; d < kHeadDim; d += kWave)
        Cu[(size_t)(nc + j) * kHeadDim + d] = Elem<DT>::from_float(mg > 0.0 ? (float)(xs[d][tok] / mg) : 0.f);
    }
  }
  if (lane == 0) {
    p.n_found[u] = nc + npicks;
    p.n_codes[u] = nc + stored;
    if (p.n_matched) p.n_matched[u] = m - r;
  }
}

spindle_status check_decode(const spindle_kv_desc *desc) {
  spindle_status s = check_desc(desc);
  if (s != SPINDLE_OK) return s;
  if (desc->stride_b || desc->stride_h || desc->stride_t)
    SPINDLE_FAIL(SPINDLE_ERR_UNSUPPORTED, "the new tokens of a decode step are contiguous: strides must be 0");
  if (desc->seq_len > kDecodeMax)
    SPINDLE_FAIL(SPINDLE_ERR_UNSUPPORTED, "at most %d new tokens per call, got %d", kDecodeMax, desc->seq_len);
  return SPINDLE_OK;
}

// Carves the workspace (or only sizes it when `ws` is null).
size_t decode_carve(const spindle_kv_desc *desc, int cap, void *ws, DecodeParams *p) {
  const size_t U = (size_t)desc->batch * desc->n_kv_heads;
  const int tiles = (desc->seq_len + kMatchTokens - 1) / kMatchTokens;
  const int slices = (cap + kSliceEntries - 1) / kSliceEntries;
  Carver cv(ws);
  double *m64 = cv.take<double>(U * desc->seq_len);
  double *Xd = cv.take<double>(U * tiles * kHeadDim * kMatchTokens);
  double *pv = cv.take<double>(U * tiles * slices * kMatchTokens);
  int *pi = cv.take<int>(U * tiles * slices * kMatchTokens);
  if (p) {
    p->m64 = m64;
    p->Xd = Xd;
    p->part_v = pv;
    p->part_i = pi;
    p->tiles = tiles;
    p->slices = slices;
  }
  return cv.total();
}

}  // namespace
}  // namespace spindle

using namespace spindle;

extern "C" spindle_status spindle_decode_workspace_bytes(const spindle_kv_desc *desc, int32_t max_codes, size_t *bytes) {
  if (!bytes) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "bytes is NULL");
  spindle_status s = check_decode(desc);
  if (s != SPINDLE_OK) return s;
  if (max_codes < 1) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "max_codes must be >= 1");
  *bytes = decode_carve(desc, max_codes, nullptr, nullptr);
  return SPINDLE_OK;
}

namespace {

// Validation both entry points share; *need = bytes of scratch memory the call uses.
spindle_status decode_check_args(const spindle_kv_desc *desc, const void *X_new, float theta, int32_t max_codes,
                                 const void *C, const int32_t *n_codes, const int32_t *n_found, const int32_t *ref,
                                 const float *mag, size_t *need) {
  spindle_status s = check_decode(desc);
  if (s != SPINDLE_OK) return s;
  if (max_codes < 1) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "max_codes must be >= 1");
  if (!(theta > -1.f && theta < 1.f)) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "theta must lie in (-1, 1)");
  if (!X_new || !C || !n_codes || !n_found || !ref || !mag)
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "X_new, C, n_codes, n_found, ref and mag are required");
  if ((reinterpret_cast<uintptr_t>(X_new) | reinterpret_cast<uintptr_t>(C)) & 15)
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");
  *need = decode_carve(desc, max_codes, nullptr, nullptr);
  return SPINDLE_OK;
}

// Enqueues the kernels of one merge; `scratch_mem` holds decode_carve's arrays and needs no
// initial content: every element a kernel reads was written by an earlier kernel of the same call.
spindle_status decode_enqueue(const spindle_kv_desc *desc, const void *X_new, float theta, int32_t max_codes,
                              void *C, int32_t *n_codes, int32_t *n_found, int32_t *n_matched, int32_t *ref,
                              float *mag, void *scratch_mem, hipStream_t st) {
  DecodeParams p;
  p.X = static_cast<const char *>(X_new);
  p.C = static_cast<char *>(C);
  p.n_codes = n_codes;
  p.n_found = n_found;
  p.n_matched = n_matched;
  p.ref = ref;
  p.mag = mag;
  decode_carve(desc, max_codes, scratch_mem, &p);
  p.dtype = desc->dtype;
  p.U = desc->batch * desc->n_kv_heads;
  p.m = desc->seq_len;
  p.cap = max_codes;
  p.theta = (double)theta;
  if (p.m <= 4) {
    ProfScope ps("decode_small", st);
#define SPINDLE_DECODE_SMALL(DT) hipLaunchKernelGGL((decode_small<DT, 4>), dim3(p.U), dim3(kSmallThreads), 0, st, p)
    if (p.dtype == SPINDLE_F16) SPINDLE_DECODE_SMALL(SPINDLE_F16);
    else if (p.dtype == SPINDLE_BF16) SPINDLE_DECODE_SMALL(SPINDLE_BF16);
    else SPINDLE_DECODE_SMALL(SPINDLE_F32);
#undef SPINDLE_DECODE_SMALL
    SPINDLE_HIP(hipGetLastError());
    return SPINDLE_OK;
  }
  const dim3 pg(p.tiles, p.U), mg(p.tiles * p.slices, p.U);
  const size_t lds = build_lds_words(p.m) * sizeof(uint32_t);
#define SPINDLE_DECODE_LAUNCH(DT)                                                                          \
  do {                                                                                                     \
    static LdsLimit lim;                                                                                   \
    if (spindle_status e = allow_lds(lim, reinterpret_cast<const void *>(&decode_build<DT>),               \
                                     build_lds_words(kDecodeMax) * sizeof(uint32_t)))                      \
      return e;                                                                                            \
    {                                                                                                      \
      ProfScope ps("decode_prep", st);                                                                     \
      hipLaunchKernelGGL(decode_prep<DT>, pg, dim3(kMatchThreads), 0, st, p);                              \
    }                                                                                                      \
    {                                                                                                      \
      ProfScope ps("decode_match", st);                                                                    \
      hipLaunchKernelGGL(decode_match<DT>, mg, dim3(kMatchThreads), 0, st, p, p.Xd, p.m64);                \
    }                                                                                                      \
    {                                                                                                      \
      ProfScope ps("decode_build", st);                                                                    \
      hipLaunchKernelGGL(decode_build<DT>, dim3(p.U), dim3(kBuildThreads), lds, st, p);                    \
    }                                                                                                      \
  } while (0)
  if (p.dtype == SPINDLE_F16) SPINDLE_DECODE_LAUNCH(SPINDLE_F16);
  else if (p.dtype == SPINDLE_BF16) SPINDLE_DECODE_LAUNCH(SPINDLE_BF16);
  else SPINDLE_DECODE_LAUNCH(SPINDLE_F32);
#undef SPINDLE_DECODE_LAUNCH
  SPINDLE_HIP(hipGetLastError());
  return SPINDLE_OK;
}

}  // namespace

extern "C" spindle_status spindle_decode_merge(const spindle_kv_desc *desc, const void *X_new, float theta,
                                               int32_t max_codes, void *C, int32_t *n_codes, int32_t *n_found,
                                               int32_t *n_matched, int32_t *ref, float *mag, void *workspace,
                                               size_t workspace_bytes, void *stream) {
  size_t need = 0;
  spindle_status s = decode_check_args(desc, X_new, theta, max_codes, C, n_codes, n_found, ref, mag, &need);
  if (s != SPINDLE_OK) return s;
  if (!workspace) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "workspace is required");
  if (reinterpret_cast<uintptr_t>(workspace) & 15) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
  if (workspace_bytes < need) SPINDLE_FAIL(SPINDLE_ERR_WORKSPACE, "workspace too small: %zu < %zu", workspace_bytes, need);
  return decode_enqueue(desc, X_new, theta, max_codes, C, n_codes, n_found, n_matched, ref, mag, workspace,
                        static_cast<hipStream_t>(stream));
}

namespace {

constexpr int kStaticMaxDevices = 64;
std::mutex g_static_mu;
void *g_static_ptr[kStaticMaxDevices] = {};     // device address of `scratch` on each GPU, once looked up

// Device address of `scratch` on the current device (each GPU holds its own copy of the array
// at its own address).
spindle_status static_scratch(void **out) {
  int dev = 0;
  SPINDLE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kStaticMaxDevices) SPINDLE_FAIL(SPINDLE_ERR_UNSUPPORTED, "device %d: at most %d devices", dev, kStaticMaxDevices);
  std::lock_guard<std::mutex> lk(g_static_mu);
  if (!g_static_ptr[dev]) {
    void *ptr = nullptr;
    SPINDLE_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) SPINDLE_FAIL(SPINDLE_ERR_HIP, "hipGetSymbolAddress returned a null address for the scratch array");
    g_static_ptr[dev] = ptr;
  }
  *out = g_static_ptr[dev];
  return SPINDLE_OK;
}

}  // namespace

extern "C" size_t spindle_decode_static_capacity(void) { return kStaticScratchBytes; }

extern "C" spindle_status spindle_decode_merge_static(const spindle_kv_desc *desc, const void *X_new, float theta,
                                                      int32_t max_codes, void *C, int32_t *n_codes, int32_t *n_found,
                                                      int32_t *n_matched, int32_t *ref, float *mag, void *stream) {
  size_t need = 0;
  spindle_status s = decode_check_args(desc, X_new, theta, max_codes, C, n_codes, n_found, ref, mag, &need);
  if (s != SPINDLE_OK) return s;
  if (need > kStaticScratchBytes)
    SPINDLE_FAIL(SPINDLE_ERR_UNSUPPORTED,
                 "this call needs %zu bytes of scratch memory, the built-in buffer holds %zu: fewer new tokens or "
                 "problems per call, a smaller max_codes, or spindle_decode_merge with a workspace",
                 need, kStaticScratchBytes);
  void *mem = nullptr;
  s = static_scratch(&mem);
  if (s != SPINDLE_OK) return s;
  return decode_enqueue(desc, X_new, theta, max_codes, C, n_codes, n_found, n_matched, ref, mag, mem,
                        static_cast<hipStream_t>(stream));
}
