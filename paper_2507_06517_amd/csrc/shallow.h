// Similarity codebook replacement (Sec. "Similarity Based Token Replacement", Alg. 1): what its
// kernels share.  ut = tensor * units + unit indexes one independent (batch, kv-head, K|V)
// problem of n tokens.  The kernels, in the order spindle_compress_shallow enqueues them:
//   shallow_init    counters, flags and outputs that must start from a known value
//   shallow_prep    magnitudes (Eq. 8) in double precision, unit vectors rounded to fp16
//   shallow_gram    cosine similarity tiles by fp16 MFMA, thresholded and bit-packed
//                   into the adjacency matrix G (Eq. 4, 9), upper triangle only; pairs whose
//                   fp16 similarity lies within kGuard of theta are deferred to shallow_fixup
//                   (shallow_gram<true>: in-place fallback when a pair list overflows)
//   shallow_fixup   exact double-precision decision for the deferred pairs;
//                   every set bit is also left as a (row, column) record
//   shallow_edge_lists  degrees (Eq. 10) and neighbour lists from those records
//   shallow_mirror  lower triangle of G by bit transposition     } only when the caller wants G,
//   shallow_lists   degrees and neighbour lists from the rows of G } or the records do not suffice
//   merge_onehop, merge_twohop, merge_update
//                   the first rounds of the greedy highest-degree codebook construction
//                   (Eq. 11-13) in its exact parallel form, one launch per phase
//   shallow_merge   the remaining rounds, one workgroup per problem
//   shallow_rank    codebook order of the picked tokens
//   shallow_emit    references in codebook order and the codebook vectors
//   shallow_assign, shallow_assign_exact, shallow_overflow
//                   tokens whose entry fell beyond the codebook cap go to the nearest
//                   stored entry
//
// shallow_graph.hip holds the kernels up to the neighbour lists, shallow_merge.hip the greedy
// merge, shallow_codebook.hip the codebook order, the outputs and the cap; shallow.hip the
// workspace layout and the entry points.
#pragma once

#include <math.h>
#include <string.h>

#include "common.h"

namespace spindle {

// Unit vectors are stored in fp16 scaled by 2^10, so that components down to 6e-8 of the
// norm stay normal numbers.  |fp16 MFMA cosine - exact cosine| then stays below kGuard:
// each component of both vectors carries a relative rounding error of at most 2^-11
// (sum over the dot product <= 2^-10 = 9.77e-4 by Cauchy-Schwarz), the fp32 normalisation
// adds < 1e-6 and the fp32 accumulation of 128 exact products < 1e-5.
constexpr float kUnitScale = 1024.f;
constexpr float kGuard = 1.05e-3f;
// shallow_gram uses the measured rounding error of the two vectors instead of that worst case:
// |fp16 MFMA cosine - exact cosine| <= err_a (1 + err_b) + err_b + kGuardSlack, where the
// slack covers the fp32 accumulation (< 1.6e-5 even with truncation) and fp16 subnormal
// components should the matrix cores flush them (< 8e-6).
constexpr float kGuardSlack = 3e-5f;

constexpr int kPanelRows = 256;   // rows of G's column range held in registers per block
constexpr int kChunkCols = 1024;  // tokens per chunk: one 128-byte line of each row of G
constexpr int kItemChunks = 4;    // chunks a block handles with the same rows in registers
constexpr int kStageCols = 64;
constexpr int kGramThreads = 256;
constexpr int kLdsRow = 272;      // fp16 row of 128 + 16 B pad (shallow_prep)
constexpr int kStageBytes = kStageCols * 256;   // staged tokens: unpadded rows, 16-byte pieces swizzled

// Edges a wave may record per chunk (64 rows x 1024 columns): what 32 MiB per problem allow,
// between 512 (n = 32768: 16384 segments) and 4096 (short sequences, where a cluster of similar
// tokens fills a larger share of every chunk).
inline int seg_cap_for(int n) {
  const long segs = 4L * ((n + 255) / 256) * ((n + 1023) / 1024);
  long cap = (32L << 20) / (segs * 4);
  cap = cap < 512 ? 512 : (cap > 4096 ? 4096 : cap);
  return (int)(cap & ~63L);
}
constexpr int kFixBucket = 2048;  // pairs decided in double precision that one row panel can take
constexpr int kCounters = 32;     // ints per ut
// Grid round r reads the list length C_ALIVE0 + r and builds C_ALIVE0 + r + 1, and has its own
// candidate and dying counters, so that nothing has to be cleared between the rounds; the
// slots 6..15 hold the phase timings of the tail kernel.
enum { C_ALIVE0 = 0, C_ALIVE1 = 1, C_CAND = 2, C_DYING = 3, C_PICKS = 4, C_ROUNDS = 5,
       C_ALIVE2 = 16, C_CAND1 = 17, C_DYING1 = 18 };
__host__ __device__ constexpr int alive_slot(int round) { return round < 2 ? C_ALIVE0 + round : C_ALIVE2; }

struct ShallowParams {
  const char *X[2];        // input tensors [U][n][128] in `dtype` (index = tensor slot)
  float theta[2];
  int dtype, U, UT, n, Wp;  // Wp = words per adjacency row (multiple of 4)
  KvLayout lay;            // rows of the input tensors
  int cap;
  // workspace
  _Float16 *Xh;            // [UT][n][128] unit vectors
  double *m64;             // [UT][n]
  float *err;              // [UT][n] distance of the stored fp16 unit vector from the exact one (units of the norm)
  unsigned *echunk;        // [UT][ceil(n/1024)] largest err of each 1024-token chunk (float bits)
  uint32_t *G;             // [UT][n][Wp]
  int *deg0, *slot, *alive, *alive2, *cand, *dying, *pick_vert, *rank, *rank_vert;   // [UT][n]
  uint16_t *nbr;           // [UT][n][kListCap] neighbour lists of the sparse rows
  uint8_t *gone8;          // [UT][n16] 1 once a token has been given a slot (grid rounds of the merge); n16 = n rounded up to 16
  int n16;
  uint32_t *key, *gone, *m1, *pick_key;                                      // [UT][n]
  int *counters;           // [UT][kCounters]
  uint32_t *fix;           // [UT][fix_cap] deferred pairs, b << 16 | a
  unsigned *fix_count;     // [UT]
  unsigned *fix_overflow;  // [1] some list was full
  // set bits of the computed part of G as (row << 16 | column), one segment per (problem, chunk,
  // row panel, wave): segment ((ut * nJc + J) * nI + I) * 4 + w, seg_cap entries
  int seg_cap;             // entries per segment
  uint32_t *edges;
  unsigned *ecount;        // entries of each segment
  uint32_t *fedges;        // [UT][panels][kFixBucket] pairs shallow_fixup found adjacent, row << 16 | column,
                           //     filed under the 256-row panel of each end whose list they extend
  unsigned *fecount;       // [UT][panels]
  unsigned *need_full;     // [1] an edge segment ran full or a row has more neighbours than a list holds:
                           //     degrees and lists are then taken from the complete bitmap
  unsigned fix_cap;        // per ut
  uint32_t *ovf;           // [UT][n] tokens whose codebook entry was cut, per problem
  unsigned *ovf_cnt;       // [UT] their number
  float2 *cstat;           // [UT][n][2] per cut token and lane group: largest approximate cosine seen, entries collected
  uint2 *ccand;            // [UT][n][2][kCandCap] (entry index, approximate cosine bits)
  uint32_t *ovf_left;      // [UT*n] cut tokens left to the exhaustive search, packed ut << 16 | token
  unsigned *ovf_count;     // [1] their number
  // outputs (index = tensor slot)
  char *C[2];
  int32_t *n_codes[2], *n_found[2], *ref[2];
  float *mag[2];
  int32_t *deg_out[2];     // optional initial degrees
};

__device__ __forceinline__ const char *x_row(const ShallowParams &p, int ut, int a) {
  const int t = ut / p.U, u = ut % p.U;
  return p.X[t] + kv_unit_offset(p.lay, u) + (size_t)a * (size_t)p.lay.st;
}

// x_a . x_b in double precision, summed in dimension order (products are exact).
template <int DT>
__device__ double dot64(const char *ra, const char *rb) {
  typedef typename Elem<DT>::type T;
  constexpr int per = 16 / sizeof(T);
  double acc = 0.0;
  constexpr int kBatch = 8;                          // pieces of each row in flight
  for (int c0 = 0; c0 < kHeadDim / per; c0 += kBatch) {
    u4 va[kBatch], vb[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      va[i] = reinterpret_cast<const u4 *>(ra)[c0 + i];
      vb[i] = reinterpret_cast<const u4 *>(rb)[c0 + i];
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const T *ea = reinterpret_cast<const T *>(&va[i]);
      const T *eb = reinterpret_cast<const T *>(&vb[i]);
#pragma unroll
      for (int j = 0; j < per; ++j)
        acc += (double)Elem<DT>::to_float(ea[j]) * (double)Elem<DT>::to_float(eb[j]);
    }
  }
  return acc;
}

__device__ inline double dot64_any(int dtype, const char *ra, const char *rb) {
  if (dtype == SPINDLE_F16) return dot64<SPINDLE_F16>(ra, rb);
  if (dtype == SPINDLE_BF16) return dot64<SPINDLE_BF16>(ra, rb);
  return dot64<SPINDLE_F32>(ra, rb);
}

// Eq. 4 evaluated the way the adjacency decision is defined: double precision,
// dimension-order dot product, 0 when either vector is zero.
__device__ inline double cos64(const ShallowParams &p, int ut, int a, int b) {
  const double den = p.m64[(size_t)ut * p.n + a] * p.m64[(size_t)ut * p.n + b];
  if (!(den > 0.0)) return 0.0;
  return dot64_any(p.dtype, x_row(p, ut, a), x_row(p, ut, b)) / den;
}

// Entries of a token's neighbour list (uint16 indices); rows with more neighbours are read from
// the bitmap G instead.
constexpr int kListCap = 256;
// Where the p-th neighbour of a row is stored: lane sl of the 8-lane segment that later walks
// the row reads the 16 entries from sl * 16 on (of each half of 128), so the neighbours are dealt
// out to the lanes in turn and a short row occupies all eight lanes instead of the first one.
__host__ __device__ constexpr int list_slot(int p) { return (p & ~127) | ((p & 7) << 4) | ((p & 127) >> 3); }

// Entries per cut token and lane group that shallow_assign hands to the exact comparison.
constexpr int kCandCap = 8;

// ---------------------------------------------------------------- launches, one per source file
// Each enqueues its kernels on `st` in order and returns SPINDLE_OK or the failed HIP call.
// force: the caller wants the adjacency matrix, so the full bitmap is completed as well.
spindle_status launch_graph(const ShallowParams &p, hipStream_t st, int force);
spindle_status launch_bare_similarity(const ShallowParams &p, hipStream_t st, int mode);   // measurement aid
spindle_status launch_merge(const ShallowParams &p, hipStream_t st);
spindle_status launch_codebook(const ShallowParams &p, hipStream_t st);

}  // namespace spindle
