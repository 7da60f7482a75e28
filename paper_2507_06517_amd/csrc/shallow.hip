// Similarity codebook replacement (Sec. "Similarity Based Token Replacement", Alg. 1).
//
// Kernels, all enqueued on the caller's stream; ut = tensor * units + unit indexes one
// independent (batch, kv-head, K|V) problem of n tokens:
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
#include <math.h>
#include <string.h>

#include <vector>

#include "common.h"
#include "mma.h"

namespace spindle {
namespace {

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

__device__ double dot64_any(int dtype, const char *ra, const char *rb) {
  if (dtype == SPINDLE_F16) return dot64<SPINDLE_F16>(ra, rb);
  if (dtype == SPINDLE_BF16) return dot64<SPINDLE_BF16>(ra, rb);
  return dot64<SPINDLE_F32>(ra, rb);
}

// Eq. 4 evaluated the way the adjacency decision is defined: double precision,
// dimension-order dot product, 0 when either vector is zero.
__device__ double cos64(const ShallowParams &p, int ut, int a, int b) {
  const double den = p.m64[(size_t)ut * p.n + a] * p.m64[(size_t)ut * p.n + b];
  if (!(den > 0.0)) return 0.0;
  return dot64_any(p.dtype, x_row(p, ut, a), x_row(p, ut, b)) / den;
}

// ---------------------------------------------------------------- prep
template <int DT>
__global__ __launch_bounds__(256) void shallow_prep(ShallowParams p) {
  typedef typename Elem<DT>::type T;
  constexpr int kRows = 64;
  constexpr int row_bytes = kHeadDim * sizeof(T);
  constexpr int lds_row = row_bytes + 16;
  constexpr int tpr = row_bytes / 16;
  __shared__ __attribute__((aligned(16))) char tile_in[kRows * lds_row];
  __shared__ __attribute__((aligned(16))) char tile_out[kRows * kLdsRow];
  __shared__ float row_err[kRows];
  __shared__ double row_inv[kRows];
  const int ut = blockIdx.y, t = ut / p.U;
  const int row0 = blockIdx.x * kRows;
  for (int i = threadIdx.x; i < kRows * tpr; i += 256) {
    const int r = i / tpr, ch = i % tpr;
    u4 v = {0, 0, 0, 0};
    if (row0 + r < p.n) v = *reinterpret_cast<const u4 *>(x_row(p, ut, row0 + r) + ch * 16);
    *reinterpret_cast<u4 *>(tile_in + r * lds_row + ch * 16) = v;
  }
  __syncthreads();
  if (threadIdx.x < kRows && row0 + threadIdx.x < p.n) {
    const int r = threadIdx.x;
    constexpr int per = 16 / sizeof(T);
    double ss = 0.0;
    for (int ch = 0; ch < tpr; ++ch) {
      const u4 v = *reinterpret_cast<const u4 *>(tile_in + r * lds_row + ch * 16);
      const T *e = reinterpret_cast<const T *>(&v);
#pragma unroll
      for (int i = 0; i < per; ++i) {
        const double x = (double)Elem<DT>::to_float(e[i]);
        ss += x * x;
      }
    }
    const double m = sqrt(ss);
    const size_t idx = (size_t)ut * p.n + row0 + r;
    p.m64[idx] = m;
    p.mag[t][(size_t)(ut % p.U) * p.n + row0 + r] = (float)m;
    row_inv[r] = m > 0.0 ? (double)kUnitScale / m : 0.0;
  } else if (threadIdx.x < kRows) {
    row_inv[threadIdx.x] = 0.0;                      // rows past the end of the sequence
  }
  __syncthreads();
  {
    // four threads per row: fp16 unit vector (x 2^10) and its distance from the exact one
    const int r = threadIdx.x >> 2, part = threadIdx.x & 3;
    constexpr int per = 16 / sizeof(T);
    const double inv64 = row_inv[r];
    const float inv = (float)inv64;
    double e2 = 0.0;                                   // squared distance stored - exact, scaled units
    for (int ch = part * (tpr / 4); ch < (part + 1) * (tpr / 4); ++ch) {
      const u4 v = *reinterpret_cast<const u4 *>(tile_in + r * lds_row + ch * 16);
      const T *e = reinterpret_cast<const T *>(&v);
#pragma unroll
      for (int i = 0; i < per; ++i) {
        const _Float16 hv = (_Float16)(Elem<DT>::to_float(e[i]) * inv);
        reinterpret_cast<_Float16 *>(tile_out + r * kLdsRow)[ch * per + i] = hv;
        const double d = (double)(float)hv - (double)Elem<DT>::to_float(e[i]) * inv64;
        e2 += d * d;
      }
    }
    e2 += __shfl_xor(e2, 1);
    e2 += __shfl_xor(e2, 2);
    if (part == 0 && row0 + r < p.n) {
      // rounded up: the double-precision evaluation above is good to 1e-15, the cast to 6e-8
      const float ev = (float)(sqrt(e2) / (double)kUnitScale) * (1.f + 1e-6f) + 1e-12f;
      p.err[(size_t)ut * p.n + row0 + r] = ev;
      row_err[r] = ev;
    }
  }
  __syncthreads();
  if (threadIdx.x < kRows) {                         // one update of the chunk's maximum per block
    float mx = row0 + (int)threadIdx.x < p.n ? row_err[threadIdx.x] : 0.f;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if (threadIdx.x == 0)
      atomicMax(p.echunk + (size_t)ut * ((p.n + kChunkCols - 1) / kChunkCols) + row0 / kChunkCols, __float_as_uint(mx));
  }
  for (int i = threadIdx.x; i < kRows * 16; i += 256) {
    const int r = i / 16, ch = i % 16;
    if (row0 + r < p.n)
      *reinterpret_cast<u4 *>(reinterpret_cast<char *>(p.Xh) + ((size_t)ut * p.n + row0 + r) * 256 + ch * 16) =
          *reinterpret_cast<const u4 *>(tile_out + r * kLdsRow + ch * 16);
  }
}

// ---------------------------------------------------------------- gram
// Block = 4 waves; wave w keeps the unit vectors of tokens a in [I*256 + 64w, +64) as
// MFMA A-fragments and streams tokens b of the column chunk through LDS.  Lane (g, c)
// of a 32-column tile holds, for token b = col + c, the similarities with 16 of the 32
// tokens a of each row block; their signs relative to theta are packed by alignbit
// into the bits of word (a / 32) of row b of G.
//
// The accumulators start at -theta (in the 2^20-scaled units of the stored vectors), so
// the sign of the result is the fp16 decision.  Results closer to zero than the guard
// band are not trusted: their bits are cleared and the pair is queued for the exact
// double-precision decision (shallow_fixup sets the bit if it is adjacent).

constexpr int kPairBuf = 256;   // queued pairs per wave before a flush
constexpr int kWordList = 384;  // listed pieces per wave before they are turned into records

// Moves a wave's queued pairs to the global list of its ut.  When that list is full the
// pairs are dropped and a flag is raised: shallow_gram<true> then decides every close
// pair of every tile in place (slow, but only for inputs with an extreme number of
// similarities within the guard band of theta).
__device__ __forceinline__ void flush_pairs(const ShallowParams &p, int ut, const uint32_t *buf, int count) {
  const int lane = lane_id();
  unsigned base = 0;
  if (lane == 0) base = atomicAdd(p.fix_count + ut, (unsigned)count);
  base = __shfl(base, 0);
  uint32_t *list = p.fix + (size_t)ut * p.fix_cap;
  if (base + (unsigned)count > p.fix_cap && lane == 0) atomicExch(p.fix_overflow, 1u);
  for (int i = lane; i < count; i += kWave)
    if (base + i < p.fix_cap) list[base + i] = buf[i];
}

// min(m, |a|, |b|) in one instruction.  `after_a`, `after_b` must be results of ordinary VALU
// instructions that read the MFMA results a and b come from: the compiler places the wait states a
// matrix-core result needs in front of instructions it knows, not in front of inline
// assembly, so this one is tied behind such an instruction by a data dependency.
__device__ __forceinline__ float min3_abs(float m, float a, float b, uint32_t after_a, uint32_t after_b) {
  float r;
  asm("v_min3_f32 %0, %1, |%2|, |%3|" : "=v"(r) : "v"(m), "v"(a), "v"(b), "v"(after_a), "v"(after_b));
  return r;
}

// 16 bytes per lane from global memory straight into LDS: lane i's piece lands at
// lds_addr + 16 i (lds_addr wave-uniform).  Issued as assembly on purpose: the compiler
// would put a wait for the load in front of every later LDS read of the kernel, since it
// cannot tell which of them touch the destination.  Completion is the caller's business
// (s_waitcnt vmcnt + barrier before any lane reads the destination).
__device__ __forceinline__ void lds_dma16(const void *src, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(src)
               : "memory", "m0");
}

// kExact = false: the fast pass described above, one block per (row panel, column chunk).
// kExact = true: fallback pass over the same tiles, run by a fixed grid that exits at once
// unless a pair list overflowed; it stores no words and decides the close pairs in place.
template <bool kExact>
__global__ __launch_bounds__(kGramThreads, 2) void shallow_gram(ShallowParams p) {
  typedef Mma<SPINDLE_F16> M;
  // two stages of 64 tokens, filled by direct global->LDS loads.  Row r keeps its 16-byte piece
  // k at position k ^ swz(r), swz(r) = (r & 7) | ((r & 16) >> 1), so that sixteen consecutive lanes
  // of a 128-bit LDS read (sixteen different rows, same k) hit sixteen different bank groups.
  __shared__ __attribute__((aligned(1024))) char stage[2 * kStageBytes];
  __shared__ uint32_t pairbuf[kGramThreads / 64][kPairBuf];
  // the 32 words (one 128-byte line) of each of a wave's 64 rows for the current chunk;
  // written out as whole lines, because partially written lines cost several times their
  // size in HBM write traffic.  Row pitch 36 words keeps 16-byte alignment.
  __shared__ __attribute__((aligned(16))) uint32_t wstage[kGramThreads / 64][64][36];
  __shared__ uint32_t wordlist[kGramThreads / 64][kWordList];   // the 16-byte pieces of a chunk that have a set bit
  const int n = p.n;
  const int nI = (n + kPanelRows - 1) / kPanelRows;
  const int nJ = (n + kChunkCols * kItemChunks - 1) / (kChunkCols * kItemChunks);
  // blocks are dealt round-robin to the 8 XCDs: give each XCD one (ut, chunk) at a time
  // and let it sweep the row panels, so the chunk is re-read from that XCD's L2
  if (kExact) {
    if (*p.fix_overflow == 0) return;
    if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(p.need_full, 1u);   // bits set here leave no edge records
  }
  const int nitems = 8 * nI * ((p.UT * nJ + 7) / 8);
  for (int item = blockIdx.x; item < nitems; item += gridDim.x) {
  const int xcd = item & 7, s_ = item >> 3;
  const int I = s_ % nI;
  const int pj = (s_ / nI) * 8 + xcd;
  if (pj >= p.UT * nJ) continue;
  // (the chunk group is rotated by ut: groups to the right hold more work, and every XCD
  // should see all of them)
  const int ut = pj / nJ, Jg = (pj % nJ + ut) % nJ;
  // G is symmetric: a row panel only computes the chunks from the one holding its own
  // tokens onwards; shallow_mirror fills the columns to the left from the transposed blocks
  const int Jfirst = (I * kPanelRows) / kChunkCols;
  if ((Jg + 1) * kItemChunks <= Jfirst) continue;
  const float theta_s = p.theta[ut / p.U] * kUnitScale * kUnitScale;
  const int lane = lane_id(), wave = threadIdx.x >> 6, g = lane >> 5, c = lane & 31;
  const char *Xh = reinterpret_cast<const char *>(p.Xh) + (size_t)ut * n * 256;
  const int arow0 = I * kPanelRows + 64 * wave;   // first of this wave's 64 rows of G
  uint32_t *buf = pairbuf[wave];
  int nbuf = 0;                                    // wave-uniform

  // unit vectors of the wave's rows: MFMA B operand (matrix columns = lanes)
  M::frag af[2][M::kSteps];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    const int a = arow0 + 32 * cb + c;
#pragma unroll
    for (int ks = 0; ks < M::kSteps; ++ks)
      af[cb][ks] = a < n ? M::load(Xh + (size_t)a * 256, ks, g) : M::zero();
  }
  float erow[2];                                   // rounding error of the stored vectors of this lane's two rows
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    const int a = arow0 + 32 * cb + c;
    erow[cb] = a < n ? p.err[(size_t)ut * n + a] : 0.f;
  }
  f16v cinit;
#pragma unroll
  for (int v = 0; v < 16; ++v) cinit[v] = -theta_s;
  // Staged token 16*g + v of a tile is fed to matrix row 8*(v/4) + 4*g + v%4, so that result
  // register v of lane group g belongs to token 16*g + v and the packed sign bits come out
  // in token order.
  const int prow = 16 * ((c >> 2) & 1) + 4 * (c >> 3) + (c & 3);
  int soff[M::kSteps];                             // byte offset of this lane's fragment ks in tile 0 of a stage
#pragma unroll
  for (int ks = 0; ks < M::kSteps; ++ks)
    soff[ks] = prow * 256 + (((2 * ks + g) ^ ((prow & 7) | ((prow & 16) >> 1))) << 4);
  uint32_t voff[4];                                // this lane's source offset within a stage, per load
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int r = (wave * 4 + q) * 4 + (lane >> 4);
    voff[q] = (uint32_t)(r * 256 + (((lane & 15) ^ ((r & 7) | ((r & 16) >> 1))) << 4));
  }
  const uint32_t wsel = g ? 0x07060302u : 0x05040100u;
  M::frag pf0, pf1;                                // fragments 0, 1 of the tile the next step multiplies
  const uint32_t stage_lds = (uint32_t)(size_t)(__attribute__((address_space(3))) char *)stage;

  bool carried = false;                            // pipeline state of the chunk to come already in place
  f16v cur0, cur1, nxt0, nxt1;
  for (int J = Jg * kItemChunks > Jfirst ? Jg * kItemChunks : Jfirst; J < (Jg + 1) * kItemChunks && J * kChunkCols < n; ++J) {
  const int col_begin = J * kChunkCols;
  const int col_end = col_begin + kChunkCols < n ? col_begin + kChunkCols : n;
  const int ntiles = (col_end - col_begin + 31) / 32;
  // guard band of this lane's two rows against the tokens of the chunk (scaled units)
  const float ech = __uint_as_float(p.echunk[(size_t)ut * ((n + kChunkCols - 1) / kChunkCols) + J]);
  const float band0 = (erow[0] * (1.f + ech) + ech + kGuardSlack) * (kUnitScale * kUnitScale);
  const float band1 = (erow[1] * (1.f + ech) + ech + kGuardSlack) * (kUnitScale * kUnitScale);
  const float band = fmaxf(band0, band1);
  // Stage s of the chunk = tokens col_begin + 64 s .. + 63, in buffer s & 1; tile x = half x & 1
  // of stage x >> 1.  Each wave fills 16 rows of a stage with four 1-KiB loads (4 rows x 16
  // pieces, lane = slot).  Rows past the end of the sequence exist (the array is padded) and
  // are never used: their bits are masked and their pairs rejected.
  auto dma = [&](int b0, int bufsel) {
    const char *sbase = Xh + (size_t)b0 * 256;
#pragma unroll
    for (int q = 0; q < 4; ++q) lds_dma16(sbase + voff[q], stage_lds + bufsel * kStageBytes + (wave * 4 + q) * 1024);
  };
  auto frag_at = [&](int bufsel, int ct, int ks) -> M::frag {
    return *reinterpret_cast<const M::frag *>(stage + bufsel * kStageBytes + ct * 32 * 256 + soff[ks]);
  };
  // One pipeline step: the matrix cores compute the similarities of the NEXT tile x (32
  // staged tokens x this wave's 64 rows, minus theta) while the vector units turn the
  // signs of the CURRENT tile (results a0, a1, first token bcol0) into the word of this
  // lane's row of G.  The two instruction streams are independent; sched_barrier pins the
  // issue order (two matrix instructions, then a slice of vector work).  The step starts
  // with matrix instructions on fragments fetched during the previous step (pf0, pf1), so
  // the matrix cores do not wait for the vector work on their previous results.
  // (bufx, ctx) = place of tile x, (bufn, ctn) = place of tile x + 1.  With sync_fetch (x is
  // the second half of its stage) the step also holds the block barrier after its last read
  // of the stage, which hands the buffer to the loads of the stage after next (tokens
  // fetch_b0 ..) and makes the next stage, loaded one barrier earlier, visible.
  auto step = [&](int bufx, int ctx, int bufn, int ctn, bool sync_fetch, int fetch_b0, int bcol0, const f16v &a0,
                  const f16v &a1, f16v &r0, f16v &r1) -> uint32_t {
    M::frag f2 = frag_at(bufx, ctx, 2), f3 = frag_at(bufx, ctx, 3);
    r0 = M::mma(pf0, af[0][0], cinit);
    r1 = M::mma(pf0, af[1][0], cinit);
    __builtin_amdgcn_sched_barrier(0);               // matrix instructions first: the vector work below waits for the previous tile
    uint32_t sg0 = 0, sg1 = 0;
    float mn = INFINITY;
#pragma unroll
    for (int v = 15; v >= 12; --v) {
      sg0 = __builtin_amdgcn_alignbit(sg0, __float_as_uint(a0[v]), 31);
      sg1 = __builtin_amdgcn_alignbit(sg1, __float_as_uint(a1[v]), 31);
      mn = min3_abs(mn, a0[v], a1[v], sg0, sg1);
    }
    __builtin_amdgcn_sched_barrier(0);
    r0 = M::mma(pf1, af[0][1], r0);
    r1 = M::mma(pf1, af[1][1], r1);
    M::frag f4 = frag_at(bufx, ctx, 4), f5 = frag_at(bufx, ctx, 5);
#pragma unroll
    for (int v = 11; v >= 9; --v) {
      sg0 = __builtin_amdgcn_alignbit(sg0, __float_as_uint(a0[v]), 31);
      sg1 = __builtin_amdgcn_alignbit(sg1, __float_as_uint(a1[v]), 31);
      mn = min3_abs(mn, a0[v], a1[v], sg0, sg1);
    }
    __builtin_amdgcn_sched_barrier(0);
    r0 = M::mma(f2, af[0][2], r0);
    r1 = M::mma(f2, af[1][2], r1);
    M::frag f6 = frag_at(bufx, ctx, 6), f7 = frag_at(bufx, ctx, 7);
#pragma unroll
    for (int v = 8; v >= 6; --v) {
      sg0 = __builtin_amdgcn_alignbit(sg0, __float_as_uint(a0[v]), 31);
      sg1 = __builtin_amdgcn_alignbit(sg1, __float_as_uint(a1[v]), 31);
      mn = min3_abs(mn, a0[v], a1[v], sg0, sg1);
    }
    __builtin_amdgcn_sched_barrier(0);
    r0 = M::mma(f3, af[0][3], r0);
    r1 = M::mma(f3, af[1][3], r1);
#pragma unroll
    for (int v = 5; v >= 3; --v) {
      sg0 = __builtin_amdgcn_alignbit(sg0, __float_as_uint(a0[v]), 31);
      sg1 = __builtin_amdgcn_alignbit(sg1, __float_as_uint(a1[v]), 31);
      mn = min3_abs(mn, a0[v], a1[v], sg0, sg1);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (sync_fetch) {
      __builtin_amdgcn_s_waitcnt(0x0070);            // vmcnt(0) lgkmcnt(0): own loads landed, own reads done
      __builtin_amdgcn_s_barrier();
      dma(fetch_b0, bufx);
    }
    __builtin_amdgcn_sched_barrier(0);
    r0 = M::mma(f4, af[0][4], r0);
    r1 = M::mma(f4, af[1][4], r1);
    pf0 = frag_at(bufn, ctn, 0);
    pf1 = frag_at(bufn, ctn, 1);
#pragma unroll
    for (int v = 2; v >= 0; --v) {
      sg0 = __builtin_amdgcn_alignbit(sg0, __float_as_uint(a0[v]), 31);
      sg1 = __builtin_amdgcn_alignbit(sg1, __float_as_uint(a1[v]), 31);
      mn = min3_abs(mn, a0[v], a1[v], sg0, sg1);
    }
    uint32_t q0 = ~sg0 & 0xFFFFu, q1 = ~sg1 & 0xFFFFu;   // bit v: staged token 16*g + v
    // pairs too close to theta for fp16: clear their bits now, queue them for the exact
    // decision.  Bit 16*cb + v of `rest` = close.
    uint32_t rest = 0;
    const bool any_close = __any(mn < band);
    __builtin_amdgcn_sched_barrier(0);
    r0 = M::mma(f5, af[0][5], r0);
    r1 = M::mma(f5, af[1][5], r1);
    if (any_close) {
      uint32_t cm0 = 0, cm1 = 0;
#pragma unroll
      for (int v = 15; v >= 0; --v) {
        cm0 = __builtin_amdgcn_alignbit(cm0, __float_as_uint(fabsf(a0[v]) - band0), 31);
        cm1 = __builtin_amdgcn_alignbit(cm1, __float_as_uint(fabsf(a1[v]) - band1), 31);
      }
      q0 &= ~cm0;
      q1 &= ~cm1;
      rest = (cm0 & 0xFFFFu) | (cm1 << 16);
    }
    if (bcol0 < arow0 + 64 && bcol0 + 32 > arow0) {   // tile touches the diagonal: G_aa = 1
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) {
        const int i = arow0 + 32 * cb + c - bcol0;    // staged index of this lane's own token
        if (i >= 0 && i < 32 && (i >> 4) == g) {
          if (cb == 0) q0 |= 1u << (i & 15); else q1 |= 1u << (i & 15);
        }
      }
    }
    if (bcol0 + 32 > n) {                             // staged tokens beyond the sequence
      const int nv = n - bcol0 - 16 * g;
      const uint32_t keep = nv >= 16 ? 0xFFFFu : (nv <= 0 ? 0u : (1u << nv) - 1u);
      q0 &= keep;
      q1 &= keep;
    }
    __builtin_amdgcn_sched_barrier(0);
    r0 = M::mma(f6, af[0][6], r0);
    r1 = M::mma(f6, af[1][6], r1);
    // halves[0] = the value of the lane with g = 0 of this column, halves[1] = that of g = 1
    const uint32_t own = q0 | (q1 << 16);
    const auto halves = __builtin_amdgcn_permlane32_swap(own, own, false, false);
    __builtin_amdgcn_sched_barrier(0);
    r0 = M::mma(f7, af[0][7], r0);
    r1 = M::mma(f7, af[1][7], r1);
    // lane group 0 keeps the word of row block 0 (low halves), group 1 that of block 1
    const uint32_t word = __builtin_amdgcn_perm(halves[1], halves[0], wsel);
    if (any_close) {
      while (__any(rest != 0)) {
        const bool has = rest != 0;
        const int i = has ? __builtin_ctz(rest) : 0;
        rest &= rest - 1;
        const int row = arow0 + 32 * (i >> 4) + c;          // row of G
        const int bit = bcol0 + 16 * g + (i & 15);           // staged token
        const bool valid = has && row < n && bit < n && row != bit;
        if (kExact) {
          if (valid && cos64(p, ut, row, bit) > (double)p.theta[ut / p.U])
            atomicOr(p.G + ((size_t)ut * n + row) * p.Wp + (bit >> 5), 1u << (bit & 31));
          continue;
        }
        const unsigned long long m = __ballot(valid);
        if (m) {                                    // wave-uniform
          if (nbuf > kPairBuf - 64) { flush_pairs(p, ut, buf, nbuf); nbuf = 0; }
          if ((m >> lane) & 1ull) buf[nbuf + __popcll(m & ((1ull << lane) - 1ull))] = ((uint32_t)row << 16) | (uint32_t)bit;
          nbuf += __popcll(m);
        }
      }
    }
    return word;
  };

  if (!carried) {
    dma(col_begin, 0);
    dma(col_begin + kStageCols, 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wave's loads have landed in LDS
    __syncthreads();
    // first tile of the chunk: nothing to pack yet
    cur0 = cinit;
    cur1 = cinit;
#pragma unroll
    for (int ks = 0; ks < M::kSteps; ++ks) {
      const M::frag f = frag_at(0, 0, ks);
      cur0 = M::mma(f, af[0][ks], cur0);
      cur1 = M::mma(f, af[1][ks], cur1);
    }
    pf0 = frag_at(0, 1, 0);
    pf1 = frag_at(0, 1, 1);
  }
  u4 words = {0, 0, 0, 0};
  // four tiles (two stages) per trip: their words are one aligned 16-byte piece of the row.
  // The trip is branch-free: tiles past the end of the chunk only occur at the end of the
  // sequence and give zero words.  Step j packs tile t0 + j and multiplies tile x = t0 + j + 1.
  for (int t0 = 0; t0 < ntiles; t0 += 4) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int bcol0 = col_begin + (t0 + j) * 32;
      const int x = j + 1;                           // tile x of the trip (mod 4: t0 is a multiple of 4)
      words[j] = step((x >> 1) & 1, x & 1, ((x + 1) >> 1) & 1, (x + 1) & 1, (x & 1) != 0,
                      col_begin + (t0 + x + 3) * 32, bcol0, cur0, cur1, nxt0, nxt1);
      cur0 = nxt0;
      cur1 = nxt1;
    }
    if (!kExact) *reinterpret_cast<u4 *>(&wstage[wave][lane][t0]) = words;
  }
  if (!kExact) {
    const int npieces = (ntiles + 3) / 4, piece = lane & 7;
    // the set bits also go out as (row, column) records, a segment per wave and chunk: sparse
    // graphs get their neighbour lists from these without another pass over G
    const int nJc = (n + kChunkCols - 1) / kChunkCols;
    const size_t seg = (((size_t)ut * nJc + J) * nI + I) * 4 + wave;
    uint32_t *eseg = p.edges + seg * p.seg_cap;
    int ecnt = 0;                                    // wave-uniform
    const unsigned long long below = (1ull << lane) - 1ull;
    // Few of the 512 16-byte pieces of a chunk (64 rows x 8) have a bit set.  First the pieces
    // that have one are listed (one ballot per eight rows), then every lane takes a listed piece
    // and the wave peels off one bit of each per pass: far fewer passes than over all pieces.
    uint32_t *wl = wordlist[wave];
    int nw = 0;                                      // wave-uniform
    auto expand = [&]() {
      for (int e0 = 0; e0 < nw; e0 += kWave) {
        const int e = e0 + lane;
        const uint32_t key = e < nw ? wl[e] : 0u;    // row in the wave << 3 | piece
        u4 v = *reinterpret_cast<const u4 *>(&wstage[wave][key >> 3][(key & 7u) * 4]);
        if (e >= nw) v = u4{0, 0, 0, 0};
        const uint32_t rec0 = ((uint32_t)(arow0 + (int)(key >> 3)) << 16) | (uint32_t)(col_begin + (int)(key & 7u) * 128);
        for (;;) {
          const bool has = (v[0] | v[1] | v[2] | v[3]) != 0;
          const unsigned long long mk = __ballot(has);
          if (mk == 0) break;
          if (has) {
            const int j = v[0] ? 0 : v[1] ? 1 : v[2] ? 2 : 3;
            const uint32_t w = v[j];
            const int t = __builtin_ctz(w);
            v[j] = w & (w - 1);
            const int at = ecnt + __popcll(mk & below);
            if (at < p.seg_cap) eseg[at] = rec0 + (uint32_t)(j * 32 + t);
          }
          ecnt += __popcll(mk);
        }
      }
      nw = 0;
    };
    for (int it = 0; it < 8; ++it) {
      const int r = it * 8 + (lane >> 3);
      const u4 v = *reinterpret_cast<const u4 *>(&wstage[wave][r][piece * 4]);
      const bool live = arow0 + r < n && piece < npieces;
      if (live)
        *reinterpret_cast<u4 *>(p.G + ((size_t)ut * n + arow0 + r) * p.Wp + (col_begin >> 5) + piece * 4) = v;
      const bool nz = live && (v[0] | v[1] | v[2] | v[3]) != 0;
      const unsigned long long mk = __ballot(nz);
      if (mk) {                                      // wave-uniform
        const int add = __popcll(mk);
        if (nw + add > kWordList) expand();
        if (nz) wl[nw + __popcll(mk & below)] = (uint32_t)(r << 3 | piece);
        nw += add;
      }
    }
    expand();
    if (lane == 0) {
      p.ecount[seg] = (unsigned)(ecnt < p.seg_cap ? ecnt : p.seg_cap);
      if (ecnt > p.seg_cap) atomicOr(p.need_full, 1u);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);              // loads issued for stages past the chunk
  __syncthreads();                                 // the stage buffers are reused by the next chunk
  // The last steps of a full chunk have staged the 128 tokens that follow it and multiplied the
  // first 32 of them (the pipeline always runs one tile and two stages ahead): when the next
  // chunk of the item follows, its first tile, the fragments of its second and both stage
  // buffers are already in place.
  carried = col_end - col_begin == kChunkCols;
  }
  if (nbuf) { flush_pairs(p, ut, buf, nbuf); nbuf = 0; }
  }
}

// ---------------------------------------------------------------- mirror
// G_ab = G_ba for the part shallow_gram leaves out: rows of the 1024-token tile TI, columns
// of every tile TJ < TI.  One block moves half such a tile: the 64-byte pieces that hold 512
// tokens a of the 1024 rows b of tile TJ go to LDS as two 512 x 512-bit squares, each is
// transposed in place (32 x 32-bit blocks in registers, swapped pairwise), and row a of the
// two squares side by side is one whole 128-byte line of G.  The two halves of a tile run on
// the same XCD one after the other, so the second finds its half of the lines in that L2.
constexpr int kMirrorThreads = 512;
constexpr int kMirrorPitch = 17;                   // words per staged row: column reads hit 32 different banks
constexpr size_t kMirrorLds = (size_t)1024 * kMirrorPitch * sizeof(uint32_t);

// One stage of the 32 x 32 bit transpose held one row per lane (lane i of a 32-lane half =
// row i): exchange with lane i ^ k, k = 16 >> st.  Lanes with bit k clear keep their bits
// at positions with bit k clear and take the partner's bits of those positions, moved up by
// k; the others the mirror image.  rot = right-rotation that moves the partner's bits into
// place (32 - k or k), keep = mask of the bits the lane keeps.
__device__ __forceinline__ uint32_t transpose_stage(uint32_t x, int st, uint32_t rot, uint32_t keep) {
  uint32_t y;
  if (st == 0) {
    y = (uint32_t)__builtin_amdgcn_ds_swizzle((int)x, 0x401F);                        // lane ^ 16
  } else if (st == 1) {
    y = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x128, 0xF, 0xF, false);  // row_ror:8 = lane ^ 8
  } else if (st == 2) {
    y = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x104, 0xF, 0x5, false);  // row_shl:4 -> lanes with bit 2 clear
    y = (uint32_t)__builtin_amdgcn_update_dpp((int)y, (int)x, 0x114, 0xF, 0xA, false);  // row_shr:4 -> lanes with bit 2 set
  } else if (st == 3) {
    y = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
  } else {
    y = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
  }
  const uint32_t moved = __builtin_amdgcn_alignbit(y, y, rot);
  uint32_t r;
  asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(r) : "v"(keep), "v"(x), "v"(moved));   // (x & keep) | (moved & ~keep)
  return r;
}

__device__ __forceinline__ void mirror_half_tile(const ShallowParams &p, uint32_t *mtile, int item) {
  const int n = p.n, Wp = p.Wp;
  const int T = (n + 1023) >> 10, npairs = T * (T - 1) / 2;
  // items b and b + 8 are the two halves of one tile
  const int q = (item >> 4) * 8 + (item & 7), ha = (item >> 3) & 1;
  if (q >= p.UT * npairs) return;
  const int ut = q / npairs, pair = q % npairs;
  int TI = (int)((1.f + sqrtf(1.f + 8.f * (float)pair)) * 0.5f);
  while (TI * (TI - 1) / 2 > pair) --TI;
  while ((TI + 1) * TI / 2 <= pair) ++TI;
  const int TJ = pair - TI * (TI - 1) / 2;          // 0 <= TJ < TI < T
  uint32_t *Gu = p.G + (size_t)ut * n * Wp;
  const int w0 = 32 * TI + 16 * ha;                 // first source word
  // rows of tile TJ all exist (TJ < T - 1); words past the row pitch read as zero
  {
    u4 v[8];
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int k = it * kMirrorThreads + threadIdx.x, r = k >> 2, c4 = k & 3;
      v[it] = u4{0, 0, 0, 0};
      if (w0 + 4 * c4 < Wp) v[it] = *reinterpret_cast<const u4 *>(Gu + (size_t)(1024 * TJ + r) * Wp + w0 + 4 * c4);
    }
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int k = it * kMirrorThreads + threadIdx.x, r = k >> 2, c4 = k & 3;
      uint32_t *d = mtile + r * kMirrorPitch + 4 * c4;
      d[0] = v[it][0]; d[1] = v[it][1]; d[2] = v[it][2]; d[3] = v[it][3];
    }
  }
  __syncthreads();
  // square s = rows 512 s ..; its block (R, C) = rows 32 R .., word C.  The transpose of the
  // block belongs at (C, R): a wave takes the two blocks of an unordered pair, one per
  // 32-lane half, and writes each where the other was.  272 pairs (136 per square), 34 per
  // wave, handled two at a time so that the lane exchanges of one hide those of the other.
  const int lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), h = lane >> 5, i = lane & 31;
  uint32_t rot[5], keep[5];
#pragma unroll
  for (int st = 0; st < 5; ++st) {
    const int k = 16 >> st;
    const uint32_t m = k == 16 ? 0x0000FFFFu : k == 8 ? 0x00FF00FFu : k == 4 ? 0x0F0F0F0Fu : k == 2 ? 0x33333333u : 0x55555555u;
    rot[st] = (i & k) ? k : 32 - k;
    keep[st] = (i & k) ? ~m : m;
  }
  const int lane_off = i * kMirrorPitch;             // word offset of this lane's row within a block
  for (int it = 0; it < 34; it += 2) {
    uint32_t *src[2], *dst[2];
    bool wr[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      // everything up to the choice between the two blocks of the pair is wave-uniform
      const int idx = (it + u) * (kMirrorThreads / 64) + wave;       // < 272
      const int sq = idx >= 136, t = idx - 136 * sq;
      // t -> the t-th pair wa <= wb < 16: rows r and 15 - r of the triangle hold 17 pairs together
      const int r = t / 17, c = t - 17 * r;
      const int wa = c < 16 - r ? r : 15 - r, wb = c < 16 - r ? r + c : c - 1;
      const int base = sq * 512 * kMirrorPitch;
      const int at_ab = base + 32 * wa * kMirrorPitch + wb;             // block (wa, wb)
      const int at_ba = base + 32 * wb * kMirrorPitch + wa;             // block (wb, wa)
      src[u] = mtile + (h ? at_ba : at_ab) + lane_off;
      dst[u] = mtile + (h ? at_ab : at_ba) + lane_off;
      wr[u] = h == 0 || wa != wb;
    }
    uint32_t x0 = *src[0], x1 = *src[1];
#pragma unroll
    for (int st = 0; st < 5; ++st) {
      x0 = transpose_stage(x0, st, rot[st], keep[st]);
      x1 = transpose_stage(x1, st, rot[st], keep[st]);
    }
    if (wr[0]) *dst[0] = x0;
    if (wr[1]) *dst[1] = x1;
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int k = it * kMirrorThreads + threadIdx.x, r = k >> 3, c4 = k & 7;   // row a, 16-byte piece of its line
    const int a = 1024 * TI + 512 * ha + r;
    const uint32_t *sp = mtile + ((c4 >> 2) * 512 + r) * kMirrorPitch + 4 * (c4 & 3);
    const u4 v = {sp[0], sp[1], sp[2], sp[3]};
    if (a < n) *reinterpret_cast<u4 *>(Gu + (size_t)a * Wp + 32 * TJ + 4 * c4) = v;
  }
}

// The launch is a fixed number of workgroups that walk over the half tiles (the grid is a
// multiple of 16, so the two halves of a tile stay on one XCD): when the gate is closed, which
// is the usual case, the launch costs a few hundred workgroups that exit at once.
__global__ __launch_bounds__(kMirrorThreads, 2) void shallow_mirror(ShallowParams p, int force, int items) {
  extern __shared__ __attribute__((aligned(16))) uint32_t mtile[];   // [1024][kMirrorPitch]
  if (!force && *p.need_full == 0) return;         // sparse graph: the lists came from the edge records
  for (int item = blockIdx.x; item < items; item += gridDim.x) {
    mirror_half_tile(p, mtile, item);
    __syncthreads();
  }
}

// ---------------------------------------------------------------- exact fix-up
__global__ __launch_bounds__(256) void shallow_fixup(ShallowParams p) {
  const int ut = blockIdx.y;                         // all problems side by side: each list is short
  const unsigned stride = gridDim.x * blockDim.x;
  unsigned count = p.fix_count[ut];
  if (count > p.fix_cap) count = p.fix_cap;
  const uint32_t *list = p.fix + (size_t)ut * p.fix_cap;
  const double theta = (double)p.theta[ut / p.U];
  for (unsigned i = blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
    const uint32_t e = list[i];
    const int b = (int)(e >> 16), a = (int)(e & 0xFFFFu);
    const bool adj = cos64(p, ut, a, b) > theta;
    if (adj) atomicOr(p.G + ((size_t)ut * p.n + b) * p.Wp + (a >> 5), 1u << (a & 31));
    // ... and as a record for the neighbour lists, filed under the panel of the row; a pair of
    // two different 1024-token tiles was only evaluated in this orientation, so it also
    // extends the list of its column
    // (consecutive pairs of the list mostly share their panels, and same-address atomics are
    // served one at a time: one counter update per wave and panel)
    const int nI = (p.n + kPanelRows - 1) / kPanelRows, lane = lane_id();
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int end = k == 0 ? b / kPanelRows : a / kPanelRows;
      const bool want = adj && (k == 0 || (a >> 10) != (b >> 10));
      unsigned long long todo = __ballot(want);
      while (todo) {                                   // wave-uniform
        const int leader = __builtin_ctzll(todo);
        const int which = __shfl(end, leader);
        const unsigned long long same = __ballot(want && end == which) & todo;
        const size_t bucket = (size_t)ut * nI + which;
        unsigned at = 0;
        if (lane == leader) at = atomicAdd(p.fecount + bucket, (unsigned)__popcll(same));
        at = __shfl(at, leader) + (unsigned)__popcll(same & ((1ull << lane) - 1ull));
        if ((same >> lane) & 1ull) {
          if (at < (unsigned)kFixBucket) p.fedges[bucket * kFixBucket + at] = e;
          else atomicOr(p.need_full, 1u);
        }
        todo &= ~same;
      }
    }
  }
}

// ---------------------------------------------------------------- degrees and neighbour lists
// One wave per row of G: degree (Eq. 10) and, for rows of at most kListCap neighbours, the
// neighbour indices as a compact uint16 list, so that the merge rounds touch a few hundred
// bytes per token instead of the whole bitmap row.  Denser rows keep using the bitmap.
constexpr int kListCap = 256;
// Where the p-th neighbour of a row is stored: lane sl of the 8-lane segment that later walks
// the row reads the 16 entries from sl * 16 on (of each half of 128), so the neighbours are dealt
// out to the lanes in turn and a short row occupies all eight lanes instead of the first one.
__host__ __device__ constexpr int list_slot(int p) { return (p & ~127) | ((p & 7) << 4) | ((p & 127) >> 3); }

__device__ __forceinline__ void lists_of_rows(const ShallowParams &p, int ut, int group) {
  const int n = p.n, Wp = p.Wp;
  const int lane = lane_id(), wave = threadIdx.x >> 6;
  const int row0 = (group * 4 + wave) * 4;
  constexpr int kHold = 8;                           // 16-byte pieces of a row a lane keeps: rows of up to 65536 bits
  for (int v = row0; v < row0 + 4 && v < n; ++v) {
    const u4 *row = reinterpret_cast<const u4 *>(p.G + ((size_t)ut * n + v) * Wp);
    u4 q[kHold];                                     // the row is read once
    int c = 0;
#pragma unroll
    for (int i = 0; i < kHold; ++i) {
      const int w4 = lane + i * kWave;
      q[i] = w4 < Wp / 4 ? row[w4] : u4{0, 0, 0, 0};
    }
#pragma unroll
    for (int i = 0; i < kHold; ++i) c += __popc(q[i][0]) + __popc(q[i][1]) + __popc(q[i][2]) + __popc(q[i][3]);
    int incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int x = __shfl_up(incl, o);
      if (lane >= o) incl += x;
    }
    const int deg = __shfl(incl, 63);
    if (lane == 0) {
      const size_t i = (size_t)ut * n + v;
      p.deg0[i] = deg;
      p.key[i] = ((uint32_t)deg << 16) | (uint32_t)(0xFFFF - v);
      p.alive[i] = v;
      p.slot[i] = -1;
      p.gone8[(size_t)ut * p.n16 + v] = 0;
      if (v == 0) p.counters[(size_t)ut * kCounters + C_ALIVE0] = n;
      if (p.deg_out[ut / p.U]) p.deg_out[ut / p.U][(size_t)(ut % p.U) * n + v] = deg;
    }
    if (deg <= kListCap) {
      uint16_t *dst = p.nbr + ((size_t)ut * n + v) * kListCap;
      int at = incl - c;                               // neighbours in the words of lower lanes
#pragma unroll
      for (int i = 0; i < kHold; ++i) {
        const int w4 = lane + i * kWave;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          uint32_t bits = q[i][j];
          while (bits) {
            const int t = __builtin_ctz(bits);
            bits &= bits - 1;
            dst[list_slot(at++)] = (uint16_t)((w4 * 4 + j) * 32 + t);
          }
        }
      }
    }
  }
}

// Fixed-size launch like shallow_mirror: the workgroups walk over the groups of 16 rows.
__global__ __launch_bounds__(256) void shallow_lists(ShallowParams p, int force) {
  if (!force && *p.need_full == 0) return;         // sparse graph: done by shallow_edge_lists
  const int groups = (p.n + 15) / 16;
  for (int group = blockIdx.x; group < groups; group += gridDim.x) lists_of_rows(p, blockIdx.y, group);
}

// ---------------------------------------------------------------- lists from edge records
// Sparse graphs: degrees (Eq. 10) and neighbour lists straight from the records of set bits
// shallow_gram and shallow_fixup left, without reading G.  One block per panel of 256 rows;
// the first 128 entries of every list are collected in LDS and written out in whole pieces.
// A record (a, b) of the panel's own segments puts b on the list of a.  G is symmetric and
// only computed from each row's own 1024-token tile on, so a record (a', b) of an earlier
// panel with b in a later tile also puts a' on the list of b: the block scans the segments
// of all earlier tiles' panels for its own chunk and keeps the records that end in its rows
// (inside a tile both orientations were computed and recorded).  Fill counts live in LDS;
// the order of a list is whatever the LDS atomics make it, which no consumer depends on.
// A row with more than kListCap neighbours, or a segment that ran full, raises need_full:
// shallow_mirror and shallow_lists then redo everything from the bitmap.
constexpr int kEdgeThreads = 1024;
constexpr int kEdgeLds = 128;                      // list entries per row collected in LDS; later ones go straight to memory

// kCap: the segment capacity when it is the smallest one (long sequences), else 0 = read it from
// the parameters; with the constant the compiler unrolls the record loop and batches its loads
// (0.14 ms against 0.21 ms on a 32k-token layer).
template <int kCap>
__global__ __launch_bounds__(kEdgeThreads) void shallow_edge_lists(ShallowParams p, int force) {
  __shared__ int cursor[kPanelRows];
  __shared__ __attribute__((aligned(16))) uint16_t part[kPanelRows][kEdgeLds];
  if (force || *p.need_full != 0) return;
  const int n = p.n, ut = blockIdx.y;
  const int nI = (n + kPanelRows - 1) / kPanelRows, nJc = (n + kChunkCols - 1) / kChunkCols;
  const int I = nI - 1 - (int)blockIdx.x;            // panels with more segments to scan first
  const int row0 = I * kPanelRows, Jm = row0 / kChunkCols;
  const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
  uint16_t *lists = p.nbr + ((size_t)ut * n + row0) * kListCap;
  if (tid < kPanelRows) cursor[tid] = 0;
  __syncthreads();
  auto add = [&](int row, int other) {
    const int r = row - row0;
    const int pos = atomicAdd(&cursor[r], 1);
    if (pos < kEdgeLds) part[r][list_slot(pos)] = (uint16_t)other;
    else if (pos < kListCap) lists[(size_t)r * kListCap + list_slot(pos)] = (uint16_t)other;
  };
  const int nown = 4 * (nJc - Jm);                   // (chunk, wave) segments of this panel
  const int nin = 16 * Jm;                           // (panel, wave) segments of earlier tiles for this tile's chunk
  constexpr int kBatch = 4;                          // segments a wave has in flight
  for (int k0 = wave * kBatch; k0 < nown + nin; k0 += (kEdgeThreads / 64) * kBatch) {
    const uint32_t *e[kBatch];
    int cnt[kBatch];
    bool own[kBatch];
    int most = 0;
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int k = k0 + u;
      own[u] = k < nown;
      const int kk = own[u] ? k : k - nown;
      const int J = own[u] ? Jm + (kk >> 2) : Jm;
      const int Ip = own[u] ? I : kk >> 2;
      const size_t seg = (((size_t)ut * nJc + J) * nI + Ip) * 4 + (kk & 3);
      const unsigned cn = k < nown + nin ? p.ecount[seg] : 0u;
      const int cap = kCap ? kCap : p.seg_cap;
      cnt[u] = cn < (unsigned)cap ? (int)cn : cap;
      e[u] = p.edges + seg * cap;
      most = cnt[u] > most ? cnt[u] : most;
    }
    for (int i0 = 0; i0 < most; i0 += kWave) {
      uint32_t rec[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) rec[u] = i0 + lane < cnt[u] ? e[u][i0 + lane] : 0xFFFFFFFFu;
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
        if (i0 + lane < cnt[u]) {
          const int a = (int)(rec[u] >> 16), b = (int)(rec[u] & 0xFFFFu);
          if (own[u]) add(a, b);
          else if (b >= row0 && b < row0 + kPanelRows) add(b, a);
        }
    }
  }
  {
    // pairs decided in double precision that have an end in this panel
    const size_t bucket = (size_t)ut * nI + I;
    const unsigned fn = p.fecount[bucket];
    const int fc = (int)(fn < (unsigned)kFixBucket ? fn : (unsigned)kFixBucket);
    const uint32_t *fe = p.fedges + bucket * kFixBucket;
    for (int i = tid; i < fc; i += kEdgeThreads) {
      const uint32_t rec = fe[i];
      const int a = (int)(rec >> 16), b = (int)(rec & 0xFFFFu);
      if (a >= row0 && a < row0 + kPanelRows) add(a, b);
      if ((a >> 10) != (b >> 10) && b >= row0 && b < row0 + kPanelRows) add(b, a);   // other tile: evaluated once
    }
  }
  __syncthreads();
  // the collected part of each list goes out in 16-byte pieces
  for (int k = tid; k < kPanelRows * (kEdgeLds / 8); k += kEdgeThreads) {
    const int r = k / (kEdgeLds / 8), piece = k % (kEdgeLds / 8);
    const int have = cursor[r] < kEdgeLds ? cursor[r] : kEdgeLds;
    // piece = half of a lane's 16 entries: entries (piece >> 1) + 8 j for j = 8 (piece & 1) ...
    if (row0 + r < n && have > (piece >> 1) + 64 * (piece & 1))
      *reinterpret_cast<u4 *>(lists + (size_t)r * kListCap + piece * 8) = *reinterpret_cast<const u4 *>(&part[r][piece * 8]);
  }
  if (tid < kPanelRows && row0 + tid < n) {
    const int v = row0 + tid, deg = cursor[tid];
    const size_t i = (size_t)ut * n + v;
    p.deg0[i] = deg;
    p.key[i] = ((uint32_t)deg << 16) | (uint32_t)(0xFFFF - v);
    p.alive[i] = v;
    p.slot[i] = -1;
    p.gone8[(size_t)ut * p.n16 + v] = 0;
    if (v == 0) p.counters[(size_t)ut * kCounters + C_ALIVE0] = n;
    if (p.deg_out[ut / p.U]) p.deg_out[ut / p.U][(size_t)(ut % p.U) * n + v] = deg;
    if (deg > kListCap) atomicOr(p.need_full, 1u);
  }
}

// ---------------------------------------------------------------- greedy merge
// Exact parallel form of the loop of Alg. 1.  With key(v) = (degree among remaining
// tokens, lower index first), the sequential loop always takes the remaining token of
// largest key.  A token whose key is the largest within two hops cannot lose a
// neighbour before it is taken itself (whoever removed one would be within two hops and
// would have needed a larger key), and tokens taken meanwhile are three or more hops away,
// so they do not touch its neighbourhood.  Each round therefore takes every two-hop
// maximum at once; sorting all picks by their key at pick time (which strictly decreases
// along the sequential loop) restores the codebook order.
//
// A round has four phases, each a loop over a list of tokens:
//   one-hop   m1[v] = largest key in v's closed neighbourhood; v is a candidate if it is its own
//   two-hop   a candidate whose neighbours' m1 never exceed its key is picked: its remaining
//             neighbours get its slot, are queued as `dying` and marked in the `dead` bitmap
//   degree    neighbours of dying tokens that stay lose one degree (Eq. 13)
//   compact   keys of dying tokens become 0, the list of remaining tokens is rebuilt
// The first kGridRounds rounds, where most tokens are still there, run as grid-wide kernels
// (one launch per phase, state in global memory); the remaining rounds run in one
// 1024-thread workgroup per problem with keys and the dead bitmap in LDS, separated by
// workgroup barriers only.  Rows are handled by 8-lane segments, four rows in flight.
constexpr int kMergeThreads = 1024;
constexpr int kSegW = 8;                 // lanes that share one row
constexpr int kGridRounds = 2;
static_assert(kGridRounds <= 2, "alive_slot and the per-round counters cover two grid rounds");
constexpr int kPhaseThreads = 256;
constexpr int kKeysInLds = 36 * 1024;   // tokens whose keys fit in LDS next to the other buffers

// The part of a row's neighbourhood one lane of a segment looks at: up to 16 entries of
// each half of the list, or (dense rows) every eighth 16-byte piece of the bitmap row.
struct Nbrs {
  u4 q[4];        // entries sl*16 .. +15 and 128 + sl*16 .. +15 of the list
  int cnt0, cnt1; // entries of this lane in each half; cnt0 = -1: dense row, walk the bitmap
  const u4 *row;
};

__device__ __forceinline__ Nbrs load_nbrs(const ShallowParams &p, size_t base, int v, int sl) {
  Nbrs r;
  const int d0 = p.deg0[base + v];
  const u4 *src = reinterpret_cast<const u4 *>(p.nbr + (base + v) * kListCap + sl * 16);
  r.q[0] = src[0];    // unconditional: the slot exists for every row, and the loads
  r.q[1] = src[1];    // then do not wait for the degree
  r.row = reinterpret_cast<const u4 *>(p.G + (base + v) * p.Wp);
  // entries sl, sl + 8, ... of each half belong to this lane (list_slot)
  const int h0 = d0 < 128 ? d0 : 128, h1 = d0 - 128;
  const int c0 = (h0 - sl + 7) >> 3, c1 = (h1 - sl + 7) >> 3;
  r.cnt0 = d0 <= kListCap ? (c0 < 0 ? 0 : c0) : -1;
  r.cnt1 = d0 <= kListCap && h1 > 0 ? (c1 < 0 ? 0 : c1) : 0;
  if (r.cnt1 > 0) {
    r.q[2] = src[16];
    r.q[3] = src[17];
  }
  return r;
}

// Calls f(b) for every neighbour b in this lane's part of the row.
template <typename F>
__device__ __forceinline__ void for_nbrs(const ShallowParams &p, const Nbrs &r, int sl, F f) {
  if (r.cnt0 >= 0) {
    // most rows are short: every fourth entry the wave checks whether any lane has more
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (j > 0 && (j & 3) == 0 && __ballot(j < r.cnt0) == 0) break;
      if (j < r.cnt0) f((int)((r.q[j >> 3][(j >> 1) & 3] >> (16 * (j & 1))) & 0xFFFFu));
    }
    if (r.cnt1 > 0) {
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        if (j > 0 && (j & 3) == 0 && __ballot(j < r.cnt1) == 0) break;
        if (j < r.cnt1) f((int)((r.q[2 + (j >> 3)][(j >> 1) & 3] >> (16 * (j & 1))) & 0xFFFFu));
      }
    }
  } else {
    for (int w4 = sl; w4 < p.Wp / 4; w4 += kSegW) {
      const u4 q = r.row[w4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        uint32_t bits = q[j];
        while (bits) {
          const int t = __builtin_ctz(bits);
          bits &= bits - 1;
          f((w4 * 4 + j) * 32 + t);
        }
      }
    }
  }
}

// Lane exchanges inside an 8-lane segment by DPP (no LDS round trip): the two quad
// permutations, then the mirror of the eight lanes, which pairs each lane with one of the
// other quad.
static_assert(kSegW == 8, "the segment reductions are written for eight lanes");
__device__ __forceinline__ uint32_t seg_xchg(uint32_t v, int step) {
  return step == 0 ? (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xF, 0xF, false)     // quad_perm [1,0,3,2]
         : step == 1 ? (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xF, 0xF, false)   // quad_perm [2,3,0,1]
                     : (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xF, 0xF, false); // row_half_mirror
}
__device__ __forceinline__ uint32_t seg_max(uint32_t v) {   // over a segment, result in every lane
#pragma unroll
  for (int step = 0; step < 3; ++step) {
    const uint32_t x = seg_xchg(v, step);
    v = x > v ? x : v;
  }
  return v;
}
__device__ __forceinline__ int seg_sum(int v) {             // over a segment, result in every lane
#pragma unroll
  for (int step = 0; step < 3; ++step) v += (int)seg_xchg((uint32_t)v, step);
  return v;
}

// The same walk four entries at a time: f4(b, ok) gets four neighbour slots of this lane
// (ok[t] false: slot t is past the end of the lane's part and b[t] is not a token) and can issue
// its look-ups together, so that a row costs a few memory round trips instead of one per
// entry; the wave stops as soon as no lane has entries left.  f1(b) handles one neighbour of
// a dense row (bitmap walk).
template <typename F4, typename F1>
__device__ __forceinline__ void for_nbrs4(const ShallowParams &p, const Nbrs &r, int sl, F4 f4, F1 f1) {
  if (r.cnt0 >= 0) {
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int cnt = half ? r.cnt1 : r.cnt0;
      if (__ballot(cnt > 0) == 0) break;               // wave-uniform
#pragma unroll
      for (int j0 = 0; j0 < 16; j0 += 4) {
        if (__ballot(j0 < cnt) == 0) break;            // wave-uniform
        int b[4];
        bool ok[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int j = j0 + t;
          ok[t] = j < cnt;
          b[t] = (int)((r.q[2 * half + (j >> 3)][(j >> 1) & 3] >> (16 * (j & 1))) & 0xFFFFu);
        }
        f4(b, ok);
      }
    }
  } else {
    for (int w4 = sl; w4 < p.Wp / 4; w4 += kSegW) {
      const u4 q = r.row[w4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        uint32_t bits = q[j];
        while (bits) {
          const int t = __builtin_ctz(bits);
          bits &= bits - 1;
          f1((w4 * 4 + j) * 32 + t);
        }
      }
    }
  }
}

// Where the state of one problem lives for the running kernel (LDS or global memory), and
// which segments of the launch work on it: segment `seg` of `nsegs`, a wave's segments
// being consecutive.
struct MergeView {
  uint32_t *key;        // (remaining degree << 16) | (0xFFFF - index); 0 once removed
  uint32_t *dead;       // bit v set once token v has been given a slot
  int *n_alive, *n_cand, *n_dying, *n_picks;
  int seg, nsegs, sl;
};

__device__ __forceinline__ void phase_onehop(const ShallowParams &p, size_t base, const MergeView &w,
                                             const int *alive, int nalive) {
  constexpr int kPer = kWave / kSegW;
  uint32_t *m1 = p.m1 + base;
  int *cand = p.cand + base;
  const int lane = lane_id();
  for (int i0 = w.seg - w.seg % kPer; i0 < nalive; i0 += 4 * w.nsegs) {
    int vv[4];
    bool on[4];
    Nbrs r[4];
    uint32_t m[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + w.seg % kPer + k * w.nsegs;
      on[k] = i < nalive;
      vv[k] = on[k] ? alive[i] : 0;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) r[k] = load_nbrs(p, base, vv[k], w.sl);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      uint32_t mk = on[k] ? w.key[vv[k]] : 0;          // a token is its own neighbour
      if (on[k]) {
        const int self = vv[k];
        for_nbrs4(p, r[k], w.sl,
                  [&](const int *b, const bool *ok) {
                    uint32_t kk[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) kk[t] = w.key[ok[t] ? b[t] : self];   // own key again: harmless
#pragma unroll
                    for (int t = 0; t < 4; ++t) mk = kk[t] > mk ? kk[t] : mk;
                  },
                  [&](int b) { const uint32_t kk = w.key[b]; mk = kk > mk ? kk : mk; });
      }
      m[k] = seg_max(mk);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const bool lead = w.sl == 0 && on[k];
      if (lead) m1[vv[k]] = m[k];
      const bool is_cand = lead && m[k] == w.key[vv[k]];
      const unsigned long long mk = __ballot(is_cand);     // one counter update per wave
      if (mk) {
        int at = 0;
        if (lane == __builtin_ctzll(mk)) at = atomicAdd(w.n_cand, __popcll(mk));
        at = __shfl(at, __builtin_ctzll(mk));
        if (is_cand) cand[at + __popcll(mk & ((1ull << lane) - 1ull))] = vv[k];
      }
    }
  }
}

// kBytes: `dead` is the byte array of the grid rounds (plain stores); else the bitmap of the tail
// kFlight: candidates a segment works on at once
template <bool kBytes, int kFlight>
__device__ __forceinline__ void phase_twohop(const ShallowParams &p, size_t base, const MergeView &w, int ncand) {
  constexpr int kPer = kWave / kSegW;
  const uint32_t *m1 = p.m1 + base;
  const int *cand = p.cand + base;
  int *slot = p.slot + base, *dying = p.dying + base, *pick_vert = p.pick_vert + base;
  uint32_t *pick_key = p.pick_key + base;
  const int lane = lane_id();
  for (int i0 = w.seg - w.seg % kPer; i0 < ncand; i0 += kFlight * w.nsegs) {
    int uv[kFlight], rem[kFlight];
    bool on[kFlight];
    uint32_t ku[kFlight], m[kFlight];
    Nbrs r[kFlight];
#pragma unroll
    for (int k = 0; k < kFlight; ++k) {
      const int i = i0 + w.seg % kPer + k * w.nsegs;
      on[k] = i < ncand;
      uv[k] = on[k] ? cand[i] : 0;
    }
#pragma unroll
    for (int k = 0; k < kFlight; ++k) {
      ku[k] = on[k] ? w.key[uv[k]] : 0xFFFFFFFFu;
      r[k] = load_nbrs(p, base, uv[k], w.sl);
    }
#pragma unroll
    for (int k = 0; k < kFlight; ++k) {
      uint32_t mk = 0;
      int rk = 0;                                    // remaining neighbours in this lane's part
      // remaining = key != 0 (keys only change in the later phases of the round)
      if (on[k]) {
        const int self = uv[k];
        for_nbrs4(p, r[k], w.sl,
                  [&](const int *b, const bool *ok) {
                    uint32_t kk[4], q[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) kk[t] = w.key[ok[t] ? b[t] : self];
                    bool there[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                      there[t] = ok[t] && kk[t] != 0;
                      q[t] = m1[there[t] ? b[t] : self];
                    }
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                      if (there[t]) { mk = q[t] > mk ? q[t] : mk; ++rk; }
                  },
                  [&](int b) {
                    if (w.key[b] != 0) { const uint32_t q = m1[b]; mk = q > mk ? q : mk; ++rk; }
                  });
      }
      m[k] = seg_max(mk);
      rem[k] = rk;
    }
#pragma unroll
    for (int k = 0; k < kFlight; ++k) {
      const bool picked = on[k] && m[k] == ku[k];
      // one update of each counter per wave: picks by the segment leaders, dying tokens by all lanes
      const unsigned long long pk = __ballot(picked && w.sl == 0);
      if (pk != 0) {                                 // wave-uniform
        int s = 0;
        {
          int at = 0;
          if (lane == __builtin_ctzll(pk)) at = atomicAdd(w.n_picks, __popcll(pk));
          at = __shfl(at, __builtin_ctzll(pk));
          if (picked && w.sl == 0) {
            s = at + __popcll(pk & ((1ull << lane) - 1ull));
            pick_key[s] = ku[k];
            pick_vert[s] = uv[k];
          }
        }
        s = __shfl(s, lane & ~(kSegW - 1));
        const int mine = picked ? rem[k] : 0;
        int incl = mine;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
          const int x = __shfl_up(incl, o);
          if (lane >= o) incl += x;
        }
        int at = 0;
        if (lane == kWave - 1) at = atomicAdd(w.n_dying, incl);
        at = __shfl(at, kWave - 1) + incl - mine;
        auto take = [&](int b) {
          slot[b] = s;
          if (kBytes) reinterpret_cast<uint8_t *>(w.dead)[b] = 1;
          else atomicOr(&w.dead[b >> 5], 1u << (b & 31));
          dying[at++] = b;
        };
        if (picked) {
          const int self = uv[k];
          for_nbrs4(p, r[k], w.sl,
                    [&](const int *b, const bool *ok) {
                      uint32_t kk[4];
#pragma unroll
                      for (int t = 0; t < 4; ++t) kk[t] = w.key[ok[t] ? b[t] : self];
#pragma unroll
                      for (int t = 0; t < 4; ++t)
                        if (ok[t] && kk[t] != 0) take(b[t]);
                    },
                    [&](int b) { if (w.key[b] != 0) take(b); });
        }
      }
    }
  }
}

__device__ __forceinline__ void phase_degree(const ShallowParams &p, size_t base, const MergeView &w, int ndying) {
  constexpr int kPer = kWave / kSegW;
  const int *dying = p.dying + base;
  for (int i0 = w.seg - w.seg % kPer; i0 < ndying; i0 += 4 * w.nsegs) {
    Nbrs r[4];
    bool on[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + w.seg % kPer + k * w.nsegs;
      on[k] = i < ndying;
      r[k] = load_nbrs(p, base, on[k] ? dying[i] : 0, w.sl);
    }
    auto drop = [&](int b) {   // tokens that stay: not marked dead (the bitmap also covers earlier rounds)
      if (!((w.dead[b >> 5] >> (b & 31)) & 1u)) atomicSub(&w.key[b], 1u << 16);
    };
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (on[k])
        for_nbrs4(p, r[k], w.sl,
                  [&](const int *b, const bool *ok) {
                    uint32_t word[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) word[t] = w.dead[(ok[t] ? b[t] : 0) >> 5];
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                      if (ok[t] && !((word[t] >> (b[t] & 31)) & 1u)) atomicSub(&w.key[b[t]], 1u << 16);
                  },
                  drop);
  }
}

// Eq. 13 the other way round: every token of the list counts its neighbours that are still
// there (dead bitmap).  Cheaper than phase_degree when more tokens left than stayed.
__device__ __forceinline__ void phase_recount(const ShallowParams &p, size_t base, const MergeView &w,
                                              const int *alive, int nalive) {
  constexpr int kPer = kWave / kSegW;
  for (int i0 = w.seg - w.seg % kPer; i0 < nalive; i0 += 4 * w.nsegs) {
    int vv[4];
    bool on[4];
    Nbrs r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + w.seg % kPer + k * w.nsegs;
      on[k] = i < nalive;
      vv[k] = on[k] ? alive[i] : 0;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) r[k] = load_nbrs(p, base, vv[k], w.sl);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      int c = 0;
      if (on[k])
        for_nbrs4(p, r[k], w.sl,
                  [&](const int *b, const bool *ok) {
                    uint32_t word[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) word[t] = w.dead[(ok[t] ? b[t] : 0) >> 5];
#pragma unroll
                    for (int t = 0; t < 4; ++t) c += ok[t] && !((word[t] >> (b[t] & 31)) & 1u);
                  },
                  [&](int b) { c += !((w.dead[b >> 5] >> (b & 31)) & 1u); });
      c = seg_sum(c);
      if (on[k] && w.sl == 0) w.key[vv[k]] = ((uint32_t)c << 16) | (uint32_t)(0xFFFF - vv[k]);
    }
  }
}

__device__ __forceinline__ MergeView global_view(const ShallowParams &p, int ut, int round) {
  MergeView w;
  const size_t base = (size_t)ut * p.n;
  int *cnt = p.counters + (size_t)ut * kCounters;
  w.key = p.key + base;
  w.dead = reinterpret_cast<uint32_t *>(p.gone8 + (size_t)ut * p.n16);
  w.n_alive = cnt + alive_slot(round);
  w.n_cand = cnt + (round ? C_CAND1 : C_CAND);
  w.n_dying = cnt + (round ? C_DYING1 : C_DYING);
  w.n_picks = cnt + C_PICKS;
  w.seg = (blockIdx.x * blockDim.x + threadIdx.x) / kSegW;
  w.nsegs = gridDim.x * blockDim.x / kSegW;
  w.sl = threadIdx.x & (kSegW - 1);
  return w;
}

// Grid-wide phases of round `round` (blockIdx.y = problem).  The list of remaining tokens
// alternates between the `alive` and `alive2` rows, its length between counters 0 and 1.
// With dynamic LDS for n keys the block first copies the keys of its problem there: the
// phase is bound by the random key look-ups, which LDS serves several times faster than L2.
__global__ __launch_bounds__(kMergeThreads) void merge_onehop(ShallowParams p, int round, int keys_in_lds) {
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  const int ut = blockIdx.y;
  const size_t base = (size_t)ut * p.n;
  MergeView w = global_view(p, ut, round);
  const int nalive = *w.n_alive;
  if ((int)(blockIdx.x * blockDim.x / kSegW) >= nalive) return;      // block-uniform: no work for this block
  if (keys_in_lds) {
    if ((p.n & 3) == 0) {                             // rows of the key array are then 16-byte aligned
      const u4 *src = reinterpret_cast<const u4 *>(p.key + base);
      for (int i = threadIdx.x; i < p.n / 4; i += blockDim.x) reinterpret_cast<u4 *>(lds)[i] = src[i];
    } else {
      for (int i = threadIdx.x; i < p.n; i += blockDim.x) lds[i] = p.key[base + i];
    }
    __syncthreads();
    w.key = lds;
  }
  phase_onehop(p, base, w, (round & 1 ? p.alive2 : p.alive) + base, nalive);
}
// Two-hop phase of a grid round.  When candidates are few (hundreds per problem: they then
// have the longest lists, and every look-up here is a trip to L2) a wave takes one candidate:
// with four slots per lane its whole list is one look-up step for the keys and one for their
// one-hop maxima, whatever its length.
__global__ __launch_bounds__(kPhaseThreads) void merge_twohop(ShallowParams p, int round) {
  const int ut = blockIdx.y, lane = lane_id();
  const size_t base = (size_t)ut * p.n;
  int *cnt = p.counters + (size_t)ut * kCounters;
  const int ncand = cnt[round ? C_CAND1 : C_CAND];
  int *n_dying = cnt + (round ? C_DYING1 : C_DYING), *n_picks = cnt + C_PICKS;
  const uint32_t *key = p.key + base, *m1 = p.m1 + base;
  const int *cand = p.cand + base;
  int *slot = p.slot + base, *dying = p.dying + base, *pick_vert = p.pick_vert + base;
  uint32_t *pick_key = p.pick_key + base;
  uint8_t *gone = p.gone8 + (size_t)ut * p.n16;
  const int wave0 = (blockIdx.x * blockDim.x + threadIdx.x) / kWave, nwaves = gridDim.x * blockDim.x / kWave;
  if (ncand > 2 * nwaves) {
    // many candidates (isolated tokens are all candidates): short lists, eight lanes per row
    const MergeView w = global_view(p, ut, round);
    phase_twohop<true, 4>(p, base, w, ncand);
    return;
  }
  for (int i = wave0; i < ncand; i += nwaves) {      // wave-uniform
    const int u = cand[i];
    const uint32_t ku = key[u];
    const int d0 = p.deg0[base + u];
    int b[4];
    bool there[4] = {false, false, false, false};
    uint32_t mk = 0;
    int rk = 0;                                       // remaining neighbours in this lane's slots
    const u4 *row = reinterpret_cast<const u4 *>(p.G + (base + u) * p.Wp);
    if (d0 <= kListCap) {
      const uint2 raw = *reinterpret_cast<const uint2 *>(p.nbr + (base + u) * kListCap + 4 * lane);
      uint32_t kk[4], q[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int s = 4 * lane + t;                  // slot -> position in the list (inverse of list_slot)
        const int at = (s & ~127) | ((s & 15) << 3) | ((s & 127) >> 4);
        b[t] = (int)(((t < 2 ? raw.x : raw.y) >> (16 * (t & 1))) & 0xFFFFu);
        there[t] = at < d0;
        kk[t] = key[there[t] ? b[t] : u];
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        there[t] = there[t] && kk[t] != 0;           // remaining = key != 0 (keys change later in the round)
        q[t] = m1[there[t] ? b[t] : u];
      }
#pragma unroll
      for (int t = 0; t < 4; ++t)
        if (there[t]) { mk = q[t] > mk ? q[t] : mk; ++rk; }
    } else {
      for (int w4 = lane; w4 < p.Wp / 4; w4 += kWave) {
        const u4 qw = row[w4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          uint32_t bits = qw[j];
          while (bits) {
            const int t = __builtin_ctz(bits);
            bits &= bits - 1;
            const int v = (w4 * 4 + j) * 32 + t;
            if (key[v] != 0) { const uint32_t q = m1[v]; mk = q > mk ? q : mk; ++rk; }
          }
        }
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const uint32_t x = __shfl_xor(mk, o);
      mk = x > mk ? x : mk;
    }
    if (mk != ku) continue;                           // wave-uniform: not the largest key within two hops
    int s = 0;
    if (lane == 0) {
      s = atomicAdd(n_picks, 1);
      pick_key[s] = ku;
      pick_vert[s] = u;
    }
    s = __shfl(s, 0);
    int incl = rk;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
      const int x = __shfl_up(incl, o);
      if (lane >= o) incl += x;
    }
    int at = 0;
    if (lane == kWave - 1) at = atomicAdd(n_dying, incl);
    at = __shfl(at, kWave - 1) + incl - rk;
    auto take = [&](int v) {
      slot[v] = s;
      gone[v] = 1;
      dying[at++] = v;
    };
    if (d0 <= kListCap) {
#pragma unroll
      for (int t = 0; t < 4; ++t)
        if (there[t]) take(b[t]);
    } else {
      for (int w4 = lane; w4 < p.Wp / 4; w4 += kWave) {
        const u4 qw = row[w4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          uint32_t bits = qw[j];
          while (bits) {
            const int t = __builtin_ctz(bits);
            bits &= bits - 1;
            const int v = (w4 * 4 + j) * 32 + t;
            if (key[v] != 0) take(v);
          }
        }
      }
    }
  }
}
// End of a grid round.  Tokens marked dead get key 0; every other token of the list counts
// its neighbours that are not dead (its new degree, Eq. 13: with most tokens leaving in the
// first rounds, recounting the few that stay is cheaper than subtracting at every
// neighbour of every leaving token), gets its new key and moves to the other list.
__global__ __launch_bounds__(kMergeThreads) void merge_update(ShallowParams p, int round) {
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];     // dead flags of the problem, one byte per token
  constexpr int kPer = kWave / kSegW;
  const int ut = blockIdx.y, lane = lane_id(), n = p.n;
  const size_t base = (size_t)ut * n;
  int *cnt = p.counters + (size_t)ut * kCounters;
  const int nalive = cnt[alive_slot(round)];
  const int seg = (blockIdx.x * blockDim.x + threadIdx.x) / kSegW, nsegs = gridDim.x * blockDim.x / kSegW;
  const int sl = threadIdx.x & (kSegW - 1);
  if ((int)(blockIdx.x * blockDim.x / kSegW) >= nalive) return;
  {
    const u4 *src8 = reinterpret_cast<const u4 *>(p.gone8 + (size_t)ut * p.n16);
    for (int i = threadIdx.x; i < p.n16 / 16; i += blockDim.x) reinterpret_cast<u4 *>(lds)[i] = src8[i];
  }
  __syncthreads();
  const uint8_t *dead = reinterpret_cast<const uint8_t *>(lds);
  const int *src = (round & 1 ? p.alive2 : p.alive) + base;
  int *dst = (round & 1 ? p.alive : p.alive2) + base;
  uint32_t *key = p.key + base;
  __shared__ int wave_total[kMergeThreads / kWave], block_at;
  const int wave = threadIdx.x / kWave;
  // block-uniform trip count (the appends below synchronise the block): waves past the end
  // of the list run with all lanes idle
  for (int b0 = blockIdx.x * blockDim.x / kSegW; b0 < nalive; b0 += 4 * nsegs) {
    const int i0 = b0 + wave * kPer;
    int vv[4];
    bool live[4];
    Nbrs r[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + seg % kPer + k * nsegs;
      vv[k] = i < nalive ? src[i] : -1;
      live[k] = vv[k] >= 0 && !dead[vv[k]];
      if (vv[k] >= 0 && !live[k] && sl == 0) key[vv[k]] = 0;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) r[k] = load_nbrs(p, base, live[k] ? vv[k] : 0, sl);
    unsigned long long mk[4];
    int mine = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      int c = 0;
      if (live[k])
        for_nbrs4(p, r[k], sl,
                  [&](const int *b, const bool *ok) {
                    uint8_t gone[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) gone[t] = dead[ok[t] ? b[t] : 0];
#pragma unroll
                    for (int t = 0; t < 4; ++t) c += ok[t] && !gone[t];
                  },
                  [&](int b) { c += !dead[b]; });
      c = seg_sum(c);
      const bool lead = live[k] && sl == 0;
      if (lead) key[vv[k]] = ((uint32_t)c << 16) | (uint32_t)(0xFFFF - vv[k]);
      mk[k] = __ballot(lead);
      mine += __popcll(mk[k]);
    }
    // one counter update per block and trip: same-address atomics are served one at a time
    if (lane == 0) wave_total[wave] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
      int t = 0;
      for (int q = 0; q < kMergeThreads / kWave; ++q) t += wave_total[q];
      block_at = t ? atomicAdd(&cnt[alive_slot(round + 1)], t) : 0;
    }
    __syncthreads();
    int at = block_at;
    for (int q = 0; q < wave; ++q) at += wave_total[q];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (live[k] && sl == 0) dst[at + __popcll(mk[k] & ((1ull << lane) - 1ull))] = vv[k];
      at += __popcll(mk[k]);
    }
    __syncthreads();                                 // wave_total is rewritten by the next trip
  }
}
template <int DT>
__device__ __forceinline__ void emit_code(const ShallowParams &p, int ut, int vert, int r) {
  typedef typename Elem<DT>::type T;
  const int t = ut / p.U, u = ut % p.U;
  const T *src = reinterpret_cast<const T *>(x_row(p, ut, vert));
  T *dst = reinterpret_cast<T *>(p.C[t]) + ((size_t)u * p.cap + r) * kHeadDim;
  const double m = p.m64[(size_t)ut * p.n + vert];
  for (int d = lane_id(); d < kHeadDim; d += kWave) {
    const double x = (double)Elem<DT>::to_float(src[d]);
    dst[d] = Elem<DT>::from_float(m > 0.0 ? (float)(x / m) : 0.f);
  }
}

#define MERGE_TICK(k)                          \
  if (tid == 0) {                              \
    const long long now_ = wall_clock64();     \
    cnt[6 + (k)] += (int)(now_ - tick_);       \
    tick_ = now_;                              \
  }

// Remaining rounds and the outputs, one workgroup per problem.
__global__ __launch_bounds__(kMergeThreads) void shallow_merge(ShallowParams p) {
  extern __shared__ __attribute__((aligned(16))) uint32_t lds[];
  __shared__ int sh_n[4];                     // alive, candidates, dying, picks
  const int ut = blockIdx.x, n = p.n, tid = threadIdx.x;
  const int lane = lane_id(), wave = tid >> 6;
  const size_t base = (size_t)ut * n;
  const bool keys_in_lds = n <= kKeysInLds;
  const int dead_words = (n + 31) / 32;
  int *cnt = p.counters + (size_t)ut * kCounters;
  MergeView w;
  w.key = keys_in_lds ? lds : p.key + base;
  w.dead = keys_in_lds ? lds + ((n + 3) & ~3) : p.gone + base;
  w.n_alive = &sh_n[0]; w.n_cand = &sh_n[1]; w.n_dying = &sh_n[2]; w.n_picks = &sh_n[3];
  w.seg = tid / kSegW; w.nsegs = kMergeThreads / kSegW; w.sl = tid & (kSegW - 1);
  int *slot = p.slot + base, *dying = p.dying + base;
  // the list the last grid round left behind; this kernel compacts it in place
  int *alive = (kGridRounds & 1 ? p.alive2 : p.alive) + base;
  long long tick_ = 0;
  if (tid == 0) tick_ = wall_clock64();

  if (keys_in_lds) {
    if ((n & 3) == 0) {                               // rows of the key array are then 16-byte aligned
      const u4 *src = reinterpret_cast<const u4 *>(p.key + base);
      for (int i = tid; i < n / 4; i += kMergeThreads) reinterpret_cast<u4 *>(w.key)[i] = src[i];
    } else {
      for (int v = tid; v < n; v += kMergeThreads) w.key[v] = p.key[base + v];
    }
  }
  {
    // the grid rounds keep one byte (0 or 1) per token; this kernel works on a bitmap
    const u4 *g8 = reinterpret_cast<const u4 *>(p.gone8 + (size_t)ut * p.n16);   // 16-byte aligned rows of n16 bytes
    for (int i = tid; i < dead_words; i += kMergeThreads) {
      uint32_t word = 0;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const u4 q = 2 * i + h < p.n16 / 16 ? g8[2 * i + h] : u4{0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 4; ++j)                    // four 0/1 bytes -> four bits
          word |= (((q[j] & 0x01010101u) * 0x01020408u) >> 24 & 0xFu) << (16 * h + 4 * j);
      }
      w.dead[i] = word;
    }
  }
  if (tid == 0) { sh_n[0] = cnt[alive_slot(kGridRounds)]; sh_n[1] = 0; sh_n[2] = 0; sh_n[3] = cnt[C_PICKS]; }
  __syncthreads();
  MERGE_TICK(0)

  // every round removes at least the token of largest key, so n rounds always suffice;
  // the bound only guards against a corrupted adjacency matrix
  int round = kGridRounds;
  for (; round <= n + kGridRounds; ++round) {
    const int nalive = sh_n[0];
    if (nalive == 0) break;
    phase_onehop(p, base, w, alive, nalive);
    __syncthreads();
    MERGE_TICK(2)
    phase_twohop<false, 2>(p, base, w, sh_n[1]);
    __syncthreads();
    MERGE_TICK(4)
    const int ndying = sh_n[2];
    for (int i = tid; i < ndying; i += kMergeThreads) w.key[dying[i]] = 0;
    if (tid == 0) { sh_n[0] = 0; sh_n[1] = 0; sh_n[2] = 0; }
    __syncthreads();
    // survivors, compacted in place (each wave appends its survivors with one LDS atomic;
    // the write index never passes the read index of a later chunk because chunks are
    // consumed by all waves in lock step)
    for (int i0 = 0; i0 < nalive; i0 += kMergeThreads) {
      const int i = i0 + tid;
      const int v = i < nalive ? alive[i] : -1;
      const bool live = v >= 0 && w.key[v] != 0;
      __syncthreads();
      const unsigned long long mk = __ballot(live);
      int at = 0;
      if (lane == 0 && mk) at = atomicAdd(&sh_n[0], __popcll(mk));
      at = __shfl(at, 0);
      if (live) alive[at + __popcll(mk & ((1ull << lane) - 1ull))] = v;
      __syncthreads();
    }
    MERGE_TICK(0)
    // degrees of the survivors (Eq. 13): subtract at the neighbours of the tokens that left,
    // or recount at the tokens that stayed, whichever list is shorter
    if (ndying <= nalive - ndying) phase_degree(p, base, w, ndying);
    else phase_recount(p, base, w, alive, nalive - ndying);
    __syncthreads();
    MERGE_TICK(6)
  }
  if (tid == 0) cnt[C_ROUNDS] = round;
  if (sh_n[0] != 0) return;                      // did not converge: n_codes stays -1

  const int P = sh_n[3];
  if (tid == 0) cnt[C_PICKS] = P;
  MERGE_TICK(8)

  const int t = ut / p.U, u = ut % p.U;
  if (tid == 0) {
    p.n_codes[t][u] = P < p.cap ? P : p.cap;
    if (p.n_found[t]) p.n_found[t][u] = P;
  }
  MERGE_TICK(9)
}

// Codebook order: the picks of a problem sorted by decreasing key at pick time (keys are
// distinct: they carry the token index).  One workgroup per problem: least-significant-digit
// radix sort, four stable passes of 8 bits over (key, pick number) pairs that ping-pong
// between two pairs of arrays left free by the merge.  A pass counts the digits, then walks
// the items in order, 1024 at a time: lanes with the same digit find each other with eight
// ballots, waves exchange their digit counts through LDS.
constexpr int kRankThreads = 1024;

__global__ __launch_bounds__(kRankThreads) void shallow_rank(ShallowParams p) {
  constexpr int kWaves = kRankThreads / 64;
  __shared__ int base_of[256];                       // next output position of each digit
  __shared__ int wave_cnt[kWaves][256];              // items of each digit per wave in the current tile
  __shared__ int scan_tmp[256];
  const int ut = blockIdx.x, tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
  const size_t base = (size_t)ut * p.n;
  if (p.n_codes[ut / p.U][ut % p.U] < 0) return;     // construction did not finish
  const int P = p.counters[(size_t)ut * kCounters + C_PICKS];
  uint32_t *keyA = p.pick_key + base, *keyB = p.m1 + base;
  uint32_t *valA = reinterpret_cast<uint32_t *>(p.cand + base), *valB = reinterpret_cast<uint32_t *>(p.dying + base);
  for (int s = tid; s < P; s += kRankThreads) valA[s] = (uint32_t)s;
  __syncthreads();
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 8 * pass;
    const uint32_t *kin = pass & 1 ? keyB : keyA, *vin = pass & 1 ? valB : valA;
    uint32_t *kout = pass & 1 ? keyA : keyB, *vout = pass & 1 ? valA : valB;
    // digit 255 - byte: larger keys first
    if (tid < 256) base_of[tid] = 0;
    __syncthreads();
    for (int s = tid; s < P; s += kRankThreads) atomicAdd(&base_of[255 - ((kin[s] >> shift) & 255u)], 1);
    __syncthreads();
    // exclusive prefix sum over the 256 counters
    if (tid < 256) scan_tmp[tid] = base_of[tid];
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
      int x = 0;
      if (tid < 256 && tid >= o) x = scan_tmp[tid - o];
      __syncthreads();
      if (tid < 256) scan_tmp[tid] += x;
      __syncthreads();
    }
    if (tid < 256) base_of[tid] = scan_tmp[tid] - base_of[tid];
    __syncthreads();
    for (int s0 = 0; s0 < P; s0 += kRankThreads) {
      const int s = s0 + tid;
      const bool on = s < P;
      const uint32_t k = on ? kin[s] : 0u, v = on ? vin[s] : 0u;
      const int d = on ? 255 - (int)((k >> shift) & 255u) : 256;      // 256: no item
      for (int j = tid; j < kWaves * 256; j += kRankThreads) (&wave_cnt[0][0])[j] = 0;
      // lanes of the wave with the same digit
      unsigned long long peers = __ballot(on);
#pragma unroll
      for (int bit = 0; bit < 8; ++bit) {
        const unsigned long long m = __ballot((d >> bit) & 1);
        peers &= ((d >> bit) & 1) ? m : ~m;
      }
      const int before = __popcll(peers & ((1ull << lane) - 1ull));
      __syncthreads();                                // counters cleared
      if (on && before == 0) wave_cnt[wave][d] = __popcll(peers);
      __syncthreads();
      if (on) {
        int at = base_of[d] + before;
        for (int w = 0; w < wave; ++w) at += wave_cnt[w][d];
        kout[at] = k;
        vout[at] = v;
      }
      __syncthreads();
      if (tid < 256) {
        int t = 0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) t += wave_cnt[w][tid];
        base_of[tid] += t;
      }
      __syncthreads();
    }
  }
  // four passes: the sorted pairs are back in the first pair of arrays
  for (int r = tid; r < P; r += kRankThreads) {
    const int s = (int)valA[r];
    p.rank[base + s] = r;
    p.rank_vert[base + r] = p.pick_vert[base + s];
  }
}

// References (Eq. 12, renumbered in codebook order) and codebook entries (Eq. 11), grid-wide.
__global__ __launch_bounds__(256) void shallow_emit(ShallowParams p) {
  const int ut = blockIdx.y, n = p.n;
  const size_t base = (size_t)ut * n;
  const int t = ut / p.U, u = ut % p.U;
  const int stored = p.n_codes[t][u];
  if (stored < 0) return;                        // the merge did not finish
  const int *rank = p.rank + base, *slot = p.slot + base, *rank_vert = p.rank_vert + base;
  const int lane = lane_id();
  for (int v0 = blockIdx.x * 256 + threadIdx.x - lane; v0 < n; v0 += gridDim.x * 256) {
    const int v = v0 + lane;
    const int r = v < n ? rank[slot[v]] : 0;
    if (v < n) p.ref[t][(size_t)u * n + v] = r;
    const bool cut = v < n && r >= p.cap;
    const unsigned long long mk = __ballot(cut);         // one counter update per wave
    if (mk) {
      unsigned at = 0;
      if (lane == __builtin_ctzll(mk)) at = atomicAdd(p.ovf_cnt + ut, (unsigned)__popcll(mk));
      at = __shfl(at, __builtin_ctzll(mk));
      if (cut) p.ovf[base + at + __popcll(mk & ((1ull << lane) - 1ull))] = (uint32_t)v;
    }
  }
  for (int r = blockIdx.x * 4 + (threadIdx.x >> 6); r < stored; r += gridDim.x * 4) {
    const int vert = rank_vert[r];
    if (p.dtype == SPINDLE_F16) emit_code<SPINDLE_F16>(p, ut, vert, r);
    else if (p.dtype == SPINDLE_BF16) emit_code<SPINDLE_BF16>(p, ut, vert, r);
    else emit_code<SPINDLE_F32>(p, ut, vert, r);
  }
}

// ---------------------------------------------------------------- codebook cap
// A token whose entry was cut goes to the stored entry of highest cosine (Eq. 4), lowest
// entry index on ties, decided as the double-precision evaluation decides it.
//
// shallow_assign finds, per cut token, the few entries that can be that maximum: fp16
// matrix-core cosines (the unit vectors of shallow_prep) against all stored entries, off
// from the exact value by less than kGuard.  With F the largest approximate cosine of a
// token, the exact maximum has an approximate value >= F - 2 kGuard, and so has every entry
// that ties with it.  Each lane keeps, for its token and its half of the entries, the
// running maximum and the entries seen within 2 kGuard of it (the list restarts whenever the
// maximum jumps by more than that, so it stays short).  shallow_assign_exact evaluates the
// surviving entries in double precision; a token whose list ran full is left to
// shallow_overflow, the exhaustive search.
constexpr int kCandCap = 8;
constexpr int kAssignThreads = 256;

__global__ __launch_bounds__(kAssignThreads, 2) void shallow_assign(ShallowParams p) {
  typedef Mma<SPINDLE_F16> M;
  __shared__ __attribute__((aligned(1024))) char stage[2 * kStageBytes];
  const int ut = blockIdx.y, n = p.n;
  const int nov = (int)p.ovf_cnt[ut];
  const int slot0 = blockIdx.x * kAssignThreads;
  if (slot0 >= nov) return;
  const int kept = p.n_codes[ut / p.U][ut % p.U];     // = cap whenever tokens were cut
  if (kept <= 0) return;
  const int lane = lane_id(), wave = threadIdx.x >> 6, g = lane >> 5, c = lane & 31;
  const char *Xh = reinterpret_cast<const char *>(p.Xh) + (size_t)ut * n * 256;
  const uint32_t *ovf = p.ovf + (size_t)ut * n;
  const int *rank_vert = p.rank_vert + (size_t)ut * n;
  const float band2 = 2.f * kGuard * kUnitScale * kUnitScale;

  // the wave's 64 cut tokens: MFMA B operand (matrix columns = lanes)
  int slot[2];
  bool valid[2];
  M::frag af[2][M::kSteps];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    slot[cb] = slot0 + 64 * wave + 32 * cb + c;
    valid[cb] = slot[cb] < nov;
    const int tok = valid[cb] ? (int)ovf[slot[cb]] : 0;
#pragma unroll
    for (int ks = 0; ks < M::kSteps; ++ks) af[cb][ks] = valid[cb] ? M::load(Xh + (size_t)tok * 256, ks, g) : M::zero();
  }
  // staged entry 16*g + v of a tile is fed to matrix row 8*(v/4) + 4*g + v%4 (as in shallow_gram)
  const int prow = 16 * ((c >> 2) & 1) + 4 * (c >> 3) + (c & 3);
  int soff[M::kSteps];
#pragma unroll
  for (int ks = 0; ks < M::kSteps; ++ks)
    soff[ks] = prow * 256 + (((2 * ks + g) ^ ((prow & 7) | ((prow & 16) >> 1))) << 4);
  // loads of a 64-entry stage: wave w, load q covers rows (4 w + q) * 4 + lane / 16
  int srow[4];
  uint32_t spiece[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    srow[q] = (wave * 4 + q) * 4 + (lane >> 4);
    spiece[q] = (uint32_t)((((lane & 15) ^ ((srow[q] & 7) | ((srow[q] & 16) >> 1))) << 4));
  }
  const uint32_t stage_lds = (uint32_t)(size_t)(__attribute__((address_space(3))) char *)stage;
  const int nstages = (kept + kStageCols - 1) / kStageCols;
  int tokq[4];                                       // tokens of the entries the next load brings in
  auto fetch_tokens = [&](int s) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int j = s * kStageCols + srow[q];
      tokq[q] = j < kept ? rank_vert[j] : 0;         // rows past the last entry are masked below
    }
  };
  auto dma = [&](int bufsel) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      lds_dma16(Xh + (size_t)tokq[q] * 256 + spiece[q], stage_lds + bufsel * kStageBytes + (wave * 4 + q) * 1024);
  };
  float runmax[2] = {-INFINITY, -INFINITY};
  int cnt[2] = {0, 0};
  uint2 *cand = p.ccand + (size_t)ut * n * 2 * kCandCap;
  auto collect = [&](f16v a, int cb, int j0) {
    if (j0 + 32 > kept) {
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (j0 + 16 * g + v >= kept) a[v] = -INFINITY;
    }
    float t = a[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) t = fmaxf(t, a[v]);
    const float nm = fmaxf(runmax[cb], t);
    if (nm > runmax[cb] + band2) cnt[cb] = 0;         // everything collected so far is out of reach
    runmax[cb] = nm;
    const float thr = nm - band2;
    if (valid[cb]) {
      uint2 *list = cand + ((size_t)slot[cb] * 2 + g) * kCandCap;
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (a[v] >= thr) {
          if (cnt[cb] < kCandCap) list[cnt[cb]] = make_uint2((uint32_t)(j0 + 16 * g + v), __float_as_uint(a[v]));
          ++cnt[cb];
        }
    }
  };

  fetch_tokens(0);
  dma(0);
  if (nstages > 1) fetch_tokens(1);
  for (int s = 0; s < nstages; ++s) {
    __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0): stage s has landed
    __syncthreads();                                  // ... for every wave; the other buffer is free
    if (s + 1 < nstages) {
      dma((s + 1) & 1);
      if (s + 2 < nstages) fetch_tokens(s + 2);
    }
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      const int j0 = s * kStageCols + 32 * ct;
      if (j0 >= kept) break;
      f16v acc0, acc1;
#pragma unroll
      for (int v = 0; v < 16; ++v) { acc0[v] = 0.f; acc1[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < M::kSteps; ++ks) {
        const M::frag f = *reinterpret_cast<const M::frag *>(stage + (s & 1) * kStageBytes + ct * 32 * 256 + soff[ks]);
        acc0 = M::mma(f, af[0][ks], acc0);
        acc1 = M::mma(f, af[1][ks], acc1);
      }
      collect(acc0, 0, j0);
      collect(acc1, 1, j0);
    }
  }
  float2 *cstat = p.cstat + (size_t)ut * n * 2;
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
    if (valid[cb]) cstat[(size_t)slot[cb] * 2 + g] = make_float2(runmax[cb], __int_as_float(cnt[cb]));
}

__global__ __launch_bounds__(256) void shallow_assign_exact(ShallowParams p) {
  const int ut = blockIdx.y, n = p.n;
  const int nov = (int)p.ovf_cnt[ut];
  const uint32_t *ovf = p.ovf + (size_t)ut * n;
  const int *rank_vert = p.rank_vert + (size_t)ut * n;
  const float2 *cstat = p.cstat + (size_t)ut * n * 2;
  const uint2 *cand = p.ccand + (size_t)ut * n * 2 * kCandCap;
  const float band2 = 2.f * kGuard * kUnitScale * kUnitScale;
  for (int s = blockIdx.x * 256 + threadIdx.x; s < nov; s += gridDim.x * 256) {
    const int a = (int)ovf[s];
    const float2 st0 = cstat[(size_t)s * 2], st1 = cstat[(size_t)s * 2 + 1];
    const int c0 = __float_as_int(st0.y), c1 = __float_as_int(st1.y);
    if (c0 > kCandCap || c1 > kCandCap) {              // a list ran full: exhaustive search
      p.ovf_left[atomicAdd(p.ovf_count, 1u)] = ((uint32_t)ut << 16) | (uint32_t)a;
      continue;
    }
    const float thr = fmaxf(st0.x, st1.x) - band2;
    double bv = -INFINITY;
    int bj = 0x7FFFFFFF;
    for (int h = 0; h < 2; ++h) {
      const int ch = h ? c1 : c0;
      for (int i = 0; i < ch; ++i) {
        const uint2 e = cand[((size_t)s * 2 + h) * kCandCap + i];
        if (__uint_as_float(e.y) >= thr) {
          const int j = (int)e.x;
          const double cv = cos64(p, ut, a, rank_vert[j]);
          if (cv > bv || (cv == bv && j < bj)) { bv = cv; bj = j; }
        }
      }
    }
    p.ref[ut / p.U][(size_t)(ut % p.U) * n + a] = bj;
  }
}

// One block per token left over: highest cosine among all stored entries.
__global__ __launch_bounds__(256) void shallow_overflow(ShallowParams p) {
  __shared__ double sh_v[256];
  __shared__ int sh_j[256];
  const unsigned count = *p.ovf_count;
  for (unsigned i = blockIdx.x; i < count; i += gridDim.x) {
    const uint32_t e = p.ovf_left[i];
    const int ut = (int)(e >> 16), a = (int)(e & 0xFFFFu);
    const int *rank_vert = p.rank_vert + (size_t)ut * p.n;
    double bv = -INFINITY;
    int bj = 0x7FFFFFFF;
    for (int j = threadIdx.x; j < p.cap; j += 256) {
      const double cv = cos64(p, ut, a, rank_vert[j]);
      if (cv > bv) { bv = cv; bj = j; }
    }
    sh_v[threadIdx.x] = bv;
    sh_j[threadIdx.x] = bj;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
      if (threadIdx.x < o) {
        const double ov = sh_v[threadIdx.x + o];
        const int oj = sh_j[threadIdx.x + o];
        if (ov > sh_v[threadIdx.x] || (ov == sh_v[threadIdx.x] && oj < sh_j[threadIdx.x])) {
          sh_v[threadIdx.x] = ov;
          sh_j[threadIdx.x] = oj;
        }
      }
      __syncthreads();
    }
    if (threadIdx.x == 0) p.ref[ut / p.U][(size_t)(ut % p.U) * p.n + a] = sh_j[0];
    __syncthreads();
  }
}

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

// ---------------------------------------------------------------- host side
struct ShallowLayout {
  size_t bytes;
};

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

extern "C" spindle_status spindle_compress_shallow(
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
  // zero: counters, list counts, error flag, barriers; codebooks
  const size_t nzero = zero_words(p.UT, n);
  const size_t cwords = (size_t)U * max_codes * kHeadDim * dtype_bytes(p.dtype) / 4;
  hipLaunchKernelGGL(shallow_init, dim3(1024), dim3(256), 0, st, p, nzero, cwords, T);

  const dim3 pgrid((n + 63) / 64, p.UT);
  { ProfScope ps("shallow_prep", st);
  if (p.dtype == SPINDLE_F16) hipLaunchKernelGGL(shallow_prep<SPINDLE_F16>, pgrid, dim3(256), 0, st, p);
  else if (p.dtype == SPINDLE_BF16) hipLaunchKernelGGL(shallow_prep<SPINDLE_BF16>, pgrid, dim3(256), 0, st, p);
  else hipLaunchKernelGGL(shallow_prep<SPINDLE_F32>, pgrid, dim3(256), 0, st, p); }

  const int nI = (n + kPanelRows - 1) / kPanelRows;
  const int nJ = (n + kChunkCols * kItemChunks - 1) / (kChunkCols * kItemChunks);
  const int pairs8 = (p.UT * nJ + 7) / 8;
  { ProfScope ps("shallow_gram", st);
  hipLaunchKernelGGL(shallow_gram<false>, dim3(8 * nI * pairs8), dim3(kGramThreads), 0, st, p); }
  { ProfScope ps("shallow_gram_exact", st);
  hipLaunchKernelGGL(shallow_gram<true>, dim3(1024), dim3(kGramThreads), 0, st, p); }
  { ProfScope ps("shallow_fixup", st);
  hipLaunchKernelGGL(shallow_fixup, dim3(128, p.UT), dim3(256), 0, st, p); }
  {
    // sparse graphs: lists from the edge records; otherwise (or when the caller wants the
    // adjacency matrix) the lower triangle is written and the lists come from the bitmap
    const int force = adj[0] || adj[1];
    { ProfScope ps("shallow_edge_lists", st);
    const dim3 eg((n + kPanelRows - 1) / kPanelRows, p.UT);
    if (p.seg_cap == 512) hipLaunchKernelGGL(shallow_edge_lists<512>, eg, dim3(kEdgeThreads), 0, st, p, force);
    else hipLaunchKernelGGL(shallow_edge_lists<0>, eg, dim3(kEdgeThreads), 0, st, p, force); }
    const int T1k = (n + 1023) / 1024, npairs = T1k * (T1k - 1) / 2;
    if (npairs > 0) {
      SPINDLE_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&shallow_mirror),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMirrorLds));
      ProfScope ps("shallow_mirror", st);
      const int items = 16 * ((p.UT * npairs + 7) / 8);
      hipLaunchKernelGGL(shallow_mirror, dim3(items < 512 ? items : 512), dim3(kMirrorThreads), kMirrorLds, st, p, force, items);
    }
    SPINDLE_HIP(hipGetLastError());
    { ProfScope ps("shallow_lists", st);
    const int groups = (n + 15) / 16;
    hipLaunchKernelGGL(shallow_lists, dim3(groups < 128 ? groups : 128, p.UT), dim3(256), 0, st, p, force); }
  }
  {
    int gx = (n + 4 * (kPhaseThreads / kSegW) - 1) / (4 * (kPhaseThreads / kSegW));
    if (gx > 256) gx = 256;
    // candidates are a small part of the tokens: an eighth of the blocks that would give every
    // 8-lane segment four rows (a grid of mostly idle blocks costs more than a second trip)
    const dim3 tg(gx / 8 > 0 ? gx / 8 : 1, p.UT);
    // one-hop phase: 1024-thread blocks with the keys of the problem in LDS when they fit
    const int keys_in_lds = n <= kKeysInLds;
    const size_t key_lds = keys_in_lds ? (size_t)((n + 3) & ~3) * sizeof(uint32_t) : 0;
    int ox = (n + 4 * (kMergeThreads / kSegW) - 1) / (4 * (kMergeThreads / kSegW));
    if (ox > 16) ox = 16;
    SPINDLE_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&merge_onehop),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)key_lds));
    const size_t dead_lds = (size_t)p.n16;
    SPINDLE_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&merge_update),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)dead_lds));
    for (int round = 0; round < kGridRounds; ++round) {
      ProfScope ps("shallow_merge_grid", st);
      hipLaunchKernelGGL(merge_onehop, dim3(ox, p.UT), dim3(kMergeThreads), key_lds, st, p, round, keys_in_lds);
      hipLaunchKernelGGL(merge_twohop, tg, dim3(kPhaseThreads), 0, st, p, round);
      hipLaunchKernelGGL(merge_update, dim3(ox, p.UT), dim3(kMergeThreads), dead_lds, st, p, round);   // 1024 threads: fewer copies of the flags

    }
  }
  const size_t merge_lds = n <= kKeysInLds ? ((size_t)((n + 3) & ~3) + (n + 31) / 32) * sizeof(uint32_t) : 0;
  SPINDLE_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&shallow_merge),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)merge_lds));
  { ProfScope ps("shallow_merge", st);
  hipLaunchKernelGGL(shallow_merge, dim3(p.UT), dim3(kMergeThreads), merge_lds, st, p); }
  { ProfScope ps("shallow_rank", st);
  hipLaunchKernelGGL(shallow_rank, dim3(p.UT), dim3(kRankThreads), 0, st, p); }
  { ProfScope ps("shallow_emit", st);
  int ex = (n + 1023) / 1024;
  hipLaunchKernelGGL(shallow_emit, dim3(ex < 64 ? ex : 64, p.UT), dim3(256), 0, st, p); }
  { ProfScope ps("shallow_assign", st);
  hipLaunchKernelGGL(shallow_assign, dim3((n + kAssignThreads - 1) / kAssignThreads, p.UT), dim3(kAssignThreads), 0, st, p);
  int ax = (n + 255) / 256;
  hipLaunchKernelGGL(shallow_assign_exact, dim3(ax < 64 ? ax : 64, p.UT), dim3(256), 0, st, p); }
  { ProfScope ps("shallow_overflow", st);
  hipLaunchKernelGGL(shallow_overflow, dim3(2048), dim3(256), 0, st, p); }

  const int W = (n + 31) / 32;
  for (int i = 0; i < T; ++i) {
    if (adj[i])
      hipLaunchKernelGGL(export_adj, dim3(1024), dim3(256), 0, st, p.G + (size_t)i * U * n * p.Wp, adj[i],
                         (size_t)U * n, p.Wp, W);
  }
  SPINDLE_HIP(hipGetLastError());
  return SPINDLE_OK;
}
