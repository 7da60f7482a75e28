// Attention-weight token eviction (Sec. "Attention Weight Based Token Eviction").
//
// Kernels, all enqueued on the caller's stream:
//   deep_stats        window logits by MFMA, per-row softmax statistics of a chunk of keys (Eq. 1)
//   deep_accumulate   merges the per-chunk statistics into max + log2(sum) per query row,
//                     recomputes the logits, forms softmax weights, sums them over the window
//                     queries and the GQA group (Eq. 2, 3)
//   deep_select       max-pool, 4096-bin histogram of the pooled scores over many workgroups;
//                     the last workgroup of a unit finds the k-th largest score from the
//                     histogram and the few scores that share its bin, then writes the kept
//                     positions in order (Eq. 7)
//   deep_gather       K_out = K[kept], V_out = V[kept]
//
// Both passes over K stream 64-KiB stages of keys through LDS with direct global->LDS loads
// (two stages, the next one in flight while the current one is multiplied); the 16-byte pieces
// of a row are XOR-swizzled by the row number so that the fragment reads of sixteen
// consecutive rows fall into different banks.
#include <math.h>

#include "common.h"
#include "mma.h"

namespace spindle {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kMaxStagesPerBlock = 4;
constexpr int kBins = 4096;          // histogram over the top 12 bits of the order-preserving score keys

// Staging geometry of one element type: a stage is 64 KiB of keys.
template <int DT>
struct Geo {
  typedef Mma<DT> M;
  static constexpr int kRowBytes = M::kRowBytes;
  static constexpr int kPieces = kRowBytes / 16;                   // 16-byte pieces per key
  static constexpr int kStageKeys = DT == SPINDLE_F32 ? 128 : 256;
  static constexpr int kStageBytes = kStageKeys * kRowBytes;
  static constexpr int kWaves = DT == SPINDLE_F32 ? 4 : 8;
  static constexpr int kThreads = 64 * kWaves;
  static constexpr int kTiles = kStageKeys / 32;                   // 32-key MFMA tiles per stage
  static constexpr int kRowsPerLoad = 1024 / kRowBytes;            // keys one wave-wide load brings
  static constexpr int kLoadsPerWave = kStageBytes / 1024 / kWaves;

  // Stage of keys key0 .. key0 + kStageKeys - 1 into the LDS buffer at byte address `lds`; keys
  // past the end of the sequence repeat the last one (the callers never use their results).
  static __device__ __forceinline__ void load(const char *Kunit, size_t pitch, int key0, int l, uint32_t lds,
                                              int wave, int lane) {
#pragma unroll
    for (int j = 0; j < kLoadsPerWave; ++j) {
      const int q = wave * kLoadsPerWave + j;
      const int r = q * kRowsPerLoad + lane / kPieces;
      const int piece = (lane % kPieces) ^ (r & (kPieces - 1));
      int key = key0 + r;
      key = key < l ? key : l - 1;
      lds_dma16(Kunit + (size_t)key * pitch + piece * 16, lds + q * 1024);
    }
  }
  // The same for a stage that lies inside the sequence, with this lane's byte offsets within a
  // stage worked out once (`offsets`): a load is then its address registers and nothing else.
  static __device__ __forceinline__ void offsets(size_t pitch, int wave, int lane, uint32_t (&off)[kLoadsPerWave]) {
#pragma unroll
    for (int j = 0; j < kLoadsPerWave; ++j) {
      const int q = wave * kLoadsPerWave + j;
      const int r = q * kRowsPerLoad + lane / kPieces;
      const int piece = (lane % kPieces) ^ (r & (kPieces - 1));
      off[j] = (uint32_t)((size_t)r * pitch + (size_t)piece * 16);
    }
  }
  static __device__ __forceinline__ void load_inside(const char *Kunit, size_t pitch, int key0, uint32_t lds, int wave,
                                                     const uint32_t (&off)[kLoadsPerWave]) {
    const char *base = Kunit + (size_t)key0 * pitch;
#pragma unroll
    for (int j = 0; j < kLoadsPerWave; ++j) lds_dma16_at(base, off[j], lds + (wave * kLoadsPerWave + j) * 1024);
  }
  // MFMA operand fragment ks of staged key `row` for lane group g
  static __device__ __forceinline__ typename M::frag frag(const char *buf, int row, int ks, int g) {
    if constexpr (DT == SPINDLE_F32) {
      const int e = 2 * ks + g;
      return *reinterpret_cast<const float *>(buf + row * kRowBytes + ((((e >> 2) ^ (row & 31)) << 4) | ((e & 3) << 2)));
    } else {
      return *reinterpret_cast<const typename M::frag *>(buf + row * kRowBytes + (((2 * ks + g) ^ (row & 15)) << 4));
    }
  }
};

// Stages a block takes: as many as leave about one block per compute unit.  The fixed cost of
// a block (query fragments, the merge of the chunk statistics) outweighs idle units only while
// the grid still covers the chip.
inline int stages_per_block(int U, int l, int stage_keys) {
  const long total = (long)U * ((l + stage_keys - 1) / stage_keys);
  const long s = total / 256;
  return s < 1 ? 1 : (s > kMaxStagesPerBlock ? kMaxStagesPerBlock : (int)s);
}

struct DeepParams {
  const char *K;       // [U][l][128] elements
  const char *Q;       // [U][R][128] elements (R = hn*lw rows, head-major)
  float2 *partial;     // [U][nchunks][Rpad] (max, sum) per chunk of keys, logits in base-2 units
  float *scores;       // [U][lc] group-averaged accumulated attention
  int *hist;           // [U][kBins] cleared here for deep_select
  int *done;           // [U]
  int l, lc, lw, hn, R, Rpad, nchunks;
  int stages;          // stages per block
  KvLayout lay;        // rows of K
  float sc2;           // scale * log2(e): logits are kept in base-2 units
  float inv_hn;
  int norm;
};

// (max, sum of exp2(. - max)) of two disjoint sets of logits
__device__ __forceinline__ void merge_stats(float &m, float &z, float m2, float z2) {
  const float mm = fmaxf(m, m2);
  if (mm == -INFINITY) return;                         // both empty
  z = z * __builtin_amdgcn_exp2f(m - mm) + z2 * __builtin_amdgcn_exp2f(m2 - mm);
  m = mm;
}

__device__ __forceinline__ uint32_t lds_address(const void *ptr) {
  return (uint32_t)(size_t)(__attribute__((address_space(3))) const char *)ptr;
}

// Pass 1.  Grid (chunks, units).  WR waves split the (padded) query rows in groups of 64, the
// other kWaves / WR split the 32-key tiles of a stage.  The matrix product is taken as keys x
// query rows, so a lane owns one query row (its column of the result) and the sixteen results
// in its registers are sixteen keys: the running (max, sum) of a row is two registers per lane
// and needs no exchange until the end of the block.
template <int DT, int WR>
__global__ __launch_bounds__(Geo<DT>::kThreads) void deep_stats(DeepParams p) {
  typedef Geo<DT> S;
  typedef Mma<DT> M;
  constexpr int WK = S::kWaves / WR;
  constexpr int kTilesPerWave = S::kTiles / WK;
  constexpr bool kPrefetch = DT != SPINDLE_F32;        // the 64 one-register fragments of a float tile are read as they are used
  static_assert(kTilesPerWave >= 1, "every wave needs a tile of each stage");
  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const int u = blockIdx.y, chunk = blockIdx.x;
  const int lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int g = lane >> 5, c = lane & 31;
  const int wr = wave % WR, wk = wave / WR;
  if (chunk == 0) {                                    // counters of this unit's selection
    for (int i = threadIdx.x; i < kBins; i += S::kThreads) p.hist[(size_t)u * kBins + i] = 0;
    if (threadIdx.x == 0) p.done[u] = 0;
  }
  const int key_begin = chunk * p.stages * S::kStageKeys;
  int nst = (p.l - key_begin + S::kStageKeys - 1) / S::kStageKeys;
  nst = nst < p.stages ? nst : p.stages;
  const char *Kunit = p.K + kv_unit_offset(p.lay, u);
  const size_t kpitch = (size_t)p.lay.st;
  const char *Qunit = p.Q + (size_t)u * p.R * M::kRowBytes;
  const uint32_t lds0 = lds_address(smem);

  uint32_t koff[S::kLoadsPerWave];
  S::offsets(kpitch, wave, lane, koff);
  const bool narrow = kpitch * S::kStageKeys <= 0xFFFFFFFFull;   // lane offsets within a stage fit 32 bits
  auto stage_load = [&](int key0, uint32_t lds) {
    if (narrow && key0 + S::kStageKeys <= p.l) S::load_inside(Kunit, kpitch, key0, lds, wave, koff);
    else S::load(Kunit, kpitch, key0, p.l, lds, wave, lane);
  };
  stage_load(key_begin, lds0);

  // query fragments stay in registers for the whole block
  typename M::frag qf[2][M::kSteps];
  int klim[2];                                         // last key this lane's query row may attend to
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int row = 64 * wr + 32 * rb + c;
#pragma unroll
    for (int ks = 0; ks < M::kSteps; ++ks)
      qf[rb][ks] = row < p.R ? M::load(Qunit + (size_t)row * M::kRowBytes, ks, g) : M::zero();
    klim[rb] = row < p.R ? p.lc + row % p.lw : -1;    // causal mask: query b of the window sits at l_c + b
  }
  float m[2] = {-INFINITY, -INFINITY}, z[2] = {0.f, 0.f};
  __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): this wave's part of the stage has landed
  __syncthreads();

  for (int s = 0; s < nst; ++s) {
    const int k0 = key_begin + s * S::kStageKeys;
    if (s + 1 < nst) stage_load(k0 + S::kStageKeys, lds0 + ((s + 1) & 1) * S::kStageBytes);
    const char *buf = smem + (s & 1) * S::kStageBytes;
    const bool tail = k0 + S::kStageKeys > p.lc;       // causal mask / end of the sequence
    // The fragments of a tile are fetched from LDS together, those of the wave's next tile right
    // after the matrix instructions of the current one are issued, so that the LDS latency falls
    // into the vector work on the results (the other wave of the SIMD multiplies meanwhile).
    typename M::frag kf[kPrefetch ? M::kSteps : 1];
    if (kPrefetch && k0 + wk * 32 < p.l) {
#pragma unroll
      for (int ks = 0; ks < M::kSteps; ++ks) kf[kPrefetch ? ks : 0] = S::frag(buf, wk * 32 + c, ks, g);
    }
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
      const int ct = wk + t * WK;
      const int tk0 = k0 + ct * 32;
      if (tk0 >= p.l) continue;                        // wave-uniform
      f16v acc[2];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][v] = 0.f;
      if (kPrefetch) {
#pragma unroll
        for (int ks = 0; ks < M::kSteps; ++ks) {
          acc[0] = M::mma(kf[kPrefetch ? ks : 0], qf[0][ks], acc[0]);
          acc[1] = M::mma(kf[kPrefetch ? ks : 0], qf[1][ks], acc[1]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < kTilesPerWave && tk0 + WK * 32 < p.l) {
#pragma unroll
          for (int ks = 0; ks < M::kSteps; ++ks) kf[kPrefetch ? ks : 0] = S::frag(buf, (ct + WK) * 32 + c, ks, g);
        }
        __builtin_amdgcn_sched_barrier(0);
      } else {
#pragma unroll
        for (int ks = 0; ks < M::kSteps; ++ks) {
          const typename M::frag f = S::frag(buf, ct * 32 + c, ks, g);
          acc[0] = M::mma(f, qf[0][ks], acc[0]);
          acc[1] = M::mma(f, qf[1][ks], acc[1]);
        }
      }
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        if (!tail) {
          float hi = acc[rb][0], lo = acc[rb][0];
#pragma unroll
          for (int v = 1; v < 16; ++v) hi = fmaxf(hi, acc[rb][v]);
          if (p.sc2 < 0.f) {                           // uniform; a negative scale turns the order round
#pragma unroll
            for (int v = 1; v < 16; ++v) lo = fminf(lo, acc[rb][v]);
            hi = lo;
          }
          const float mn = fmaxf(m[rb], hi * p.sc2);
          float sum = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(fmaf(acc[rb][v], p.sc2, -mn));
          z[rb] = z[rb] * __builtin_amdgcn_exp2f(m[rb] - mn) + sum;
          m[rb] = mn;
        } else {
          float tv[16];
          float hi = -INFINITY;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = tk0 + mma_row(v, g);
            tv[v] = key <= klim[rb] && key < p.l ? acc[rb][v] * p.sc2 : -INFINITY;
            hi = fmaxf(hi, tv[v]);
          }
          const float mn = fmaxf(m[rb], hi);
          if (mn > -INFINITY) {
            float sum = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) sum += __builtin_amdgcn_exp2f(tv[v] - mn);
            z[rb] = z[rb] * __builtin_amdgcn_exp2f(m[rb] - mn) + sum;
            m[rb] = mn;
          }
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
  }

  // the two lane groups of a wave hold different keys of the same rows; then the WK waves of a
  // row group through LDS, in wave order
  float2 *red = reinterpret_cast<float2 *>(smem);      // [WK][64 * WR]
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const float m2 = __shfl_xor(m[rb], 32), z2 = __shfl_xor(z[rb], 32);
    float mm = g ? m2 : m[rb], zz = g ? z2 : z[rb];    // same operand order in both lane groups
    merge_stats(mm, zz, g ? m[rb] : m2, g ? z[rb] : z2);
    if (g == 0) red[wk * (64 * WR) + 64 * wr + 32 * rb + c] = make_float2(mm, zz);
  }
  __syncthreads();
  const int row = threadIdx.x;
  if (row < 64 * WR) {
    float2 e = red[row];
#pragma unroll
    for (int j = 1; j < WK; ++j) {
      const float2 o = red[j * (64 * WR) + row];
      merge_stats(e.x, e.y, o.x, o.y);
    }
    p.partial[((size_t)u * p.nchunks + chunk) * p.Rpad + row] = e;
  }
}

// Pass 2.  Grid (chunks of context keys, units).  Here the product is taken as query rows x
// keys: a lane owns one key and its registers hold sixteen query rows, so the sum over the
// window queries and the heads of the group is a sum over the lane's own registers.  The
// weight of (row, key) is exp2(logit - c_row) with c_row = max + log2(sum) of the row.
template <int DT, int WR>
__global__ __launch_bounds__(Geo<DT>::kThreads) void deep_accumulate(DeepParams p) {
  typedef Geo<DT> S;
  typedef Mma<DT> M;
  constexpr int WK = S::kWaves / WR;
  constexpr int kTilesPerWave = S::kTiles / WK;
  constexpr bool kPrefetch = DT != SPINDLE_F32;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  float *colpart = reinterpret_cast<float *>(smem + 2 * S::kStageBytes);      // [2][WR][kStageKeys]
  float *row_const = colpart + 2 * WR * S::kStageKeys;                          // [256]

  const int u = blockIdx.y, chunk = blockIdx.x;
  const int lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int g = lane >> 5, c = lane & 31;
  const int wr = wave % WR, wk = wave / WR;
  const int key_begin = chunk * p.stages * S::kStageKeys;
  int nst = (p.lc - key_begin + S::kStageKeys - 1) / S::kStageKeys;            // only context keys get a score
  nst = nst < p.stages ? nst : p.stages;
  const char *Kunit = p.K + kv_unit_offset(p.lay, u);
  const size_t kpitch = (size_t)p.lay.st;
  const char *Qunit = p.Q + (size_t)u * p.R * M::kRowBytes;
  const uint32_t lds0 = lds_address(smem);

  uint32_t koff[S::kLoadsPerWave];
  S::offsets(kpitch, wave, lane, koff);
  const bool narrow = kpitch * S::kStageKeys <= 0xFFFFFFFFull;   // lane offsets within a stage fit 32 bits
  auto stage_load = [&](int key0, uint32_t lds) {
    if (narrow && key0 + S::kStageKeys <= p.l) S::load_inside(Kunit, kpitch, key0, lds, wave, koff);
    else S::load(Kunit, kpitch, key0, p.l, lds, wave, lane);
  };
  stage_load(key_begin, lds0);

  // max + log2(sum) of every query row from the per-chunk statistics of the first pass, merged
  // in chunk order by one thread per row (every block of the unit does the same sum in the same
  // order)
  if ((int)threadIdx.x < p.Rpad) {
    const int row = threadIdx.x;
    const float2 *part = p.partial + (size_t)u * p.nchunks * p.Rpad + row;
    float mm = -INFINITY, zz = 0.f;
    for (int ch0 = 0; ch0 < p.nchunks; ch0 += 32) {   // 32 records in flight: one trip for 32 k keys
      float2 e[32];
#pragma unroll
      for (int j = 0; j < 32; ++j) e[j] = ch0 + j < p.nchunks ? part[(size_t)(ch0 + j) * p.Rpad] : make_float2(-INFINITY, 0.f);
#pragma unroll
      for (int j = 0; j < 32; ++j) merge_stats(mm, zz, e[j].x, e[j].y);
    }
    row_const[row] = row < p.R && zz > 0.f ? mm + log2f(zz) : INFINITY;        // rows of the padding weigh nothing
  }

  typename M::frag qf[2][M::kSteps];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int row = 64 * wr + 32 * rb + c;
#pragma unroll
    for (int ks = 0; ks < M::kSteps; ++ks)
      qf[rb][ks] = row < p.R ? M::load(Qunit + (size_t)row * M::kRowBytes, ks, g) : M::zero();
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  float cst[2][16];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) cst[rb][v] = row_const[64 * wr + 32 * rb + mma_row(v, g)];

  for (int s = 0; s < nst; ++s) {
    const int k0 = key_begin + s * S::kStageKeys;
    if (s + 1 < nst) stage_load(k0 + S::kStageKeys, lds0 + ((s + 1) & 1) * S::kStageBytes);
    const char *buf = smem + (s & 1) * S::kStageBytes;
    float *cp = colpart + (s & 1) * (WR * S::kStageKeys);
    typename M::frag kf[kPrefetch ? M::kSteps : 1];    // as in deep_stats
    if (kPrefetch && k0 + wk * 32 < p.lc) {
#pragma unroll
      for (int ks = 0; ks < M::kSteps; ++ks) kf[kPrefetch ? ks : 0] = S::frag(buf, wk * 32 + c, ks, g);
    }
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
      const int ct = wk + t * WK;
      if (k0 + ct * 32 >= p.lc) continue;              // wave-uniform
      f16v acc[2];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][v] = 0.f;
      if (kPrefetch) {
#pragma unroll
        for (int ks = 0; ks < M::kSteps; ++ks) {
          acc[0] = M::mma(qf[0][ks], kf[kPrefetch ? ks : 0], acc[0]);
          acc[1] = M::mma(qf[1][ks], kf[kPrefetch ? ks : 0], acc[1]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < kTilesPerWave && k0 + (ct + WK) * 32 < p.lc) {
#pragma unroll
          for (int ks = 0; ks < M::kSteps; ++ks) kf[kPrefetch ? ks : 0] = S::frag(buf, (ct + WK) * 32 + c, ks, g);
        }
        __builtin_amdgcn_sched_barrier(0);
      } else {
#pragma unroll
        for (int ks = 0; ks < M::kSteps; ++ks) {
          const typename M::frag f = S::frag(buf, ct * 32 + c, ks, g);
          acc[0] = M::mma(qf[0][ks], f, acc[0]);
          acc[1] = M::mma(qf[1][ks], f, acc[1]);
        }
      }
      float cs0 = 0.f, cs1 = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        cs0 += __builtin_amdgcn_exp2f(fmaf(acc[0][v], p.sc2, -cst[0][v]));
        cs1 += __builtin_amdgcn_exp2f(fmaf(acc[1][v], p.sc2, -cst[1][v]));
      }
      // the other sixteen rows of each block of 32 sit in the other lane group
      const uint32_t csb = __float_as_uint(cs0 + cs1);
      const auto both = __builtin_amdgcn_permlane32_swap(csb, csb, false, false);   // [0]: group 0's value, [1]: group 1's
      if (g == 0) cp[wr * S::kStageKeys + ct * 32 + c] = __uint_as_float(both[0]) + __uint_as_float(both[1]);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    if ((int)threadIdx.x < S::kStageKeys) {            // fixed-order sum over the row groups
      const int a = k0 + threadIdx.x;
      if (a < p.lc) {
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < WR; ++j) sum += cp[j * S::kStageKeys + threadIdx.x];
        float v = sum * p.inv_hn;
        if (p.norm == SPINDLE_NORM_PAPER) v = v / (float)(p.l - a);
        p.scores[(size_t)u * p.lc + a] = v;
      }
    }
  }
}

// ---------------------------------------------------------------- pool + top-k
struct SelectParams {
  const float *scores;   // [U][lc]
  uint32_t *pooled;      // [U][lc] pooled scores as order-preserving keys
  float *scores_out;     // optional [U][lc]
  int *hist;             // [U][kBins], zero on entry
  int *done;             // [U], zero on entry
  const int32_t *budgets;
  int32_t *kept;         // [U][out_stride]
  int l, lc, lw, pool, budget, out_stride, nseg;
};

constexpr int kSelThreads = 1024;
constexpr int kSegLen = 2048;        // context positions per workgroup
constexpr int kHaloMax = 256;        // pooling radius up to which the raw scores of a segment sit in LDS
constexpr int kCandMax = 8192;       // scores sharing the threshold's bin that are ranked in LDS

__device__ __forceinline__ uint32_t orderable(float f) {
  const uint32_t b = __float_as_uint(f);
  return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

// Stores and loads that workgroups of one launch use to hand data to each other: performed at
// device scope (they go through to, and come from, memory that every compute unit sees), so
// that no cache has to be written back or invalidated as a fence would do; the writer waits for
// its stores (s_waitcnt vmcnt(0)) before it takes its ticket.
__device__ __forceinline__ void store_shared(uint32_t *ptr, uint32_t v) {
  __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t load_shared(const uint32_t *ptr) {
  return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Counts, from the top, the digits of the keys `src[0 .. nsrc)` that match `prefix` above
// `bits_left`, and narrows (prefix, krem) by one digit of width w: afterwards the krem-th
// largest matching key still matches.  All threads of the block call it with the same arguments.
__device__ void radix_step(const uint32_t *src, int nsrc, bool other_groups_wrote, uint32_t &prefix, int &krem, int &bits_left, int *hist,
                           uint32_t *sh_prefix, int *sh_krem) {
  const int tid = threadIdx.x, lane = lane_id();
  const int w = bits_left < 8 ? bits_left : 8, shift = bits_left - w;
  const uint32_t dmask = (1u << w) - 1u;
  if (tid < 256) hist[tid] = 0;
  __syncthreads();
  constexpr int kAtOnce = 4;                           // independent keys per thread and trip
  for (int a0 = 0; a0 < nsrc; a0 += kAtOnce * kSelThreads) {
    uint32_t x[kAtOnce];
#pragma unroll
    for (int q = 0; q < kAtOnce; ++q) {
      const int a = a0 + q * kSelThreads + tid;
      x[q] = a < nsrc ? (other_groups_wrote ? load_shared(src + a) : src[a]) : 0u;
    }
#pragma unroll
    for (int q = 0; q < kAtOnce; ++q) {
      const int a = a0 + q * kSelThreads + tid;
      const bool in = a < nsrc && (bits_left == 32 || (x[q] >> bits_left) == (prefix >> bits_left));
      const int d = (int)((x[q] >> shift) & dmask);
      if (in) {
        // keys crowd into few digits: the digit of the first lane that takes part is counted
        // once for all lanes that share it
        const int d0 = __builtin_amdgcn_readfirstlane(d);
        const unsigned long long same = __ballot(d == d0);
        if (d != d0) atomicAdd(&hist[d], 1);
        else if (lane == __builtin_ctzll(same)) atomicAdd(&hist[d0], __popcll(same));
      }
    }
  }
  __syncthreads();
  if (tid < 64) {
    // lane t owns counters 4t .. 4t+3; find the digit at which the count from the top reaches krem
    const int h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2], h3 = hist[4 * tid + 3];
    const int mine = h0 + h1 + h2 + h3;
    int above = mine;                                  // inclusive sum over lanes >= t
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int x = __shfl_down(above, o);
      if (tid + o < 64) above += x;
    }
    above -= mine;                                     // keys in counters of higher lanes
    const int hh[4] = {h0, h1, h2, h3};
    int run = above;
#pragma unroll
    for (int j = 3; j >= 0; --j) {
      if (run < krem && krem <= run + hh[j]) {
        *sh_prefix = prefix | ((uint32_t)(4 * tid + j) << shift);
        *sh_krem = krem - run;
      }
      run += hh[j];
    }
  }
  __syncthreads();
  prefix = *sh_prefix;
  krem = *sh_krem;
  bits_left = shift;
  __syncthreads();
}

// Grid (segments, units).  Every workgroup pools its segment of the raw scores, stores the
// pooled scores as keys and adds its 4096-bin histogram to the unit's.  The workgroup that
// finishes last for a unit carries on alone: threshold bin from the histogram, exact value of
// the k-th largest key among the keys of that bin, ordered compaction of the unit.
__global__ __launch_bounds__(kSelThreads) void deep_select(SelectParams p) {
  __shared__ float rawl[kSegLen + 2 * kHaloMax];
  __shared__ int hist[kBins];
  __shared__ uint32_t cand[kCandMax];
  __shared__ int wsum[kSelThreads / 64][2];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_krem, sh_last, sh_ncand;
  const int seg = blockIdx.x, u = blockIdx.y, tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
  const int lc = p.lc;
  const float *raw = p.scores + (size_t)u * lc;
  uint32_t *pooled = p.pooled + (size_t)u * lc;
  int *ghist = p.hist + (size_t)u * kBins;

  // ---- every workgroup: pooling and histogram of its segment
  for (int i = tid; i < kBins; i += kSelThreads) hist[i] = 0;
  const int a_begin = seg * kSegLen;
  const int a_end = a_begin + kSegLen < lc ? a_begin + kSegLen : lc;
  const int r = (p.pool - 1) / 2;
  const bool in_lds = r <= kHaloMax;
  const int h_begin = a_begin - r < 0 ? 0 : a_begin - r;
  const int h_end = a_end + r > lc ? lc : a_end + r;
  if (in_lds)
    for (int a = h_begin + tid; a < h_end; a += kSelThreads) rawl[a - h_begin] = raw[a];
  __syncthreads();
  for (int a = a_begin + tid; a < a_end; a += kSelThreads) {
    const int lo = a - r < 0 ? 0 : a - r, hi = a + r >= lc ? lc - 1 : a + r;
    float mx = -INFINITY;
    if (in_lds) for (int j = lo; j <= hi; ++j) mx = fmaxf(mx, rawl[j - h_begin]);
    else for (int j = lo; j <= hi; ++j) mx = fmaxf(mx, raw[j]);
    const uint32_t x = orderable(mx);
    store_shared(pooled + a, x);
    if (p.scores_out) p.scores_out[(size_t)u * lc + a] = mx;
    const int d = (int)(x >> 20);
    const int d0 = __builtin_amdgcn_readfirstlane(d);
    const unsigned long long same = __ballot(d == d0);
    if (d != d0) atomicAdd(&hist[d], 1);
    else if (lane == __builtin_ctzll(same)) atomicAdd(&hist[d0], __popcll(same));
  }
  __syncthreads();
  for (int i = tid; i < kBins; i += kSelThreads) {
    const int v = hist[i];
    if (v) __hip_atomic_fetch_add(&ghist[i], v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): this thread's keys and counts have arrived
  __syncthreads();
  if (tid == 0) sh_last = __hip_atomic_fetch_add(&p.done[u], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == p.nseg - 1;
  __syncthreads();
  if (!sh_last) return;

  // ---- the last workgroup of the unit
  int32_t *kept = p.kept + (size_t)u * p.out_stride;
  int budget = p.budgets ? p.budgets[u] : p.budget;
  if (budget < p.lw) budget = p.lw;
  int k = budget - p.lw;
  if (k > lc) k = lc;
  if (k > p.out_stride - p.lw) k = p.out_stride - p.lw;   // never write past the row pitch

  constexpr int kWaves = kSelThreads / 64;
  constexpr int kBatch = 32;
  const int run = (((lc + kWaves - 1) / kWaves) + 63) & ~63;      // positions per wave
  const int w0 = wave * run, w1 = w0 + run < lc ? w0 + run : lc;
  const bool one_trip = run <= 64 * kBatch;
  const unsigned long long below = (1ull << lane) - 1ull;
  uint32_t x[kBatch];
  auto load_keys = [&](int b0) {
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const int a = b0 + 64 * i + lane;
      x[i] = a < w1 ? load_shared(pooled + a) : 0u;
    }
  };
  uint32_t prefix = 0;                                 // key of the k-th largest pooled score
  int krem = k;                                        // how many keys equal to it are taken
  if (k > 0 && k < lc) {
    if (one_trip) load_keys(w0);
    // threshold bin: thread t owns bins 4t .. 4t+3, counts from the top
    {
      int h[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) h[j] = (int)load_shared(reinterpret_cast<const uint32_t *>(ghist) + 4 * tid + j);
      const int mine = h[0] + h[1] + h[2] + h[3];
      int above = mine;                                // inclusive sum over the higher lanes of the wave
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_down(above, o);
        if (lane + o < 64) above += up;
      }
      if (lane == 0) wsum[wave][0] = above;            // total of the wave
      __syncthreads();
      above -= mine;
      for (int w2 = wave + 1; w2 < kSelThreads / 64; ++w2) above += wsum[w2][0];
      int seen = above;
#pragma unroll
      for (int j = 3; j >= 0; --j) {
        if (seen < k && k <= seen + h[j]) {
          sh_prefix = (uint32_t)(4 * tid + j) << 20;
          sh_krem = k - seen;
        }
        seen += h[j];
      }
      if (tid == 0) sh_ncand = 0;
      __syncthreads();
      prefix = sh_prefix;
      krem = sh_krem;
    }
    // The unit's keys, dealt to the waves in contiguous runs (the order of the compaction below),
    // thirty-two 64-position steps per lane and trip, all loads of a trip in flight together.  A
    // unit of up to 32768 positions is one trip: its keys stay in registers for all three uses.
    // First use: the keys of the threshold's bin, ranked in LDS when they fit (a few hundred as a
    // rule), else where they are.
    for (int b0 = w0; b0 < w1; b0 += 64 * kBatch) {
      if (!one_trip) load_keys(b0);
#pragma unroll
      for (int i = 0; i < kBatch; ++i) {
        const int a = b0 + 64 * i + lane;
        const bool in = a < w1 && (x[i] >> 20) == (prefix >> 20);
        const unsigned long long mk = __ballot(in);
        if (mk) {                                      // wave-uniform
          int at = 0;
          if (lane == __builtin_ctzll(mk)) at = atomicAdd(&sh_ncand, __popcll(mk));
          at = __shfl(at, __builtin_ctzll(mk)) + __popcll(mk & below);
          if (in && at < kCandMax) cand[at] = x[i];
        }
      }
    }
    __syncthreads();
    const int ncand = sh_ncand;
    const uint32_t *src = ncand <= kCandMax ? cand : pooled;
    const int nsrc = ncand <= kCandMax ? ncand : lc;
    int bits_left = 20;
    while (bits_left > 0) radix_step(src, nsrc, ncand > kCandMax, prefix, krem, bits_left, hist, &sh_prefix, &sh_krem);
  }
  // ordered compaction: everything above the threshold, then the first `krem` equal to it.
  // Ranks within a 64-position step come from ballots, the offset of the wave from a count pass
  // and a scan over the waves.
  if (k >= lc) {
    for (int a = tid; a < lc; a += kSelThreads) kept[a] = a;
  } else if (k > 0) {
    int ngt = 0, neq = 0;                              // wave-uniform
    for (int b0 = w0; b0 < w1; b0 += 64 * kBatch) {
      if (!one_trip) load_keys(b0);
#pragma unroll
      for (int i = 0; i < kBatch; ++i) {
        const int a = b0 + 64 * i + lane;
        ngt += __popcll(__ballot(a < w1 && x[i] > prefix));
        neq += __popcll(__ballot(a < w1 && x[i] == prefix));
      }
    }
    __syncthreads();                                   // wsum was read above
    if (lane == 0) { wsum[wave][0] = ngt; wsum[wave][1] = neq; }
    __syncthreads();
    int gt_seen = 0, eq_seen = 0;
    for (int w = 0; w < wave; ++w) { gt_seen += wsum[w][0]; eq_seen += wsum[w][1]; }
    for (int b0 = w0; b0 < w1; b0 += 64 * kBatch) {
      if (!one_trip) load_keys(b0);
#pragma unroll
      for (int i = 0; i < kBatch; ++i) {
        const int a = b0 + 64 * i + lane;
        const bool gt = a < w1 && x[i] > prefix, eq = a < w1 && x[i] == prefix;
        const unsigned long long mgt = __ballot(gt), meq = __ballot(eq);
        const int gt_before = gt_seen + __popcll(mgt & below), eq_before = eq_seen + __popcll(meq & below);
        if (gt) kept[gt_before + (eq_before < krem ? eq_before : krem)] = a;
        else if (eq && eq_before < krem) kept[gt_before + eq_before] = a;
        gt_seen += __popcll(mgt);
        eq_seen += __popcll(meq);
      }
    }
  }
  for (int b = tid; b < p.lw; b += kSelThreads) kept[k + b] = lc + b;
  for (int j = k + p.lw + tid; j < p.out_stride; j += kSelThreads) kept[j] = -1;
}

// ---------------------------------------------------------------- gather
struct GatherParams {
  const char *K, *V;
  char *Ko, *Vo;
  const int32_t *kept;
  int l, out_stride, row_bytes;
  KvLayout lay;        // rows of K and V
};

__global__ __launch_bounds__(256) void deep_gather(GatherParams p) {
  const int tpr = p.row_bytes / 16;
  const int rows_per_block = 256 / tpr;
  const int u = blockIdx.y;
  const int j = blockIdx.x * rows_per_block + threadIdx.x / tpr;
  const int t = threadIdx.x % tpr;
  if (j >= p.out_stride) return;
  const int idx = p.kept[(size_t)u * p.out_stride + j];
  const size_t dst = ((size_t)u * p.out_stride + j) * p.row_bytes + t * 16;
  const size_t src = kv_unit_offset(p.lay, u) + (size_t)(idx < 0 ? 0 : idx) * (size_t)p.lay.st + t * 16;
  u4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
  if (idx >= 0) {
    kv = *reinterpret_cast<const u4 *>(p.K + src);
    if (p.V) vv = *reinterpret_cast<const u4 *>(p.V + src);
  }
  *reinterpret_cast<u4 *>(p.Ko + dst) = kv;
  if (p.Vo) *reinterpret_cast<u4 *>(p.Vo + dst) = vv;
}

// ---------------------------------------------------------------- host side
struct DeepLayout {
  float2 *partial;
  float *scores;
  uint32_t *pooled;
  int *hist, *done;
  int stages, nchunks;
  size_t bytes;
};

int stage_keys_of(int dtype) { return dtype == SPINDLE_F32 ? Geo<SPINDLE_F32>::kStageKeys : Geo<SPINDLE_F16>::kStageKeys; }
static_assert(Geo<SPINDLE_F16>::kStageKeys == Geo<SPINDLE_BF16>::kStageKeys, "one stage size for the 16-bit types");

DeepLayout deep_layout(void *ws, int U, int l, int lw, int Rpad, int dtype) {
  Carver cv(ws);
  DeepLayout L;
  const int sk = stage_keys_of(dtype);
  L.stages = stages_per_block(U, l, sk);
  L.nchunks = (l + L.stages * sk - 1) / (L.stages * sk);
  const int lc = l - lw;
  L.partial = cv.take<float2>((size_t)U * L.nchunks * Rpad);
  L.scores = cv.take<float>((size_t)U * (lc > 0 ? lc : 1));
  L.pooled = cv.take<uint32_t>((size_t)U * (lc > 0 ? lc : 1));
  L.hist = cv.take<int>((size_t)U * kBins);
  L.done = cv.take<int>((size_t)U);
  L.bytes = cv.total();
  return L;
}

int padded_rows(int R) { return R <= 64 ? 64 : (R <= 128 ? 128 : 256); }

template <int DT, int WR>
spindle_status launch_passes(const DeepParams &p, int U, hipStream_t st) {
  typedef Geo<DT> S;
  const size_t smem_stats = 2 * (size_t)S::kStageBytes;
  const size_t smem_acc = 2 * (size_t)S::kStageBytes + (2 * WR * S::kStageKeys + 256) * sizeof(float);
  static LdsLimit lim_stats, lim_acc;                  // one pair per instantiation; the sizes are constants of it
  if (spindle_status e = allow_lds(lim_stats, reinterpret_cast<const void *>(&deep_stats<DT, WR>), smem_stats)) return e;
  if (spindle_status e = allow_lds(lim_acc, reinterpret_cast<const void *>(&deep_accumulate<DT, WR>), smem_acc)) return e;
  { ProfScope ps("deep_stats", st);
  hipLaunchKernelGGL((deep_stats<DT, WR>), dim3(p.nchunks, U), dim3(S::kThreads), smem_stats, st, p); }
  if (p.lc > 0) {
    const int per = p.stages * S::kStageKeys;
    ProfScope ps("deep_accumulate", st);
    hipLaunchKernelGGL((deep_accumulate<DT, WR>), dim3((p.lc + per - 1) / per, U), dim3(S::kThreads), smem_acc, st, p);
  }
  SPINDLE_HIP(hipGetLastError());
  return SPINDLE_OK;
}

template <int DT>
spindle_status launch_dtype(const DeepParams &p, int U, hipStream_t st) {
  if (p.Rpad == 64) return launch_passes<DT, 1>(p, U, st);
  if (p.Rpad == 128) return launch_passes<DT, 2>(p, U, st);
  return launch_passes<DT, 4>(p, U, st);
}

}  // namespace
}  // namespace spindle

using namespace spindle;

extern "C" spindle_status spindle_deep_workspace_bytes(const spindle_kv_desc *desc, int32_t window,
                                                       size_t *bytes) {
  spindle_status s = check_desc(desc);
  if (s != SPINDLE_OK) return s;
  if (!bytes) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "bytes is NULL");
  if (window < 1 || window > desc->seq_len) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "window must be in [1, seq_len]");
  if (desc->group_size < 1 || (int64_t)window * desc->group_size > 256)
    SPINDLE_FAIL(SPINDLE_ERR_UNSUPPORTED, "window * group_size must be in [1, 256]");
  const int U = desc->batch * desc->n_kv_heads;
  *bytes = deep_layout(nullptr, U, desc->seq_len, window, padded_rows(window * desc->group_size), desc->dtype).bytes;
  return SPINDLE_OK;
}

extern "C" spindle_status spindle_compress_deep(const spindle_kv_desc *desc, const void *K, const void *V,
                                                const void *Qw, int32_t window, int32_t pool_kernel,
                                                float scale, int32_t norm, int32_t budget,
                                                const int32_t *budgets, int32_t out_stride,
                                                int32_t *kept_idx, void *K_out, void *V_out,
                                                float *scores_out, void *workspace,
                                                size_t workspace_bytes, void *stream) {
  size_t need = 0;
  spindle_status s = spindle_deep_workspace_bytes(desc, window, &need);
  if (s != SPINDLE_OK) return s;
  if (!K || !Qw || !kept_idx || !K_out) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "K, Qw, kept_idx and K_out are required");
  if ((V == nullptr) != (V_out == nullptr)) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "V and V_out must both be given or both NULL");
  if (pool_kernel < 1 || (pool_kernel & 1) == 0) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "pool_kernel must be odd and >= 1");
  if (norm != SPINDLE_NORM_PAPER && norm != SPINDLE_NORM_NONE) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "unknown norm mode %d", norm);
  if (!(scale == scale) || fabsf(scale) > 3.0e38f) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "scale must be finite");
  const int l = desc->seq_len, lw = window, lc = l - lw;
  if (!budgets && budget < lw) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "budget (%d) must be >= window (%d)", budget, lw);
  if (out_stride < lw || (!budgets && out_stride < (budget < l ? budget : l)))
    SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "out_stride (%d) is smaller than the kept-token count", out_stride);
  if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255))
    SPINDLE_FAIL(SPINDLE_ERR_WORKSPACE, "workspace needs %zu bytes, 256-byte aligned (got %zu)", need, workspace_bytes);
  const uintptr_t al = reinterpret_cast<uintptr_t>(K) | reinterpret_cast<uintptr_t>(V) |
                       reinterpret_cast<uintptr_t>(Qw) | reinterpret_cast<uintptr_t>(K_out) |
                       reinterpret_cast<uintptr_t>(V_out);
  if (al & 15) SPINDLE_FAIL(SPINDLE_ERR_INVALID_ARG, "tensor pointers must be 16-byte aligned");

  hipStream_t st = static_cast<hipStream_t>(stream);
  const int U = desc->batch * desc->n_kv_heads;
  const int R = lw * desc->group_size, Rpad = padded_rows(R);
  DeepLayout L = deep_layout(workspace, U, l, lw, Rpad, desc->dtype);

  DeepParams p;
  KvLayout lay;
  s = kv_layout(desc, &lay);
  if (s != SPINDLE_OK) return s;
  p.K = static_cast<const char *>(K);
  p.lay = lay;
  p.Q = static_cast<const char *>(Qw);
  p.partial = L.partial;
  p.scores = L.scores;
  p.hist = L.hist;
  p.done = L.done;
  p.l = l; p.lc = lc; p.lw = lw; p.hn = desc->group_size; p.R = R; p.Rpad = Rpad;
  p.stages = L.stages;
  p.nchunks = L.nchunks;
  p.sc2 = scale * kLog2e;
  p.inv_hn = 1.0f / (float)desc->group_size;
  p.norm = norm;
  if (desc->dtype == SPINDLE_F16) s = launch_dtype<SPINDLE_F16>(p, U, st);
  else if (desc->dtype == SPINDLE_BF16) s = launch_dtype<SPINDLE_BF16>(p, U, st);
  else s = launch_dtype<SPINDLE_F32>(p, U, st);
  if (s != SPINDLE_OK) return s;

  SelectParams sp;
  sp.scores = L.scores; sp.pooled = L.pooled; sp.scores_out = scores_out;
  sp.hist = L.hist; sp.done = L.done;
  sp.budgets = budgets; sp.kept = kept_idx;
  sp.l = l; sp.lc = lc; sp.lw = lw; sp.pool = pool_kernel; sp.budget = budget; sp.out_stride = out_stride;
  sp.nseg = lc > 0 ? (lc + kSegLen - 1) / kSegLen : 1;
  {
    ProfScope ps("deep_select", st);
    hipLaunchKernelGGL(deep_select, dim3(sp.nseg, U), dim3(kSelThreads), 0, st, sp);
  }

  GatherParams gp;
  gp.K = static_cast<const char *>(K); gp.V = static_cast<const char *>(V);
  gp.Ko = static_cast<char *>(K_out); gp.Vo = static_cast<char *>(V_out);
  gp.kept = kept_idx; gp.l = l; gp.out_stride = out_stride;
  gp.row_bytes = kHeadDim * dtype_bytes(desc->dtype);
  gp.lay = lay;
  const int rows_per_block = 256 / (gp.row_bytes / 16);
  { ProfScope ps("deep_gather", st);
  hipLaunchKernelGGL(deep_gather, dim3((out_stride + rows_per_block - 1) / rows_per_block, U), dim3(256), 0, st, gp); }
  SPINDLE_HIP(hipGetLastError());
  return SPINDLE_OK;
}
