// Attention-weight token eviction (Sec. "Attention Weight Based Token Eviction").
//
// Kernels, all enqueued on the caller's stream:
//   deep_pass<.., false>  window logits by MFMA, per-row softmax statistics (Eq. 1)
//   deep_pass<.., true>   merges the per-chunk statistics into (max, 1/sum) per query row,
//                         recomputes the logits, forms softmax weights, sums them over
//                         the window queries and the GQA group (Eq. 2, 3)
//   deep_select           max-pool, radix select of the k largest, ordered compaction (Eq. 7)
//   deep_gather           K_out = K[kept], V_out = V[kept]
#include <math.h>

#include "common.h"
#include "mma.h"

namespace spindle {
namespace {

constexpr int kStageKeys = 128;      // keys per LDS stage
constexpr int kMaxStagesPerBlock = 8; // at most 1024 keys per block
// Stages a block takes: as many as leave about one block per compute unit.  The fixed cost of
// a block (query fragments, the merge of the chunk statistics) outweighs idle units only while
// the grid still covers the chip.
inline int stages_per_block(int U, int l) {
  const long total = (long)U * ((l + kStageKeys - 1) / kStageKeys);
  const long s = total / 256;
  return s < 1 ? 1 : (s > kMaxStagesPerBlock ? kMaxStagesPerBlock : (int)s);
}
constexpr int kDeepThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

struct DeepParams {
  const char *K;       // [U][l][128] elements
  const char *Q;       // [U][R][128] elements (R = hn*lw rows, head-major)
  float2 *partial;     // [U][nchunks][Rpad] (max, sum) per chunk of keys
  float *scores;       // [U][lc] group-averaged accumulated attention
  int l, lc, lw, hn, R, Rpad, nchunks;
  int stages;          // 128-key stages per block
  KvLayout lay;        // rows of K
  float sc2;           // scale * log2(e): logits are kept in base-2 units
  float inv_hn;
  int norm;
};

// ---------------------------------------------------------------- stage loading
template <int DT>
struct Stage {
  typedef Mma<DT> M;
  static constexpr int kThreadsPerRow = M::kRowBytes / 16;
  static constexpr int kRowsPerPass = kDeepThreads / kThreadsPerRow;
  static constexpr int kPasses = kStageKeys / kRowsPerPass;
  static constexpr int kBytes = kStageKeys * M::kLdsRow;

  // global -> registers; keys at or beyond `l` read as zero
  static __device__ __forceinline__ void fetch(u4 (&r)[kPasses], const char *Kunit, size_t pitch, int k0, int l) {
    const int tr = threadIdx.x / kThreadsPerRow, tc = threadIdx.x % kThreadsPerRow;
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
      const int key = k0 + p * kRowsPerPass + tr;
      u4 v = {0, 0, 0, 0};
      if (key < l) v = *reinterpret_cast<const u4 *>(Kunit + (size_t)key * pitch + tc * 16);
      r[p] = v;
    }
  }
  static __device__ __forceinline__ void store(const u4 (&r)[kPasses], char *lds) {
    const int tr = threadIdx.x / kThreadsPerRow, tc = threadIdx.x % kThreadsPerRow;
#pragma unroll
    for (int p = 0; p < kPasses; ++p)
      *reinterpret_cast<u4 *>(lds + (p * kRowsPerPass + tr) * M::kLdsRow + tc * 16) = r[p];
  }
};

// One pass over a block's keys.  ACCUM = false: softmax statistics; true: weights.
// WR waves split the (padded) query rows in groups of 64, the other 4/WR split the
// four 32-key tiles of a stage.
template <int DT, int WR, bool ACCUM>
__global__ __launch_bounds__(kDeepThreads) void deep_pass(DeepParams p) {
  typedef Mma<DT> M;
  typedef Stage<DT> S;
  constexpr int WK = 4 / WR;
  constexpr int kTilesPerWave = 4 / WK;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // ACCUM: column partial sums [2][2*WR][kStageKeys] placed after the stage buffers
  float *colpart = reinterpret_cast<float *>(smem + 2 * S::kBytes);

  const int u = blockIdx.y;
  const int chunk = blockIdx.x;
  const int lane = lane_id(), wave = threadIdx.x >> 6;
  const int g = lane >> 5, c = lane & 31;
  const int wr = wave % WR, wk = wave / WR;
  const int key_begin = chunk * p.stages * kStageKeys;
  const int key_limit = ACCUM ? p.lc : p.l;   // keys at or beyond this index are not needed
  const char *Kunit = p.K + kv_unit_offset(p.lay, u);
  const size_t kpitch = (size_t)p.lay.st;
  const char *Qunit = p.Q + (size_t)u * p.R * M::kRowBytes;

  // query fragments stay in registers for the whole block
  typename M::frag qf[2][M::kSteps];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int row = 64 * wr + 32 * rb + c;
#pragma unroll
    for (int ks = 0; ks < M::kSteps; ++ks)
      qf[rb][ks] = row < p.R ? M::load(Qunit + (size_t)row * M::kRowBytes, ks, g) : M::zero();
  }

  // accumulate pass: (max, 1/sum) of every query row from the per-chunk statistics of the
  // first pass, merged in chunk order by one thread per row (every block of the unit does
  // the same sum in the same order)
  __shared__ float2 row_stats[ACCUM ? 256 : 1];
  if (ACCUM) {
    if ((int)threadIdx.x < p.Rpad) {
      const int row = threadIdx.x;
      const float2 *part = p.partial + (size_t)u * p.nchunks * p.Rpad + row;
      float m = -INFINITY, z = 0.f;
#pragma unroll 8
      for (int ch = 0; ch < p.nchunks; ++ch) {
        const float2 e = part[(size_t)ch * p.Rpad];
        if (e.y > 0.f) {
          if (e.x > m) {
            z = z * __builtin_amdgcn_exp2f(m - e.x) + e.y;
            m = e.x;
          } else {
            z += e.y * __builtin_amdgcn_exp2f(e.x - m);
          }
        }
      }
      const bool ok = row < p.R && z > 0.f;
      row_stats[row] = make_float2(ok ? m : 0.f, ok ? 1.f / z : 0.f);
    }
    __syncthreads();
  }

  // per-row state of this lane: stats pass (reference, sum); accumulate pass (max, weight)
  float s0[2][16], s1[2][16];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      if (ACCUM) {
        const int row = 64 * wr + 32 * rb + mma_row(v, g);
        const float2 st = row_stats[row];
        s0[rb][v] = st.x;
        s1[rb][v] = st.y;
      } else {
        s0[rb][v] = -INFINITY;
        s1[rb][v] = 0.f;
      }
    }

  u4 regs[S::kPasses];
  S::fetch(regs, Kunit, kpitch, key_begin, key_limit);
  S::store(regs, smem);
  __syncthreads();

  for (int s = 0; s < p.stages; ++s) {
    const int k0 = key_begin + s * kStageKeys;
    if (k0 >= key_limit) break;                       // uniform over the block
    const bool more = (s + 1 < p.stages) && (k0 + kStageKeys < key_limit);
    if (more) S::fetch(regs, Kunit, kpitch, k0 + kStageKeys, key_limit);

    if (ACCUM && s > 0 && threadIdx.x < kStageKeys) {
      // finish the previous stage: fixed-order sum of the partial column sums
      const float *cp = colpart + ((s - 1) & 1) * (2 * WR * kStageKeys);
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 2 * WR; ++j) sum += cp[j * kStageKeys + threadIdx.x];
      const int a = k0 - kStageKeys + threadIdx.x;
      if (a < p.lc) {
        float v = sum * p.inv_hn;
        if (p.norm == SPINDLE_NORM_PAPER) v = v / (float)(p.l - a);
        p.scores[(size_t)u * p.lc + a] = v;
      }
    }

    const char *lds = smem + (s & 1) * S::kBytes;
    const bool tail = !ACCUM && (k0 + kStageKeys > p.lc);   // causal mask / end of sequence
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
      const int ct = wk + t * WK;
      f16v acc[2];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][v] = 0.f;
      const char *krow = lds + (ct * 32 + c) * M::kLdsRow;
#pragma unroll
      for (int ks = 0; ks < M::kSteps; ++ks) {
        const typename M::frag kf = M::load(krow, ks, g);
        acc[0] = M::mma(qf[0][ks], kf, acc[0]);
        acc[1] = M::mma(qf[1][ks], kf, acc[1]);
      }
      if (ACCUM) {
        float cs0 = 0.f, cs1 = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          cs0 = fmaf(__builtin_amdgcn_exp2f(fmaf(acc[0][v], p.sc2, -s0[0][v])), s1[0][v], cs0);
          cs1 = fmaf(__builtin_amdgcn_exp2f(fmaf(acc[1][v], p.sc2, -s0[1][v])), s1[1][v], cs1);
        }
        colpart[(s & 1) * (2 * WR * kStageKeys) + (2 * wr + g) * kStageKeys + ct * 32 + c] = cs0 + cs1;
      } else if (!tail) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          float d[16], t_[16];
          float dmax = -INFINITY;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            t_[v] = acc[rb][v] * p.sc2;
            d[v] = t_[v] - s0[rb][v];
            dmax = fmaxf(dmax, d[v]);
          }
          if (__any(dmax > 40.f)) {      // move the reference up (always on the first tile)
#pragma unroll
            for (int v = 0; v < 16; ++v)
              if (d[v] > 0.f) {
                s1[rb][v] *= __builtin_amdgcn_exp2f(s0[rb][v] - t_[v]);
                s0[rb][v] = t_[v];
                d[v] = 0.f;
              }
          }
#pragma unroll
          for (int v = 0; v < 16; ++v) s1[rb][v] += __builtin_amdgcn_exp2f(d[v]);
        }
      } else {
        const int key = k0 + ct * 32 + c;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int row = 64 * wr + 32 * rb + mma_row(v, g);
            const bool valid = row < p.R && key < p.l && key <= p.lc + (row % p.lw);
            if (valid) {
              const float t = acc[rb][v] * p.sc2;
              if (t > s0[rb][v]) {
                s1[rb][v] = s1[rb][v] * __builtin_amdgcn_exp2f(s0[rb][v] - t) + 1.f;
                s0[rb][v] = t;
              } else {
                s1[rb][v] += __builtin_amdgcn_exp2f(t - s0[rb][v]);
              }
            }
          }
      }
    }
    if (more) S::store(regs, smem + ((s + 1) & 1) * S::kBytes);
    __syncthreads();
    if (ACCUM && !more && threadIdx.x < kStageKeys) {
      const float *cp = colpart + (s & 1) * (2 * WR * kStageKeys);
      float sum = 0.f;
#pragma unroll
      for (int j = 0; j < 2 * WR; ++j) sum += cp[j * kStageKeys + threadIdx.x];
      const int a = k0 + threadIdx.x;
      if (a < p.lc) {
        float v = sum * p.inv_hn;
        if (p.norm == SPINDLE_NORM_PAPER) v = v / (float)(p.l - a);
        p.scores[(size_t)u * p.lc + a] = v;
      }
    }
  }

  if (!ACCUM) {
    // lane partials -> LDS (swizzled slot so that the row-wise readers spread over banks)
    constexpr int kSlots = WK * 32;
    __syncthreads();
    float2 *red = reinterpret_cast<float2 *>(smem);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = 64 * wr + 32 * rb + mma_row(v, g);
        const int slot = (wk * 32 + c + row) % kSlots;
        red[row * kSlots + slot] = make_float2(s0[rb][v], s1[rb][v]);
      }
    __syncthreads();
    const int row = threadIdx.x;
    if (row < 64 * WR) {
      float m = -INFINITY;
      for (int j = 0; j < kSlots; ++j) m = fmaxf(m, red[row * kSlots + (j + row) % kSlots].x);
      float z = 0.f;
      if (m > -INFINITY)
        for (int j = 0; j < kSlots; ++j) {
          const float2 e = red[row * kSlots + (j + row) % kSlots];
          if (e.y > 0.f) z += e.y * __builtin_amdgcn_exp2f(e.x - m);
        }
      p.partial[((size_t)u * p.nchunks + chunk) * p.Rpad + row] = make_float2(m, z);
    }
  }
}

// ---------------------------------------------------------------- pool + top-k
struct SelectParams {
  const float *scores;   // [U][lc]
  float *pooled;         // [U][lc]
  float *scores_out;     // optional [U][lc]
  const int32_t *budgets;
  int32_t *kept;         // [U][out_stride]
  int l, lc, lw, pool, budget, out_stride;
};

constexpr int kSelThreads = 1024;

__device__ __forceinline__ uint32_t orderable(float f) {
  const uint32_t b = __float_as_uint(f);
  return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

constexpr int kSelInLds = 36 * 1024;   // pooled scores of a unit that fit in LDS

__global__ __launch_bounds__(kSelThreads) void deep_select(SelectParams p, int vals_in_lds) {
  extern __shared__ __attribute__((aligned(16))) uint32_t sel_lds[];
  __shared__ int hist[256];
  __shared__ int wsum[kSelThreads / 64][2];
  __shared__ uint32_t sh_prefix, sh_min, sh_max;
  __shared__ int sh_krem;
  const int u = blockIdx.x, tid = threadIdx.x, lane = lane_id();
  const int lc = p.lc;
  const float *raw = p.scores + (size_t)u * lc;
  // pooled scores as order-preserving unsigned keys: in LDS when they fit, else in the workspace
  uint32_t *pooled = vals_in_lds ? sel_lds : reinterpret_cast<uint32_t *>(p.pooled + (size_t)u * lc);
  int32_t *kept = p.kept + (size_t)u * p.out_stride;
  int budget = p.budgets ? p.budgets[u] : p.budget;
  if (budget < p.lw) budget = p.lw;
  int k = budget - p.lw;
  if (k > lc) k = lc;
  if (k > p.out_stride - p.lw) k = p.out_stride - p.lw;   // never write past the row pitch

  // 1-D max pooling, window clipped to the context; smallest and largest key of the unit
  if (tid == 0) { sh_min = 0xFFFFFFFFu; sh_max = 0u; }
  __syncthreads();
  const int r = (p.pool - 1) / 2;
  uint32_t mn = 0xFFFFFFFFu, mx = 0u;
  if (vals_in_lds) {
    // raw scores to LDS with independent coalesced loads, pooled in registers, keys back in place
    constexpr int kPer = kSelInLds / kSelThreads;
    float *rawl = reinterpret_cast<float *>(sel_lds);
    float pm[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {                 // all loads of the thread in flight together
      const int a = tid + i * kSelThreads;
      pm[i] = a < lc ? raw[a] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int a = tid + i * kSelThreads;
      if (a < lc) rawl[a] = pm[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int a = tid + i * kSelThreads;
      float m = -INFINITY;
      if (a < lc) {
        const int lo = a - r < 0 ? 0 : a - r, hi = a + r >= lc ? lc - 1 : a + r;
        for (int j = lo; j <= hi; ++j) m = fmaxf(m, rawl[j]);
      }
      pm[i] = m;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int a = tid + i * kSelThreads;
      if (a < lc) {
        const uint32_t x = orderable(pm[i]);
        pooled[a] = x;
        mn = x < mn ? x : mn;
        mx = x > mx ? x : mx;
        if (p.scores_out) p.scores_out[(size_t)u * lc + a] = pm[i];
      }
    }
  } else {
    for (int a = tid; a < lc; a += kSelThreads) {
      float m = raw[a];
      const int lo = a - r < 0 ? 0 : a - r, hi = a + r >= lc ? lc - 1 : a + r;
      for (int j = lo; j <= hi; ++j) m = fmaxf(m, raw[j]);
      const uint32_t x = orderable(m);
      pooled[a] = x;
      mn = x < mn ? x : mn;
      mx = x > mx ? x : mx;
      if (p.scores_out) p.scores_out[(size_t)u * lc + a] = m;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const uint32_t a = __shfl_xor(mn, o), b = __shfl_xor(mx, o);
    mn = a < mn ? a : mn;
    mx = b > mx ? b : mx;
  }
  if (lane == 0) { atomicMin(&sh_min, mn); atomicMax(&sh_max, mx); }
  __syncthreads();

  // Value of the k-th largest pooled score by most-significant-digit radix select.  The bits
  // all keys share (scores of one unit have similar exponents) are skipped: they would send
  // every key to the same counter.
  uint32_t prefix = sh_max;
  int krem = k;   // how many still to take among the keys matching `prefix`
  if (k > 0 && k < lc && sh_min != sh_max) {
    int bits_left = 32 - __builtin_clz(sh_min ^ sh_max);      // 1 .. 32 low bits still undecided
    prefix = bits_left == 32 ? 0u : (sh_max >> bits_left) << bits_left;
    while (bits_left > 0) {
      const int w = bits_left < 8 ? bits_left : 8, shift = bits_left - w;
      const uint32_t dmask = (1u << w) - 1u;
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      constexpr int kAtOnce = 4;                        // independent keys per thread and trip
      for (int a0 = 0; a0 < lc; a0 += kAtOnce * kSelThreads) {
        uint32_t x[kAtOnce];
#pragma unroll
        for (int q = 0; q < kAtOnce; ++q) {
          const int a = a0 + q * kSelThreads + tid;
          x[q] = a < lc ? pooled[a] : 0u;
        }
#pragma unroll
        for (int q = 0; q < kAtOnce; ++q) {
          const int a = a0 + q * kSelThreads + tid;
          const bool in = a < lc && (bits_left == 32 || (x[q] >> bits_left) == (prefix >> bits_left));
          const int d = (int)((x[q] >> shift) & dmask);
          if (in) {
            // scores of one unit crowd into few digits: the digit of the first lane that takes
            // part is counted once for all lanes that share it
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
        int above = mine;                                     // inclusive sum over lanes >= t
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const int x = __shfl_down(above, o);
          if (tid + o < 64) above += x;
        }
        above -= mine;                                        // keys in counters of higher lanes
        const int hh[4] = {h0, h1, h2, h3};
        int run = above;
#pragma unroll
        for (int j = 3; j >= 0; --j) {
          if (run < krem && krem <= run + hh[j]) {
            sh_prefix = prefix | ((uint32_t)(4 * tid + j) << shift);
            sh_krem = krem - run;
          }
          run += hh[j];
        }
      }
      __syncthreads();
      prefix = sh_prefix;
      krem = sh_krem;
      bits_left = shift;
      __syncthreads();
    }
  }
  // ordered compaction: everything above the threshold, then the first `krem` equal to it.
  // Each wave owns a contiguous run of positions and walks it 64 at a time (coalesced,
  // conflict-free); ranks within a step come from ballots, the offset of the wave from a
  // count pass and a scan over the waves.
  if (k >= lc) {
    for (int a = tid; a < lc; a += kSelThreads) kept[a] = a;
  } else if (k > 0) {
    constexpr int kWaves = kSelThreads / 64;
    const int wave = tid >> 6;
    const int run = (((lc + kWaves - 1) / kWaves) + 63) & ~63;
    const int w0 = wave * run, w1 = w0 + run < lc ? w0 + run : lc;
    const unsigned long long below = (1ull << lane) - 1ull;
    int ngt = 0, neq = 0;                              // wave-uniform
    for (int a0 = w0; a0 < w1; a0 += 64) {
      const int a = a0 + lane;
      const uint32_t x = a < w1 ? pooled[a] : 0u;
      ngt += __popcll(__ballot(a < w1 && x > prefix));
      neq += __popcll(__ballot(a < w1 && x == prefix));
    }
    if (lane == 0) { wsum[wave][0] = ngt; wsum[wave][1] = neq; }
    __syncthreads();
    int gt_seen = 0, eq_seen = 0;
    for (int w = 0; w < wave; ++w) { gt_seen += wsum[w][0]; eq_seen += wsum[w][1]; }
    for (int a0 = w0; a0 < w1; a0 += 64) {
      const int a = a0 + lane;
      const uint32_t x = a < w1 ? pooled[a] : 0u;
      const bool gt = a < w1 && x > prefix, eq = a < w1 && x == prefix;
      const unsigned long long mgt = __ballot(gt), meq = __ballot(eq);
      const int gt_before = gt_seen + __popcll(mgt & below), eq_before = eq_seen + __popcll(meq & below);
      if (gt) kept[gt_before + (eq_before < krem ? eq_before : krem)] = a;
      else if (eq && eq_before < krem) kept[gt_before + eq_before] = a;
      gt_seen += __popcll(mgt);
      eq_seen += __popcll(meq);
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
  float *scores, *pooled;
  size_t bytes;
};

DeepLayout deep_layout(void *ws, int U, int l, int lw, int Rpad) {
  Carver cv(ws);
  DeepLayout L;
  const int keys = stages_per_block(U, l) * kStageKeys;
  const int nchunks = (l + keys - 1) / keys;
  const int lc = l - lw;
  L.partial = cv.take<float2>((size_t)U * nchunks * Rpad);
  L.scores = cv.take<float>((size_t)U * (lc > 0 ? lc : 1));
  L.pooled = cv.take<float>((size_t)U * (lc > 0 ? lc : 1));
  L.bytes = cv.total();
  return L;
}

int padded_rows(int R) { return R <= 64 ? 64 : (R <= 128 ? 128 : 256); }

template <int DT, int WR>
spindle_status launch_passes(const DeepParams &p, int U, hipStream_t st) {
  typedef Stage<DT> S;
  const size_t smem_stats = 2 * (size_t)S::kBytes > 65536 ? 2 * (size_t)S::kBytes : 65536;
  const size_t smem_acc = 2 * (size_t)S::kBytes + 2 * 2 * WR * kStageKeys * sizeof(float);
  static LdsLimit lim_stats, lim_acc;                     // one pair per instantiation; the sizes are constants of it
  if (spindle_status e = allow_lds(lim_stats, reinterpret_cast<const void *>(&deep_pass<DT, WR, false>), smem_stats)) return e;
  if (spindle_status e = allow_lds(lim_acc, reinterpret_cast<const void *>(&deep_pass<DT, WR, true>), smem_acc)) return e;
  { ProfScope ps("deep_stats", st);
  hipLaunchKernelGGL((deep_pass<DT, WR, false>), dim3(p.nchunks, U), dim3(kDeepThreads), smem_stats, st, p); }
  if (p.lc > 0) {
    const int nacc = (p.lc + p.stages * kStageKeys - 1) / (p.stages * kStageKeys);
    ProfScope ps("deep_accumulate", st);
    hipLaunchKernelGGL((deep_pass<DT, WR, true>), dim3(nacc, U), dim3(kDeepThreads), smem_acc, st, p);
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
  *bytes = deep_layout(nullptr, U, desc->seq_len, window, padded_rows(window * desc->group_size)).bytes;
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
  DeepLayout L = deep_layout(workspace, U, l, lw, Rpad);

  DeepParams p;
  KvLayout lay;
  s = kv_layout(desc, &lay);
  if (s != SPINDLE_OK) return s;
  p.K = static_cast<const char *>(K);
  p.lay = lay;
  p.Q = static_cast<const char *>(Qw);
  p.partial = L.partial;
  p.scores = L.scores;
  p.l = l; p.lc = lc; p.lw = lw; p.hn = desc->group_size; p.R = R; p.Rpad = Rpad;
  p.stages = stages_per_block(U, l);
  p.nchunks = (l + p.stages * kStageKeys - 1) / (p.stages * kStageKeys);
  p.sc2 = scale * kLog2e;
  p.inv_hn = 1.0f / (float)desc->group_size;
  p.norm = norm;
  if (desc->dtype == SPINDLE_F16) s = launch_dtype<SPINDLE_F16>(p, U, st);
  else if (desc->dtype == SPINDLE_BF16) s = launch_dtype<SPINDLE_BF16>(p, U, st);
  else s = launch_dtype<SPINDLE_F32>(p, U, st);
  if (s != SPINDLE_OK) return s;

  SelectParams sp;
  sp.scores = L.scores; sp.pooled = L.pooled; sp.scores_out = scores_out;
  sp.budgets = budgets; sp.kept = kept_idx;
  sp.l = l; sp.lc = lc; sp.lw = lw; sp.pool = pool_kernel; sp.budget = budget; sp.out_stride = out_stride;
  {
    const int vals_in_lds = lc <= kSelInLds;
    const size_t sel_lds = vals_in_lds ? (size_t)lc * sizeof(uint32_t) : 0;
    static LdsLimit lim_select;
    if (spindle_status e = allow_lds(lim_select, reinterpret_cast<const void *>(&deep_select), kSelInLds * sizeof(uint32_t))) return e;
    ProfScope ps("deep_select", st);
    hipLaunchKernelGGL(deep_select, dim3(U), dim3(kSelThreads), sel_lds, st, sp, vals_in_lds);
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
