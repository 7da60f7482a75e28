// Codebook order, outputs and the codebook cap (Alg. 1; Eq. 4 for the re-pointed tokens).
#include "mma.h"
#include "shallow.h"

namespace spindle {
namespace {

// One codebook vector: the unit vector of a picked token, in the input type.
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
  const int lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), g = lane >> 5, c = lane & 31;
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
      lds_dma16_at(Xh, (uint32_t)tokq[q] * 256u + spiece[q], stage_lds + bufsel * kStageBytes + (wave * 4 + q) * 1024);
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
    // bit v of `hits`: a[v] >= thr, from the sign of a[v] - thr (sixteen tests and branches, one per
    // value, cost several times the matrix instructions of the tile; hits are rare)
    uint32_t miss = 0;
#pragma unroll
    for (int v = 15; v >= 0; --v) miss = __builtin_amdgcn_alignbit(miss, __float_as_uint(a[v] - thr), 31);
    uint32_t hits = valid[cb] ? ~miss & 0xFFFFu : 0u;
    if (hits) {
      uint2 *list = cand + ((size_t)slot[cb] * 2 + g) * kCandCap;
      do {
        const int v = __builtin_ctz(hits);
        hits &= hits - 1;
        float val = a[0];
#pragma unroll
        for (int u = 1; u < 16; ++u) val = v == u ? a[u] : val;
        if (cnt[cb] < kCandCap) list[cnt[cb]] = make_uint2((uint32_t)(j0 + 16 * g + v), __float_as_uint(val));
        ++cnt[cb];
      } while (hits);
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

}  // namespace

spindle_status launch_codebook(const ShallowParams &p, hipStream_t st) {
  const int n = p.n;
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
  SPINDLE_HIP(hipGetLastError());
  return SPINDLE_OK;
}

}  // namespace spindle
