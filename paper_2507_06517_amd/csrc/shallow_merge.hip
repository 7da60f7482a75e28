// Greedy highest-degree codebook construction (Alg. 1, Eq. 11-13) on the neighbour lists.
#include "shallow.h"

namespace spindle {
namespace {

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

}  // namespace

spindle_status launch_merge(const ShallowParams &p, hipStream_t st) {
  const int n = p.n;
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
  static LdsLimit lim_onehop, lim_update, lim_merge;      // raised once per device to the largest size in use
  if (spindle_status e = allow_lds(lim_onehop, reinterpret_cast<const void *>(&merge_onehop), kKeysInLds * sizeof(uint32_t))) return e;
  const size_t dead_lds = (size_t)p.n16;
  if (spindle_status e = allow_lds(lim_update, reinterpret_cast<const void *>(&merge_update), 65536)) return e;
  if (spindle_status e = allow_lds(lim_merge, reinterpret_cast<const void *>(&shallow_merge),
                                   (kKeysInLds + kKeysInLds / 32) * sizeof(uint32_t))) return e;
  for (int round = 0; round < kGridRounds; ++round) {
    ProfScope ps("shallow_merge_grid", st);
    hipLaunchKernelGGL(merge_onehop, dim3(ox, p.UT), dim3(kMergeThreads), key_lds, st, p, round, keys_in_lds);
    hipLaunchKernelGGL(merge_twohop, tg, dim3(kPhaseThreads), 0, st, p, round);
    hipLaunchKernelGGL(merge_update, dim3(ox, p.UT), dim3(kMergeThreads), dead_lds, st, p, round);   // 1024 threads: fewer copies of the flags
  }
  const size_t merge_lds = n <= kKeysInLds ? ((size_t)((n + 3) & ~3) + (n + 31) / 32) * sizeof(uint32_t) : 0;
  { ProfScope ps("shallow_merge", st);
  hipLaunchKernelGGL(shallow_merge, dim3(p.UT), dim3(kMergeThreads), merge_lds, st, p); }
  SPINDLE_HIP(hipGetLastError());
  return SPINDLE_OK;
}

}  // namespace spindle
