// Shared host/device helpers of the HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <atomic>

#include "spindle.h"

namespace spindle {

constexpr int kHeadDim = 128;
constexpr int kWave = 64;

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------- error reporting
void set_error(const char *fmt, ...);
spindle_status check_desc(const spindle_kv_desc *d);

// Where the rows of the input tensors K and V are: byte strides between batches, heads and tokens.
struct KvLayout {
  long long sb, sh, st;
  int H;
};
spindle_status kv_layout(const spindle_kv_desc *d, KvLayout *out);   // validates the strides of d
__host__ __device__ inline size_t kv_unit_offset(const KvLayout &L, int unit) {
  return (size_t)(unit / L.H) * (size_t)L.sb + (size_t)(unit % L.H) * (size_t)L.sh;
}

#define SPINDLE_FAIL(code, ...)        \
  do {                                 \
    ::spindle::set_error(__VA_ARGS__); \
    return (code);                     \
  } while (0)

#define SPINDLE_HIP(call)                                                            \
  do {                                                                               \
    hipError_t e_ = (call);                                                          \
    if (e_ != hipSuccess) SPINDLE_FAIL(SPINDLE_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

// Brackets one kernel launch with HIP events on its stream while profiling is enabled.
struct ProfScope {
  int idx;
  hipStream_t st;
  ProfScope(const char *name, hipStream_t s);
  ~ProfScope();
};

// A kernel may only be launched with more dynamic LDS than the default limit after that limit
// was raised for it, per device.  allow_lds raises it to `bytes`, the largest size the kernel is
// ever launched with, on the first call per device (one LdsLimit object per kernel), so that
// no call depends on what another thread asked for and later calls cost nothing.
struct LdsLimit {
  std::atomic<uint64_t> devices{0};   // bit d: done on device d
};
spindle_status allow_lds(LdsLimit &state, const void *kernel, size_t bytes);

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline int dtype_bytes(int dt) { return dt == SPINDLE_F32 ? 4 : 2; }

// Bump allocator over the caller's workspace.
struct Carver {
  char *base;
  size_t off = 0;
  explicit Carver(void *p) : base(static_cast<char *>(p)) {}
  template <typename T>
  T *take(size_t count) {
    off = align_up(off, 256);
    T *r = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off += count * sizeof(T);
    return r;
  }
  size_t total() const { return align_up(off, 256); }
};

// ---------------------------------------------------------------- element access
template <int DT>
struct Elem;
template <>
struct Elem<SPINDLE_F32> {
  typedef float type;
  static __device__ __forceinline__ float to_float(float v) { return v; }
  static __device__ __forceinline__ float from_float(float v) { return v; }
};
template <>
struct Elem<SPINDLE_F16> {
  typedef _Float16 type;
  static __device__ __forceinline__ float to_float(_Float16 v) { return (float)v; }
  static __device__ __forceinline__ _Float16 from_float(float v) { return (_Float16)v; }
};
template <>
struct Elem<SPINDLE_BF16> {
  typedef uint16_t type;
  static __device__ __forceinline__ float to_float(uint16_t v) {
    return __uint_as_float(((uint32_t)v) << 16);
  }
  static __device__ __forceinline__ uint16_t from_float(float v) {  // round to nearest even
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
  }
};

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

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

// The same load with the address split into a base that is the same for the whole wave (scalar
// registers) and a 32-bit byte offset per lane: no vector instruction is spent on the address.
__device__ __forceinline__ void lds_dma16_at(const void *wave_base, uint32_t lane_offset, uint32_t lds_addr) {
  const uint64_t b = reinterpret_cast<uint64_t>(wave_base);
  // (readfirstlane returns a signed int: widen it as unsigned, or a low half with its top bit set
  // would fill the high half with ones)
  const uint64_t sb = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(b >> 32)) << 32) |
                      (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(lane_offset), "s"(sb)
               : "memory", "m0");
}

// Spread the four nibbles of a 16-bit value to bits [8k, 8k+4) of a 32-bit word.
__device__ __forceinline__ uint32_t spread_nibbles(uint32_t p) {
  return (p & 0xFu) | ((p & 0xF0u) << 4) | ((p & 0xF00u) << 8) | ((p & 0xF000u) << 12);
}

}  // namespace spindle
