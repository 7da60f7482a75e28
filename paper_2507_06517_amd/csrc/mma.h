// MFMA operand traits for the 32x32 matrix-core tiles used by both paths.
//
// D[i][j] += sum_k A[i][k] * B[k][j] on one 64-lane wave.  Lane l = 32*g + c supplies
//   A: row i = c, and B: column j = c, each with the k-slice owned by lane group g
//   (fp16/bf16: 8 consecutive k at 16*ks + 8*g; fp32: the single k = 2*ks + g).
// Both operands are therefore read from row-major [row][k] storage with the same
// address pattern.  The result register v = 4*blk + e of lane (g, c) holds
//   D[8*blk + 4*g + e][c].
#pragma once

#include "common.h"

namespace spindle {

template <int DT>
struct Mma;

template <>
struct Mma<SPINDLE_F16> {
  typedef h8 frag;
  static constexpr int kSteps = 8;
  static constexpr int kRowBytes = 256;
  static constexpr int kLdsRow = 272;  // +16 B pad: rows start 4 banks apart
  static __device__ __forceinline__ frag load(const char *row, int ks, int g) {
    return *reinterpret_cast<const frag *>(row + ks * 32 + g * 16);
  }
  static __device__ __forceinline__ frag zero() { return frag{0, 0, 0, 0, 0, 0, 0, 0}; }
  static __device__ __forceinline__ f16v mma(frag a, frag b, f16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
};

template <>
struct Mma<SPINDLE_BF16> {
  typedef b8 frag;
  static constexpr int kSteps = 8;
  static constexpr int kRowBytes = 256;
  static constexpr int kLdsRow = 272;
  static __device__ __forceinline__ frag load(const char *row, int ks, int g) {
    return *reinterpret_cast<const frag *>(row + ks * 32 + g * 16);
  }
  static __device__ __forceinline__ frag zero() {
    u4 z = {0, 0, 0, 0};
    return __builtin_bit_cast(frag, z);
  }
  static __device__ __forceinline__ f16v mma(frag a, frag b, f16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};

template <>
struct Mma<SPINDLE_F32> {
  typedef float frag;
  static constexpr int kSteps = 64;
  static constexpr int kRowBytes = 512;
  static constexpr int kLdsRow = 528;  // keeps 16-byte alignment of staged chunks
  static __device__ __forceinline__ frag load(const char *row, int ks, int g) {
    return *reinterpret_cast<const float *>(row + (2 * ks + g) * 4);
  }
  static __device__ __forceinline__ frag zero() { return 0.f; }
  static __device__ __forceinline__ f16v mma(frag a, frag b, f16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
  }
};

// Row of the 32-row tile that result register v of lane group g holds.
__device__ __forceinline__ int mma_row(int v, int g) { return 8 * (v >> 2) + 4 * g + (v & 3); }

}  // namespace spindle
