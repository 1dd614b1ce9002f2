// Shared device/host helpers of the MaskKV HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/maskkv.h"

namespace maskkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

struct bf16_t {
  uint16_t bits;
};

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;  // finite stand-in for -inf in running maxima

// Device-side view of a [B, H, T, d] tensor: per-sequence base offsets are resolved on the host.
struct View {
  char* ptr;
  int64_t stride_h;             // bytes
  int64_t stride_t;             // bytes
  int64_t boff[MASKKV_MAX_BATCH];  // bytes: b*stride_b + seq_start[b]*stride_t

  __device__ __forceinline__ char* row(int b, int h, int64_t t) const {
    return ptr + boff[b] + (int64_t)h * stride_h + t * stride_t;
  }
  // Query row r of key/value head h when g query heads of n_per rows each share that head:
  // rows [gi*n_per, (gi+1)*n_per) are query head h*g + gi.
  __device__ __forceinline__ char* group_row(int b, int h, int g, int n_per, int r) const {
    const int gi = r / n_per;
    return row(b, h * g + gi, r - gi * n_per);
  }
};

// Query heads that share one key/value head (1 for plain multi-head attention).
__host__ __device__ inline int query_heads_per_kv(const maskkv_desc* d) { return d->q_per_kv > 1 ? d->q_per_kv : 1; }

struct Lens {
  int32_t P[MASKKV_MAX_BATCH];  // prompt length per sequence
};

// ---------------------------------------------------------------------------------------------
// MFMA 32x32 fragments.  A "fragment" is 16 bytes per lane: lane (r = lane%32, g = lane/32) holds
// bytes [32*ks + 16*g, +16) of row r of its operand.  For bf16 that is one 32x32x16 MFMA (k-slot
// 8g+e <-> element 16ks+8g+e); for fp32 it is four 32x32x2 MFMAs (MFMA q, k-slot g <-> element
// 8ks+4g+q).  Both operands use the same map, so the contraction over the head dimension is exact.
// Accumulator element i of lane (c = lane%32, g) is row 8*(i/4) + 4*g + i%4, column c.
// ---------------------------------------------------------------------------------------------
// Scalar bit reinterpretation by value.  (A bit_cast applied directly to a vector element expression
// was observed to read element 0 for every index, so elements are always copied to a scalar first.)
__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

template <typename T>
__device__ __forceinline__ void mfma_step(const u32x4& a, const u32x4& b, f32x16& acc);

template <>
__device__ __forceinline__ void mfma_step<bf16_t>(const u32x4& a, const u32x4& b, f32x16& acc) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                acc, 0, 0, 0);
}

template <>
__device__ __forceinline__ void mfma_step<float>(const u32x4& a, const u32x4& b, f32x16& acc) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint32_t ua = a[q], ub = b[q];
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(as_f32(ua), as_f32(ub), acc, 0, 0, 0);
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = as_u32(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// Two floats -> two bf16 (round to nearest even) in one 32-bit word, lo in the low half.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ float xor32(float v) { return __shfl_xor(v, 32, 64); }

// Host-side error plumbing (api.hip).
void set_error(const char* fmt, ...);
int check_launch(const char* what);

}  // namespace maskkv
