// Shared declarations of the gfx950 clustered sparse-attention library (internal).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/adacluster.h"

namespace adac {

typedef uint16_t bf16raw;   // storage of one bfloat16

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;

__device__ __forceinline__ float bf16_to_f32(bf16raw v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even fp32 -> bf16 (inputs here are finite)
__device__ __forceinline__ bf16raw f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16raw)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_t x = {lo, hi};
  bf16x2_t y = __builtin_convertvector(x, bf16x2_t);
  return *reinterpret_cast<uint32_t*>(&y);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
};
template <> struct Elem<bf16raw> {
  static __device__ __forceinline__ float load(const bf16raw* p) { return bf16_to_f32(*p); }
};

// per-head state of the multi-stage key clustering (Algorithm 1), device resident
struct KState {
  int32_t ucount;      // |U|
  int32_t ccount;      // |C| so far
  int32_t m_t;         // centres of the running stage
  int32_t stage;       // t
  int32_t done;        // the stage loop has ended for this head
  int32_t full;        // F
  int32_t active;      // this stage runs (set by stage_begin)
  int32_t pad;
  int32_t stage_offs[ADACLUSTER_MAX_STAGES + 1];
  int32_t u_hist[ADACLUSTER_MAX_STAGES + 1];   // |U| at the head of stage t; entry `stage` = what staging left over
};

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace adac
