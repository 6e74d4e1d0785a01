// Shared device/host helpers of the POET-X HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "poetx.h"

namespace poetx {

typedef long long i64;

// Raw bf16 storage; arithmetic is always done in fp32.
struct bf16_t {
  uint16_t v;
};

__host__ __device__ inline float bf16_bits_to_float(uint16_t v) {
  union {
    uint32_t u;
    float f;
  } c;
  c.u = ((uint32_t)v) << 16;
  return c.f;
}

// Round to nearest even on the fp32 bit pattern (inputs here are finite).
__host__ __device__ inline uint16_t float_to_bf16_bits(float f) {
  union {
    uint32_t u;
    float f;
  } c;
  c.f = f;
  uint32_t u = c.u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ inline float to_float(float x) { return x; }
__device__ inline float to_float(bf16_t x) { return bf16_bits_to_float(x.v); }

template <class T>
__device__ inline T from_float(float f);
template <>
__device__ inline float from_float<float>(float f) {
  return f;
}
template <>
__device__ inline bf16_t from_float<bf16_t>(float f) {
  bf16_t r;
  r.v = float_to_bf16_bits(f);
  return r;
}

// Slot of (i, j), i < j, in the row-major strict upper triangle of a b x b matrix (Sec. 3.4).
__host__ __device__ inline i64 packed_index(int i, int j, int b) {
  return (i64)i * b - ((i64)i * (i + 1)) / 2 + (j - i - 1);
}

__host__ __device__ inline int ceil_div(i64 a, i64 b) { return (int)((a + b - 1) / b); }

// Side of block j of a dimension d tiled by b (b except possibly for the last block).
__host__ __device__ inline int block_side(int d, int b, int j) {
  int rem = d - j * b;
  return rem < b ? rem : b;
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Convert the status of the launches enqueued so far into a poetx_status.
inline int launch_status() { return hipGetLastError() == hipSuccess ? POETX_OK : POETX_ERR_HIP; }

}  // namespace poetx
