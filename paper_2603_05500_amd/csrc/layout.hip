// Token-major <-> feature-major conversion of activations (the permutation operator of
// Sec. 3.2 / Eq. 5 acts on features: in the library's native feature-major layout it is a gather of
// whole rows and costs nothing; a caller that holds [tokens][features] tensors gets them
// re-laid once on the way in and once on the way out).  Plain out-of-place transpose through an
// LDS tile: 16-byte coalesced loads along the source rows, 16-byte coalesced stores along the
// destination rows; HBM bound.
#include "poetx_kernels.h"

namespace poetx {
namespace {

constexpr int TT = 64;   // tile side in elements

// in: R x C row major (ld_in), out: C x R row major (ld_out).  One 64 x 64 tile per workgroup.
template <class T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* __restrict__ in, T* __restrict__ out, i64 R, i64 C,
                                                        i64 ld_in, i64 ld_out) {
  constexpr int V = 16 / sizeof(T);          // elements per 16-byte vector
  constexpr int VPR = TT / V;                // vectors per tile row
  constexpr int RPP = 256 / VPR;             // tile rows per pass
  __shared__ T tile[TT][TT + 2];             // +2: column walks hit different banks
  const i64 r0 = (i64)blockIdx.y * TT, c0 = (i64)blockIdx.x * TT;
  const int tid = threadIdx.x;
  const int vr = tid / VPR, vc = (tid % VPR) * V;
  const bool full = r0 + TT <= R && c0 + TT <= C && (ld_in % V) == 0 && (ld_out % V) == 0 &&
                    ((uintptr_t)in % 16) == 0 && ((uintptr_t)out % 16) == 0;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  union Vec {
    u32x4 v;
    T e[V];
  };
  if (full) {
#pragma unroll
    for (int p = 0; p < TT / RPP; ++p) {
      const int r = vr + p * RPP;
      Vec x;
      x.v = *reinterpret_cast<const u32x4*>(in + (r0 + r) * ld_in + c0 + vc);
#pragma unroll
      for (int e = 0; e < V; ++e) tile[r][vc + e] = x.e[e];
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < TT / RPP; ++p) {
      const int c = vr + p * RPP;             // source column = destination row
      Vec x;
#pragma unroll
      for (int e = 0; e < V; ++e) x.e[e] = tile[vc + e][c];
      *reinterpret_cast<u32x4*>(out + (c0 + c) * ld_out + r0 + vc) = x.v;
    }
  } else {   // ragged edge or unaligned: element by element
    for (int i = tid; i < TT * TT; i += 256) {
      const int r = i / TT, c = i % TT;
      if (r0 + r < R && c0 + c < C) tile[r][c] = in[(r0 + r) * ld_in + c0 + c];
    }
    __syncthreads();
    for (int i = tid; i < TT * TT; i += 256) {
      const int c = i / TT, r = i % TT;
      if (r0 + r < R && c0 + c < C) out[(c0 + c) * ld_out + r0 + r] = tile[r][c];
    }
  }
}

}  // namespace

void transpose_launch(int dtype, const void* in, void* out, i64 R, i64 C, hipStream_t st) {
  dim3 grid((unsigned)ceil_div(C, TT), (unsigned)ceil_div(R, TT));
  if (dtype == POETX_F32)
    hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, st, (const float*)in, (float*)out, R, C, C, R);
  else
    hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)in, (uint16_t*)out, R, C, C, R);
}

}  // namespace poetx
