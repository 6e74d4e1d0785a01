// INT8 storage of the frozen base weight (Sec. 3.6, POET-XQ): symmetric absmax codes with one
// fp32 scale per output row, W[i][k] ~ scale[i] * q[i][k].  The layer calls dequantise the
// weight into the caller's workspace right before the dense product and keep nothing, so
// the only weight that persists is the 8-bit one.  Both kernels are plain HBM streams.
#include "poetx_kernels.h"

namespace poetx {
namespace {

template <class T>
__global__ __launch_bounds__(256) void quantize_rows_kernel(const T* __restrict__ W, int m, int8_t* __restrict__ q,
                                                            float* __restrict__ scale) {
  __shared__ float red[256];
  const int i = blockIdx.x, tid = threadIdx.x;
  const T* row = W + (i64)i * m;
  float amax = 0.f;
  for (int k = tid; k < m; k += 256) amax = fmaxf(amax, fabsf(to_float(row[k])));
  red[tid] = amax;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) red[tid] = fmaxf(red[tid], red[tid + s]);
    __syncthreads();
  }
  amax = red[0];
  const float sc = amax > 0.f ? amax / 127.0f : 1.0f;
  if (tid == 0) scale[i] = sc;
  int8_t* out = q + (i64)i * m;
  for (int k = tid; k < m; k += 256) {
    float c = rintf(to_float(row[k]) / sc);   // IEEE division and round-half-even, as the definition says
    c = fminf(fmaxf(c, -127.f), 127.f);
    out[k] = (int8_t)c;
  }
}

// 16 codes per thread: one 16-byte load, the row's scale, 16 products, stores in the layer's dtype.
template <class T>
__global__ __launch_bounds__(256) void dequantize_kernel(const int8_t* __restrict__ q, const float* __restrict__ scale,
                                                         int m, i64 total16, T* __restrict__ W) {
  const i64 g = (i64)blockIdx.x * 256 + threadIdx.x;
  if (g >= total16) return;
  const i64 e0 = g * 16;
  const float sc = scale[e0 / m];
  typedef int int4v __attribute__((ext_vector_type(4)));
  const int4v v = *reinterpret_cast<const int4v*>(q + e0);
  T* o = W + e0;
#pragma unroll
  for (int w = 0; w < 4; ++w)
#pragma unroll
    for (int c = 0; c < 4; ++c) o[4 * w + c] = from_float<T>(sc * (float)(int8_t)(v[w] >> (8 * c)));
}

template <class T>
__global__ void dequantize_tail_kernel(const int8_t* __restrict__ q, const float* __restrict__ scale, int m, i64 first,
                                       i64 total, T* __restrict__ W) {
  const i64 e = first + (i64)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < total) W[e] = from_float<T>(scale[e / m] * (float)q[e]);
}

}  // namespace

size_t weight_q8_scale_offset(int n, int m) { return align256((size_t)n * m); }

void weight_quantize_q8_launch(int dtype, const void* W, int n, int m, void* Wq, hipStream_t st) {
  int8_t* q = (int8_t*)Wq;
  float* scale = (float*)((char*)Wq + weight_q8_scale_offset(n, m));
  if (dtype == POETX_F32)
    hipLaunchKernelGGL(quantize_rows_kernel<float>, dim3(n), dim3(256), 0, st, (const float*)W, m, q, scale);
  else
    hipLaunchKernelGGL(quantize_rows_kernel<bf16_t>, dim3(n), dim3(256), 0, st, (const bf16_t*)W, m, q, scale);
}

// A row may start anywhere modulo 16 when m is not a multiple of 16, so groups of 16 codes are
// only used when m is; otherwise every element goes through the scalar kernel.
void weight_dequantize_q8_launch(const void* Wq, int n, int m, int dtype, void* W_out, hipStream_t st) {
  const int8_t* q = (const int8_t*)Wq;
  const float* scale = (const float*)((const char*)Wq + weight_q8_scale_offset(n, m));
  const i64 total = (i64)n * m;
  const i64 total16 = (m % 16 == 0) ? total / 16 : 0;
  if (total16 > 0) {
    if (dtype == POETX_F32)
      hipLaunchKernelGGL(dequantize_kernel<float>, dim3(ceil_div(total16, 256)), dim3(256), 0, st, q, scale, m, total16,
                         (float*)W_out);
    else
      hipLaunchKernelGGL(dequantize_kernel<bf16_t>, dim3(ceil_div(total16, 256)), dim3(256), 0, st, q, scale, m,
                         total16, (bf16_t*)W_out);
  } else {
    if (dtype == POETX_F32)
      hipLaunchKernelGGL(dequantize_tail_kernel<float>, dim3(ceil_div(total, 256)), dim3(256), 0, st, q, scale, m,
                         (i64)0, total, (float*)W_out);
    else
      hipLaunchKernelGGL(dequantize_tail_kernel<bf16_t>, dim3(ceil_div(total, 256)), dim3(256), 0, st, q, scale, m,
                         (i64)0, total, (bf16_t*)W_out);
  }
}

}  // namespace poetx
