// poetx_limits: what the MI355X in front of you sustains, next to what the dense product of the
// library gets out of it.  Measurement tool, not part of the library.
//   1. matrix-core rate of a loop of nothing but v_mfma_f32_32x32x16_bf16 (one wave per SIMD with a
//      128 x 128 accumulator tile, and two waves per SIMD), with operands of zeros and with normally
//      distributed operands: the sustained clock, and with it the ceiling of any bf16 product,
//      depends on how many bits the operands toggle;
//   2. plain device-to-device copy rate (the ceiling of the HBM-bound stages);
//   3. the library's dense product (same kernel, same launch) on one llama-8B shape, as it is and
//      with its direct-to-LDS loads and / or its LDS fragment reads switched off inside the loop
//      (results are then wrong; the timing shows what feeding the matrix cores costs).
// Every timing is taken after a sustained warm-up: the first ~10 ms after an idle period run at a
// higher clock than the chip holds.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "mfma_dense_kernel.h"

namespace poetx {
StageTimer::StageTimer(int, hipStream_t st) : st_(st), idx_(-1) {}
StageTimer::~StageTimer() {}
}  // namespace poetx

using namespace poetx;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

#define CHECK(x)                                                                    \
  do {                                                                              \
    hipError_t e_ = (x);                                                            \
    if (e_ != hipSuccess) {                                                         \
      printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
      exit(1);                                                                      \
    }                                                                               \
  } while (0)

// 4 x 4 MFMA tiles per wave (the dense kernel's wave tile), operands fixed in registers
__global__ __launch_bounds__(256) void mfma_loop_kernel(const bf16x8* __restrict__ src, float* out, int iters) {
  bf16x8 a[4], b[4];
  const int tid = blockIdx.x * 256 + threadIdx.x;
  for (int i = 0; i < 4; ++i) a[i] = src[(size_t)i * 65536 + (tid & 65535)];
  for (int i = 0; i < 4; ++i) b[i] = src[(size_t)(4 + i) * 65536 + (tid & 65535)];
  floatx16 acc[4][4];
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j)
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    bf16x8 t = a[0];   // rotate, so that consecutive iterations do not repeat operand / accumulator pairs
    a[0] = a[1]; a[1] = a[2]; a[2] = a[3]; a[3] = t;
  }
  float s = 0;
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j)
      for (int v = 0; v < 16; ++v) s += acc[i][j][v];
  out[tid] = s;
}

// the same wave tile (128 x 128) out of 8 x 8 tiles of v_mfma_f32_16x16x32_bf16: twice the operand
// register reads per flop, half the accumulator traffic
__global__ __launch_bounds__(256) void mfma16_loop_kernel(const bf16x8* __restrict__ src, float* out, int iters) {
  typedef float floatx4 __attribute__((ext_vector_type(4)));
  bf16x8 a[8], b[8];
  const int tid = blockIdx.x * 256 + threadIdx.x;
  for (int i = 0; i < 8; ++i) a[i] = src[(size_t)(i & 3) * 65536 + ((tid + 4096 * (i >> 2)) & 65535)];
  for (int i = 0; i < 8; ++i) b[i] = src[(size_t)(4 + (i & 3)) * 65536 + ((tid + 4096 * (i >> 2)) & 65535)];
  floatx4 acc[8][8];
  for (int i = 0; i < 8; ++i)
    for (int j = 0; j < 8; ++j)
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    bf16x8 t = a[0];
    for (int i = 0; i < 7; ++i) a[i] = a[i + 1];
    a[7] = t;
  }
  float s = 0;
  for (int i = 0; i < 8; ++i)
    for (int j = 0; j < 8; ++j)
      for (int v = 0; v < 4; ++v) s += acc[i][j][v];
  out[tid] = s;
}

// the same copy with one contiguous piece per workgroup (16 KB per pass): fewer, longer streams
__global__ __launch_bounds__(256) void copy_chunk_kernel(const float4* __restrict__ in, float4* __restrict__ out, size_t n4) {
  const size_t per = n4 / gridDim.x;
  const float4* a = in + per * blockIdx.x;
  float4* b = out + per * blockIdx.x;
  for (size_t i = threadIdx.x; i + 768 < per; i += 1024) {
    const float4 v0 = a[i], v1 = a[i + 256], v2 = a[i + 512], v3 = a[i + 768];
    b[i] = v0;
    b[i + 256] = v1;
    b[i + 512] = v2;
    b[i + 768] = v3;
  }
}

__global__ void copy_kernel(const float4* __restrict__ in, float4* __restrict__ out, size_t n4) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n4; i += stride) out[i] = in[i];
}

static uint16_t f2b(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFF + ((u >> 16) & 1);
  return (uint16_t)(u >> 16);
}

template <class F>
static float sustained_ms(F launch, int warm, int iters) {
  for (int i = 0; i < warm; ++i) launch();
  hipEvent_t e0, e1;
  CHECK(hipEventCreate(&e0));
  CHECK(hipEventCreate(&e1));
  CHECK(hipEventRecord(e0));
  for (int i = 0; i < iters; ++i) launch();
  CHECK(hipEventRecord(e1));
  CHECK(hipEventSynchronize(e1));
  float ms;
  CHECK(hipEventElapsedTime(&ms, e0, e1));
  CHECK(hipGetLastError());
  return ms / iters;
}

template <bool A_KMAJOR, int DIAG>
static void time_dense(const char* what, const dense::DenseArgs& g, double flops) {
  auto kern = dense::dense_stream_kernel<A_KMAJOR, DIAG>;
  CHECK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, dense::LDS_BYTES));
  const float ms = sustained_ms([&] { hipLaunchKernelGGL(kern, dim3(256), dim3(256), dense::LDS_BYTES, 0, g); }, 60, 40);
  // the same variant with the cycle counters in (DIAG bit 3): main loop and output of each workgroup's second tile
  auto kclk = dense::dense_stream_kernel<A_KMAJOR, DIAG | 8>;
  CHECK(hipFuncSetAttribute((const void*)kclk, hipFuncAttributeMaxDynamicSharedMemorySize, dense::LDS_BYTES));
  for (int i = 0; i < 10; ++i) hipLaunchKernelGGL(kclk, dim3(256), dim3(256), dense::LDS_BYTES, 0, g);
  CHECK(hipDeviceSynchronize());
  static long long hc[4][1024];
  CHECK(hipMemcpyFromSymbol(hc, HIP_SYMBOL(dense::g_diag_cycles), sizeof(hc)));
  double loop = 0, outc = 0, ticks = 0;
  for (int i = 0; i < 1024; ++i) {
    loop += (double)hc[0][i];
    outc += (double)hc[1][i];
    ticks += (double)hc[2][i];
  }
  // workgroup w runs on XCD w % 8: mean life of a workgroup per XCD, fastest and slowest XCD
  double xmin = 1e30, xmax = 0;
  for (int x = 0; x < 8; ++x) {
    double d = 0;
    for (int w = x; w < 256; w += 8) d += (double)hc[3][w * 4];
    d /= 32 * 100.0;
    xmin = fmin(xmin, d);
    xmax = fmax(xmax, d);
  }
  printf("  %-58s %.3f ms  %7.1f TFLOP/s   %6.0f cycles per 32-deep stage (32 MFMAs = 1024), %5.0f per tile output, %.2f GHz, "
         "workgroups live %.0f-%.0f us by XCD\n", what, ms, flops / ms / 1e9, loop / 1024 / g.ktiles, outc / 1024, loop / ticks / 10.0, xmin, xmax);
}

int main() {
  std::mt19937 rng(3);
  std::normal_distribution<float> nd(0.f, 1.f);
  // ---- 1. matrix cores alone
  {
    const size_t n = 8 * 65536 * 8;
    std::vector<uint16_t> h(n);
    uint16_t* d;
    float* out;
    CHECK(hipMalloc(&d, n * 2));
    CHECK(hipMalloc(&out, 512 * 256 * 4));
    printf("1. v_mfma_f32_32x32x16_bf16 alone (16 independent accumulator tiles per wave)\n");
    for (int mode = 0; mode < 2; ++mode) {
      for (size_t i = 0; i < n; ++i) h[i] = f2b(mode == 0 ? 0.f : nd(rng) * (i < 4 * 65536 * 8 ? 0.02f : 1.f));
      CHECK(hipMemcpy(d, h.data(), n * 2, hipMemcpyHostToDevice));
      for (int wps = 1; wps <= 2; ++wps) {
        const int grid = 256 * wps, iters = 3000;
        const float ms = sustained_ms([&] { hipLaunchKernelGGL(mfma_loop_kernel, dim3(grid), dim3(256), 0, 0, (const bf16x8*)d, out, iters); }, 12, 8);
        printf("  %-40s %d wave(s) per SIMD: %7.1f TFLOP/s\n", mode == 0 ? "operands all zero" : "operands N(0, 0.02^2) x N(0, 1)", wps,
               (double)grid * 4 * iters * 16 * 32768.0 / ms / 1e9);
        const float ms16 = sustained_ms([&] { hipLaunchKernelGGL(mfma16_loop_kernel, dim3(grid), dim3(256), 0, 0, (const bf16x8*)d, out, iters / 2); }, 12, 8);
        printf("  %-40s %d wave(s) per SIMD: %7.1f TFLOP/s  (16x16x32 tiles)\n", "", wps, (double)grid * 4 * (iters / 2) * 64 * 16384.0 / ms16 / 1e9);
      }
    }
    CHECK(hipFree(d));
    CHECK(hipFree(out));
  }
  // ---- 2. copy
  {
    const size_t bytes = (size_t)1 << 30;
    float4 *a, *b;
    CHECK(hipMalloc(&a, bytes));
    CHECK(hipMalloc(&b, bytes));
    CHECK(hipMemset(a, 1, bytes));
    const float ms = sustained_ms([&] { hipLaunchKernelGGL(copy_kernel, dim3(256 * 16), dim3(256), 0, 0, a, b, bytes / 16); }, 20, 20);
    printf("2. device-to-device copy of 1 GiB: %.3f ms, %.0f GB/s read + write\n", ms, 2.0 * bytes / ms / 1e6);
    const float msc = sustained_ms([&] { hipLaunchKernelGGL(copy_chunk_kernel, dim3(2048), dim3(256), 0, 0, a, b, bytes / 16); }, 20, 20);
    printf("   the same with one contiguous 512 KB piece per workgroup: %.3f ms, %.0f GB/s\n", msc, 2.0 * bytes / msc / 1e6);
    CHECK(hipFree(a));
    CHECK(hipFree(b));
  }
  // ---- 3. the dense product and what feeds it
  {
    const int M = 4096, K = 4096;
    const long N = 16384;
    std::vector<uint16_t> hW((size_t)M * K), hA((size_t)K * N);
    for (auto& x : hW) x = f2b(0.02f * nd(rng));
    for (auto& x : hA) x = f2b(nd(rng));
    uint16_t *dW, *dA, *dC;
    CHECK(hipMalloc(&dW, hW.size() * 2));
    CHECK(hipMalloc(&dA, hA.size() * 2));
    CHECK(hipMalloc(&dC, (size_t)M * N * 2));
    CHECK(hipMemcpy(dW, hW.data(), hW.size() * 2, hipMemcpyHostToDevice));
    CHECK(hipMemcpy(dA, hA.data(), hA.size() * 2, hipMemcpyHostToDevice));
    dense::DenseArgs g{};
    g.A = dW; g.B = dA; g.C = dC; g.lda = K; g.ldb = N; g.ldc = N;
    g.tiles_m = M / 256; g.tiles_n = (int)(N / 256); g.ktiles = K / 32;
    const double flops = 2.0 * M * K * N;
    printf("3. dense product %d x %d x %ld, W ~ N(0, 0.02^2), activations ~ N(0, 1), sustained\n", M, K, N);
    time_dense<true, 0>("forward B = W A (weight rows contiguous)", g, flops);
    time_dense<false, 0>("backward dA = W^T dB (both operands strided)", g, flops);
    time_dense<false, 1>("backward, no direct-to-LDS loads in the loop", g, flops);
    time_dense<false, 2>("backward, no fragment reads in the loop", g, flops);
    time_dense<false, 3>("backward, neither (MFMAs, barrier, epilogue only)", g, flops);
    time_dense<false, 4>("backward, every load re-fetches the first stage (cache hits)", g, flops);
    time_dense<false, 6>("backward, cache-hit loads and no fragment reads", g, flops);
    // spot check of the unmodified kernel (forward)
    auto kern = dense::dense_stream_kernel<true, 0>;
    hipLaunchKernelGGL(kern, dim3(256), dim3(256), dense::LDS_BYTES, 0, g);
    std::vector<uint16_t> hC((size_t)M * N);
    CHECK(hipMemcpy(hC.data(), dC, hC.size() * 2, hipMemcpyDeviceToHost));
    double maxerr = 0, maxref = 0;
    for (int s = 0; s < 64; ++s) {
      const int i = rng() % M;
      const long j = rng() % N;
      double r = 0;
      for (int k = 0; k < K; ++k) r += (double)bf16_bits_to_float(hW[(size_t)i * K + k]) * bf16_bits_to_float(hA[(size_t)k * N + j]);
      maxerr = fmax(maxerr, fabs(r - bf16_bits_to_float(hC[(size_t)i * N + j])));
      maxref = fmax(maxref, fabs(r));
    }
    printf("  spot check of the forward product: max |err| %.4g on max |ref| %.4g\n", maxerr, maxref);
    // the same kernels on zero operands: the same cycles at the clock the power limit then allows
    CHECK(hipMemset(dW, 0, hW.size() * 2));
    CHECK(hipMemset(dA, 0, hA.size() * 2));
    time_dense<true, 0>("forward, all operands zero", g, flops);
    time_dense<false, 0>("backward, all operands zero", g, flops);
  }
  return 0;
}
