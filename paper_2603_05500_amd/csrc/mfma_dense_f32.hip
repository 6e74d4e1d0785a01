// Dense products of the POET-X linear layer for fp32 tensors on the matrix cores
// (v_mfma_f32_32x32x2_f32: fp32 operands, fp32 accumulation -- no reduced-precision step):
//   forward  (Eq. 10, mm2):       B  (n x N) = W   (n x m) * A  (m x N)
//   backward (Sec. 3.5, mm2 bwd): dA (m x N) = W^T (m x n) * dB (n x N)
// Same layouts as the bf16 kernel: W row major n x m, activations feature major.  The fp32 path
// is the accuracy path (1e-4 tolerance), not the fast one: a plain 128 x 128 x 16 tiling, 4 waves of
// 64 x 64, register-staged global loads one tile ahead, two LDS stages, one barrier per tile.
// Both operands sit in LDS as [k][x] rows (x contiguous), which is the order the MFMA wants its
// lanes in (lane = x + 32 * (k & 1)), so fragment reads are conflict-free 4-byte reads.
#include "poetx_kernels.h"

namespace poetx {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BN = 128, BK = 16, PADX = 4;   // rows of 128 + 4 floats: the transposed store of W spreads over banks
constexpr int LDX = BM + PADX;

struct Args {
  const float* W;     // n x m row major
  const float* act;   // K x N row major
  float* out;         // M x N row major
  int n, m;
  i64 N;
  int K;
};

template <bool TRANS_W>
__global__ __launch_bounds__(256) void dense_f32_kernel(Args g) {
  __shared__ float As[2][BK][LDX];
  __shared__ float Bs[2][BK][LDX];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
  const i64 i0 = (i64)blockIdx.y * BM, j0 = (i64)blockIdx.x * BN;
  const int lda = g.m;   // row stride of W
  // ---- global -> registers.  A tile: 128 x 16.  Forward: W rows are contiguous along k: 4 lanes per
  // row, a float4 (4 k) each, two passes of 64 rows.  Backward: W^T, contiguous along the output row
  // index: 32 lanes per k row, two passes of 8 k rows.  B tile: 16 x 128, 32 lanes per k row.
  floatx4 ra[2], rb[2];
  auto gload = [&](int kt) {
    const i64 k0 = (i64)kt * BK;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      if (!TRANS_W) {
        const int r = p * 64 + (tid >> 2), kq = tid & 3;
        ra[p] = *reinterpret_cast<const floatx4*>(g.W + (i0 + r) * lda + k0 + 4 * kq);
      } else {
        const int k = p * 8 + (tid >> 5), c = tid & 31;
        ra[p] = *reinterpret_cast<const floatx4*>(g.W + (k0 + k) * lda + i0 + 4 * c);
      }
      const int k = p * 8 + (tid >> 5), c = tid & 31;
      rb[p] = *reinterpret_cast<const floatx4*>(g.act + (k0 + k) * g.N + j0 + 4 * c);
    }
  };
  auto lstore = [&](int s) {
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      if (!TRANS_W) {
        const int r = p * 64 + (tid >> 2), kq = tid & 3;
#pragma unroll
        for (int e = 0; e < 4; ++e) As[s][4 * kq + e][r] = ra[p][e];
      } else {
        const int k = p * 8 + (tid >> 5), c = tid & 31;
        *reinterpret_cast<floatx4*>(&As[s][k][4 * c]) = ra[p];
      }
      const int k = p * 8 + (tid >> 5), c = tid & 31;
      *reinterpret_cast<floatx4*>(&Bs[s][k][4 * c]) = rb[p];
    }
  };
  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][c][v] = 0.f;
  const int KT = g.K / BK;
  gload(0);
  lstore(0);
  __syncthreads();
  const int x = lane & 31, kh = lane >> 5;
  for (int kt = 0; kt < KT; ++kt) {
    const int s = kt & 1;
    if (kt + 1 < KT) gload(kt + 1);
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      float fa[2], fb[2];
#pragma unroll
      for (int a = 0; a < 2; ++a) fa[a] = As[s][kk + kh][wm * 64 + a * 32 + x];
#pragma unroll
      for (int c = 0; c < 2; ++c) fb[c] = Bs[s][kk + kh][wn * 64 + c * 32 + x];
      // operands swapped: the accumulator tile is transposed, a lane owns one output row and groups of
      // four consecutive columns
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c) acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x2f32(fb[c], fa[a], acc[a][c], 0, 0, 0);
    }
    if (kt + 1 < KT) lstore(s ^ 1);   // the other stage: nobody reads it before the barrier below
    __syncthreads();
  }
  // lane (x, kh) of accumulator tile (a, c): row wm*64 + a*32 + x, columns wn*64 + c*32 + 8 q + 4 kh + 0..3
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const floatx4 o = {acc[a][c][4 * q], acc[a][c][4 * q + 1], acc[a][c][4 * q + 2], acc[a][c][4 * q + 3]};
        *reinterpret_cast<floatx4*>(g.out + (i0 + wm * 64 + a * 32 + x) * g.N + j0 + wn * 64 + c * 32 + 8 * q + 4 * kh) = o;
      }
}

}  // namespace

bool mfma_dense_f32_supported(int n, int m, i64 N) { return n % BM == 0 && m % BM == 0 && N % BN == 0; }

void mfma_dense_f32(int trans_w, const void* W, int n, int m, const void* act, void* out, i64 N, hipStream_t st) {
  Args g{(const float*)W, (const float*)act, (float*)out, n, m, N, trans_w ? n : m};
  const int M = trans_w ? m : n;
  const dim3 grid((unsigned)(N / BN), (unsigned)(M / BM));
  if (trans_w) hipLaunchKernelGGL(dense_f32_kernel<true>, grid, dim3(256), 0, st, g);
  else hipLaunchKernelGGL(dense_f32_kernel<false>, grid, dim3(256), 0, st, g);
}

}  // namespace poetx
