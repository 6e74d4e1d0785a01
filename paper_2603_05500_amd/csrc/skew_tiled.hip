// Q = skew(theta) and its adjoint on the packed parameters (Sec. 3.4), tile by tile.
//   materialise: Q[i][c] = +theta[idx(i, c)] for i < c, -theta[idx(c, i)] for i > c, 0 on the diagonal
//   project:     dtheta[idx(i, c)] (+)= M[i][c] - M[c][i] for i < c
// idx is the row-major strict upper triangle, so a row segment of the upper triangle is contiguous in
// theta while its mirror image is a column.  A workgroup takes a 64 x 64 tile (I, J), I <= J, together
// with its mirror tile (J, I) and passes the transposed half through LDS: every global access of both
// kernels runs along contiguous addresses.  For blocks whose side is a multiple of 64 and dimensions
// that are whole blocks (the matrix-core paths); other shapes keep the element-wise kernels.
#include "poetx_kernels.h"

namespace poetx {
namespace {

constexpr int ST = 64;

// tile pair p of the upper triangle (diagonal included) of a T x T tile grid, row by row
__device__ inline void pair_decode(int p, int T, int& I, int& J) {
  I = 0;
  while (p >= T - I) {
    p -= T - I;
    ++I;
  }
  J = I + p;
}

__global__ __launch_bounds__(256) void skew_materialize_tiled_kernel(const float* __restrict__ theta, int b, float* __restrict__ Qf,
                                                                     uint16_t* __restrict__ Qb, uint16_t* __restrict__ Tb) {
  __shared__ float tile[ST][ST + 1];
  int I, J;
  pair_decode(blockIdx.x, b / ST, I, J);
  const i64 j = blockIdx.y;
  const float* th = theta + j * ((i64)b * (b - 1) / 2);
  const int c = threadIdx.x & 63, r0 = threadIdx.x >> 6;
#pragma unroll 4
  for (int r = r0; r < ST; r += 4) {
    const int i = I * ST + r, col = J * ST + c;
    tile[r][c] = i < col ? th[packed_index(i, col, b)] : 0.f;
  }
  __syncthreads();
  auto put = [&](i64 at, float q) {
    if (Qf) Qf[at] = q;
    if (Qb) Qb[at] = float_to_bf16_bits(q);
    if (Tb) Tb[at] = float_to_bf16_bits(-q);
  };
#pragma unroll 4
  for (int r = r0; r < ST; r += 4) {
    float q = tile[r][c];                               // strictly above the diagonal where I < J
    if (I == J) q = c > r ? tile[r][c] : (c < r ? -tile[c][r] : 0.f);
    put((j * b + I * ST + r) * b + J * ST + c, q);
    if (I != J) put((j * b + J * ST + r) * b + I * ST + c, -tile[c][r]);   // Q[J*64 + r][I*64 + c] = -Q[I*64 + c][J*64 + r]
  }
}

__global__ __launch_bounds__(256) void skew_project_tiled_kernel(const float* __restrict__ M, int b, float* __restrict__ dtheta,
                                                                 int accumulate) {
  __shared__ float up[ST][ST + 1], lo[ST][ST + 1];
  int I, J;
  pair_decode(blockIdx.x, b / ST, I, J);
  const i64 j = blockIdx.y;
  const float* Mj = M + j * (i64)b * b;
  float* dt = dtheta + j * ((i64)b * (b - 1) / 2);
  const int c = threadIdx.x & 63, r0 = threadIdx.x >> 6;
#pragma unroll 4
  for (int r = r0; r < ST; r += 4) {
    up[r][c] = Mj[(i64)(I * ST + r) * b + J * ST + c];
    lo[r][c] = Mj[(i64)(J * ST + r) * b + I * ST + c];
  }
  __syncthreads();
#pragma unroll 4
  for (int r = r0; r < ST; r += 4) {
    const int i = I * ST + r, col = J * ST + c;
    if (i < col) {
      const float v = up[r][c] - lo[c][r];   // M[i][col] - M[col][i]
      float* dst = dt + packed_index(i, col, b);
      *dst = accumulate ? *dst + v : v;
    }
  }
}

}  // namespace

bool skew_tiled_supported(int b, i64 d) { return b % ST == 0 && d % b == 0; }

void skew_materialize_tiled_launch(const float* theta, int b, i64 nb, float* Qf, uint16_t* Qb, uint16_t* Tb, hipStream_t st) {
  const int T = b / ST;
  hipLaunchKernelGGL(skew_materialize_tiled_kernel, dim3(T * (T + 1) / 2, (unsigned)nb), dim3(256), 0, st, theta, b, Qf, Qb, Tb);
}

void skew_project_tiled_launch(const float* M, int b, i64 nb, float* dtheta, int accumulate, hipStream_t st) {
  const int T = b / ST;
  hipLaunchKernelGGL(skew_project_tiled_kernel, dim3(T * (T + 1) / 2, (unsigned)nb), dim3(256), 0, st, M, b, dtheta, accumulate);
}

}  // namespace poetx
