// Block gradients on the matrix cores (Sec. 3.5, mm1/mm3 backward):
//   dG_j = U'_j V'_j^T,  U'_j / V'_j = rows j*b .. j*b+b-1 of U / V gathered by the
//   side's permutation, contraction over the N tokens.
// Both operands are contracted over their contiguous (token) index.  The output
// is only nb blocks of b x b, so the token range is split over `splits`
// workgroups per tile; each writes an fp32 partial tile and a second kernel
// adds the partials in a fixed order (deterministic, no atomics).
#include "mfma_gemm.h"

namespace poetx {
namespace {

constexpr int GBM = 256, GBN = 256, GBK = 64;

struct EpiPartial {
  float* out;
  int b;
  i64 split_stride;
  __device__ void operator()(int batch, int split, int row, int col, float4 v) const {
    *reinterpret_cast<float4*>(out + split * split_stride + ((i64)batch * b + row) * b + col) = v;
  }
  __device__ void wide(int batch, int split, int row, int col, float4 lo, float4 hi) const {   // whole 32-byte sectors
    float* p = out + split * split_stride + ((i64)batch * b + row) * b + col;
    *reinterpret_cast<float4*>(p) = lo;
    *reinterpret_cast<float4*>(p + 4) = hi;
  }
};

__global__ void reduce_partials_kernel(const float4* __restrict__ part, float4* __restrict__ out, i64 n4, int splits) {
  i64 idx = (i64)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n4) return;
  float4 s = part[idx];
  for (int z = 1; z < splits; ++z) {
    float4 p = part[(i64)z * n4 + idx];
    s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
  }
  out[idx] = s;
}

int pick_splits(int d, i64 N, int b) {
  const int tiles = (d / b) * (b / GBM) * (b / GBN);
  const int ktiles = (int)(N / GBK);
  int s = 1;
  while (s * 2 * tiles <= 256 && s * 2 <= 64 && ktiles % (s * 2) == 0 && ktiles / (s * 2) >= 4) s *= 2;
  return s;
}

}  // namespace

bool mfma_blockgrad_supported(int d, i64 N, int b) {
  return (b == 256 || b == 512) && d % b == 0 && N % GBK == 0 && N >= 4 * GBK && N < (1ll << 31);
}

size_t mfma_blockgrad_workspace_bytes(int d, i64 N, int b) {
  return (size_t)pick_splits(d, N, b) * d * b * sizeof(float);
}

void mfma_blockgrad(const void* U, const void* V, int d, i64 N, const int32_t* perm, int b, float* dG, void* ws,
                    hipStream_t st) {
  const int nb = d / b;
  const int splits = pick_splits(d, N, b);
  mm::Args g{};
  g.nsrc = 1;
  g.s[0].A = (const uint16_t*)U;
  g.s[0].B = (const uint16_t*)V;
  g.s[0].lda = N;
  g.s[0].ldb = N;
  g.s[0].ktiles = (int)(N / GBK) / splits;
  g.tiles_m = b / GBM;
  g.tiles_n = b / GBN;
  g.perm = perm;
  g.rows_per_batch = b;
  const i64 total = (i64)nb * b * b;
  float* part = splits > 1 ? (float*)ws : dG;
  // a split contracts as few as 8 stages: no redundant tail loads
  mm::launch<GBM, GBN, 2, 4, true, true, true, 4, true>(g, EpiPartial{part, b, total}, nb, splits, st);
  if (splits > 1)
    hipLaunchKernelGGL(reduce_partials_kernel, dim3(ceil_div(total / 4, 256)), dim3(256), 0, st, (const float4*)part,
                       (float4*)dG, total / 4, splits);
}

}  // namespace poetx
