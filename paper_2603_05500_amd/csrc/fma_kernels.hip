// Plain fp32-FMA kernels for every step of the POET-X linear hot path.
//
// This is the path used for fp32 tensors (where the 1e-4 tolerance rules out
// bf16 matrix-core products) and for shapes the matrix-core kernels do not
// cover.  Every step is one instance of a small LDS-tiled batched product
//     C[batch](i, j) = sum_k A[batch](i, k) * B[batch](k, j)
// whose operands are described by accessor structs, so gather-by-permutation,
// scatter-by-permutation and on-the-fly skew construction are fused into the loads
// and stores.  The projection of the series gradient onto the packed parameters is a
// separate element-wise kernel (skew_project_kernel), shared with the matrix-core path.
#include "poetx_kernels.h"

namespace poetx {
namespace {

constexpr int BM = 64, BN = 64, BK = 16, NT = 256;

// FA: float operator()(int batch, int i, int k), static bool k_fast (k contiguous in memory)
// FB: float operator()(int batch, int k, int j), static bool k_fast
// FC: void  operator()(int batch, int i, int j, float acc)
template <class FA, class FB, class FC>
__global__ __launch_bounds__(NT) void gemm_fma_kernel(int M, int N, int K, FA fa, FB fb, FC fc) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int tid = threadIdx.x;
  const int batch = blockIdx.z;
  const int i0 = blockIdx.y * BM;
  const int j0 = blockIdx.x * BN;
  const int tx = tid % 16, ty = tid / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int s = 0; s < (BM * BK) / NT; ++s) {
      int idx = tid + s * NT;
      int kk, ii;
      if (FA::k_fast) { kk = idx % BK; ii = idx / BK; } else { ii = idx % BM; kk = idx / BM; }
      float v = 0.f;
      if (i0 + ii < M && k0 + kk < K) v = fa(batch, i0 + ii, k0 + kk);
      As[kk][ii] = v;
    }
#pragma unroll
    for (int s = 0; s < (BN * BK) / NT; ++s) {
      int idx = tid + s * NT;
      int kk, jj;
      if (FB::k_fast) { kk = idx % BK; jj = idx / BK; } else { jj = idx % BN; kk = idx / BN; }
      float v = 0.f;
      if (j0 + jj < N && k0 + kk < K) v = fb(batch, k0 + kk, j0 + jj);
      Bs[kk][jj] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) a[r] = As[kk][ty * 4 + r];
#pragma unroll
      for (int c = 0; c < 4; ++c) b[c] = Bs[kk][tx * 4 + c];
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(a[r], b[c], acc[r][c]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      int i = i0 + ty * 4 + r, j = j0 + tx * 4 + c;
      if (i < M && j < N) fc(batch, i, j, acc[r][c]);
    }
}

template <class FA, class FB, class FC>
void launch_gemm(int batch, i64 M, i64 N, i64 K, FA fa, FB fb, FC fc, hipStream_t st) {
  if (batch <= 0 || M <= 0 || N <= 0) return;
  dim3 grid(ceil_div(N, BN), ceil_div(M, BM), batch);
  hipLaunchKernelGGL((gemm_fma_kernel<FA, FB, FC>), grid, dim3(NT), 0, st, (int)M, (int)N, (int)K, fa, fb, fc);
}

// ---------------------------------------------------------------- accessors
template <class T>
struct RowMajorA {  // A(i,k) = p[batch*bs + i*ld + k]
  const T* p; i64 ld; i64 bs;
  static constexpr bool k_fast = true;
  __device__ float operator()(int bt, int i, int k) const { return to_float(p[bt * bs + (i64)i * ld + k]); }
};
template <class T>
struct ColMajorA {  // A(i,k) = p[batch*bs + k*ld + i]
  const T* p; i64 ld; i64 bs;
  static constexpr bool k_fast = false;
  __device__ float operator()(int bt, int i, int k) const { return to_float(p[bt * bs + (i64)k * ld + i]); }
};
template <class T>
struct RowMajorB {  // B(k,j) = p[batch*bs + k*ld + j]
  const T* p; i64 ld; i64 bs;
  static constexpr bool k_fast = false;
  __device__ float operator()(int bt, int k, int j) const { return to_float(p[bt * bs + (i64)k * ld + j]); }
};
template <class T>
struct StoreRowMajor {
  T* p; i64 ld;
  __device__ void operator()(int, int i, int j, float v) const { p[(i64)i * ld + j] = from_float<T>(v); }
};

// op(G_j)(i,l) for the structured apply.  RES = false: float G[nb][b][b].  RES = true: bf16
// pairs [nb][2][b][b] holding G - I and its transpose; the identity is added back here.
template <class T, bool TRANS, bool RES>
struct BlockOpA {
  const T* blocks; int b; int d;
  static constexpr bool k_fast = RES || !TRANS;
  __device__ float operator()(int j, int i, int l) const {
    int s = block_side(d, b, j);
    if (i >= s || l >= s) return 0.f;
    const i64 bb = (i64)b * b;
    if (RES) {
      float g = to_float(blocks[(i64)j * 2 * bb + (TRANS ? bb : 0) + (i64)i * b + l]);
      return i == l ? g + 1.f : g;
    }
    return to_float(TRANS ? blocks[j * bb + (i64)l * b + i] : blocks[j * bb + (i64)i * b + l]);
  }
};
// op(G_j)(l,i) as the right-hand operand (apply_right).
template <class T, bool TRANS, bool RES>
struct BlockOpB {
  const T* blocks; int b; int d;
  static constexpr bool k_fast = !RES && TRANS;
  __device__ float operator()(int j, int l, int i) const {
    int s = block_side(d, b, j);
    if (i >= s || l >= s) return 0.f;
    const i64 bb = (i64)b * b;
    if (RES) {
      float g = to_float(blocks[(i64)j * 2 * bb + (TRANS ? bb : 0) + (i64)l * b + i]);
      return i == l ? g + 1.f : g;
    }
    return to_float(TRANS ? blocks[j * bb + (i64)i * b + l] : blocks[j * bb + (i64)l * b + i]);
  }
};
template <class T>
struct GatherRowsB {  // B(l, c) = V[perm[j*b + l]][c]
  const T* V; i64 ld; const int32_t* perm; int b; int d;
  static constexpr bool k_fast = false;
  __device__ float operator()(int j, int l, int c) const {
    int row = j * b + l;
    if (row >= d) return 0.f;
    return to_float(V[(i64)perm[row] * ld + c]);
  }
};
template <class T>
struct ScatterRowsC {  // out[perm[j*b + i]][c] = acc
  T* out; i64 ld; const int32_t* perm; int b; int d;
  __device__ void operator()(int j, int i, int c, float v) const {
    int row = j * b + i;
    if (row < d) out[(i64)perm[row] * ld + c] = from_float<T>(v);
  }
};
template <class T>
struct GatherColsA {  // A(r, l) = V[r][perm[j*b + l]]
  const T* V; i64 ld; const int32_t* perm; int b; int d;
  static constexpr bool k_fast = true;
  __device__ float operator()(int j, int r, int l) const {
    int col = j * b + l;
    if (col >= d) return 0.f;
    return to_float(V[(i64)r * ld + perm[col]]);
  }
};
template <class T>
struct ScatterColsC {
  T* out; i64 ld; const int32_t* perm; int b; int d;
  __device__ void operator()(int j, int r, int i, float v) const {
    int col = j * b + i;
    if (col < d) out[(i64)r * ld + perm[col]] = from_float<T>(v);
  }
};
// token-contraction operands of the block gradient
template <class T>
struct GatherRowsTokA {  // A(i, t) = U[perm[j*b+i]][t]
  const T* U; i64 ld; const int32_t* perm; int b; int d;
  static constexpr bool k_fast = true;
  __device__ float operator()(int j, int i, int t) const {
    int row = j * b + i;
    if (row >= d) return 0.f;
    return to_float(U[(i64)perm[row] * ld + t]);
  }
};
template <class T>
struct GatherRowsTokB {  // B(t, c) = V[perm[j*b+c]][t]
  const T* V; i64 ld; const int32_t* perm; int b; int d;
  static constexpr bool k_fast = true;
  __device__ float operator()(int j, int t, int c) const {
    int row = j * b + c;
    if (row >= d) return 0.f;
    return to_float(V[(i64)perm[row] * ld + t]);
  }
};
struct StoreBlock {  // C[j][i][c]
  float* p; int b;
  __device__ void operator()(int j, int i, int c, float v) const { p[((i64)j * b + i) * b + c] = v; }
};

// sign * skew(theta_j)(r, c), tail rows/columns masked (Sec. 3.4).
struct SkewB {
  const float* theta; int b; int d; float sign;
  static constexpr bool k_fast = false;
  __device__ float operator()(int j, int r, int c) const {
    int s = block_side(d, b, j);
    if (r >= s || c >= s || r == c) return 0.f;
    const float* th = theta + (i64)j * ((i64)b * (b - 1) / 2);
    return r < c ? sign * th[packed_index(r, c, b)] : -sign * th[packed_index(c, r, b)];
  }
};
// C = acc + cdiag * I; optionally also the bf16 residual (acc itself).
struct StoreHorner {
  float* out; uint16_t* e; int b; float cdiag; float ediag;
  __device__ void operator()(int j, int i, int c, float v) const {
    i64 o = ((i64)j * b + i) * b + c;
    if (out) out[o] = (i == c) ? v + cdiag : v;
    if (e) {  // bf16 pair: value, then its transpose
      const i64 bb = (i64)b * b;
      const uint16_t r = float_to_bf16_bits((i == c) ? v + ediag : v);
      e[(i64)j * 2 * bb + (i64)i * b + c] = r;
      e[(i64)j * 2 * bb + bb + (i64)c * b + i] = r;
    }
  }
};
// [A | Bm](i, kk) and [D ; T](kk, c) for the backward recursion step Bm <- A D + Bm T.
struct CatA {
  const float* A; const float* Bm; int b;
  static constexpr bool k_fast = true;
  __device__ float operator()(int j, int i, int kk) const {
    i64 base = ((i64)j * b + i) * b;
    return kk < b ? A[base + kk] : Bm[base + kk - b];
  }
};
struct CatB {
  const float* D; SkewB T; int b;
  static constexpr bool k_fast = false;
  __device__ float operator()(int j, int kk, int c) const {
    return kk < b ? D[((i64)j * b + kk) * b + c] : T(j, kk - b, c);
  }
};

// H = sign*Q + cdiag*I (first Horner coefficient pair), elementwise.
__global__ void skew_affine_kernel(SkewB q, float cdiag, float* out, i64 total) {
  i64 idx = (i64)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  int b = q.b;
  int c = (int)(idx % b);
  int r = (int)((idx / b) % b);
  int j = (int)(idx / ((i64)b * b));
  out[idx] = q(j, r, c) + (r == c ? cdiag : 0.f);
}

// dtheta[j][idx(i,c)] (+)= M[j][i][c] - M[j][c][i], i < c < tail side; dead slots get 0.
__global__ void skew_project_kernel(const float* M, int b, int d, int nb, float* dtheta, int accumulate) {
  i64 L = (i64)b * (b - 1) / 2;
  i64 idx = (i64)blockIdx.x * blockDim.x + threadIdx.x;
  i64 total = (i64)nb * b * b;
  if (idx >= total) return;
  int c = (int)(idx % b);
  int i = (int)((idx / b) % b);
  int j = (int)(idx / ((i64)b * b));
  if (i >= c) return;
  int s = block_side(d, b, j);
  float v = 0.f;
  if (c < s) v = M[((i64)j * b + i) * b + c] - M[((i64)j * b + c) * b + i];
  float* dst = dtheta + j * L + packed_index(i, c, b);
  *dst = accumulate ? *dst + v : v;
}

__global__ void zero_i32_kernel(int32_t* p, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

__global__ void perm_mark_kernel(const int32_t* perm, int d, int32_t* scratch) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= d) return;
  int p = perm[i];
  if (p < 0 || p >= d) { atomicAdd(&scratch[d], 1); return; }
  if (atomicAdd(&scratch[p], 1) != 0) atomicAdd(&scratch[d], 1);
}

template <class T, bool RES>
void apply_left_t(const T* V, T* out, int d, i64 cols, i64 ld, const int32_t* perm, const T* blocks, int b,
                  int trans, hipStream_t st) {
  int nb = ceil_div(d, b);
  GatherRowsB<T> fb{V, ld, perm, b, d};
  ScatterRowsC<T> fc{out, ld, perm, b, d};
  if (trans) launch_gemm(nb, b, cols, b, BlockOpA<T, true, RES>{blocks, b, d}, fb, fc, st);
  else launch_gemm(nb, b, cols, b, BlockOpA<T, false, RES>{blocks, b, d}, fb, fc, st);
}
template <class T, bool RES>
void apply_right_t(const T* V, T* out, i64 rows, int d, i64 ld, const int32_t* perm, const T* blocks, int b,
                   int trans, hipStream_t st) {
  int nb = ceil_div(d, b);
  GatherColsA<T> fa{V, ld, perm, b, d};
  ScatterColsC<T> fc{out, ld, perm, b, d};
  if (trans) launch_gemm(nb, rows, b, b, fa, BlockOpB<T, true, RES>{blocks, b, d}, fc, st);
  else launch_gemm(nb, rows, b, b, fa, BlockOpB<T, false, RES>{blocks, b, d}, fc, st);
}
template <class T>
void dense_t(int trans_w, const T* W, int n, int m, const T* act, T* out, i64 N, hipStream_t st) {
  RowMajorB<T> fb{act, N, 0};
  StoreRowMajor<T> fc{out, N};
  if (!trans_w) launch_gemm(1, n, N, m, RowMajorA<T>{W, m, 0}, fb, fc, st);
  else launch_gemm(1, m, N, n, ColMajorA<T>{W, m, 0}, fb, fc, st);
}

}  // namespace

void fma_dense(int dtype, int trans_w, const void* W, int n, int m, const void* act, void* out, i64 N,
               hipStream_t st) {
  if (dtype == POETX_F32) dense_t<float>(trans_w, (const float*)W, n, m, (const float*)act, (float*)out, N, st);
  else dense_t<bf16_t>(trans_w, (const bf16_t*)W, n, m, (const bf16_t*)act, (bf16_t*)out, N, st);
}

void fma_apply_left(int dtype, const void* V, void* out, int d, i64 cols, i64 ld, const int32_t* perm,
                    const void* blocks, int b, int transpose_G, hipStream_t st) {
  if (dtype == POETX_F32)
    apply_left_t<float, false>((const float*)V, (float*)out, d, cols, ld, perm, (const float*)blocks, b, transpose_G, st);
  else
    apply_left_t<bf16_t, true>((const bf16_t*)V, (bf16_t*)out, d, cols, ld, perm, (const bf16_t*)blocks, b, transpose_G, st);
}

void fma_apply_right(int dtype, const void* V, void* out, i64 rows, int d, i64 ld, const int32_t* perm,
                     const void* blocks, int b, int transpose_G, hipStream_t st) {
  if (dtype == POETX_F32)
    apply_right_t<float, false>((const float*)V, (float*)out, rows, d, ld, perm, (const float*)blocks, b, transpose_G, st);
  else
    apply_right_t<bf16_t, true>((const bf16_t*)V, (bf16_t*)out, rows, d, ld, perm, (const bf16_t*)blocks, b, transpose_G, st);
}

void fma_blockgrad(int dtype, const void* U, const void* V, int d, i64 N, const int32_t* perm, int b, float* dG,
                   hipStream_t st) {
  int nb = ceil_div(d, b);
  StoreBlock fc{dG, b};
  if (dtype == POETX_F32)
    launch_gemm(nb, b, b, N, GatherRowsTokA<float>{(const float*)U, N, perm, b, d},
                GatherRowsTokB<float>{(const float*)V, N, perm, b, d}, fc, st);
  else
    launch_gemm(nb, b, b, N, GatherRowsTokA<bf16_t>{(const bf16_t*)U, N, perm, b, d},
                GatherRowsTokB<bf16_t>{(const bf16_t*)V, N, perm, b, d}, fc, st);
}

// G = I + 2 sum_{p<=k} Q^p + Q^{k+1} by Horner's rule in Q (Eq. 8 for general k):
// H <- Q + 2I, then k times H <- H Q + c I with c = 2 except c = 1 at the end.
// The last product alone is G - I, which is what the bf16 residual stores.
void fma_cnp_build(const float* theta, int d, int b, int k, float* G_f32, void* E_bf16, float* ws,
                   hipStream_t st) {
  int nb = ceil_div(d, b);
  i64 total = (i64)nb * b * b;
  float* buf[2] = {ws, ws + total};
  SkewB q{theta, b, d, 1.f};
  int cur = 0;
  hipLaunchKernelGGL(skew_affine_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, q, 2.f, buf[cur], total);
  for (int step = 0; step < k; ++step) {
    bool last = step == k - 1;
    RowMajorA<float> fa{buf[cur], b, (i64)b * b};
    if (last) {
      launch_gemm(nb, b, b, b, fa, q, StoreHorner{G_f32, (uint16_t*)E_bf16, b, 1.f, 0.f}, st);
    } else {
      launch_gemm(nb, b, b, b, fa, q, StoreHorner{buf[1 - cur], nullptr, b, 2.f, 0.f}, st);
      cur = 1 - cur;
    }
  }
}

// Chain rule through the series for any k.  With T = Q^T = -Q and D = dL/dG, the
// gradient sum_p c_p sum_{i+j=p-1} T^i D T^j is the upper-right block of the matrix
// polynomial evaluated at [[T, D], [0, T]]; Horner's rule on that block matrix gives
//   A <- c_{k+1} T + c_k I,  Bm <- c_{k+1} D,  then for p = k-1 .. 0:
//   Bm <- A D + Bm T,  A <- A T + c_p I.
// At k = 3 the result equals the paper's 2 grad_1 + 2 grad_2 + 2 grad_3 + grad_4.
// The projection onto the packed parameters is dtheta[i,j] = Bm[i,j] - Bm[j,i].
void fma_cnp_bwd(const float* theta, const float* dG, int d, int b, int k, float* dtheta, int accumulate,
                 float* ws, hipStream_t st) {
  int nb = ceil_div(d, b);
  i64 total = (i64)nb * b * b;
  float* A[2] = {ws, ws + total};
  float* Bm[2] = {ws + 2 * total, ws + 3 * total};
  SkewB t{theta, b, d, -1.f};
  hipLaunchKernelGGL(skew_affine_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, t, 2.f, A[0], total);
  const float* bcur = dG;  // c_{k+1} = 1
  int ca = 0, cb = 0;
  for (int p = k - 1; p >= 0; --p) {
    if (bcur == dG) {
      // Bm = D: the concatenated product needs Bm T with Bm = D
      launch_gemm(nb, b, b, 2 * b, CatA{A[ca], dG, b}, CatB{dG, t, b}, StoreBlock{Bm[cb], b}, st);
    } else {
      launch_gemm(nb, b, b, 2 * b, CatA{A[ca], bcur, b}, CatB{dG, t, b}, StoreBlock{Bm[1 - cb], b}, st);
      cb = 1 - cb;
    }
    bcur = Bm[cb];
    if (p > 0) {
      launch_gemm(nb, b, b, b, RowMajorA<float>{A[ca], b, (i64)b * b}, t,
                  StoreHorner{A[1 - ca], nullptr, b, 2.f, 0.f}, st);
      ca = 1 - ca;
    }
  }
  skew_project_launch(bcur, b, d, dtheta, accumulate, st);
}

void skew_project_launch(const float* M, int b, int d, float* dtheta, int accumulate, hipStream_t st) {
  const int nb = ceil_div(d, b);
  if (skew_tiled_supported(b, d)) {
    skew_project_tiled_launch(M, b, nb, dtheta, accumulate, st);
    return;
  }
  const i64 total = (i64)nb * b * b;
  hipLaunchKernelGGL(skew_project_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, M, b, d, nb, dtheta,
                     accumulate);
}

void perm_validate_launch(const int32_t* perm, int d, int32_t* scratch, hipStream_t st) {
  hipLaunchKernelGGL(zero_i32_kernel, dim3(ceil_div(d + 1, 256)), dim3(256), 0, st, scratch, d + 1);
  hipLaunchKernelGGL(perm_mark_kernel, dim3(ceil_div(d, 256)), dim3(256), 0, st, perm, d, scratch);
}

}  // namespace poetx
