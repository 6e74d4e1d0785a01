// Dense bf16 products of the POET-X linear layer on the gfx950 matrix cores:
//   forward  (Eq. 10, mm2):      B  (n x N) = W   (n x m) * A  (m x N)
//   backward (Sec. 3.5, mm2 bwd): dA (m x N) = W^T (m x n) * dB (n x N)
// W is row major n x m, activations are feature major (token index contiguous).
//
// The contraction runs over the feature index, which is the strided one for the
// activations (and for W in the backward product).  The tiles are therefore
// staged in LDS as they lie in memory and the matrix-core operands are fetched
// with the transposing LDS read (ds_read_b64_tr_b16), which hands each lane four
// consecutive contraction elements of one column.
//
// Tile: BM x BN outputs per workgroup, 4 waves in a 2 x 2 grid, each wave owns
// (BM/2) x (BN/2) as 32x32x16 bf16 MFMA tiles with fp32 accumulators; K is
// walked in steps of BK through a double-buffered LDS stage; global loads of the
// next stage are in flight while the current one is multiplied.
#include "poetx_kernels.h"

namespace poetx {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) short4v* lds_s4p;

// Pad of the row-major [k][x] tiles: 32 elements (64 B) puts four consecutive k rows
// on four different 16-bank groups, which is what one transposing read touches.
constexpr int PAD_T = 32;
// Pad of the [row][k] tile read with 16-byte loads: 8 elements (row stride 144 B at BK=64).
constexpr int PAD_K = 8;

__device__ inline short4v lds_read_tr(const uint16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(p));
}

// One 32 x 16 operand fragment (32 rows/cols x 16 contraction elements) out of a
// [k][x] LDS tile with row stride `stride` (elements): lane l ends up with column
// x0 + l%32 and contraction elements k0 + 8*(l/32) + 0..7.
__device__ inline bf16x8 frag_from_kx(const uint16_t* tile, int stride, int k0, int x0, int lane) {
  const int q = lane >> 4, i = lane & 15;
  const int krow = k0 + 8 * (q >> 1) + (i >> 2);
  const int col = x0 + 16 * (q & 1) + 4 * (i & 3);
  const uint16_t* p = tile + krow * stride + col;
  short4v lo = lds_read_tr(p);
  short4v hi = lds_read_tr(p + 4 * stride);
  short8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// Same fragment out of a [x][k] LDS tile (contraction index contiguous).
__device__ inline bf16x8 frag_from_xk(const uint16_t* tile, int stride, int k0, int x0, int lane) {
  const uint16_t* p = tile + (x0 + (lane & 31)) * stride + k0 + 8 * (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(p);
}

__device__ inline uint32_t pack2_bf16(float a, float b) {
  return (uint32_t)float_to_bf16_bits(a) | ((uint32_t)float_to_bf16_bits(b) << 16);
}

template <int BM, int BN, int BK, bool A_KMAJOR>
struct DenseCfg {
  static constexpr int NT = 256;
  static constexpr int SA = A_KMAJOR ? BK + PAD_K : BM + PAD_T;      // A tile row stride
  static constexpr int A_ROWS = A_KMAJOR ? BM : BK;
  static constexpr int SB = BN + PAD_T;
  static constexpr int A_ELEMS = A_ROWS * SA;
  static constexpr int B_ELEMS = BK * SB;
  static constexpr int STAGE = A_ELEMS + B_ELEMS;
  static constexpr size_t LDS_BYTES = (size_t)2 * STAGE * sizeof(uint16_t);
  static constexpr int A_CHUNKS = BM * BK / 8 / NT;  // 16-byte chunks per thread per stage
  static constexpr int B_CHUNKS = BK * BN / 8 / NT;
};

// C (M x N, ldc) = A * Bm,  Bm is K x N row major (ldb).
// A_KMAJOR: A is M x K row major (lda).  Otherwise A is given as K x M row major (lda): A(i,k) = A[k*lda + i].
// Requires M % BM == 0, N % BN == 0, K % BK == 0 and 16-byte aligned rows.
template <int BM, int BN, int BK, bool A_KMAJOR>
__global__ __launch_bounds__(256) void dense_bf16_kernel(const uint16_t* __restrict__ A, const uint16_t* __restrict__ Bm,
                                                          uint16_t* __restrict__ C, int M, int N, int K, i64 lda,
                                                          i64 ldb, i64 ldc, int tiles_m, int tiles_n) {
  using Cfg = DenseCfg<BM, BN, BK, A_KMAJOR>;
  constexpr int TM = BM / 2 / 32, TN = BN / 2 / 32;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];

  // Workgroups are handed to the 8 XCDs round robin; give each XCD one contiguous
  // chunk of the tile list so that neighbouring tiles share its L2, and walk the
  // chunk in groups of 4 tile rows.
  int wg = blockIdx.x;
  const int total = tiles_m * tiles_n;
  if ((total & 7) == 0) wg = (wg & 7) * (total >> 3) + (wg >> 3);
  constexpr int GROUP = 4;
  const int per_group = GROUP * tiles_n;
  const int grp = wg / per_group;
  const int first_m = grp * GROUP;
  const int gsz = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
  const int tile_m = first_m + (wg % per_group) % gsz;
  const int tile_n = (wg % per_group) / gsz;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const i64 i0 = (i64)tile_m * BM, j0 = (i64)tile_n * BN;

  uint4 ra[Cfg::A_CHUNKS], rb[Cfg::B_CHUNKS];

  auto load_global = [&](int kt) {
    const i64 k0 = (i64)kt * BK;
#pragma unroll
    for (int s = 0; s < Cfg::A_CHUNKS; ++s) {
      const int c = tid + s * 256;
      if (A_KMAJOR) {
        const int row = c / (BK / 8), ch = c % (BK / 8);
        ra[s] = *reinterpret_cast<const uint4*>(A + (i0 + row) * lda + k0 + ch * 8);
      } else {
        const int row = c / (BM / 8), ch = c % (BM / 8);
        ra[s] = *reinterpret_cast<const uint4*>(A + (k0 + row) * lda + i0 + ch * 8);
      }
    }
#pragma unroll
    for (int s = 0; s < Cfg::B_CHUNKS; ++s) {
      const int c = tid + s * 256;
      const int row = c / (BN / 8), ch = c % (BN / 8);
      rb[s] = *reinterpret_cast<const uint4*>(Bm + (k0 + row) * ldb + j0 + ch * 8);
    }
  };
  auto store_lds = [&](int stage) {
    uint16_t* As = lds + stage * Cfg::STAGE;
    uint16_t* Bs = As + Cfg::A_ELEMS;
#pragma unroll
    for (int s = 0; s < Cfg::A_CHUNKS; ++s) {
      const int c = tid + s * 256;
      const int row = A_KMAJOR ? c / (BK / 8) : c / (BM / 8);
      const int ch = A_KMAJOR ? c % (BK / 8) : c % (BM / 8);
      *reinterpret_cast<uint4*>(As + row * Cfg::SA + ch * 8) = ra[s];
    }
#pragma unroll
    for (int s = 0; s < Cfg::B_CHUNKS; ++s) {
      const int c = tid + s * 256;
      const int row = c / (BN / 8), ch = c % (BN / 8);
      *reinterpret_cast<uint4*>(Bs + row * Cfg::SB + ch * 8) = rb[s];
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int c = 0; c < TN; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][c][v] = 0.f;

  const int KT = K / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) load_global(kt + 1);
    const uint16_t* As = lds + cur * Cfg::STAGE;
    const uint16_t* Bs = As + Cfg::A_ELEMS;
#pragma unroll 2
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int a = 0; a < TM; ++a) {
        const int x0 = wm * (BM / 2) + a * 32;
        fa[a] = A_KMAJOR ? frag_from_xk(As, Cfg::SA, ks * 16, x0, lane) : frag_from_kx(As, Cfg::SA, ks * 16, x0, lane);
      }
#pragma unroll
      for (int c = 0; c < TN; ++c) fb[c] = frag_from_kx(Bs, Cfg::SB, ks * 16, wn * (BN / 2) + c * 32, lane);
      // Operands are passed swapped so that the accumulator tile is the transpose:
      // each lane then owns one output row and four consecutive token columns,
      // which store as one packed 8-byte write.
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int c = 0; c < TN; ++c)
          acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c], fa[a], acc[a][c], 0, 0, 0);
    }
    if (kt + 1 < KT) store_lds(cur ^ 1);
    __syncthreads();
  }

  const int h = lane >> 5, li = lane & 31;
#pragma unroll
  for (int a = 0; a < TM; ++a) {
    const i64 row = i0 + wm * (BM / 2) + a * 32 + li;
#pragma unroll
    for (int c = 0; c < TN; ++c) {
      const i64 col = j0 + wn * (BN / 2) + c * 32 + 4 * h;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint2 v;
        v.x = pack2_bf16(acc[a][c][4 * q + 0], acc[a][c][4 * q + 1]);
        v.y = pack2_bf16(acc[a][c][4 * q + 2], acc[a][c][4 * q + 3]);
        *reinterpret_cast<uint2*>(C + row * ldc + col + 8 * q) = v;
      }
    }
  }
}

template <int BM, int BN, int BK, bool A_KMAJOR>
void launch_dense(const uint16_t* A, const uint16_t* Bm, uint16_t* C, int M, i64 N, int K, i64 lda, hipStream_t st) {
  using Cfg = DenseCfg<BM, BN, BK, A_KMAJOR>;
  auto kern = dense_bf16_kernel<BM, BN, BK, A_KMAJOR>;
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cfg::LDS_BYTES);
    configured = true;
  }
  const int tiles_m = M / BM, tiles_n = (int)(N / BN);
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), Cfg::LDS_BYTES, st, A, Bm, C, M, (int)N, K, lda, N, N,
                     tiles_m, tiles_n);
}

constexpr int DBM = 256, DBN = 256, DBK = 64;

}  // namespace

bool mfma_dense_supported(int n, int m, i64 N) {
  return n % DBM == 0 && m % DBM == 0 && N % DBN == 0 && n % DBK == 0 && m % DBK == 0;
}

void mfma_dense(int trans_w, const void* W, int n, int m, const void* act, void* out, i64 N, hipStream_t st) {
  const uint16_t* w = (const uint16_t*)W;
  if (!trans_w) launch_dense<DBM, DBN, DBK, true>(w, (const uint16_t*)act, (uint16_t*)out, n, N, m, m, st);
  else launch_dense<DBM, DBN, DBK, false>(w, (const uint16_t*)act, (uint16_t*)out, m, N, n, m, st);
}

}  // namespace poetx
