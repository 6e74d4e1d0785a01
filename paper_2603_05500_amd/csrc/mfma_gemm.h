// Tiled bf16 matrix-core product shared by the dense, Cayley-Neumann and
// block-gradient stages (gfx950, wave64, v_mfma_f32_32x32x16_bf16).
//
//   C[batch] (M x N) = sum over up to two sources s of  A_s[batch] * B_s[batch]
//
// Each operand tile is staged in LDS exactly as it lies in memory.  An operand
// whose contraction index is contiguous ("K major": A given as M x K, B given as
// N x K) is fetched from LDS with 16-byte reads; one whose contraction index is
// the strided one (A given as K x M, B given as K x N) is fetched with the
// transposing LDS read ds_read_b64_tr_b16, which hands a lane four consecutive
// contraction elements of a single row/column.  Rows of K-major operands may be
// gathered through a permutation (block gradients).
//
// Workgroup: 256 threads = 2 x 2 waves, wave tile (BM/2) x (BN/2), fp32
// accumulators, double-buffered LDS stage of depth BK with the next stage's
// global loads in flight during the multiply.  The MFMA operands are passed
// swapped so the accumulator tile is transposed: a lane owns one output row
// and four consecutive columns, handed to the epilogue as one float4.
#pragma once

#include "poetx_kernels.h"

namespace poetx {
namespace mm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4v* lds_s4p;

// Row pad of [k][x] tiles: 32 elements (64 B) spreads the four k rows one
// transposing read touches over four different 16-bank groups.
constexpr int PAD_T = 32;
// Row pad of [x][k] tiles read with 16-byte loads.
constexpr int PAD_K = 8;

__device__ inline short4v lds_read_tr(const uint16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(p));
}

// 32 x 16 operand fragment from a [k][x] tile: lane l gets column x0 + l%32,
// contraction elements k0 + 8*(l/32) + 0..7.
__device__ inline bf16x8 frag_from_kx(const uint16_t* tile, int stride, int k0, int x0, int lane) {
  const int q = lane >> 4, i = lane & 15;
  const uint16_t* p = tile + (k0 + 8 * (q >> 1) + (i >> 2)) * stride + x0 + 16 * (q & 1) + 4 * (i & 3);
  short4v lo = lds_read_tr(p);
  short4v hi = lds_read_tr(p + 4 * stride);
  short8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// Same fragment from a [x][k] tile.
__device__ inline bf16x8 frag_from_xk(const uint16_t* tile, int stride, int k0, int x0, int lane) {
  return *reinterpret_cast<const bf16x8*>(tile + (x0 + (lane & 31)) * stride + k0 + 8 * (lane >> 5));
}

__device__ inline uint32_t pack2_bf16(float a, float b) {
  return (uint32_t)float_to_bf16_bits(a) | ((uint32_t)float_to_bf16_bits(b) << 16);
}

struct Source {
  const uint16_t* A;
  const uint16_t* B;
  i64 lda, ldb;        // row strides (elements)
  i64 sA, sB;          // batch strides (elements)
  int ktiles;          // BK-deep tiles taken from this source (per split)
};

struct Args {
  Source s[2];
  int nsrc;
  int tiles_m, tiles_n;      // output tiles per batch
  const int32_t* perm;       // GATHER: row r of batch j of both operands is memory row perm[j*rows_per_batch + r]
  int rows_per_batch;
};

template <int BM, int BN, int BK, bool A_KMAJOR, bool B_KMAJOR>
struct Cfg {
  static constexpr int SA = A_KMAJOR ? BK + PAD_K : BM + PAD_T;
  static constexpr int SB = B_KMAJOR ? BK + PAD_K : BN + PAD_T;
  static constexpr int A_ELEMS = (A_KMAJOR ? BM : BK) * SA;
  static constexpr int B_ELEMS = (B_KMAJOR ? BN : BK) * SB;
  static constexpr int STAGE = A_ELEMS + B_ELEMS;
  static constexpr size_t LDS_BYTES = (size_t)2 * STAGE * sizeof(uint16_t);
  static constexpr int A_CHUNKS = BM * BK / 8 / 256;
  static constexpr int B_CHUNKS = BK * BN / 8 / 256;
};

// Epi: __device__ void operator()(int batch, int split, int row, int col, float4 v) -- four
// consecutive columns col..col+3 of output row `row` (indices local to the batch).
// grid = (tiles_m * tiles_n, batches, splits).  With splits > 1 split z contracts k tiles
// [z * ktiles, (z+1) * ktiles) of source 0.
template <int BM, int BN, int BK, bool A_KMAJOR, bool B_KMAJOR, bool GATHER, class Epi>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(Args g, Epi epi) {
  using C = Cfg<BM, BN, BK, A_KMAJOR, B_KMAJOR>;
  constexpr int TM = BM / 64, TN = BN / 64;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];

  // Workgroups go to the 8 XCDs round robin: give each XCD a contiguous chunk of
  // the tile list (its own L2 then serves neighbouring tiles), walked in groups
  // of 4 tile rows.
  int wg = blockIdx.x;
  const int total = g.tiles_m * g.tiles_n;
  if ((total & 7) == 0) wg = (wg & 7) * (total >> 3) + (wg >> 3);
  constexpr int GROUP = 4;
  const int per_group = GROUP * g.tiles_n;
  const int first_m = (wg / per_group) * GROUP;
  const int gsz = (g.tiles_m - first_m) < GROUP ? (g.tiles_m - first_m) : GROUP;
  const int tile_m = first_m + (wg % per_group) % gsz;
  const int tile_n = (wg % per_group) / gsz;
  const int batch = blockIdx.y, split = blockIdx.z;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int i0 = tile_m * BM, j0 = tile_n * BN;

  u32x4 ra[C::A_CHUNKS], rb[C::B_CHUNKS];
  // Gathered rows: element offsets of this thread's rows, fixed over the k loop.
  i64 ga[GATHER ? C::A_CHUNKS : 1], gb[GATHER ? C::B_CHUNKS : 1];
  if (GATHER) {
    const int32_t* pm = g.perm + (i64)batch * g.rows_per_batch;
#pragma unroll
    for (int s = 0; s < C::A_CHUNKS; ++s) ga[s] = (i64)pm[i0 + (tid + s * 256) / (BK / 8)] * g.s[0].lda;
#pragma unroll
    for (int s = 0; s < C::B_CHUNKS; ++s) gb[s] = (i64)pm[j0 + (tid + s * 256) / (BK / 8)] * g.s[0].ldb;
  }

  auto load_global = [&](const Source& src, int kt) {
    const i64 k0 = (i64)kt * BK;
    const uint16_t* Ab = src.A + (GATHER ? 0 : batch * src.sA);
    const uint16_t* Bb = src.B + (GATHER ? 0 : batch * src.sB);
#pragma unroll
    for (int s = 0; s < C::A_CHUNKS; ++s) {
      const int c = tid + s * 256;
      if (A_KMAJOR) {
        const int row = c / (BK / 8), ch = c % (BK / 8);
        const i64 off = GATHER ? ga[s] : (i64)(i0 + row) * src.lda;
        ra[s] = *reinterpret_cast<const u32x4*>(Ab + off + k0 + ch * 8);
      } else {
        const int row = c / (BM / 8), ch = c % (BM / 8);
        ra[s] = *reinterpret_cast<const u32x4*>(Ab + (k0 + row) * src.lda + i0 + ch * 8);
      }
    }
#pragma unroll
    for (int s = 0; s < C::B_CHUNKS; ++s) {
      const int c = tid + s * 256;
      if (B_KMAJOR) {
        const int row = c / (BK / 8), ch = c % (BK / 8);
        const i64 off = GATHER ? gb[s] : (i64)(j0 + row) * src.ldb;
        rb[s] = *reinterpret_cast<const u32x4*>(Bb + off + k0 + ch * 8);
      } else {
        const int row = c / (BN / 8), ch = c % (BN / 8);
        rb[s] = *reinterpret_cast<const u32x4*>(Bb + (k0 + row) * src.ldb + j0 + ch * 8);
      }
    }
  };
  auto store_lds = [&](int stage) {
    uint16_t* As = lds + stage * C::STAGE;
    uint16_t* Bs = As + C::A_ELEMS;
#pragma unroll
    for (int s = 0; s < C::A_CHUNKS; ++s) {
      const int c = tid + s * 256;
      const int row = A_KMAJOR ? c / (BK / 8) : c / (BM / 8);
      const int ch = A_KMAJOR ? c % (BK / 8) : c % (BM / 8);
      *reinterpret_cast<u32x4*>(As + row * C::SA + ch * 8) = ra[s];
    }
#pragma unroll
    for (int s = 0; s < C::B_CHUNKS; ++s) {
      const int c = tid + s * 256;
      const int row = B_KMAJOR ? c / (BK / 8) : c / (BN / 8);
      const int ch = B_KMAJOR ? c % (BK / 8) : c % (BN / 8);
      *reinterpret_cast<u32x4*>(Bs + row * C::SB + ch * 8) = rb[s];
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int c = 0; c < TN; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][c][v] = 0.f;

  // k tiles of source 0 then source 1, as one sequence
  const int kt0 = g.s[0].ktiles;
  const int KT = kt0 + (g.nsrc > 1 ? g.s[1].ktiles : 0);
  const int kbase = split * kt0;
  auto fetch = [&](int kt) {
    if (kt < kt0) load_global(g.s[0], kbase + kt);
    else load_global(g.s[1], kt - kt0);
  };

  auto multiply = [&](int stage) {
    const uint16_t* As = lds + stage * C::STAGE;
    const uint16_t* Bs = As + C::A_ELEMS;
#pragma unroll 2
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int a = 0; a < TM; ++a) {
        const int x0 = wm * (BM / 2) + a * 32;
        fa[a] = A_KMAJOR ? frag_from_xk(As, C::SA, ks * 16, x0, lane) : frag_from_kx(As, C::SA, ks * 16, x0, lane);
      }
#pragma unroll
      for (int c = 0; c < TN; ++c) {
        const int x0 = wn * (BN / 2) + c * 32;
        fb[c] = B_KMAJOR ? frag_from_xk(Bs, C::SB, ks * 16, x0, lane) : frag_from_kx(Bs, C::SB, ks * 16, x0, lane);
      }
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int c = 0; c < TN; ++c)
          acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c], fa[a], acc[a][c], 0, 0, 0);
    }
  };

  // The last tile is peeled so that the loads inside the loop are unconditional: the
  // staging registers then have a single definition per iteration and nothing has to
  // wait for them before the multiply.
  fetch(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt + 1 < KT; ++kt) {
    fetch(kt + 1);
    multiply(kt & 1);
    store_lds((kt & 1) ^ 1);
    __syncthreads();
  }
  multiply((KT - 1) & 1);

  const int h = lane >> 5, li = lane & 31;
#pragma unroll
  for (int a = 0; a < TM; ++a) {
    const int row = i0 + wm * (BM / 2) + a * 32 + li;
#pragma unroll
    for (int c = 0; c < TN; ++c) {
      const int col = j0 + wn * (BN / 2) + c * 32 + 4 * h;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        epi(batch, split, row, col + 8 * q,
            make_float4(acc[a][c][4 * q], acc[a][c][4 * q + 1], acc[a][c][4 * q + 2], acc[a][c][4 * q + 3]));
    }
  }
}

template <int BM, int BN, int BK, bool A_KMAJOR, bool B_KMAJOR, bool GATHER, class Epi>
void launch(const Args& g, Epi epi, int batches, int splits, hipStream_t st) {
  using C = Cfg<BM, BN, BK, A_KMAJOR, B_KMAJOR>;
  auto kern = gemm_bf16_kernel<BM, BN, BK, A_KMAJOR, B_KMAJOR, GATHER, Epi>;
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
    configured = true;
  }
  hipLaunchKernelGGL(kern, dim3(g.tiles_m * g.tiles_n, batches, splits), dim3(256), C::LDS_BYTES, st, g, epi);
}

// Plain bf16 store of the output tile.
struct EpiStoreBf16 {
  uint16_t* C;
  i64 ldc, sC;
  __device__ void operator()(int batch, int, int row, int col, float4 v) const {
    uint2 o;
    o.x = pack2_bf16(v.x, v.y);
    o.y = pack2_bf16(v.z, v.w);
    *reinterpret_cast<uint2*>(C + batch * sC + (i64)row * ldc + col) = o;
  }
};

}  // namespace mm
}  // namespace poetx
