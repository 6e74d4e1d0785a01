// Fused permutation-gather + block-diagonal product + permutation-scatter on bf16
// activations (Eq. 2 with Eq. 5 and Eq. 7; mm1 / mm3 of Eq. 10 and their input
// gradients):
//     out[pi[j*b + i], t] = V[pi[j*b + i], t] + sum_l op(E_j)(i, l) * V[pi[j*b + l], t]
// with E = G - I, so neither the permutation nor the orthogonal matrix is ever
// materialised and the identity part of G is carried exactly.
//
// The stage is HBM bound (b/2 flop per byte), so the kernel is organised around
// the memory stream: one workgroup owns block j and a tile of BN tokens, gathers
// the b rows of that tile once into LDS (each row is a contiguous run of tokens,
// so the gather is coalesced), multiplies from LDS with transposing reads, adds
// the identity term from the same LDS tile, writes the result back into the tile
// and streams it out with the same coalesced row pattern (scatter by the same
// index map).  The block operand op(E_j) is read straight from global memory in
// matrix-core fragment order: blocks are stored as the pair (E, E^T) so that
// op(E)(i, .) is always a contiguous row; the pair stays L2 resident because every
// token tile of block j reuses it.
#include "mfma_gemm.h"

namespace poetx {
namespace {

using mm::bf16x8;
using mm::floatx16;
using mm::short4v;
using mm::short8v;

// Row pad of the gathered [l][token] tile: 32 elements (64 B) spreads the four l rows one
// transposing read touches over different bank groups.
constexpr int PAD_T = 32;

// 32 x 16 matrix-core operand fragment from a padded [k][x] LDS tile (row stride `stride`
// elements): lane gets column x0 + lane%32 and contraction elements k0 + 8*(lane/32) + 0..7.
__device__ inline bf16x8 frag_from_kx(const uint16_t* tile, int stride, int k0, int x0, int lane) {
  const int q = lane >> 4, i = lane & 15;
  const uint16_t* p = tile + (k0 + 8 * (q >> 1) + (i >> 2)) * stride + x0 + 16 * (q & 1) + 4 * (i & 3);
  short4v lo = mm::lds_read_tr((const char*)p);
  short4v hi = mm::lds_read_tr((const char*)(p + 4 * stride));
  short8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// B: block side.  BN: tokens per workgroup.  4 waves, wave w owns output rows
// [w*B/4, (w+1)*B/4) for all BN tokens.
template <int B, int BN>
__global__ __launch_bounds__(256) void apply_left_bf16_kernel(const uint16_t* __restrict__ V, uint16_t* __restrict__ out,
                                                               i64 ld, const int32_t* __restrict__ perm,
                                                               const uint16_t* __restrict__ blocks, int trans) {
  constexpr int SX = BN + PAD_T;
  constexpr int TM = B / 4 / 32, TN = BN / 32;
  constexpr int CPR = BN / 8;                 // 16-byte chunks per row
  constexpr int CHUNKS = B * CPR / 256;       // per thread
  constexpr int ROWS_PER_PASS = 256 / CPR;
  extern __shared__ __attribute__((aligned(16))) uint16_t xs[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int j = blockIdx.y;
  const i64 t0 = (i64)blockIdx.x * BN;
  const int32_t* pm = perm + (i64)j * B;
  const int crow = tid / CPR, cch = tid % CPR;

  // gather: rows pi[j*B + l] of V, BN tokens each
#pragma unroll 4
  for (int s = 0; s < CHUNKS; ++s) {
    const int row = crow + s * ROWS_PER_PASS;
    const uint4 v = *reinterpret_cast<const uint4*>(V + (i64)pm[row] * ld + t0 + cch * 8);
    *reinterpret_cast<uint4*>(xs + row * SX + cch * 8) = v;
  }
  __syncthreads();

  floatx16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int c = 0; c < TN; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][c][v] = 0.f;

  const int li = lane & 31, h = lane >> 5;
  const int row0 = wave * (B / 4);
  const uint16_t* Eb = blocks + ((i64)j * 2 + (trans ? 1 : 0)) * B * B + (i64)(row0 + li) * B + 8 * h;

  bf16x8 fa[TM], fa_next[TM];
#pragma unroll
  for (int a = 0; a < TM; ++a) fa[a] = *reinterpret_cast<const bf16x8*>(Eb + (i64)a * 32 * B);
#pragma unroll 4
  for (int ks = 0; ks < B / 16; ++ks) {
    if (ks + 1 < B / 16) {
#pragma unroll
      for (int a = 0; a < TM; ++a) fa_next[a] = *reinterpret_cast<const bf16x8*>(Eb + (i64)a * 32 * B + (ks + 1) * 16);
    }
    bf16x8 fb[TN];
#pragma unroll
    for (int c = 0; c < TN; ++c) fb[c] = frag_from_kx(xs, SX, ks * 16, c * 32, lane);
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int c = 0; c < TN; ++c)
        acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[c], fa[a], acc[a][c], 0, 0, 0);
#pragma unroll
    for (int a = 0; a < TM; ++a) fa[a] = fa_next[a];
  }
  __syncthreads();  // every wave is done reading the gathered tile

  // identity term + rounding, in place: lane owns row (row0 + a*32 + li), tokens c*32 + 8q + 4h .. +3
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int c = 0; c < TN; ++c)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint16_t* p = xs + (row0 + a * 32 + li) * SX + c * 32 + 8 * q + 4 * h;
        const uint2 x = *reinterpret_cast<const uint2*>(p);
        uint2 o;
        o.x = mm::pack2_bf16(acc[a][c][4 * q + 0] + bf16_bits_to_float((uint16_t)(x.x & 0xFFFF)),
                             acc[a][c][4 * q + 1] + bf16_bits_to_float((uint16_t)(x.x >> 16)));
        o.y = mm::pack2_bf16(acc[a][c][4 * q + 2] + bf16_bits_to_float((uint16_t)(x.y & 0xFFFF)),
                             acc[a][c][4 * q + 3] + bf16_bits_to_float((uint16_t)(x.y >> 16)));
        *reinterpret_cast<uint2*>(p) = o;
      }
  __syncthreads();

  // scatter: same row map, coalesced 16-byte stores
#pragma unroll 4
  for (int s = 0; s < CHUNKS; ++s) {
    const int row = crow + s * ROWS_PER_PASS;
    const uint4 v = *reinterpret_cast<const uint4*>(xs + row * SX + cch * 8);
    *reinterpret_cast<uint4*>(out + (i64)pm[row] * ld + t0 + cch * 8) = v;
  }
}

template <int B, int BN>
void launch_apply(const uint16_t* V, uint16_t* out, int d, i64 cols, i64 ld, const int32_t* perm, const uint16_t* E,
                  int trans, hipStream_t st) {
  constexpr size_t LDS = (size_t)B * (BN + PAD_T) * sizeof(uint16_t);
  auto kern = apply_left_bf16_kernel<B, BN>;
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
    configured = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(cols / BN), d / B), dim3(256), LDS, st, V, out, ld, perm, E, trans);
}

constexpr int BN256 = 128, BN512 = 64;

}  // namespace

bool mfma_apply_left_supported(int d, i64 cols, i64 ld, int b) {
  if (d % b != 0 || ld % 8 != 0) return false;
  if (b == 256) return cols % BN256 == 0;
  if (b == 512) return cols % BN512 == 0;
  return false;
}

void mfma_apply_left(const void* V, void* out, int d, i64 cols, i64 ld, const int32_t* perm, const void* E, int b,
                     int transpose_G, hipStream_t st) {
  if (b == 256)
    launch_apply<256, BN256>((const uint16_t*)V, (uint16_t*)out, d, cols, ld, perm, (const uint16_t*)E, transpose_G, st);
  else
    launch_apply<512, BN512>((const uint16_t*)V, (uint16_t*)out, d, cols, ld, perm, (const uint16_t*)E, transpose_G, st);
}

}  // namespace poetx
