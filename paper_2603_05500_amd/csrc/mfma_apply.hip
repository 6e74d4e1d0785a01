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


// ---------------------------------------------------------------------------------------
// Streaming variant: one persistent workgroup per (block, 256-row slice of it, token range).
//   * 8 waves; wave w owns 32 output rows of the slice for computing and storing.
//   * those rows of op(E_j) stay in registers as matrix-core fragments for the whole range
//     (B/16 k steps x 4 VGPRs), so the block operand is read once per workgroup.
//   * token tiles of BN go from HBM straight into a 2-stage LDS ring (global_load_lds, all B
//     rows of the block gathered through the permutation, XOR-swizzled chunks, no bank
//     conflicts); the tile of the next step is in flight while the current one is multiplied.
//   * the identity part of G is applied as one exact extra MFMA per k step that covers the
//     wave's own rows (1.0 * x accumulates exactly in fp32), so nothing is re-read.
//   * results leave from registers: a lane owns one row and 4 consecutive tokens (8-byte
//     packed stores), scattered through the same index map that gathered them.
// b = 256: one slice, 128-token tiles.  b = 512: two slices per block (the block operand of
// a whole block does not fit the register file), 64-token tiles; the two workgroups of a
// block read the same token tiles, the second read being served by L2 / Infinity Cache.
template <int B, int BN>
__global__ __launch_bounds__(512) void apply_left_stream_kernel(const uint16_t* __restrict__ V,
                                                                 uint16_t* __restrict__ out, i64 ld,
                                                                 const int32_t* __restrict__ perm,
                                                                 const uint16_t* __restrict__ blocks, int trans,
                                                                 int tiles_per_wg, int paired_chunks) {
  constexpr int MSPLIT = B / 256, TN = BN / 32, KS = B / 16;
  constexpr int STAGE_BYTES = B * BN * 2;
  constexpr int CPR = BN / 8;                        // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;                      // rows filled by one direct-to-LDS instruction
  constexpr int IPW = STAGE_BYTES / 1024 / 8;        // such instructions per wave per stage
  extern __shared__ __attribute__((aligned(1024))) char ring[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Which (block, slice, token range).  With two slices per block (paired_chunks > 0, one-dimensional
  // grid) the two workgroups that read the same token tiles get ids 8 apart: consecutive ids go to the
  // 8 XCDs in turn, so the pair shares one L2 and the tiles cross the fabric once.
  int j = blockIdx.y, slice = blockIdx.x % MSPLIT, chunk = blockIdx.x / MSPLIT;
  if (MSPLIT == 2 && paired_chunks > 0) {
    const int id = blockIdx.x, pair = (id >> 4) * 8 + (id & 7);
    slice = (id >> 3) & 1;
    j = pair / paired_chunks;
    chunk = pair % paired_chunks;
  }
  const i64 tok0 = (i64)chunk * tiles_per_wg * BN;
  const int32_t* pm = perm + (i64)j * B;
  const int li = lane & 31, h = lane >> 5;
  const uint32_t ring_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)ring;

  // direct-to-LDS instruction s of this wave fills chunk slots [(IPW*w+s)*64, +64) of a stage:
  // row k = (IPW*w+s)*RPI + lane/CPR, chunk position lane%CPR -> logical chunk through the swizzle.
  i64 goff[IPW];
#pragma unroll
  for (int s = 0; s < IPW; ++s) {
    const int k = (wave * IPW + s) * RPI + lane / CPR;
    const int c = mm::kx_unchunk<BN>(lane % CPR, k);
    goff[s] = (i64)pm[k] * ld + tok0 + c * 8;
  }
  auto issue = [&](int t) {
    const uint32_t stage = ring_base + (t & 1) * STAGE_BYTES + wave * IPW * 1024;
#pragma unroll
    for (int s = 0; s < IPW; ++s) mm::dma16(V + goff[s] + (i64)t * BN, stage + s * 1024);
  };
  issue(0);

  // block operand fragments (rows of op(E_j) are contiguous in the stored pair)
  const int row_own = slice * 256 + wave * 32 + li;
  const uint16_t* Eb = blocks + ((i64)j * 2 + (trans ? 1 : 0)) * B * B + (i64)row_own * B + 8 * h;
  bf16x8 fa[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) fa[ks] = *reinterpret_cast<const bf16x8*>(Eb + ks * 16);
  // identity fragments for the two k steps that cover the wave's own 32 rows
  bf16x8 fi[2];
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int e = 0; e < 8; ++e) fi[u][e] = (li == u * 16 + 8 * h + e) ? (__bf16)1.0f : (__bf16)0.0f;
  const int own_kpair = slice * 8 + wave;  // k steps 2*own_kpair and 2*own_kpair + 1

  // LDS byte offsets of this lane's token fragments at k step 0
  int fragB[TN];
  {
    const int q = lane >> 4, i = lane & 15;
    const int k = 8 * (q >> 1) + (i >> 2);
#pragma unroll
    for (int c2 = 0; c2 < TN; ++c2) {
      const int c = c2 * 4 + 2 * (q & 1) + ((i & 3) >> 1);
      fragB[c2] = k * (BN * 2) + 16 * mm::kx_chunk<BN>(c, k) + 8 * (i & 1);
    }
  }
  // Results leave through a per-wave staging area behind the ring (32 rows x 64 tokens = 4 KB): the
  // wave writes a 64-token half of its tile there in accumulator order and reads it back with 8
  // consecutive lanes on one row, so that every global store instruction writes whole 128-byte row
  // segments (scattered through the same index map that gathered the rows).  Only the wave itself
  // touches its area, so its own lgkmcnt wait is all the synchronisation this needs.
  constexpr int NH = TN / 2;                          // 64-token halves of a tile
  char* stg = ring + 2 * STAGE_BYTES + wave * 4096;
  // write side: row li, chunk (8 tokens) cl*4 + 2p + h of the half, XOR-swizzled by the row pair
  const int stg_w = li * 128 + 16 * (h ^ ((li >> 1) & 7));
  // read side / stores: rows (lane >> 3) + 8 i, chunk lane & 7
  i64 soff[4];
  int stg_r[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = (lane >> 3) + 8 * i;
    soff[i] = (i64)pm[slice * 256 + wave * 32 + r] * ld + tok0 + 8 * (lane & 7);
    stg_r[i] = r * 128 + 16 * ((lane & 7) ^ ((r >> 1) & 7));
  }

  // The stores of a tile are issued one iteration late, right after the next barrier: by the
  // following barrier both those stores and the loads of the next tile are old, so a plain
  // vmcnt(0) there waits for nothing that is not already due (loads and stores share one counter
  // and may retire out of order with respect to each other).
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 pend[NH * 4];
  auto flush = [&](int t) {
#pragma unroll
    for (int hf = 0; hf < NH; ++hf)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        *reinterpret_cast<u32x4*>(out + soff[i] + (i64)t * BN + hf * 64) = pend[hf * 4 + i];
  };
  for (int t = 0; t < tiles_per_wg; ++t) {
    // tile t has landed and every wave is done reading the stage that tile t+1 overwrites: the
    // wait covers this wave's own LDS reads too (lgkmcnt), so the ring does not depend on where the
    // compiler places the MFMAs that consume them
    mm::wait_all_reads_and_barrier<0>();
    if (t > 0) flush(t - 1);
    if (t + 1 < tiles_per_wg) issue(t + 1);
    const char* stage = ring + (t & 1) * STAGE_BYTES;
    auto load_tok = [&](bf16x8* fb, int ks) {
#pragma unroll
      for (int c = 0; c < TN; ++c) {
        const char* p = stage + fragB[c] + ks * 16 * (BN * 2);
        short4v lo = mm::lds_read_tr(p);
        short4v hi = mm::lds_read_tr(p + 4 * (BN * 2));
        short8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        fb[c] = __builtin_bit_cast(bf16x8, v);
      }
    };
    floatx16 acc[TN];
#pragma unroll
    for (int c = 0; c < TN; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
    // identity part first (the two k steps that cover the wave's own rows: a wave-uniform LDS
    // address, no branch in the main loop), then the block operand with the token fragments of
    // the next k step always in flight under the MFMAs of the current one
    bf16x8 fo[2][TN], fb[2][TN];
    load_tok(fo[0], 2 * own_kpair);
    load_tok(fo[1], 2 * own_kpair + 1);
    load_tok(fb[0], 0);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int c = 0; c < TN; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo[u][c], fi[u], acc[c], 0, 0, 0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) load_tok(fb[(ks + 1) & 1], ks + 1);
#pragma unroll
      for (int c = 0; c < TN; ++c)
        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks & 1][c], fa[ks], acc[c], 0, 0, 0);
    }
    // round; registers 4q..4q+3 hold tokens 8q + 4h + 0..3.  v_permlane32_swap exchanges the upper
    // lane half of its first operand with the lower half of its second, which leaves the lower lanes
    // with tokens 16p .. 16p+7 and the upper lanes with tokens 16p+8 .. 16p+15 of the 32-token
    // tile: 16-byte pieces, written to the staging area and read back row by row
#pragma unroll
    for (int hf = 0; hf < NH; ++hf) {
#pragma unroll
      for (int cl = 0; cl < 2; ++cl) {
        const int c = 2 * hf + cl;
        uint32_t w[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = mm::pack2_bf16(acc[c][2 * e], acc[c][2 * e + 1]);
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          typedef unsigned uint2v __attribute__((ext_vector_type(2)));
          const uint2v r0 = __builtin_amdgcn_permlane32_swap(w[4 * p], w[4 * p + 2], false, false);
          const uint2v r1 = __builtin_amdgcn_permlane32_swap(w[4 * p + 1], w[4 * p + 3], false, false);
          // chunk cl*4 + 2p + h: the XOR with the row pair commutes with adding the even part
          *reinterpret_cast<u32x4*>(stg + (stg_w ^ (16 * (cl * 4 + 2 * p)))) = u32x4{r0[0], r1[0], r0[1], r1[1]};
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int i = 0; i < 4; ++i) pend[hf * 4 + i] = *reinterpret_cast<const u32x4*>(stg + stg_r[i]);
      if (hf + 1 < NH) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // read back before the area is rewritten
    }
  }
  flush(tiles_per_wg - 1);
}

// token ranges per block slice: fill the 256 CUs in whole rounds, at least 2 tiles per workgroup
int stream_chunks(int slices, int tiles) {
  int best = 1;
  double best_eff = 0.0;
  for (int c = 1; c <= tiles; c *= 2) {
    if (tiles % c != 0 || tiles / c < 2) break;
    const double wgs = (double)slices * c;
    const double rounds = (double)(long long)((wgs + 255) / 256);
    const double eff = wgs / 256.0 / rounds;
    if (eff > best_eff + 1e-9) { best_eff = eff; best = c; }
  }
  return best;
}

template <int B, int BN>
void launch_apply_stream(const uint16_t* V, uint16_t* out, int d, i64 cols, i64 ld, const int32_t* perm,
                         const uint16_t* E, int trans, hipStream_t st) {
  constexpr size_t LDS = 2 * (size_t)B * BN * 2 + 8 * 4096;   // 2-stage ring + per-wave output staging
  constexpr int MSPLIT = B / 256;
  auto kern = apply_left_stream_kernel<B, BN>;
  // once per kernel instance; a function-local static is initialised exactly once, whichever thread gets there first
  static const bool configured =
      hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS) == hipSuccess;
  (void)configured;
  const int nb = d / B, tiles = (int)(cols / BN);
  const int chunks = stream_chunks(nb * MSPLIT, tiles);
  if (MSPLIT == 2 && (nb * chunks) % 8 == 0)
    hipLaunchKernelGGL(kern, dim3(chunks * MSPLIT * nb), dim3(512), LDS, st, V, out, ld, perm, E, trans, tiles / chunks, chunks);
  else
    hipLaunchKernelGGL(kern, dim3(chunks * MSPLIT, nb), dim3(512), LDS, st, V, out, ld, perm, E, trans, tiles / chunks, 0);
}
constexpr int SBN256 = 128, SBN512 = 64;   // tokens per tile of the streaming kernel

template <int B, int BN>
void launch_apply(const uint16_t* V, uint16_t* out, int d, i64 cols, i64 ld, const int32_t* perm, const uint16_t* E,
                  int trans, hipStream_t st) {
  constexpr size_t LDS = (size_t)B * (BN + PAD_T) * sizeof(uint16_t);
  auto kern = apply_left_bf16_kernel<B, BN>;
  // once per kernel instance; a function-local static is initialised exactly once, whichever thread gets there first
  static const bool configured =
      hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS) == hipSuccess;
  (void)configured;
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
  if (b == 256 && cols % (2 * SBN256) == 0)
    launch_apply_stream<256, SBN256>((const uint16_t*)V, (uint16_t*)out, d, cols, ld, perm, (const uint16_t*)E, transpose_G, st);
  else if (b == 512 && cols % (2 * SBN512) == 0)
    launch_apply_stream<512, SBN512>((const uint16_t*)V, (uint16_t*)out, d, cols, ld, perm, (const uint16_t*)E, transpose_G, st);
  else if (b == 256)
    launch_apply<256, BN256>((const uint16_t*)V, (uint16_t*)out, d, cols, ld, perm, (const uint16_t*)E, transpose_G, st);
  else
    launch_apply<512, BN512>((const uint16_t*)V, (uint16_t*)out, d, cols, ld, perm, (const uint16_t*)E, transpose_G, st);
}

}  // namespace poetx
