// Tiled bf16 matrix-core product shared by the dense, Cayley-Neumann and
// block-gradient stages (gfx950, wave64, v_mfma_f32_32x32x16_bf16).
//
//   C[batch] (M x N) = sum over up to two sources s of  A_s[batch] * B_s[batch]
//
// Operand tiles go from global memory straight into LDS (global_load_lds, 16
// bytes per lane, no staging registers) through a ring of NS stages of BK = 32
// (4 for the long contractions, deeper for the short ones of the series kernels),
// so up to NS - 1 tiles are in flight while one is multiplied and the only per-tile
// synchronisation is one barrier.  A tile is stored unpadded; bank conflicts are
// avoided by an XOR swizzle of the 16-byte chunks, which costs nothing because
// every lane may fetch any global chunk.
//
// An operand whose contraction index is contiguous in memory ("K major": A given
// as M x K, B given as N x K) is read from LDS with 16-byte loads; one whose
// contraction index is the strided one (A given as K x M, B given as K x N) is
// read with the transposing LDS load ds_read_b64_tr_b16, which hands a lane four
// consecutive contraction elements of one row/column.  Rows of K-major operands
// may be gathered through a permutation (block gradients).
//
// Workgroup: WGM x WGN waves (2 x 4 for the 256 x 256 tile, i.e. two waves per SIMD),
// wave tile (BM/WGM) x (BN/WGN), fp32 accumulators.  The MFMA operands are passed swapped so the accumulator tile is
// transposed: a lane owns one output row and four consecutive columns, handed to
// the epilogue as one float4.
#pragma once
#include <type_traits>

#include "poetx_kernels.h"

namespace poetx {
namespace mm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) short4v* lds_s4p;

constexpr int BK = 32;       // contraction depth of one stage

__device__ inline short4v lds_read_tr(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(p));
}

// Two floats to two bf16 (round to nearest even) in one v_cvt_pk_bf16_f32; a in the low half.
__device__ inline uint32_t pack2_bf16(float a, float b) {
  typedef float float2v __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const float2v f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// ---- swizzled tile layouts (16-byte chunk granularity) --------------------------------
// [x][k] tile ("xk", K major): row = BK elements = 4 chunks.  16 consecutive rows read the
// same logical chunk at once, so the chunk position is XORed with bits 2..3 of the row.
__device__ inline int xk_chunk(int c, int row) { return c ^ ((row >> 2) & 3); }
// [k][x] tile ("kx", K strided): row = X elements.  A transposing read touches 4
// consecutive k rows x 2 chunks; XOR with the k row spreads them over 8 chunk positions,
// and for wide tiles bit 1 of the chunk index is folded into bit 3 so that the two column
// halves of a 32-wide fragment use different 128-byte halves of the bank space.
template <int X>
__device__ inline int kx_chunk(int c, int k) {
  int p = c ^ (2 * (k & 3));
  if (X >= 128) p ^= ((c >> 1) & 1) << 3;
  return p;
}
template <int X>
__device__ inline int kx_unchunk(int p, int k) {
  int c = p ^ (2 * (k & 3));
  if (X >= 128) c ^= ((c >> 1) & 1) << 3;   // bit 1 of c is already final here
  return c;
}

struct Source {
  const uint16_t* A;
  const uint16_t* B;
  i64 lda, ldb;        // row strides (elements)
  i64 sA, sB;          // batch strides (elements)
  int ktiles;          // 64-deep k tiles taken from this source (per split)
};

struct Args {
  Source s[2];
  int nsrc;
  // Optional second problem in the same launch: batches >= alt_from run it (with batch index
  // batch - alt_from for the operand strides; the epilogue still sees the raw batch index).
  // Same tile shape, strides and layout flags as the first; alt_from = 0 disables it.
  Source alt[2];
  int alt_nsrc;
  int alt_from;
  int tiles_m, tiles_n;      // output tiles per batch
  const int32_t* perm;       // GATHER: row r of batch j of both operands is memory row perm[j*rows_per_batch + r]
  int rows_per_batch;
  // Set by launch(): > 0 means a one-dimensional grid in which the tiles of one (batch, split) get
  // workgroup ids 8 apart, i.e. run on one XCD at the same time and share their operand panels in its
  // L2 (consecutive ids go to the 8 XCDs in turn); the value is the number of batches.
  int xcd_batches;
};

// NS = ring depth (stages); up to NS - 1 tiles are in flight while one is multiplied.
template <int BM, int BN, int WGM, int WGN, int NS>
struct Cfg {
  static constexpr int NWAVE = WGM * WGN;
  static constexpr int A_BYTES = BM * BK * 2;
  static constexpr int B_BYTES = BN * BK * 2;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr size_t LDS_BYTES = (size_t)NS * STAGE_BYTES;
  static constexpr int IPW_A = A_BYTES / 1024 / NWAVE;   // direct-to-LDS instructions per wave per stage
  static constexpr int IPW_B = B_BYTES / 1024 / NWAVE;
  static_assert(IPW_A >= 1 && IPW_B >= 1, "tile too small for this many waves");
};

// Wait until at most N of this wave's vector-memory operations are outstanding, then
// meet the other waves.  Written as one asm statement because __syncthreads() would
// drain every outstanding load (it carries a full fence) and so serialise the ring; the
// memory clobber keeps the compiler from moving LDS accesses across the barrier.
// 16 bytes per lane from global memory straight into LDS at lds_addr + 16 * lane.  Inline
// asm (not the builtin) so that the compiler does not drain vmcnt before later LDS reads:
// completion is tracked by hand with wait_vmcnt_and_barrier.  lds_addr is wave uniform.
__device__ inline void dma16(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory");
}

template <int N>
__device__ inline void wait_vmcnt_and_barrier() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}
// The same, and this wave's LDS reads have returned too (so that the stage they came from may
// be overwritten by whoever passes the barrier).
template <int N>
__device__ inline void wait_all_reads_and_barrier() {
  static_assert(N >= 0 && N < 64, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// The same with a run-time (wave uniform) bound: at most min(tiles, MAXT) tiles of LPT loads
// each may stay outstanding.  The count must be an immediate, hence the chain of cases.
template <int LPT, int MAXT>
__device__ inline void wait_tiles_and_barrier(int tiles) {
  if constexpr (MAXT <= 0) {
    wait_all_reads_and_barrier<0>();
  } else {
    if (tiles >= MAXT) wait_all_reads_and_barrier<MAXT * LPT>();
    else wait_tiles_and_barrier<LPT, MAXT - 1>(tiles);
  }
}

// An epilogue may also offer  void wide(int batch, int split, int row, int col, float4 lo, float4 hi)  for
// eight consecutive columns col..col+7; the kernel then calls that instead (wider loads and stores).
template <class E, class = void>
struct has_wide : std::false_type {};
template <class E>
struct has_wide<E, std::void_t<decltype(&E::wide)>> : std::true_type {};

// Epi: __device__ void operator()(int batch, int split, int row, int col, float4 v) -- four
// consecutive columns col..col+3 of output row `row` (indices local to the batch).
// grid = (tiles_m * tiles_n, batches, splits).  With splits > 1 split z contracts k tiles
// [z * ktiles, (z+1) * ktiles) of source 0.  Source::ktiles counts 64-deep tiles.
//
// EXACT_TAIL = false keeps the loop free of branches: loads past the last tile re-fetch it, so
// one fixed vmcnt bound serves every iteration (NS - 1 redundant tile loads per workgroup:
// nothing next to a long contraction).  With EXACT_TAIL the kernel stops issuing after the last
// tile and shrinks the bound instead -- for short contractions, where redundant loads and the
// latency of the first tiles are a visible share of the work.
template <int BM, int BN, int WGM, int WGN, bool A_KMAJOR, bool B_KMAJOR, bool GATHER, int NS, bool EXACT_TAIL, class Epi>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_kernel(Args g, Epi epi) {
  using C = Cfg<BM, BN, WGM, WGN, NS>;
  constexpr int NSTAGE = NS;
  constexpr int TM = BM / WGM / 32, TN = BN / WGN / 32;
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  // Workgroups go to the 8 XCDs round robin: give each XCD a contiguous chunk of
  // the tile list (its own L2 then serves neighbouring tiles), walked in groups
  // of 4 tile rows.
  int wg = blockIdx.x;
  const int total = g.tiles_m * g.tiles_n;
  int batch = blockIdx.y, split = blockIdx.z;
  if (g.xcd_batches > 0) {
    const int slot = blockIdx.x >> 3, work = (slot / total) * 8 + (blockIdx.x & 7);
    wg = slot % total;
    batch = work % g.xcd_batches;
    split = work / g.xcd_batches;
  } else if ((total & 7) == 0) wg = (wg & 7) * (total >> 3) + (wg >> 3);
  constexpr int GROUP = 4;
  const int per_group = GROUP * g.tiles_n;
  const int first_m = (wg / per_group) * GROUP;
  const int gsz = (g.tiles_m - first_m) < GROUP ? (g.tiles_m - first_m) : GROUP;
  const int tile_m = first_m + (wg % per_group) % gsz;
  const int tile_n = (wg % per_group) / gsz;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const int i0 = tile_m * BM, j0 = tile_n * BN;

  // ---- global element offsets of this lane's chunk for each direct-to-LDS instruction.
  // Instruction (wave, s) fills LDS slots [(wave*IPW + s)*64, +64) of the operand tile; the
  // lane's slot decides, through the inverse swizzle, which global chunk it fetches.
  i64 offA[C::IPW_A], offB[C::IPW_B];
  {
    const int32_t* pm = GATHER ? g.perm + (i64)batch * g.rows_per_batch : nullptr;
#pragma unroll
    for (int s = 0; s < C::IPW_A; ++s) {
      const int slot = (wave * C::IPW_A + s) * 64 + lane;
      if (A_KMAJOR) {
        const int r = slot >> 2, c = xk_chunk(slot & 3, r);
        const i64 row = GATHER ? (i64)pm[i0 + r] : (i64)(i0 + r);
        offA[s] = row * g.s[0].lda + c * 8;
      } else {
        constexpr int CPR = BM / 8;
        const int k = slot / CPR, c = kx_unchunk<BM>(slot % CPR, k);
        offA[s] = (i64)k * g.s[0].lda + i0 + c * 8;
      }
    }
#pragma unroll
    for (int s = 0; s < C::IPW_B; ++s) {
      const int slot = (wave * C::IPW_B + s) * 64 + lane;
      if (B_KMAJOR) {
        const int r = slot >> 2, c = xk_chunk(slot & 3, r);
        const i64 row = GATHER ? (i64)pm[j0 + r] : (i64)(j0 + r);
        offB[s] = row * g.s[0].ldb + c * 8;
      } else {
        constexpr int CPR = BN / 8;
        const int k = slot / CPR, c = kx_unchunk<BN>(slot % CPR, k);
        offB[s] = (i64)k * g.s[0].ldb + j0 + c * 8;
      }
    }
  }

  const bool use_alt = g.alt_from > 0 && batch >= g.alt_from;
  const Source* S = use_alt ? g.alt : g.s;
  const int nsrc = use_alt ? g.alt_nsrc : g.nsrc;
  const int bidx = use_alt ? batch - g.alt_from : batch;
  const int kt0 = S[0].ktiles * 2;  // in BK = 32 tiles
  const int KT = kt0 + (nsrc > 1 ? S[1].ktiles * 2 : 0);
  const int kbase = split * kt0;

  // LDS byte address of the ring (wave uniform) for the direct-to-LDS loads
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;

  auto issue_at = [&](int t, int ring_slot) {
    const bool second = t >= kt0;
    const Source& src = S[second ? 1 : 0];
    const i64 kt = second ? (t - kt0) : (kbase + t);
    const uint16_t* Ab = src.A + (GATHER ? 0 : bidx * src.sA) + (A_KMAJOR ? kt * BK : kt * BK * src.lda);
    const uint16_t* Bb = src.B + (GATHER ? 0 : bidx * src.sB) + (B_KMAJOR ? kt * BK : kt * BK * src.ldb);
    const uint32_t stage = lds_base + ring_slot * C::STAGE_BYTES;
#pragma unroll
    for (int s = 0; s < C::IPW_A; ++s) dma16(Ab + offA[s], stage + (wave * C::IPW_A + s) * 1024);
#pragma unroll
    for (int s = 0; s < C::IPW_B; ++s) dma16(Bb + offB[s], stage + C::A_BYTES + (wave * C::IPW_B + s) * 1024);
  };

  // ---- LDS byte offsets of this lane's fragments inside a stage (k step 0)
  int fragA[TM], fragB[TN];
  {
    const int q = lane >> 4, i = lane & 15;
#pragma unroll
    for (int a = 0; a < TM; ++a) {
      const int x0 = wm * (BM / WGM) + a * 32;
      if (A_KMAJOR) {
        const int r = x0 + (lane & 31);
        fragA[a] = r * 64 + 16 * xk_chunk(lane >> 5, r);
      } else {
        const int k = 8 * (q >> 1) + (i >> 2);
        const int c = (x0 >> 3) + 2 * (q & 1) + ((i & 3) >> 1);
        fragA[a] = k * (BM * 2) + 16 * kx_chunk<BM>(c, k) + 8 * (i & 1);
      }
    }
#pragma unroll
    for (int c2 = 0; c2 < TN; ++c2) {
      const int x0 = wn * (BN / WGN) + c2 * 32;
      if (B_KMAJOR) {
        const int r = x0 + (lane & 31);
        fragB[c2] = C::A_BYTES + r * 64 + 16 * xk_chunk(lane >> 5, r);
      } else {
        const int k = 8 * (q >> 1) + (i >> 2);
        const int c = (x0 >> 3) + 2 * (q & 1) + ((i & 3) >> 1);
        fragB[c2] = C::A_BYTES + k * (BN * 2) + 16 * kx_chunk<BN>(c, k) + 8 * (i & 1);
      }
    }
  }

  floatx16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int c = 0; c < TN; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][c][v] = 0.f;

  auto load_frag = [&](const char* stage, int off, bool kmajor, int row_bytes, int ks) -> bf16x8 {
    if (kmajor) {
      // k step 1 is logical chunk + 2: flips bit 1 of the swizzled position
      return *reinterpret_cast<const bf16x8*>(stage + (ks ? (off ^ 32) : off));
    }
    const char* p = stage + off + ks * 16 * row_bytes;
    short4v lo = lds_read_tr(p);
    short4v hi = lds_read_tr(p + 4 * row_bytes);
    short8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };
  struct Frags {
    bf16x8 a[TM], b[TN];
  };
  auto load_frags = [&](Frags& f, int t, int ks) {
    const char* stage = lds + (t % NSTAGE) * C::STAGE_BYTES;
#pragma unroll
    for (int a = 0; a < TM; ++a) f.a[a] = load_frag(stage, fragA[a], A_KMAJOR, BM * 2, ks);
#pragma unroll
    for (int c = 0; c < TN; ++c) f.b[c] = load_frag(stage, fragB[c], B_KMAJOR, BN * 2, ks);
  };
  auto mfma_all = [&](const Frags& f) {
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int c = 0; c < TN; ++c)
        acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[c], f.a[a], acc[a][c], 0, 0, 0);
  };

  // Ask the scheduler to alternate one MFMA with one LDS read (0x008 = MFMA, 0x100 = DS read)
  // so the fragment reads of the next k step trickle in under the current MFMAs.
  auto interleave_hint = [&]() {
#pragma unroll
    for (int i = 0; i < TM * TN; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
  };

  // Ring schedule.  All NS stages are in use: while tile kt is multiplied, tiles kt+1 ..
  // kt+NS-1 are in flight or landed.  The one barrier per tile sits in the middle of the
  // iteration: by then every wave holds all of tile kt in registers (its k step 0 fragments
  // were prefetched during tile kt-1, its k step 1 fragments are waited for here), so the
  // stage of tile kt is refilled at once with tile kt+NS, and tile kt+1 -- whose arrival the
  // same wait checks -- can be prefetched under the second half of the MFMAs.
  constexpr int LPT = C::IPW_A + C::IPW_B;  // direct-to-LDS loads per tile per wave
  static_assert(NSTAGE * LPT < 64, "vmcnt range");
  // !EXACT_TAIL: loads past the last tile re-fetch the last tile into a free stage, which keeps
  // the number of outstanding loads constant (no branches, one fixed vmcnt bound).
  auto issue_clamped = [&](int t) {
    if (EXACT_TAIL) {
      if (t < KT) issue_at(t, t % NSTAGE);
    } else {
      issue_at(t < KT ? t : KT - 1, t % NSTAGE);
    }
  };
  // with `issued` tiles issued so far, the number of tiles younger than tile `need`
  auto younger_than = [&](int issued, int need) { return (issued < KT ? issued : KT) - 1 - need; };
#pragma unroll
  for (int t = 0; t < NSTAGE; ++t) issue_clamped(t);
  if (EXACT_TAIL) wait_tiles_and_barrier<LPT, NSTAGE - 1>(younger_than(NSTAGE, 0));
  else wait_vmcnt_and_barrier<(NSTAGE - 1) * LPT>();
  Frags F, G;
  load_frags(F, 0, 0);
  for (int kt = 0; kt < KT; ++kt) {
    load_frags(G, kt, 1);
    mfma_all(F);
    interleave_hint();
    // tile kt+1 has landed and tile kt is in registers, for every wave
    if (EXACT_TAIL) wait_tiles_and_barrier<LPT, NSTAGE - 2>(younger_than(kt + NSTAGE, kt + 1));
    else wait_all_reads_and_barrier<(NSTAGE - 2) * LPT>();
    issue_clamped(kt + NSTAGE);                     // into the stage of tile kt
    load_frags(F, kt + 1, 0);                       // stale but harmless after the last tile
    mfma_all(G);
    interleave_hint();
  }
  wait_vmcnt_and_barrier<0>();

  const int h = lane >> 5, li = lane & 31;
  if constexpr (has_wide<Epi>::value) {
    // An epilogue that takes 8 consecutive columns: register groups q and q + 1 are swapped between the
    // lane halves (v_permlane32_swap: the upper half of its first operand against the lower half of its
    // second), after which the lower lanes hold columns 8q .. 8q + 7 and the upper lanes 8(q+1) .. + 7.
    typedef unsigned uint2v __attribute__((ext_vector_type(2)));
#pragma unroll
    for (int a = 0; a < TM; ++a) {
      const int row = i0 + wm * (BM / WGM) + a * 32 + li;
#pragma unroll
      for (int c = 0; c < TN; ++c) {
        const int col = j0 + wn * (BN / WGN) + c * 32 + 8 * h;
#pragma unroll
        for (int q = 0; q < 4; q += 2) {
          float lo[4], hi[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float x = acc[a][c][4 * q + e], y = acc[a][c][4 * q + 4 + e];   // scalars first: a bit cast straight from a vector element reads element 0
            const uint2v r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, y), false, false);
            const unsigned r0 = r[0], r1 = r[1];
            lo[e] = __builtin_bit_cast(float, r0);
            hi[e] = __builtin_bit_cast(float, r1);
          }
          epi.wide(batch, split, row, col + 8 * q, make_float4(lo[0], lo[1], lo[2], lo[3]), make_float4(hi[0], hi[1], hi[2], hi[3]));
        }
      }
    }
  } else {
#pragma unroll
    for (int a = 0; a < TM; ++a) {
      const int row = i0 + wm * (BM / WGM) + a * 32 + li;
#pragma unroll
      for (int c = 0; c < TN; ++c) {
        const int col = j0 + wn * (BN / WGN) + c * 32 + 4 * h;
#pragma unroll
        for (int q = 0; q < 4; ++q)
          epi(batch, split, row, col + 8 * q,
              make_float4(acc[a][c][4 * q], acc[a][c][4 * q + 1], acc[a][c][4 * q + 2], acc[a][c][4 * q + 3]));
      }
    }
  }
}

template <int BM, int BN, int WGM, int WGN, bool A_KMAJOR, bool B_KMAJOR, bool GATHER, int NS = 4, bool EXACT_TAIL = (NS > 4),
          class Epi>
void launch(const Args& g, Epi epi, int batches, int splits, hipStream_t st) {
  using C = Cfg<BM, BN, WGM, WGN, NS>;
  auto kern = gemm_bf16_kernel<BM, BN, WGM, WGN, A_KMAJOR, B_KMAJOR, GATHER, NS, EXACT_TAIL, Epi>;
  // once per kernel instance; a function-local static is initialised exactly once, whichever thread gets there first
  static const bool configured =
      hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES) == hipSuccess;
  (void)configured;
  // a few tiles per (batch, split) that read the same operand rows: keep them on one XCD
  const int tiles = g.tiles_m * g.tiles_n;
  if (tiles > 1 && tiles <= 16 && ((i64)batches * splits) % 8 == 0) {
    Args h = g;
    h.xcd_batches = batches;
    hipLaunchKernelGGL(kern, dim3(tiles * batches * splits), dim3(64 * WGM * WGN), C::LDS_BYTES, st, h, epi);
    return;
  }
  hipLaunchKernelGGL(kern, dim3(g.tiles_m * g.tiles_n, batches, splits), dim3(64 * WGM * WGN), C::LDS_BYTES, st, g, epi);
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
