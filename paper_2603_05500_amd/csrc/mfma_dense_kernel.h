// Dense bf16 products of the POET-X linear layer on the matrix cores:
//   forward  (Eq. 10, mm2):       B  (n x N) = W   (n x m) * A  (m x N)
//   backward (Sec. 3.5, mm2 bwd): dA (m x N) = W^T (m x n) * dB (n x N)   -- no weight gradient
// W is row major n x m; activations are feature major (token index contiguous), so the
// activation operand (and W in the backward product) is contracted over its strided index and
// is read from LDS with the transposing load.
//
// The kernel is a persistent stream: one workgroup per CU, 4 waves (2 x 2, one per SIMD), each
// wave owning a 128 x 128 piece of a 256 x 256 output tile in 256 accumulator registers
// (v_mfma_f32_32x32x16_bf16, fp32).  A workgroup walks its list of output tiles; the 32-deep
// operand stages of ALL its tiles form one stream that flows through a ring of 4 LDS stages
// (a fifth buys nothing measurable; its 32 KB stage the output instead),
// filled by direct-to-LDS loads issued that many stages ahead of the multiplication -- across tile
// boundaries, so a new tile starts multiplying the moment the previous one is rounded and stored.
// Per stage there is one barrier, placed after the first of the two k steps, where every wave
// holds the rest of the stage in registers: the stage's slot is refilled at once.  Loads and
// fragment reads are pinned to fixed places between the MFMAs (each wave spreads its loads
// over different places), and the load addresses are a uniform base plus a per-lane offset that
// never changes, so the loop carries no vector address arithmetic.
#pragma once
#include <type_traits>

#include "mfma_gemm.h"

namespace poetx {
namespace dense {


using mm::bf16x8;
using mm::floatx16;
using mm::short4v;
using mm::short8v;

constexpr int BM = 256, BN = 256, BK = 32, NW = 4, NS = 4;
constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
constexpr int OUT_BYTES = 8192;                  // per-wave output staging: two 32-row x 64-column pieces
constexpr int LDS_BYTES = NS * STAGE_BYTES + NW * OUT_BYTES;   // 128 + 32 = 160 KB: the whole LDS of a CU
constexpr int IPW = A_BYTES / 1024 / NW;         // direct-to-LDS instructions per wave per operand per stage
constexpr int LPT = 2 * IPW;                     // loads per stage per wave
constexpr int TM = 4, TN = 4;                    // 32 x 32 MFMA tiles of a wave
constexpr int GROUP = 4;                         // tile rows walked together
static_assert(NS * LPT < 64, "vmcnt range");
static_assert(IPW == 4, "dma16g_s covers groups of four loads");

struct DenseArgs {
  const uint16_t* A;     // A_KMAJOR: M x K row major (lda = K stride); else K x M
  const uint16_t* B;     // K x N row major
  uint16_t* C;           // M x N row major
  i64 lda, ldb, ldc;
  int tiles_m, tiles_n, ktiles;   // ktiles counts 32-deep stages
};

// 16 bytes per lane from (uniform base + per-lane byte offset + OFF) straight into LDS at
// lds_group + OFF + 16 * lane: the instruction offset moves the LDS address and the global address
// alike, so the per-lane offsets of a group of loads are biased by -OFF and the whole group shares
// one value of M0 (written once by the compiler, which tracks it as an operand).  Completion is
// tracked by hand through vmcnt.
template <int OFF>
__device__ inline void dma16g(const void* sbase, uint32_t voff, uint32_t lds_group) {
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(voff), "s"(sbase), "n"(OFF), "{m0}"(lds_group) : "memory");
}
// load s of a wave's group of IPW = 4 (s is a constant wherever this is called)
__device__ inline void dma16g_s(int s, const void* sbase, uint32_t voff, uint32_t lds_group) {
  switch (s) {
    case 0: dma16g<0>(sbase, voff, lds_group); break;
    case 1: dma16g<1024>(sbase, voff, lds_group); break;
    case 2: dma16g<2048>(sbase, voff, lds_group); break;
    default: dma16g<3072>(sbase, voff, lds_group); break;
  }
}

// DIAG bit 3: counts of this workgroup's second tile, per wave: [0] core cycles of its main loop, [1] of its
// output, [2] the main loop again in ticks of the constant 100 MHz counter (cycles / ticks = the clock the
// CU ran at); [3] ticks from the wave's start to its end.
static __device__ long long g_diag_cycles[4][4 * 256];

// DIAG (measurement builds only; the library instantiates DIAG = 0): bit 0 stops the direct-to-LDS loads
// after the prologue, bit 1 stops the fragment reads inside the loop, bit 2 keeps the load addresses on
// the first stage of the first tile (all loads hit in cache) -- the results are then wrong,
// bit 3 (harmless to the result) records the cycle counts above --
// every address stays what it was, and the timing shows what the loads or the reads cost.
template <bool A_KMAJOR, int DIAG = 0>
__global__ __launch_bounds__(256) void dense_stream_kernel(DenseArgs g) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  long long t_start = 0;
  if (DIAG & 8) t_start = __builtin_amdgcn_s_memrealtime();

  // ---- this workgroup's tiles.  Workgroups go to the 8 XCDs round robin; in every step of
  // gridDim.x tiles each XCD takes a contiguous run of the tile order (GROUP tile rows walked
  // together), so the tiles an XCD works on at a time share operand panels in its L2.
  const int T = g.tiles_m * g.tiles_n;
  const int G = gridDim.x;
  int wq = blockIdx.x;
  if ((G & 7) == 0) wq = (wq & 7) * (G >> 3) + (wq >> 3);
  const int n_my = wq < T ? (T - 1 - wq) / G + 1 : 0;
  if (n_my == 0) return;
  const int per_group = GROUP * g.tiles_n;
  auto tile_origin = [&](int ti, int& i0, int& j0) {
    const int u = ti * G + wq;
    const int first_m = (u / per_group) * GROUP;
    const int gsz = (g.tiles_m - first_m) < GROUP ? (g.tiles_m - first_m) : GROUP;
    i0 = (first_m + (u % per_group) % gsz) * BM;
    j0 = ((u % per_group) / gsz) * BN;
  };

  // per-lane byte offsets of the direct-to-LDS loads (the same for every stage and tile), less the
  // instruction offset s * 1024 of load s (never negative: load s starts 16 s rows, or 2 s rows of at
  // least 256 elements, into the tile).
  // Instruction (wave, s) fills LDS chunk slots [(wave*IPW + s)*64, +64) of the operand's part of
  // a stage; the lane's slot decides, through the inverse swizzle, which global chunk it fetches.
  uint32_t voffA[IPW], voffB[IPW];
#pragma unroll
  for (int s = 0; s < IPW; ++s) {
    const int slot = (wave * IPW + s) * 64 + lane;
    if (A_KMAJOR) {
      const int r = slot >> 2, c = mm::xk_chunk(slot & 3, r);
      voffA[s] = (uint32_t)((r * g.lda + c * 8) * 2) - s * 1024;
    } else {
      const int k = slot / (BM / 8), c = mm::kx_unchunk<BM>(slot % (BM / 8), k);
      voffA[s] = (uint32_t)((k * g.lda + c * 8) * 2) - s * 1024;
    }
    const int k = slot / (BN / 8), c = mm::kx_unchunk<BN>(slot % (BN / 8), k);
    voffB[s] = (uint32_t)((k * g.ldb + c * 8) * 2) - s * 1024;
  }
  const i64 stepA = A_KMAJOR ? (i64)BK * 2 : (i64)BK * g.lda * 2;
  const i64 stepB = (i64)BK * g.ldb * 2;
  const int KT = g.ktiles;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;

  // ---- issue side of the stream: runs NS stages ahead of the multiplication, across tiles
  const char* Ab;
  const char* Bb;
  int itile = 0, ikt = 0, islot = 0;
  auto issue_base = [&](int ti) {
    int i0, j0;
    tile_origin(ti, i0, j0);
    Ab = (const char*)(g.A + (A_KMAJOR ? (i64)i0 * g.lda : (i64)i0));
    Bb = (const char*)(g.B + j0);
  };
  issue_base(0);
  bool loads_on = true;   // DIAG bit 0 switches it off after the prologue
  auto issue_a = [&](int s) { if (!(DIAG & 1) || loads_on) dma16g_s(s, Ab, voffA[s], lds_base + islot * STAGE_BYTES + wave * IPW * 1024); };
  auto issue_b = [&](int s) { if (!(DIAG & 1) || loads_on) dma16g_s(s, Bb, voffB[s], lds_base + islot * STAGE_BYTES + A_BYTES + wave * IPW * 1024); };
  // After the last stage of the last tile the stream keeps re-fetching that stage, so the number
  // of loads in flight -- and with it the vmcnt bound of the barrier -- never changes.
  auto issue_advance = [&]() {
    islot = islot + 1 == NS ? 0 : islot + 1;
    if (DIAG & 4) return;   // every stage re-fetches the first one: the loads stay, their misses go
    if (ikt + 1 < KT) {
      ++ikt;
      Ab += stepA;
      Bb += stepB;
    } else if (itile + 1 < n_my) {
      ++itile;
      ikt = 0;
      issue_base(itile);
    }
  };

  // ---- LDS byte offsets of this lane's fragments inside a stage (k step 0)
  int fragA[TM], fragB[TN];
  {
    const int q = lane >> 4, i = lane & 15;
#pragma unroll
    for (int a = 0; a < TM; ++a) {
      const int x0 = wm * (BM / 2) + a * 32;
      if (A_KMAJOR) {
        const int r = x0 + (lane & 31);
        fragA[a] = r * 64 + 16 * mm::xk_chunk(lane >> 5, r);
      } else {
        const int k = 8 * (q >> 1) + (i >> 2);
        const int c = (x0 >> 3) + 2 * (q & 1) + ((i & 3) >> 1);
        fragA[a] = k * (BM * 2) + 16 * mm::kx_chunk<BM>(c, k) + 8 * (i & 1);
      }
    }
#pragma unroll
    for (int c2 = 0; c2 < TN; ++c2) {
      const int x0 = wn * (BN / 2) + c2 * 32;
      const int k = 8 * (q >> 1) + (i >> 2);
      const int c = (x0 >> 3) + 2 * (q & 1) + ((i & 3) >> 1);
      fragB[c2] = A_BYTES + k * (BN * 2) + 16 * mm::kx_chunk<BN>(c, k) + 8 * (i & 1);
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
    // K major: k step 1 is logical chunk + 2, which flips bit 1 of the swizzled position
    if (kmajor) return *reinterpret_cast<const bf16x8*>(stage + (ks ? (off ^ 32) : off));
    const char* p = stage + off + ks * 16 * row_bytes;
    short4v lo = mm::lds_read_tr(p);
    short4v hi = mm::lds_read_tr(p + 4 * row_bytes);
    short8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };
  struct Frags {
    bf16x8 a[TM], b[TN];
  };
  // piece p of a k step's fragments, in the order the MFMAs first need them: A0 B0 A1 A2 A3 B1 B2 B3
  auto load_piece = [&](Frags& f, const char* stage, int ks, int p) {
    switch (p) {
      case 0: f.a[0] = load_frag(stage, fragA[0], A_KMAJOR, BM * 2, ks); break;
      case 1: f.b[0] = load_frag(stage, fragB[0], false, BN * 2, ks); break;
      case 2: f.a[1] = load_frag(stage, fragA[1], A_KMAJOR, BM * 2, ks); break;
      case 3: f.a[2] = load_frag(stage, fragA[2], A_KMAJOR, BM * 2, ks); break;
      case 4: f.a[3] = load_frag(stage, fragA[3], A_KMAJOR, BM * 2, ks); break;
      case 5: f.b[1] = load_frag(stage, fragB[1], false, BN * 2, ks); break;
      case 6: f.b[2] = load_frag(stage, fragB[2], false, BN * 2, ks); break;
      default: f.b[3] = load_frag(stage, fragB[3], false, BN * 2, ks); break;
    }
  };
  // MFMA i of a k step.  The operands go in swapped, so the accumulator tile is transposed: a lane
  // owns one output row and four consecutive columns per group of four registers.
  auto mfma_one = [&](const Frags& f, int i) {
    const int c = i >> 2, a = i & 3;
    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[c], f.a[a], acc[a][c], 0, 0, 0);
  };

  // ---- prologue: stages 0 .. NS-2 and the A half of stage NS-1
#pragma unroll
  for (int t = 0; t < NS - 1; ++t) {
#pragma unroll
    for (int s = 0; s < IPW; ++s) issue_a(s);
#pragma unroll
    for (int s = 0; s < IPW; ++s) issue_b(s);
    issue_advance();
  }
#pragma unroll
  for (int s = 0; s < IPW; ++s) issue_a(s);
  mm::wait_vmcnt_and_barrier<(NS - 2) * LPT + IPW>();   // stage 0 has landed
  Frags F, Gf;
  int cslot = 0;
#pragma unroll
  for (int p = 0; p < 8; ++p) load_piece(F, lds, 0, p);

  if (DIAG & 2) {   // the loop reads no fragments: both sets come from the first stage
#pragma unroll
    for (int p = 0; p < 8; ++p) load_piece(Gf, lds, 1, p);
  }
  loads_on = false;
  const int h = lane >> 5, li = lane & 31;

  // The body is instantiated once per wave: wave W issues its four loads of a k step after MFMAs
  // W, W+4, W+8 and W+12, so the four waves never hand the memory pipeline a load in the same place.
  auto run = [&](auto WC) {
    constexpr int W = decltype(WC)::value;
    for (int ti = 0; ti < n_my; ++ti) {
      long long tc0 = 0, tc1 = 0, tr0 = 0, tr1 = 0;
      if ((DIAG & 8) && ti == 1) {
        tc0 = __builtin_readcyclecounter();
        tr0 = __builtin_amdgcn_s_memrealtime();
      }
      for (int kt = 0; kt < KT; ++kt) {
        const char* stage = lds + cslot * STAGE_BYTES;
        // k step 0 from F; fetch k step 1 of this stage; B half of the stage in issue (its A half
        // went out during the previous k step, into the slot the last barrier released)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          mfma_one(F, i);
          if (i < 8 && !(DIAG & 2)) load_piece(Gf, stage, 1, i);
          if ((i & 3) == W) issue_b(i >> 2);
          if (i == 15) issue_advance();
          __builtin_amdgcn_sched_barrier(0);
        }
        // Every wave holds the rest of this stage in registers (lgkmcnt(0)) and the next stage has
        // landed: stages up to kt + NS - 1 are issued, so at most NS - 2 of them may be in flight.
        // Stores of a finished tile share the counter and only make this wait stricter.
        mm::wait_all_reads_and_barrier<(NS - 2) * LPT>();
        const int nslot = cslot + 1 == NS ? 0 : cslot + 1;
        const char* nstage = lds + nslot * STAGE_BYTES;
        // k step 1 from Gf; fetch k step 0 of the next stage (the next tile's first stage after
        // the last one of this tile); A half of the next stage to issue, into the slot just released
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          mfma_one(Gf, i);
          if (i < 8 && !(DIAG & 2)) load_piece(F, nstage, 0, i);
          if ((i & 3) == W) issue_a(i >> 2);
          __builtin_amdgcn_sched_barrier(0);
        }
        cslot = nslot;
      }
      if ((DIAG & 8) && ti == 1) {
        tc1 = __builtin_readcyclecounter();
        tr1 = __builtin_amdgcn_s_memrealtime();
      }
      // ---- tile done: round to bf16 and store, clear the accumulators.  The accumulator layout gives a
      // lane 4 consecutive columns of its row per register group; swapping groups between the lane halves
      // (v_permlane32_swap: the upper half of its first operand against the lower half of its second)
      // makes that 8 columns = 16 bytes.  Stored like this an instruction would write 32 contiguous bytes
      // per row, and all workgroups finish their tiles together: the burst drains twice as fast when
      // every instruction writes whole 128-byte lines.  So the wave passes its piece through LDS, 32 rows
      // x 64 columns at a time (rows XOR-swizzled in 16-byte chunks, conflict free both ways), and reads
      // it back with 8 lanes per row.
      {
        typedef unsigned uint2v __attribute__((ext_vector_type(2)));
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        int i0, j0;
        tile_origin(ti, i0, j0);
        char* stg = lds + NS * STAGE_BYTES + wave * OUT_BYTES;
        const int wsw = (li >> 1) & 7;
        uint16_t* Cw = g.C + (i64)(i0 + wm * (BM / 2)) * g.ldc + j0 + wn * (BN / 2);
#pragma unroll
        for (int a = 0; a < TM; ++a) {
#pragma unroll
          for (int c = 0; c < TN; ++c) {
            uint32_t p[8];   // p[2q], p[2q+1]: columns 8q + 4h + 0..3 of the 32-column tile
#pragma unroll
            for (int e = 0; e < 8; ++e) p[e] = mm::pack2_bf16(acc[a][c][2 * e], acc[a][c][2 * e + 1]);
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][c][v] = 0.f;
#pragma unroll
            for (int q = 0; q < 4; q += 2) {
              const uint2v r0 = __builtin_amdgcn_permlane32_swap(p[2 * q], p[2 * q + 2], false, false);
              const uint2v r1 = __builtin_amdgcn_permlane32_swap(p[2 * q + 1], p[2 * q + 3], false, false);
              const u32x4 o = {r0[0], r1[0], r0[1], r1[1]};   // columns 8 (q + h) .. + 7 of tile c
              const int ch = (c & 1) * 4 + q + h;             // 16-byte chunk of the 64-column piece
              *reinterpret_cast<u32x4*>(stg + (c >> 1) * 4096 + li * 128 + 16 * (ch ^ wsw)) = o;
            }
          }
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's own writes; the area is private to it
#pragma unroll
          for (int cp = 0; cp < 2; ++cp)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int r = (lane >> 3) + 8 * i, ch = lane & 7;
              const u32x4 o = *reinterpret_cast<const u32x4*>(stg + cp * 4096 + r * 128 + 16 * (ch ^ ((r >> 1) & 7)));
              *reinterpret_cast<u32x4*>(Cw + (i64)(a * 32 + r) * g.ldc + cp * 64 + ch * 8) = o;
            }
        }
      }
      if ((DIAG & 8) && ti == 1 && lane == 0 && blockIdx.x < 256) {
        g_diag_cycles[0][blockIdx.x * 4 + W] = tc1 - tc0;
        g_diag_cycles[1][blockIdx.x * 4 + W] = __builtin_readcyclecounter() - tc1;
        g_diag_cycles[2][blockIdx.x * 4 + W] = tr1 - tr0;
      }
    }
  };
  switch (wave) {
    case 0: run(std::integral_constant<int, 0>{}); break;
    case 1: run(std::integral_constant<int, 1>{}); break;
    case 2: run(std::integral_constant<int, 2>{}); break;
    default: run(std::integral_constant<int, 3>{}); break;
  }
  mm::wait_vmcnt_and_barrier<0>();   // the re-fetched stages land before the LDS is released
  if ((DIAG & 8) && lane == 0 && blockIdx.x < 256) g_diag_cycles[3][blockIdx.x * 4 + wave] = __builtin_amdgcn_s_memrealtime() - t_start;
}


}  // namespace dense
}  // namespace poetx
