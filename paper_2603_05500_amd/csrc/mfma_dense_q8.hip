// Dense bf16 products on an INT8 base weight (Sec. 3.6, POET-XQ): the weight is dequantised on the
// fly inside the product, no high-precision copy of it is ever written to memory.
//   forward : B  (n x N) = W   A,   backward: dA (m x N) = W^T dB,   W[i][k] = scale[i] * q[i][k].
//
// Same persistent stream as the bf16 product (mfma_dense.hip: one wave per SIMD, 128 x 128 wave
// tiles, 32-deep stages through an LDS ring, one barrier per stage); only the weight operand takes
// another road into its ring slot.  Its 8-bit codes (8 KB per stage) and the scales the stage needs
// arrive by direct-to-LDS loads in a small side ring; two stages ahead of the multiplication each
// wave converts exactly the bytes it loaded itself -- so its own vmcnt wait is all the
// synchronisation the side ring needs -- into bf16(scale * q) and writes them into the weight half
// of the stage's slot, in the layout the bf16 kernel uses.  The conversion (one cvt + one fma per
// element, rounded once to fp32 and once to bf16, i.e. bit for bit the stand-alone dequantiser)
// runs in the shadow of the MFMAs.
#include <type_traits>

#include "mfma_gemm.h"

namespace poetx {
namespace {

using mm::bf16x8;
using mm::floatx16;
using mm::short4v;
using mm::short8v;

constexpr int BM = 256, BN = 256, BK = 32, NW = 4, NS = 4, NQ = 3;
constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
constexpr int Q_CODES = BM * BK;                 // 8 KB of codes per stage
constexpr int Q_SLOT = Q_CODES + 1024;           // + 256 floats of scales
constexpr int Q_BASE = NS * STAGE_BYTES;         // side ring behind the main ring
constexpr int LDS_BYTES = Q_BASE + NQ * Q_SLOT;  // 155648
constexpr int IPW = B_BYTES / 1024 / NW;         // 4 direct-to-LDS instructions per wave per stage for the activations
constexpr int QLOADS = 3;                        // per wave per stage: 2 x 16 bytes of codes per lane + 1 x 4 bytes of scale
constexpr int TM = 4, TN = 4, GROUP = 4;
// At the barrier of stage kt the wave's own codes of stage kt+2 and everybody's activations of
// stage kt+1 must have landed.  Issue order: ... B(kt+1), Q(kt+2), B(kt+2), Q(kt+3), B(kt+3), barrier:
// the loads younger than Q(kt+2) are two activation stages and one code stage.
constexpr int VM_BOUND = 2 * IPW + QLOADS;
static_assert(NS * IPW + NQ * QLOADS < 64, "vmcnt range");

struct DenseQ8Args {
  const int8_t* Q;       // codes, n x m row major
  const float* scale;    // n
  const uint16_t* B;     // activations, K x N row major
  uint16_t* C;           // M x N row major
  i64 ldq, ldb, ldc;
  int tiles_m, tiles_n, ktiles;
};

// Direct-to-LDS loads as in the bf16 kernel: the instruction offset moves the LDS and the global
// address alike, so a group of loads shares one M0 and the per-lane offsets carry the bias.
template <int OFF>
__device__ inline void dma16g(const void* sbase, uint32_t voff, uint32_t lds_group) {
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(voff), "s"(sbase), "n"(OFF), "{m0}"(lds_group) : "memory");
}
__device__ inline void dma16g_s(int s, const void* sbase, uint32_t voff, uint32_t lds_group) {
  switch (s) {
    case 0: dma16g<0>(sbase, voff, lds_group); break;
    case 1: dma16g<1024>(sbase, voff, lds_group); break;
    case 2: dma16g<2048>(sbase, voff, lds_group); break;
    default: dma16g<3072>(sbase, voff, lds_group); break;
  }
}
__device__ inline void dma4s(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("global_load_lds_dword %0, %1" ::"v"(voff), "s"(sbase), "{m0}"(lds_addr) : "memory");
}

// A_KMAJOR: forward (weight rows are output rows, contraction along a row).  Otherwise backward
// (weight rows are the contraction index).
template <bool A_KMAJOR>
__global__ __launch_bounds__(256) void dense_q8_stream_kernel(DenseQ8Args g) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

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
  const int KT = g.ktiles;
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;

  // ---- activations: as in the bf16 kernel
  uint32_t voffB[IPW];
#pragma unroll
  for (int s = 0; s < IPW; ++s) {
    const int slot = (wave * IPW + s) * 64 + lane;
    const int k = slot / (BN / 8), c = mm::kx_unchunk<BN>(slot % (BN / 8), k);
    voffB[s] = (uint32_t)((k * g.ldb + c * 8) * 2) - s * 1024;   // less the instruction offset of load s
  }
  const i64 stepB = (i64)BK * g.ldb * 2;
  const char* Bb;
  int b_tile = 0, b_kt = 0, b_slot = 0;
  auto b_base = [&](int ti) {
    int i0, j0;
    tile_origin(ti, i0, j0);
    Bb = (const char*)(g.B + j0);
  };
  b_base(0);
  auto issue_b = [&](int s) { dma16g_s(s, Bb, voffB[s], lds_base + b_slot * STAGE_BYTES + A_BYTES + wave * IPW * 1024); };
  auto b_advance = [&]() {
    b_slot = b_slot + 1 == NS ? 0 : b_slot + 1;
    if (b_kt + 1 < KT) { ++b_kt; Bb += stepB; }
    else if (b_tile + 1 < n_my) { ++b_tile; b_kt = 0; b_base(b_tile); }
  };

  // ---- codes and scales.  Code instruction j of wave w fills 16-byte chunks [(2w+j)*64, +64) of the
  // side-ring slot; lane l owns chunk ch = (2w+j)*64 + l and converts it itself later.
  //   forward : the stage's codes are [256 rows][32 bytes]: row = ch >> 1, bytes 16 (ch & 1) ..
  //   backward: [32 k rows][256 bytes]: row = ch >> 4, bytes 16 (ch & 15) ..
  // The scale instruction of wave w fills floats [64w, 64w + 64) of the slot's scale area with the
  // scales of the rows its chunks belong to (forward: rows 64w + l; backward: k rows 8w + (l & 7)).
  uint32_t voffQ[2], voffS;
  int cvt_dst[2][2];     // byte offsets (inside the weight half of a stage) of the two bf16 chunks a code chunk becomes
  int cvt_scale[2];      // byte offset of the chunk's scale inside the slot
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int ch = (wave * 2 + j) * 64 + lane;
    if (A_KMAJOR) {
      const int r = ch >> 1, c = ch & 1;
      voffQ[j] = (uint32_t)(r * g.ldq + 16 * c) - j * 1024;
      cvt_dst[j][0] = r * 64 + 16 * mm::xk_chunk(2 * c, r);
      cvt_dst[j][1] = r * 64 + 16 * mm::xk_chunk(2 * c + 1, r);
      cvt_scale[j] = Q_CODES + 4 * r;
    } else {
      const int k = ch >> 4, c = ch & 15;
      voffQ[j] = (uint32_t)(k * g.ldq + 16 * c) - j * 1024;
      cvt_dst[j][0] = k * (BM * 2) + 16 * mm::kx_chunk<BM>(2 * c, k);
      cvt_dst[j][1] = k * (BM * 2) + 16 * mm::kx_chunk<BM>(2 * c + 1, k);
      cvt_scale[j] = Q_CODES + 4 * (64 * wave + (k - 8 * wave));
    }
  }
  voffS = A_KMAJOR ? (uint32_t)(4 * (64 * wave + lane)) : (uint32_t)(4 * (8 * wave + (lane & 7)));
  const i64 stepQ = A_KMAJOR ? (i64)BK : (i64)BK * g.ldq;          // bytes per stage along the contraction
  const char* Qb;
  const char* Sb;
  int q_tile = 0, q_kt = 0, q_slot = 0;
  auto q_base = [&](int ti) {
    int i0, j0;
    tile_origin(ti, i0, j0);
    Qb = (const char*)g.Q + (A_KMAJOR ? (i64)i0 * g.ldq : (i64)i0);
    Sb = (const char*)(g.scale + (A_KMAJOR ? i0 : 0));
  };
  q_base(0);
  auto issue_q = [&]() {
    const uint32_t slot = lds_base + Q_BASE + q_slot * Q_SLOT;
    dma16g<0>(Qb, voffQ[0], slot + wave * 2 * 1024);
    dma16g<1024>(Qb, voffQ[1], slot + wave * 2 * 1024);
    dma4s(Sb, voffS, slot + Q_CODES + wave * 256);
    q_slot = q_slot + 1 == NQ ? 0 : q_slot + 1;
    if (q_kt + 1 < KT) {
      ++q_kt;
      Qb += stepQ;
      if (!A_KMAJOR) Sb += BK * 4;
    } else if (q_tile + 1 < n_my) {
      ++q_tile;
      q_kt = 0;
      q_base(q_tile);
    }
  };
  // conversion side: which side-ring slot and which main-ring slot come next
  int c_qslot = 0, c_slot = 0;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  struct Codes {
    u32x4 q[2];
    float s[2];
  };
  auto cvt_read = [&](Codes& c) {
    const char* slot = lds + Q_BASE + c_qslot * Q_SLOT;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      c.q[j] = *reinterpret_cast<const u32x4*>(slot + (wave * 2 + j) * 1024 + lane * 16);
      c.s[j] = *reinterpret_cast<const float*>(slot + cvt_scale[j]);
    }
    c_qslot = c_qslot + 1 == NQ ? 0 : c_qslot + 1;
  };
  // Conversion of chunk j in eight steps of two codes each (about six vector instructions: few enough
  // to sit between two MFMAs without delaying the second); after steps 3 and 7 one 16-byte chunk of
  // bf16 goes into the weight half of main-ring slot c_slot.
  uint32_t cvo[8];
  auto cvt_step = [&](const Codes& c, int j, int hw) {
    char* stage = lds + c_slot * STAGE_BYTES;
    const float s = c.s[j], off = -128.f * s;
    const uint32_t u = c.q[j][hw >> 1] ^ 0x80808080u;      // signed code + 128 as an unsigned byte
    const uint32_t b0 = (hw & 1) ? ((u >> 16) & 0xffu) : (u & 0xffu);
    const uint32_t b1 = (hw & 1) ? (u >> 24) : ((u >> 8) & 0xffu);
    // (u - 128) * s, rounded once: the fma adds the exact products u*s and -128*s
    cvo[hw] = mm::pack2_bf16(__builtin_fmaf((float)b0, s, off), __builtin_fmaf((float)b1, s, off));
    if (hw == 3) *reinterpret_cast<u32x4*>(stage + cvt_dst[j][0]) = u32x4{cvo[0], cvo[1], cvo[2], cvo[3]};
    if (hw == 7) *reinterpret_cast<u32x4*>(stage + cvt_dst[j][1]) = u32x4{cvo[4], cvo[5], cvo[6], cvo[7]};
  };
  auto cvt_write = [&](const Codes& c, int j) {
#pragma unroll
    for (int hw = 0; hw < 8; ++hw) cvt_step(c, j, hw);
  };
  auto cvt_done = [&]() { c_slot = c_slot + 1 == NS ? 0 : c_slot + 1; };

  // ---- fragments
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
  auto mfma_one = [&](const Frags& f, int i) {
    const int c = i >> 2, a = i & 3;
    acc[a][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[c], f.a[a], acc[a][c], 0, 0, 0);
  };

  // ---- prologue: codes of stages 0..2, activations of stages 0..2; stage 0 and half of stage 1
  // converted (the loop's first k step finishes stage 1, as every k step finishes the stage the
  // previous one began); then the codes of stage 3 into the slot stage 0 has left
  Codes cd;
  issue_q();
  issue_q();
  issue_q();
#pragma unroll
  for (int t = 0; t < NS - 1; ++t) {
#pragma unroll
    for (int s = 0; s < IPW; ++s) issue_b(s);
    b_advance();
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  cvt_read(cd);            // stage 0, whole
  cvt_write(cd, 0);
  cvt_write(cd, 1);
  cvt_done();
  cvt_read(cd);            // stage 1: first chunk here, second chunk in the first k step of the loop
  cvt_write(cd, 0);
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // conversion reads done before the slot is refilled
  issue_q();
  mm::wait_all_reads_and_barrier<QLOADS>();           // everybody's stage 0 is in place
  Frags F, Gf;
  int cslot = 0;
#pragma unroll
  for (int p = 0; p < 8; ++p) load_piece(F, lds, 0, p);

  const int h = lane >> 5, li = lane & 31;
  const i64 coff = (i64)(wm * (BM / 2) + li) * g.ldc + wn * (BN / 2) + 8 * h;

  auto run = [&](auto WC) {
    constexpr int W = decltype(WC)::value;
    for (int ti = 0; ti < n_my; ++ti) {
      for (int kt = 0; kt < KT; ++kt) {
        const char* stage = lds + cslot * STAGE_BYTES;
        // k step 0 from F; fetch k step 1; activations of stage kt + NS - 1 into the slot the last
        // barrier released; second half of the conversion that the previous k step began
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          mfma_one(F, i);
          if (i < 8) load_piece(Gf, stage, 1, i);
          if ((i & 3) == W) issue_b(i >> 2);
          if (i >= 8) cvt_step(cd, 1, i - 8);          // second chunk of the codes read after the last barrier
          if (i == 15) { cvt_done(); b_advance(); }
          __builtin_amdgcn_sched_barrier(0);
        }
        // every wave holds the rest of this stage in registers; the activations of the next stage and
        // this wave's codes of the stage after it have landed; the next stage's weights are converted
        mm::wait_all_reads_and_barrier<VM_BOUND>();
        const int nslot = cslot + 1 == NS ? 0 : cslot + 1;
        const char* nstage = lds + nslot * STAGE_BYTES;
        // k step 1 from Gf; fetch k step 0 of the next stage; read this wave's codes of stage kt + 2,
        // convert their first half, refill the side-ring slot that stage kt + 1 has left
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          mfma_one(Gf, i);
          if (i < 8) load_piece(F, nstage, 0, i);
          if (i == 0) cvt_read(cd);
          if (i >= 8) cvt_step(cd, 0, i - 8);          // first chunk, into the slot of stage kt + 2
          if (i == 15) issue_q();
          __builtin_amdgcn_sched_barrier(0);
        }
        cslot = nslot;
      }
      int i0, j0;
      tile_origin(ti, i0, j0);
      uint16_t* Ct = g.C + (i64)i0 * g.ldc + j0 + coff;
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int c = 0; c < TN; ++c) {
          uint32_t p[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) p[e] = mm::pack2_bf16(acc[a][c][2 * e], acc[a][c][2 * e + 1]);
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[a][c][v] = 0.f;
#pragma unroll
          for (int q = 0; q < 4; q += 2) {
            typedef unsigned uint2v __attribute__((ext_vector_type(2)));
            const uint2v r0 = __builtin_amdgcn_permlane32_swap(p[2 * q], p[2 * q + 2], false, false);
            const uint2v r1 = __builtin_amdgcn_permlane32_swap(p[2 * q + 1], p[2 * q + 3], false, false);
            const u32x4 o = {r0[0], r1[0], r0[1], r1[1]};
            *reinterpret_cast<u32x4*>(Ct + (i64)a * 32 * g.ldc + c * 32 + 8 * q) = o;
          }
        }
    }
  };
  switch (wave) {
    case 0: run(std::integral_constant<int, 0>{}); break;
    case 1: run(std::integral_constant<int, 1>{}); break;
    case 2: run(std::integral_constant<int, 2>{}); break;
    default: run(std::integral_constant<int, 3>{}); break;
  }
  mm::wait_vmcnt_and_barrier<0>();
}

int compute_units_q8() {
  static const int n = [] {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0)
      cu = 256;
    return cu;
  }();
  return n;
}

template <bool A_KMAJOR>
void launch_dense_q8(const DenseQ8Args& g, hipStream_t st) {
  auto kern = dense_q8_stream_kernel<A_KMAJOR>;
  static const bool configured =
      hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) == hipSuccess;
  (void)configured;
  const int T = g.tiles_m * g.tiles_n, cus = compute_units_q8();
  hipLaunchKernelGGL(kern, dim3(T < cus ? T : cus), dim3(256), LDS_BYTES, st, g);
}

}  // namespace

bool mfma_dense_q8_supported(int n, int m, i64 N) {
  // a stream of at least 3 stages per workgroup keeps the prologue simple; 32-bit lane offsets
  return mfma_dense_supported(n, m, N) && n >= 3 * BK && m >= 3 * BK;
}

void mfma_dense_q8(int trans_w, const void* Wq, int n, int m, const void* act, void* out, i64 N, hipStream_t st) {
  DenseQ8Args g{};
  g.Q = (const int8_t*)Wq;
  g.scale = (const float*)((const char*)Wq + weight_q8_scale_offset(n, m));
  g.B = (const uint16_t*)act;
  g.C = (uint16_t*)out;
  g.ldq = m;
  g.ldb = N;
  g.ldc = N;
  g.tiles_n = (int)(N / BN);
  if (!trans_w) {
    g.tiles_m = n / BM;
    g.ktiles = m / BK;
    launch_dense_q8<true>(g, st);
  } else {
    g.tiles_m = m / BM;
    g.ktiles = n / BK;
    launch_dense_q8<false>(g, st);
  }
}

}  // namespace poetx
