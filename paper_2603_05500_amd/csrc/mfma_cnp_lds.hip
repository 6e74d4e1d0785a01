// Cayley-Neumann series and its backward for b = 256 with the block resident on chip
// (Sec. 3.4, Eq. 8-9): one launch runs the whole chain of a block.
//
// Every quantity of the series is a polynomial in Q applied from the left to a matrix whose
// column stripes do not mix:
//   forward    H_1 = Q,  H_{s+1} = 2Q + Q H_s,  G = I + H_{k+1}          (Horner, residual form)
//   backward   V_0 = D^T, V_m = Q V_{m-1}       (D = dL/dG)               pass 1
//              W_m = 2 (V_0 + .. + V_m) - V_m,  stored transposed
//              Y_0 = D,   Y_m = W_m^T - Q Y_{m-1},  dL/dQ = Y_k            pass 2
// (the backward is dQ = sum_{a+c<=k} c_{a+c+1} (Q^T)^a D (Q^T)^c regrouped as
// sum_a (-Q)^a W_{k-a}^T; both passes cost k products instead of the 3k-1 of the two-sided
// Horner scheme).  So one kernel serves all three: bf16(Q) (materialised once per call from the
// packed parameters by a small element-wise kernel) sits in LDS as the left operand,
// a wave owns 32 columns of the running matrix and keeps them in registers as matrix-core
// B fragments, multiplies (v_mfma_f32_32x32x16_bf16, fp32 accumulators, 8 row tiles), adds
// the step's fp32 term and rounds the result straight back into B fragments: with the
// contraction index permuted inside each group of 16 (k = 16s + 8a + 4h + j is taken at
// fragment slot 8h + 4a + j) accumulator registers 8u..8u+7 of row tile t ARE fragment
// 2t+u, so the chain never leaves the register file and nothing is transposed.  The same
// permutation is applied to the columns of Q in LDS, which keeps its fragment reads 16 bytes
// wide.  A workgroup is 4 waves = 128 columns; two workgroups share a block.
//
// Precision as in the tiled kernels: products in bf16 with fp32 accumulation, the dominant
// terms (2Q in the final forward step, D in both backward passes) enter in fp32.
#include "mfma_gemm.h"

namespace poetx {
namespace {

using mm::bf16x8;
using mm::floatx16;

constexpr int LB = 256;                  // block side
constexpr int LROW = LB * 2 + 16;        // LDS row stride in bytes: 16 lanes of a 16-byte read hit 16 bank groups
constexpr int CHAIN_LDS = LB * LROW;     // 135168 bytes
constexpr int NT = LB / 32;              // row tiles of a stripe
constexpr int NKS = LB / 16;             // k steps of a product

enum { CHAIN_FWD = 0, CHAIN_BWD1 = 1, CHAIN_BWD2 = 2 };

struct ChainArgs {
  const uint16_t* Qb;   // bf16(Q), [nb][LB][LB] row major
  const float* Qf;      // Q in fp32, same layout (forward only)
  int k, nb;
  float* G;             // forward: I + H, [nb][LB][LB] (nullable)
  uint16_t* E;          // forward: bf16 pair [nb][2][LB][LB] (nullable)
  const float* D;       // backward: dL/dG [nb][LB][LB]
  float* M;             // backward: [k][nb][LB][LB], M[m-1] = W_m^T
  float* dQ;            // backward pass 2: dL/dQ [nb][LB][LB]
};

// p + n with the sum hidden from the optimiser: walking a column row by row with this keeps
// one live address instead of one precomputed 64-bit address per unrolled access.
template <class T>
__device__ inline T* bump(T* p, i64 n) {
  p += n;
  asm volatile("" : "+v"(p));
  return p;
}

__device__ inline bf16x8 negate(bf16x8 v) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 u = __builtin_bit_cast(u32x4, v);
  u ^= 0x80008000u;
  return __builtin_bit_cast(bf16x8, u);
}

__device__ inline bf16x8 pack8(const floatx16& a, int u) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 r;
#pragma unroll
  for (int e = 0; e < 4; ++e) r[e] = mm::pack2_bf16(a[8 * u + 2 * e], a[8 * u + 2 * e + 1]);
  return __builtin_bit_cast(bf16x8, r);
}

template <int MODE>
__global__ __launch_bounds__(256) void cnp_chain_kernel(ChainArgs a) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = blockIdx.y;
  const int wg0 = blockIdx.x * 128;             // first column of the workgroup
  const int n = lane & 31, h = lane >> 5;
  const int col = wg0 + wave * 32 + n;          // this lane's column of the running matrix
  const i64 blk = (i64)j * LB * LB;

  // ---- bf16(Q) into LDS, contraction slots permuted: a 16-byte chunk (8 consecutive k, i.e.
  // one value of a and both values of h) becomes two 8-byte pieces 16 bytes apart.
  {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr int NCH = LB * LB / 8 / 256;   // chunks per thread
    const u32x4* src = reinterpret_cast<const u32x4*>(a.Qb + blk);
    u32x4 v[NCH];
    // Chunk (row, kc) of a wave's two rows goes to lane 16 * (2 * (kc >> 4) + (row & 1)) + (kc & 15): the 8-byte
    // writes of a half wave then cover rows 2p and 2p + 1 (4 banks apart) over 16 chunks each = all 64 banks once.
    auto chunk_of = [&](int id, int& row, int& kc) {
      const int l = id & 63;
      row = 2 * (id >> 6) + ((l >> 4) & 1);
      kc = (l & 15) + 16 * (l >> 5);
    };
#pragma unroll
    for (int it = 0; it < NCH; ++it) {
      int row, kc;
      chunk_of(tid + 256 * it, row, kc);
      v[it] = src[row * 32 + kc];
    }
#pragma unroll
    for (int it = 0; it < NCH; ++it) {
      int row, kc;
      chunk_of(tid + 256 * it, row, kc);
      char* dst = lds + row * LROW + 32 * (kc >> 1) + 8 * (kc & 1);
      *reinterpret_cast<uint2*>(dst) = make_uint2(v[it][0], v[it][1]);
      *reinterpret_cast<uint2*>(dst + 16) = make_uint2(v[it][2], v[it][3]);
    }
  }
  __syncthreads();

  // A fragment (row tile tm, k step s): 16 bytes at row 32 tm + n, slot 16 s + 8 h.
  const char* qa = lds + n * LROW + 16 * h;
  // The lane's own column of Q read as row `col` (Q[k][col] = -Q[col][k]): same slots.
  const char* qown = lds + col * LROW + 16 * h;

  bf16x8 Y[NKS];
  floatx16 acc[NT];
  floatx16 S[MODE == CHAIN_BWD1 ? NT : 1];

  // ---- first value of the running matrix
  if (MODE == CHAIN_FWD) {
#pragma unroll
    for (int s = 0; s < NKS; ++s) Y[s] = negate(*reinterpret_cast<const bf16x8*>(qown + s * 32));
  } else if (MODE == CHAIN_BWD1) {
    // V_0 = D^T: element (r, col) is D[col][r]; registers 4g..4g+3 of tile t are 4 consecutive r
    const float* drow = a.D + blk + (i64)col * LB + 4 * h;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 v = *reinterpret_cast<const float4*>(drow + 32 * t + 8 * g);
        S[t][4 * g + 0] = v.x; S[t][4 * g + 1] = v.y; S[t][4 * g + 2] = v.z; S[t][4 * g + 3] = v.w;
      }
      Y[2 * t] = pack8(S[t], 0);
      Y[2 * t + 1] = pack8(S[t], 1);
    }
  } else {
    // Y_0 = D: element (r, col) is D[r][col]
    const float* p = a.D + blk + col + (i64)4 * h * LB;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      floatx16 v;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[4 * g + e] = p[e * LB];
        p = bump(p, 8 * LB);
      }
      Y[2 * t] = pack8(v, 0);
      Y[2 * t + 1] = pack8(v, 1);
    }
  }

  // acc = Q * running matrix; the fragments of the next k step are read under the MFMAs of this one
  auto product = [&]() {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
    bf16x8 A[2][NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) A[0][t] = *reinterpret_cast<const bf16x8*>(qa + t * 32 * LROW);
#pragma unroll
    for (int s = 0; s < NKS; ++s) {
      if (s + 1 < NKS) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
          A[(s + 1) & 1][t] = *reinterpret_cast<const bf16x8*>(qa + t * 32 * LROW + (s + 1) * 32);
      }
#pragma unroll
      for (int t = 0; t < NT; ++t)
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[s & 1][t], Y[s], acc[t], 0, 0, 0);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);   // keep the reads of step s+1 in the shadow of step s
    }
  };
  // fp32 column `col` of a row-major matrix in accumulator layout, fetched before a product so
  // that it lands under it
  auto fetch_col = [&](floatx16* W, const float* base) {
    const float* p = base + (i64)4 * h * LB;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
#pragma unroll
        for (int e = 0; e < 4; ++e) W[t][4 * g + e] = p[e * LB];
        p = bump(p, 8 * LB);
      }
  };
  auto repack = [&]() {
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      Y[2 * t] = pack8(acc[t], 0);
      Y[2 * t + 1] = pack8(acc[t], 1);
    }
  };

  if (MODE == CHAIN_FWD) {
    for (int step = 1; step < a.k; ++step) {
      product();
      // H = 2Q + acc with Q[r][col] = -Q[col][r] taken from LDS (bf16: the chain value is rounded anyway)
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 q = *reinterpret_cast<const bf16x8*>(qown + (2 * t + u) * 32);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[t][8 * u + e] -= 2.f * (float)q[e];
        }
      repack();
    }
    floatx16 Qt[NT];            // last step: 2Q enters in fp32
    fetch_col(Qt, a.Qf + blk + col);
    product();
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[t][v] += 2.f * Qt[t][v];
  } else if (MODE == CHAIN_BWD1) {
    for (int step = 1; step <= a.k; ++step) {
      product();
      // V_m = acc;  W_m = 2 (V_0 + .. + V_m) - V_m, written as row `col` of W_m^T
      float* mrow = a.M + ((i64)(step - 1) * a.nb + j) * LB * LB + (i64)col * LB + 4 * h;
#pragma unroll
      for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int v = 0; v < 16; ++v) S[t][v] += acc[t][v];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float4 w;
          w.x = 2.f * S[t][4 * g + 0] - acc[t][4 * g + 0];
          w.y = 2.f * S[t][4 * g + 1] - acc[t][4 * g + 1];
          w.z = 2.f * S[t][4 * g + 2] - acc[t][4 * g + 2];
          w.w = 2.f * S[t][4 * g + 3] - acc[t][4 * g + 3];
          *reinterpret_cast<float4*>(mrow + 32 * t + 8 * g) = w;
        }
      }
      if (step < a.k) repack();
    }
  } else {
    for (int step = 1; step <= a.k; ++step) {
      floatx16 Wt[NT];          // W_m^T
      fetch_col(Wt, a.M + ((i64)(step - 1) * a.nb + j) * LB * LB + col);
      product();
      // Y_m = W_m^T - acc; the last one is dL/dQ
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = Wt[t][v] - acc[t][v];
      if (step < a.k) repack();
    }
  }

  if (MODE == CHAIN_BWD2) {
    float* p = a.dQ + blk + col + (i64)4 * h * LB;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
#pragma unroll
        for (int e = 0; e < 4; ++e) p[e * LB] = acc[t][4 * g + e];
        p = bump(p, 8 * LB);
      }
  }

  if (MODE == CHAIN_FWD) {
    // rows r0 .. r0+3 of column `col`, r0 = 32 t + 8 g + 4 h: four strided elements of G and of
    // E, one 8-byte run of E^T
    uint16_t* e0 = a.E ? a.E + (i64)j * 2 * LB * LB + col + (i64)4 * h * LB : nullptr;
    uint16_t* e1 = a.E ? a.E + (i64)j * 2 * LB * LB + (i64)LB * LB + (i64)col * LB + 4 * h : nullptr;
    float* gc = a.G ? a.G + blk + col + (i64)4 * h * LB : nullptr;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int r0 = 32 * t + 8 * g + 4 * h;
        if (gc) {
#pragma unroll
          for (int e = 0; e < 4; ++e) gc[e * LB] = acc[t][4 * g + e] + ((r0 + e) == col ? 1.f : 0.f);
          gc = bump(gc, 8 * LB);
        }
        if (e0) {
          uint2 pk;
          pk.x = mm::pack2_bf16(acc[t][4 * g + 0], acc[t][4 * g + 1]);
          pk.y = mm::pack2_bf16(acc[t][4 * g + 2], acc[t][4 * g + 3]);
          e0[0 * LB] = (uint16_t)pk.x;
          e0[1 * LB] = (uint16_t)(pk.x >> 16);
          e0[2 * LB] = (uint16_t)pk.y;
          e0[3 * LB] = (uint16_t)(pk.y >> 16);
          e0 = bump(e0, 8 * LB);
          *reinterpret_cast<uint2*>(e1 + 32 * t + 8 * g) = pk;
        }
      }
    }
  }
}

template <int MODE>
void launch_chain(const ChainArgs& a, hipStream_t st) {
  auto kern = cnp_chain_kernel<MODE>;
  // once per kernel instance; a function-local static is initialised exactly once, whichever thread gets there first
  static const bool configured =
      hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, CHAIN_LDS) == hipSuccess;
  (void)configured;
  hipLaunchKernelGGL(kern, dim3(LB / 128, a.nb), dim3(256), CHAIN_LDS, st, a);
}

}  // namespace

bool lds_cnp_supported(int d, int b) { return b == LB && d % LB == 0; }

// floats of scratch per block element for the backward: W_1^T .. W_k^T and dL/dQ
size_t lds_cnp_bwd_ws_floats_per_elem(int k) { return (size_t)k + 1; }

void lds_cnp_build(const float* Qf, const uint16_t* Qb, int d, int k, float* G_f32, void* E_bf16, hipStream_t st) {
  ChainArgs a{};
  a.Qf = Qf;
  a.Qb = Qb;
  a.k = k;
  a.nb = d / LB;
  a.G = G_f32;
  a.E = (uint16_t*)E_bf16;
  launch_chain<CHAIN_FWD>(a, st);
}

const float* lds_cnp_bwd_chain(const uint16_t* Qb, const float* dG, int nb, int k, float* ws, hipStream_t st) {
  ChainArgs a{};
  a.Qb = Qb;
  a.k = k;
  a.nb = nb;
  a.D = dG;
  a.M = ws;
  a.dQ = ws + (size_t)k * nb * LB * LB;
  launch_chain<CHAIN_BWD1>(a, st);
  launch_chain<CHAIN_BWD2>(a, st);
  return a.dQ;
}

}  // namespace poetx
