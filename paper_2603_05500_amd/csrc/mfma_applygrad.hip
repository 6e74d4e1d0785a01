// Backward block stage of one side in a single pass over the gradient (Sec. 3.5, mm3 / mm1
// backward), b = 256, bf16:
//     out   = Psi^T Diag(G) Psi * V                 (dB = P dZ,   dX = R dA)
//     dG_j  = U'_j V'_j^T                            (dG_P = B' dZ'^T, dG_R = X' dA'^T)
// with V the incoming gradient (d x N, feature major), U the tensor saved by the forward pass
// and primes denoting rows gathered through the side's permutation.  Both results need the
// gathered rows V'_j of block j, so one kernel streams them once: a token tile of V'_j lands
// in LDS, is multiplied by the block from the left (contraction over its rows, transposing LDS
// reads) and, with the matching tile of U'_j, extends the block gradient (contraction over its
// tokens, plain 16-byte LDS reads of the same tile).
//
// A workgroup owns block j, one 128-row half of it and a token range.  The two halves of a
// block run side by side on the same XCD, so the V tile the second one asks for comes out of
// that XCD's L2.  8 waves: waves 0..3 each produce 32 output rows of the half for the 64 tokens
// of a tile (their rows of the block operand stay in registers); waves 4..7 each hold a 32 x 256
// stripe of the half's block gradient in 128 accumulator registers for the whole token range.
// Tiles flow through a 3-stage ring of direct-to-LDS loads (two tiles in flight under the one
// being multiplied).  The V tile is stored [row][64 tokens] with its 16-byte chunks XORed by a
// bit-reversed function of the row pair, which keeps both the transposing reads (4 consecutive
// rows x 32 bytes) and the row-wise reads (16 consecutive rows x 16 bytes) free of bank conflicts.
// Each workgroup writes its partial block gradient once, at the end; a small kernel adds the
// partials of a block in a fixed order (deterministic, no atomics).
#include "mfma_gemm.h"

namespace poetx {
namespace {

using mm::bf16x8;
using mm::floatx16;
using mm::short4v;
using mm::short8v;

constexpr int GB = 256;                      // block side
constexpr int GBN = 64;                      // tokens per tile: one 128-byte line per row
constexpr int V_BYTES = GB * GBN * 2;        // 32 KB
constexpr int U_BYTES = (GB / 2) * GBN * 2;  // 16 KB
constexpr int G_STAGE = V_BYTES + U_BYTES;   // 48 KB
constexpr int G_NS = 3;
constexpr int G_STG = G_NS * G_STAGE;        // output staging of the apply waves: 4 x 4 KB
constexpr int G_LDS = G_STG + 4 * 4096;      // 160 KB
constexpr int G_LOADS = 6;                   // direct-to-LDS instructions per wave per tile (4 V + 2 U)

// chunk position of logical 16-byte chunk c in row k of a [row][64 tokens] tile
__device__ inline int rc_swz(int c, int k) {
  const int t = (k >> 1) & 7;
  return c ^ (((t & 1) << 2) | (t & 2) | ((t >> 2) & 1));
}

struct GradArgs {
  const uint16_t* V;
  const uint16_t* U;
  uint16_t* out;
  i64 ld;
  const int32_t* perm;
  const uint16_t* blocks;   // bf16 pairs [nb][2][256][256]
  int trans;                // which member of the pair multiplies V
  float* partial;           // [chunks][nb][256][256]
  int nb, tiles_per_wg, n_pairs;
};

__global__ __launch_bounds__(512) void apply_grad_stream_kernel(GradArgs g) {
  extern __shared__ __attribute__((aligned(1024))) char ring[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // workgroups go to the XCDs round robin: ids 8 apart are neighbours on one XCD
  const int id = blockIdx.x;
  const int half = (id >> 3) & 1;
  const int pair = (id >> 4) * 8 + (id & 7);
  if (pair >= g.n_pairs) return;
  const int j = pair % g.nb, chunk = pair / g.nb;
  const i64 tok0 = (i64)chunk * g.tiles_per_wg * GBN;
  const int32_t* pm = g.perm + (i64)j * GB;
  const int li = lane & 31, h = lane >> 5;
  const uint32_t ring_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)ring;
  const int T = g.tiles_per_wg;

  // ---- direct-to-LDS loads: V instruction s of wave w fills chunk slots [(4w+s)*64, +64) of the V
  // part (8 rows of 8 chunks), U instruction s fills [(2w+s)*64, +64) of the U part
  i64 goff[G_LOADS];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int slot = (wave * 4 + s) * 64 + lane, k = slot >> 3, c = rc_swz(slot & 7, k);
    goff[s] = (i64)pm[k] * g.ld + tok0 + c * 8;
  }
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const int slot = (wave * 2 + s) * 64 + lane, r = slot >> 3, c = rc_swz(slot & 7, r);
    goff[4 + s] = (i64)pm[half * 128 + r] * g.ld + tok0 + c * 8;
  }
  auto issue = [&](int t, int slot) {
    const uint32_t stage = ring_base + slot * G_STAGE;
#pragma unroll
    for (int s = 0; s < 4; ++s) mm::dma16(g.V + goff[s] + (i64)t * GBN, stage + (wave * 4 + s) * 1024);
#pragma unroll
    for (int s = 0; s < 2; ++s) mm::dma16(g.U + goff[4 + s] + (i64)t * GBN, stage + V_BYTES + (wave * 2 + s) * 1024);
  };
  issue(0, 0);
  if (T > 1) issue(1, 1);

  // Wait for tile t (loads return in order; at most the loads of one younger tile may stay in
  // flight; stores share the counter and only make the wait stricter), then meet the other waves:
  // every wave is then also done reading the stage that the next issue overwrites.
  auto wait_tile = [&](bool younger_in_flight) {
    if (younger_in_flight) mm::wait_all_reads_and_barrier<G_LOADS>();
    else mm::wait_all_reads_and_barrier<0>();
  };

  if (wave < 4) {
    // =========================== apply waves: out rows half*128 + 32 wave + 0..31 ===========
    const int row_own = half * 128 + wave * 32 + li;
    const uint16_t* Eb = g.blocks + ((i64)j * 2 + (g.trans ? 1 : 0)) * GB * GB + (i64)row_own * GB + 8 * h;
    bf16x8 fa[GB / 16];
#pragma unroll
    for (int ks = 0; ks < GB / 16; ++ks) fa[ks] = *reinterpret_cast<const bf16x8*>(Eb + ks * 16);
    // identity fragments for the two k steps that cover the wave's own 32 rows (1.0 * x is exact)
    bf16x8 fi[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int e = 0; e < 8; ++e) fi[u][e] = (li == u * 16 + 8 * h + e) ? (__bf16)1.0f : (__bf16)0.0f;
    const int own_kpair = half * 4 + wave;
    // token fragments (transposing reads): 4 consecutive rows x 2 chunks per group of 16 lanes
    int fragT[2], fragT4[2];
    {
      const int q = lane >> 4, i = lane & 15;
      const int k = 8 * (q >> 1) + (i >> 2);
#pragma unroll
      for (int c2 = 0; c2 < 2; ++c2) {
        const int c = c2 * 4 + 2 * (q & 1) + ((i & 3) >> 1);
        fragT[c2] = k * 128 + 16 * rc_swz(c, k) + 8 * (i & 1);
        fragT4[c2] = (k + 4) * 128 + 16 * rc_swz(c, k + 4) + 8 * (i & 1);
      }
    }
    // output staging (4 KB per wave) and coalesced stores: see apply_left_stream_kernel
    char* stg = ring + G_STG + wave * 4096;
    const int stg_w = li * 128 + 16 * (h ^ ((li >> 1) & 7));
    i64 soff[4];
    int stg_r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = (lane >> 3) + 8 * i;
      soff[i] = (i64)pm[half * 128 + wave * 32 + r] * g.ld + tok0 + 8 * (lane & 7);
      stg_r[i] = r * 128 + 16 * ((lane & 7) ^ ((r >> 1) & 7));
    }
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 pend[4];
    auto flush = [&](int t) {
#pragma unroll
      for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(g.out + soff[i] + (i64)t * GBN) = pend[i];
    };
    int slot = 0;
    for (int t = 0; t < T; ++t) {
      wait_tile(t + 1 < T);
      if (t > 0) flush(t - 1);                       // one tile late: old by the next wait
      if (t + 2 < T) issue(t + 2, slot == 0 ? 2 : slot - 1);
      const char* stage = ring + slot * G_STAGE;
      // the swizzle depends on the row only through (k >> 1) & 7, so a k step (16 rows) further down
      // uses the same offsets
      auto load_tok = [&](bf16x8* fb, int ks) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          short4v lo = mm::lds_read_tr(stage + fragT[c] + ks * 16 * 128);
          short4v hi = mm::lds_read_tr(stage + fragT4[c] + ks * 16 * 128);
          short8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          fb[c] = __builtin_bit_cast(bf16x8, v);
        }
      };
      floatx16 acc[2];
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
      bf16x8 fo[2][2], fb[2][2];
      load_tok(fo[0], 2 * own_kpair);
      load_tok(fo[1], 2 * own_kpair + 1);
      load_tok(fb[0], 0);
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int c = 0; c < 2; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo[u][c], fi[u], acc[c], 0, 0, 0);
#pragma unroll
      for (int ks = 0; ks < GB / 16; ++ks) {
        if (ks + 1 < GB / 16) load_tok(fb[(ks + 1) & 1], ks + 1);
#pragma unroll
        for (int c = 0; c < 2; ++c)
          acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks & 1][c], fa[ks], acc[c], 0, 0, 0);
      }
      // round, swap register pairs between the lane halves (a lane then holds 8 consecutive
      // tokens), stage, read back row by row
#pragma unroll
      for (int cl = 0; cl < 2; ++cl) {
        uint32_t w[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = mm::pack2_bf16(acc[cl][2 * e], acc[cl][2 * e + 1]);
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          typedef unsigned uint2v __attribute__((ext_vector_type(2)));
          const uint2v r0 = __builtin_amdgcn_permlane32_swap(w[4 * p], w[4 * p + 2], false, false);
          const uint2v r1 = __builtin_amdgcn_permlane32_swap(w[4 * p + 1], w[4 * p + 3], false, false);
          *reinterpret_cast<u32x4*>(stg + (stg_w ^ (16 * (cl * 4 + 2 * p)))) = u32x4{r0[0], r1[0], r0[1], r1[1]};
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int i = 0; i < 4; ++i) pend[i] = *reinterpret_cast<const u32x4*>(stg + stg_r[i]);
      slot = slot + 1 == G_NS ? 0 : slot + 1;
    }
    flush(T - 1);
  } else {
    // =========================== gradient waves: dG rows half*128 + 32 g + 0..31, all 256 columns
    const int gw = wave - 4;
    // row-wise fragment reads: lane -> row (lane & 31), chunk 2 ks + (lane >> 5)
    int fragU, fragV[8];
    {
      const int r = gw * 32 + li;
      fragU = V_BYTES + r * 128 + 16 * rc_swz(h, r);
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const int c = ct * 32 + li;
        fragV[ct] = c * 128 + 16 * rc_swz(h, c);
      }
    }
    floatx16 acc[8];
#pragma unroll
    for (int ct = 0; ct < 8; ++ct)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[ct][v] = 0.f;
    int slot = 0;
    for (int t = 0; t < T; ++t) {
      wait_tile(t + 1 < T);
      if (t + 2 < T) issue(t + 2, slot == 0 ? 2 : slot - 1);
      const char* stage = ring + slot * G_STAGE;
      // k step ks covers tokens 16 ks .. 16 ks + 15 = logical chunks 2 ks, 2 ks + 1: XOR of the
      // swizzled position with 2 ks (the swizzle is an XOR, so it commutes)
      bf16x8 fu[2], fv[2][8];
      fu[0] = *reinterpret_cast<const bf16x8*>(stage + fragU);
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) fv[0][ct] = *reinterpret_cast<const bf16x8*>(stage + fragV[ct]);
#pragma unroll
      for (int ks = 0; ks < GBN / 16; ++ks) {
        if (ks + 1 < GBN / 16) {
          fu[(ks + 1) & 1] = *reinterpret_cast<const bf16x8*>(stage + (fragU ^ (32 * (ks + 1))));
#pragma unroll
          for (int ct = 0; ct < 8; ++ct)
            fv[(ks + 1) & 1][ct] = *reinterpret_cast<const bf16x8*>(stage + (fragV[ct] ^ (32 * (ks + 1))));
        }
        // operands swapped: the lane owns gradient row (its U row) and 4 consecutive columns
#pragma unroll
        for (int ct = 0; ct < 8; ++ct)
          acc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[ks & 1][ct], fu[ks & 1], acc[ct], 0, 0, 0);
      }
      slot = slot + 1 == G_NS ? 0 : slot + 1;
    }
    // A lane holds columns 8q + 4h .. + 3 of its row for q = 0..3.  Swapping register groups between the lane
    // halves (v_permlane32_swap: the upper half of its first operand against the lower half of its second)
    // leaves the lower lanes with columns 8q .. 8q + 7 and the upper lanes with 8(q+1) .. 8(q+1) + 7:
    // every lane stores whole 32-byte sectors.
    typedef unsigned uint2v __attribute__((ext_vector_type(2)));
    float* P = g.partial + (((i64)chunk * g.nb + j) * GB + half * 128 + gw * 32 + li) * GB + 8 * h;
#pragma unroll
    for (int ct = 0; ct < 8; ++ct)
#pragma unroll
      for (int q = 0; q < 4; q += 2) {
        float lo[4], hi[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float x = acc[ct][4 * q + e], y = acc[ct][4 * q + 4 + e];   // scalars first: a bit cast straight from a vector element reads element 0
          const uint2v r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, y), false, false);
          const unsigned r0 = r[0], r1 = r[1];
          lo[e] = __builtin_bit_cast(float, r0);
          hi[e] = __builtin_bit_cast(float, r1);
        }
        *reinterpret_cast<float4*>(P + ct * 32 + 8 * q) = make_float4(lo[0], lo[1], lo[2], lo[3]);
        *reinterpret_cast<float4*>(P + ct * 32 + 8 * q + 4) = make_float4(hi[0], hi[1], hi[2], hi[3]);
      }
  }
}

__global__ void reduce_grad_partials_kernel(const float4* __restrict__ part, float4* __restrict__ out, i64 n4, int chunks) {
  i64 idx = (i64)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n4) return;
  float4 s = part[idx];
  for (int z = 1; z < chunks; ++z) {
    float4 p = part[(i64)z * n4 + idx];
    s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
  }
  out[idx] = s;
}

// token ranges per block: workgroups = 2 nb chunks; fill the CUs in whole rounds, keep at least
// 4 tiles per workgroup (the two tiles of lead-in are then a small share)
// Token chunks per half block.  More chunks fill the 256 CUs in whole rounds, but every chunk writes an
// fp32 partial of its half block that the reduction reads again: the choice minimises the bytes moved,
// with the three activation passes weighted by the share of the CUs that the workgroups keep busy.
int grad_chunks(int nb, int tiles) {
  int best = 1;
  double best_cost = 0.0;
  const double act = 3.0 * nb * GB * (double)tiles * GBN * 2.0;
  for (int c = 1; c <= tiles; c *= 2) {
    if (tiles % c != 0 || tiles / c < 4) break;
    const double wgs = 2.0 * nb * c;
    const double rounds = (double)(long long)((wgs + 255) / 256);
    const double eff = wgs / 256.0 / rounds;
    const double cost = act / eff + (c > 1 ? 2.0 * c * nb * GB * GB * 4.0 : 0.0);
    if (c == 1 || cost < best_cost) { best_cost = cost; best = c; }
  }
  return best;
}

}  // namespace

bool mfma_apply_grad_supported(int d, i64 N, i64 ld, int b) {
  return b == GB && d % GB == 0 && N % GBN == 0 && N / GBN >= 4 && ld % 8 == 0 && N < (1ll << 31);
}

size_t mfma_apply_grad_workspace_bytes(int d, i64 N) {
  return (size_t)grad_chunks(d / GB, (int)(N / GBN)) * d * GB * sizeof(float);
}

void mfma_apply_grad(const void* V, const void* U, void* out, int d, i64 N, i64 ld, const int32_t* perm, const void* E,
                     int transpose_G, float* dG, void* ws, hipStream_t st) {
  static const bool configured =
      hipFuncSetAttribute((const void*)apply_grad_stream_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, G_LDS) == hipSuccess;
  (void)configured;
  GradArgs g{};
  g.V = (const uint16_t*)V;
  g.U = (const uint16_t*)U;
  g.out = (uint16_t*)out;
  g.ld = ld;
  g.perm = perm;
  g.blocks = (const uint16_t*)E;
  g.trans = transpose_G;
  g.nb = d / GB;
  const int tiles = (int)(N / GBN), chunks = grad_chunks(g.nb, tiles);
  g.tiles_per_wg = tiles / chunks;
  g.n_pairs = g.nb * chunks;
  g.partial = chunks > 1 ? (float*)ws : dG;
  const int grid = ceil_div(g.n_pairs, 8) * 16;
  hipLaunchKernelGGL(apply_grad_stream_kernel, dim3(grid), dim3(512), G_LDS, st, g);
  if (chunks > 1) {
    const i64 n4 = (i64)d * GB / 4;
    hipLaunchKernelGGL(reduce_grad_partials_kernel, dim3(ceil_div(n4, 256)), dim3(256), 0, st, (const float4*)ws, (float4*)dG, n4, chunks);
  }
}

}  // namespace poetx
