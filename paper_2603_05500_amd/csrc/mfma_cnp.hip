// Cayley-Neumann series and its backward on the matrix cores (Sec. 3.4, Eq. 8-9),
// batched over the blocks of one side, for block sides that are multiples of 256.
//
// Every b x b product runs as bf16 x bf16 -> fp32 on the batched tile kernel.  To
// keep the small terms, the chain is carried in residual form: with H = 2I + H'
// Horner's rule H <- H Q + 2I becomes H' <- 2Q + H' Q, where only the small
// product H' Q goes through bf16 and the 2Q term is added in fp32.
// After k steps H' is G - I.  The backward recursion (see fma_cnp_bwd) is carried
// the same way: A = 2I + A', A' <- 2T + A' T and Bm <- 2D + A' D + Bm T with
// T = -Q, the 2D term added in fp32; the two products of one step are independent
// and share one launch.
#include "mfma_gemm.h"

namespace poetx {
namespace {

// Tiled products (block sides that do not fit on chip, i.e. b = 512): 128 x 128 tiles, 2 x 2 waves,
// 64 KB of LDS so that two workgroups share a CU; a contraction is only b deep, so the loop
// stops loading after the last tile instead of re-fetching it.
constexpr int CBM = 128, CBN = 128, CBK = 64, CNS = 4;

__device__ inline float skew_at(const float* th, int i, int c, int b) {
  if (i == c) return 0.f;
  return i < c ? th[packed_index(i, c, b)] : -th[packed_index(c, i, b)];
}

// Q from the packed parameters: Qf = Q (fp32), Qb = bf16(Q), Tb = bf16(-Q); any may be null.
__global__ void skew_materialize_kernel(const float* __restrict__ theta, int b, i64 total, float* __restrict__ Qf,
                                        uint16_t* __restrict__ Qb, uint16_t* __restrict__ Tb) {
  i64 idx = (i64)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  int c = (int)(idx % b);
  int i = (int)((idx / b) % b);
  i64 j = idx / ((i64)b * b);
  float q = skew_at(theta + j * ((i64)b * (b - 1) / 2), i, c, b);
  if (Qf) Qf[idx] = q;
  if (Qb) Qb[idx] = float_to_bf16_bits(q);
  if (Tb) Tb[idx] = float_to_bf16_bits(-q);
}

__global__ void to_bf16_kernel(const float4* __restrict__ in, uint2* __restrict__ out, i64 n4) {
  i64 idx = (i64)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n4) return;
  float4 v = in[idx];
  uint2 o;
  o.x = mm::pack2_bf16(v.x, v.y);
  o.y = mm::pack2_bf16(v.z, v.w);
  out[idx] = o;
}

// value = acc + coef * Qf(row, col).  Writes whichever outputs are set:
// Hn (bf16 chain value), G (fp32, + I), E (bf16 pair [nb][2][b][b]: value and its transpose).
struct EpiHorner {
  const float* Qf;
  float coef;
  int b;
  uint16_t* Hn;
  float* G;
  uint16_t* E;
  __device__ void operator()(int j, int, int row, int col, float4 a) const {
    const i64 o = ((i64)j * b + row) * b + col;
    const float4 q = *reinterpret_cast<const float4*>(Qf + o);
    float v[4] = {a.x + coef * q.x, a.y + coef * q.y, a.z + coef * q.z, a.w + coef * q.w};
    uint2 pk;
    pk.x = mm::pack2_bf16(v[0], v[1]);
    pk.y = mm::pack2_bf16(v[2], v[3]);
    if (Hn) *reinterpret_cast<uint2*>(Hn + o) = pk;
    if (G) {
      float4 gv = make_float4(v[0], v[1], v[2], v[3]);
      gv.x += (row == col) ? 1.f : 0.f;
      gv.y += (row == col + 1) ? 1.f : 0.f;
      gv.z += (row == col + 2) ? 1.f : 0.f;
      gv.w += (row == col + 3) ? 1.f : 0.f;
      *reinterpret_cast<float4*>(G + o) = gv;
    }
    if (E) {
      const i64 base = (i64)j * 2 * b * b;
      *reinterpret_cast<uint2*>(E + base + (i64)row * b + col) = pk;
#pragma unroll
      for (int e = 0; e < 4; ++e) E[base + (i64)b * b + (i64)(col + e) * b + row] = float_to_bf16_bits(v[e]);
    }
  }
  // eight consecutive columns: 32-byte reads of Q, 16-byte stores of the bf16 outputs
  __device__ void wide(int j, int, int row, int col, float4 lo, float4 hi) const {
    const i64 o = ((i64)j * b + row) * b + col;
    const float4 q0 = *reinterpret_cast<const float4*>(Qf + o), q1 = *reinterpret_cast<const float4*>(Qf + o + 4);
    const float v[8] = {lo.x + coef * q0.x, lo.y + coef * q0.y, lo.z + coef * q0.z, lo.w + coef * q0.w,
                        hi.x + coef * q1.x, hi.y + coef * q1.y, hi.z + coef * q1.z, hi.w + coef * q1.w};
    const uint4 pk = make_uint4(mm::pack2_bf16(v[0], v[1]), mm::pack2_bf16(v[2], v[3]), mm::pack2_bf16(v[4], v[5]), mm::pack2_bf16(v[6], v[7]));
    if (Hn) *reinterpret_cast<uint4*>(Hn + o) = pk;
    if (G) {
      float gv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) gv[e] = v[e] + (row == col + e ? 1.f : 0.f);
      *reinterpret_cast<float4*>(G + o) = make_float4(gv[0], gv[1], gv[2], gv[3]);
      *reinterpret_cast<float4*>(G + o + 4) = make_float4(gv[4], gv[5], gv[6], gv[7]);
    }
    if (E) {
      const i64 base = (i64)j * 2 * b * b;
      *reinterpret_cast<uint4*>(E + base + (i64)row * b + col) = pk;
#pragma unroll
      for (int e = 0; e < 8; ++e) E[base + (i64)b * b + (i64)(col + e) * b + row] = float_to_bf16_bits(v[e]);
    }
  }
};

// One backward step in one launch.  Batches [0, nb): Bm_next = acc + 2 D  (bf16 chain value and/or
// the final fp32 result).  Batches [nb, 2nb): A'_next = acc - 2 Q (bf16).
struct EpiBwdStep {
  const float* D;
  const float* Qf;
  int b, nb;
  uint16_t* Bn;
  float* Bf;
  uint16_t* An;
  __device__ void operator()(int batch, int, int row, int col, float4 a) const {
    const bool second = batch >= nb;
    const int j = second ? batch - nb : batch;
    const i64 o = ((i64)j * b + row) * b + col;
    const float4 d = *reinterpret_cast<const float4*>((second ? Qf : D) + o);
    const float coef = second ? -2.f : 2.f;
    const float4 v = make_float4(a.x + coef * d.x, a.y + coef * d.y, a.z + coef * d.z, a.w + coef * d.w);
    uint2 pk;
    pk.x = mm::pack2_bf16(v.x, v.y);
    pk.y = mm::pack2_bf16(v.z, v.w);
    if (second) {
      *reinterpret_cast<uint2*>(An + o) = pk;
    } else {
      if (Bn) *reinterpret_cast<uint2*>(Bn + o) = pk;
      if (Bf) *reinterpret_cast<float4*>(Bf + o) = v;
    }
  }
  __device__ void wide(int batch, int, int row, int col, float4 lo, float4 hi) const {
    const bool second = batch >= nb;
    const int j = second ? batch - nb : batch;
    const i64 o = ((i64)j * b + row) * b + col;
    const float* src = (second ? Qf : D) + o;
    const float4 d0 = *reinterpret_cast<const float4*>(src), d1 = *reinterpret_cast<const float4*>(src + 4);
    const float coef = second ? -2.f : 2.f;
    const float4 v0 = make_float4(lo.x + coef * d0.x, lo.y + coef * d0.y, lo.z + coef * d0.z, lo.w + coef * d0.w);
    const float4 v1 = make_float4(hi.x + coef * d1.x, hi.y + coef * d1.y, hi.z + coef * d1.z, hi.w + coef * d1.w);
    const uint4 pk = make_uint4(mm::pack2_bf16(v0.x, v0.y), mm::pack2_bf16(v0.z, v0.w), mm::pack2_bf16(v1.x, v1.y), mm::pack2_bf16(v1.z, v1.w));
    if (second) {
      *reinterpret_cast<uint4*>(An + o) = pk;
    } else {
      if (Bn) *reinterpret_cast<uint4*>(Bn + o) = pk;
      if (Bf) {
        *reinterpret_cast<float4*>(Bf + o) = v0;
        *reinterpret_cast<float4*>(Bf + o + 4) = v1;
      }
    }
  }
};

// 512-wide blocks take 256 x 256 output tiles (8 waves of 128 x 64): four times the work per
// workgroup for the same 512-deep contraction, whose fill and drain dominate a 128 x 128 tile.
inline bool big_tiles(int b) { return b % 256 == 0 && b >= 512; }
mm::Args batched_args(int b) {
  mm::Args g{};
  const int t = big_tiles(b) ? 256 : CBM;
  g.tiles_m = b / t;
  g.tiles_n = b / t;
  return g;
}
template <class Epi>
void launch_product(int b, const mm::Args& g, Epi epi, int batches, hipStream_t st) {
  if (big_tiles(b)) mm::launch<256, 256, 2, 4, true, false, false, CNS, true>(g, epi, batches, 1, st);
  else mm::launch<CBM, CBN, 2, 2, true, false, false, CNS, true>(g, epi, batches, 1, st);
}
void set_src(mm::Source& s, const uint16_t* A, const uint16_t* B, int b) {
  s.A = A; s.B = B; s.lda = b; s.ldb = b; s.sA = (i64)b * b; s.sB = (i64)b * b; s.ktiles = b / CBK;
}

}  // namespace

void skew_materialize_launch(const float* theta, int b, i64 nb, float* Qf, uint16_t* Qb, uint16_t* Tb, hipStream_t st) {
  if (skew_tiled_supported(b, (i64)b)) {
    skew_materialize_tiled_launch(theta, b, nb, Qf, Qb, Tb, st);
    return;
  }
  const i64 total = nb * b * b;
  hipLaunchKernelGGL(skew_materialize_kernel, dim3(ceil_div(total, 256)), dim3(256), 0, st, theta, b, total, Qf, Qb, Tb);
}

bool mfma_cnp_supported(int d, int b) { return (b == 256 || b == 512) && d % b == 0; }

// bytes of scratch per block element (nb*b*b elements): forward Qf(4) + Qb, H0, H1 (2 each);
// backward Qf(4) + Tb, Db, A0, A1, B0, B1 (2 each) + Bfinal(4).
size_t mfma_cnp_build_ws_bytes_per_elem() { return 10; }
size_t mfma_cnp_bwd_ws_bytes_per_elem() { return 20; }

void mfma_cnp_build(const float* theta, int d, int b, int k, float* G_f32, void* E_bf16, float* ws, hipStream_t st) {
  const int nb = d / b;
  const i64 total = (i64)nb * b * b;
  float* Qf = ws;
  uint16_t* Qb = (uint16_t*)(Qf + total);
  uint16_t* H[2] = {Qb + total, Qb + 2 * total};
  skew_materialize_launch(theta, b, nb, Qf, Qb, nullptr, st);
  if (lds_cnp_supported(d, b)) {   // whole chain in one launch, block resident in LDS
    lds_cnp_build(Qf, Qb, d, k, G_f32, E_bf16, st);
    return;
  }
  const uint16_t* cur = Qb;  // H'_1 = Q
  for (int step = 0; step < k; ++step) {
    const bool last = step == k - 1;
    mm::Args g = batched_args(b);
    g.nsrc = 1;
    set_src(g.s[0], cur, Qb, b);
    uint16_t* nxt = H[step & 1];
    EpiHorner epi{Qf, 2.f, b, last ? nullptr : nxt, last ? G_f32 : nullptr, last ? (uint16_t*)E_bf16 : nullptr};
    launch_product(b, g, epi, nb, st);
    cur = nxt;
  }
}

void mfma_cnp_bwd(const float* theta, const float* dG, int d, int b, int k, float* dtheta, int accumulate, float* ws,
                  hipStream_t st) {
  const int nb = d / b;
  const i64 total = (i64)nb * b * b;
  if (lds_cnp_supported(d, b)) {   // two launches, block resident in LDS; scratch = bf16(Q) + (k + 1) fp32 matrices
    uint16_t* Qb = (uint16_t*)ws;
    skew_materialize_launch(theta, b, nb, nullptr, Qb, nullptr, st);
    const float* dQ = lds_cnp_bwd_chain(Qb, dG, nb, k, ws + total, st);
    skew_project_launch(dQ, b, d, dtheta, accumulate, st);
    return;
  }
  float* Qf = ws;
  uint16_t* Tb = (uint16_t*)(Qf + total);
  skew_materialize_launch(theta, b, nb, Qf, nullptr, Tb, st);
  const float* dQ = mfma_cnp_bwd_chain(Qf, Tb, dG, nb, b, k, Qf + total + total / 2, st);
  skew_project_launch(dQ, b, d, dtheta, accumulate, st);
}

// Tiled two-sided Horner backward for nb blocks (of any sides) given Q in fp32 and T = -Q in
// bf16; ws: 3.5 floats per block element.  Returns dL/dQ (inside ws).
const float* mfma_cnp_bwd_chain(const float* Qf, const uint16_t* Tb, const float* dG, int nb, int b, int k, float* ws,
                                hipStream_t st) {
  const i64 total = (i64)nb * b * b;
  float* Bfinal = ws;
  uint16_t* Db = (uint16_t*)(Bfinal + total);
  uint16_t* A[2] = {Db + total, Db + 2 * total};
  uint16_t* Bb[2] = {Db + 3 * total, Db + 4 * total};
  hipLaunchKernelGGL(to_bf16_kernel, dim3(ceil_div(total / 4, 256)), dim3(256), 0, st, (const float4*)dG, (uint2*)Db,
                     total / 4);
  const uint16_t* acur = Tb;  // A'_1 = T
  const uint16_t* bcur = Db;  // Bm_1 = D
  int ia = 0, ib = 0;
  for (int p = k - 1; p >= 0; --p) {
    const bool last = p == 0;
    mm::Args g = batched_args(b);
    g.nsrc = 2;
    set_src(g.s[0], acur, Db, b);  // A' D
    set_src(g.s[1], bcur, Tb, b);  // Bm T
    if (!last) {                   // second problem of the launch: A' T
      g.alt_from = nb;
      g.alt_nsrc = 1;
      set_src(g.alt[0], acur, Tb, b);
    }
    EpiBwdStep epi{dG, Qf, b, nb, last ? nullptr : Bb[ib], last ? Bfinal : nullptr, last ? nullptr : A[ia]};
    launch_product(b, g, epi, last ? nb : 2 * nb, st);
    if (!last) {
      acur = A[ia];
      ia ^= 1;
      bcur = Bb[ib];
      ib ^= 1;
    }
  }
  return Bfinal;
}

}  // namespace poetx
