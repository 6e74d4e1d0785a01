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
// operand stages of ALL its tiles form one stream that flows through a ring of 4 LDS stages,
// filled by direct-to-LDS loads issued that many stages ahead of the multiplication -- across tile
// boundaries, so a new tile starts multiplying the moment the previous one is rounded and stored.
// Per stage there is one barrier, placed after the first of the two k steps, where every wave
// holds the rest of the stage in registers: the stage's slot is refilled at once.  Loads and
// fragment reads are pinned to fixed places between the MFMAs (each wave spreads its loads
// over different places), and the load addresses are a uniform base plus a per-lane offset that
// never changes, so the loop carries no vector address arithmetic.
#include "mfma_dense_kernel.h"

namespace poetx {
namespace {

using namespace dense;

int compute_units() {
  static const int n = [] {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0)
      cu = 256;
    return cu;
  }();
  return n;
}

template <bool A_KMAJOR>
void launch_dense(const DenseArgs& g, hipStream_t st) {
  auto kern = dense_stream_kernel<A_KMAJOR>;
  static const bool configured =
      hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) == hipSuccess;
  (void)configured;
  const int T = g.tiles_m * g.tiles_n, cus = compute_units();
  hipLaunchKernelGGL(kern, dim3(T < cus ? T : cus), dim3(256), LDS_BYTES, st, g);
}

}  // namespace

bool mfma_dense_supported(int n, int m, i64 N) {
  // per-lane load offsets are 32-bit: 255 rows of the wider operand must stay below 4 GB
  return n % BM == 0 && m % BM == 0 && N % BN == 0 && N < (1ll << 22) && (i64)(n > m ? n : m) < (1ll << 22);
}

void mfma_dense(int trans_w, const void* W, int n, int m, const void* act, void* out, i64 N, hipStream_t st) {
  DenseArgs g{};
  g.A = (const uint16_t*)W;
  g.B = (const uint16_t*)act;
  g.C = (uint16_t*)out;
  g.lda = m;
  g.ldb = N;
  g.ldc = N;
  g.tiles_n = (int)(N / BN);
  if (!trans_w) {
    g.tiles_m = n / BM;
    g.ktiles = m / BK;
    launch_dense<true>(g, st);
  } else {
    g.tiles_m = m / BM;
    g.ktiles = n / BK;
    launch_dense<false>(g, st);
  }
}

}  // namespace poetx
