// Dense bf16 products of the POET-X linear layer on the matrix cores:
//   forward  (Eq. 10, mm2):       B  (n x N) = W   (n x m) * A  (m x N)
//   backward (Sec. 3.5, mm2 bwd): dA (m x N) = W^T (m x n) * dB (n x N)   -- no weight gradient
// W is row major n x m; activations are feature major (token index contiguous),
// so the activation operand (and W in the backward product) is contracted over
// its strided index and goes through the transposing LDS read.
#include "mfma_gemm.h"

namespace poetx {
namespace {
constexpr int DBM = 256, DBN = 256, DBK = 64;
}

bool mfma_dense_supported(int n, int m, i64 N) {
  return n % DBM == 0 && m % DBM == 0 && N % DBN == 0 && N < (1ll << 31);
}

void mfma_dense(int trans_w, const void* W, int n, int m, const void* act, void* out, i64 N, hipStream_t st) {
  mm::Args g{};
  g.nsrc = 1;
  g.s[0].A = (const uint16_t*)W;
  g.s[0].B = (const uint16_t*)act;
  g.s[0].lda = m;
  g.s[0].ldb = N;
  g.tiles_n = (int)(N / DBN);
  mm::EpiStoreBf16 epi{(uint16_t*)out, N, 0};
  if (!trans_w) {
    g.tiles_m = n / DBM;
    g.s[0].ktiles = m / DBK;
    mm::launch<DBM, DBN, 2, 4, true, false, false>(g, epi, 1, 1, st);
  } else {
    g.tiles_m = m / DBM;
    g.s[0].ktiles = n / DBK;
    mm::launch<DBM, DBN, 2, 4, false, false, false>(g, epi, 1, 1, st);
  }
}

}  // namespace poetx
