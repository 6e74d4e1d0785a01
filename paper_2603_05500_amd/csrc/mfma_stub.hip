// Placeholder: matrix-core kernels not built yet; everything reports unsupported.
#include "poetx_kernels.h"
namespace poetx {
bool mfma_apply_left_supported(int, i64, i64, int) { return false; }
void mfma_apply_left(const void*, void*, int, i64, i64, const int32_t*, const void*, int, int, hipStream_t) {}
bool mfma_blockgrad_supported(int, i64, int) { return false; }
size_t mfma_blockgrad_workspace_bytes(int, i64, int) { return 0; }
void mfma_blockgrad(const void*, const void*, int, i64, const int32_t*, int, float*, void*, hipStream_t) {}
bool mfma_cnp_supported(int) { return false; }
void mfma_cnp_build(const float*, int, int, int, float*, void*, float*, hipStream_t) {}
void mfma_cnp_bwd(const float*, const float*, int, int, int, float*, int, float*, hipStream_t) {}
}
