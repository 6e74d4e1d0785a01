// Internal launch interface between the C-ABI layer and the kernel files.
// Every launcher enqueues on `st` and returns; shapes were validated by the caller.
#pragma once

#include "poetx_common.h"

namespace poetx {

// Brackets the launches of one stage with HIP events when stage profiling is on.
class StageTimer {
 public:
  StageTimer(int stage, hipStream_t st);
  ~StageTimer();
 private:
  hipStream_t st_;
  long idx_;
};

// ---- plain fp32-FMA path (fma_kernels.hip): any dtype, any block size ---------------
// out = op(W) * act:  W is n x m row major.  trans_w == 0: out (n x N) = W act (m x N);
// trans_w == 1: out (m x N) = W^T act (n x N).
void fma_dense(int dtype, int trans_w, const void* W, int n, int m, const void* act, void* out,
               i64 N, hipStream_t st);
void fma_apply_left(int dtype, const void* V, void* out, int d, i64 cols, i64 ld, const int32_t* perm,
                    const void* blocks, int b, int transpose_G, hipStream_t st);
void fma_apply_right(int dtype, const void* V, void* out, i64 rows, int d, i64 ld, const int32_t* perm,
                     const void* blocks, int b, int transpose_G, hipStream_t st);
// dG[j] = U'_j V'_j^T with rows of U and V (d x N each) gathered by perm; dG is [nb][b][b] float.
void fma_blockgrad(int dtype, const void* U, const void* V, int d, i64 N, const int32_t* perm, int b,
                   float* dG, hipStream_t st);
// ws: 2 * nb*b*b floats.
void fma_cnp_build(const float* theta, int d, int b, int k, float* G_f32, void* E_bf16, float* ws,
                   hipStream_t st);
// dG -> dtheta.  ws: 4 * nb*b*b floats.
void fma_cnp_bwd(const float* theta, const float* dG, int d, int b, int k, float* dtheta, int accumulate,
                 float* ws, hipStream_t st);

// dtheta[j][idx(i,c)] (+)= M[j][i][c] - M[j][c][i] (Sec. 3.4: gradient on the packed parameters).
void skew_project_launch(const float* M, int b, int d, float* dtheta, int accumulate, hipStream_t st);

// ---- INT8 base weight (weight_q8.hip): codes [n][m] then, 256-byte aligned, float scale[n]
size_t weight_q8_scale_offset(int n, int m);
void weight_quantize_q8_launch(int dtype, const void* W, int n, int m, void* Wq, hipStream_t st);
void weight_dequantize_q8_launch(const void* Wq, int n, int m, int dtype, void* W_out, hipStream_t st);

// out (C x R) = in (R x C)^T, both row major and dense (layout.hip)
void transpose_launch(int dtype, const void* in, void* out, i64 R, i64 C, hipStream_t st);

void perm_validate_launch(const int32_t* perm, int d, int32_t* scratch, hipStream_t st);

// ---- matrix-core path for bf16 (mfma_*.hip) -------------------------------------------
bool mfma_dense_supported(int n, int m, i64 N);
void mfma_dense(int trans_w, const void* W, int n, int m, const void* act, void* out, i64 N,
                hipStream_t st);
// the same products for fp32 tensors (fp32 MFMA, mfma_dense_f32.hip)
bool mfma_dense_f32_supported(int n, int m, i64 N);
void mfma_dense_f32(int trans_w, const void* W, int n, int m, const void* act, void* out, i64 N, hipStream_t st);
// the same products on a quantised weight buffer (codes + row scales), dequantised inside the kernel (mfma_dense_q8.hip)
bool mfma_dense_q8_supported(int n, int m, i64 N);
void mfma_dense_q8(int trans_w, const void* Wq, int n, int m, const void* act, void* out, i64 N, hipStream_t st);
bool mfma_apply_left_supported(int d, i64 cols, i64 ld, int b);
void mfma_apply_left(const void* V, void* out, int d, i64 cols, i64 ld, const int32_t* perm,
                     const void* E, int b, int transpose_G, hipStream_t st);
bool mfma_blockgrad_supported(int d, i64 N, int b);
size_t mfma_blockgrad_workspace_bytes(int d, i64 N, int b);
void mfma_blockgrad(const void* U, const void* V, int d, i64 N, const int32_t* perm, int b, float* dG,
                    void* ws, hipStream_t st);
// One pass over the incoming gradient V (d x N) for one side (mfma_applygrad.hip, b = 256):
// out = Psi^T Diag(op(G)) Psi V and dG[j] = U'_j V'_j^T (rows gathered by perm).  ws: the bytes the
// query reports (partial block gradients of the token ranges).
bool mfma_apply_grad_supported(int d, i64 N, i64 ld, int b);
size_t mfma_apply_grad_workspace_bytes(int d, i64 N);
void mfma_apply_grad(const void* V, const void* U, void* out, int d, i64 N, i64 ld, const int32_t* perm, const void* E,
                     int transpose_G, float* dG, void* ws, hipStream_t st);
bool mfma_cnp_supported(int d, int b);
void mfma_cnp_build(const float* theta, int d, int b, int k, float* G_f32, void* E_bf16, float* ws,
                    hipStream_t st);
void mfma_cnp_bwd(const float* theta, const float* dG, int d, int b, int k, float* dtheta, int accumulate,
                  float* ws, hipStream_t st);
// b = 256: whole chain of a block in one launch, block resident in LDS (mfma_cnp_lds.hip).
// Qf / Qb: Q in fp32 / bf16, [nb][b][b].  The backward needs (k + 1) * nb*b*b floats of scratch.
bool lds_cnp_supported(int d, int b);
void lds_cnp_build(const float* Qf, const uint16_t* Qb, int d, int k, float* G_f32, void* E_bf16, hipStream_t st);
// dL/dG of nb blocks -> dL/dQ (returned pointer lies inside ws); the blocks may belong to
// several sides, the chain does not care.
const float* lds_cnp_bwd_chain(const uint16_t* Qb, const float* dG, int nb, int k, float* ws, hipStream_t st);
// Q of nb blocks from packed parameters: Qf fp32 and/or Qb bf16, [nb][b][b] (either may be null).
// Tb = bf16(-Q).
void skew_materialize_launch(const float* theta, int b, i64 nb, float* Qf, uint16_t* Qb, uint16_t* Tb, hipStream_t st);
// skew_tiled.hip: the same two operations through 64 x 64 tiles (coalesced on both sides of the transpose)
bool skew_tiled_supported(int b, i64 d);
void skew_materialize_tiled_launch(const float* theta, int b, i64 nb, float* Qf, uint16_t* Qb, uint16_t* Tb, hipStream_t st);
void skew_project_tiled_launch(const float* M, int b, i64 nb, float* dtheta, int accumulate, hipStream_t st);
// Series backward on the tiled kernels (b = 512) for nb blocks: Qf fp32, Tb = bf16(-Q); ws holds
// 3.5 floats per block element; returns dL/dQ (inside ws).
const float* mfma_cnp_bwd_chain(const float* Qf, const uint16_t* Tb, const float* dG, int nb, int b, int k, float* ws,
                                hipStream_t st);

}  // namespace poetx
