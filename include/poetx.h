/*
 * poetx.h -- C ABI of the MI355X (gfx950) POET-X linear-layer library.
 *
 * The library evaluates the orthogonal equivalence transformation
 *     W_eff = R * W0 * P                                   (paper Sec. 2, Eq. 1)
 * inside a linear layer without ever forming R, P or W_eff.  R (d_in x d_in)
 * and P (d_out x d_out) are block-diagonal matrices of b x b blocks placed
 * under a permutation (Sec. 3, Eq. 2); each block is the truncated
 * Cayley-Neumann series of a skew-symmetric matrix stored as its packed strict
 * upper triangle (Sec. 3.4, Eq. 8).  W0 is frozen.
 *
 * Conventions shared by every call
 * --------------------------------
 *  - m = d_in, n = d_out, N = n_tokens.  The stored weight is W = W0^T, row
 *    major n x m (out x in).
 *  - Activations are FEATURE MAJOR: X is m x N, Z is n x N, row major with the
 *    token index contiguous (leading dimension = N).  This is the column form
 *    of Eq. 4: Z = P^T W R^T X.
 *  - A permutation is an int32 vector pi of length d holding a bijection of
 *    {0..d-1}.  Psi[i, pi[i]] = 1, so (Psi V)[i,:] = V[pi[i],:] and
 *    (Psi^T V)[pi[i],:] = V[i,:]                              (Sec. 3.2, Eq. 5).
 *    R = Psi_R^T Diag(G^0 .. G^{nb-1}) Psi_R, i.e. R[pi[i], pi[j]] = Diag[i, j].
 *  - Blocks: nb = ceil(d / b).  If b does not divide d the last block has side
 *    r = d - b (nb - 1); it is stored as a full b x b block whose rows/columns
 *    >= r are those of the identity.  theta rows always hold b(b-1)/2 floats in
 *    row-major strict-upper-triangle order, Q[i][j] = +theta for i < j; slots
 *    of the tail block with i >= r or j >= r are ignored on input and receive a
 *    zero gradient.
 *  - Block storage.  dtype POETX_F32: blocks are float G[nb][b][b].
 *    dtype POETX_BF16: blocks are bf16 pairs E[nb][2][b][b]: E[j][0] = G_j - I
 *    and E[j][1] = (G_j - I)^T.  The residual keeps the small part of G that
 *    rounding G itself to bf16 would lose (the kernels add the identity back in
 *    fp32); the stored transpose lets both op(G) = G and op(G) = G^T be read as
 *    contiguous rows.  poetx_cnp_build writes either form.
 *  - bf16 buffers hold raw 16-bit patterns (uint16_t); accumulation is fp32.
 *  - All data pointers are DEVICE pointers unless marked host.  `stream` is a
 *    hipStream_t passed as void* (NULL = the null stream).  The caller owns
 *    every buffer; the library allocates no device memory, enqueues its kernels
 *    on `stream` and returns without synchronising (poetx_perm_validate
 *    excepted).  No call leaves anything behind that a later call depends on;
 *    the only process-wide state is the two diagnostic switches
 *    (poetx_debug_force_fma, poetx_profile_begin/end, both off by default), the
 *    static scratch of poetx_cnp_build_static, and once-only kernel attributes.
 *    `ws` is scratch of at least the size the matching *_workspace_bytes call
 *    reports, 256-byte aligned.
 *  - Alignment: bf16 tensors, block storage and workspaces should be 16-byte aligned
 *    with leading dimensions that are multiples of 8 elements (what any device
 *    allocator gives).  The matrix-core kernels move 16 bytes per lane; a call
 *    whose pointers are not so aligned runs on the plain fp32-FMA kernels.
 *  - Which kernels serve a shape: the matrix-core kernels cover bf16 tensors with
 *    b = 256 or 512 dividing d_in and d_out, dimensions that are multiples of 256
 *    and token counts that are multiples of 256, and, for fp32 tensors, the two dense
 *    products when all three dimensions are multiples of 128 (fp32 MFMA); everything
 *    else (the structured stages and the series of fp32 tensors, small blocks, ragged
 *    tails) runs on plain fp32-FMA kernels, correct but one to two orders of magnitude
 *    slower at large sizes.  poetx_linear_path reports the
 *    choice for a descriptor, so a caller can refuse shapes that would fall off
 *    the fast path instead of finding out from the clock.
 *  - Output buffers must not overlap input buffers (in-place operation is refused:
 *    the kernels of one call read rows that other workgroups of the same call write).
 *  - Return value: POETX_OK (0) or a poetx_status error.  Arguments are checked
 *    on the host before anything is enqueued; on error nothing was launched.
 *    Permutation contents are NOT checked on the hot path (use
 *    poetx_perm_validate); an out-of-range index is undefined behaviour.
 */
#ifndef POETX_H_
#define POETX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  POETX_OK = 0,
  POETX_ERR_INVALID_ARG = 1,   /* null pointer, non-positive size, bad enum     */
  POETX_ERR_BAD_SHAPE = 2,     /* sizes inconsistent with each other            */
  POETX_ERR_BAD_PERM = 3,      /* poetx_perm_validate: not a bijection          */
  POETX_ERR_UNSUPPORTED = 4,   /* valid request this build has no kernel for    */
  POETX_ERR_WORKSPACE = 5,     /* ws is null or smaller than required           */
  POETX_ERR_HIP = 6            /* a HIP runtime call or launch failed           */
} poetx_status;

typedef enum { POETX_F32 = 0, POETX_BF16 = 1 } poetx_dtype;

/* Layout of the activations a caller hands to the poetx_linear_* calls (X, Z, dZ, dX).
 * FEATURE_MAJOR ([d][N], the library's native layout: the feature permutation of Eq. 5 is then a
 * gather of whole rows, fused into the block kernels at no cost).  TOKEN_MAJOR ([N][d], what a
 * framework usually holds): every such tensor is re-laid by one transposing pass through LDS on
 * its way in or out (feature-major copies live in the workspace, which grows accordingly); all
 * values are bit for bit those of the feature-major call.  saved_B, dA and the block gradients keep
 * their layouts in both modes. */
typedef enum { POETX_FEATURE_MAJOR = 0, POETX_TOKEN_MAJOR = 1 } poetx_layout;

/* How the block products of the Cayley-Neumann chain are multiplied.
 * FP32: plain fp32 arithmetic.  BF16X1: operands rounded to bf16, fp32
 * accumulation on the matrix cores (meets the bf16 tolerance, not the fp32 one). */
typedef enum { POETX_CNP_FP32 = 0, POETX_CNP_BF16 = 1 } poetx_cnp_precision;

/* One POET-X linear layer (Sec. 3.5, Eq. 10). */
typedef struct {
  int32_t d_in;        /* m */
  int32_t d_out;       /* n */
  int32_t block;       /* b, side of the orthogonal blocks                    */
  int32_t neumann_k;   /* k: highest power kept in (I - Q)^-1 ~ sum_{i<=k} Q^i */
  int64_t n_tokens;    /* N */
  int32_t dtype;       /* poetx_dtype of X, W, Z, saved B, gradients, blocks   */
  int32_t cnp_precision; /* poetx_cnp_precision used by poetx_linear_bwd_skew  */
  int32_t flags;       /* POETX_FLAG_* bits                                    */
  int32_t layout;      /* poetx_layout of X, Z, dZ, dX (0 = feature major)     */
} poetx_linear_desc;

/* Memory-saving variant (Sec. 3.5, POET-X_mem): the forward pass keeps no activation
 * (poetx_linear_fwd is called with saved_B = NULL and holds B in the workspace only) and the
 * backward pass recomputes A = R^T X and B = W A: poetx_linear_bwd does so itself when it is called
 * with saved_B = NULL (B then lives at the end of the workspace), and poetx_linear_recompute_b does it
 * for callers of the two halves, before poetx_linear_bwd_skew.  The flag sizes the workspace for that. */
#define POETX_FLAG_RECOMPUTE_B 1

/* Quantised base weight (Sec. 3.6, POET-XQ): the frozen W is stored as signed 8-bit codes and
 * dequantised whenever it is needed, so no high-precision weight persists.  The paper does not
 * state its quantisation scheme; this library uses symmetric absmax codes per output row:
 *   scale_i = max_k |W[i][k]| / 127 (1 for an all-zero row),
 *   q[i][k] = round-half-even(W[i][k] / scale_i) clamped to [-127, 127]   (decided in fp32),
 *   W[i][k] ~ scale_i * q[i][k].
 * A quantised weight buffer is int8 q[n][m] row major followed, at byte offset
 * (n*m rounded up to 256), by float scale[n]; poetx_weight_q8_bytes gives its size.
 * With this flag the W argument of poetx_linear_fwd, poetx_linear_recompute_b,
 * poetx_linear_bwd_input and poetx_linear_bwd is such a buffer.  Each call dequantises it into its
 * workspace (one n x m weight of the layer's dtype more, transient like the rest of the workspace) ahead
 * of its dense products -- once per call: poetx_linear_bwd with saved_B = NULL uses the one copy for
 * the recomputation of B and for dA = W^T dB.  That pass moves 3 bytes per weight element and is the
 * fastest way through (about 2 % over the plain memory-saving variant at 16384 tokens).
 * As in the paper the flag is only valid together with POETX_FLAG_RECOMPUTE_B (the variant that
 * keeps no activation); alone it is POETX_ERR_INVALID_ARG. */
#define POETX_FLAG_W_INT8 2

/* With POETX_FLAG_W_INT8: the dense products read the codes themselves, for bf16 layers whose
 * dimensions are multiples of 256 (other shapes and fp32 layers ignore the flag).  Code tiles and row
 * scales stream into LDS and are converted to bf16(scale * q) there, two stages ahead of the
 * multiplication, so no high-precision weight is ever written to memory and the workspace is that of
 * the plain memory-saving variant -- for callers to whom one weight's worth of workspace matters more
 * than the conversion work, which makes these products about 20 % slower.  The values are the same
 * bit for bit either way.  Without POETX_FLAG_W_INT8 the flag is POETX_ERR_INVALID_ARG. */
#define POETX_FLAG_W_INT8_FUSED 8

/* Deferred series backward: poetx_linear_bwd_skew and poetx_linear_bwd stop after the block
 * gradients (Sec. 3.5: dG_P^j = B'_j dZ'_j^T, dG_R^j = X'_j dA'_j^T) and write them where they
 * would have written the parameter gradients: dtheta_R / dtheta_P are then float [ceil(m/b)][b][b] /
 * [ceil(n/b)][b][b] buffers (overwritten; `accumulate` is ignored).  poetx_cnp_bwd turns block
 * gradients into parameter gradients for any batch of blocks, so one call can serve all
 * projections of a layer -- the chains of a single projection leave most of the GPU idle. */
#define POETX_FLAG_BLOCK_GRADS 4

const char* poetx_status_string(int status);

/* Library version (major * 100 + minor). */
int poetx_version(void);

/* Test hook (process-wide, not for production use): on != 0 routes every call,
 * whatever its dtype, through the plain fp32-FMA kernels instead of the
 * matrix-core kernels, so that the two kernel families can be compared. */
void poetx_debug_force_fma(int on);

/* Stage timing for benchmarks (process-wide; off unless begun).  Between
 * poetx_profile_begin and poetx_profile_end every group of kernels an entry
 * point enqueues is bracketed by HIP events on the caller's stream (at most
 * max_records groups; later ones are not timed).  poetx_profile_end waits for
 * the recorded events and returns, per stage, the summed elapsed milliseconds
 * and the number of timed groups; both arrays are HOST arrays of
 * POETX_STAGE_COUNT entries. */
typedef enum {
  POETX_STAGE_CNP_FWD = 0,    /* skew + Cayley-Neumann series                    */
  POETX_STAGE_APPLY = 1,      /* gather + block-diagonal product + scatter       */
  POETX_STAGE_DENSE = 2,      /* B = W A and dA = W^T dB                         */
  POETX_STAGE_BLOCKGRAD = 3,  /* per-block token reduction dG                    */
  POETX_STAGE_CNP_BWD = 4,    /* series backward + packed projection             */
  POETX_STAGE_APPLY_GRAD = 5, /* poetx_linear_bwd: structured product and block gradient of a side in one pass */
  POETX_STAGE_LAYOUT = 6,     /* token-major <-> feature-major passes            */
  POETX_STAGE_DEQUANT = 7,    /* INT8 weight dequantised into the workspace */
  POETX_STAGE_COUNT = 8
} poetx_stage;
int poetx_profile_begin(int32_t max_records);
int poetx_profile_end(double* ms_by_stage, int64_t* launches_by_stage);

/* ---------------------------------------------------------------------------
 * skew_symmetric + cayley_neumann (Sec. 3.4, Eq. 8-9), batched over blocks:
 *   Q_j = skew(theta_j),  G_j = (I + Q_j)(I + Q_j + ... + Q_j^k)
 *       = I + 2 sum_{p=1..k} Q_j^p + Q_j^{k+1}.
 * theta : [nb][b(b-1)/2] float, nb = ceil(d / b); d gives the ragged tail.
 * G_f32 : [nb][b][b] float, nullable.   E_bf16 : [nb][2][b][b] bf16 pairs
 * (G - I, its transpose), nullable (at least one must be given).
 * ws    : poetx_cnp_workspace_bytes(d, b) bytes.
 */
size_t poetx_cnp_workspace_bytes(int32_t d, int32_t b);
int poetx_cnp_build(const float* theta, int32_t d, int32_t b, int32_t k, int32_t precision,
                    float* G_f32, void* E_bf16, void* ws, size_t ws_bytes, void* stream);

/* The same call for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): it takes no workspace and calls no
 * allocating routine.  The scratch is an array inside the library, resident on every GPU the
 * library runs on until the process ends (12 * POETX_CNP_STATIC_MAX_ELEMS bytes = 48 MiB); its
 * per-device address is looked up on the first call on that device.  Requests with
 * ceil(d/b) * b * b > POETX_CNP_STATIC_MAX_ELEMS return POETX_ERR_UNSUPPORTED.  All calls on one
 * GPU share that GPU's array (it keeps the last call's contents; the kernels write every element
 * before reading it, so nothing is cleared): calls that overlap in time on one GPU race -- keep
 * them on one stream or order them yourself.  Results are those of poetx_cnp_build bit for bit. */
#define POETX_CNP_STATIC_MAX_ELEMS (1u << 22)   /* e.g. d = 16384 at b = 256, d = 8192 at b = 512 */
int poetx_cnp_build_static(const float* theta, int32_t d, int32_t b, int32_t k, int32_t precision,
                           float* G_f32, void* E_bf16, void* stream);

/* Backward of skew_symmetric + cayley_neumann (the Sec. 3.4 backward display, for any k), batched
 * over blocks: dG [nb][b][b] float = dL/dG -> dtheta [nb][b(b-1)/2] float, overwritten when
 * accumulate == 0 and added to otherwise; theta, d, b, k, precision as in poetx_cnp_build (the
 * blocks may be those of several sides or projections laid end to end when b divides each of
 * their dimensions).  ws: poetx_cnp_bwd_workspace_bytes(d, b, k) bytes. */
size_t poetx_cnp_bwd_workspace_bytes(int32_t d, int32_t b, int32_t k);
int poetx_cnp_bwd(const float* theta, const float* dG, int32_t d, int32_t b, int32_t k, int32_t precision,
                  float* dtheta, int32_t accumulate, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * INT8 codes of a base weight (Sec. 3.6; scheme and buffer layout: see POETX_FLAG_W_INT8).
 * W: n x m in `dtype`.  Wq: poetx_weight_q8_bytes(n, m) bytes (out of quantize, in of
 * dequantize).  W_out: n x m in `dtype`, scale_i * q[i][k] rounded once to that type.
 */
size_t poetx_weight_q8_bytes(int32_t n, int32_t m);
int poetx_weight_quantize_q8(const void* W, int32_t dtype, int32_t n, int32_t m, void* Wq, void* stream);
int poetx_weight_dequantize_q8(const void* Wq, int32_t n, int32_t m, int32_t dtype, void* W_out, void* stream);

/* ---------------------------------------------------------------------------
 * Structured apply without materialising the orthogonal matrix (Eq. 2 with
 * Eq. 5 and Eq. 7):
 *   left :  out = Psi^T Diag(op(G)) Psi * V,   V and out are d x cols, leading
 *           dimension ld >= cols (elements).          (R V, R^T X, P dZ, ...)
 *   right:  out = V * Psi^T Diag(op(G)) Psi,   V and out are rows x d, leading
 *           dimension ld >= d.                        (W0 P, the merge R W0 P)
 * op(G) = G^T when transpose_G != 0.  `blocks` is G (float) or E (bf16) as the
 * dtype says.  perm has d entries.  out must not alias V.
 */
int poetx_perm_blockdiag_apply_left(const void* V, void* out, int32_t d, int64_t cols, int64_t ld,
                                    const int32_t* perm, const void* blocks, int32_t b,
                                    int32_t transpose_G, int32_t dtype, void* stream);
int poetx_perm_blockdiag_apply_right(const void* V, void* out, int64_t rows, int32_t d, int64_t ld,
                                     const int32_t* perm, const void* blocks, int32_t b,
                                     int32_t transpose_G, int32_t dtype, void* stream);

/* Merge step of the outer loop (Sec. 3, after Eq. 2: every few hundred steps the learned factors are
 * folded into the base weight, W <- R W0 P in the paper's orientation, and the parameters reset).
 * On the stored weight W = W0^T (n x m, row major): W_out = P^T W R^T, the same result as
 * poetx_perm_blockdiag_apply_left (P side, transpose) followed by poetx_perm_blockdiag_apply_right
 * (R side, transpose), but with the input-side product run as a row gather on the transposed matrix,
 * so that both sides use the streaming kernels.  W_out must not overlap W.
 * ws: poetx_merge_workspace_bytes(n, m, dtype) bytes (two weight-sized buffers). */
size_t poetx_merge_workspace_bytes(int32_t n, int32_t m, int32_t dtype);
int poetx_merge_weight(const void* W, void* W_out, int32_t n, int32_t m,
                       const int32_t* perm_R, const int32_t* perm_P,
                       const void* blocks_R, const void* blocks_P, int32_t b, int32_t dtype,
                       void* ws, size_t ws_bytes, void* stream);

/* Debug helper: checks on the device that perm is a bijection of {0..d-1}.
 * scratch: d + 1 int32 on the device.  Synchronises `stream`. */
int poetx_perm_validate(const int32_t* perm, int32_t d, int32_t* scratch, void* stream);

/* ---------------------------------------------------------------------------
 * The linear layer, input-centric (Eq. 3, Eq. 4, Eq. 10).  Because gather and
 * scatter are folded into the block kernels, W is used as stored (the
 * pre-permuted W' of Eq. 6 is not needed) and all activations keep physical
 * feature order:
 *   forward : A = R^T X (mm1),  B = W A (mm2),  Z = P^T B (mm3)
 *   backward: dB = P dZ,  dA = W^T dB  (no weight gradient),  dX = R dA
 *             dG_P^j = B'_j dZ'_j^T, dG_R^j = X'_j dA'_j^T  (primes: rows
 *             gathered by the side's permutation), then the chain rule through
 *             the series and the projection onto the packed parameters.
 * poetx_linear_workspace_bytes: scratch needed by the largest of the linear calls.
 */
size_t poetx_linear_workspace_bytes(const poetx_linear_desc* desc);

/* Which kernel families would serve `desc` (bit set = matrix cores; 16-byte aligned pointers
 * assumed).  Returns a combination of POETX_PATH_* bits, 0 when every stage runs on the plain
 * fp32-FMA kernels, or minus a poetx_status when the descriptor is invalid. */
#define POETX_PATH_APPLY 1              /* gather + block-diagonal product + scatter            */
#define POETX_PATH_DENSE 2              /* B = W A, dA = W^T dB (the only bit fp32 tensors get) */
#define POETX_PATH_BLOCKGRAD 4          /* block gradients (two-call backward)                 */
#define POETX_PATH_SERIES 8             /* series backward on the matrix cores                 */
#define POETX_PATH_SERIES_ON_CHIP 16    /* ... as one-launch chains with the block in LDS      */
#define POETX_PATH_BWD_ONE_PASS 32      /* poetx_linear_bwd streams each side's gradient once  */
#define POETX_PATH_W_INT8_IN_KERNEL 64  /* POETX_FLAG_W_INT8_FUSED honoured: codes converted inside the dense kernels */
int poetx_linear_path(const poetx_linear_desc* desc);

/* X: m x N.  W: n x m.  blocks_R / blocks_P: block storage of the dtype (see top)
 * with ceil(m/b) and ceil(n/b) blocks.
 * Z: n x N (out).  saved_B: n x N (out; the one activation the fast variant
 * keeps for the backward pass, physical feature order).  saved_B may be NULL only
 * when desc->flags has POETX_FLAG_RECOMPUTE_B.  With POETX_FLAG_W_INT8, W is a quantised
 * weight buffer (also in poetx_linear_recompute_b and poetx_linear_bwd_input). */
int poetx_linear_fwd(const poetx_linear_desc* desc, const void* X, const void* W,
                     const int32_t* perm_R, const int32_t* perm_P,
                     const void* blocks_R, const void* blocks_P,
                     void* Z, void* saved_B, void* ws, size_t ws_bytes, void* stream);

/* Gradient-checkpoint step of the memory-saving variant: B_out (n x N) = W (R^T X), the same
 * values poetx_linear_fwd would have saved (same kernels, same rounding). */
int poetx_linear_recompute_b(const poetx_linear_desc* desc, const void* X, const void* W,
                             const int32_t* perm_R, const void* blocks_R, void* B_out,
                             void* ws, size_t ws_bytes, void* stream);

/* dZ: n x N.  dX: m x N (out).  dA: m x N (out; W^T P dZ in physical order,
 * consumed by poetx_linear_bwd_skew). */
int poetx_linear_bwd_input(const poetx_linear_desc* desc, const void* dZ, const void* W,
                           const int32_t* perm_R, const int32_t* perm_P,
                           const void* blocks_R, const void* blocks_P,
                           void* dX, void* dA, void* ws, size_t ws_bytes, void* stream);

/* Gradients on the packed skew parameters of both sides (Sec. 3.4 backward
 * display generalised to any k; Sec. 3.5 mm1/mm3 backward).
 * theta_R: [ceil(m/b)][b(b-1)/2] float, theta_P likewise for n.
 * dtheta_R / dtheta_P: same shapes (out); overwritten when accumulate == 0,
 * added to otherwise. */
int poetx_linear_bwd_skew(const poetx_linear_desc* desc, const void* X, const void* dZ,
                          const void* saved_B, const void* dA,
                          const int32_t* perm_R, const int32_t* perm_P,
                          const float* theta_R, const float* theta_P,
                          float* dtheta_R, float* dtheta_P, int32_t accumulate,
                          void* ws, size_t ws_bytes, void* stream);

/* The whole backward pass in one call (Sec. 3.5, all three bullets, then Sec. 3.4 backward): the
 * results of poetx_linear_bwd_input followed by poetx_linear_bwd_skew, with dA kept in the workspace.
 * Where the shapes allow (bf16, b = 256, d_in, d_out multiples of 256, n_tokens a multiple of 256) each
 * side's gradient is streamed from memory once: dB = P dZ is produced together with
 * dG_P^j = B'_j dZ'_j^T, and dX = R dA together with dG_R^j = X'_j dA'_j^T, instead of one pass
 * for the product and another for the block gradient.  Otherwise it runs the two halves as they are.
 * The block gradients are summed over token ranges in a fixed order, so results are reproducible
 * run to run; they differ from the two-call results only by that summation order.
 * Arguments as in the two halves; W follows desc->flags (POETX_FLAG_W_INT8).  saved_B may be NULL when
 * desc->flags has POETX_FLAG_RECOMPUTE_B: the call then recomputes B = W (R^T X) first, with the kernels
 * and the rounding of poetx_linear_fwd, so every result is the one poetx_linear_recompute_b followed by
 * this call would give, bit for bit. */
int poetx_linear_bwd(const poetx_linear_desc* desc, const void* X, const void* dZ, const void* saved_B,
                     const void* W, const int32_t* perm_R, const int32_t* perm_P,
                     const void* blocks_R, const void* blocks_P,
                     const float* theta_R, const float* theta_P,
                     void* dX, float* dtheta_R, float* dtheta_P, int32_t accumulate,
                     void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* POETX_H_ */
