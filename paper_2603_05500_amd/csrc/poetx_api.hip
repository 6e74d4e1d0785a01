// C-ABI entry points: host-side argument checks and kernel dispatch.
// Every step of the path runs in the kernels of this library; this file only
// validates, carves the workspace and enqueues.
#include <atomic>
#include <mutex>

#include "poetx_kernels.h"

using namespace poetx;

namespace {

std::atomic<int> g_force_fma{0};

// ---- scratch of the entry point that allocates nothing (poetx_cnp_build_static) ------------
// One copy of this array lives on every GPU the library runs on, for as long as the process
// lives.  Its name is only a host-side handle: kernels get the per-device address that
// hipGetSymbolAddress returns, looked up once per device with that device current.
constexpr size_t kStaticCnpElems = POETX_CNP_STATIC_MAX_ELEMS;           // block elements: ceil(d/b) * b * b
constexpr size_t kStaticCnpBytes = 12 * kStaticCnpElems;                 // poetx_cnp_workspace_bytes per element
static __device__ __align__(256) unsigned char scratch[kStaticCnpBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return POETX_ERR_HIP;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return POETX_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return POETX_OK;
}

inline bool use_mfma(int dtype) { return dtype == POETX_BF16 && !g_force_fma.load(); }
// the matrix-core kernels move 16 bytes per lane: every tensor they touch must be 16-byte aligned
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
inline size_t esize(int dtype) { return dtype == POETX_F32 ? 4 : 2; }
inline bool dtype_ok(int dtype) { return dtype == POETX_F32 || dtype == POETX_BF16; }
inline bool overlap(const void* a, size_t na, const void* b, size_t nb) {
  const char* x = (const char*)a;
  const char* y = (const char*)b;
  return x < y + nb && y < x + na;
}

int check_desc(const poetx_linear_desc* d) {
  if (!d) return POETX_ERR_INVALID_ARG;
  if (d->d_in <= 0 || d->d_out <= 0 || d->block <= 0 || d->neumann_k < 1 || d->n_tokens <= 0)
    return POETX_ERR_INVALID_ARG;
  if (!dtype_ok(d->dtype)) return POETX_ERR_INVALID_ARG;
  if (d->cnp_precision != POETX_CNP_FP32 && d->cnp_precision != POETX_CNP_BF16) return POETX_ERR_INVALID_ARG;
  if ((d->flags & ~(POETX_FLAG_RECOMPUTE_B | POETX_FLAG_W_INT8 | POETX_FLAG_BLOCK_GRADS | POETX_FLAG_W_INT8_FUSED)) != 0 || (d->layout != POETX_FEATURE_MAJOR && d->layout != POETX_TOKEN_MAJOR))
    return POETX_ERR_INVALID_ARG;
  if ((d->flags & POETX_FLAG_W_INT8) && !(d->flags & POETX_FLAG_RECOMPUTE_B)) return POETX_ERR_INVALID_ARG;
  if ((d->flags & POETX_FLAG_W_INT8_FUSED) && !(d->flags & POETX_FLAG_W_INT8)) return POETX_ERR_INVALID_ARG;
  if (d->block > d->d_in || d->block > d->d_out) return POETX_ERR_BAD_SHAPE;
  if (d->n_tokens >= (1ll << 31) || (i64)d->n_tokens * (d->d_in > d->d_out ? d->d_in : d->d_out) >= (1ll << 40))
    return POETX_ERR_UNSUPPORTED;
  return POETX_OK;
}

// dG plus chain scratch per block element: five floats cover the tiled kernel families, the
// on-chip chain keeps bf16(Q), k transposed terms and the result (k + 2 floats)
size_t cnp_bwd_ws_floats(int d, int b, int k) {
  const size_t per_elem = 1 + (size_t)(k + 2 > 5 ? k + 2 : 5);
  return per_elem * ceil_div(d, b) * b * b;
}
// The same when both sides of a layer go through the series backward together.
size_t cnp_bwd_ws_floats_both(int m, int n, int b, int k) {
  const size_t per_elem = (size_t)(k + 3 > 6 ? k + 3 : 6);   // tiled kernels: dG, Q, -Q (half), 3.5 of chain
  return per_elem * (ceil_div(m, b) + ceil_div(n, b)) * b * b;
}

void apply_left_dispatch(int dtype, const void* V, void* out, int d, i64 cols, i64 ld, const int32_t* perm,
                         const void* blocks, int b, int trans, hipStream_t st) {
  StageTimer tm(POETX_STAGE_APPLY, st);
  if (use_mfma(dtype) && mfma_apply_left_supported(d, cols, ld, b) && aligned16(V) && aligned16(out) && aligned16(blocks))
    mfma_apply_left(V, out, d, cols, ld, perm, blocks, b, trans, st);
  else
    fma_apply_left(dtype, V, out, d, cols, ld, perm, blocks, b, trans, st);
}

// w_q8: W is a quantised weight buffer that the product dequantises itself (see weight_in_kernel)
void dense_dispatch(int dtype, int trans_w, const void* W, int n, int m, const void* act, void* out, i64 N,
                    hipStream_t st, bool w_q8 = false) {
  StageTimer tm(POETX_STAGE_DENSE, st);
  if (w_q8) mfma_dense_q8(trans_w, W, n, m, act, out, N, st);
  else if (use_mfma(dtype) && mfma_dense_supported(n, m, N) && aligned16(W) && aligned16(act) && aligned16(out))
    mfma_dense(trans_w, W, n, m, act, out, N, st);
  else if (dtype == POETX_F32 && !g_force_fma.load() && mfma_dense_f32_supported(n, m, N) && aligned16(W) && aligned16(act) && aligned16(out))
    mfma_dense_f32(trans_w, W, n, m, act, out, N, st);
  else fma_dense(dtype, trans_w, W, n, m, act, out, N, st);
}

// POET-XQ: do the dense kernels read the 8-bit weight directly (conversion inside the operand path; asked for
// with POETX_FLAG_W_INT8_FUSED)?  Otherwise the weight is dequantised into the workspace before the products.
bool weight_in_kernel(const poetx_linear_desc* d) {
  return (d->flags & POETX_FLAG_W_INT8) && (d->flags & POETX_FLAG_W_INT8_FUSED) && use_mfma(d->dtype) && mfma_dense_q8_supported(d->d_out, d->d_in, d->n_tokens);
}

size_t blockgrad_ws_bytes(int dtype, int d, i64 N, int b) {
  if (dtype == POETX_BF16 && mfma_blockgrad_supported(d, N, b)) return align256(mfma_blockgrad_workspace_bytes(d, N, b));
  return 0;
}

}  // namespace

extern "C" {

const char* poetx_status_string(int s) {
  switch (s) {
    case POETX_OK: return "ok";
    case POETX_ERR_INVALID_ARG: return "invalid argument";
    case POETX_ERR_BAD_SHAPE: return "inconsistent shapes";
    case POETX_ERR_BAD_PERM: return "not a permutation";
    case POETX_ERR_UNSUPPORTED: return "unsupported configuration";
    case POETX_ERR_WORKSPACE: return "workspace missing or too small";
    case POETX_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int poetx_version(void) { return 100; }

// Test hook: path != 0 forces the plain fp32-FMA kernels for every dtype.
void poetx_debug_force_fma(int on) { g_force_fma.store(on ? 1 : 0); }

size_t poetx_cnp_workspace_bytes(int32_t d, int32_t b) {
  if (d <= 0 || b <= 0) return 0;
  return align256((size_t)3 * ceil_div(d, b) * b * b * sizeof(float));  // covers both kernel families
}

int poetx_cnp_build(const float* theta, int32_t d, int32_t b, int32_t k, int32_t precision, float* G_f32,
                    void* E_bf16, void* ws, size_t ws_bytes, void* stream) {
  if (!theta || (!G_f32 && !E_bf16) || d <= 0 || b <= 0 || k < 1) return POETX_ERR_INVALID_ARG;
  if (precision != POETX_CNP_FP32 && precision != POETX_CNP_BF16) return POETX_ERR_INVALID_ARG;
  if (b > d) return POETX_ERR_BAD_SHAPE;
  if (!ws || ws_bytes < poetx_cnp_workspace_bytes(d, b)) return POETX_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  StageTimer tm(POETX_STAGE_CNP_FWD, st);
  if (precision == POETX_CNP_BF16 && !g_force_fma.load() && mfma_cnp_supported(d, b))
    mfma_cnp_build(theta, d, b, k, G_f32, E_bf16, (float*)ws, st);
  else
    fma_cnp_build(theta, d, b, k, G_f32, E_bf16, (float*)ws, st);
  return launch_status();
}

int poetx_cnp_build_static(const float* theta, int32_t d, int32_t b, int32_t k, int32_t precision, float* G_f32,
                           void* E_bf16, void* stream) {
  if (!theta || (!G_f32 && !E_bf16) || d <= 0 || b <= 0 || k < 1) return POETX_ERR_INVALID_ARG;
  if (precision != POETX_CNP_FP32 && precision != POETX_CNP_BF16) return POETX_ERR_INVALID_ARG;
  if (b > d) return POETX_ERR_BAD_SHAPE;
  if ((size_t)ceil_div(d, b) * b * b > kStaticCnpElems) return POETX_ERR_UNSUPPORTED;   // beyond the static scratch
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != POETX_OK) return rc;
  // every scratch element the kernels read was written earlier in the same call: nothing to clear
  return poetx_cnp_build(theta, d, b, k, precision, G_f32, E_bf16, ws, kStaticCnpBytes, stream);
}

size_t poetx_cnp_bwd_workspace_bytes(int32_t d, int32_t b, int32_t k) {
  if (d <= 0 || b <= 0 || k < 1) return 0;
  return align256((cnp_bwd_ws_floats(d, b, k) - (size_t)ceil_div(d, b) * b * b) * sizeof(float));   // without dG itself
}

int poetx_cnp_bwd(const float* theta, const float* dG, int32_t d, int32_t b, int32_t k, int32_t precision,
                  float* dtheta, int32_t accumulate, void* ws, size_t ws_bytes, void* stream) {
  if (!theta || !dG || !dtheta || d <= 0 || b <= 0 || k < 1) return POETX_ERR_INVALID_ARG;
  if (precision != POETX_CNP_FP32 && precision != POETX_CNP_BF16) return POETX_ERR_INVALID_ARG;
  if (b > d) return POETX_ERR_BAD_SHAPE;
  if (!ws || ws_bytes < poetx_cnp_bwd_workspace_bytes(d, b, k)) return POETX_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  StageTimer tm(POETX_STAGE_CNP_BWD, st);
  if (precision == POETX_CNP_BF16 && !g_force_fma.load() && mfma_cnp_supported(d, b))
    mfma_cnp_bwd(theta, dG, d, b, k, dtheta, accumulate != 0, (float*)ws, st);
  else
    fma_cnp_bwd(theta, dG, d, b, k, dtheta, accumulate != 0, (float*)ws, st);
  return launch_status();
}

size_t poetx_weight_q8_bytes(int32_t n, int32_t m) {
  if (n <= 0 || m <= 0) return 0;
  return weight_q8_scale_offset(n, m) + align256((size_t)n * sizeof(float));
}

int poetx_weight_quantize_q8(const void* W, int32_t dtype, int32_t n, int32_t m, void* Wq, void* stream) {
  if (!W || !Wq || n <= 0 || m <= 0 || !dtype_ok(dtype)) return POETX_ERR_INVALID_ARG;
  weight_quantize_q8_launch(dtype, W, n, m, Wq, (hipStream_t)stream);
  return launch_status();
}

int poetx_weight_dequantize_q8(const void* Wq, int32_t n, int32_t m, int32_t dtype, void* W_out, void* stream) {
  if (!Wq || !W_out || n <= 0 || m <= 0 || !dtype_ok(dtype)) return POETX_ERR_INVALID_ARG;
  weight_dequantize_q8_launch(Wq, n, m, dtype, W_out, (hipStream_t)stream);
  return launch_status();
}

int poetx_perm_blockdiag_apply_left(const void* V, void* out, int32_t d, int64_t cols, int64_t ld,
                                    const int32_t* perm, const void* blocks, int32_t b, int32_t transpose_G,
                                    int32_t dtype, void* stream) {
  if (!V || !out || !perm || !blocks || d <= 0 || cols <= 0 || b <= 0 || !dtype_ok(dtype)) return POETX_ERR_INVALID_ARG;
  if (ld < cols || b > d) return POETX_ERR_BAD_SHAPE;
  if (cols >= (1ll << 31)) return POETX_ERR_UNSUPPORTED;
  size_t bytes = (size_t)d * ld * esize(dtype);
  if (overlap(V, bytes, out, bytes)) return POETX_ERR_INVALID_ARG;
  apply_left_dispatch(dtype, V, out, d, cols, ld, perm, blocks, b, transpose_G != 0, (hipStream_t)stream);
  return launch_status();
}

int poetx_perm_blockdiag_apply_right(const void* V, void* out, int64_t rows, int32_t d, int64_t ld,
                                     const int32_t* perm, const void* blocks, int32_t b, int32_t transpose_G,
                                     int32_t dtype, void* stream) {
  if (!V || !out || !perm || !blocks || d <= 0 || rows <= 0 || b <= 0 || !dtype_ok(dtype)) return POETX_ERR_INVALID_ARG;
  if (ld < d || b > d) return POETX_ERR_BAD_SHAPE;
  if (rows >= (1ll << 31)) return POETX_ERR_UNSUPPORTED;
  size_t bytes = (size_t)rows * ld * esize(dtype);
  if (overlap(V, bytes, out, bytes)) return POETX_ERR_INVALID_ARG;
  StageTimer tm(POETX_STAGE_APPLY, (hipStream_t)stream);
  fma_apply_right(dtype, V, out, rows, d, ld, perm, blocks, b, transpose_G != 0, (hipStream_t)stream);
  return launch_status();
}

size_t poetx_merge_workspace_bytes(int32_t n, int32_t m, int32_t dtype) {
  if (n <= 0 || m <= 0 || !dtype_ok(dtype)) return 0;
  return 2 * align256((size_t)n * m * esize(dtype));
}

int poetx_merge_weight(const void* W, void* W_out, int32_t n, int32_t m, const int32_t* perm_R, const int32_t* perm_P,
                       const void* blocks_R, const void* blocks_P, int32_t b, int32_t dtype, void* ws, size_t ws_bytes,
                       void* stream) {
  if (!W || !W_out || !perm_R || !perm_P || !blocks_R || !blocks_P || n <= 0 || m <= 0 || b <= 0 || !dtype_ok(dtype))
    return POETX_ERR_INVALID_ARG;
  if (b > n || b > m) return POETX_ERR_BAD_SHAPE;
  const size_t bytes = (size_t)n * m * esize(dtype);
  if (overlap(W, bytes, W_out, bytes)) return POETX_ERR_INVALID_ARG;
  if (!ws || ws_bytes < poetx_merge_workspace_bytes(n, m, dtype)) return POETX_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  void* T1 = ws;
  void* T2 = (char*)ws + align256(bytes);
  // W (n x m) is feature major for the output side (rows = output features): P^T W is a left apply.
  // The input side acts on the columns; a column gather is a row gather of the transpose, so the
  // product with R^T runs as R (P^T W)^T on the transposed matrix and is transposed back.
  apply_left_dispatch(dtype, W, T1, n, m, m, perm_P, blocks_P, b, 1, st);        // T1 = P^T W         (n x m)
  {
    StageTimer tm(POETX_STAGE_LAYOUT, st);
    transpose_launch(dtype, T1, T2, n, m, st);                                   // T2 = T1^T          (m x n)
  }
  apply_left_dispatch(dtype, T2, T1, m, n, n, perm_R, blocks_R, b, 0, st);       // T1 = R T2          (m x n)
  {
    StageTimer tm(POETX_STAGE_LAYOUT, st);
    transpose_launch(dtype, T1, W_out, m, n, st);                                // W_out = (R T2)^T = P^T W R^T
  }
  return launch_status();
}

int poetx_perm_validate(const int32_t* perm, int32_t d, int32_t* scratch, void* stream) {
  if (!perm || !scratch || d <= 0) return POETX_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  perm_validate_launch(perm, d, scratch, st);
  int32_t bad = 0;
  if (hipMemcpyAsync(&bad, scratch + d, sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess) return POETX_ERR_HIP;
  if (hipStreamSynchronize(st) != hipSuccess) return POETX_ERR_HIP;
  return bad ? POETX_ERR_BAD_PERM : POETX_OK;
}

// The weight the dense product reads: W itself, or its dequantised copy made at `scratch`.
static const void* resolve_weight(const poetx_linear_desc* desc, const void* W, void* scratch, hipStream_t st) {
  if (!(desc->flags & POETX_FLAG_W_INT8) || weight_in_kernel(desc)) return W;
  StageTimer tm(POETX_STAGE_DEQUANT, st);
  weight_dequantize_q8_launch(W, desc->d_out, desc->d_in, desc->dtype, scratch, st);
  return scratch;
}

// Token-major callers: feature-major copies of the call's activations (at most X, dZ / Z and dX)
// live behind the regular workspace.
static size_t layout_staging_bytes(const poetx_linear_desc* d) {
  if (d->layout != POETX_TOKEN_MAJOR) return 0;
  const size_t es = esize(d->dtype), N = (size_t)d->n_tokens;
  return 2 * align256((size_t)d->d_in * N * es) + align256((size_t)d->d_out * N * es);
}
static size_t core_workspace_bytes(const poetx_linear_desc* desc);

size_t poetx_linear_workspace_bytes(const poetx_linear_desc* desc) {
  if (check_desc(desc) != POETX_OK) return 0;
  return core_workspace_bytes(desc) + layout_staging_bytes(desc);
}

int poetx_linear_path(const poetx_linear_desc* d) {
  const int rc = check_desc(d);
  if (rc) return -rc;
  const int m = d->d_in, n = d->d_out, b = d->block;
  const i64 N = d->n_tokens;
  int path = 0;
  if (d->dtype == POETX_F32 && !g_force_fma.load() && mfma_dense_f32_supported(n, m, N)) path |= POETX_PATH_DENSE;   // fp32 MFMA; the other stages of fp32 tensors stay on the plain-FMA kernels
  if (!use_mfma(d->dtype)) return path;
  if (mfma_apply_left_supported(m, N, N, b) && mfma_apply_left_supported(n, N, N, b)) path |= POETX_PATH_APPLY;
  if (mfma_dense_supported(n, m, N)) path |= POETX_PATH_DENSE;
  if (mfma_blockgrad_supported(m, N, b) && mfma_blockgrad_supported(n, N, b)) path |= POETX_PATH_BLOCKGRAD;
  if (d->cnp_precision == POETX_CNP_BF16 && mfma_cnp_supported(m, b) && mfma_cnp_supported(n, b)) {
    path |= POETX_PATH_SERIES;
    if (lds_cnp_supported(m, b) && lds_cnp_supported(n, b)) path |= POETX_PATH_SERIES_ON_CHIP;
    if (lds_cnp_supported(m, b) && lds_cnp_supported(n, b) && mfma_apply_grad_supported(m, N, N, b) &&
        mfma_apply_grad_supported(n, N, N, b))
      path |= POETX_PATH_BWD_ONE_PASS;
  }
  if (weight_in_kernel(d)) path |= POETX_PATH_W_INT8_IN_KERNEL;
  return path;
}

// Feature-major <-> token-major copies around a call.  in(): the feature-major copy of a
// token-major input (or the pointer itself); out(): where the call should write a feature-major
// output; finish(): transposes the registered outputs into the caller's token-major buffers.
class LayoutStaging {
 public:
  LayoutStaging(const poetx_linear_desc* d, void* ws, hipStream_t st)
      : on_(d->layout == POETX_TOKEN_MAJOR), dt_(d->dtype), N_(d->n_tokens), st_(st),
        next_((char*)ws + core_workspace_bytes(d)), n_out_(0) {}
  const void* in(const void* p, int rows) {
    if (!on_ || !p) return p;
    void* t = take(rows);
    StageTimer tm(POETX_STAGE_LAYOUT, st_);
    transpose_launch(dt_, p, t, N_, rows, st_);        // [N][rows] -> [rows][N]
    return t;
  }
  void* out(void* p, int rows) {
    if (!on_ || !p) return p;
    void* t = take(rows);
    outs_[n_out_].user = p; outs_[n_out_].tmp = t; outs_[n_out_].rows = rows; ++n_out_;
    return t;
  }
  void finish() {
    for (int i = 0; i < n_out_; ++i) {
      StageTimer tm(POETX_STAGE_LAYOUT, st_);
      transpose_launch(dt_, outs_[i].tmp, outs_[i].user, outs_[i].rows, N_, st_);   // [rows][N] -> [N][rows]
    }
  }
 private:
  void* take(int rows) {
    void* t = next_;
    next_ += align256((size_t)rows * N_ * esize(dt_));
    return t;
  }
  bool on_; int dt_; i64 N_; hipStream_t st_; char* next_;
  struct { void* user; void* tmp; int rows; } outs_[2];
  int n_out_;
};

// poetx_linear_bwd called without saved_B recomputes B itself: B, then the dequantised weight (kept for both
// of the call's dense products), sit at the very end of the workspace.
static size_t dequantised_weight_bytes(const poetx_linear_desc* desc) {
  return ((desc->flags & POETX_FLAG_W_INT8) && !weight_in_kernel(desc))
             ? align256((size_t)desc->d_out * desc->d_in * esize(desc->dtype)) : 0;
}
static size_t recompute_tail_bytes(const poetx_linear_desc* desc) {
  if (!(desc->flags & POETX_FLAG_RECOMPUTE_B)) return 0;
  return align256((size_t)desc->d_out * (size_t)desc->n_tokens * esize(desc->dtype)) + dequantised_weight_bytes(desc);
}

static size_t core_workspace_bytes(const poetx_linear_desc* desc) {
  size_t es = esize(desc->dtype);
  size_t N = (size_t)desc->n_tokens;
  size_t fwd = align256((size_t)desc->d_in * N * es);   // A = R^T X
  if (desc->flags & POETX_FLAG_RECOMPUTE_B) fwd += align256((size_t)desc->d_out * N * es);  // B lives here too
  const size_t wdeq = ((desc->flags & POETX_FLAG_W_INT8) && !weight_in_kernel(desc))
                          ? align256((size_t)desc->d_out * desc->d_in * es) : 0;   // dequantised copy, only where no kernel converts on the fly
  fwd += wdeq;                                          // dequantised weight behind A (and B)
  size_t bwi = align256((size_t)desc->d_out * N * es) + wdeq;  // dB = P dZ
  int dmax = desc->d_in > desc->d_out ? desc->d_in : desc->d_out;
  size_t bg_in = blockgrad_ws_bytes(desc->dtype, desc->d_in, desc->n_tokens, desc->block);
  size_t bg_out = blockgrad_ws_bytes(desc->dtype, desc->d_out, desc->n_tokens, desc->block);
  size_t chain = cnp_bwd_ws_floats(dmax, desc->block, desc->neumann_k);
  const size_t both = cnp_bwd_ws_floats_both(desc->d_in, desc->d_out, desc->block, desc->neumann_k);
  if (both > chain) chain = both;
  size_t skew = align256(chain * sizeof(float)) + (bg_in > bg_out ? bg_in : bg_out);
  size_t w = fwd > bwi ? fwd : bwi;
  if (skew > w) w = skew;
  // poetx_linear_bwd keeps dA (and, on its one-pass path, dB) in the workspace next to what the two
  // halves need: dA | two-call scratch, or dA | dB | dG + chain | partials or dequantised weight
  const size_t two_calls = bwi > skew ? bwi : skew;
  size_t bwd = align256((size_t)desc->d_in * N * es) + two_calls;
  if (desc->dtype == POETX_BF16 && mfma_apply_grad_supported(desc->d_in, desc->n_tokens, desc->n_tokens, desc->block) &&
      mfma_apply_grad_supported(desc->d_out, desc->n_tokens, desc->n_tokens, desc->block)) {
    size_t tail = align256(mfma_apply_grad_workspace_bytes(desc->d_in, desc->n_tokens));
    const size_t po = align256(mfma_apply_grad_workspace_bytes(desc->d_out, desc->n_tokens));
    if (po > tail) tail = po;
    if (wdeq > tail) tail = wdeq;
    const size_t one_pass = align256((size_t)desc->d_in * N * es) + align256((size_t)desc->d_out * N * es) +
                            align256(chain * sizeof(float)) + tail;
    if (one_pass > bwd) bwd = one_pass;
  }
  bwd += recompute_tail_bytes(desc);
  return w > bwd ? w : bwd;
}

int poetx_linear_fwd(const poetx_linear_desc* desc, const void* X, const void* W, const int32_t* perm_R,
                     const int32_t* perm_P, const void* blocks_R, const void* blocks_P, void* Z, void* saved_B,
                     void* ws, size_t ws_bytes, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!X || !W || !perm_R || !perm_P || !blocks_R || !blocks_P || !Z) return POETX_ERR_INVALID_ARG;
  if (!saved_B && !(desc->flags & POETX_FLAG_RECOMPUTE_B)) return POETX_ERR_INVALID_ARG;
  if (!ws || ws_bytes < poetx_linear_workspace_bytes(desc)) return POETX_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int m = desc->d_in, n = desc->d_out, b = desc->block, dt = desc->dtype;
  const i64 N = desc->n_tokens;
  LayoutStaging lay(desc, ws, st);
  X = lay.in(X, m);
  Z = lay.out(Z, n);
  void* A = ws;
  char* after = (char*)ws + align256((size_t)m * N * esize(dt));
  if (!saved_B) {  // memory-saving variant: scratch only
    saved_B = after;
    after += align256((size_t)n * N * esize(dt));
  }
  W = resolve_weight(desc, W, after, st);
  apply_left_dispatch(dt, X, A, m, N, N, perm_R, blocks_R, b, 1, st);        // mm1: A = R^T X
  dense_dispatch(dt, 0, W, n, m, A, saved_B, N, st, weight_in_kernel(desc));                        // mm2: B = W A
  apply_left_dispatch(dt, saved_B, Z, n, N, N, perm_P, blocks_P, b, 1, st);  // mm3: Z = P^T B
  lay.finish();
  return launch_status();
}

int poetx_linear_recompute_b(const poetx_linear_desc* desc, const void* X, const void* W, const int32_t* perm_R,
                             const void* blocks_R, void* B_out, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!X || !W || !perm_R || !blocks_R || !B_out) return POETX_ERR_INVALID_ARG;
  if (!ws || ws_bytes < poetx_linear_workspace_bytes(desc)) return POETX_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int m = desc->d_in, n = desc->d_out, b = desc->block, dt = desc->dtype;
  const i64 N = desc->n_tokens;
  LayoutStaging lay(desc, ws, st);
  X = lay.in(X, m);
  W = resolve_weight(desc, W, (char*)ws + align256((size_t)m * N * esize(dt)), st);
  apply_left_dispatch(dt, X, ws, m, N, N, perm_R, blocks_R, b, 1, st);  // A = R^T X
  dense_dispatch(dt, 0, W, n, m, ws, B_out, N, st, weight_in_kernel(desc));                    // B = W A
  return launch_status();
}

// dB = P dZ, dA = W^T dB, dX = R dA; ws holds dB (and the dequantised weight behind it)
static void bwd_input_impl(const poetx_linear_desc* desc, const void* dZ, const void* W, const int32_t* perm_R,
                           const int32_t* perm_P, const void* blocks_R, const void* blocks_P, void* dX, void* dA,
                           void* ws, hipStream_t st, const void* W_resolved = nullptr) {
  const int m = desc->d_in, n = desc->d_out, b = desc->block, dt = desc->dtype;
  const i64 N = desc->n_tokens;
  void* dB = ws;
  W = W_resolved ? W_resolved : resolve_weight(desc, W, (char*)ws + align256((size_t)n * N * esize(dt)), st);
  apply_left_dispatch(dt, dZ, dB, n, N, N, perm_P, blocks_P, b, 0, st);  // dB = P dZ
  dense_dispatch(dt, 1, W, n, m, dB, dA, N, st, weight_in_kernel(desc));                        // dA = W^T dB
  apply_left_dispatch(dt, dA, dX, m, N, N, perm_R, blocks_R, b, 0, st);  // dX = R dA
}

int poetx_linear_bwd_input(const poetx_linear_desc* desc, const void* dZ, const void* W, const int32_t* perm_R,
                           const int32_t* perm_P, const void* blocks_R, const void* blocks_P, void* dX, void* dA,
                           void* ws, size_t ws_bytes, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!dZ || !W || !perm_R || !perm_P || !blocks_R || !blocks_P || !dX || !dA) return POETX_ERR_INVALID_ARG;
  if (!ws || ws_bytes < poetx_linear_workspace_bytes(desc)) return POETX_ERR_WORKSPACE;
  LayoutStaging lay(desc, ws, (hipStream_t)stream);
  dZ = lay.in(dZ, desc->d_out);
  dX = lay.out(dX, desc->d_in);
  bwd_input_impl(desc, dZ, W, perm_R, perm_P, blocks_R, blocks_P, dX, dA, ws, (hipStream_t)stream);
  lay.finish();
  return launch_status();
}

// Series backward of both sides as one batch on the on-chip chains (b = 256): dG holds the block
// gradients of the P side, then of the R side; Qb and chain are scratch behind it.
static void cnp_bwd_both_on_chip(const float* theta_R, const float* theta_P, float* dG, int m, int n, int b, int k,
                                 float* dtheta_R, float* dtheta_P, int accumulate, hipStream_t st) {
  const int nbP = n / b, nbR = m / b, nbt = nbP + nbR;
  const size_t bb = (size_t)b * b;
  uint16_t* Qb = (uint16_t*)(dG + nbt * bb);                // [nbt][b][b] bf16 (one float slot per element)
  float* chain = dG + 2 * nbt * bb;                         // (k + 1) * nbt * b * b floats
  StageTimer tm(POETX_STAGE_CNP_BWD, st);
  skew_materialize_launch(theta_P, b, nbP, nullptr, Qb, nullptr, st);
  skew_materialize_launch(theta_R, b, nbR, nullptr, Qb + nbP * bb, nullptr, st);
  const float* dQ = lds_cnp_bwd_chain(Qb, dG, nbt, k, chain, st);
  skew_project_launch(dQ, b, n, dtheta_P, accumulate != 0, st);
  skew_project_launch(dQ + nbP * bb, b, m, dtheta_R, accumulate != 0, st);
}

static void bwd_skew_impl(const poetx_linear_desc* desc, const void* X, const void* dZ, const void* saved_B,
                          const void* dA, const int32_t* perm_R, const int32_t* perm_P, const float* theta_R,
                          const float* theta_P, float* dtheta_R, float* dtheta_P, int32_t accumulate, void* ws,
                          hipStream_t st) {
  const int m = desc->d_in, n = desc->d_out, b = desc->block, dt = desc->dtype, k = desc->neumann_k;
  const i64 N = desc->n_tokens;
  const int dmax = m > n ? m : n;
  size_t chain_floats = cnp_bwd_ws_floats(dmax, b, k);
  if (cnp_bwd_ws_floats_both(m, n, b, k) > chain_floats) chain_floats = cnp_bwd_ws_floats_both(m, n, b, k);
  void* bg_ws = (char*)ws + align256(chain_floats * sizeof(float));
  // POETX_FLAG_BLOCK_GRADS: the block gradients go to the caller (in place of dtheta) and the series
  // backward is left to poetx_cnp_bwd
  const bool defer = (desc->flags & POETX_FLAG_BLOCK_GRADS) != 0;
  if (desc->cnp_precision == POETX_CNP_BF16 && !g_force_fma.load() && use_mfma(dt) && mfma_cnp_supported(m, b) &&
      mfma_cnp_supported(n, b) && mfma_blockgrad_supported(m, N, b) && mfma_blockgrad_supported(n, N, b)) {
    // Both sides' blocks go through the series backward as one batch (P side first): the chains
    // are latency bound and a side alone leaves most CUs empty.
    const int nbP = n / b, nbR = m / b, nbt = nbP + nbR;
    const size_t bb = (size_t)b * b;
    float* dG = (float*)ws;                                   // [nbt][b][b]
    if (defer) {
      StageTimer tm(POETX_STAGE_BLOCKGRAD, st);
      mfma_blockgrad(saved_B, dZ, n, N, perm_P, b, dtheta_P, bg_ws, st);
      mfma_blockgrad(X, dA, m, N, perm_R, b, dtheta_R, bg_ws, st);
      return;
    }
    if (!lds_cnp_supported(m, b)) {                            // tiled kernels (b = 512)
      float* Qf = dG + nbt * bb;
      uint16_t* Tb = (uint16_t*)(Qf + nbt * bb);
      float* chain = Qf + nbt * bb + nbt * bb / 2;            // 3.5 floats per element follow: 6 in all
      {
        StageTimer tm(POETX_STAGE_BLOCKGRAD, st);
        mfma_blockgrad(saved_B, dZ, n, N, perm_P, b, dG, bg_ws, st);
        mfma_blockgrad(X, dA, m, N, perm_R, b, dG + nbP * bb, bg_ws, st);
      }
      StageTimer tm(POETX_STAGE_CNP_BWD, st);
      skew_materialize_launch(theta_P, b, nbP, Qf, nullptr, Tb, st);
      skew_materialize_launch(theta_R, b, nbR, Qf + nbP * bb, nullptr, Tb + nbP * bb, st);
      const float* dQ = mfma_cnp_bwd_chain(Qf, Tb, dG, nbt, b, k, chain, st);
      skew_project_launch(dQ, b, n, dtheta_P, accumulate != 0, st);
      skew_project_launch(dQ + nbP * bb, b, m, dtheta_R, accumulate != 0, st);
      return;
    }
    {
      StageTimer tm(POETX_STAGE_BLOCKGRAD, st);
      mfma_blockgrad(saved_B, dZ, n, N, perm_P, b, dG, bg_ws, st);            // dG_P = B' dZ'^T
      mfma_blockgrad(X, dA, m, N, perm_R, b, dG + nbP * bb, bg_ws, st);       // dG_R = X' dA'^T
    }
    cnp_bwd_both_on_chip(theta_R, theta_P, dG, m, n, b, k, dtheta_R, dtheta_P, accumulate, st);
    return;
  }
  float* dG = (float*)ws;
  float* chain = dG + (size_t)ceil_div(dmax, b) * b * b;
  for (int side = 0; side < 2; ++side) {
    const void* U = side == 0 ? saved_B : X;   // mm3 backward: dG_P = B' dZ'^T; mm1 backward: dG_R = X' dA'^T
    const void* V = side == 0 ? dZ : dA;
    const int d = side == 0 ? n : m;
    const int32_t* perm = side == 0 ? perm_P : perm_R;
    const float* theta = side == 0 ? theta_P : theta_R;
    float* dtheta = side == 0 ? dtheta_P : dtheta_R;
    const bool fast_cnp = desc->cnp_precision == POETX_CNP_BF16 && !g_force_fma.load() && mfma_cnp_supported(d, b);
    float* dGs = defer ? dtheta : dG;
    {
      StageTimer tm(POETX_STAGE_BLOCKGRAD, st);
      if (use_mfma(dt) && mfma_blockgrad_supported(d, N, b)) mfma_blockgrad(U, V, d, N, perm, b, dGs, bg_ws, st);
      else fma_blockgrad(dt, U, V, d, N, perm, b, dGs, st);
    }
    if (!defer) {
      StageTimer tm(POETX_STAGE_CNP_BWD, st);
      if (fast_cnp) mfma_cnp_bwd(theta, dG, d, b, k, dtheta, accumulate != 0, chain, st);
      else fma_cnp_bwd(theta, dG, d, b, k, dtheta, accumulate != 0, chain, st);
    }
  }
}

int poetx_linear_bwd_skew(const poetx_linear_desc* desc, const void* X, const void* dZ, const void* saved_B,
                          const void* dA, const int32_t* perm_R, const int32_t* perm_P, const float* theta_R,
                          const float* theta_P, float* dtheta_R, float* dtheta_P, int32_t accumulate, void* ws,
                          size_t ws_bytes, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!X || !dZ || !saved_B || !dA || !perm_R || !perm_P || !theta_R || !theta_P || !dtheta_R || !dtheta_P)
    return POETX_ERR_INVALID_ARG;
  if (!ws || ws_bytes < poetx_linear_workspace_bytes(desc)) return POETX_ERR_WORKSPACE;
  LayoutStaging lay(desc, ws, (hipStream_t)stream);
  X = lay.in(X, desc->d_in);
  dZ = lay.in(dZ, desc->d_out);
  bwd_skew_impl(desc, X, dZ, saved_B, dA, perm_R, perm_P, theta_R, theta_P, dtheta_R, dtheta_P, accumulate, ws,
                (hipStream_t)stream);
  return launch_status();
}

int poetx_linear_bwd(const poetx_linear_desc* desc, const void* X, const void* dZ, const void* saved_B, const void* W,
                     const int32_t* perm_R, const int32_t* perm_P, const void* blocks_R, const void* blocks_P,
                     const float* theta_R, const float* theta_P, void* dX, float* dtheta_R, float* dtheta_P,
                     int32_t accumulate, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!X || !dZ || !W || !perm_R || !perm_P || !blocks_R || !blocks_P || !theta_R || !theta_P || !dX ||
      !dtheta_R || !dtheta_P)
    return POETX_ERR_INVALID_ARG;
  if (!saved_B && !(desc->flags & POETX_FLAG_RECOMPUTE_B)) return POETX_ERR_INVALID_ARG;
  if (!ws || ws_bytes < poetx_linear_workspace_bytes(desc)) return POETX_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const int m = desc->d_in, n = desc->d_out, b = desc->block, dt = desc->dtype, k = desc->neumann_k;
  const i64 N = desc->n_tokens;
  LayoutStaging lay(desc, ws, st);
  X = lay.in(X, m);
  dZ = lay.in(dZ, n);
  dX = lay.out(dX, m);
  void* dA = ws;                                                   // m x N, lives until the R side is done
  char* rest = (char*)ws + align256((size_t)m * N * esize(dt));
  const void* W_resolved = nullptr;
  if (!saved_B) {
    // Gradient checkpoint inside the call (Sec. 3.5, memory-saving variant): A = R^T X goes where dA will
    // be, B = W A to the end of the workspace; a quantised weight is dequantised once for both products.
    char* end = (char*)ws + core_workspace_bytes(desc);
    char* w_keep = end - dequantised_weight_bytes(desc);
    char* B_re = w_keep - align256((size_t)n * N * esize(dt));
    W_resolved = resolve_weight(desc, W, w_keep, st);
    apply_left_dispatch(dt, X, dA, m, N, N, perm_R, blocks_R, b, 1, st);
    dense_dispatch(dt, 0, W_resolved, n, m, dA, B_re, N, st, weight_in_kernel(desc));
    saved_B = B_re;
  }
  const bool one_pass = desc->cnp_precision == POETX_CNP_BF16 && use_mfma(dt) && lds_cnp_supported(m, b) &&
                        lds_cnp_supported(n, b) && mfma_apply_grad_supported(m, N, N, b) &&
                        mfma_apply_grad_supported(n, N, N, b);
  if (!one_pass) {   // the same values through the two halves
    bwd_input_impl(desc, dZ, W, perm_R, perm_P, blocks_R, blocks_P, dX, dA, rest, st, W_resolved);
    bwd_skew_impl(desc, X, dZ, saved_B, dA, perm_R, perm_P, theta_R, theta_P, dtheta_R, dtheta_P, accumulate, rest, st);
    lay.finish();
    return launch_status();
  }
  // Each side's gradient is streamed once: dB = P dZ together with dG_P = B' dZ'^T, then
  // dA = W^T dB, then dX = R dA together with dG_R = X' dA'^T (Sec. 3.5), then the series backward.
  void* dB = rest;
  char* after_dB = rest + align256((size_t)n * N * esize(dt));
  const int nbP = n / b;
  const size_t bb = (size_t)b * b;
  float* dG = (float*)after_dB;                                    // both sides' block gradients, then chain scratch
  size_t chain_floats = cnp_bwd_ws_floats(m > n ? m : n, b, k);
  if (cnp_bwd_ws_floats_both(m, n, b, k) > chain_floats) chain_floats = cnp_bwd_ws_floats_both(m, n, b, k);
  void* part = after_dB + align256(chain_floats * sizeof(float));
  const bool defer = (desc->flags & POETX_FLAG_BLOCK_GRADS) != 0;   // block gradients to the caller, no series backward
  float* dG_P = defer ? dtheta_P : dG;
  float* dG_R = defer ? dtheta_R : dG + nbP * bb;
  {
    StageTimer tm(POETX_STAGE_APPLY_GRAD, st);
    mfma_apply_grad(dZ, saved_B, dB, n, N, N, perm_P, blocks_P, 0, dG_P, part, st);
  }
  W = W_resolved ? W_resolved : resolve_weight(desc, W, part, st);   // the P side's partials are reduced by now (stream order): same space
  dense_dispatch(dt, 1, W, n, m, dB, dA, N, st, weight_in_kernel(desc));
  {
    StageTimer tm(POETX_STAGE_APPLY_GRAD, st);
    mfma_apply_grad(dA, X, dX, m, N, N, perm_R, blocks_R, 0, dG_R, part, st);
  }
  lay.finish();
  if (defer) return launch_status();
  cnp_bwd_both_on_chip(theta_R, theta_P, dG, m, n, b, k, dtheta_R, dtheta_P, accumulate, st);
  return launch_status();
}

}  // extern "C"
