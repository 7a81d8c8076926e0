// C ABI of libcca (declared in include/cca.h): host-side validation, workspace
// carving and the chaining of the four stages on the caller's stream.
#include <math.h>

#include <mutex>

#include "cca_internal.h"

// Scratch of cca_decode_step_static: part of the loaded code object, one copy per GPU, never allocated or freed.
// In host code this name is only a handle for hipGetSymbolAddress; kernels get the device address it returns.
static __device__ __align__(256) unsigned char cca_decode_static_scratch[CCA_DECODE_STATIC_BYTES];

namespace cca {

// Device address of the static scratch on the current device, looked up once per device.
static hipError_t decode_static_scratch(void **ptr) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex mu;
  static void *addr[MAX_DEVICES] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(cca_decode_static_scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    addr[dev] = p;
  }
  *ptr = addr[dev];
  return hipSuccess;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Validates cfg and fills Dims.  Touches no HIP API.
static cca_status make_dims(const cca_config *cfg, Dims *d) {
  if (!cfg || !d) return CCA_ERR_NULL;
  if (cfg->dtype != CCA_BF16 && cfg->dtype != CCA_F32) return CCA_ERR_DTYPE;
  if (cfg->B <= 0 || cfg->T <= 0 || cfg->d_model <= 0 || cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0 ||
      cfg->head_dim <= 0)
    return CCA_ERR_SHAPE;
  if ((long long)cfg->B * cfg->T > (1ll << 30)) return CCA_ERR_SHAPE;
  if (cfg->n_q_heads % cfg->n_kv_heads != 0) return CCA_ERR_LAYOUT;
  const uint32_t known = CCA_CAUSAL | CCA_CONV_SEQ | CCA_CONV_CH | CCA_QK_MEAN | CCA_V_SHIFT | CCA_QK_NORM |
                         CCA_KEY_TEMP | CCA_ROPE | CCA_ROPE_INTERLEAVED;
  if (cfg->flags & ~known) return CCA_ERR_UNSUPPORTED;
  if ((cfg->flags & CCA_KEY_TEMP) && !(cfg->flags & CCA_QK_NORM)) return CCA_ERR_UNSUPPORTED;
  if ((cfg->flags & CCA_ROPE_INTERLEAVED) && !(cfg->flags & CCA_ROPE)) return CCA_ERR_UNSUPPORTED;
  if ((cfg->flags & CCA_CONV_SEQ) && (cfg->k_seq < 1 || cfg->k_seq > 4)) return CCA_ERR_UNSUPPORTED;
  if ((cfg->flags & CCA_CONV_CH) && (cfg->k_ch < 1 || cfg->k_ch > 4)) return CCA_ERR_UNSUPPORTED;
  if (cfg->head_dim > 256) return CCA_ERR_UNSUPPORTED;
  // rows of every tensor must keep 16-byte alignment
  const int per16 = cfg->dtype == CCA_BF16 ? 8 : 4;
  if (cfg->head_dim % per16 != 0 || cfg->d_model % per16 != 0) return CCA_ERR_UNSUPPORTED;
  if ((cfg->flags & CCA_ROPE) && (cfg->head_dim % 2 != 0)) return CCA_ERR_LAYOUT;
  if ((cfg->flags & CCA_ROPE) && !(cfg->rope_base > 0.f)) return CCA_ERR_SHAPE;
  if (cfg->softmax_scale < 0.f || isnan(cfg->softmax_scale)) return CCA_ERR_SHAPE;
  if (!(cfg->norm_eps >= 0.f) || isinf(cfg->norm_eps)) return CCA_ERR_SHAPE;
  const long long e_kv = (long long)cfg->n_kv_heads * cfg->head_dim;
  const long long e_q = (long long)cfg->n_q_heads * cfg->head_dim;
  if (e_q > 65536 || e_kv > 65536 || cfg->d_model > 65536) return CCA_ERR_SHAPE;
  if ((cfg->flags & CCA_V_SHIFT) && (e_kv % 2 != 0)) return CCA_ERR_LAYOUT;
  // the latent must not be wider than the residual stream (compression factors >= 1)
  if (e_q > cfg->d_model || e_kv > e_q) return CCA_ERR_SHAPE;
  // stated compression factors (Sec. 2.2: latent widths E/C1 and E/C2) must agree with the head layout
  if (cfg->compress_q < 0 || cfg->compress_kv < 0) return CCA_ERR_SHAPE;
  if (cfg->compress_q > 0 && (long long)cfg->compress_q * e_q != cfg->d_model) return CCA_ERR_SHAPE;
  if (cfg->compress_kv > 0 && (long long)cfg->compress_kv * e_kv != cfg->d_model) return CCA_ERR_SHAPE;
  d->B = cfg->B; d->T = cfg->T; d->E = cfg->d_model;
  d->Hq = cfg->n_q_heads; d->Hk = cfg->n_kv_heads; d->dh = cfg->head_dim;
  d->R = d->Hq / d->Hk;
  d->e_q = (int)e_q; d->e_kv = (int)e_kv; d->n_lat = d->e_q + 2 * d->e_kv;
  d->v_half = d->e_kv / 2;
  d->k_seq = (cfg->flags & CCA_CONV_SEQ) ? cfg->k_seq : 1;
  d->k_ch = (cfg->flags & CCA_CONV_CH) ? cfg->k_ch : 1;
  d->bf16 = cfg->dtype == CCA_BF16;
  d->flags = cfg->flags;
  d->rope_base = cfg->rope_base;
  d->norm_eps = cfg->norm_eps;
  d->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / sqrtf((float)cfg->head_dim);
  return CCA_OK;
}

// The first three parts depend on the weights and the config only (not on x, not on B): they are what
// cca_prepare writes into a caller-owned buffer, in this layout.
struct FwdLayout {
  size_t wt_down, wt_out, pro, lat, q, k, v, o, total;  // byte offsets
  size_t prepared_bytes() const { return lat; }
};

static FwdLayout fwd_layout(const Dims &d) {
  FwdLayout L;
  const size_t es = d.esize();
  const size_t rows = (size_t)d.rows();
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  // (the transposed weights are only made when the matrix-core GEMM runs, which does not depend on B: see
  // both_projections_mfma)
  L.wt_down = take(d.bf16 ? (size_t)d.E * d.n_lat * 2 : 0);
  L.wt_out = take(d.bf16 ? (size_t)d.E * d.e_q * 2 : 0);
  L.pro = take(prologue_fused_scratch_bytes(d));
  L.lat = take(rows * d.n_lat * es);
  L.q = take(rows * d.e_q * es);
  L.k = take(rows * d.e_kv * es);
  L.v = take(rows * d.e_kv * es);
  L.o = take(rows * d.e_q * es);
  L.total = off;
  return L;
}

// C (M,N) = A (M,K) * W (K,N); the MFMA path first writes W^T into `wt` (unless the caller already has).
static cca_status project(const Dims &d, const void *A, const void *W, void *C, long long M, int N, int K, void *wt,
                          size_t wt_bytes, hipStream_t s, bool wt_ready = false) {
  hipError_t e;
  if (d.bf16 && gemm_mfma_supported(M, N, K)) {
    if (!wt || wt_bytes < (size_t)N * K * 2) return CCA_ERR_WORKSPACE;
    if (!wt_ready) {
      e = transpose_bf16(W, wt, K, N, s);
      if (e != hipSuccess) return CCA_ERR_LAUNCH;
    }
    e = gemm_mfma_bf16(A, wt, C, M, N, K, s);
  } else {
    e = gemm_generic(d.bf16, A, W, C, M, N, K, s);
  }
  return e == hipSuccess ? CCA_OK : CCA_ERR_LAUNCH;
}

// `ready`: scratch already holds the folded filters and RoPE tables (cca_prepare made them)
static cca_status run_prologue(const Dims &d, const cca_weights *w, const void *lat, void *q, void *k, void *v,
                               float *rnorm, void *scratch, size_t scratch_bytes, hipStream_t s, bool ready = false) {
  hipError_t e;
  if (prologue_is_split_copy(d)) {
    e = prologue_split_copy(d, lat, q, k, v, rnorm, s);
  } else if (prologue_fused_supported(d)) {
    if (!scratch || scratch_bytes < prologue_fused_scratch_bytes(d)) return CCA_ERR_WORKSPACE;
    e = ready ? prologue_fused_run(d, *w, lat, q, k, v, rnorm, scratch, s)
              : prologue_fused_bf16(d, *w, lat, q, k, v, rnorm, scratch, s);
  } else {
    e = prologue_generic(d, *w, lat, q, k, v, rnorm, s);
  }
  return e == hipSuccess ? CCA_OK : CCA_ERR_LAUNCH;
}

static cca_status run_attention(const Dims &d, const void *q, const void *k, const void *v, void *o, void *o_lo,
                                float *lse, const float *temp, hipStream_t s) {
  hipError_t e = attention_mfma_supported(d) ? attention_mfma_bf16(d, q, k, v, o, o_lo, lse, temp, s)
                                             : attention_generic(d, q, k, v, o, o_lo, lse, s);
  return e == hipSuccess ? CCA_OK : CCA_ERR_LAUNCH;
}

struct BwdLayout {
  size_t d_o, d_q, d_k, d_v, delta, d_lat, pro, gemm, total;  // byte offsets
  size_t pro_bytes, gemm_bytes;
};

static size_t prologue_bwd_scratch_bytes(const Dims &d) {
  if (prologue_is_split_copy(d)) return 0;
  return prologue_bwd_fused_supported(d) ? prologue_bwd_fused_scratch_bytes(d) : prologue_bwd_generic_scratch_bytes(d);
}

static bool tn_mfma(const Dims &d, int Mo, int No) { return d.bf16 && gemm_tn_mfma_supported(Mo, No, d.rows()); }

static BwdLayout bwd_layout(const Dims &d) {
  BwdLayout L;
  const size_t es = d.esize();
  const size_t rows = (size_t)d.rows();
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  L.d_o = take(rows * d.e_q * es);
  L.d_q = take(rows * d.e_q * es);
  L.d_k = take(rows * d.e_kv * es);
  L.d_v = take(rows * d.e_kv * es);
  L.delta = take(attention_bwd_scratch_bytes(d));  // Delta and the attention backward's per-head partial sums
  L.d_lat = take(rows * d.n_lat * es);
  L.pro_bytes = prologue_bwd_scratch_bytes(d);
  L.pro = take(L.pro_bytes);
  size_t g1 = tn_mfma(d, d.e_q, d.E) ? gemm_tn_scratch_bytes(d.e_q, d.E, d.rows()) : 0;
  size_t g2 = tn_mfma(d, d.E, d.n_lat) ? gemm_tn_scratch_bytes(d.E, d.n_lat, d.rows()) : 0;
  L.gemm_bytes = g1 > g2 ? g1 : g2;
  L.gemm = take(L.gemm_bytes);
  L.total = off;
  return L;
}

// C (M,N) = A (M,K) * W (N,K)^T with W as stored (no transpose pass): d_o = d_out W_O^T, d_x = d_lat W_down^T
static cca_status project_t(const Dims &d, const void *A, const void *W, void *C, long long M, int N, int K,
                            hipStream_t s) {
  hipError_t e = (d.bf16 && gemm_mfma_supported(M, N, K)) ? gemm_mfma_bf16(A, W, C, M, N, K, s)
                                                          : gemm_generic_ex(d.bf16, A, K, false, W, K, true, C, N, M, N, K, s);
  return e == hipSuccess ? CCA_OK : CCA_ERR_LAUNCH;
}

// dW (Mo,No) = A (rows,Mo)^T * Bm (rows,No)
static cca_status weight_grad(const Dims &d, const void *A, const void *Bm, void *dW, int Mo, int No, void *scratch,
                              hipStream_t s) {
  hipError_t e = tn_mfma(d, Mo, No)
                     ? gemm_tn_mfma_bf16(A, Mo, Bm, No, dW, Mo, No, d.rows(), static_cast<float *>(scratch), s)
                     : gemm_generic_ex(d.bf16, A, Mo, true, Bm, No, false, dW, No, Mo, No, d.rows(), s);
  return e == hipSuccess ? CCA_OK : CCA_ERR_LAUNCH;
}

static cca_status run_attention_bwd(const Dims &d, const void *q, const void *k, const void *v, const void *o,
                                    const void *o_lo, const float *lse, const void *d_o, void *d_q, void *d_k, void *d_v, float *delta,
                                    hipStream_t s) {
  hipError_t e = attention_bwd_supported(d) ? attention_bwd_bf16(d, q, k, v, o, o_lo, lse, d_o, d_q, d_k, d_v, delta, s)
                                            : attention_bwd_generic(d, q, k, v, o, o_lo, lse, d_o, d_q, d_k, d_v, delta, s);
  return e == hipSuccess ? CCA_OK : CCA_ERR_LAUNCH;
}

static cca_status run_prologue_bwd(const Dims &d, const cca_weights *w, const void *lat, const void *q, const void *k,
                                   const float *rnorm, const void *d_q, const void *d_k, const void *d_v, void *d_lat,
                                   const cca_grads *gr, void *scratch, size_t scratch_bytes, hipStream_t s) {
  if (prologue_is_split_copy(d))  // plain MHA / GQA: nothing to differentiate but the column split
    return prologue_split_copy_bwd(d, d_q, d_k, d_v, d_lat, s) == hipSuccess ? CCA_OK : CCA_ERR_LAUNCH;
  if (!scratch || scratch_bytes < prologue_bwd_scratch_bytes(d)) return CCA_ERR_WORKSPACE;
  hipError_t e = prologue_bwd_fused_supported(d)
                     ? prologue_bwd_fused_bf16(d, *w, lat, q, k, rnorm, d_q, d_k, d_v, d_lat, gr, scratch, s)
                     : prologue_bwd_generic(d, *w, lat, q, k, rnorm, d_q, d_k, d_v, d_lat, gr, scratch, s);
  return e == hipSuccess ? CCA_OK : CCA_ERR_LAUNCH;
}

// Both projections of cca_forward on the matrix-core GEMM (then their weights are wanted K-contiguous).  The GEMM's
// conditions on the row count are met or missed by every B alike only through M = B*T >= 1, so a buffer prepared
// under one B serves any other.
static bool both_projections_mfma(const Dims &d) {
  return d.bf16 && gemm_mfma_supported(d.rows(), d.n_lat, d.E) && gemm_mfma_supported(d.rows(), d.E, d.e_q);
}

static cca_status check_grads(const cca_grads *g) {
  if (!g) return CCA_OK;
  if (!aligned16(g->w_down) || !aligned16(g->w_conv_seq) || !aligned16(g->w_conv_ch) || !aligned16(g->w_out) ||
      (reinterpret_cast<uintptr_t>(g->temp) & 3u))
    return CCA_ERR_ALIGN;
  return CCA_OK;
}

static cca_status check_prologue_weights(const Dims &d, const cca_weights *w) {
  if (!w) return CCA_ERR_NULL;
  if ((d.flags & CCA_CONV_SEQ) && !w->w_conv_seq) return CCA_ERR_NULL;
  if ((d.flags & CCA_CONV_CH) && !w->w_conv_ch) return CCA_ERR_NULL;
  if ((d.flags & CCA_KEY_TEMP) && !w->temp) return CCA_ERR_NULL;
  if (!aligned16(w->w_conv_seq) || !aligned16(w->w_conv_ch) || (reinterpret_cast<uintptr_t>(w->temp) & 3u))
    return CCA_ERR_ALIGN;
  return CCA_OK;
}

}  // namespace cca

using namespace cca;

extern "C" {

cca_status cca_workspace_size(const cca_config *cfg, size_t *fwd_bytes, size_t *bwd_bytes) {
  if (!fwd_bytes && !bwd_bytes) return CCA_ERR_NULL;
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  if (fwd_bytes) *fwd_bytes = fwd_layout(d).total;
  if (bwd_bytes) *bwd_bytes = bwd_layout(d).total;
  return CCA_OK;
}

cca_status cca_prepared_size(const cca_config *cfg, size_t *bytes) {
  if (!bytes) return CCA_ERR_NULL;
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  *bytes = fwd_layout(d).prepared_bytes();
  return CCA_OK;
}

cca_status cca_prepare(const cca_config *cfg, const cca_weights *w, void *prepared, size_t prepared_bytes,
                       void *hip_stream) {
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  if (!w || !w->w_down || !w->w_out) return CCA_ERR_NULL;
  st = check_prologue_weights(d, w);
  if (st != CCA_OK) return st;
  const FwdLayout L = fwd_layout(d);
  if (L.prepared_bytes() == 0) return CCA_OK;  // nothing to prepare for this config
  if (!prepared || prepared_bytes < L.prepared_bytes()) return CCA_ERR_WORKSPACE;
  if (!aligned16(prepared) || !aligned16(w->w_down) || !aligned16(w->w_out)) return CCA_ERR_ALIGN;
  char *pb = static_cast<char *>(prepared);
  hipStream_t s = (hipStream_t)hip_stream;
  if (both_projections_mfma(d) &&
      transpose2_bf16(w->w_down, pb + L.wt_down, d.E, d.n_lat, w->w_out, pb + L.wt_out, d.e_q, d.E, s) != hipSuccess)
    return CCA_ERR_LAUNCH;
  if (!prologue_is_split_copy(d) && prologue_fused_supported(d) &&
      prologue_fused_prepare(d, *w, pb + L.pro, s) != hipSuccess)
    return CCA_ERR_LAUNCH;
  return CCA_OK;
}

cca_status cca_backward_workspace_size(const cca_config *cfg, size_t *bwd_bytes) {
  if (!bwd_bytes) return CCA_ERR_NULL;
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  *bwd_bytes = bwd_layout(d).total;
  return CCA_OK;
}

cca_status cca_down_project(const cca_config *cfg, const void *x, const void *w_down, void *lat, void *workspace,
                            size_t workspace_bytes, void *hip_stream) {
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  if (!x || !w_down || !lat) return CCA_ERR_NULL;
  if (!aligned16(x) || !aligned16(w_down) || !aligned16(lat) || !aligned16(workspace)) return CCA_ERR_ALIGN;
  return project(d, x, w_down, lat, d.rows(), d.n_lat, d.E, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

cca_status cca_up_project(const cca_config *cfg, const void *o, const void *w_out, void *out, void *workspace,
                          size_t workspace_bytes, void *hip_stream) {
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  if (!o || !w_out || !out) return CCA_ERR_NULL;
  if (!aligned16(o) || !aligned16(w_out) || !aligned16(out) || !aligned16(workspace)) return CCA_ERR_ALIGN;
  return project(d, o, w_out, out, d.rows(), d.E, d.e_q, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

cca_status cca_prologue(const cca_config *cfg, const cca_weights *w, const void *lat, void *q, void *k, void *v,
                        float *rnorm, void *workspace, size_t workspace_bytes, void *hip_stream) {
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  if (!lat || !q || !k || !v) return CCA_ERR_NULL;
  st = check_prologue_weights(d, w);
  if (st != CCA_OK) return st;
  if (!aligned16(lat) || !aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(workspace))
    return CCA_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(rnorm) & 3u) return CCA_ERR_ALIGN;
  return run_prologue(d, w, lat, q, k, v, rnorm, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

cca_status cca_attention(const cca_config *cfg, const void *q, const void *k, const void *v, void *o, void *o_lo,
                         float *lse, const float *temp, void *hip_stream) {
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  if (!q || !k || !v || !o) return CCA_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(o_lo) ||
      (reinterpret_cast<uintptr_t>(lse) & 3u))
    return CCA_ERR_ALIGN;
  if ((d.flags & CCA_KEY_TEMP) && !temp) return CCA_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(temp) & 3u) return CCA_ERR_ALIGN;
  return run_attention(d, q, k, v, o, o_lo, lse, temp, (hipStream_t)hip_stream);
}

cca_status cca_attention_backward(const cca_config *cfg, const void *q, const void *k, const void *v, const void *o,
                                  const void *o_lo, const float *lse, const void *d_o, void *d_q, void *d_k, void *d_v, void *workspace,
                                  size_t workspace_bytes, void *hip_stream) {
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  if (!q || !k || !v || !o || !lse || !d_o || !d_q || !d_k || !d_v) return CCA_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(d_o) || !aligned16(d_q) ||
      !aligned16(d_k) || !aligned16(d_v) || !aligned16(workspace) || !aligned16(o_lo) ||
      (reinterpret_cast<uintptr_t>(lse) & 3u))
    return CCA_ERR_ALIGN;
  if (!workspace || workspace_bytes < attention_bwd_scratch_bytes(d)) return CCA_ERR_WORKSPACE;
  return run_attention_bwd(d, q, k, v, o, o_lo, lse, d_o, d_q, d_k, d_v, static_cast<float *>(workspace),
                           (hipStream_t)hip_stream);
}

cca_status cca_prologue_backward(const cca_config *cfg, const cca_weights *w, const void *lat, const void *q,
                                 const void *k, const float *rnorm, const void *d_q, const void *d_k, const void *d_v,
                                 void *d_lat, const cca_grads *grads, void *workspace, size_t workspace_bytes,
                                 void *hip_stream) {
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  if (!lat || !q || !k || !rnorm || !d_q || !d_k || !d_v || !d_lat) return CCA_ERR_NULL;
  st = check_prologue_weights(d, w);
  if (st != CCA_OK) return st;
  st = check_grads(grads);
  if (st != CCA_OK) return st;
  if (!aligned16(lat) || !aligned16(q) || !aligned16(k) || !aligned16(d_q) || !aligned16(d_k) || !aligned16(d_v) ||
      !aligned16(d_lat) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(rnorm) & 3u))
    return CCA_ERR_ALIGN;
  return run_prologue_bwd(d, w, lat, q, k, rnorm, d_q, d_k, d_v, d_lat, grads, workspace, workspace_bytes,
                          (hipStream_t)hip_stream);
}

cca_status cca_backward(const cca_config *cfg, const cca_weights *w, const void *x, const cca_saved *saved,
                        const void *d_out, void *d_x, const cca_grads *grads, void *workspace, size_t workspace_bytes,
                        void *hip_stream) {
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  if (!w || !x || !saved || !d_out || !w->w_down || !w->w_out) return CCA_ERR_NULL;
  if (!saved->lat || !saved->q || !saved->k || !saved->v || !saved->o || !saved->lse || !saved->rnorm)
    return CCA_ERR_NULL;
  st = check_prologue_weights(d, w);
  if (st != CCA_OK) return st;
  st = check_grads(grads);
  if (st != CCA_OK) return st;
  if (!aligned16(x) || !aligned16(d_out) || !aligned16(d_x) || !aligned16(w->w_down) || !aligned16(w->w_out) ||
      !aligned16(saved->lat) || !aligned16(saved->q) || !aligned16(saved->k) || !aligned16(saved->v) ||
      !aligned16(saved->o) || !aligned16(saved->o_lo) || (reinterpret_cast<uintptr_t>(saved->lse) & 3u) ||
      (reinterpret_cast<uintptr_t>(saved->rnorm) & 3u))
    return CCA_ERR_ALIGN;
  const BwdLayout L = bwd_layout(d);
  if (!workspace || workspace_bytes < L.total) return CCA_ERR_WORKSPACE;
  if (!aligned16(workspace)) return CCA_ERR_ALIGN;
  char *ws = static_cast<char *>(workspace);
  void *d_o = ws + L.d_o, *d_q = ws + L.d_q, *d_k = ws + L.d_k, *d_v = ws + L.d_v, *d_lat = ws + L.d_lat;
  hipStream_t s = (hipStream_t)hip_stream;
  // last step first: out = o W_O
  if (grads && grads->w_out) {
    st = weight_grad(d, saved->o, d_out, grads->w_out, d.e_q, d.E, ws + L.gemm, s);
    if (st != CCA_OK) return st;
  }
  st = project_t(d, d_out, w->w_out, d_o, d.rows(), d.e_q, d.E, s);
  if (st != CCA_OK) return st;
  st = run_attention_bwd(d, saved->q, saved->k, saved->v, saved->o, saved->o_lo, saved->lse, d_o, d_q, d_k, d_v,
                         reinterpret_cast<float *>(ws + L.delta), s);
  if (st != CCA_OK) return st;
  st = run_prologue_bwd(d, w, saved->lat, saved->q, saved->k, saved->rnorm, d_q, d_k, d_v, d_lat, grads, ws + L.pro,
                        L.pro_bytes, s);
  if (st != CCA_OK) return st;
  if (d_x) {
    st = project_t(d, d_lat, w->w_down, d_x, d.rows(), d.E, d.n_lat, s);
    if (st != CCA_OK) return st;
  }
  if (grads && grads->w_down) {
    st = weight_grad(d, x, d_lat, grads->w_down, d.E, d.n_lat, ws + L.gemm, s);
    if (st != CCA_OK) return st;
  }
  return CCA_OK;
}

cca_status cca_forward(const cca_config *cfg, const cca_weights *w, const void *x, void *out, const cca_saved *saved,
                       void *workspace, size_t workspace_bytes, void *hip_stream) {
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  if (!w || !x || !out || !w->w_down || !w->w_out) return CCA_ERR_NULL;
  st = check_prologue_weights(d, w);
  if (st != CCA_OK) return st;
  if (!aligned16(x) || !aligned16(out) || !aligned16(w->w_down) || !aligned16(w->w_out) || !aligned16(w->prepared))
    return CCA_ERR_ALIGN;
  const FwdLayout L = fwd_layout(d);
  if (!workspace || workspace_bytes < L.total) return CCA_ERR_WORKSPACE;
  if (!aligned16(workspace)) return CCA_ERR_ALIGN;
  char *ws = static_cast<char *>(workspace);
  void *lat = ws + L.lat, *q = ws + L.q, *k = ws + L.k, *v = ws + L.v, *o = ws + L.o;
  float *lse = nullptr, *rnorm = nullptr;
  void *o_lo = nullptr;
  if (saved) {
    if (!aligned16(saved->lat) || !aligned16(saved->q) || !aligned16(saved->k) || !aligned16(saved->v) ||
        !aligned16(saved->o) || !aligned16(saved->o_lo) || (reinterpret_cast<uintptr_t>(saved->lse) & 3u))
      return CCA_ERR_ALIGN;
    if (saved->lat) lat = saved->lat;
    if (saved->q) q = saved->q;
    if (saved->k) k = saved->k;
    if (saved->v) v = saved->v;
    if (saved->o) o = saved->o;
    lse = saved->lse;
    rnorm = saved->rnorm;
    o_lo = saved->o_lo;
    if (reinterpret_cast<uintptr_t>(rnorm) & 3u) return CCA_ERR_ALIGN;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  // What depends on the weights only: taken from the caller's prepared buffer, else derived into the workspace
  // (both weight transposes in one launch when both projections run on the MFMA GEMM).
  const bool prepared = w->prepared != nullptr;
  char *pre = prepared ? static_cast<char *>(const_cast<void *>(w->prepared)) : ws;
  const bool both = both_projections_mfma(d);
  if (both && !prepared &&
      transpose2_bf16(w->w_down, pre + L.wt_down, d.E, d.n_lat, w->w_out, pre + L.wt_out, d.e_q, d.E, s) != hipSuccess)
    return CCA_ERR_LAUNCH;
  st = project(d, x, w->w_down, lat, d.rows(), d.n_lat, d.E, pre + L.wt_down, (size_t)d.E * d.n_lat * 2, s, both);
  if (st != CCA_OK) return st;
  st = run_prologue(d, w, lat, q, k, v, rnorm, pre + L.pro, L.lat - L.pro, s, prepared);
  if (st != CCA_OK) return st;
  st = run_attention(d, q, k, v, o, o_lo, lse, w->temp, s);
  if (st != CCA_OK) return st;
  return project(d, o, w->w_out, out, d.rows(), d.E, d.e_q, pre + L.wt_out, (size_t)d.E * d.e_q * 2, s, both);
}

cca_status cca_decode_workspace_size(const cca_config *cfg, size_t *bytes, int32_t *ring_rows) {
  if (!bytes) return CCA_ERR_NULL;
  Dims d;
  cca_status st = make_dims(cfg, &d);
  if (st != CCA_OK) return st;
  if (d.dh % 8 != 0) return CCA_ERR_UNSUPPORTED;
  *bytes = decode_scratch_bytes(d);
  if (ring_rows) *ring_rows = decode_ring_rows(d);
  return CCA_OK;
}

// Argument checks shared by the two decode entry points (no HIP call).
static cca_status decode_validate(const cca_config *cfg, Dims *d, const cca_weights *w, const void *x_new,
                                  const cca_decode_state *state, int32_t pos, const void *out) {
  cca_status st = make_dims(cfg, d);
  if (st != CCA_OK) return st;
  if (d->dh % 8 != 0) return CCA_ERR_UNSUPPORTED;
  if (!w || !x_new || !state || !out || !state->k_cache || !state->v_cache || !state->lat_ring) return CCA_ERR_NULL;
  if (!w->w_down || !w->w_out) return CCA_ERR_NULL;
  if (pos < 0 || pos >= d->T) return CCA_ERR_SHAPE;
  st = check_prologue_weights(*d, w);
  if (st != CCA_OK) return st;
  if (!aligned16(x_new) || !aligned16(out) || !aligned16(state->k_cache) || !aligned16(state->v_cache) ||
      !aligned16(state->lat_ring) || !aligned16(w->w_down) || !aligned16(w->w_out))
    return CCA_ERR_ALIGN;
  return CCA_OK;
}

cca_status cca_decode_step(const cca_config *cfg, const cca_weights *w, const void *x_new, const cca_decode_state *state,
                           int32_t pos, void *out, void *workspace, size_t workspace_bytes, void *hip_stream) {
  Dims d;
  cca_status st = decode_validate(cfg, &d, w, x_new, state, pos, out);
  if (st != CCA_OK) return st;
  if (!aligned16(workspace)) return CCA_ERR_ALIGN;
  if (!workspace || workspace_bytes < decode_scratch_bytes(d)) return CCA_ERR_WORKSPACE;
  return decode_step(d, *w, x_new, state->k_cache, state->v_cache, state->lat_ring, pos, nullptr, out, workspace,
                     (hipStream_t)hip_stream) == hipSuccess
             ? CCA_OK
             : CCA_ERR_LAUNCH;
}

cca_status cca_decode_step_static(const cca_config *cfg, const cca_weights *w, const void *x_new,
                                  const cca_decode_state *state, int32_t pos, void *out, void *hip_stream) {
  Dims d;
  cca_status st = decode_validate(cfg, &d, w, x_new, state, pos, out);
  if (st != CCA_OK) return st;
  if (decode_scratch_bytes(d) > (size_t)CCA_DECODE_STATIC_BYTES) return CCA_ERR_WORKSPACE;  // does not fit the array
  void *scratch = nullptr;  // first HIP call: everything above is host arithmetic
  if (decode_static_scratch(&scratch) != hipSuccess) return CCA_ERR_LAUNCH;
  return decode_step(d, *w, x_new, state->k_cache, state->v_cache, state->lat_ring, pos, nullptr, out, scratch,
                     (hipStream_t)hip_stream) == hipSuccess
             ? CCA_OK
             : CCA_ERR_LAUNCH;
}

cca_status cca_decode_step_ragged(const cca_config *cfg, const cca_weights *w, const void *x_new,
                                  const cca_decode_state *state, const int32_t *pos, int32_t max_pos, void *out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream) {
  Dims d;
  cca_status st = decode_validate(cfg, &d, w, x_new, state, max_pos, out);
  if (st != CCA_OK) return st;
  if (!pos) return CCA_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(pos) % 4 != 0 || !aligned16(workspace)) return CCA_ERR_ALIGN;
  if (!workspace || workspace_bytes < decode_scratch_bytes(d)) return CCA_ERR_WORKSPACE;
  static_assert(sizeof(int) == sizeof(int32_t), "positions are passed to the kernels as int");
  return decode_step(d, *w, x_new, state->k_cache, state->v_cache, state->lat_ring, max_pos,
                     reinterpret_cast<const int *>(pos), out, workspace, (hipStream_t)hip_stream) == hipSuccess
             ? CCA_OK
             : CCA_ERR_LAUNCH;
}

cca_status cca_probe_mfma_rate(void *out, size_t out_bytes, int32_t blocks, int32_t iters, int32_t operands,
                               double *flops, void *hip_stream) {
  if (!out || !flops) return CCA_ERR_NULL;
  if (blocks <= 0 || iters <= 0 || blocks > (1 << 20) || iters > (1 << 24) || (iters & 1)) return CCA_ERR_SHAPE;
  if (operands != 0 && operands != 1) return CCA_ERR_UNSUPPORTED;
  if (out_bytes < (size_t)blocks * 256 * sizeof(float)) return CCA_ERR_WORKSPACE;
  if (!aligned16(out)) return CCA_ERR_ALIGN;
  *flops = (double)blocks * 4.0 * (double)iters * 4.0 * (2.0 * 32 * 32 * 16);
  return mfma_probe(static_cast<float *>(out), blocks, iters, operands == 1, (hipStream_t)hip_stream) == hipSuccess
             ? CCA_OK
             : CCA_ERR_LAUNCH;
}

const char *cca_strerror(cca_status s) {
  switch (s) {
    case CCA_OK: return "ok";
    case CCA_ERR_NULL: return "a required pointer is NULL";
    case CCA_ERR_SHAPE: return "a size is non-positive or the sizes are inconsistent";
    case CCA_ERR_LAYOUT: return "invalid head / group layout";
    case CCA_ERR_UNSUPPORTED: return "request not supported by this build";
    case CCA_ERR_WORKSPACE: return "workspace missing or too small";
    case CCA_ERR_ALIGN: return "a pointer is not 16-byte aligned";
    case CCA_ERR_DTYPE: return "dtype must be CCA_BF16 or CCA_F32";
    case CCA_ERR_LAUNCH: return "HIP reported an error while enqueuing";
  }
  return "unknown status";
}

int cca_version(void) { return 200; }

}  // extern "C"
