/*
 * cca.h — C ABI of the MI355X (gfx950) implementation of the prefill hot path
 * of Compressed Convolutional Attention (CCA) and its grouped-query variant
 * CCGQA (arXiv 2510.04476, Sec. 2.2 and App. A).
 *
 * The block maps hidden states x (B,T,E) to out (B,T,E):
 *   down-projection to latent q, k and two value streams  (Sec. 2.2, down-projection eq.; value-shift eq.)
 *   conv1_seq, conv2_seq+ch on q and k                     (Sec. 2.2, convolution eq.)
 *   qk-mean                                                (Sec. 2.2, qk-mean eq.)
 *   value-shift                                            (Sec. 2.2, value-shift eq.)
 *   L2 norm * sqrt(d_h), key temperature, RoPE             (Sec. 2.2, final eq. block, lines 1-2)
 *   causal softmax attention in the latent space, KV heads
 *   shared by groups of query heads (CCGQA)                (final eq. block, line 3; CCGQA paragraph)
 *   up-projection                                          (final eq. block, line 4)
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer (HIP), row-major, contiguous,
 *     16-byte aligned, owned by the caller.  The config / weight / saved
 *     structs themselves live in HOST memory.
 *   - The library never allocates, frees or synchronises (the one buffer it
 *     owns is the fixed array behind cca_decode_step_static).  All work is
 *     enqueued on the caller's stream (`hip_stream` is a hipStream_t, NULL =
 *     the default stream) and the call returns at once.
 *   - Arguments are validated on the host before the first HIP call; a failed
 *     validation enqueues nothing.  Errors are negative cca_status values.
 *   - Storage type (`dtype`) applies to x, weights (except temp), latents and
 *     out.  Accumulation is always fp32.  bf16 tensors are rounded to nearest
 *     even once per stored tensor.
 *   - No global mutable state: calls on different streams may run
 *     concurrently as long as their buffers (workspace included) are disjoint
 *     (cca_decode_step_static is the exception: see there).
 *
 * Symbols: B batch, T sequence length, E = d_model, H_q / H_k latent query /
 * KV heads, d_h latent head width, e_q = H_q*d_h (= E/C1), e_kv = H_k*d_h
 * (= E/C2), R = H_q/H_k query heads per KV head, N_lat = e_q + 2*e_kv.
 */
#ifndef CCA_H_
#define CCA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
/* The library is built with hidden visibility; only what is declared here is exported. */
#pragma GCC visibility push(default)

typedef enum {
  CCA_OK = 0,
  CCA_ERR_NULL = -1,        /* a required pointer is NULL */
  CCA_ERR_SHAPE = -2,       /* a size is non-positive or the sizes are inconsistent */
  CCA_ERR_LAYOUT = -3,      /* head/group layout invalid (H_q % H_k, odd e_kv with value-shift, odd d_h with RoPE) */
  CCA_ERR_UNSUPPORTED = -4, /* valid request this build has no kernel for */
  CCA_ERR_WORKSPACE = -5,   /* workspace NULL or smaller than cca_workspace_size says */
  CCA_ERR_ALIGN = -6,       /* a pointer is not 16-byte aligned */
  CCA_ERR_DTYPE = -7,       /* dtype is neither CCA_BF16 nor CCA_F32 */
  CCA_ERR_LAUNCH = -8       /* HIP reported an error while enqueuing */
} cca_status;

typedef enum { CCA_BF16 = 0, CCA_F32 = 1 } cca_dtype;

/* Feature flags: each optional transform of Sec. 2.2 can be switched on its
 * own (the paper's ablation tables switch the same ones). */
enum {
  CCA_CAUSAL = 1u << 0,           /* attend to s <= t only */
  CCA_CONV_SEQ = 1u << 1,         /* conv1_seq: depth-wise causal conv, width k_seq */
  CCA_CONV_CH = 1u << 2,          /* conv2_seq+ch: per-head dense d_h x d_h causal conv, width k_ch */
  CCA_QK_MEAN = 1u << 3,          /* qk-mean skip branch from the pre-conv latents */
  CCA_V_SHIFT = 1u << 4,          /* second half of the value channels comes from token t-1 */
  CCA_QK_NORM = 1u << 5,          /* L2 norm over d_h, times sqrt(d_h) */
  CCA_KEY_TEMP = 1u << 6,         /* key times exp(temp[g]); requires CCA_QK_NORM */
  CCA_ROPE = 1u << 7,             /* rotary embedding on q and k, full head width, positions 0..T-1 */
  CCA_ROPE_INTERLEAVED = 1u << 8  /* pairs (2i,2i+1) instead of (i, i+d_h/2) */
};
#define CCA_FLAGS_PAPER                                                                         \
  (CCA_CAUSAL | CCA_CONV_SEQ | CCA_CONV_CH | CCA_QK_MEAN | CCA_V_SHIFT | CCA_QK_NORM | CCA_KEY_TEMP | \
   CCA_ROPE)
/* Plain MHA / GQA (Sec. 2.1) through the same kernels: e_q = E, no transforms. */
#define CCA_FLAGS_MHA (CCA_CAUSAL)

typedef struct {
  int32_t B, T, d_model;
  int32_t compress_q, compress_kv;         /* C1, C2 of Sec. 2.2 (query / key-value compression, C2 >= C1; equal for
                                              plain CCA).  Each is either 0 (derived from the head layout, not
                                              checked) or must satisfy d_model == C * heads * head_dim exactly
                                              (compress_q with n_q_heads, compress_kv with n_kv_heads), else
                                              CCA_ERR_SHAPE.  Plain MHA: 1 and 1. */
  int32_t n_q_heads, n_kv_heads, head_dim; /* H_q, H_k, d_h; H_q % H_k == 0 */
  int32_t k_seq, k_ch;                     /* conv widths, 1..4; ignored when the conv's flag is off */
  int32_t dtype;                           /* cca_dtype */
  uint32_t flags;
  float rope_base;                         /* e.g. 10000; must be > 0 when CCA_ROPE */
  float softmax_scale;                     /* 0 => 1/sqrt(d_h) */
  float norm_eps;                          /* CCA_QK_NORM divides by sqrt(sum u^2 + norm_eps).  0 => the paper's form
                                              (App. A listing: plain L2 norm, no epsilon).  Must be >= 0. */
} cca_config;

/* Weights (device pointers, read-only).  Pointers whose flag is off may be NULL. */
typedef struct {
  const void *w_down;     /* (E, N_lat): columns [W_Q (e_q) | W_K (e_kv) | W_V (e_kv/2) | W_Vbar (e_kv - e_kv/2)] */
  const void *w_conv_seq; /* (e_q + e_kv, k_seq): depth-wise filter per packed q|k channel; tap k_seq-1 multiplies token t */
  const void *w_conv_ch;  /* (H_q + H_k, d_h_out, d_h_in, k_ch): q heads first, then KV heads; tap k_ch-1 multiplies token t */
  const float *temp;      /* (H_k) fp32 log-temperature, beta_g = exp(temp[g]) */
  const void *w_out;      /* (e_q, E) */
  const void *prepared;   /* optional, may be NULL: a buffer that cca_prepare filled from THESE weights under a
                             config equal to the call's in every field but B (cca_prepared_size bytes, caller-
                             owned).  It holds what depends on the weights and the config only - both projection
                             weights in the layout the matrix-core GEMM reads, the two convolutions folded into
                             one filter per head, the RoPE angle tables - so that cca_forward does not derive
                             them again on every call.  Results are bit-identical with and without it.  Read by
                             cca_forward only; the library cannot check that it matches the weights. */
} cca_weights;

/* Intermediates (device pointers, caller-owned).  Any member may be NULL; a
 * non-NULL member is written by cca_forward in place of workspace storage. */
typedef struct {
  void *lat;  /* (B,T,N_lat) down-projection output, columns as in w_down */
  void *q;    /* (B,T,H_q,d_h) query as it enters attention */
  void *k;    /* (B,T,H_k,d_h) key   as it enters attention */
  void *v;    /* (B,T,H_k,d_h) value as it enters attention */
  void *o;    /* (B,T,H_q*d_h) attention output */
  float *lse; /* (B,H_q,T) natural-log sum-exp of the scaled logits */
  float *rnorm; /* (B,T,H_q+H_k) factor the norm step multiplied each head vector by: sqrt(d_h) [* beta] / |x|;
                   1 when CCA_QK_NORM is off.  Needed by cca_backward. */
  void *o_lo;   /* (B,T,H_q*d_h), bf16 storage only (not written with CCA_F32): the part of the fp32 attention
                   result that rounding `o` to bf16 dropped, itself rounded to bf16.  Optional for
                   cca_backward: with it <d_o, o> is formed from o + o_lo; without it the rounding error of o
                   can dominate d_q and d_k when the softmax is flat. */
} cca_saved;

/* Gradients of the weights (device pointers, caller-owned, same shapes and
 * storage type as cca_weights; temp fp32).  cca_backward OVERWRITES each
 * non-NULL member (it does not accumulate); a NULL member is not computed. */
typedef struct {
  void *w_down;     /* (E, N_lat) */
  void *w_conv_seq; /* (e_q + e_kv, k_seq); ignored when CCA_CONV_SEQ is off */
  void *w_conv_ch;  /* (H_q + H_k, d_h, d_h, k_ch); ignored when CCA_CONV_CH is off */
  float *temp;      /* (H_k) fp32; ignored when CCA_KEY_TEMP is off */
  void *w_out;      /* (e_q, E) */
} cca_grads;

/* Bytes of device workspace cca_forward (*fwd_bytes) and cca_backward
 * (*bwd_bytes) need for `cfg`, independent of which cca_saved members are
 * given.  Either out-pointer may be NULL (not wanted), not both.  Returns
 * CCA_OK or a validation error. */
cca_status cca_workspace_size(const cca_config *cfg, size_t *fwd_bytes, size_t *bwd_bytes);

/* The second figure alone (same as cca_workspace_size(cfg, NULL, bwd_bytes)). */
cca_status cca_backward_workspace_size(const cca_config *cfg, size_t *bwd_bytes);

/* Bytes of the buffer cca_prepare fills for `cfg` (0 when this config has
 * nothing to prepare: fp32 storage, or shapes off the matrix-core kernels). */
cca_status cca_prepared_size(const cca_config *cfg, size_t *bytes);

/* One-time set-up per set of weights (Sec. 2.2: the projection weights, the
 * two convolution filters and the RoPE angles do not change between calls):
 * fills `prepared` (device memory, 16-byte aligned, at least
 * cca_prepared_size bytes, caller-owned) on the caller's stream.  Pass the
 * buffer as cca_weights.prepared to cca_forward.  Allocates nothing. */
cca_status cca_prepare(const cca_config *cfg, const cca_weights *w, void *prepared, size_t prepared_bytes,
                       void *hip_stream);

/* Whole block.  x: (B,T,E) in, out: (B,T,E) overwritten.  `saved` may be NULL.
 * `workspace` is scratch of at least cca_workspace_size() bytes whose
 * contents are undefined afterwards. */
cca_status cca_forward(const cca_config *cfg, const cca_weights *w, const void *x, void *out,
                       const cca_saved *saved, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Gradient of the whole block (the paper gives no backward equations: this is
 * the adjoint of the steps of Sec. 2.2, last step first).  Given d_out =
 * dLoss/d out (B,T,E) and the intermediates `saved` that cca_forward wrote for
 * the SAME cfg, weights and x (every member required except o_lo), computes
 *   d_x (B,T,E)            overwritten; may be NULL (then not computed)
 *   grads->...             see cca_grads; `grads` itself may be NULL.
 * Attention probabilities are recomputed from saved->lse (nothing of size
 * T x T is stored); the convolution inputs are re-read from saved->lat.
 * Deterministic: no floating-point atomics, a repeated call gives the same
 * bits.  `workspace`: at least cca_backward_workspace_size() bytes, contents
 * undefined afterwards. */
cca_status cca_backward(const cca_config *cfg, const cca_weights *w, const void *x, const cca_saved *saved,
                        const void *d_out, void *d_x, const cca_grads *grads, void *workspace,
                        size_t workspace_bytes, void *hip_stream);

/* ---- the four stages of cca_forward, callable on their own ---------------
 * Same validation and conventions.  They exist so that each stage can be
 * checked against the oracle and timed separately.  Where a stage takes a
 * workspace, cca_workspace_size() bytes always suffice (a stage may need
 * none; then NULL / 0 is accepted). */

/* lat (B*T, N_lat) = x (B*T, E) * w_down (E, N_lat).  Down-projection eq. of Sec. 2.2. */
cca_status cca_down_project(const cca_config *cfg, const void *x, const void *w_down, void *lat,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/* lat -> q, k, v: convolutions, qk-mean, value-shift, norm, temperature, RoPE
 * as selected by cfg->flags.  w->w_down / w->w_out are not read.  The
 * workspace holds the folded convolution filters and the RoPE tables. */
cca_status cca_prologue(const cca_config *cfg, const cca_weights *w, const void *lat, void *q, void *k,
                        void *v, float *rnorm_or_null, void *workspace, size_t workspace_bytes, void *hip_stream);

/* o (B,T,H_q*d_h) = softmax(scale * q k^T [causal]) v per latent head, query
 * head h reading KV head h / R.  lse and o_lo (see cca_saved) may be NULL.
 * With bf16 storage the probabilities enter the PV product rounded to bf16.
 * When lse or o_lo is requested (a backward pass will consume o) the row is
 * normalised by the sum of those rounded probabilities, so o is exactly the
 * convex combination that was formed; when neither is requested it is
 * normalised by the fp32 sum (a common factor 1 + delta per row, |delta| <=
 * 2^-8, at most the rounding of o itself) and the kernel is a few percent faster.
 * If cfg->flags has CCA_QK_NORM the caller PROMISES that q and k are what
 * cca_prologue writes under that flag: |q[t,h]| = sqrt(d_h) and |k[t,g]| =
 * sqrt(d_h) * exp(temp[g]) (temp: H_k fp32 log-temperatures on the device,
 * required with CCA_KEY_TEMP, else ignored and may be NULL).  The kernel uses
 * the resulting bound on the scores in place of the running row max; q / k
 * that break the promise give undefined results.  Clear CCA_QK_NORM in cfg to
 * attend over arbitrary q, k. */
cca_status cca_attention(const cca_config *cfg, const void *q, const void *k, const void *v, void *o,
                         void *o_lo, float *lse, const float *temp, void *hip_stream);

/* Backward of cca_attention (the paper gives no backward equations; this is
 * the adjoint of the attention line of the final eq. block): from q, k, v, o,
 * lse of the forward pass and d_o (B,T,H_q*d_h) computes d_q (B,T,H_q,d_h),
 * d_k, d_v (B,T,H_k,d_h), overwritten; d_k, d_v are summed over the query
 * heads sharing a KV head.  Probabilities are recomputed from lse.
 * workspace: B*H_q*T*4 bytes (rounded up to 256) plus, when H_q > H_k,
 * 2*B*T*H_q*d_h*4 bytes for the per-query-head partial sums of d_k and d_v,
 * plus B*T*H_q*d_h*2 bytes for the rescaled q;
 * cca_backward_workspace_size() bytes always suffice. */
cca_status cca_attention_backward(const cca_config *cfg, const void *q, const void *k, const void *v,
                                  const void *o, const void *o_lo_or_null, const float *lse, const void *d_o, void *d_q, void *d_k,
                                  void *d_v, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Backward of cca_prologue: from d_q (B,T,H_q,d_h), d_k, d_v (B,T,H_k,d_h)
 * (gradients of what cca_prologue wrote), the saved lat, q, k and rnorm of the
 * forward pass, computes d_lat (B,T,N_lat) and, where the pointer is non-NULL
 * and the flag is on, grads->w_conv_seq, grads->w_conv_ch, grads->temp
 * (grads->w_down / w_out are not touched).  workspace:
 * cca_backward_workspace_size() bytes always suffice. */
cca_status cca_prologue_backward(const cca_config *cfg, const cca_weights *w, const void *lat, const void *q,
                                 const void *k, const float *rnorm, const void *d_q, const void *d_k,
                                 const void *d_v, void *d_lat, const cca_grads *grads, void *workspace,
                                 size_t workspace_bytes, void *hip_stream);

/* out (B*T, E) = o (B*T, e_q) * w_out (e_q, E).  Last line of the final eq. block. */
cca_status cca_up_project(const cca_config *cfg, const void *o, const void *w_out, void *out,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---- decode: one new token per sequence against the latent KV cache -------
 * Sec. 2.2 and the cost table (KV-cache and decode-FLOPs columns): what is
 * cached per token are the latent key and value AFTER every transform, i.e.
 * the k and v that cca_prologue / cca_forward write (cca_saved.k, .v), so a
 * prefill leaves the cache ready.  cfg->T is the CAPACITY of the cache. */
typedef struct {
  void *k_cache;  /* (B, T, H_k, d_h): rows 0..pos-1 valid on entry; row pos is written */
  void *v_cache;  /* (B, T, H_k, d_h): likewise */
  void *lat_ring; /* (B, P, N_lat): the down-projected rows of the last P tokens, token s in slot s % P, where
                     P = max(k_seq + k_ch - 2, 1) + 1 counting only the convolutions whose flag is on
                     (cca_decode_workspace_size reports it): the earlier rows the convolutions and the value
                     shift reach back to, plus the new token's own row, which the step writes into slot
                     pos % P.  After a prefill: copy the last P - 1 (or P) rows of cca_saved.lat.  Slots of
                     tokens before the sequence start are never read. */
} cca_decode_state;

/* Bytes of device workspace one step needs, and (optional) the ring depth P. */
cca_status cca_decode_workspace_size(const cca_config *cfg, size_t *bytes, int32_t *ring_rows);

/* out (B, E) = the block's output for the token at position `pos` (0-based;
 * `pos` tokens are already in the cache) given its hidden state x_new (B, E).
 * By causality this equals row `pos` of cca_forward over tokens 0..pos.  All
 * sequences of the batch are at the same position.  Requires d_h % 8 == 0 and
 * CCA_CAUSAL semantics (a new token attends to everything cached).  Updates
 * `state` in place; every pointer is device memory, 16-byte aligned.
 * Errors as for cca_forward; CCA_ERR_SHAPE when pos is outside [0, T). */
cca_status cca_decode_step(const cca_config *cfg, const cca_weights *w, const void *x_new,
                           const cca_decode_state *state, int32_t pos, void *out, void *workspace,
                           size_t workspace_bytes, void *hip_stream);

/* The same step for a batch whose sequences are at DIFFERENT positions (a serving batch of mixed lengths):
 * `pos` is a DEVICE array of B int32 (4-byte aligned), sequence b's new token is at position pos[b] and attends
 * to its cache rows 0..pos[b]; `max_pos` (host) is an upper bound of every entry, 0 <= max_pos < T
 * (CCA_ERR_SHAPE otherwise) - it sizes the split of the key range, and every entry is clamped into
 * [0, max_pos] on the device, so that no value in the array can carry an access outside the cache.  Row b of the
 * result equals row pos[b] of cca_forward over that sequence's tokens 0..pos[b] (Sec. 2.2; causality).  The
 * array is read by the kernels of this call only; everything else as for cca_decode_step. */
cca_status cca_decode_step_ragged(const cca_config *cfg, const cca_weights *w, const void *x_new,
                                  const cca_decode_state *state, const int32_t *pos, int32_t max_pos, void *out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

/* cca_decode_step for callers that cannot hand over a workspace and must not
 * allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, results and errors as
 * cca_decode_step, but the step's scratch (new query, attention partial sums
 * per cache split, split-K sums of the two projections) lives in a
 * CCA_DECODE_STATIC_BYTES array that is part of the loaded library (one copy
 * per GPU, held until the process ends).  Calls no allocating routine.
 * Returns CCA_ERR_WORKSPACE when cca_decode_workspace_size(cfg) exceeds
 * CCA_DECODE_STATIC_BYTES (nothing is enqueued then) and CCA_ERR_LAUNCH when
 * the array's address cannot be obtained on the current device.  Every call
 * on a GPU uses that GPU's one array: two calls whose kernels may overlap in
 * time on the same GPU (different streams, or concurrent host threads) race;
 * calls on one stream are ordered and safe.  Nothing in the array has to
 * start at zero: each step writes every partial sum before reading it. */
#define CCA_DECODE_STATIC_BYTES (16u << 20)
cca_status cca_decode_step_static(const cca_config *cfg, const cca_weights *w, const void *x_new,
                                  const cca_decode_state *state, int32_t pos, void *out, void *hip_stream);

/* Measurement aid (not a step of the method): enqueues a kernel of `blocks`
 * workgroups x 4 wavefronts that issue iters x 4 independent 32x32x16 bf16
 * matrix-core instructions each and nothing else, and stores the number of
 * floating-point operations that is (2*32*32*16 per instruction) in *flops
 * (host memory).  Timing the launch gives the matrix-core rate the chip
 * sustains - the measured ceiling quoted beside the nominal peak.
 * `operands` = 0: every instruction multiplies the same few small constants;
 * 1: the operands are pseudo-random values in (-2, 2), as activations are
 * (8 register sets in rotation) - the chip draws more power multiplying
 * those and holds a lower clock, so this is the ceiling a kernel on real
 * data meets.
 * `iters` must be even.  `out`: device scratch of at least
 * blocks * 256 * 4 bytes, overwritten.  CCA_ERR_UNSUPPORTED for another `operands`. */
cca_status cca_probe_mfma_rate(void *out, size_t out_bytes, int32_t blocks, int32_t iters, int32_t operands,
                               double *flops, void *hip_stream);

/* Human-readable text for a status; never NULL; static storage. */
const char *cca_strerror(cca_status s);

/* Library version: major*10000 + minor*100 + patch. */
int cca_version(void);

#pragma GCC visibility pop
#ifdef __cplusplus
}
#endif
#endif /* CCA_H_ */
