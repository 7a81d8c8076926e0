// Internal declarations shared by the HIP translation units of libcca.
// Not part of the C ABI (that is include/cca.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "cca.h"

namespace cca {

// Derived sizes of a validated config.
struct Dims {
  int B, T, E, Hq, Hk, dh, R;
  int e_q, e_kv, n_lat, v_half;  // v_half = channels of the current-token value stream
  int k_seq, k_ch;
  bool bf16;
  uint32_t flags;
  float rope_base, scale;
  float norm_eps;  // added to the sum of squares under the L2 norm (0: the paper's form)
  long long rows() const { return (long long)B * T; }
  size_t esize() const { return bf16 ? 2 : 4; }
};

typedef uint16_t bf16_t;  // raw bf16 bits in memory

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float load_f(const float *p) { return *p; }
__device__ __forceinline__ float load_f(const bf16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void store_f(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_f(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// Raises a kernel's dynamic-LDS limit (needed above 64 KB).  The attribute belongs to the device's copy of the
// kernel and never changes afterwards, so it is set on the first launch per (kernel, device) and remembered in one
// atomic bit mask per kernel: the only state the launchers keep, idempotent and safe from any thread.
template <auto Kernel>
inline hipError_t raise_lds_limit(size_t bytes) {
  static std::atomic<unsigned long long> done{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const unsigned long long bit = 1ull << (dev & 63);
  if (dev < 64 && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess && dev < 64) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// ---- generic kernels (any supported shape, fp32 or bf16 storage) ----------
// C (M,N) = A (M,K) * Bm (K,N), all row-major.
hipError_t gemm_generic(bool bf16, const void *A, const void *Bm, void *C, long long M, int N, int K,
                        hipStream_t s);
hipError_t prologue_generic(const Dims &d, const cca_weights &w, const void *lat, void *q, void *k, void *v,
                            float *rnorm, hipStream_t s);
// o_lo (may be NULL): bf16 storage only, receives the part of the fp32 result that rounding o to bf16 dropped
hipError_t attention_generic(const Dims &d, const void *q, const void *k, const void *v, void *o, void *o_lo,
                             float *lse, hipStream_t s);

// ---- gfx950 MFMA kernels (bf16 storage) -----------------------------------
// C (M,N) = A (M,K) * Bt (N,K)^T; Bt is the K-contiguous ("transposed") weight.
bool gemm_mfma_supported(long long M, int N, int K);
hipError_t gemm_mfma_bf16(const void *A, const void *Bt, void *C, long long M, int N, int K, hipStream_t s);
// dst (cols, rows) = src (rows, cols)^T, bf16.
hipError_t transpose_bf16(const void *src, void *dst, int rows, int cols, hipStream_t s);
// two independent transposes in one launch (src2 may be NULL)
hipError_t transpose2_bf16(const void *src1, void *dst1, int rows1, int cols1, const void *src2, void *dst2, int rows2,
                           int cols2, hipStream_t s);

// measurement aid: blocks x 4 wavefronts x iters x 4 MFMAs (32x32x16 bf16), one float per thread written to out
hipError_t mfma_probe(float *out, int blocks, int iters, bool random_operands, hipStream_t s);

bool attention_mfma_supported(const Dims &d);
// temp (H_k log-temperatures, device) is read only when d.flags has QK_NORM and KEY_TEMP: it bounds the scores
hipError_t attention_mfma_bf16(const Dims &d, const void *q, const void *k, const void *v, void *o, void *o_lo,
                               float *lse, const float *temp, hipStream_t s);

// no transform selected: q, k, v are slices of the latent rows (plus the optional value-shift)
bool prologue_is_split_copy(const Dims &d);
hipError_t prologue_split_copy(const Dims &d, const void *lat, void *q, void *k, void *v, float *rnorm, hipStream_t s);
// its adjoint: no weights, no scratch
hipError_t prologue_split_copy_bwd(const Dims &d, const void *d_q, const void *d_k, const void *d_v, void *d_lat,
                                   hipStream_t s);

// ---- backward of the attention stage (bf16, d_h = 128) ----------------------
bool attention_bwd_supported(const Dims &d);
size_t attention_bwd_scratch_bytes(const Dims &d);  // Delta (B,H_q,T) fp32
hipError_t attention_bwd_bf16(const Dims &d, const void *q, const void *k, const void *v, const void *o,
                              const void *o_lo, const float *lse, const void *d_o, void *d_q, void *d_k, void *d_v, float *delta,
                              hipStream_t s);

// C (Mo,No) = A (K,Mo)^T * B (K,No): weight gradients, contraction over token rows, split over K into fp32
// partial sums in `part` (gemm_tn_scratch_bytes), added in a fixed order.
bool gemm_tn_mfma_supported(int Mo, int No, long long K);
size_t gemm_tn_scratch_bytes(int Mo, int No, long long K);
hipError_t gemm_tn_mfma_bf16(const void *A, long long lda, const void *Bm, long long ldb, void *C, int Mo, int No,
                             long long K, float *part, hipStream_t s);

// ---- generic backward kernels (any supported shape, fp32 or bf16 storage) ----
// C (M,N) = op(A) op(B); ta: A is stored (K,M); tb: B is stored (N,K)
hipError_t gemm_generic_ex(bool bf16, const void *A, long long lda, bool ta, const void *Bm, long long ldb, bool tb,
                           void *C, long long ldc, long long M, int N, long long K, hipStream_t s);
hipError_t attention_bwd_generic(const Dims &d, const void *q, const void *k, const void *v, const void *o,
                                 const void *o_lo, const float *lse, const void *d_o, void *d_q, void *d_k, void *d_v, float *delta,
                                 hipStream_t s);
size_t prologue_bwd_generic_scratch_bytes(const Dims &d);
hipError_t prologue_bwd_generic(const Dims &d, const cca_weights &w, const void *lat, const void *q, const void *k,
                                const float *rnorm, const void *d_q, const void *d_k, const void *d_v, void *d_lat,
                                const cca_grads *gr, void *scratch, hipStream_t s);

// ---- backward of the fused prologue (bf16, d_h = 128, same shapes as the fused forward) ----
bool prologue_bwd_fused_supported(const Dims &d);
size_t prologue_bwd_fused_scratch_bytes(const Dims &d);
hipError_t prologue_bwd_fused_bf16(const Dims &d, const cca_weights &w, const void *lat, const void *q, const void *k,
                                   const float *rnorm, const void *d_q, const void *d_k, const void *d_v, void *d_lat,
                                   const cca_grads *gr, void *scratch, hipStream_t s);

bool prologue_fused_supported(const Dims &d);
size_t prologue_fused_scratch_bytes(const Dims &d);  // folded filters + RoPE tables; 0 if unsupported
hipError_t prologue_fused_bf16(const Dims &d, const cca_weights &w, const void *lat, void *q, void *k, void *v,
                               float *rnorm, void *scratch, hipStream_t s);
// The two halves of prologue_fused_bf16: `scratch` (folded filters, RoPE tables) depends on the weights and the
// config only, so a caller may fill it once (prepare) and run the main kernel many times.
hipError_t prologue_fused_prepare(const Dims &d, const cca_weights &w, void *scratch, hipStream_t s);
hipError_t prologue_fused_run(const Dims &d, const cca_weights &w, const void *lat, void *q, void *k, void *v,
                              float *rnorm, const void *scratch, hipStream_t s);

// ---- decode step (one new token per sequence against the latent KV cache) ----
int decode_ring_rows(const Dims &d);            // latent rows of history the transforms need: max(taps - 1, 1)
size_t decode_scratch_bytes(const Dims &d);
// pos: the position of every sequence; with pos_seq (device, one int per sequence) the largest position, and each
// sequence takes its own (clamped to [0, pos] in the kernels)
hipError_t decode_step(const Dims &d, const cca_weights &w, const void *x_new, void *k_cache, void *v_cache, void *hist,
                       int pos, const int *pos_seq, void *out, void *workspace, hipStream_t s);

}  // namespace cca
