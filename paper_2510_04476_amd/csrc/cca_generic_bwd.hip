// Shape-generic backward kernels (adjoints of the steps of Sec. 2.2, which the
// paper states forward only): fp32 or bf16 storage, fp32 arithmetic on the
// vector ALUs.  They serve the fp32 configuration and every bf16 shape the
// MFMA backward kernels do not cover.  Every sum runs in a fixed order (no
// atomics), so results are reproducible bit for bit.
#include "cca_internal.h"

namespace cca {

// ---------------------------------------------------------------------------
// GEMM with optional transposes: C (M,N) = op(A) * op(B),
//   op(A)[m][k] = ta ? A[k*lda + m] : A[m*lda + k],  op(B)[k][n] = tb ? B[n*ldb + k] : B[k*ldb + n].
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_ex_kernel(const T *__restrict__ A, long long lda, int ta,
                                                             const T *__restrict__ Bm, long long ldb, int tb,
                                                             T *__restrict__ C, long long ldc, long long M, int N,
                                                             long long K) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 1];
  __shared__ float Bs[BK][BN + 1];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const long long m0 = (long long)blockIdx.y * BM;
  const int n0 = blockIdx.x * BN;
  float acc[4][4] = {};
  for (long long k0 = 0; k0 < K; k0 += BK) {
    for (int i = tid; i < BM * BK; i += 256) {
      // walk the contiguous direction of A with consecutive threads
      const int r = ta ? i % BM : i / BK, c = ta ? i / BM : i % BK;
      const long long gm = m0 + r, gk = k0 + c;
      As[c][r] = (gm < M && gk < K) ? load_f(A + (ta ? gk * lda + gm : gm * lda + gk)) : 0.f;
    }
    for (int i = tid; i < BK * BN; i += 256) {
      const int r = tb ? i % BK : i / BN, c = tb ? i / BK : i % BN;
      const long long gk = k0 + r;
      const int gn = n0 + c;
      Bs[r][c] = (gk < K && gn < N) ? load_f(Bm + (tb ? (long long)gn * ldb + gk : gk * ldb + gn)) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i) {
    const long long gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn < N) store_f(C + gm * ldc + gn, acc[i][j]);
    }
  }
}

hipError_t gemm_generic_ex(bool bf16, const void *A, long long lda, bool ta, const void *Bm, long long ldb, bool tb,
                           void *C, long long ldc, long long M, int N, long long K, hipStream_t s) {
  dim3 grid((N + 63) / 64, (unsigned)((M + 63) / 64));
  if (bf16)
    gemm_generic_ex_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)A, lda, ta, (const bf16_t *)Bm, ldb, tb,
                                                       (bf16_t *)C, ldc, M, N, K);
  else
    gemm_generic_ex_kernel<float><<<grid, 256, 0, s>>>((const float *)A, lda, ta, (const float *)Bm, ldb, tb,
                                                      (float *)C, ldc, M, N, K);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Attention backward.  With P = softmax(scale Q K^T) row-wise and
// Delta_t = <dO_t, O_t>:  dS = P * (dO V^T - Delta),  dQ = scale dS K,
// dK = scale dS^T Q,  dV = P^T dO;  dK, dV summed over the query heads of a group.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void delta_generic_kernel(const T *__restrict__ dO, const T *__restrict__ O,
                                                           const T *__restrict__ OLO, float *__restrict__ delta,
                                                           long long n_rows, int Tn, int Hq, int dh) {
  const long long row = (long long)blockIdx.x * 256 + threadIdx.x;  // (b*T + t)*Hq + h
  if (row >= n_rows) return;
  float acc = 0.f;
  for (int i = 0; i < dh; ++i)
    acc = fmaf(load_f(dO + row * dh + i), load_f(O + row * dh + i) + (OLO ? load_f(OLO + row * dh + i) : 0.f), acc);
  const long long bt = row / Hq;
  const int h = (int)(row % Hq);
  delta[((bt / Tn) * Hq + h) * Tn + (bt % Tn)] = acc;
}

// log2-unit score against the forward MFMA kernel's own rounding of q (q * scale * log2(e) rounded to bf16):
// used when that kernel produced lse, so that the recomputed probabilities are exactly its probabilities
__device__ __forceinline__ float q_log2_rounded(float q, float c) { return bf16_to_f32(f32_to_bf16(q * c)); }
constexpr float kLog2e = 1.44269504088896340736f;

// one wavefront per query row (b, h, t); lane l walks keys l, l + 64, ...
template <typename T, int DH_MAX>
__global__ __launch_bounds__(64) void attn_bwd_dq_generic_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                                const T *__restrict__ v, const T *__restrict__ dO,
                                                                const float *__restrict__ lse,
                                                                const float *__restrict__ delta, T *__restrict__ dq,
                                                                int Tn, int Hq, int Hk, int dh, float scale,
                                                                int causal, int q_rounded) {
  __shared__ float qs[DH_MAX], ds_[DH_MAX];
  const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int g = h / (Hq / Hk);
  const int lane = threadIdx.x;
  const long long qrow = ((long long)b * Tn + t) * Hq + h;
  for (int i = lane; i < dh; i += 64) {
    const float qv = load_f(q + qrow * dh + i);
    qs[i] = q_rounded ? q_log2_rounded(qv, scale * kLog2e) : qv * scale;
    ds_[i] = load_f(dO + qrow * dh + i);
  }
  __syncthreads();
  const float L = lse[((long long)b * Hq + h) * Tn + t] * (q_rounded ? kLog2e : 1.f);
  const float Dl = delta[((long long)b * Hq + h) * Tn + t];
  float acc[DH_MAX];
#pragma unroll
  for (int i = 0; i < DH_MAX; ++i) acc[i] = 0.f;
  const int s_end = causal ? t + 1 : Tn;
  for (int s = lane; s < s_end; s += 64) {
    const long long krow = ((long long)b * Tn + s) * Hk + g;
    const T *kp = k + krow * dh, *vp = v + krow * dh;
    float dot = 0.f, dp = 0.f;
    for (int i = 0; i < dh; ++i) {
      dot = fmaf(qs[i], load_f(kp + i), dot);
      dp = fmaf(ds_[i], load_f(vp + i), dp);
    }
    const float dsv = (q_rounded ? exp2f(dot - L) : expf(dot - L)) * (dp - Dl);
#pragma unroll
    for (int i = 0; i < DH_MAX; ++i)
      if (i < dh) acc[i] = fmaf(dsv, load_f(kp + i), acc[i]);
  }
#pragma unroll
  for (int i = 0; i < DH_MAX; ++i) {
    if (i < dh) {
      float a = acc[i];
      for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off);
      if (lane == 0) store_f(dq + qrow * dh + i, a * scale);
    }
  }
}

// one wavefront per key (b, g, s); lanes walk the (query head of the group, query row) pairs that see the key.
// WHICH = 0: dK, 1: dV (one accumulator per lane).
template <typename T, int DH_MAX, int WHICH>
__global__ __launch_bounds__(64) void attn_bwd_dkv_generic_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                                 const T *__restrict__ v, const T *__restrict__ dO,
                                                                 const float *__restrict__ lse,
                                                                 const float *__restrict__ delta, T *__restrict__ out,
                                                                 int Tn, int Hq, int Hk, int dh, float scale,
                                                                 int causal, int q_rounded) {
  __shared__ float ks[DH_MAX], vs[DH_MAX];
  const int s = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int R = Hq / Hk;
  const int lane = threadIdx.x;
  const long long krow = ((long long)b * Tn + s) * Hk + g;
  for (int i = lane; i < dh; i += 64) {
    ks[i] = load_f(k + krow * dh + i) * (q_rounded ? 1.f : scale);
    vs[i] = load_f(v + krow * dh + i);
  }
  __syncthreads();
  float acc[DH_MAX];
#pragma unroll
  for (int i = 0; i < DH_MAX; ++i) acc[i] = 0.f;
  const int t_begin = causal ? s : 0;
  const int nt = Tn - t_begin;
  for (int idx = lane; idx < nt * R; idx += 64) {
    const int h = g * R + idx / nt, t = t_begin + idx % nt;
    const long long qrow = ((long long)b * Tn + t) * Hq + h;
    const T *qp = q + qrow * dh, *dp_ = dO + qrow * dh;
    float dot = 0.f, dp = 0.f;
    for (int i = 0; i < dh; ++i) {
      const float qv = load_f(qp + i);
      dot = fmaf(ks[i], q_rounded ? q_log2_rounded(qv, scale * kLog2e) : qv, dot);
      dp = fmaf(vs[i], load_f(dp_ + i), dp);
    }
    const long long st = ((long long)b * Hq + h) * Tn + t;
    const float p = q_rounded ? exp2f(dot - lse[st] * kLog2e) : expf(dot - lse[st]);
    const float w = WHICH == 0 ? p * (dp - delta[st]) * scale : p;
    const T *src = WHICH == 0 ? qp : dp_;
#pragma unroll
    for (int i = 0; i < DH_MAX; ++i)
      if (i < dh) acc[i] = fmaf(w, load_f(src + i), acc[i]);
  }
#pragma unroll
  for (int i = 0; i < DH_MAX; ++i) {
    if (i < dh) {
      float a = acc[i];
      for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off);
      if (lane == 0) store_f(out + krow * dh + i, a);
    }
  }
}

template <typename T>
static hipError_t attention_bwd_generic_t(const Dims &d, const void *q, const void *k, const void *v, const void *o,
                                          const void *o_lo, const float *lse, const void *d_o, void *d_q, void *d_k, void *d_v,
                                          float *delta, hipStream_t s) {
  const long long n_rows = d.rows() * d.Hq;
  delta_generic_kernel<T><<<(unsigned)((n_rows + 255) / 256), 256, 0, s>>>((const T *)d_o, (const T *)o, (const T *)o_lo, delta, n_rows,
                                                                          d.T, d.Hq, d.dh);
  const int causal = (d.flags & CCA_CAUSAL) ? 1 : 0;
  const int q_rounded = attention_mfma_supported(d) ? 1 : 0;  // lse then comes from the MFMA forward kernel
  dim3 gq(d.T, d.Hq, d.B), gk(d.T, d.Hk, d.B);
#define LAUNCH(DH)                                                                                                    \
  do {                                                                                                                \
    attn_bwd_dq_generic_kernel<T, DH><<<gq, 64, 0, s>>>((const T *)q, (const T *)k, (const T *)v, (const T *)d_o, lse, \
                                                        delta, (T *)d_q, d.T, d.Hq, d.Hk, d.dh, d.scale, causal,      \
                                                        q_rounded);                                                   \
    attn_bwd_dkv_generic_kernel<T, DH, 0><<<gk, 64, 0, s>>>((const T *)q, (const T *)k, (const T *)v, (const T *)d_o,  \
                                                            lse, delta, (T *)d_k, d.T, d.Hq, d.Hk, d.dh, d.scale,     \
                                                            causal, q_rounded);                                       \
    attn_bwd_dkv_generic_kernel<T, DH, 1><<<gk, 64, 0, s>>>((const T *)q, (const T *)k, (const T *)v, (const T *)d_o,  \
                                                            lse, delta, (T *)d_v, d.T, d.Hq, d.Hk, d.dh, d.scale,     \
                                                            causal, q_rounded);                                       \
  } while (0)
  if (d.dh <= 32) LAUNCH(32);
  else if (d.dh <= 64) LAUNCH(64);
  else if (d.dh <= 128) LAUNCH(128);
  else LAUNCH(256);
#undef LAUNCH
  return hipGetLastError();
}

hipError_t attention_bwd_generic(const Dims &d, const void *q, const void *k, const void *v, const void *o,
                                 const void *o_lo, const float *lse, const void *d_o, void *d_q, void *d_k, void *d_v, float *delta,
                                 hipStream_t s) {
  return d.bf16 ? attention_bwd_generic_t<bf16_t>(d, q, k, v, o, o_lo, lse, d_o, d_q, d_k, d_v, delta, s)
                : attention_bwd_generic_t<float>(d, q, k, v, o, nullptr, lse, d_o, d_q, d_k, d_v, delta, s);
}

// ---------------------------------------------------------------------------
// Prologue backward.  Notation: y5 = q / k as they enter attention, d3 = gradient
// of the vectors entering the norm step (= gradient of the conv2 output, since
// qk-mean adds to it), d1 = gradient of the conv1_seq output.  d3, d1 are fp32
// scratch of shape (B*T, e_q + e_kv), q channels first.
// ---------------------------------------------------------------------------
struct ProBwdArgs {
  int T, Hq, Hk, dh, R, e_q, e_kv, n_lat, v_half, k_seq, k_ch;
  long long rows;
  uint32_t flags;
  float rope_base;
};

// RoPE^T, norm / temperature backward.  One workgroup per (token, q or k head).
//   y = x * mul with mul = sqrt(d_h) beta / |x|:  dx = mul * (dy - y <y,dy> / (d_h beta^2)).
template <typename T>
__global__ void pro_bwd_point_generic_kernel(ProBwdArgs a, const T *__restrict__ q, const T *__restrict__ k,
                                             const float *__restrict__ rnorm, const float *__restrict__ temp,
                                             const T *__restrict__ dq, const T *__restrict__ dk,
                                             float *__restrict__ d3, float *__restrict__ rowdot) {
  extern __shared__ float sm[];  // tmp[dh] | red[blockDim]
  const long long row = blockIdx.x;
  const int t = (int)(row % a.T);
  const int head = blockIdx.y, dh = a.dh, tid = threadIdx.x;
  const bool is_q = head < a.Hq;
  const int g = head - a.Hq;
  const T *y5 = is_q ? q + (row * a.Hq + head) * dh : k + (row * a.Hk + g) * dh;
  const T *dy5 = is_q ? dq + (row * a.Hq + head) * dh : dk + (row * a.Hk + g) * dh;
  float *tmp = sm, *red = sm + dh;
  float part = 0.f;
  for (int o = tid; o < dh; o += blockDim.x) part = fmaf(load_f(y5 + o), load_f(dy5 + o), part);
  red[tid] = part;
  __syncthreads();
  for (int s = blockDim.x / 2; s > 0; s >>= 1) {
    if (tid < s) red[tid] += red[tid + s];
    __syncthreads();
  }
  const float dot = red[0];
  float mul = 1.f, c = 0.f;
  if (a.flags & CCA_QK_NORM) {
    mul = rnorm[row * (a.Hq + a.Hk) + head];
    const float beta2 = (!is_q && (a.flags & CCA_KEY_TEMP)) ? expf(2.f * temp[g]) : 1.f;
    c = dot / ((float)dh * beta2);
  }
  if (!is_q && rowdot && tid == 0) rowdot[row * a.Hk + g] = dot;
  for (int o = tid; o < dh; o += blockDim.x) tmp[o] = load_f(dy5 + o) - load_f(y5 + o) * c;
  __syncthreads();
  const int ch0 = is_q ? head * dh : a.e_q + g * dh;
  for (int o = tid; o < dh; o += blockDim.x) {
    float val = tmp[o];
    if (a.flags & CCA_ROPE) {
      const int half = dh / 2;
      int pair, partner;
      bool first;
      if (a.flags & CCA_ROPE_INTERLEAVED) {
        pair = o / 2; first = (o % 2) == 0; partner = first ? o + 1 : o - 1;
      } else {
        pair = o % half; first = o < half; partner = first ? o + half : o - half;
      }
      const double theta = pow((double)a.rope_base, -2.0 * (double)pair / (double)dh);
      double sn, cs;
      sincos((double)t * theta, &sn, &cs);
      // forward: (a, b) -> (a c - b s, b c + a s); adjoint rotates back
      val = first ? (val * (float)cs + tmp[partner] * (float)sn) : (val * (float)cs - tmp[partner] * (float)sn);
    }
    d3[row * (a.e_q + a.e_kv) + ch0 + o] = val * mul;
  }
}

// out[col] = sum over rows of src[row*ncol + col]; one workgroup per column, fixed summation order
__global__ __launch_bounds__(256) void column_sum_kernel(const float *__restrict__ src, long long rows, int ncol,
                                                        float *__restrict__ out) {
  __shared__ float red[256];
  const int col = blockIdx.x, tid = threadIdx.x;
  float acc = 0.f;
  for (long long r = tid; r < rows; r += 256) acc += src[r * ncol + col];
  red[tid] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) red[tid] += red[tid + s];
    __syncthreads();
  }
  if (tid == 0) out[col] = red[0];
}

// conv2_seq+ch transposed: d1[t,h,i] = sum_j sum_o w1[h,o,i,j] d3[t + (k_ch-1-j), h, o] within the sequence
template <typename T>
__global__ void pro_bwd_convch_generic_kernel(ProBwdArgs a, const T *__restrict__ w1, const float *__restrict__ d3,
                                              float *__restrict__ d1) {
  extern __shared__ float sm[];  // d3 rows of the k_ch taps: [kc][dh]
  const long long row = blockIdx.x;
  const int t = (int)(row % a.T);
  const int head = blockIdx.y, dh = a.dh, kc = a.k_ch, tid = threadIdx.x;
  const int ch0 = head < a.Hq ? head * dh : a.e_q + (head - a.Hq) * dh;
  const int ld = a.e_q + a.e_kv;
  for (int idx = tid; idx < kc * dh; idx += blockDim.x) {
    const int j = idx / dh, o = idx % dh;
    const int fwd = kc - 1 - j;
    sm[idx] = (t + fwd < a.T) ? d3[(row + fwd) * ld + ch0 + o] : 0.f;
  }
  __syncthreads();
  for (int i = tid; i < dh; i += blockDim.x) {
    float acc = 0.f;
    for (int o = 0; o < dh; ++o) {
      const T *wp = w1 + (((long long)head * dh + o) * dh + i) * kc;
      for (int j = 0; j < kc; ++j) acc = fmaf(load_f(wp + j), sm[j * dh + o], acc);
    }
    d1[row * ld + ch0 + i] = acc;
  }
}

// conv1_seq transposed + qk-mean adjoint + value-shift adjoint: one thread per element of d_lat
template <typename T>
__global__ __launch_bounds__(256) void pro_bwd_dlat_generic_kernel(ProBwdArgs a, const T *__restrict__ w0,
                                                                  const float *__restrict__ d3,
                                                                  const float *__restrict__ d1,
                                                                  const T *__restrict__ dv, T *__restrict__ d_lat) {
  const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
  if (id >= a.rows * a.n_lat) return;
  const long long row = id / a.n_lat;
  const int c = (int)(id % a.n_lat);
  const int t = (int)(row % a.T);
  const int ld = a.e_q + a.e_kv, dh = a.dh;
  float val;
  if (c < ld) {
    if (a.flags & CCA_CONV_SEQ) {
      val = 0.f;
      for (int jj = 0; jj < a.k_seq; ++jj) {
        const int fwd = a.k_seq - 1 - jj;
        if (t + fwd < a.T) val = fmaf(load_f(w0 + (long long)c * a.k_seq + jj), d1[(row + fwd) * ld + c], val);
      }
    } else {
      val = d1[row * ld + c];
    }
    if (a.flags & CCA_QK_MEAN) {
      // m_q[h] = (q0[h] + k0[g]) / 2 enters q3[h] and, averaged over the group, k3[g]
      if (c < a.e_q) {
        const int h = c / dh, i = c % dh, g = h / a.R;
        val += 0.5f * d3[row * ld + c] + (0.5f / (float)a.R) * d3[row * ld + a.e_q + g * dh + i];
      } else {
        const int g = (c - a.e_q) / dh, i = (c - a.e_q) % dh;
        float sq = 0.f;
        for (int r = 0; r < a.R; ++r) sq += d3[row * ld + (g * a.R + r) * dh + i];
        val += 0.5f * sq + 0.5f * d3[row * ld + c];
      }
    }
  } else {
    const int cc = c - ld;
    const bool shifted = (a.flags & CCA_V_SHIFT) && cc >= a.v_half;
    if (!shifted) val = load_f(dv + row * a.e_kv + cc);
    else val = (t + 1 < a.T) ? load_f(dv + (row + 1) * a.e_kv + cc) : 0.f;
  }
  store_f(d_lat + id, val);
}

// conv1_seq output u1[row, ch] recomputed from the pre-conv latent (zero before the sequence start)
template <typename T>
__device__ __forceinline__ float conv_seq_at(const ProBwdArgs &a, const T *__restrict__ lat, const T *__restrict__ w0,
                                             long long row, int t, int ch) {
  if (!(a.flags & CCA_CONV_SEQ)) return load_f(lat + row * a.n_lat + ch);
  float acc = 0.f;
  for (int jj = 0; jj < a.k_seq; ++jj) {
    const int back = a.k_seq - 1 - jj;
    if (t >= back) acc = fmaf(load_f(w0 + (long long)ch * a.k_seq + jj), load_f(lat + (row - back) * a.n_lat + ch), acc);
  }
  return acc;
}

// dw1[h,o,i,j] = sum_rows d3[row,h,o] * u1[row - (k_ch-1-j), h, i]; one thread per filter element
template <typename T>
__global__ __launch_bounds__(256) void pro_bwd_dw1_generic_kernel(ProBwdArgs a, const T *__restrict__ lat,
                                                                 const T *__restrict__ w0,
                                                                 const float *__restrict__ d3, T *__restrict__ dw1) {
  const int dh = a.dh, kc = a.k_ch;
  const long long id = (long long)blockIdx.x * 256 + threadIdx.x;  // ((h*dh + o)*kc + j)*dh + i: i fastest
  if (id >= (long long)(a.Hq + a.Hk) * dh * dh * kc) return;
  const int i = (int)(id % dh), j = (int)((id / dh) % kc), o = (int)((id / ((long long)dh * kc)) % dh);
  const int h = (int)(id / ((long long)dh * kc * dh));
  const int ch0 = h < a.Hq ? h * dh : a.e_q + (h - a.Hq) * dh;
  const int ld = a.e_q + a.e_kv, back = kc - 1 - j;
  float acc = 0.f;
  for (long long row = 0; row < a.rows; ++row) {
    const int t = (int)(row % a.T);
    if (t < back) continue;
    acc = fmaf(d3[row * ld + ch0 + o], conv_seq_at(a, lat, w0, row - back, t - back, ch0 + i), acc);
  }
  store_f(dw1 + (((long long)h * dh + o) * dh + i) * kc + j, acc);
}

// dw0[c,jj] = sum_rows d1[row,c] * lat[row - (k_seq-1-jj), c]; one thread per filter element
template <typename T>
__global__ __launch_bounds__(256) void pro_bwd_dw0_generic_kernel(ProBwdArgs a, const T *__restrict__ lat,
                                                                 const float *__restrict__ d1, T *__restrict__ dw0) {
  const int ld = a.e_q + a.e_kv;
  const int id = blockIdx.x * 256 + threadIdx.x;  // jj * ld + c: c fastest
  if (id >= ld * a.k_seq) return;
  const int c = id % ld, jj = id / ld, back = a.k_seq - 1 - jj;
  float acc = 0.f;
  for (long long row = 0; row < a.rows; ++row) {
    const int t = (int)(row % a.T);
    if (t < back) continue;
    acc = fmaf(d1[row * ld + c], load_f(lat + (row - back) * a.n_lat + c), acc);
  }
  store_f(dw0 + (long long)c * a.k_seq + jj, acc);
}

size_t prologue_bwd_generic_scratch_bytes(const Dims &d) {
  const size_t plane = (size_t)d.rows() * (d.e_q + d.e_kv) * sizeof(float);
  return 2 * ((plane + 255) / 256 * 256) + (size_t)d.rows() * d.Hk * sizeof(float);
}

template <typename T>
static hipError_t prologue_bwd_generic_t(const Dims &d, const cca_weights &w, const void *lat, const void *q,
                                         const void *k, const float *rnorm, const void *d_q, const void *d_k,
                                         const void *d_v, void *d_lat, const cca_grads *gr, void *scratch,
                                         hipStream_t s) {
  ProBwdArgs a{d.T, d.Hq, d.Hk, d.dh, d.R, d.e_q, d.e_kv, d.n_lat, d.v_half, d.k_seq, d.k_ch, d.rows(), d.flags,
               d.rope_base};
  const size_t plane = ((size_t)d.rows() * (d.e_q + d.e_kv) * sizeof(float) + 255) / 256 * 256;
  float *d3 = reinterpret_cast<float *>(scratch);
  float *d1 = reinterpret_cast<float *>(static_cast<char *>(scratch) + plane);
  float *rowdot = reinterpret_cast<float *>(static_cast<char *>(scratch) + 2 * plane);
  const bool want_temp = (d.flags & CCA_KEY_TEMP) && gr && gr->temp;
  int threads = 64;
  while (threads < d.dh && threads < 256) threads *= 2;
  const int NH = d.Hq + d.Hk;
  dim3 grid_rh((unsigned)d.rows(), NH);
  pro_bwd_point_generic_kernel<T><<<grid_rh, threads, sizeof(float) * (d.dh + threads), s>>>(
      a, (const T *)q, (const T *)k, rnorm, w.temp, (const T *)d_q, (const T *)d_k, d3, want_temp ? rowdot : nullptr);
  if (want_temp) column_sum_kernel<<<d.Hk, 256, 0, s>>>(rowdot, d.rows(), d.Hk, gr->temp);
  if (d.flags & CCA_CONV_CH)
    pro_bwd_convch_generic_kernel<T><<<grid_rh, threads, sizeof(float) * d.k_ch * d.dh, s>>>(
        a, (const T *)w.w_conv_ch, d3, d1);
  else
    d1 = d3;
  const long long n = d.rows() * d.n_lat;
  pro_bwd_dlat_generic_kernel<T><<<(unsigned)((n + 255) / 256), 256, 0, s>>>(a, (const T *)w.w_conv_seq, d3, d1,
                                                                            (const T *)d_v, (T *)d_lat);
  if ((d.flags & CCA_CONV_CH) && gr && gr->w_conv_ch) {
    const long long nw = (long long)NH * d.dh * d.dh * d.k_ch;
    pro_bwd_dw1_generic_kernel<T><<<(unsigned)((nw + 255) / 256), 256, 0, s>>>(a, (const T *)lat,
                                                                              (const T *)w.w_conv_seq, d3,
                                                                              (T *)gr->w_conv_ch);
  }
  if ((d.flags & CCA_CONV_SEQ) && gr && gr->w_conv_seq) {
    const int nw = (d.e_q + d.e_kv) * d.k_seq;
    pro_bwd_dw0_generic_kernel<T><<<(nw + 255) / 256, 256, 0, s>>>(a, (const T *)lat, d1, (T *)gr->w_conv_seq);
  }
  return hipGetLastError();
}

hipError_t prologue_bwd_generic(const Dims &d, const cca_weights &w, const void *lat, const void *q, const void *k,
                                const float *rnorm, const void *d_q, const void *d_k, const void *d_v, void *d_lat,
                                const cca_grads *gr, void *scratch, hipStream_t s) {
  return d.bf16 ? prologue_bwd_generic_t<bf16_t>(d, w, lat, q, k, rnorm, d_q, d_k, d_v, d_lat, gr, scratch, s)
                : prologue_bwd_generic_t<float>(d, w, lat, q, k, rnorm, d_q, d_k, d_v, d_lat, gr, scratch, s);
}

}  // namespace cca
