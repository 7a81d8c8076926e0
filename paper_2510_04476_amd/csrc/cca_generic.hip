// Shape-generic kernels for every stage of the CCA block: fp32 or bf16 storage,
// fp32 arithmetic on the vector ALUs.  They serve the fp32 configuration and
// every bf16 shape the MFMA kernels do not cover.  Simple data-parallel
// mappings, no tuning.
#include "cca_internal.h"

namespace cca {

// ---------------------------------------------------------------------------
// GEMM: C (M,N) = A (M,K) * Bm (K,N).  64x64 tile, 256 threads, 4x4 per thread.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const T *__restrict__ A, const T *__restrict__ Bm,
                                                          T *__restrict__ C, long long M, int N, int K) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 1];
  __shared__ float Bs[BK][BN + 1];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const long long m0 = (long long)blockIdx.y * BM;
  const int n0 = blockIdx.x * BN;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    for (int i = tid; i < BM * BK; i += 256) {
      int r = i / BK, c = i % BK;
      long long gm = m0 + r;
      int gk = k0 + c;
      As[c][r] = (gm < M && gk < K) ? load_f(A + gm * K + gk) : 0.f;
    }
    for (int i = tid; i < BK * BN; i += 256) {
      int r = i / BN, c = i % BN;
      int gk = k0 + r, gn = n0 + c;
      Bs[r][c] = (gk < K && gn < N) ? load_f(Bm + (long long)gk * N + gn) : 0.f;
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
    long long gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
    for (int j = 0; j < 4; ++j) {
      int gn = n0 + tx * 4 + j;
      if (gn < N) store_f(C + gm * N + gn, acc[i][j]);
    }
  }
}

hipError_t gemm_generic(bool bf16, const void *A, const void *Bm, void *C, long long M, int N, int K,
                        hipStream_t s) {
  dim3 grid((N + 63) / 64, (unsigned)((M + 63) / 64));
  if (bf16)
    gemm_generic_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)A, (const bf16_t *)Bm, (bf16_t *)C, M, N, K);
  else
    gemm_generic_kernel<float><<<grid, 256, 0, s>>>((const float *)A, (const float *)Bm, (float *)C, M, N, K);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Prologue: one workgroup per (token, head).  Heads 0..Hq-1 are query heads,
// Hq..Hq+Hk-1 key heads, Hq+Hk..Hq+2Hk-1 value heads.
// ---------------------------------------------------------------------------
struct PrologueArgs {
  int T, Hq, Hk, dh, R, e_q, e_kv, n_lat, v_half, k_seq, k_ch;
  uint32_t flags;
  float rope_base, norm_eps;
};

template <typename T>
__global__ void prologue_generic_kernel(PrologueArgs a, const T *__restrict__ lat, const T *__restrict__ w0,
                                        const T *__restrict__ w1, const float *__restrict__ temp,
                                        T *__restrict__ q, T *__restrict__ k, T *__restrict__ v,
                                        float *__restrict__ rnorm) {
  extern __shared__ float sm[];  // y0[k_ch][dh] | red[blockDim] | yrot[dh]
  const long long row = blockIdx.x;  // b*T + t
  const int t = (int)(row % a.T);
  const int head = blockIdx.y;
  const int dh = a.dh;
  const int tid = threadIdx.x;

  if (head >= a.Hq + a.Hk) {  // value head: copy, second stream delayed by one token
    const int g = head - a.Hq - a.Hk;
    for (int i = tid; i < dh; i += blockDim.x) {
      const int c = g * dh + i;  // channel within e_kv
      float val;
      if (c < a.v_half || !(a.flags & CCA_V_SHIFT))
        val = load_f(lat + row * a.n_lat + a.e_q + a.e_kv + c);
      else
        val = (t == 0) ? 0.f : load_f(lat + (row - 1) * a.n_lat + a.e_q + a.e_kv + c);
      store_f(v + row * a.e_kv + c, val);
    }
    return;
  }

  const bool is_q = head < a.Hq;
  const int ch0 = is_q ? head * dh : a.e_q + (head - a.Hq) * dh;  // first packed q|k channel of this head
  const int kc = (a.flags & CCA_CONV_CH) ? a.k_ch : 1;
  const int ks = (a.flags & CCA_CONV_SEQ) ? a.k_seq : 1;
  float *y0 = sm;                 // [kc][dh]
  float *red = sm + kc * dh;      // [blockDim.x]
  float *yrot = red + blockDim.x; // [dh]

  // conv1_seq output at the kc time steps conv2 needs (zero before the sequence start)
  for (int idx = tid; idx < kc * dh; idx += blockDim.x) {
    const int j = idx / dh, i = idx % dh;
    const int tj = t - (kc - 1) + j;
    float acc = 0.f;
    if (tj >= 0) {
      if (a.flags & CCA_CONV_SEQ) {
        for (int jj = 0; jj < ks; ++jj) {
          const int ts = tj - (ks - 1) + jj;
          if (ts >= 0)
            acc = fmaf(load_f(w0 + (long long)(ch0 + i) * ks + jj),
                       load_f(lat + (row - t + ts) * a.n_lat + ch0 + i), acc);
        }
      } else {
        acc = load_f(lat + (row - t + tj) * a.n_lat + ch0 + i);
      }
    }
    y0[idx] = acc;
  }
  __syncthreads();

  float ssq = 0.f;
  // each thread owns output channels o = tid, tid + blockDim, ...
  for (int o = tid; o < dh; o += blockDim.x) {
    float y;
    if (a.flags & CCA_CONV_CH) {
      y = 0.f;
      const T *wp = w1 + ((long long)head * dh + o) * dh * kc;
      for (int i = 0; i < dh; ++i)
        for (int j = 0; j < kc; ++j) y = fmaf(load_f(wp + i * kc + j), y0[j * dh + i], y);
    } else {
      y = y0[(kc - 1) * dh + o];
    }
    if (a.flags & CCA_QK_MEAN) {
      float m;
      if (is_q) {
        m = 0.5f * (load_f(lat + row * a.n_lat + head * dh + o) +
                    load_f(lat + row * a.n_lat + a.e_q + (head / a.R) * dh + o));
      } else {
        const int g = head - a.Hq;
        float sq = 0.f;
        for (int r = 0; r < a.R; ++r) sq += load_f(lat + row * a.n_lat + (g * a.R + r) * dh + o);
        m = 0.5f * (sq / (float)a.R + load_f(lat + row * a.n_lat + a.e_q + g * dh + o));
      }
      y += m;
    }
    yrot[o] = y;
    ssq = fmaf(y, y, ssq);
  }
  red[tid] = ssq;
  __syncthreads();
  for (int s = blockDim.x / 2; s > 0; s >>= 1) {
    if (tid < s) red[tid] += red[tid + s];
    __syncthreads();
  }
  float mul = 1.f;
  if (a.flags & CCA_QK_NORM) {
    mul = sqrtf((float)dh) / sqrtf(red[0] + a.norm_eps);
    if (!is_q && (a.flags & CCA_KEY_TEMP)) mul *= expf(temp[head - a.Hq]);
  }
  if (rnorm && tid == 0) rnorm[row * (a.Hq + a.Hk) + head] = mul;
  T *dst = is_q ? q + row * a.e_q + head * dh : k + row * a.e_kv + (head - a.Hq) * dh;
  for (int o = tid; o < dh; o += blockDim.x) {
    float y = yrot[o] * mul;
    if (a.flags & CCA_ROPE) {
      const int half = dh / 2;
      int pair, partner;
      bool first;
      if (a.flags & CCA_ROPE_INTERLEAVED) {
        pair = o / 2; first = (o % 2) == 0; partner = first ? o + 1 : o - 1;
      } else {
        pair = o % half; first = o < half; partner = first ? o + half : o - half;
      }
      // angle in fp64: t * theta loses ~1e-3 rad in fp32 at t ~ 16k
      const double theta = pow((double)a.rope_base, -2.0 * (double)pair / (double)dh);
      double sn, cs;
      sincos((double)t * theta, &sn, &cs);
      const float yp = yrot[partner] * mul;
      y = first ? (y * (float)cs - yp * (float)sn) : (y * (float)cs + yp * (float)sn);
    }
    store_f(dst + o, y);
  }
}

hipError_t prologue_generic(const Dims &d, const cca_weights &w, const void *lat, void *q, void *k, void *v,
                            float *rnorm, hipStream_t s) {
  PrologueArgs a{d.T, d.Hq, d.Hk, d.dh, d.R, d.e_q, d.e_kv, d.n_lat, d.v_half, d.k_seq, d.k_ch, d.flags, d.rope_base,
                 d.norm_eps};
  int threads = 64;
  while (threads < d.dh && threads < 256) threads *= 2;
  const int kc = (d.flags & CCA_CONV_CH) ? d.k_ch : 1;
  size_t smem = sizeof(float) * ((size_t)kc * d.dh + threads + d.dh);
  dim3 grid((unsigned)d.rows(), d.Hq + 2 * d.Hk);
  if (d.bf16)
    prologue_generic_kernel<bf16_t><<<grid, threads, smem, s>>>(a, (const bf16_t *)lat, (const bf16_t *)w.w_conv_seq,
                                                               (const bf16_t *)w.w_conv_ch, w.temp, (bf16_t *)q,
                                                               (bf16_t *)k, (bf16_t *)v, rnorm);
  else
    prologue_generic_kernel<float><<<grid, threads, smem, s>>>(a, (const float *)lat, (const float *)w.w_conv_seq,
                                                              (const float *)w.w_conv_ch, w.temp, (float *)q,
                                                              (float *)k, (float *)v, rnorm);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Attention: one wavefront per query row (b, h, t).  Lane l walks keys
// l, l+64, ... with its own running (max, sum, accumulator); the 64 partial
// results are merged at the end.  DH_MAX bounds the per-lane accumulator.
// ---------------------------------------------------------------------------
template <typename T, int DH_MAX>
__global__ __launch_bounds__(64) void attention_generic_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                              const T *__restrict__ v, T *__restrict__ o,
                                                              T *__restrict__ o_lo, float *__restrict__ lse, int Tn,
                                                              int Hq, int Hk, int dh,
                                                              float scale, int causal) {
  __shared__ float qs[DH_MAX];
  const int t = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int g = h / (Hq / Hk);
  const int lane = threadIdx.x;
  const long long qrow = ((long long)b * Tn + t) * Hq + h;
  for (int i = lane; i < dh; i += 64) qs[i] = load_f(q + qrow * dh + i) * scale;
  __syncthreads();
  float m = -INFINITY, z = 0.f;
  float acc[DH_MAX];
#pragma unroll
  for (int i = 0; i < DH_MAX; ++i) acc[i] = 0.f;
  const int s_end = causal ? t + 1 : Tn;
  for (int s = lane; s < s_end; s += 64) {
    const long long krow = ((long long)b * Tn + s) * Hk + g;
    const T *kp = k + krow * dh;
    float dot = 0.f;
    for (int i = 0; i < dh; ++i) dot = fmaf(qs[i], load_f(kp + i), dot);
    const float mn = fmaxf(m, dot);
    const float corr = expf(m - mn);  // exp(-inf) = 0 on the first key
    const float p = expf(dot - mn);
    z = z * corr + p;
    const T *vp = v + krow * dh;
#pragma unroll
    for (int i = 0; i < DH_MAX; ++i)
      if (i < dh) acc[i] = fmaf(p, load_f(vp + i), acc[i] * corr);
    m = mn;
  }
  // merge the 64 lanes
  float M = m;
  for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
  const float f = (m == -INFINITY) ? 0.f : expf(m - M);
  float Z = z * f;
  for (int off = 32; off > 0; off >>= 1) Z += __shfl_xor(Z, off);
  const float inv = 1.f / Z;
#pragma unroll
  for (int i = 0; i < DH_MAX; ++i) {
    if (i < dh) {
      float a = acc[i] * f;
      for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off);
      if (lane == 0) {
        store_f(o + qrow * dh + i, a * inv);
        if (o_lo) store_f(o_lo + qrow * dh + i, a * inv - load_f(o + qrow * dh + i));  // what the rounding dropped
      }
    }
  }
  if (lse && lane == 0) lse[((long long)b * Hq + h) * Tn + t] = M + logf(Z);
}

template <typename T>
static hipError_t attention_generic_t(const Dims &d, const void *q, const void *k, const void *v, void *o,
                                      void *o_lo, float *lse, hipStream_t s) {
  dim3 grid(d.T, d.Hq, d.B);
  const int causal = (d.flags & CCA_CAUSAL) ? 1 : 0;
#define LAUNCH(DH)                                                                                      \
  attention_generic_kernel<T, DH><<<grid, 64, 0, s>>>((const T *)q, (const T *)k, (const T *)v, (T *)o, (T *)o_lo, lse, d.T, \
                                                      d.Hq, d.Hk, d.dh, d.scale, causal)
  if (d.dh <= 32) LAUNCH(32);
  else if (d.dh <= 64) LAUNCH(64);
  else if (d.dh <= 128) LAUNCH(128);
  else LAUNCH(256);
#undef LAUNCH
  return hipGetLastError();
}

hipError_t attention_generic(const Dims &d, const void *q, const void *k, const void *v, void *o, void *o_lo,
                             float *lse, hipStream_t s) {
  // fp32 storage rounds nothing away: no low part
  return d.bf16 ? attention_generic_t<bf16_t>(d, q, k, v, o, o_lo, lse, s)
                : attention_generic_t<float>(d, q, k, v, o, nullptr, lse, s);
}

}  // namespace cca
