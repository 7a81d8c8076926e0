// One autoregressive decode step of the block (Sec. 2.2; the cost table's KV-cache and decode-FLOPs columns):
// what is cached per token are the latent keys and values AFTER every transform, exactly what the prefill
// prologue writes, so prefill and decode share one cache.  By causality the result of a step at position t is
// row t of the whole block applied to the tokens 0..t; that identity is what the tests check.
//
// Per step and sequence:  lat = x W_down (small GEMM);  conv / qk-mean / value-shift / norm / temperature / RoPE
// for the ONE new token from a ring of latent rows (the D-1 earlier rows the D = k_seq + k_ch - 1 taps reach, one
// at least for the value shift, plus the new row, which the projection writes straight into its slot);  k, v appended to the cache;  attention of the new query against the cache;  out = o W_O.
// The attention is bound by reading the cache (2 * len * H_k * d_h elements per sequence), so the key range is
// split over workgroups (each serves all R query heads of one KV head: the cache is read once per group, not
// once per query head) and a second kernel merges the partial softmax states in a fixed order.
#include <type_traits>

#include "cca_internal.h"

namespace cca {

namespace {

constexpr int R_MAX = 8;       // query heads of a group handled per pass over the cache
constexpr int DEC_WAVES = 4;   // wavefronts per workgroup of the attention kernel
constexpr int MAX_SPLITS = 32;

struct DecArgs {
  int B, S, Hq, Hk, dh, R, e_q, e_kv, n_lat, v_half, k_seq, k_ch, P, pos;
  uint32_t flags;
  float rope_base, scale, norm_eps;
  const int *pos_seq;  // per-sequence positions (device, B entries) or null: every sequence at `pos`
};

// Position of sequence b's new token.  With per-sequence positions `pos` is the largest one the host vouched for
// (it is below the cache capacity); a value outside [0, pos] is clamped into that range, so whatever the array
// holds no cache or ring access can leave its allocation.
__device__ __forceinline__ int seq_pos(const DecArgs &a, int b) {
  if (!a.pos_seq) return a.pos;
  const int p = a.pos_seq[b];
  return p < 0 ? 0 : (p > a.pos ? a.pos : p);
}

// N consecutive elements as one vector load (N * sizeof(T) bytes, aligned by construction: head offsets and
// channel offsets are multiples of N elements)
template <int N>
__device__ __forceinline__ void load_vec(const float *p, float *dst) {
  typedef float fv __attribute__((ext_vector_type(N)));
  if constexpr (N == 1) {
    dst[0] = *p;
  } else if constexpr (N == 8) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 a = *reinterpret_cast<const f4 *>(p), b = *reinterpret_cast<const f4 *>(p + 4);
    dst[0] = a.x; dst[1] = a.y; dst[2] = a.z; dst[3] = a.w; dst[4] = b.x; dst[5] = b.y; dst[6] = b.z; dst[7] = b.w;
  } else {
    const fv v = *reinterpret_cast<const fv *>(p);
#pragma unroll
    for (int i = 0; i < N; ++i) dst[i] = v[i];
  }
}
template <int N>
__device__ __forceinline__ void load_vec(const bf16_t *p, float *dst) {
  if constexpr (N == 1) {
    dst[0] = bf16_to_f32(*p);
  } else {
    typedef uint32_t uv __attribute__((ext_vector_type(N / 2)));
    if constexpr (N == 2) {
      const uint32_t w = *reinterpret_cast<const uint32_t *>(p);
      dst[0] = __uint_as_float(w << 16);
      dst[1] = __uint_as_float(w & 0xffff0000u);
    } else {
      const uv v = *reinterpret_cast<const uv *>(p);
#pragma unroll
      for (int i = 0; i < N / 2; ++i) {
        dst[2 * i] = __uint_as_float(v[i] << 16);
        dst[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
      }
    }
  }
}

// latent row of token `tok` of sequence b: ring slot tok % P (the new token's row is written there by the projection)
template <typename T>
__device__ __forceinline__ const T *lat_row(const DecArgs &a, const T *hist, int b, int tok) {
  return hist + ((long long)b * a.P + tok % a.P) * a.n_lat;
}

// ---------------------------------------------------------------------------
// Transforms of the new token: one workgroup per (sequence, head); heads 0..Hq-1 query, then Hk key, then Hk value.
// Same arithmetic, in the same order, as the shape-generic prefill prologue.
// ---------------------------------------------------------------------------
template <typename T>
__global__ void decode_prologue_kernel(DecArgs a, const T *__restrict__ hist,
                                       const T *__restrict__ w0, const T *__restrict__ w1,
                                       const float *__restrict__ temp, float *__restrict__ q_new,
                                       T *__restrict__ k_cache, T *__restrict__ v_cache) {
  extern __shared__ float sm[];  // y0[dh][k_ch] | red[blockDim] | yrot[dh]
  const int b = blockIdx.x, head = blockIdx.y, dh = a.dh, tid = threadIdx.x, t = seq_pos(a, b);
  const long long crow = (long long)b * a.S + t;  // cache row of the new token

  if (head >= a.Hq + a.Hk) {  // value head: second stream delayed by one token
    const int g = head - a.Hq - a.Hk;
    const T *cur = lat_row(a, hist, b, t) + a.e_q + a.e_kv;
    const T *prev = t > 0 ? lat_row(a, hist, b, t - 1) + a.e_q + a.e_kv : nullptr;
    for (int i = tid; i < dh; i += blockDim.x) {
      const int c = g * dh + i;
      float val;
      if (c < a.v_half || !(a.flags & CCA_V_SHIFT)) val = load_f(cur + c);
      else val = prev ? load_f(prev + c) : 0.f;
      store_f(v_cache + crow * a.e_kv + c, val);
    }
    return;
  }

  const bool is_q = head < a.Hq;
  const int ch0 = is_q ? head * dh : a.e_q + (head - a.Hq) * dh;
  const int kc = (a.flags & CCA_CONV_CH) ? a.k_ch : 1;
  const int ks = (a.flags & CCA_CONV_SEQ) ? a.k_seq : 1;
  float *y0 = sm, *red = sm + kc * dh, *yrot = red + blockDim.x;

  for (int idx = tid; idx < kc * dh; idx += blockDim.x) {
    const int j = idx / dh, i = idx % dh;
    const int tj = t - (kc - 1) + j;
    float acc = 0.f;
    if (tj >= 0) {
      if (a.flags & CCA_CONV_SEQ) {
        for (int jj = 0; jj < ks; ++jj) {
          const int ts = tj - (ks - 1) + jj;
          if (ts >= 0)
            acc = fmaf(load_f(w0 + (long long)(ch0 + i) * ks + jj), load_f(lat_row(a, hist, b, ts) + ch0 + i), acc);
        }
      } else {
        acc = load_f(lat_row(a, hist, b, tj) + ch0 + i);
      }
    }
    y0[i * kc + j] = acc;  // in the order the channel filter stores its (input channel, tap) pairs
  }
  __syncthreads();

  const T *me = lat_row(a, hist, b, t);
  float ssq = 0.f;
  for (int o = tid; o < dh; o += blockDim.x) {
    float y;
    if (a.flags & CCA_CONV_CH) {
      y = 0.f;
      const T *wp = w1 + ((long long)head * dh + o) * dh * kc;  // one contiguous row of d_h * k_ch weights
      int c8 = 0;
      for (; c8 + 32 <= dh * kc; c8 += 32) {  // four 16-byte loads in flight; the sum keeps its order
        float wv[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) load_vec<8>(wp + c8 + 8 * u, wv[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int e = 0; e < 8; ++e) y = fmaf(wv[u][e], y0[c8 + 8 * u + e], y);
      }
      for (; c8 < dh * kc; c8 += 8) {
        float wv[8];
        load_vec<8>(wp + c8, wv);
#pragma unroll
        for (int e = 0; e < 8; ++e) y = fmaf(wv[e], y0[c8 + e], y);
      }
    } else {
      y = y0[o * kc + (kc - 1)];
    }
    if (a.flags & CCA_QK_MEAN) {
      float m;
      if (is_q) {
        m = 0.5f * (load_f(me + head * dh + o) + load_f(me + a.e_q + (head / a.R) * dh + o));
      } else {
        const int g = head - a.Hq;
        float sq = 0.f;
        for (int r = 0; r < a.R; ++r) sq += load_f(me + (g * a.R + r) * dh + o);
        m = 0.5f * (sq / (float)a.R + load_f(me + a.e_q + g * dh + o));
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
      const double theta = pow((double)a.rope_base, -2.0 * (double)pair / (double)dh);
      double sn, cs;
      sincos((double)t * theta, &sn, &cs);
      const float yp = yrot[partner] * mul;
      y = first ? (y * (float)cs - yp * (float)sn) : (y * (float)cs + yp * (float)sn);
    }
    if (is_q) {
      // the query goes through the storage type once, as the prefill's q does, then stays fp32 for the dot products
      T tmp;
      store_f(&tmp, y);
      q_new[((long long)b * a.Hq + head) * dh + o] = load_f(&tmp);
    } else {
      store_f(k_cache + crow * a.e_kv + (head - a.Hq) * dh + o, y);
    }
  }
}

// ---------------------------------------------------------------------------
// Attention of the new queries against the cache.  Workgroup = (sequence, KV head, split of the key range), 4
// wavefronts, each walking its share of the split 64 keys at a time: for the scores a lane owns ONE key (its row
// of K, 8 elements per load) and all R query heads; for P V a lane owns CPL adjacent channels and the probabilities come
// from LDS.  Online softmax per wavefront in log2 units; the wavefronts' states are merged through LDS.
// Partial result per (sequence, query head, split): m, l, o[d_h] in fp32.
// ---------------------------------------------------------------------------
// CPL = channels per lane in the P V phase (d_h <= 64 * CPL); DHC = d_h when it is one of the common widths (the
// loops over channels then unroll and their loads are all in flight together), 0 for any other multiple of 8.
template <typename T, int CPL, int DHC>
__global__ __launch_bounds__(DEC_WAVES * 64) void decode_attn_kernel(DecArgs a, const float *__restrict__ q_new,
                                                                    const T *__restrict__ k_cache,
                                                                    const T *__restrict__ v_cache,
                                                                    float *__restrict__ part, int nsplit, int r0) {
  extern __shared__ float sm[];
  const int dh = DHC ? DHC : a.dh;
  const int split = blockIdx.x % nsplit, g = (blockIdx.x / nsplit) % a.Hk, b = blockIdx.x / (nsplit * a.Hk);
  const int len = seq_pos(a, b) + 1;  // a short sequence leaves its last splits empty: they write (-inf, 0, 0)
  const int nr = min(R_MAX, a.R - r0);  // query heads of this pass: g*R + r0 .. + nr
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float *qs = sm;                             // [R_MAX][dh], scaled to log2 units
  float *ps = qs + R_MAX * dh + wave * 64 * R_MAX;  // [64][R_MAX] probabilities of this wavefront's current keys
  float *mrg = sm + R_MAX * dh + DEC_WAVES * 64 * R_MAX;  // merge area: [DEC_WAVES][R_MAX][2 + dh]
  const float c = a.scale * 1.44269504088896340736f;
  for (int i = tid; i < R_MAX * dh; i += blockDim.x) {
    const int r = i / dh, ch = i % dh;
    qs[i] = r < nr ? q_new[((long long)b * a.Hq + g * a.R + r0 + r) * dh + ch] * c : 0.f;
  }
  __syncthreads();

  // keys of this split, dealt to the wavefronts in blocks of 64
  const int per = (len + nsplit - 1) / nsplit;
  const int k_begin = split * per, k_end = min(len, k_begin + per);
  float m[R_MAX], l[R_MAX], o[R_MAX][CPL];
#pragma unroll
  for (int r = 0; r < R_MAX; ++r) {
    m[r] = -INFINITY;
    l[r] = 0.f;
#pragma unroll
    for (int x = 0; x < CPL; ++x) o[r][x] = 0.f;
  }
  const long long row_elems = (long long)a.Hk * dh;
  const T *kb = k_cache + ((long long)b * a.S * a.Hk + g) * dh;
  const T *vb = v_cache + ((long long)b * a.S * a.Hk + g) * dh;
  for (int k0 = k_begin + wave * 64; k0 < k_end; k0 += DEC_WAVES * 64) {
    const int key = k0 + lane;
    const bool live = key < k_end;
    float s[R_MAX];
#pragma unroll
    for (int r = 0; r < R_MAX; ++r) s[r] = 0.f;
    if (live) {
      const T *kp = kb + (long long)key * row_elems;
#pragma unroll
      for (int ch = 0; ch < dh; ch += 8) {
        float kv[8];
        load_vec<8>(kp + ch, kv);
#pragma unroll
        for (int r = 0; r < R_MAX; ++r)
          if (r < nr) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s[r] = fmaf(kv[e], qs[r * dh + ch + e], s[r]);
          }
      }
    }
    float alpha[R_MAX];
#pragma unroll
    for (int r = 0; r < R_MAX; ++r) {
      float mx = live ? s[r] : -INFINITY;
      for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
      const float mn = fmaxf(m[r], mx);  // finite: the block holds at least one live key
      const float p = live ? exp2f(s[r] - mn) : 0.f;
      float sum = p;
      for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
      alpha[r] = exp2f(m[r] - mn);  // 0 on the first block
      l[r] = l[r] * alpha[r] + sum;
      m[r] = mn;
      ps[lane * R_MAX + r] = p;
    }
#pragma unroll
    for (int r = 0; r < R_MAX; ++r)
#pragma unroll
      for (int x = 0; x < CPL; ++x) o[r][x] *= alpha[r];
    // the probabilities written above are read by the same wavefront only: LDS serves a wavefront in order
    const int nk = min(64, k_end - k0);
    constexpr int VB = 16;  // value rows requested together
    for (int j0 = 0; j0 < nk; j0 += VB) {
      float vv[VB][CPL];
#pragma unroll
      for (int u = 0; u < VB; ++u) {
#pragma unroll
        for (int x = 0; x < CPL; ++x) vv[u][x] = 0.f;
        const int j = min(j0 + u, nk - 1);  // rows past the end repeat the last one; their probability is 0
        if (lane * CPL < dh) load_vec<CPL>(vb + (long long)(k0 + j) * row_elems + lane * CPL, vv[u]);
      }
#pragma unroll
      for (int u = 0; u < VB; ++u) {
#pragma unroll
        for (int r = 0; r < R_MAX; ++r) {
          const float p = j0 + u < nk ? ps[(j0 + u) * R_MAX + r] : 0.f;
#pragma unroll
          for (int x = 0; x < CPL; ++x) o[r][x] = fmaf(p, vv[u][x], o[r][x]);
        }
      }
    }
  }
  // merge the wavefronts in a fixed order
  const int stride = 2 + dh;
#pragma unroll
  for (int r = 0; r < R_MAX; ++r) {
    float *dst = mrg + (wave * R_MAX + r) * stride;
    if (lane == 0) {
      dst[0] = m[r];
      dst[1] = l[r];
    }
#pragma unroll
    for (int x = 0; x < CPL; ++x) {
      const int ch = lane * CPL + x;
      if (ch < dh) dst[2 + ch] = o[r][x];
    }
  }
  __syncthreads();
  for (int i = tid; i < nr * dh; i += blockDim.x) {
    const int r = i / dh, ch = i % dh;
    float M = -INFINITY;
    for (int w = 0; w < DEC_WAVES; ++w) M = fmaxf(M, mrg[(w * R_MAX + r) * stride]);
    float L = 0.f, acc = 0.f;
    for (int w = 0; w < DEC_WAVES; ++w) {
      const float *src = mrg + (w * R_MAX + r) * stride;
      const float f = src[0] == -INFINITY ? 0.f : exp2f(src[0] - M);
      L += src[1] * f;
      acc += src[2 + ch] * f;
    }
    float *out = part + (((long long)b * a.Hq + g * a.R + r0 + r) * nsplit + split) * stride;
    if (ch == 0) {
      out[0] = M;  // -inf when the split holds no key
      out[1] = L;
    }
    out[2 + ch] = acc;
  }
}

// ---------------------------------------------------------------------------
// The same attention for bf16 caches with d_h in {64, 128, 256}: rows of K and V are read the way they lie in
// memory.  A row is d_h / 8 chunks of 16 bytes; lane = (row of a group of 64 / LPR rows, chunk), so one load
// instruction fetches whole adjacent rows and every byte of every cache line it touches.  A lane's share of a score
// is the dot product over its 8 channels (bf16 pair dot instructions against the query, which the prologue has
// already rounded to bf16, packed in registers); the LPR shares of a row are added with DPP lane exchanges inside a
// row of 16 lanes, after which every lane of the row holds the score.  Each row group of a wavefront keeps its own
// online-softmax state (m, l, o over its 8 channels) so the main loop has no other cross-lane step; the groups, then
// the wavefronts, are merged once at the end.  The next block's K loads are issued as soon as the scores of the
// current one have left the K registers and the next V loads after the P V step, so a wavefront always has one or
// two blocks of loads in flight.  NR = query heads per pass, U = load instructions (groups of rows) per block.
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  return x + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}

template <int NR, int DH, int U>
__global__ __launch_bounds__(DEC_WAVES * 64) void decode_attn_rows_kernel(DecArgs a, const float *__restrict__ q_new,
                                                                         const bf16_t *__restrict__ k_cache,
                                                                         const bf16_t *__restrict__ v_cache,
                                                                         float *__restrict__ part, int nsplit, int r0) {
  constexpr int LPR = DH / 8, RPL = 64 / LPR, BLK = U * RPL;  // lanes per row, rows per load, rows per block
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  typedef float f4 __attribute__((ext_vector_type(4)));
  typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
  __shared__ float mrg[DEC_WAVES][NR][2 + DH];
  const int split = blockIdx.x % nsplit, g = (blockIdx.x / nsplit) % a.Hk, b = blockIdx.x / (nsplit * a.Hk);
  const int len = seq_pos(a, b) + 1;  // a short sequence leaves its last splits empty: they write (-inf, 0, 0)
  const int nr = min(NR, a.R - r0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rr = lane / LPR, cc = lane % LPR;
  const float c = a.scale * 1.44269504088896340736f;

  uint32_t q2[NR][4];  // this lane's 8 channels of each query head, bf16 pairs (exact: q_new holds bf16 values)
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    f4 lo = {0.f, 0.f, 0.f, 0.f}, hi = lo;
    if (r < nr) {
      const float *qp = q_new + ((long long)b * a.Hq + g * a.R + r0 + r) * DH + cc * 8;
      lo = *reinterpret_cast<const f4 *>(qp);
      hi = *reinterpret_cast<const f4 *>(qp + 4);
    }
    q2[r][0] = (__float_as_uint(lo.x) >> 16) | (__float_as_uint(lo.y) & 0xffff0000u);
    q2[r][1] = (__float_as_uint(lo.z) >> 16) | (__float_as_uint(lo.w) & 0xffff0000u);
    q2[r][2] = (__float_as_uint(hi.x) >> 16) | (__float_as_uint(hi.y) & 0xffff0000u);
    q2[r][3] = (__float_as_uint(hi.z) >> 16) | (__float_as_uint(hi.w) & 0xffff0000u);
  }

  float m[NR], l[NR], o[NR][8];
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    m[r] = -INFINITY;
    l[r] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[r][e] = 0.f;
  }
  const int per = (len + nsplit - 1) / nsplit;
  const int k_begin = split * per, k_end = min(len, k_begin + per);
  int k0 = k_begin + wave * BLK;
  if (k0 < k_end) {  // wave-uniform
    const uint32_t rowb = (uint32_t)a.Hk * DH * 2;  // bytes between consecutive tokens (S * rowb < 2^31: host check)
    const unsigned char *kb = reinterpret_cast<const unsigned char *>(k_cache + ((long long)b * a.S * a.Hk + g) * DH);
    const unsigned char *vb = reinterpret_cast<const unsigned char *>(v_cache + ((long long)b * a.S * a.Hk + g) * DH);
    // byte offsets of this lane's chunk in the U row groups of a block (the same for K and V); rows past the end of
    // the split repeat its last row (in bounds) and their probabilities are set to zero
    uint32_t off[U];
    auto offsets = [&](int kk) {
#pragma unroll
      for (int u = 0; u < U; ++u) off[u] = (uint32_t)min(kk + u * RPL + rr, k_end - 1) * rowb + cc * 16;
    };
    u4 kr[U], vr[U];
    offsets(k0);
#pragma unroll
    for (int u = 0; u < U; ++u) kr[u] = *reinterpret_cast<const u4 *>(kb + off[u]);
    __builtin_amdgcn_sched_barrier(0);  // K before V, as in the loop: the first wait is then for the K loads only
#pragma unroll
    for (int u = 0; u < U; ++u) vr[u] = *reinterpret_cast<const u4 *>(vb + off[u]);
    __builtin_amdgcn_sched_barrier(0);
    for (; k0 < k_end; k0 += DEC_WAVES * BLK) {
      float s[U][NR];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int r = 0; r < NR; ++r) {
          float acc = 0.f;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const uint32_t kw = kr[u][i], qw = q2[r][i];  // scalars first: a bit cast straight from a vector element is not safe
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf2, kw), __builtin_bit_cast(bf2, qw), acc, false);
          }
          s[u][r] = acc;
        }
      // the next block of this wavefront (clamped to the last row when there is none): K now, V after the P V step
      offsets(k0 + DEC_WAVES * BLK);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < U; ++u) kr[u] = *reinterpret_cast<const u4 *>(kb + off[u]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool live = k0 + u * RPL + rr < k_end;
#pragma unroll
        for (int r = 0; r < NR; ++r) {
          float x = s[u][r];
          x = dpp_add<0xB1>(x);   // quad_perm [1,0,3,2]
          x = dpp_add<0x4E>(x);   // quad_perm [2,3,0,1]
          x = dpp_add<0x141>(x);  // row_half_mirror
          if constexpr (LPR >= 16) x = dpp_add<0x140>(x);  // row_mirror
          if constexpr (LPR >= 32) x += __shfl_xor(x, 16);
          s[u][r] = live ? x * c : -INFINITY;
        }
      }
#pragma unroll
      for (int r = 0; r < NR; ++r) {
        float mx = s[0][r];
#pragma unroll
        for (int u = 1; u < U; ++u) mx = fmaxf(mx, s[u][r]);
        const float mn = fmaxf(m[r], mx);
        const float ms = mn == -INFINITY ? 0.f : mn;  // a row group that has seen no live key yet
        const float alpha = exp2f(m[r] - ms);
        float sum = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          s[u][r] = exp2f(s[u][r] - ms);
          sum += s[u][r];
        }
        l[r] = l[r] * alpha + sum;
        m[r] = mn;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[r][e] *= alpha;
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float vf[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          vf[2 * i] = __uint_as_float(vr[u][i] << 16);
          vf[2 * i + 1] = __uint_as_float(vr[u][i] & 0xffff0000u);
        }
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
          for (int e = 0; e < 8; ++e) o[r][e] = fmaf(s[u][r], vf[e], o[r][e]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < U; ++u) vr[u] = *reinterpret_cast<const u4 *>(vb + off[u]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // merge the row groups of the wavefront (lane <-> lane ^ step), then the wavefronts through LDS
#pragma unroll
  for (int step = LPR; step < 64; step *= 2) {
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const float mo = __shfl_xor(m[r], step), lo = __shfl_xor(l[r], step);
      const float M = fmaxf(m[r], mo), Ms = M == -INFINITY ? 0.f : M;
      const float f = exp2f(m[r] - Ms), fo = exp2f(mo - Ms);
      l[r] = l[r] * f + lo * fo;
      m[r] = M;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[r][e] = o[r][e] * f + __shfl_xor(o[r][e], step) * fo;
    }
  }
  if (rr == 0) {
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      if (cc == 0) {
        mrg[wave][r][0] = m[r];
        mrg[wave][r][1] = l[r];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) mrg[wave][r][2 + cc * 8 + e] = o[r][e];
    }
  }
  __syncthreads();
  constexpr int stride = 2 + DH;
  for (int i = tid; i < nr * DH; i += DEC_WAVES * 64) {
    const int r = i / DH, ch = i % DH;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < DEC_WAVES; ++w) M = fmaxf(M, mrg[w][r][0]);
    float L = 0.f, acc = 0.f;
#pragma unroll
    for (int w = 0; w < DEC_WAVES; ++w) {
      const float f = mrg[w][r][0] == -INFINITY ? 0.f : exp2f(mrg[w][r][0] - M);
      L += mrg[w][r][1] * f;
      acc += mrg[w][r][2 + ch] * f;
    }
    float *out = part + (((long long)b * a.Hq + g * a.R + r0 + r) * nsplit + split) * stride;
    if (ch == 0) {
      out[0] = M;  // -inf when the split holds no key
      out[1] = L;
    }
    out[2 + ch] = acc;
  }
}

// o[b, h, :] = sum_s part_o * 2^(m_s - M) / sum_s l_s * 2^(m_s - M), splits in index order
template <typename T>
__global__ __launch_bounds__(128) void decode_combine_kernel(DecArgs a, const float *__restrict__ part, int nsplit,
                                                            T *__restrict__ o) {
  __shared__ float f[MAX_SPLITS];  // 2^(m_s - M) / L per split (0 for an empty split)
  const int bh = blockIdx.x, dh = a.dh, stride = 2 + dh, tid = threadIdx.x;
  const float *src = part + (long long)bh * nsplit * stride;
  if (tid < 64) {  // one wavefront: lane s holds split s
    const float ms = tid < nsplit ? src[tid * stride] : -INFINITY;
    const float ls = tid < nsplit ? src[tid * stride + 1] : 0.f;
    float M = ms;
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    const float w = ms == -INFINITY ? 0.f : exp2f(ms - M);
    float L = 0.f;
    for (int s = 0; s < nsplit; ++s) L += __shfl(ls * w, s);  // index order
    if (tid < nsplit) f[tid] = w / L;
  }
  __syncthreads();
  for (int ch = tid; ch < dh; ch += blockDim.x) {
    float acc = 0.f;
    for (int s = 0; s < nsplit; ++s) acc = fmaf(src[s * stride + 2 + ch], f[s], acc);
    store_f(o + (long long)bh * dh + ch, acc);
  }
}

// ---------------------------------------------------------------------------
// Projections of a decode step: C (M, N) = A (M, K) W (K, N) with M = batch size (a handful of rows), bound by
// reading W once.  Workgroup = 128 columns x one slice of K; a lane owns 2 adjacent columns (one 4- or 8-byte load
// per row of W), the 4 wavefronts take quarters of the slice and are added through LDS, rows of A go through LDS
// 16 or 32 at a time ([k][rows] floats, so one 16-byte broadcast read feeds 4 rows).  K slices write fp32 partial sums
// that a second kernel adds in index order (no atomics).
// ---------------------------------------------------------------------------
constexpr int SK_COLS = 128, SK_MAXCHUNK = 128, SK_KB = 16, SK_PAD = 4;

// ROWS = rows of A per pass (16 or 32).  A wavefront requests SK_KB rows of W at a time and the next batch before it
// multiplies the current one, so its loads overlap the arithmetic instead of being waited for one by one.
template <typename T, int ROWS>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(const T *__restrict__ A, const T *__restrict__ W,
                                                         float *__restrict__ part, int M, int N, int K, int chunk) {
  constexpr int XS = ROWS + SK_PAD;  // padded row of the A tile: the transposing store spreads over 8 banks
  constexpr int XS_FLOATS = SK_MAXCHUNK * XS, RED_FLOATS = 3 * 64 * ROWS * 2;
  __shared__ float buf[XS_FLOATS > RED_FLOATS ? XS_FLOATS : RED_FLOATS];
  float *xs = buf;   // [klen][XS] A tile, fp32
  float *red = buf;  // [3][64][2 * ROWS] sums of wavefronts 1..3 (after the A tile is no longer read)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = blockIdx.x * SK_COLS + lane * 2;
  const int k_begin = blockIdx.y * chunk, k_end = min(K, k_begin + chunk);
  const int klen = k_end - k_begin;
  const int per_wave = (klen + 3) / 4;
  const int kw0 = wave * per_wave, kw1 = min(klen, kw0 + per_wave);
  const bool col_ok = n0 < N;
  // rows of W past the wavefront's range are read from its last row (in bounds) and multiplied by nothing
  const T *wp = W + (long long)k_begin * N + (col_ok ? n0 : 0);
  auto load_rows = [&](int kk0, float (&wv)[SK_KB][2]) {
#pragma unroll
    for (int j = 0; j < SK_KB; ++j) load_vec<2>(wp + (long long)min(kk0 + j, max(kw1 - 1, 0)) * N, wv[j]);
  };
  for (int m0 = 0; m0 < M; m0 += ROWS) {
    __syncthreads();  // the previous pass no longer reads buf
    for (int i = tid; i < klen * ROWS; i += 256) {
      const int m = i / klen, kk = i % klen;  // consecutive threads read consecutive k of one row
      xs[kk * XS + m] = m0 + m < M ? load_f(A + (long long)(m0 + m) * K + k_begin + kk) : 0.f;
    }
    __syncthreads();
    float acc[ROWS][2];
#pragma unroll
    for (int m = 0; m < ROWS; ++m) acc[m][0] = acc[m][1] = 0.f;
    if (kw0 < kw1) {
      float wa[SK_KB][2], wb[SK_KB][2];
      load_rows(kw0, wa);
      for (int kk0 = kw0; kk0 < kw1; kk0 += SK_KB) {
        load_rows(kk0 + SK_KB, wb);
#pragma unroll
        for (int j = 0; j < SK_KB; ++j) {
          if (kk0 + j < kw1) {  // wave-uniform
#pragma unroll
            for (int m4 = 0; m4 < ROWS; m4 += 4) {
              typedef float f4 __attribute__((ext_vector_type(4)));
              const f4 xv = *reinterpret_cast<const f4 *>(&xs[(kk0 + j) * XS + m4]);
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                acc[m4 + e][0] = fmaf(xv[e], wa[j][0], acc[m4 + e][0]);
                acc[m4 + e][1] = fmaf(xv[e], wa[j][1], acc[m4 + e][1]);
              }
            }
          }
        }
#pragma unroll
        for (int j = 0; j < SK_KB; ++j) wa[j][0] = wb[j][0], wa[j][1] = wb[j][1];
      }
    }
    __syncthreads();  // every wavefront is done with the A tile: its memory now takes the partial sums
    if (wave > 0) {
#pragma unroll
      for (int m = 0; m < ROWS; ++m) {
        red[((wave - 1) * 64 + lane) * 2 * ROWS + 2 * m] = acc[m][0];
        red[((wave - 1) * 64 + lane) * 2 * ROWS + 2 * m + 1] = acc[m][1];
      }
    }
    __syncthreads();
    if (wave == 0 && col_ok) {
#pragma unroll
      for (int m = 0; m < ROWS; ++m) {
        if (m0 + m < M) {
          float a0 = acc[m][0], a1 = acc[m][1];
          for (int w = 0; w < 3; ++w) a0 += red[(w * 64 + lane) * 2 * ROWS + 2 * m], a1 += red[(w * 64 + lane) * 2 * ROWS + 2 * m + 1];
          float *dst = part + ((long long)blockIdx.y * M + m0 + m) * N + n0;
          dst[0] = a0;
          dst[1] = a1;
        }
      }
    }
  }
}

// The same product on the matrix cores for bf16 (N and K multiples of 8).  The W tile (a K slice x 128 columns) is
// staged row-major in LDS and read as MFMA fragments with the transposing LDS read (the contraction index is the ROW
// of W); the fragments of A (32 rows x 16 k) come straight from memory: lane (row l % 32, half l / 32) holds
// k = 4*half .. +3 and 8 + 4*half .. +3 of each group of 16, the order the transposing read delivers W in.  Each
// wavefront owns 32 of the 128 columns over the whole slice, so nothing is added across wavefronts.
typedef __bf16 sk_bf16x8 __attribute__((ext_vector_type(8)));
typedef float sk_f32x16 __attribute__((ext_vector_type(16)));
typedef float sk_f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t sk_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t sk_u32x2 __attribute__((ext_vector_type(2)));
typedef short sk_v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) sk_v4i16 sk_lds_v4i16;
constexpr int SM_ROW = SK_COLS * 2 + 64;  // LDS row of the W tile, bytes: padded so that the 4 rows a transposing read touches differ in bank group

__global__ __launch_bounds__(256) void gemm_skinny_mfma_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W,
                                                              float *__restrict__ part, int M, int N, int K, int chunk) {
  __shared__ __attribute__((aligned(16))) unsigned char wt[SK_MAXCHUNK * SM_ROW];
  constexpr int NK16 = SK_MAXCHUNK / 16, STAGE = SK_MAXCHUNK * 16 / 256;  // k groups of a slice; 16-byte chunks per thread
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
  const int n0 = blockIdx.x * SK_COLS;
  const int k_begin = blockIdx.y * chunk, k_end = min(K, k_begin + chunk);
  const int nk16 = (k_end - k_begin + 15) / 16;
  // W tile: all loads first, then the LDS stores; rows past the slice and columns past N are zero
  sk_u32x4 wv[STAGE];
#pragma unroll
  for (int i = 0; i < STAGE; ++i) {
    const int id = tid + i * 256, row = id >> 4, c = id & 15;
    sk_u32x4 v = {0, 0, 0, 0};
    if (row < nk16 * 16 && k_begin + row < k_end && n0 + c * 8 < N)
      v = *reinterpret_cast<const sk_u32x4 *>(W + (long long)(k_begin + row) * N + n0 + c * 8);
    wv[i] = v;
  }
  // fragments of the first 32 rows of A for the whole slice (k past the slice reads as zero)
  auto load_a = [&](int m0, sk_u32x4 (&xa)[NK16]) {
    const bf16_t *ap = A + (long long)min(m0 + l32, M - 1) * K + k_begin + 4 * half;
#pragma unroll
    for (int kk = 0; kk < NK16; ++kk) {
      sk_u32x2 lo = {0, 0}, hi = {0, 0};
      if (kk < nk16) {
        if (k_begin + kk * 16 + 4 * half < k_end) lo = *reinterpret_cast<const sk_u32x2 *>(ap + kk * 16);
        if (k_begin + kk * 16 + 8 + 4 * half < k_end) hi = *reinterpret_cast<const sk_u32x2 *>(ap + kk * 16 + 8);
      }
      xa[kk] = sk_u32x4{lo.x, lo.y, hi.x, hi.y};
    }
  };
  sk_u32x4 xa[NK16];
  load_a(0, xa);
#pragma unroll
  for (int i = 0; i < STAGE; ++i) {
    const int id = tid + i * 256, row = id >> 4, c = id & 15;
    if (row < nk16 * 16) *reinterpret_cast<sk_u32x4 *>(wt + row * SM_ROW + c * 16) = wv[i];
  }
  __syncthreads();
  const unsigned char *pw = wt + (4 * half + ((lane & 15) >> 2)) * SM_ROW + (wave * 32 + ((lane >> 4) & 1) * 16 + 4 * (lane & 3)) * 2;
  for (int m0 = 0; m0 < M; m0 += 32) {
    if (m0 > 0) load_a(m0, xa);
    sk_f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < NK16; ++kk) {
      if (kk < nk16) {
        const unsigned char *p = pw + kk * 16 * SM_ROW;
        const sk_v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((sk_lds_v4i16 *)p);
        const sk_v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((sk_lds_v4i16 *)(p + 8 * SM_ROW));
        const sk_bf16x8 fw = __builtin_bit_cast(sk_bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw, __builtin_bit_cast(sk_bf16x8, xa[kk]), acc, 0, 0, 0);
      }
    }
    // acc[r] = C[m0 + l32][n0 + 32*wave + 8*(r/4) + 4*half + r%4]
    const int m = m0 + l32;
    if (m < M) {
      float *dst = part + ((long long)blockIdx.y * M + m) * N + n0 + wave * 32 + half * 4;
#pragma unroll
      for (int rg = 0; rg < 4; ++rg)
        if (n0 + wave * 32 + rg * 8 + half * 4 < N)  // N % 8 == 0: the four columns are inside
          *reinterpret_cast<sk_f32x4 *>(dst + rg * 8) = sk_f32x4{acc[rg * 4], acc[rg * 4 + 1], acc[rg * 4 + 2], acc[rg * 4 + 3]};
    }
  }
}

// C row m starts at C + m * ldc (the rows of a projection may go straight into a strided destination).  With
// `row_pos` row m goes to ring slot clamp(row_pos[m], 0, pos_max) % ring of its sequence: C + m * ldc + slot * N.
template <typename T>
__global__ void skinny_reduce_kernel(const float *__restrict__ part, T *__restrict__ C, long long mn, int N,
                                     long long ldc, int splits, const int *__restrict__ row_pos, int pos_max,
                                     int ring) {
  const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
  if (id >= mn) return;
  float a = 0.f;
  int s = 0;
  for (; s + 8 <= splits; s += 8) {  // 8 loads in flight, added in split order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = part[(long long)(s + u) * mn + id];
#pragma unroll
    for (int u = 0; u < 8; ++u) a += v[u];
  }
  for (; s < splits; ++s) a += part[(long long)s * mn + id];
  const long long m = id / N;
  long long slot_off = 0;
  if (row_pos) {
    const int p = row_pos[m];
    slot_off = (long long)((p < 0 ? 0 : (p > pos_max ? pos_max : p)) % ring) * N;
  }
  store_f(C + m * ldc + slot_off + id % N, a);
}

int skinny_splits(int N, int K) {
  const int col_blocks = (N + SK_COLS - 1) / SK_COLS;
  int splits = (256 + col_blocks - 1) / col_blocks;          // about one workgroup per CU
  const int min_splits = (K + SK_MAXCHUNK - 1) / SK_MAXCHUNK;  // a slice must fit the LDS tile
  splits = splits < min_splits ? min_splits : splits;
  return splits > K / 16 ? (K / 16 > min_splits ? K / 16 : min_splits) : splits;
}
size_t skinny_scratch_bytes(int M, int N, int K) { return (size_t)skinny_splits(N, K) * M * N * sizeof(float); }

template <typename T>
hipError_t gemm_skinny(const T *A, const T *W, T *C, long long ldc, float *part, int M, int N, int K, hipStream_t s,
                       const int *row_pos = nullptr, int pos_max = 0, int ring = 1) {
  const int splits = skinny_splits(N, K);
  int chunk = (K + splits - 1) / splits;
  const dim3 grid((N + SK_COLS - 1) / SK_COLS, (K + chunk - 1) / chunk);
  if constexpr (std::is_same<T, bf16_t>::value) {
    if (N % 8 == 0 && K % 8 == 0) {
      chunk = (chunk + 15) / 16 * 16;  // whole groups of 16 k (never above SK_MAXCHUNK, itself a multiple of 16)
      const dim3 grid_m((N + SK_COLS - 1) / SK_COLS, (K + chunk - 1) / chunk);
      gemm_skinny_mfma_kernel<<<grid_m, 256, 0, s>>>(A, W, part, M, N, K, chunk);
      hipError_t em = hipGetLastError();
      if (em != hipSuccess) return em;
      const long long mn_m = (long long)M * N;
      skinny_reduce_kernel<T><<<(unsigned)((mn_m + 255) / 256), 256, 0, s>>>(part, C, mn_m, N, ldc, (int)grid_m.y, row_pos,
                                                                             pos_max, ring);
      return hipGetLastError();
    }
  }
  if (M > 16) gemm_skinny_kernel<T, 32><<<grid, 256, 0, s>>>(A, W, part, M, N, K, chunk);
  else gemm_skinny_kernel<T, 16><<<grid, 256, 0, s>>>(A, W, part, M, N, K, chunk);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const long long mn = (long long)M * N;
  skinny_reduce_kernel<T><<<(unsigned)((mn + 255) / 256), 256, 0, s>>>(part, C, mn, N, ldc, (int)grid.y, row_pos, pos_max,
                                                                         ring);
  return hipGetLastError();
}

// slots of the latent ring: the taps - 1 earlier rows the convolutions reach back to (one at least, for the value
// shift) plus the slot the new row is written to
int ring_rows(const Dims &d) {
  const int ks = (d.flags & CCA_CONV_SEQ) ? d.k_seq : 1, kc = (d.flags & CCA_CONV_CH) ? d.k_ch : 1;
  const int taps = ks + kc - 1;
  return (taps - 1 > 1 ? taps - 1 : 1) + 1;
}

size_t align256(size_t n) { return (n + 255) / 256 * 256; }

struct DecLayout {
  size_t q_new, o, part, gemm, total;
};
DecLayout layout(const Dims &d) {
  DecLayout L;
  size_t off = 0;
  auto take = [&](size_t n) {
    const size_t at = off;
    off += align256(n);
    return at;
  };
  L.q_new = take((size_t)d.B * d.e_q * sizeof(float));
  L.o = take((size_t)d.B * d.e_q * d.esize());
  L.part = take((size_t)d.B * d.Hq * MAX_SPLITS * (2 + d.dh) * sizeof(float));
  const size_t g1 = skinny_scratch_bytes(d.B, d.n_lat, d.E), g2 = skinny_scratch_bytes(d.B, d.E, d.e_q);
  L.gemm = take(g1 > g2 ? g1 : g2);
  L.total = off;
  return L;
}

template <typename T>
hipError_t step_t(const Dims &d, const cca_weights &w, const void *x_new, void *k_cache, void *v_cache, void *hist,
                  int pos, const int *pos_seq, void *out, unsigned char *ws, hipStream_t s) {
  // pos: the position of every sequence, or with pos_seq (device, one entry per sequence) the largest of them
  const DecLayout L = layout(d);
  const int P = ring_rows(d);
  DecArgs a{d.B, d.T, d.Hq, d.Hk, d.dh, d.R, d.e_q, d.e_kv, d.n_lat, d.v_half, d.k_seq, d.k_ch, P, pos,
            d.flags, d.rope_base, d.scale, d.norm_eps, pos_seq};
  float *q_new = reinterpret_cast<float *>(ws + L.q_new);
  T *o = reinterpret_cast<T *>(ws + L.o);
  float *part = reinterpret_cast<float *>(ws + L.part);
  float *gpart = reinterpret_cast<float *>(ws + L.gemm);
  // the new latent rows go straight into their ring slot
  hipError_t e = pos_seq ? gemm_skinny<T>((const T *)x_new, (const T *)w.w_down, (T *)hist, (long long)P * d.n_lat, gpart,
                                          d.B, d.n_lat, d.E, s, pos_seq, pos, P)
                         : gemm_skinny<T>((const T *)x_new, (const T *)w.w_down,
                                          (T *)hist + (long long)(pos % P) * d.n_lat, (long long)P * d.n_lat, gpart, d.B,
                                          d.n_lat, d.E, s);
  if (e != hipSuccess) return e;
  {
    int threads = 64;
    while (threads < d.dh && threads < 256) threads *= 2;
    const int kc = (d.flags & CCA_CONV_CH) ? d.k_ch : 1;
    const size_t smem = sizeof(float) * ((size_t)kc * d.dh + threads + d.dh);
    decode_prologue_kernel<T><<<dim3(d.B, d.Hq + 2 * d.Hk), threads, smem, s>>>(
        a, (const T *)hist, (const T *)w.w_conv_seq, (const T *)w.w_conv_ch, w.temp, q_new, (T *)k_cache,
        (T *)v_cache);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  {
    const int len = pos + 1;  // the longest sequence sizes the splits
    // enough workgroups to fill the chip, at least 256 keys each, at most MAX_SPLITS
    int nsplit = (1024 + d.B * d.Hk - 1) / (d.B * d.Hk);
    nsplit = nsplit < (len + 255) / 256 ? nsplit : (len + 255) / 256;
    nsplit = nsplit < 1 ? 1 : (nsplit > MAX_SPLITS ? MAX_SPLITS : nsplit);
    const size_t smem = sizeof(float) * ((size_t)R_MAX * d.dh + DEC_WAVES * 64 * R_MAX + DEC_WAVES * R_MAX * (2 + d.dh));
    const unsigned grid = (unsigned)((long long)d.B * d.Hk * nsplit);
    if constexpr (std::is_same<T, bf16_t>::value) {
      // the row kernel addresses a sequence's cache with 32-bit byte offsets
      if ((d.dh == 64 || d.dh == 128 || d.dh == 256) && (long long)d.T * d.Hk * d.dh * 2 < (1ll << 31)) {
        for (int r0 = 0; r0 < d.R; r0 += R_MAX) {
          const int left = d.R - r0;
#define CCA_DEC_ROWS(NR, DH, U)                                                                                    \
  decode_attn_rows_kernel<NR, DH, U><<<grid, DEC_WAVES * 64, 0, s>>>(a, q_new, (const bf16_t *)k_cache,             \
                                                                     (const bf16_t *)v_cache, part, nsplit, r0)
#define CCA_DEC_ROWS_DH(NR, U)                                                                                     \
  {                                                                                                                \
    if (d.dh == 64) CCA_DEC_ROWS(NR, 64, U);                                                                       \
    else if (d.dh == 128) CCA_DEC_ROWS(NR, 128, U);                                                                \
    else CCA_DEC_ROWS(NR, 256, U);                                                                                 \
  }
          if (left == 1) CCA_DEC_ROWS_DH(1, 8)
          else if (left == 2) CCA_DEC_ROWS_DH(2, 8)
          else if (left <= 4) CCA_DEC_ROWS_DH(4, 8)
          else CCA_DEC_ROWS_DH(8, 4)
#undef CCA_DEC_ROWS_DH
#undef CCA_DEC_ROWS
          if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        decode_combine_kernel<T><<<(unsigned)(d.B * d.Hq), 128, 0, s>>>(a, part, nsplit, o);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        return gemm_skinny<T>(o, (const T *)w.w_out, (T *)out, d.E, gpart, d.B, d.E, d.e_q, s);
      }
    }
    for (int r0 = 0; r0 < d.R; r0 += R_MAX) {
#define CCA_DEC_ATTN(CPL, DHC)                                                                                  \
  {                                                                                                             \
    e = raise_lds_limit<decode_attn_kernel<T, CPL, DHC>>(smem);                                                 \
    if (e != hipSuccess) return e;                                                                              \
    decode_attn_kernel<T, CPL, DHC><<<grid, DEC_WAVES * 64, smem, s>>>(a, q_new, (const T *)k_cache,              \
                                                                           (const T *)v_cache, part, nsplit, r0); \
  }
      if (d.dh == 64) CCA_DEC_ATTN(1, 64)
      else if (d.dh == 128) CCA_DEC_ATTN(2, 128)
      else if (d.dh == 256) CCA_DEC_ATTN(4, 256)
      else if (d.dh <= 64) CCA_DEC_ATTN(1, 0)
      else if (d.dh <= 128) CCA_DEC_ATTN(2, 0)
      else CCA_DEC_ATTN(4, 0)
#undef CCA_DEC_ATTN
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    decode_combine_kernel<T><<<(unsigned)(d.B * d.Hq), 128, 0, s>>>(a, part, nsplit, o);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return gemm_skinny<T>(o, (const T *)w.w_out, (T *)out, d.E, gpart, d.B, d.E, d.e_q, s);
}

}  // namespace

int decode_ring_rows(const Dims &d) { return ring_rows(d); }
size_t decode_scratch_bytes(const Dims &d) { return layout(d).total; }

hipError_t decode_step(const Dims &d, const cca_weights &w, const void *x_new, void *k_cache, void *v_cache, void *hist,
                       int pos, const int *pos_seq, void *out, void *workspace, hipStream_t s) {
  unsigned char *ws = static_cast<unsigned char *>(workspace);
  return d.bf16 ? step_t<bf16_t>(d, w, x_new, k_cache, v_cache, hist, pos, pos_seq, out, ws, s)
                : step_t<float>(d, w, x_new, k_cache, v_cache, hist, pos, pos_seq, out, ws, s);
}

}  // namespace cca
