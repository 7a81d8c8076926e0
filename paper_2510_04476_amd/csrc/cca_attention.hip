// Latent-space softmax attention on the gfx950 matrix cores (Sec. 2.2, third
// line of the final equation block; KV heads shared by groups of query heads
// as in the CCGQA paragraph).  bf16 in, fp32 accumulation, online softmax.
//
// One workgroup = 4 wavefronts = 128 query rows of one (batch, query head);
// each wavefront owns 32 rows (one MFMA tile) and all of d_h, so the softmax
// statistics of a row never leave a wavefront.  Two workgroups share a CU
// (2 wavefronts per SIMD): while one wavefront does softmax arithmetic on
// the vector ALU, the other keeps the matrix core busy.  Keys / values arrive
// in tiles of 64 through double-buffered LDS; the next tile travels HBM ->
// registers while the current one is multiplied.
//
// The scores are produced transposed, S^T = K Q^T, with the 32x32x16 bf16
// MFMA.  Its accumulator layout then gives every lane 16 keys of ONE query
// row, so (a) the row max / sum are in-lane reductions plus a single exchange
// between the two half-waves, and (b) the exponentiated scores, packed to
// bf16 in place, are already the second operand of O^T += V^T P^T: P never
// goes through LDS.  V is transposed on its way into LDS (4 keys x 8 channels
// per lane, in registers) into the key order that accumulator layout dictates.
#include "cca_internal.h"

namespace cca {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int BQ = 128;   // query rows per workgroup (4 wavefronts x 32 rows)
constexpr int BKV = 64;   // keys per LDS tile
constexpr int NT = 256;   // threads
constexpr float RESCALE_LOG2 = 8.f;  // the running max is only raised when it would grow by more than 2^8

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  // round-to-nearest-even pair; inputs are finite and non-negative
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

template <int DH, bool CAUSAL>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_fwd_kernel(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K, const bf16_t *__restrict__ V, bf16_t *__restrict__ O,
    float *__restrict__ LSE, int T, int Hq, int Hk, int BH, int nqb, float scale) {
  constexpr int KK = DH / 16;   // MFMA k-steps over the head width
  constexpr int DT = DH / 32;   // 32-wide output tiles over the head width
  constexpr int KCH = DH / 8;   // 16-byte chunks per key row
  constexpr int K_PER_THREAD = BKV * KCH / NT;
  constexpr int V_UNITS = (BKV / 4) * (DH / 8);  // 4-key x 8-channel units per tile
  static_assert(V_UNITS <= NT, "one V unit per thread at most");
  __shared__ u32x4 sK[2][BKV * KCH];
  __shared__ u32x4 sV[2][DH * 8];  // V^T: d_h rows of 64 keys

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  // heaviest (latest) query blocks first; the head index is the fast one, so with
  // B*Hq a multiple of 8 every XCD keeps working on the K/V of the same head
  const int idx = blockIdx.x;
  const int bh = idx % BH, qb = nqb - 1 - idx / BH;
  const int b = bh / Hq, h = bh % Hq, g = h / (Hq / Hk);
  const int q0 = qb * BQ, qw0 = q0 + wave * 32;
  const float c = scale * 1.44269504088896340736f;  // exp(x * scale) = exp2(x * c)

  // ---- query fragments: row qw0 + l32, all of d_h, straight from HBM
  bf16x8 qf[KK];
  {
    int row = qw0 + l32;
    row = row < T ? row : T - 1;
    const bf16_t *p = Q + (((long long)b * T + row) * Hq + h) * DH + half * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      qf[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(p + kk * 16));
  }

  f32x16 oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float m_run = -INFINITY;  // reference max of the raw scores of this lane's query row
  float l_run = 0.f;        // running sum; each half-wave keeps its own part

  const int kv_end = CAUSAL ? min(q0 + BQ, T) : T;  // keys [0, kv_end) matter to this workgroup
  const int ntiles = (kv_end + BKV - 1) / BKV;
  const int wave_last = min(qw0 + 31, T - 1);
  const bool wave_live = qw0 < T;

  // ---- global -> register staging of one K/V tile
  u32x4 rk[K_PER_THREAD];
  u32x4 rv[4];
  const int v_kg = tid / (DH / 8), v_dg = tid % (DH / 8);  // V unit of this thread: keys 4*v_kg.., channels 8*v_dg..
  auto load_tile = [&](int kv0) {
#pragma unroll
    for (int i = 0; i < K_PER_THREAD; ++i) {
      const int id = tid + i * NT, r = id / KCH, ch = id % KCH;
      int s = kv0 + r;
      s = s < T ? s : T - 1;
      rk[i] = *reinterpret_cast<const u32x4 *>(K + (((long long)b * T + s) * Hk + g) * DH + ch * 8);
    }
    if (tid < V_UNITS) {
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        int s = kv0 + v_kg * 4 + rr;
        s = s < T ? s : T - 1;
        rv[rr] = *reinterpret_cast<const u32x4 *>(V + (((long long)b * T + s) * Hk + g) * DH + v_dg * 8);
      }
    }
  };
  auto kswz = [](int r, int ch) {
    return KCH == 16 ? (ch ^ (r & 15)) : (ch ^ ((r & 7) ^ ((r >> 3) & 1)));
  };
  auto vswz = [](int d, int ch) { return ch ^ ((d & 7) ^ ((d >> 3) & 7)); };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < K_PER_THREAD; ++i) {
      const int id = tid + i * NT, r = id / KCH, ch = id % KCH;
      sK[buf][r * KCH + kswz(r, ch)] = rk[i];
    }
    if (tid < V_UNITS) {
      // position of key group v_kg inside a V^T row: chunk = ks*4 + j*2 + hf, 8-byte slot blk
      const int ks = v_kg >> 3, k8 = v_kg & 7;
      const int chunk = ks * 4 + (k8 >> 2) * 2 + (k8 & 1), blk = (k8 & 3) >> 1;
      unsigned char *base = reinterpret_cast<unsigned char *>(sV[buf]);
#pragma unroll
      for (int e = 0; e < 8; ++e) {  // channel d = 8*v_dg + e: gather its 4 keys
        const int d = v_dg * 8 + e;
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        u32x2 p;
        p.x = __builtin_amdgcn_perm(rv[1][e >> 1], rv[0][e >> 1], sel);
        p.y = __builtin_amdgcn_perm(rv[3][e >> 1], rv[2][e >> 1], sel);
        *reinterpret_cast<u32x2 *>(base + d * 128 + vswz(d, chunk) * 16 + blk * 8) = p;
      }
    }
  };

  load_tile(0);
  store_tile(0);
  __syncthreads();
  for (int j = 0; j < ntiles; ++j) {
    const int kv0 = j * BKV, buf = j & 1;
    const bool more = j + 1 < ntiles;
    if (more) load_tile(kv0 + BKV);  // in flight while this tile is multiplied
    if (wave_live && !(CAUSAL && kv0 > wave_last)) {
      // ---- S^T = K Q^T for 64 keys x 32 query rows
      f32x16 sacc[2];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[ks][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          const int r = ks * 32 + l32;
          const bf16x8 kf = __builtin_bit_cast(bf16x8, sK[buf][r * KCH + kswz(r, kk * 2 + half)]);
          sacc[ks] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[ks], 0, 0, 0);
        }

      // ---- online softmax; lane (l32, half) holds keys kv0 + ks*32 + 8*(r/4) + 4*half + r%4 of row l32
      if ((CAUSAL && kv0 + BKV - 1 > qw0) || (kv0 + BKV > T)) {
        const int t = qw0 + l32;
        const int lim = CAUSAL ? min(t, T - 1) : T - 1;  // last visible key
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int s = kv0 + ks * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
            if (s > lim) sacc[ks][r] = -INFINITY;
          }
      }
      float mx = max3(sacc[0][0], sacc[0][1], sacc[1][0]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = max3(mx, sacc[0][r], sacc[0][r + 1]);
#pragma unroll
      for (int r = 1; r < 16; r += 2) mx = max3(mx, sacc[1][r], sacc[1][(r + 1) & 15]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      // Raise the reference max only when it would grow by more than 2^RESCALE_LOG2:
      // exp2 arguments stay <= RESCALE_LOG2, far from fp32 / bf16 overflow, and the
      // accumulator is rescaled on few tiles only.
      if (__any((mx - m_run) * c > RESCALE_LOG2)) {
        const float m_new = fmaxf(m_run, mx);  // finite: key 0 is visible to every row in tile 0
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);  // 0 on the first tile
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
      }
      const float mc = m_run * c;
      bf16x8 pf[2][2];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = __builtin_amdgcn_exp2f(fmaf(sacc[ks][r], c, -mc));
          l_run += p[r];
        }
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          u32x4 w;
          w.x = pack2(p[8 * jj + 0], p[8 * jj + 1]);
          w.y = pack2(p[8 * jj + 2], p[8 * jj + 3]);
          w.z = pack2(p[8 * jj + 4], p[8 * jj + 5]);
          w.w = pack2(p[8 * jj + 6], p[8 * jj + 7]);
          pf[ks][jj] = __builtin_bit_cast(bf16x8, w);
        }
      }

      // ---- O^T += V^T P^T
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            const int d = dt * 32 + l32;
            const bf16x8 vf = __builtin_bit_cast(bf16x8, sV[buf][d * 8 + vswz(d, ks * 4 + jj * 2 + half)]);
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ks][jj], oacc[dt], 0, 0, 0);
          }
    }
    if (more) store_tile(buf ^ 1);  // last read before the barrier that ended the previous iteration
    __syncthreads();
  }

  // ---- epilogue: normalise, round once to bf16, store; log-sum-exp of the scaled logits
  if (!wave_live) return;
  {
    const int t = qw0 + l32;
    const float l = l_run + __shfl_xor(l_run, 32);
    if (t < T) {
      const float inv = 1.f / l;
      bf16_t *orow = O + (((long long)b * T + t) * Hq + h) * DH;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          u32x2 w;
          w.x = pack2(oacc[dt][rg * 4 + 0] * inv, oacc[dt][rg * 4 + 1] * inv);
          w.y = pack2(oacc[dt][rg * 4 + 2] * inv, oacc[dt][rg * 4 + 3] * inv);
          *reinterpret_cast<u32x2 *>(orow + dt * 32 + rg * 8 + half * 4) = w;
        }
      if (LSE && half == 0) LSE[((long long)b * Hq + h) * T + t] = m_run * scale + logf(l);
    }
  }
}

template <int DH>
hipError_t launch(const Dims &d, const void *q, const void *k, const void *v, void *o, float *lse, hipStream_t s) {
  const int nqb = (d.T + BQ - 1) / BQ;
  const int BH = d.B * d.Hq;
  const long long blocks = (long long)nqb * BH;
  if (d.flags & CCA_CAUSAL)
    attn_fwd_kernel<DH, true><<<(unsigned)blocks, NT, 0, s>>>((const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                                                            (bf16_t *)o, lse, d.T, d.Hq, d.Hk, BH, nqb, d.scale);
  else
    attn_fwd_kernel<DH, false><<<(unsigned)blocks, NT, 0, s>>>((const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                                                             (bf16_t *)o, lse, d.T, d.Hq, d.Hk, BH, nqb, d.scale);
  return hipGetLastError();
}

}  // namespace

bool attention_mfma_supported(const Dims &d) {
  return d.bf16 && (d.dh == 128 || d.dh == 64) && (long long)d.B * d.Hq * ((d.T + BQ - 1) / BQ) < (1ll << 31);
}

hipError_t attention_mfma_bf16(const Dims &d, const void *q, const void *k, const void *v, void *o, float *lse,
                               hipStream_t s) {
  return d.dh == 128 ? launch<128>(d, q, k, v, o, lse, s) : launch<64>(d, q, k, v, o, lse, s);
}

}  // namespace cca
