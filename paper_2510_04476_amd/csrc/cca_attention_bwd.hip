// Backward of the latent softmax attention on the gfx950 matrix cores (flash
// style: probabilities are recomputed from the saved log-sum-exp, nothing of
// size T x T is stored).  The paper gives no backward equations; with
// P = softmax(scale * Q K^T) per row and Delta_t = <dO_t, O_t>:
//     dV = P^T dO,  dP = dO V^T,  dS = P * (dP - Delta),  dQ = scale * dS K,  dK = scale * dS^T Q,
// dK and dV summed over the query heads that share a KV head (CCGQA paragraph).
//
// Three kernels, no atomics, deterministic:
//   delta_kernel      Delta (B,H_q,T) fp32.
//   attn_bwd_dq       one workgroup = 256 query rows of one head (8 wavefronts x 32 rows), loops over key
//                     tiles like the forward kernel; S^T and dP^T come out with one query row per lane, dS^T
//                     packed to bf16 is the second MFMA operand of dQ^T += K^T dS^T, K^T fetched with the
//                     transposing LDS read.
//   scale_q           q * scale * log2(e) rounded to bf16 (what the forward kernel multiplies), once, for the next kernel.
//   attn_bwd_dkdv     one workgroup = 256 keys x one QUERY head (8 wavefronts x 32 keys), loops over the query
//                     tiles of that head; S and dP come out with one key per lane, P and dS packed to bf16 are
//                     the second operands of dV^T += dO^T P and dK^T += Q^T dS, with dO^T and Q^T fetched by
//                     transposing LDS reads.  With R > 1 query heads per KV head each workgroup writes its
//                     head's fp32 contribution and group_sum_kernel adds the R of them in a fixed order
//                     (one workgroup looping over the whole group leaves a causal grid of only B*H_k*T/128
//                     unequal workgroups: measured 4.2 ms against 0.86 ms for dQ at the 16k CCGQA shape).
// S and dP are recomputed in both kernels (7 contractions instead of 5) in exchange for having no atomics.
//
// The probabilities must be the forward kernel's own: that kernel multiplies q by scale*log2(e) and rounds it
// to bf16 before the score MFMAs, and lse is the log-sum-exp of THOSE scores.  Recomputing the scores from
// the unrounded q against that lse leaves every row of P off by a common factor exp(lse_exact - lse) (about
// 1 % where logits reach ~10: measured 0.8 % on d_q, d_k).  So q is scaled and rounded here exactly as there;
// d_k then contracts dS with the scaled q and is multiplied by ln 2 instead of scale.
#include <type_traits>

#include "cca_internal.h"

namespace cca {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef short v8i16 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4i16 lds_v4i16;

namespace {

// Shapes that follow from the head width d_h (128 or 64): KK fragments of 16 channels, DT tiles of 32 channels,
// KCH 16-byte chunks per row, ROW = LDS row of one token in bytes (64 bytes of padding: see below).
#define CCA_BWD_GEOMETRY(DH) \
  constexpr int KK = (DH) / 16, DT = (DH) / 32, KCH = (DH) / 8, ROW = (DH) * 2 + 64; \
  (void)KK; (void)DT; (void)KCH; (void)ROW

// LDS tiles of this file are read two ways: 16-byte reads down a column of 16 rows (first MFMA operand of the score
// products) and transposing reads that touch 4 consecutive rows x 64 consecutive bytes (operands of the products
// that contract over tokens).  Padding alone cannot serve both: a stride that spreads 16 rows over the banks (+16
// bytes) makes neighbouring rows overlap within 64 bytes, and the transposing reads then ran 4-way conflicted (half
// of all LDS cycles of these kernels).  So: the row stride is a multiple of 64 bytes that is odd in units of 64
// (4 consecutive rows land in 4 different 64-byte bank groups: transposing reads conflict-free), and chunk c of
// row r is stored at chunk position c ^ ((r >> 2) & 3): among 16 rows, those that share a bank group (r & 3 equal)
// differ in r >> 2 and so in the low two bits of the position (column reads conflict-free).  The XOR touches only
// bits 4-5 of the address, so every read is a per-lane base plus a compile-time offset.
__device__ __forceinline__ int swz(int r) { return (r >> 2) & 3; }

// Per-lane byte offsets of the two read patterns.  Column read of this lane's chunk 2*kk + half of row 32*blk + l32:
//   tile + blk*32*ROW + col[kk & 1] + 64*(kk >> 1).
// Transposing read of rows r0 + {4*half + q, 8 + 4*half + q} (q = (lane & 15) >> 2; r0 a multiple of 16), channel
// tile dt (32 channels = 64 bytes), this lane's 8 bytes:  tile + r0*ROW + tr[x] + 64*dt  for x = lo, hi.
struct LaneSwz {
  uint32_t col[2], tr[2];
};
template <int DH>
__device__ __forceinline__ LaneSwz lane_swz(int lane) {
  constexpr int ROW = DH * 2 + 64;
  const int l32 = lane & 31, half = lane >> 5;
  LaneSwz L;
#pragma unroll
  for (int x = 0; x < 2; ++x) L.col[x] = (uint32_t)l32 * ROW + (((2 * x + half) ^ swz(l32)) << 4);
  const int l2 = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1), sub8 = (lane & 1) * 8;
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const int rr = 8 * x + 4 * half + ((lane & 15) >> 2);
    L.tr[x] = (uint32_t)rr * ROW + ((l2 ^ swz(rr)) << 4) + sub8;
  }
  return L;
}

constexpr float LOG2E = 1.44269504088896340736f;
constexpr float LN2 = 0.69314718055994530942f;  // the scaled q carries scale * log2(e): scale * q = ln 2 * q_scaled

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// MFMA first-operand fragment of the TRANSPOSE of a row-major LDS tile (layout above): lane (c = l32, half) receives
// tile[r0 + 4*half + {0..3}][32*dt + c] and tile[r0 + 8 + 4*half + {0..3}][32*dt + c].
template <int ROW>
__device__ __forceinline__ bf16x8 tr_frag(const unsigned char *tile, const LaneSwz &L, int r0, int dt) {
  const unsigned char *a = tile + r0 * ROW + dt * 64;
  const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16 *)(a + L.tr[0]));
  const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16 *)(a + L.tr[1]));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// S and dP chains of the one-wavefront dK / dV kernel, as inline assembly so that their accumulators live in ordinary
// vector registers: in a kernel that may use more than 256 registers the compiler keeps every MFMA accumulator it
// selects itself in the accumulation registers, and the two 32 x 256 accumulators of that kernel already fill those.
// The compiler does not track matrix-core hazards through inline assembly: the result of a chain must not be touched
// by another instruction until 11 issue slots after its last MFMA.  chain_fence() orders the readers of a chain
// behind whatever was issued before it (the other chain; the arithmetic on the other chain's result).
__device__ __forceinline__ f32x16 chain_mfma0(bf16x8 a, bf16x8 b) {
  f32x16 d;
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "v"(b));
  return d;
}
__device__ __forceinline__ f32x16 chain_mfma(bf16x8 a, bf16x8 b, f32x16 acc) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
  return acc;
}
// The same for the products that accumulate dK and dV, with the accumulator pinned to the accumulation registers
// (left to the compiler, part of the 256 accumulator registers ends up in ordinary registers and the K fragments in
// scratch memory).  Successive MFMAs on one accumulator are interlocked by the hardware; acc_settle() pads the one
// place where other instructions read them: after the loop.
__device__ __forceinline__ void acc_mfma(bf16x8 a, bf16x8 b, f32x16 &acc) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// 0 * 0 + 0: the accumulator is born in an accumulation register.  The compiler materialises the zero operand with
// vector-ALU moves right in front of the statement; the idle slots keep the MFMA from reading it before it is
// written (seen on the GPU: without them the first accumulator zeroed this way came out non-finite now and then).
__device__ __forceinline__ f32x16 acc_zero() {
  f32x16 d;
  const bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
  asm volatile("s_nop 7\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %1, 0" : "=a"(d) : "v"(z));
  return d;
}
__device__ __forceinline__ void acc_settle(f32x16 *x, f32x16 *y) {  // 8 + 8 accumulators
  asm volatile("s_nop 15\n\ts_nop 1"
               : "+a"(x[0]), "+a"(x[1]), "+a"(x[2]), "+a"(x[3]), "+a"(x[4]), "+a"(x[5]), "+a"(x[6]), "+a"(x[7]));
  asm volatile("" : "+a"(y[0]), "+a"(y[1]), "+a"(y[2]), "+a"(y[3]), "+a"(y[4]), "+a"(y[5]), "+a"(y[6]), "+a"(y[7]));
}
__device__ __forceinline__ void acc_settle(f32x16 *x) {  // 8 accumulators
  asm volatile("s_nop 15\n\ts_nop 1"
               : "+a"(x[0]), "+a"(x[1]), "+a"(x[2]), "+a"(x[3]), "+a"(x[4]), "+a"(x[5]), "+a"(x[6]), "+a"(x[7]));
}
__device__ __forceinline__ void chain_fence(f32x16 &acc) { asm volatile("" : "+v"(acc)); }
__device__ __forceinline__ void chain_fence(f32x16 &acc, f32x16 &other) { asm volatile("" : "+v"(acc), "+v"(other)); }
__device__ __forceinline__ void chain_fence(f32x16 &acc, u32x4 &a, u32x4 &b) { asm volatile("" : "+v"(acc), "+v"(a), "+v"(b)); }

// ---------------------------------------------------------------------------
// Delta[b,h,t] = sum_d dO[b,t,h,d] * O[b,t,h,d]; d_h / 8 lanes x 16 bytes per (t,h) row
// ---------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void delta_kernel(const bf16_t *__restrict__ dO, const bf16_t *__restrict__ O,
                                                   const bf16_t *__restrict__ OLO, float *__restrict__ delta,
                                                   long long n_rows, int T, int Hq) {
  constexpr int LPR = DH / 8;  // lanes per row
  const long long row = (long long)blockIdx.x * (256 / LPR) + threadIdx.x / LPR;  // row = (b*T + t)*Hq + h
  const int sub = threadIdx.x % LPR;
  float acc = 0.f;
  if (row < n_rows) {
    const u32x4 a = *reinterpret_cast<const u32x4 *>(dO + row * DH + sub * 8);
    const u32x4 b = *reinterpret_cast<const u32x4 *>(O + row * DH + sub * 8);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc += bf_lo(a[i]) * bf_lo(b[i]) + bf_hi(a[i]) * bf_hi(b[i]);
    if (OLO) {  // O to ~16 mantissa bits: with O rounded to bf16 alone, the error of Delta dominates dQ and dK
                // whenever the softmax is flat (measured 2 % at T = 700 with 0.02-scaled weights)
      const u32x4 c = *reinterpret_cast<const u32x4 *>(OLO + row * DH + sub * 8);
#pragma unroll
      for (int i = 0; i < 4; ++i) acc += bf_lo(a[i]) * bf_lo(c[i]) + bf_hi(a[i]) * bf_hi(c[i]);
    }
  }
#pragma unroll
  for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
  if (sub == 0 && row < n_rows) {
    const long long bt = row / Hq;
    const int h = (int)(row % Hq);
    const long long b = bt / T;
    const int t = (int)(bt % T);
    delta[(b * Hq + h) * T + t] = acc;
  }
}

// ---------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------
constexpr int DQ_NT = 512, BKV = 64;

// DQ_NT_ threads = DQ_NT_ / 64 wavefronts x 32 query rows per workgroup: 512 threads (two wavefronts per SIMD) for
// d_h <= 128; 256 threads (one wavefront per SIMD, twice the registers: the 32 x 256 accumulator moves to the
// accumulation registers) for d_h = 256.
template <int DH, bool CAUSAL, int DQ_NT_>
__device__ __forceinline__ void attn_bwd_dq_body(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K, const bf16_t *__restrict__ V,
    const bf16_t *__restrict__ dO, const float *__restrict__ LSE, const float *__restrict__ DELTA,
    bf16_t *__restrict__ dQ, int T, int Hq, int Hk, int BH, int nqb, int paired, float scale, unsigned char *smem) {
  CCA_BWD_GEOMETRY(DH);
  constexpr int DQ_BQ = DQ_NT_ / 2;
  constexpr bool WIDE = DQ_NT_ == 256;
  constexpr int TILE = BKV * ROW;
  constexpr int PER_THREAD = BKV * KCH / DQ_NT_;  // 16-byte chunks of K (and of V) per thread per tile
  constexpr int ROWS_PER_PASS = DQ_NT_ / KCH;
  unsigned char *const sK = smem, *const sV = smem + 2 * TILE;  // K0 K1 V0 V1

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int idx = blockIdx.x;
  const int bh = idx % BH, slot = idx / BH;
  const int b = bh / Hq, h = bh % Hq, g = h / (Hq / Hk);
  const float c = scale * LOG2E;
  const int row_bytes = Hk * DH * 2;
  const unsigned char *const Kg = reinterpret_cast<const unsigned char *>(K + ((long long)b * T * Hk + g) * DH);
  const unsigned char *const Vg = reinterpret_cast<const unsigned char *>(V + ((long long)b * T * Hk + g) * DH);

  const int s_r0 = tid / KCH, s_ch = tid % KCH;
  // chunk i of this thread lies ROWS_PER_PASS * i rows further down; the swizzle of a row depends on its index
  // modulo 16, so with 8 rows per pass the odd passes flip bit 1 of the chunk position
  static_assert(ROWS_PER_PASS % 8 == 0, "the swizzle of a row depends on its index modulo 16");
  const uint32_t s_off = (uint32_t)s_r0 * ROW + ((s_ch ^ swz(s_r0)) << 4);
  const uint32_t s_off_odd = ROWS_PER_PASS % 16 == 0 ? s_off : (s_off ^ 32u);
  const LaneSwz LS = lane_swz<DH>(lane);

  // Staging registers of the next tile.  One wavefront per SIMD: a single set carries K and V in turn (K of tile
  // j+1 is put into LDS and V of tile j+1 requested before tile j is multiplied, V put down and K of tile j+2
  // requested after), because the query and dO fragments alone take half of the ordinary registers.
  u32x4 rk[PER_THREAD], rv[WIDE ? 1 : PER_THREAD];
  auto load_half = [&](const unsigned char *src, u32x4 *r, int kv0) {
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int s = min(kv0 + s_r0 + i * ROWS_PER_PASS, T - 1);  // clamped keys are masked below
      r[i] = *reinterpret_cast<const u32x4 *>(src + (long long)s * row_bytes + s_ch * 16);
    }
  };
  auto store_half = [&](unsigned char *dst, const u32x4 *r, int buf) {
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const uint32_t o = ((i & 1) ? s_off_odd : s_off) + i * ROWS_PER_PASS * ROW;
      *reinterpret_cast<u32x4 *>(dst + buf * TILE + o) = r[i];
    }
  };
  auto load_tile = [&](int kv0) {  // two wavefronts per SIMD only
    if constexpr (!WIDE) {
      load_half(Kg, rk, kv0);
      load_half(Vg, rv, kv0);
    }
  };
  auto store_tile = [&](int buf) {
    if constexpr (!WIDE) {
      store_half(sK, rk, buf);
      store_half(sV, rv, buf);
    }
  };

  // Causal work per query block grows with its index: heavy blocks are issued first (unpaired), or each
  // workgroup takes one heavy and one light block (paired) so that all workgroups do equal work (as in the
  // forward kernel; measured 7 % faster for this kernel at B * H_q = 8, T = 16384).
  const int npass = paired ? 2 : 1;
  for (int pass = 0; pass < npass; ++pass) {
  const int qb = (paired && pass == 1) ? slot : nqb - 1 - slot;
  if (pass == 1 && slot >= nqb - 1 - slot) break;  // odd count: the middle block was done in pass 0
  const int q0 = qb * DQ_BQ, qw0 = q0 + wave * 32;
  const bool wave_live = qw0 < T;
  const int wave_last = min(qw0 + 31, T - 1);
  const int trow = min(qw0 + l32, T - 1);
  bf16x8 qf[KK], dof[KK];
  {
    const bf16_t *pq = Q + (((long long)b * T + trow) * Hq + h) * DH + half * 8;
    const bf16_t *pd = dO + (((long long)b * T + trow) * Hq + h) * DH + half * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      u32x4 w = *reinterpret_cast<const u32x4 *>(pq + kk * 16);
      w.x = pack2(bf_lo(w.x) * c, bf_hi(w.x) * c);
      w.y = pack2(bf_lo(w.y) * c, bf_hi(w.y) * c);
      w.z = pack2(bf_lo(w.z) * c, bf_hi(w.z) * c);
      w.w = pack2(bf_lo(w.w) * c, bf_hi(w.w) * c);
      qf[kk] = __builtin_bit_cast(bf16x8, w);  // log2 units, rounded as in the forward kernel
      dof[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(pd + kk * 16));
    }
  }
  const float lse2 = LSE[((long long)b * Hq + h) * T + trow] * LOG2E;  // exp(s*scale - lse) = exp2(s*c - lse2)
  float delta = DELTA[((long long)b * Hq + h) * T + trow];
  // taken through an empty asm once: as a value still "in flight" from memory it made the first use in every tile
  // iteration wait for all vector memory operations, i.e. for the tile loads issued just before
  asm volatile("" : "+v"(delta));

  f32x16 acc[DT];  // dQ^T: lane = query row, registers = channels
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    if constexpr (WIDE) {
      acc[dt] = acc_zero();
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[dt][r] = 0.f;
    }
  }
  if constexpr (WIDE) acc_settle(acc);  // the compiler may move the fresh accumulators around

  // One block of 32 keys of the tile at kp / vp against this wavefront's 32 query rows.  LDS fragments are requested
  // PF products ahead of their use, the first transposed ones before the arithmetic that precedes their chain (left
  // to itself the compiler issues read, wait, MFMA one at a time).
  constexpr int PF = WIDE ? 4 : 2, PT = WIDE ? 4 : 3;  // deeper with one wavefront per SIMD: nothing else hides the LDS latency
  auto block = [&](const unsigned char *kp, const unsigned char *vp, int kv0, int ks, auto masked_t) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_t)::value;
    auto col = [&](const unsigned char *tile, int kk) {
      return *reinterpret_cast<const u32x4 *>(tile + LS.col[kk & 1] + ks * 32 * ROW + 64 * (kk >> 1));
    };
    auto frag_of = [&](int i) { return tr_frag<ROW>(kp, LS, ks * 32 + (i / DT) * 16, i % DT); };  // i -> (jj, dt)
    constexpr int NP = 2 * DT;
    static_assert(PT <= NP && PF <= KK, "prefetch depth");
    u32x4 fk[PF], fv[PF];
    bf16x8 tk[PT];
    f32x16 s, dp;
    // lane (l32, half) holds keys kv0 + ks*32 + 8*(r/4) + 4*half + r%4 of query row qw0 + l32
    float ds[16];
    const int lim = (CAUSAL ? min(qw0 + l32, T - 1) : T - 1) - kv0 - ks * 32 - 4 * half;
    if constexpr (WIDE) {
      // the S chain, then the dP chain, as inline assembly on ordinary registers; S is first read after the whole dP
      // chain was issued, dP after the probabilities were formed (chain_fence)
#pragma unroll
      for (int i = 0; i < PF; ++i) fk[i] = col(kp, i);
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 kf = __builtin_bit_cast(bf16x8, fk[kk % PF]);
        if (kk + PF < KK) fk[kk % PF] = col(kp, kk + PF);
        else fv[kk + PF - KK] = col(vp, kk + PF - KK);
        s = kk == 0 ? chain_mfma0(kf, qf[0]) : chain_mfma(kf, qf[kk], s);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 vf = __builtin_bit_cast(bf16x8, fv[kk % PF]);
        if (kk + PF < KK) fv[kk % PF] = col(vp, kk + PF);
        else if (kk + PF - KK < PT) tk[kk + PF - KK] = frag_of(kk + PF - KK);
        dp = kk == 0 ? chain_mfma0(vf, dof[0]) : chain_mfma(vf, dof[kk], dp);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = PF; i < PT; ++i) tk[i] = frag_of(i);
      chain_fence(s);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(s[r] - lse2);
        if (MASKED) p = (8 * (r >> 2) + (r & 3) <= lim) ? p : 0.f;
        s[r] = p;
      }
      chain_fence(dp, s);
#pragma unroll
      for (int r = 0; r < 16; ++r) ds[r] = s[r] * (dp[r] - delta);
    } else {
#pragma unroll
      for (int i = 0; i < PF; ++i) fk[i] = col(kp, i), fv[i] = col(vp, i);
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f, dp[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 kf = __builtin_bit_cast(bf16x8, fk[kk % PF]), vf = __builtin_bit_cast(bf16x8, fv[kk % PF]);
        if (kk + PF < KK) fk[kk % PF] = col(kp, kk + PF), fv[kk % PF] = col(vp, kk + PF);
        else if (kk + PF - KK < PT) tk[kk + PF - KK] = frag_of(kk + PF - KK);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[kk], dp, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = PF; i < PT; ++i) tk[i] = frag_of(i);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(s[r] - lse2);
        if (MASKED) p = (8 * (r >> 2) + (r & 3) <= lim) ? p : 0.f;
        ds[r] = p * (dp[r] - delta);
      }
    }
    bf16x8 dsf[2];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      u32x4 w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = pack2(ds[8 * jj + 2 * e], ds[8 * jj + 2 * e + 1]);
      dsf[jj] = __builtin_bit_cast(bf16x8, w);
    }
    __builtin_amdgcn_sched_barrier(0);
    // dQ^T += K^T dS^T
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const bf16x8 f = tk[i % PT];
      if (i + PT < NP) tk[i % PT] = frag_of(i + PT);
      if constexpr (WIDE) acc_mfma(f, dsf[i / DT], acc[i % DT]);
      else acc[i % DT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, dsf[i / DT], acc[i % DT], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  const int kv_end = CAUSAL ? min(q0 + DQ_BQ, T) : T;
  const int ntiles = (kv_end + BKV - 1) / BKV;
  if constexpr (WIDE) {
    load_half(Kg, rk, 0);
    store_half(sK, rk, 0);
    load_half(Vg, rk, 0);
    store_half(sV, rk, 0);
    if (ntiles > 1) load_half(Kg, rk, BKV);
  } else {
    load_tile(0);
    store_tile(0);
    if (ntiles > 1) load_tile(BKV);
  }
  __syncthreads();
  for (int j = 0; j < ntiles; ++j) {
    const int kv0 = j * BKV, buf = j & 1;
    if constexpr (WIDE) {
      if (j + 1 < ntiles) {
        store_half(sK, rk, buf ^ 1);
        load_half(Vg, rk, kv0 + BKV);
      }
    } else {
      if (j + 1 < ntiles) store_tile(buf ^ 1);
      if (j + 2 < ntiles) load_tile(kv0 + 2 * BKV);
    }
    if (wave_live && !(CAUSAL && kv0 > wave_last)) {
      const unsigned char *kp = sK + buf * TILE, *vp = sV + buf * TILE;
      // wave-uniform: tiles below the diagonal and inside the sequence need no mask
      const bool need_mask = (CAUSAL && kv0 + BKV - 1 > qw0) || (kv0 + BKV > T);
      if (WIDE || need_mask) {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) block(kp, vp, kv0, ks, std::true_type{});
      } else {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) block(kp, vp, kv0, ks, std::false_type{});
      }
    }
    if constexpr (WIDE) {
      if (j + 1 < ntiles) {
        store_half(sV, rk, buf ^ 1);
        if (j + 2 < ntiles) load_half(Kg, rk, kv0 + 2 * BKV);
      }
    }
    __syncthreads();
  }
  if constexpr (WIDE) {
    static_assert(!WIDE || DT == 8, "acc_settle takes 8 accumulators");
    acc_settle(acc);
  }
  if (wave_live && qw0 + l32 < T) {
    bf16_t *row = dQ + (((long long)b * T + qw0 + l32) * Hq + h) * DH;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        u32x2 w;
        w.x = pack2(acc[dt][rg * 4 + 0] * scale, acc[dt][rg * 4 + 1] * scale);
        w.y = pack2(acc[dt][rg * 4 + 2] * scale, acc[dt][rg * 4 + 3] * scale);
        *reinterpret_cast<u32x2 *>(row + dt * 32 + rg * 8 + half * 4) = w;
      }
  }
  }  // pass
}

template <int DH, bool CAUSAL>
__global__ __launch_bounds__(DQ_NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dq_kernel(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K, const bf16_t *__restrict__ V,
    const bf16_t *__restrict__ dO, const float *__restrict__ LSE, const float *__restrict__ DELTA,
    bf16_t *__restrict__ dQ, int T, int Hq, int Hk, int BH, int nqb, int paired, float scale) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * BKV * (DH * 2 + 64)];
  attn_bwd_dq_body<DH, CAUSAL, DQ_NT>(Q, K, V, dO, LSE, DELTA, dQ, T, Hq, Hk, BH, nqb, paired, scale, smem);
}

template <int DH, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_bwd_dq_wide_kernel(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K, const bf16_t *__restrict__ V,
    const bf16_t *__restrict__ dO, const float *__restrict__ LSE, const float *__restrict__ DELTA,
    bf16_t *__restrict__ dQ, int T, int Hq, int Hk, int BH, int nqb, int paired, float scale) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * BKV * (DH * 2 + 64)];
  attn_bwd_dq_body<DH, CAUSAL, 256>(Q, K, V, dO, LSE, DELTA, dQ, T, Hq, Hk, BH, nqb, paired, scale, smem);
}

// q in log2 units, rounded to bf16 exactly as the forward kernel rounds it (see the note at the top): written once
// so that the dK / dV kernel can move its Q tiles global -> LDS directly
__global__ __launch_bounds__(256) void scale_q_kernel(const bf16_t *__restrict__ Q, bf16_t *__restrict__ Qs, long long n8,
                                                     float c) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  u32x4 w = *reinterpret_cast<const u32x4 *>(Q + i * 8);
  w.x = pack2(bf_lo(w.x) * c, bf_hi(w.x) * c);
  w.y = pack2(bf_lo(w.y) * c, bf_hi(w.y) * c);
  w.z = pack2(bf_lo(w.z) * c, bf_hi(w.z) * c);
  w.w = pack2(bf_lo(w.w) * c, bf_hi(w.w) * c);
  *reinterpret_cast<u32x4 *>(Qs + i * 8) = w;
}

// ---------------------------------------------------------------------------
// dK, dV
// ---------------------------------------------------------------------------
constexpr int KV_NT = 512;  // threads; a workgroup owns KV_NT / 2 keys

// PARTIAL = false (one query head per KV head): dK, dV written as bf16 (B,T,H_k,d_h).
// PARTIAL = true: this head's contribution written as fp32 to dKp, dVp (B,T,H_q,d_h).
// dK and dV in one pass (S, dP, dV, dK).  The two accumulators and the resident K / V fragments take 192 of the 256
// registers two wavefronts per SIMD leave each lane: the Q and dO tiles therefore go global -> LDS directly (no
// staging registers; q arrives pre-scaled from scale_q_kernel), S is turned into bf16 P before dP is formed, and
// dS is computed from that bf16 P.  (With register staging and fp32 P the pass spilled 98 registers; split into a
// dV pass and a dK pass it cost a fifth contraction.)
// KV_NT_ threads = KV_NT_ / 64 wavefronts x 32 keys per workgroup: 512 (two wavefronts per SIMD, 64-row Q / dO tiles)
// for d_h <= 128; 256 (one wavefront per SIMD, 32-row tiles so that tiles and V fragments fit the LDS) for d_h = 256,
// where dK and dV, 128 registers each, fill the accumulation registers and the S and dP chains run as inline assembly
// on ordinary registers (chain_mfma above).
constexpr int kv_tile_rows(int threads) { return threads == 256 ? 32 : 64; }

template <int DH, bool CAUSAL, bool PARTIAL, int KV_NT_>
__device__ __forceinline__ void attn_bwd_dkdv_body(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K, const bf16_t *__restrict__ V,
    const bf16_t *__restrict__ dO, const float *__restrict__ LSE, const float *__restrict__ DELTA,
    bf16_t *__restrict__ dK, bf16_t *__restrict__ dV, float *__restrict__ dKp, float *__restrict__ dVp, int T, int Hq,
    int Hk, int BH, int nkb, float scale, unsigned char *smem) {
  CCA_BWD_GEOMETRY(DH);
  constexpr int KV_NT = KV_NT_, KV_BK = KV_NT_ / 2, BQT = kv_tile_rows(KV_NT_);
  constexpr bool WIDE = KV_NT_ == 256;
  constexpr int TILE = BQT * ROW;
  // smem: Q0 Q1 dO0 dO1, 4 * TILE bytes of dynamic LDS (with a static array the compiler makes every LDS read wait
  // for the tile loads in flight (vmcnt(0): a load into LDS might alias what is read), which puts the latency of the
  // next tile's loads in front of each step)
  // [buf][-lse2 | -Delta][row]: the S and dP chains START from these (lane = key, register = query row), so that the
  // chains deliver S - lse and dP - Delta and the arithmetic needs no subtraction
  __shared__ __attribute__((aligned(16))) float sStat[2][2][BQT];
  // this workgroup's V rows as MFMA operand fragments, [wavefront][kk][lane] x 16 bytes: each wavefront keeps its own
  // (read back one fragment per dP product; holding them in registers next to the K fragments and the two
  // accumulators leaves no room for fragments requested ahead of their use)
  __shared__ __attribute__((aligned(16))) u32x4 sVf[KV_NT / 64][KK][64];
  unsigned char *const sQ = smem, *const sD = smem + 2 * TILE;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int idx = blockIdx.x;
  const int bh = idx % BH, kb = idx / BH;  // early key blocks (most query tiles when causal) first
  const int b = bh / Hq, h = bh % Hq, g = h / (Hq / Hk);
  const int k0 = kb * KV_BK, kw0 = k0 + wave * 32;
  const float c = scale * LOG2E;
  const int qrow_bytes = Hq * DH * 2;

  const LaneSwz LS = lane_swz<DH>(lane);

  // this wavefront's 32 keys: K and V rows as second MFMA operands, resident in registers
  bf16x8 kf[KK];
  {
    const int s = min(kw0 + l32, T - 1);
    const bf16_t *pk = K + (((long long)b * T + s) * Hk + g) * DH + half * 8;
    const bf16_t *pv = V + (((long long)b * T + s) * Hk + g) * DH + half * 8;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      kf[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(pk + kk * 16));
      sVf[wave][kk][lane] = *reinterpret_cast<const u32x4 *>(pv + kk * 16);
    }
  }
  f32x16 dk[DT], dv[DT];  // dK^T, dV^T: lane = key, registers = channels
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    if constexpr (WIDE) {
      dk[dt] = acc_zero(), dv[dt] = acc_zero();
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) dk[dt][r] = 0.f, dv[dt][r] = 0.f;
    }
  }
  if constexpr (WIDE) acc_settle(dk, dv);  // the compiler may move the fresh accumulators around

  // query tiles that see keys of this block
  const int qt_first = CAUSAL ? k0 / BQT : 0;
  const int nqt = (T + BQT - 1) / BQT;
  const int steps = nqt - qt_first;

  // Q (pre-scaled) and dO tiles travel global -> LDS directly: wave instruction i deposits 64 x 16 bytes at LDS
  // chunks [i*64, i*64+64) of the tile, so each lane fetches the chunk that the layout puts at its position (lanes
  // landing on padding fetch a duplicate).
  constexpr int CPR = ROW / 16;                 // chunk positions per padded row: 20 (d_h = 128), 12 (d_h = 64)
  constexpr int T_INSTR = BQT * CPR / 64;       // wave instructions per tile
  static_assert(BQT * CPR % 64 == 0, "tile must be a whole number of wave instructions");
  constexpr int PER_WAVE = (2 * T_INSTR + KV_NT / 64 - 1) / (KV_NT / 64);
  typedef __attribute__((address_space(3))) void lds_void;
  typedef __attribute__((address_space(1))) void glb_void;
  const unsigned char *const Qg = reinterpret_cast<const unsigned char *>(Q + ((long long)b * T * Hq + h) * DH);
  const unsigned char *const Dg = reinterpret_cast<const unsigned char *>(dO + ((long long)b * T * Hq + h) * DH);
  float rstat = 0.f;
  // per lane and wave instruction: (row of the tile, byte offset of the chunk in its row), packed; the global address
  // is a wave-uniform base plus a 32-bit offset (T * H_q * d_h * 2 < 2^31 is a precondition of this path)
  uint32_t dma_rc[PER_WAVE];
#pragma unroll
  for (int u = 0; u < PER_WAVE; ++u) {
    const int i = wave + u * (KV_NT / 64);
    const int ii = i >= T_INSTR ? i - T_INSTR : i;
    const int L = ii * 64 + lane;
    const int row = L / CPR, ch = min(L % CPR, KCH - 1) ^ swz(row);
    dma_rc[u] = (uint32_t)row | ((uint32_t)ch << 12);  // ch * 16 = dma_rc >> 8 with the row bits masked off
  }
  auto issue_tile = [&](int step, int buf) {
    const int t0 = (qt_first + step) * BQT;
    // the row statistics first, untouched until they land: arithmetic on them here would wait for them and, loads
    // completing in order, for every tile load issued before
    if (tid < 2 * BQT) {
      const int t = min(t0 + (tid & (BQT - 1)), T - 1);
      const long long o = ((long long)b * Hq + h) * T + t;
      rstat = tid < BQT ? LSE[o] : DELTA[o];
    }
#pragma unroll
    for (int u = 0; u < PER_WAVE; ++u) {
      const int i = wave + u * (KV_NT / 64);
      if (i < 2 * T_INSTR) {
        const bool isd = i >= T_INSTR;
        const int ii = isd ? i - T_INSTR : i;
        const int t = min(t0 + (int)(dma_rc[u] & 0xfffu), T - 1);  // clamped rows get probability 0 below
        const uint32_t off = (uint32_t)t * (uint32_t)qrow_bytes + ((dma_rc[u] >> 8) & 0xfff0u);
        const unsigned char *src = (isd ? Dg : Qg) + off;
        unsigned char *dst = (isd ? sD : sQ) + buf * TILE + ii * 1024;
        __builtin_amdgcn_global_load_lds((glb_void *)src, (lds_void *)dst, 16, 0, 0);
      }
    }
  };
  auto land_tile = [&](int buf) {  // before the barrier that publishes the tile
    if (tid < 2 * BQT) sStat[buf][tid / BQT][tid & (BQT - 1)] = tid < BQT ? -rstat * LOG2E : -rstat;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };

  // One block of 32 query rows of the tile in stage `buf` against this wavefront's 32 keys.  LDS fragments are
  // requested PF MFMAs ahead of their use (the compiler on its own issues read, wait, MFMA one at a time, and the
  // wavefronts then spend most of their cycles waiting for LDS), the first ones of a chain before the arithmetic
  // that precedes it.
  constexpr int PF = WIDE ? 4 : 2;  // one wavefront per SIMD: nothing else hides the LDS latency
  auto block = [&](const unsigned char *qp, const unsigned char *dp_, int buf, int t0, int qs, auto masked_t) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_t)::value;
    auto col = [&](const unsigned char *tile, int kk) {
      return *reinterpret_cast<const u32x4 *>(tile + LS.col[kk & 1] + qs * 32 * ROW + 64 * (kk >> 1));
    };
    bf16x8 pf[2], dsf[2];
    u32x4 fr[PF], fd[PF], fv[PF];
    constexpr int NP = 4 * DT;  // products of the last phase: dV (jj, dt), then dK (jj, dt)
    auto frag_of = [&](int i) {  // i -> (dO | Q, jj, dt)
      const int which = i / (2 * DT), jj = (i / DT) & 1, dt = i % DT;
      return tr_frag<ROW>(which ? qp : dp_, LS, qs * 32 + jj * 16, dt);
    };
    bf16x8 tv[PF];  // transposed fragments of the first products of the last phase, requested under the dP chain
#pragma unroll
    for (int i = 0; i < PF; ++i) fr[i] = col(qp, i);
    // S[t, key] - lse[t] and dP[t, key] - Delta[t]: the chains start from minus the row statistics
    auto stats = [&](int which) __attribute__((always_inline)) {
      f32x16 v;
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const f32x4 q4 = *reinterpret_cast<const f32x4 *>(&sStat[buf][which][qs * 32 + rg * 8 + half * 4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) v[rg * 4 + e] = q4[e];
      }
      return v;
    };
    f32x16 s = stats(0), dp;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8 qa = __builtin_bit_cast(bf16x8, fr[kk % PF]);
      if (kk + PF < KK) fr[kk % PF] = col(qp, kk + PF);
      else {  // first fragments of the dP chain
        fd[kk + PF - KK] = col(dp_, kk + PF - KK);
        fv[kk + PF - KK] = sVf[wave][kk + PF - KK][lane];
      }
      if constexpr (WIDE) s = chain_mfma(qa, kf[kk], s);
      else s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf[kk], s, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    // S -> P, packed to bf16 at once.  Lane (l32, half) holds key kw0 + l32 and query rows t0 + qs*32 + 8*(r/4) +
    // 4*half + r%4.  Masked tiles: the row index relative to t0 + qs*32 + 4*half must lie in [lo, hi] (lo: causal,
    // hi: end of the sequence; a key past the end has an empty range).
    u32x4 w[2], x[2];
    const int key = kw0 + l32, tb = t0 + qs * 32 + 4 * half;
    const int lo = CAUSAL ? key - tb : -(1 << 20);
    const unsigned span = key < T ? (unsigned)(T - 1 - tb - lo) : 0u;
    const bool none = MASKED && (key >= T || T - 1 - tb < lo);
    // slice g = 0..7 of the arithmetic on S / dP: values 2g, 2g+1 of this lane -> one packed word
    auto p_slice = [&](int g) __attribute__((always_inline)) {
      const int rg = g >> 1, pr = g & 1;
      float pv[2];
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        pv[e] = __builtin_amdgcn_exp2f(s[rg * 4 + 2 * pr + e]);
        if (MASKED) pv[e] = (!none & ((unsigned)(rg * 8 + 2 * pr + e - lo) <= span)) ? pv[e] : 0.f;
      }
      w[rg >> 1][(rg & 1) * 2 + pr] = pack2(pv[0], pv[1]);
    };
    auto ds_slice = [&](int g) __attribute__((always_inline)) {  // dS = P (dP - Delta): P taken back from its bf16 form, times the chain's result
      const int rg = g >> 1, pr = g & 1;
      const uint32_t pw = w[rg >> 1][(rg & 1) * 2 + pr];
      x[rg >> 1][(rg & 1) * 2 + pr] = pack2(bf_lo(pw) * dp[rg * 4 + 2 * pr], bf_hi(pw) * dp[rg * 4 + 2 * pr + 1]);
    };
    // Two wavefronts per SIMD: P is formed between the chains (one accumulator live at a time) and dS after the dP
    // chain.  One wavefront: nothing else fills the matrix core while this wavefront does arithmetic, so the
    // arithmetic on S is issued in slices between the MFMAs of the dP chain and the arithmetic on dP between the
    // dV products (which need P only); each chain's result is first touched behind an MFMA that had to wait for
    // one issued after the chain's last.
    if constexpr (!WIDE) {
#pragma unroll
      for (int g = 0; g < 8; ++g) p_slice(g);
      __builtin_amdgcn_sched_barrier(0);
    }
    dp = stats(1);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {  // dP[t, key]
      const bf16x8 da = __builtin_bit_cast(bf16x8, fd[kk % PF]), vb = __builtin_bit_cast(bf16x8, fv[kk % PF]);
      if (kk + PF < KK) {
        fd[kk % PF] = col(dp_, kk + PF);
        fv[kk % PF] = sVf[wave][kk + PF][lane];
      } else {
        tv[kk + PF - KK] = frag_of(kk + PF - KK);
      }
      if constexpr (WIDE) dp = chain_mfma(da, vb, dp);
      else dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da, vb, dp, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (WIDE) {
        // S is first read after the third MFMA of this chain: each link waits for the one before it, so two whole
        // MFMAs have run since the S chain's last one was issued
        static_assert(!WIDE || KK >= 11, "eight slices after the third MFMA of the chain");
        if (kk == 2) chain_fence(s);
        if (kk >= 3 && kk < 11) {
          p_slice(kk - 3);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    pf[0] = __builtin_bit_cast(bf16x8, w[0]);
    pf[1] = __builtin_bit_cast(bf16x8, w[1]);
    if constexpr (!WIDE) {
#pragma unroll
      for (int g = 0; g < 8; ++g) ds_slice(g);
      dsf[0] = __builtin_bit_cast(bf16x8, x[0]);
      dsf[1] = __builtin_bit_cast(bf16x8, x[1]);
    }
    __builtin_amdgcn_sched_barrier(0);
    // dV^T += dO^T P (all of them first: they do not wait for dS), then dK^T += Q^T dS; product i of the 4*DT
    // uses fragment i, requested PF products earlier
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const bf16x8 f = tv[i % PF];
      if (i + PF < NP) tv[i % PF] = frag_of(i + PF);
      const int which = i / (2 * DT), jj = (i / DT) & 1, dt = i % DT;
      if constexpr (WIDE) {
        if (which == 0) acc_mfma(f, pf[jj], dv[dt]);
        else acc_mfma(f, dsf[jj], dk[dt]);
      } else {
        if (which == 0) dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, pf[jj], dv[dt], 0, 0, 0);
        else dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, dsf[jj], dk[dt], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (WIDE) {
        // dP is first read after dV product DT: it waits for product 0 on the same accumulator, which entered the
        // matrix core behind the dP chain's last MFMA.  (This does not rely on how many independent MFMAs the core
        // accepts before it holds the wavefront back, which is not documented.)
        static_assert(!WIDE || DT == 8, "eight slices under the second half of the dV products");
        if (i == DT) chain_fence(dp);
        if (i >= DT && i < 2 * DT) {
          ds_slice(i - DT);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (i == 2 * DT - 1) {
          // both halves of dS packed here, in registers of their own: packed later, the second half landed in the
          // registers of the first right behind the last MFMA that read them, and dK came out wrong on the GPU
          asm volatile("" : "+v"(x[0]), "+v"(x[1]));
          dsf[0] = __builtin_bit_cast(bf16x8, x[0]);
          dsf[1] = __builtin_bit_cast(bf16x8, x[1]);
        }
      }
    }
  };

  const bool wave_live = kw0 < T;
  if (steps > 0) {
    issue_tile(0, 0);
    land_tile(0);
    __syncthreads();
  }
  for (int step = 0; step < steps; ++step) {
    const int buf = step & 1;
    const int t0 = (qt_first + step) * BQT;
    if (step + 1 < steps) issue_tile(step + 1, buf ^ 1);  // that buffer was last read before the previous barrier
    if (wave_live && !(CAUSAL && t0 + BQT - 1 < kw0)) {
      const unsigned char *qp = sQ + buf * TILE, *dp_ = sD + buf * TILE;
      // wave-uniform: tiles away from the diagonal and from the end of the sequence need no mask at all
      const bool need_mask = (CAUSAL && t0 < kw0 + 31) || (t0 + BQT > T) || (kw0 + 32 > T);
      if (need_mask) {
#pragma unroll
        for (int qs = 0; qs < BQT / 32; ++qs) block(qp, dp_, buf, t0, qs, std::true_type{});
      } else {
#pragma unroll
        for (int qs = 0; qs < BQT / 32; ++qs) block(qp, dp_, buf, t0, qs, std::false_type{});
      }
    }
    if (step + 1 < steps) land_tile(buf ^ 1);
    __syncthreads();
  }
  if constexpr (WIDE) {
    static_assert(!WIDE || DT == 8, "acc_settle takes 8 + 8 accumulators");
    acc_settle(dk, dv);
  }
  if (PARTIAL) {
    if (wave_live && kw0 + l32 < T) {
      float *rk_ = dKp + (((long long)b * T + kw0 + l32) * Hq + h) * DH;
      float *rv_ = dVp + (((long long)b * T + kw0 + l32) * Hq + h) * DH;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          const f32x4 w = {dk[dt][rg * 4 + 0] * LN2, dk[dt][rg * 4 + 1] * LN2, dk[dt][rg * 4 + 2] * LN2,
                           dk[dt][rg * 4 + 3] * LN2};
          const f32x4 x = {dv[dt][rg * 4 + 0], dv[dt][rg * 4 + 1], dv[dt][rg * 4 + 2], dv[dt][rg * 4 + 3]};
          *reinterpret_cast<f32x4 *>(rk_ + dt * 32 + rg * 8 + half * 4) = w;
          *reinterpret_cast<f32x4 *>(rv_ + dt * 32 + rg * 8 + half * 4) = x;
        }
    }
    return;
  }
  if (wave_live && kw0 + l32 < T) {
    bf16_t *rk_ = dK + (((long long)b * T + kw0 + l32) * Hk + g) * DH;
    bf16_t *rv_ = dV + (((long long)b * T + kw0 + l32) * Hk + g) * DH;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        u32x2 w, x;
        w.x = pack2(dk[dt][rg * 4 + 0] * LN2, dk[dt][rg * 4 + 1] * LN2);
        w.y = pack2(dk[dt][rg * 4 + 2] * LN2, dk[dt][rg * 4 + 3] * LN2);
        x.x = pack2(dv[dt][rg * 4 + 0], dv[dt][rg * 4 + 1]);
        x.y = pack2(dv[dt][rg * 4 + 2], dv[dt][rg * 4 + 3]);
        *reinterpret_cast<u32x2 *>(rk_ + dt * 32 + rg * 8 + half * 4) = w;
        *reinterpret_cast<u32x2 *>(rv_ + dt * 32 + rg * 8 + half * 4) = x;
      }
  }
}

template <int DH, bool CAUSAL, bool PARTIAL>
__global__ __launch_bounds__(KV_NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dkdv_kernel(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K, const bf16_t *__restrict__ V,
    const bf16_t *__restrict__ dO, const float *__restrict__ LSE, const float *__restrict__ DELTA,
    bf16_t *__restrict__ dK, bf16_t *__restrict__ dV, float *__restrict__ dKp, float *__restrict__ dVp, int T, int Hq,
    int Hk, int BH, int nkb, float scale) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  attn_bwd_dkdv_body<DH, CAUSAL, PARTIAL, KV_NT>(Q, K, V, dO, LSE, DELTA, dK, dV, dKp, dVp, T, Hq, Hk, BH, nkb, scale, smem);
}

template <int DH, bool CAUSAL, bool PARTIAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_bwd_dkdv_wide_kernel(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K, const bf16_t *__restrict__ V,
    const bf16_t *__restrict__ dO, const float *__restrict__ LSE, const float *__restrict__ DELTA,
    bf16_t *__restrict__ dK, bf16_t *__restrict__ dV, float *__restrict__ dKp, float *__restrict__ dVp, int T, int Hq,
    int Hk, int BH, int nkb, float scale) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  attn_bwd_dkdv_body<DH, CAUSAL, PARTIAL, 256>(Q, K, V, dO, LSE, DELTA, dK, dV, dKp, dVp, T, Hq, Hk, BH, nkb, scale, smem);
}

// out[(row, g), :] = bf16(sum_r part[(row, g*R + r), :]) for dK and dV, 4 channels per thread, fixed order
template <int DH>
__global__ __launch_bounds__(256) void group_sum_kernel(const float *__restrict__ pk, const float *__restrict__ pv,
                                                       bf16_t *__restrict__ dK, bf16_t *__restrict__ dV,
                                                       long long n_out, int R) {
  const long long id = (long long)blockIdx.x * 256 + threadIdx.x;  // (row*Hk + g) * (DH/4) + c4
  if (id >= n_out) return;
  const long long rg = id / (DH / 4);
  const int c = (int)(id % (DH / 4)) * 4;
  f32x4 ak = {0.f, 0.f, 0.f, 0.f}, av = {0.f, 0.f, 0.f, 0.f};
  for (int r = 0; r < R; ++r) {
    const f32x4 a = *reinterpret_cast<const f32x4 *>(pk + (rg * R + r) * DH + c);
    const f32x4 b = *reinterpret_cast<const f32x4 *>(pv + (rg * R + r) * DH + c);
    ak.x += a.x; ak.y += a.y; ak.z += a.z; ak.w += a.w;
    av.x += b.x; av.y += b.y; av.z += b.z; av.w += b.w;
  }
  u32x2 w, x;
  w.x = pack2(ak.x, ak.y); w.y = pack2(ak.z, ak.w);
  x.x = pack2(av.x, av.y); x.y = pack2(av.z, av.w);
  *reinterpret_cast<u32x2 *>(dK + rg * DH + c) = w;
  *reinterpret_cast<u32x2 *>(dV + rg * DH + c) = x;
}

}  // namespace

bool attention_bwd_supported(const Dims &d) {
  return d.bf16 && (d.dh == 256 || d.dh == 128 || d.dh == 64) && (long long)d.T * d.Hq * d.dh * 2 < (1ll << 31);
}

// Delta (B,H_q,T) fp32, then (R > 1 only) the per-query-head fp32 contributions to dK and dV, (B,T,H_q,d_h) each,
// then the scaled q (B,T,H_q,d_h) bf16
static size_t delta_bytes(const Dims &d) { return ((size_t)d.B * d.Hq * d.T * sizeof(float) + 255) / 256 * 256; }
size_t attention_bwd_scratch_bytes(const Dims &d) {
  if (!attention_bwd_supported(d)) return (size_t)d.B * d.Hq * d.T * sizeof(float);
  return delta_bytes(d) + (d.R > 1 ? 2 * (size_t)d.rows() * d.e_q * sizeof(float) : 0) + (size_t)d.rows() * d.e_q * 2;
}

template <int DH>
static hipError_t attention_bwd_run(const Dims &d, const void *q, const void *k, const void *v, const void *o,
                                    const void *o_lo, const float *lse, const void *d_o, void *d_q, void *d_k, void *d_v,
                                    float *delta, hipStream_t s) {
  const bool causal = d.flags & CCA_CAUSAL;
  const long long n_rows = d.rows() * d.Hq;
  constexpr int DELTA_ROWS = 256 / (DH / 8);  // rows per workgroup of delta_kernel
  delta_kernel<DH><<<(unsigned)((n_rows + DELTA_ROWS - 1) / DELTA_ROWS), 256, 0, s>>>((const bf16_t *)d_o, (const bf16_t *)o, (const bf16_t *)o_lo, delta,
                                                             n_rows, d.T,
                                                             d.Hq);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  constexpr bool WIDE = DH > 128;                 // one wavefront per SIMD, half as many rows per workgroup
  constexpr int NTH = WIDE ? 256 : DQ_NT;         // threads of both kernels (DQ_NT == KV_NT)
  constexpr int ROWS = NTH / 2;                   // query rows (dQ) or keys (dK / dV) per workgroup
  static_assert(DQ_NT == KV_NT, "one thread count for both kernels");
  const int BH = d.B * d.Hq, nqb = (d.T + ROWS - 1) / ROWS;
  const int nkb = (d.T + ROWS - 1) / ROWS;
  float *pk = reinterpret_cast<float *>(reinterpret_cast<char *>(delta) + delta_bytes(d));
  float *pv = pk + (size_t)d.rows() * d.e_q;
  bf16_t *qs = reinterpret_cast<bf16_t *>(reinterpret_cast<char *>(delta) + delta_bytes(d) +
                                          (d.R > 1 ? 2 * (size_t)d.rows() * d.e_q * sizeof(float) : 0));
  {
    const long long n8 = d.rows() * d.e_q / 8;
    scale_q_kernel<<<(unsigned)((n8 + 255) / 256), 256, 0, s>>>((const bf16_t *)q, qs, n8, d.scale * LOG2E);
  }
#define ARGS_DQ (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v, (const bf16_t *)d_o, lse, delta, (bf16_t *)d_q, \
                d.T, d.Hq, d.Hk, BH, nqb, paired, d.scale
#define ARGS_KV (const bf16_t *)qs, (const bf16_t *)k, (const bf16_t *)v, (const bf16_t *)d_o, lse, delta, (bf16_t *)d_k, \
                (bf16_t *)d_v, pk, pv, d.T, d.Hq, d.Hk, BH, nkb, d.scale
  const unsigned gkv = (unsigned)((long long)BH * nkb);
  constexpr size_t kv_smem = 4ull * kv_tile_rows(NTH) * (DH * 2 + 64);  // the Q / dO tiles of the dK / dV kernel
  // pairing query blocks only pays while it still leaves a workgroup for each of the 256 CUs; the dK / dV kernel
  // gains nothing from it (measured)
  const int paired = causal && (long long)BH * ((nqb + 1) / 2) >= 256 ? 1 : 0;
  const bool partial = d.R > 1;
  // (the dynamic-LDS limit is raised once per kernel and device: raise_lds_limit)
#define LAUNCH_KV(C_, P_)                                                                                     \
  if constexpr (WIDE) {                                                                                       \
    e = raise_lds_limit<attn_bwd_dkdv_wide_kernel<DH, C_, P_>>(kv_smem);                                      \
    if (e != hipSuccess) return e;                                                                            \
    attn_bwd_dkdv_wide_kernel<DH, C_, P_><<<gkv, NTH, kv_smem, s>>>(ARGS_KV);                                  \
  } else {                                                                                                    \
    e = raise_lds_limit<attn_bwd_dkdv_kernel<DH, C_, P_>>(kv_smem);                                           \
    if (e != hipSuccess) return e;                                                                            \
    attn_bwd_dkdv_kernel<DH, C_, P_><<<gkv, NTH, kv_smem, s>>>(ARGS_KV);                                       \
  }
#define LAUNCH_DQ(C_, G_)                                                                                     \
  if constexpr (WIDE) attn_bwd_dq_wide_kernel<DH, C_><<<(unsigned)(G_), NTH, 0, s>>>(ARGS_DQ);                 \
  else attn_bwd_dq_kernel<DH, C_><<<(unsigned)(G_), NTH, 0, s>>>(ARGS_DQ);
  if (causal) {
    LAUNCH_DQ(true, (long long)BH * (paired ? (nqb + 1) / 2 : nqb));
    if (partial) {
      LAUNCH_KV(true, true);
    } else {
      LAUNCH_KV(true, false);
    }
  } else {
    LAUNCH_DQ(false, (long long)BH * nqb);
    if (partial) {
      LAUNCH_KV(false, true);
    } else {
      LAUNCH_KV(false, false);
    }
  }
#undef LAUNCH_KV
#undef LAUNCH_DQ
#undef ARGS_DQ
#undef ARGS_KV
  if (partial) {
    const long long n_out = d.rows() * d.Hk * (DH / 4);
    group_sum_kernel<DH><<<(unsigned)((n_out + 255) / 256), 256, 0, s>>>(pk, pv, (bf16_t *)d_k, (bf16_t *)d_v, n_out, d.R);
  }
  return hipGetLastError();
}

hipError_t attention_bwd_bf16(const Dims &d, const void *q, const void *k, const void *v, const void *o,
                              const void *o_lo, const float *lse, const void *d_o, void *d_q, void *d_k, void *d_v, float *delta,
                              hipStream_t s) {
  return d.dh == 64    ? attention_bwd_run<64>(d, q, k, v, o, o_lo, lse, d_o, d_q, d_k, d_v, delta, s)
         : d.dh == 128 ? attention_bwd_run<128>(d, q, k, v, o, o_lo, lse, d_o, d_q, d_k, d_v, delta, s)
                       : attention_bwd_run<256>(d, q, k, v, o, o_lo, lse, d_o, d_q, d_k, d_v, delta, s);
}

}  // namespace cca
