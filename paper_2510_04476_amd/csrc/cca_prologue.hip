// Fused latent-space prologue for gfx950, bf16 storage (Sec. 2.2: convolution
// equation, qk-mean equation, value-shift equation and the first two lines of
// the final equation block).  One pass over the down-projected latents yields
// the q, k, v that enter attention.
//
// The two causal convolutions have no bias and no nonlinearity between them,
// so conv2_seq+ch(conv1_seq(u)) is one causal convolution of width
// D = k_seq + k_ch - 1 with per-head filters
//     Wc[h,o,i,d] = sum_{j + jj = d} w1[h,o,i,j] * w0[c(h,i),jj].
// A small set-up kernel forms Wc (fp32, rounded once to bf16) and the RoPE
// tables; the main kernel then runs the convolution as a bf16 MFMA
// contraction per head (M = d_h outputs, N = tokens, K = D*d_h), straight on
// the latent rows: the filter of one head lives in LDS for the lifetime of a
// workgroup, the token operands are the latent rows of tokens t-D+1..t.
//
// The MFMA is issued with the filter as its first operand, so each lane ends
// up with half of the d_h output channels of ONE token (the other half-wave has
// the rest; d_h = 128 or 64): the L2 norm is an in-lane sum plus one half-wave exchange, and
// the rotate-half RoPE partner (o, o + d_h/2) sits in the same lane.  The
// qk-mean skip branch is added by the matrix core as well (a scaled identity
// times the pre-conv latent rows), so it needs no loads in another layout.
//
// RoPE angles: t * theta_i is split as (t >> 7) * 128 * theta_i + (t & 127) *
// theta_i; both parts come from tables made in fp64, combined by the angle
// addition formulas in fp32 (an fp32 product t * theta_i alone is off by up to
// 1e-3 rad at t ~ 16k).
#include "cca_internal.h"

namespace cca {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int NT = 512;
constexpr int MAX_TILES_PER_WAVE = 3;  // a workgroup takes 256 * tiles_per_wave tokens, tiles dealt round-robin

struct FusedArgs {
  int T, Hq, Hk, R, e_q, e_kv, n_lat, v_half, k_seq, k_ch;
  long long rows;
  uint32_t flags;
  int n_conv_blocks;
  int tiles_per_wave;
  float rope_base, norm_eps;
  // Row strides (elements).  Forward: the source is the latent (n_lat), q / k / v are dense.  Backward: the source
  // is the gradient entering the convolutions (e_q + e_kv wide), q / k destinations are column ranges of d_lat,
  // the value role reads d_v (e_kv) and writes the value columns of d_lat.
  int src_stride, q_stride, k_stride, vsrc_stride, vdst_stride;
  // qk-mean weights of the other stream: a q head adds mean_q_other * (k row of its group), a k head adds
  // mean_k_other * (each q row of its group).  Forward 1/2 and 1/(2R); the adjoint swaps them.
  float mean_q_other, mean_k_other;
  // Key-head workgroups come first in the grid and take tiles_per_wave_k tiles per wavefront (a key-head tile
  // costs more: its qk-mean adds the rows of all R query heads of the group); `tiles_per_wave` is the query heads'.
  int n_k_blocks, tiles_per_wave_k;
};

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float lo_f(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_f(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ---------------------------------------------------------------------------
// set-up: folded filters Wc [h][o][d][i] (bf16) and the two RoPE tables
//   ropeA [t_hi][i]            float2 (cos, sin) of t_hi * 128 * theta_i
//   ropeB [i / 4][t_lo][i % 4] float2 (cos, sin) of t_lo * theta_i
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prologue_setup_kernel(FusedArgs a, int D, const bf16_t *__restrict__ w0,
                                                            const bf16_t *__restrict__ w1, bf16_t *__restrict__ wc,
                                                            float2 *__restrict__ ropeA, float2 *__restrict__ ropeB,
                                                            int n_fold_blocks, int n_thi, int transposed, int DH) {
  const int NH = a.Hq + a.Hk;
  if ((int)blockIdx.x < n_fold_blocks) {
    const long long id = (long long)blockIdx.x * 256 + threadIdx.x;  // (h, o, i)
    if (id >= (long long)NH * DH * DH) return;
    const int i = (int)(id % DH), o = (int)((id / DH) % DH), h = (int)(id / (DH * DH));
    const int ch = h * DH + i;  // packed q|k channel: q heads first, then k heads
    const int ks = (a.flags & CCA_CONV_SEQ) ? a.k_seq : 1, kc = (a.flags & CCA_CONV_CH) ? a.k_ch : 1;
    for (int d = 0; d < D; ++d) {
      float acc = 0.f;
      for (int j = 0; j < kc; ++j) {
        const int jj = d - j;
        if (jj < 0 || jj >= ks) continue;
        const float f0 = (a.flags & CCA_CONV_SEQ) ? bf16_to_f32(w0[(long long)ch * ks + jj]) : 1.f;
        acc = fmaf(bf16_to_f32(w1[(((long long)h * DH + o) * DH + i) * kc + j]), f0, acc);
      }
      // the adjoint convolution contracts over the output channel: filter stored [h][i][d][o]
      if (transposed) wc[(((long long)h * DH + i) * D + d) * DH + o] = f32_to_bf16(acc);
      else wc[(((long long)h * DH + o) * D + d) * DH + i] = f32_to_bf16(acc);
    }
    return;
  }
  const int id = ((int)blockIdx.x - n_fold_blocks) * 256 + threadIdx.x;
  const int nA = n_thi * (DH / 2), nB = (DH / 2) * 128;
  if (id < nA) {
    const int i = id % (DH / 2), thi = id / (DH / 2);
    const double theta = pow((double)a.rope_base, -2.0 * (double)i / (double)DH);
    double sn, cs;
    sincos((double)thi * 128.0 * theta, &sn, &cs);
    ropeA[id] = make_float2((float)cs, (float)sn);
  } else if (id < nA + nB) {
    const int k = id - nA;
    const int i = k / 128, tlo = k % 128;
    const double theta = pow((double)a.rope_base, -2.0 * (double)i / (double)DH);
    double sn, cs;
    sincos((double)tlo * theta, &sn, &cs);
    ropeB[((i >> 2) * 128 + tlo) * 4 + (i & 3)] = make_float2((float)cs, (float)sn);
  }
}

// ---------------------------------------------------------------------------
// main kernel: one workgroup = one head x (256 * tiles per wavefront) tokens, 8 wavefronts x 32-token tiles.
// BWD = false: the forward prologue.  BWD = true: its adjoint from the gradient d3 of the conv2 output to
// d_lat: the same contraction with the transposed filter and the taps reaching FORWARD in time (token t reads
// rows t .. t+D-1, zero past the end of its sequence), the qk-mean adjoint through the same identity MFMAs, no
// norm / RoPE (those are undone by a pointwise kernel before), and the value role running the shift backwards.
// ---------------------------------------------------------------------------
// DH = d_h (64 or 128): KK fragments of 16 input channels, NTL tiles of 32 output channels, CPR 16-byte chunks per
// tap of a filter row.
template <int DH, int D, bool BWD>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void prologue_fused_kernel(
    FusedArgs a, const bf16_t *__restrict__ lat, const bf16_t *__restrict__ vsrc, const u32x4 *__restrict__ wc,
    const float2 *__restrict__ ropeA, const float2 *__restrict__ ropeB, const float *__restrict__ temp,
    bf16_t *__restrict__ q, bf16_t *__restrict__ k, bf16_t *__restrict__ v, float *__restrict__ rnorm) {
  constexpr int KK = DH / 16, NTL = DH / 32, CPR = DH / 8;
  constexpr int WROW = D * CPR;  // 16-byte chunks per filter row (one output channel)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4 *sW = reinterpret_cast<u32x4 *>(smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;

  if ((int)blockIdx.x >= a.n_conv_blocks) {
    // ---- value-shift role: v[t] = [vc[t] | vp[t-1]], 16 bytes per thread, whole rows per wavefront
    const int cpr = a.e_kv / 8;  // chunks per row
    const long long total = a.rows * cpr;
    const long long first = ((long long)blockIdx.x - a.n_conv_blocks) * (NT * 4);
    for (int it = 0; it < 4; ++it) {
      const long long id = first + it * NT + tid;
      if (id >= total) break;
      const long long row = id / cpr;
      const int ch = (int)(id % cpr) * 8;
      const int t = (int)(row % a.T);
      u32x4 val = {0, 0, 0, 0};
      const bool shifted = (a.flags & CCA_V_SHIFT) && ch >= a.v_half;
      // forward: the shifted half comes from token t-1; adjoint: its gradient goes back to token t, read at t+1
      const bool live = !shifted || (BWD ? t + 1 < a.T : t > 0);
      if (live) val = *reinterpret_cast<const u32x4 *>(vsrc + (row + (shifted ? (BWD ? 1 : -1) : 0)) * a.vsrc_stride + ch);
      *reinterpret_cast<u32x4 *>(v + row * a.vdst_stride + ch) = val;
    }
    return;
  }

  const int NH = a.Hq + a.Hk;
  const bool is_q = (int)blockIdx.x >= a.n_k_blocks;
  const int bid = is_q ? (int)blockIdx.x - a.n_k_blocks : (int)blockIdx.x;
  const int head = is_q ? bid % a.Hq : a.Hq + bid % a.Hk;
  const int tiles_per_wave = is_q ? a.tiles_per_wave : a.tiles_per_wave_k;
  const long long row_begin = (long long)(bid / (is_q ? a.Hq : a.Hk)) * (256 * tiles_per_wave);
  const int g = is_q ? head / a.R : head - a.Hq;
  const int ch0 = is_q ? head * DH : a.e_q + g * DH;

  // ---- filter of this head -> LDS, chunk-swizzled by output channel
  {
    const u32x4 *src = wc + (long long)head * DH * WROW;
#pragma unroll 4
    for (int id = tid; id < DH * WROW; id += NT) {
      const int o = id / WROW, c = id % WROW;
      sW[o * WROW + ((c & ~(CPR - 1)) | ((c ^ o) & (CPR - 1)))] = src[id];
    }
  }
  __syncthreads();  // the only workgroup-wide synchronisation
  const float beta = (!is_q && (a.flags & CCA_KEY_TEMP)) ? expf(temp[g]) : 1.f;
  bf16_t *dst = is_q ? q + head * DH : k + g * DH;
  const int dst_stride = is_q ? a.q_stride : a.k_stride;

  // ---- qk-mean through the matrix core: m = c * I * u adds c times a latent row, already in the
  // accumulator layout, with no extra loads or conversions.  Fragment j of c*I for output tile nt pairs with
  // operand fragment kk = 2*nt + j of the source row; lane (l32, half) is non-zero in fragment l32 >> 4 when
  // (l32 >> 3) & 1 == half, element l32 & 7.
  const bool mean = a.flags & CCA_QK_MEAN;
  // The weight of the other stream, 1/2 or 1/(2R), is an exact mean in the qk-mean equation.  As a single bf16
  // it is exact only for R a power of two, so it is fed as the sum of two bf16 numbers, w = hi + lo (the MFMA forms
  // bf16 products exactly and adds in fp32, so hi*u + lo*u carries w to 2^-17 relative); the second pass is skipped
  // when lo is zero.
  // c * I as fragments: lane (l32, half) holds c in ONE half-word of fragment j = l32 >> 4 (when (l32 >> 3) & 1 == half:
  // element l32 & 7) and zeros elsewhere, so one mask per fragment is kept and c is and-ed in where it is used.
  const float w_other = is_q ? a.mean_q_other : a.mean_k_other;
  const bf16_t w_other_hi = f32_to_bf16(w_other);
  const bf16_t w_other_lo = f32_to_bf16(w_other - bf16_to_f32(w_other_hi));
  const bool grp_lo = (w_other_lo & 0x7fffu) != 0;  // uniform over the workgroup
  u32x4 id_sel[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const bool on = ((l32 >> 4) == j) && (((l32 >> 3) & 1) == half);
    const int e = l32 & 7;
    id_sel[j] = u32x4{0, 0, 0, 0};
    if (on) id_sel[j][e >> 1] = 0xffffu << ((e & 1) * 16);
  }
  auto identity_frag = [&](bf16_t c, int j) {
    const uint32_t cc = (uint32_t)c | ((uint32_t)c << 16);
    const u32x4 w = {id_sel[j].x & cc, id_sel[j].y & cc, id_sel[j].z & cc, id_sel[j].w & cc};
    return __builtin_bit_cast(bf16x8, w);
  };

  for (int tt = 0; tt < tiles_per_wave; ++tt) {
    const long long trow0 = row_begin + (tt * 8 + wave) * 32;
    if (trow0 >= a.rows) break;  // wave-uniform; nothing below synchronises across wavefronts
    const long long row = trow0 + l32;
    const long long rowc = row < a.rows ? row : a.rows - 1;
    const int tpos = (int)(rowc % a.T);
    // Taps outside the token's sequence contribute zeros.  Only the first (adjoint: last) tile of a sequence
    // has such taps: everywhere else the loads are unconditional and all in flight together.
    const bool any_pad = __any(BWD ? tpos + D - 1 >= a.T : tpos < D - 1) != 0;

    // ---- operands: source rows of tokens t-D+1 .. t (adjoint: t .. t+D-1) of this head.  The taps of a tile are
    //      the same 32 rows shifted by a token, so the rows are fetched ONCE, whole (16 bytes per lane, 64 / CPR rows
    //      per load instruction: every cache line touched is used in full), parked in this wavefront's staging rows
    //      in LDS (chunk c of row r at position c ^ (r mod CPR)) and read from there as MFMA fragments, tap by tap.
    //      Fetched as fragments straight from memory, each tap cost 8 load instructions that touch 32 rows with 32
    //      bytes each; the vector memory pipeline works per cache line touched (timing without the D-1 earlier taps'
    //      loads: 56 -> 46 us).  The D-1 rows before the tile (adjoint: after it) are handled below (`halo`).
    constexpr int RPI = 64 / CPR, NLD = 32 / RPI, ROWB = DH * 2;
    unsigned char *const stg = smem + (size_t)DH * WROW * 16 + wave * (32 * ROWB);
    // Addresses of the whole-row transfers: a wave-uniform pointer to the tile's first row plus a 32-bit offset per
    // lane (row it * RPI + lane / CPR of the tile, clamped to the last row of the tensor on a ragged last tile).
    const int rows_left = (int)(a.rows - trow0 < 32 ? a.rows - trow0 : 32);  // >= 1
    auto stage_rows = [&](const bf16_t *tile_src, int stride) {  // rows of `tile_src` -> staging rows (swizzled)
      u32x4 rreg[NLD];
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        const int rr = it * RPI + lane / CPR, p = lane % CPR, c = p ^ (rr & (CPR - 1));
        const int rs = rr < rows_left ? rr : rows_left - 1;
        rreg[it] = *reinterpret_cast<const u32x4 *>(tile_src + rs * stride + c * 8);
      }
#pragma unroll
      for (int it = 0; it < NLD; ++it) {
        const int rr = it * RPI + lane / CPR, p = lane % CPR;
        *reinterpret_cast<u32x4 *>(stg + rr * ROWB + p * 16) = rreg[it];
      }
    };
    stage_rows(lat + trow0 * a.src_stride + ch0, a.src_stride);
    // The D-1 rows before the tile (adjoint: after it), which the first (last) D-1 tokens' taps reach: fetched whole as
    // well, one 16-byte chunk per lane - halo row j, chunk c in lane j * CPR + c - and handed to the lane that needs a
    // fragment of them by a lane gather (4 registers instead of a set of fragments in every lane).
    u32x4 halo = {0, 0, 0, 0};
    if (D > 1 && lane < (D - 1) * CPR) {
      const long long lo = -trow0, hi = a.rows - 1 - trow0;  // clamped in bounds; a clamped row is zeroed below:
      int hrel = BWD ? 32 + lane / CPR : lane / CPR - (D - 1);  // it lies outside the token's sequence
      hrel = hrel < lo ? (int)lo : (hrel > hi ? (int)hi : hrel);
      const bf16_t *tile_src = lat + trow0 * a.src_stride + ch0;  // wave-uniform
      halo = *reinterpret_cast<const u32x4 *>(tile_src + hrel * a.src_stride + (lane % CPR) * 8);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // LDS handles a wavefront's accesses in order
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // fragment kk of tap `back` for this lane's token: row l32 -+ back of the tile, or the halo row
    auto row_frag = [&](auto back_c, int kk, int l32v) {
      constexpr int back = decltype(back_c)::value;
      const int r = BWD ? l32v + back : l32v - back;
      const bool inside = BWD ? r < 32 : r >= 0;
      const int rc = inside ? r : l32v;  // the lanes that take the halo read their own row and drop it
      u32x4 raw = *reinterpret_cast<const u32x4 *>(stg + rc * ROWB + (((2 * kk + half) ^ (rc & (CPR - 1))) * 16));
      if constexpr (back > 0) {
        // halo row of this lane's tap: index r + (D-1) (adjoint: r - 32); its chunk 2 kk + half sits in lane
        // index * CPR + chunk (the index is clamped for the lanes that do not take the halo)
        int hj = BWD ? r - 32 : r + (D - 1);
        hj = hj < 0 ? 0 : (hj > D - 2 ? D - 2 : hj);
        const int src = (hj * CPR + 2 * kk + half) * 4;
        u32x4 h;
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)halo[e]);
        if (!inside) raw = h;
      }
      return __builtin_bit_cast(bf16x8, raw);
    };

    // ---- y1^T = Wc * [u(t-D+1) .. u(t)]^T
    f32x16 acc[NTL];
#pragma unroll
    for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nt][r] = 0.f;
    bf16x8 uf[KK];  // the fragments of the tap being multiplied; after the loop: the token's own row (back = 0)
    auto conv_tap = [&](auto d_c) {
      constexpr int d = decltype(d_c)::value;
      constexpr int back = D - 1 - d;
      // the LDS addresses of a tap (one per k-step: the swizzle is an XOR, not an offset) are formed here, per tap
      // and tile, from a copy of the lane index the compiler cannot see through: hoisted out of the tile loop as
      // loop invariants they cost 8 registers per tap for the whole kernel
      int l32v = l32;
      asm volatile("" : "+v"(l32v));
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) uf[kk] = row_frag(std::integral_constant<int, back>{}, kk, l32v);
      if (back > 0 && any_pad) {  // wave-uniform and rare: a tap that reaches outside the token's sequence is zero
        const bool outside = BWD ? tpos + back >= a.T : tpos < back;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
          if (outside) uf[kk] = __builtin_bit_cast(bf16x8, u32x4{0, 0, 0, 0});
      }
      // the tap's KK * NTL products in a fixed order, the filter fragment of product i + PFW requested before product
      // i is issued (left to the compiler each fragment is read, waited for and consumed one at a time, and the LDS
      // latency of every read is paid in full)
      constexpr int NPW = KK * NTL, PFW = 4;
      bf16x8 wfr[PFW + 1];  // ring: fragment i lives in slot i mod (PFW + 1)
      auto fetch_w = [&](int i) {
        const int kk = i / NTL, nt = i % NTL;
        const int o = nt * 32 + l32v;
        const int c = d * CPR + kk * 2 + half;
        wfr[i % (PFW + 1)] = __builtin_bit_cast(bf16x8, sW[o * WROW + ((c & ~(CPR - 1)) | ((c ^ o) & (CPR - 1)))]);
      };
#pragma unroll
      for (int i = 0; i < PFW; ++i) fetch_w(i);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < NPW; ++i) {
        if (i + PFW < NPW) fetch_w(i + PFW);
        acc[i % NTL] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfr[i % (PFW + 1)], uf[i / NTL], acc[i % NTL], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      __builtin_amdgcn_sched_barrier(0);  // one tap's fragments at a time: the next tap's reads stay behind this one's products
    };
    conv_tap(std::integral_constant<int, 0>{});
    if constexpr (D > 1) conv_tap(std::integral_constant<int, 1>{});
    if constexpr (D > 2) conv_tap(std::integral_constant<int, 2>{});

    // ---- qk-mean.  q head: + (q0 + k0[g]) / 2.  k head: + (mean_r q0[gR + r] + k0) / 2.
    //      Adjoint: q head + d3_q / 2 + d3_k[g] / (2R);  k head: + (sum_r d3_q[gR + r] + d3_k) / 2.
    if (mean) {
#pragma unroll
      for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(identity_frag(f32_to_bf16(0.5f), j), uf[2 * nt + j], acc[nt], 0, 0, 0);
      const int nsrc = is_q ? 1 : a.R;
      for (int sidx = 0; sidx < nsrc; ++sidx) {
        // the other stream's rows of this tile travel like the tile's own: whole rows -> staging rows -> fragments
        const int col = is_q ? a.e_q + g * DH : (g * a.R + sidx) * DH;
        __builtin_amdgcn_sched_barrier(0);  // not hoisted above the products before: their registers are needed there
        stage_rows(lat + trow0 * a.src_stride + col, a.src_stride);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        int l32v = l32;
        asm volatile("" : "+v"(l32v));
        bf16x8 mf[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
          mf[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(
                                                  stg + l32v * ROWB + (((2 * kk + half) ^ (l32v & (CPR - 1))) * 16)));
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(identity_frag(w_other_hi, j), mf[2 * nt + j], acc[nt], 0, 0, 0);
        if (grp_lo) {
#pragma unroll
          for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
            for (int j = 0; j < 2; ++j)
              acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(identity_frag(w_other_lo, j), mf[2 * nt + j], acc[nt], 0, 0, 0);
        }
      }
    }

    __builtin_amdgcn_sched_barrier(0);
    // ---- per token: norm, temperature, RoPE.  Lane (l32, half) holds channels
    //      o = 32*nt + 8*rg + 4*half + e of token l32 in acc[nt][4*rg + e].
    if (!BWD && (a.flags & CCA_QK_NORM)) {
      float ssq = 0.f;
#pragma unroll
      for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) ssq = fmaf(acc[nt][r], acc[nt][r], ssq);
      ssq += __shfl_xor(ssq, 32);
      const float mul = sqrtf((float)DH) / sqrtf(ssq + a.norm_eps) * beta;
#pragma unroll
      for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[nt][r] *= mul;
      if (rnorm && half == 0 && row < a.rows) rnorm[row * NH + head] = mul;
    } else if (!BWD && rnorm && half == 0 && row < a.rows) {
      rnorm[row * NH + head] = 1.f;
    }
    __builtin_amdgcn_sched_barrier(0);
    if (!BWD && (a.flags & CCA_ROPE)) {
      const int thi = tpos >> 7, tlo = tpos & 127;
#pragma unroll
      for (int nt = 0; nt < NTL / 2; ++nt)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          const int i0 = nt * 32 + rg * 8 + half * 4;  // 4 consecutive pair indices
          const f32x4 *pa = reinterpret_cast<const f32x4 *>(ropeA + thi * (DH / 2) + i0);
          const f32x4 *pb = reinterpret_cast<const f32x4 *>(ropeB + ((i0 >> 2) * 128 + tlo) * 4);
          const f32x4 a01 = pa[0], a23 = pa[1], b01 = pb[0], b23 = pb[1];
          const float ca[4] = {a01.x, a01.z, a23.x, a23.z}, sa[4] = {a01.y, a01.w, a23.y, a23.w};
          const float cb[4] = {b01.x, b01.z, b23.x, b23.z}, sb[4] = {b01.y, b01.w, b23.y, b23.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float cs = ca[e] * cb[e] - sa[e] * sb[e];
            const float sn = sa[e] * cb[e] + ca[e] * sb[e];
            const float x1 = acc[nt][rg * 4 + e], x2 = acc[nt + NTL / 2][rg * 4 + e];
            acc[nt][rg * 4 + e] = x1 * cs - x2 * sn;
            acc[nt + NTL / 2][rg * 4 + e] = x2 * cs + x1 * sn;
          }
        }
    }
    // ---- round once to bf16 and store.  In the accumulator layout a lane holds 4 consecutive channels (8 bytes) of
    //      one token per (nt, rg): stored from there, a wavefront's store instruction would touch 32 rows with 16
    //      bytes each, and the vector memory pipeline works per cache line touched (timing the kernel with 1 such
    //      store per lane instead of 16: 56 -> 45 us).  So the tile is transposed through this wavefront's private
    //      staging rows in LDS (16-byte chunk c of row r at position c ^ (r mod CPR): conflict-free both ways) and
    //      leaves as whole rows, 16 bytes per lane, 64 / CPR rows per instruction.
    {
      int l32w = l32;  // as for the tap reads: the 16 swizzled positions are formed here, not kept across tiles
      asm volatile("" : "+v"(l32w));
#pragma unroll
      for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          u32x2 w;
          w.x = pack2(acc[nt][rg * 4 + 0], acc[nt][rg * 4 + 1]);
          w.y = pack2(acc[nt][rg * 4 + 2], acc[nt][rg * 4 + 3]);
          const int pos = (nt * 4 + rg) ^ (l32w & (CPR - 1));
          *reinterpret_cast<u32x2 *>(stg + l32w * (DH * 2) + pos * 16 + half * 8) = w;
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // LDS handles a wavefront's accesses in order
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      bf16_t *const tile_dst = dst + trow0 * dst_stride;
#pragma unroll
      for (int it = 0; it < 32 / RPI; ++it) {
        const int rr = it * RPI + lane / CPR, p = lane % CPR, c = p ^ (rr & (CPR - 1));
        const u32x4 val = *reinterpret_cast<const u32x4 *>(stg + rr * (DH * 2) + p * 16);
        if (rr < rows_left) *reinterpret_cast<u32x4 *>(tile_dst + rr * dst_stride + c * 8) = val;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // the next tile's writes come after these reads
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// ---------------------------------------------------------------------------
// The same prologue for d_h = 256, where one head's folded filter (D x 256 x 256 bf16 = 128 KB per tap) cannot
// stay in LDS: the filter is STREAMED through a double-buffered LDS slab of 256 outputs x 64 input channels
// (one slab per tap and quarter of the head width), all 8 wavefronts of a workgroup walking the slabs in step.
// Workgroup = one head x 256 tokens, wavefront = 32 tokens x all 256 outputs (8 accumulator tiles).  The token
// operands of a slab (4 fragments) come straight from the latent rows as in the kernel above; the qk-mean, norm,
// temperature, RoPE and the value role are the same code.  BWD = true is the adjoint, as for the kernel above:
// transposed filter, taps reaching forward in time, the value shift running backwards; the host passes only the
// qk-mean and value-shift flags, so the norm and RoPE steps are skipped.
// ---------------------------------------------------------------------------
template <int DH, int D, bool BWD>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void prologue_stream_kernel(
    FusedArgs a, const bf16_t *__restrict__ lat, const bf16_t *__restrict__ vsrc, const u32x4 *__restrict__ wc,
    const float2 *__restrict__ ropeA, const float2 *__restrict__ ropeB, const float *__restrict__ temp,
    bf16_t *__restrict__ q, bf16_t *__restrict__ k, bf16_t *__restrict__ v, float *__restrict__ rnorm) {
  constexpr int NTL = DH / 32, CPR = DH / 8;
  constexpr int WROW = D * CPR;              // 16-byte chunks per filter row (one output channel) in memory
  constexpr int KC = 64, KCK = KC / 16;      // input channels per slab, MFMA k-steps per slab
  constexpr int NCH = DH / KC, NSLAB = D * NCH;
  constexpr int SROW = KC * 2 + 16;          // padded slab row in LDS: conflict-free 16-byte reads down a column of rows
  constexpr int SLAB = DH * SROW;
  constexpr int W_PER_THREAD = DH * (KC / 8) / NT;  // 16-byte chunks of a slab per thread
  __shared__ __attribute__((aligned(16))) unsigned char sW[2 * SLAB];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;

  if ((int)blockIdx.x >= a.n_conv_blocks) {
    // ---- value-shift role (as in prologue_fused_kernel)
    const int cpr = a.e_kv / 8;
    const long long total = a.rows * cpr;
    const long long first = ((long long)blockIdx.x - a.n_conv_blocks) * (NT * 4);
    for (int it = 0; it < 4; ++it) {
      const long long id = first + it * NT + tid;
      if (id >= total) break;
      const long long row = id / cpr;
      const int ch = (int)(id % cpr) * 8;
      const int t = (int)(row % a.T);
      u32x4 val = {0, 0, 0, 0};
      const bool shifted = (a.flags & CCA_V_SHIFT) && ch >= a.v_half;
      const bool live = !shifted || (BWD ? t + 1 < a.T : t > 0);
      if (live) val = *reinterpret_cast<const u32x4 *>(vsrc + (row + (shifted ? (BWD ? 1 : -1) : 0)) * a.vsrc_stride + ch);
      *reinterpret_cast<u32x4 *>(v + row * a.vdst_stride + ch) = val;
    }
    return;
  }

  const int NH = a.Hq + a.Hk;
  const bool is_q = (int)blockIdx.x >= a.n_k_blocks;
  const int bid = is_q ? (int)blockIdx.x - a.n_k_blocks : (int)blockIdx.x;
  const int head = is_q ? bid % a.Hq : a.Hq + bid % a.Hk;
  const long long row_begin = (long long)(bid / (is_q ? a.Hq : a.Hk)) * 256;
  const int g = is_q ? head / a.R : head - a.Hq;
  const int ch0 = is_q ? head * DH : a.e_q + g * DH;
  const float beta = (!is_q && (a.flags & CCA_KEY_TEMP)) ? expf(temp[g]) : 1.f;
  bf16_t *dst = is_q ? q + head * DH : k + g * DH;
  const int dst_stride = is_q ? a.q_stride : a.k_stride;

  // qk-mean weights as identity fragments (see prologue_fused_kernel); the other stream's are made after the
  // convolution, when fewer registers are live
  const bool mean = a.flags & CCA_QK_MEAN;
  auto identity_frag = [&](bf16_t wbits, int j) {
    const bool on = ((l32 >> 4) == j) && (((l32 >> 3) & 1) == half);
    u32x4 w = {0, 0, 0, 0};
    const int e = l32 & 7;
    if (on) w[e >> 1] = (uint32_t)wbits << ((e & 1) * 16);
    return __builtin_bit_cast(bf16x8, w);
  };
  bf16x8 id_half[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) id_half[j] = identity_frag(f32_to_bf16(0.5f), j);

  // this wavefront's 32 tokens (a wavefront past the end keeps walking the slabs: it stages filter chunks too)
  const long long trow0 = row_begin + wave * 32;
  const long long row = trow0 + l32;
  const long long rowc = row < a.rows ? row : a.rows - 1;
  const int tpos = (int)(rowc % a.T);

  // slab s = (tap d = s / NCH, channel quarter c = s % NCH): rows o = 0..DH-1, bytes [c*128, c*128+128) of tap d
  const u32x4 *wsrc = wc + (long long)head * DH * WROW;
  u32x4 wreg[W_PER_THREAD];
  auto load_slab = [&](int s_) {
    const int d = s_ / NCH, c = s_ % NCH;
#pragma unroll
    for (int i = 0; i < W_PER_THREAD; ++i) {
      const int id = tid + i * NT, o = id / (KC / 8), cc = id % (KC / 8);
      wreg[i] = wsrc[o * WROW + d * CPR + c * (KC / 8) + cc];
    }
  };
  auto store_slab = [&](int buf) {
#pragma unroll
    for (int i = 0; i < W_PER_THREAD; ++i) {
      const int id = tid + i * NT, o = id / (KC / 8), cc = id % (KC / 8);
      *reinterpret_cast<u32x4 *>(sW + buf * SLAB + o * SROW + cc * 16) = wreg[i];
    }
  };

  f32x16 acc[NTL];
#pragma unroll
  for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nt][r] = 0.f;

  load_slab(0);
  store_slab(0);
#pragma unroll  // tap and channel quarter must be compile-time: they pick accumulator tiles
  for (int s_ = 0; s_ < NSLAB; ++s_) {
    const int d = s_ / NCH, c = s_ % NCH;
    if (s_ + 1 < NSLAB) load_slab(s_ + 1);
    // token operands of this slab: row t - (D-1-d) (adjoint: t + (D-1-d)), channels c*64 .. c*64+63; rows outside
    // the token's sequence are zero
    const int back = D - 1 - d;
    bf16x8 uf[KCK];
    {
      long long src_row = BWD ? rowc + back : rowc - back;
      src_row = src_row < 0 ? 0 : (src_row > a.rows - 1 ? a.rows - 1 : src_row);
      const bf16_t *p = lat + src_row * a.src_stride + ch0 + c * KC + half * 8;
#pragma unroll
      for (int kk = 0; kk < KCK; ++kk) {
        u32x4 raw = *reinterpret_cast<const u32x4 *>(p + kk * 16);
        if (BWD ? tpos + back >= a.T : tpos < back) raw = u32x4{0, 0, 0, 0};
        uf[kk] = __builtin_bit_cast(bf16x8, raw);
      }
    }
    __syncthreads();  // slab s_ is in LDS (stored one step ago); the other buffer is no longer read
    if (s_ + 1 < NSLAB) store_slab((s_ + 1) & 1);
    const unsigned char *sw = sW + (s_ & 1) * SLAB + l32 * SROW + half * 16;
#pragma unroll
    for (int kk = 0; kk < KCK; ++kk)
#pragma unroll
      for (int nt = 0; nt < NTL; ++nt) {
        const bf16x8 wf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(sw + nt * 32 * SROW + kk * 32));
        acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, uf[kk], acc[nt], 0, 0, 0);
      }
    if (mean && d == D - 1) {  // own stream of the qk-mean: + 1/2 of the token's own latent row
#pragma unroll
      for (int kk = 0; kk < KCK; ++kk) {
        // channels c*64 + kk*16 .. +15 lie in output tile 2c + kk/2, half kk % 2 of it
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt)
          if (nt == 2 * c + kk / 2) acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(id_half[kk & 1], uf[kk], acc[nt], 0, 0, 0);
      }
    }
  }

  // ---- other stream of the qk-mean, a quarter of the head width at a time
  if (mean) {
    const float w_other = is_q ? a.mean_q_other : a.mean_k_other;
    const bf16_t w_other_hi = f32_to_bf16(w_other);
    const bf16_t w_other_lo = f32_to_bf16(w_other - bf16_to_f32(w_other_hi));
    const bool grp_lo = (w_other_lo & 0x7fffu) != 0;  // uniform over the workgroup
    bf16x8 id_grp[2], id_grp_lo[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      id_grp[j] = identity_frag(w_other_hi, j);
      id_grp_lo[j] = identity_frag(w_other_lo, j);
    }
    const int nsrc = is_q ? 1 : a.R;
    for (int sidx = 0; sidx < nsrc; ++sidx) {
      const int col = is_q ? a.e_q + g * DH : (g * a.R + sidx) * DH;
      const bf16_t *p = lat + rowc * a.src_stride + col + half * 8;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        bf16x8 mf[KCK];
#pragma unroll
        for (int kk = 0; kk < KCK; ++kk)
          mf[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(p + c * KC + kk * 16));
#pragma unroll
        for (int kk = 0; kk < KCK; ++kk) {
          acc[2 * c + kk / 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(id_grp[kk & 1], mf[kk], acc[2 * c + kk / 2], 0, 0, 0);
          if (grp_lo)
            acc[2 * c + kk / 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(id_grp_lo[kk & 1], mf[kk], acc[2 * c + kk / 2], 0, 0, 0);
        }
      }
    }
  }

  // ---- per token: norm, temperature, RoPE, store (lane (l32, half): channels 32*nt + 8*rg + 4*half + e)
  if (a.flags & CCA_QK_NORM) {
    float ssq = 0.f;
#pragma unroll
    for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) ssq = fmaf(acc[nt][r], acc[nt][r], ssq);
    ssq += __shfl_xor(ssq, 32);
    const float mul = sqrtf((float)DH) / sqrtf(ssq + a.norm_eps) * beta;
#pragma unroll
    for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nt][r] *= mul;
    if (rnorm && half == 0 && row < a.rows) rnorm[row * NH + head] = mul;
  } else if (rnorm && half == 0 && row < a.rows) {
    rnorm[row * NH + head] = 1.f;
  }
  if (a.flags & CCA_ROPE) {
    const int thi = tpos >> 7, tlo = tpos & 127;
#pragma unroll
    for (int nt = 0; nt < NTL / 2; ++nt)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int i0 = nt * 32 + rg * 8 + half * 4;
        const f32x4 *pa = reinterpret_cast<const f32x4 *>(ropeA + thi * (DH / 2) + i0);
        const f32x4 *pb = reinterpret_cast<const f32x4 *>(ropeB + ((i0 >> 2) * 128 + tlo) * 4);
        const f32x4 a01 = pa[0], a23 = pa[1], b01 = pb[0], b23 = pb[1];
        const float ca[4] = {a01.x, a01.z, a23.x, a23.z}, sa[4] = {a01.y, a01.w, a23.y, a23.w};
        const float cb[4] = {b01.x, b01.z, b23.x, b23.z}, sb[4] = {b01.y, b01.w, b23.y, b23.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float cs = ca[e] * cb[e] - sa[e] * sb[e];
          const float sn = sa[e] * cb[e] + ca[e] * sb[e];
          const float x1 = acc[nt][rg * 4 + e], x2 = acc[nt + NTL / 2][rg * 4 + e];
          acc[nt][rg * 4 + e] = x1 * cs - x2 * sn;
          acc[nt + NTL / 2][rg * 4 + e] = x2 * cs + x1 * sn;
        }
      }
  }
  if (row < a.rows) {
    bf16_t *orow = dst + row * dst_stride;
#pragma unroll
    for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        u32x2 w;
        w.x = pack2(acc[nt][rg * 4 + 0], acc[nt][rg * 4 + 1]);
        w.y = pack2(acc[nt][rg * 4 + 2], acc[nt][rg * 4 + 3]);
        *reinterpret_cast<u32x2 *>(orow + nt * 32 + rg * 8 + half * 4) = w;
      }
  }
}

// ---------------------------------------------------------------------------
// No transform selected (plain MHA / GQA, Sec. 2.1): q, k, v are column slices
// of the latent rows; only the optional value-shift moves data in time.
// 16 bytes per thread, storage-type agnostic (`es` = bytes per element).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void split_copy_kernel(const unsigned char *__restrict__ lat,
                                                        unsigned char *__restrict__ q, unsigned char *__restrict__ k,
                                                        unsigned char *__restrict__ v, long long rows, int T, int e_q,
                                                        int e_kv, int v_half, int es, int v_shift) {
  const int n_lat = e_q + 2 * e_kv;
  const int cpr = n_lat * es / 16;  // chunks per latent row
  const long long total = rows * cpr;
  for (long long id = (long long)blockIdx.x * 256 + threadIdx.x; id < total; id += (long long)gridDim.x * 256) {
    const long long row = id / cpr;
    const int col = (int)(id % cpr) * (16 / es);  // first element of the chunk
    const int t = (int)(row % T);
    u32x4 val = {0, 0, 0, 0};
    const bool shifted = v_shift && col >= e_q + e_kv + v_half;
    if (!shifted || t > 0)
      val = *reinterpret_cast<const u32x4 *>(lat + ((row - (shifted ? 1 : 0)) * n_lat + col) * es);
    unsigned char *dstp;
    if (col < e_q) dstp = q + (row * e_q + col) * es;
    else if (col < e_q + e_kv) dstp = k + (row * e_kv + (col - e_q)) * es;
    else dstp = v + (row * e_kv + (col - e_q - e_kv)) * es;
    *reinterpret_cast<u32x4 *>(dstp) = val;
  }
}

// Adjoint of split_copy_kernel: d_lat is d_q | d_k | d_v side by side, the shifted half of d_v read one token later
// (zero for the last token of a sequence).
__global__ __launch_bounds__(256) void split_copy_bwd_kernel(const unsigned char *__restrict__ dq,
                                                            const unsigned char *__restrict__ dk,
                                                            const unsigned char *__restrict__ dv,
                                                            unsigned char *__restrict__ d_lat, long long rows, int T,
                                                            int e_q, int e_kv, int v_half, int es, int v_shift) {
  const int n_lat = e_q + 2 * e_kv;
  const int cpr = n_lat * es / 16;
  const long long total = rows * cpr;
  for (long long id = (long long)blockIdx.x * 256 + threadIdx.x; id < total; id += (long long)gridDim.x * 256) {
    const long long row = id / cpr;
    const int col = (int)(id % cpr) * (16 / es);
    const int t = (int)(row % T);
    u32x4 val = {0, 0, 0, 0};
    if (col < e_q) {
      val = *reinterpret_cast<const u32x4 *>(dq + (row * e_q + col) * es);
    } else if (col < e_q + e_kv) {
      val = *reinterpret_cast<const u32x4 *>(dk + (row * e_kv + (col - e_q)) * es);
    } else {
      const int cc = col - e_q - e_kv;
      const bool shifted = v_shift && cc >= v_half;
      if (!shifted || t + 1 < T) val = *reinterpret_cast<const u32x4 *>(dv + ((row + (shifted ? 1 : 0)) * e_kv + cc) * es);
    }
    *reinterpret_cast<u32x4 *>(d_lat + (row * n_lat + col) * es) = val;
  }
}

template <int DH, int D, bool BWD>
hipError_t launch_main(const FusedArgs &a, const void *lat, const void *vsrc, const void *wc, const float2 *ropeA,
                       const float2 *ropeB, const float *temp, void *q, void *k, void *v, float *rnorm, int grid,
                       hipStream_t s) {
  // the head's filter, then 32 staging rows of d_h channels per wavefront (160 KB at d_h = 128 with 3 taps)
  constexpr size_t smem = (size_t)DH * D * (DH / 8) * 16 + (size_t)(NT / 64) * 32 * DH * 2;
  static_assert(smem <= 160 * 1024, "filter and staging rows must fit the LDS");
  if (hipError_t e = raise_lds_limit<prologue_fused_kernel<DH, D, BWD>>(smem); e != hipSuccess) return e;
  prologue_fused_kernel<DH, D, BWD><<<grid, NT, smem, s>>>(a, (const bf16_t *)lat, (const bf16_t *)vsrc, (const u32x4 *)wc,
                                                       ropeA, ropeB, temp, (bf16_t *)q, (bf16_t *)k, (bf16_t *)v, rnorm);
  return hipGetLastError();
}

// Tokens per workgroup: each workgroup first loads its head's filter (about one tile's worth of time), and one
// workgroup fits per CU, so minimise rounds-on-256-CUs x (1 + tiles per wavefront).  Returns the grid size.
int plan_grid(const Dims &d, FusedArgs &a) {
  // One workgroup = one head x 256 * tiles tokens.  Cost of a workgroup in units of a query-head tile: about one
  // for loading its filter, one per query-head tile, 1 + 0.11 R per key-head tile when the qk-mean is on (measured
  // 1.43 at R = 4).  The slowest workgroup of a round sets the round's length, so key heads take fewer tiles.
  const double ck = (a.flags & CCA_QK_MEAN) ? 1.0 + 0.11 * d.R : 1.0;
  double best_cost = -1.0;
  long long best_q = 0, best_k = 0;
  for (int tq = 1; tq <= MAX_TILES_PER_WAVE; ++tq)
    for (int tk = 1; tk <= MAX_TILES_PER_WAVE; ++tk) {
      const long long nq = d.Hq * ((d.rows() + 256 * tq - 1) / (256 * tq));
      const long long nk = d.Hk * ((d.rows() + 256 * tk - 1) / (256 * tk));
      const double slowest = 1.0 + (tq > ck * tk ? (double)tq : ck * tk);
      const double cost = (double)((nq + nk + 255) / 256) * slowest;
      if (best_cost < 0 || cost < best_cost - 1e-9) {
        best_cost = cost;
        a.tiles_per_wave = tq;
        a.tiles_per_wave_k = tk;
        best_q = nq;
        best_k = nk;
      }
    }
  a.n_k_blocks = (int)best_k;
  a.n_conv_blocks = (int)(best_q + best_k);
  const long long v_chunks = d.rows() * (d.e_kv / 8);
  const int v_blocks = (int)((v_chunks + NT * 4 - 1) / (NT * 4));
  return a.n_conv_blocks + v_blocks;
}

struct FusedScratch {
  bf16_t *wc;
  float2 *ropeA, *ropeB;
  size_t bytes;
};
FusedScratch carve(const Dims &d, void *scratch, int D) {
  const int NH = d.Hq + d.Hk, n_thi = (d.T + 127) / 128, DH = d.dh;
  const size_t wc_bytes = ((size_t)NH * DH * D * DH * 2 + 255) / 256 * 256;
  const size_t ra_bytes = ((size_t)n_thi * (DH / 2) * 8 + 255) / 256 * 256;
  const size_t rb_bytes = (size_t)(DH / 2) * 128 * 8;
  char *base = static_cast<char *>(scratch);
  return FusedScratch{reinterpret_cast<bf16_t *>(base), reinterpret_cast<float2 *>(base + wc_bytes),
                      reinterpret_cast<float2 *>(base + wc_bytes + ra_bytes), wc_bytes + ra_bytes + rb_bytes};
}

hipError_t run_setup(const Dims &d, const FusedArgs &a, const cca_weights &w, const FusedScratch &fs, int D,
                     bool transposed, hipStream_t s) {
  const int NH = d.Hq + d.Hk, n_thi = (d.T + 127) / 128, DH = d.dh;
  const int n_fold = (NH * DH * DH + 255) / 256;
  const int n_rope = (n_thi * (DH / 2) + (DH / 2) * 128 + 255) / 256;
  prologue_setup_kernel<<<n_fold + n_rope, 256, 0, s>>>(a, D, (const bf16_t *)w.w_conv_seq, (const bf16_t *)w.w_conv_ch,
                                                        fs.wc, fs.ropeA, fs.ropeB, n_fold, n_thi, transposed ? 1 : 0, DH);
  return hipGetLastError();
}

int taps(const Dims &d) { return ((d.flags & CCA_CONV_SEQ) ? d.k_seq : 1) + d.k_ch - 1; }

}  // namespace

bool prologue_is_split_copy(const Dims &d) {
  const uint32_t transforms = CCA_CONV_SEQ | CCA_CONV_CH | CCA_QK_MEAN | CCA_QK_NORM | CCA_KEY_TEMP | CCA_ROPE;
  const int per16 = d.bf16 ? 8 : 4;
  return !(d.flags & transforms) && d.e_q % per16 == 0 && d.e_kv % per16 == 0 && d.v_half % per16 == 0;
}

__global__ void fill_f32_kernel(float *p, long long n, float val) {
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x)
    p[i] = val;
}

hipError_t prologue_split_copy(const Dims &d, const void *lat, void *q, void *k, void *v, float *rnorm, hipStream_t s) {
  if (rnorm) fill_f32_kernel<<<256, 256, 0, s>>>(rnorm, d.rows() * (d.Hq + d.Hk), 1.f);
  const long long total = d.rows() * ((long long)d.n_lat * d.esize() / 16);
  const int grid = (int)((total + 255) / 256 < 256 * 64 ? (total + 255) / 256 : 256 * 64);
  split_copy_kernel<<<grid, 256, 0, s>>>((const unsigned char *)lat, (unsigned char *)q, (unsigned char *)k,
                                         (unsigned char *)v, d.rows(), d.T, d.e_q, d.e_kv, d.v_half, (int)d.esize(),
                                         (d.flags & CCA_V_SHIFT) ? 1 : 0);
  return hipGetLastError();
}

hipError_t prologue_split_copy_bwd(const Dims &d, const void *d_q, const void *d_k, const void *d_v, void *d_lat,
                                   hipStream_t s) {
  const long long total = d.rows() * ((long long)d.n_lat * d.esize() / 16);
  const int grid = (int)((total + 255) / 256 < 256 * 64 ? (total + 255) / 256 : 256 * 64);
  split_copy_bwd_kernel<<<grid, 256, 0, s>>>((const unsigned char *)d_q, (const unsigned char *)d_k,
                                             (const unsigned char *)d_v, (unsigned char *)d_lat, d.rows(), d.T, d.e_q,
                                             d.e_kv, d.v_half, (int)d.esize(), (d.flags & CCA_V_SHIFT) ? 1 : 0);
  return hipGetLastError();
}

bool prologue_fused_supported(const Dims &d) {
  return d.bf16 && (d.dh == 256 || d.dh == 128 || d.dh == 64) && (d.flags & CCA_CONV_CH) && !(d.flags & CCA_ROPE_INTERLEAVED) && taps(d) <= 3 &&
         d.v_half % 8 == 0;
}

size_t prologue_fused_scratch_bytes(const Dims &d) {
  if (!prologue_fused_supported(d)) return 0;
  return carve(d, nullptr, taps(d)).bytes;
}

static FusedArgs forward_args(const Dims &d) {
  return FusedArgs{d.T, d.Hq, d.Hk, d.R, d.e_q, d.e_kv, d.n_lat, d.v_half, d.k_seq, d.k_ch, d.rows(), d.flags, 0, 1,
                   d.rope_base, d.norm_eps, d.n_lat, d.e_q, d.e_kv, d.n_lat, d.e_kv, 0.5f, 0.5f / (float)d.R};
}

hipError_t prologue_fused_prepare(const Dims &d, const cca_weights &w, void *scratch, hipStream_t s) {
  const int D = taps(d);
  return run_setup(d, forward_args(d), w, carve(d, scratch, D), D, false, s);
}

template <int D, bool BWD>
static hipError_t launch_stream(const Dims &d, FusedArgs a, const float *temp, const void *lat, const void *vsrc,
                                const FusedScratch &fs, void *q, void *k, void *v, float *rnorm, hipStream_t s) {
  // one 256-token block per workgroup for every head, key heads first (the kernel's block map)
  const long long blocks = (d.rows() + 255) / 256;
  a.tiles_per_wave = a.tiles_per_wave_k = 1;
  a.n_k_blocks = (int)(d.Hk * blocks);
  a.n_conv_blocks = (int)((d.Hq + d.Hk) * blocks);
  const long long v_chunks = d.rows() * (d.e_kv / 8);
  const int grid = a.n_conv_blocks + (int)((v_chunks + NT * 4 - 1) / (NT * 4));
  prologue_stream_kernel<256, D, BWD><<<grid, NT, 0, s>>>(a, (const bf16_t *)lat, (const bf16_t *)vsrc,
                                                        (const u32x4 *)fs.wc, fs.ropeA, fs.ropeB, temp, (bf16_t *)q,
                                                        (bf16_t *)k, (bf16_t *)v, rnorm);
  return hipGetLastError();
}

hipError_t prologue_fused_run(const Dims &d, const cca_weights &w, const void *lat, void *q, void *k, void *v,
                              float *rnorm, const void *scratch, hipStream_t s) {
  const int D = taps(d);
  FusedArgs a = forward_args(d);
  const FusedScratch fs = carve(d, const_cast<void *>(scratch), D);
  const bf16_t *vsrc = (const bf16_t *)lat + d.e_q + d.e_kv;
  if (d.dh == 256) {
    switch (D) {
      case 1: return launch_stream<1, false>(d, a, w.temp, lat, vsrc, fs, q, k, v, rnorm, s);
      case 2: return launch_stream<2, false>(d, a, w.temp, lat, vsrc, fs, q, k, v, rnorm, s);
      default: return launch_stream<3, false>(d, a, w.temp, lat, vsrc, fs, q, k, v, rnorm, s);
    }
  }
  const int grid = plan_grid(d, a);
#define LAUNCH_DH(D_, B_) (d.dh == 64 ? launch_main<64, D_, B_> : launch_main<128, D_, B_>)
  switch (D) {
    case 1: return LAUNCH_DH(1, false)(a, lat, vsrc, fs.wc, fs.ropeA, fs.ropeB, w.temp, q, k, v, rnorm, grid, s);
    case 2: return LAUNCH_DH(2, false)(a, lat, vsrc, fs.wc, fs.ropeA, fs.ropeB, w.temp, q, k, v, rnorm, grid, s);
    default: return LAUNCH_DH(3, false)(a, lat, vsrc, fs.wc, fs.ropeA, fs.ropeB, w.temp, q, k, v, rnorm, grid, s);
  }
}

hipError_t prologue_fused_bf16(const Dims &d, const cca_weights &w, const void *lat, void *q, void *k, void *v,
                               float *rnorm, void *scratch, hipStream_t s) {
  hipError_t e = prologue_fused_prepare(d, w, scratch, s);
  if (e != hipSuccess) return e;
  return prologue_fused_run(d, w, lat, q, k, v, rnorm, scratch, s);
}

// ---- adjoint: d3 (B*T, e_q+e_kv), d_v -> d_lat.  `scratch` as for the forward; the RoPE tables it leaves
// behind are the ones the pointwise backward kernel reads, so this runs its set-up first (see fused_bwd_setup).
hipError_t prologue_fused_bwd_setup(const Dims &d, const cca_weights &w, void *scratch, const float2 **ropeA,
                                    const float2 **ropeB, hipStream_t s) {
  const int D = taps(d);
  FusedArgs a{d.T, d.Hq, d.Hk, d.R, d.e_q, d.e_kv, d.n_lat, d.v_half, d.k_seq, d.k_ch, d.rows(), d.flags, 0, 1,
              d.rope_base, 0.f, 0, 0, 0, 0, 0, 0.f, 0.f};
  const FusedScratch fs = carve(d, scratch, D);
  *ropeA = fs.ropeA;
  *ropeB = fs.ropeB;
  return run_setup(d, a, w, fs, D, true, s);
}

hipError_t prologue_fused_bwd_dlat(const Dims &d, const void *d3, const void *d_v, void *d_lat, void *scratch,
                                   hipStream_t s) {
  const int D = taps(d);
  const int ld = d.e_q + d.e_kv;
  // only the qk-mean and value-shift flags matter to the adjoint kernel
  FusedArgs a{d.T, d.Hq, d.Hk, d.R, d.e_q, d.e_kv, d.n_lat, d.v_half, d.k_seq, d.k_ch, d.rows(),
              d.flags & (CCA_QK_MEAN | CCA_V_SHIFT), 0, 1, d.rope_base, 0.f, ld, d.n_lat, d.n_lat, d.e_kv, d.n_lat,
              0.5f / (float)d.R, 0.5f};
  const FusedScratch fs = carve(d, scratch, D);
  bf16_t *dl = (bf16_t *)d_lat;
  if (d.dh == 256) {
    switch (D) {
      case 1: return launch_stream<1, true>(d, a, nullptr, d3, d_v, fs, dl, dl + d.e_q, dl + ld, nullptr, s);
      case 2: return launch_stream<2, true>(d, a, nullptr, d3, d_v, fs, dl, dl + d.e_q, dl + ld, nullptr, s);
      default: return launch_stream<3, true>(d, a, nullptr, d3, d_v, fs, dl, dl + d.e_q, dl + ld, nullptr, s);
    }
  }
  const int grid = plan_grid(d, a);
  switch (D) {
    case 1: return LAUNCH_DH(1, true)(a, d3, d_v, fs.wc, fs.ropeA, fs.ropeB, nullptr, dl, dl + d.e_q, dl + ld, nullptr, grid, s);
    case 2: return LAUNCH_DH(2, true)(a, d3, d_v, fs.wc, fs.ropeA, fs.ropeB, nullptr, dl, dl + d.e_q, dl + ld, nullptr, grid, s);
    default: return LAUNCH_DH(3, true)(a, d3, d_v, fs.wc, fs.ropeA, fs.ropeB, nullptr, dl, dl + d.e_q, dl + ld, nullptr, grid, s);
  }
}

}  // namespace cca
