// Backward of the fused latent-space prologue for gfx950, bf16 storage,
// d_h = 256, 128 or 64 (adjoint of the convolution, qk-mean and value-shift equations
// and of the first two lines of the final equation block of Sec. 2.2; the
// paper states these steps forward only).
//
//   1. pointwise kernel: undoes RoPE (a rotation: rotate back) and the norm /
//      temperature step on the gradients of q and k.  With y = x * mul,
//      mul = sqrt(d_h) beta / |x|:   dx = mul * (dy - y <y,dy> / (d_h beta^2)),
//      where y is the saved q / k (the dot product is invariant under RoPE, so
//      it is taken on the rotated vectors), mul the saved norm factor.  Result
//      d3 (B*T, e_q + e_kv) bf16 = gradient of the conv2 output; also
//      <dk,k> per (token, KV head), whose sum over tokens is d temp.
//   2. d_lat: the forward kernel run as its own adjoint (cca_prologue.hip).
//   3. filter gradients: dWc[h,o,d,i] = sum_t d3[t,h,o] * u[t-(D-1-d),h,i] for
//      the folded filter Wc of width D = k_seq + k_ch - 1, as an MFMA
//      contraction over tokens (both operands fetched from row-major LDS tiles
//      with the transposing read), split over chunks of tokens into fp32
//      partial sums that a second kernel adds in a fixed order; Wc is bilinear
//      in (w0, w1), so d w1[h,o,i,j] = sum_jj dWc[h,o,j+jj,i] w0[c,jj] and
//      d w0[c,jj] = sum_o sum_j dWc[h,o,j+jj,i] w1[h,o,i,j].
// No atomics anywhere: a repeated call gives the same bits.
#include "cca_internal.h"

namespace cca {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16 lds_v4i16;

// from cca_prologue.hip
bool prologue_fused_supported(const Dims &d);
size_t prologue_fused_scratch_bytes(const Dims &d);
hipError_t prologue_fused_bwd_setup(const Dims &d, const cca_weights &w, void *scratch, const float2 **ropeA,
                                    const float2 **ropeB, hipStream_t s);
hipError_t prologue_fused_bwd_dlat(const Dims &d, const void *d3, const void *d_v, void *d_lat, void *scratch,
                                   hipStream_t s);

namespace {

// ROW below = DH * 2 + 16: padded LDS row of one token, bytes

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

struct PointArgs {
  int T, Hq, Hk, e_q, e_kv;
  long long rows;
  uint32_t flags;
};

// ---------------------------------------------------------------------------
// 1. pointwise: d_h / 8 lanes per (token, head); lane j holds channels 4j..4j+3 and d_h/2 + 4j .. + 3, so the
//    rotate-half partner sits in the same lane and the row dot product is a butterfly over those lanes.
// ---------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void pro_bwd_point_kernel(PointArgs a, const bf16_t *__restrict__ q,
                                                           const bf16_t *__restrict__ k,
                                                           const float *__restrict__ rnorm,
                                                           const float *__restrict__ temp,
                                                           const bf16_t *__restrict__ dq, const bf16_t *__restrict__ dk,
                                                           const float2 *__restrict__ ropeA,
                                                           const float2 *__restrict__ ropeB, bf16_t *__restrict__ d3,
                                                           float *__restrict__ rowdot) {
  const int NH = a.Hq + a.Hk;
  constexpr int LPI = DH / 8, HALF = DH / 2;  // lanes per item
  const long long item = (long long)blockIdx.x * (256 / LPI) + threadIdx.x / LPI;  // row * NH + head
  const int j = threadIdx.x % LPI;
  const bool live = item < a.rows * NH;
  const long long it = live ? item : 0;
  const long long row = it / NH;
  const int head = (int)(it % NH);
  const int tpos = (int)(row % a.T);
  const bool is_q = head < a.Hq;
  const int g = head - a.Hq;
  const bf16_t *y5 = is_q ? q + (row * a.Hq + head) * DH : k + (row * a.Hk + g) * DH;
  const bf16_t *dy5 = is_q ? dq + (row * a.Hq + head) * DH : dk + (row * a.Hk + g) * DH;
  const u32x2 ya = *reinterpret_cast<const u32x2 *>(y5 + 4 * j), yb = *reinterpret_cast<const u32x2 *>(y5 + HALF + 4 * j);
  const u32x2 da = *reinterpret_cast<const u32x2 *>(dy5 + 4 * j), db = *reinterpret_cast<const u32x2 *>(dy5 + HALF + 4 * j);
  float y[8] = {bf_lo(ya.x), bf_hi(ya.x), bf_lo(ya.y), bf_hi(ya.y), bf_lo(yb.x), bf_hi(yb.x), bf_lo(yb.y), bf_hi(yb.y)};
  float dy[8] = {bf_lo(da.x), bf_hi(da.x), bf_lo(da.y), bf_hi(da.y), bf_lo(db.x), bf_hi(db.x), bf_lo(db.y), bf_hi(db.y)};
  float dot = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) dot = fmaf(y[e], dy[e], dot);
#pragma unroll
  for (int off = LPI / 2; off > 0; off >>= 1) dot += __shfl_xor(dot, off);
  float mul = 1.f, c = 0.f;
  if (a.flags & CCA_QK_NORM) {
    mul = rnorm[row * NH + head];
    const float beta2 = (!is_q && (a.flags & CCA_KEY_TEMP)) ? expf(2.f * temp[g]) : 1.f;
    c = dot / ((float)DH * beta2);
  }
  if (live && !is_q && rowdot && j == 0) rowdot[row * a.Hk + g] = dot;
  float r[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = dy[e] - y[e] * c;
  if (a.flags & CCA_ROPE) {
    const int thi = tpos >> 7, tlo = tpos & 127;
    const f32x4 *pa = reinterpret_cast<const f32x4 *>(ropeA + thi * (DH / 2) + 4 * j);
    const f32x4 *pb = reinterpret_cast<const f32x4 *>(ropeB + (j * 128 + tlo) * 4);
    const f32x4 a01 = pa[0], a23 = pa[1], b01 = pb[0], b23 = pb[1];
    const float ca[4] = {a01.x, a01.z, a23.x, a23.z}, sa[4] = {a01.y, a01.w, a23.y, a23.w};
    const float cb[4] = {b01.x, b01.z, b23.x, b23.z}, sb[4] = {b01.y, b01.w, b23.y, b23.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float cs = ca[e] * cb[e] - sa[e] * sb[e];
      const float sn = sa[e] * cb[e] + ca[e] * sb[e];
      // forward: (x1, x2) -> (x1 c - x2 s, x2 c + x1 s); the adjoint rotates back
      const float g1 = r[e], g2 = r[e + 4];
      r[e] = g1 * cs + g2 * sn;
      r[e + 4] = g2 * cs - g1 * sn;
    }
  }
  if (live) {
    bf16_t *dst = d3 + row * (a.e_q + a.e_kv) + (is_q ? head * DH : a.e_q + g * DH);
    u32x2 lo, hi;
    lo.x = pack2(r[0] * mul, r[1] * mul);
    lo.y = pack2(r[2] * mul, r[3] * mul);
    hi.x = pack2(r[4] * mul, r[5] * mul);
    hi.y = pack2(r[6] * mul, r[7] * mul);
    *reinterpret_cast<u32x2 *>(dst + 4 * j) = lo;
    *reinterpret_cast<u32x2 *>(dst + HALF + 4 * j) = hi;
  }
}

// out[col] = sum over rows of src[row*ncol + col]; one workgroup per column, fixed summation order
__global__ __launch_bounds__(256) void column_sum_f32_kernel(const float *__restrict__ src, long long rows, int ncol,
                                                            float *__restrict__ out) {
  __shared__ float red[256];
  const int col = blockIdx.x, tid = threadIdx.x;
  float acc = 0.f;
  long long r = tid;
  for (; r + 7 * 256 < rows; r += 8 * 256) {  // 8 loads in flight, added in row order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[(r + u * 256) * ncol + col];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  for (; r < rows; r += 256) acc += src[r * ncol + col];
  red[tid] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) red[tid] += red[tid + s];
    __syncthreads();
  }
  if (tid == 0) out[col] = red[0];
}

// ---------------------------------------------------------------------------
// 3. folded-filter gradient, partial sums per chunk of tokens.
//    Workgroup = (head, chunk of `chunk` tokens of one sequence[, slice of the output channels at d_h = 256]);
//    wavefront w owns OX output-channel tiles starting at OX*(w&1) and IX input-channel tiles starting at
//    IX*(w>>1), for all D taps (OX = d_h / 64 and IX = 1 up to d_h = 128).
// ---------------------------------------------------------------------------
// MFMA operand fragment of the TRANSPOSE of a row-major LDS tile: lane (c = lane & 31, half) receives
// tile[r0 + 4*half + {0..3}][c0 + c] and tile[r0 + 8 + 4*half + {0..3}][c0 + c].  `base` already holds the
// per-lane part  (4*half + ((lane & 15) >> 2)) * ROW + (((lane >> 4) & 1) * 16 + 4 * (lane & 3)) * 2.
template <int ROW>
__device__ __forceinline__ bf16x8 tr_frag(const unsigned char *base, int r0, int c0) {
  const unsigned char *p = base + r0 * ROW + c0 * 2;
  const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16 *)p);
  const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16 *)(p + 8 * ROW));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

constexpr int DW_BT = 64;  // tokens per LDS tile

// Output slices per head and threads per workgroup: at d_h <= 128 one workgroup of d_h * 4 threads owns all of a head's
// d_h x D x d_h sums; at d_h = 256 they would not fit its registers, so 512 threads own a slice of 128 (D <= 2) or 64
// (D = 3) output channels (blockIdx.y) and each such workgroup re-reads the token rows of all 256 input channels.
constexpr int dwc_slices(int DH, int D) { return DH <= 128 ? 1 : (D <= 2 ? 2 : 4); }
constexpr int dwc_threads(int DH) { return DH <= 128 ? DH * 4 : 512; }

template <int DH, int D>
__global__ __launch_bounds__(dwc_threads(DH)) void pro_bwd_dwc_kernel(const bf16_t *__restrict__ d3,
                                                                      const bf16_t *__restrict__ lat,
                                                                      float *__restrict__ part, int T, int Hq, int Hk,
                                                                      int e_q, int e_kv, int n_lat, int chunk,
                                                                      int chunks_per_seq) {
  constexpr int OS = dwc_slices(DH, D), DHO = DH / OS, DW_NT = dwc_threads(DH), NW = DW_NT / 64;
  // LDS rows of the gradient tile (this slice's output channels) and of the token tile (all input channels); the
  // 64-byte pad keeps the transposing reads conflict-free
  constexpr int ROWY = DHO * 2 + 64, ROWU = DH * 2 + 64, CPWY = DHO / 8, CPWU = DH / 8;
  constexpr int OX = DHO / 64, IX = (DH / 32) / (NW / 2);  // output / input channel tiles per wavefront
  static_assert(OX >= 1 && IX >= 1 && OX * 2 * 32 == DHO && IX * (NW / 2) * 32 == DH, "wavefront tiling");
  constexpr int UROWS = DW_BT + D - 1;
  constexpr int DY_TILE = DW_BT * ROWY, U_TILE = UROWS * ROWU;
  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * (DY_TILE + U_TILE)];
  unsigned char *const sDy = smem, *const sU = smem + 2 * DY_TILE;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int NH = Hq + Hk;
  const int head = blockIdx.x % NH, cid = blockIdx.x / NH;  // cid = b * chunks_per_seq + chunk index
  const int o_base = (int)blockIdx.y * DHO;                 // first output channel of this slice
  const int b = cid / chunks_per_seq, t_begin = (cid % chunks_per_seq) * chunk;
  const int t_end = min(T, t_begin + chunk);
  const int ch0 = head < Hq ? head * DH : e_q + (head - Hq) * DH;
  const int ld3 = e_q + e_kv;
  const bf16_t *const d3b = d3 + (long long)b * T * ld3 + ch0 + o_base;
  const bf16_t *const ub = lat + (long long)b * T * n_lat + ch0;

  constexpr int DY_CHUNKS = DW_BT * CPWY, U_CHUNKS = UROWS * CPWU;  // 16-byte chunks per tile
  constexpr int DY_PER = DY_CHUNKS / DW_NT, U_PER = (U_CHUNKS + DW_NT - 1) / DW_NT;
  static_assert(DY_CHUNKS % DW_NT == 0, "gradient tile must divide over the threads");
  u32x4 rdy[DY_PER], ru[U_PER];
  auto load_tile = [&](int t0) {
#pragma unroll
    for (int i = 0; i < DY_PER; ++i) {
      const int id = tid + i * DW_NT, r = id / CPWY, c = id % CPWY;
      const int t = t0 + r;
      u32x4 val = {0, 0, 0, 0};
      if (t < t_end) val = *reinterpret_cast<const u32x4 *>(d3b + (long long)t * ld3 + c * 8);
      rdy[i] = val;
    }
#pragma unroll
    for (int i = 0; i < U_PER; ++i) {
      const int id = tid + i * DW_NT, r = id / CPWU, c = id % CPWU;
      const int t = t0 - (D - 1) + r;  // row r of the tile holds token t0 - (D-1) + r
      u32x4 val = {0, 0, 0, 0};
      if (id < U_CHUNKS && t >= 0 && t < t_end) val = *reinterpret_cast<const u32x4 *>(ub + (long long)t * n_lat + c * 8);
      ru[i] = val;
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < DY_PER; ++i) {
      const int id = tid + i * DW_NT, r = id / CPWY, c = id % CPWY;
      *reinterpret_cast<u32x4 *>(sDy + buf * DY_TILE + r * ROWY + c * 16) = rdy[i];
    }
#pragma unroll
    for (int i = 0; i < U_PER; ++i) {
      const int id = tid + i * DW_NT, r = id / CPWU, c = id % CPWU;
      if (id < U_CHUNKS) *reinterpret_cast<u32x4 *>(sU + buf * U_TILE + r * ROWU + c * 16) = ru[i];
    }
  };

  const uint32_t tr_row = (uint32_t)(4 * half + ((lane & 15) >> 2)), tr_col = (((lane >> 4) & 1) * 16 + 4 * (lane & 3)) * 2;
  const uint32_t tr_off_y = tr_row * ROWY + tr_col, tr_off_u = tr_row * ROWU + tr_col;
  const int o_tile0 = OX * (wave & 1), i_tile0 = IX * (wave >> 1);

  f32x16 acc[OX][IX][D];
#pragma unroll
  for (int x = 0; x < OX; ++x)
#pragma unroll
    for (int y = 0; y < IX; ++y)
#pragma unroll
      for (int d = 0; d < D; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[x][y][d][r] = 0.f;

  const int ntiles = (t_end - t_begin + DW_BT - 1) / DW_BT;
  load_tile(t_begin);
  store_tile(0);
  if (ntiles > 1) load_tile(t_begin + DW_BT);
  __syncthreads();
  for (int it = 0; it < ntiles; ++it) {
    const int buf = it & 1;
    if (it + 1 < ntiles) store_tile(buf ^ 1);
    if (it + 2 < ntiles) load_tile(t_begin + (it + 2) * DW_BT);
    const unsigned char *dyp = sDy + buf * DY_TILE + tr_off_y, *up = sU + buf * U_TILE + tr_off_u;
#pragma unroll
    for (int kk = 0; kk < DW_BT / 16; ++kk) {
      bf16x8 fo[OX], fu[IX][D];
#pragma unroll
      for (int x = 0; x < OX; ++x) fo[x] = tr_frag<ROWY>(dyp, kk * 16, (o_tile0 + x) * 32);
#pragma unroll
      for (int y = 0; y < IX; ++y)
#pragma unroll
        for (int d = 0; d < D; ++d) fu[y][d] = tr_frag<ROWU>(up, kk * 16 + d, (i_tile0 + y) * 32);  // token t - (D-1-d)
#pragma unroll
      for (int x = 0; x < OX; ++x)
#pragma unroll
        for (int y = 0; y < IX; ++y)
#pragma unroll
          for (int d = 0; d < D; ++d)
            acc[x][y][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo[x], fu[y][d], acc[x][y][d], 0, 0, 0);
    }
    __syncthreads();
  }
  // acc[x][y][d][r]: o = o_base + (o_tile0 + x)*32 + 8*(r/4) + 4*half + r%4,  i = (i_tile0 + y)*32 + l32
  float *out = part + (long long)blockIdx.x * DH * D * DH;  // [o][d][i] of (cid, head); blockIdx.x = cid*NH + head
#pragma unroll
  for (int x = 0; x < OX; ++x)
#pragma unroll
    for (int y = 0; y < IX; ++y)
#pragma unroll
      for (int d = 0; d < D; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int o = o_base + (o_tile0 + x) * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
          out[(o * D + d) * DH + (i_tile0 + y) * 32 + l32] = acc[x][y][d][r];
        }
}

// dwc[h][o][d][i] = sum over chunks (fixed order); then d w1[h,o,i,j] = sum_jj dwc[h,o,j+jj,i] * w0[c(h,i),jj]
__global__ __launch_bounds__(256) void pro_bwd_unfold_w1_kernel(const float *__restrict__ part, int n_chunks, int NH,
                                                               int D, int ks, int kc, int use_w0,
                                                               const bf16_t *__restrict__ w0, float *__restrict__ dwc,
                                                               bf16_t *__restrict__ dw1, int DH) {
  const long long id = (long long)blockIdx.x * 256 + threadIdx.x;  // (h*DH + o)*DH + i
  if (id >= (long long)NH * DH * DH) return;
  const int i = (int)(id % DH), o = (int)((id / DH) % DH), h = (int)(id / (DH * DH));
  float sum[4] = {0.f, 0.f, 0.f, 0.f};  // D <= 3 on this path
  const long long cstride = (long long)NH * DH * D * DH;
  const float *p0 = part + ((long long)h * DH + o) * D * DH + i;
  int c = 0;
  for (; c + 8 <= n_chunks; c += 8) {  // 8 chunks of loads in flight, added in chunk order
    float v[8][3];
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int d = 0; d < 3; ++d) v[u][d] = d < D ? p0[(c + u) * cstride + d * DH] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int d = 0; d < 3; ++d) sum[d] += v[u][d];
  }
  for (; c < n_chunks; ++c)
    for (int d = 0; d < D; ++d) sum[d] += p0[c * cstride + d * DH];
  for (int d = 0; d < D; ++d) dwc[(((long long)h * DH + o) * D + d) * DH + i] = sum[d];
  if (!dw1) return;
  for (int j = 0; j < kc; ++j) {
    float acc = 0.f;
    for (int jj = 0; jj < ks; ++jj) {
      const float f0 = use_w0 ? bf16_to_f32(w0[(long long)(h * DH + i) * ks + jj]) : 1.f;
      acc = fmaf(sum[j + jj], f0, acc);
    }
    dw1[(((long long)h * DH + o) * DH + i) * kc + j] = f32_to_bf16(acc);
  }
}

// d w0[c(h,i), jj] = sum_o sum_j dwc[h,o,j+jj,i] * w1[h,o,i,j].  Workgroup = (head, 16 input channels): 8 groups of
// d_h / 8 output channels x 16 input channels; the 8 partial sums are added through LDS in a fixed order.
constexpr int W0_IW = 16;
template <int DH>
__global__ __launch_bounds__(W0_IW * 8) void pro_bwd_unfold_w0_kernel(const float *__restrict__ dwc, int D, int ks, int kc,
                                                                     const bf16_t *__restrict__ w1, bf16_t *__restrict__ dw0) {
  __shared__ float red[8][4][W0_IW];
  const int h = blockIdx.x, il = threadIdx.x % W0_IW, i = blockIdx.y * W0_IW + il, og = threadIdx.x / W0_IW;
  // D = ks + kc - 1 <= 3 on this path: every load of the d_h / 8 output channels is issued before the first use
  // (absent taps read as zero), so the thread waits for memory once instead of once per channel
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  float pv[DH / 8][3], wv[DH / 8][3];
#pragma unroll
  for (int x = 0; x < DH / 8; ++x) {
    const int o = og * (DH / 8) + x;
    const float *p = dwc + (((long long)h * DH + o) * D) * DH + i;
    const bf16_t *wp = w1 + (((long long)h * DH + o) * DH + i) * kc;
#pragma unroll
    for (int t = 0; t < 3; ++t) {
      pv[x][t] = t < D ? p[t * DH] : 0.f;
      wv[x][t] = t < kc ? bf16_to_f32(wp[t]) : 0.f;
    }
  }
#pragma unroll
  for (int x = 0; x < DH / 8; ++x)
#pragma unroll
    for (int j = 0; j < 3; ++j)
#pragma unroll
      for (int jj = 0; jj < 3; ++jj)
        if (j + jj < 3) acc[jj] = fmaf(pv[x][j + jj], wv[x][j], acc[jj]);  // j >= kc: wv = 0; j + jj >= D: pv = 0
  for (int jj = 0; jj < 4; ++jj) red[og][jj][il] = acc[jj];
  __syncthreads();
  if (og == 0)
    for (int jj = 0; jj < ks; ++jj) {
      float sum = 0.f;
      for (int x = 0; x < 8; ++x) sum += red[x][jj][il];
      dw0[(long long)(h * DH + i) * ks + jj] = f32_to_bf16(sum);
    }
}

int taps(const Dims &d) { return ((d.flags & CCA_CONV_SEQ) ? d.k_seq : 1) + d.k_ch - 1; }

// tokens per chunk of the filter-gradient kernel: the largest of 512..64 that still gives >= 256 workgroups
int dwc_chunk(const Dims &d) {
  const int NH = d.Hq + d.Hk, os = dwc_slices(d.dh, taps(d));
  for (int c = 512; c > 64; c >>= 1)
    if ((long long)d.B * ((d.T + c - 1) / c) * NH * os >= 256) return c;
  return 64;
}

struct BwdScratch {
  size_t fused, d3, rowdot, part, dwc, total;  // byte offsets
};
BwdScratch bwd_layout(const Dims &d) {
  BwdScratch L;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
  const int D = taps(d), NH = d.Hq + d.Hk, chunk = dwc_chunk(d), DH = d.dh;
  const size_t n_chunks = (size_t)d.B * ((d.T + chunk - 1) / chunk);
  L.fused = take(prologue_fused_scratch_bytes(d));
  L.d3 = take((size_t)d.rows() * (d.e_q + d.e_kv) * 2);
  L.rowdot = take((size_t)d.rows() * d.Hk * 4);
  L.part = take(n_chunks * NH * DH * D * DH * 4);
  L.dwc = take((size_t)NH * DH * D * DH * 4);
  L.total = off;
  return L;
}

}  // namespace

bool prologue_bwd_fused_supported(const Dims &d) { return prologue_fused_supported(d); }

size_t prologue_bwd_fused_scratch_bytes(const Dims &d) {
  return prologue_bwd_fused_supported(d) ? bwd_layout(d).total : 0;
}

template <int DH>
static hipError_t prologue_bwd_run(const Dims &d, const cca_weights &w, const void *lat, const void *q, const void *k,
                                   const float *rnorm, const void *d_q, const void *d_k, const void *d_v, void *d_lat,
                                   const cca_grads *gr, void *scratch, hipStream_t s) {
  const BwdScratch L = bwd_layout(d);
  char *base = static_cast<char *>(scratch);
  bf16_t *d3 = reinterpret_cast<bf16_t *>(base + L.d3);
  float *rowdot = reinterpret_cast<float *>(base + L.rowdot);
  float *part = reinterpret_cast<float *>(base + L.part);
  float *dwc = reinterpret_cast<float *>(base + L.dwc);
  const int D = taps(d), NH = d.Hq + d.Hk;

  const float2 *ropeA, *ropeB;
  hipError_t e = prologue_fused_bwd_setup(d, w, base + L.fused, &ropeA, &ropeB, s);
  if (e != hipSuccess) return e;

  const bool want_temp = (d.flags & CCA_KEY_TEMP) && gr && gr->temp;
  PointArgs pa{d.T, d.Hq, d.Hk, d.e_q, d.e_kv, d.rows(), d.flags};
  const long long items = d.rows() * NH;
  constexpr int IPB = 256 / (DH / 8);  // items per workgroup of the pointwise kernel
  pro_bwd_point_kernel<DH><<<(unsigned)((items + IPB - 1) / IPB), 256, 0, s>>>(pa, (const bf16_t *)q, (const bf16_t *)k, rnorm,
                                                                    w.temp, (const bf16_t *)d_q, (const bf16_t *)d_k,
                                                                    ropeA, ropeB, d3, want_temp ? rowdot : nullptr);
  if (want_temp) column_sum_f32_kernel<<<d.Hk, 256, 0, s>>>(rowdot, d.rows(), d.Hk, gr->temp);
  e = hipGetLastError();
  if (e != hipSuccess) return e;

  e = prologue_fused_bwd_dlat(d, d3, d_v, d_lat, base + L.fused, s);
  if (e != hipSuccess) return e;

  const bool want_w1 = gr && gr->w_conv_ch;  // CONV_CH is on whenever this path runs
  const bool want_w0 = (d.flags & CCA_CONV_SEQ) && gr && gr->w_conv_seq;
  if (!want_w1 && !want_w0) return hipSuccess;
  const int chunk = dwc_chunk(d), cps = (d.T + chunk - 1) / chunk, n_chunks = d.B * cps;
#define DWC(DD)                                                                                                     \
  pro_bwd_dwc_kernel<DH, DD><<<dim3(n_chunks * NH, dwc_slices(DH, DD)), dwc_threads(DH), 0, s>>>(                    \
      d3, (const bf16_t *)lat, part, d.T, d.Hq, d.Hk, d.e_q, d.e_kv, d.n_lat, chunk, cps)
  switch (D) {
    case 1: DWC(1); break;
    case 2: DWC(2); break;
    default: DWC(3); break;
  }
#undef DWC
  const int ks = (d.flags & CCA_CONV_SEQ) ? d.k_seq : 1;
  pro_bwd_unfold_w1_kernel<<<(NH * DH * DH + 255) / 256, 256, 0, s>>>(part, n_chunks, NH, D, ks, d.k_ch,
                                                                     (d.flags & CCA_CONV_SEQ) ? 1 : 0,
                                                                     (const bf16_t *)w.w_conv_seq, dwc,
                                                                     want_w1 ? (bf16_t *)gr->w_conv_ch : nullptr, DH);
  if (want_w0)
    pro_bwd_unfold_w0_kernel<DH><<<dim3(NH, DH / W0_IW), W0_IW * 8, 0, s>>>(dwc, D, ks, d.k_ch, (const bf16_t *)w.w_conv_ch,
                                               (bf16_t *)gr->w_conv_seq);
  return hipGetLastError();
}

hipError_t prologue_bwd_fused_bf16(const Dims &d, const cca_weights &w, const void *lat, const void *q, const void *k,
                                   const float *rnorm, const void *d_q, const void *d_k, const void *d_v, void *d_lat,
                                   const cca_grads *gr, void *scratch, hipStream_t s) {
  return d.dh == 64    ? prologue_bwd_run<64>(d, w, lat, q, k, rnorm, d_q, d_k, d_v, d_lat, gr, scratch, s)
         : d.dh == 128 ? prologue_bwd_run<128>(d, w, lat, q, k, rnorm, d_q, d_k, d_v, d_lat, gr, scratch, s)
                       : prologue_bwd_run<256>(d, w, lat, q, k, rnorm, d_q, d_k, d_v, d_lat, gr, scratch, s);
}

}  // namespace cca
