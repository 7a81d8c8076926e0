// bf16 GEMM on the gfx950 matrix cores for the down- and up-projection
// (Sec. 2.2: down-projection equation and last line of the final equation
// block):  C (M,N) = A (M,K) * Bt (N,K)^T, fp32 accumulation, bf16 output.
//
// Both operands are K-contiguous, so a lane's 8-element MFMA fragment is one
// 16-byte LDS read.  Workgroup tile 256 x BN x 64 with 8 wavefronts; LDS is
// double-buffered and XOR-swizzled per 16-byte chunk; K-slab k+1 travels HBM ->
// LDS directly (global_load_lds, no staging registers, no ds_write) while slab k
// is multiplied, its loads spread over the first two of the slab's four 16-wide
// MFMA steps so that the LDS writes trickle in between the fragment reads
// instead of arriving in one burst (the LDS write port, ~75 B/clk against ~230 B/clk for
// reads, is what this kernel feels first: without the stores it runs a third
// faster).  The MFMA is issued with the weight rows as its first operand,
// which leaves every lane with 4 consecutive output columns of one row, so
// the epilogue packs them to bf16, stages the tile in LDS and writes whole
// rows with 16-byte stores.
#include "cca_internal.h"

namespace cca {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int BM = 256, BK = 64;
constexpr int SPREAD = 2;  // k-steps of a slab over which the next slab's loads are issued (4 k-steps per slab)

// LDS position of the 16-byte chunk c (0..7) of row r in a [rows][64] bf16 tile
__device__ __forceinline__ int swz(int r, int c) { return r * 8 + (c ^ ((r & 7) ^ ((r >> 3) & 1))); }

// two floats -> one word of two bf16 (round to nearest even) with the hardware conversion instruction
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

template <int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(WAVES_M *WAVES_N * 64) void gemm_bf16_nt_kernel(const bf16_t *__restrict__ A,
                                                               const bf16_t *__restrict__ Bt,
                                                               bf16_t *__restrict__ C, long long M, int N, int K,
                                                               int tiles_n, int tiles_total) {
  constexpr int NTHREADS = WAVES_M * WAVES_N * 64;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wave tile
  constexpr int MI = WM / 32, NI = WN / 32;            // 32x32 MFMA tiles per wave
  static_assert(MI * 32 == WM && NI * 32 == WN, "wave tile must be a multiple of 32");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int STAGE = (BM + BN) * 8;  // 16-byte chunks per pipeline stage
  u32x4 *const sbase = reinterpret_cast<u32x4 *>(smem);

  // XCD-aware tile order: workgroup ids are dealt round-robin over the 8 XCDs,
  // so give each XCD a contiguous range of tiles; within it the N tiles of one
  // M block are adjacent and share the A panel in that XCD's L2.
  const int wg = blockIdx.x;
  const int per_xcd = (tiles_total + 7) / 8;
  const int tile = (wg % 8) * per_xcd + wg / 8;
  if (tile >= tiles_total) return;
  const long long m0 = (long long)(tile / tiles_n) * BM;
  const int n0 = (tile % tiles_n) * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int l32 = lane & 31, half = lane >> 5;

  // Direct global -> LDS loads: wave instruction i deposits 64 x 16 bytes at LDS chunks [i*64, i*64+64) of the
  // stage (A rows first, then B rows; 8 chunks per row), so lane L fetches the chunk that the XOR swizzle puts
  // at that position.  No staging registers, no ds_write.
  constexpr int N_INSTR = (BM + BN) * 8 / 64;
  constexpr int PER_WAVE = N_INSTR / (NTHREADS / 64);
  static_assert(N_INSTR % (NTHREADS / 64) == 0, "instructions must divide evenly over the wavefronts");
  const bf16_t *g_src[PER_WAVE];
#pragma unroll
  for (int u = 0; u < PER_WAVE; ++u) {
    const int i = wave + u * (NTHREADS / 64);
    const int pos = i * 64 + lane;            // chunk position inside the stage
    const bool isb = pos >= BM * 8;
    const int r = (isb ? pos - BM * 8 : pos) >> 3, cs = pos & 7;
    const int c = cs ^ ((r & 7) ^ ((r >> 3) & 1));  // inverse of swz(): the chunk stored at this position
    if (!isb) {
      long long gr = m0 + r;
      gr = gr < M ? gr : M - 1;
      g_src[u] = A + gr * K + c * 8;
    } else {
      int gr = n0 + r;
      gr = gr < N ? gr : N - 1;
      g_src[u] = Bt + (long long)gr * K + c * 8;
    }
  }
  typedef __attribute__((address_space(3))) void lds_void;
  typedef __attribute__((address_space(1))) void glb_void;
  auto issue_slab = [&](int k0, int buf) {
#pragma unroll
    for (int u = 0; u < PER_WAVE; ++u) {
      const int i = wave + u * (NTHREADS / 64);
      __builtin_amdgcn_global_load_lds((glb_void *)(g_src[u] + k0), (lds_void *)(sbase + buf * STAGE + i * 64), 16, 0, 0);
    }
  };

  f32x16 acc[NI][MI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[ni][mi][r] = 0.f;

  const int nk = K / BK;
  issue_slab(0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  // Within a slab the fragments of k-step kk+1 are requested before the MFMAs of k-step kk are issued (two register
  // sets): only the first k-step of a slab, right after the slab barrier, pays its LDS latency in the open.
  // Warm same-box A/B: the projections timed alone, back to back, are 2-5 % SLOWER this way (102 -> 104, 74 -> 78 us),
  // the forward pass they are part of is 0.8 % faster (0.668 -> 0.6625 ms, repeated in both orders): inside a pass
  // their operands come from further away than in a loop over the same GEMM.
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    bf16x8 fa[2][MI], fb[2][NI];
    auto read_frags = [&](int kk, int set) {
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int r = wm * WM + mi * 32 + l32;
        fa[set][mi] = __builtin_bit_cast(bf16x8, sbase[buf * STAGE + swz(r, kk * 2 + half)]);
      }
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        const int r = wn * WN + ni * 32 + l32;
        fb[set][ni] = __builtin_bit_cast(bf16x8, sbase[buf * STAGE + BM * 8 + swz(r, kk * 2 + half)]);
      }
    };
    read_frags(0, 0);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      // the loads of slab kt+1 are issued over the first SPREAD k-steps: not in one burst (the LDS write port), not
      // over all four either (the last quarter then has a fraction of a slab to land before the wait below).
      // Warm same-box A/B of the whole forward pass: spread over 4 / 3 / 2 / 1 steps 0.6935 / 0.687 / 0.6865 / 0.690 ms
      if (kt + 1 < nk && kk < SPREAD) {
#pragma unroll
        for (int u = kk * PER_WAVE / SPREAD; u < (kk + 1) * PER_WAVE / SPREAD; ++u) {
          const int i = wave + u * (NTHREADS / 64);
          __builtin_amdgcn_global_load_lds((glb_void *)(g_src[u] + (kt + 1) * BK), (lds_void *)(sbase + (buf ^ 1) * STAGE + i * 64), 16, 0, 0);
        }
      }
      if (kk + 1 < BK / 16) read_frags(kk + 1, (kk + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[kk & 1][ni], fa[kk & 1][mi], acc[ni][mi], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }
  // Epilogue.  acc[ni][mi][r] = C[m][n] with m = wm*WM + mi*32 + l32 and
  // n = wn*WN + ni*32 + 8*(r/4) + 4*half + r%4.
  constexpr int ROW_BYTES = BN * 2 + 16;  // padded row: 8-byte column writes of 32 rows hit distinct banks
  unsigned char *sC = smem;
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int m = wm * WM + mi * 32 + l32;
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int n = wn * WN + ni * 32 + rg * 8 + half * 4;
        u32x2 p;
        p.x = pack_bf16x2(acc[ni][mi][rg * 4 + 0], acc[ni][mi][rg * 4 + 1]);
        p.y = pack_bf16x2(acc[ni][mi][rg * 4 + 2], acc[ni][mi][rg * 4 + 3]);
        *reinterpret_cast<u32x2 *>(sC + m * ROW_BYTES + n * 2) = p;
      }
    }
  __syncthreads();
  constexpr int CH_ROW = BN / 8;  // 16-byte chunks per tile row
  for (int id = tid; id < BM * CH_ROW; id += NTHREADS) {
    const int r = id / CH_ROW, c = id % CH_ROW;
    const long long gm = m0 + r;
    const int gn = n0 + c * 8;
    if (gm < M && gn < N)
      *reinterpret_cast<u32x4 *>(C + gm * N + gn) = *reinterpret_cast<const u32x4 *>(sC + r * ROW_BYTES + c * 16);
  }
}

// Up to two independent transposes in one launch (both projection weights of a forward pass): workgroups
// [0, n1) serve the first matrix, the rest the second.  64 x 64 tiles; both sizes are multiples of 8 (checked by the
// launcher) and a thread moves 16 bytes per memory access (the tile is transposed element by element on its way into LDS).
__global__ __launch_bounds__(256) void transpose_bf16_kernel(const bf16_t *__restrict__ src1, bf16_t *__restrict__ dst1,
                                                            int rows1, int cols1, int n1,
                                                            const bf16_t *__restrict__ src2, bf16_t *__restrict__ dst2,
                                                            int rows2, int cols2) {
  __shared__ __attribute__((aligned(16))) bf16_t tile[64][72];  // [source column][source row], rows of 144 bytes
  const bool second = (int)blockIdx.x >= n1;
  const bf16_t *src = second ? src2 : src1;
  bf16_t *dst = second ? dst2 : dst1;
  const int rows = second ? rows2 : rows1, cols = second ? cols2 : cols1;
  const int id = second ? blockIdx.x - n1 : blockIdx.x, tiles_c = (cols + 63) / 64;
  const int c0 = (id % tiles_c) * 64, r0 = (id / tiles_c) * 64;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int ch = threadIdx.x + i * 256, r = ch >> 3, c = (ch & 7) * 8;  // chunk of 8 columns of source row r0 + r
    u32x4 v = {0, 0, 0, 0};
    if (r0 + r < rows && c0 + c < cols) v = *reinterpret_cast<const u32x4 *>(src + (long long)(r0 + r) * cols + c0 + c);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      tile[c + 2 * e][r] = (bf16_t)(v[e] & 0xffffu);
      tile[c + 2 * e + 1][r] = (bf16_t)(v[e] >> 16);
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int ch = threadIdx.x + i * 256, c = ch >> 3, r = (ch & 7) * 8;  // 8 source rows of source column c0 + c
    if (c0 + c < cols && r0 + r < rows)
      *reinterpret_cast<u32x4 *>(dst + (long long)(c0 + c) * rows + r0 + r) = *reinterpret_cast<const u32x4 *>(&tile[c][r]);
  }
}

// ---------------------------------------------------------------------------
// Weight-gradient GEMM (adjoint of the two projections): C (Mo,No) = A (K,Mo)^T * B (K,No), contraction over
// the B*T token rows.  Both operands are row-major with the contraction index as the ROW, so the tiles are
// staged row-major in LDS and the MFMA fragments (8 values along K for one column) come from the transposing
// LDS read.  The output is small (a weight matrix) and K is long, so K is split over `gridDim.y` workgroups
// that write fp32 partial sums; a second kernel adds them in a fixed order and rounds to bf16.
// ---------------------------------------------------------------------------
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16 lds_v4i16;

constexpr int TN_BN = 256, TN_ROW = 256 * 2 + 64;  // tile width (both operands); LDS row in bytes, padded by 64 so
                                                   // that the 4 rows a transposing read touches fall in 4 different bank groups

__device__ __forceinline__ bf16x8 tr_frag_tn(const unsigned char *base, int r0, int c0) {
  const unsigned char *p = base + r0 * TN_ROW + c0 * 2;
  const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16 *)p);
  const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16 *)(p + 8 * TN_ROW));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__global__ __launch_bounds__(512) void gemm_bf16_tn_kernel(const bf16_t *__restrict__ A, long long lda,
                                                          const bf16_t *__restrict__ Bm, long long ldb,
                                                          float *__restrict__ part, int Mo, int No, long long K,
                                                          int tiles_n, int tiles_total, int slabs_per_split) {
  constexpr int NTHREADS = 512, WAVES_N = 4;
  constexpr int WM = BM / 2, WN = TN_BN / WAVES_N;  // 128 x 64 wave tile
  constexpr int MI = WM / 32, NI = WN / 32;
  constexpr int CHUNKS = BK * (BM / 8) / NTHREADS;  // 16-byte chunks per thread per operand per slab (4)
  constexpr int TILE = BK * TN_ROW;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [2 stages][A tile | B tile]

  const int wg = blockIdx.x;
  const int per_xcd = (tiles_total + 7) / 8;
  const int tile = (wg % 8) * per_xcd + wg / 8;
  if (tile >= tiles_total) return;
  const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * TN_BN;
  const int split = blockIdx.y;
  const long long nk_all = (K + BK - 1) / BK;
  const long long slab0 = (long long)split * slabs_per_split;
  const int nk = (int)((slab0 + slabs_per_split <= nk_all ? slabs_per_split : nk_all - slab0));

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int l32 = lane & 31, half = lane >> 5;

  // chunk id -> (row r of the slab, 16-byte column chunk c); columns past the matrix edge are clamped to
  // column 0 (they only feed outputs that are never stored), rows past K are zero-filled
  int c_row[CHUNKS], c_col[CHUNKS];
  const bf16_t *a_src[CHUNKS], *b_src[CHUNKS];
#pragma unroll
  for (int i = 0; i < CHUNKS; ++i) {
    const int id = tid + i * NTHREADS;
    c_row[i] = id >> 5;
    c_col[i] = id & 31;
    const int am = m0 + c_col[i] * 8, bn = n0 + c_col[i] * 8;
    a_src[i] = A + (am < Mo ? am : 0);
    b_src[i] = Bm + (bn < No ? bn : 0);
  }
  u32x4 ra[CHUNKS], rb[CHUNKS];
  auto load_slab = [&](long long k0) {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const long long gk = k0 + c_row[i];
      u32x4 va = {0, 0, 0, 0}, vb = {0, 0, 0, 0};
      if (gk < K) {
        va = *reinterpret_cast<const u32x4 *>(a_src[i] + gk * lda);
        vb = *reinterpret_cast<const u32x4 *>(b_src[i] + gk * ldb);
      }
      ra[i] = va;
      rb[i] = vb;
    }
  };
  auto store_slab = [&](int buf) {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      *reinterpret_cast<u32x4 *>(smem + buf * 2 * TILE + c_row[i] * TN_ROW + c_col[i] * 16) = ra[i];
      *reinterpret_cast<u32x4 *>(smem + buf * 2 * TILE + TILE + c_row[i] * TN_ROW + c_col[i] * 16) = rb[i];
    }
  };

  f32x16 acc[NI][MI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[ni][mi][r] = 0.f;

  const uint32_t tr_off = (uint32_t)(4 * half + ((lane & 15) >> 2)) * TN_ROW + (((lane >> 4) & 1) * 16 + 4 * (lane & 3)) * 2;
  const long long kbase = slab0 * BK;
  if (nk > 0) {
    load_slab(kbase);
    store_slab(0);
    if (nk > 1) load_slab(kbase + BK);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) store_slab(buf ^ 1);
    if (kt + 2 < nk) load_slab(kbase + (long long)(kt + 2) * BK);
    const unsigned char *pa = smem + buf * 2 * TILE + tr_off, *pb = pa + TILE;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 fa[MI], fb[NI];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) fa[mi] = tr_frag_tn(pa, kk * 16, wm * WM + mi * 32);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) fb[ni] = tr_frag_tn(pb, kk * 16, wn * WN + ni * 32);
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ni], fa[mi], acc[ni][mi], 0, 0, 0);
    }
    __syncthreads();
  }
  // acc[ni][mi][r] = C[m][n], m = m0 + wm*WM + mi*32 + l32, n = n0 + wn*WN + ni*32 + 8*(r/4) + 4*half + r%4
  float *out = part + (long long)split * Mo * No;
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int m = m0 + wm * WM + mi * 32 + l32;
      if (m >= Mo) continue;
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int n = n0 + wn * WN + ni * 32 + rg * 8 + half * 4;
        if (n < No) {  // No % 8 == 0 and n % 4 == 0: the four columns are inside
          f32x4 v4 = {acc[ni][mi][rg * 4 + 0], acc[ni][mi][rg * 4 + 1], acc[ni][mi][rg * 4 + 2], acc[ni][mi][rg * 4 + 3]};
          *reinterpret_cast<f32x4 *>(out + (long long)m * No + n) = v4;
        }
      }
    }
}

// C[i] = bf16(sum_s part[s][i]), 4 elements per thread, fixed summation order
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ part, int splits, long long n,
                                                           bf16_t *__restrict__ C) {
  const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= n) return;
  f32x4 acc = *reinterpret_cast<const f32x4 *>(part + i);
  for (int s = 1; s < splits; ++s) {
    const f32x4 v = *reinterpret_cast<const f32x4 *>(part + (long long)s * n + i);
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  u32x2 w;
  w.x = pack_bf16x2(acc.x, acc.y);
  w.y = pack_bf16x2(acc.z, acc.w);
  *reinterpret_cast<u32x2 *>(C + i) = w;
}

// Number of K splits: minimise (rounds on 256 CUs) x (slabs per split) x (time of one 256x256x64 slab at ~70 % of
// the MFMA rate, 1.2 us) + the traffic of the fp32 partial sums (written once, read once, ~3 TB/s).
int tn_splits(int Mo, int No, long long K) {
  const long long tiles = (long long)((Mo + BM - 1) / BM) * ((No + TN_BN - 1) / TN_BN);
  const long long nk = (K + BK - 1) / BK;
  int best = 1;
  double best_t = -1.0;
  for (int sp = 1; sp <= 32; ++sp) {
    const long long per = (nk + sp - 1) / sp;
    if (sp > 1 && per < 4) break;
    if ((per * (sp - 1)) >= nk) continue;  // an empty last split
    const double t = (double)((tiles * sp + 255) / 256) * (double)per * 1.2e-6 + (double)sp * Mo * No * 8.0 / 3e12;
    if (best_t < 0 || t < best_t) best_t = t, best = sp;
  }
  return best;
}

template <int BN, int WAVES_M, int WAVES_N>
hipError_t launch_gemm(const void *A, const void *Bt, void *C, long long M, int N, int K, hipStream_t s) {
  const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (N + BN - 1) / BN;
  const int total = tiles_m * tiles_n;
  const int per_xcd = (total + 7) / 8;
  constexpr size_t epi_bytes = (size_t)BM * (BN * 2 + 16);
  constexpr size_t main_bytes = 2ull * (BM + BN) * BK * 2;
  constexpr size_t smem = main_bytes > epi_bytes ? main_bytes : epi_bytes;
  if (hipError_t e = raise_lds_limit<gemm_bf16_nt_kernel<BN, WAVES_M, WAVES_N>>(smem); e != hipSuccess) return e;
  gemm_bf16_nt_kernel<BN, WAVES_M, WAVES_N><<<per_xcd * 8, WAVES_M * WAVES_N * 64, smem, s>>>((const bf16_t *)A, (const bf16_t *)Bt, (bf16_t *)C, M, N,
                                                             K, tiles_n, total);
  return hipGetLastError();
}

}  // namespace

// Measurement aid: nothing but matrix-core instructions (four independent accumulator chains per wavefront, no
// memory traffic inside the loop), to read off the MFMA rate the chip sustains, i.e. the clock it holds under
// matrix-core load.  One float per thread is written so that the work cannot be removed.
__global__ __launch_bounds__(256) void mfma_probe_kernel(float *__restrict__ out, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (__bf16)((float)(threadIdx.x & 7) * 0.125f);
    b[i] = (__bf16)((float)i * 0.25f);
  }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  for (int it = 0; it < iters; ++it) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
  }
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = c0[0] + c1[1] + c2[2] + c3[3];
}

// The same loop on varied operands: 8 register sets of pseudo-random values in (-2, 2) with random mantissas, as
// activations and weights have.  The matrix cores draw more power multiplying such values than the few small
// constants above (it is the values, not their changing: one random set used for every instruction costs the
// same), and the clock the chip holds follows the power.
__global__ __launch_bounds__(256) void mfma_probe_random_kernel(float *__restrict__ out, int iters) {
  bf16x8 a[8], b[8];
  unsigned h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int s = 0; s < 8; ++s)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      h = h * 1664525u + 1013904223u;
      a[s][i] = (__bf16)((float)(int)(h >> 8) * (1.0f / 4194304.0f) - 2.0f);
      h = h * 1664525u + 1013904223u;
      b[s][i] = (__bf16)((float)(int)(h >> 8) * (1.0f / 4194304.0f) - 2.0f);
    }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  for (int it = 0; it < iters; it += 2) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[1], c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2], b[2], c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[3], b[3], c3, 0, 0, 0);
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[4], b[4], c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[5], b[5], c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[6], b[6], c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[7], b[7], c3, 0, 0, 0);
  }
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = c0[0] + c1[1] + c2[2] + c3[3];
}

hipError_t mfma_probe(float *out, int blocks, int iters, bool random_operands, hipStream_t s) {
  if (random_operands) mfma_probe_random_kernel<<<blocks, 256, 0, s>>>(out, iters);
  else mfma_probe_kernel<<<blocks, 256, 0, s>>>(out, iters);
  return hipGetLastError();
}

bool gemm_mfma_supported(long long M, int N, int K) { return M >= 1 && K % BK == 0 && K >= BK && N % 8 == 0 && N >= 8; }

hipError_t gemm_mfma_bf16(const void *A, const void *Bt, void *C, long long M, int N, int K, hipStream_t s) {
  // Tile width by the number of rounds the grid needs on 256 CUs:
  // N = 1536, M = 16384 gives 384 tiles of 256 (2 rounds, half empty) or 512 tiles of 192 (2 full rounds).
  auto cost = [&](int bn) {
    const long long tiles = ((M + BM - 1) / BM) * ((N + bn - 1) / bn);
    return ((tiles + 255) / 256) * bn;
  };
  // 8 wavefronts (2 per SIMD) measured 15-20 % faster than 4 wavefronts with 128x128 wave tiles: a second
  // wavefront hides LDS latency better than the compiler's in-wave schedule does
  if (cost(192) < cost(256)) return launch_gemm<192, 4, 2>(A, Bt, C, M, N, K, s);
  return launch_gemm<256, 2, 4>(A, Bt, C, M, N, K, s);
}

bool gemm_tn_mfma_supported(int Mo, int No, long long K) { return Mo % 8 == 0 && No % 8 == 0 && Mo >= 8 && No >= 8 && K >= 1; }

size_t gemm_tn_scratch_bytes(int Mo, int No, long long K) {
  return (size_t)tn_splits(Mo, No, K) * Mo * No * sizeof(float);
}

hipError_t gemm_tn_mfma_bf16(const void *A, long long lda, const void *Bm, long long ldb, void *C, int Mo, int No,
                             long long K, float *part, hipStream_t s) {
  const int tiles_m = (Mo + BM - 1) / BM, tiles_n = (No + TN_BN - 1) / TN_BN;
  const int total = tiles_m * tiles_n, per_xcd = (total + 7) / 8;
  const int splits = tn_splits(Mo, No, K);
  const long long nk = (K + BK - 1) / BK;
  const int per = (int)((nk + splits - 1) / splits);
  constexpr size_t smem = 2ull * 2 * BK * TN_ROW;
  if (hipError_t e = raise_lds_limit<gemm_bf16_tn_kernel>(smem); e != hipSuccess) return e;
  gemm_bf16_tn_kernel<<<dim3(per_xcd * 8, splits), 512, smem, s>>>((const bf16_t *)A, lda, (const bf16_t *)Bm, ldb, part,
                                                                  Mo, No, K, tiles_n, total, per);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const long long n = (long long)Mo * No;
  splitk_reduce_kernel<<<(unsigned)((n / 4 + 255) / 256), 256, 0, s>>>(part, splits, n, (bf16_t *)C);
  return hipGetLastError();
}

hipError_t transpose_bf16(const void *src, void *dst, int rows, int cols, hipStream_t s) {
  return transpose2_bf16(src, dst, rows, cols, nullptr, nullptr, 0, 0, s);
}

hipError_t transpose2_bf16(const void *src1, void *dst1, int rows1, int cols1, const void *src2, void *dst2, int rows2,
                           int cols2, hipStream_t s) {
  if (rows1 % 8 || cols1 % 8 || (src2 && (rows2 % 8 || cols2 % 8))) return hipErrorInvalidValue;
  const int n1 = ((cols1 + 63) / 64) * ((rows1 + 63) / 64);
  const int n2 = src2 ? ((cols2 + 63) / 64) * ((rows2 + 63) / 64) : 0;
  transpose_bf16_kernel<<<n1 + n2, 256, 0, s>>>((const bf16_t *)src1, (bf16_t *)dst1, rows1, cols1, n1,
                                                 (const bf16_t *)src2, (bf16_t *)dst2, rows2, cols2);
  return hipGetLastError();
}

}  // namespace cca
