// Dense contractions of the training step: bf16 MFMA GEMM (gfx950
// v_mfma_f32_32x32x16_bf16, fp32 accumulate) and an fp32 FMA GEMM for the
// full-precision mode, both with the fused epilogues the step needs
// (bias, bias+GeLU with saved pre-activation, GeLU-gradient multiply, residual
// add, scale, fp32 output).  Pattern-based "GEMM + elementwise epilogue"
// fusion in the sense of the paper's Section 3.2.2.
#include "gemm_device.hpp"

namespace raf {

// ------------------------------------------------------------- bf16 MFMA --
constexpr int BK = 64;          // k extent of one LDS stage

// Operand tile in LDS.
//  K-major operands (contraction index contiguous in memory) are kept
//  [row][BK+8]: the 16-byte pad makes the 128-bit fragment reads conflict-free.
//  MN-major operands (row index contiguous in memory, i.e. the operand arrives
//  transposed) are kept [k][ROWS+32] and read with the transposing LDS load
//  ds_read_b64_tr_b16; a pitch of 16 dwords modulo 32 spreads the four k-rows a
//  16-lane group touches over distinct banks.
template <int ROWS, bool KMAJOR, int NTHREADS>
struct TileLds {
  static constexpr int PITCH = KMAJOR ? (BK + 8) : (ROWS + 32);
  static constexpr int ELEMS = KMAJOR ? ROWS * PITCH : BK * PITCH;
  static constexpr int VEC_PER_THREAD = ROWS * BK / 8 / NTHREADS;
  static_assert(VEC_PER_THREAD >= 1, "tile too small for the workgroup");
};

template <int ROWS, bool KMAJOR, int NTHREADS>
__device__ __forceinline__ void tile_load_global(const bf16_t* __restrict__ base, long ld, int row0, int nrows, int k0,
                                                 int K, uint4 (&reg)[TileLds<ROWS, KMAJOR, NTHREADS>::VEC_PER_THREAD]) {
  constexpr int NV = TileLds<ROWS, KMAJOR, NTHREADS>::VEC_PER_THREAD;
  const int tid = threadIdx.x;
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int v = tid + t * NTHREADS;
    if (KMAJOR) {
      int r = row0 + v / (BK / 8);
      r = r < nrows ? r : nrows - 1;
      const int k = k0 + (v % (BK / 8)) * 8;
      reg[t] = k < K ? *reinterpret_cast<const uint4*>(base + (long)r * ld + k) : make_uint4(0, 0, 0, 0);
    } else {
      const int kr = v / (ROWS / 8);
      int r = row0 + (v % (ROWS / 8)) * 8;
      r = r < nrows ? r : nrows - 8;
      reg[t] = k0 + kr < K ? *reinterpret_cast<const uint4*>(base + (long)(k0 + kr) * ld + r) : make_uint4(0, 0, 0, 0);
    }
  }
}

template <int ROWS, bool KMAJOR, int NTHREADS>
__device__ __forceinline__ void tile_store_lds(bf16_t* lds,
                                               const uint4 (&reg)[TileLds<ROWS, KMAJOR, NTHREADS>::VEC_PER_THREAD]) {
  constexpr int NV = TileLds<ROWS, KMAJOR, NTHREADS>::VEC_PER_THREAD;
  constexpr int PITCH = TileLds<ROWS, KMAJOR, NTHREADS>::PITCH;
  const int tid = threadIdx.x;
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int v = tid + t * NTHREADS;
    if (KMAJOR) {
      *reinterpret_cast<uint4*>(lds + (v / (BK / 8)) * PITCH + (v % (BK / 8)) * 8) = reg[t];
    } else {
      *reinterpret_cast<uint4*>(lds + (v / (ROWS / 8)) * PITCH + (v % (ROWS / 8)) * 8) = reg[t];
    }
  }
}

// MFMA operand fragment for 32 rows starting at `row` and the 16 k values of
// sub-step kk: lane l supplies row (l & 31), k = kk*16 + (l >> 5)*8 + 0..7.
//
// Transposing read (measured lane layout of ds_read_b64_tr_b16): inside each
// group of 16 lanes, lane s points at 4 consecutive 16-bit elements and lane t
// receives element (t & 3) of lanes (t >> 2), 4 + (t >> 2), 8 + (t >> 2),
// 12 + (t >> 2).  With lane s pointing at k-row (s >> 2), columns 4*(s & 3)..+3
// of a [k][row] tile, lane t ends up with 4 consecutive k of column t.
template <int PITCH, bool KMAJOR>
__device__ __forceinline__ bf16x8_t tile_fragment(const bf16_t* lds, int row, int kk) {
  const int lane = threadIdx.x & 63;
  if (KMAJOR) {
    const int r = row + (lane & 31);
    const int k = kk * 16 + (lane >> 5) * 8;
    return *reinterpret_cast<const bf16x8_t*>(lds + r * PITCH + k);
  } else {
    const int grp = lane >> 4, s = lane & 15;
    const int k = kk * 16 + (grp >> 1) * 8 + (s >> 2);
    const int col = row + (grp & 1) * 16 + (s & 3) * 4;
    typedef s16x4_t __attribute__((address_space(3))) * lds_v4_ptr;
    const bf16_t* p = lds + k * PITCH + col;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p + 4 * PITCH));
    const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, both);
  }
}

// One BM x BN output tile of problem g (batch index z) by a workgroup of
// WGM x WGN wavefronts: operand tiles are staged global -> registers -> LDS
// with the next k-step's global loads in flight during the MFMAs.
template <int BM, int BN, int WGM, int WGN, bool A_KMAJOR, bool B_KMAJOR, typename TC>
__device__ __forceinline__ void staged_tile(const GemmDev& g, int m0, int n0, int z, bf16_t* lds_a, bf16_t* lds_b) {
  constexpr int NTHREADS = 64 * WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile below one MFMA block");
  typedef TileLds<BM, A_KMAJOR, NTHREADS> LA;
  typedef TileLds<BN, B_KMAJOR, NTHREADS> LB;

  const int zb = z / g.nz_inner, zi = z % g.nz_inner;
  const bf16_t* __restrict__ A = (const bf16_t*)g.a + zb * g.sa0 + zi * g.sa1;
  const bf16_t* __restrict__ B = (const bf16_t*)g.b + zb * g.sb0 + zi * g.sb1;
  TC* __restrict__ C = (TC*)g.c + zb * g.sc0 + zi * g.sc1;
  bf16_t* __restrict__ AUX = g.aux ? (bf16_t*)g.aux + zb * g.sc0 + zi * g.sc1 : nullptr;

  const int wave = threadIdx.x >> 6;
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  uint4 ra[LA::VEC_PER_THREAD], rb[LB::VEC_PER_THREAD];
  tile_load_global<BM, A_KMAJOR, NTHREADS>(A, g.lda, m0, g.M, 0, g.K, ra);
  tile_load_global<BN, B_KMAJOR, NTHREADS>(B, g.ldb, n0, g.N, 0, g.K, rb);

  for (int k0 = 0; k0 < g.K; k0 += BK) {
    __syncthreads();   // previous stage fully consumed
    tile_store_lds<BM, A_KMAJOR, NTHREADS>(lds_a, ra);
    tile_store_lds<BN, B_KMAJOR, NTHREADS>(lds_b, rb);
    __syncthreads();
    if (k0 + BK < g.K) {
      tile_load_global<BM, A_KMAJOR, NTHREADS>(A, g.lda, m0, g.M, k0 + BK, g.K, ra);
      tile_load_global<BN, B_KMAJOR, NTHREADS>(B, g.ldb, n0, g.N, k0 + BK, g.K, rb);
    }
    // fragment loads run one sub-step ahead of the MFMAs that consume them
    bf16x8_t fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = tile_fragment<LA::PITCH, A_KMAJOR>(lds_a, wm + i * 32, 0);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = tile_fragment<LB::PITCH, B_KMAJOR>(lds_b, wn + j * 32, 0);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      const int cur = kk & 1, nx = cur ^ 1;
      if (kk + 1 < BK / 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[nx][i] = tile_fragment<LA::PITCH, A_KMAJOR>(lds_a, wm + i * 32, kk + 1);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[nx][j] = tile_fragment<LB::PITCH, B_KMAJOR>(lds_b, wn + j * 32, kk + 1);
      }
      // operands swapped: the MFMA produces the transposed 32x32 block, so that
      // a lane ends up with 4 consecutive output columns per register group
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][j], fa[cur][i], acc[i][j], 0, 0, 0);
    }
  }

  // accumulator layout of the (transposed) 32x32 block: register r of lane l
  // holds output row (l & 31), column 8*(r/4) + 4*(l/32) + r%4.
  epilogue_tile32<TC, TM, TN>(g, C, AUX, acc, m0 + wm, n0 + wn);
}

// Consecutive workgroup ids are dealt round-robin to the 8 XCDs (each with its
// own L2).  Give XCD x the contiguous range [x*per, (x+1)*per) of the row-major
// tile list, so that tiles sharing A rows / B columns meet in one L2.
__device__ __forceinline__ int xcd_tile(int block, int ntile) {
  const int per = (ntile + 7) >> 3;
  return (block & 7) * per + (block >> 3);
}

template <int BM, int BN, int WGM, int WGN, bool A_KMAJOR, bool B_KMAJOR, typename TC>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_kernel(GemmDev g, int tiles_m, int tiles_n, int remap) {
  constexpr int NTHREADS = 64 * WGM * WGN;
  __shared__ __attribute__((aligned(16))) bf16_t lds_a[TileLds<BM, A_KMAJOR, NTHREADS>::ELEMS];
  __shared__ __attribute__((aligned(16))) bf16_t lds_b[TileLds<BN, B_KMAJOR, NTHREADS>::ELEMS];
  const int ntile = tiles_m * tiles_n;
  const int t = remap ? xcd_tile(blockIdx.x, ntile) : (int)blockIdx.x;
  if (t >= ntile) return;
  staged_tile<BM, BN, WGM, WGN, A_KMAJOR, B_KMAJOR, TC>(g, (t / tiles_n) * BM, (t % tiles_n) * BN, blockIdx.y, lds_a,
                                                          lds_b);
}

// Several independent problems of one layout in a single launch (the four
// weight-gradient GEMMs of a layer: each alone has too few tiles to fill the
// chip).  tile_start[p] is the first linear tile of problem p.

template <int BM, int BN, int WGM, int WGN, bool A_KMAJOR, bool B_KMAJOR, typename TC>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_group_kernel(GemmGroupDev grp) {
  constexpr int NTHREADS = 64 * WGM * WGN;
  __shared__ __attribute__((aligned(16))) bf16_t lds_a[TileLds<BM, A_KMAJOR, NTHREADS>::ELEMS];
  __shared__ __attribute__((aligned(16))) bf16_t lds_b[TileLds<BN, B_KMAJOR, NTHREADS>::ELEMS];
  const int ntile = grp.tile_start[grp.count];
  const int t = xcd_tile(blockIdx.x, ntile);
  if (t >= ntile) return;
  int p = 0;
#pragma unroll
  for (int q = 1; q < GEMM_GROUP_MAX; ++q)
    if (q < grp.count && t >= grp.tile_start[q]) p = q;
  const int lt = t - grp.tile_start[p];
  const int tn = grp.tiles_n[p];
  // the problem descriptor is selected with wave-uniform scalar loads
  staged_tile<BM, BN, WGM, WGN, A_KMAJOR, B_KMAJOR, TC>(grp.p[p], (lt / tn) * BM, (lt % tn) * BN, 0, lds_a, lds_b);
}

// -------------------------------------------------------------- fp32 FMA --
// Plain LDS-tiled FMA kernel for the full-precision mode (small validation
// shapes): 64x64 tile, 16x16 threads, 4x4 outputs each, any strides.
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmDev g, long sa_i, long sa_k, long sb_k, long sb_j) {
  constexpr int T = 64, KT = 16;
  __shared__ float As[KT][T + 1];
  __shared__ float Bs[KT][T + 1];
  const int z = blockIdx.z;
  const int zb = z / g.nz_inner, zi = z % g.nz_inner;
  const float* __restrict__ A = (const float*)g.a + zb * g.sa0 + zi * g.sa1;
  const float* __restrict__ B = (const float*)g.b + zb * g.sb0 + zi * g.sb1;
  float* __restrict__ C = (float*)g.c + zb * g.sc0 + zi * g.sc1;
  float* __restrict__ AUX = g.aux ? (float*)g.aux + zb * g.sc0 + zi * g.sc1 : nullptr;
  const int m0 = blockIdx.y * T, n0 = blockIdx.x * T;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < g.K; k0 += KT) {
    for (int e = threadIdx.x; e < T * KT; e += 256) {
      const int r = e / KT, k = e % KT;     // k fastest: good for k-major operands
      const int i = m0 + r, j = n0 + r, kk = k0 + k;
      As[k][r] = (i < g.M && kk < g.K) ? A[i * sa_i + kk * sa_k] : 0.f;
      Bs[k][r] = (j < g.N && kk < g.K) ? B[kk * sb_k + j * sb_j] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < KT; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        a[u] = As[k][ty * 4 + u];
        b[u] = Bs[k][tx * 4 + u];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[u][w] = fmaf(a[u], b[w], acc[u][w]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int i = m0 + ty * 4 + u, j = n0 + tx * 4 + w;
      if (i < g.M && j < g.N) epilogue_store<float, float>(g, C, AUX, i, j, acc[u][w]);
    }
}

// ---------------------------------------------------------------- launch --
template <int BM, int BN, int WGM, int WGN, bool AK, bool BKM>
static void launch_bf16_tile(const GemmDev& d, int out_f32, int batch, hipStream_t st) {
  const int tiles_m = (d.M + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
  const int ntile = tiles_m * tiles_n;
  const int remap = (batch == 1 && ntile >= 64) ? 1 : 0;   // XCD-aware order only pays for one large problem
  dim3 grid(remap ? ((ntile + 7) / 8) * 8 : ntile, batch);
  dim3 block(64 * WGM * WGN);
  if (out_f32)
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WGM, WGN, AK, BKM, float>), grid, block, 0, st, d, tiles_m, tiles_n,
                       remap);
  else
    hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WGM, WGN, AK, BKM, bf16_t>), grid, block, 0, st, d, tiles_m, tiles_n,
                       remap);
}

// Few tiles: one workgroup per CU at most, so use 8 wavefronts per workgroup
// (2 per SIMD) to overlap LDS/global latency with MFMA inside the workgroup.
static bool few_tiles(const GemmDev& d, int batch) {
  const long tiles = (long)((d.M + 127) / 128) * ((d.N + 127) / 128) * batch;
  return tiles < 384;
}

template <bool AK, bool BKM>
static void launch_bf16_layout(const GemmDev& d, int out_f32, int batch, hipStream_t st) {
  if (d.M <= 64 && d.N <= 64)
    launch_bf16_tile<64, 64, 2, 2, AK, BKM>(d, out_f32, batch, st);
  else if (d.N <= 64)
    launch_bf16_tile<128, 64, 2, 2, AK, BKM>(d, out_f32, batch, st);
  else if (few_tiles(d, batch))
    launch_bf16_tile<128, 128, 2, 4, AK, BKM>(d, out_f32, batch, st);
  else
    launch_bf16_tile<128, 128, 2, 2, AK, BKM>(d, out_f32, batch, st);
}

static raf_status check_gemm_args(const GemmArgs& g) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0 || g.batch <= 0 || g.nz_inner <= 0) return RAF_EINVAL;
  if ((g.M % 32) || (g.N % 32) || (g.K % 32)) return RAF_ENOTSUP;
  if (!g.a || !g.b || !g.c) return RAF_EINVAL;
  if (!aligned16(g.a) || !aligned16(g.b) || !aligned16(g.c)) return RAF_EINVAL;
  if ((g.epilogue == EPI_BIAS || g.epilogue == EPI_BIAS_GELU || g.epilogue == EPI_BIAS_GELU_DERIV) && !g.bias) return RAF_EINVAL;
  if (g.epilogue >= EPI_BIAS_GELU && !g.aux) return RAF_EINVAL;
  if (g.epilogue < 0 || g.epilogue > EPI_MUL_AUX) return RAF_EINVAL;
  if ((g.lda % 8) || (g.ldb % 8) || (g.ldc % 8) || (g.aux && (g.ldaux % 8))) return RAF_EINVAL;
  if (g.batch > 65535) return RAF_ENOTSUP;
  return RAF_OK;
}

static GemmDev to_dev(const GemmArgs& g) {
  GemmDev d;
  d.M = g.M; d.N = g.N; d.K = g.K;
  d.a = g.a; d.lda = g.lda; d.b = g.b; d.ldb = g.ldb; d.c = g.c; d.ldc = g.ldc;
  d.alpha = g.alpha; d.epilogue = g.epilogue; d.bias = g.bias; d.aux = g.aux; d.ldaux = g.ldaux;
  d.gelu_tanh = g.gelu_tanh; d.nz_inner = g.nz_inner;
  d.sa0 = g.sa[0]; d.sa1 = g.sa[1]; d.sb0 = g.sb[0]; d.sb1 = g.sb[1]; d.sc0 = g.sc[0]; d.sc1 = g.sc[1];
  return d;
}

// ------------------------------------------------------- bf16 transposes --
// The input-gradient products dX = dY . W contract over the rows of the
// row-major weight, i.e. over its strided dimension.  With a transposed copy of
// W both operands are contiguous along the contraction and the product runs on
// the K-major kernels, the fastest ones; writing the copy costs about as much as
// reading the weight once.  64x64 tiles through LDS, 16-byte accesses both ways.
constexpr int TRANSPOSE_MAX = 4;
struct TransposeDev {
  const uint16_t* src[TRANSPOSE_MAX];
  uint16_t* dst[TRANSPOSE_MAX];
  int rows[TRANSPOSE_MAX], cols[TRANSPOSE_MAX], tiles_c[TRANSPOSE_MAX];
  int tile_start[TRANSPOSE_MAX + 1];
};

__global__ __launch_bounds__(256) void transpose_bf16_kernel(TransposeDev g) {
  __shared__ uint16_t tile[64][64 + 2];
  int j = 0;
  while (j + 1 < TRANSPOSE_MAX && (int)blockIdx.x >= g.tile_start[j + 1]) ++j;
  const int t = blockIdx.x - g.tile_start[j];
  const int r0 = (t / g.tiles_c[j]) * 64, c0 = (t % g.tiles_c[j]) * 64;
  const int rows = g.rows[j], cols = g.cols[j];
  const uint16_t* __restrict__ src = g.src[j];
  uint16_t* __restrict__ dst = g.dst[j];
  const int chunk = threadIdx.x & 7, line = threadIdx.x >> 3;   // 8 chunks of 8 elements per 64-wide line
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = line + 32 * pass;
    if (r0 + r < rows && c0 + chunk * 8 < cols) {
      const uint4 v = *reinterpret_cast<const uint4*>(src + (long)(r0 + r) * cols + c0 + chunk * 8);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        tile[r][chunk * 8 + 2 * e] = (uint16_t)(w[e] & 0xffffu);
        tile[r][chunk * 8 + 2 * e + 1] = (uint16_t)(w[e] >> 16);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int c = line + 32 * pass;             // output row = input column
    if (c0 + c < cols && r0 + chunk * 8 < rows) {
      uint32_t w[4];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        w[e] = (uint32_t)tile[chunk * 8 + 2 * e][c] | ((uint32_t)tile[chunk * 8 + 2 * e + 1][c] << 16);
      *reinterpret_cast<uint4*>(dst + (long)(c0 + c) * rows + r0 + chunk * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
}

raf_status launch_transpose_bf16(const TransposeJob* jobs, int count, hipStream_t st) {
  if (!jobs || count <= 0 || count > TRANSPOSE_MAX) return RAF_EINVAL;
  TransposeDev g{};
  int tiles = 0;
  for (int i = 0; i < count; ++i) {
    if (!jobs[i].src || !jobs[i].dst || jobs[i].rows <= 0 || jobs[i].cols <= 0) return RAF_EINVAL;
    if ((jobs[i].rows % 8) || (jobs[i].cols % 8) || !aligned16(jobs[i].src) || !aligned16(jobs[i].dst)) return RAF_EINVAL;
    g.src[i] = (const uint16_t*)jobs[i].src; g.dst[i] = (uint16_t*)jobs[i].dst;
    g.rows[i] = jobs[i].rows; g.cols[i] = jobs[i].cols;
    g.tiles_c[i] = (jobs[i].cols + 63) / 64;
    g.tile_start[i] = tiles;
    tiles += ((jobs[i].rows + 63) / 64) * g.tiles_c[i];
  }
  for (int i = count; i <= TRANSPOSE_MAX; ++i) g.tile_start[i] = tiles;
  for (int i = count; i < TRANSPOSE_MAX; ++i) { g.src[i] = g.src[0]; g.dst[i] = g.dst[0]; g.rows[i] = g.cols[i] = 8; g.tiles_c[i] = 1; }
  hipLaunchKernelGGL(transpose_bf16_kernel, dim3(tiles), dim3(256), 0, st, g);
  return check_launch();
}

// Weight-gradient form only: A and B both MN-major, float output, no batch.
raf_status launch_gemm_group_wgrad(int precision, const GemmArgs* gs, int count, hipStream_t st, const ColsumJob* side,
                                   int nside, const ReduceJob* reds, int nred, bool* side_taken, int* nonfinite) {
  if (side_taken) *side_taken = false;
  if (count <= 0 || count > GEMM_GROUP_MAX || !gs) return RAF_EINVAL;
  bool groupable = precision == RAF_BF16_AMP;
  for (int i = 0; i < count; ++i) {
    raf_status rc = check_gemm_args(gs[i]);
    if (rc != RAF_OK) return rc;
    if (gs[i].a_kmajor || gs[i].b_kmajor || !gs[i].out_f32 || gs[i].batch != 1 || gs[i].epilogue != EPI_NONE ||
        gs[i].M < 128 || gs[i].N < 128)
      groupable = false;
  }
  if (!groupable) {
    for (int i = 0; i < count; ++i) {
      raf_status rc = launch_gemm(precision, gs[i], st);
      if (rc != RAF_OK) return rc;
    }
    return RAF_OK;
  }
  if (precision == RAF_BF16_AMP) {
    GemmDev ds[GEMM_GROUP_MAX];
    for (int i = 0; i < count; ++i) ds[i] = to_dev(gs[i]);
    // column sums of up to two bf16 matrices with a common row count can ride along on idle CUs
    ColsumSide sd{};
    sd.nonfinite = nonfinite;
    if (side && nside >= 1 && nside <= 2) {
      bool ok = true;
      for (int i = 0; i < nside; ++i)
        ok = ok && side[i].precision == RAF_BF16_AMP && side[i].x && side[i].out && side[i].cols > 0 &&
             side[i].cols % 8 == 0 && side[i].ld % 8 == 0 && side[i].rows == side[0].rows && aligned16(side[i].x) &&
             (side[i].out_cols == 0 || side[i].out_cols == side[i].cols);
      if (ok) {
        sd.count = nside;
        sd.rows = side[0].rows;
        for (int i = 0; i < nside; ++i) {
          sd.x[i] = (const bf16_t*)side[i].x;
          sd.out[i] = side[i].out;
          sd.ld[i] = side[i].ld;
          sd.cols[i] = side[i].cols;
        }
        if (nside == 1) { sd.x[1] = sd.x[0]; sd.out[1] = sd.out[0]; sd.ld[1] = sd.ld[0]; sd.cols[1] = 0; }
        sd.nred = 0;
        if (reds && nred > 0 && nred <= 3) {
          for (int i = 0; i < nred; ++i) sd.red[i] = reds[i];
          sd.nred = nred;
        } else if (nred > 3) {
          sd.count = 0;   // more second stages than the side workers take: the caller launches everything itself
        }
      }
    }
    if (launch_gemm_group_spec(ds, count, st, sd.count ? &sd : nullptr, side_taken)) return check_launch();
  }
  GemmGroupDev grp;
  grp.count = count;
  int tiles = 0;
  for (int i = 0; i < count; ++i) {
    grp.p[i] = to_dev(gs[i]);
    grp.tile_start[i] = tiles;
    grp.tiles_n[i] = (gs[i].N + 127) / 128;
    tiles += ((gs[i].M + 127) / 128) * grp.tiles_n[i];
  }
  for (int i = count; i <= GEMM_GROUP_MAX; ++i) grp.tile_start[i] = tiles;
  for (int i = 0; i < GEMM_GROUP_MAX; ++i) grp.tiles_m_first[i] = 0;
  for (int i = count; i < GEMM_GROUP_MAX; ++i) { grp.p[i] = grp.p[0]; grp.tiles_n[i] = 1; }
  dim3 grid(((tiles + 7) / 8) * 8);
  // 8 wavefronts per workgroup measured faster than 4 even with ~1.7 workgroups per CU
  hipLaunchKernelGGL((gemm_bf16_group_kernel<128, 128, 2, 4, false, false, float>), grid, dim3(512), 0, st, grp);
  return check_launch();
}

raf_status launch_gemm(int precision, const GemmArgs& g, hipStream_t st) {
  raf_status rc = check_gemm_args(g);
  if (rc != RAF_OK) return rc;
  const GemmDev d = to_dev(g);
  if (precision == RAF_F32) {
    dim3 grid((g.N + 63) / 64, (g.M + 63) / 64, g.batch);
    const long sa_i = g.a_kmajor ? g.lda : 1, sa_k = g.a_kmajor ? 1 : g.lda;
    const long sb_k = g.b_kmajor ? 1 : g.ldb, sb_j = g.b_kmajor ? g.ldb : 1;
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, st, d, sa_i, sa_k, sb_k, sb_j);
  } else if (precision == RAF_BF16_AMP) {
    if (!g.a_kmajor && !g.b_kmajor && g.out_f32 && g.batch == 1 && g.epilogue == EPI_NONE &&
        launch_gemm_group_spec(&d, 1, st))
      return check_launch();
    if (launch_gemm_pipe(d, g.a_kmajor, g.b_kmajor, g.out_f32, g.batch, st)) return check_launch();
    if (g.a_kmajor && g.b_kmajor) launch_bf16_layout<true, true>(d, g.out_f32, g.batch, st);
    else if (g.a_kmajor && !g.b_kmajor) launch_bf16_layout<true, false>(d, g.out_f32, g.batch, st);
    else if (!g.a_kmajor && !g.b_kmajor) launch_bf16_layout<false, false>(d, g.out_f32, g.batch, st);
    else launch_bf16_layout<false, true>(d, g.out_f32, g.batch, st);
  } else {
    return RAF_EINVAL;
  }
  return check_launch();
}

}  // namespace raf
