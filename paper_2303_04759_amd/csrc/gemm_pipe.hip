// Pipelined bf16 MFMA GEMM for gfx950: operand tiles go from global memory
// straight into LDS (global_load_lds, 16 bytes per lane) through an NS-stage
// ring, so several k-steps of loads are in flight while the matrix cores work
// on the oldest stage; one workgroup barrier per k-step.
//
// LDS layout (no padding is possible with direct loads: one instruction fills
// 1 KiB contiguously, 16 bytes per lane, so bank conflicts are avoided by
// permuting which global 16-byte chunk each lane fetches):
//   K-major tile  [ROWS][64]  : chunk c of row r sits at position c ^ ((r>>1)&7)
//   MN-major tile [64][ROWS]  : chunk cc of k-row k sits at position cc ^ ((k&3)<<2)
// K-major fragments are read with ds_read_b128, MN-major ones with the
// transposing ds_read_b64_tr_b16.
#include "gemm_device.hpp"

namespace raf {

constexpr int PBK = 64;

template <int ROWS, bool KMAJOR, int NW>
struct PipeTile {
  static constexpr int BYTES = ROWS * PBK * 2;
  static constexpr int LOADS = BYTES / 1024 / NW;       // direct-load instructions per wave per stage
  static_assert(LOADS >= 1 && LOADS * NW * 1024 == BYTES, "tile must split evenly over the waves");
  static constexpr int CPR = KMAJOR ? 8 : ROWS / 8;     // 16-byte chunks per LDS row
  static __device__ __forceinline__ int swz_k(int r) { return (r >> 1) & 7; }
  static __device__ __forceinline__ int swz_mn(int k) { return CPR >= 16 ? ((k & 3) << 2) : ((k & 1) << 2); }
};

typedef __attribute__((address_space(3))) void* lds_void_ptr;

// per-lane global source addresses of this wave's direct loads for k-step 0
template <int ROWS, bool KMAJOR, int NW>
__device__ __forceinline__ void pipe_src_init(const bf16_t* base, long ld, int row0, int nrows,
                                              const bf16_t* (&src)[PipeTile<ROWS, KMAJOR, NW>::LOADS]) {
  typedef PipeTile<ROWS, KMAJOR, NW> PT;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < PT::LOADS; ++i) {
    const int q = wave * PT::LOADS + i;       // which KiB of the tile
    if (KMAJOR) {
      const int r = q * 8 + (lane >> 3);
      const int c = (lane & 7) ^ PT::swz_k(r);
      int gr = row0 + r;
      gr = gr < nrows ? gr : nrows - 1;
      src[i] = base + (long)gr * ld + c * 8;
    } else {
      constexpr int RPK = 64 / PT::CPR;       // k-rows per KiB
      const int k = q * RPK + lane / PT::CPR;
      const int cc = (lane % PT::CPR) ^ PT::swz_mn(k);
      int col = row0 + cc * 8;
      col = col < nrows ? col : nrows - 8;
      src[i] = base + (long)k * ld + col;
    }
  }
}

template <int ROWS, bool KMAJOR, int NW>
__device__ __forceinline__ void pipe_issue(const bf16_t* (&src)[PipeTile<ROWS, KMAJOR, NW>::LOADS], long koff,
                                           char* lds_tile) {
  typedef PipeTile<ROWS, KMAJOR, NW> PT;
  const int wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < PT::LOADS; ++i) {
    char* dst = lds_tile + (wave * PT::LOADS + i) * 1024;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[i] + koff),
                                     (lds_void_ptr)dst, 16, 0, 0);
  }
}

template <int ROWS, bool KMAJOR>
__device__ __forceinline__ bf16x8_t pipe_fragment(const char* lds_tile, int row, int kk) {
  typedef PipeTile<ROWS, KMAJOR, 1> PT;
  const int lane = threadIdx.x & 63;
  if (KMAJOR) {
    const int r = row + (lane & 31);
    const int c = kk * 2 + (lane >> 5);
    return *reinterpret_cast<const bf16x8_t*>(lds_tile + r * 128 + ((c ^ PT::swz_k(r)) << 4));
  } else {
    const int grp = lane >> 4, s = lane & 15;
    const int k = kk * 16 + (grp >> 1) * 8 + (s >> 2);
    const int col = row + (grp & 1) * 16 + (s & 3) * 4;
    const char* p = lds_tile + k * (ROWS * 2) + (((col >> 3) ^ PT::swz_mn(k)) << 4) + (col & 7) * 2;
    typedef s16x4_t __attribute__((address_space(3))) * lds_v4_ptr;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p + 4 * ROWS * 2));
    const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, both);
  }
}

// s_waitcnt on the vector-memory counter only (expcnt / lgkmcnt left at max)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

template <int BM, int BN, int WGM, int WGN, bool A_KMAJOR, bool B_KMAJOR, typename TC, int NS>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_pipe_kernel(GemmDev g, int tiles_m, int tiles_n) {
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile below one MFMA block");
  typedef PipeTile<BM, A_KMAJOR, NW> PA;
  typedef PipeTile<BN, B_KMAJOR, NW> PB;
  constexpr int STAGE_BYTES = PA::BYTES + PB::BYTES;
  constexpr int LPS = PA::LOADS + PB::LOADS;          // loads per wave per stage
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  // Tile assignment.  Consecutive workgroup ids go round-robin over the 8
  // XCDs (each with its own L2), so XCD x takes the contiguous range
  // [x*per, (x+1)*per) of the row-major tile list: tiles sharing A rows and B
  // columns meet in one L2.
  const int ntile = tiles_m * tiles_n;
  const int per = (ntile + 7) >> 3;
  const int t = (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);
  if (t >= ntile) return;
  const int m0 = (t / tiles_n) * BM, n0 = (t % tiles_n) * BN;

  const int z = blockIdx.y;
  const int zb = z / g.nz_inner, zi = z % g.nz_inner;
  const bf16_t* __restrict__ A = (const bf16_t*)g.a + zb * g.sa0 + zi * g.sa1;
  const bf16_t* __restrict__ B = (const bf16_t*)g.b + zb * g.sb0 + zi * g.sb1;
  TC* __restrict__ C = (TC*)g.c + zb * g.sc0 + zi * g.sc1;
  bf16_t* __restrict__ AUX = g.aux ? (bf16_t*)g.aux + zb * g.sc0 + zi * g.sc1 : nullptr;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;

  const bf16_t* srca[PA::LOADS];
  const bf16_t* srcb[PB::LOADS];
  pipe_src_init<BM, A_KMAJOR, NW>(A, g.lda, m0, g.M, srca);
  pipe_src_init<BN, B_KMAJOR, NW>(B, g.ldb, n0, g.N, srcb);
  const long stepa = A_KMAJOR ? PBK : (long)PBK * g.lda;
  const long stepb = B_KMAJOR ? PBK : (long)PBK * g.ldb;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = g.K / PBK;
#pragma unroll
  for (int s = 0; s < NS - 1; ++s) {
    if (s < nk) {
      pipe_issue<BM, A_KMAJOR, NW>(srca, s * stepa, lds + s * STAGE_BYTES);
      pipe_issue<BN, B_KMAJOR, NW>(srcb, s * stepb, lds + s * STAGE_BYTES + PA::BYTES);
    }
  }

  int stage = 0;
  for (int it = 0; it < nk; ++it) {
    // loads of k-steps it+1 .. it+NS-2 may stay in flight; those of k-step `it` must have landed
    const int ahead = nk - 1 - it;
    if (NS >= 4 && ahead >= 2) wait_vmcnt<(NS >= 4 ? 2 : 0) * LPS>();
    else if (NS >= 3 && ahead >= 1) wait_vmcnt<(NS >= 3 ? 1 : 0) * LPS>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();   // stage `it` is complete for every wave; stage it-1 is free
    const int nxt = it + NS - 1;
    if (nxt < nk) {
      int ns = stage + NS - 1;
      ns = ns >= NS ? ns - NS : ns;
      pipe_issue<BM, A_KMAJOR, NW>(srca, nxt * stepa, lds + ns * STAGE_BYTES);
      pipe_issue<BN, B_KMAJOR, NW>(srcb, nxt * stepb, lds + ns * STAGE_BYTES + PA::BYTES);
    }
    const char* ta = lds + stage * STAGE_BYTES;
    const char* tb = ta + PA::BYTES;
    // fragment loads run one sub-step ahead of the MFMAs that consume them
    bf16x8_t fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = pipe_fragment<BM, A_KMAJOR>(ta, wm + i * 32, 0);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = pipe_fragment<BN, B_KMAJOR>(tb, wn + j * 32, 0);
#pragma unroll
    for (int kk = 0; kk < PBK / 16; ++kk) {
      const int cur = kk & 1, nx = cur ^ 1;
      if (kk + 1 < PBK / 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[nx][i] = pipe_fragment<BM, A_KMAJOR>(ta, wm + i * 32, kk + 1);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[nx][j] = pipe_fragment<BN, B_KMAJOR>(tb, wn + j * 32, kk + 1);
      }
      // operands swapped: the MFMA yields the transposed 32x32 block, so a lane
      // holds 4 consecutive output columns per register group
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][j], fa[cur][i], acc[i][j], 0, 0, 0);
    }
    stage = stage + 1 == NS ? 0 : stage + 1;
  }

  // register r of lane l holds output row (l & 31), column 8*(r/4) + 4*(l/32) + r%4 of its 32x32 block
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + wm + i * 32 + (lane & 31);
    if (row < g.M) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = n0 + wn + j * 32 + 8 * q + 4 * (lane >> 5);
          if (col < g.N) {
            float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
            epilogue_store4<TC>(g, C, AUX, row, col, v);
          }
        }
    }
  }
}

template <int BM, int BN, int WGM, int WGN, bool AK, bool BKM, typename TC, int NS>
static bool launch_pipe_inst(const GemmDev& d, int batch, hipStream_t st) {
  constexpr int NW = WGM * WGN;
  constexpr int LDS_BYTES = NS * (PipeTile<BM, AK, NW>::BYTES + PipeTile<BN, BKM, NW>::BYTES);
  auto kern = gemm_bf16_pipe_kernel<BM, BN, WGM, WGN, AK, BKM, TC, NS>;
  static bool attr_done = false;   // per instantiation
  if (!attr_done) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess) {
      (void)hipGetLastError();
      return false;
    }
    attr_done = true;
  }
  const int tiles_m = (d.M + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
  const int ntile = tiles_m * tiles_n;
  dim3 grid(((ntile + 7) / 8) * 8, batch);
  hipLaunchKernelGGL(kern, grid, dim3(64 * NW), LDS_BYTES, st, d, tiles_m, tiles_n);
  return true;
}

// 128x128 tiles, 8 wavefronts (2 x 4), two 32 KiB stages: two workgroups share a
// CU (16 waves).  Measured on MI355X against 4-wave workgroups, deeper rings and
// 256-wide tiles, this is the fastest variant for every shape of the layer.
template <bool AK, bool BKM, typename TC>
static bool launch_pipe_layout(const GemmDev& d, int batch, hipStream_t st) {
  return launch_pipe_inst<128, 128, 2, 4, AK, BKM, TC, 2>(d, batch, st);
}

bool launch_gemm_pipe(const GemmDev& d, int a_kmajor, int b_kmajor, int out_f32, int batch, hipStream_t st) {
  if (d.K % PBK) return false;
  if (d.M < 128 || d.N < 128 || batch != 1 || out_f32) return false;
  const long tiles = (long)((d.M + 127) / 128) * ((d.N + 127) / 128);
  if (a_kmajor && b_kmajor) return launch_pipe_layout<true, true, bf16_t>(d, batch, st);
  // with a transposed B operand the ring only wins when there are enough tiles
  // for two workgroups per CU; below that the register-staged kernel is faster
  if (a_kmajor && !b_kmajor && tiles >= 384) return launch_pipe_layout<true, false, bf16_t>(d, batch, st);
  return false;
}

}  // namespace raf
