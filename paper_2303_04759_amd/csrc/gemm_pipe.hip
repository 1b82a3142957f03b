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
                                              const bf16_t* (&src)[PipeTile<ROWS, KMAJOR, NW>::LOADS], int wave) {
  typedef PipeTile<ROWS, KMAJOR, NW> PT;
  const int lane = threadIdx.x & 63;
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
                                           char* lds_tile, int wave) {
  typedef PipeTile<ROWS, KMAJOR, NW> PT;
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

// s_waitcnt vmcnt(n) for a wave-uniform run-time n (conservative above 24)
__device__ __forceinline__ void wait_vmcnt_dyn(int n) {
  switch (n) {
#define RAF_VMCNT_CASE(N) case N: wait_vmcnt<N>(); break;
    RAF_VMCNT_CASE(1) RAF_VMCNT_CASE(2) RAF_VMCNT_CASE(3) RAF_VMCNT_CASE(4) RAF_VMCNT_CASE(5) RAF_VMCNT_CASE(6)
    RAF_VMCNT_CASE(7) RAF_VMCNT_CASE(8) RAF_VMCNT_CASE(9) RAF_VMCNT_CASE(10) RAF_VMCNT_CASE(11) RAF_VMCNT_CASE(12)
    RAF_VMCNT_CASE(13) RAF_VMCNT_CASE(14) RAF_VMCNT_CASE(15) RAF_VMCNT_CASE(16) RAF_VMCNT_CASE(17) RAF_VMCNT_CASE(18)
    RAF_VMCNT_CASE(19) RAF_VMCNT_CASE(20) RAF_VMCNT_CASE(21) RAF_VMCNT_CASE(22) RAF_VMCNT_CASE(23) RAF_VMCNT_CASE(24)
#undef RAF_VMCNT_CASE
    default: wait_vmcnt<0>(); break;
  }
}

template <int BM, int BN, int WGM, int WGN, bool A_KMAJOR, bool B_KMAJOR, typename TC, int NS>
__device__ __forceinline__ void pipe_body(const GemmDev& g, int tiles_m, int tiles_n, int remap, int z) {
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
  // batched launches (many problems of a few tiles) keep the plain order: consecutive workgroups already spread
  // over the XCDs
  const int t = remap ? (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3) : (int)blockIdx.x;
  if (t >= ntile) return;
  const int m0 = (t / tiles_n) * BM, n0 = (t % tiles_n) * BN;

  const int zb = z / g.nz_inner, zi = z % g.nz_inner;
  const bf16_t* __restrict__ A = (const bf16_t*)g.a + zb * g.sa0 + zi * g.sa1;
  const bf16_t* __restrict__ B = (const bf16_t*)g.b + zb * g.sb0 + zi * g.sb1;
  TC* __restrict__ C = (TC*)g.c + zb * g.sc0 + zi * g.sc1;
  bf16_t* __restrict__ AUX = g.aux ? (bf16_t*)g.aux + zb * g.sc0 + zi * g.sc1 : nullptr;

  const int wave = threadIdx.x >> 6;
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;

  const bf16_t* srca[PA::LOADS];
  const bf16_t* srcb[PB::LOADS];
  pipe_src_init<BM, A_KMAJOR, NW>(A, g.lda, m0, g.M, srca, wave);
  pipe_src_init<BN, B_KMAJOR, NW>(B, g.ldb, n0, g.N, srcb, wave);
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
      pipe_issue<BM, A_KMAJOR, NW>(srca, s * stepa, lds + s * STAGE_BYTES, wave);
      pipe_issue<BN, B_KMAJOR, NW>(srcb, s * stepb, lds + s * STAGE_BYTES + PA::BYTES, wave);
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
      pipe_issue<BM, A_KMAJOR, NW>(srca, nxt * stepa, lds + ns * STAGE_BYTES, wave);
      pipe_issue<BN, B_KMAJOR, NW>(srcb, nxt * stepb, lds + ns * STAGE_BYTES + PA::BYTES, wave);
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
  epilogue_tile32<TC, TM, TN>(g, C, AUX, acc, m0 + wm, n0 + wn);
}

template <int BM, int BN, int WGM, int WGN, bool A_KMAJOR, bool B_KMAJOR, typename TC, int NS>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_pipe_kernel(GemmDev g, int tiles_m, int tiles_n, int remap) {
  pipe_body<BM, BN, WGM, WGN, A_KMAJOR, B_KMAJOR, TC, NS>(g, tiles_m, tiles_n, remap, (int)blockIdx.y);
}

template <int BM, int BN, int WGM, int WGN, bool AK, bool BKM, typename TC, int NS>
static bool launch_pipe_inst(const GemmDev& d, int batch, hipStream_t st) {
  constexpr int NW = WGM * WGN;
  constexpr int LDS_BYTES = NS * (PipeTile<BM, AK, NW>::BYTES + PipeTile<BN, BKM, NW>::BYTES);
  auto kern = gemm_bf16_pipe_kernel<BM, BN, WGM, WGN, AK, BKM, TC, NS>;
  static LdsLimitOnce lds_limit;   // per instantiation
  if (!lds_limit.ensure((const void*)kern, LDS_BYTES)) return false;
  const int tiles_m = (d.M + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
  const int ntile = tiles_m * tiles_n;
  const int remap = batch == 1 ? 1 : 0;
  dim3 grid(remap ? ((ntile + 7) / 8) * 8 : ntile, batch);
  hipLaunchKernelGGL(kern, grid, dim3(64 * NW), LDS_BYTES, st, d, tiles_m, tiles_n, remap);
  return true;
}

// ---------------------------------------------------------------------------
// Producer/consumer form of the ring for a group of problems (the four weight
// gradients of a layer: long contraction, operands contiguous along M and N).
// A wave is held for roughly a hundred cycles per 1-KiB direct load, so loads
// issued by the computing waves serialise with their MFMAs, and loads that go
// through registers are capped near 16 bytes/clock/CU.  Here NP producer waves
// do nothing but issue the direct-to-LDS loads, NS-1 k-steps ahead, while the
// WGM*WGN consumer waves only read fragments and issue MFMAs.  One workgroup
// barrier per k-step keeps both sides in step: after barrier `it` the consumers
// work on stage it while the producers refill the stage that was just freed
// and then wait until stage it+1 has landed.
// Side work of the grouped launch: worker w of nworkers takes a contiguous range of the 8-column vectors of the
// (concatenated) column space; its threads are dealt to (vector, row group), every row group sums its rows in
// registers, and the row groups are added in a fixed order through LDS, so the sums are reproducible.
__device__ __forceinline__ void colsum_side_worker(const ColsumSide& sd, int w, int nworkers, char* lds) {
  const int nvec0 = sd.cols[0] / 8, total = nvec0 + sd.cols[1] / 8;
  const int per = (total + nworkers - 1) / nworkers;
  const int v0 = w * per;
  const int nv = total - v0 < per ? total - v0 : per;
  if (per > (int)blockDim.x) return;               // uniform over the launch; the host never asks for it
  const int ngroups = (int)blockDim.x / per;
  const int vec = threadIdx.x % per, rg = threadIdx.x / per;
  const bool active = rg < ngroups && vec < nv;     // nv <= 0: a worker beyond the last vector idles through the barrier
  const int uv = v0 + vec;
  const int j = uv < nvec0 ? 0 : 1;
  const bf16_t* __restrict__ x = sd.x[j] + (long)(j ? uv - nvec0 : uv) * 8;
  const long ld = sd.ld[j];
  float acc[8] = {};
  if (active) {
    long r = rg;
    // eight independent 16-byte loads in flight per lane
    for (; r + 7L * ngroups < sd.rows; r += 8L * ngroups) {
      float v[8][8];
#pragma unroll
      for (int u = 0; u < 8; ++u) Vec8<bf16_t>::load(x + (r + (long)u * ngroups) * ld, v[u]);
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += v[u][e];
    }
    for (; r < sd.rows; r += ngroups) {
      float v[8];
      Vec8<bf16_t>::load(x + r * ld, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += v[e];
    }
  }
  float* red = reinterpret_cast<float*>(lds);   // [ngroups][per * 8]
  if (active) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[(rg * per + vec) * 8 + e] = acc[e];
  }
  __syncthreads();
  bool bad = false;
  for (int c = threadIdx.x; c < nv * 8; c += blockDim.x) {
    float sum = red[c];
    for (int g = 1; g < ngroups; ++g) sum += red[g * per * 8 + c];
    const int u = v0 + c / 8;
    const int jj = u < nvec0 ? 0 : 1;
    sd.out[jj][(long)(jj ? u - nvec0 : u) * 8 + (c & 7)] = sum;
    bad |= !(sum - sum == 0.f);   // x - x is 0 for finite x and nan for inf and nan
  }
  if (bad && sd.nonfinite) *sd.nonfinite = 1;   // every writer stores the same value
}

// out_k[c] = sum_p partial[p][k][c] for the columns of worker w: threads are dealt to (column, slice of the partial
// rows), slices are added in a fixed order through LDS
__device__ __forceinline__ void reduce_side_worker(const ReduceJob& job, int w, int nworkers, char* lds, int* nonfinite) {
  const int chunk = (job.width_out + nworkers - 1) / nworkers;
  const int c0 = w * chunk;
  const int nc = job.width_out - c0 < chunk ? job.width_out - c0 : chunk;
  float* red = reinterpret_cast<float*>(lds);   // [nslices][chunk]
  const bool fits = chunk <= (int)blockDim.x;
  const int nslices = fits ? (int)blockDim.x / chunk : 1;
  const int cl = fits ? threadIdx.x % chunk : 0, slice = fits ? threadIdx.x / chunk : nslices;
  const long width = (long)job.nout * job.ncols;   // stride between partial rows
  __syncthreads();                                 // the previous user of the LDS buffer is done
  if (nc > 0 && fits && slice < nslices) {
    float acc = 0.f;
    if (cl < nc) {
      // eight loads in flight; rows past the end re-read the last row and are not added
      for (int p = slice; p < job.nparts; p += 8 * nslices) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int q = p + u * nslices;
          v[u] = job.partial[(long)(q < job.nparts ? q : job.nparts - 1) * width + c0 + cl];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += p + u * nslices < job.nparts ? v[u] : 0.f;
      }
    }
    red[slice * chunk + cl] = acc;
  }
  __syncthreads();
  if (nc > 0 && fits && slice == 0 && cl < nc) {
    float sum = 0.f;
    for (int sl = 0; sl < nslices; ++sl) sum += red[sl * chunk + cl];
    const int c = c0 + cl;
    const int k = c / job.ncols;
    int cc = c % job.ncols;
    if (job.perm_nvec > 0) cc = (cc % job.perm_nvec) * 8 + cc / job.perm_nvec;   // partial rows stored element-major
    float* o = k == 0 ? job.o0 : (k == 1 ? job.o1 : job.o2);
    if (o) {
      o[cc] = sum;
      if (nonfinite && !(sum - sum == 0.f)) *nonfinite = 1;
    }
  }
}

template <int BM, int BN, int WGM, int WGN, bool A_KMAJOR, bool B_KMAJOR, typename TC, int NS, int NP>
__global__ __launch_bounds__(64 * (WGM * WGN + NP)) void gemm_bf16_spec_kernel(GemmGroupDev grp, ColsumSide side,
                                                                               int tile_blocks) {
  constexpr int NC = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile below one MFMA block");
  static_assert(NS >= 3, "the producers need a stage to fill while one is read and one is in flight");
  typedef PipeTile<BM, A_KMAJOR, NP> PA;
  typedef PipeTile<BN, B_KMAJOR, NP> PB;
  constexpr int STAGE_BYTES = PA::BYTES + PB::BYTES;
  constexpr int LPS = PA::LOADS + PB::LOADS;          // loads per producer wave per stage
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  if ((int)blockIdx.x >= tile_blocks) {   // a workgroup without a tile: column sums on a CU that the tiles leave idle
    const int w = (int)blockIdx.x - tile_blocks, nworkers = (int)gridDim.x - tile_blocks;
    colsum_side_worker(side, w, nworkers, lds);
    // static indices: a run-time index would copy the descriptors to scratch memory
    if (side.nred > 0) reduce_side_worker(side.red[0], w, nworkers, lds, side.nonfinite);
    if (side.nred > 1) reduce_side_worker(side.red[1], w, nworkers, lds, side.nonfinite);
    if (side.nred > 2) reduce_side_worker(side.red[2], w, nworkers, lds, side.nonfinite);
    return;
  }
  const int ntile = grp.tile_start[grp.count];
  const int per = (ntile + 7) >> 3;
  const int t = (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);   // XCD x takes tiles [x*per, (x+1)*per)
  if (t >= ntile) return;
  // the problem is selected with static indices (a run-time index would copy the descriptors to scratch memory)
  GemmDev g = grp.p[0];
  int lt = t, tn = grp.tiles_n[0], tmf = grp.tiles_m_first[0];
#pragma unroll
  for (int q = 1; q < GEMM_GROUP_MAX; ++q)
    if (q < grp.count && t >= grp.tile_start[q]) {
      g = grp.p[q];
      lt = t - grp.tile_start[q];
      tn = grp.tiles_n[q];
      tmf = grp.tiles_m_first[q];
    }
  const int m0 = (tmf ? lt % tmf : lt / tn) * BM, n0 = (tmf ? lt / tmf : lt % tn) * BN;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nk = g.K / PBK;

  if (wave >= NC) {
    // ------------------------------------------------------------ producer
    const int pw = wave - NC;
    const bf16_t* srca[PA::LOADS];
    const bf16_t* srcb[PB::LOADS];
    pipe_src_init<BM, A_KMAJOR, NP>((const bf16_t*)g.a, g.lda, m0, g.M, srca, pw);
    pipe_src_init<BN, B_KMAJOR, NP>((const bf16_t*)g.b, g.ldb, n0, g.N, srcb, pw);
    const long stepa = A_KMAJOR ? PBK : (long)PBK * g.lda;
    const long stepb = B_KMAJOR ? PBK : (long)PBK * g.ldb;
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
      if (s < nk) {
        pipe_issue<BM, A_KMAJOR, NP>(srca, s * stepa, lds + s * STAGE_BYTES, pw);
        pipe_issue<BN, B_KMAJOR, NP>(srcb, s * stepb, lds + s * STAGE_BYTES + PA::BYTES, pw);
      }
    int stage = 0;
    for (int it = 0; it < nk; ++it) {
      // k-steps it+1 .. it+NS-2 may stay in flight; k-step `it` must have landed
      const int ahead = nk - 1 - it < NS - 2 ? nk - 1 - it : NS - 2;
      wait_vmcnt_dyn(ahead * LPS);
      __builtin_amdgcn_s_barrier();   // stage `it` handed to the consumers; stage it-1 is free
      const int nxt = it + NS - 1;
      if (nxt < nk) {
        int ns = stage + NS - 1;
        ns = ns >= NS ? ns - NS : ns;
        pipe_issue<BM, A_KMAJOR, NP>(srca, nxt * stepa, lds + ns * STAGE_BYTES, pw);
        pipe_issue<BN, B_KMAJOR, NP>(srcb, nxt * stepb, lds + ns * STAGE_BYTES + PA::BYTES, pw);
      }
      stage = stage + 1 == NS ? 0 : stage + 1;
    }
    return;
  }

  // -------------------------------------------------------------- consumer
  const int wm = (wave / WGN) * WM, wn = (wave % WGN) * WN;
  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  int stage = 0;
  for (int it = 0; it < nk; ++it) {
    __builtin_amdgcn_s_barrier();   // stage `it` is complete
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
      // operands swapped: a lane holds 4 consecutive output columns per register group
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][j], fa[cur][i], acc[i][j], 0, 0, 0);
    }
    stage = stage + 1 == NS ? 0 : stage + 1;
  }

  TC* __restrict__ C = (TC*)g.c;
  bf16_t* __restrict__ AUX = (bf16_t*)g.aux;
  if (side.nonfinite) {
    // non-finite test of the weight gradients while they are still in registers (rows and columns past the edge of a
    // ragged tile repeat operand rows that also feed real outputs, so they raise the flag only when those do)
    bool bad = false;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) bad |= !(acc[i][j][r] - acc[i][j][r] == 0.f);
    if (bad) *side.nonfinite = 1;   // every writer stores the same value
  }
  // register r of lane l holds output row (l & 31), column 8*(r/4) + 4*(l/32) + r%4 of its 32x32 block
  if constexpr (sizeof(TC) == 4) {
    // every consumer has passed the last barrier, so the stage after the last one is read by nobody and no load
    // is in flight to it: each wave stages its blocks in a slice of it
    static_assert(NC * epilogue_stage32_bytes <= STAGE_BYTES, "staging exceeds a ring stage");
    if (epilogue_can_stage32(g)) {
      epilogue_tile32_staged<TM, TN>(g, C, acc, m0 + wm, n0 + wn, lds + stage * STAGE_BYTES + wave * epilogue_stage32_bytes);
      return;
    }
  }
  epilogue_tile32<TC, TM, TN>(g, C, AUX, acc, m0 + wm, n0 + wn);
}

bool launch_gemm_group_spec(const GemmDev* ds, int count, hipStream_t st, const ColsumSide* side, bool* side_taken) {
  constexpr int BM = 256, BN = 128, WGM = 4, WGN = 2, NS = 3, NP = 8;
  if (side_taken) *side_taken = false;
  if (!ds || count <= 0 || count > GEMM_GROUP_MAX) return false;
  GemmGroupDev grp;
  grp.count = count;
  int tiles = 0;
  for (int i = 0; i < count; ++i) {
    if (ds[i].K % PBK || ds[i].M < BM || ds[i].N < BN || (ds[i].M % 8) || (ds[i].N % 8)) return false;
    grp.p[i] = ds[i];
    grp.tile_start[i] = tiles;
    grp.tiles_n[i] = (ds[i].N + BN - 1) / BN;
    const int tiles_m = (ds[i].M + BM - 1) / BM;
    // Each XCD takes a contiguous share of the tile list and its L2 fetches every operand panel its tiles touch:
    // numbering the tiles along the side with fewer tiles first keeps the panels of the long side to one XCD each
    // (the 768 x 3072 gradient: 3 x 24 tiles, 78 -> 42 MB of L2 fills).
    grp.tiles_m_first[i] = tiles_m < grp.tiles_n[i] ? tiles_m : 0;
    tiles += tiles_m * grp.tiles_n[i];
  }
  for (int i = count; i <= GEMM_GROUP_MAX; ++i) grp.tile_start[i] = tiles;
  for (int i = count; i < GEMM_GROUP_MAX; ++i) { grp.p[i] = grp.p[0]; grp.tiles_n[i] = 1; grp.tiles_m_first[i] = 0; }
  constexpr int LDS_BYTES = NS * (BM + BN) * PBK * 2;
  static_assert(LDS_BYTES <= 160 * 1024, "ring exceeds the LDS of a CU");
  auto kern = gemm_bf16_spec_kernel<BM, BN, WGM, WGN, false, false, float, NS, NP>;
  static LdsLimitOnce lds_limit;   // per instantiation
  if (!lds_limit.ensure((const void*)kern, LDS_BYTES)) return false;
  const int tile_blocks = ((tiles + 7) / 8) * 8;
  // side workers only where the tiles leave CUs free (one workgroup per CU: the ring takes most of the LDS), and
  // enough of them that a worker's columns take less time than a tile.  With more tiles than CUs the free CUs are
  // those of the last round: the workers come last in the grid and start when the tiles of that round have theirs.
  ColsumSide sd{};
  int workers = 0;
  if (side && side->count > 0) {
    constexpr int NUM_CUS = 256, THREADS = 64 * (WGM * WGN + NP);
    const int total_vecs = (side->cols[0] + side->cols[1]) / 8;
    const int last_round = tile_blocks % NUM_CUS;
    const int free_cus = last_round ? NUM_CUS - last_round : 0;
    if (free_cus > 0 && total_vecs > 0) {
      const int per = (total_vecs + free_cus - 1) / free_cus;
      // per row of the contraction a worker reads per*16 bytes through registers (about 16 bytes/clock/CU: `per`
      // clocks) while a tile needs about 30 clocks (1 us per 64-deep step, measured)
      const bool short_enough = per <= 24;
      const int nw = free_cus < total_vecs ? free_cus : total_vecs;
      bool red_ok = side->nred >= 0 && side->nred <= 3;
      for (int i = 0; red_ok && i < side->nred; ++i)
        red_ok = side->red[i].partial && side->red[i].nparts > 0 && side->red[i].ncols > 0 &&
                 side->red[i].nout >= 1 && side->red[i].nout <= 3 && side->red[i].width_out > 0 &&
                 (side->red[i].width_out + nw - 1) / nw <= THREADS;
      if (per <= THREADS && short_enough && red_ok && (long)(THREADS / per) * per * 32 <= LDS_BYTES) {
        sd = *side;
        workers = nw;
        if (side_taken) *side_taken = true;
      }
    }
  }
  dim3 grid(tile_blocks + workers);
  hipLaunchKernelGGL(kern, grid, dim3(64 * (WGM * WGN + NP)), LDS_BYTES, st, grp, sd, tile_blocks);
  return true;
}

// ---------------------------------------------------------------------------
// Tiles of 64*WGM x 48*WGN outputs for K-major operands.  The widths 48, 96,
// 144 and 192 let the launcher pick a tile count that fills the 256 CUs in
// whole rounds when 128-wide tiles would leave most of the last round idle
// (N = 2304: 16 x 16 tiles of 256x144, one per CU, instead of 576 of 128x128),
// and the tall variants halve the bytes fetched per flop, which is what bounds
// these kernels (direct loads deliver at most about 52 bytes/clock/CU).  Each of the
// WGM x WGN wavefronts owns 64 x 48 outputs as 4 x 3 blocks of
// v_mfma_f32_16x16x32_bf16.  Same direct-to-LDS ring and swizzle as above, NS
// stages deep; the KiB chunks of a stage are dealt round-robin to the waves, so
// some waves issue one load more than others and each wave counts its own.
template <int CHUNKS, int NW>
__device__ __forceinline__ void w48_src_init(const bf16_t* base, long ld, int row0, int nrows, int first,
                                             const bf16_t* (&src)[(CHUNKS + NW - 1) / NW + 1]) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < (CHUNKS + NW - 1) / NW + 1; ++i) {
    int q = i * NW + wave - first;            // which KiB (8 rows) of the tile
    q = q < 0 ? 0 : (q < CHUNKS ? q : CHUNKS - 1);   // out-of-range slots keep a valid address they never use
    const int r = q * 8 + (lane >> 3);
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    int gr = row0 + r;
    gr = gr < nrows ? gr : nrows - 1;
    src[i] = base + (long)gr * ld + c * 8;
  }
}

// `first` shifts the dealing so that the B chunks continue where the A chunks stopped
template <int CHUNKS, int NW>
__device__ __forceinline__ void w48_issue(const bf16_t* (&src)[(CHUNKS + NW - 1) / NW + 1], long koff, char* lds_tile,
                                          int first) {
  const int wave = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < (CHUNKS + NW - 1) / NW + 1; ++i) {
    const int q = i * NW + wave - first;
    if (q >= 0 && q < CHUNKS)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[i] + koff),
                                       (lds_void_ptr)(lds_tile + q * 1024), 16, 0, 0);
  }
}

// 16 rows x 32 contraction values of a K-major tile: lane l holds row l&15, elements 8*(l>>4) .. +7 of k-half kk
__device__ __forceinline__ bf16x8_t w48_fragment(const char* lds_tile, int row0, int kk) {
  const int lane = threadIdx.x & 63;
  const int r = row0 + (lane & 15);
  const int c = kk * 4 + (lane >> 4);
  return *reinterpret_cast<const bf16x8_t*>(lds_tile + r * 128 + ((c ^ ((r >> 1) & 7)) << 4));
}

// KS = 2 doubles the waves of a workgroup without adding LDS traffic: waves w and w + WGM*WGN share one 64x48
// output block, each takes one 32-deep half of every k-step, and the halves are added through LDS at the end (each
// wave of the pair then finishes half of the rows).  For tiles with only 4-8 waves this gives every SIMD a second
// wave to issue MFMAs while the first waits for its LDS fragments.
template <int WGM, int WGN, int NS, int KS, typename TC, int NB = 3>
__global__ __launch_bounds__(64 * WGM * WGN * KS) void gemm_bf16_w48_kernel(GemmDev g, int tiles_m, int tiles_n) {
  constexpr int NT = WGM * WGN, NW = NT * KS, BM = 64 * WGM, BN = 16 * NB * WGN;
  constexpr int ACH = BM / 8, BCH = BN / 8;           // KiB per operand tile
  constexpr int STAGE_BYTES = (ACH + BCH) * 1024;
  constexpr int BFIRST = ACH % NW;                    // wave that takes B chunk 0
  static_assert(KS == 1 || KS == 2, "one or two waves per output block");
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  const int ntile = tiles_m * tiles_n;
  const int per = (ntile + 7) >> 3;
  const int t = (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);   // XCD x takes tiles [x*per, (x+1)*per)
  if (t >= ntile) return;
  const int m0 = (t / tiles_n) * BM, n0 = (t % tiles_n) * BN;

  const bf16_t* __restrict__ A = (const bf16_t*)g.a;
  const bf16_t* __restrict__ B = (const bf16_t*)g.b;
  TC* __restrict__ C = (TC*)g.c;
  bf16_t* __restrict__ AUX = (bf16_t*)g.aux;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int wt = wave % NT, kg = wave / NT;           // output block of this wave, its half of each k-step
  const int wm = (wt / WGN) * 64, wn = (wt % WGN) * 16 * NB;

  const bf16_t* srca[(ACH + NW - 1) / NW + 1];
  const bf16_t* srcb[(BCH + NW - 1) / NW + 1];
  w48_src_init<ACH, NW>(A, g.lda, m0, g.M, 0, srca);
  w48_src_init<BCH, NW>(B, g.ldb, n0, g.N, BFIRST, srcb);
  // loads this wave issues per stage: chunk f of the ACH+BCH goes to wave f % NW
  const int my_loads = (ACH + BCH) / NW + (wave < (ACH + BCH) % NW ? 1 : 0);

  f32x4_t acc[4][NB];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int nk = g.K / PBK;
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < nk) {
      w48_issue<ACH, NW>(srca, (long)s * PBK, lds + s * STAGE_BYTES, 0);
      w48_issue<BCH, NW>(srcb, (long)s * PBK, lds + s * STAGE_BYTES + ACH * 1024, BFIRST);
    }
  int stage = 0;
  for (int it = 0; it < nk; ++it) {
    // k-steps it+1 .. it+NS-2 may stay in flight; k-step `it` must have landed
    const int ahead = nk - 1 - it < NS - 2 ? nk - 1 - it : NS - 2;
    wait_vmcnt_dyn(ahead * my_loads);
    __builtin_amdgcn_s_barrier();   // stage `it` is complete for every wave; stage it-1 is free
    if (it + NS - 1 < nk) {
      int ns = stage + NS - 1;
      ns = ns >= NS ? ns - NS : ns;
      char* nxt = lds + ns * STAGE_BYTES;
      w48_issue<ACH, NW>(srca, (long)(it + NS - 1) * PBK, nxt, 0);
      w48_issue<BCH, NW>(srcb, (long)(it + NS - 1) * PBK, nxt + ACH * 1024, BFIRST);
    }
    const char* ta = lds + stage * STAGE_BYTES;
    const char* tb = ta + ACH * 1024;
#pragma unroll
    for (int kh = 0; kh < 2 / KS; ++kh) {
      const int kk = KS == 2 ? kg : kh;
      bf16x8_t fa[4], fb[NB];
#pragma unroll
      for (int i = 0; i < 4; ++i) fa[i] = w48_fragment(ta, wm + i * 16, kk);
#pragma unroll
      for (int j = 0; j < NB; ++j) fb[j] = w48_fragment(tb, wn + j * 16, kk);
      // operands swapped: a lane ends with output row (l & 15) and 4 consecutive columns 4*(l>>4) + r
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    stage = stage + 1 == NS ? 0 : stage + 1;
  }

  int i_begin = 0, i_end = 4;
  // wave-private LDS for the staged epilogue: with one wave per block a slice of the ring stage that nobody reads
  // any more (every wave has passed the last barrier, so all reads of the stage before the last one are done and no
  // load is in flight), with wave pairs the slot this wave received its partner's accumulators in
  // (waves whose slice does not fit that stage any more take one behind the ring: w48_stage_spill)
  constexpr int SB = epilogue_stage_bytes<NB>(), FIT = STAGE_BYTES / SB;
  static_assert(epilogue_stage_bytes<NB>() <= 2 * NB * 64 * 16, "staging exceeds an exchange slot");
  char* stg = wave < FIT ? lds + stage * STAGE_BYTES + wave * SB : lds + NS * STAGE_BYTES + (wave - FIT) * SB;
  if (KS == 2) {
    // exchange: the wave with kg = 0 finishes row blocks 0-1, its partner row blocks 2-3; each sends the other half
    __builtin_amdgcn_s_barrier();   // every wave is done with the ring
    f32x4_t* xch = reinterpret_cast<f32x4_t*>(lds) + (wt * 2 + (kg ^ 1)) * 2 * NB * 64;   // slot read by the partner
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int j = 0; j < NB; ++j) xch[(ii * NB + j) * 64 + lane] = kg ? acc[ii][j] : acc[2 + ii][j];   // static indices: no scratch
    __syncthreads();
    const f32x4_t* got = reinterpret_cast<const f32x4_t*>(lds) + (wt * 2 + kg) * 2 * NB * 64;
    stg = lds + (wt * 2 + kg) * 2 * NB * 64 * 16;
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const f32x4_t o = got[(ii * NB + j) * 64 + lane];
        // fixed order: first k-half plus second k-half
        if (kg == 0) acc[ii][j] = acc[ii][j] + o;
        else acc[2 + ii][j] = o + acc[2 + ii][j];
      }
    i_begin = kg * 2;
    i_end = i_begin + 2;
  }

  if constexpr (sizeof(TC) == 2) {
    if (epilogue_can_stage(g)) {
      epilogue_tile16_staged<NB>(g, C, AUX, acc, m0 + wm, n0 + wn, i_begin, i_end, stg);
      return;
    }
  }
  epilogue_tile16<TC, NB>(g, C, AUX, acc, m0 + wm, n0 + wn, i_begin, i_end);
}

// Same tiles with the waves specialised: NP producer waves only issue the direct-to-LDS loads (a wave is held for
// roughly a hundred cycles per 1-KiB load instruction, so loads issued by the computing waves serialise with their
// MFMAs), the WGM*WGN*KS consumer waves only read fragments and issue MFMAs.  One workgroup barrier per k-step keeps
// both sides in step: after barrier `it` the consumers work on stage it while the producers refill the stage that was
// freed and then wait until stage it+1 has landed.
template <int WGM, int WGN, int NB, int NS, int KS, int NP, typename TC>
__global__ __launch_bounds__(64 * (WGM * WGN * KS + NP)) void gemm_bf16_w48s_kernel(GemmDev g, int tiles_m, int tiles_n) {
  constexpr int NT = WGM * WGN, NC = NT * KS, BM = 64 * WGM, BN = 16 * NB * WGN;
  constexpr int ACH = BM / 8, BCH = BN / 8;           // KiB per operand tile
  constexpr int STAGE_BYTES = (ACH + BCH) * 1024;
  constexpr int BFIRST = ACH % NP;                    // producer that takes B chunk 0
  static_assert(KS == 1 || KS == 2, "one or two waves per output block");
  static_assert(NS >= 2, "one stage is read while another is filled");
  extern __shared__ __attribute__((aligned(1024))) char lds[];

  const int ntile = tiles_m * tiles_n;
  const int per = (ntile + 7) >> 3;
  const int t = (int)(blockIdx.x & 7) * per + (int)(blockIdx.x >> 3);   // XCD x takes tiles [x*per, (x+1)*per)
  if (t >= ntile) return;
  const int m0 = (t / tiles_n) * BM, n0 = (t % tiles_n) * BN;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int nk = g.K / PBK;

  if (wave >= NC) {
    // ------------------------------------------------------------ producer
    const int pw = wave - NC;
    const bf16_t* __restrict__ A = (const bf16_t*)g.a;
    const bf16_t* __restrict__ B = (const bf16_t*)g.b;
    constexpr int LA = (ACH + NP - 1) / NP + 1, LB = (BCH + NP - 1) / NP + 1;
    const bf16_t* srca[LA];
    const bf16_t* srcb[LB];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
      int q = i * NP + pw;
      q = q < ACH ? q : ACH - 1;
      const int r = q * 8 + (lane >> 3);
      int gr = m0 + r;
      gr = gr < g.M ? gr : g.M - 1;
      srca[i] = A + (long)gr * g.lda + (((lane & 7) ^ ((r >> 1) & 7)) << 3);
    }
#pragma unroll
    for (int i = 0; i < LB; ++i) {
      int q = i * NP + pw - BFIRST;
      q = q < 0 ? 0 : (q < BCH ? q : BCH - 1);
      const int r = q * 8 + (lane >> 3);
      int gr = n0 + r;
      gr = gr < g.N ? gr : g.N - 1;
      srcb[i] = B + (long)gr * g.ldb + (((lane & 7) ^ ((r >> 1) & 7)) << 3);
    }
    const int my_loads = (ACH + BCH) / NP + (pw < (ACH + BCH) % NP ? 1 : 0);
    auto issue = [&](int kstep, int stage) {
      char* base = lds + stage * STAGE_BYTES;
      const long koff = (long)kstep * PBK;
#pragma unroll
      for (int i = 0; i < LA; ++i) {
        const int q = i * NP + pw;
        if (q < ACH)
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srca[i] + koff),
                                           (lds_void_ptr)(base + q * 1024), 16, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < LB; ++i) {
        const int q = i * NP + pw - BFIRST;
        if (q >= 0 && q < BCH)
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srcb[i] + koff),
                                           (lds_void_ptr)(base + (ACH + q) * 1024), 16, 0, 0);
      }
    };
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
      if (s < nk) issue(s, s);
    int stage = 0;
    for (int it = 0; it < nk; ++it) {
      // k-steps it+1 .. it+NS-2 may stay in flight; k-step `it` must have landed
      const int ahead = nk - 1 - it < NS - 2 ? nk - 1 - it : NS - 2;
      wait_vmcnt_dyn(ahead * my_loads);
      __builtin_amdgcn_s_barrier();   // stage `it` handed to the consumers; stage it-1 is free
      if (it + NS - 1 < nk) {
        int ns = stage + NS - 1;
        ns = ns >= NS ? ns - NS : ns;
        issue(it + NS - 1, ns);
      }
      stage = stage + 1 == NS ? 0 : stage + 1;
    }
    if (KS == 2) {   // the consumers' exchange has two more barriers
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_s_barrier();
    }
    return;
  }

  // -------------------------------------------------------------- consumer
  TC* __restrict__ C = (TC*)g.c;
  bf16_t* __restrict__ AUX = (bf16_t*)g.aux;
  const int wt = wave % NT, kg = wave / NT;           // output block of this wave, its half of each k-step
  const int wm = (wt / WGN) * 64, wn = (wt % WGN) * 16 * NB;
  f32x4_t acc[4][NB];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  int stage = 0;
  for (int it = 0; it < nk; ++it) {
    __builtin_amdgcn_s_barrier();   // stage `it` is complete
    const char* ta = lds + stage * STAGE_BYTES;
    const char* tb = ta + ACH * 1024;
#pragma unroll
    for (int kh = 0; kh < 2 / KS; ++kh) {
      const int kk = KS == 2 ? kg : kh;
      bf16x8_t fa[4], fb[NB];
#pragma unroll
      for (int i = 0; i < 4; ++i) fa[i] = w48_fragment(ta, wm + i * 16, kk);
#pragma unroll
      for (int j = 0; j < NB; ++j) fb[j] = w48_fragment(tb, wn + j * 16, kk);
      // operands swapped: a lane ends with output row (l & 15) and 4 consecutive columns 4*(l>>4) + r
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    stage = stage + 1 == NS ? 0 : stage + 1;
  }

  int i_begin = 0, i_end = 4;
  // wave-private LDS for the staged epilogue: with one wave per block a slice of the ring stage that nobody reads
  // any more (every consumer has passed the last barrier, so all reads of the stage before the last one are done,
  // and the producers have no load in flight), with wave pairs the slot this wave received its partner's
  // accumulators in
  // (waves whose slice does not fit that stage any more take one behind the ring: w48_stage_spill)
  constexpr int SB = epilogue_stage_bytes<NB>(), FIT = STAGE_BYTES / SB;
  static_assert(epilogue_stage_bytes<NB>() <= 2 * NB * 64 * 16, "staging exceeds an exchange slot");
  char* stg = KS == 2 ? lds + (wt * 2 + kg) * 2 * NB * 64 * 16
                      : (wave < FIT ? lds + stage * STAGE_BYTES + wave * SB : lds + NS * STAGE_BYTES + (wave - FIT) * SB);
  if (KS == 2) {
    // exchange: the wave with kg = 0 finishes row blocks 0-1, its partner row blocks 2-3; each sends the other half
    __builtin_amdgcn_s_barrier();   // every wave is done with the ring
    f32x4_t* xch = reinterpret_cast<f32x4_t*>(lds) + (wt * 2 + (kg ^ 1)) * 2 * NB * 64;   // slot read by the partner
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int j = 0; j < NB; ++j) xch[(ii * NB + j) * 64 + lane] = kg ? acc[ii][j] : acc[2 + ii][j];   // static indices: no scratch
    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): the writes above have reached LDS
    __builtin_amdgcn_s_barrier();
    const f32x4_t* got = reinterpret_cast<const f32x4_t*>(lds) + (wt * 2 + kg) * 2 * NB * 64;
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const f32x4_t o = got[(ii * NB + j) * 64 + lane];
        // fixed order: first k-half plus second k-half
        if (kg == 0) acc[ii][j] = acc[ii][j] + o;
        else acc[2 + ii][j] = o + acc[2 + ii][j];
      }
    i_begin = kg * 2;
    i_end = i_begin + 2;
  }

  if constexpr (sizeof(TC) == 2) {
    if (epilogue_can_stage(g)) {
      epilogue_tile16_staged<NB>(g, C, AUX, acc, m0 + wm, n0 + wn, i_begin, i_end, stg);
      return;
    }
  }
  epilogue_tile16<TC, NB>(g, C, AUX, acc, m0 + wm, n0 + wn, i_begin, i_end);
}

// LDS behind the ring for the epilogue staging of the waves (of `waves`, one wave per output block) whose slice does
// not fit one ring stage
template <int NB>
constexpr int w48_stage_spill(int stage_bytes, int waves) {
  const int fit = stage_bytes / epilogue_stage_bytes<NB>();
  return waves > fit ? (waves - fit) * epilogue_stage_bytes<NB>() : 0;
}

template <int WGM, int WGN, int NB, int NS, int KS, int NP, typename TC>
static bool launch_w48s_inst(const GemmDev& d, hipStream_t st) {
  constexpr int BM = 64 * WGM, BN = 16 * NB * WGN;
  constexpr int RING_BYTES = NS * (BM / 8 + BN / 8) * 1024 +
                             (KS == 1 ? w48_stage_spill<NB>((BM / 8 + BN / 8) * 1024, WGM * WGN) : 0);
  constexpr int XCH_BYTES = KS == 2 ? WGM * WGN * 2 * 2 * NB * 64 * 16 : 0;   // accumulator exchange of the wave pairs
  constexpr int LDS_BYTES = RING_BYTES > XCH_BYTES ? RING_BYTES : XCH_BYTES;
  static_assert(LDS_BYTES <= 160 * 1024, "ring exceeds the LDS of a CU");
  static_assert((NS - 2) * ((BM / 8 + BN / 8 + NP - 1) / NP) <= 24, "in-flight loads exceed wait_vmcnt_dyn");
  static_assert(64 * (WGM * WGN * KS + NP) <= 1024, "workgroup too large");
  auto kern = gemm_bf16_w48s_kernel<WGM, WGN, NB, NS, KS, NP, TC>;
  static LdsLimitOnce lds_limit;   // per instantiation
  if (!lds_limit.ensure((const void*)kern, LDS_BYTES)) return false;
  const int tiles_m = (d.M + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
  const int ntile = tiles_m * tiles_n;
  dim3 grid(((ntile + 7) / 8) * 8);
  hipLaunchKernelGGL(kern, grid, dim3(64 * (WGM * WGN * KS + NP)), LDS_BYTES, st, d, tiles_m, tiles_n);
  return true;
}

template <int WGM, int WGN, int NS, int KS, typename TC, int NB = 3>
static bool launch_w48_inst(const GemmDev& d, hipStream_t st) {
  constexpr int BM = 64 * WGM, BN = 16 * NB * WGN;
  constexpr int RING_BYTES = NS * (BM / 8 + BN / 8) * 1024 +
                             (KS == 1 ? w48_stage_spill<NB>((BM / 8 + BN / 8) * 1024, WGM * WGN) : 0);
  constexpr int XCH_BYTES = KS == 2 ? WGM * WGN * 2 * 2 * NB * 64 * 16 : 0;   // accumulator exchange of the wave pairs
  constexpr int LDS_BYTES = RING_BYTES > XCH_BYTES ? RING_BYTES : XCH_BYTES;
  static_assert(LDS_BYTES <= 160 * 1024, "ring exceeds the LDS of a CU");
  static_assert((NS - 2) * ((BM / 8 + BN / 8 + WGM * WGN * KS - 1) / (WGM * WGN * KS)) <= 24, "in-flight loads exceed wait_vmcnt_dyn");
  auto kern = gemm_bf16_w48_kernel<WGM, WGN, NS, KS, TC, NB>;
  static LdsLimitOnce lds_limit;   // per instantiation
  if (!lds_limit.ensure((const void*)kern, LDS_BYTES)) return false;
  const int tiles_m = (d.M + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
  const int ntile = tiles_m * tiles_n;
  dim3 grid(((ntile + 7) / 8) * 8);
  hipLaunchKernelGGL(kern, grid, dim3(64 * WGM * WGN * KS), LDS_BYTES, st, d, tiles_m, tiles_n);
  return true;
}

// 128x128 tiles, 8 wavefronts (2 x 4), two 32 KiB stages, two workgroups per CU (16 waves): the variant for a
// K-major A with an MN-major B (products against an untransposed row-major weight, e.g. the tied decoder of the
// MLM head) when there are enough tiles for two workgroups per CU.
template <bool AK, bool BKM, typename TC>
static bool launch_pipe_layout(const GemmDev& d, int batch, hipStream_t st) {
  return launch_pipe_inst<128, 128, 2, 4, AK, BKM, TC, 2>(d, batch, st);
}

bool launch_gemm_pipe(const GemmDev& d, int a_kmajor, int b_kmajor, int out_f32, int batch, hipStream_t st) {
  if (d.K % PBK) return false;
  if (out_f32) return false;
  // per-head attention products (N = 64, contraction <= 128): the whole problem fits the ring, so every load is
  // issued before the first barrier instead of one memory round trip per k-step
  if (!b_kmajor && d.N == 64 && d.K <= 2 * PBK && d.M >= 128 && d.M % 128 == 0) {
    if (a_kmajor) return launch_pipe_inst<128, 64, 2, 2, true, false, bf16_t, 3>(d, batch, st);
    return launch_pipe_inst<128, 64, 2, 2, false, false, bf16_t, 3>(d, batch, st);
  }
  if (d.M < 128 || d.N < 128 || batch != 1) return false;
  const long tiles = (long)((d.M + 127) / 128) * ((d.N + 127) / 128);
  if (a_kmajor && b_kmajor) {
    // Tile choice.  Every CU has to work through ceil(tiles / 256) tiles, so the cost of a tiling is that count
    // times the tile area; among equals the larger tile fetches fewer bytes per flop, then the squarer one.
    struct Cand { int bm, bn; };
    static const Cand cands[] = {{128, 128}, {128, 96}, {128, 144}, {128, 192}, {256, 144}, {256, 192}, {256, 256}};
    int best = 0;
    long best_cost = 0, best_area = 0, best_perim = 0;
    for (int i = 0; i < 7; ++i) {
      const Cand& c = cands[i];
      if (i > 0 && d.N % c.bn) continue;
      const long tl = (long)((d.M + c.bm - 1) / c.bm) * ((d.N + c.bn - 1) / c.bn);
      const long area = (long)c.bm * c.bn, cost = ((tl + 255) / 256) * area, perim = c.bm + c.bn;
      if (i == 0 || cost < best_cost || (cost == best_cost && (area > best_area || (area == best_area && perim < best_perim)))) {
        best = i; best_cost = cost; best_area = area; best_perim = perim;
      }
    }
    switch (best) {
      // one 128x96 tile per CU: 8 consumer + 8 producer waves, three stages (measured 24 us against 33 us for the
      // 4096x768x3072 product)
      case 1: return launch_w48s_inst<2, 2, 3, 3, 2, 8, bf16_t>(d, st);
      case 2: return launch_w48s_inst<2, 3, 3, 3, 2, 4, bf16_t>(d, st);   // 128x144: 12 + 4 waves
      case 3: return launch_w48s_inst<2, 4, 3, 3, 1, 8, bf16_t>(d, st);   // 128x192: 8 + 8 waves
      case 4: return launch_w48s_inst<4, 3, 3, 3, 1, 4, bf16_t>(d, st);   // 256x144: 12 + 4 waves
      case 5: {
        // 256x192: two stages only (112 KiB).  8 consumer waves with 64x96 wave tiles + 4 producers reach 975 TFLOP/s
        // on a 3072-deep contraction (16 symmetric waves: 840), but run the epilogue on half the waves, which costs
        // more than the loop gains on a 768-deep one whenever the epilogue does more than add a bias (GeLU forward
        // 40 against 56 us, multiply by the saved derivative 28 against 34 us).
        const bool heavy_epilogue = d.epilogue == EPI_BIAS_GELU || d.epilogue == EPI_MUL_GELU_GRAD ||
                                    d.epilogue == EPI_BIAS_GELU_DERIV || d.epilogue == EPI_MUL_AUX;
        if (heavy_epilogue && d.K <= 1536) return launch_w48_inst<4, 4, 2, 1, bf16_t>(d, st);
        return launch_w48s_inst<4, 2, 6, 2, 1, 4, bf16_t>(d, st);
      }
      // 256x256 (a 4096 x 4096 output: one tile per CU instead of four 128x128 ones, half the operand bytes per
      // flop): 16 symmetric waves with 64x64 wave tiles, two stages.  Measured on 4096 x 4096 x 1024: 35 us against
      // 56 us (bias), 50 against 78 (GeLU + derivative); 1.2 PFLOP/s on a 4096-deep contraction.  The
      // producer/consumer form would need 8 computing waves with 64x128 wave tiles, which do not fit the registers
      // of three waves per SIMD (146 spilled).
      case 6: return launch_w48_inst<4, 4, 2, 1, bf16_t, 4>(d, st);
      default: break;
    }
    // 128x128: the same producer/consumer kernel with 64x64 wave tiles
    return launch_w48s_inst<2, 2, 4, 3, 2, 8, bf16_t>(d, st);
  }
  // with a transposed B operand the ring only wins when there are enough tiles
  // for two workgroups per CU; below that the register-staged kernel is faster
  if (a_kmajor && !b_kmajor && tiles >= 384) return launch_pipe_layout<true, false, bf16_t>(d, batch, st);
  return false;
}

}  // namespace raf
