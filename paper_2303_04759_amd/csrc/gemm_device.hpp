// Device-side pieces shared by the GEMM kernels: the launch descriptor and the
// fused epilogues (bias, bias+GeLU with saved pre-activation, GeLU-gradient
// multiply, residual add, scale, fp32 output).
#pragma once
#include "common.hpp"

namespace raf {

struct GemmDev {
  int M, N, K;
  const void* a; long lda;
  const void* b; long ldb;
  void* c; long ldc;
  float alpha;
  int epilogue;
  const float* bias;
  void* aux; long ldaux;
  int gelu_tanh;
  int nz_inner;
  long sa0, sa1, sb0, sb1, sc0, sc1;
};

template <typename TC, typename TAUX>
__device__ __forceinline__ float epilogue_value(const GemmDev& g, TAUX* __restrict__ aux, int i, int j, float acc) {
  float v = acc * g.alpha;
  switch (g.epilogue) {
    case EPI_BIAS:
      v += g.bias[j];
      break;
    case EPI_BIAS_GELU: {
      v += g.bias[j];
      aux[(long)i * g.ldaux + j] = (TAUX)v;
      // GeLU is evaluated on the value the backward pass will read back
      v = gelu_f((float)(TAUX)v, g.gelu_tanh);
      break;
    }
    case EPI_MUL_GELU_GRAD:
      v *= gelu_grad_f((float)aux[(long)i * g.ldaux + j], g.gelu_tanh);
      break;
    case EPI_ADD_RES:
      v += (float)aux[(long)i * g.ldaux + j];
      break;
    case EPI_BIAS_GELU_DERIV: {
      v += g.bias[j];
      float y, dy;
      gelu_and_grad_f(v, g.gelu_tanh, y, dy);
      aux[(long)i * g.ldaux + j] = (TAUX)dy;
      v = y;
      break;
    }
    case EPI_MUL_AUX:
      v *= (float)aux[(long)i * g.ldaux + j];
      break;
    default:
      break;
  }
  return v;
}

template <typename TC, typename TAUX>
__device__ __forceinline__ void epilogue_store(const GemmDev& g, TC* __restrict__ c, TAUX* __restrict__ aux, int i,
                                               int j, float acc) {
  c[(long)i * g.ldc + j] = (TC)epilogue_value<TC, TAUX>(g, aux, i, j, acc);
}

// four consecutive columns j..j+3 of row i (j a multiple of 4; all pointers and
// leading dimensions keep 8-byte alignment of such groups)
__device__ __forceinline__ void load4(const bf16_t* p, float (&o)[4]) {
  const uint2 r = *reinterpret_cast<const uint2*>(p);
  o[0] = bf16_bits_to_f32(r.x & 0xffffu); o[1] = __uint_as_float(r.x & 0xffff0000u);
  o[2] = bf16_bits_to_f32(r.y & 0xffffu); o[3] = __uint_as_float(r.y & 0xffff0000u);
}
__device__ __forceinline__ void store4(bf16_t* p, const float (&v)[4]) {
  uint2 r;
  r.x = pack_bf16x2(v[0], v[1]);
  r.y = pack_bf16x2(v[2], v[3]);
  *reinterpret_cast<uint2*>(p) = r;
}
__device__ __forceinline__ void store4(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}

// The epilogue kind is a template parameter here and the kernels switch on it once, outside their unrolled store
// loops: with the run-time switch inside, every one of the 12-64 store groups of a wave carried all cases and the
// epilogue of the plain-bias GEMMs slowed down by several microseconds when a case was added.
template <typename TC, int EPI>
__device__ __forceinline__ void epilogue_store4(const GemmDev& g, TC* __restrict__ c, bf16_t* __restrict__ aux, int i,
                                                int j, float (&v)[4]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] *= g.alpha;
  if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_GELU_DERIV) {
    const float4 b = *reinterpret_cast<const float4*>(g.bias + j);
    v[0] += b.x; v[1] += b.y; v[2] += b.z; v[3] += b.w;
  }
  if constexpr (EPI == EPI_BIAS_GELU) {
    store4(aux + (long)i * g.ldaux + j, v);
    // GeLU is evaluated on the value the backward pass will read back
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = gelu_f((float)(bf16_t)v[e], g.gelu_tanh);
  } else if constexpr (EPI == EPI_MUL_GELU_GRAD) {
    float u[4];
    load4(aux + (long)i * g.ldaux + j, u);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] *= gelu_grad_f(u[e], g.gelu_tanh);
  } else if constexpr (EPI == EPI_ADD_RES) {
    float r[4];
    load4(aux + (long)i * g.ldaux + j, r);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += r[e];
  } else if constexpr (EPI == EPI_BIAS_GELU_DERIV) {
    float dy[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) gelu_and_grad_f(v[e], g.gelu_tanh, v[e], dy[e]);
    store4(aux + (long)i * g.ldaux + j, dy);
  } else if constexpr (EPI == EPI_MUL_AUX) {
    float r[4];
    load4(aux + (long)i * g.ldaux + j, r);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] *= r[e];
  }
  store4(c + (long)i * g.ldc + j, v);
}

template <int V>
struct EpiTag {
  static constexpr int value = V;
};
template <typename F>
__device__ __forceinline__ void epilogue_dispatch(int epi, F&& f) {
  switch (epi) {
    case EPI_BIAS: f(EpiTag<EPI_BIAS>{}); break;
    case EPI_BIAS_GELU: f(EpiTag<EPI_BIAS_GELU>{}); break;
    case EPI_MUL_GELU_GRAD: f(EpiTag<EPI_MUL_GELU_GRAD>{}); break;
    case EPI_ADD_RES: f(EpiTag<EPI_ADD_RES>{}); break;
    case EPI_BIAS_GELU_DERIV: f(EpiTag<EPI_BIAS_GELU_DERIV>{}); break;
    case EPI_MUL_AUX: f(EpiTag<EPI_MUL_AUX>{}); break;
    default: f(EpiTag<EPI_NONE>{}); break;
  }
}

// A wave's TM x TN blocks of the (transposed) 32x32 MFMA result: register r of lane l holds output row (l & 31),
// column 8*(r/4) + 4*(l/32) + r%4 of its block.  row0 / col0: the wave tile's origin.
template <typename TC, int TM, int TN>
__device__ __forceinline__ void epilogue_tile32(const GemmDev& g, TC* __restrict__ C, bf16_t* __restrict__ AUX,
                                                f32x16_t (&acc)[TM][TN], int row0, int col0) {
  const int lane = threadIdx.x & 63;
  epilogue_dispatch(g.epilogue, [&](auto tag) {
    constexpr int EPI = decltype(tag)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = row0 + i * 32 + (lane & 31);
      if (row < g.M) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int col = col0 + j * 32 + 8 * q + 4 * (lane >> 5);
            if (col < g.N) {
              float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
              epilogue_store4<TC, EPI>(g, C, AUX, row, col, v);
            }
          }
      }
    }
  });
}

// A wave's 4 x NB blocks of the (transposed) 16x16 MFMA result: a lane holds output row (l & 15) and the 4
// consecutive columns 4*(l>>4) + r of each block; only row blocks [i_begin, i_end) are written.
template <typename TC, int NB>
__device__ __forceinline__ void epilogue_tile16(const GemmDev& g, TC* __restrict__ C, bf16_t* __restrict__ AUX,
                                                f32x4_t (&acc)[4][NB], int row0, int col0, int i_begin, int i_end) {
  const int lane = threadIdx.x & 63;
  epilogue_dispatch(g.epilogue, [&](auto tag) {
    constexpr int EPI = decltype(tag)::value;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i < i_begin || i >= i_end) continue;
      const int row = row0 + i * 16 + (lane & 15);
      if (row < g.M) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const int col = col0 + j * 16 + 4 * (lane >> 4);
          if (col < g.N) {
            float v[4] = {acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
            epilogue_store4<TC, EPI>(g, C, AUX, row, col, v);
          }
        }
      }
    }
  });
}


// Bytes of LDS one wave needs for epilogue_tile16_staged.
template <int NB>
constexpr int epilogue_stage_bytes() {
  return 2 * 16 * (32 * NB + 16);
}

// True when the output (and aux) rows of a problem can be written 16 bytes at a time.
__device__ __forceinline__ bool epilogue_can_stage(const GemmDev& g) {
  const unsigned long long p = (unsigned long long)g.c | (unsigned long long)g.aux;
  return ((g.ldc | g.ldaux | (long)g.N) & 7) == 0 && (p & 15) == 0;
}

// Same result as epilogue_tile16 for bf16 outputs, written through a wave-private LDS buffer: the accumulator
// layout gives a lane 4 columns of one row, so a direct store instruction touches 16 rows with 32 bytes each, and
// such stores cost several times the time of full-row ones (5.5 us against 0.7 us for the 19-MB output of a
// 4096 x 2304 product).  The blocks are therefore finished in registers, laid out row-major in LDS and written
// (aux operands: read) as 16-byte pieces that run along the rows of the wave tile: two 16-row blocks per trip, an
// aux operand being replaced in place by the result; one block per trip with two buffers for the epilogues that
// write a second output.  LDS operations of one wave execute in order, so no barrier is needed; `stg` must not be
// touched by any other wave.
template <int NB>
__device__ __forceinline__ void epilogue_tile16_staged(const GemmDev& g, bf16_t* __restrict__ C,
                                                       bf16_t* __restrict__ AUX, f32x4_t (&acc)[4][NB], int row0,
                                                       int col0, int i_begin, int i_end, char* stg) {
  constexpr int P = 32 * NB + 16;         // row pitch in LDS, bytes
  constexpr int CPR = 2 * NB;             // 16-byte pieces per row
  const int lane = threadIdx.x & 63;
  const int lr = lane & 15, lg = lane >> 4;
  epilogue_dispatch(g.epilogue, [&](auto tag) {
    constexpr int EPI = decltype(tag)::value;
    constexpr bool AUX_IN = EPI == EPI_MUL_GELU_GRAD || EPI == EPI_ADD_RES || EPI == EPI_MUL_AUX;
    constexpr bool AUX_OUT = EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_GELU_DERIV;
    constexpr bool BIAS = EPI == EPI_BIAS || EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_GELU_DERIV;
    constexpr int BLK = AUX_OUT ? 1 : 2;  // row blocks per trip through LDS
    constexpr int ROWS = 16 * BLK, NCH = ROWS * CPR, IT = (NCH + 63) / 64;
    char* s_out = stg;
    char* s_aux = AUX_OUT ? stg + 16 * P : stg;
    // piece `it` of this lane: row and 16-byte column within a trip
    int pr[IT], pc[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
      const int q = it * 64 + lane;
      pr[it] = q / CPR;
      pc[it] = q - pr[it] * CPR;
    }
    // aux pieces of one trip; the next trip's are requested as soon as these have gone to LDS
    uint4 ain[IT];
    auto load_aux = [&](int t) {
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const int row = row0 + t * ROWS + pr[it], col = col0 + pc[it] * 8;
        ain[it] = make_uint4(0u, 0u, 0u, 0u);
        if (pr[it] < ROWS && row < g.M && col < g.N)
          ain[it] = *reinterpret_cast<const uint4*>(AUX + (long)row * g.ldaux + col);
      }
    };
    if constexpr (AUX_IN) load_aux(i_begin / BLK);
    float4 bias[BIAS ? NB : 1];
    if constexpr (BIAS) {
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int col = col0 + j * 16 + 4 * lg;
        bias[j] = col < g.N ? *reinterpret_cast<const float4*>(g.bias + col) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int t = 0; t < 4 / BLK; ++t) {
      if (t * BLK < i_begin || t * BLK >= i_end) continue;
      if constexpr (AUX_IN) {
#pragma unroll
        for (int it = 0; it < IT; ++it)
          if (pr[it] < ROWS) *reinterpret_cast<uint4*>(s_aux + pr[it] * P + pc[it] * 16) = ain[it];
        if ((t + 1) * BLK < i_end) load_aux(t + 1);
      }
#pragma unroll
      for (int b = 0; b < BLK; ++b)
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const int i = t * BLK + b;
          const int off = (b * 16 + lr) * P + j * 32 + lg * 8;
          float v[4] = {acc[i][j][0] * g.alpha, acc[i][j][1] * g.alpha, acc[i][j][2] * g.alpha, acc[i][j][3] * g.alpha};
          if constexpr (BIAS) {
            v[0] += bias[j].x; v[1] += bias[j].y; v[2] += bias[j].z; v[3] += bias[j].w;
          }
          if constexpr (EPI == EPI_BIAS_GELU) {
            store4(reinterpret_cast<bf16_t*>(s_aux + off), v);
            // GeLU is evaluated on the value the backward pass will read back
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = gelu_fast((float)(bf16_t)v[e], g.gelu_tanh);
          } else if constexpr (EPI == EPI_BIAS_GELU_DERIV) {
            float dy[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) gelu_and_grad_fast(v[e], g.gelu_tanh, v[e], dy[e]);
            store4(reinterpret_cast<bf16_t*>(s_aux + off), dy);
          } else if constexpr (AUX_IN) {
            float u[4];
            load4(reinterpret_cast<const bf16_t*>(s_aux + off), u);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if constexpr (EPI == EPI_MUL_GELU_GRAD) v[e] *= gelu_grad_fast(u[e], g.gelu_tanh);
              else if constexpr (EPI == EPI_ADD_RES) v[e] += u[e];
              else v[e] *= u[e];
            }
          }
          store4(reinterpret_cast<bf16_t*>(s_out + off), v);
        }
#pragma unroll
      for (int it = 0; it < IT; ++it) {
        const int row = row0 + t * ROWS + pr[it], col = col0 + pc[it] * 8;
        if (pr[it] < ROWS && row < g.M && col < g.N) {
          *reinterpret_cast<uint4*>(C + (long)row * g.ldc + col) =
              *reinterpret_cast<const uint4*>(s_out + pr[it] * P + pc[it] * 16);
          if constexpr (AUX_OUT)
            *reinterpret_cast<uint4*>(AUX + (long)row * g.ldaux + col) =
                *reinterpret_cast<const uint4*>(s_aux + pr[it] * P + pc[it] * 16);
        }
      }
    }
  });
}

// Float outputs of the 32x32 layout without elementwise epilogue (weight gradients), one 32x32 block per trip
// through a wave-private LDS buffer of epilogue_stage32_bytes: a direct store instruction writes 32-byte pieces of
// 32 rows, the staged one whole 128-byte rows.
constexpr int epilogue_stage32_bytes = 32 * (128 + 16);
__device__ __forceinline__ bool epilogue_can_stage32(const GemmDev& g) {
  return g.epilogue == EPI_NONE && ((g.ldc | (long)g.N) & 3) == 0 && ((unsigned long long)g.c & 15) == 0;
}
template <int TM, int TN>
__device__ __forceinline__ void epilogue_tile32_staged(const GemmDev& g, float* __restrict__ C,
                                                       f32x16_t (&acc)[TM][TN], int row0, int col0, char* stg) {
  constexpr int P = 128 + 16;
  const int lane = threadIdx.x & 63;
  const int wr = lane & 31, wh = lane >> 5;     // accumulator layout: row, which 4 of every 8 columns
  const int rr = lane >> 3, rc = lane & 7;      // copy-out: row within 8, 16-byte piece of the row
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4*>(stg + wr * P + q * 32 + wh * 16) =
            make_float4(acc[i][j][4 * q] * g.alpha, acc[i][j][4 * q + 1] * g.alpha, acc[i][j][4 * q + 2] * g.alpha,
                        acc[i][j][4 * q + 3] * g.alpha);
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int r = it * 8 + rr;
        const int row = row0 + i * 32 + r, col = col0 + j * 32 + rc * 4;
        if (row < g.M && col < g.N)
          *reinterpret_cast<float4*>(C + (long)row * g.ldc + col) = *reinterpret_cast<const float4*>(stg + r * P + rc * 16);
      }
    }
}

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

// Several independent problems of one layout in a single launch; tile_start[p]
// is the first linear tile of problem p, tiles_n[p] its tile columns.
constexpr int GEMM_GROUP_MAX = 4;
struct GemmGroupDev {
  GemmDev p[GEMM_GROUP_MAX];
  int tile_start[GEMM_GROUP_MAX + 1];
  int tiles_n[GEMM_GROUP_MAX];
  // > 0: the problem's tiles are numbered along M first (that many row tiles), so that a contiguous share of the tile
  // list covers whole strips of the side with fewer tiles; 0: along N first
  int tiles_m_first[GEMM_GROUP_MAX];
  int count;
};


// Column sums out[j][c] = sum_r x[j][r*ld + c] of up to two bf16 matrices with the same row count (the bias
// gradients next to the weight gradients), taken by workgroups of the weight-gradient launch that would otherwise
// find no tile: the grouped launch of a BERT-base layer has 216 tiles for 256 CUs.
struct ColsumSide {
  const bf16_t* x[2];
  float* out[2];
  long ld[2];
  int cols[2];     // multiples of 8; cols[1] = 0 for a single matrix
  long rows;
  int count;       // 0: no side work
  // second stages of earlier two-stage column sums (sums over partial rows, see ReduceJob), taken after the above
  ReduceJob red[3];
  int nred;
  // not null: set to 1 when any sum written here, or any weight-gradient value of the launch's tiles, is inf or nan
  int* nonfinite;
};

// Weight-gradient group (both operands MN-major, float output) on the
// producer/consumer direct-to-LDS kernel (gemm_pipe.hip); false when a problem
// does not fit it (K % 64, sizes below one tile).  side: optional column sums; *side_taken tells whether the launch
// computed them (it does when enough CUs are left without a tile), otherwise the caller has to.
// side->nonfinite is honoured only when the side work is taken (*side_taken).
bool launch_gemm_group_spec(const GemmDev* ds, int count, hipStream_t st, const ColsumSide* side = nullptr,
                            bool* side_taken = nullptr);

// Pipelined direct-to-LDS kernel family (gemm_pipe.hip).  Returns false when
// the problem does not meet its requirements (K % 64, tile fit) and the
// caller must use the staged kernel instead.
bool launch_gemm_pipe(const GemmDev& d, int a_kmajor, int b_kmajor, int out_f32, int batch, hipStream_t st);

}  // namespace raf
