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

template <typename TC>
__device__ __forceinline__ void epilogue_store4(const GemmDev& g, TC* __restrict__ c, bf16_t* __restrict__ aux, int i,
                                                int j, float (&v)[4]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] *= g.alpha;
  if (g.epilogue == EPI_BIAS || g.epilogue == EPI_BIAS_GELU) {
    const float4 b = *reinterpret_cast<const float4*>(g.bias + j);
    v[0] += b.x; v[1] += b.y; v[2] += b.z; v[3] += b.w;
  }
  if (g.epilogue == EPI_BIAS_GELU) {
    store4(aux + (long)i * g.ldaux + j, v);
    // GeLU is evaluated on the value the backward pass will read back
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = gelu_f((float)(bf16_t)v[e], g.gelu_tanh);
  } else if (g.epilogue == EPI_MUL_GELU_GRAD) {
    float u[4];
    load4(aux + (long)i * g.ldaux + j, u);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] *= gelu_grad_f(u[e], g.gelu_tanh);
  } else if (g.epilogue == EPI_ADD_RES) {
    float r[4];
    load4(aux + (long)i * g.ldaux + j, r);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += r[e];
  }
  store4(c + (long)i * g.ldc + j, v);
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
  int count;
};

// Weight-gradient group (both operands MN-major, float output) on the
// producer/consumer direct-to-LDS kernel (gemm_pipe.hip); false when a problem
// does not fit it (K % 64, sizes below one tile).
bool launch_gemm_group_spec(const GemmDev* ds, int count, hipStream_t st);

// Pipelined direct-to-LDS kernel family (gemm_pipe.hip).  Returns false when
// the problem does not meet its requirements (K % 64, tile fit) and the
// caller must use the staged kernel instead.
bool launch_gemm_pipe(const GemmDev& d, int a_kmajor, int b_kmajor, int out_f32, int batch, hipStream_t st);

}  // namespace raf
