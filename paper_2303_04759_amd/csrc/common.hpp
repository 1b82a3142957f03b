// Shared device helpers for the gfx950 kernels: 8-wide typed vector access,
// bf16 conversion, the Philox4x32-10 dropout generator, wavefront reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "raf_mi355.h"

namespace raf {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int WAVE = 64;

// ---------------------------------------------------------------- status --
void set_hip_error(hipError_t e);
inline raf_status check_launch() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_hip_error(e);
    return RAF_EHIP;
  }
  return RAF_OK;
}
// Raises a kernel's dynamic-LDS limit once per device.  One object per kernel instantiation (a function-local
// static); safe from several host threads: two racing callers both set the same value.
struct LdsLimitOnce {
  std::atomic<uint64_t> done{0};
  bool ensure(const void* kern, int bytes) {
    int dev = 0;
    const bool tracked = hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64;
    const uint64_t bit = tracked ? (uint64_t)1 << dev : 0;
    if (tracked && (done.load(std::memory_order_acquire) & bit)) return true;
    const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) {   // recorded for raf_last_hip_error and cleared: callers may fall back to another kernel
      (void)hipGetLastError();
      set_hip_error(e);
      return false;
    }
    done.fetch_or(bit, std::memory_order_release);
    return true;
  }
};

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ------------------------------------------------------- typed 8-vectors --
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t hi16) { return __uint_as_float(hi16 << 16); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  // round-to-nearest-even; lowers to v_cvt_pk_bf16_f32 on gfx950
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  bf16x2_t v = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, v);
}

template <typename T>
struct Vec8;

template <>
struct Vec8<float> {
  static __device__ __forceinline__ void load(const float* p, float (&o)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
  // value as it will read back from storage
  static __device__ __forceinline__ float round(float v) { return v; }
  // 8 elements as loaded, converted to float later (lets a kernel request the next row before it works on this one)
  struct Raw { float4 a, b; };
  static __device__ __forceinline__ Raw load_raw(const float* p) {
    return Raw{*reinterpret_cast<const float4*>(p), *reinterpret_cast<const float4*>(p + 4)};
  }
  static __device__ __forceinline__ void unpack(const Raw& r, float (&o)[8]) {
    o[0] = r.a.x; o[1] = r.a.y; o[2] = r.a.z; o[3] = r.a.w;
    o[4] = r.b.x; o[5] = r.b.y; o[6] = r.b.z; o[7] = r.b.w;
  }
};

template <>
struct Vec8<bf16_t> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&o)[8]) {
    const uint4 r = *reinterpret_cast<const uint4*>(p);
    o[0] = bf16_bits_to_f32(r.x & 0xffffu); o[1] = __uint_as_float(r.x & 0xffff0000u);
    o[2] = bf16_bits_to_f32(r.y & 0xffffu); o[3] = __uint_as_float(r.y & 0xffff0000u);
    o[4] = bf16_bits_to_f32(r.z & 0xffffu); o[5] = __uint_as_float(r.z & 0xffff0000u);
    o[6] = bf16_bits_to_f32(r.w & 0xffffu); o[7] = __uint_as_float(r.w & 0xffff0000u);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    uint4 r;
    r.x = pack_bf16x2(v[0], v[1]);
    r.y = pack_bf16x2(v[2], v[3]);
    r.z = pack_bf16x2(v[4], v[5]);
    r.w = pack_bf16x2(v[6], v[7]);
    *reinterpret_cast<uint4*>(p) = r;
  }
  static __device__ __forceinline__ float round(float v) { return (float)(__bf16)v; }
  typedef uint4 Raw;
  static __device__ __forceinline__ Raw load_raw(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
  static __device__ __forceinline__ void unpack(const Raw& r, float (&o)[8]) {
    o[0] = bf16_bits_to_f32(r.x & 0xffffu); o[1] = __uint_as_float(r.x & 0xffff0000u);
    o[2] = bf16_bits_to_f32(r.y & 0xffffu); o[3] = __uint_as_float(r.y & 0xffff0000u);
    o[4] = bf16_bits_to_f32(r.z & 0xffffu); o[5] = __uint_as_float(r.z & 0xffff0000u);
    o[6] = bf16_bits_to_f32(r.w & 0xffffu); o[7] = __uint_as_float(r.w & 0xffff0000u);
  }
};

__device__ __forceinline__ void load8f(const float* p, float (&o)[8]) { Vec8<float>::load(p, o); }

// ----------------------------------------------------------------- Philox --
// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies
// with a Weyl-sequence key schedule.
struct Philox4 {
  uint32_t x, y, z, w;
};

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                 uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one 32x32->64 multiply per product (v_mad_u64_u32) instead of separate high and low multiplies
    const uint64_t p0 = (uint64_t)M0 * c0, p1 = (uint64_t)M1 * c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    // three-input xor in one instruction (v_bitop3_b32, truth table 0x96)
    const uint32_t n0 = __builtin_amdgcn_bitop3_b32(hi1, c1, k0, 0x96);
    const uint32_t n2 = __builtin_amdgcn_bitop3_b32(hi0, c3, k1, 0x96);
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += W0;
    k1 += W1;
    // the key is wave-uniform: keep its schedule as two scalar adds per round; hoisted out of the callers' loops, the
    // twenty round keys do not fit the scalar registers and come back through v_readlane, two extra instructions per xor
    asm volatile("" : "+s"(k0), "+s"(k1));
  }
  return Philox4{c0, c1, c2, c3};
}

// Everything a kernel needs to regenerate one dropout site's mask.
struct DropSite {
  uint32_t k0, k1;      // seed lo, hi
  uint32_t c1, c2, c3;  // step hi, site | layer<<8, step lo
  uint32_t thr;         // keep iff the element's 16 random bits are >= thr
  float scale;          // 1/(1-p)
  int enabled;          // 0: p == 0 or no dropout at this call
};

inline DropSite make_drop_site(const raf_layer_desc& d, int site, uint64_t step) {
  DropSite s;
  s.k0 = (uint32_t)(d.seed & 0xffffffffu);
  s.k1 = (uint32_t)(d.seed >> 32);
  s.c1 = (uint32_t)(step >> 32);
  s.c2 = ((uint32_t)site & 0xffu) | ((d.layer_id & 0xffffffu) << 8);
  s.c3 = (uint32_t)(step & 0xffffffffu);
  const double t = d.dropout_p * 65536.0;
  s.thr = (uint32_t)t;  // floor for t >= 0
  s.scale = (float)(1.0 / (1.0 - d.dropout_p));
  s.enabled = (site != 0 && d.dropout_p > 0.0) ? 1 : 0;
  return s;
}

// keep-multipliers (0 or scale) for 8 consecutive elements starting at flat
// index idx8 (a multiple of 8): one Philox block, 16 bits per element (the
// 32x32 multiplies of the generator are the main arithmetic cost of every
// kernel with a dropout site, so no output bit is thrown away beyond that).
__device__ __forceinline__ void drop_mult8(const DropSite& s, uint64_t idx8, float (&mult)[8]) {
  const Philox4 a = philox4x32_10((uint32_t)(idx8 >> 3), s.c1, s.c2, s.c3, s.k0, s.k1);
  mult[0] = (a.x & 0xffffu) >= s.thr ? s.scale : 0.f; mult[1] = (a.x >> 16) >= s.thr ? s.scale : 0.f;
  mult[2] = (a.y & 0xffffu) >= s.thr ? s.scale : 0.f; mult[3] = (a.y >> 16) >= s.thr ? s.scale : 0.f;
  mult[4] = (a.z & 0xffffu) >= s.thr ? s.scale : 0.f; mult[5] = (a.z >> 16) >= s.thr ? s.scale : 0.f;
  mult[6] = (a.w & 0xffffu) >= s.thr ? s.scale : 0.f; mult[7] = (a.w >> 16) >= s.thr ? s.scale : 0.f;
}

// the same, and the decisions as bits (bit e = element idx8 + e is kept)
__device__ __forceinline__ void drop_mult8_bits(const DropSite& s, uint64_t idx8, float (&mult)[8], uint32_t& bits) {
  const Philox4 a = philox4x32_10((uint32_t)(idx8 >> 3), s.c1, s.c2, s.c3, s.k0, s.k1);
  const uint32_t f[8] = {a.x & 0xffffu, a.x >> 16, a.y & 0xffffu, a.y >> 16, a.z & 0xffffu, a.z >> 16, a.w & 0xffffu, a.w >> 16};
  bits = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const bool kept = f[e] >= s.thr;
    mult[e] = kept ? s.scale : 0.f;
    bits |= kept ? (1u << e) : 0u;
  }
}

// ------------------------------------------------------------- reductions --
template <int WIDTH>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = WIDTH / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
template <int WIDTH>
__device__ __forceinline__ float group_max(float v) {
#pragma unroll
  for (int o = WIDTH / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

// ------------------------------------------------------------------- GeLU --
// erf by the rational approximation 7.1.28 of Abramowitz & Stegun:
// erf(x) = 1 - (1 + a1 x + ... + a6 x^6)^-16 for x >= 0, |error| <= 3e-7;
// branch-free and about a third of the instructions of the library erff.
__device__ __forceinline__ float erf_as(float x) {
  const float ax = fabsf(x);
  float p = 0.0000430638f;
  p = fmaf(p, ax, 0.0002765672f);
  p = fmaf(p, ax, 0.0001520143f);
  p = fmaf(p, ax, 0.0092705272f);
  p = fmaf(p, ax, 0.0422820123f);
  p = fmaf(p, ax, 0.0705230784f);
  p = fmaf(p, ax, 1.0f);
  p = p * p;
  p = p * p;
  p = p * p;
  p = p * p;
  const float r = 1.0f - __frcp_rn(p);
  return copysignf(r, x);
}
__device__ __forceinline__ float gelu_f(float u, int tanh_form) {
  if (tanh_form) {
    const float k = 0.7978845608028654f;
    return 0.5f * u * (1.0f + tanhf(k * (u + 0.044715f * u * u * u)));
  }
  return 0.5f * u * (1.0f + erf_as(u * 0.7071067811865476f));
}
__device__ __forceinline__ float gelu_grad_f(float u, int tanh_form) {
  if (tanh_form) {
    const float k = 0.7978845608028654f;
    const float t = tanhf(k * (u + 0.044715f * u * u * u));
    return 0.5f * (1.0f + t) + 0.5f * u * (1.0f - t * t) * k * (1.0f + 0.134145f * u * u);
  }
  const float Phi = 0.5f * (1.0f + erf_as(u * 0.7071067811865476f));
  const float phi = 0.3989422804014327f * __expf(-0.5f * u * u);
  return Phi + u * phi;
}

// GeLU and its derivative at once (they share the erf / tanh evaluation)
__device__ __forceinline__ void gelu_and_grad_f(float u, int tanh_form, float& y, float& dy) {
  if (tanh_form) {
    const float k = 0.7978845608028654f;
    const float t = tanhf(k * (u + 0.044715f * u * u * u));
    y = 0.5f * u * (1.0f + t);
    dy = 0.5f * (1.0f + t) + 0.5f * u * (1.0f - t * t) * k * (1.0f + 0.134145f * u * u);
  } else {
    const float Phi = 0.5f * (1.0f + erf_as(u * 0.7071067811865476f));
    y = u * Phi;
    dy = Phi + u * (0.3989422804014327f * __expf(-0.5f * u * u));
  }
}

// Cheaper forms for results that are stored as bf16 (2^-9 relative): Phi(u) = (1 + erf(u / sqrt 2)) / 2 and
// phi(u) = exp(-u^2/2) / sqrt(2 pi) by the approximation 7.1.25 of Abramowitz & Stegun,
// erf(z) = 1 - (a1 t + a2 t^2 + a3 t^3) exp(-z^2), t = 1/(1 + p z), z >= 0, |error| <= 2.5e-5: with z = |u| / sqrt 2
// its exponential is exp(-u^2/2), the one phi needs, so GeLU and its derivative cost one v_exp_f32, one v_rcp_f32
// and about a dozen multiply-adds together (|Phi error| <= 1.1e-5, |gelu error| <= 2.6e-5).  The epilogue of the
// 4096 x 3072 product that applies both is bound by these instructions.
__device__ __forceinline__ void gauss_cdf_pdf_fast(float u, float& Phi, float& phi) {
  const float z = fabsf(u) * 0.7071067811865476f;
  const float t = __frcp_rn(fmaf(0.47047f, z, 1.0f));
  const float e = __builtin_amdgcn_exp2f(u * u * -0.7213475204444817f);   // exp(-u^2/2)
  const float poly = t * fmaf(t, fmaf(t, 0.7478556f, -0.0958798f), 0.3480242f);
  const float erf_abs = fmaf(-poly, e, 1.0f);
  Phi = fmaf(0.5f, copysignf(erf_abs, u), 0.5f);
  phi = 0.3989422804014327f * e;
}
__device__ __forceinline__ float gelu_fast(float u, int tanh_form) {
  if (tanh_form) return gelu_f(u, 1);
  float Phi, phi;
  gauss_cdf_pdf_fast(u, Phi, phi);
  return u * Phi;
}
__device__ __forceinline__ float gelu_grad_fast(float u, int tanh_form) {
  if (tanh_form) return gelu_grad_f(u, 1);
  float Phi, phi;
  gauss_cdf_pdf_fast(u, Phi, phi);
  return fmaf(u, phi, Phi);
}
__device__ __forceinline__ void gelu_and_grad_fast(float u, int tanh_form, float& y, float& dy) {
  if (tanh_form) {
    gelu_and_grad_f(u, 1, y, dy);
  } else {
    float Phi, phi;
    gauss_cdf_pdf_fast(u, Phi, phi);
    y = u * Phi;
    dy = fmaf(u, phi, Phi);
  }
}

// ---------------------------------------------------------- row geometry --
struct RowGeom {
  int lpr, nv;
};
inline RowGeom row_geom(int len) {
  const int nvec = len / 8;
  int lpr = 4;
  while (lpr < 64 && lpr < nvec) lpr <<= 1;
  int nv = 1;
  while (lpr * nv < nvec) nv <<= 1;
  // three vectors per lane keep every lane busy for rows of 3 * 2^k vectors (768 = 32 lanes x 3 x 8)
  if (lpr * nv != nvec && lpr >= 32 && (lpr / 2) * 3 == nvec) return RowGeom{lpr / 2, 3};
  if (lpr * nv != nvec && lpr == 64 && nvec == 192) return RowGeom{64, 3};
  return RowGeom{lpr, nv};
}

#define RAF_DISPATCH_GEOM(GEOM, CALL)                   \
  do {                                                  \
    const RowGeom _g = (GEOM);                          \
    if (_g.nv == 3 && _g.lpr == 16) { CALL(16, 3); }    \
    else if (_g.nv == 3 && _g.lpr == 32) { CALL(32, 3); } \
    else if (_g.nv == 3) { CALL(64, 3); }               \
    else if (_g.lpr == 4) { CALL(4, 1); }               \
    else if (_g.lpr == 8) { CALL(8, 1); }               \
    else if (_g.lpr == 16) { CALL(16, 1); }             \
    else if (_g.lpr == 32) { CALL(32, 1); }             \
    else if (_g.nv == 1) { CALL(64, 1); }               \
    else if (_g.nv == 2) { CALL(64, 2); }               \
    else if (_g.nv == 4) { CALL(64, 4); }               \
    else { CALL(64, 8); }                               \
  } while (0)

// --------------------------------------------------------- internal ops ---
// EPI_BIAS_GELU_DERIV stores gelu'(pre-activation) in aux instead of the pre-activation, so that the matching
// backward epilogue EPI_MUL_AUX is one multiply (the derivative shares the erf of the forward evaluation).
enum Epilogue { EPI_NONE = 0, EPI_BIAS = 1, EPI_BIAS_GELU = 2, EPI_MUL_GELU_GRAD = 3, EPI_ADD_RES = 4,
                EPI_BIAS_GELU_DERIV = 5, EPI_MUL_AUX = 6 };

// One (optionally batched) GEMM problem.  Batch index z = zb*nz_inner + zi
// moves each pointer by zb*stride_*[0] + zi*stride_*[1] elements.
struct GemmArgs {
  int M, N, K;
  const void* a; long lda; int a_kmajor;
  const void* b; long ldb; int b_kmajor;
  void* c; long ldc; int out_f32;
  float alpha;
  int epilogue;
  const float* bias;
  void* aux; long ldaux;   // EPI_BIAS_GELU: written; EPI_MUL_GELU_GRAD / EPI_ADD_RES: read
  int gelu_tanh;
  int batch;               // number of problems (>= 1)
  int nz_inner;            // inner batch extent (>= 1)
  long sa[2], sb[2], sc[2];
};
inline GemmArgs gemm_args_default() {
  GemmArgs g{};
  g.alpha = 1.0f;
  g.batch = 1;
  g.nz_inner = 1;
  return g;
}

raf_status launch_gemm(int precision, const GemmArgs& g, hipStream_t st);
// up to 4 independent weight-gradient GEMMs (A, B MN-major, float out) in one launch
// side / nside: optional column sums (ColsumJob, at most two, bf16, same row count), reds / nred: optional second
// stages of two-stage column sums (at most three), that the launch may take along on CUs its tiles leave idle;
// *side_taken tells whether it did (all of them or none), otherwise the caller launches them itself.
// nonfinite: optional device flag; when the side work is taken the launch also sets it to 1 if any weight gradient
// or any of the side sums is inf or nan (otherwise it is left alone and the caller has to check by other means)
struct ColsumJob;
struct ReduceJob;
raf_status launch_gemm_group_wgrad(int precision, const GemmArgs* gs, int count, hipStream_t st,
                                   const ColsumJob* side = nullptr, int nside = 0, const ReduceJob* reds = nullptr,
                                   int nred = 0, bool* side_taken = nullptr, int* nonfinite = nullptr);
// *flag = 1 if any element of the `count` float tensors ptrs[i][0 .. n[i]) is inf or nan (count <= 48)
raf_status launch_nonfinite_check(const float* const* ptrs, const long* n, int count, int* flag, hipStream_t st);
// dst[c][r] = src[r][c] for up to 4 dense row-major bf16 matrices (rows, cols multiples of 8) in one launch
struct TransposeJob {
  const void* src; void* dst; int rows, cols;
};
raf_status launch_transpose_bf16(const TransposeJob* jobs, int count, hipStream_t st);

raf_status launch_softmax_fwd(const raf_layer_desc& d, const void* s, const int32_t* lens, void* prob, void* prob_d,
                              uint64_t step, hipStream_t st);
raf_status launch_softmax_bwd(const raf_layer_desc& d, const void* prob, const void* prob_d, const void* dprob_d,
                              void* ds, float scale_out, hipStream_t st);
// S <= 128 in bf16 AMP: no S x S tensor reaches memory.  Forward: ctx = P~ . V written to [T,H], the probabilities
// are not stored.  Backward: P and the dropout mask are recomputed from qkv, the same lens and the same step; dQ, dK
// and dV are written to dqkv [T,3H].
// field and shape checks shared by every entry point that takes a layer description (layer.hip)
raf_status validate_desc(const raf_layer_desc* d);
bool attn_fused_supported(const raf_layer_desc& d);
raf_status launch_attn_fwd_fused(const raf_layer_desc& d, const void* qkv, const int32_t* lens, void* ctx, uint64_t step,
                                 hipStream_t st);
// S > 128 in bf16 AMP: blockwise with running softmax statistics; lse [B*heads*S] floats goes from forward to
// backward, dvec [B*heads*S] floats is backward scratch
bool attn_flash_supported(const raf_layer_desc& d);
// keep (optional, attn_flash_keep_bytes(d) bytes): the forward kernel leaves the keep decisions of dropout site 1
// there, one bit per score, and the adjoint kernels read them instead of running the generator again
size_t attn_flash_keep_bytes(const raf_layer_desc& d);
raf_status launch_attn_flash_fwd(const raf_layer_desc& d, const void* qkv, const int32_t* lens, void* ctx, float* lse,
                                 uint64_t step, hipStream_t st, uint32_t* keep = nullptr);
raf_status launch_attn_flash_bwd(const raf_layer_desc& d, const void* dc, const void* qkv, const void* ctx,
                                 const float* lse, const int32_t* lens, void* dqkv, float* dvec, uint64_t step,
                                 hipStream_t st, const uint32_t* keep = nullptr);
raf_status launch_attn_bwd_full(const raf_layer_desc& d, const void* dc, const void* qkv, const int32_t* lens, void* dqkv,
                                uint64_t step, hipStream_t st);
// Loss seed taken by the kernel that writes the layer's output: partial sums of out * G (one per workgroup, ln_fwd_blocks
// of them) and dy = scale * G; scale_ptr != nullptr: the scale is read from device memory
struct LossSeedDev {
  const void* G; void* dy; float* partial; float scale; const float* scale_ptr;
};
int ln_fwd_blocks(int hidden, int64_t rows);
raf_status launch_ln_fwd(const raf_layer_desc& d, int site, int64_t rows, const void* a, const void* res,
                         const float* gamma, const float* beta, void* out, void* z_out, float* mu, float* rstd,
                         uint64_t step, hipStream_t st, const LossSeedDev* loss = nullptr);
// Deferred second stages.  The column sums that only the optimizer reads (LayerNorm and bias gradients) are
// produced in two stages: per-block partial rows, then a reduction over the partial rows.  A caller with several of
// them can collect the second stages (and whole column-sum problems) and run each kind in one launch at the end of
// its schedule instead of one small launch after every producer.
struct ReduceJob {
  const float* partial; int nparts, ncols, nout;
  float *o0, *o1, *o2;
  int width_out, perm_nvec;
};
struct ColsumJob {
  int precision; const void* x; int64_t rows; int cols; long ld; float* out; float* partial; int out_cols;
};
constexpr int REDUCE_GROUP_MAX = 6, COLSUM_GROUP_MAX = 2;
raf_status launch_reduce_group(const ReduceJob* jobs, int count, hipStream_t st);
// first stage of up to COLSUM_GROUP_MAX column sums in one launch; their second stages are appended to reduce_jobs
raf_status launch_colsum_group(const ColsumJob* jobs, int count, ReduceJob* reduce_jobs, int* nreduce, hipStream_t st);

size_t ln_bwd_partial_floats(int hidden, int64_t rows);
// defer != nullptr: the reduction of the partial sums is not launched but described in *defer
raf_status launch_ln_bwd(const raf_layer_desc& d, int site, int64_t rows, const void* dout, const void* dout2,
                         const void* z, const float* mu, const float* rstd, const float* gamma, const void* dres,
                         void* dz, void* da, float* dgamma, float* dbeta, float* dbias, float* partial,
                         uint64_t step, hipStream_t st, int site_in = 0, ReduceJob* defer = nullptr);
// out[j] = sum_i x[i*ld + j], x in compute dtype, rows x cols; partial scratch
size_t colsum_partial_floats(int cols, int64_t rows);
// only the first out_cols (<= cols, 0 = all) sums are written
raf_status launch_colsum(int precision, const void* x, int64_t rows, int cols, long ld, float* out, float* partial,
                         hipStream_t st, int out_cols = 0);
// loss_out[0] = sum of partial[0..nparts) in a fixed order
raf_status launch_sum_partials(const float* partial, int nparts, float* out, hipStream_t st);

}  // namespace raf
