// Fused attention-probability kernels for the bf16 AMP path (head dim 64):
//   forward : scores = Q K^T / 8 -> mask -> softmax -> dropout, written as P and P~
//   backward: dP~ = dC V^T -> dropout adjoint -> softmax adjoint (x 1/8), written as ds
// Both contract over the head dimension, which is contiguous in memory for both
// operands, so every MFMA fragment is a plain 16-byte global load: no LDS, no
// barriers.  A wavefront owns 32 query rows and walks the keys in chunks of 128
// (4 MFMA blocks); with the operands swapped, a lane holds one query row and 4
// consecutive keys per register group, so row reductions are in-lane plus one
// exchange with lane^32.  Rows longer than 128 keys take two passes
// (statistics, then values) and recompute the cheap 64-deep product.
// The S x S score / dP~ tensors never reach memory (rule-based fusion of the
// elementwise + reduction chain into its producer, paper Section 3.2.2; softmax
// arithmetic in fp32, Section 3.1.2).
#include "common.hpp"

namespace raf {

constexpr int ATT_KC = 128;              // keys per chunk
constexpr int ATT_TILES = ATT_KC / 32;   // MFMA blocks per chunk

// 32 rows x 64 contraction values starting at `base` (row stride ld): the four
// k-step fragments of lane l: row l&31, elements 16*kk + 8*(l>>5) .. +7
__device__ __forceinline__ void load_frags(const bf16_t* base, long ld, int row_lim, bf16x8_t (&f)[4]) {
  const int lane = threadIdx.x & 63;
  int r = lane & 31;
  r = r < row_lim ? r : row_lim - 1;     // rows past the end are clamped (their results are never stored)
  const bf16_t* p = base + (long)r * ld + (lane >> 5) * 8;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) f[kk] = *reinterpret_cast<const bf16x8_t*>(p + kk * 16);
}

// acc[t] = X_t . Y^T for the 32-row blocks X_t (rows = keys) against the wave's
// 32 query rows Y; lane l ends with query row l&31 and keys 8*(r/4)+4*(l>>5)+r%4.
__device__ __forceinline__ void chunk_products(const bf16_t* keys_base, long ld, int key0, int S,
                                               const bf16x8_t (&qf)[4], f32x16_t (&acc)[ATT_TILES], int ntiles) {
#pragma unroll
  for (int t = 0; t < ATT_TILES; ++t) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    if (t < ntiles) {
      bf16x8_t kf[4];
      load_frags(keys_base + (long)(key0 + t * 32) * ld, ld, S - (key0 + t * 32), kf);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk], qf[kk], acc[t], 0, 0, 0);
    }
  }
}

__device__ __forceinline__ float xhalf_sum(float v) { return v + __shfl_xor(v, 32, WAVE); }
__device__ __forceinline__ float xhalf_max(float v) { return fmaxf(v, __shfl_xor(v, 32, WAVE)); }

__device__ __forceinline__ void store4_bf16(bf16_t* p, float a, float b, float c, float d) {
  uint2 r;
  r.x = pack_bf16x2(a, b);
  r.y = pack_bf16x2(c, d);
  *reinterpret_cast<uint2*>(p) = r;
}
__device__ __forceinline__ void load4_bf16(const bf16_t* p, float (&o)[4]) {
  const uint2 r = *reinterpret_cast<const uint2*>(p);
  o[0] = bf16_bits_to_f32(r.x & 0xffffu); o[1] = __uint_as_float(r.x & 0xffff0000u);
  o[2] = bf16_bits_to_f32(r.y & 0xffffu); o[3] = __uint_as_float(r.y & 0xffff0000u);
}

// ---------------------------------------------------------------- forward --
__global__ __launch_bounds__(256) void attn_prob_fwd_kernel(const bf16_t* __restrict__ qkv, const int32_t* __restrict__ lens,
                                                            bf16_t* __restrict__ prob, bf16_t* __restrict__ prob_d,
                                                            int S, int H, int heads, int causal, float alpha,
                                                            DropSite drop) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = blockIdx.y, b = bh / heads, h = bh % heads;
  const int i0 = (blockIdx.x * 4 + wave) * 32;          // first query row of this wave
  if (i0 >= S) return;
  const long ld = 3L * H;
  const bf16_t* Q = qkv + ((long)b * S) * ld + h * 64;
  const bf16_t* K = Q + H;
  const int i = i0 + (lane & 31);                        // this lane's query row
  int len = lens ? lens[b] : S;
  len = len < 0 ? 0 : (len > S ? S : len);
  const int limit = causal ? (len < i + 1 ? len : i + 1) : len;      // keys >= limit are masked
  const int wave_limit = causal ? (len < i0 + 32 ? len : i0 + 32) : len;   // no row of the wave sees keys beyond

  bf16x8_t qf[4];
  load_frags(Q + (long)i0 * ld, ld, S - i0, qf);

  const int nchunks = (S + ATT_KC - 1) / ATT_KC;
  f32x16_t acc[ATT_TILES];
  float mx = -INFINITY, sum = 0.f;
  // pass 1: row maximum and sum of exponentials (online over the chunks)
  for (int c = 0; c < nchunks; ++c) {
    const int key0 = c * ATT_KC;
    if (key0 >= wave_limit) break;                       // fully masked from here on
    const int ntiles = (S - key0) >= ATT_KC ? ATT_TILES : (S - key0) / 32;
    chunk_products(K, ld, key0, S, qf, acc, ntiles);
    float cm = -INFINITY;
#pragma unroll
    for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int j = key0 + t * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const float s = (t < ntiles && j < limit) ? acc[t][r] * alpha : -INFINITY;
        acc[t][r] = s;
        cm = fmaxf(cm, s);
      }
    cm = xhalf_max(cm);
    const float nm = fmaxf(mx, cm);
    if (nm != -INFINITY) {
      float cs = 0.f;
#pragma unroll
      for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) cs += expf(acc[t][r] - nm);     // exp(-inf) == 0
      cs = xhalf_sum(cs);
      sum = sum * (mx == -INFINITY ? 0.f : expf(mx - nm)) + cs;
      mx = nm;
    }
  }
  const float inv = sum > 0.f ? 1.0f / sum : 0.f;        // a row without admissible keys gives zeros
  // pass 2: probabilities, dropout, stores (scores of a single chunk are still in registers)
  const long row_off = ((long)bh * S + i) * S;
  for (int c = 0; c < nchunks; ++c) {
    const int key0 = c * ATT_KC;
    const int ntiles = (S - key0) >= ATT_KC ? ATT_TILES : (S - key0) / 32;
    const bool live = key0 < wave_limit;
    if (live && nchunks > 1) {
      chunk_products(K, ld, key0, S, qf, acc, ntiles);
#pragma unroll
      for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = key0 + t * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          acc[t][r] = (t < ntiles && j < limit) ? acc[t][r] * alpha : -INFINITY;
        }
    }
    if (i < S) {
#pragma unroll
      for (int t = 0; t < ATT_TILES; ++t) {
        if (t < ntiles) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int j = key0 + t * 32 + 8 * q + 4 * (lane >> 5);
            float p[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) p[e] = (live && inv > 0.f) ? expf(acc[t][4 * q + e] - mx) * inv : 0.f;
            store4_bf16(prob + row_off + j, p[0], p[1], p[2], p[3]);
            if (drop.enabled) {
              const Philox4 rnd = philox4x32_10((uint32_t)((uint64_t)(row_off + j) >> 2), drop.c1, drop.c2, drop.c3,
                                                drop.k0, drop.k1);
              p[0] *= rnd.x >= drop.thr ? drop.scale : 0.f;
              p[1] *= rnd.y >= drop.thr ? drop.scale : 0.f;
              p[2] *= rnd.z >= drop.thr ? drop.scale : 0.f;
              p[3] *= rnd.w >= drop.thr ? drop.scale : 0.f;
            }
            store4_bf16(prob_d + row_off + j, p[0], p[1], p[2], p[3]);
          }
        }
      }
    }
  }
}

// --------------------------------------------------------------- backward --
__global__ __launch_bounds__(256) void attn_prob_bwd_kernel(const bf16_t* __restrict__ dc, const bf16_t* __restrict__ qkv,
                                                            const bf16_t* __restrict__ prob,
                                                            const bf16_t* __restrict__ prob_d, bf16_t* __restrict__ ds,
                                                            int S, int H, int heads, float drop_scale, float alpha) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = blockIdx.y, b = bh / heads, h = bh % heads;
  const int i0 = (blockIdx.x * 4 + wave) * 32;
  if (i0 >= S) return;
  const long ldv = 3L * H;
  const bf16_t* DC = dc + ((long)b * S) * H + h * 64;
  const bf16_t* V = qkv + ((long)b * S) * ldv + 2 * H + h * 64;
  const int i = i0 + (lane & 31);
  const long row_off = ((long)bh * S + (i < S ? i : S - 1)) * S;

  bf16x8_t gf[4];
  load_frags(DC + (long)i0 * H, H, S - i0, gf);

  const int nchunks = (S + ATT_KC - 1) / ATT_KC;
  f32x16_t acc[ATT_TILES];
  float dot = 0.f;
  // pass 1: D_i = sum_j dP_ij * P_ij
  for (int c = 0; c < nchunks; ++c) {
    const int key0 = c * ATT_KC;
    const int ntiles = (S - key0) >= ATT_KC ? ATT_TILES : (S - key0) / 32;
    chunk_products(V, ldv, key0, S, gf, acc, ntiles);
#pragma unroll
    for (int t = 0; t < ATT_TILES; ++t) {
      if (t < ntiles) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int j = key0 + t * 32 + 8 * q + 4 * (lane >> 5);
          float p[4], pd[4];
          load4_bf16(prob + row_off + j, p);
          load4_bf16(prob_d + row_off + j, pd);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            // dropped iff the probability is non-zero but the post-dropout value is zero
            const bool keep = (pd[e] != 0.f) || (p[e] == 0.f);
            const float dp = keep ? acc[t][4 * q + e] * drop_scale : 0.f;
            dot += dp * p[e];
            if (nchunks == 1) acc[t][4 * q + e] = p[e] * dp;     // single chunk: keep P*dP for pass 2
          }
        }
      }
    }
  }
  dot = xhalf_sum(dot);
  // pass 2: ds = alpha * P * (dP - D)
  for (int c = 0; c < nchunks; ++c) {
    const int key0 = c * ATT_KC;
    const int ntiles = (S - key0) >= ATT_KC ? ATT_TILES : (S - key0) / 32;
    if (nchunks > 1) chunk_products(V, ldv, key0, S, gf, acc, ntiles);
    if (i < S) {
#pragma unroll
      for (int t = 0; t < ATT_TILES; ++t) {
        if (t < ntiles) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int j = key0 + t * 32 + 8 * q + 4 * (lane >> 5);
            float p[4], o[4];
            load4_bf16(prob + row_off + j, p);
            if (nchunks == 1) {
              // acc holds P*dP
#pragma unroll
              for (int e = 0; e < 4; ++e) o[e] = alpha * (acc[t][4 * q + e] - p[e] * dot);
            } else {
              float pd[4];
              load4_bf16(prob_d + row_off + j, pd);
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const bool keep = (pd[e] != 0.f) || (p[e] == 0.f);
                const float dp = keep ? acc[t][4 * q + e] * drop_scale : 0.f;
                o[e] = alpha * p[e] * (dp - dot);
              }
            }
            store4_bf16(ds + row_off + j, o[0], o[1], o[2], o[3]);
          }
        }
      }
    }
  }
}

// ----------------------------------------------------------------- launch --
raf_status launch_attn_prob_fwd(const raf_layer_desc& d, const void* qkv, const int32_t* lens, void* prob, void* prob_d,
                                uint64_t step, hipStream_t st) {
  if (!qkv || !prob || !prob_d) return RAF_EINVAL;
  if (d.precision != RAF_BF16_AMP || d.hidden / d.heads != 64 || (d.seq % 32)) return RAF_ENOTSUP;
  const DropSite drop = make_drop_site(d, 1, step);
  dim3 grid((d.seq + 127) / 128, d.batch * d.heads);
  hipLaunchKernelGGL(attn_prob_fwd_kernel, grid, dim3(256), 0, st, (const bf16_t*)qkv, lens, (bf16_t*)prob,
                     (bf16_t*)prob_d, d.seq, d.hidden, d.heads, d.causal, 0.125f, drop);
  return check_launch();
}

raf_status launch_attn_prob_bwd(const raf_layer_desc& d, const void* dc, const void* qkv, const void* prob,
                                const void* prob_d, void* ds, hipStream_t st) {
  if (!dc || !qkv || !prob || !prob_d || !ds) return RAF_EINVAL;
  if (d.precision != RAF_BF16_AMP || d.hidden / d.heads != 64 || (d.seq % 32)) return RAF_ENOTSUP;
  dim3 grid((d.seq + 127) / 128, d.batch * d.heads);
  hipLaunchKernelGGL(attn_prob_bwd_kernel, grid, dim3(256), 0, st, (const bf16_t*)dc, (const bf16_t*)qkv,
                     (const bf16_t*)prob, (const bf16_t*)prob_d, (bf16_t*)ds, d.seq, d.hidden, d.heads,
                     (float)(1.0 / (1.0 - d.dropout_p)), 0.125f);
  return check_launch();
}

}  // namespace raf
