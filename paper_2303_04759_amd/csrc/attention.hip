// Fused attention-probability kernels for the bf16 AMP path (head dim 64):
//   forward : scores = Q K^T / 8 -> mask -> softmax -> dropout, written as P and P~
//   backward: dP~ = dC V^T -> dropout adjoint -> softmax adjoint (x 1/8), written as ds
// Both contract over the head dimension, which is contiguous in memory for both
// operands, so every MFMA fragment is a plain 16-byte global load: no LDS, no
// barriers.  A wavefront owns 16 query rows (v_mfma_f32_16x16x32_bf16, so that a
// BERT-base layer yields 3072 waves: 3 per SIMD) and walks the keys in chunks of
// 128 (8 MFMA blocks); with the operands swapped, a lane holds one query row and
// 8 consecutive keys per 32-key group, so row reductions are in-lane plus two
// exchanges (lane^16, lane^32).  Rows longer than 128 keys take two passes
// (statistics, then values) and recompute the cheap 64-deep product.
// The S x S score / dP~ tensors never reach memory (rule-based fusion of the
// elementwise + reduction chain into its producer, paper Section 3.2.2; softmax
// arithmetic in fp32, Section 3.1.2).
#include "common.hpp"

namespace raf {

constexpr int ATT_KC = 128;              // keys per chunk
constexpr int ATT_TILES = ATT_KC / 16;   // 16-key MFMA blocks per chunk
constexpr int ATT_ROWS = 16;             // query rows per wavefront

constexpr int ATT_PAIRS = ATT_TILES / 2; // 32-key groups per chunk

// 16 rows x 64 contraction values (row stride ld): the two k-step fragments of
// lane l: row `row`, elements 32*kk + 8*(l>>4) .. +7
__device__ __forceinline__ void load_frags(const bf16_t* base, long row, long ld, bf16x8_t (&f)[2]) {
  const int lane = threadIdx.x & 63;
  const bf16_t* p = base + row * ld + (lane >> 4) * 8;
  f[0] = *reinterpret_cast<const bf16x8_t*>(p);
  f[1] = *reinterpret_cast<const bf16x8_t*>(p + 32);
}

// acc[t] = X_t . Y^T for eight 16-key blocks X_t against the wave's 16 query rows
// Y.  The MFMA leaves lane l with query row l&15 and block rows 4*(l>>4) + r; the
// keys are dealt to block rows so that those are keys
//     32*(t/2) + 8*(l>>4) + 4*(t%2) + r          (block t, register r)
// i.e. per 32-key group a lane owns 8 consecutive keys and the four lanes of a
// query row own 64 contiguous bytes of the probability row: P, P~ and ds move as
// 16-byte accesses.  Every load is issued before the first product and none sits
// under a branch (groups past the end of a ragged chunk re-read the first group
// and their products are discarded by the caller), so the fragment loads of a
// chunk are in flight together instead of one memory round trip per block.
__device__ __forceinline__ void chunk_products(const bf16_t* keys_base, long ld, int key0, const bf16x8_t (&qf)[2],
                                               f32x4_t (&acc)[ATT_TILES], int npairs) {
  const int m = threadIdx.x & 15;
  bf16x8_t kf[ATT_TILES][2];
#pragma unroll
  for (int t = 0; t < ATT_TILES; ++t) {
    const int u = t >> 1, v = t & 1;
    load_frags(keys_base, key0 + (u < npairs ? 32 * u : 0) + 8 * (m >> 2) + 4 * v + (m & 3), ld, kf[t]);
  }
#pragma unroll
  for (int t = 0; t < ATT_TILES; ++t) {
    const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][0], qf[0], zero, 0, 0, 0);
    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][1], qf[1], acc[t], 0, 0, 0);
  }
}

__device__ __forceinline__ float xgroup_sum(float v) {
  v += __shfl_xor(v, 16, WAVE);
  return v + __shfl_xor(v, 32, WAVE);
}
__device__ __forceinline__ float xgroup_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 16, WAVE));
  return fmaxf(v, __shfl_xor(v, 32, WAVE));
}

__device__ __forceinline__ void store8_bf16(bf16_t* p, const float (&v)[8]) { Vec8<bf16_t>::store(p, v); }
__device__ __forceinline__ uint4 load8_raw(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ void unpack8_bf16(const uint4 r, float (&o)[8]) {
  o[0] = bf16_bits_to_f32(r.x & 0xffffu); o[1] = __uint_as_float(r.x & 0xffff0000u);
  o[2] = bf16_bits_to_f32(r.y & 0xffffu); o[3] = __uint_as_float(r.y & 0xffff0000u);
  o[4] = bf16_bits_to_f32(r.z & 0xffffu); o[5] = __uint_as_float(r.z & 0xffff0000u);
  o[6] = bf16_bits_to_f32(r.w & 0xffffu); o[7] = __uint_as_float(r.w & 0xffff0000u);
}

// 2^x by the hardware instruction alone; arguments here are <= 0 or -inf (-> 0)
__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

// ---------------------------------------------------------------- forward --
// alpha2 = log2(e) / sqrt(head dim): scores are kept in base-2 units so that the
// exponential is one v_exp_f32.
__global__ __launch_bounds__(256) void attn_prob_fwd_kernel(const bf16_t* __restrict__ qkv, const int32_t* __restrict__ lens,
                                                            bf16_t* __restrict__ prob, bf16_t* __restrict__ prob_d,
                                                            int S, int H, int heads, int causal, float alpha2,
                                                            DropSite drop) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = blockIdx.y, b = bh / heads, h = bh % heads;
  const int i0 = (blockIdx.x * 4 + wave) * ATT_ROWS;    // first query row of this wave
  if (i0 >= S) return;                                   // S is a multiple of 32: a wave is all in or all out
  const long ld = 3L * H;
  const bf16_t* Q = qkv + ((long)b * S) * ld + h * 64;
  const bf16_t* K = Q + H;
  const int i = i0 + (lane & 15);                        // this lane's query row
  const int jl = 8 * (lane >> 4);                        // this lane's first key within a 32-key group
  int len = lens ? lens[b] : S;
  len = len < 0 ? 0 : (len > S ? S : len);
  const int limit = causal ? (len < i + 1 ? len : i + 1) : len;      // keys >= limit are masked
  const int wave_limit = causal ? (len < i0 + ATT_ROWS ? len : i0 + ATT_ROWS) : len;   // no row of the wave sees keys beyond
  const long row_off = ((long)bh * S + i) * S;

  bf16x8_t qf[2];
  load_frags(Q, i, ld, qf);

  const int nchunks = (S + ATT_KC - 1) / ATT_KC;
  f32x4_t acc[ATT_TILES];

  // probabilities of one 8-key group -> P, dropout -> P~
  auto emit = [&](int j, float (&p)[8]) {
    store8_bf16(prob + row_off + j, p);
    if (drop.enabled) {
      float mult[8];
      drop_mult8(drop, (uint64_t)(row_off + j), mult);
#pragma unroll
      for (int e = 0; e < 8; ++e) p[e] *= mult[e];
    }
    store8_bf16(prob_d + row_off + j, p);
  };

  if (nchunks == 1) {
    // whole row in registers: one exponential per element
    const int npairs = S / 32;
    chunk_products(K, ld, 0, qf, acc, npairs);
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int j = 32 * (t >> 1) + jl + 4 * (t & 1) + r;
        const float s = ((t >> 1) < npairs && j < limit) ? acc[t][r] * alpha2 : -INFINITY;
        acc[t][r] = s;
        mx = fmaxf(mx, s);
      }
    mx = xgroup_max(mx);
    const float ref = mx == -INFINITY ? 0.f : mx;         // row without admissible keys: every term is 2^-inf = 0
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        acc[t][r] = exp2_hw(acc[t][r] - ref);
        sum += acc[t][r];
      }
    sum = xgroup_sum(sum);
    const float inv = sum > 0.f ? 1.0f / sum : 0.f;
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u)
      if (u < npairs) {
        float p[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) p[e] = acc[2 * u + (e >> 2)][e & 3] * inv;
        emit(32 * u + jl, p);
      }
    return;
  }

  float mx = -INFINITY, sum = 0.f;
  // pass 1: row maximum and sum of exponentials (online over the chunks)
  for (int c = 0; c < nchunks; ++c) {
    const int key0 = c * ATT_KC;
    if (key0 >= wave_limit) break;                       // fully masked from here on
    const int npairs = (S - key0) >= ATT_KC ? ATT_PAIRS : (S - key0) / 32;
    chunk_products(K, ld, key0, qf, acc, npairs);
    float cm = -INFINITY;
#pragma unroll
    for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int j = key0 + 32 * (t >> 1) + jl + 4 * (t & 1) + r;
        const float s = ((t >> 1) < npairs && j < limit) ? acc[t][r] * alpha2 : -INFINITY;
        acc[t][r] = s;
        cm = fmaxf(cm, s);
      }
    cm = xgroup_max(cm);
    const float nm = fmaxf(mx, cm);
    if (nm != -INFINITY) {
      float cs = 0.f;
#pragma unroll
      for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) cs += exp2_hw(acc[t][r] - nm);
      cs = xgroup_sum(cs);
      sum = sum * (mx == -INFINITY ? 0.f : exp2_hw(mx - nm)) + cs;
      mx = nm;
    }
  }
  const float inv = sum > 0.f ? 1.0f / sum : 0.f;        // a row without admissible keys gives zeros
  // pass 2: recompute the scores, then probabilities, dropout, stores
  for (int c = 0; c < nchunks; ++c) {
    const int key0 = c * ATT_KC;
    const int npairs = (S - key0) >= ATT_KC ? ATT_PAIRS : (S - key0) / 32;
    const bool live = key0 < wave_limit && inv > 0.f;
    if (live) chunk_products(K, ld, key0, qf, acc, npairs);
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u)
      if (u < npairs) {
        const int j = key0 + 32 * u + jl;
        float p[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
          p[e] = (live && j + e < limit) ? exp2_hw(acc[2 * u + (e >> 2)][e & 3] * alpha2 - mx) * inv : 0.f;
        emit(j, p);
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
  const int i0 = (blockIdx.x * 4 + wave) * ATT_ROWS;
  if (i0 >= S) return;
  const long ldv = 3L * H;
  const bf16_t* DC = dc + ((long)b * S) * H + h * 64;
  const bf16_t* V = qkv + ((long)b * S) * ldv + 2 * H + h * 64;
  const int i = i0 + (lane & 15);
  const int jl = 8 * (lane >> 4);
  const long row_off = ((long)bh * S + i) * S;

  bf16x8_t gf[2];
  load_frags(DC, i, H, gf);

  const int nchunks = (S + ATT_KC - 1) / ATT_KC;
  f32x4_t acc[ATT_TILES];
  uint4 pr[ATT_PAIRS], pdr[ATT_PAIRS];
  // P and P~ of this lane's key groups in one chunk; groups past a ragged end re-read the first one
  auto load_probs = [&](int key0, int npairs) {
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u) {
      const long o = row_off + key0 + (u < npairs ? 32 * u : 0) + jl;
      pr[u] = load8_raw(prob + o);
      pdr[u] = load8_raw(prob_d + o);
    }
  };
  // dP of one element: dropout adjoint of the product dP~ (dropped iff P != 0 but P~ == 0)
  auto dprob = [&](float dpd, float p, float pd) { return ((pd != 0.f) || (p == 0.f)) ? dpd * drop_scale : 0.f; };

  if (nchunks == 1) {
    // whole row in registers: P*dP is kept between the two passes
    const int npairs = S / 32;
    load_probs(0, npairs);
    chunk_products(V, ldv, 0, gf, acc, npairs);
    float dot = 0.f;
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u) {
      float p[8], pd[8];
      unpack8_bf16(pr[u], p);
      unpack8_bf16(pdr[u], pd);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float a = u < npairs ? p[e] * dprob(acc[2 * u + (e >> 2)][e & 3], p[e], pd[e]) : 0.f;
        acc[2 * u + (e >> 2)][e & 3] = a;
        dot += a;
      }
    }
    dot = xgroup_sum(dot);
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u)
      if (u < npairs) {
        float p[8], o[8];
        unpack8_bf16(pr[u], p);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = alpha * (acc[2 * u + (e >> 2)][e & 3] - p[e] * dot);
        store8_bf16(ds + row_off + 32 * u + jl, o);
      }
    return;
  }

  float dot = 0.f;
  // pass 1: D_i = sum_j dP_ij * P_ij
  for (int c = 0; c < nchunks; ++c) {
    const int key0 = c * ATT_KC;
    const int npairs = (S - key0) >= ATT_KC ? ATT_PAIRS : (S - key0) / 32;
    load_probs(key0, npairs);
    chunk_products(V, ldv, key0, gf, acc, npairs);
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u) {
      float p[8], pd[8];
      unpack8_bf16(pr[u], p);
      unpack8_bf16(pdr[u], pd);
#pragma unroll
      for (int e = 0; e < 8; ++e) dot += u < npairs ? p[e] * dprob(acc[2 * u + (e >> 2)][e & 3], p[e], pd[e]) : 0.f;
    }
  }
  dot = xgroup_sum(dot);
  // pass 2: ds = alpha * P * (dP - D)
  for (int c = 0; c < nchunks; ++c) {
    const int key0 = c * ATT_KC;
    const int npairs = (S - key0) >= ATT_KC ? ATT_PAIRS : (S - key0) / 32;
    load_probs(key0, npairs);
    chunk_products(V, ldv, key0, gf, acc, npairs);
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u)
      if (u < npairs) {
        float p[8], pd[8], o[8];
        unpack8_bf16(pr[u], p);
        unpack8_bf16(pdr[u], pd);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = alpha * p[e] * (dprob(acc[2 * u + (e >> 2)][e & 3], p[e], pd[e]) - dot);
        store8_bf16(ds + row_off + key0 + 32 * u + jl, o);
      }
  }
}

// ------------------------------------------- fused kernels for S <= 128 --
// With the whole key range in one chunk the probabilities of a wave are already in registers in the layout of an
// MFMA operand (a lane holds 8 consecutive keys of its query row per 32-key group), so the product that follows
// them is taken in the same kernel: context = P~ . V in the forward pass, dQ = ds . K in the backward pass.  The
// other operand ([S keys][64] of this head) is staged once per workgroup in LDS and read with the transposing
// ds_read_b64_tr_b16; two batched GEMM launches (and their reads of P~ and ds) disappear.
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
constexpr int HT_PITCH = 160;   // bytes per key row of a staged tile: 128 data + 32 pad; rows with bit 3 set swap
                                // their 64-byte halves, so the 8 key rows x 16 bytes one half-wave reads are conflict-free

__device__ __forceinline__ void stage_head_tile(const bf16_t* __restrict__ src, long ld, int S, char* tile) {
  for (int idx = threadIdx.x; idx < S * 8; idx += 256) {
    const int r = idx >> 3, c = idx & 7;
    const uint4 v = *reinterpret_cast<const uint4*>(src + (long)r * ld + c * 8);
    *reinterpret_cast<uint4*>(tile + r * HT_PITCH + ((c * 16) ^ (((r >> 3) & 1) << 6))) = v;
  }
}

// X^T fragment of the staged tile X [keys][64]: lane l gets row d = 16*nb + (l & 15), keys 32*u + 8*(l >> 4) .. +7
__device__ __forceinline__ bf16x8_t head_tile_frag_t(const char* tile, int u, int nb) {
  const int lane = threadIdx.x & 63, g = lane >> 4, s = lane & 15;
  const int r = 32 * u + 8 * g + (s >> 2);                    // key row of the first four values; +4 for the rest
  const int boff = (32 * nb + 8 * (s & 3)) ^ ((g & 1) << 6);  // (r >> 3) & 1 == g & 1 for both rows
  typedef s16x4_t __attribute__((address_space(3))) * lds_v4_ptr;
  const char* p = tile + r * HT_PITCH + boff;
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p));
  const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4_ptr)(p + 4 * HT_PITCH));
  const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8_t, both);
}

__device__ __forceinline__ uint4 pack8_bf16(const float (&v)[8]) {
  uint4 r;
  r.x = pack_bf16x2(v[0], v[1]); r.y = pack_bf16x2(v[2], v[3]);
  r.z = pack_bf16x2(v[4], v[5]); r.w = pack_bf16x2(v[6], v[7]);
  return r;
}

// out[query][64*h + d] = sum_keys frag[u] (this lane's 8 keys per group) x tile[key][d]; 8-byte stores
__device__ __forceinline__ void head_product_store(const char* tile, const uint4 (&frag)[ATT_PAIRS], int npairs,
                                                   bf16_t* __restrict__ out_row) {
  const int lane = threadIdx.x & 63;
  f32x4_t acc[4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int u = 0; u < ATT_PAIRS; ++u)
    if (u < npairs) {
      const bf16x8_t pf = __builtin_bit_cast(bf16x8_t, frag[u]);
#pragma unroll
      for (int nb = 0; nb < 4; ++nb)
        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(head_tile_frag_t(tile, u, nb), pf, acc[nb], 0, 0, 0);
    }
  // the lane ends with its query row and d = 16*nb + 4*(l >> 4) + r
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) {
    uint2 r;
    r.x = pack_bf16x2(acc[nb][0], acc[nb][1]);
    r.y = pack_bf16x2(acc[nb][2], acc[nb][3]);
    *reinterpret_cast<uint2*>(out_row + 16 * nb + 4 * (lane >> 4)) = r;
  }
}

__global__ __launch_bounds__(256) void attn_fwd_fused_kernel(const bf16_t* __restrict__ qkv, const int32_t* __restrict__ lens,
                                                             bf16_t* __restrict__ prob, bf16_t* __restrict__ prob_d,
                                                             bf16_t* __restrict__ ctx, int S, int H, int heads, int causal,
                                                             float alpha2, DropSite drop) {
  __shared__ __attribute__((aligned(16))) char vt[ATT_KC * HT_PITCH];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = blockIdx.y, b = bh / heads, h = bh % heads;
  const long ld = 3L * H;
  const bf16_t* Q = qkv + ((long)b * S) * ld + h * 64;
  const bf16_t* K = Q + H;
  stage_head_tile(Q + 2 * H, ld, S, vt);                // V of this head; read after the barrier below
  const int i0 = (blockIdx.x * 4 + wave) * ATT_ROWS;    // first query row of this wave
  const bool active = i0 < S;                            // S is a multiple of 32: a wave is all in or all out
  const int npairs = S / 32;
  uint4 pdf[ATT_PAIRS];
  const int i = i0 + (lane & 15);                        // this lane's query row
  if (active) {
    const int jl = 8 * (lane >> 4);                      // this lane's first key within a 32-key group
    int len = lens ? lens[b] : S;
    len = len < 0 ? 0 : (len > S ? S : len);
    const int limit = causal ? (len < i + 1 ? len : i + 1) : len;      // keys >= limit are masked
    const long row_off = ((long)bh * S + i) * S;
    bf16x8_t qf[2];
    load_frags(Q, i, ld, qf);
    f32x4_t acc[ATT_TILES];
    chunk_products(K, ld, 0, qf, acc, npairs);
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int j = 32 * (t >> 1) + jl + 4 * (t & 1) + r;
        const float sc = ((t >> 1) < npairs && j < limit) ? acc[t][r] * alpha2 : -INFINITY;
        acc[t][r] = sc;
        mx = fmaxf(mx, sc);
      }
    mx = xgroup_max(mx);
    const float ref = mx == -INFINITY ? 0.f : mx;         // row without admissible keys: every term is 2^-inf = 0
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        acc[t][r] = exp2_hw(acc[t][r] - ref);
        sum += acc[t][r];
      }
    sum = xgroup_sum(sum);
    const float inv = sum > 0.f ? 1.0f / sum : 0.f;
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u) {
      pdf[u] = make_uint4(0, 0, 0, 0);
      if (u < npairs) {
        float p[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) p[e] = acc[2 * u + (e >> 2)][e & 3] * inv;
        const int j = 32 * u + jl;
        store8_bf16(prob + row_off + j, p);
        if (drop.enabled) {
          float mult[8];
          drop_mult8(drop, (uint64_t)(row_off + j), mult);
#pragma unroll
          for (int e = 0; e < 8; ++e) p[e] *= mult[e];
        }
        pdf[u] = pack8_bf16(p);
        *reinterpret_cast<uint4*>(prob_d + row_off + j) = pdf[u];
      }
    }
  }
  __syncthreads();                                        // V tile complete
  if (active) head_product_store(vt, pdf, npairs, ctx + ((long)b * S + i) * H + h * 64);
}

__global__ __launch_bounds__(256) void attn_bwd_fused_kernel(const bf16_t* __restrict__ dc, const bf16_t* __restrict__ qkv,
                                                             const bf16_t* __restrict__ prob,
                                                             const bf16_t* __restrict__ prob_d, bf16_t* __restrict__ ds,
                                                             bf16_t* __restrict__ dq, int S, int H, int heads,
                                                             float drop_scale, float alpha) {
  __shared__ __attribute__((aligned(16))) char kt[ATT_KC * HT_PITCH];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = blockIdx.y, b = bh / heads, h = bh % heads;
  const long ldv = 3L * H;
  const bf16_t* Kp = qkv + ((long)b * S) * ldv + H + h * 64;
  stage_head_tile(Kp, ldv, S, kt);                       // K of this head; read after the barrier below
  const int i0 = (blockIdx.x * 4 + wave) * ATT_ROWS;
  const bool active = i0 < S;
  const int npairs = S / 32;
  const int i = i0 + (lane & 15);
  uint4 dsf[ATT_PAIRS];
  if (active) {
    const bf16_t* DC = dc + ((long)b * S) * H + h * 64;
    const bf16_t* V = qkv + ((long)b * S) * ldv + 2 * H + h * 64;
    const int jl = 8 * (lane >> 4);
    const long row_off = ((long)bh * S + i) * S;
    bf16x8_t gf[2];
    load_frags(DC, i, H, gf);
    uint4 pr[ATT_PAIRS], pdr[ATT_PAIRS];
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u) {
      const long o = row_off + (u < npairs ? 32 * u : 0) + jl;
      pr[u] = load8_raw(prob + o);
      pdr[u] = load8_raw(prob_d + o);
    }
    f32x4_t acc[ATT_TILES];
    chunk_products(V, ldv, 0, gf, acc, npairs);
    float dot = 0.f;
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u) {
      float p[8], pd[8];
      unpack8_bf16(pr[u], p);
      unpack8_bf16(pdr[u], pd);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // dropout adjoint of dP~: an element was dropped iff P != 0 but P~ == 0
        const float dp = ((pd[e] != 0.f) || (p[e] == 0.f)) ? acc[2 * u + (e >> 2)][e & 3] * drop_scale : 0.f;
        const float a = u < npairs ? p[e] * dp : 0.f;
        acc[2 * u + (e >> 2)][e & 3] = a;
        dot += a;
      }
    }
    dot = xgroup_sum(dot);
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u) {
      dsf[u] = make_uint4(0, 0, 0, 0);
      if (u < npairs) {
        float p[8], o[8];
        unpack8_bf16(pr[u], p);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = alpha * (acc[2 * u + (e >> 2)][e & 3] - p[e] * dot);
        dsf[u] = pack8_bf16(o);
        *reinterpret_cast<uint4*>(ds + row_off + 32 * u + jl) = dsf[u];
      }
    }
  }
  __syncthreads();                                        // K tile complete
  if (active) head_product_store(kt, dsf, npairs, dq + ((long)b * S + i) * ldv + h * 64);
}

// ----------------------------------------------------------------- launch --
raf_status launch_attn_prob_fwd(const raf_layer_desc& d, const void* qkv, const int32_t* lens, void* prob, void* prob_d,
                                uint64_t step, hipStream_t st) {
  if (!qkv || !prob || !prob_d) return RAF_EINVAL;
  if (d.precision != RAF_BF16_AMP || d.hidden / d.heads != 64 || (d.seq % 32)) return RAF_ENOTSUP;
  const DropSite drop = make_drop_site(d, 1, step);
  dim3 grid((d.seq + 4 * ATT_ROWS - 1) / (4 * ATT_ROWS), d.batch * d.heads);
  hipLaunchKernelGGL(attn_prob_fwd_kernel, grid, dim3(256), 0, st, (const bf16_t*)qkv, lens, (bf16_t*)prob,
                     (bf16_t*)prob_d, d.seq, d.hidden, d.heads, d.causal, 0.125f * 1.44269504088896341f, drop);
  return check_launch();
}

raf_status launch_attn_prob_bwd(const raf_layer_desc& d, const void* dc, const void* qkv, const void* prob,
                                const void* prob_d, void* ds, hipStream_t st) {
  if (!dc || !qkv || !prob || !prob_d || !ds) return RAF_EINVAL;
  if (d.precision != RAF_BF16_AMP || d.hidden / d.heads != 64 || (d.seq % 32)) return RAF_ENOTSUP;
  dim3 grid((d.seq + 4 * ATT_ROWS - 1) / (4 * ATT_ROWS), d.batch * d.heads);
  hipLaunchKernelGGL(attn_prob_bwd_kernel, grid, dim3(256), 0, st, (const bf16_t*)dc, (const bf16_t*)qkv,
                     (const bf16_t*)prob, (const bf16_t*)prob_d, (bf16_t*)ds, d.seq, d.hidden, d.heads,
                     (float)(1.0 / (1.0 - d.dropout_p)), 0.125f);
  return check_launch();
}

bool attn_fused_supported(const raf_layer_desc& d) {
  return d.precision == RAF_BF16_AMP && d.hidden / d.heads == 64 && d.seq % 32 == 0 && d.seq <= ATT_KC;
}

raf_status launch_attn_fwd_fused(const raf_layer_desc& d, const void* qkv, const int32_t* lens, void* prob, void* prob_d,
                                 void* ctx, uint64_t step, hipStream_t st) {
  if (!qkv || !prob || !prob_d || !ctx) return RAF_EINVAL;
  if (!attn_fused_supported(d)) return RAF_ENOTSUP;
  const DropSite drop = make_drop_site(d, 1, step);
  dim3 grid((d.seq + 4 * ATT_ROWS - 1) / (4 * ATT_ROWS), d.batch * d.heads);
  hipLaunchKernelGGL(attn_fwd_fused_kernel, grid, dim3(256), 0, st, (const bf16_t*)qkv, lens, (bf16_t*)prob,
                     (bf16_t*)prob_d, (bf16_t*)ctx, d.seq, d.hidden, d.heads, d.causal, 0.125f * 1.44269504088896341f,
                     drop);
  return check_launch();
}

raf_status launch_attn_bwd_fused(const raf_layer_desc& d, const void* dc, const void* qkv, const void* prob,
                                 const void* prob_d, void* ds, void* dqkv, hipStream_t st) {
  if (!dc || !qkv || !prob || !prob_d || !ds || !dqkv) return RAF_EINVAL;
  if (!attn_fused_supported(d)) return RAF_ENOTSUP;
  dim3 grid((d.seq + 4 * ATT_ROWS - 1) / (4 * ATT_ROWS), d.batch * d.heads);
  hipLaunchKernelGGL(attn_bwd_fused_kernel, grid, dim3(256), 0, st, (const bf16_t*)dc, (const bf16_t*)qkv,
                     (const bf16_t*)prob, (const bf16_t*)prob_d, (bf16_t*)ds, (bf16_t*)dqkv, d.seq, d.hidden, d.heads,
                     (float)(1.0 / (1.0 - d.dropout_p)), 0.125f);
  return check_launch();
}

}  // namespace raf
