// Attention kernels of the bf16 AMP path (head dim 64): scores = Q K^T / 8 -> mask -> softmax -> dropout ->
// context, and the adjoints, without any S x S tensor in memory (rule-based fusion of the elementwise + reduction
// chain into its producers, paper Section 3.2.2; softmax arithmetic in fp32, Section 3.1.2).
// A wavefront owns 16 rows (v_mfma_f32_16x16x32_bf16) and sees the other index in blocks of 128 (8 MFMA blocks);
// with the operands swapped, a lane holds one of its rows and 8 consecutive columns per 32-column group, so row
// reductions are in-lane plus two exchanges (lane^16, lane^32) and the probabilities are already laid out as the
// operand of the product that follows them.
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

// Layout of a 16 x 128 score block acc[t] = X_t . Y^T (eight 16-key blocks X_t against the wave's 16 rows Y): the
// MFMA leaves lane l with own row l&15 and block rows 4*(l>>4) + r; the keys are dealt to block rows so that those are
//     32*(t/2) + 8*(l>>4) + 4*(t%2) + r          (block t, register r)
// i.e. per 32-key group a lane owns 8 consecutive keys.
__device__ __forceinline__ float xgroup_sum(float v) {
  v += __shfl_xor(v, 16, WAVE);
  return v + __shfl_xor(v, 32, WAVE);
}
__device__ __forceinline__ float xgroup_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 16, WAVE));
  return fmaxf(v, __shfl_xor(v, 32, WAVE));
}

// 2^x by the hardware instruction alone; arguments here are <= 0 or -inf (-> 0)
__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

// ------------------------------------------- fused kernels for S <= 128 --
// With the whole key range in one chunk the probabilities of a wave are already in registers in the layout of an
// MFMA operand (a lane holds 8 consecutive keys of its query row per 32-key group), so the products that follow
// them are taken in the same kernel and no S x S tensor reaches memory at all:
//   forward : context = P~ . V; the probabilities are not stored
//   backward: P and the dropout mask are recomputed from Q, K and the counter-based generator, ds is formed in
//             registers, and dQ = ds . K, dV = P~^T . dC and dK = ds^T . Q follow, the last two through LDS copies
//             of P~ and ds (their contraction runs over the query index, which is spread over the waves).
// A wave owns 16 query rows; the backward pass runs one workgroup of 8 waves per (batch, head).  The [S][64] operands of the
// head (K, V, dC, Q) are brought into LDS once per workgroup by direct-to-LDS loads: loads into registers sustain
// only about 16 bytes/clock/CU, and with every wave fetching its own K and V fragments from global memory that rate,
// not the arithmetic, set the time of these kernels.  Fragments whose contraction index is the row index of the
// tile are read with the transposing ds_read_b64_tr_b16.
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* att_lds_ptr;
typedef s16x4_t __attribute__((address_space(3))) * att_lds_v4_ptr;

// [rows][64] bf16 tile, 128 bytes per row (the direct loads fill whole KiB of 8 rows); the 16-byte chunk c of row r
// sits at chunk position c ^ hd_swz(r).  The swizzle makes both access patterns conflict-free: the 16 key rows
// {0-3, 8-11, 16-19, 24-27} + 4v that one 16-lane group reads at a common chunk, and the 8 rows {0-3, 8-11} x 32
// bytes that a half-wave reads transposed.
constexpr int HD_TILE = ATT_KC * 128;
__device__ __forceinline__ int hd_swz(int r) {
  return (((r >> 1) & 1) << 1) | (((r >> 3) & 1) << 2) | (((r >> 2) ^ (r >> 4)) & 1);
}

// rows [0, S) of a head ([S][64] at row stride ld) -> tile, issued by all waves of the workgroup; complete for the
// workgroup after hd_tile_wait() and a barrier
__device__ __forceinline__ void hd_tile_load(const bf16_t* __restrict__ src, long ld, int S, char* tile) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
  for (int q = wave; q < S / 8; q += nw) {
    const int r = q * 8 + (lane >> 3);
    const bf16_t* g = src + (long)r * ld + (((lane & 7) ^ hd_swz(r)) << 3);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g, (att_lds_ptr)(tile + q * 1024), 16,
                                     0, 0);
  }
}
__device__ __forceinline__ void hd_tile_wait() { __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8)); }   // vmcnt(0)

// operand fragment of a tile row: elements 32*kk + 8*(l >> 4) .. +7 of row `row`
__device__ __forceinline__ bf16x8_t hd_frag(const char* tile, int row, int kk) {
  const int c = 4 * kk + ((threadIdx.x & 63) >> 4);
  return *reinterpret_cast<const bf16x8_t*>(tile + row * 128 + ((c ^ hd_swz(row)) << 4));
}

// X^T fragment of a tile X [rows][64]: lane l gets d = 16*nb + (l & 15), rows 32*u + 8*(l >> 4) .. +7
__device__ __forceinline__ bf16x8_t hd_frag_t(const char* tile, int u, int nb) {
  const int lane = threadIdx.x & 63, g = lane >> 4, s = lane & 15;
  const int r = 32 * u + 8 * g + (s >> 2);                    // row of the first four values; +4 for the rest
  const int c = 2 * nb + ((s & 3) >> 1), half = (s & 1) << 3;
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((att_lds_v4_ptr)(tile + r * 128 + ((c ^ hd_swz(r)) << 4) + half));
  const s16x4_t hi =
      __builtin_amdgcn_ds_read_tr16_b64_v4i16((att_lds_v4_ptr)(tile + (r + 4) * 128 + ((c ^ hd_swz(r + 4)) << 4) + half));
  const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8_t, both);
}

// chunk_products with the key-side operand (K or V) in an LDS tile
__device__ __forceinline__ void tile_products(const char* tile, const bf16x8_t (&qf)[2], f32x4_t (&acc)[ATT_TILES],
                                              int npairs) {
  const int m = threadIdx.x & 15;
#pragma unroll
  for (int t = 0; t < ATT_TILES; ++t) {
    const int u = t >> 1, v = t & 1;
    const int row = (u < npairs ? 32 * u : 0) + 8 * (m >> 2) + 4 * v + (m & 3);
    const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hd_frag(tile, row, 0), qf[0], zero, 0, 0, 0);
    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hd_frag(tile, row, 1), qf[1], acc[t], 0, 0, 0);
  }
}

// the two 16-row blocks of 32-row group u only: a[v][r] = acc[2u+v][r] of tile_products (the blockwise kernels take
// one group at a time, which keeps 48 accumulator registers fewer alive)
__device__ __forceinline__ void group_products(const char* tile, const bf16x8_t (&qf)[2], int u, f32x4_t (&a)[2]) {
  const int m = threadIdx.x & 15;
#pragma unroll
  for (int v = 0; v < 2; ++v) {
    const int row = 32 * u + 8 * (m >> 2) + 4 * v + (m & 3);
    const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
    a[v] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hd_frag(tile, row, 0), qf[0], zero, 0, 0, 0);
    a[v] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hd_frag(tile, row, 1), qf[1], a[v], 0, 0, 0);
  }
}

__device__ __forceinline__ uint4 pack8_bf16(const float (&v)[8]) {
  uint4 r;
  r.x = pack_bf16x2(v[0], v[1]); r.y = pack_bf16x2(v[2], v[3]);
  r.z = pack_bf16x2(v[4], v[5]); r.w = pack_bf16x2(v[6], v[7]);
  return r;
}

__device__ __forceinline__ void store_head_row(bf16_t* __restrict__ out_row, const f32x4_t (&acc)[4]) {
  // the lane holds its row and d = 16*nb + 4*(l >> 4) + r
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) {
    uint2 r;
    r.x = pack_bf16x2(acc[nb][0], acc[nb][1]);
    r.y = pack_bf16x2(acc[nb][2], acc[nb][3]);
    *reinterpret_cast<uint2*>(out_row + 16 * nb + 4 * (lane >> 4)) = r;
  }
}

// out[query][64*h + d] = sum_keys frag[u] (this lane's 8 keys per group) x tile[key][d]
__device__ __forceinline__ void head_product_store(const char* tile, const uint4 (&frag)[ATT_PAIRS], int npairs,
                                                   bf16_t* __restrict__ out_row) {
  f32x4_t acc[4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int u = 0; u < ATT_PAIRS; ++u)
    if (u < npairs) {
      const bf16x8_t pf = __builtin_bit_cast(bf16x8_t, frag[u]);
#pragma unroll
      for (int nb = 0; nb < 4; ++nb)
        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hd_frag_t(tile, u, nb), pf, acc[nb], 0, 0, 0);
    }
  store_head_row(out_row, acc);
}

// scores -> mask -> softmax of this lane's query row: acc holds P (not yet divided by the sum) on return, the
// reciprocal of the row sum is returned (0 for a row without admissible keys)
__device__ __forceinline__ float row_softmax(f32x4_t (&acc)[ATT_TILES], int npairs, int limit, float alpha2) {
  const int jl = 8 * ((threadIdx.x & 63) >> 4);
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
  return sum > 0.f ? 1.0f / sum : 0.f;
}

// Forward: a workgroup of 4 waves takes 64 query rows of one head (two workgroups per head at S = 128, so that the
// 256 CUs get three workgroups each instead of one and a half); each stages K and V for itself.
__global__ __launch_bounds__(256) void attn_fwd_fused_kernel(const bf16_t* __restrict__ qkv, const int32_t* __restrict__ lens,
                                                             bf16_t* __restrict__ ctx, int S, int H, int heads, int causal,
                                                             float alpha2, DropSite drop) {
  __shared__ __attribute__((aligned(1024))) char kt[HD_TILE];
  __shared__ __attribute__((aligned(1024))) char vt[HD_TILE];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = blockIdx.x, b = bh / heads, h = bh % heads;
  const long ld = 3L * H;
  const bf16_t* Q = qkv + ((long)b * S) * ld + h * 64;
  hd_tile_load(Q + H, ld, S, kt);
  hd_tile_load(Q + 2 * H, ld, S, vt);
  const int i0 = ((int)blockIdx.y * 4 + wave) * ATT_ROWS;   // first query row of this wave
  const bool active = i0 < S;                            // S is a multiple of 32: a wave is all in or all out
  const int npairs = S / 32;
  const int i = i0 + (lane & 15);                        // this lane's query row
  bf16x8_t qf[2];
  if (active) load_frags(Q, i, ld, qf);
  hd_tile_wait();
  __syncthreads();                                        // K and V tiles complete
  if (!active) return;
  const int jl = 8 * (lane >> 4);                        // this lane's first key within a 32-key group
  int len = lens ? lens[b] : S;
  len = len < 0 ? 0 : (len > S ? S : len);
  const int limit = causal ? (len < i + 1 ? len : i + 1) : len;      // keys >= limit are masked
  const long row_off = ((long)bh * S + i) * S;
  f32x4_t acc[ATT_TILES];
  tile_products(kt, qf, acc, npairs);
  const float inv = row_softmax(acc, npairs, limit, alpha2);
  uint4 pdf[ATT_PAIRS];
#pragma unroll
  for (int u = 0; u < ATT_PAIRS; ++u) {
    pdf[u] = make_uint4(0, 0, 0, 0);
    if (u < npairs) {
      float p[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) p[e] = acc[2 * u + (e >> 2)][e & 3] * inv;
      if (drop.enabled) {
        float mult[8];
        drop_mult8(drop, (uint64_t)(row_off + 32 * u + jl), mult);
#pragma unroll
        for (int e = 0; e < 8; ++e) p[e] *= mult[e];
      }
      pdf[u] = pack8_bf16(p);
    }
  }
  head_product_store(vt, pdf, npairs, ctx + ((long)b * S + i) * H + h * 64);
}

// [S][S] tile of P~ or ds in LDS, row = query: 256 data bytes per row at a pitch of 288, rows with bit 3 set have
// their 128-byte halves swapped, so that the 8 rows x 32 bytes one half-wave reads transposed are conflict-free.
constexpr int SQ_PITCH = 288;
// K | dC, later Q | V, later P~ and ds (the last tile is longer than V and extends beyond it)
constexpr int ATT_BWD_LDS = 2 * HD_TILE + ATT_KC * SQ_PITCH;

// this lane's 8 values of each 32-key group of query row `row` (0 .. S-1 within the head)
__device__ __forceinline__ void sq_tile_write(char* tile, int row, const uint4 (&frag)[ATT_PAIRS], int npairs) {
  const int g = (threadIdx.x & 63) >> 4;
  char* p = tile + row * SQ_PITCH;
  const int swap = ((row >> 3) & 1) << 7;
#pragma unroll
  for (int u = 0; u < ATT_PAIRS; ++u)
    if (u < npairs) *reinterpret_cast<uint4*>(p + ((64 * u + 16 * g) ^ swap)) = frag[u];
}

// X^T fragment of such a tile: lane l gets row key = 16*kb + (l & 15), queries 32*u + 8*(l >> 4) .. +7
__device__ __forceinline__ bf16x8_t sq_tile_frag_t(const char* tile, int u, int kb) {
  const int lane = threadIdx.x & 63, g = lane >> 4, s = lane & 15;
  const int r = 32 * u + 8 * g + (s >> 2);                    // query row of the first four values; +4 for the rest
  const int boff = (32 * kb + 8 * (s & 3)) ^ ((g & 1) << 7);  // (r >> 3) & 1 == g & 1 for both rows
  const char* p = tile + r * SQ_PITCH + boff;
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((att_lds_v4_ptr)(p));
  const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((att_lds_v4_ptr)(p + 4 * SQ_PITCH));
  const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8_t, both);
}

// out[key][64*h + d] = sum_queries sq[query][key] x xt[query][d] for the 16 keys of block kb
__device__ __forceinline__ void key_product_store(const char* sq, const char* xt, int npairs, int kb,
                                                  bf16_t* __restrict__ out_row) {
  f32x4_t acc[4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) acc[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int u = 0; u < ATT_PAIRS; ++u)
    if (u < npairs) {
      const bf16x8_t yf = sq_tile_frag_t(sq, u, kb);
#pragma unroll
      for (int nb = 0; nb < 4; ++nb)
        acc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hd_frag_t(xt, u, nb), yf, acc[nb], 0, 0, 0);
    }
  store_head_row(out_row, acc);
}

// Wave w owns query rows 16w .. 16w+15 until ds is formed and key rows 16w .. 16w+15 of dV and dK afterwards.
// alpha2 = log2(e)/8 as in the forward pass, alpha = 1/8.
__global__ __launch_bounds__(512) void attn_bwd_full_kernel(const bf16_t* __restrict__ dc, const bf16_t* __restrict__ qkv,
                                                            const int32_t* __restrict__ lens, bf16_t* __restrict__ dqkv,
                                                            int S, int H, int heads, int causal, float alpha2,
                                                            float alpha, DropSite drop) {
  extern __shared__ __attribute__((aligned(1024))) char att_lds[];
  char* kt = att_lds;                          // K of this head
  char* xt = kt + HD_TILE;                     // dC, later Q
  char* vt = xt + HD_TILE;                     // V
  char* sq = vt;                               // P~, later ds: written only after every wave is done with V
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = blockIdx.x, b = bh / heads, h = bh % heads;
  const long ld = 3L * H;
  const bf16_t* Q = qkv + ((long)b * S) * ld + h * 64;
  const bf16_t* DC = dc + ((long)b * S) * H + h * 64;
  hd_tile_load(Q + H, ld, S, kt);
  hd_tile_load(Q + 2 * H, ld, S, vt);
  hd_tile_load(DC, H, S, xt);
  const int i0 = wave * ATT_ROWS;
  const bool active = i0 < S;                            // S is a multiple of 32: a wave is all in or all out
  const int npairs = S / 32;
  const int i = i0 + (lane & 15);                        // this lane's query row, later its key row
  bf16_t* out_row = dqkv + ((long)b * S + i) * ld + h * 64;
  bf16x8_t qf[2], gf[2];
  if (active) {
    load_frags(Q, i, ld, qf);
    load_frags(DC, i, H, gf);
  }
  hd_tile_wait();
  __syncthreads();                                        // K, V and dC tiles complete
  uint4 pdf[ATT_PAIRS], dsf[ATT_PAIRS];
  if (active) {
    const int jl = 8 * (lane >> 4);                      // this lane's first key within a 32-key group
    int len = lens ? lens[b] : S;
    len = len < 0 ? 0 : (len > S ? S : len);
    const int limit = causal ? (len < i + 1 ? len : i + 1) : len;      // keys >= limit are masked
    const long row_off = ((long)bh * S + i) * S;
    // P as in the forward pass
    f32x4_t acc[ATT_TILES];
    tile_products(kt, qf, acc, npairs);
    const float inv = row_softmax(acc, npairs, limit, alpha2);
    // dP~ = dC V^T
    f32x4_t dacc[ATT_TILES];
    tile_products(vt, gf, dacc, npairs);
    float dot = 0.f;
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u) {
      pdf[u] = make_uint4(0, 0, 0, 0);
      if (u < npairs) {
        float mult[8], pd[8];
        if (drop.enabled) {
          drop_mult8(drop, (uint64_t)(row_off + 32 * u + jl), mult);
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) mult[e] = 1.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pe = acc[2 * u + (e >> 2)][e & 3] * inv;
          acc[2 * u + (e >> 2)][e & 3] = pe;
          pd[e] = pe * mult[e];
          const float a = pe * (dacc[2 * u + (e >> 2)][e & 3] * mult[e]);   // P (.) dP, dropout adjoint applied
          dacc[2 * u + (e >> 2)][e & 3] = a;
          dot += a;
        }
        pdf[u] = pack8_bf16(pd);
      }
    }
    dot = xgroup_sum(dot);
#pragma unroll
    for (int u = 0; u < ATT_PAIRS; ++u) {
      dsf[u] = make_uint4(0, 0, 0, 0);
      if (u < npairs) {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = alpha * (dacc[2 * u + (e >> 2)][e & 3] - acc[2 * u + (e >> 2)][e & 3] * dot);
        dsf[u] = pack8_bf16(o);
      }
    }
  }
  __syncthreads();                                        // every wave is done with the V tile
  if (active) sq_tile_write(sq, i, pdf, npairs);
  __syncthreads();                                        // P~ tile complete
  if (active) {
    head_product_store(kt, dsf, npairs, out_row);                     // dQ = ds . K
    key_product_store(sq, xt, npairs, wave, out_row + 2 * H);         // dV = P~^T . dC
  }
  __syncthreads();                                        // every wave is done with the P~ and dC tiles
  if (active) sq_tile_write(sq, i, dsf, npairs);
  hd_tile_load(Q, ld, S, xt);
  hd_tile_wait();
  __syncthreads();                                        // ds and Q tiles complete
  if (active) key_product_store(sq, xt, npairs, wave, out_row + H);   // dK = ds^T . Q
}

// --------------------------------------------- longer rows (S > 128) --
// The same three products per 128-key block with a running maximum and sum (the rescaling form of the softmax), so
// that rows of any length keep their probabilities on chip as well.  The forward pass leaves one number per query
// row, lse = max + log2(sum) in the base-2 units of the scores, from which the backward kernels recompute
// P = 2^(s - lse) block by block.  The backward pass is two kernels with opposite ownership, each deterministic:
//   attn_flash_dq_kernel   waves own query rows and walk the key blocks   (dQ; also D = rowsum(dC (.) ctx))
//   attn_flash_dkv_kernel  waves own key rows and walk the query blocks   (dK, dV)
// In the second one the score block is formed transposed (own key row, 8 consecutive queries per lane and 32-query
// group), which is already the operand layout of dV = P~^T dC and dK = ds^T Q: no exchange between waves is needed.
// Dropout blocks cover 8 consecutive keys of one query, so there each lane generates the block of one (query,
// key octet) of its 16 x 32 sub-block and the keep bits are exchanged with lane permutes.
// KEPT: the generator (twenty 32x32 multiplies per 8 scores) runs in the forward kernel only, which leaves its
// decisions in memory, one bit per score: 16 bytes per (query row, 128-key block), dword g holding the octets
// 32u + 8g .. +7 (u = 0..3 in bytes 0..3), which is what lane group g of the row's wavefront holds.  The adjoint
// kernels read them back (dQ: one dword per lane and key block; dK/dV: the 2 KiB of a block pair staged through LDS
// with the Q and dC blocks).
constexpr int FL_QB = 128;   // query rows per workgroup (8 waves x 16)
constexpr int FL_KEEP_TILE = FL_QB * 16;                   // keep bits of 128 queries x 128 keys
// Block of the sequence that workgroup (blockIdx.x, blockIdx.y) takes.  Under a causal mask the work of a block
// grows (query blocks) or shrinks (key blocks) along the sequence; two workgroups share a CU and are dealt to the
// CUs round-robin, so every other round of 256 workgroups walks the sequence backwards and a long block meets a
// short one instead of another long one.
__device__ __forceinline__ int fl_seq_block() {
  const int n = gridDim.x;
  const long linear = (long)blockIdx.y * n + blockIdx.x;
  return ((linear >> 8) & 1) ? n - 1 - (int)blockIdx.x : (int)blockIdx.x;
}
constexpr int FL_STAGE = 2 * HD_TILE;                      // K and V (or Q and dC) block
constexpr int FL_DKV_STAGE = 2 * HD_TILE + 2 * FL_QB * 4;  // plus lse and D of the query rows

// keep bits (bit e = element idx8 + e is kept) of one Philox block
__device__ __forceinline__ uint32_t drop_keep8(const DropSite& s, uint64_t idx8) {
  const Philox4 a = philox4x32_10((uint32_t)(idx8 >> 3), s.c1, s.c2, s.c3, s.k0, s.k1);
  uint32_t bits = 0;
  bits |= ((a.x & 0xffffu) >= s.thr ? 1u : 0u) | ((a.x >> 16) >= s.thr ? 2u : 0u);
  bits |= ((a.y & 0xffffu) >= s.thr ? 4u : 0u) | ((a.y >> 16) >= s.thr ? 8u : 0u);
  bits |= ((a.z & 0xffffu) >= s.thr ? 16u : 0u) | ((a.z >> 16) >= s.thr ? 32u : 0u);
  bits |= ((a.w & 0xffffu) >= s.thr ? 64u : 0u) | ((a.w >> 16) >= s.thr ? 128u : 0u);
  return bits;
}

__device__ __forceinline__ float frag_dot(const bf16x8_t (&a)[2], const bf16x8_t (&b)[2]) {
  float d = 0.f;
#pragma unroll
  for (int k = 0; k < 2; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) d += (float)a[k][e] * (float)b[k][e];
  return d;
}

template <bool KEPT>
__global__ __launch_bounds__(512) void attn_flash_fwd_kernel(const bf16_t* __restrict__ qkv, const int32_t* __restrict__ lens,
                                                             bf16_t* __restrict__ ctx, float* __restrict__ lse, int S,
                                                             int H, int heads, int causal, float alpha2, DropSite drop,
                                                             uint32_t* __restrict__ keep) {
  extern __shared__ __attribute__((aligned(1024))) char fl_lds[];   // two stages of (K block, V block)
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = blockIdx.y, b = bh / heads, h = bh % heads;
  const long ld = 3L * H;
  const bf16_t* Q = qkv + ((long)b * S) * ld + h * 64;
  const int q0 = fl_seq_block() * FL_QB;
  const int i0 = q0 + wave * ATT_ROWS;
  const bool active = i0 < S;                            // S is a multiple of 32: a wave is all in or all out
  const int i = i0 + (lane & 15);                        // this lane's query row
  const int jl = 8 * (lane >> 4);                        // this lane's first key within a 32-key group
  int len = lens ? lens[b] : S;
  len = len < 0 ? 0 : (len > S ? S : len);
  const int limit = causal ? (len < i + 1 ? len : i + 1) : len;      // keys >= limit are masked
  const int q_end = q0 + FL_QB < S ? q0 + FL_QB : S;
  const int kmax = causal ? (len < q_end ? len : q_end) : len;       // no row of the workgroup sees keys beyond
  const int nkb = (kmax + ATT_KC - 1) / ATT_KC;
  const long row_off = ((long)bh * S + i) * S;
  bf16x8_t qf[2];
  if (active) load_frags(Q, i, ld, qf);
  float mx = -INFINITY, sum = 0.f;
  f32x4_t o[4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) o[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  auto fetch = [&](int jb) {   // K and V rows of key block jb -> stage jb & 1
    const int key0 = jb * ATT_KC;
    const int rows = S - key0 < ATT_KC ? S - key0 : ATT_KC;
    char* st = fl_lds + (jb & 1) * 2 * HD_TILE;
    hd_tile_load(Q + H + (long)key0 * ld, ld, rows, st);
    hd_tile_load(Q + 2 * H + (long)key0 * ld, ld, rows, st + HD_TILE);
  };
  if (nkb > 0) fetch(0);
  for (int jb = 0; jb < nkb; ++jb) {
    const int key0 = jb * ATT_KC;
    const int rows = S - key0 < ATT_KC ? S - key0 : ATT_KC;
    const int npairs = rows / 32;
    const char* kt = fl_lds + (jb & 1) * 2 * HD_TILE;
    const char* vt = kt + HD_TILE;
    hd_tile_wait();
    __syncthreads();                                      // block jb has landed; every wave is done with block jb-1
    if (jb + 1 < nkb) fetch(jb + 1);                      // overlaps the arithmetic below
    if (active) {
      f32x4_t acc[ATT_TILES];
      tile_products(kt, qf, acc, npairs);
      float bm = -INFINITY;
#pragma unroll
      for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int j = key0 + 32 * (t >> 1) + jl + 4 * (t & 1) + r;
          const float sc = ((t >> 1) < npairs && j < limit) ? acc[t][r] * alpha2 : -INFINITY;
          acc[t][r] = sc;
          bm = fmaxf(bm, sc);
        }
      bm = xgroup_max(bm);
      const float nm = fmaxf(mx, bm);
      const float ref = nm == -INFINITY ? 0.f : nm;       // nothing admissible so far: every term is 2^-inf = 0
      const float corr = exp2_hw(mx - ref);
      float bs = 0.f;
#pragma unroll
      for (int t = 0; t < ATT_TILES; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          acc[t][r] = exp2_hw(acc[t][r] - ref);
          bs += acc[t][r];
        }
      bs = xgroup_sum(bs);
      sum = sum * corr + bs;
      mx = nm;
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) o[nb] = o[nb] * corr;
      uint32_t kw = 0;
#pragma unroll
      for (int u = 0; u < ATT_PAIRS; ++u)
        if (u < npairs) {
          float p[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) p[e] = acc[2 * u + (e >> 2)][e & 3];
          if (drop.enabled) {
            float mult[8];
            if (KEPT) {
              uint32_t bits;
              drop_mult8_bits(drop, (uint64_t)(row_off + key0 + 32 * u + jl), mult, bits);
              kw |= bits << (8 * u);
            } else {
              drop_mult8(drop, (uint64_t)(row_off + key0 + 32 * u + jl), mult);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) p[e] *= mult[e];
          }
          const bf16x8_t pf = __builtin_bit_cast(bf16x8_t, pack8_bf16(p));
#pragma unroll
          for (int nb = 0; nb < 4; ++nb)
            o[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hd_frag_t(vt, u, nb), pf, o[nb], 0, 0, 0);
        }
      if (KEPT && drop.enabled) keep[(((long)bh * S + i) * ((S + ATT_KC - 1) / ATT_KC) + jb) * 4 + (lane >> 4)] = kw;
    }
  }
  if (!active) return;
  const float inv = sum > 0.f ? 1.0f / sum : 0.f;         // a row without admissible keys gives zeros
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) o[nb] = o[nb] * inv;
  store_head_row(ctx + ((long)b * S + i) * H + h * 64, o);
  if (lane < 16) lse[(long)bh * S + i] = sum > 0.f ? mx + __log2f(sum) : INFINITY;
}

// dQ = ds . K over all key blocks; also writes D = rowsum(dC (.) ctx) for the dK/dV kernel
template <bool KEPT>
__global__ __launch_bounds__(512) void attn_flash_dq_kernel(const bf16_t* __restrict__ dc, const bf16_t* __restrict__ qkv,
                                                            const bf16_t* __restrict__ ctx, const float* __restrict__ lse,
                                                            const int32_t* __restrict__ lens, bf16_t* __restrict__ dqkv,
                                                            float* __restrict__ dvec, int S, int H, int heads, int causal,
                                                            float alpha2, float alpha, DropSite drop,
                                                            const uint32_t* __restrict__ keep) {
  extern __shared__ __attribute__((aligned(1024))) char fl_lds[];   // two stages of (K block, V block)
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = blockIdx.y, b = bh / heads, h = bh % heads;
  const long ld = 3L * H;
  const bf16_t* Q = qkv + ((long)b * S) * ld + h * 64;
  const int q0 = fl_seq_block() * FL_QB;
  const int i0 = q0 + wave * ATT_ROWS;
  const bool active = i0 < S;
  const int i = i0 + (lane & 15);
  const int jl = 8 * (lane >> 4);
  int len = lens ? lens[b] : S;
  len = len < 0 ? 0 : (len > S ? S : len);
  const int limit = causal ? (len < i + 1 ? len : i + 1) : len;
  const int q_end = q0 + FL_QB < S ? q0 + FL_QB : S;
  const int kmax = causal ? (len < q_end ? len : q_end) : len;
  const int nkb = (kmax + ATT_KC - 1) / ATT_KC;
  const long row_off = ((long)bh * S + i) * S;
  bf16x8_t qf[2], gf[2];
  float L = INFINITY, D = 0.f;
  if (active) {
    bf16x8_t of[2];
    load_frags(Q, i, ld, qf);
    load_frags(dc + ((long)b * S) * H + h * 64, i, H, gf);
    load_frags(ctx + ((long)b * S) * H + h * 64, i, H, of);
    L = lse[(long)bh * S + i];
    D = xgroup_sum(frag_dot(gf, of));
    if (lane < 16) dvec[(long)bh * S + i] = D;
  }
  f32x4_t dq[4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) dq[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  auto fetch = [&](int jb) {   // K and V rows of key block jb -> stage jb & 1
    const int key0 = jb * ATT_KC;
    const int rows = S - key0 < ATT_KC ? S - key0 : ATT_KC;
    char* st = fl_lds + (jb & 1) * 2 * HD_TILE;
    hd_tile_load(Q + H + (long)key0 * ld, ld, rows, st);
    hd_tile_load(Q + 2 * H + (long)key0 * ld, ld, rows, st + HD_TILE);
  };
  // this lane's keep bits of key block jb: one dword, requested one block ahead
  const bool kept = KEPT && active && drop.enabled;
  const uint32_t* kp = keep + ((long)bh * S + (kept ? i : 0)) * ((S + ATT_KC - 1) / ATT_KC) * 4 + (lane >> 4);
  uint32_t kw_next = 0;
  if (kept && nkb > 0) kw_next = kp[0];
  if (nkb > 0) fetch(0);
  for (int jb = 0; jb < nkb; ++jb) {
    const int key0 = jb * ATT_KC;
    const int rows = S - key0 < ATT_KC ? S - key0 : ATT_KC;
    const int npairs = rows / 32;
    const char* kt = fl_lds + (jb & 1) * 2 * HD_TILE;
    const char* vt = kt + HD_TILE;
    hd_tile_wait();
    __syncthreads();                                      // block jb has landed; every wave is done with block jb-1
    if (jb + 1 < nkb) fetch(jb + 1);
    const uint32_t kw = kw_next;
    if (kept && jb + 1 < nkb) kw_next = kp[(jb + 1) * 4];
    if (active) {
#pragma unroll
      for (int u = 0; u < ATT_PAIRS; ++u)
        if (u < npairs) {
          f32x4_t acc[2], dacc[2];
          group_products(kt, qf, u, acc);
          group_products(vt, gf, u, dacc);
          float mult[8], dsv[8];
          if (KEPT && drop.enabled) {
#pragma unroll
            for (int e = 0; e < 8; ++e) mult[e] = ((kw >> (8 * u + e)) & 1u) ? drop.scale : 0.f;
          } else if (drop.enabled) {
            drop_mult8(drop, (uint64_t)(row_off + key0 + 32 * u + jl), mult);
          } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) mult[e] = 1.f;
          }
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int j = key0 + 32 * u + jl + e;
            const float pe = j < limit ? exp2_hw(acc[e >> 2][e & 3] * alpha2 - L) : 0.f;
            dsv[e] = alpha * pe * (dacc[e >> 2][e & 3] * mult[e] - D);
          }
          const bf16x8_t df = __builtin_bit_cast(bf16x8_t, pack8_bf16(dsv));
#pragma unroll
          for (int nb = 0; nb < 4; ++nb)
            dq[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hd_frag_t(kt, u, nb), df, dq[nb], 0, 0, 0);
        }
    }
  }
  if (active) store_head_row(dqkv + ((long)b * S + i) * ld + h * 64, dq);
}

// dV = P~^T dC and dK = ds^T Q for the 128 keys of one block, over all query blocks
template <bool KEPT>
__global__ __launch_bounds__(512, 4) void attn_flash_dkv_kernel(const bf16_t* __restrict__ dc, const bf16_t* __restrict__ qkv,
                                                             const float* __restrict__ lse, const float* __restrict__ dvec,
                                                             const int32_t* __restrict__ lens, bf16_t* __restrict__ dqkv,
                                                             int S, int H, int heads, int causal, float alpha2,
                                                             float alpha, DropSite drop, const uint32_t* __restrict__ keep) {
  // two stages of (Q block, dC block, lse and D of its rows; KEPT: the keep bits of the block pair)
  extern __shared__ __attribute__((aligned(1024))) char fl_lds[];
  constexpr int STAGE = FL_DKV_STAGE + (KEPT ? FL_KEEP_TILE : 0);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bh = blockIdx.y, b = bh / heads, h = bh % heads;
  const long ld = 3L * H;
  const bf16_t* Q = qkv + ((long)b * S) * ld + h * 64;
  const bf16_t* DC = dc + ((long)b * S) * H + h * 64;
  const int jb = fl_seq_block();
  const int kbase = jb * ATT_KC + wave * ATT_ROWS;       // first key row of this wave
  const bool active = kbase < S;
  const int m = lane & 15, g = lane >> 4;
  const int k = kbase + m;                               // this lane's key row
  int len = lens ? lens[b] : S;
  len = len < 0 ? 0 : (len > S ? S : len);
  bf16x8_t kf[2], vf[2];
  if (active) {
    load_frags(Q + H, k, ld, kf);
    load_frags(Q + 2 * H, k, ld, vf);
  }
  f32x4_t dv[4], dk[4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) dv[nb] = dk[nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  const int nqb = (S + FL_QB - 1) / FL_QB;
  // causal: query blocks before this key block see none of its keys; keys beyond every length contribute nothing
  const int ib0 = causal ? jb : 0;
  const int ib1 = jb * ATT_KC < len ? nqb : ib0;
  auto fetch = [&](int ib) {   // Q and dC rows of query block ib and their row statistics -> stage ib & 1
    const int q0 = ib * FL_QB;
    const int rows = S - q0 < FL_QB ? S - q0 : FL_QB;
    char* st = fl_lds + (ib & 1) * STAGE;
    hd_tile_load(Q + (long)q0 * ld, ld, rows, st);
    hd_tile_load(DC + (long)q0 * H, H, rows, st + HD_TILE);
    if (wave < 4) {   // 4 bytes per lane: lse rows 0-63, 64-127, then D likewise (rows past the end re-read the last row)
      int q = q0 + (wave & 1) * 64 + lane;
      q = q < S ? q : S - 1;
      const float* src = (wave < 2 ? lse : dvec) + (long)bh * S + q;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (att_lds_ptr)(st + 2 * HD_TILE + wave * 256), 4, 0, 0);
    }
    if (KEPT && drop.enabled) {   // 4 bytes per lane: dword (thread & 3) of query row thread >> 2, this key block
      int q = q0 + (int)(threadIdx.x >> 2);
      q = q < S ? q : S - 1;
      const uint32_t* src = keep + (((long)bh * S + q) * ((S + ATT_KC - 1) / ATT_KC) + jb) * 4 + (threadIdx.x & 3);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (att_lds_ptr)(st + FL_DKV_STAGE + wave * 256), 4, 0, 0);
    }
  };
  if (ib0 < ib1) fetch(ib0);
  for (int ib = ib0; ib < ib1; ++ib) {
    const int q0 = ib * FL_QB;
    const int rows = S - q0 < FL_QB ? S - q0 : FL_QB;
    const int npairs = rows / 32;
    const char* qt = fl_lds + (ib & 1) * STAGE;
    const char* ct = qt + HD_TILE;
    const float* lse_t = reinterpret_cast<const float*>(ct + HD_TILE);
    const float* dvec_t = lse_t + FL_QB;
    hd_tile_wait();
    __syncthreads();                                      // block ib has landed; every wave is done with block ib-1
    if (ib + 1 < ib1) fetch(ib + 1);
    if (active) {
#pragma unroll
      for (int u = 0; u < ATT_PAIRS; ++u)
        if (u < npairs) {
          f32x4_t acc[2], dacc[2];
          group_products(qt, kf, u, acc);                 // own key row x 8 consecutive queries of the 32-query group
          group_products(ct, vf, u, dacc);
          const int qg = q0 + 32 * u + 8 * g;             // first of this lane's 8 queries in the group
          float Lv[8], Dv[8];
          *reinterpret_cast<float4*>(&Lv[0]) = *reinterpret_cast<const float4*>(lse_t + 32 * u + 8 * g);
          *reinterpret_cast<float4*>(&Lv[4]) = *reinterpret_cast<const float4*>(lse_t + 32 * u + 8 * g + 4);
          *reinterpret_cast<float4*>(&Dv[0]) = *reinterpret_cast<const float4*>(dvec_t + 32 * u + 8 * g);
          *reinterpret_cast<float4*>(&Dv[4]) = *reinterpret_cast<const float4*>(dvec_t + 32 * u + 8 * g + 4);
          // this lane's Philox block: query qg + (m & 7), keys kbase + 8*(m >> 3) .. +7; the lane that needs the bit
          // of (query qg + e, key k) fetches the block of lane (g, e + 8*(m >> 3)) and takes bit m & 7
          uint32_t mine = 0xffu;
          if (KEPT && drop.enabled) {
            // keys 16*wave + 8*(m >> 3) .. +7 of the block: octet 2*wave + (m >> 3) = 4*byte + dword
            const int row = 32 * u + 8 * g + (m & 7);
            mine = *reinterpret_cast<const uint8_t*>(qt + FL_DKV_STAGE + row * 16 + (2 * (wave & 1) + (m >> 3)) * 4 + (wave >> 1));
          } else if (drop.enabled) {
            mine = drop_keep8(drop, (uint64_t)(((long)bh * S + qg + (m & 7)) * S + kbase + 8 * (m >> 3)));
          }
          float pd[8], dsv[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t theirs = (uint32_t)__shfl((int)mine, (g << 4) | (e + 8 * (m >> 3)), WAVE);
            const float mult = drop.enabled ? (((theirs >> (m & 7)) & 1u) ? drop.scale : 0.f) : 1.f;
            const int q = qg + e;
            const bool admissible = k < len && (!causal || k <= q);
            const float pe = admissible ? exp2_hw(acc[e >> 2][e & 3] * alpha2 - Lv[e]) : 0.f;
            pd[e] = pe * mult;
            dsv[e] = alpha * pe * (dacc[e >> 2][e & 3] * mult - Dv[e]);
          }
          const bf16x8_t pf = __builtin_bit_cast(bf16x8_t, pack8_bf16(pd));
          const bf16x8_t df = __builtin_bit_cast(bf16x8_t, pack8_bf16(dsv));
#pragma unroll
          for (int nb = 0; nb < 4; ++nb) {
            dv[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hd_frag_t(ct, u, nb), pf, dv[nb], 0, 0, 0);
            dk[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hd_frag_t(qt, u, nb), df, dk[nb], 0, 0, 0);
          }
        }
    }
  }
  if (active) {
    bf16_t* out_row = dqkv + ((long)b * S + k) * ld + h * 64;
    store_head_row(out_row + H, dk);
    store_head_row(out_row + 2 * H, dv);
  }
}

// ----------------------------------------------------------------- launch --
bool attn_fused_supported(const raf_layer_desc& d) {
  return d.precision == RAF_BF16_AMP && d.hidden / d.heads == 64 && d.seq % 32 == 0 && d.seq <= ATT_KC;
}

raf_status launch_attn_fwd_fused(const raf_layer_desc& d, const void* qkv, const int32_t* lens, void* ctx, uint64_t step,
                                 hipStream_t st) {
  if (!qkv || !ctx) return RAF_EINVAL;
  if (!attn_fused_supported(d)) return RAF_ENOTSUP;
  const DropSite drop = make_drop_site(d, 1, step);
  hipLaunchKernelGGL(attn_fwd_fused_kernel, dim3(d.batch * d.heads, (d.seq + 63) / 64), dim3(256), 0, st, (const bf16_t*)qkv, lens,
                     (bf16_t*)ctx, d.seq, d.hidden, d.heads, d.causal, 0.125f * 1.44269504088896341f, drop);
  return check_launch();
}

raf_status launch_attn_bwd_full(const raf_layer_desc& d, const void* dc, const void* qkv, const int32_t* lens, void* dqkv,
                                uint64_t step, hipStream_t st) {
  if (!dc || !qkv || !dqkv) return RAF_EINVAL;
  if (!attn_fused_supported(d)) return RAF_ENOTSUP;
  static LdsLimitOnce lds_limit;
  if (!lds_limit.ensure((const void*)attn_bwd_full_kernel, ATT_BWD_LDS)) return RAF_EHIP;
  const DropSite drop = make_drop_site(d, 1, step);
  hipLaunchKernelGGL(attn_bwd_full_kernel, dim3(d.batch * d.heads), dim3(512), ATT_BWD_LDS, st, (const bf16_t*)dc,
                     (const bf16_t*)qkv, lens, (bf16_t*)dqkv, d.seq, d.hidden, d.heads, d.causal,
                     0.125f * 1.44269504088896341f, 0.125f, drop);
  return check_launch();
}

bool attn_flash_supported(const raf_layer_desc& d) {
  return d.precision == RAF_BF16_AMP && d.hidden / d.heads == 64 && d.seq % 32 == 0 && d.seq > ATT_KC;
}

size_t attn_flash_keep_bytes(const raf_layer_desc& d) {
  if (!attn_flash_supported(d) || !(d.dropout_p > 0.0)) return 0;
  return (size_t)d.batch * d.heads * d.seq * ((d.seq + ATT_KC - 1) / ATT_KC) * 16;
}

raf_status launch_attn_flash_fwd(const raf_layer_desc& d, const void* qkv, const int32_t* lens, void* ctx, float* lse,
                                 uint64_t step, hipStream_t st, uint32_t* keep) {
  if (!qkv || !ctx || !lse || ((uintptr_t)keep & 15u)) return RAF_EINVAL;
  if (!attn_flash_supported(d)) return RAF_ENOTSUP;
  const DropSite drop = make_drop_site(d, 1, step);
  dim3 grid((d.seq + FL_QB - 1) / FL_QB, d.batch * d.heads);
  static LdsLimitOnce lds_limit, lds_limit_kept;
  if (keep && drop.enabled) {
    if (!lds_limit_kept.ensure((const void*)attn_flash_fwd_kernel<true>, 2 * FL_STAGE)) return RAF_EHIP;
    hipLaunchKernelGGL(attn_flash_fwd_kernel<true>, grid, dim3(512), 2 * FL_STAGE, st, (const bf16_t*)qkv, lens, (bf16_t*)ctx,
                       lse, d.seq, d.hidden, d.heads, d.causal, 0.125f * 1.44269504088896341f, drop, keep);
  } else {
    if (!lds_limit.ensure((const void*)attn_flash_fwd_kernel<false>, 2 * FL_STAGE)) return RAF_EHIP;
    hipLaunchKernelGGL(attn_flash_fwd_kernel<false>, grid, dim3(512), 2 * FL_STAGE, st, (const bf16_t*)qkv, lens, (bf16_t*)ctx,
                       lse, d.seq, d.hidden, d.heads, d.causal, 0.125f * 1.44269504088896341f, drop, (uint32_t*)nullptr);
  }
  return check_launch();
}

raf_status launch_attn_flash_bwd(const raf_layer_desc& d, const void* dc, const void* qkv, const void* ctx,
                                 const float* lse, const int32_t* lens, void* dqkv, float* dvec, uint64_t step,
                                 hipStream_t st, const uint32_t* keep) {
  if (!dc || !qkv || !ctx || !lse || !dqkv || !dvec || ((uintptr_t)keep & 15u)) return RAF_EINVAL;
  if (!attn_flash_supported(d)) return RAF_ENOTSUP;
  const DropSite drop = make_drop_site(d, 1, step);
  const float alpha2 = 0.125f * 1.44269504088896341f;
  dim3 grid((d.seq + FL_QB - 1) / FL_QB, d.batch * d.heads);
  static LdsLimitOnce lds_dq, lds_dkv, lds_dq_kept, lds_dkv_kept;
  if (keep && drop.enabled) {
    constexpr int DKV_LDS = 2 * (FL_DKV_STAGE + FL_KEEP_TILE);
    if (!lds_dq_kept.ensure((const void*)attn_flash_dq_kernel<true>, 2 * FL_STAGE) ||
        !lds_dkv_kept.ensure((const void*)attn_flash_dkv_kernel<true>, DKV_LDS))
      return RAF_EHIP;
    hipLaunchKernelGGL(attn_flash_dq_kernel<true>, grid, dim3(512), 2 * FL_STAGE, st, (const bf16_t*)dc, (const bf16_t*)qkv,
                       (const bf16_t*)ctx, lse, lens, (bf16_t*)dqkv, dvec, d.seq, d.hidden, d.heads, d.causal, alpha2,
                       0.125f, drop, keep);
    const raf_status rc = check_launch();
    if (rc != RAF_OK) return rc;
    hipLaunchKernelGGL(attn_flash_dkv_kernel<true>, grid, dim3(512), DKV_LDS, st, (const bf16_t*)dc, (const bf16_t*)qkv, lse,
                       (const float*)dvec, lens, (bf16_t*)dqkv, d.seq, d.hidden, d.heads, d.causal, alpha2, 0.125f, drop,
                       keep);
    return check_launch();
  }
  if (!lds_dq.ensure((const void*)attn_flash_dq_kernel<false>, 2 * FL_STAGE) ||
      !lds_dkv.ensure((const void*)attn_flash_dkv_kernel<false>, 2 * FL_DKV_STAGE))
    return RAF_EHIP;
  hipLaunchKernelGGL(attn_flash_dq_kernel<false>, grid, dim3(512), 2 * FL_STAGE, st, (const bf16_t*)dc, (const bf16_t*)qkv,
                     (const bf16_t*)ctx, lse, lens, (bf16_t*)dqkv, dvec, d.seq, d.hidden, d.heads, d.causal, alpha2,
                     0.125f, drop, (const uint32_t*)nullptr);
  const raf_status rc = check_launch();
  if (rc != RAF_OK) return rc;
  hipLaunchKernelGGL(attn_flash_dkv_kernel<false>, grid, dim3(512), 2 * FL_DKV_STAGE, st, (const bf16_t*)dc, (const bf16_t*)qkv,
                     lse, (const float*)dvec, lens, (bf16_t*)dqkv, d.seq, d.hidden, d.heads, d.causal, alpha2, 0.125f, drop,
                     (const uint32_t*)nullptr);
  return check_launch();
}

}  // namespace raf
