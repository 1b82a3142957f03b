// Fused multi-tensor Adam with loss-scale removal and the bf16 weight copy
// (optimizer inside the training step with in-place parameter update, paper
// Section 3; the AMP cast fused into its producer, Section 3.1.2), the loss
// seed of the benchmark workload, and the dropout-mask test hook.
#include <cmath>

#include "common.hpp"

namespace raf {

constexpr int ADAM_MAX_TENSORS = 48;       // per launch (kernel-argument budget)
constexpr int ADAM_CHUNK = 256 * 4 * 4;    // elements per block
// tensors with a transposed copy are walked in tiles of 32 rows x 128 columns (= one chunk): row pieces of 512 bytes
// on the float side, 64-byte column pieces on the transposed bf16 side (measured against 64 x 64 and 16 x 256)
constexpr int ADAM_TILE_R = 32, ADAM_TILE_C = ADAM_CHUNK / ADAM_TILE_R;

struct AdamTable {
  float* master[ADAM_MAX_TENSORS];
  const float* grad[ADAM_MAX_TENSORS];
  float* m[ADAM_MAX_TENSORS];
  float* v[ADAM_MAX_TENSORS];
  bf16_t* lowp[ADAM_MAX_TENSORS];
  bf16_t* lowp_t[ADAM_MAX_TENSORS];        // transposed bf16 copy, or null
  long n[ADAM_MAX_TENSORS];
  int rows[ADAM_MAX_TENSORS], cols[ADAM_MAX_TENSORS];   // matrix view of a tensor with lowp_t
  int block_start[ADAM_MAX_TENSORS + 1];   // first block of each tensor
  int count;
};

struct AdamHyper {
  float lr_over_bc1, inv_bc2, beta1, beta2, one_minus_beta1, one_minus_beta2, eps, weight_decay, inv_scale;
  float lr, ln_beta1, ln_beta2;   // dynamic entry point only: the step count is read on the device
};

__device__ __forceinline__ void adam_update(float& w, float g, float& m, float& v, const AdamHyper& h) {
  g = g * h.inv_scale + h.weight_decay * w;
  m = h.beta1 * m + h.one_minus_beta1 * g;
  v = h.beta2 * v + h.one_minus_beta2 * g * g;
  w = w - h.lr_over_bc1 * m / (sqrtf(v * h.inv_bc2) + h.eps);
}

// One block's share of one tensor: chunk `block` of the flat element range, or tile `block` of a matrix that keeps a
// transposed bf16 copy.
// The optimizer's fp32 streams (master weights, moments, gradients) are touched once per step and are as large as
// the memory-side cache: loaded and stored with the non-temporal hint they do not push the bf16 weights and the
// activations of the next forward pass out of L2 and the memory-side cache, and less dirty data is left for the
// write-back at the end of the kernel (BERT-base step 0.368 -> 0.342 ms).  The bf16 copies are stored normally:
// the next pass reads them.
__device__ __forceinline__ float4 stream_load4(const float* p) {
  const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
  return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void stream_store4(float* p, const float4& v) {
  const f32x4_t o = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(o, reinterpret_cast<f32x4_t*>(p));
}
__device__ __forceinline__ void adam_block(float* __restrict__ W, const float* __restrict__ G, float* __restrict__ Mo,
                                           float* __restrict__ Vo, bf16_t* __restrict__ L, bf16_t* __restrict__ LT,
                                           long n, int rows, int cols, int block, const AdamHyper& h) {
  if (LT) {
    // A matrix that also keeps a transposed bf16 copy: one tile per block.  Each thread updates pieces of 4 consecutive
    // elements, leaves the rounded weights in an LDS tile stored transposed, and the block then writes the tile's
    // columns as rows of the transposed copy, 16 bytes per store.
    __shared__ uint16_t tile[ADAM_TILE_C][ADAM_TILE_R + 2];   // [column][row] of the tile
    constexpr int LANES_C = ADAM_TILE_C / 4;                   // threads along a row piece
    constexpr int ROWS_PASS = 256 / LANES_C;                   // rows per pass of the workgroup
    const int tiles_c = (cols + ADAM_TILE_C - 1) / ADAM_TILE_C;
    const int tb = block;
    const int r0 = (tb / tiles_c) * ADAM_TILE_R, c0 = (tb % tiles_c) * ADAM_TILE_C;
    const int cl = (threadIdx.x % LANES_C) * 4;
#pragma unroll
    for (int it = 0; it < ADAM_TILE_R / ROWS_PASS; ++it) {
      const int rl = it * ROWS_PASS + (threadIdx.x / LANES_C);
      const int r = r0 + rl, c = c0 + cl;
      if (r < rows && c < cols) {      // cols is a multiple of 8: a 4-element piece is inside or outside as a whole
        const long i = (long)r * cols + c;
        float4 w = stream_load4(W + i);
        const float4 g = stream_load4(G + i);
        float4 m = stream_load4(Mo + i);
        float4 v = stream_load4(Vo + i);
        adam_update(w.x, g.x, m.x, v.x, h);
        adam_update(w.y, g.y, m.y, v.y, h);
        adam_update(w.z, g.z, m.z, v.z, h);
        adam_update(w.w, g.w, m.w, v.w, h);
        stream_store4(W + i, w);
        stream_store4(Mo + i, m);
        stream_store4(Vo + i, v);
        uint2 p;
        p.x = pack_bf16x2(w.x, w.y);
        p.y = pack_bf16x2(w.z, w.w);
        if (L) *reinterpret_cast<uint2*>(L + i) = p;
        tile[cl + 0][rl] = (uint16_t)(p.x & 0xffffu);
        tile[cl + 1][rl] = (uint16_t)(p.x >> 16);
        tile[cl + 2][rl] = (uint16_t)(p.y & 0xffffu);
        tile[cl + 3][rl] = (uint16_t)(p.y >> 16);
      }
    }
    __syncthreads();
    // transposed copy: row (c0 + tc) of [cols, rows], 8 consecutive elements (16 bytes) per store
    constexpr int PIECES = ADAM_TILE_R / 8;                    // 16-byte pieces per tile column
    for (int q = threadIdx.x; q < ADAM_TILE_C * PIECES; q += 256) {
      const int tc = q / PIECES, rl = (q % PIECES) * 8;
      if (c0 + tc < cols && r0 + rl < rows) {   // rows is a multiple of 8
        const uint16_t* src = &tile[tc][rl];
        uint4 o;
        o.x = (uint32_t)src[0] | ((uint32_t)src[1] << 16);
        o.y = (uint32_t)src[2] | ((uint32_t)src[3] << 16);
        o.z = (uint32_t)src[4] | ((uint32_t)src[5] << 16);
        o.w = (uint32_t)src[6] | ((uint32_t)src[7] << 16);
        *reinterpret_cast<uint4*>(LT + (long)(c0 + tc) * rows + r0 + rl) = o;
      }
    }
    return;
  }
  const long base = (long)block * ADAM_CHUNK;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const long i = base + ((long)it * 256 + threadIdx.x) * 4;
    if (i + 3 < n) {
      float4 w = stream_load4(W + i);
      const float4 g = stream_load4(G + i);
      float4 m = stream_load4(Mo + i);
      float4 v = stream_load4(Vo + i);
      adam_update(w.x, g.x, m.x, v.x, h);
      adam_update(w.y, g.y, m.y, v.y, h);
      adam_update(w.z, g.z, m.z, v.z, h);
      adam_update(w.w, g.w, m.w, v.w, h);
      stream_store4(W + i, w);
      stream_store4(Mo + i, m);
      stream_store4(Vo + i, v);
      if (L) {
        uint2 p;
        p.x = pack_bf16x2(w.x, w.y);
        p.y = pack_bf16x2(w.z, w.w);
        *reinterpret_cast<uint2*>(L + i) = p;
      }
    } else {
      for (long j = i; j < n && j < i + 4; ++j) {
        float w = W[j], m = Mo[j], v = Vo[j];
        adam_update(w, G[j], m, v, h);
        W[j] = w;
        Mo[j] = m;
        Vo[j] = v;
        if (L) L[j] = (bf16_t)w;
      }
    }
  }
}

// the dynamic entry points: step count and loss scale come from the device-resident scaler state; false: the step's
// gradients held a non-finite value and the whole launch is a no-op
__device__ __forceinline__ bool adam_dynamic(AdamHyper& h, const raf_scaler_state* __restrict__ dyn) {
  if (dyn->found_inf) return false;
  h.inv_scale = dyn->inv_scale;
  // bias corrections 1 - beta^t of step t + 1 as -expm1(t ln beta): accurate to a few float ulps also where
  // beta^t is close to 1, and cheap enough to be formed by every thread instead of by a launch of its own
  const float tf = (float)(dyn->t + 1);
  h.lr_over_bc1 = h.lr / -expm1f(tf * h.ln_beta1);
  h.inv_bc2 = 1.0f / -expm1f(tf * h.ln_beta2);
  return true;
}

// tensor table in the kernel arguments (at most ADAM_MAX_TENSORS tensors)
__global__ __launch_bounds__(256) void adam_kernel(AdamTable tab, AdamHyper h, const raf_scaler_state* __restrict__ dyn) {
  if (dyn && !adam_dynamic(h, dyn)) return;
  int ti = 0;
  while (ti + 1 < tab.count && (int)blockIdx.x >= tab.block_start[ti + 1]) ++ti;
  adam_block(tab.master[ti], tab.grad[ti], tab.m[ti], tab.v[ti], tab.lowp[ti], tab.lowp_t[ti], tab.n[ti], tab.rows[ti],
             tab.cols[ti], (int)blockIdx.x - tab.block_start[ti], h);
}

// Tensor table in device memory, for lists of any length in ONE launch: `entries` is a device copy of the caller's
// list without its empty tensors, block_start[i] the first block of entry i, block_entry[b] the entry block b works on
// (one dependent read instead of a search).
__global__ __launch_bounds__(256) void adam_table_kernel(const raf_adam_tensor* __restrict__ entries,
                                                         const int* __restrict__ block_start,
                                                         const int* __restrict__ block_entry, AdamHyper h,
                                                         const raf_scaler_state* __restrict__ dyn) {
  if (dyn && !adam_dynamic(h, dyn)) return;
  const int ti = block_entry[blockIdx.x];
  const raf_adam_tensor e = entries[ti];
  adam_block(e.master, e.grad, e.m, e.v, (bf16_t*)e.lowp, (bf16_t*)e.lowp_t, (long)e.n, e.rows, e.cols,
             (int)blockIdx.x - block_start[ti], h);
}

// writes entries [first, first + n) of the device table from kernel arguments: workgroup i takes entry first + i and
// the block numbers that belong to it
constexpr int ADAM_FILL = 32;
struct AdamFillChunk {
  raf_adam_tensor e[ADAM_FILL];
  int start[ADAM_FILL + 1];
};
__global__ __launch_bounds__(256) void adam_table_fill_kernel(AdamFillChunk c, raf_adam_tensor* __restrict__ entries,
                                                              int* __restrict__ block_start,
                                                              int* __restrict__ block_entry, int first) {
  const int i = blockIdx.x;
  if (threadIdx.x == 0) {
    entries[first + i] = c.e[i];
    block_start[first + i] = c.start[i];
    block_start[first + i + 1] = c.start[i + 1];   // the next entry's workgroup writes the same value
  }
  for (int b = c.start[i] + (int)threadIdx.x; b < c.start[i + 1]; b += 256) block_entry[b] = first + i;
}

// ------------------------------------------------------------- loss seed --
template <typename T>
__global__ __launch_bounds__(256) void loss_seed_kernel(const T* __restrict__ y, const T* __restrict__ G, long n,
                                                        float loss_scale, const float* __restrict__ scale_ptr,
                                                        T* __restrict__ dy, float* __restrict__ partial) {
  __shared__ float red[4];
  if (scale_ptr) loss_scale = *scale_ptr;   // dynamic loss scale, device-resident
  float acc = 0.f;
  for (long i = ((long)blockIdx.x * 256 + threadIdx.x) * 8; i < n; i += (long)gridDim.x * 256 * 8) {
    float a[8], g[8];
    Vec8<T>::load(y + i, a);
    Vec8<T>::load(G + i, g);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      acc += a[e] * g[e];
      g[e] *= loss_scale;
    }
    Vec8<T>::store(dy + i, g);
  }
  acc = group_sum<64>(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// one wavefront: each lane adds its share of the partial sums in ascending order, the 64 lane sums are then folded by
// xor shuffles; no LDS, no barrier, a fixed order
__global__ __launch_bounds__(64) void loss_final_kernel(const float* __restrict__ partial, int nparts,
                                                        float* __restrict__ loss_out) {
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  int i = threadIdx.x;
  for (; i + 192 < nparts; i += 256) {   // four loads in flight
    const float a = partial[i], b = partial[i + 64], c = partial[i + 128], d = partial[i + 192];
    acc[0] += a; acc[1] += b; acc[2] += c; acc[3] += d;
  }
  for (; i < nparts; i += 64) acc[0] += partial[i];
  const float sum = group_sum<64>((acc[0] + acc[1]) + (acc[2] + acc[3]));
  if (threadIdx.x == 0) *loss_out = sum;
}

raf_status launch_sum_partials(const float* partial, int nparts, float* out, hipStream_t st) {
  if (!partial || !out || nparts <= 0) return RAF_EINVAL;
  hipLaunchKernelGGL(loss_final_kernel, dim3(1), dim3(64), 0, st, partial, nparts, out);
  return check_launch();
}

// -------------------------------------------------- dynamic loss scale ---
__global__ void scaler_init_kernel(raf_scaler_state* st, float scale) {
  st->scale = scale;
  st->inv_scale = 1.0f / scale;
  st->good_steps = 0;
  st->found_inf = 0;
  st->t = 0;
  st->lr_over_bc1 = 0.f;
  st->inv_bc2 = 0.f;
}

// one chunk of one gradient tensor per block (the Adam partition); any non-finite element raises the flag
__global__ __launch_bounds__(256) void grads_check_kernel(AdamTable tab, int* flag) {
  int ti = 0;
  while (ti + 1 < tab.count && (int)blockIdx.x >= tab.block_start[ti + 1]) ++ti;
  const long n = tab.n[ti];
  const float* __restrict__ G = tab.grad[ti];
  const long base = (long)(blockIdx.x - tab.block_start[ti]) * ADAM_CHUNK;
  bool bad = false;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const long i = base + ((long)it * 256 + threadIdx.x) * 4;
    if (i + 3 < n) {
      const float4 g = *reinterpret_cast<const float4*>(G + i);
      // x - x is 0 for finite x and nan for inf and nan
      bad |= !((g.x - g.x) + (g.y - g.y) + (g.z - g.z) + (g.w - g.w) == 0.f);
    } else {
      for (long j = i; j < n && j < i + 4; ++j) bad |= !(G[j] - G[j] == 0.f);
    }
  }
  if (__any(bad) && (threadIdx.x & 63) == 0) *flag = 1;   // every writer stores the same value
}

__global__ void scaler_update_kernel(raf_scaler_state* st, float growth, float backoff, int interval) {
  float scale = st->scale;
  if (st->found_inf) {
    scale *= backoff;
    st->good_steps = 0;
  } else {
    st->t += 1;
    const int good = st->good_steps + 1;
    if (good == interval) {
      scale *= growth;
      st->good_steps = 0;
    } else {
      st->good_steps = good;
    }
  }
  st->scale = scale;
  st->inv_scale = 1.0f / scale;
  st->found_inf = 0;
}

// ------------------------------------------------------- mask test hook ---
__global__ __launch_bounds__(256) void dropout_mask_kernel(uint8_t* __restrict__ out, long n, DropSite drop) {
  const long i8 = ((long)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i8 >= n) return;
  float mult[8];
  if (drop.enabled) {
    drop_mult8(drop, (uint64_t)i8, mult);
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) mult[e] = 1.f;
  }
  for (int e = 0; e < 8 && i8 + e < n; ++e) out[i8 + e] = mult[e] != 0.f ? 1 : 0;
}

raf_status launch_nonfinite_check(const float* const* ptrs, const long* n, int count, int* flag, hipStream_t st) {
  if (!ptrs || !n || !flag || count <= 0 || count > ADAM_MAX_TENSORS) return RAF_EINVAL;
  AdamTable tab{};
  long blocks = 0;
  for (int i = 0; i < count; ++i) {
    if (!ptrs[i] || n[i] <= 0 || !aligned16(ptrs[i])) return RAF_EINVAL;
    const int k = tab.count++;
    tab.grad[k] = ptrs[i];
    tab.n[k] = n[i];
    tab.block_start[k] = (int)blocks;
    blocks += (n[i] + ADAM_CHUNK - 1) / ADAM_CHUNK;
  }
  tab.block_start[tab.count] = (int)blocks;
  hipLaunchKernelGGL(grads_check_kernel, dim3((unsigned)blocks), dim3(256), 0, st, tab, flag);
  return check_launch();
}

}  // namespace raf

using namespace raf;

#define RAF_TRY(expr)                \
  do {                               \
    const raf_status _rc = (expr);   \
    if (_rc != RAF_OK) return _rc;   \
  } while (0)

static raf_status check_adam_list(const raf_adam_tensor* list, int32_t count) {
  if (count < 0 || (count > 0 && !list)) return RAF_EINVAL;
  for (int i = 0; i < count; ++i) {
    const raf_adam_tensor& a = list[i];
    if (a.n < 0) return RAF_EINVAL;
    if (a.n == 0) continue;
    if (!a.master || !a.grad || !a.m || !a.v) return RAF_EINVAL;
    if (!aligned16(a.master) || !aligned16(a.grad) || !aligned16(a.m) || !aligned16(a.v) || !aligned16(a.lowp))
      return RAF_EINVAL;
    if (a.lowp_t) {
      if (!aligned16(a.lowp_t) || a.rows <= 0 || a.cols <= 0 || (a.rows % 8) || (a.cols % 8)) return RAF_EINVAL;
      if ((int64_t)a.rows * a.cols != a.n) return RAF_EINVAL;
    }
  }
  return RAF_OK;
}

// Splits the list into kernel-argument tables of at most ADAM_MAX_TENSORS tensors, one chunk of one tensor per
// block, and calls launch(table, blocks) for each.
template <typename F>
static raf_status for_each_adam_table(const raf_adam_tensor* list, int32_t count, F&& launch) {
  int i = 0;
  while (i < count) {
    AdamTable tab;
    tab.count = 0;
    long blocks = 0;
    while (i < count && tab.count < ADAM_MAX_TENSORS) {
      const raf_adam_tensor& a = list[i++];
      if (a.n == 0) continue;
      const long nb = a.lowp_t ? (long)((a.rows + ADAM_TILE_R - 1) / ADAM_TILE_R) * ((a.cols + ADAM_TILE_C - 1) / ADAM_TILE_C)
                               : (a.n + ADAM_CHUNK - 1) / ADAM_CHUNK;
      if (blocks + nb > 0x7fffffff) return RAF_ENOTSUP;
      const int k = tab.count++;
      tab.master[k] = a.master; tab.grad[k] = a.grad; tab.m[k] = a.m; tab.v[k] = a.v;
      tab.lowp[k] = (bf16_t*)a.lowp; tab.n[k] = a.n;
      tab.lowp_t[k] = (bf16_t*)a.lowp_t; tab.rows[k] = a.lowp_t ? a.rows : 0; tab.cols[k] = a.lowp_t ? a.cols : 0;
      tab.block_start[k] = (int)blocks;
      blocks += nb;
    }
    if (tab.count == 0) continue;
    tab.block_start[tab.count] = (int)blocks;
    launch(tab, (unsigned)blocks);
    raf_status rc = check_launch();
    if (rc != RAF_OK) return rc;
  }
  return RAF_OK;
}

static AdamHyper adam_constants(double beta1, double beta2, double eps, double weight_decay) {
  AdamHyper h{};
  h.beta1 = (float)beta1;
  h.beta2 = (float)beta2;
  h.one_minus_beta1 = (float)(1.0 - beta1);
  h.one_minus_beta2 = (float)(1.0 - beta2);
  h.eps = (float)eps;
  h.weight_decay = (float)weight_decay;
  return h;
}

extern "C" raf_status raf_adam_step(const raf_adam_tensor* list, int32_t count, double lr, double beta1, double beta2,
                                    double eps, double weight_decay, int64_t t, double inv_loss_scale,
                                    void* hip_stream) {
  RAF_TRY(check_adam_list(list, count));
  if (t < 1 || !(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0)) return RAF_EINVAL;
  AdamHyper h = adam_constants(beta1, beta2, eps, weight_decay);
  const double bc1 = 1.0 - pow(beta1, (double)t);
  const double bc2 = 1.0 - pow(beta2, (double)t);
  h.lr_over_bc1 = (float)(lr / bc1);
  h.inv_bc2 = (float)(1.0 / bc2);
  h.inv_scale = (float)inv_loss_scale;
  hipStream_t st = (hipStream_t)hip_stream;
  return for_each_adam_table(list, count, [&](const AdamTable& tab, unsigned blocks) {
    hipLaunchKernelGGL(adam_kernel, dim3(blocks), dim3(256), 0, st, tab, h, (const raf_scaler_state*)nullptr);
  });
}

// ---- tensor table in device memory: any number of tensors in one launch
static long adam_blocks_of(const raf_adam_tensor& a) {
  return a.lowp_t ? (long)((a.rows + ADAM_TILE_R - 1) / ADAM_TILE_R) * ((a.cols + ADAM_TILE_C - 1) / ADAM_TILE_C)
                  : (a.n + ADAM_CHUNK - 1) / ADAM_CHUNK;
}
static size_t pad256(size_t n) { return (n + 255) & ~(size_t)255; }
// entries | block_start[live + 1] | block_entry[blocks]; false: too many blocks for one launch
static bool adam_table_layout(const raf_adam_tensor* list, int32_t count, int* live, long* blocks, size_t* off_start,
                              size_t* off_entry, size_t* bytes) {
  *live = 0;
  *blocks = 0;
  for (int i = 0; i < count; ++i) {
    if (list[i].n == 0) continue;   // empty tensors take no entry
    ++*live;
    *blocks += adam_blocks_of(list[i]);
    if (*blocks > 0x7fffffff) return false;
  }
  *off_start = pad256((size_t)*live * sizeof(raf_adam_tensor));
  *off_entry = *off_start + pad256(((size_t)*live + 1) * sizeof(int));
  *bytes = *off_entry + pad256((size_t)*blocks * sizeof(int));
  return true;
}

extern "C" size_t raf_adam_table_bytes(const raf_adam_tensor* list, int32_t count) {
  if (check_adam_list(list, count) != RAF_OK) return 0;
  int live; long blocks; size_t o1, o2, bytes;
  if (!adam_table_layout(list, count, &live, &blocks, &o1, &o2, &bytes)) return 0;
  return bytes;
}

extern "C" raf_status raf_adam_table_fill(const raf_adam_tensor* list, int32_t count, void* table, void* hip_stream) {
  RAF_TRY(check_adam_list(list, count));
  int live; long total; size_t o1, o2, bytes;
  if (!adam_table_layout(list, count, &live, &total, &o1, &o2, &bytes)) return RAF_ENOTSUP;
  if (live == 0) return RAF_OK;
  if (!table || ((uintptr_t)table & 255u)) return RAF_EINVAL;
  raf_adam_tensor* entries = (raf_adam_tensor*)table;
  int* block_start = (int*)((char*)table + o1);
  int* block_entry = (int*)((char*)table + o2);
  hipStream_t st = (hipStream_t)hip_stream;
  AdamFillChunk c;
  int filled = 0, first = 0;
  long blocks = 0;
  auto flush = [&]() -> raf_status {
    if (filled == 0) return RAF_OK;
    c.start[filled] = (int)blocks;
    hipLaunchKernelGGL(adam_table_fill_kernel, dim3(filled), dim3(256), 0, st, c, entries, block_start, block_entry, first);
    first += filled;
    filled = 0;
    return check_launch();
  };
  for (int i = 0; i < count; ++i) {
    if (list[i].n == 0) continue;
    c.e[filled] = list[i];
    c.start[filled] = (int)blocks;
    blocks += adam_blocks_of(list[i]);
    if (++filled == ADAM_FILL) RAF_TRY(flush());
  }
  return flush();
}

extern "C" raf_status raf_adam_step_table(const raf_adam_tensor* list, int32_t count, const void* table, double lr,
                                          double beta1, double beta2, double eps, double weight_decay, int64_t t,
                                          double inv_loss_scale, const raf_scaler_state* state, void* hip_stream) {
  RAF_TRY(check_adam_list(list, count));
  if (!(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0)) return RAF_EINVAL;
  if (!state && t < 1) return RAF_EINVAL;
  if (state && !aligned16(state)) return RAF_EINVAL;
  // the partition of fill time, recomputed from the list (which must be the one the table was filled from)
  int live; long blocks; size_t o1, o2, bytes;
  if (!adam_table_layout(list, count, &live, &blocks, &o1, &o2, &bytes)) return RAF_ENOTSUP;
  if (live == 0) return RAF_OK;
  if (!table || ((uintptr_t)table & 255u)) return RAF_EINVAL;
  AdamHyper h = adam_constants(beta1, beta2, eps, weight_decay);
  if (state) {
    h.lr = (float)lr;
    h.ln_beta1 = (float)log(beta1);
    h.ln_beta2 = (float)log(beta2);
  } else {
    const double bc1 = 1.0 - pow(beta1, (double)t), bc2 = 1.0 - pow(beta2, (double)t);
    h.lr_over_bc1 = (float)(lr / bc1);
    h.inv_bc2 = (float)(1.0 / bc2);
    h.inv_scale = (float)inv_loss_scale;
  }
  hipLaunchKernelGGL(adam_table_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                     (const raf_adam_tensor*)table, (const int*)((const char*)table + o1),
                     (const int*)((const char*)table + o2), h, state);
  return check_launch();
}

extern "C" raf_status raf_scaler_init(raf_scaler_state* state, float init_scale, void* hip_stream) {
  if (!state || !aligned16(state) || !(init_scale > 0.f) || !(init_scale <= 3.0e38f)) return RAF_EINVAL;
  hipLaunchKernelGGL(scaler_init_kernel, dim3(1), dim3(1), 0, (hipStream_t)hip_stream, state, init_scale);
  return check_launch();
}

extern "C" raf_status raf_grads_check(const raf_adam_tensor* list, int32_t count, raf_scaler_state* state,
                                      void* hip_stream) {
  RAF_TRY(check_adam_list(list, count));
  if (!state || !aligned16(state)) return RAF_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  return for_each_adam_table(list, count, [&](const AdamTable& tab, unsigned blocks) {
    hipLaunchKernelGGL(grads_check_kernel, dim3(blocks), dim3(256), 0, st, tab, &state->found_inf);
  });
}

extern "C" raf_status raf_adam_step_scaled(const raf_adam_tensor* list, int32_t count, double lr, double beta1,
                                           double beta2, double eps, double weight_decay, raf_scaler_state* state,
                                           void* hip_stream) {
  RAF_TRY(check_adam_list(list, count));
  if (!state || !aligned16(state)) return RAF_EINVAL;
  if (!(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0)) return RAF_EINVAL;
  AdamHyper h = adam_constants(beta1, beta2, eps, weight_decay);
  h.lr = (float)lr;
  h.ln_beta1 = (float)log(beta1);   // -inf for beta = 0: the correction is then 1
  h.ln_beta2 = (float)log(beta2);
  hipStream_t st = (hipStream_t)hip_stream;
  return for_each_adam_table(list, count, [&](const AdamTable& tab, unsigned blocks) {
    hipLaunchKernelGGL(adam_kernel, dim3(blocks), dim3(256), 0, st, tab, h, (const raf_scaler_state*)state);
  });
}

extern "C" raf_status raf_scaler_update(raf_scaler_state* state, float growth_factor, float backoff_factor,
                                        int32_t growth_interval, void* hip_stream) {
  if (!state || !aligned16(state)) return RAF_EINVAL;
  if (!(growth_factor >= 1.f) || !(backoff_factor > 0.f && backoff_factor <= 1.f) || growth_interval < 1)
    return RAF_EINVAL;
  hipLaunchKernelGGL(scaler_update_kernel, dim3(1), dim3(1), 0, (hipStream_t)hip_stream, state, growth_factor,
                     backoff_factor, growth_interval);
  return check_launch();
}

static raf_status loss_seed_impl(int32_t precision, const void* y, const void* G, int64_t n, float loss_scale,
                                 const float* scale_ptr, float* loss_out, void* dy, float* partial, hipStream_t st) {
  if (!y || !G || !loss_out || !dy || !partial || n <= 0 || (n % 8)) return RAF_EINVAL;
  if (!aligned16(y) || !aligned16(G) || !aligned16(dy)) return RAF_EINVAL;
  if (precision != RAF_F32 && precision != RAF_BF16_AMP) return RAF_EINVAL;
  long nb = (n / 8 + 255) / 256;
  if (nb > RAF_LOSS_PARTIALS) nb = RAF_LOSS_PARTIALS;
  if (precision == RAF_F32)
    hipLaunchKernelGGL((loss_seed_kernel<float>), dim3(nb), dim3(256), 0, st, (const float*)y, (const float*)G,
                       (long)n, loss_scale, scale_ptr, (float*)dy, partial);
  else
    hipLaunchKernelGGL((loss_seed_kernel<bf16_t>), dim3(nb), dim3(256), 0, st, (const bf16_t*)y, (const bf16_t*)G,
                       (long)n, loss_scale, scale_ptr, (bf16_t*)dy, partial);
  raf_status rc = check_launch();
  if (rc != RAF_OK) return rc;
  hipLaunchKernelGGL(loss_final_kernel, dim3(1), dim3(64), 0, st, partial, (int)nb, loss_out);
  return check_launch();
}

extern "C" raf_status raf_loss_seed(int32_t precision, const void* y, const void* G, int64_t n, float loss_scale,
                                    float* loss_out, void* dy, float* partial, void* hip_stream) {
  return loss_seed_impl(precision, y, G, n, loss_scale, nullptr, loss_out, dy, partial, (hipStream_t)hip_stream);
}

extern "C" raf_status raf_loss_seed_scaled(int32_t precision, const void* y, const void* G, int64_t n,
                                           const raf_scaler_state* state, float* loss_out, void* dy, float* partial,
                                           void* hip_stream) {
  if (!state || !aligned16(state)) return RAF_EINVAL;
  return loss_seed_impl(precision, y, G, n, 1.0f, &state->scale, loss_out, dy, partial, (hipStream_t)hip_stream);
}

extern "C" raf_status raf_debug_dropout_mask(const raf_layer_desc* desc, int32_t site, uint64_t step,
                                             uint8_t* mask_out, int64_t n, void* hip_stream) {
  if (!desc || !mask_out || n <= 0 || site < 1 || site > 255) return RAF_EINVAL;
  if (!(desc->dropout_p >= 0.0 && desc->dropout_p < 1.0)) return RAF_EINVAL;
  if ((uint64_t)n / 4 > 0xffffffffull) return RAF_ENOTSUP;
  const DropSite drop = make_drop_site(*desc, site, step);
  const long nb = ((n + 7) / 8 + 255) / 256;
  hipLaunchKernelGGL(dropout_mask_kernel, dim3(nb), dim3(256), 0, (hipStream_t)hip_stream, mask_out, (long)n, drop);
  return check_launch();
}
