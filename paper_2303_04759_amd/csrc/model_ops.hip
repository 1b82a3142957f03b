// Whole-model pieces around the layer stack: token + position embedding with
// LayerNorm and dropout (forward and adjoint, including the reproducible
// scatter-add into the word-table gradient), and the masked-language-model head
// with a decoder tied to the word table and a fused softmax cross-entropy.
// Same composition (paper Section 2.1), adjoint (3.1.1), precision (3.1.2) and
// fusion (3.2.2) rules as the layer.
#include "common.hpp"

namespace raf {

// ------------------------------------------------------------- embedding --
// One row per LPR-lane group: z0 = word[id] + pos[s]; e = LN(z0); x0 = e * keep/(1-p).
template <typename T, int LPR, int NV>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const int32_t* __restrict__ ids, const T* __restrict__ word,
                                                        const T* __restrict__ pos, const float* __restrict__ gamma,
                                                        const float* __restrict__ beta, T* __restrict__ x0,
                                                        T* __restrict__ z_out, float* __restrict__ mu,
                                                        float* __restrict__ rstd, long nrows, int S, int H, int vocab,
                                                        float eps, DropSite drop) {
  const int lane = threadIdx.x & (LPR - 1);
  const long row = ((long)blockIdx.x * 256 + threadIdx.x) / LPR;
  if (row >= nrows) return;
  const int nvec = H / 8;
  int id = ids[row];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);   // out-of-range ids are clamped, never read out of bounds
  const int s = (int)(row % S);
  float z[NV][8];
  float sum = 0.f;
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    if (vec < nvec) {
      float w[8], p[8];
      Vec8<T>::load(word + (long)id * H + vec * 8, w);
      Vec8<T>::load(pos + (long)s * H + vec * 8, p);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        z[t][e] = Vec8<T>::round(w[e] + p[e]);
        sum += z[t][e];
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) z[t][e] = 0.f;
    }
  }
  const float mean = group_sum<LPR>(sum) / (float)H;
  float sq = 0.f;
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    if (vec < nvec) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float d = z[t][e] - mean;
        sq += d * d;
      }
    }
  }
  const float rs = 1.0f / sqrtf(group_sum<LPR>(sq) / (float)H + eps);
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    if (vec < nvec) {
      const long off = row * H + vec * 8;
      float gm[8], bt[8], o[8];
      load8f(gamma + vec * 8, gm);
      load8f(beta + vec * 8, bt);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (z[t][e] - mean) * rs * gm[e] + bt[e];
      if (drop.enabled) {
        float mult[8];
        drop_mult8(drop, (uint64_t)off, mult);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= mult[e];
      }
      Vec8<T>::store(x0 + off, o);
      Vec8<T>::store(z_out + off, z[t]);
    }
  }
  if (lane == 0) {
    mu[row] = mean;
    rstd[row] = rs;
  }
}

// dword[id] += sum over positions t with ids[t] == id of dz[t], in ascending t.
// One workgroup per position; only the first position of each id (its
// "leader") does the work, so every table row has one writer and the order of
// the additions is fixed.
template <typename T>
__global__ __launch_bounds__(256) void embed_dword_kernel(const int32_t* __restrict__ ids, const T* __restrict__ dz,
                                                          float* __restrict__ dword, int nrows, int H, int vocab) {
  const int t0 = blockIdx.x;
  int id = ids[t0];
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
  const int lane = threadIdx.x & 63;
  // the id list is scanned 256 positions at a time: four independent loads per lane and round trip (one load per
  // round trip made the two scans, 128 round trips for 8192 positions, the whole cost of the kernel)
  auto clamped = [&](int t, int limit) {
    int other = ids[t < limit ? t : limit - 1];
    other = other < 0 ? 0 : (other >= vocab ? vocab - 1 : other);
    return t < limit ? other : -1;
  };
  // is there an earlier position with the same (clamped) id?
  for (int base = 0; base < t0; base += 256) {
    int o[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) o[u] = clamped(base + 64 * u + lane, t0);
    const bool hit = o[0] == id || o[1] == id || o[2] == id || o[3] == id;
    if (__ballot(hit)) return;   // wave-uniform: every wave scans the same ids
  }
  // every thread takes part in the ballots (the scan must see all 64 candidates
  // of a chunk); a thread owns up to two 8-column vectors (H <= 4096)
  const int nvec = H / 8;
  float acc[2][8];
#pragma unroll
  for (int v = 0; v < 2; ++v) {
    const int vec = threadIdx.x + 256 * v;
    if (vec < nvec) {
      Vec8<T>::load(dz + (long)t0 * H + vec * 8, acc[v]);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[v][e] = 0.f;
    }
  }
  for (int base0 = t0 + 1; base0 < nrows; base0 += 256) {
    int o[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) o[u] = clamped(base0 + 64 * u + lane, nrows);
#pragma unroll
    for (int u = 0; u < 4; ++u) {      // ascending positions: chunk by chunk, lowest bit first
      const int base = base0 + 64 * u;
      unsigned long long m = __ballot(o[u] == id);
      while (m) {
        const int b = __builtin_ctzll(m);
        m &= m - 1;
#pragma unroll
        for (int v = 0; v < 2; ++v) {
          const int vec = threadIdx.x + 256 * v;
          if (vec < nvec) {
            float x[8];
            Vec8<T>::load(dz + (long)(base + b) * H + vec * 8, x);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[v][e] += x[e];
          }
        }
      }
    }
  }
#pragma unroll
  for (int v = 0; v < 2; ++v) {
    const int vec = threadIdx.x + 256 * v;
    if (vec < nvec) {
      float* dst = dword + (long)id * H + vec * 8;
      float cur[8];
      load8f(dst, cur);
#pragma unroll
      for (int e = 0; e < 8; ++e) cur[e] += acc[v][e];
      Vec8<float>::store(dst, cur);
    }
  }
}

// dpos[s] = sum_b dz[b*S + s] (ascending b) for s < S, zero for S <= s < max_pos
template <typename T>
__global__ __launch_bounds__(256) void embed_dpos_kernel(const T* __restrict__ dz, float* __restrict__ dpos, int B,
                                                         int S, int H) {
  const int s = blockIdx.x;
  for (int vec = threadIdx.x; vec < H / 8; vec += 256) {
    float acc[8] = {};
    if (s < S) {
      for (int b = 0; b < B; ++b) {
        float v[8];
        Vec8<T>::load(dz + ((long)b * S + s) * H + vec * 8, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += v[e];
      }
    }
    Vec8<float>::store(dpos + (long)s * H + vec * 8, acc);
  }
}

// ------------------------------------------------------------- MLM head ---
// r[i] = x[sel[i]] for i < n_sel, zero rows up to n_pad
template <typename T>
__global__ __launch_bounds__(256) void gather_rows_kernel(const T* __restrict__ x, const int32_t* __restrict__ sel,
                                                          T* __restrict__ r, int n_sel, int rows, int H) {
  const int i = blockIdx.x;
  int src = i < n_sel ? sel[i] : -1;
  if (src >= rows) src = -1;
  for (int vec = threadIdx.x; vec < H / 8; vec += 256) {
    float v[8] = {};
    if (src >= 0) Vec8<T>::load(x + (long)src * H + vec * 8, v);
    Vec8<T>::store(r + (long)i * H + vec * 8, v);
  }
}

// dx[t] = dr[j] if sel[j] == t (sel ascending: binary search), else zero
template <typename T>
__global__ __launch_bounds__(256) void scatter_rows_kernel(const T* __restrict__ dr, const int32_t* __restrict__ sel,
                                                           T* __restrict__ dx, int n_sel, int H) {
  const int t = blockIdx.x;
  int lo = 0, hi = n_sel - 1, found = -1;
  while (lo <= hi) {
    const int mid = (lo + hi) >> 1;
    const int v = sel[mid];
    if (v == t) { found = mid; break; }
    if (v < t) lo = mid + 1; else hi = mid - 1;
  }
  for (int vec = threadIdx.x; vec < H / 8; vec += 256) {
    float v[8] = {};
    if (found >= 0) Vec8<T>::load(dr + (long)found * H + vec * 8, v);
    Vec8<T>::store(dx + (long)t * H + vec * 8, v);
  }
}

// dt1 = dt2 * gelu'(t1)
template <typename T>
__global__ __launch_bounds__(256) void gelu_bwd_kernel(const T* __restrict__ dt2, const T* __restrict__ t1,
                                                       T* __restrict__ dt1, long n, int tanh_form) {
  const long i = ((long)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= n) return;
  float g[8], u[8];
  Vec8<T>::load(dt2 + i, g);
  Vec8<T>::load(t1 + i, u);
#pragma unroll
  for (int e = 0; e < 8; ++e) g[e] *= gelu_grad_f(u[e], tanh_form);
  Vec8<T>::store(dt1 + i, g);
}

// One workgroup per selected row: z = logits + bias over the first `vocab`
// columns; loss_row = logsumexp(z) - z[label]; the row is overwritten with
// loss_scale * (softmax(z) - onehot(label)); columns >= vocab and rows without a
// label (padding) become zero.  The row lives in registers between the passes.
constexpr int CE_MAX_VEC = 32;   // 8-element vectors per thread: vocab_pad <= 65536
template <typename T, int NVT>
__global__ __launch_bounds__(256) void softmax_ce_kernel(T* __restrict__ logits, const float* __restrict__ bias,
                                                         const int32_t* __restrict__ labels, float* __restrict__ loss_rows,
                                                         int n_sel, int vocab, int vocab_pad, float loss_scale) {
  __shared__ float red[4];
  __shared__ float red2[4];
  const int i = blockIdx.x;
  T* row = logits + (long)i * vocab_pad;
  const int nvec = vocab_pad / 8;
  const int label = i < n_sel ? labels[i] : -1;
  const bool live = label >= 0 && label < vocab;
  float v[NVT][8];
  float mx = -INFINITY;
  // every load of the row is issued before the first use and none sits under a branch (vectors past the end re-read
  // the last one and are discarded): one memory round trip instead of one per vector
  typename Vec8<T>::Raw raw[NVT];
#pragma unroll
  for (int t = 0; t < NVT; ++t) {
    const int vec = threadIdx.x + 256 * t;
    raw[t] = Vec8<T>::load_raw(row + (vec < nvec ? vec : nvec - 1) * 8);
  }
#pragma unroll
  for (int t = 0; t < NVT; ++t) {
    const int vec = threadIdx.x + 256 * t;
    Vec8<T>::unpack(raw[t], v[t]);
    if (vec * 8 + 8 <= vocab) {          // whole vector inside the vocabulary (all but the last one or two)
      float b[8];
      load8f(bias + vec * 8, b);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        v[t][e] += b[e];
        mx = fmaxf(mx, v[t][e]);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int c = vec * 8 + e;
        v[t][e] = (vec < nvec && c < vocab) ? v[t][e] + bias[c] : -INFINITY;
        mx = fmaxf(mx, v[t][e]);
      }
    }
  }
  mx = group_max<64>(mx);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float sum = 0.f, zl = 0.f;
#pragma unroll
  for (int t = 0; t < NVT; ++t) {
    const int vec = threadIdx.x + 256 * t;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (vec * 8 + e == label) zl = v[t][e];
      v[t][e] = expf(v[t][e] - mx);   // exp(-inf) = 0 on the padding
      sum += v[t][e];
    }
  }
  sum = group_sum<64>(sum);
  zl = group_sum<64>(zl);
  if ((threadIdx.x & 63) == 0) {
    red2[threadIdx.x >> 6] = sum;
  }
  __syncthreads();
  sum = (red2[0] + red2[1]) + (red2[2] + red2[3]);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = zl;
  __syncthreads();
  zl = (red[0] + red[1]) + (red[2] + red[3]);
  if (threadIdx.x == 0) loss_rows[i] = live ? (mx + logf(sum)) - zl : 0.f;
  const float scale = live ? loss_scale / sum : 0.f;
#pragma unroll
  for (int t = 0; t < NVT; ++t) {
    const int vec = threadIdx.x + 256 * t;
    if (vec < nvec) {
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        o[e] = v[t][e] * scale;
        if (live && vec * 8 + e == label) o[e] -= loss_scale;
      }
      Vec8<T>::store(row + vec * 8, o);
    }
  }
}

// ----------------------------------------------------------------- plans --
static inline size_t bump256(size_t& off, size_t bytes) {
  const size_t at = off;
  off += (bytes + 255) & ~(size_t)255;
  return at;
}
static inline int vocab_pad_of(int vocab) { return (vocab + 31) / 32 * 32; }

static raf_status validate_embed(const raf_embed_desc* d) {
  if (!d) return RAF_EINVAL;
  if (d->batch <= 0 || d->seq <= 0 || d->hidden <= 0 || d->vocab <= 0 || d->max_pos <= 0) return RAF_EINVAL;
  if (d->precision != RAF_F32 && d->precision != RAF_BF16_AMP) return RAF_EINVAL;
  if (!(d->dropout_p >= 0.0 && d->dropout_p < 1.0) || !(d->ln_eps >= 0.f)) return RAF_EINVAL;
  if (d->seq > d->max_pos) return RAF_EINVAL;
  if ((d->hidden % 32) || d->hidden > 4096) return RAF_ENOTSUP;
  if ((long)d->batch * d->seq > (1l << 24)) return RAF_ENOTSUP;
  return RAF_OK;
}

static raf_layer_desc as_layer_desc(int hidden, int precision, float eps, double p, uint64_t seed, uint32_t layer_id,
                                    int gelu_tanh) {
  raf_layer_desc l{};
  l.batch = 1; l.seq = 32; l.hidden = hidden; l.heads = hidden / 64 > 0 ? hidden / 64 : 1; l.ffn = 32;
  l.precision = precision; l.ln_eps = eps; l.dropout_p = p; l.seed = seed; l.layer_id = layer_id;
  l.gelu_tanh = gelu_tanh;
  return l;
}

struct EmbedPlan {
  size_t e, z0, mu, rstd, saved_bytes, dz0, partial, scratch_bytes;
  long T;
};
static EmbedPlan embed_plan(const raf_embed_desc& d) {
  EmbedPlan p{};
  p.e = d.precision == RAF_F32 ? 4 : 2;
  p.T = (long)d.batch * d.seq;
  size_t o = 0;
  p.z0 = bump256(o, (size_t)p.T * d.hidden * p.e);
  p.mu = bump256(o, p.T * 4);
  p.rstd = bump256(o, p.T * 4);
  p.saved_bytes = o;
  size_t s = 0;
  p.dz0 = bump256(s, (size_t)p.T * d.hidden * p.e);
  p.partial = bump256(s, ln_bwd_partial_floats(d.hidden, p.T) * 4);
  p.scratch_bytes = s;
  return p;
}

static raf_status validate_mlm(const raf_mlm_desc* d) {
  if (!d) return RAF_EINVAL;
  if (d->rows <= 0 || d->hidden <= 0 || d->vocab <= 0 || d->n_sel <= 0 || d->n_sel > d->rows) return RAF_EINVAL;
  if (d->precision != RAF_F32 && d->precision != RAF_BF16_AMP) return RAF_EINVAL;
  // ln_eps must be positive here: the selected rows are padded to the GEMM tile height with zero rows, which reach
  // the LayerNorm as constant rows (gelu of the bias), variance exactly 0; with eps = 0 they would turn into NaN and
  // spread through the tied decoder's gradient.
  if ((d->gelu_tanh | 1) != 1 || d->reserved != 0 || !(d->ln_eps > 0.f)) return RAF_EINVAL;
  if ((d->hidden % 32) || d->hidden > 4096) return RAF_ENOTSUP;
  if (vocab_pad_of(d->vocab) > 256 * 8 * CE_MAX_VEC) return RAF_ENOTSUP;
  return RAF_OK;
}

// out[i] = sum_s part[s*n + i] (fixed order), 8 elements per thread
template <typename T>
__global__ __launch_bounds__(256) void sum_slices_kernel(const float* __restrict__ part, int nslices, long n,
                                                         T* __restrict__ out) {
  const long i = ((long)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= n) return;
  float acc[8] = {};
  for (int s = 0; s < nslices; ++s) {
    float v[8];
    load8f(part + (long)s * n + i, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += v[e];
  }
  Vec8<T>::store(out + i, acc);
}

struct MlmPlan {
  size_t e;
  int n_pad, vp;
  size_t r, t1, t2, t, mu, rstd, logits, dt, dt2, dt1, dr, loss_rows, partial, dt_part, scratch_bytes;
  int dt_splits;   // the vocabulary-deep product dt = dlogits . Word is taken in this many slices of the contraction
};

// dt has only n_pad/128 x hidden/128 output tiles (60 for the BERT-base head) under a contraction as deep as the
// vocabulary: slicing the contraction fills the chip.  Largest count up to 16 that divides the 64-deep steps.
static int dt_split_count(int vp) {
  if (vp % 64) return 1;
  const int steps = vp / 64;
  for (int s = 16; s > 1; --s)
    if (steps % s == 0 && steps / s >= 8) return s;
  return 1;
}
static MlmPlan mlm_plan(const raf_mlm_desc& d) {
  MlmPlan p{};
  p.e = d.precision == RAF_F32 ? 4 : 2;
  p.n_pad = (d.n_sel + 127) / 128 * 128;
  p.vp = vocab_pad_of(d.vocab);
  const size_t NH = (size_t)p.n_pad * d.hidden * p.e;
  size_t o = 0;
  p.r = bump256(o, NH); p.t1 = bump256(o, NH); p.t2 = bump256(o, NH); p.t = bump256(o, NH);
  p.mu = bump256(o, (size_t)p.n_pad * 4); p.rstd = bump256(o, (size_t)p.n_pad * 4);
  p.logits = bump256(o, (size_t)p.n_pad * p.vp * p.e);
  p.dt = bump256(o, NH); p.dt2 = bump256(o, NH); p.dt1 = bump256(o, NH); p.dr = bump256(o, NH);
  p.loss_rows = bump256(o, (size_t)p.n_pad * 4);
  size_t pf = ln_bwd_partial_floats(d.hidden, p.n_pad);
  const size_t c1 = colsum_partial_floats(p.vp, p.n_pad), c2 = colsum_partial_floats(d.hidden, p.n_pad);
  if (c1 > pf) pf = c1;
  if (c2 > pf) pf = c2;
  p.partial = bump256(o, pf * 4);
  p.dt_splits = d.precision == RAF_BF16_AMP ? dt_split_count(p.vp) : 1;
  p.dt_part = bump256(o, p.dt_splits > 1 ? (size_t)p.dt_splits * p.n_pad * d.hidden * 4 : 0);
  p.scratch_bytes = o;
  return p;
}

}  // namespace raf

using namespace raf;

#define RAF_TRY(expr)                \
  do {                               \
    raf_status _rc = (expr);         \
    if (_rc != RAF_OK) return _rc;   \
  } while (0)

extern "C" raf_status raf_embed_workspace(const raf_embed_desc* desc, size_t* saved_bytes, size_t* scratch_bytes) {
  RAF_TRY(validate_embed(desc));
  if (!saved_bytes || !scratch_bytes) return RAF_EINVAL;
  const EmbedPlan p = embed_plan(*desc);
  *saved_bytes = p.saved_bytes;
  *scratch_bytes = p.scratch_bytes;
  return RAF_OK;
}

extern "C" raf_status raf_embed_fwd(const raf_embed_desc* desc, const int32_t* ids, const void* word, const void* pos,
                                    const float* gamma, const float* beta, void* x0, void* saved, uint64_t step,
                                    void* hip_stream) {
  RAF_TRY(validate_embed(desc));
  if (!ids || !word || !pos || !gamma || !beta || !x0 || !saved) return RAF_EINVAL;
  if (!aligned16(word) || !aligned16(pos) || !aligned16(gamma) || !aligned16(beta) || !aligned16(x0) ||
      !aligned16(saved) || ((uintptr_t)ids & 3u))
    return RAF_EINVAL;
  const raf_embed_desc& d = *desc;
  const EmbedPlan p = embed_plan(d);
  hipStream_t st = (hipStream_t)hip_stream;
  const raf_layer_desc ld = as_layer_desc(d.hidden, d.precision, d.ln_eps, d.dropout_p, d.seed, d.layer_id, 0);
  const DropSite drop = make_drop_site(ld, 4, step);
  char* sv = (char*)saved;
  const int H = d.hidden;
#define CALL(LPR, NV)                                                                                               \
  {                                                                                                                 \
    const long nblk = (p.T * LPR + 255) / 256;                                                                      \
    if (d.precision == RAF_F32)                                                                                     \
      hipLaunchKernelGGL((embed_fwd_kernel<float, LPR, NV>), dim3(nblk), dim3(256), 0, st, ids, (const float*)word, \
                         (const float*)pos, gamma, beta, (float*)x0, (float*)(sv + p.z0), (float*)(sv + p.mu),      \
                         (float*)(sv + p.rstd), p.T, d.seq, H, d.vocab, d.ln_eps, drop);                            \
    else                                                                                                            \
      hipLaunchKernelGGL((embed_fwd_kernel<bf16_t, LPR, NV>), dim3(nblk), dim3(256), 0, st, ids,                   \
                         (const bf16_t*)word, (const bf16_t*)pos, gamma, beta, (bf16_t*)x0, (bf16_t*)(sv + p.z0),   \
                         (float*)(sv + p.mu), (float*)(sv + p.rstd), p.T, d.seq, H, d.vocab, d.ln_eps, drop);       \
  }
  RAF_DISPATCH_GEOM(row_geom(H), CALL);
#undef CALL
  return check_launch();
}

extern "C" raf_status raf_embed_bwd(const raf_embed_desc* desc, const int32_t* ids, const void* dx0, const void* saved,
                                    const float* gamma, float* dword, float* dpos, float* dgamma, float* dbeta,
                                    void* scratch, uint64_t step, void* hip_stream) {
  RAF_TRY(validate_embed(desc));
  if (!ids || !dx0 || !saved || !gamma || !dword || !dpos || !dgamma || !dbeta || !scratch) return RAF_EINVAL;
  if (!aligned16(dx0) || !aligned16(saved) || !aligned16(gamma) || !aligned16(dword) || !aligned16(dpos) ||
      !aligned16(scratch) || ((uintptr_t)ids & 3u))
    return RAF_EINVAL;
  const raf_embed_desc& d = *desc;
  const EmbedPlan p = embed_plan(d);
  hipStream_t st = (hipStream_t)hip_stream;
  const raf_layer_desc ld = as_layer_desc(d.hidden, d.precision, d.ln_eps, d.dropout_p, d.seed, d.layer_id, 0);
  const char* sv = (const char*)saved;
  char* sc = (char*)scratch;
  void* dz0 = sc + p.dz0;
  // de = dx0 * keep4/(1-p) on load; dz0 = LN'(de); dgamma, dbeta
  RAF_TRY(launch_ln_bwd(ld, 0, p.T, dx0, nullptr, sv + p.z0, (const float*)(sv + p.mu), (const float*)(sv + p.rstd),
                        gamma, nullptr, dz0, nullptr, dgamma, dbeta, nullptr, (float*)(sc + p.partial), step, st, 4));
  if (d.precision == RAF_F32) {
    hipLaunchKernelGGL((embed_dword_kernel<float>), dim3((unsigned)p.T), dim3(256), 0, st, ids, (const float*)dz0,
                       dword, (int)p.T, d.hidden, d.vocab);
    hipLaunchKernelGGL((embed_dpos_kernel<float>), dim3(d.max_pos), dim3(256), 0, st, (const float*)dz0, dpos, d.batch,
                       d.seq, d.hidden);
  } else {
    hipLaunchKernelGGL((embed_dword_kernel<bf16_t>), dim3((unsigned)p.T), dim3(256), 0, st, ids, (const bf16_t*)dz0,
                       dword, (int)p.T, d.hidden, d.vocab);
    hipLaunchKernelGGL((embed_dpos_kernel<bf16_t>), dim3(d.max_pos), dim3(256), 0, st, (const bf16_t*)dz0, dpos,
                       d.batch, d.seq, d.hidden);
  }
  return check_launch();
}

extern "C" raf_status raf_mlm_workspace(const raf_mlm_desc* desc, size_t* scratch_bytes) {
  RAF_TRY(validate_mlm(desc));
  if (!scratch_bytes) return RAF_EINVAL;
  *scratch_bytes = mlm_plan(*desc).scratch_bytes;
  return RAF_OK;
}

template <typename T>
static raf_status launch_ce(T* logits, const float* bias, const int32_t* labels, float* loss_rows, int n_pad, int n_sel,
                            int vocab, int vp, float loss_scale, hipStream_t st) {
  const int nvt = (vp / 8 + 255) / 256;
#define CE(NVT) \
  hipLaunchKernelGGL((softmax_ce_kernel<T, NVT>), dim3(n_pad), dim3(256), 0, st, logits, bias, labels, loss_rows, n_sel, \
                     vocab, vp, loss_scale)
  if (nvt <= 1) CE(1);
  else if (nvt <= 2) CE(2);
  else if (nvt <= 4) CE(4);
  else if (nvt <= 8) CE(8);
  else if (nvt <= 16) CE(16);
  else CE(32);
#undef CE
  return check_launch();
}

static raf_status head_gemm(int prec, hipStream_t st, int M, int N, int K, const void* a, long lda, int ak,
                            const void* b, long ldb, int bk, void* c, long ldc, int out_f32 = 0, int epi = EPI_NONE,
                            const float* bias = nullptr, void* aux = nullptr, int gelu_tanh = 0) {
  GemmArgs g = gemm_args_default();
  g.M = M; g.N = N; g.K = K;
  g.a = a; g.lda = lda; g.a_kmajor = ak;
  g.b = b; g.ldb = ldb; g.b_kmajor = bk;
  g.c = c; g.ldc = ldc; g.out_f32 = out_f32;
  g.epilogue = epi; g.bias = bias; g.aux = aux; g.ldaux = ldc; g.gelu_tanh = gelu_tanh;
  return launch_gemm(prec, g, st);
}

extern "C" raf_status raf_mlm_head_fwd_bwd(const raf_mlm_desc* desc, const raf_mlm_tensors* w, const void* x,
                                           const int32_t* sel, const int32_t* labels, float loss_scale,
                                           float* loss_out, void* dx, raf_mlm_tensors* grads, void* scratch,
                                           void* hip_stream) {
  RAF_TRY(validate_mlm(desc));
  if (!w || !grads || !x || !sel || !labels || !loss_out || !dx || !scratch) return RAF_EINVAL;
  const void* const* wp = (const void* const*)w;
  const void* const* gp = (const void* const*)grads;
  for (int i = 0; i < 6; ++i)
    if (!wp[i] || !gp[i] || !aligned16(wp[i]) || !aligned16(gp[i])) return RAF_EINVAL;
  if (!aligned16(x) || !aligned16(dx) || !aligned16(scratch)) return RAF_EINVAL;
  const raf_mlm_desc& d = *desc;
  const MlmPlan p = mlm_plan(d);
  hipStream_t st = (hipStream_t)hip_stream;
  const int prec = d.precision, H = d.hidden, NP = p.n_pad, VP = p.vp;
  const raf_layer_desc ld = as_layer_desc(H, prec, d.ln_eps, 0.0, 0, 0, d.gelu_tanh);
  char* sc = (char*)scratch;
  void *r = sc + p.r, *t1 = sc + p.t1, *t2 = sc + p.t2, *t = sc + p.t, *logits = sc + p.logits;
  void *dt = sc + p.dt, *dt2 = sc + p.dt2, *dt1 = sc + p.dt1, *dr = sc + p.dr;
  float *mu = (float*)(sc + p.mu), *rstd = (float*)(sc + p.rstd), *loss_rows = (float*)(sc + p.loss_rows);
  float* partial = (float*)(sc + p.partial);

  // forward
  if (prec == RAF_F32)
    hipLaunchKernelGGL((gather_rows_kernel<float>), dim3(NP), dim3(256), 0, st, (const float*)x, sel, (float*)r,
                       d.n_sel, d.rows, H);
  else
    hipLaunchKernelGGL((gather_rows_kernel<bf16_t>), dim3(NP), dim3(256), 0, st, (const bf16_t*)x, sel, (bf16_t*)r,
                       d.n_sel, d.rows, H);
  RAF_TRY(check_launch());
  RAF_TRY(head_gemm(prec, st, NP, H, H, r, H, 1, w->head_w, H, 1, t2, H, 0, EPI_BIAS_GELU, (const float*)w->head_b, t1,
                    d.gelu_tanh));
  RAF_TRY(launch_ln_fwd(ld, 0, NP, nullptr, t2, (const float*)w->ln_g, (const float*)w->ln_b, t, nullptr, mu, rstd, 0,
                        st));
  RAF_TRY(head_gemm(prec, st, NP, VP, H, t, H, 1, w->word, H, 1, logits, VP));
  // loss and dlogits (in place), decoder bias added here
  if (prec == RAF_F32)
    RAF_TRY(launch_ce<float>((float*)logits, (const float*)w->dec_b, labels, loss_rows, NP, d.n_sel, d.vocab, VP,
                             loss_scale, st));
  else
    RAF_TRY(launch_ce<bf16_t>((bf16_t*)logits, (const float*)w->dec_b, labels, loss_rows, NP, d.n_sel, d.vocab, VP,
                              loss_scale, st));
  RAF_TRY(launch_sum_partials(loss_rows, NP, loss_out, st));

  // backward
  RAF_TRY(launch_colsum(prec, logits, NP, VP, VP, (float*)grads->dec_b, partial, st, d.vocab));
  RAF_TRY(head_gemm(prec, st, VP, H, NP, logits, VP, 0, t, H, 0, grads->word, H, 1));          // dWord = dlogits^T t
  if (p.dt_splits > 1) {
    // dt = dlogits Word in slices of the contraction (float partial results), then their sum
    GemmArgs g = gemm_args_default();
    const int kc = VP / p.dt_splits;
    g.M = NP; g.N = H; g.K = kc;
    g.a = logits; g.lda = VP; g.a_kmajor = 1;
    g.b = w->word; g.ldb = H; g.b_kmajor = 0;
    g.c = sc + p.dt_part; g.ldc = H; g.out_f32 = 1;
    g.batch = p.dt_splits;
    g.sa[0] = kc; g.sb[0] = (long)kc * H; g.sc[0] = (long)NP * H;
    RAF_TRY(launch_gemm(prec, g, st));
    const long n = (long)NP * H;
    hipLaunchKernelGGL((sum_slices_kernel<bf16_t>), dim3((n / 8 + 255) / 256), dim3(256), 0, st,
                       (const float*)(sc + p.dt_part), p.dt_splits, n, (bf16_t*)dt);
    RAF_TRY(check_launch());
  } else {
    RAF_TRY(head_gemm(prec, st, NP, H, VP, logits, VP, 1, w->word, H, 0, dt, H));              // dt = dlogits Word
  }
  RAF_TRY(launch_ln_bwd(ld, 0, NP, dt, nullptr, t2, mu, rstd, (const float*)w->ln_g, nullptr, dt2, nullptr,
                        (float*)grads->ln_g, (float*)grads->ln_b, nullptr, partial, 0, st));
  const long nh = (long)NP * H;
  if (prec == RAF_F32)
    hipLaunchKernelGGL((gelu_bwd_kernel<float>), dim3((nh / 8 + 255) / 256), dim3(256), 0, st, (const float*)dt2,
                       (const float*)t1, (float*)dt1, nh, d.gelu_tanh);
  else
    hipLaunchKernelGGL((gelu_bwd_kernel<bf16_t>), dim3((nh / 8 + 255) / 256), dim3(256), 0, st, (const bf16_t*)dt2,
                       (const bf16_t*)t1, (bf16_t*)dt1, nh, d.gelu_tanh);
  RAF_TRY(check_launch());
  RAF_TRY(launch_colsum(prec, dt1, NP, H, H, (float*)grads->head_b, partial, st));
  RAF_TRY(head_gemm(prec, st, H, H, NP, dt1, H, 0, r, H, 0, grads->head_w, H, 1));             // dWt = dt1^T r
  RAF_TRY(head_gemm(prec, st, NP, H, H, dt1, H, 1, w->head_w, H, 0, dr, H));                   // dr = dt1 Wt
  if (prec == RAF_F32)
    hipLaunchKernelGGL((scatter_rows_kernel<float>), dim3(d.rows), dim3(256), 0, st, (const float*)dr, sel, (float*)dx,
                       d.n_sel, H);
  else
    hipLaunchKernelGGL((scatter_rows_kernel<bf16_t>), dim3(d.rows), dim3(256), 0, st, (const bf16_t*)dr, sel,
                       (bf16_t*)dx, d.n_sel, H);
  return check_launch();
}
