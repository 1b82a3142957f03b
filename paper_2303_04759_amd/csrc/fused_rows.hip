// Memory-bound fused row kernels of the training step (rule-based fusion of
// elementwise + reduction operators, paper Section 3.2.2): masked softmax with
// dropout and its adjoint, dropout + residual + LayerNorm and its adjoint,
// column sums for bias gradients.  All arithmetic and statistics in fp32
// (numerically sensitive operators stay in full precision, Section 3.1.2);
// storage in the compute dtype with the casts fused into loads and stores.
//
// A row of L elements is owned by LPR lanes (a power of two <= 64) of one
// wavefront, each holding NV vectors of 8 elements in registers:
// vector index = lane_in_row + LPR * t, t < NV, valid while < L/8.
#include "common.hpp"

namespace raf {

// ---------------------------------------------------------- softmax fwd ---
template <typename T, int LPR, int NV>
__global__ __launch_bounds__(256) void softmax_fwd_kernel(const T* __restrict__ s, const int32_t* __restrict__ lens,
                                                          T* __restrict__ prob, T* __restrict__ prob_d, long nrows,
                                                          int S, int heads, int causal, DropSite drop) {
  const int lane = threadIdx.x & (LPR - 1);
  const long row = ((long)blockIdx.x * 256 + threadIdx.x) / LPR;
  if (row >= nrows) return;   // whole LPR-group leaves together; shuffles below stay inside a group
  const int nvec = S / 8;
  const int i = (int)(row % S);
  const int b = (int)(row / ((long)S * heads));
  int limit = lens ? lens[b] : S;
  limit = limit < 0 ? 0 : (limit > S ? S : limit);
  if (causal) limit = limit < i + 1 ? limit : i + 1;

  float v[NV][8];
  float mx = -INFINITY;
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    if (vec < nvec) {
      Vec8<T>::load(s + row * S + vec * 8, v[t]);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (vec * 8 + e >= limit) v[t][e] = -INFINITY;
        mx = fmaxf(mx, v[t][e]);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[t][e] = -INFINITY;
    }
  }
  mx = group_max<LPR>(mx);
  const bool empty = (mx == -INFINITY);
  float sum = 0.f;
#pragma unroll
  for (int t = 0; t < NV; ++t)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      v[t][e] = empty ? 0.f : expf(v[t][e] - mx);   // exp(-inf) == 0 exactly
      sum += v[t][e];
    }
  sum = group_sum<LPR>(sum);
  const float inv = empty ? 0.f : 1.0f / sum;
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    if (vec < nvec) {
      float p[8], pd[8], mult[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) p[e] = v[t][e] * inv;
      if (drop.enabled) {
        drop_mult8(drop, (uint64_t)row * S + vec * 8, mult);
#pragma unroll
        for (int e = 0; e < 8; ++e) pd[e] = p[e] * mult[e];
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) pd[e] = p[e];
      }
      Vec8<T>::store(prob + row * S + vec * 8, p);
      Vec8<T>::store(prob_d + row * S + vec * 8, pd);
    }
  }
}

// ---------------------------------------------------------- softmax bwd ---
template <typename T, int LPR, int NV>
__global__ __launch_bounds__(256) void softmax_bwd_kernel(const T* __restrict__ prob, const T* __restrict__ prob_d,
                                                          const T* __restrict__ dprob_d, T* __restrict__ ds,
                                                          long nrows, int S, float drop_scale, float scale_out) {
  const int lane = threadIdx.x & (LPR - 1);
  const long row = ((long)blockIdx.x * 256 + threadIdx.x) / LPR;
  if (row >= nrows) return;
  const int nvec = S / 8;
  float p[NV][8], dp[NV][8];
  float dot = 0.f;
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    if (vec < nvec) {
      float pd[8], g[8];
      Vec8<T>::load(prob + row * S + vec * 8, p[t]);
      Vec8<T>::load(prob_d + row * S + vec * 8, pd);
      Vec8<T>::load(dprob_d + row * S + vec * 8, g);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // an element was dropped iff its probability is non-zero but the
        // post-dropout value is zero; for p == 0 the product below is 0 anyway
        const bool keep = (pd[e] != 0.f) || (p[t][e] == 0.f);
        dp[t][e] = keep ? g[e] * drop_scale : 0.f;
        dot += dp[t][e] * p[t][e];
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) p[t][e] = dp[t][e] = 0.f;
    }
  }
  dot = group_sum<LPR>(dot);
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    if (vec < nvec) {
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = scale_out * p[t][e] * (dp[t][e] - dot);
      Vec8<T>::store(ds + row * S + vec * 8, o);
    }
  }
}

// -------------------------------------------- dropout + residual + LN fwd --
// LOSS: the kernel that produces the layer's output also takes the loss seed of the benchmark workload on it:
// loss partial sums of out * G (out as stored, one partial per workgroup) and dy = loss_scale * G.
template <typename T, int LPR, int NV, bool LOSS>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T* __restrict__ a, const T* __restrict__ res,
                                                     const float* __restrict__ gamma, const float* __restrict__ beta,
                                                     T* __restrict__ out, T* __restrict__ z_out, float* __restrict__ mu,
                                                     float* __restrict__ rstd, long nrows, int H, float eps,
                                                     DropSite drop, LossSeedDev ls) {
  const int lane = threadIdx.x & (LPR - 1);
  const long row_raw = ((long)blockIdx.x * 256 + threadIdx.x) / LPR;
  const bool live = row_raw < nrows;
  if (!LOSS && !live) return;
  const long row = live ? row_raw : nrows - 1;   // LOSS: a group without a row stays for the block sum and adds zero
  const int nvec = H / 8;
  float z[NV][8];
  float sum = 0.f;
  // every operand of the row is requested before the first use (one memory round trip, not one per vector)
  typename Vec8<T>::Raw rres[NV], ra[NV], rG[NV];
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    const long off = row * H + (vec < nvec ? vec : nvec - 1) * 8;
    rres[t] = Vec8<T>::load_raw(res + off);
    if (a) ra[t] = Vec8<T>::load_raw(a + off);
    if (LOSS) rG[t] = Vec8<T>::load_raw((const T*)ls.G + off);
  }
  float loss_scale = ls.scale, loss_acc = 0.f;
  if (LOSS && ls.scale_ptr) loss_scale = *ls.scale_ptr;   // dynamic loss scale, device-resident
  // out[vec] is final: store it and take the loss seed on the value as stored
  auto emit = [&](int t, int vec, float (&o)[8]) {
    if (live) Vec8<T>::store(out + row * H + vec * 8, o);
    if (LOSS) {
      float g[8];
      Vec8<T>::unpack(rG[t], g);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        loss_acc += Vec8<T>::round(o[e]) * g[e];
        g[e] *= loss_scale;
      }
      if (live) Vec8<T>::store((T*)ls.dy + row * H + vec * 8, g);
    }
  };
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    if (vec < nvec) {
      const long off = row * H + vec * 8;
      Vec8<T>::unpack(rres[t], z[t]);
      if (a) {
        float av[8];
        Vec8<T>::unpack(ra[t], av);
        if (drop.enabled) {
          float mult[8];
          drop_mult8(drop, (uint64_t)off, mult);
#pragma unroll
          for (int e = 0; e < 8; ++e) z[t][e] += av[e] * mult[e];
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) z[t][e] += av[e];
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        z[t][e] = Vec8<T>::round(z[t][e]);   // statistics of the value the backward pass reads back
        sum += z[t][e];
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) z[t][e] = 0.f;
    }
  }
  if (!gamma) {   // no normalisation: out = z
#pragma unroll
    for (int t = 0; t < NV; ++t) {
      const int vec = lane + LPR * t;
      if (vec < nvec) emit(t, vec, z[t]);
    }
  } else {
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
    const float var = group_sum<LPR>(sq) / (float)H;
    const float rs = 1.0f / sqrtf(var + eps);
#pragma unroll
    for (int t = 0; t < NV; ++t) {
      const int vec = lane + LPR * t;
      if (vec < nvec) {
        float gm[8], bt[8], o[8];
        load8f(gamma + vec * 8, gm);
        load8f(beta + vec * 8, bt);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (z[t][e] - mean) * rs * gm[e] + bt[e];
        emit(t, vec, o);
        if (z_out && live) Vec8<T>::store(z_out + row * H + vec * 8, z[t]);
      }
    }
    if (lane == 0 && live) {
      mu[row] = mean;
      rstd[row] = rs;
    }
  }
  if (LOSS) {
    // one partial per workgroup, summed in a fixed order (lanes of a wavefront, then the four wavefronts)
    __shared__ float red[4];
    if (!live) loss_acc = 0.f;
    loss_acc = group_sum<64>(loss_acc);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = loss_acc;
    __syncthreads();
    if (threadIdx.x == 0) ls.partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}

// -------------------------------------------- dropout + residual + LN bwd --
// Each LPR-lane group walks rows (group-strided) and keeps per-column partial
// sums for dgamma, dbeta and dbias in registers; a block reduces them through
// LDS and writes one partial row; a second kernel sums the partial rows in a
// fixed order, so the result does not depend on scheduling.
constexpr int LN_BWD_MAX_BLOCKS = 256;

template <typename T, int LPR, int NV, bool HAS_LN, int LN_BWD_THREADS>
__global__ __launch_bounds__(LN_BWD_THREADS) void ln_bwd_kernel(const T* __restrict__ dout, const T* __restrict__ dout2,
                                                     const T* __restrict__ z, const float* __restrict__ mu,
                                                     const float* __restrict__ rstd, const float* __restrict__ gamma,
                                                     const T* __restrict__ dres, T* __restrict__ dz,
                                                     T* __restrict__ da, float* __restrict__ partial, long nrows,
                                                     int H, DropSite drop, DropSite drop_in, int slices) {
  extern __shared__ float red[];   // [slices][3][8][H/8]: column vec*8+e of sum k sits at k*H + e*(H/8) + vec
  const int lane = threadIdx.x & (LPR - 1);
  const int groups_per_block = LN_BWD_THREADS / LPR;
  const long group = (long)blockIdx.x * groups_per_block + threadIdx.x / LPR;
  const long ngroups = (long)gridDim.x * groups_per_block;
  const int nvec = H / 8;

  float cg[NV][8], cb[NV][8], cd[NV][8];
  float gm[NV][8];
#pragma unroll
  for (int t = 0; t < NV; ++t) {
#pragma unroll
    for (int e = 0; e < 8; ++e) cg[t][e] = cb[t][e] = cd[t][e] = 0.f, gm[t][e] = 0.f;
    const int vec = lane + LPR * t;
    if (HAS_LN && vec < nvec) load8f(gamma + vec * 8, gm[t]);
  }

  // The operands of a row are requested one row ahead (kept as loaded, converted when used), so that the loads of the
  // next row overlap the arithmetic and the stores of this one.
  typedef typename Vec8<T>::Raw Raw;
  struct RowIn {
    Raw g[NV], g2[NV], z[NV], res[NV];
    float mean, rs;
  };
  auto request = [&](long row, RowIn& in) {
    in.mean = in.rs = 0.f;
    if (HAS_LN) {
      in.mean = mu[row];
      in.rs = rstd[row];
    }
#pragma unroll
    for (int t = 0; t < NV; ++t) {
      const int vec = lane + LPR * t;
      if (vec < nvec) {
        const long off = row * H + vec * 8;
        in.g[t] = Vec8<T>::load_raw(dout + off);
        if (dout2) in.g2[t] = Vec8<T>::load_raw(dout2 + off);
        if (HAS_LN) in.z[t] = Vec8<T>::load_raw(z + off);
        if (dres) in.res[t] = Vec8<T>::load_raw(dres + off);
      }
    }
  };
  RowIn cur, nxt;
  if (group < nrows) request(group, cur);
  for (long row = group; row < nrows; row += ngroups) {
    const bool more = row + ngroups < nrows;
    if (more) request(row + ngroups, nxt);
    float g[NV][8], xh[NV][8];
    float s1 = 0.f, s2 = 0.f;
    const float mean = cur.mean, rs = cur.rs;
#pragma unroll
    for (int t = 0; t < NV; ++t) {
      const int vec = lane + LPR * t;
      if (vec < nvec) {
        const long off = row * H + vec * 8;
        Vec8<T>::unpack(cur.g[t], g[t]);
        if (dout2) {
          float g2[8];
          Vec8<T>::unpack(cur.g2[t], g2);
#pragma unroll
          for (int e = 0; e < 8; ++e) g[t][e] += g2[e];
        }
        if (drop_in.enabled) {   // the incoming gradient passes a dropout that follows the LayerNorm
          float mult[8];
          drop_mult8(drop_in, (uint64_t)off, mult);
#pragma unroll
          for (int e = 0; e < 8; ++e) g[t][e] *= mult[e];
        }
        if (HAS_LN) {
          float zv[8];
          Vec8<T>::unpack(cur.z[t], zv);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            xh[t][e] = (zv[e] - mean) * rs;
            cg[t][e] += g[t][e] * xh[t][e];
            cb[t][e] += g[t][e];
            g[t][e] *= gm[t][e];           // dxhat
            s1 += g[t][e];
            s2 += g[t][e] * xh[t][e];
          }
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) g[t][e] = xh[t][e] = 0.f;
      }
    }
    if (HAS_LN) {
      s1 = group_sum<LPR>(s1) / (float)H;
      s2 = group_sum<LPR>(s2) / (float)H;
    }
#pragma unroll
    for (int t = 0; t < NV; ++t) {
      const int vec = lane + LPR * t;
      if (vec < nvec) {
        const long off = row * H + vec * 8;
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = HAS_LN ? rs * (g[t][e] - s1 - xh[t][e] * s2) : g[t][e];
        if (dres) {
          float r[8];
          Vec8<T>::unpack(cur.res[t], r);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] += r[e];
        }
        if (dz) Vec8<T>::store(dz + off, o);
        if (da) {
          if (drop.enabled) {
            float mult[8];
            drop_mult8(drop, (uint64_t)off, mult);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] *= mult[e];
          }
          Vec8<T>::store(da + off, o);
#pragma unroll
          for (int e = 0; e < 8; ++e) cd[t][e] += o[e];
        }
      }
    }
    if (more) cur = nxt;
  }

  // lanes of different groups inside a wave that own the same columns
#pragma unroll
  for (int t = 0; t < NV; ++t)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma unroll
      for (int o = LPR; o < WAVE; o <<= 1) {
        cg[t][e] += __shfl_xor(cg[t][e], o, WAVE);
        cb[t][e] += __shfl_xor(cb[t][e], o, WAVE);
        cd[t][e] += __shfl_xor(cd[t][e], o, WAVE);
      }
    }
  // The waves deposit their sums in `slices` LDS copies ([slice][3][H], element-major columns so that consecutive
  // lanes hit consecutive banks): wave w owns copy w % slices in round w / slices, and the copies are then added in
  // a fixed order.  With one copy per wave (small H) this is a single barrier.
  const int wave = threadIdx.x >> 6;
  const int wlane = threadIdx.x & 63;
  constexpr int NWAVE = LN_BWD_THREADS / 64;
  float* mine = red + (wave % slices) * 3 * H;
  for (int round = 0; round < NWAVE / slices; ++round) {
    if (wave / slices == round && wlane < LPR) {
#pragma unroll
      for (int t = 0; t < NV; ++t) {
        const int vec = lane + LPR * t;
        if (vec < nvec) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int c = e * nvec + vec;
            if (round == 0) {
              mine[c] = cg[t][e];
              mine[H + c] = cb[t][e];
              mine[2 * H + c] = cd[t][e];
            } else {
              mine[c] += cg[t][e];
              mine[H + c] += cb[t][e];
              mine[2 * H + c] += cd[t][e];
            }
          }
        }
      }
    }
    __syncthreads();
  }
  for (int c = threadIdx.x; c < 3 * H; c += LN_BWD_THREADS) {
    float v = red[c];
    for (int sl = 1; sl < slices; ++sl) v += red[sl * 3 * H + c];
    partial[(long)blockIdx.x * 3 * H + c] = v;
  }
}

// The same operator with one row per lane group and no row loop: 512 threads (two or more wavefronts per SIMD, so
// the arithmetic of one overlaps the memory round trips of another), every operand of the row requested up front,
// and the three column contributions of a row reduced across the lane groups of a wavefront and handed to LDS as
// soon as they exist instead of being carried in registers.  Partial rows have the layout of ln_bwd_kernel.
constexpr int LN_ROW_THREADS = 512;

// Adds the eight values of a column vector over the lane groups of a wavefront that own the same columns and stores
// the totals at dst[e * nvec + vec].  Groups narrower than half a wavefront are first folded with xor shuffles; the two
// halves are then folded with v_permlane32_swap, which exchanges the upper half of one register with the lower half of
// another: after swapping (a, b) the sum of the pair holds a's total in lanes 0..31 and b's in lanes 32..63, one
// exchange and one store instruction per two elements.
template <int LPR>
__device__ __forceinline__ void store_column_totals(float* dst, float (&v)[8], int nvec, int vec, bool on) {
  const int wlane = threadIdx.x & 63;
  if (LPR == 64) {
    if (on) {
#pragma unroll
      for (int e = 0; e < 8; ++e) dst[e * nvec + vec] = v[e];
    }
    return;
  }
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int o = LPR; o < 32; o <<= 1) v[e] += __shfl_xor(v[e], o, WAVE);
  const int half = wlane >> 5;
  const bool writer = on && (wlane & 31) < LPR;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[2 * j]), __float_as_uint(v[2 * j + 1]), false, false);
    const float total = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    if (writer) dst[(2 * j + half) * nvec + vec] = total;
  }
}

template <typename T, int LPR, int NV, bool HAS_LN>
__global__ __launch_bounds__(LN_ROW_THREADS) void ln_bwd_row_kernel(
    const T* __restrict__ dout, const T* __restrict__ dout2, const T* __restrict__ z, const float* __restrict__ mu,
    const float* __restrict__ rstd, const float* __restrict__ gamma, const T* __restrict__ dres, T* __restrict__ dz,
    T* __restrict__ da, float* __restrict__ partial, long nrows, int H, DropSite drop, DropSite drop_in) {
  extern __shared__ float red[];   // [wavefront][3][8][H/8]: column vec*8+e of sum k sits at k*H + e*(H/8) + vec
  constexpr int NWAVE = LN_ROW_THREADS / 64;
  const int lane = threadIdx.x & (LPR - 1);
  const int nvec = H / 8;
  const long row_raw = (long)blockIdx.x * (LN_ROW_THREADS / LPR) + threadIdx.x / LPR;
  const bool live = row_raw < nrows;
  const long row = live ? row_raw : nrows - 1;   // a group without a row reads the last one and contributes zeros
  float* mine = red + (threadIdx.x >> 6) * 3 * H;
  typedef typename Vec8<T>::Raw Raw;
  Raw rg[NV], rg2[NV], rz[NV], rres[NV];
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    const long off = row * H + (vec < nvec ? vec : nvec - 1) * 8;
    rg[t] = Vec8<T>::load_raw(dout + off);
    if (dout2) rg2[t] = Vec8<T>::load_raw(dout2 + off);
    if (HAS_LN) rz[t] = Vec8<T>::load_raw(z + off);
    if (dres) rres[t] = Vec8<T>::load_raw(dres + off);
  }
  float mean = 0.f, rs = 0.f;
  if (HAS_LN) {
    mean = mu[row];
    rs = rstd[row];
  }
  float g[NV][8], xh[NV][8];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    const bool on = vec < nvec;
    const long off = row * H + (on ? vec : nvec - 1) * 8;
    Vec8<T>::unpack(rg[t], g[t]);
    if (dout2) {
      float g2[8];
      Vec8<T>::unpack(rg2[t], g2);
#pragma unroll
      for (int e = 0; e < 8; ++e) g[t][e] += g2[e];
    }
    if (drop_in.enabled) {   // the incoming gradient passes a dropout that follows the LayerNorm
      float mult[8];
      drop_mult8(drop_in, (uint64_t)off, mult);
#pragma unroll
      for (int e = 0; e < 8; ++e) g[t][e] *= mult[e];
    }
    if (!(on && live)) {
#pragma unroll
      for (int e = 0; e < 8; ++e) g[t][e] = 0.f;
    }
    if (HAS_LN) {
      float zv[8], gm[8], cg[8], cb[8];
      Vec8<T>::unpack(rz[t], zv);
      load8f(gamma + (on ? vec : nvec - 1) * 8, gm);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        xh[t][e] = (zv[e] - mean) * rs;
        cg[e] = g[t][e] * xh[t][e];
        cb[e] = g[t][e];
        g[t][e] *= gm[e];           // dxhat
        s1 += g[t][e];
        s2 += g[t][e] * xh[t][e];
      }
      store_column_totals<LPR>(mine, cg, nvec, vec, on);
      store_column_totals<LPR>(mine + H, cb, nvec, vec, on);
    }
  }
  if (HAS_LN) {
    s1 = group_sum<LPR>(s1) / (float)H;
    s2 = group_sum<LPR>(s2) / (float)H;
  }
#pragma unroll
  for (int t = 0; t < NV; ++t) {
    const int vec = lane + LPR * t;
    const bool on = vec < nvec;
    const long off = row * H + (on ? vec : nvec - 1) * 8;
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = HAS_LN ? rs * (g[t][e] - s1 - xh[t][e] * s2) : g[t][e];
    if (dres) {
      float r[8];
      Vec8<T>::unpack(rres[t], r);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] += r[e];
    }
    if (dz && on && live) Vec8<T>::store(dz + off, o);
    if (da) {
      if (drop.enabled) {
        float mult[8];
        drop_mult8(drop, (uint64_t)off, mult);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= mult[e];
      }
      if (on && live) Vec8<T>::store(da + off, o);
      else {
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.f;
      }
      store_column_totals<LPR>(mine + 2 * H, o, nvec, vec, on);
    }
  }
  __syncthreads();
  const int k_begin = HAS_LN ? 0 : 2 * H, k_end = da ? 3 * H : 2 * H;
  for (int c = (int)threadIdx.x; c < 3 * H; c += LN_ROW_THREADS) {
    float v = 0.f;
    if (c >= k_begin && c < k_end) {   // sums this call does not form (no LayerNorm, no da) are written as zeros
      v = red[c];
#pragma unroll
      for (int w = 1; w < NWAVE; ++w) v += red[w * 3 * H + c];
    }
    partial[(long)blockIdx.x * 3 * H + c] = v;
  }
}

// out_k[c] = sum_p partial[p][k][c], k < nout.  16 columns per block; the 16
// slices of a block take parts p = slice, slice+16, ... eight loads at a time
// and are combined in a fixed order, so the sum is reproducible.
constexpr int RED_COLS = 16, RED_SLICES = 16, RED_UNROLL = 8;
struct ReduceGroupDev {
  ReduceJob j[REDUCE_GROUP_MAX];
  int block_start[REDUCE_GROUP_MAX + 1];
};
__global__ __launch_bounds__(256) void reduce_partials_kernel(ReduceGroupDev grp) {
  __shared__ float red[RED_SLICES][RED_COLS];
  int ji = 0;
#pragma unroll
  for (int q = 1; q < REDUCE_GROUP_MAX; ++q)
    if ((int)blockIdx.x >= grp.block_start[q]) ji = q;
  const ReduceJob& job = grp.j[ji];                 // wave-uniform selection
  const float* __restrict__ partial = job.partial;
  const int nparts = job.nparts, ncols = job.ncols, width_out = job.width_out;
  const int cl = threadIdx.x % RED_COLS;
  const int c = ((int)blockIdx.x - grp.block_start[ji]) * RED_COLS + cl;
  const int slice = threadIdx.x / RED_COLS;
  const long width = (long)job.nout * ncols;   // stride between partial rows; only c < width_out is produced
  float acc[RED_UNROLL];
#pragma unroll
  for (int u = 0; u < RED_UNROLL; ++u) acc[u] = 0.f;
  if (c < width_out) {
    int p = slice;
    for (; p + (RED_UNROLL - 1) * RED_SLICES < nparts; p += RED_UNROLL * RED_SLICES) {
      float v[RED_UNROLL];
#pragma unroll
      for (int u = 0; u < RED_UNROLL; ++u) v[u] = partial[(long)(p + u * RED_SLICES) * width + c];
#pragma unroll
      for (int u = 0; u < RED_UNROLL; ++u) acc[u] += v[u];
    }
    for (; p < nparts; p += RED_SLICES) acc[0] += partial[(long)p * width + c];
  }
  red[slice][cl] = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
  __syncthreads();
  if (slice == 0 && c < width_out) {
    float sum = 0.f;
#pragma unroll
    for (int sl = 0; sl < RED_SLICES; ++sl) sum += red[sl][cl];
    const int k = c / ncols;
    int cc = c % ncols;
    if (job.perm_nvec > 0) cc = (cc % job.perm_nvec) * 8 + cc / job.perm_nvec;   // partial rows stored element-major
    float* o = k == 0 ? job.o0 : (k == 1 ? job.o1 : job.o2);
    if (o) o[cc] = sum;
  }
}

raf_status launch_reduce_group(const ReduceJob* jobs, int count, hipStream_t st) {
  if (!jobs || count <= 0 || count > REDUCE_GROUP_MAX) return RAF_EINVAL;
  ReduceGroupDev g{};
  int blocks = 0;
  for (int i = 0; i < count; ++i) {
    if (!jobs[i].partial || jobs[i].nparts <= 0 || jobs[i].ncols <= 0 || jobs[i].nout < 1 || jobs[i].nout > 3) return RAF_EINVAL;
    g.j[i] = jobs[i];
    g.block_start[i] = blocks;
    blocks += (jobs[i].width_out + RED_COLS - 1) / RED_COLS;
  }
  for (int i = count; i <= REDUCE_GROUP_MAX; ++i) g.block_start[i] = blocks;
  for (int i = count; i < REDUCE_GROUP_MAX; ++i) g.j[i] = g.j[0];
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(blocks), dim3(256), 0, st, g);
  return check_launch();
}

// ------------------------------------------------------------ column sum --
constexpr int COLSUM_MAX_PARTS = 64;
struct ColsumGroupDev {
  const void* x[COLSUM_GROUP_MAX];
  float* partial[COLSUM_GROUP_MAX];
  long rows[COLSUM_GROUP_MAX], ld[COLSUM_GROUP_MAX];
  int cols[COLSUM_GROUP_MAX], parts[COLSUM_GROUP_MAX];
  int block_start[COLSUM_GROUP_MAX + 1];
};
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(ColsumGroupDev g) {
  __shared__ float red[4][64 * 8];
  int ji = 0;
#pragma unroll
  for (int q = 1; q < COLSUM_GROUP_MAX; ++q)
    if ((int)blockIdx.x >= g.block_start[q]) ji = q;
  if ((int)blockIdx.y >= g.parts[ji]) return;
  const T* __restrict__ x = (const T*)g.x[ji];
  const long rows = g.rows[ji], ld = g.ld[ji];
  const int cols = g.cols[ji], nparts = g.parts[ji];
  const int bx = (int)blockIdx.x - g.block_start[ji];
  const int cv = bx * 64 + (threadIdx.x & 63);
  const int rl = threadIdx.x >> 6;
  float acc[8] = {};
  if (cv * 8 < cols) {
    const long stride = (long)nparts * 4;
    long r = (long)blockIdx.y * 4 + rl;
    // eight independent 16-byte loads in flight per lane
    for (; r + 7 * stride < rows; r += 8 * stride) {
      float v[8][8];
#pragma unroll
      for (int u = 0; u < 8; ++u) Vec8<T>::load(x + (r + u * stride) * ld + cv * 8, v[u]);
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += v[u][e];
    }
    for (; r < rows; r += stride) {
      float v[8];
      Vec8<T>::load(x + r * ld + cv * 8, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += v[e];
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rl][(threadIdx.x & 63) * 8 + e] = acc[e];
  __syncthreads();
  for (int c = threadIdx.x; c < 64 * 8; c += 256) {
    const int col = bx * 512 + c;
    if (col < cols) g.partial[ji][(long)blockIdx.y * cols + col] = red[0][c] + red[1][c] + red[2][c] + red[3][c];
  }
}

// ---------------------------------------------------------------- launch --
static bool row_shape_ok(long len) { return len >= 32 && len % 8 == 0 && len <= 4096; }

raf_status launch_softmax_fwd(const raf_layer_desc& d, const void* s, const int32_t* lens, void* prob, void* prob_d,
                              uint64_t step, hipStream_t st) {
  if (!s || !prob || !prob_d) return RAF_EINVAL;
  if (!aligned16(s) || !aligned16(prob) || !aligned16(prob_d)) return RAF_EINVAL;
  if (!row_shape_ok(d.seq)) return RAF_ENOTSUP;
  const long nrows = (long)d.batch * d.heads * d.seq;
  if ((uint64_t)nrows * d.seq / 4 > 0xffffffffull) return RAF_ENOTSUP;
  const DropSite drop = make_drop_site(d, 1, step);
#define CALL(LPR, NV)                                                                                          \
  {                                                                                                            \
    const long nblk = (nrows * LPR + 255) / 256;                                                               \
    if (d.precision == RAF_F32)                                                                                \
      hipLaunchKernelGGL((softmax_fwd_kernel<float, LPR, NV>), dim3(nblk), dim3(256), 0, st, (const float*)s, \
                         lens, (float*)prob, (float*)prob_d, nrows, d.seq, d.heads, d.causal, drop);           \
    else                                                                                                       \
      hipLaunchKernelGGL((softmax_fwd_kernel<bf16_t, LPR, NV>), dim3(nblk), dim3(256), 0, st,                 \
                         (const bf16_t*)s, lens, (bf16_t*)prob, (bf16_t*)prob_d, nrows, d.seq, d.heads,        \
                         d.causal, drop);                                                                      \
  }
  RAF_DISPATCH_GEOM(row_geom(d.seq), CALL);
#undef CALL
  return check_launch();
}

raf_status launch_softmax_bwd(const raf_layer_desc& d, const void* prob, const void* prob_d, const void* dprob_d,
                              void* ds, float scale_out, hipStream_t st) {
  if (!prob || !prob_d || !dprob_d || !ds) return RAF_EINVAL;
  if (!aligned16(prob) || !aligned16(prob_d) || !aligned16(dprob_d) || !aligned16(ds)) return RAF_EINVAL;
  if (!row_shape_ok(d.seq)) return RAF_ENOTSUP;
  const long nrows = (long)d.batch * d.heads * d.seq;
  const float drop_scale = (float)(1.0 / (1.0 - d.dropout_p));
#define CALL(LPR, NV)                                                                                             \
  {                                                                                                               \
    const long nblk = (nrows * LPR + 255) / 256;                                                                  \
    if (d.precision == RAF_F32)                                                                                   \
      hipLaunchKernelGGL((softmax_bwd_kernel<float, LPR, NV>), dim3(nblk), dim3(256), 0, st, (const float*)prob, \
                         (const float*)prob_d, (const float*)dprob_d, (float*)ds, nrows, d.seq, drop_scale,       \
                         scale_out);                                                                              \
    else                                                                                                          \
      hipLaunchKernelGGL((softmax_bwd_kernel<bf16_t, LPR, NV>), dim3(nblk), dim3(256), 0, st,                    \
                         (const bf16_t*)prob, (const bf16_t*)prob_d, (const bf16_t*)dprob_d, (bf16_t*)ds, nrows,  \
                         d.seq, drop_scale, scale_out);                                                           \
  }
  RAF_DISPATCH_GEOM(row_geom(d.seq), CALL);
#undef CALL
  return check_launch();
}

int ln_fwd_blocks(int hidden, int64_t rows) {
  const RowGeom g = row_geom(hidden);
  return (int)(((long)rows * g.lpr + 255) / 256);
}

raf_status launch_ln_fwd(const raf_layer_desc& d, int site, int64_t rows, const void* a, const void* res,
                         const float* gamma, const float* beta, void* out, void* z_out, float* mu, float* rstd,
                         uint64_t step, hipStream_t st, const LossSeedDev* loss) {
  if (!res || !out || rows <= 0) return RAF_EINVAL;
  if (gamma && (!beta || !mu || !rstd)) return RAF_EINVAL;
  if (a && site != 2 && site != 3) return RAF_EINVAL;
  if (!aligned16(a) || !aligned16(res) || !aligned16(out) || !aligned16(z_out) || !aligned16(gamma) ||
      !aligned16(beta))
    return RAF_EINVAL;
  if (loss && (!loss->G || !loss->dy || !loss->partial || !aligned16(loss->G) || !aligned16(loss->dy))) return RAF_EINVAL;
  if (!row_shape_ok(d.hidden)) return RAF_ENOTSUP;
  if ((uint64_t)rows * d.hidden / 4 > 0xffffffffull) return RAF_ENOTSUP;
  const DropSite drop = make_drop_site(d, a ? site : 0, step);
  const int H = d.hidden;
  const LossSeedDev ls = loss ? *loss : LossSeedDev{};
#define CALL_T(T, LPR, NV)                                                                                           \
  {                                                                                                                  \
    const long nblk = ((long)rows * LPR + 255) / 256;                                                                \
    if (loss)                                                                                                        \
      hipLaunchKernelGGL((ln_fwd_kernel<T, LPR, NV, true>), dim3(nblk), dim3(256), 0, st, (const T*)a, (const T*)res, \
                         gamma, beta, (T*)out, (T*)z_out, mu, rstd, (long)rows, H, d.ln_eps, drop, ls);              \
    else                                                                                                             \
      hipLaunchKernelGGL((ln_fwd_kernel<T, LPR, NV, false>), dim3(nblk), dim3(256), 0, st, (const T*)a, (const T*)res, \
                         gamma, beta, (T*)out, (T*)z_out, mu, rstd, (long)rows, H, d.ln_eps, drop, ls);              \
  }
#define CALL(LPR, NV)                                        \
  {                                                          \
    if (d.precision == RAF_F32) CALL_T(float, LPR, NV)       \
    else CALL_T(bf16_t, LPR, NV)                             \
  }
  RAF_DISPATCH_GEOM(row_geom(H), CALL);
#undef CALL
#undef CALL_T
  return check_launch();
}

// Which of the two adjoint kernels a shape takes, and with how many workgroups (= partial rows): one row per lane
// group (ln_bwd_row_kernel) while its LDS copies fit and the partial rows stay few, the looping kernel otherwise.
constexpr int LN_ROW_MAX_BLOCKS = 1024;
struct LnBwdPlan {
  bool row_kernel;
  int blocks;
};
static LnBwdPlan ln_bwd_plan(int hidden, int64_t rows) {
  const RowGeom g = row_geom(hidden);
  const long per_block = LN_ROW_THREADS / g.lpr;
  const long nb_row = (rows + per_block - 1) / per_block;
  const size_t lds_row = (size_t)(LN_ROW_THREADS / 64) * 3 * hidden * sizeof(float);
  if (lds_row <= 144 * 1024 && nb_row <= LN_ROW_MAX_BLOCKS) return LnBwdPlan{true, (int)(nb_row < 1 ? 1 : nb_row)};
  const long groups_per_block = 256 / g.lpr;
  long nb = (rows + groups_per_block - 1) / groups_per_block;   // one row per group until the block cap
  if (nb < 1) nb = 1;
  if (nb > LN_BWD_MAX_BLOCKS) nb = LN_BWD_MAX_BLOCKS;
  return LnBwdPlan{false, (int)nb};
}

size_t ln_bwd_partial_floats(int hidden, int64_t rows) {
  if (hidden <= 0 || rows <= 0) return 0;
  return (size_t)ln_bwd_plan(hidden, rows).blocks * 3 * (size_t)hidden;
}

struct LnBwdArgs {
  const void *dout, *dout2, *z, *dres;
  const float *mu, *rstd, *gamma;
  void *dz, *da;
  float* partial;
  long rows;
  int H;
  DropSite drop, drop_in;
  int slices;
};
template <typename T, int LPR, int NV, bool HAS_LN, int TH>
static bool launch_ln_bwd_inst(const LnBwdArgs& a, int nb, size_t shm, hipStream_t st) {
  auto kern = ln_bwd_kernel<T, LPR, NV, HAS_LN, TH>;
  static LdsLimitOnce lds_limit;   // per instantiation
  if (shm > 48 * 1024 && !lds_limit.ensure((const void*)kern, (int)shm)) return false;
  hipLaunchKernelGGL(kern, dim3(nb), dim3(TH), shm, st, (const T*)a.dout, (const T*)a.dout2, (const T*)a.z, a.mu, a.rstd,
                     a.gamma, (const T*)a.dres, (T*)a.dz, (T*)a.da, a.partial, a.rows, a.H, a.drop, a.drop_in, a.slices);
  return true;
}
template <typename T, int LPR, int NV, bool HAS_LN>
static bool launch_ln_bwd_row_inst(const LnBwdArgs& a, int nb, size_t shm, hipStream_t st) {
  auto kern = ln_bwd_row_kernel<T, LPR, NV, HAS_LN>;
  static LdsLimitOnce lds_limit;   // per instantiation
  if (shm > 48 * 1024 && !lds_limit.ensure((const void*)kern, (int)shm)) return false;
  hipLaunchKernelGGL(kern, dim3(nb), dim3(LN_ROW_THREADS), shm, st, (const T*)a.dout, (const T*)a.dout2, (const T*)a.z,
                     a.mu, a.rstd, a.gamma, (const T*)a.dres, (T*)a.dz, (T*)a.da, a.partial, a.rows, a.H, a.drop,
                     a.drop_in);
  return true;
}
template <typename T, int LPR, int NV>
static bool launch_ln_bwd_geom(const LnBwdArgs& a, bool row_kernel, int nb, size_t shm, hipStream_t st) {
  if (row_kernel)
    return a.gamma ? launch_ln_bwd_row_inst<T, LPR, NV, true>(a, nb, shm, st)
                   : launch_ln_bwd_row_inst<T, LPR, NV, false>(a, nb, shm, st);
  return a.gamma ? launch_ln_bwd_inst<T, LPR, NV, true, 256>(a, nb, shm, st)
                 : launch_ln_bwd_inst<T, LPR, NV, false, 256>(a, nb, shm, st);
}

raf_status launch_ln_bwd(const raf_layer_desc& d, int site, int64_t rows, const void* dout, const void* dout2,
                         const void* z, const float* mu, const float* rstd, const float* gamma, const void* dres,
                         void* dz, void* da, float* dgamma, float* dbeta, float* dbias, float* partial,
                         uint64_t step, hipStream_t st, int site_in, ReduceJob* defer) {
  if (!dout || !partial || rows <= 0) return RAF_EINVAL;
  if (gamma && (!z || !mu || !rstd || !dgamma || !dbeta)) return RAF_EINVAL;
  if (!dz && !da) return RAF_EINVAL;
  if (da && !dbias) return RAF_EINVAL;
  if (site != 0 && site != 2 && site != 3) return RAF_EINVAL;
  if (site_in != 0 && site_in != 4) return RAF_EINVAL;
  if (!aligned16(dout) || !aligned16(dout2) || !aligned16(z) || !aligned16(gamma) || !aligned16(dres) ||
      !aligned16(dz) || !aligned16(da))
    return RAF_EINVAL;
  if (!row_shape_ok(d.hidden)) return RAF_ENOTSUP;
  if ((uint64_t)rows * d.hidden / 4 > 0xffffffffull) return RAF_ENOTSUP;
  const int H = d.hidden;
  const LnBwdPlan plan = ln_bwd_plan(H, rows);
  const int nb = plan.blocks;
  // LDS copies of the column sums (3 * H floats each): one per wavefront in the row kernel, at most 48 KiB otherwise
  const int slices = plan.row_kernel ? LN_ROW_THREADS / 64 : (H <= 1024 ? 4 : (H <= 2048 ? 2 : 1));
  const size_t shm = (size_t)slices * 3 * H * sizeof(float);
  const LnBwdArgs a{dout, dout2, z, dres, mu, rstd, gamma, dz, da, partial, (long)rows, H,
                    make_drop_site(d, site, step), make_drop_site(d, site_in, step), slices};
  bool ok = false;
#define CALL(LPR, NV)                                                                       \
  {                                                                                         \
    if (d.precision == RAF_F32) ok = launch_ln_bwd_geom<float, LPR, NV>(a, plan.row_kernel, nb, shm, st); \
    else ok = launch_ln_bwd_geom<bf16_t, LPR, NV>(a, plan.row_kernel, nb, shm, st);                \
  }
  RAF_DISPATCH_GEOM(row_geom(H), CALL);
#undef CALL
  if (!ok) return RAF_EHIP;
  raf_status rc = check_launch();
  if (rc != RAF_OK) return rc;
  const ReduceJob job{partial, nb, H, 3, gamma ? dgamma : nullptr, gamma ? dbeta : nullptr, da ? dbias : nullptr, 3 * H, H / 8};
  if (defer) {
    *defer = job;
    return RAF_OK;
  }
  return launch_reduce_group(&job, 1, st);
}

static int colsum_parts(int64_t rows) {
  long p = (rows + 63) / 64;
  if (p < 1) p = 1;
  if (p > COLSUM_MAX_PARTS) p = COLSUM_MAX_PARTS;
  return (int)p;
}
size_t colsum_partial_floats(int cols, int64_t rows) { return (size_t)colsum_parts(rows) * (size_t)cols; }

raf_status launch_colsum_group(const ColsumJob* jobs, int count, ReduceJob* reduce_jobs, int* nreduce, hipStream_t st) {
  if (!jobs || count <= 0 || count > COLSUM_GROUP_MAX || !reduce_jobs || !nreduce) return RAF_EINVAL;
  ColsumGroupDev g{};
  int blocks = 0, max_parts = 0;
  for (int i = 0; i < count; ++i) {
    const ColsumJob& j = jobs[i];
    if (!j.x || !j.out || !j.partial || j.rows <= 0 || j.cols <= 0) return RAF_EINVAL;
    if ((j.cols % 8) || (j.ld % 8) || !aligned16(j.x) || j.precision != jobs[0].precision) return RAF_EINVAL;
    const int out_cols = (j.out_cols <= 0 || j.out_cols > j.cols) ? j.cols : j.out_cols;
    g.x[i] = j.x; g.partial[i] = j.partial; g.rows[i] = (long)j.rows; g.ld[i] = j.ld; g.cols[i] = j.cols;
    g.parts[i] = colsum_parts(j.rows);
    g.block_start[i] = blocks;
    blocks += (j.cols + 511) / 512;
    max_parts = g.parts[i] > max_parts ? g.parts[i] : max_parts;
    reduce_jobs[(*nreduce)++] = ReduceJob{j.partial, g.parts[i], j.cols, 1, j.out, nullptr, nullptr, out_cols, 0};
  }
  for (int i = count; i <= COLSUM_GROUP_MAX; ++i) g.block_start[i] = blocks;
  for (int i = count; i < COLSUM_GROUP_MAX; ++i) { g.x[i] = g.x[0]; g.partial[i] = g.partial[0]; g.rows[i] = g.rows[0]; g.ld[i] = g.ld[0]; g.cols[i] = g.cols[0]; g.parts[i] = 0; }
  dim3 grid(blocks, max_parts);
  if (jobs[0].precision == RAF_F32) hipLaunchKernelGGL((colsum_kernel<float>), grid, dim3(256), 0, st, g);
  else hipLaunchKernelGGL((colsum_kernel<bf16_t>), grid, dim3(256), 0, st, g);
  return check_launch();
}

raf_status launch_colsum(int precision, const void* x, int64_t rows, int cols, long ld, float* out, float* partial,
                         hipStream_t st, int out_cols) {
  const ColsumJob job{precision, x, rows, cols, ld, out, partial, out_cols};
  ReduceJob rj[1];
  int nr = 0;
  raf_status rc = launch_colsum_group(&job, 1, rj, &nr, st);
  if (rc != RAF_OK) return rc;
  return launch_reduce_group(rj, nr, st);
}

}  // namespace raf
