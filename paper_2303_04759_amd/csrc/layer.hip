// The training step of one transformer layer as a fixed kernel schedule:
// forward graph and the reverse chain of adjoints (paper Sections 2.1, 3.1.1),
// with the fused operators of Section 3.2.2.  Host code only: it validates
// the descriptor, lays out the saved/scratch buffers and enqueues kernels on
// the caller's stream; it never allocates or synchronises.
#include <mutex>
#include <string>

#include "common.hpp"

namespace raf {

static std::mutex g_err_mutex;
static std::string g_err = "";
void set_hip_error(hipError_t e) {
  std::lock_guard<std::mutex> lk(g_err_mutex);
  g_err = hipGetErrorString(e);
}

static raf_status validate_desc(const raf_layer_desc* d) {
  if (!d) return RAF_EINVAL;
  if (d->batch <= 0 || d->seq <= 0 || d->hidden <= 0 || d->heads <= 0 || d->ffn <= 0) return RAF_EINVAL;
  if (d->precision != RAF_F32 && d->precision != RAF_BF16_AMP) return RAF_EINVAL;
  if ((d->pre_ln | 1) != 1 || (d->causal | 1) != 1 || (d->gelu_tanh | 1) != 1) return RAF_EINVAL;
  if (!(d->dropout_p >= 0.0 && d->dropout_p < 1.0)) return RAF_EINVAL;
  if (!(d->ln_eps >= 0.f)) return RAF_EINVAL;
  if (d->reserved != 0) return RAF_EINVAL;
  if (d->hidden % d->heads) return RAF_ENOTSUP;
  if (d->hidden / d->heads != 64) return RAF_ENOTSUP;
  if ((d->seq % 32) || (d->hidden % 32) || (d->ffn % 32)) return RAF_ENOTSUP;
  if (d->seq > 4096 || d->hidden > 4096 || d->ffn > 65536) return RAF_ENOTSUP;
  const long T = (long)d->batch * d->seq;
  if (T > (1l << 24) || (long)d->batch * d->heads > 65535) return RAF_ENOTSUP;
  // 32-bit Philox block counters per site
  if ((unsigned long)d->batch * d->heads * d->seq * d->seq / 4 > 0xfffffffful) return RAF_ENOTSUP;
  return RAF_OK;
}

// Byte offsets into the two caller-provided buffers.
struct Plan {
  size_t e;   // element size of the compute dtype
  long T, H, F, S, NH, B, PS;   // PS = B*heads*S*S
  // saved
  size_t qkv, prob, prob_d, c, z1, ffn_in, u, g, z2, n1, mu1, rstd1, mu2, rstd2, lse, saved_bytes;
  // scratch, forward
  size_t s, a;
  // scratch, backward
  size_t dz2, da, da1, du, dffn, dz1, dc, dprob_d, ds, dqkv, dattn, dvec, partial_ln[3], partial_cs[2], wt_qkv, wt_o, wt_1, wt_2;
  size_t scratch_bytes;
};

static size_t bump(size_t& off, size_t bytes) {
  const size_t at = off;
  off += (bytes + 255) & ~(size_t)255;
  return at;
}

static Plan make_plan(const raf_layer_desc& d) {
  Plan p{};
  p.e = d.precision == RAF_F32 ? 4 : 2;
  p.B = d.batch; p.S = d.seq; p.H = d.hidden; p.F = d.ffn; p.NH = d.heads;
  p.T = p.B * p.S;
  p.PS = p.B * p.NH * p.S * p.S;
  // the bf16 attention kernels keep every S x S tensor on chip: no room is reserved for them
  const bool onchip = attn_fused_supported(d) || attn_flash_supported(d);
  const size_t TH = (size_t)p.T * p.H * p.e, TF = (size_t)p.T * p.F * p.e, PSb = onchip ? 0 : (size_t)p.PS * p.e;
  const size_t rowstat = attn_flash_supported(d) ? (size_t)p.B * p.NH * p.S * 4 : 0;   // one float per query row and head
  size_t o = 0;
  p.qkv = bump(o, 3 * TH);
  p.prob = bump(o, PSb);
  p.prob_d = bump(o, PSb);
  p.c = bump(o, TH);
  p.z1 = bump(o, TH);
  p.ffn_in = bump(o, TH);
  p.u = bump(o, TF);
  p.g = bump(o, TF);
  p.z2 = bump(o, TH);
  p.n1 = bump(o, TH);
  p.mu1 = bump(o, p.T * 4);
  p.rstd1 = bump(o, p.T * 4);
  p.mu2 = bump(o, p.T * 4);
  p.rstd2 = bump(o, p.T * 4);
  p.lse = bump(o, rowstat);
  p.saved_bytes = o;
  size_t f = 0;
  p.s = bump(f, PSb);
  p.a = bump(f, TH);
  size_t b = 0;
  p.dz2 = bump(b, TH);
  p.da = bump(b, TH);
  p.da1 = bump(b, TH);
  p.du = bump(b, TF);
  p.dffn = bump(b, TH);
  p.dz1 = bump(b, TH);
  p.dc = bump(b, TH);
  p.dprob_d = bump(b, PSb);
  p.ds = bump(b, PSb);
  p.dqkv = bump(b, 3 * TH);
  p.dattn = bump(b, TH);
  p.dvec = bump(b, rowstat);
  // one partial-sum buffer per producer: their second stages run together at the end of the backward pass
  for (int i = 0; i < 3; ++i) p.partial_ln[i] = bump(b, ln_bwd_partial_floats((int)p.H, p.T) * 4);
  p.partial_cs[0] = bump(b, colsum_partial_floats((int)p.F, p.T) * 4);
  p.partial_cs[1] = bump(b, colsum_partial_floats((int)(3 * p.H), p.T) * 4);
  if (d.precision == RAF_BF16_AMP) {   // transposed bf16 weight copies for the input-gradient products
    p.wt_qkv = bump(b, (size_t)3 * p.H * p.H * 2);
    p.wt_o = bump(b, (size_t)p.H * p.H * 2);
    p.wt_1 = bump(b, (size_t)p.F * p.H * 2);
    p.wt_2 = bump(b, (size_t)p.H * p.F * 2);
  }
  p.scratch_bytes = f > b ? f : b;
  return p;
}

static inline char* at(void* base, size_t off) { return (char*)base + off; }
static inline const char* at(const void* base, size_t off) { return (const char*)base + off; }

static bool tensors_ok(const raf_layer_tensors* t) {
  if (!t) return false;
  const void* const* p = (const void* const*)t;
  for (int i = 0; i < 12; ++i)
    if (!p[i] || !aligned16(p[i])) return false;
  return true;
}

#define RAF_TRY(expr)                \
  do {                               \
    raf_status _rc = (expr);         \
    if (_rc != RAF_OK) return _rc;   \
  } while (0)

// plain (un-batched) GEMM helper: C[M,N] = A.B, see GemmArgs
static raf_status gemm(int prec, hipStream_t st, int M, int N, int K, const void* a, long lda, int ak, const void* b,
                       long ldb, int bk, void* c, long ldc, int out_f32 = 0, int epi = EPI_NONE,
                       const float* bias = nullptr, void* aux = nullptr, long ldaux = 0, int gelu_tanh = 0) {
  GemmArgs g = gemm_args_default();
  g.M = M; g.N = N; g.K = K;
  g.a = a; g.lda = lda; g.a_kmajor = ak;
  g.b = b; g.ldb = ldb; g.b_kmajor = bk;
  g.c = c; g.ldc = ldc; g.out_f32 = out_f32;
  g.epilogue = epi; g.bias = bias; g.aux = aux; g.ldaux = ldaux; g.gelu_tanh = gelu_tanh;
  return launch_gemm(prec, g, st);
}

// weight-gradient form: C[M,N] (float) = A^T B with A [K,M], B [K,N] row-major
static GemmArgs wgrad_args(int M, int N, int K, const void* a, long lda, const void* b, long ldb, void* c, long ldc) {
  GemmArgs g = gemm_args_default();
  g.M = M; g.N = N; g.K = K;
  g.a = a; g.lda = lda; g.a_kmajor = 0;
  g.b = b; g.ldb = ldb; g.b_kmajor = 0;
  g.c = c; g.ldc = ldc; g.out_f32 = 1;
  return g;
}

// per-(batch, head) GEMM over views of [T, ld] tensors (64 columns per head)
// and/or [B, heads, S, S] tensors
struct HeadView {
  const void* p; long ld; int kmajor; bool is_prob;   // is_prob: [B,heads,S,S] else [T, ld] with head offset 64*h
};
static GemmArgs heads_args(const Plan& p, int M, int N, int K, HeadView a, HeadView b, void* c, long ldc, bool c_is_prob,
                           float alpha) {
  GemmArgs g = gemm_args_default();
  g.M = M; g.N = N; g.K = K;
  g.a = a.p; g.lda = a.ld; g.a_kmajor = a.kmajor;
  g.b = b.p; g.ldb = b.ld; g.b_kmajor = b.kmajor;
  g.c = c; g.ldc = ldc; g.alpha = alpha;
  g.batch = (int)(p.B * p.NH);
  g.nz_inner = (int)p.NH;
  g.sa[0] = a.is_prob ? p.NH * p.S * p.S : p.S * a.ld; g.sa[1] = a.is_prob ? p.S * p.S : 64;
  g.sb[0] = b.is_prob ? p.NH * p.S * p.S : p.S * b.ld; g.sb[1] = b.is_prob ? p.S * p.S : 64;
  g.sc[0] = c_is_prob ? p.NH * p.S * p.S : p.S * ldc;  g.sc[1] = c_is_prob ? p.S * p.S : 64;
  return g;
}
static raf_status gemm_heads(const Plan& p, int prec, hipStream_t st, int M, int N, int K, HeadView a, HeadView b,
                             void* c, long ldc, bool c_is_prob, float alpha) {
  return launch_gemm(prec, heads_args(p, M, N, K, a, b, c, ldc, c_is_prob, alpha), st);
}

}  // namespace raf

using namespace raf;

extern "C" raf_status raf_layer_workspace(const raf_layer_desc* desc, size_t* saved_bytes, size_t* scratch_bytes) {
  RAF_TRY(validate_desc(desc));
  if (!saved_bytes || !scratch_bytes) return RAF_EINVAL;
  const Plan p = make_plan(*desc);
  *saved_bytes = p.saved_bytes;
  *scratch_bytes = p.scratch_bytes;
  return RAF_OK;
}

extern "C" raf_status raf_layer_fwd(const raf_layer_desc* desc, const raf_layer_tensors* w, const void* x,
                                    const int32_t* seq_lens, void* y, void* saved, void* scratch, uint64_t step,
                                    void* hip_stream) {
  RAF_TRY(validate_desc(desc));
  if (!tensors_ok(w) || !x || !y || !saved || !scratch) return RAF_EINVAL;
  if (!aligned16(x) || !aligned16(y) || !aligned16(saved) || !aligned16(scratch)) return RAF_EINVAL;
  if (seq_lens && ((uintptr_t)seq_lens & 3u)) return RAF_EINVAL;
  const raf_layer_desc& d = *desc;
  const Plan p = make_plan(d);
  hipStream_t st = (hipStream_t)hip_stream;
  const int prec = d.precision;
  const int T = (int)p.T, H = (int)p.H, F = (int)p.F, S = (int)p.S;
  const size_t e = p.e;
  const float alpha = 0.125f;   // 1/sqrt(64)

  void* qkv = at(saved, p.qkv);
  void* prob = at(saved, p.prob);
  void* prob_d = at(saved, p.prob_d);
  void* c = at(saved, p.c);
  void* z1 = at(saved, p.z1);
  void* ffn_in = at(saved, p.ffn_in);
  void* u = at(saved, p.u);
  void* g = at(saved, p.g);
  void* z2 = at(saved, p.z2);
  void* n1 = at(saved, p.n1);
  float* mu1 = (float*)at(saved, p.mu1);
  float* rstd1 = (float*)at(saved, p.rstd1);
  float* mu2 = (float*)at(saved, p.mu2);
  float* rstd2 = (float*)at(saved, p.rstd2);
  void* s = at(scratch, p.s);
  void* a = at(scratch, p.a);

  const void* attn_in = x;
  if (d.pre_ln) {
    RAF_TRY(launch_ln_fwd(d, 0, T, nullptr, x, (const float*)w->ln1_g, (const float*)w->ln1_b, n1, nullptr, mu1,
                          rstd1, step, st));
    attn_in = n1;
  }
  // F1: qkv = attn_in . Wqkv^T + bqkv
  RAF_TRY(gemm(prec, st, T, 3 * H, H, attn_in, H, 1, w->w_qkv, H, 1, qkv, 3 * H, 0, EPI_BIAS, (const float*)w->b_qkv));
  const bool attn_fused = attn_fused_supported(d) || attn_flash_supported(d);   // F4 is taken inside the attention kernel
  if (attn_fused_supported(d)) {
    // F2+F3+F4 fused: scores, mask, softmax, dropout site 1, context; the backward pass recomputes the
    // probabilities, so they are not stored
    RAF_TRY(launch_attn_fwd_fused(d, qkv, seq_lens, c, step, st));
  } else if (attn_flash_supported(d)) {
    // the same for longer rows, 128 keys at a time; leaves one softmax statistic per query row for the backward pass
    RAF_TRY(launch_attn_flash_fwd(d, qkv, seq_lens, c, (float*)at(saved, p.lse), step, st));
  } else {   // fp32
    // F2: s = Q K^T / 8 per (batch, head)
    RAF_TRY(gemm_heads(p, prec, st, S, S, 64, HeadView{qkv, 3 * H, 1, false},
                       HeadView{at(qkv, (size_t)H * e), 3 * H, 1, false}, s, S, true, alpha));
    // F3: masked softmax + dropout site 1
    RAF_TRY(launch_softmax_fwd(d, s, seq_lens, prob, prob_d, step, st));
  }
  // F4: c = prob_d . V, heads merged on store
  if (!attn_fused)
    RAF_TRY(gemm_heads(p, prec, st, S, 64, S, HeadView{prob_d, S, 1, true},
                       HeadView{at(qkv, (size_t)2 * H * e), 3 * H, 0, false}, c, H, false, 1.0f));
  // F5: a1 = c . Wo^T + bo
  RAF_TRY(gemm(prec, st, T, H, H, c, H, 1, w->w_o, H, 1, a, H, 0, EPI_BIAS, (const float*)w->b_o));
  // F6: z1 = x + drop2(a1); ffn_in = LN(z1)   (LN1 in post-LN, LN2 in pre-LN)
  if (d.pre_ln)
    RAF_TRY(launch_ln_fwd(d, 2, T, a, x, (const float*)w->ln2_g, (const float*)w->ln2_b, ffn_in, z1, mu2, rstd2, step,
                          st));
  else
    RAF_TRY(launch_ln_fwd(d, 2, T, a, x, (const float*)w->ln1_g, (const float*)w->ln1_b, ffn_in, z1, mu1, rstd1, step,
                          st));
  // F7: u = ffn_in . W1^T + b1; g = gelu(u).  Saved for the backward pass: u (fp32 mode) or, in bf16 AMP,
  // gelu'(u), which shares the erf of the forward evaluation and makes the backward epilogue one multiply
  RAF_TRY(gemm(prec, st, T, F, H, ffn_in, H, 1, w->w_1, H, 1, g, F, 0,
               prec == RAF_BF16_AMP ? EPI_BIAS_GELU_DERIV : EPI_BIAS_GELU, (const float*)w->b_1, u, F, d.gelu_tanh));
  // F8: a2 = g . W2^T + b2
  RAF_TRY(gemm(prec, st, T, H, F, g, F, 1, w->w_2, F, 1, a, H, 0, EPI_BIAS, (const float*)w->b_2));
  // F9: post-LN: z2 = ffn_in + drop3(a2), y = LN2(z2); pre-LN: y = z1 + drop3(a2)
  if (d.pre_ln)
    RAF_TRY(launch_ln_fwd(d, 3, T, a, z1, nullptr, nullptr, y, nullptr, nullptr, nullptr, step, st));
  else
    RAF_TRY(launch_ln_fwd(d, 3, T, a, ffn_in, (const float*)w->ln2_g, (const float*)w->ln2_b, y, z2, mu2, rstd2, step,
                          st));
  return RAF_OK;
}

extern "C" raf_status raf_layer_bwd(const raf_layer_desc* desc, const raf_layer_tensors* w, const void* x,
                                    const void* dy, const int32_t* seq_lens, const void* saved, void* dx,
                                    raf_layer_tensors* grads, void* scratch, uint64_t step, void* hip_stream) {
  RAF_TRY(validate_desc(desc));
  if (!tensors_ok(w) || !tensors_ok(grads) || !x || !dy || !dx || !saved || !scratch) return RAF_EINVAL;
  if (!aligned16(x) || !aligned16(dy) || !aligned16(dx) || !aligned16(saved) || !aligned16(scratch)) return RAF_EINVAL;
  const raf_layer_desc& d = *desc;
  const Plan p = make_plan(d);
  hipStream_t st = (hipStream_t)hip_stream;
  const int prec = d.precision;
  const int T = (int)p.T, H = (int)p.H, F = (int)p.F, S = (int)p.S;
  const size_t e = p.e;
  const float alpha = 0.125f;

  const void* qkv = at(saved, p.qkv);
  const void* prob = at(saved, p.prob);
  const void* prob_d = at(saved, p.prob_d);
  const void* c = at(saved, p.c);
  const void* z1 = at(saved, p.z1);
  const void* ffn_in = at(saved, p.ffn_in);
  void* u = (void*)at(saved, p.u);
  const void* g = at(saved, p.g);
  const void* z2 = at(saved, p.z2);
  const void* n1 = at(saved, p.n1);
  const float* mu1 = (const float*)at(saved, p.mu1);
  const float* rstd1 = (const float*)at(saved, p.rstd1);
  const float* mu2 = (const float*)at(saved, p.mu2);
  const float* rstd2 = (const float*)at(saved, p.rstd2);

  void* dz2 = at(scratch, p.dz2);
  void* da = at(scratch, p.da);     // da2, kept until the grouped weight-gradient launch
  void* da1 = at(scratch, p.da1);
  void* du = at(scratch, p.du);
  void* dffn = at(scratch, p.dffn);
  void* dz1 = at(scratch, p.dz1);
  void* dc = at(scratch, p.dc);
  void* dprob_d = at(scratch, p.dprob_d);
  void* ds = at(scratch, p.ds);
  void* dqkv = at(scratch, p.dqkv);
  void* dattn = at(scratch, p.dattn);
  float* partial_ln[3] = {(float*)at(scratch, p.partial_ln[0]), (float*)at(scratch, p.partial_ln[1]),
                          (float*)at(scratch, p.partial_ln[2])};
  // second stages of the LayerNorm / bias gradient sums and the two bias column sums, launched together at the end
  ReduceJob rj[REDUCE_GROUP_MAX];
  int nr = 0;
  ColsumJob cj[COLSUM_GROUP_MAX];

  // bf16: the input-gradient products below use K-major transposed copies of the four weights
  const bool wt = prec == RAF_BF16_AMP;
  const void* wt_qkv = at(scratch, p.wt_qkv);   // [H][3H]
  const void* wt_o = at(scratch, p.wt_o);       // [H][H]
  const void* wt_1 = at(scratch, p.wt_1);       // [H][F]
  const void* wt_2 = at(scratch, p.wt_2);       // [F][H]
  if (wt) {
    const TransposeJob jobs[4] = {{w->w_qkv, (void*)wt_qkv, 3 * H, H}, {w->w_o, (void*)wt_o, H, H},
                                  {w->w_1, (void*)wt_1, F, H}, {w->w_2, (void*)wt_2, H, F}};
    RAF_TRY(launch_transpose_bf16(jobs, 4, st));
  }
  // B9: adjoint of the output block
  if (d.pre_ln)   // y = z1 + drop3(a2): da2 = dy * keep3/(1-p)
    RAF_TRY(launch_ln_bwd(d, 3, T, dy, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, da, nullptr,
                          nullptr, (float*)grads->b_2, partial_ln[0], step, st, 0, &rj[nr++]));
  else            // y = LN2(z2), z2 = ffn_in + drop3(a2)
    RAF_TRY(launch_ln_bwd(d, 3, T, dy, nullptr, z2, mu2, rstd2, (const float*)w->ln2_g, nullptr, dz2, da,
                          (float*)grads->ln2_g, (float*)grads->ln2_b, (float*)grads->b_2, partial_ln[0], step, st, 0,
                          &rj[nr++]));
  // The four weight gradients (dW = dY^T X) are deferred to one grouped launch
  // at the end: each alone has too few output tiles to fill 256 CUs.
  // B8: a2 = g W2^T + b2  ->  du = (da2 W2) * gelu'(u)      [dW2 = da2^T g deferred]
  RAF_TRY(gemm(prec, st, T, F, H, da, H, 1, wt ? wt_2 : w->w_2, wt ? H : F, wt ? 1 : 0, du, F, 0,
               prec == RAF_BF16_AMP ? EPI_MUL_AUX : EPI_MUL_GELU_GRAD, nullptr, u, F, d.gelu_tanh));
  // B7: u = ffn_in W1^T + b1  ->  db1 ; dffn = du W1          [dW1 = du^T ffn_in deferred]
  cj[0] = ColsumJob{prec, du, T, F, F, (float*)grads->b_1, (float*)at(scratch, p.partial_cs[0]), 0};
  RAF_TRY(gemm(prec, st, T, H, F, du, F, 1, wt ? wt_1 : w->w_1, wt ? F : H, wt ? 1 : 0, dffn, H));
  // B6: the LayerNorm between the two halves, the residual, dropout site 2
  if (d.pre_ln)   // ffn_in = LN2(z1); dz1 = dy + LN2'(dffn); da1 = dz1 * keep2/(1-p)
    RAF_TRY(launch_ln_bwd(d, 2, T, dffn, nullptr, z1, mu2, rstd2, (const float*)w->ln2_g, dy, dz1, da1,
                          (float*)grads->ln2_g, (float*)grads->ln2_b, (float*)grads->b_o, partial_ln[1], step, st, 0,
                          &rj[nr++]));
  else            // ffn_in = LN1(z1) feeds the ffn and the residual: g_in = dz2 + dffn
    RAF_TRY(launch_ln_bwd(d, 2, T, dz2, dffn, z1, mu1, rstd1, (const float*)w->ln1_g, nullptr, dz1, da1,
                          (float*)grads->ln1_g, (float*)grads->ln1_b, (float*)grads->b_o, partial_ln[1], step, st, 0,
                          &rj[nr++]));
  // B5: a1 = c Wo^T + bo  ->  dc = da1 Wo                   [dWo = da1^T c deferred]
  RAF_TRY(gemm(prec, st, T, H, H, da1, H, 1, wt ? wt_o : w->w_o, H, wt ? 1 : 0, dc, H));
  // B4, B3, B2: adjoint of the attention core; dQ, dK, dV are written to dqkv
  if (attn_fused_supported(d)) {
    // bf16, S <= 128: one kernel; probabilities and dropout mask recomputed from qkv, seq_lens and the step counter
    RAF_TRY(launch_attn_bwd_full(d, dc, qkv, seq_lens, dqkv, step, st));
  } else if (attn_flash_supported(d)) {
    // bf16, longer rows: the same from the row statistics of the forward pass, 128 keys / queries at a time
    RAF_TRY(launch_attn_flash_bwd(d, dc, qkv, c, (const float*)at(saved, p.lse), seq_lens, dqkv,
                                  (float*)at(scratch, p.dvec), step, st));
  } else {   // fp32
    // B4: c = prob_d V  ->  dV = prob_d^T dc ; dprob_d = dc V^T
    RAF_TRY(gemm_heads(p, prec, st, S, S, 64, HeadView{dc, H, 1, false},
                       HeadView{at(qkv, (size_t)2 * H * e), 3 * H, 1, false}, dprob_d, S, true, 1.0f));
    RAF_TRY(gemm_heads(p, prec, st, S, 64, S, HeadView{prob_d, S, 0, true}, HeadView{dc, H, 0, false},
                       at(dqkv, (size_t)2 * H * e), 3 * H, false, 1.0f));
    // B3: softmax + dropout adjoint, with the 1/8 of the score scaling folded in
    RAF_TRY(launch_softmax_bwd(d, prob, prob_d, dprob_d, ds, alpha, st));
    // B2: s = Q K^T / 8  ->  dQ = ds K ; dK = ds^T Q
    RAF_TRY(gemm_heads(p, prec, st, S, 64, S, HeadView{ds, S, 1, true},
                       HeadView{at(qkv, (size_t)H * e), 3 * H, 0, false}, dqkv, 3 * H, false, 1.0f));
    RAF_TRY(gemm_heads(p, prec, st, S, 64, S, HeadView{ds, S, 0, true}, HeadView{qkv, 3 * H, 0, false},
                       at(dqkv, (size_t)H * e), 3 * H, false, 1.0f));
  }
  // B1: qkv = attn_in Wqkv^T + bqkv
  cj[1] = ColsumJob{prec, dqkv, T, 3 * H, 3 * H, (float*)grads->b_qkv, (float*)at(scratch, p.partial_cs[1]), 0};
  if (d.pre_ln) {
    RAF_TRY(gemm(prec, st, T, H, 3 * H, dqkv, 3 * H, 1, wt ? wt_qkv : w->w_qkv, wt ? 3 * H : H, wt ? 1 : 0, dattn, H));
    // attn_in = LN1(x); dx = dz1 + LN1'(dattn)
    RAF_TRY(launch_ln_bwd(d, 0, T, dattn, nullptr, x, mu1, rstd1, (const float*)w->ln1_g, dz1, dx, nullptr,
                          (float*)grads->ln1_g, (float*)grads->ln1_b, nullptr, partial_ln[2], step, st, 0, &rj[nr++]));
  } else {
    // dx = dz1 + dqkv Wqkv (residual add in the epilogue)
    RAF_TRY(gemm(prec, st, T, H, 3 * H, dqkv, 3 * H, 1, wt ? wt_qkv : w->w_qkv, wt ? 3 * H : H, wt ? 1 : 0, dx, H, 0,
                 EPI_ADD_RES, nullptr, dz1, H));
  }
  // dW2 = da2^T g ; dW1 = du^T ffn_in ; dWqkv = dqkv^T attn_in ; dWo = da1^T c   (float outputs)
  GemmArgs wg[4];
  wg[0] = wgrad_args(H, F, T, da, H, g, F, grads->w_2, F);
  wg[1] = wgrad_args(F, H, T, du, F, ffn_in, H, grads->w_1, H);
  wg[2] = wgrad_args(3 * H, H, T, dqkv, 3 * H, d.pre_ln ? n1 : x, H, grads->w_qkv, H);
  wg[3] = wgrad_args(H, H, T, da1, H, c, H, grads->w_o, H);
  // db1 = column sums of du, dbqkv = column sums of dqkv (both still intact) and every deferred reduction: taken
  // inside the weight-gradient launch when its tiles leave CUs idle, else by their own two launches
  bool side_taken = false;
  RAF_TRY(launch_gemm_group_wgrad(prec, wg, 4, st, cj, 2, rj, nr, &side_taken));
  if (side_taken) return RAF_OK;
  RAF_TRY(launch_colsum_group(cj, 2, rj, &nr, st));
  return launch_reduce_group(rj, nr, st);
}

// ------------------------------------------------------ single operators --
extern "C" raf_status raf_op_gemm(int32_t precision, int32_t M, int32_t N, int32_t K, const void* a, int32_t lda,
                                  int32_t a_kmajor, const void* b, int32_t ldb, int32_t b_kmajor, void* c,
                                  int32_t ldc, int32_t out_f32, float alpha, int32_t epilogue, const float* bias,
                                  void* aux, int32_t gelu_tanh, void* hip_stream) {
  if (precision != RAF_F32 && precision != RAF_BF16_AMP) return RAF_EINVAL;
  GemmArgs g = gemm_args_default();
  g.M = M; g.N = N; g.K = K;
  g.a = a; g.lda = lda; g.a_kmajor = a_kmajor ? 1 : 0;
  g.b = b; g.ldb = ldb; g.b_kmajor = b_kmajor ? 1 : 0;
  g.c = c; g.ldc = ldc; g.out_f32 = out_f32 ? 1 : 0;
  g.alpha = alpha; g.epilogue = epilogue; g.bias = bias; g.aux = aux; g.ldaux = ldc; g.gelu_tanh = gelu_tanh ? 1 : 0;
  if (aux && !aligned16(aux)) return RAF_EINVAL;
  return launch_gemm(precision, g, (hipStream_t)hip_stream);
}

extern "C" raf_status raf_op_softmax_fwd(const raf_layer_desc* desc, const void* s, const int32_t* seq_lens,
                                         void* prob, void* prob_d, uint64_t step, void* hip_stream) {
  RAF_TRY(validate_desc(desc));
  return launch_softmax_fwd(*desc, s, seq_lens, prob, prob_d, step, (hipStream_t)hip_stream);
}

extern "C" raf_status raf_op_attention_fwd(const raf_layer_desc* desc, const void* qkv, const int32_t* seq_lens,
                                           void* ctx, float* lse, uint64_t step, void* hip_stream) {
  RAF_TRY(validate_desc(desc));
  if (!qkv || !ctx || !aligned16(qkv) || !aligned16(ctx) || !aligned16(lse)) return RAF_EINVAL;
  if (attn_fused_supported(*desc)) return launch_attn_fwd_fused(*desc, qkv, seq_lens, ctx, step, (hipStream_t)hip_stream);
  if (attn_flash_supported(*desc))
    return launch_attn_flash_fwd(*desc, qkv, seq_lens, ctx, lse, step, (hipStream_t)hip_stream);
  return RAF_ENOTSUP;
}

extern "C" raf_status raf_op_attention_bwd(const raf_layer_desc* desc, const void* dctx, const void* qkv,
                                           const void* ctx, const float* lse, const int32_t* seq_lens, void* dqkv,
                                           float* dvec, uint64_t step, void* hip_stream) {
  RAF_TRY(validate_desc(desc));
  if (!dctx || !qkv || !dqkv || !aligned16(dctx) || !aligned16(qkv) || !aligned16(dqkv) || !aligned16(ctx) ||
      !aligned16(lse) || !aligned16(dvec))
    return RAF_EINVAL;
  if (attn_fused_supported(*desc))
    return launch_attn_bwd_full(*desc, dctx, qkv, seq_lens, dqkv, step, (hipStream_t)hip_stream);
  if (attn_flash_supported(*desc))
    return launch_attn_flash_bwd(*desc, dctx, qkv, ctx, lse, seq_lens, dqkv, dvec, step, (hipStream_t)hip_stream);
  return RAF_ENOTSUP;
}

extern "C" raf_status raf_op_softmax_bwd(const raf_layer_desc* desc, const void* prob, const void* prob_d,
                                         const void* dprob_d, void* ds, float scale_out, void* hip_stream) {
  RAF_TRY(validate_desc(desc));
  return launch_softmax_bwd(*desc, prob, prob_d, dprob_d, ds, scale_out, (hipStream_t)hip_stream);
}

extern "C" raf_status raf_op_dropout_residual_ln_fwd(const raf_layer_desc* desc, int32_t site, int64_t rows,
                                                     const void* a, const void* res, const float* gamma,
                                                     const float* beta, void* out, void* z_out, float* mu,
                                                     float* rstd, uint64_t step, void* hip_stream) {
  RAF_TRY(validate_desc(desc));
  return launch_ln_fwd(*desc, site, rows, a, res, gamma, beta, out, z_out, mu, rstd, step, (hipStream_t)hip_stream);
}

extern "C" size_t raf_op_ln_bwd_partial_floats(int32_t hidden, int64_t rows) {
  if (hidden < 32 || hidden > 4096 || (hidden % 8)) return 0;
  return ln_bwd_partial_floats(hidden, rows);
}

extern "C" raf_status raf_op_dropout_residual_ln_bwd(const raf_layer_desc* desc, int32_t site, int64_t rows,
                                                     const void* dout, const void* dout2, const void* z,
                                                     const float* mu, const float* rstd, const float* gamma,
                                                     const void* dres, void* dz, void* da, float* dgamma,
                                                     float* dbeta, float* dbias, float* partial, uint64_t step,
                                                     void* hip_stream) {
  RAF_TRY(validate_desc(desc));
  return launch_ln_bwd(*desc, site, rows, dout, dout2, z, mu, rstd, gamma, dres, dz, da, dgamma, dbeta, dbias, partial,
                       step, (hipStream_t)hip_stream);
}

extern "C" const char* raf_status_string(raf_status s) {
  switch (s) {
    case RAF_OK: return "ok";
    case RAF_EINVAL: return "invalid argument";
    case RAF_ENOTSUP: return "unsupported shape or mode";
    case RAF_EWORKSPACE: return "workspace too small";
    case RAF_EHIP: return "HIP error";
  }
  return "unknown status";
}

extern "C" const char* raf_last_hip_error(void) {
  static thread_local std::string copy;
  std::lock_guard<std::mutex> lk(g_err_mutex);
  copy = g_err;
  return copy.c_str();
}

extern "C" const char* raf_version(void) { return "raf_mi355 0.1 gfx950"; }
