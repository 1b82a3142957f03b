/*
 * raf_mi355.h - C ABI of the single-GPU mixed-precision training step of one
 * transformer layer on MI355X (gfx950): forward, backward, fused Adam.
 *
 * What the calls compute follows the paper (RAF, arXiv 2303.04759):
 *   - a training workload is forward graph + loss + backward graph + optimizer
 *     over learnable parameters (Section 2.1, Fig. "Deep learning training
 *     workload");
 *   - the backward graph is the chain of adjoints of the forward operators
 *     (Section 3.1.1);
 *   - mixed precision keeps numerically sensitive operators in full precision
 *     and fuses every cast into its consumer (Section 3.1.2);
 *   - the optimizer is part of the step and updates parameters in place
 *     (Section 3, graph-generation phase);
 *   - elementwise / reduction operators are fused into their producers or with
 *     each other (Section 3.2.2).
 * The forward model is the only model input and the training graph is derived
 * from it (Section 1); here the forward model is the plain-data descriptor below.
 *
 * General conventions (all entry points)
 *   - Every pointer marked [dev] is device memory owned by the caller; the
 *     library never allocates, frees or synchronises, and keeps no pointer
 *     after a call returns.  [host] pointers are read during the call only.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream).  Calls are asynchronous; they are safe to
 *     record into a HIP graph (no memset/memcpy nodes are issued).  Scalar
 *     arguments (the dropout `step`, Adam's `t`, lr, loss_scale) are host values
 *     frozen into the recorded launches: a replay repeats the same dropout masks
 *     and bias corrections.  Only the *_scaled entry points, which read t and the
 *     loss scale from a raf_scaler_state on the device, advance across replays.
 *   - Tensors are dense, row-major, 16-byte aligned (else RAF_EINVAL).
 *   - "compute dtype" is float in RAF_F32 mode and bfloat16 (round to nearest
 *     even) in RAF_BF16_AMP mode.  Vectors (biases, LayerNorm gamma/beta),
 *     gradients, optimizer state and all statistics are always float.
 *   - No C++ exception crosses the ABI; every call returns a raf_status.
 *     After RAF_EHIP, raf_last_hip_error() names the HIP error.
 *   - Supported shapes: hidden/heads == 64; seq, hidden, ffn multiples of 32;
 *     seq <= 4096, hidden <= 4096; 0 <= dropout_p < 1.  Others: RAF_ENOTSUP.
 *   - Calls on different streams may overlap only if their buffers differ.
 */
#ifndef RAF_MI355_H
#define RAF_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  RAF_OK = 0,
  RAF_EINVAL = -1,     /* null / misaligned pointer, bad field value            */
  RAF_ENOTSUP = -2,    /* well-formed but outside the supported shapes          */
  RAF_EWORKSPACE = -3, /* an output capacity given by the caller is too small      */
  RAF_EHIP = -4        /* a HIP launch failed; see raf_last_hip_error()         */
} raf_status;

typedef enum { RAF_F32 = 0, RAF_BF16_AMP = 1 } raf_precision;

/* The forward model: one transformer layer (plain data, no pointers).
 *   post-LN (pre_ln=0):  h1 = LN1(x + drop2(attn(x)));  y = LN2(h1 + drop3(ffn(h1)))
 *   pre-LN  (pre_ln=1):  h  = x + drop2(attn(LN1(x)));  y = h + drop3(ffn(LN2(h)))
 * attn = out_proj(merge_heads(drop1(softmax(mask(Q K^T / 8))) V)), ffn = W2 gelu(W1 . + b1) + b2.
 * Dropout sites: 1 = attention probabilities [B,heads,S,S], 2 = attention
 * output [T,H], 3 = ffn output [T,H]; element idx of a site is kept iff the
 * 16-bit half (idx & 1: 0 = low, 1 = high) of word ((idx>>1) & 3) of
 * Philox4x32-10(counter = (idx>>3, step>>32, site | layer_id<<8,
 * step & 0xffffffff), key = (seed lo, seed hi)) is >= floor(dropout_p * 2^16);
 * kept values are scaled by 1/(1-dropout_p). */
typedef struct {
  int32_t batch, seq, hidden, heads, ffn;
  int32_t pre_ln;    /* 0 = post-LN (BERT style), 1 = pre-LN (GPT style)                 */
  int32_t causal;    /* 1: key j > query i is masked (in addition to padding)            */
  int32_t gelu_tanh; /* 0 = erf GeLU, 1 = tanh approximation                             */
  int32_t precision; /* raf_precision                                                     */
  float ln_eps;      /* added to the biased variance                                      */
  double dropout_p;  /* [0,1); the keep threshold is floor(dropout_p * 2^16) in double    */
  uint64_t seed;     /* dropout key                                                       */
  uint32_t layer_id; /* folded into the dropout counter (24 bits used)                    */
  uint32_t remat;    /* OR of raf_remat_bits: tensors the forward pass does not keep      */
} raf_layer_desc;

/* Rematerialisation (Section 3.1.5): a tensor named here is not written to
 * `saved` by raf_layer_fwd; raf_layer_bwd regenerates it in scratch by replaying
 * the operator that produced it (same kernel, same inputs: bit-identical values,
 * so every output of the step is unchanged).  Which tensors to name under a byte
 * budget is what raf_remat_plan decides.
 *   RAF_REMAT_QKV   the [T,3H] output of the QKV projection (replay: that product)
 *   RAF_REMAT_CTX   the [T,H] attention context (replay: the attention forward
 *                   kernel; RAF_ENOTSUP where attention is not taken on chip, i.e. RAF_F32)
 *   RAF_REMAT_FFN1  the two [T,F] outputs of the first feed-forward product: the
 *                   activation and the second tensor kept with it for the
 *                   adjoint (replay: that product with its GeLU epilogue) */
typedef enum { RAF_REMAT_QKV = 1, RAF_REMAT_CTX = 2, RAF_REMAT_FFN1 = 4 } raf_remat_bits;

/* The twelve parameter tensors of a layer, or their gradients.
 * Shapes ([out,in] row-major for matrices): w_qkv [3H,H] (rows: Q block, K
 * block, V block), b_qkv [3H], w_o [H,H], b_o [H], ln1_g/ln1_b [H],
 * w_1 [F,H], b_1 [F], w_2 [H,F], b_2 [H], ln2_g/ln2_b [H].
 * As weights: w_* in compute dtype, all vectors float.  As gradients: all float.
 * wt_*: optional, read by raf_layer_bwd in RAF_BF16_AMP mode only (ignored
 * elsewhere, and in a gradient struct): bfloat16 transposed copies [in,out] of the
 * four matrices (wt_qkv [H,3H], wt_o [H,H], wt_1 [H,F], wt_2 [F,H]), which the
 * input-gradient products contract over.  All four non-NULL: they must hold exactly
 * the transposes of w_* (raf_adam_step keeps them so through raf_adam_tensor.lowp_t).
 * Any of them NULL: the backward pass forms the transposes itself in scratch.
 * nonfinite: optional, read in the gradient struct of raf_layer_bwd only: [dev] int32
 * (4-byte aligned) that the call sets to 1 if any of the twelve gradients it writes is
 * inf or nan, and leaves alone otherwise (the caller clears it; raf_scaler_state
 * .found_inf is such a flag).  Where the weight gradients and their reductions leave
 * in one launch the test rides in that launch's epilogues; other shapes take one
 * extra pass over the gradients. */
typedef struct {
  void *w_qkv, *b_qkv, *w_o, *b_o, *ln1_g, *ln1_b, *w_1, *b_1, *w_2, *b_2, *ln2_g, *ln2_b;
  void *wt_qkv, *wt_o, *wt_1, *wt_2;
  void *nonfinite;
} raf_layer_tensors;

/* Sizes in bytes of the two caller-provided buffers of a layer.
 * `saved` carries activations from raf_layer_fwd to raf_layer_bwd of the same
 * step (opaque layout); `scratch` is dead outside a call and may be shared by
 * all layers on one stream.  Both sizes are multiples of 256. */
raf_status raf_layer_workspace(const raf_layer_desc *desc /*host*/, size_t *saved_bytes /*host out*/,
                               size_t *scratch_bytes /*host out*/);

/* Forward pass (Section 2.1 "forward graph"; fused operators per Section 3.2.2).
 *   w        [host struct of dev pointers] weights, see raf_layer_tensors
 *   x        [dev] input  [B*S, H], compute dtype
 *   seq_lens [dev] int32 [B], valid keys per sequence (key j >= len is masked,
 *            probability exactly 0; a row with no admissible key gives zeros);
 *            NULL = all sequences full length
 *   y        [dev] output [B*S, H], compute dtype
 *   saved    [dev] >= saved_bytes,  written
 *   scratch  [dev] >= scratch_bytes, clobbered
 *   step     dropout step counter (use the optimizer step) */
raf_status raf_layer_fwd(const raf_layer_desc *desc, const raf_layer_tensors *w, const void *x,
                         const int32_t *seq_lens, void *y, void *saved, void *scratch, uint64_t step,
                         void *hip_stream);

/* Backward pass: adjoints of the forward operators in reverse order (Section
 * 3.1.1), dropout masks recomputed from the counter, not stored (one exception:
 * with seq > 128 the forward pass leaves the keep decisions of the attention
 * probabilities in saved, one bit each: the two attention adjoint kernels of
 * that path would each run the generator again over all seq x seq scores).
 *   x, seq_lens, saved, step: exactly what the matching raf_layer_fwd saw/wrote
 *   dy     [dev] gradient w.r.t. y [B*S,H], compute dtype (already loss-scaled)
 *   dx     [dev] gradient w.r.t. x [B*S,H], compute dtype, overwritten
 *   grads  [host struct of dev pointers] twelve float tensors, OVERWRITTEN
 *          with the (loss-scaled) gradients; no accumulation across calls */
raf_status raf_layer_bwd(const raf_layer_desc *desc, const raf_layer_tensors *w, const void *x, const void *dy,
                         const int32_t *seq_lens, const void *saved, void *dx, raf_layer_tensors *grads,
                         void *scratch, uint64_t step, void *hip_stream);

/* Loss seed of the benchmark workload: loss = sum(y * G) (float accumulate,
 * deterministic), dy = loss_scale * G in compute dtype.
 *   y, G [dev] [n] compute dtype; loss_out [dev] one float; dy [dev] [n];
 *   partial [dev] float[RAF_LOSS_PARTIALS] scratch.  n must be a multiple of 8. */
#define RAF_LOSS_PARTIALS 1024
raf_status raf_loss_seed(int32_t precision, const void *y, const void *G, int64_t n, float loss_scale,
                         float *loss_out, void *dy, float *partial, void *hip_stream);

/* One tensor of the optimizer's list.  master/grad/m/v: [dev] float[n];
 * lowp: [dev] bfloat16[n] copy of the updated master (the AMP cast fused into
 * the producer, Section 3.1.2), or NULL.  n >= 0; pointers 16-byte aligned.
 * lowp_t: [dev] bfloat16 [cols, rows], or NULL: a second copy of the updated master,
 * transposed, the tensor being viewed as a [rows, cols] row-major matrix
 * (rows * cols == n, both multiples of 8, else RAF_EINVAL): the operand layout the
 * input-gradient products of raf_layer_bwd want (raf_layer_tensors.wt_*), written by
 * the optimizer so that no transpose pass runs in the backward pass.  rows and cols
 * are ignored when lowp_t is NULL. */
typedef struct {
  float *master;
  const float *grad;
  float *m;
  float *v;
  void *lowp;
  int64_t n;
  void *lowp_t;
  int32_t rows, cols;
} raf_adam_tensor;

/* Fused multi-tensor Adam (optimizer inside the step, in-place update; Section 3).
 * Per element: g = grad*inv_loss_scale (+ weight_decay*w); m = b1 m + (1-b1) g;
 * v = b2 v + (1-b2) g^2; w -= lr * (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps).
 *   list [host] array of `count` tensors (copied into kernel arguments);
 *   t is 1-based.  count == 0 is a no-op.  Hyper-parameters are doubles; the
 *   derived constants (1-b1, 1-b2, lr/(1-b1^t), 1/(1-b2^t)) are formed in double
 *   on the host and rounded once to float for the kernel. */
raf_status raf_adam_step(const raf_adam_tensor *list, int32_t count, double lr, double beta1, double beta2,
                         double eps, double weight_decay, int64_t t, double inv_loss_scale, void *hip_stream);

/* ---- Dynamic loss scaling with a non-finite skip (mixed precision applied by the
 * system, Section 3.1.2; the paper's float16 AMP runs of Section 5.1 need it).
 * The paper prints no rule; this is the standard one: the loss gradient is
 * multiplied by the scale; if any gradient of the step is non-finite the optimizer
 * step is skipped and the scale multiplied by backoff_factor, otherwise the step is
 * taken on gradients divided by the scale and after growth_interval consecutive
 * good steps the scale is multiplied by growth_factor.  Every decision is taken on
 * the device from this state, so a captured step replays correctly:
 *   raf_loss_seed_scaled -> raf_layer_bwd ... -> raf_grads_check ->
 *   raf_adam_step_scaled -> raf_scaler_update.
 * The state lives in device memory (16-byte aligned); read it back with a copy. */
typedef struct {
  float scale;          /* current loss scale                                   */
  float inv_scale;      /* 1/scale                                              */
  int32_t good_steps;   /* consecutive steps without a non-finite gradient      */
  int32_t found_inf;    /* set by raf_grads_check, cleared by raf_scaler_update */
  int64_t t;            /* optimizer steps taken so far (skipped ones excluded) */
  float lr_over_bc1;    /* reserved (kept for the 32-byte layout; not read or    */
  float inv_bc2;        /*   written by the present kernels)                     */
} raf_scaler_state;

/* state [dev] written: scale = init_scale (> 0, finite), counters zero. */
raf_status raf_scaler_init(raf_scaler_state *state, float init_scale, void *hip_stream);
/* raf_loss_seed with loss_scale read from state->scale on the device. */
raf_status raf_loss_seed_scaled(int32_t precision, const void *y, const void *G, int64_t n,
                                const raf_scaler_state *state, float *loss_out, void *dy, float *partial,
                                void *hip_stream);
/* raf_layer_fwd and raf_loss_seed in one call: the kernel that writes y also forms
 * dy = loss_scale * G and the partial sums of loss = sum(y * G) (y as stored), so the
 * loss (Section 2.1: part of the training graph) costs no pass of its own (fusion of an
 * elementwise + reduction operator into its producer, Section 3.2.2).  y and dy are
 * bit-identical to the two separate calls; the loss differs by the order of the float
 * summation only.  state == NULL: loss_scale is used; otherwise the scale is read from
 * the device-resident state (as raf_loss_seed_scaled does) and loss_scale is ignored.
 * The partial sums live in scratch. */
raf_status raf_layer_fwd_loss(const raf_layer_desc *desc, const raf_layer_tensors *w, const void *x,
                              const int32_t *seq_lens, void *y, const void *G, float loss_scale,
                              const raf_scaler_state *state, float *loss_out, void *dy, void *saved, void *scratch,
                              uint64_t step, void *hip_stream);

/* state->found_inf = 1 if any element of any list[i].grad is inf or nan (it is not cleared here). */
raf_status raf_grads_check(const raf_adam_tensor *list, int32_t count, raf_scaler_state *state, void *hip_stream);
/* raf_adam_step with t = state->t + 1 and inv_loss_scale = state->inv_scale, both read on the
 * device (the bias corrections 1 - beta^t are formed there in float as -expm1(t ln beta)); a
 * no-op on every tensor when state->found_inf is set. */
raf_status raf_adam_step_scaled(const raf_adam_tensor *list, int32_t count, double lr, double beta1, double beta2,
                                double eps, double weight_decay, raf_scaler_state *state, void *hip_stream);
/* The scale rule above; also advances state->t on a good step and clears found_inf.
 * growth_factor >= 1, 0 < backoff_factor <= 1, growth_interval >= 1. */
raf_status raf_scaler_update(raf_scaler_state *state, float growth_factor, float backoff_factor,
                             int32_t growth_interval, void *hip_stream);

/* The same update for lists of any length in ONE launch (the optimizer of a whole model
 * as one operator of the step, Section 3): raf_adam_step holds its tensor table in
 * the kernel arguments and splits lists of more than 48 tensors into several launches;
 * here the table lives in device memory.
 *   raf_adam_table_bytes(list, count): size of the caller's table buffer for this list
 *     (0 for a malformed list).
 *   raf_adam_table_fill: writes the table for `list` with small kernels on the stream
 *     (no copies, no allocation); once per list, again whenever a pointer changes.
 *     table [dev]: >= raf_adam_table_bytes(list, count) bytes, 256-byte aligned.
 *   raf_adam_step_table: one launch over all tensors.  list [host] must be the list the
 *     table was filled from (the launch geometry is recomputed from it).  state == NULL:
 *     t and inv_loss_scale as in raf_adam_step; otherwise both are read on the device
 *     as in raf_adam_step_scaled and the two arguments are ignored. */
size_t raf_adam_table_bytes(const raf_adam_tensor *list, int32_t count);
raf_status raf_adam_table_fill(const raf_adam_tensor *list, int32_t count, void *table, void *hip_stream);
raf_status raf_adam_step_table(const raf_adam_tensor *list, int32_t count, const void *table, double lr,
                               double beta1, double beta2, double eps, double weight_decay, int64_t t,
                               double inv_loss_scale, const raf_scaler_state *state, void *hip_stream);

/* Test hook: the keep-mask of one dropout site as bytes (1 = kept).
 *   mask_out [dev] uint8[n]; element order is the site's flat index. */
raf_status raf_debug_dropout_mask(const raf_layer_desc *desc, int32_t site, uint64_t step, uint8_t *mask_out,
                                  int64_t n, void *hip_stream);

/* ---- whole-model pieces around the layer stack (largest workload): token +
 * position embedding with LayerNorm and dropout, and the masked-language-model
 * head with a decoder tied to the word table and a summed softmax
 * cross-entropy.  Same composition rule as the layer (Section 2.1) and the same
 * fusion / precision policy (Sections 3.1.2, 3.2.2).
 *
 * The word table is stored with vocab_pad = vocab rounded up to a multiple of 32
 * rows; rows >= vocab must be zero (they take part in padded GEMM tiles with a
 * zero coefficient).  Its gradient has the same vocab_pad rows. */
typedef struct {
  int32_t batch, seq, hidden, vocab, max_pos;
  int32_t precision; /* raf_precision */
  float ln_eps;
  uint32_t layer_id; /* dropout counter id of the embedding (site 4) */
  double dropout_p;
  uint64_t seed;
} raf_embed_desc;

raf_status raf_embed_workspace(const raf_embed_desc *desc, size_t *saved_bytes, size_t *scratch_bytes);

/* x0 = dropout_site4(LayerNorm(word[ids] + pos[position])).
 *   ids [dev] int32 [B*S] in [0,vocab); word [dev] [vocab_pad,H] and pos [dev]
 *   [max_pos,H] in compute dtype; gamma/beta [dev] float [H]; x0 [dev] [B*S,H]
 *   compute dtype; saved [dev] >= saved_bytes (written). */
raf_status raf_embed_fwd(const raf_embed_desc *desc, const int32_t *ids, const void *word, const void *pos,
                         const float *gamma, const float *beta, void *x0, void *saved, uint64_t step,
                         void *hip_stream);

/* Adjoint.  dx0 [dev] [B*S,H] compute dtype.  dword [dev] float [vocab_pad,H]:
 * the embedding's contribution is ADDED to what is there (call after
 * raf_mlm_head_fwd_bwd, which overwrites it with the tied decoder's gradient);
 * rows with the same id are summed in ascending position order, so the result
 * is reproducible.  dpos [dev] float [max_pos,H], dgamma/dbeta [dev] float [H]:
 * overwritten. */
raf_status raf_embed_bwd(const raf_embed_desc *desc, const int32_t *ids, const void *dx0, const void *saved,
                         const float *gamma, float *dword, float *dpos, float *dgamma, float *dbeta, void *scratch,
                         uint64_t step, void *hip_stream);

typedef struct {
  int32_t rows;      /* B*S rows of the final hidden state                      */
  int32_t hidden, vocab;
  int32_t n_sel;     /* number of selected (masked) positions, >= 1             */
  int32_t precision; /* raf_precision */
  int32_t gelu_tanh;
  float ln_eps;      /* > 0 (RAF_EINVAL otherwise): the selected rows are padded to the
                        tile height with rows of zero variance                     */
  int32_t reserved;  /* must be 0 */
} raf_mlm_desc;

/* head_w [H,H] and word [vocab_pad,H] in compute dtype as weights; everything
 * else float.  As gradients: all float, word with vocab_pad rows. */
typedef struct {
  void *head_w, *head_b, *ln_g, *ln_b, *word, *dec_b;
} raf_mlm_tensors;

raf_status raf_mlm_workspace(const raf_mlm_desc *desc, size_t *scratch_bytes);

/* Forward and backward of the head in one call:
 *   r = x[sel]; t = LN(gelu(r head_w^T + head_b)); logits = t word^T + dec_b;
 *   loss = sum_i (logsumexp(logits_i) - logits_i[labels_i]);
 *   gradients of loss_scale * loss.
 *   x [dev] [rows,H] compute dtype; sel [dev] int32 [n_sel] flat row indices,
 *   strictly ascending; labels [dev] int32 [n_sel] in [0,vocab).
 *   loss_out [dev] one float (unscaled loss); dx [dev] [rows,H] compute dtype,
 *   fully overwritten (zero on unselected rows); grads overwritten. */
raf_status raf_mlm_head_fwd_bwd(const raf_mlm_desc *desc, const raf_mlm_tensors *w, const void *x,
                                const int32_t *sel, const int32_t *labels, float loss_scale, float *loss_out,
                                void *dx, raf_mlm_tensors *grads, void *scratch, void *hip_stream);

/* ---- single fused operators, exported for per-kernel parity tests and
 * per-kernel roofline measurement; the layer calls above use the same kernels. */

/* C[M,N] = epilogue(alpha * A.B) on the MFMA (bf16) or FMA (f32) GEMM kernel.
 * a_kmajor=1: A element (i,k) at a[i*lda+k]; 0: at a[k*lda+i].
 * b_kmajor=1: B element (k,j) at b[j*ldb+k]; 0: at b[k*ldb+j].
 * epilogue: 0 none, 1 +bias[j], 2 +bias then GeLU (pre-activation stored to
 * aux, same shape/ld as C), 3 multiply by gelu'(aux[i,j]), 4 +residual aux[i,j],
 * 5 +bias then GeLU with gelu'(pre-activation) stored to aux, 6 multiply by aux[i,j]
 * (5 and 6 are the forward / backward pair the bf16 layer uses).
 * out_f32=1 stores C as float regardless of precision. M,N,K multiples of 32. */
raf_status raf_op_gemm(int32_t precision, int32_t M, int32_t N, int32_t K, const void *a, int32_t lda,
                       int32_t a_kmajor, const void *b, int32_t ldb, int32_t b_kmajor, void *c, int32_t ldc,
                       int32_t out_f32, float alpha, int32_t epilogue, const float *bias, void *aux,
                       int32_t gelu_tanh, void *hip_stream);

/* Masked softmax (+ dropout site 1) over the last axis of s [B,heads,S,S]:
 * writes prob (softmax) and prob_d (after dropout), both compute dtype. */
raf_status raf_op_softmax_fwd(const raf_layer_desc *desc, const void *s, const int32_t *seq_lens, void *prob,
                              void *prob_d, uint64_t step, void *hip_stream);
/* ds = scale_out * prob * (dprob - sum_j dprob*prob), dprob = dprob_d * keep/(1-p)
 * where keep is recovered as (prob_d != 0 or prob == 0). */
raf_status raf_op_softmax_bwd(const raf_layer_desc *desc, const void *prob, const void *prob_d,
                              const void *dprob_d, void *ds, float scale_out, void *hip_stream);

/* Attention core of the bf16 AMP path (precision must be RAF_BF16_AMP), all S x S
 * tensors kept on chip: ctx = merge_heads(dropout1(softmax(mask(Q K^T / 8))) V)
 * from qkv [B*S,3H] (column blocks Q | K | V, head h = columns 64h .. 64h+63).
 *   ctx [dev] [B*S,H] written; lse [dev] float[B*heads*S] written when
 *   seq > 128 (row statistic max + log2(sum) in base-2 score units that the
 *   backward call needs), ignored and may be NULL otherwise.
 *   keep [dev] raf_op_attention_keep_bytes(desc) bytes, 16-byte aligned, or NULL:
 *   written when given and seq > 128 and dropout_p > 0: the keep decisions of
 *   dropout site 1, one bit per score (16 bytes per query row and 128-key block;
 *   bit 8u + e of dword g = key 32u + 8g + e of the block), so that the backward
 *   call need not run the random number generator again. */
raf_status raf_op_attention_fwd(const raf_layer_desc *desc, const void *qkv, const int32_t *seq_lens, void *ctx,
                                float *lse, void *keep, uint64_t step, void *hip_stream);
/* Bytes of the keep buffer above; 0 where none is used (seq <= 128 or dropout_p == 0). */
size_t raf_op_attention_keep_bytes(const raf_layer_desc *desc);
/* Adjoint: dqkv [B*S,3H] (dQ | dK | dV) from dctx [B*S,H]; probabilities and
 * dropout mask are recomputed from qkv, seq_lens and step, which must be those of
 * the forward call.  seq > 128 also needs ctx and lse of the forward call and
 * dvec [dev] float[B*heads*S] scratch; they are ignored (may be NULL) otherwise.
 * keep: NULL (the dropout mask is generated again), or the buffer the forward call
 * wrote (the same results, bit for bit, without the generator). */
raf_status raf_op_attention_bwd(const raf_layer_desc *desc, const void *dctx, const void *qkv, const void *ctx,
                                const float *lse, const void *keep, const int32_t *seq_lens, void *dqkv, float *dvec,
                                uint64_t step, void *hip_stream);

/* z = res + dropout_site(a); out = LayerNorm(z) with float statistics.
 * a == NULL: z = res (plain LayerNorm).  gamma == NULL: no LayerNorm, out = z
 * (z_out, mu, rstd ignored).  site in {2,3}. rows*H elements, compute dtype. */
raf_status raf_op_dropout_residual_ln_fwd(const raf_layer_desc *desc, int32_t site, int64_t rows, const void *a,
                                          const void *res, const float *gamma, const float *beta, void *out,
                                          void *z_out, float *mu, float *rstd, uint64_t step, void *hip_stream);

/* Adjoint of the above.  g_in = dout (+ dout2 if not NULL).
 * gamma != NULL: dz = LN-backward(g_in; z, mu, rstd, gamma) (+ dres if not
 * NULL), dgamma/dbeta = column sums; gamma == NULL: dz = g_in.
 * site != 0: da = dz * keep_site/(1-p) and dbias = column sums of da.
 * partial: [dev] float scratch of raf_op_ln_bwd_partial_floats(H) floats. */
size_t raf_op_ln_bwd_partial_floats(int32_t hidden, int64_t rows);
raf_status raf_op_dropout_residual_ln_bwd(const raf_layer_desc *desc, int32_t site, int64_t rows, const void *dout,
                                          const void *dout2, const void *z, const float *mu, const float *rstd,
                                          const float *gamma, const void *dres, void *dz, void *da, float *dgamma,
                                          float *dbeta, float *dbias, float *partial, uint64_t step,
                                          void *hip_stream);

/* The same operator for callers that cannot allocate device memory (code under HIP
 * graph capture, serving loops and harnesses that forbid hipMalloc): identical to
 * raf_op_dropout_residual_ln_bwd except that the partial-sum buffer is a device array
 * inside the library, RAF_NOALLOC_LN_BWD_PARTIAL_FLOATS floats (3 MiB) per GPU, held
 * until the process ends.  Same kernels, bit-identical results.  The call allocates
 * nothing.  RAF_EWORKSPACE when raf_op_ln_bwd_partial_floats(hidden, rows) exceeds
 * that size (with the present kernels it holds hidden = 768 up to 5456 rows and hidden
 * = 1024 up to 4096 rows); nothing is launched then.  All
 * calls on one GPU share the array: calls that overlap on one GPU (different streams
 * or host threads) race and must be serialised by the caller; calls in stream order
 * need no clearing in between.  The first call on a device looks the array up (it may
 * load the code object): make it outside a graph capture. */
#define RAF_NOALLOC_LN_BWD_PARTIAL_FLOATS (256 * 3 * 1024)
raf_status raf_op_dropout_residual_ln_bwd_noalloc(const raf_layer_desc *desc, int32_t site, int64_t rows,
                                                  const void *dout, const void *dout2, const void *z,
                                                  const float *mu, const float *rstd, const float *gamma,
                                                  const void *dres, void *dz, void *da, float *dgamma, float *dbeta,
                                                  float *dbias, uint64_t step, void *hip_stream);

/* ---- Memory passes on an operator list (host only, no GPU work; Sections 3.1.4
 * "operator scheduling" and 3.1.5 "rematerialization").  The paper names the
 * ingredients and prints no formulas; the rules used are stated with each call.
 *
 * An operator list in execution order, in CSR form.  A tensor has at most one
 * producer and must be produced before its first reader; a tensor that no operator
 * produces is external (parameters, inputs) and counts as resident throughout.
 * Duplicate ids inside one operator's list count once.  All arrays are host memory,
 * read only, owned by the caller. */
typedef enum { RAF_TENSOR_REMAT_OK = 1, RAF_TENSOR_PERSISTENT = 2 } raf_tensor_flags;
typedef struct {
  int32_t n_ops, n_tensors;
  const int32_t *in_begin;  /* [n_ops+1] offsets into in_ids: tensors op k reads        */
  const int32_t *in_ids;
  const int32_t *out_begin; /* [n_ops+1] offsets into out_ids: tensors op k writes      */
  const int32_t *out_ids;
  const double *latency;    /* [n_ops] run time of the operator, any unit, >= 0          */
  const int64_t *bytes;     /* [n_tensors] >= 0                                          */
  const uint8_t *flags;     /* [n_tensors] raf_tensor_flags: REMAT_OK = an intermediate
                               that may be dropped and regenerated; PERSISTENT = must
                               outlive the list (a result)                               */
} raf_op_graph;

/* Liveness estimate: mem_out[p] = bytes of all tensors alive while item p of the
 * sequence runs (its inputs and outputs included).  A tensor is alive from the item
 * that writes it to the last item that reads it before it is written again.
 *   sequence: item k >= 0 runs operator k; item -1-t replays the producer of tensor
 *   t and regenerates t alone.  NULL = operators 0..n_ops-1 in order (seq_len unused).
 * RAF_EINVAL for a malformed graph or a sequence that reads a tensor before it exists. */
raf_status raf_memory_profile(const raf_op_graph *graph, const int32_t *sequence, int32_t seq_len,
                              int64_t *mem_out /* [seq_len or n_ops] */);

/* Operator scheduling (Section 3.1.4): with p the bytes an operator produces and c
 * the bytes that can be released once it has run, operators with p - c < 0 move
 * forward and those with p - c > 0 backward.  Taken as list scheduling: of the
 * operators whose inputs exist, the one with the smallest p - c runs next (ties in
 * the given order).  c counts the inputs whose other readers have all run, and
 * outputs that nothing reads (unless PERSISTENT).  The list only has to be acyclic
 * here (RAF_EINVAL otherwise).  order_out [n_ops]: a permutation of the operators
 * that respects every dependence. */
raf_status raf_schedule_ops(const raf_op_graph *graph, int32_t *order_out);

typedef struct {
  int64_t peak_before;  /* liveness estimate of the given order                            */
  int64_t peak_after;   /* of the sequence with replays                                    */
  int32_t fits;         /* 1 if every point is within the budget                           */
  int32_t reserved;
  double extra_latency; /* sum of the replayed operators' latencies                        */
} raf_remat_summary;

/* Rematerialisation (Section 3.1.5): the order is walked once; where the liveness
 * estimate exceeds budget_bytes, alive intermediates are dropped in ascending cost
 *   latency(producer) * (readers still to come) / bytes     (ties: larger, lower id)
 * and a replay of the producer is placed directly in front of the next reader, until
 * the point fits or nothing qualifies.  A tensor qualifies if it is REMAT_OK, the
 * current item neither reads nor writes it, its next reader is not the very next
 * item, and every input of its producer is still alive where the replay goes (one
 * operator is replayed, never a chain).
 *   sequence_out [sequence_cap], *sequence_len: the order with replays (item coding
 *     as in raf_memory_profile); evicted_tensor/evicted_pos [evicted_cap], *n_evicted:
 *     which tensor was dropped at which position of the final sequence.
 * RAF_EWORKSPACE if a capacity is too small (the needed lengths and the summary are
 * still written; 9*n_ops+8 items always suffice). */
raf_status raf_remat_plan(const raf_op_graph *graph, int64_t budget_bytes, int32_t *sequence_out,
                          int32_t sequence_cap, int32_t *sequence_len, int32_t *evicted_tensor,
                          int32_t *evicted_pos, int32_t evicted_cap, int32_t *n_evicted,
                          raf_remat_summary *summary);

/* The operator list of `layers` identical layers run forward, a loss seed, and
 * backward (the kernels of raf_layer_fwd / raf_layer_bwd in launch order, the grouped
 * weight-gradient launch last in each layer), activations only: parameters,
 * gradients and optimizer state are outside this budget.  Tensors that raf_layer_desc
 * .remat can drop carry REMAT_OK, with owner_layer / owner_bit naming layer and bit
 * (else -1 / 0); the context qualifies only where attention runs on chip.
 *   replay_us [3] or NULL: measured run times of the QKV product, the attention
 *   forward kernel and the first feed-forward product; NULL = an estimate from the
 *   operation counts (800 TFLOP/s, 4 TB/s).
 * 1 <= layers <= 512 (the planner's run time grows with the cube of the list length).
 * Two-call protocol: with in_begin == NULL only sizes->n_ops, sizes->n_tensors,
 * *n_in_ids and *n_out_ids are written; then call again with arrays of those sizes
 * (in_begin/out_begin n_ops+1). */
raf_status raf_layer_stack_graph(const raf_layer_desc *desc, int32_t layers, const double *replay_us,
                                 raf_op_graph *sizes, int32_t *in_begin, int32_t *in_ids, int32_t *out_begin,
                                 int32_t *out_ids, double *latency, int64_t *bytes, uint8_t *flags,
                                 int32_t *owner_layer, int32_t *owner_bit, int32_t *n_in_ids, int32_t *n_out_ids);

/* raf_remat_plan on that list: remat_out [layers] receives the raf_layer_desc.remat
 * value of every layer under an activation budget of budget_bytes.  The kernels
 * replay a dropped tensor at the start of the layer's backward call rather than in
 * front of its reader; replayed tensors sit in the scratch buffer all layers share,
 * so the peak is not affected. */
raf_status raf_layer_stack_remat(const raf_layer_desc *desc, int32_t layers, int64_t budget_bytes,
                                 const double *replay_us, uint32_t *remat_out, raf_remat_summary *summary);

const char *raf_status_string(raf_status s);
const char *raf_last_hip_error(void);
/* Library version string, e.g. "raf_mi355 0.1 gfx950". */
const char *raf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RAF_MI355_H */
