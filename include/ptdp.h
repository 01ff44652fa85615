/*
 * ptdp.h - C ABI of the per-GPU compute path of PTD-P training
 * (Narayanan et al., "Efficient Large-Scale Language Model Training on GPU
 * Clusters Using Megatron-LM", arXiv 2104.04473) for AMD MI355X (gfx950).
 *
 * What the library computes: forward and backward of GPT transformer layers
 * on ONE pipeline stage holding ONE tensor-parallel shard (paper sections 2.2
 * and 2.3), for one microbatch at a time, plus the order in which one device
 * of an (interleaved) 1F1B pipeline runs those passes over its model chunks.
 * Communication between devices is not part of this library: on a single
 * shard the conjugate all-reduce operators f and g of section 2.3 are the
 * identity.
 *
 * Notation (paper section 3.1 and section 5.1): t tensor-parallel degree,
 * h hidden size, a attention heads, s sequence length, b microbatch size,
 * p pipeline stages, v model chunks per device, m microbatches per batch.
 * Derived: dh = h/a, hp = h/t (width of the local heads), fp = 4h/t,
 * T = s*b tokens.
 *
 * General conventions
 *  - Every function returns PTDP_OK (0) or a negative PTDP_E_* code; nothing
 *    throws or aborts.  All argument checks happen before any device work.
 *  - "dev" pointers are device (HBM) addresses, "host" pointers host addresses.
 *    All device memory is owned by the caller; the library borrows it for the
 *    duration of the enqueued work and never allocates device memory.
 *  - All device work is enqueued on the caller's HIP stream (`stream` is a
 *    hipStream_t passed as void*; NULL = the null stream) and the call returns
 *    without synchronising.
 *  - Activations are row-major [s, b, width] (section 4.2), i.e. a [T, width]
 *    matrix whose row index is si*b + bi.  Weights are row-major [in, out] so
 *    that Y = X A (section 2.3).  The columns of w_qkv are ordered
 *    [Q of all local heads | K | V], each head's dh columns contiguous.
 *  - dtype PTDP_F32: storage and arithmetic fp32.  dtype PTDP_BF16: parameters,
 *    activations and stash are bf16 (round-to-nearest-even), every reduction
 *    and accumulator is fp32, LayerNorm statistics and the attention
 *    log-sum-exp are fp32, parameter gradients are fp32.
 *  - Parameter gradients ACCUMULATE (+=) until the caller zeroes them: the
 *    optimizer steps only at the pipeline flush (section 2.2).
 *  - Device buffers must be 16-byte aligned; h, hp, fp and dh must be
 *    multiples of 8.
 *  - A ptdp_chunk may be used by one thread at a time; different chunks may be
 *    used from different threads (on streams of the device that is current in
 *    the calling thread).  Calls that share a workspace or stash must be
 *    ordered on one stream.
 */
#ifndef PTDP_H
#define PTDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#pragma GCC visibility push(default)
#endif

/* ------------------------------------------------------------------ status */
enum {
  PTDP_OK = 0,
  PTDP_E_INVALID_ARG = -1, /* a size or flag violates the documented limits   */
  PTDP_E_UNSUPPORTED = -2, /* valid in the paper's terms, not built here      */
  PTDP_E_NULL_PTR = -3,    /* a required pointer is NULL                      */
  PTDP_E_TOO_SMALL = -4,   /* an output array / capacity is too small         */
  PTDP_E_HIP = -5,         /* a HIP runtime call failed (launch, event, ...)  */
  PTDP_E_STATE = -6        /* object not ready (e.g. parameters not bound)    */
};
const char* ptdp_status_string(int status);

enum { PTDP_F32 = 0, PTDP_BF16 = 1 };
enum { PTDP_GELU_ERF = 0, PTDP_GELU_TANH = 1 };

/* --------------------------------------------------------------- structures */

/* One layer's shape on one shard.  struct_size must be sizeof(ptdp_layer_cfg). */
typedef struct ptdp_layer_cfg {
  uint32_t struct_size;
  int32_t h, a, t, s, b; /* full hidden, full heads, TP degree, sequence, microbatch */
  int32_t dtype;         /* PTDP_F32 or PTDP_BF16 */
  int32_t causal;        /* 1: implicit causal mask; 0: general mask, see ptdp_chunk_set_mask (section 4.2) */
  int32_t gelu_mode;     /* PTDP_GELU_ERF (default) or PTDP_GELU_TANH */
  float p_hidden;        /* dropout probability of the two bias+dropout+add sites, 0 <= p < 1 */
  float ln_eps;          /* LayerNorm epsilon (> 0) */
  uint64_t seed;         /* dropout seed */
} ptdp_layer_cfg;

/* Device pointers to one shard's parameters of one layer, in the storage dtype.
 * Shapes: ln*_g, ln*_b, b_o, b_2 [h]; w_qkv [h, 3hp]; b_qkv [3hp]; w_o [hp, h];
 * w_1 [h, fp]; b_1 [fp]; w_2 [fp, h].  That all four linear maps carry a bias
 * and that there are two LayerNorms follows from the 13h term of eq. (2).
 * b_o and b_2 are added once, after the (identity) reduction of the row-split
 * GEMMs (section 2.3). */
typedef struct ptdp_layer_params {
  const void *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  const void *ln2_g, *ln2_b, *w_1, *b_1, *w_2, *b_2;
} ptdp_layer_params;

/* Device pointers to the fp32 gradient accumulators, same shapes. */
typedef struct ptdp_layer_grads {
  float *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_o, *b_o;
  float *ln2_g, *ln2_b, *w_1, *b_1, *w_2, *b_2;
} ptdp_layer_grads;

/* Fields of the per-layer, per-microbatch activation stash (what the backward
 * pass needs, section 2.2 "stashed intermediate activations"). */
enum {
  PTDP_STASH_X = 0,  /* layer input           [T, h]   storage dtype */
  PTDP_STASH_U,      /* LayerNorm-1 output    [T, h]                 */
  PTDP_STASH_QKV,    /* Q|K|V                 [T, 3hp]               */
  PTDP_STASH_CTX,    /* attention output      [T, hp]                */
  PTDP_STASH_X1,     /* after first residual  [T, h]                 */
  PTDP_STASH_U2,     /* LayerNorm-2 output    [T, h]                 */
  PTDP_STASH_Z,      /* first MLP GEMM output, before bias [T, fp]   */
  PTDP_STASH_G,      /* GeLU(z + b_1)         [T, fp]                */
  PTDP_STASH_MU1,    /* LayerNorm-1 mean      [T] fp32               */
  PTDP_STASH_RSTD1,  /* LayerNorm-1 1/sqrt(var+eps) [T] fp32         */
  PTDP_STASH_MU2,
  PTDP_STASH_RSTD2,
  PTDP_STASH_LSE,    /* log-sum-exp of scaled masked scores [b, a/t, s] fp32 */
  PTDP_STASH_NFIELDS
};

/* ------------------------------------------------------------ host helpers */

/* Checks a configuration: struct_size, h % a == 0, a % t == 0, (4h) % t == 0,
 * dh % 8 == 0, sizes > 0, 0 <= p_hidden < 1, ln_eps > 0, causal in {0, 1}, known
 * dtype / gelu_mode.  bf16 needs dh in {32, 64, 96, 128, 160} for the MFMA attention
 * kernels, otherwise PTDP_E_UNSUPPORTED. */
int ptdp_cfg_validate(const ptdp_layer_cfg* cfg);

/* Bytes of one layer's stash for one microbatch / byte offset of a field in
 * it (every field 256-byte aligned).  0 / (size_t)-1 on an invalid cfg. */
size_t ptdp_layer_stash_bytes(const ptdp_layer_cfg* cfg);
size_t ptdp_stash_offset(const ptdp_layer_cfg* cfg, int field);

/* Bytes of scratch one forward or backward call needs (contents are garbage
 * between calls; one workspace may serve every call on the same stream). */
size_t ptdp_workspace_bytes(const ptdp_layer_cfg* cfg);

/* Where ptdp_layer_backward leaves the intermediate gradients of the appendix's
 * dgrad / wgrad products inside the workspace when it returns (valid until the
 * next call that uses the workspace; storage dtype, row-major).  On a
 * tensor-parallel shard these are also the buffers an all-reduce of section 2.3
 * would act on (PTDP_WS_DU: the operator f of the attention block). */
enum {
  PTDP_WS_DO = 0,  /* grad of (o + b_o) = dx1 * mask_0 / (1-p)        [T, h]   */
  PTDP_WS_DU,      /* grad of LayerNorm-1's output u                   [T, h]   */
  PTDP_WS_DX1,     /* grad of x1 (after LayerNorm-2's backward)        [T, h]   */
  PTDP_WS_CHAIN,   /* gradient handed from layer l+1 to layer l by ptdp_chunk_backward [T, h] */
  PTDP_WS_DZ,      /* grad of (z + b_1)                                [T, fp]  */
  PTDP_WS_DCTX,    /* grad of the attention output                     [T, hp]  */
  PTDP_WS_DQKV,    /* grad of Q|K|V                                    [T, 3hp] */
  PTDP_WS_DMO,     /* grad of (mo + b_2) = dy * mask_1 / (1-p)         [T, h]   */
  PTDP_WS_NFIELDS
};
/* Byte offset of such a field in the workspace; (size_t)-1 on an invalid cfg or field. */
size_t ptdp_workspace_offset(const ptdp_layer_cfg* cfg, int field);

/* Model FLOPs of one layer's forward pass on this shard for one microbatch:
 * (24 b s h^2 + 4 b s^2 h) / t  (paper appendix; GEMMs only, full s x s
 * attention matrix).  Backward is counted as twice this.  -1 on invalid cfg. */
int64_t ptdp_layer_flops_fwd(const ptdp_layer_cfg* cfg);

/* Time to process one batch on a p-stage pipeline without interleaving,
 * ignoring communication (section 3.4, eq. (1)): a data-parallel replica's
 * share b_prime = B/d of the batch is cut into b_prime/b microbatches of size
 * b, each costing t_fwd + t_bwd per stage, plus p - 1 bubble slots:
 *   (b_prime / b + p - 1) * (t_fwd + t_bwd).
 * Host-only.  NaN unless b_prime, b, p >= 1, b divides b_prime and both times
 * are finite and >= 0. */
double ptdp_batch_time(int64_t b_prime, int64_t b, int p, double t_fwd, double t_bwd);

/* The 64-bit word of the dropout stream that serves elements 4*group ..
 * 4*group+3 of dropout site `site` (0 after attention, 1 after the MLP) of
 * global layer `layer` for microbatch `microbatch`.  SplitMix64 mixing;
 * key = mix(mix(mix(seed) + G*(2*layer+site+1)) + G*(microbatch+1)),
 * word = mix(key + G*group), G = 0x9E3779B97F4A7C15.  Element i of the
 * [s, b, h] tensor uses bits 16*(i&3) .. +15 of word(i>>2) and is KEPT iff
 * that field >= floor(p*65536 + 0.5); kept values are scaled by 1/(1-p).
 * Host function; the kernels evaluate the same integers on the device. */
uint64_t ptdp_hash(uint64_t seed, uint32_t layer, uint32_t site, uint64_t microbatch, uint64_t group);

/* ------------------------------------------------------------------ chunks */

/* A model chunk: n_layers consecutive layers held by this device (section 2.2,
 * "Schedule with Interleaved Stages").  first_global_layer numbers the chunk's
 * first layer in the whole model; it only selects dropout streams. */
typedef struct ptdp_chunk ptdp_chunk;

int ptdp_chunk_create(const ptdp_layer_cfg* cfg, int n_layers, int first_global_layer, ptdp_chunk** out);
void ptdp_chunk_destroy(ptdp_chunk* chunk);
int ptdp_chunk_n_layers(const ptdp_chunk* chunk);

/* Records the (borrowed) device pointers of layer `layer` (0-based inside the
 * chunk).  All twelve pointers must be non-NULL. */
int ptdp_chunk_bind_params(ptdp_chunk* chunk, int layer, const ptdp_layer_params* dev_ptrs);
int ptdp_chunk_bind_grads(ptdp_chunk* chunk, int layer, const ptdp_layer_grads* dev_ptrs);

/* General attention mask for a chunk whose cfg.causal is 0 (section 4.2 names
 * two fused softmax kernels: general masking, as in BERT-style models, and
 * the implicit causal mask).  mask: dev bytes [b, s, s], 4-byte aligned,
 * borrowed; mask[j][q][k] != 0 hides key k from query q of sample j; NULL
 * (the default) hides nothing.  A hidden scaled score is replaced by -10000
 * before the softmax: a query with some visible key gives hidden keys
 * probability 0; a query with none attends uniformly; no gradient reaches q
 * or k through a hidden score.  PTDP_E_INVALID_ARG on a causal chunk. */
int ptdp_chunk_set_mask(ptdp_chunk* chunk, const uint8_t* mask);

/* Forward of one layer for one microbatch (section 2.3):
 *   u = LN1(x); qkv = u Wqkv + bqkv; ctx = causal softmax(q k^T/sqrt(dh)) v per
 *   (sample, local head); o = ctx Wo; x1 = x + Drop0(o + bo); u2 = LN2(x1);
 *   z = u2 W1; g = GeLU(z + b1); mo = g W2; y = x1 + Drop1(mo + b2).
 * x [T,h] dev in, y [T,h] dev out (may not alias x), stash: ptdp_layer_stash_bytes
 * dev bytes written, workspace: ptdp_workspace_bytes dev bytes scratch.
 * `microbatch` selects the dropout stream.  If x already is the stash's X
 * field the copy into the stash is skipped. */
int ptdp_layer_forward(ptdp_chunk* chunk, int layer, int64_t microbatch, const void* x, void* y,
                       void* stash, void* workspace, void* stream);

/* Backward of the same layer/microbatch: given dy [T,h] returns dx [T,h] (may
 * alias dy) and adds this microbatch's parameter gradients into the bound
 * gradient buffers.  Dropout masks are recomputed from the hash; the attention
 * probabilities are recomputed from the stashed log-sum-exp. */
int ptdp_layer_backward(ptdp_chunk* chunk, int layer, int64_t microbatch, const void* dy, void* dx,
                        const void* stash, void* workspace, void* stream);

/* The chunk's layers in order (forward) / reverse order (backward).  `stash`
 * holds n_layers consecutive layer stashes. */
int ptdp_chunk_forward(ptdp_chunk* chunk, int64_t microbatch, const void* x, void* y,
                       void* stash, void* workspace, void* stream);
int ptdp_chunk_backward(ptdp_chunk* chunk, int64_t microbatch, const void* dy, void* dx,
                        const void* stash, void* workspace, void* stream);

/* Activation recomputation (section 3.5).  The chunk is cut into segments of
 * seg_layers consecutive layers (the last may be shorter); only the input
 * activation of each segment is kept per in-flight microbatch:
 *   ckpt: dev, ptdp_chunk_n_checkpoints(chunk, seg_layers) * ptdp_checkpoint_bytes
 *         bytes (written by the forward, read by the backward);
 *   seg_stash: dev scratch for seg_layers layer stashes, shared by every
 *         microbatch (garbage between calls).
 * The backward reruns each segment's forward from its checkpoint (same dropout
 * masks: they are a pure function of seed, layer, site, microbatch and element
 * index) and then runs that segment's backward, last segment first.  With c
 * checkpoints over l layers the kept bytes are c*A_input + (l/c)*A_intermediate
 * (A_input = ptdp_checkpoint_bytes, A_intermediate = ptdp_layer_stash_bytes).
 * Results are bit-identical to ptdp_chunk_forward / ptdp_chunk_backward.
 * seg_layers in [1, n_layers], else PTDP_E_INVALID_ARG. */
size_t ptdp_checkpoint_bytes(const ptdp_layer_cfg* cfg);
int ptdp_chunk_n_checkpoints(const ptdp_chunk* chunk, int seg_layers);
int ptdp_chunk_forward_ckpt(ptdp_chunk* chunk, int64_t microbatch, const void* x, void* y, void* ckpt,
                            int seg_layers, void* seg_stash, void* workspace, void* stream);
int ptdp_chunk_backward_ckpt(ptdp_chunk* chunk, int64_t microbatch, const void* dy, void* dx,
                             const void* ckpt, int seg_layers, void* seg_stash, void* workspace,
                             void* stream);

/* ---------------------------------------------------------------- schedule */

/* One pass of the device's order: kind 0 = forward, 1 = backward. */
typedef struct ptdp_step {
  int32_t kind, chunk, microbatch;
} ptdp_step;

/* Order in which device `rank` of `p` runs its passes for one batch of m
 * microbatches with v chunks per device (section 2.2): v = 1 is the
 * PipeDream-Flush 1F1B schedule (warm-up of p-rank-1 forwards, steady 1F1B,
 * cool-down); v > 1 is the interleaved schedule and needs m % p == 0.
 * Writes 2*m*v steps to out (host) if cap allows, the count to *n_out (host).
 * Host-only, integer-only. */
int ptdp_schedule_build(int p, int v, int m, int rank, ptdp_step* out, int cap, int* n_out);

/* Largest number of (chunk, microbatch) stashes alive at once under that
 * order (<= p for v = 1), or a negative status. */
int ptdp_schedule_peak_inflight(int p, int v, int m, int rank);

/* Runs a step list on one device.  chunks[c] is the device's c-th chunk.
 * stage_in[c*m + mb]  : dev input activations of (chunk c, microbatch mb), [T,h]
 * stage_dout[c*m + mb]: dev output gradients of the same pair
 * stage_out / stage_din: dev buffers receiving the chunk's output / input
 *   gradient (what would be sent to the neighbouring stage); entries may
 *   repeat, NULL entries are not allowed.
 * stash_pool: dev memory for n_slots chunk stashes (slot_bytes each =
 *   n_layers * ptdp_layer_stash_bytes); a slot is taken at a forward and
 *   released at the matching backward; PTDP_E_TOO_SMALL (before any device
 *   work) if the order needs more than n_slots. */
int ptdp_schedule_run(ptdp_chunk* const* chunks, int v, int m, const ptdp_step* steps, int n_steps,
                      const void* const* stage_in, void* const* stage_out,
                      const void* const* stage_dout, void* const* stage_din,
                      void* stash_pool, size_t slot_bytes, int n_slots, void* workspace, void* stream);

/* The same with activation recomputation: ckpt_pool holds n_slots checkpoint
 * sets of slot_bytes each (>= n_checkpoints * ptdp_checkpoint_bytes of every
 * chunk); seg_stash as in ptdp_chunk_forward_ckpt, one for the whole run. */
int ptdp_schedule_run_ckpt(ptdp_chunk* const* chunks, int v, int m, const ptdp_step* steps, int n_steps,
                           const void* const* stage_in, void* const* stage_out,
                           const void* const* stage_dout, void* const* stage_din,
                           void* ckpt_pool, size_t slot_bytes, int n_slots, int seg_layers,
                           void* seg_stash, void* workspace, void* stream);

/* ------------------------------------------- first / last stage extras */
/* What the first and last pipeline stage run besides transformer layers: the
 * V x h word table and s x h position table of eq. (2), and the logit layer of
 * the appendix (2 b s h V FLOPs forward, 4 b s h V backward).  The paper fixes
 * no more than that; the readings taken are: hidden dropout after the
 * embedding sum (stream of layer id PTDP_EMBED_LAYER, site 0), a final
 * LayerNorm before the logits, the word table shared by input and output, mean
 * token loss.  One tensor-parallel shard holds the vocabulary rows
 * [vocab_first, vocab_first + vocab_rows) (vocab_rows % 8 == 0): ids outside
 * contribute zero rows / no target term, and maximum and sum of exponentials
 * run over the shard's rows (the cross-shard reductions are the identity on
 * one shard, as for the layers).  cfg supplies h, s, b, dtype, p_hidden,
 * ln_eps, seed.  tokens / targets: dev int32 [s, b]. */
#define PTDP_EMBED_LAYER 0x7fffffffu

/* Bytes of scratch for the three calls below. */
size_t ptdp_lm_workspace_bytes(const ptdp_layer_cfg* cfg, int vocab_rows);
/* 2 b s h vocab_rows: the shard's logit GEMM, forward. */
int64_t ptdp_logit_flops_fwd(const ptdp_layer_cfg* cfg, int vocab_rows);

/* x[i,j,:] = Drop(e_word[tokens[i,j] - vocab_first] + e_pos[i]);  e_word
 * [vocab_rows, h], e_pos [s, h], x [T, h] out, all dev in cfg's dtype. */
int ptdp_embedding_forward(const ptdp_layer_cfg* cfg, int vocab_first, int vocab_rows, const int32_t* tokens,
                           const void* e_word, const void* e_pos, void* x, int64_t microbatch, void* stream);
/* d_e_word [vocab_rows, h] and d_e_pos [s, h] (dev fp32) += the gradients for
 * dx [T, h].  Rows of repeated ids are added in token order (no atomics). */
int ptdp_embedding_backward(const ptdp_layer_cfg* cfg, int vocab_first, int vocab_rows, const int32_t* tokens,
                            const void* dx, float* d_e_word, float* d_e_pos, void* workspace,
                            int64_t microbatch, void* stream);
/* Forward and backward of the model head for one microbatch (the last stage
 * runs them back to back under 1F1B): u = LN(y); logits = u e_word^T;
 * token_loss[r] = log sum_v exp(logit[r,v]) - logit[r,target[r]] (dev fp32
 * [T]); loss[0] = mean (dev fp32); then gradients of loss_scale * loss:
 * dy [T, h] out (may alias y), d_lnf_g / d_lnf_b [h] and d_e_word
 * [vocab_rows, h] (dev fp32) +=. */
int ptdp_lm_head_step(const ptdp_layer_cfg* cfg, int vocab_first, int vocab_rows, const void* y, const void* lnf_g,
                      const void* lnf_b, const void* e_word, const int32_t* targets, float loss_scale,
                      float* loss, float* token_loss, void* dy, float* d_lnf_g, float* d_lnf_b,
                      float* d_e_word, void* workspace, void* stream);

/* ------------------------------------------------- single kernels (per-op) */
/* Exported for per-operation parity tests and roofline measurements.  dtype as
 * in ptdp_layer_cfg; all pointers dev; rows = T. */

/* LayerNorm over the last dimension (biased variance, two-pass):
 * u = g*(x-mu)*rstd + beta; mu, rstd [rows] fp32 out.  If x_copy != NULL the
 * input row is also copied there. */
int ptdp_layernorm_fwd(int dtype, const void* x, const void* gain, const void* bias, void* u, float* mu,
                       float* rstd, void* x_copy, int rows, int width, float eps, void* stream);
/* dx = resid + LN'(du): resid [rows,width] may be NULL (treated as 0), dx may
 * alias resid or du.  dgain, dbias [width] fp32 +=.  scratch: dev,
 * >= ptdp_layernorm_bwd_scratch_bytes(rows, width). */
int ptdp_layernorm_bwd(int dtype, const void* du, const void* x, const void* gain, const float* mu,
                       const float* rstd, const void* resid, void* dx, float* dgain, float* dbias,
                       void* scratch, int rows, int width, void* stream);
/* g = GeLU(z + bias) (bias + GeLU fusion of section 4.2). */
int ptdp_bias_gelu_fwd(int dtype, int gelu_mode, const void* z, const void* bias, void* g, int rows,
                       int width, void* stream);
/* dz = dg * GeLU'(z + bias) (dz may alias dg); dbias [width] fp32 += column sums of dz. */
int ptdp_bias_gelu_bwd(int dtype, int gelu_mode, const void* dg, const void* z, const void* bias, void* dz,
                       float* dbias, void* scratch, int rows, int width, void* stream);
/* out = resid + keep*(in + bias)/(1-p) (bias + dropout + add fusion of section
 * 4.2); mask from ptdp_hash(seed, layer, site, microbatch, .). */
int ptdp_bias_dropout_add_fwd(int dtype, const void* in, const void* bias, const void* resid, void* out,
                              int rows, int width, float p, uint64_t seed, uint32_t layer, uint32_t site,
                              uint64_t microbatch, void* stream);
/* din = keep*dout/(1-p) (din may not alias dout); dbias [width] fp32 += column sums of din. */
int ptdp_bias_dropout_add_bwd(int dtype, const void* dout, void* din, float* dbias, void* scratch, int rows,
                              int width, float p, uint64_t seed, uint32_t layer, uint32_t site,
                              uint64_t microbatch, void* stream);
size_t ptdp_colsum_scratch_bytes(int rows, int width);
size_t ptdp_layernorm_bwd_scratch_bytes(int rows, int width);
/* For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): ptdp_bias_dropout_add_bwd
 * without the scratch argument.  The column-sum partials live in a static device
 * array of ptdp_noalloc_scratch_bytes() (8 MiB) that each GPU the library runs on
 * holds until the process ends; the call allocates and frees nothing.  Same
 * kernels, same results, bit for bit.  PTDP_E_TOO_SMALL when
 * ptdp_colsum_scratch_bytes(rows, width) exceeds the array (nothing is launched),
 * PTDP_E_STATE while profiling is on (profiling creates events).  Every call on a
 * GPU shares that GPU's array: calls that overlap on one GPU (two streams, two
 * threads) race; calls in stream order do not, and nothing needs clearing between
 * them. */
int ptdp_bias_dropout_add_bwd_noalloc(int dtype, const void* dout, void* din, float* dbias, int rows, int width,
                                      float p, uint64_t seed, uint32_t layer, uint32_t site, uint64_t microbatch,
                                      void* stream);
size_t ptdp_noalloc_scratch_bytes(void);
/* keep[i] = 1/0 for i < n: the dropout keep-mask as bytes (test hook). */
int ptdp_dropout_mask(uint8_t* keep, int64_t n, float p, uint64_t seed, uint32_t layer, uint32_t site,
                      uint64_t microbatch, void* stream);

/* C[M,N] (op)= A' B' + bias, the three GEMM forms of a linear map Y = X W:
 *   mode PTDP_GEMM_NN: A [M,K] row-major, B [K,N] row-major      (forward)
 *   mode PTDP_GEMM_NT: A [M,K] row-major, B [N,K] row-major      (input grad: dX = dY W^T)
 *   mode PTDP_GEMM_TN: A [K,M] row-major, B [K,N] row-major      (weight grad: dW = X^T dY)
 * A, B in `dtype`.  out_f32 = 0: C in `dtype`, overwritten; out_f32 = 1: C fp32,
 * accumulated (+=) when accumulate != 0.  bias [N] in `dtype` or NULL.  bf16
 * needs M, N, K multiples of 8 and operands below 2 GiB.  workspace (dev, may
 * be NULL): ptdp_gemm_workspace_bytes() bytes of scratch; with it, a tile count
 * that does not fill the compute units evenly is finished by giving each tile of
 * the last, incomplete round to several workgroups that split its k range:
 * partial tiles go to the workspace and are summed in a fixed order, so results
 * stay bit-reproducible. */
enum { PTDP_GEMM_NN = 0, PTDP_GEMM_NT = 1, PTDP_GEMM_TN = 2 };
int ptdp_gemm(int dtype, int mode, const void* A, const void* B, void* C, const void* bias, int M, int N,
              int K, int out_f32, int accumulate, void* workspace, size_t workspace_bytes, void* stream);
size_t ptdp_gemm_workspace_bytes(void);
/* Host only (no device work): how ptdp_gemm cuts a bf16 call (appendix: the
 * GEMMs of a layer).  *dp_columns = columns of C computed in whole rounds, one
 * workgroup per 256 x 256 tile (a multiple of 256, or N when nothing is split).
 * The remaining tiles, numbered row tile fastest, form *n_groups (0..2)
 * consecutive groups: group j has group_tiles[j] tiles and gives each of them to
 * group_parts[j] workgroups, part p of which takes the 64-wide k-steps
 * [nk*p/parts, nk*(p+1)/parts) of that tile; tiles x parts never exceeds the
 * number of compute units.  group_tiles / group_parts: two ints each.
 * has_bias / workspace_bytes as in the call being planned.  Returns 0, or
 * PTDP_E_INVALID_ARG / PTDP_E_NULL_PTR. */
int ptdp_gemm_plan(int M, int N, int K, int out_f32, int accumulate, int has_bias, size_t workspace_bytes,
                   int* dp_columns, int* n_groups, int* group_tiles, int* group_parts);

/* Fused causal attention over qkv [s, b, 3hp] (scale 1/sqrt(dh), implicit
 * causal mask, softmax, times V; section 4.2's scale+mask+softmax fusion
 * extended over both batched GEMMs): ctx [s, b, hp], lse [b, heads, s] fp32. */
int ptdp_attn_fwd(int dtype, const void* qkv, void* ctx, float* lse, int s, int b, int heads, int dh,
                  void* stream);
/* The same with a general mask instead of the causal one (mask as in
 * ptdp_chunk_set_mask; NULL = full bidirectional attention). */
int ptdp_attn_masked_fwd(int dtype, const void* qkv, const uint8_t* mask, void* ctx, float* lse, int s, int b,
                         int heads, int dh, void* stream);
int ptdp_attn_masked_bwd(int dtype, const void* qkv, const uint8_t* mask, const void* ctx, const float* lse,
                         const void* dctx, void* dqkv, float* delta, int s, int b, int heads, int dh,
                         void* stream);
/* dqkv [s, b, 3hp] from dctx; delta: dev scratch of b*heads*s floats. */
int ptdp_attn_bwd(int dtype, const void* qkv, const void* ctx, const float* lse, const void* dctx, void* dqkv,
                  float* delta, int s, int b, int heads, int dh, void* stream);

/* ---------------------------------------------------------------- ceilings */
/* What the chip is seen to do, for reading roofline fractions: a loop of
 * v_mfma_f32_32x32x16_bf16 on registers only (workgroups x 8 waves x 8
 * accumulators x iters instructions; random_operands 0: small constant
 * integers, 1: hash-derived values spread like N(0,1), rotated between
 * instructions as in a GEMM (more toggling bits, lower sustained clock); +2:
 * the same loop on v_mfma_f32_16x16x32_bf16, the shape of the forward and
 * data-gradient GEMMs);
 * *flops (host) receives the FLOP count of the launch; sink: dev, >= 4 bytes,
 * not written in practice), and a copy of
 * `bytes` (multiple of 16, 16-byte aligned pointers) with 16 bytes per lane.
 * The caller times them with events on `stream`. */
int ptdp_ceiling_mfma(float* sink, int workgroups, int iters, int random_operands, double* flops, void* stream);
int ptdp_ceiling_copy(const void* src, void* dst, size_t bytes, void* stream);

/* ---------------------------------------------------------------- profiling */
/* Optional per-kernel timing with HIP events on the launch stream.  While
 * enabled every kernel launch of the library is bracketed by an event pair
 * (this serialises nothing but adds a few microseconds per launch, so
 * whole-step throughput is measured with profiling disabled).
 * ptdp_prof_collect synchronises the recorded events and adds their elapsed
 * times to per-family totals.  The profiling state is process-wide and not
 * thread-safe: enable it from one thread, on one device, while no other
 * thread calls the library. */
enum {
  PTDP_K_GEMM_NN = 0, PTDP_K_GEMM_NT, PTDP_K_GEMM_TN, PTDP_K_ATTN_FWD, PTDP_K_ATTN_BWD,
  PTDP_K_LN_FWD, PTDP_K_LN_BWD, PTDP_K_GELU_FWD, PTDP_K_GELU_BWD, PTDP_K_BDA_FWD, PTDP_K_BDA_BWD,
  PTDP_K_COLSUM, PTDP_K_OTHER, PTDP_K_EMBED, PTDP_K_XENT, PTDP_K_NFAMILIES
};
typedef struct ptdp_prof_entry {
  double ms;     /* summed elapsed time of the family's launches */
  double work;   /* summed algorithmic work: FLOPs for GEMM/attention, bytes for the rest */
  int64_t launches;
} ptdp_prof_entry;
int ptdp_prof_enable(int on);         /* also clears the totals when switching on */
int ptdp_prof_collect(ptdp_prof_entry* out /* [PTDP_K_NFAMILIES], host */);
const char* ptdp_prof_family_name(int family);

#ifdef __cplusplus
#pragma GCC visibility pop
}
#endif
#endif /* PTDP_H */
