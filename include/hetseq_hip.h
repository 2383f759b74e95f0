/*
 * hetseq_hip.h - C ABI of libhetseq_hip.so: one worker's share of a HetSeq training step on
 * one MI355X (gfx950).
 *
 * The HetSeq paper ("Distributed GPU Training on Heterogeneous Infrastructure") describes a
 * synchronous data-parallel step in which workers with unequal memory run unequal batches:
 * forward pass and a per-worker loss with a weight (figure 1; section "Forward Pass"; section
 * "Optimizer and Learning Rate Scheduler"), back-propagation with an all-zero contribution from
 * workers that have no data (section "Backpropagation"), aggregation of several passes before
 * one update (section "Delayed Update (Gradient Accumulation)"), division by the global weight
 * so that the result equals the non-distributed large batch, and a local optimizer update
 * (Adam for BERT, section "BERT Language Model").  The calls below are those steps.
 *
 * Conventions (all calls):
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses.
 *  - The caller owns every buffer and the stream.  The library allocates no device memory (the one
 *    built-in array of hs_op_layernorm_bwd_noalloc aside) and keeps no pointer after a call returns, with one
 *    exception: hs_arm_update records the pointers of w, m, v, G and the low-precision copy in the context
 *    until the next hs_encoder_bwd / hs_s2s_bwd call on it has used them; those buffers must stay valid
 *    until then.  hs_ctx holds host state only: tables, the error text, that armed update, the dropout
 *    state, and the handles of up to two further HIP streams (default priority) with the events that
 *    order them, created on first use and destroyed with the context.
 *  - Device calls enqueue on `stream` (a hipStream_t passed as void*; NULL = the default stream)
 *    and return without synchronising.  Results are valid once the caller synchronises that
 *    stream: work a call puts on the context's own streams is joined to `stream` before it returns.
 *    Calls on one context must not overlap in time from different host threads.
 *  - Errors are return codes.  Arguments and shapes are checked on the host before any launch;
 *    a call that fails launches nothing.  hs_last_error() gives the reason as text.
 *  - Matrices are row-major.  Weights are [out, in] (y = x W^T + b).  The flat parameter order
 *    is the one hs_param_layout() reports and is the same for w, m, v, g and G.
 *  - Element type of weights ("w") and activations follows cfg.compute: HS_FP32 -> float,
 *    HS_BF16 -> bfloat16 (fp32 accumulation everywhere; gradients, LayerNorm/softmax/loss
 *    statistics and optimizer state are always fp32).
 *  - Every dev buffer must be 256-byte aligned (what any device allocator returns).
 */
#ifndef HETSEQ_HIP_H
#define HETSEQ_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HS_OK = 0,
  HS_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad flag */
  HS_ERR_SHAPE = 2,       /* sizes the kernels do not support (see each call) */
  HS_ERR_WORKSPACE = 3,   /* workspace smaller than hs_workspace_bytes() */
  HS_ERR_STATE = 4,
  HS_ERR_HIP = 5,         /* a HIP runtime call failed; text in hs_last_error() */
  HS_ERR_UNIMPLEMENTED = 6
} hs_status;

typedef enum { HS_FP32 = 0, HS_BF16 = 1 } hs_dtype;

/* Model shape.  Supported: hidden a multiple of 64 and <= 1024, hidden / n_heads == 64,
 * ffn a multiple of 64, vocab >= 8, 1 <= n_layers, 8 <= max_pos. */
typedef struct {
  int32_t n_layers, hidden, n_heads, ffn, vocab, max_pos;
  float ln_eps;
  int32_t compute; /* hs_dtype */
} hs_model_cfg;

/* One slice of the flat parameter buffer.  Vectors have rows == 1. */
typedef struct {
  char name[48];
  int64_t offset; /* in elements */
  int32_t rows, cols;
} hs_param_entry;

typedef struct hs_ctx hs_ctx; /* opaque, host-side */

/* ---- context, layout, sizes (host only) ------------------------------------------------- */

/* Validates cfg and builds the host-side tables.  *out is NULL on failure. */
hs_status hs_ctx_create(const hs_model_cfg* cfg, hs_ctx** out);
hs_status hs_ctx_destroy(hs_ctx* ctx);
/* Text of the last error on this context (ctx-owned, valid until the next call on ctx), or of
 * the last context-free call when ctx is NULL (thread-local). */
const char* hs_last_error(const hs_ctx* ctx);

/* Number of parameters P of the model (0 when cfg is invalid). */
size_t hs_param_count(const hs_model_cfg* cfg);
/* Writes the layout table.  On entry *n is the capacity of out, on exit the number of entries;
 * with out == NULL only *n is written.  Order: emb.word [V,H], emb.pos [max_pos,H], emb.ln.g,
 * emb.ln.b, then per layer i: l<i>.qkv.w [3H,H] (rows 0..H-1 query, H..2H-1 key, 2H..3H-1
 * value), l<i>.qkv.b, l<i>.o.w [H,H], l<i>.o.b, l<i>.ln1.g, l<i>.ln1.b, l<i>.ffn1.w [F,H],
 * l<i>.ffn1.b, l<i>.ffn2.w [H,F], l<i>.ffn2.b, l<i>.ln2.g, l<i>.ln2.b, then head.t.w [H,H],
 * head.t.b, head.ln.g, head.ln.b, head.dec.b [V]. */
hs_status hs_param_layout(const hs_model_cfg* cfg, hs_param_entry* out, int32_t* n);

/* Bytes of the saved-activation arena written by hs_encoder_fwd and read by hs_encoder_bwd for
 * a batch of B sequences padded to L (M, the number of masked-LM targets, does not enter). */
size_t hs_acts_bytes(const hs_model_cfg* cfg, int32_t B, int32_t L, int32_t M);
/* Bytes of scratch that hs_encoder_fwd / hs_mlm_loss / hs_encoder_bwd need for (B, L, M): the
 * maximum over the three calls, so one buffer serves all. */
size_t hs_workspace_bytes(const hs_model_cfg* cfg, int32_t B, int32_t L, int32_t M);

/* ---- optimizer update inside the last backward pass ----------------------------------------
 * Sections "Backpropagation" / "Optimizer and Learning Rate Scheduler": once the gradients of all
 * micro-batches are summed, they are divided by the global weight and the optimizer updates the
 * parameters.  hs_arm_update arms exactly that (hs_grad_accum_normalize with `denom`, then
 * hs_adam_step with the given arguments, same arithmetic, same results bit for bit) for the NEXT
 * hs_encoder_bwd call on ctx whose gradient buffer g is G: that call then normalises and updates
 * every parameter group (head, each layer, embeddings) on a stream of its own as soon as the
 * group's gradient is final, beside the rest of the backward pass, and joins that work before it
 * returns work to the caller's stream.  Arm it for the LAST micro-batch of an update only (denom is
 * the global sample count of the whole update); hs_mlm_loss of that micro-batch must already have been
 * enqueued on the same stream with the same G.  All pointers dev, sizes = hs_param_count; the
 * armed state is cleared by the backward call that consumes it (also when that call fails).
 * HS_ERR_STATE from hs_encoder_bwd if an update is armed for another buffer. */
hs_status hs_arm_update(hs_ctx* ctx, float* w, float* m, float* v, float* G, void* w_lowp_out /*nullable*/, double denom, double lr,
                        double beta1, double beta2, double eps, double weight_decay, int64_t t);

/* ---- dropout --------------------------------------------------------------------------------
 * Section "Transformer Translation Model" trains with dropout 0.1 and section "Checkpointing" keeps
 * the run's random seed; the cited BERT model drops its embedding output, attention probabilities,
 * attention output and feed-forward output (the last two before the residual is added).
 * hs_set_dropout sets the rate p in [0, 1), the seed and a 32-bit stream number for the following
 * hs_encoder_fwd / hs_encoder_bwd calls on ctx (host state only; p = 0, the initial state, switches
 * dropout off).  A mask is a pure function of (seed, stream, site, element): element e of a site
 * uses word e % 4 of the Philox4x32-10 block with counter (e / 4 low, e / 4 high, site, stream) and
 * key (seed low, seed high), is dropped when that word is below floor(p * 2^32), and is scaled by
 * 1 / (1 - p) otherwise.  Sites: 0 = embedding output [B, L, H]; for layer l: 1 + 3 l = attention
 * probabilities [B, heads, L, L], 2 + 3 l = attention output [B, L, H], 3 + 3 l = feed-forward
 * output [B, L, H]; elements in row-major order of those shapes (L = the padded length).
 * The backward call of a micro-batch must see the state its forward call saw; give every
 * micro-batch of every update its own stream number.  The masked-LM head has no dropout. */
hs_status hs_set_dropout(hs_ctx* ctx, double p, uint64_t seed, uint32_t stream);
/* Test aid: writes the keep mask (1 = survives) of the first n elements of `site` under the current
 * state of ctx to mask_out [n] (dev). */
hs_status hs_dropout_keep_mask(hs_ctx* ctx, uint32_t site, size_t n, uint8_t* mask_out, void* stream);

/* ---- host data path ---------------------------------------------------------------------------
 * Section "Dataset and Dataloader": the dataset is split into shards, the lengths of the shards are
 * accumulated and the index of a training instance is mapped to an offset inside its shard; the
 * shuffle is reproducible.  Section "Forward Pass": batches under the max-tokens criterion.
 * Section "Prefetch and Cache": the next batches are fetched while the current one trains, and a
 * least-recently-used cache keeps instances in memory.  Everything here is host code.
 * Shard file (little-endian): the 8 bytes "HSSHARD1", int64 n_seq, int64 n_tokens, int32
 * lengths[n_seq], int32 tokens[n_tokens].  Instances are numbered through the shards in the order
 * the shards are given. */
typedef struct hs_dataset hs_dataset;
/* Writes a shard (for synthetic data and tests).  lengths [n_seq], tokens [sum of lengths], host. */
hs_status hs_shard_write(const char* path, const int32_t* lengths, int64_t n_seq, const int32_t* tokens);
/* Opens the shards and reads their headers and lengths only (tokens are read on demand).
 * cache_instances: capacity of the least-recently-used instance cache (0: none); prefetch_batches
 * (1..64): how many batches the background thread may be ahead of hs_dataset_next.
 * HS_ERR_STATE for a missing, malformed or truncated shard. */
hs_status hs_dataset_open(const char* const* paths, int32_t n_shards, int64_t cache_instances, int32_t prefetch_batches, hs_dataset** out);
hs_status hs_dataset_close(hs_dataset* d);
int64_t hs_dataset_size(const hs_dataset* d);                                   /* number of instances */
hs_status hs_dataset_lengths(const hs_dataset* d, int32_t* lengths_out /*[size]*/);
/* The index map: shard and row of a global instance index. */
hs_status hs_dataset_locate(const hs_dataset* d, int64_t instance, int32_t* shard_out, int64_t* row_out);
/* Starts an epoch: forms the batches of the whole dataset with hs_make_batches(bucket_width, max_tokens,
 * cap_mode), shuffles their order (Fisher-Yates: for i = n-1 .. 1 swap batch i with batch
 * w mod (i + 1), w = word 0 of the Philox4x32-10 block with counter (i low, i high, epoch, 0x5AFF1E) and
 * key (seed low, seed high)), keeps the batches rank, rank + world, ... for this worker and starts the
 * background thread.  *n_batches_out = this worker's number of batches.  An epoch in progress is
 * abandoned. */
hs_status hs_dataset_begin_epoch(hs_dataset* d, uint64_t seed, int64_t epoch, int32_t bucket_width, int64_t max_tokens, int32_t cap_mode,
                                 int32_t world, int32_t rank, int64_t* n_batches_out);
/* Shape of the next batch (sequences, padded length); 0, 0 when the epoch is over. */
hs_status hs_dataset_peek(hs_dataset* d, int32_t* B_out, int32_t* L_out);
/* Copies the next batch into the caller's host buffers (pinned memory makes the following upload
 * asynchronous): ids_out [B * L] padded with 0, lens_out [B], instance_out [B] (nullable) the global
 * instance indices.  Blocks until the background thread has assembled the batch.  HS_ERR_STATE at
 * the end of the epoch or after a read error.  One consumer thread per dataset. */
hs_status hs_dataset_next(hs_dataset* d, int32_t* ids_out, int32_t* lens_out, int64_t* instance_out);
/* Instances read from the shards and instances served by the cache, over the batches assembled so far. */
hs_status hs_dataset_stats(hs_dataset* d, int64_t* loads_out, int64_t* hits_out);

/* ---- learning-rate schedule (host) ---------------------------------------------------------
 * Section "BERT Language Model": linear-decay schedule with a maximum rate, `warmup` warm-up
 * updates and `total` updates in all.  Returns the rate of update number t (1-based):
 * max_lr * t / warmup while t <= warmup, then max_lr * (total - t) / (total - warmup), and 0 from
 * t = total on.  No device work.  Returns NaN (and records an error text) when t < 1, warmup < 0,
 * total < max(warmup, 1), or max_lr is negative or not finite. */
double hs_lr_linear(int64_t t, double max_lr, int64_t warmup, int64_t total);

/* ---- checkpoints (host files) -------------------------------------------------------------
 * Section "Checkpointing": a snapshot holds the model parameters, the completed epochs and steps,
 * the optimizer status including the scheduler's, and the random seed, so that training continues
 * exactly where it stopped.  The file is: the magic "HSCKPT01", this header, the three fp32 arrays
 * w, m, v of n_params elements each, and a 64-bit FNV-1a checksum of everything before it
 * (little-endian, no padding beyond the struct's own).
 * All pointers are HOST pointers; the caller copies device state to the host first.  Nothing is
 * kept after a call returns.  A failed write leaves no file under `path` (it is written under a
 * temporary name and renamed). */
typedef struct {
  hs_model_cfg cfg;        /* the model the state belongs to */
  int64_t n_params;        /* = hs_param_count(&cfg) */
  int64_t epoch, step;     /* completed epochs and completed updates (Adam's t of the last update) */
  uint64_t seed;           /* seed of the run's random processes */
  double max_lr;           /* scheduler status: the three numbers of hs_lr_linear */
  int64_t warmup, total;
  double beta1, beta2, eps, weight_decay;   /* optimizer hyper-parameters (its moments are m and v) */
} hs_ckpt_header;
/* HS_ERR_INVALID_ARG: NULL argument, n_params != hs_param_count(&cfg); HS_ERR_STATE: the file
 * cannot be created or written completely. */
hs_status hs_checkpoint_write(const char* path, const hs_ckpt_header* header, const float* w, const float* m, const float* v);
/* Reads and validates magic and header only. */
hs_status hs_checkpoint_read_header(const char* path, hs_ckpt_header* header_out);
/* Reads the arrays into w, m, v (each n elements, n must equal the file's n_params) and verifies the
 * checksum; HS_ERR_STATE on a missing, truncated or corrupted file (the arrays may then be partly
 * written), HS_ERR_SHAPE when n does not match. */
hs_status hs_checkpoint_read(const char* path, hs_ckpt_header* header_out, float* w, float* m, float* v, size_t n);

/* ---- batch formation (host, integer) ----------------------------------------------------
 * Section "Forward Pass": batches are formed under a max-instances or max-tokens criterion; the
 * last batch may be partially filled (section "Optimizer and Learning Rate Scheduler").
 * Sequences are ordered by (length, index); a sequence of length n is padded to
 * ceil(n / bucket_width) * bucket_width; inside one padded length, sequences join the open
 * batch in order until the cap would be exceeded.  cap_mode 0 caps the real tokens of a batch
 * (sum of lengths), cap_mode 1 caps its padded size (sequences x padded length).
 * lengths [n] host, each >= 1 and admissible under the cap alone.  Outputs (host, caller
 * allocated): seq_index_out [n], batch_offsets_out [n + 1] (n_batches + 1 entries used),
 * batch_pad_len_out [n] (n_batches used).  Returns HS_ERR_INVALID_ARG on a bad argument or a
 * length that cannot fit; nothing is written in that case except *n_batches_out = 0. */
hs_status hs_make_batches(const int32_t* lengths, int64_t n, int32_t bucket_width, int64_t max_tokens,
                          int32_t cap_mode, int32_t* seq_index_out, int64_t* batch_offsets_out,
                          int32_t* batch_pad_len_out, int64_t* n_batches_out);

/* Key mask of a padded batch: mask_out[b * L + l] = (l < lens[b]) as uint8.  lens [B] dev,
 * mask_out [B, L] dev.  The attention kernels apply exactly this predicate. */
hs_status hs_key_mask(const int32_t* lens, int32_t B, int32_t L, uint8_t* mask_out, void* stream);

/* ---- the training step ------------------------------------------------------------------ */

/* Encoder forward (figure 1 "forward step"; section "Forward Pass").
 * x0 = LN(E[ids] + Pos); per layer (post-LN): attention over the real keys only
 * (key l' of sequence b takes part iff l' < lens[b]), x' = LN(x + attn W_o^T + b_o),
 * x'' = LN(x' + GELU(x' W_1^T + b_1) W_2^T + b_2); GELU is the exact erf form.
 * w: flat parameters, dev, element type per cfg.compute.  ids [B, L] dev int32 in [0, vocab),
 * lens [B] dev int32 with 1 <= lens[b] <= L (also given on the host as lens_host, which is only
 * validated, may be NULL to skip validation).  L a multiple of 8, L <= max_pos.
 * acts: dev, hs_acts_bytes(); hidden_out [B, L, H] dev, activation type.  Rows of padded
 * positions hold finite don't-care values. */
hs_status hs_encoder_fwd(hs_ctx* ctx, const void* w, const int32_t* ids, const int32_t* lens,
                         const int32_t* lens_host, int32_t B, int32_t L, void* acts, void* hidden_out,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Masked-LM head, loss SUM and its backward (section "Optimizer and Learning Rate Scheduler":
 * a worker reports a loss together with a weight; no division happens here).
 * g_m = hidden[mlm_pos[m]]; t = LN(GELU(g W_t^T + b_t)); logits = t E^T + b_dec (decoder tied to
 * the word embedding); *loss_sum = sum_m [logsumexp(logits_m) - logits_m[label_m]].
 * Backward with d loss_sum = 1: gradients of head.* and the decoder's share of emb.word go to g
 * (flat fp32 [P] dev; overwritten in those slices when accumulate == 0, added when 1), and
 * d_hidden [B, L, H] dev (activation type) is fully written: zeros off the target rows.
 * mlm_pos [M] dev int32 = b * L + l, strictly ascending, each a real position; mlm_label [M] dev
 * int32 in [0, vocab).  M == 0 is defined: loss 0, zero d_hidden, g untouched. */
hs_status hs_mlm_loss(hs_ctx* ctx, const void* w, const void* hidden, const int32_t* mlm_pos,
                      const int32_t* mlm_label, int32_t M, int32_t B, int32_t L, float* loss_sum,
                      void* d_hidden, float* g, int32_t accumulate, void* workspace,
                      size_t workspace_bytes, void* stream);

/* Encoder backward (figure 1 "backpropagation"; section "Backpropagation").
 * Chain rule through everything hs_encoder_fwd computed, from d_hidden down to the embeddings.
 * Parameter gradients go to g (flat fp32 [P] dev): slices l<i>.*, emb.pos, emb.ln.* are
 * overwritten when accumulate == 0 and added when 1; emb.word is ALWAYS added to (the tied
 * decoder's share is already there), so call hs_mlm_loss first.  With accumulate == 1 and
 * g == the accumulation buffer G, gradients of successive micro-batches sum in place and no
 * separate accumulation pass is needed.  Rows of emb.pos beyond L are zero-filled when
 * accumulate == 0.  d_hidden is read only. */
hs_status hs_encoder_bwd(hs_ctx* ctx, const void* w, const void* acts, const int32_t* ids,
                         const int32_t* lens, int32_t B, int32_t L, const void* d_hidden, float* g,
                         int32_t accumulate, void* workspace, size_t workspace_bytes, void* stream);

/* Delayed update and weighting (sections "Delayed Update (Gradient Accumulation)",
 * "Backpropagation", "Optimizer and Learning Rate Scheduler").
 * If ignore == 0 and g != NULL: G += g.  If ignore != 0 (dummy batch of a worker without data)
 * g is not read at all.  Then, if denom > 0: G /= denom (denom = the global weight: sample or
 * token count over all micro-batches and workers; the library never counts, the caller does).
 * denom == 0 means no scaling.  G, g flat fp32 [n] dev.  denom < 0 or NaN -> HS_ERR_INVALID_ARG. */
hs_status hs_grad_accum_normalize(float* G, const float* g, size_t n, int32_t ignore, double denom,
                                  void* stream);

/* Fused Adam (section "BERT Language Model": beta1 0.9, beta2 0.999, eps 1e-8, max lr 1e-4; the
 * learning rate of the step is a host scalar from the caller's schedule).
 * m = b1 m + (1-b1) G; v = b2 v + (1-b2) G^2; w -= lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps);
 * weight_decay, when non-zero, is decoupled (w -= lr * wd * w, applied before the Adam term).
 * w, m, v (in/out) and G (in) flat fp32 [n] dev; w_lowp_out [n] dev bfloat16 or NULL: the
 * rounded (nearest-even) copy of the new w for the next forward pass.  t >= 1. */
hs_status hs_adam_step(float* w, float* m, float* v, const float* G, void* w_lowp_out, size_t n,
                       double lr, double beta1, double beta2, double eps, double weight_decay, int64_t t,
                       void* stream);

/* The loss that a step reports (section "Optimizer and Learning Rate Scheduler": every worker's loss comes with a
 * weight, and the weighted sum over all workers divided by the global weight equals the non-distributed loss):
 * *loss_out = (loss_sums[0] + ... + loss_sums[n - 1]) / denom, the sums added in index order.  loss_sums [n] dev:
 * the loss SUMs that hs_mlm_loss (hs_s2s_loss) wrote for the micro-batches of the step, zeros for workers or passes
 * without data; denom > 0: the global weight, the one given to hs_grad_accum_normalize; loss_out: dev scalar. */
hs_status hs_weighted_loss(const float* loss_sums, int32_t n, double denom, float* loss_out, void* stream);

/* Zero-fills `bytes` bytes at dst (dev): the start state of the gradient buffer of an update whose first micro-batch
 * has no target, and of the loss sums of workers without data (sections "Backpropagation" and "Delayed Update
 * (Gradient Accumulation)": such a worker contributes nothing).  Buffers above 4096 bytes must be 16-byte aligned. */
hs_status hs_fill_zero(void* dst, size_t bytes, void* stream);

/* fp32 -> activation-type copy of a flat buffer (dst bfloat16 [n] for HS_BF16, float for
 * HS_FP32); used once to seed the low-precision weights before the first step. */
hs_status hs_cast_params(const float* src, void* dst, size_t n, int32_t dst_dtype, void* stream);

/* ---- translation workload: encoder-decoder step ---------------------------------------------
 * Section "Transformer Translation Model": the base Transformer (6 + 6 layers, hidden 512, 8 heads,
 * dropout 0.1, label-smoothed cross-entropy with epsilon 0.1, Adam 0.9 / 0.98 / 1e-9), trained with
 * 4096 tokens per worker (table 1).  The model is the cited one written out: one embedding matrix E
 * shared by source tokens, target tokens and the output projection; inputs sqrt(H) E[id] + PE[pos] with
 * PE[p, 2i] = sin(p / 10000^(2i/H)), PE[p, 2i+1] = cos(p / 10000^(2i/H)); post-LN sub-layers
 * x <- LN(x + drop(sublayer(x))); encoder layer = self-attention over the real source tokens, ReLU
 * feed-forward; decoder layer = causal self-attention, attention over the encoder output (masked by
 * the source lengths), ReLU feed-forward; dropout (hs_set_dropout) on the two embedding sums and on
 * every sub-layer output; logits = decoder output times E^T.  The optimizer calls above serve this
 * workload unchanged (the caller passes the token count as denom). */
typedef struct {
  int32_t n_enc, n_dec, hidden, n_heads, ffn, vocab, max_pos;
  float ln_eps;
  int32_t compute; /* hs_dtype */
} hs_s2s_cfg;

/* A context for the calls below (destroyed with hs_ctx_destroy; hs_set_dropout, hs_profile_* and
 * hs_last_error apply).  hidden = 64 * n_heads, a multiple of 64 and <= 1024; ffn and vocab as in hs_ctx_create. */
hs_status hs_s2s_ctx_create(const hs_s2s_cfg* cfg, hs_ctx** out);
size_t hs_s2s_param_count(const hs_s2s_cfg* cfg);
/* Same protocol as hs_param_layout.  Order: emb; enc<i>.{qkv.w, qkv.b, o.w, o.b, ln1.g, ln1.b, ffn1.w, ffn1.b,
 * ffn2.w, ffn2.b, ln2.g, ln2.b}; dec<i>.{qkv, o, ln1, cq.w, cq.b, ckv.w, ckv.b, co.w, co.b, lnc.g, lnc.b, ffn1, ffn2, ln2}. */
hs_status hs_s2s_param_layout(const hs_s2s_cfg* cfg, hs_param_entry* out, int32_t* n);
size_t hs_s2s_acts_bytes(const hs_s2s_cfg* cfg, int32_t B, int32_t Ls, int32_t Lt);
size_t hs_s2s_workspace_bytes(const hs_s2s_cfg* cfg, int32_t B, int32_t Ls, int32_t Lt);

/* Forward pass of one batch of sentence pairs.  src [B, Ls], tgt_in [B, Lt] dev int32 in [0, vocab) (tgt_in is the
 * target shifted right); src_lens, tgt_lens [B] dev int32 with 1 <= len <= Ls (Lt).  Ls, Lt multiples of 8, <= max_pos.
 * acts: dev, hs_s2s_acts_bytes(); dec_out [B, Lt, H] dev, activation type (rows of padding: finite don't-care).
 * Sub-layer dropout needs H * Ls and H * Lt to be multiples of 4 (always true). */
hs_status hs_s2s_fwd(hs_ctx* ctx, const void* w, const int32_t* src, const int32_t* src_lens, const int32_t* tgt_in,
                     const int32_t* tgt_lens, int32_t B, int32_t Ls, int32_t Lt, void* acts, void* dec_out, void* stream);

/* Output projection, label-smoothed loss SUM over the real target positions and its backward.
 * Per real position with label y: nll = logsumexp(z) - z_y; loss = (1 - eps) nll + eps (logsumexp(z) - mean_v z_v), i.e.
 * the cross-entropy to the target (1 - eps) onehot(y) + eps / V.  *loss_sum and *nll_sum (dev scalars, nll_sum may be
 * NULL) are overwritten; nothing is divided (the weight, normally the number of real target tokens, travels beside the sum).
 * tgt_out [B, Lt] dev int32 labels.  tgt_lens_host: the same lengths on the host, or NULL; when given they are validated
 * (1 <= len <= Lt) and the padding rows are left out of the projection (the real rows are gathered first), which changes
 * nothing but the order of the fp32 loss sums.  d_dec_out [B, Lt, H] dev is fully written (zero rows at padding); the projection's
 * share of the emb gradient goes to g (flat fp32 [P] dev): overwritten when accumulate == 0, added when 1. */
hs_status hs_s2s_loss(hs_ctx* ctx, const void* w, const void* dec_out, const int32_t* tgt_out, const int32_t* tgt_lens,
                      const int32_t* tgt_lens_host, int32_t B, int32_t Lt, double eps, float* loss_sum, float* nll_sum, void* d_dec_out,
                      float* g, int32_t accumulate, void* workspace, size_t workspace_bytes, void* stream);

/* Backward through decoder and encoder down to the embedding.  Gradients of enc*. and dec*. go to g (overwritten when
 * accumulate == 0, added when 1); emb is ALWAYS added to (call hs_s2s_loss first).  An update armed with hs_arm_update is
 * consumed by this call as by hs_encoder_bwd: each layer's slice of the flat buffers is normalised and updated as soon as
 * its gradient is final, the shared embedding last. */
hs_status hs_s2s_bwd(hs_ctx* ctx, const void* w, const void* acts, const int32_t* src, const int32_t* src_lens, const int32_t* tgt_in,
                     const int32_t* tgt_lens, int32_t B, int32_t Ls, int32_t Lt, const void* d_dec_out, float* g, int32_t accumulate,
                     void* workspace, size_t workspace_bytes, void* stream);

/* Building block, exported for tests: attention with separate query and key/value sequences (head dimension 64).
 * q rows b*Lq + i (stride ldq elements), k and v rows b*Lk + j (stride ldkv); key j takes part iff j < klens[b] and, when
 * causal != 0 (needs Lq == Lk), j <= i.  ctx_out [B*Lq, A*64]; lse [B, A, Lq] fp32.  Backward: queries at or beyond
 * qlens[b] get zero gradients; dq (stride lddq), dk, dv (stride lddkv) are written for every row; dvec [B, A, Lq] scratch. */
hs_status hs_op_attention_general_fwd(int32_t dtype, const void* q, int64_t ldq, const void* k, const void* v, int64_t ldkv,
                                      const int32_t* qlens, const int32_t* klens, int32_t B, int32_t Lq, int32_t Lk, int32_t A,
                                      int32_t causal, void* ctx_out, float* lse, void* stream);
hs_status hs_op_attention_general_bwd(int32_t dtype, const void* q, int64_t ldq, const void* k, const void* v, int64_t ldkv,
                                      const int32_t* qlens, const int32_t* klens, int32_t B, int32_t Lq, int32_t Lk, int32_t A,
                                      int32_t causal, const void* ctx_in, const float* lse, const void* d_ctx, void* dq, int64_t lddq,
                                      void* dk, void* dv, int64_t lddkv, float* dvec, void* stream);

/* ---- per-kernel timing (optional) -------------------------------------------------------
 * When enabled, every kernel launch of the ctx-taking calls is bracketed by a pair of HIP
 * events on the launch stream.  hs_profile_read synchronises those events and returns, per
 * kernel class, launches, summed milliseconds and the algorithmic flops and bytes the launches
 * were asked to do.  Off by default; costs two event records per launch when on. */
typedef struct {
  char name[32];
  int64_t launches;
  double ms;
  double flops; /* algorithmic: 2*M*N*K for contractions */
  double bytes; /* algorithmic HBM bytes: operands read once, results written once */
} hs_profile_entry;
hs_status hs_profile_enable(hs_ctx* ctx, int32_t on);
/* On entry *n = capacity of out; on exit the number of classes written.  Resets the counters. */
hs_status hs_profile_read(hs_ctx* ctx, hs_profile_entry* out, int32_t* n);

/* ---- building blocks (exported so that each kernel can be checked on its own) ------------
 * Same conventions as above.  dtype is an hs_dtype and selects both element type and kernel
 * family (HS_FP32: plain fp32 kernels; HS_BF16: MFMA kernels with fp32 accumulation). */

/* C[M,N] = sum_k A(m,k) B(n,k) (+ epilogue).  a_kmajor: A stored [M, lda] with k contiguous,
 * else [K, lda] with m contiguous; same for B with n.  C is float (c_f32 != 0; C = beta*C + acc)
 * or the activation type (beta ignored).  bias [N] activation type or NULL.  epi: 0 none;
 * 1 C += R[m,n] (aux = R, activation type, leading dimension ldaux); 2 C = pre-activation,
 * C2 = GELU(C) (C2 same type and ldc as C); 3 C = acc * GELU'(aux[m,n]).
 * In bf16 mode rows of operands must be 16-byte aligned (leading dimensions multiples of 8) and
 * the 8-element chunk that contains the last valid element of a contiguous row must be readable
 * and finite.  scratch (dev, scratch_bytes, may be NULL): when given and the output has too few
 * tiles to fill the chip, the contraction is split, the fp32 partial sums go to scratch and are
 * added in a fixed order. */
hs_status hs_op_gemm(int32_t dtype, int32_t a_kmajor, int32_t b_kmajor, int32_t M, int32_t N, int32_t K,
                     const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                     int32_t c_f32, float beta, const void* bias, int32_t epi, const void* aux,
                     int64_t ldaux, void* C2, void* scratch, size_t scratch_bytes, void* stream);

/* Timing aid, not part of the method: the library holds several tilings of its bf16 GEMM kernel (numbered 0 .. 11: block
 * tile, k-tile depth, blocks per CU, operands staged through registers or loaded into LDS directly) and normally picks
 * one per product from its shape.  variant >= 0 makes every later bf16 product of this process with M, N, K >= 256
 * that the variant can serve use it (the grouped weight-gradient launch of the backward pass keeps its own tiling);
 * -1 restores the automatic choice.
 * Results stay within the same tolerance for every variant.  Host call, process-wide, not thread-safe: set it while no
 * other thread launches work.  HS_ERR_INVALID_ARG for numbers outside [-1, 11]. */
hs_status hs_tune_gemm_variant(int32_t variant);

/* y = LN(x) over rows of length H; writes mean and reciprocal std per row (stats [2, R] float). */
hs_status hs_op_layernorm_fwd(int32_t dtype, const void* x, const void* gain, const void* bias, void* y,
                              float* stats, int32_t R, int32_t H, float eps, void* stream);
/* dx = LN backward of dy given the saved input x and stats; d_gain/d_bias/d_colsum [H] float get
 * beta * old + (sum over rows of dy*xhat / dy / dx); any of the three may be NULL.
 * partials: dev scratch of hs_op_layernorm_bwd_scratch(R, H) bytes. */
size_t hs_op_layernorm_bwd_scratch(int32_t R, int32_t H);
hs_status hs_op_layernorm_bwd(int32_t dtype, const void* dy, const void* x, const float* stats,
                              const void* gain, void* dx, float* d_gain, float* d_bias, float* d_colsum,
                              float beta, int32_t R, int32_t H, void* partials, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): hs_op_layernorm_bwd with the same arguments, results and kernels, except
 * that the per-block partial column sums go to a 9437184-byte array built into the library (one copy per GPU,
 * held until the process ends) instead of a caller buffer.  Allocates nothing.  Limits: H a multiple of 64 and
 * <= 1024, R <= 2^24 (HS_ERR_SHAPE beyond).  Every call on one GPU uses that GPU's one array: calls that
 * overlap in time on one GPU (different streams or threads) race; order them.  Nothing in the array has to
 * start at zero: a call overwrites what it reads. */
hs_status hs_op_layernorm_bwd_noalloc(int32_t dtype, const void* dy, const void* x, const float* stats,
                                      const void* gain, void* dx, float* d_gain, float* d_bias, float* d_colsum,
                                      float beta, int32_t R, int32_t H, void* stream);

/* Attention over qkv [B*L, 3H] (per row: query | key | value, head h at columns h*64..h*64+63 of
 * each third): ctx [B*L, H], lse [B, A, L] float (log-sum-exp of the scaled, masked scores). */
hs_status hs_op_attention_fwd(int32_t dtype, const void* qkv, const int32_t* lens, int32_t B, int32_t L,
                              int32_t A, void* ctx, float* lse, void* stream);
/* Backward: dqkv [B*L, 3H] from d_ctx, the saved qkv, ctx and lse.  dvec: dev scratch [B, A, L]
 * float.  Rows of padded positions are written as zeros. */
hs_status hs_op_attention_bwd(int32_t dtype, const void* qkv, const void* ctx, const float* lse,
                              const void* d_ctx, const int32_t* lens, int32_t B, int32_t L, int32_t A,
                              void* dqkv, float* dvec, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HETSEQ_HIP_H */
