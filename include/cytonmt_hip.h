/* cytonmt_hip.h — C ABI of the MI355X (gfx950) training-step library.
 *
 * One call of cmt_train_step runs one full training step (forward + backward) of the
 * attention-based stacked-LSTM encoder-decoder of the paper's Method section (Eq. 1-7):
 * bidirectional bottom encoder layer, input-feeding decoder, multiplicative ("general")
 * attention, attentional tanh layer H_o = tanh(W_c [C_s; H_t]), and the vocabulary projection
 * with log-softmax cross-entropy of Eq. 1.  Every step of the path runs in hand-written HIP
 * kernels; the host side only validates arguments and enqueues launches.
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary host memory.
 *   - The caller owns every device buffer (parameters, gradients, workspace, ids, lengths) and
 *     the HIP stream; the library owns only the host-side handle, a few bytes of pinned host
 *     memory, one internal non-blocking stream of default priority and a pool of events.  It
 *     never allocates or frees device memory.
 *   - All work is ordered on the stream given to cmt_create: inside a training step the
 *     library forks work that is off the recurrences' critical path onto its internal stream
 *     and joins it back before the step's last kernel, so whatever the caller enqueues on its
 *     stream afterwards sees the finished step.  Calls that return data to host memory
 *     synchronise that stream before returning.  Environment variable CMT_SIDE_STREAM=0 (read
 *     in cmt_create) keeps everything on the caller's stream.
 *   - Every function returns CMT_OK (0) or a negative error code; nothing throws or aborts
 *     across this boundary.  cmt_last_error gives the text of the last failure on a handle.
 *   - Matrices are row-major [out, in].  Flat parameter / gradient vectors are fp32 in the
 *     canonical order listed at cmt_param_info.
 */
#ifndef CYTONMT_HIP_H
#define CYTONMT_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CMT_OK          0
#define CMT_EINVAL     -1   /* null pointer, bad shape, B/S/T beyond the configured maxima        */
#define CMT_ERANGE     -2   /* a token id outside [0, vocab) or a length outside [1, S] / [1, T]   */
#define CMT_ENONFINITE -3   /* the loss came out NaN or Inf                                        */
#define CMT_EHIP       -4   /* a HIP runtime call failed                                           */

/* Network shape (hyperparameter table of the paper: embedding size, hidden size, depth,
 * bidirectional encoder, LSTM) and the largest batch the workspace must hold. */
typedef struct cmt_config {
  int32_t src_vocab, tgt_vocab;  /* vocabulary sizes; both multiples of 8                          */
  int32_t emb_dim;               /* embedding size, multiple of 8                                   */
  int32_t hidden;                /* hidden size H, multiple of 16, at most 1024; the bottom encoder */
                                 /* layer is two LSTMs of width H/2                                 */
  int32_t layers;                /* encoder depth = decoder depth, 1..8                             */
  int32_t max_batch, max_src_len, max_tgt_len;
  int32_t precision;             /* 0: fp32 storage and fp32 matrix cores; 1: bf16 operands with    */
                                 /* fp32 accumulation, fp32 master weights, fp32 state and sums     */
  int32_t bos_id, pad_id;        /* decoder input at step 0; id stored in padded slots              */
} cmt_config;

typedef struct cmt_handle cmt_handle;

/* Bytes the caller must provide: flat fp32 parameters, flat fp32 gradients, workspace.
 * Returns CMT_EINVAL for a configuration the kernels do not support. */
int cmt_query_sizes(const cmt_config* cfg, size_t* param_bytes, size_t* grad_bytes, size_t* workspace_bytes);

/* Binds caller-owned device buffers (each 256-byte aligned, sizes from cmt_query_sizes) and a
 * HIP stream (hipStream_t passed as void*; NULL = the default stream).  The buffers must stay
 * alive until cmt_destroy.  Parameters are uninitialised until cmt_init_params / cmt_set_params. */
int cmt_create(const cmt_config* cfg, void* params_dev, void* grads_dev, void* workspace_dev,
               void* hip_stream, cmt_handle** out);
/* Releases the handle, its pinned host memory, its internal stream and events (it waits for the
 * internal stream first).  The caller synchronises its own stream before freeing the device buffers
 * that asynchronous calls may still be using.  NULL is accepted. */
void cmt_destroy(cmt_handle* h);

/* Parameter table.  Canonical order: E_src[Vs,E], E_tgt[Vt,E], enc.l0.fwd.W[4Hd,E+Hd], .b[4Hd],
 * enc.l0.bwd.W, .b, enc.l{1..}.W[4H,2H], .b[4H], dec.l0.W[4H,E+2H] (columns [emb; H_o feed; h]),
 * .b, dec.l{1..}.W[4H,2H], .b, W_a[H,H], W_c[H,2H] (columns [C_s; H_t]), W_o[Vt,H], B_o[Vt].
 * LSTM weight rows are the gate blocks i, f, g, o; columns are [input; recurrent].
 * name points into the handle (valid until cmt_destroy); cols = 1 for vectors. */
int cmt_param_count(const cmt_handle* h);
int cmt_param_info(const cmt_handle* h, int idx, const char** name, int64_t* rows, int64_t* cols,
                   size_t* offset_elems);

/* uniform[-scale, scale) from a counter-based generator: flat element n takes the top 24 bits u
 * of SplitMix64(seed + n) and becomes (u * 2^-23 - 1) * scale in fp32.  Device-side. */
int cmt_init_params(cmt_handle* h, uint64_t seed, float scale);
/* Copy the whole flat fp32 parameter vector from / to host memory. */
int cmt_set_params(cmt_handle* h, const float* host_src);
int cmt_get_params(cmt_handle* h, float* host_dst);

/* One training step (Eq. 1-7 forward, then the gradient of the mean cross-entropy).
 *   src_ids_dev [B,S] row-major int32, src_len_dev [B] int32 in [1,S],
 *   tgt_ids_dev [B,T] row-major int32, tgt_len_dev [B] int32 in [1,T]  (device memory, read only).
 * The decoder runs tgt_len[b] steps: its input at step j is bos_id for j = 0, else tgt_ids[b,j-1];
 * the label at step j is tgt_ids[b,j].  Slots beyond a length are ignored.
 * On return the gradient buffer holds d(loss)/d(parameter) for every parameter (overwritten, not
 * accumulated; rows of unused embedding ids are zero) and *loss_host the mean cross-entropy per
 * valid target token.  Synchronises the stream.  Parameters are never modified.
 * CMT_ERANGE / CMT_ENONFINITE leave the gradient buffer undefined. */
int cmt_train_step(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev,
                   const int32_t* tgt_ids_dev, const int32_t* tgt_len_dev,
                   int32_t B, int32_t S, int32_t T, float* loss_host);
/* Same work, but only enqueues it: no synchronisation, no error-flag or loss read-back.  The loss of
 * the last enqueued step is fetched (with a synchronisation) by cmt_fetch_loss.  The error flags are
 * sticky: cmt_fetch_loss reports CMT_ERANGE / CMT_ENONFINITE if ANY step enqueued since the previous
 * read-back raised one, and clears them; until then cmt_sgd_update applies nothing (the gradients of
 * a failed step are undefined), so parameters stay as they were before the failed step. */
int cmt_train_step_async(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev,
                         const int32_t* tgt_ids_dev, const int32_t* tgt_len_dev,
                         int32_t B, int32_t S, int32_t T);
int cmt_fetch_loss(cmt_handle* h, float* loss_host);

/* The forward half of a step only (Eq. 1-7, no gradient): the development-set cross-entropy that
 * the training procedure of the Settings section monitors.  Arguments as for cmt_train_step.
 * Evaluation mode: no dropout and no label smoothing, whatever cmt_set_regularization says.
 *   *loss_host  mean cross-entropy per valid target token of this batch,
 *   *n_tok_host the number of valid target tokens (sum of tgt_len), so that a caller can average
 *               over several batches; either may be NULL.
 * Synchronises the stream.  Parameters and the gradient buffer are untouched; the intermediates of
 * the last training step are overwritten.  Errors as for cmt_train_step. */
int cmt_eval_loss(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev,
                  const int32_t* tgt_ids_dev, const int32_t* tgt_len_dev,
                  int32_t B, int32_t S, int32_t T, float* loss_host, float* n_tok_host);

/* cmt_eval_loss for callers that cannot provide (or allocate) a workspace for the call: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same result
 * (the same kernels in the same order), but every intermediate — including the working copies of the
 * parameters, which are rebuilt on each call — lives in one array of CMT_STATIC_SCRATCH_BYTES that is
 * part of the library's device code, laid out for exactly this call's B, S and T; the handle's
 * workspace, its last step's intermediates and the gradient buffer are untouched.  The call allocates
 * and frees nothing.  A shape whose intermediates do not fit is refused with CMT_EINVAL (cmt_last_error
 * names both sizes): the tiny configuration (hidden 64, vocabulary 1000, 8 x 10 tokens) needs about
 * 20 MB.  Each GPU holds one such array until the process ends, shared by all handles; it keeps the last
 * call's contents and is cleared at the start of each call.  Calls that overlap on one GPU — from
 * several handles, streams or threads — race on it: serialise them.  Like cmt_eval_loss it leaves its
 * own loss in the handle's pinned read-back slot (what a later cmt_fetch_loss returns). */
#define CMT_STATIC_SCRATCH_BYTES (32u << 20)
int cmt_eval_loss_static(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev,
                         const int32_t* tgt_ids_dev, const int32_t* tgt_len_dev,
                         int32_t B, int32_t S, int32_t T, float* loss_host, float* n_tok_host);

int cmt_get_grads(cmt_handle* h, float* host_dst);

/* Regularisation of the training step (Settings section; hyperparameter table: dropout 0.2, label
 * smoothing 0.1).  Both are off (0) after cmt_create; the values set here apply to every later step.
 *   dropout p in [0, 1): the hidden states a recurrent layer hands to the layer above it (encoder
 *     and decoder, all layers but the top one) and the output H_o (as seen by the output layer and
 *     by the next step's input feed) are multiplied by keep / (1 - p).  Element (t, b, h) of dropout
 *     site s is kept iff the top 24 bits of SplitMix64(dropout_seed + s * 2^48 + (t * B + b) * H + h)
 *     are >= floor(p * 2^24); s = l for the encoder layer l output, 16 + l for the decoder layer l
 *     output, 32 for H_o; B is the step's batch size, H = hidden.  Nothing is stored: forward and
 *     backward recompute the decision.  The caller changes dropout_seed from step to step.
 *   label_smoothing eps in [0, 1): the target distribution of Eq. 1 becomes
 *     (1 - eps) onehot(y) + eps / V; the loss returned is the cross-entropy against it.
 * Returns CMT_EINVAL for values outside those ranges (the previous setting is kept). */
int cmt_set_regularization(cmt_handle* h, float dropout, float label_smoothing, uint64_t dropout_seed);

/* Forward-only translation with beam size 1 (the hyperparameter table's beam search reduced to its
 * first hypothesis): the encoder as in a training step, then max_len decoder steps in which the input
 * token is bos_id at step 0 and the previous output token afterwards, and the output token is
 * argmax_v (W_o H_o + B_o)_v, the lowest index winning a tie.  A sentence ends with the step that emits
 * eos_id (which is kept) or at step max_len - 1.  No dropout, whatever cmt_set_regularization says.
 *   src_ids_dev [B, S] int32 row-major, src_len_dev [B]: as for cmt_train_step (device pointers).
 *   out_ids_dev [B, max_len] int32 (device): the tokens, pad_id after a sentence's end;
 *   out_len_dev [B] int32 (device): tokens emitted per sentence, in [1, max_len].
 * 1 <= max_len <= max_tgt_len.  Synchronises the stream.  Overwrites the intermediates of the last
 * training step (cmt_debug_fetch needs a new step afterwards); parameters and gradients are untouched.
 * Errors: CMT_EINVAL (shape / pointer / eos_id), CMT_ERANGE (source id or length out of range). */
int cmt_greedy_decode(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev, int32_t B, int32_t S,
                      int32_t max_len, int32_t eos_id, int32_t* out_ids_dev, int32_t* out_len_dev);

/* Beam search (hyperparameter table: beam search size 10, length penalty 0.6; the Settings section
 * names the length normalisation of Wu et al. 2016: lp(Y) = ((5 + |Y|) / 6) ^ length_penalty).
 * The decoder runs on B * beam rows, one per hypothesis, so B * beam <= max_batch is required.
 * A hypothesis carries the sum of log p(token) of its tokens.  At every step the `beam` best
 * one-token extensions over a sentence's live hypotheses are taken (equal scores: the lower
 * (hypothesis slot, token) pair first); an extension ending in eos_id leaves the beam as a finished
 * hypothesis of length = its token count (eos included), the others stay live, best first.  A
 * sentence is done when no hypothesis is live or after max_len steps (hypotheses still live then
 * are finished as they are).  Returned per sentence: the finished hypothesis with the largest
 * score / lp(length) (equal values: the one finished first).  No dropout.
 *   out_ids_dev [B, max_len] int32, pad_id after the end; out_len_dev [B] int32; out_score_dev [B]
 *   fp32 normalised scores (all device pointers).  1 <= beam <= 16, 1 <= max_len <= max_tgt_len
 *   (max_tgt_len >= 2).  Scores are accumulated in fp32.  Synchronises the stream; overwrites the
 *   intermediates of the last training step.  Errors as for cmt_greedy_decode. */
int cmt_beam_decode(cmt_handle* h, const int32_t* src_ids_dev, const int32_t* src_len_dev, int32_t B, int32_t S,
                    int32_t max_len, int32_t beam, float length_penalty, int32_t eos_id, int32_t* out_ids_dev,
                    int32_t* out_len_dev, float* out_score_dev);

/* Plain SGD (hyperparameter table: optimizer SGD, learning rate 1.0): p <- p - lr * g on the flat
 * fp32 master vector, then refreshes the kernels' working copies (bf16 casts, transposes).  The
 * update is skipped on the device while an error flag of an earlier step is pending (see
 * cmt_train_step_async). */
int cmt_sgd_update(cmt_handle* h, float lr);

/* Copies a named intermediate of the last step to host memory as fp32, for per-kernel parity
 * tests.  Names: "x_src" [S,Bp,E], "x_tgt" [T,Bp,E], "mask_src" [S,Bp], "mask_tgt" [T,Bp],
 * "h_s" [S,Bp,H], "h_t" [T,Bp,H], "att_a" [T,Bp,S], "att_cs" [T,Bp,H], "h_o" [T,Bp,H] (before
 * dropout), "h_o_drop" [T,Bp,H] (after), "lse" [T,Bp], "nll" [T,Bp] (the per-token loss), "att_s" [T,Bp,S]
 * (the scores F_a of Eq. 4 before the softmax; training step only), and per LSTM "enc.l0.fwd", "enc.l0.bwd"
 * (width H/2), "enc.l<k>" (k >= 1), "dec.l<k>": "<lstm>.h" and "<lstm>.c" [len,Bp,width] (the state after every
 * step, a padded step carrying the previous state) and "<lstm>.gates" [len,Bp,4 width] (gate activations
 * i, f, g, o of every step), len = S or T; Bp = B rounded up to a multiple of 16 (extra rows are padding).
 * bytes must equal the tensor's size; values at masked positions are unspecified except for
 * the masks, "att_a" (exactly 0 on padded source positions) and "nll" (0 on padded targets). */
int cmt_debug_fetch(cmt_handle* h, const char* name, float* host_dst, size_t bytes);
/* Padded batch pitch Bp used by cmt_debug_fetch for the last step. */
int cmt_padded_batch(const cmt_handle* h);

/* Measurement aid: launches one kernel of the last step `iters` times back to back on the handle's
 * stream, with the operands that step used, timed by HIP events (the forward kernels rewrite their results
 * with identical values; the backward replays update the state gradients they find in place, which changes
 * those values, not the timing: run a step before using gradients again).  Returns the mean microseconds per launch and the algorithmic work of one launch:
 * bytes (operands read once, outputs written once) for the bandwidth-bound kernels, flops
 * (2 per multiply-add) for the matrix-core-bound ones.  Names:
 *   "lstm_fwd_dec"   fused decoder LSTM step (gate GEMM + cell), cycling over the layers   bytes
 *   "step2d_bwd_dec" [dx; dh] = dgates [W_x; W_h] of a decoder layer's backward step       bytes
 *   "att_fwd"        attention forward of one decoder step as the step runs it: below 256 sentences the scores
 *                    (with the H_t half of the attentional layer's product in the same launch), then softmax,
 *                    mix of the projected source rows and tanh -> H_o; else scores + softmax + context     bytes
 *   "att_bwd"        attention backward of one decoder step as the step runs it (with the top layer's cell; in
 *                    the fused loop below 256 sentences also the product dpre W_c, whose launch carries the
 *                    score gradients)                                                      bytes
 *   "gemm_gx"        time-batched input-side GEMM [T Bp, E] x [E, 4H]                      flops
 *   "gemm_dw"        the decoder's weight-gradient GEMMs (W_c and every layer, k = T Bp), one grouped launch  flops
 *   "ce_fwd"         vocabulary projection + log-sum-exp partials of the first slab of rows flops
 *   "step_bwd_fused_dec" the same product as step2d_bwd_dec in the form the decoder's backward loop runs:
 *                    whole contraction per workgroup, cell backward of the layer below in the epilogue bytes
 *   "grid_barrier", "grid_barrier_nofence"  100 chip-wide barriers between 256 resident workgroups, with /
 *                    without device-scope fences (bounded polling; what a persistent recurrence would pay
 *                    per time step); work = the number of barriers
 *   "mfma_rate"      matrix-core instructions alone (bf16 32x32x16 on registers): the rate the chip's
 *                    matrix cores reach, to be read beside the nominal peak                 flops
 * The replays of the backward kernels leave the in-place state gradients of the last step in whatever
 * state they reach; the next step re-initialises them.  Synchronises the stream. */
int cmt_time_kernel(cmt_handle* h, const char* name, int iters, float* us_per_launch, double* algo_work);

const char* cmt_last_error(const cmt_handle* h);

#ifdef __cplusplus
}
#endif
#endif
