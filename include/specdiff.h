/*
 * specdiff.h -- C ABI of the MI355X (gfx950) implementation of one Speculative Diffusion
 * Decoding round (arxiv 2408.05636, Algorithm 1).
 *
 * Conventions
 *   - Every function returns an sd_status (0 = SD_OK) unless stated; nothing aborts or throws.
 *   - "host" pointers are ordinary CPU memory owned by the caller; "device" pointers are HIP
 *     device memory of the current device, owned by the caller unless stated otherwise.
 *   - Token ids are int32.  The output vocabulary is [0, vocab); the diffusion drafter's
 *     absorbing [MASK] state has id == vocab and is never an output class.
 *   - Logit / probability rows have a leading dimension ld = sd_vocab_pad(vocab) floats
 *     (vocab rounded up to 256); columns >= vocab are undefined.
 *   - Batches are ragged: sequence b has prefix_len[b] tokens, stored back to back in `prefix`.
 *   - All work is enqueued on the HIP stream given at creation (or per call for the
 *     stand-alone kernels); calls that return host data synchronise that stream.
 *   - Random draws come from Philox4x32-10 keyed by `seed`, counter =
 *     (position k, step j, sequence b, stream) with stream 1 = draft (word 0: reveal decision,
 *     word 1: token sample) and stream 2 = verify (word 0: acceptance, word 1: final token);
 *     a uniform is (word >> 8) * 2^-24.
 */
#ifndef SPECDIFF_H
#define SPECDIFF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sd_status {
    SD_OK = 0,
    SD_ERR_ARG = 1,       /* NULL pointer, non-positive size, unknown enum                         */
    SD_ERR_SHAPE = 2,     /* batch / gamma / length beyond what the handle or the model allows     */
    SD_ERR_TOKEN = 3,     /* a token id outside the vocabulary                                      */
    SD_ERR_STATE = 4,     /* call needs state that is missing (e.g. q of a previous sd_draft)       */
    SD_ERR_WORKSPACE = 5, /* workspace too small or misaligned                                      */
    SD_ERR_HIP = 6        /* a HIP runtime call failed; see sd_last_error                           */
} sd_status;

enum { SD_ARCH_GPT2 = 0, SD_ARCH_LLAMA = 1 };
enum { SD_DTYPE_F32 = 0, SD_DTYPE_BF16 = 1 };

/* Shape of one transformer.  The paper names the model families (Evaluation, Experimental
 * Setup: GPT-2 XL / GPT-Neo / Vicuna targets, MDLM drafter) but not their arithmetic; see
 * the weight inventory below for what each field selects. */
typedef struct sd_model_config {
    int32_t arch;          /* SD_ARCH_GPT2: LayerNorm, biases, tanh-GELU MLP, learned positions
                              SD_ARCH_LLAMA: RMSNorm, no biases, SwiGLU, rotary positions, GQA  */
    int32_t dtype;         /* storage type of matrices / embeddings and of the KV cache         */
    int32_t n_layer, d_model, n_head, n_kv_head, d_ff, vocab, n_ctx;
    int32_t bidirectional; /* 1 = diffusion drafter M_q: non-causal attention, an extra embedding
                              row for [MASK], additive timestep embedding; 0 = causal target M_p */
    float norm_eps;
    float rope_theta;
} sd_model_config;

typedef struct sd_handle sd_handle;

int32_t sd_vocab_pad(int32_t vocab);

/* ---- weight buffer layout (host logic only; no GPU needed) -----------------------------
 * A model's parameters live in ONE device buffer.  Tensor i of sd_weight_count() sits at
 * byte offset `offset` (256-byte aligned), row-major [rows, cols] (cols contiguous; linear
 * layers are stored [out_features, in_features]).  elem_bytes is 4 for gains and biases
 * (always fp32) and 4 or 2 for matrices and embeddings according to dtype (bf16 = upper 16
 * bits of the fp32 pattern).  Names: wte, wpe, t_w1, t_b1, t_w2, t_b2, l<i>.ln1_g, l<i>.ln1_b,
 * l<i>.w_qkv, l<i>.b_qkv, l<i>.w_o, l<i>.b_o, l<i>.ln2_g, l<i>.ln2_b, l<i>.w_fc, l<i>.b_fc,
 * l<i>.w_gate, l<i>.w_up, l<i>.w_proj, l<i>.b_proj, lnf_g, lnf_b, w_head. */
int32_t sd_weight_count(const sd_model_config *cfg);
int32_t sd_weight_desc(const sd_model_config *cfg, int32_t index, char *name, int32_t name_cap,
                       int64_t *rows, int64_t *cols, int32_t *elem_bytes, int64_t *offset);
int64_t sd_weight_bytes(const sd_model_config *cfg);

/* Bytes of device workspace sd_create needs for these models and limits (0 on bad input). */
int64_t sd_workspace_bytes(const sd_model_config *target, const sd_model_config *drafter,
                           int32_t max_batch, int32_t gamma_max);

/* Create a decoder.  target_w / drafter_w: device weight buffers in the layout above,
 * borrowed -- the caller keeps them alive and unchanged.  workspace: device memory,
 * 256-byte aligned, at least sd_workspace_bytes(); borrowed for the handle's lifetime and
 * holding every activation, the target's KV cache and q.  hip_stream: a hipStream_t (NULL =
 * default stream).  The library itself allocates only small pinned host staging buffers. */
int32_t sd_create(const sd_model_config *target, const sd_model_config *drafter,
                  const void *target_w, const void *drafter_w, int32_t max_batch, int32_t gamma_max,
                  void *workspace, int64_t workspace_bytes, void *hip_stream, sd_handle **out);
void sd_destroy(sd_handle *h);
/* Library-owned message describing the last failure on this handle (never NULL); with
 * h == NULL, the reason the last sd_create failed. */
const char *sd_last_error(const sd_handle *h);

/* Fill the target's KV cache for tokens [0, prefix_len[b]-1) of every sequence (prompt
 * processing; Table 1 of the paper costs a round "following the initial prompt", so this is
 * outside the timed round).  prefix, prefix_len: host. */
int32_t sd_prefill(sd_handle *h, int32_t batch, const int32_t *prefix, const int32_t *prefix_len);

/* Algorithm 1, drafting part: start from gamma [MASK] slots, run T reverse-diffusion steps
 * j = T..1 (time j/T), each one bidirectional forward of the drafter over prefix o block,
 * a vocabulary softmax on the block rows and the reveal / categorical-sampling step: a
 * masked slot is revealed at step j with probability 1/j (always at j = 1), its token is
 * drawn by inverse CDF from that step's softmax row, which becomes q_k.
 *   draft_out: host [batch, gamma]; qtok_out: host [batch, gamma] = q_k(x_k), may be NULL;
 *   q_dev_out: receives a device pointer to q, fp32 [batch, gamma, ld], library-owned,
 *   valid until the next sd_draft / sd_round on this handle (NULL at temperature 0, which
 *   produces no q). */
int32_t sd_draft(sd_handle *h, int32_t batch, const int32_t *prefix, const int32_t *prefix_len,
                 int32_t gamma, int32_t T, uint64_t seed, int32_t *draft_out, float *qtok_out,
                 const float **q_dev_out);

/* Algorithm 1, verification part: one causal forward of the target over the last prefix
 * token and the gamma draft tokens against its KV cache (prefilled on demand when the cache
 * does not hold this prefix), giving gamma+1 next-token laws P[0..gamma]; token k is accepted
 * iff r_k * q_k(x_k) <= P[k](x_k) (fp32 product); n = number of leading accepted tokens; the
 * extra token is drawn from norm(max(0, P[n] - q_n)) if n < gamma, else from P[gamma].
 *   draft: host [batch, gamma]; q_dev: device fp32 [batch, gamma, ld];
 *   n_accepted_out, token_out: host [batch]. */
int32_t sd_verify(sd_handle *h, int32_t batch, const int32_t *prefix, const int32_t *prefix_len,
                  int32_t gamma, const int32_t *draft, const float *q_dev, uint64_t seed,
                  int32_t *n_accepted_out, int32_t *token_out);

/* sd_draft followed by sd_verify with the same seed, the draft and q handed over on the
 * device and a single synchronisation at the end.  Same results as the two calls. */
int32_t sd_round(sd_handle *h, int32_t batch, const int32_t *prefix, const int32_t *prefix_len,
                 int32_t gamma, int32_t T, uint64_t seed, int32_t *draft_out,
                 int32_t *n_accepted_out, int32_t *token_out);

/* After sd_verify / sd_round: keep the n accepted tokens.  The target's KV cache then counts the rows of
 * the last prefix token and of draft[0 .. n) as cached, so that the next call whose prefix is
 * old prefix o draft[0 .. n) o token runs without a prefill (multi-round generation: the loop around
 * Algorithm 1).  n_accepted: host [batch], each in [0, gamma].  Without this call the next round with a
 * longer prefix prefills again (correct, only slower).  SD_ERR_STATE if no verification is pending. */
int32_t sd_commit(sd_handle *h, int32_t batch, const int32_t *n_accepted);

/* Temperature 0, the setting of the paper's experiments (Section 4.1): the one-hot limit of Algorithm 1.
 * enable != 0: a slot revealed by the drafter takes the argmax of its row (reveal schedule unchanged;
 * no q is produced, qtok = 1), a drafted token is accepted iff it is the argmax of the target's row,
 * and the extra token is the argmax of row n; seeds only drive the reveal schedule.  Arg-maxima are taken
 * on the fp32 logits, lowest id on ties.  Applies to sd_draft, sd_verify (its q_dev is ignored and may be
 * NULL) and sd_round of this handle until switched off. */
int32_t sd_set_greedy(sd_handle *h, int32_t enable);

/* Leaving out drafting steps that reveal nothing (in the spirit of the cached sampling strategy that the appendix's
 * table of parametric setups names for the drafter, applied to the reveal rule of Algorithm 1's sampling loop).  Which masked slots step j reveals is decided by the
 * seed alone (probability 1/j per slot), and the logits of step j are read by the slots revealed at step j and by
 * nothing else; enable != 0: sd_draft and sd_round replay the reveal schedule on the host and run the drafter only
 * at the steps that reveal at least one slot -- same draft, same q, same verification, fewer forwards (each
 * step is uniformly distributed per slot, so a step is idle with probability (1 - 1/T)^(batch gamma)).  Off by
 * default.  sd_steps_run: drafter forwards of the last sd_draft / sd_round of this handle (T when off). */
int32_t sd_set_step_skipping(sd_handle *h, int32_t enable);
int32_t sd_steps_run(const sd_handle *h);

/* ---- standard speculative decoding (SpS): the paper's baseline and its sequence initialisation ---------------
 * Section 3, "Speculative decoding", and Table 1, row SpS (depth D_p + gamma D_q): the drafter is a small
 * autoregressive model that produces the gamma draft tokens one after the other, x_k ~ q_k = M_q(prefix o x_0 ..
 * x_{k-1}) by inverse CDF with the Philox draw (position k, step 0, sequence b, stream 3) word 1; verification is
 * sd_verify's.  Section 4, "Sequence initialization": the first tokens of a generation are produced this way, the
 * rest with the diffusion drafter -- the caller alternates sd_sps_round and sd_round on one handle (both share the
 * target, its KV cache and sd_commit).
 *
 * sd_sps_attach adds the autoregressive drafter to a handle: a causal model (bidirectional = 0) with the target's
 * vocabulary and storage type whose widths do not exceed the handle's activation buffers (d_model, QKV and MLP widths
 * at most those of the wider of target and diffusion drafter, no more heads, n_ctx * max_batch rows at most; a
 * Llama-shaped one only beside a Llama-shaped target).  sps_w: device weights in the layout of sd_weight_desc, borrowed;
 * workspace: device, 256-byte aligned, sd_sps_workspace_bytes() bytes (its KV cache, folded-norm vectors, row maps),
 * borrowed for the handle's lifetime.  The drafter keeps a KV cache of its own and brings it up to the prefix by itself
 * (only the rows it does not hold yet); sd_commit advances it together with the target's. */
int64_t sd_sps_workspace_bytes(const sd_handle *h, const sd_model_config *sps);
int32_t sd_sps_attach(sd_handle *h, const sd_model_config *sps, const void *sps_w, void *workspace,
                      int64_t workspace_bytes);
/* gamma sequential drafter evaluations.  Outputs as sd_draft: draft_out host [batch, gamma], qtok_out host or NULL,
 * q_dev_out device fp32 [batch, gamma, ld] (NULL at temperature 0, where x_k is the argmax of its row). */
int32_t sd_sps_draft(sd_handle *h, int32_t batch, const int32_t *prefix, const int32_t *prefix_len,
                     int32_t gamma, uint64_t seed, int32_t *draft_out, float *qtok_out,
                     const float **q_dev_out);
/* sd_sps_draft followed by the target pass and the acceptance / residual sampling of sd_verify, one
 * synchronisation at the end.  Same results as the two calls. */
int32_t sd_sps_round(sd_handle *h, int32_t batch, const int32_t *prefix, const int32_t *prefix_len,
                     int32_t gamma, uint64_t seed, int32_t *draft_out, int32_t *n_accepted_out,
                     int32_t *token_out);
/* Parity hook: next-token logits of the autoregressive drafter after each sequence (tokens: host, back to back,
 * seq_len[b] tokens each).  logits_dev_out: device fp32 [batch, ld], library-owned. */
int32_t sd_sps_logits(sd_handle *h, int32_t batch, const int32_t *tokens, const int32_t *seq_len,
                      const float **logits_dev_out);

/* ---- single steps of the path, for parity checks and profiling --------------------------- */

/* One drafter evaluation M_q(prefix o block, t = step/T) (Algorithm 1, loop body).
 * tokens: host, sequences back to back, sequence b = its prefix followed by gamma block
 * slots (ids in [0, vocab], vocab = [MASK]); seq_len[b] includes the gamma block slots.
 * logits_dev_out: device fp32 [batch*gamma, ld], row b*gamma+k = slot k; library-owned. */
int32_t sd_drafter_logits(sd_handle *h, int32_t batch, const int32_t *tokens, const int32_t *seq_len,
                          int32_t gamma, int32_t step, int32_t T, const float **logits_dev_out);

/* The target's parallel scoring M_p(x_{0:i}) .. M_p(x_{0:i+gamma}) (Algorithm 1).
 * logits_dev_out: device fp32 [batch*(gamma+1), ld], row b*(gamma+1)+k = logits of P[k]. */
int32_t sd_target_logits(sd_handle *h, int32_t batch, const int32_t *prefix, const int32_t *prefix_len,
                         int32_t gamma, const int32_t *draft, const float **logits_dev_out);

/* Stand-alone kernels on caller-provided device rows (all pointers device, asynchronous on
 * hip_stream).  scratch: device, sd_sampling_scratch_bytes(rows, vocab) bytes. */
int64_t sd_sampling_scratch_bytes(int32_t rows, int32_t vocab);

/* Reveal / sample step j of the drafting loop on logits [batch*gamma, ld]:
 * for every slot with z == vocab ([MASK]) that is revealed at this step, z <- token,
 * q row <- softmax row, qtok <- its probability; other slots are left untouched. */
int32_t sd_unmask_sample(const float *logits, int32_t batch, int32_t gamma, int32_t vocab,
                         int32_t step, uint64_t seed, int32_t *z, float *q, float *qtok,
                         void *scratch, int64_t scratch_bytes, void *hip_stream);

/* Acceptance, first rejection and residual / bonus sampling on target logits
 * [batch*(gamma+1), ld], q [batch*gamma, ld] and draft [batch, gamma];
 * writes n_accepted[batch] and token[batch]. */
int32_t sd_accept_resample(const float *p_logits, const float *q, const int32_t *draft,
                           int32_t batch, int32_t gamma, int32_t vocab, uint64_t seed,
                           int32_t *n_accepted, int32_t *token,
                           void *scratch, int64_t scratch_bytes, void *hip_stream);

/* sd_accept_resample for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results, no scratch
 * argument: the partial row statistics live in a fixed buffer of sd_static_scratch_bytes() bytes (4 MiB) that the
 * library holds in device memory on every GPU it runs on, for the life of the process.  The call allocates nothing
 * (no hipMalloc / hipFree, no staging copy: the seed travels as a kernel argument) and is asynchronous on
 * hip_stream.  Shapes whose statistics do not fit, i.e. sd_sampling_scratch_bytes(batch * (gamma + 1), vocab) >
 * sd_static_scratch_bytes(), are rejected with SD_ERR_WORKSPACE (text in sd_last_error(NULL)); nothing is launched
 * then.  All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU (two streams, two
 * threads) race and give undefined results; calls on one stream, or otherwise ordered, are fine.  The call clears the
 * few counters that must start at zero itself (a fill kernel, no memset); nothing is kept between calls. */
int64_t sd_static_scratch_bytes(void);
int32_t sd_accept_resample_static(const float *p_logits, const float *q, const int32_t *draft,
                                  int32_t batch, int32_t gamma, int32_t vocab, uint64_t seed,
                                  int32_t *n_accepted, int32_t *token, void *hip_stream);

/* y = epilogue(x W^T + bias): the dense contraction used by every QKV / MLP / LM-head layer.
 * x: [m, k] (dtype), w: [n, k] (dtype), bias: fp32 [n] or NULL.
 * epilogue 0: y (dtype) = acc; 1: y (dtype) = gelu_tanh(acc); 2: y (fp32) += acc (residual);
 * 3: y (fp32) = acc.  ldy in elements of y.
 * split_workspace: device, 256-byte aligned, or NULL.  With few rows (the target's gamma + 1 query
 * rows) the K range of an output tile is divided over several workgroups, which needs memory for their
 * partial sums: the first sd_linear_split_ticket_bytes() bytes are counters that must be zero before
 * the first call (every call leaves them zero), the rest holds partial tiles; a larger workspace allows
 * a finer split, NULL none.  Calls that share a workspace must not overlap.  Results are deterministic
 * (partials are added in a fixed order). */
int64_t sd_linear_split_ticket_bytes(void);
int32_t sd_linear(int32_t dtype, const void *x, const void *w, const float *bias, void *y,
                  int32_t m, int32_t n, int32_t k, int32_t ldy, int32_t epilogue,
                  void *split_workspace, int64_t split_workspace_bytes, void *hip_stream);

/* y = epilogue(W norm(h) + bias): the normalisation in front of a contraction folded into it, as the
 * forwards of bf16 models do it.  norm_kind 1: LayerNorm(h; gain, beta, eps), 2: RMSNorm(h; gain, eps).
 * The A operand is bf16(h * gain) and the row sums of h are prepared by a row kernel (inside a forward: by
 * the kernel that wrote h), the contraction applies mean and variance in its epilogue:
 *   y_n = rstd_m (acc_mn - mu_m u_n) + v_n,  u = W gain,  v = W beta + bias   (RMSNorm: mu = 0, v = bias).
 * h: fp32 [m, k] (the residual stream), w: bf16 [n, k], gain / beta: fp32 [k], bias: fp32 [n] or NULL,
 * epilogue 0, 1 or 3 as in sd_linear.  fold_scratch: device, 256-byte aligned,
 * sd_norm_linear_scratch_floats(m, n, k) floats (receives u, v, the row sums and the bf16 operand).
 * split_workspace as in sd_linear.  All pointers device; asynchronous. */
int64_t sd_norm_linear_scratch_floats(int32_t m, int32_t n, int32_t k);
int32_t sd_norm_linear(int32_t norm_kind, const float *h, const void *w, const float *gain, const float *beta,
                       const float *bias, void *y, int32_t m, int32_t n, int32_t k, int32_t ldy, int32_t epilogue,
                       float eps, float *fold_scratch, void *split_workspace, int64_t split_workspace_bytes,
                       void *hip_stream);

/* The producer side of a folded normalisation (bf16 weights): y (fp32 [m, n], the residual stream) += x W^T + bias
 * as sd_linear's epilogue 2, and for the normalisation that follows: xg (bf16 [m, n]) = bf16(y * gain) and
 * stats (fp32 [m, ceil(n/32), 2]) = per row and 32-column tile the sums of y and of y^2 over the tile's columns.
 * gain: fp32 [n].  split_workspace as in sd_linear.  All pointers device; asynchronous. */
int32_t sd_linear_resid_norm(const void *x, const void *w, const float *bias, float *y, const float *gain,
                             void *xg, float *stats, int32_t m, int32_t n, int32_t k,
                             void *split_workspace, int64_t split_workspace_bytes, void *hip_stream);

/* Tuning hook for sd_linear and every contraction inside the forwards: force tile variant
 * `variant` of the matrix-core kernel (0, 3, 5, 6: few-row / mid-size tiles; 7, 8: workgroup-shared 128 x 128, 64 x 128 tiles;
 * 9: the weight-streaming kernel for up to 64 rows wherever the shape fits it, the choice by shape elsewhere;
 * 10-13: 64 x 64, 64 x 128, 128 x 128, 256 x 128 tiles fed straight from global memory into a ring of LDS stages, 14, 15: the
 * first two with two 64-wide chunks of K per stage -- the choice by shape when K is shorter than the ring or no multiple of
 * the stage width; see the kernel sources; other values are rejected at the next contraction), -1 = choose by shape (default).
 * Process-wide (captured launch sequences are keyed by it, so a change takes effect at the next call); results do not
 * depend on the variant beyond fp32 summation order. */
int32_t sd_set_linear_variant(int32_t variant);
/* Same for the number of workgroups that share the K range of one output tile (clamped to what the
 * shape and the workspace allow); <= 0 = choose by shape (default). */
int32_t sd_set_linear_split(int32_t split);

/* The launch sequences of sd_draft / sd_verify / sd_round are captured into HIP graphs on first
 * use (one per combination of batch, gamma, T and sequence lengths) and replayed afterwards; the
 * results are identical to eager launches.  (A sequence is launched eagerly the first time it is seen
 * and captured the second time.)  enable = 0 turns replay off (it is also off while
 * profiling and when the handle runs on the NULL stream). */
int32_t sd_set_graph_replay(sd_handle *h, int32_t enable);
/* What became of the launch sequences of this handle since creation: replays = sequences sent as a graph replay;
 * failures = captures or instantiations that failed (the first failure switches replay off for the handle: results
 * stay correct, every sequence is launched eagerly from then on); eager_after_failure = sequences launched eagerly
 * because of that; captured = graphs currently held.  Any pointer may be NULL.  sd_graph_error: library-owned text
 * naming the call that failed ("" if none).  A caller that times rounds checks failures == 0. */
int32_t sd_graph_stats(const sd_handle *h, int64_t *replays, int64_t *eager_after_failure, int32_t *failures,
                       int32_t *captured);
const char *sd_graph_error(const sd_handle *h);

/* ---- per-kernel timing ----------------------------------------------------------------------
 * Between sd_profile_begin and sd_profile_end every kernel of the handle is launched with a pair of HIP events on
 * its stream that receive the kernel's own start and end of execution (hipExtLaunchKernelGGL), and launch
 * sequences run eagerly instead of as graph replays; entries accumulate, per part of the round and kernel name
 * ("draft:", "verify:" or "accept:" followed by the name; the bare name for launches outside a round), the launch
 * count, the summed kernel milliseconds (gaps between kernels are not in them) and the summed algorithmic bytes
 * and flops of those launches (operands read once, results written once).  The eager launches are slower than
 * a replay: time a round without profiling.  One handle of the process profiles at a time.
 * name: caller buffer of name_cap bytes. */
int32_t sd_profile_begin(sd_handle *h);
int32_t sd_profile_end(sd_handle *h);
int32_t sd_profile_count(const sd_handle *h);
int32_t sd_profile_entry(const sd_handle *h, int32_t index, char *name, int32_t name_cap, int64_t *launches,
                         double *total_ms, double *bytes, double *flops);

#ifdef __cplusplus
}
#endif
#endif /* SPECDIFF_H */
