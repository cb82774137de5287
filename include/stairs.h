/*
 * stairs.h -- C ABI of the MI355X (gfx950) library for "stairs" assisted greedy generation.
 *
 * The method (paper Sec. 3.3): an assistant ("draft") model greedily generates k tokens; the
 * current sequence S (length L) is turned into the k+1 "stair" rows S, S+d_1, ..., S+d_1..d_k;
 * the main ("target") model predicts one more token for every row in one batched iteration;
 * "stairs" validation keeps the first row's prediction and every following row's prediction as
 * long as the row equals the running ground truth, i.e. as long as d_i == t_{i-1}.  The output
 * is the one the target alone would generate greedily (abstract, Sec. 3.1).
 *
 * On the GPU the stair batch is one causal forward of the k+1 new rows [S[L-1], d_1..d_k]
 * against the target's key/value cache: its k+1 output rows are exactly the last-position
 * logits of the k+1 stair rows.
 *
 * Conventions
 *  - Every function returns 0 (STAIRS_OK) or a negative error code; nothing throws across the
 *    ABI.  stairs_last_error() gives the text of the last failure of a context.
 *  - Pointers are HOST pointers unless the argument is documented "host or device".
 *  - The caller owns every buffer it passes; the library copies what it needs during the call
 *    and keeps no reference afterwards.  The library owns the context and everything in it.
 *  - One context serves one sequence at a time and is not thread-safe.
 *  - All device work is issued on the HIP stream given to stairs_init (NULL = default stream)
 *    on the device current at that time.  Calls return after their device work has finished
 *    unless stated otherwise.
 */
#ifndef STAIRS_H
#define STAIRS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define STAIRS_OK          0
#define STAIRS_EINVAL     (-1)   /* bad argument or unsupported model shape               */
#define STAIRS_ECAPACITY  (-2)   /* sequence would exceed max_seq                          */
#define STAIRS_ESTATE     (-3)   /* call order (e.g. verify before prefill / propose)      */
#define STAIRS_ENOMEM     (-4)   /* host or device allocation failed                       */
#define STAIRS_EHIP       (-5)   /* a HIP runtime call or kernel launch failed             */

#define STAIRS_DTYPE_FP32  0     /* matrices are float                                     */
#define STAIRS_DTYPE_BF16  1     /* matrices are bfloat16 bit patterns (uint16_t)          */

#define STAIRS_MAX_ROWS    32    /* most rows one forward takes: k + 1 <= STAIRS_MAX_ROWS  */
#define STAIRS_MAX_BATCH        128   /* most sequences stairs_reserve_batch makes room for          */
#define STAIRS_MAX_STREAM_ROWS  64    /* most rows of several sequences the weight-streaming kernels take */
#define STAIRS_MAX_BATCH_ROWS   256   /* most rows one forward of several sequences takes            */

/* Shape of one decoder-only pre-RMSNorm transformer (RoPE in the rotate-half pairing
 * (i, i + head_dim/2), SwiGLU feed-forward, no biases, untied embedding / unembedding).
 * Supported: head_dim = d_model / n_heads in {64, 128}; bf16 models need d_model and d_ffn
 * to be multiples of 256 and vocab, 3*d_model, 2*d_ffn multiples of 16; fp32 models need
 * d_model, d_ffn multiples of 4. */
typedef struct {
  int32_t n_layers, d_model, n_heads, d_ffn, vocab;
  int32_t max_seq;        /* most positions the key/value cache must hold                  */
  float rope_theta;       /* e.g. 10000                                                     */
  float rms_eps;          /* e.g. 1e-5                                                      */
  int32_t dtype;          /* STAIRS_DTYPE_*: type of the matrices AND of the KV cache       */
} stairs_model_cfg;

/* Host pointers to the weights.  Matrices are [out_features, in_features] row-major in
 * cfg.dtype; norm gains are float[d_model].  The per-layer members point to arrays of
 * n_layers pointers.  Two models may share tensors (same host address): the library keeps
 * one device copy per distinct address. */
typedef struct {
  const void *tok_emb;          /* [vocab, d_model] */
  const void *lm_head;          /* [vocab, d_model] */
  const float *final_norm;      /* [d_model]        */
  const float *const *attn_norm;
  const void *const *wq, *const *wk, *const *wv, *const *wo;   /* [d, d]             */
  const float *const *ffn_norm;
  const void *const *w_gate, *const *w_up;                     /* [d_ffn, d_model]   */
  const void *const *w_down;                                   /* [d_model, d_ffn]   */
} stairs_weights;

typedef struct {
  int32_t iterations;           /* target iterations (stair batches) run                   */
  int32_t tokens;               /* tokens produced (= G unless an end token stopped it)    */
  int64_t accepted;             /* assistant tokens kept, summed over iterations           */
  float ms_prefill;             /* prompt ingestion, both models                           */
  float ms_decode;              /* everything after prefill until the last token           */
  float ms_draft;               /* part of ms_decode spent in the draft's k-step proposals */
  float ms_verify;              /* part of ms_decode spent in stair verification + accept  */
  int32_t accept_hist[STAIRS_MAX_ROWS + 1];   /* accept_hist[n] = iterations that kept n   */
} stairs_stats;

/* Environment variables read by the library (all optional; for measurements and tests, never needed in use):
 *   STAIRS_NO_GRAPH=1          launch every kernel one by one instead of replaying captured iterations
 *   STAIRS_NO_BLOCK_PREFILL=1  ingest prompts with the decode kernels, 32 rows per forward (read at stairs_init)
 *   STAIRS_SYNC_LAUNCHES=1|2   wait after every kernel (counter-collecting profilers); 1 also ingests prompts with
 *                              the decode kernels, 2 keeps the block kernels
 *   STAIRS_WIDE_CFG, STAIRS_ROWS_MAX, STAIRS_ROWS_TPW   launch shapes of the GEMM kernels (tuning aids, read once per
 *                              process; results are bit-identical whatever they say) */
typedef struct stairs_ctx stairs_ctx;   /* opaque */

const char *stairs_strerror(int code);
const char *stairs_last_error(const stairs_ctx *ctx);

/* Build a context: upload both models, re-lay the matrices out for the kernels, allocate the
 * KV caches (max_seq positions each) and workspaces.  dcfg/dw may be NULL (no assistant; only
 * k = 0 is then legal, which is plain greedy generation of the target -- the paper's
 * "batch size 1", Sec. 4.3).  k_max: largest draft length that will be used, 0 <= k_max <
 * STAIRS_MAX_ROWS.  Both models must have the same vocab.  hip_stream: a hipStream_t or NULL.
 * Errors: EINVAL (shapes, NULLs), ENOMEM, EHIP.  On error *out is NULL. */
int stairs_init(stairs_ctx **out, const stairs_model_cfg *tcfg, const stairs_weights *tw,
                const stairs_model_cfg *dcfg, const stairs_weights *dw, int32_t k_max,
                void *hip_stream);

void stairs_free(stairs_ctx *ctx);

/* Start a new sequence S = prompt[0..P) (the text both models start from, Sec. 3.3 first
 * paragraph): both models ingest prompt[0..P-2] into their KV caches; the last prompt token is
 * the first row of the first stair batch.  Prompts of 64 rows and more are ingested in blocks of
 * up to 2048 rows (bf16 models; the library's own MFMA block GEMM on the same weight tiles the
 * decode kernels read), shorter ones with the decode kernels.  Requires 1 <= P and
 * P + k_max + 1 <= max_seq of both models.
 * Errors: EINVAL (NULL, P < 1, token id outside [0, vocab)), ECAPACITY. */
int stairs_prefill(stairs_ctx *ctx, const int32_t *prompt, int32_t P);

/* Sec. 3.3, first step: the assistant greedily generates d_1..d_k after the current S.
 * draft_out: k ints or NULL.  Must be followed by stairs_verify with the same k before the
 * next draft_propose.  1 <= k <= k_max.  Errors: EINVAL, ESTATE (no prefill, or a proposal is
 * already pending, or no draft model), ECAPACITY. */
int draft_propose(stairs_ctx *ctx, int32_t k, int32_t *draft_out);

/* Sec. 3.3, stair batch + validation: score the k+1 stair rows built from the pending
 * proposal (k = 0: no proposal needed, one plain greedy step), take the per-row argmax
 * t_0..t_k (ties -> lowest token id), keep n = max{ n : d_i == t_{i-1}, i <= n } assistant
 * tokens, append t_0..t_n to S and roll both KV caches back to the accepted length.
 * target_tok_out: k+1 ints or NULL.  n_accepted_out: 1 int or NULL.  logits_out: host or
 * device buffer of (k+1)*vocab floats (row i = stair row i's next-token logits) or NULL.
 * Errors: EINVAL, ESTATE (k > 0 without a pending proposal of the same k), ECAPACITY. */
int stairs_verify(stairs_ctx *ctx, int32_t k, int32_t *target_tok_out, int32_t *n_accepted_out,
                  float *logits_out);

/* Same as stairs_verify but the assistant tokens d_1..d_k are given by the caller (tests:
 * forced acceptance / rejection, replaying another implementation's trace).  Any pending
 * proposal is discarded; the draft model's cache is brought up to date lazily by its next
 * proposal.  0 <= k <= k_max.  Token ids outside [0, vocab) -> EINVAL. */
int stairs_verify_tokens(stairs_ctx *ctx, const int32_t *draft, int32_t k, int32_t *target_tok_out,
                         int32_t *n_accepted_out, float *logits_out);

/* Whole loop (the iteration of Sec. 3.3 repeated until the answer is complete, Sec. 3.2; the
 * synthetic models have no end token, so here: until exactly G tokens exist): prefill, then
 * propose / verify until G tokens are produced; the last iteration is truncated to G.  tokens_out: G ints.  stats: optional.
 * Requires P + G + k + 1 <= max_seq.  k = 0 is plain greedy generation of the target. */
int stairs_generate(stairs_ctx *ctx, const int32_t *prompt, int32_t P, int32_t G, int32_t k,
                    int32_t *tokens_out, stairs_stats *stats);

/* End token of the generation loops (Sec. 3.2, last sentence: the cycle runs until the answer is complete; for a
 * real checkpoint that is the main model emitting its end-of-sequence token).  With 0 <= eos_id < vocab every
 * generation call (stairs_generate, stairs_decode, stairs_decode_adaptive, the sampled and encoder-decoder
 * variants, and per sequence stairs_generate_batch) stops after the first emitted token equal to eos_id: the
 * sequence keeps that token and nothing after it, stats->tokens counts what was produced (<= G, summed over the
 * sequences of a batch), and the entries of tokens_out after the end token are filled with eos_id.  eos_id = -1
 * (the default) turns this off: exactly G tokens.  Errors: EINVAL (eos_id outside [-1, vocab)). */
int stairs_set_eos(stairs_ctx *ctx, int32_t eos_id);

/* The loop of stairs_generate without the prefill: continue the current sequence (after
 * stairs_prefill, or after an earlier stairs_decode) by exactly G tokens.  stats->ms_prefill
 * is 0.  Requires L + G + k + 1 <= max_seq.  Errors: EINVAL, ESTATE (no prefill, pending
 * proposal, k > 0 without a draft model), ECAPACITY. */
int stairs_decode(stairs_ctx *ctx, int32_t G, int32_t k, int32_t *tokens_out, stairs_stats *stats);

/* stairs_decode with a draft length that follows the acceptance: the first iteration proposes k_first tokens
 * (1 <= k_first <= k_max); after an iteration that kept all k the next one proposes min(k + 1, k_max), after one that
 * kept n < k the next one proposes max(1, n + 1).  The output does not depend on the draft lengths (it is the
 * target's greedy continuation, abstract / Sec. 3.1); only the number of iterations does (the paper picks one best
 * length per model pair by a sweep, Sec. 4.3).  Requires L + G + k_max + 1 <= max_seq.  Errors as stairs_decode. */
int stairs_decode_adaptive(stairs_ctx *ctx, int32_t G, int32_t k_first, int32_t *tokens_out, stairs_stats *stats);

/* Several independent sequences in one context (a batch of stair batches): the k+1 stair rows of B sequences are
 * scored by ONE forward of B*(k+1) rows, so the weights are streamed once for all of them; every sequence keeps its
 * own key/value caches, length and acceptance (Sec. 3.3 applied per sequence).  Up to STAIRS_MAX_STREAM_ROWS rows per
 * forward run on the kernels of the single-sequence path (models with d_model, d_ffn <= 16384; else STAIRS_MAX_ROWS)
 * and each sequence's output is bit for bit what stairs_generate gives
 * for it alone; forwards of more rows (up to STAIRS_MAX_BATCH_ROWS) run on the block kernels of the prompt ingestion
 * (one order of additions per output whatever the batch, so a sequence's output does not depend on which others share
 * the forward; against the sequence alone it is the same greedy choice up to near-ties of the logits).
 * stairs_reserve_batch makes room for up to max_batch sequences (caches and token arrays grow max_batch-fold;
 * 1 <= max_batch <= STAIRS_MAX_BATCH; bf16 models only; more than STAIRS_MAX_ROWS / 2 sequences also widen the
 * row workspaces) and drops the current sequence; call it once after stairs_init.  Errors: EINVAL, ENOMEM, EHIP. */
int stairs_reserve_batch(stairs_ctx *ctx, int32_t max_batch);

/* prompts: B host pointers, prompts[b] has P[b] tokens (lengths may differ).  Generates exactly G tokens for every
 * sequence with draft length k (a sequence that has its G tokens stops taking part; the loop ends when all have):
 * tokens_out is [B][G] row-major.  Requires B <= reserved batch, max(B * (k+1), B * 2) <= STAIRS_MAX_STREAM_ROWS (or, with
 * more than STAIRS_MAX_ROWS / 2 sequences reserved, <= STAIRS_MAX_BATCH_ROWS), P[b] + G + k + 1 <= max_seq.  stats (optional): iterations = batched iterations, tokens = B * G,
 * accepted / accept_hist summed over sequences.  Afterwards the context holds no current sequence for the
 * single-sequence calls (stairs_prefill starts one).  Errors: EINVAL, ESTATE (k > 0 without a draft), ECAPACITY, EHIP. */
int stairs_generate_batch(stairs_ctx *ctx, const int32_t *const *prompts, const int32_t *P, int32_t B, int32_t G,
                          int32_t k, int32_t *tokens_out, stairs_stats *stats);

/* ---- sampling variant (the paper's future work, Sec. 5: sampling instead of greedy choice for the assistant and
 * the main model, with a temperature; validation by the rejection scheme its related work describes, Sec. 2.2) ----
 * The assistant DRAWS its k tokens from softmax(logits / temperature); the main model scores the k + 1 stair rows as
 * in stairs_verify; the walk keeps d_i while u_i < p_{i-1}(d_i) / q_i(d_i) (p, q: main model's and assistant's
 * probabilities at the temperature, u_i uniform); at the first token not kept one token is drawn from the normalised
 * positive part of p - q and the walk stops; if all are kept one more token is drawn from p_k.  Each iteration emits
 * n + 1 tokens distributed as the main model's own sampling.  Random numbers come from a counter-based generator
 * (Widynski's "squares", key derived from `seed`) indexed by (position of the token being decided, purpose,
 * vocabulary index), so a run is reproducible and independent of launch shapes; draws are Gumbel-max argmaxes.
 * One sequence per context (not after stairs_reserve_batch); works on decoder-only and encoder-decoder contexts.
 * temperature > 0.  Errors as for the greedy calls. */
int stairs_decode_sampled(stairs_ctx *ctx, int32_t G, int32_t k, float temperature, uint64_t seed,
                          int32_t *tokens_out, stairs_stats *stats);
/* stairs_prefill followed by stairs_decode_sampled. */
int stairs_generate_sampled(stairs_ctx *ctx, const int32_t *prompt, int32_t P, int32_t G, int32_t k,
                            float temperature, uint64_t seed, int32_t *tokens_out, stairs_stats *stats);
/* One iteration in two steps (as draft_propose / stairs_verify).  draft_out: k tokens (host, optional);
 * draft_logits_out: the k logits rows they were drawn from, [k][vocab] float (host, optional). */
int draft_propose_sampled(stairs_ctx *ctx, int32_t k, float temperature, uint64_t seed, int32_t *draft_out,
                          float *draft_logits_out);
/* Needs the pending proposal of draft_propose_sampled with the same k (k = 0: none), temperature and seed.
 * emitted_out: the n + 1 tokens appended to the sequence (room for k + 1); logits_out: [k+1][vocab] main-model
 * logits (host, optional). */
int stairs_verify_sampled(stairs_ctx *ctx, int32_t k, float temperature, uint64_t seed, int32_t *emitted_out,
                          int32_t *n_accepted_out, float *logits_out);

/* ---- encoder-decoder models (the model family of the paper's experiments, Sec. 2.3 / 4.3 / 4.4) -----------
 * The source text goes through the encoder once; the stair batch of Sec. 3.3 is made of prefixes of the DECODER
 * sequence, and every stair row reads the same encoder output (its per-layer cross-attention keys and values are
 * computed once by stairs_encode).  Model: the original T5 layout -- RMS layer norm before every block, attention
 * scores q.k + bias[bucket(key position - query position)][head] without 1/sqrt(head_dim), one bias table per
 * stack (two-sided buckets in the encoder, one-sided with the causal mask in the decoder, none in cross-attention),
 * feed-forward W_out relu(W_in x), no other biases, untied unembedding.  bf16 matrices only.  Supported: head_dim in
 * {64, 128}; d_model, n_heads * head_dim and d_ffn multiples of 256; vocab a multiple of 16; max_src <= 4096. */
typedef struct {
  int32_t n_enc_layers, n_dec_layers, d_model, n_heads, head_dim, d_ffn, vocab;
  int32_t max_src;            /* most source (encoder) positions                              */
  int32_t max_seq;            /* most decoder positions (start token included)                */
  int32_t rel_buckets;        /* rows of the bias tables, e.g. 32 (even)                      */
  int32_t rel_max_distance;   /* distance from which the last bucket is used, e.g. 128        */
  float rms_eps;              /* e.g. 1e-6                                                    */
} stairs_encdec_cfg;

/* Host pointers; matrices are bf16 bit patterns [out_features, in_features] row-major, a = n_heads * head_dim;
 * gains float[d_model]; bias tables float[rel_buckets][n_heads].  enc_* members point to arrays of n_enc_layers
 * pointers, dec_* to arrays of n_dec_layers pointers.  Tensors two models share (same host address) are kept once. */
typedef struct {
  const void *tok_emb;                       /* [vocab, d_model], encoder and decoder inputs */
  const void *lm_head;                       /* [vocab, d_model]                             */
  const float *enc_rel_bias, *dec_rel_bias;
  const float *enc_final_norm, *dec_final_norm;
  const float *const *enc_attn_norm, *const *enc_ffn_norm;
  const void *const *enc_wq, *const *enc_wk, *const *enc_wv;   /* [a, d_model]     */
  const void *const *enc_wo;                                   /* [d_model, a]     */
  const void *const *enc_w_in;                                 /* [d_ffn, d_model] */
  const void *const *enc_w_out;                                /* [d_model, d_ffn] */
  const float *const *dec_attn_norm, *const *dec_cross_norm, *const *dec_ffn_norm;
  const void *const *dec_wq, *const *dec_wk, *const *dec_wv, *const *dec_wo;   /* self-attention  */
  const void *const *dec_cq, *const *dec_ck, *const *dec_cv, *const *dec_co;   /* cross-attention */
  const void *const *dec_w_in, *const *dec_w_out;
} stairs_encdec_weights;

/* As stairs_init, for a target (and optional assistant) of the encoder-decoder kind.  start_token: the id every
 * decoder sequence begins with.  Afterwards stairs_encode starts a sequence; draft_propose, stairs_verify,
 * stairs_verify_tokens, stairs_decode, stairs_decode_adaptive and stairs_get_tokens then work on the decoder
 * sequence exactly as for a decoder-only model (its "prompt" is the start token, P = 1).  stairs_prefill, the
 * several-sequences calls and stairs_time_kernel return EINVAL on such a context. */
int stairs_encdec_init(stairs_ctx **out, const stairs_encdec_cfg *tcfg, const stairs_encdec_weights *tw,
                       const stairs_encdec_cfg *dcfg, const stairs_encdec_weights *dw, int32_t k_max,
                       int32_t start_token, void *hip_stream);

/* Run the encoder of both models over the S source tokens (host pointer), fill every decoder layer's
 * cross-attention keys and values, and start a new decoder sequence [start_token].  1 <= S <= max_src of both
 * models.  Errors: EINVAL, ECAPACITY (S > max_src), EHIP. */
int stairs_encode(stairs_ctx *ctx, const int32_t *src, int32_t S);

/* stairs_encode followed by stairs_decode(G, k): tokens_out[0..G) are the G tokens after the start token;
 * requires 1 + G + k + 1 <= max_seq.  stats->ms_prefill is the time of stairs_encode. */
int stairs_encdec_generate(stairs_ctx *ctx, const int32_t *src, int32_t S, int32_t G, int32_t k,
                           int32_t *tokens_out, stairs_stats *stats);

/* The bucket the library's bias tables use for rel = key position - query position (host arithmetic, no GPU needed;
 * two_sided: the encoder's rule, else the decoder's): lets a caller or a test check the rule against its own.
 * Returns -1 for table shapes stairs_encdec_init would reject. */
int32_t stairs_rel_bucket(int32_t rel, int32_t two_sided, int32_t buckets, int32_t max_distance);

/* Copy the current sequence (prompt + generated) into out[0..min(cap, len)); *len = length. */
int stairs_get_tokens(stairs_ctx *ctx, int32_t *out, int32_t cap, int32_t *len);

/* ---- diagnostics (kernel-level tests and roofline measurement) ------------------------ */

/* Y[M, N] = X[M, K] . W[N, K]^T through the same weight re-layout and skinny GEMM kernels the
 * forward pass uses (bf16: X is split into a bf16 high and low part, fp32 accumulation).
 * All pointers are host pointers; W is in `dtype`; X, Y are float.  1 <= M <= STAIRS_MAX_ROWS. */
int stairs_gemm_host(int32_t dtype, const void *W, const float *X, float *Y, int32_t M, int32_t N,
                     int32_t K, void *hip_stream);

/* stairs_gemm_host for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same kernels, but W [N, K] (row-major, `dtype`), X [M, K] and Y [M, N]
 * (float) are DEVICE pointers the caller owns, and everything stairs_gemm_host allocates per call (hand-off counters,
 * partial sums, the re-laid-out bf16 weights, the activation fragments) lives in a fixed device array inside the
 * library (about 9.3 MiB per GPU the call is used on, held until the process ends).  The call allocates nothing,
 * frees nothing and does not wait: the work is enqueued on hip_stream (a hipStream_t or NULL) and Y is valid once
 * that stream has reached the end of it.  Limits (ECAPACITY beyond them): K <= STAIRS_GEMM_DEVICE_MAX_K; bf16:
 * N * K * 2 <= STAIRS_GEMM_DEVICE_MAX_WEIGHT; ceil(K / 512) * M * N * 4 (bf16) or M * N * 4 (fp32) <=
 * STAIRS_GEMM_DEVICE_MAX_PARTIAL; shape rules as stairs_gemm_host (EINVAL).  All calls on one GPU share the one
 * array: calls that overlap on a GPU (two streams, two threads) race; issue them on one stream or order them. */
#define STAIRS_GEMM_DEVICE_MAX_K        8192
#define STAIRS_GEMM_DEVICE_MAX_WEIGHT   (4u << 20)
#define STAIRS_GEMM_DEVICE_MAX_PARTIAL  (4u << 20)
int stairs_gemm_device(int32_t dtype, const void *W, const float *X, float *Y, int32_t M, int32_t N,
                       int32_t K, void *hip_stream);

/* Time `reps` back-to-back launches of one kernel of the target's forward at M rows, cycling
 * through the layers so that the weights come from HBM, bracketed by HIP events on the
 * context's stream.  which: 0 = gate/up projection GEMM (the largest), 1 = QKV GEMM,
 * 2 = attention output GEMM, 3 = down projection GEMM, 4 = unembedding GEMM,
 * 5 = KV-cache attention at context length ctx_len, 6 = one whole target forward of M rows
 * ending at position ctx_len-1 with all rows' logits (a stair verification without the
 * validation step), 7 = one whole draft forward of M rows with the last row's logits,
 * 8 = the gate/up projection GEMM in situ: `reps` whole target forwards as in 6, with an event
 * pair around every layer's gate/up launch; the mean over reps * n_layers launches is returned,
 * 9 = the same forwards with each event pair recorded back to back in front of the gate/up launch: what a pair
 * reads with no kernel inside (the overhead contained in 8's figure),
 * 10 = the same forwards with every layer's gate/up launch recording its own start and end events (the launch's
 * events, nothing added to the stream): the kernel's duration in situ without the pair's overhead.
 * *ms_per_launch: mean duration; *bytes_per_launch: algorithmic bytes (matrix bytes; K and V
 * bytes of ctx_len positions; for 6/7 all matrices of the model plus its K and V bytes).
 * 0, 2, 3, 4 and 5 do not disturb the sequence state but overwrite workspaces (not allowed between
 * draft_propose and stairs_verify: ESTATE); 1 (its epilogue appends keys and values at positions
 * ctx_len-M .. ctx_len-1; M <= ctx_len <= max_seq) and 6..10 overwrite cache rows: they END the current
 * sequence, and the generation calls return ESTATE until stairs_prefill starts a new one. */
int stairs_time_kernel(stairs_ctx *ctx, int32_t which, int32_t M, int32_t ctx_len, int32_t reps,
                       float *ms_per_launch, double *bytes_per_launch);

/* Launch a plain copy kernel (dst[i] = src[i], `bytes` read + `bytes` written, library-owned
 * buffers) reps+1 times; the reference point that scales a profiler's HBM traffic counters.
 * bytes: multiple of 16.  *ms_per_launch (optional): mean duration of the last reps launches. */
int stairs_copy_probe(int64_t bytes, int32_t reps, float *ms_per_launch, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* STAIRS_H */
