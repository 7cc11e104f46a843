/*
 * sd.h -- C ABI of the MI355X speculative-decoding hot path.
 *
 * One iteration of Algorithm 1 (SpeculativeDecodingStep) of "Fast Inference
 * from Transformers via Speculative Decoding": gamma serial draft steps of
 * the approximation model Mq, one target-model (Mp) forward over the gamma+1
 * draft positions, the acceptance test r_i <= p_i(x_i)/q_i(x_i), the draw from
 * the adjusted distribution norm(max(0, p_{n+1} - q_{n+1})), and the roll-back
 * of both KV caches.  Every step runs in HIP kernels for gfx950.
 *
 * Conventions
 *  - "host" / "dev" in a comment says where a pointer must live.
 *  - All calls are synchronous with respect to their host outputs: they
 *    enqueue on the context's stream and wait for it before returning.
 *  - A context is not thread-safe.  Calls on one context must not overlap.
 *  - Errors are return codes only; a failed call leaves the decoding state
 *    unchanged.  sd_last_error() gives a human-readable reason.
 *  - The library never allocates device memory: everything it needs on the
 *    device lives in the caller's workspace (sd_workspace_bytes()).
 */
#ifndef SD_H
#define SD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sd_ctx sd_ctx;     /* opaque: one (Mp, Mq) pair plus decoding state */

typedef enum {
  SD_OK = 0,
  SD_EINVAL = 1,   /* bad argument: gamma out of range, NULL pointer, unknown tensor, shape mismatch */
  SD_ESTATE = 2,   /* call out of order (step before prefill), or prefix check failed */
  SD_ERANGE = 3,   /* token id >= vocab, sequence would exceed max_len, uniform outside (0,1) */
  SD_ENOMEM = 4,   /* workspace too small */
  SD_EHIP   = 5    /* a HIP call failed */
} sd_status;

typedef enum { SD_F32 = 0, SD_BF16 = 1 } sd_dtype;

enum { SD_ARCH_GPT = 0, SD_ARCH_T5DEC = 1, SD_ARCH_GQA = 2 };
enum { SD_MAX_GAMMA = 15 };       /* a sequence contributes at most SD_MAX_GAMMA+1 rows to a forward */
enum { SD_MAX_BATCH = 64 };       /* sequences decoded together */
enum { SD_ATTN_MAX_ROWS_X_GROUP = 32 };  /* the attention kernels keep (query rows) x (query heads per KV head)
                                     <= 32 rows per KV head: sd_load_models refuses (max_gamma + 1) x
                                     (n_heads / n_kv_heads) beyond it (SD_EINVAL), e.g. 4 query heads per
                                     KV head allow max_gamma <= 7 */

/* Flags of sd_runtime_cfg.flags */
enum {
  SD_FLAG_GRAPH   = 1,  /* replay each iteration as one hipGraph (draft loop, verify, accept) */
  SD_FLAG_PROFILE = 2,  /* record HIP events around the draft / verify / accept phases */
  SD_FLAG_BETA    = 4,  /* also compute beta_i = sum_x min(p_i(x), q_i(x)) of every guess (section 3.1)
                           in each sd_step: one more small launch; feeds sd_stats.beta_sum */
  SD_FLAG_SCATTER_PAGES = 8, /* at load only: every sequence's page table lists its KV-cache pages back to
                           front instead of in order.  Results are identical; it exists to show that
                           every kernel finds its pages through the table.  sd_set_flags leaves it as
                           it was at load. */
  SD_FLAG_SEPARATE_CROSS_Q = 16 /* small T5-type models (bf16, heads of 64, d_model <= 512, at most 16 rows)
                           let the cross-attention kernel compute its own queries, one launch less
                           per layer; with this flag the query projection stays a launch of its own.
                           Results are identical; it exists so that a test can show that. */
};

/*
 * Sampling options beyond the temperature.
 *   lenience : appendix A.5.  q is multiplied by l in (0, 1] before the
 *       comparison with p: guess x_i is kept iff r_i <= p_i(x_i) / (l q_i(x_i)),
 *       so no token is produced with more than 1/l times its probability under
 *       Mp.  After a rejection the extra token is drawn from
 *       norm(max(0, p - l q)) (the appendix leaves this distribution open; this
 *       one keeps the 1/l bound).  With temperature 0 the variant the appendix
 *       sketches for argmax sampling is used: x_i is kept iff
 *       p_i(x_i) >= l max p_i with p_i = softmax of the unscaled logits, decided
 *       as z[x_i] - max z >= ln l in double precision.  l = 1 is Algorithm 1.
 *   top_k, top_p : section 2.2 names top-k and nucleus sampling among the
 *       samplers that amount to plain sampling from an adjusted distribution.
 *       top_k > 0 keeps the tokens whose logit is >= the k-th largest logit;
 *       0 < top_p < 1 then keeps the tokens whose logit is >= that of the token
 *       at which the descending cumulative probability first reaches top_p
 *       (tokens tied with the last kept one are kept); the rest is renormalised.
 *       The same rule is applied to Mp and Mq rows.  0 switches either off;
 *       temperature 0 ignores both.  Needs vocab <= 32768 and vocab % 4 == 0
 *       (the row is filtered in registers); SD_EINVAL otherwise.
 */
typedef struct {
  float   lenience;
  int32_t top_k;
  float   top_p;
} sd_sampling;

/*
 * Model description.  The paper treats Mp and Mq as black boxes (section 2.1)
 * and gives only sizes for its experiments (section 4); the block types are:
 *   SD_ARCH_GPT    pre-LayerNorm (gain+bias), learned positions, biased linear
 *                  layers, tanh-GELU MLP, attention scale 1/sqrt(d_head)
 *   SD_ARCH_T5DEC  RMSNorm, no biases, unscaled attention + one shared
 *                  relative-position bias table, cross-attention over a fixed
 *                  encoder output, gated tanh-GELU MLP
 *   SD_ARCH_GQA    RMSNorm, rotary on adjacent pairs, grouped KV heads, SwiGLU
 * dtype is the storage type of weights, activations and KV cache (accumulation
 * is always fp32; logits are fp32).
 */
typedef struct {
  int32_t arch;
  int32_t n_layers, d_model, n_heads, n_kv_heads, d_head, d_ff, vocab, max_len;
  int32_t enc_len;                 /* T5DEC: rows of the encoder output, else 0 */
  int32_t rel_buckets, rel_max_dist;
  float   rope_theta;
  float   logit_scale;             /* logits = logit_scale * (norm(x) @ head^T) */
  float   norm_eps;
  int32_t dtype;                   /* sd_dtype */
} sd_model_cfg;

/*
 * One weight tensor.  dev: device pointer, row-major, dtype == model dtype.
 * Linear weights are [out_features, in_features].  Names:
 *   tok_emb [V,d]  head [V,d]  lnf.g [d]  (GPT: lnf.b, pos_emb [max_len,d])
 *   (T5DEC: rel_bias [n_heads, rel_buckets])
 *   per layer i, prefix "l<i>.":  ln1.g ln2.g  wq wk wv wo  w2
 *     GPT   : ln1.b ln2.b bq bk bv bo  w1 b1 b2
 *     T5DEC : wg wu  lnc.g cq ck cv co
 *     GQA   : wg wu
 * All tensors are copied (linear weights re-tiled) into the workspace during
 * sd_load_models; the caller may release them when it returns.
 */
typedef struct {
  const char* name;
  const void* dev;
  int32_t     ndim;
  int64_t     shape[4];
  int32_t     dtype;
} sd_tensor;

typedef struct {
  int32_t batch;            /* sequences decoded together, 1..SD_MAX_BATCH (1 for T5DEC models).  Rows are
                               independent: own prompt, own uniforms, own n, own KV pages.  The paper's
                               runs are single-sequence; this is the same algorithm per row. */
  int32_t max_gamma;        /* largest gamma sd_step will be called with, 1..SD_MAX_GAMMA */
  int32_t page_size;        /* KV-cache page, positions; power of two, >= 16 */
  void*   workspace;        /* dev, 256-byte aligned, caller-owned, outlives the context */
  size_t  workspace_bytes;
  void*   stream;           /* hipStream_t every call enqueues on (default priority, capturable: not the
                               legacy default stream), or NULL: the context creates a non-blocking stream
                               of its own and destroys it in sd_free */
  int32_t flags;
} sd_runtime_cfg;

typedef struct {
  double  draft_ms, verify_ms, accept_ms;   /* last sd_step, valid with SD_FLAG_PROFILE */
  int64_t steps;                            /* sd_step calls since load / reset */
  int64_t tokens;                           /* tokens they produced */
  int64_t accepted;                         /* sum of n */
  int64_t fallbacks;                        /* zero-residual fallbacks taken */
  double  ffn_in_ms_sum;                    /* SD_FLAG_PROFILE, RMSNorm targets: time between HIP events around */
  int64_t ffn_in_launches;                  /*   every gated FFN-in GEMM of the verify forwards, and their count */
  int64_t tested;                           /* acceptance tests that counted: sum of min(n+1, gamma) */
  double  beta_sum;                         /* SD_FLAG_BETA: sum of beta_i over those same guesses */
  int64_t beta_count;                       /*   and their number; beta_sum / beta_count estimates alpha = E(beta) */
} sd_stats;

/* Device bytes sd_load_models needs for this pair (weights, KV caches,
 * activations, logits).  Returns 0 for an invalid configuration. */
size_t sd_workspace_bytes(const sd_model_cfg* p_cfg, const sd_model_cfg* q_cfg,
                          const sd_runtime_cfg* rt);

/* Section 2.1: bind the target model Mp and the approximation model Mq.
 * out: host, receives the context.  p_w / q_w: host arrays of descriptors of
 * device tensors.  Fails with SD_EINVAL on a missing / unknown / misshapen
 * tensor, SD_ENOMEM if the workspace is too small. */
sd_status sd_load_models(sd_ctx** out,
                         const sd_model_cfg* p_cfg, const sd_tensor* p_w, int32_t n_p,
                         const sd_model_cfg* q_cfg, const sd_tensor* q_w, int32_t n_q,
                         const sd_runtime_cfg* rt);

/* Condition both models on a prefix (the "prefix" input of Algorithm 1):
 * fills both KV caches for prompt[0 .. prompt_len-2] and records the last
 * token.  prompt: host, prompt_len >= 1 ids.  enc_out_p / enc_out_q: dev,
 * [enc_len, d_model] of the respective model in its dtype (T5DEC), else NULL;
 * their cross-attention keys / values are computed here, once.
 * row: the sequence, 0..batch-1; sd_step needs every sequence prefilled.
 * Requires prompt_len + max_gamma + 1 <= max_len of both models. */
sd_status sd_prefill(sd_ctx* ctx, int32_t row, const int32_t* prompt, int32_t prompt_len,
                     const void* enc_out_p, const void* enc_out_q);

/*
 * Algorithm 1, one run.
 *   prefix, prefix_len : host; optional consistency check of the committed
 *       sequence (length must equal the internal length and the last token
 *       must match, else SD_ESTATE).  prefix == NULL skips the check.
 *   gamma       : number of guesses, 1..max_gamma.
 *   temperature : section 2.2 standardisation; 0 = argmax sampling, > 0 =
 *       softmax(logits / temperature); the same for Mp and Mq.
 *   uniforms    : host, [2*gamma+1] floats strictly inside (0,1):
 *       [0,gamma) draw x_i ~ q_i, [gamma,2*gamma) the acceptance tests r_i,
 *       [2*gamma] the final draw t ~ p'.  All draws are inverse-CDF in
 *       vocabulary order.  May be NULL iff temperature == 0.
 *   out_tokens  : host, [gamma+1]; receives x_1..x_n, t, then -1 padding.
 *   out_n       : host, receives n, the number of accepted guesses.
 * On return the committed sequence is n+1 tokens longer and both KV caches
 * are rolled back to it.
 * With batch > 1 every sequence takes one run, all in the same launches:
 * uniforms is [batch][2*gamma+1], out_tokens [batch][gamma+1], out_n [batch];
 * each sequence has its own n and its own roll-back; prefix must be NULL.
 */
sd_status sd_step(sd_ctx* ctx, const int32_t* prefix, int32_t prefix_len,
                  int32_t gamma, float temperature, const float* uniforms,
                  int32_t* out_tokens, int32_t* out_n);

/* Standard decoding (section 1 / the denominator of Theorem 3.8): one Mp
 * forward on the last token, one draw from p with uniforms[0] (host; may be
 * NULL iff temperature == 0).  out_token: host.  With batch > 1: uniforms
 * [batch], out_token [batch], one token per sequence.  Leaves Mq's cache behind:
 * sd_step after sd_step_baseline needs sd_reset + sd_prefill first
 * (SD_ESTATE otherwise). */
sd_status sd_step_baseline(sd_ctx* ctx, float temperature, const float* uniforms,
                           int32_t* out_token);

/* Forget sequence `row` (-1: all of them, and the statistics): it must be prefilled again
 * before the next sd_step. */
sd_status sd_reset(sd_ctx* ctx, int32_t row);

void sd_free(sd_ctx* ctx);

/* Reason of the last failure on this context (or of the last failed
 * sd_load_models when ctx == NULL).  The string is owned by the library. */
const char* sd_last_error(const sd_ctx* ctx);

/* Measurement / test access.  which = 0: Mp logits of the last step,
 * [batch, gamma+1, vocab]; which = 1: Mq logits, [batch, gamma, vocab]; which = 2
 * after sd_step_baseline: [batch, vocab].  host_out: host, n floats (n <= rows*vocab). */
sd_status sd_debug_logits(sd_ctx* ctx, int32_t which, float* host_out, size_t n);
sd_status sd_get_stats(sd_ctx* ctx, sd_stats* out);
/* Replace the flags given at load for the following calls (captured graphs are rebuilt).
 * SD_FLAG_SCATTER_PAGES keeps the value it had at load whatever is passed here. */
sd_status sd_set_flags(sd_ctx* ctx, int32_t flags);
/* Sampling options for the following sd_step / sd_step_baseline calls (host
 * struct, copied).  SD_EINVAL unless 0 < lenience <= 1, top_k >= 0,
 * 0 <= top_p <= 1, and the vocabulary fits the filter when one is on. */
sd_status sd_set_sampling(sd_ctx* ctx, const sd_sampling* opt);

/*
 * Section 3.6, negligible-cost approximation models: an n-gram table in place
 * of Mq.  With a table set, the draft loop of sd_step does no Mq forward:
 * the logits of guess x_i are the table row row_of[previous token] (a bigram
 * model; the previous token is the last committed token for x_1, else x_{i-1});
 * row_of == NULL selects row 0 for every context (a unigram model).  The rows
 * then go through the same standardisation, acceptance test and adjusted
 * distribution as Mq's logits would; c is the cost of a table lookup and a draw.
 *   table  : dev, [n_rows, vocab] fp32 logits, caller-owned, must outlive its use
 *   row_of : dev, [vocab] int32 row per previous token (values clamped to the table), or NULL
 * table == NULL (with row_of NULL, n_rows 0) goes back to Mq; Mq's cache was not
 * kept up meanwhile, so sd_step then needs sd_reset + sd_prefill first (SD_ESTATE).
 * Mq must still be given to sd_load_models.  Synchronises the stream.
 */
sd_status sd_set_table_draft(sd_ctx* ctx, const float* table, const int32_t* row_of, int32_t n_rows);

/*
 * Section 3.6, the parameter-less approximation model that copies from the
 * context.  With match > 0 the draft loop of sd_step does no Mq forward: for
 * each guess the context (the committed tokens of the sequence, then this
 * iteration's earlier guesses) is searched for earlier occurrences of its own
 * last `match` tokens; the most recent occurrence that has a successor decides,
 * and the draft distribution is all mass on that successor.  Without an
 * occurrence the draft is the table row of sd_set_table_draft when a table is
 * set, else the uniform distribution (the random model that closes the
 * section).  The paper names the idea only; this rule is this library's.
 * The rows go through the same test and adjusted distribution as Mq's would:
 * a copied guess x is kept with probability p(x).
 * The token history lives on the device and is kept up by sd_prefill and by
 * every step taken while match > 0; sequences that advanced with match == 0
 * must be reset and prefilled before a copying step (SD_ESTATE).
 *   match : tokens to match, 1..SD_MAX_COPY_MATCH; 0 goes back to the table
 *           draft or Mq (Mq's cache is stale then, as for sd_set_table_draft)
 * For T5DEC models the context is the decoder's tokens.  Synchronises the stream.
 */
#define SD_MAX_COPY_MATCH 8
sd_status sd_set_copy_draft(sd_ctx* ctx, int32_t match);

/*
 * Section 3.5 (choosing gamma): the integer gamma in 1..gamma_max that maximises
 * the expected walltime improvement of Theorem 3.8,
 *     (1 - alpha^(gamma+1)) / ((1 - alpha) (gamma c + 1)),
 * for an acceptance rate alpha in [0, 1) and a cost coefficient c >= 0
 * (Definition 3.7: time of one Mq run over time of one Mp run); ties go to the
 * smaller gamma.  gamma, improvement: host outputs (improvement may be NULL).
 * Pure host arithmetic: needs no GPU and no context.
 */
sd_status sd_choose_gamma(double alpha, double c, int32_t gamma_max, int32_t* gamma, double* improvement);

/*
 * Measure the two run times behind the cost coefficient c on a prefilled
 * sequence: one draft step of Mq (1-row forward + draw) and one standard
 * decoding step of Mp (1-row forward + draw), each replayed reps (1..1000)
 * times from a hipGraph between two HIP events.  mq_us, mp_us: host outputs,
 * microseconds per run.  The runs write only cache rows beyond the committed
 * sequence (or rewrite a committed row with the same values) and commit
 * nothing.  SD_ESTATE unless the context is prefilled and no sd_step_baseline
 * has made Mq's cache stale.
 */
sd_status sd_measure_cost(sd_ctx* ctx, int32_t reps, double* mq_us, double* mp_us);

/*
 * gamma for this pair from what the context has measured so far: alpha from
 * all sd_step calls since load (sd_reset does not clear it: alpha describes the
 * pair and the task, not one sequence), as the mean of beta_i over the guesses
 * whose test counted when SD_FLAG_BETA was on, else as accepted / tested (both
 * estimate E(beta), Definition 3.1 and Corollary 3.6); c from
 * sd_measure_cost(reps) (needs the prefilled sequence); then sd_choose_gamma with
 * gamma_max = max_gamma of the context.  All outputs host; alpha, c, improvement
 * may be NULL.  SD_ESTATE if no acceptance test has been recorded yet.
 */
sd_status sd_autotune_gamma(sd_ctx* ctx, int32_t reps, int32_t* gamma, double* alpha, double* c,
                            double* improvement);
/* Measurement: the FFN-in GEMM of every Mp layer (the kernel that streams the
 * most weight bytes of the verify forward, section 3.4), `rows` activation rows
 * (1..16), launched reps times over all layers from one hipGraph between two HIP
 * events on the library's stream.  Every launch streams another layer's weights
 * (2 * d_ff * d_model elements for gated blocks, half for GPT blocks), so none is
 * served from cache.  *us_per_launch (host) = mean time of one launch in
 * microseconds.  Needs a prefilled sequence only in so far as the activations it
 * multiplies are whatever the last forward left; it overwrites Mp's FFN scratch
 * rows, nothing else.  Synchronous. */
sd_status sd_time_ffn_in(sd_ctx* ctx, int32_t rows, int32_t reps, double* us_per_launch);

/* Measurement: the time of one whole forward inside a replayed graph, with chosen launches left
 * out, so that a launch's share of the forward is the difference of two calls (kernels of a graph
 * run back to back, so the difference is that launch's duration in its real surroundings).
 *   which    : 0 = Mp over `rows` rows (1 = the standard decoding step of section 1, r > 1 = the
 *              scoring of r - 1 guesses, section 2.3), rows <= max_gamma + 1;
 *              1 = Mq, rows 1 (a draft step) or 2 (the first draft step of an iteration)
 *   skip_ops : SD_OP_* bits: the launches of these kinds are not recorded (their outputs keep
 *              whatever the last forward left, so the remaining launches do the same work).
 *              Where the cross-attention launch computes its own queries (small T5-type models,
 *              see SD_FLAG_SEPARATE_CROSS_Q), SD_OP_CROSS_Q leaves that part of the launch out
 *              and SD_OP_CROSS_ATTN the whole launch.
 *   reps     : graph replays between the two HIP events, 1..1000
 *   us_per_forward : host output, microseconds per replay.
 * Writes cache rows beyond the committed sequence and the logits buffers only; commits nothing.
 * SD_ESTATE unless every sequence is prefilled.  Synchronous. */
enum {
  SD_OP_QKV = 1, SD_OP_ATTN = 2, SD_OP_O = 4, SD_OP_CROSS_Q = 8, SD_OP_CROSS_ATTN = 16, SD_OP_CROSS_O = 32,
  SD_OP_FFN_IN = 64, SD_OP_FFN_OUT = 128, SD_OP_HEAD = 256, SD_OP_ALL = 511
};
sd_status sd_time_forward(sd_ctx* ctx, int32_t which, int32_t rows, int32_t skip_ops, int32_t reps,
                          double* us_per_forward);

/* Measurement: what this chip delivers to a kernel that does nothing but read (the ceiling the
 * weight-streaming GEMMs of section 3.4's memory-bound regime can approach).  One pass reads the
 * whole resident weight block of Mp (which = 0) or Mq (1) exactly once with one persistent
 * 512-thread workgroup per compute unit, 1 KB per wavefront and load, 8 KB in flight per
 * wavefront: the GEMMs' access shape without their arithmetic.  reps passes between two HIP
 * events; us_per_pass, bytes_per_pass: host outputs.  Reads only.  Synchronous. */
sd_status sd_time_stream_read(sd_ctx* ctx, int32_t which, int32_t reps, double* us_per_pass, double* bytes_per_pass);

/*
 * The accept / resample part of Algorithm 1 on explicit logits, for `rows`
 * independent sequences:  n = number of guesses before the first
 * r_i > p_i(x_i)/q_i(x_i);  t ~ norm(max(0, p_{n+1} - q_{n+1})) if n < gamma
 * else t ~ p_{gamma+1};  p_i, q_i = section-2.2 standardisation of the logits.
 *   p_logits : dev, [rows, gamma+1, vocab] fp32      q_logits : dev, [rows, gamma, vocab] fp32
 *   x        : dev, [rows, gamma] int32 guesses      r : dev, [rows, gamma] fp32
 *   s        : dev, [rows] fp32                      out_n, out_t : dev, [rows] int32
 *   scratch  : dev, sd_spec_sample_scratch_bytes(rows, gamma) bytes, zeroed
 *              once by the caller before the first call.
 * Asynchronous on `stream`; no host output.
 */
size_t    sd_spec_sample_scratch_bytes(int32_t rows, int32_t gamma);
/* The same with sampling options (opt: host, NULL = defaults) and, when beta is
 * not NULL, the acceptance probabilities as a side output: beta: dev,
 * [rows, gamma] fp32, beta[b][i] = sum_x min(p_{i+1}(x) / l, q_{i+1}(x))
 * (section 3.1, appendix A.5).  sd_spec_sample is this with opt = beta = NULL. */
sd_status sd_spec_sample_ex(const float* p_logits, const float* q_logits, const int32_t* x,
                            const float* r, const float* s, int32_t rows, int32_t gamma,
                            int32_t vocab, float temperature, const sd_sampling* opt,
                            int32_t* out_n, int32_t* out_t, float* beta,
                            void* scratch, void* stream);
sd_status sd_spec_sample(const float* p_logits, const float* q_logits, const int32_t* x,
                         const float* r, const float* s, int32_t rows, int32_t gamma,
                         int32_t vocab, float temperature,
                         int32_t* out_n, int32_t* out_t,
                         void* scratch, void* stream);


/*
 * sd_spec_sample_ex for callers that cannot allocate device memory or pass a
 * scratch buffer: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same kernels and same results; the
 * scratch (tickets and row statistics, 250 KB) is a fixed array in device
 * memory that the library holds on every GPU it runs on until the process ends.
 * The call allocates nothing (no hipMalloc / hipFree, no allocating library
 * routine) and clears the tickets it uses with a small fill kernel, so it may
 * be recorded into a graph.
 *   rows <= SD_SPEC_SAMPLE_STATIC_MAX_ROWS, else SD_ERANGE (sd_last_error(NULL)
 *   says so); other argument errors as for sd_spec_sample_ex.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one
 * GPU (different streams, different threads) race and give undefined results;
 * calls on one stream are ordered and safe.  Asynchronous on `stream`.
 */
enum { SD_SPEC_SAMPLE_STATIC_MAX_ROWS = 256 };
sd_status sd_spec_sample_static(const float* p_logits, const float* q_logits, const int32_t* x,
                                const float* r, const float* s, int32_t rows, int32_t gamma,
                                int32_t vocab, float temperature, const sd_sampling* opt,
                                int32_t* out_n, int32_t* out_t, float* beta, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SD_H */
