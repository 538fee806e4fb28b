/*
 * tasc.h -- C ABI of the MI355X (gfx950) library for TASC-spec: batched, greedy, n-gram-drafted
 * speculative decoding of a small decoder-only language model.
 *
 * The method is the inference-time method of "Task-Centric Acceleration of Small-Language Models"
 * (section "n-Gram Speculative Decoding Method"): a drafter made of pruned corpus n-gram tables M_n
 * (n <= n_max), queried in descending order of n with the most frequent token as the fallback,
 * mixed with an n-gram drafter over the available context,
 *     p_mixed(x|c) = lambda p_corp(x|c) + (1 - lambda) p_prompt(x|c),
 * proposes a run of tokens that the target model verifies in a single forward pass, of which a
 * prefix is accepted (subsection "Speculative Decoding"; greedy, beam size 1, p_min = 5 and
 * lambda = 0.75 in the paper's Results).
 *
 * Conventions
 *   - Every function returns a tasc_status; on error nothing is written to the outputs and
 *     tasc_last_error() holds a thread-local message.
 *   - "device" pointers are HIP device memory of the current device, "host" pointers ordinary
 *     host memory.  The caller owns every buffer it passes in; the library owns only the opaque
 *     handles (and the device memory it allocates for the n-gram tables and the packed weights)
 *     and releases them in *_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Unless stated
 *     otherwise a call only enqueues work on `stream`; results are valid once the stream has
 *     been synchronised.
 *   - Same inputs give bit-identical outputs, run to run.
 *   - There is no CPU fallback: without a gfx950 device every compute call fails with TASC_EHIP.
 */
#ifndef TASC_H
#define TASC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t tasc_status;
enum {
    TASC_OK = 0,
    TASC_EINVAL = -1,  /* null pointer, shape or range error                       */
    TASC_ENOMEM = -2,  /* caller buffer too small, allocation failure, table full  */
    TASC_EHIP = -3,    /* HIP runtime error (text in tasc_last_error)              */
    TASC_ESTATE = -4   /* call out of order (e.g. verify before prefill)           */
};

typedef enum { TASC_MEM_HOST = 0, TASC_MEM_DEVICE = 1 } tasc_mem;
typedef enum { TASC_F32 = 0, TASC_BF16 = 1 } tasc_dtype;

#define TASC_MAX_ORDER 8   /* n_max <= 8 and n_max * ceil(log2(vocab)) <= 128 */
#define TASC_MAX_K 15      /* at most 15 draft tokens per step                */

typedef struct tasc_model tasc_model;     /* packed weights, LM-head bias, RoPE table            */
typedef struct tasc_ngram tasc_ngram;     /* corpus tables M_2..M_nmax and the fallback token    */
typedef struct tasc_session tasc_session; /* B sequences: committed tokens, lengths, paged KV    */

const char* tasc_last_error(void);

/* ------------------------------------------------------------------------------------------
 * Corpus n-gram drafter (section "Proposed Method: TASC-spec", first paragraph).
 * ---------------------------------------------------------------------------------------- */

/*
 * Builds M_n for n = 2..n_max from the n-gram frequencies of the corpus, prunes every element
 * whose count is below p_min, and finds the most frequent token.
 *   tokens       int32[doc_offsets[n_docs]], every token in [0, vocab); host or device per `where`
 *   doc_offsets  HOST int64[n_docs + 1], non-decreasing, doc_offsets[0] = 0; n-grams never span
 *                two documents.  The corpus must hold fewer than 2^32 - 1 tokens.
 *   n_max        in [2, TASC_MAX_ORDER];  p_min >= 1.
 * An element (c, x) of M_n is kept iff count(c, x) >= p_min; per kept context c the table holds
 * T(c) = sum of kept counts and its most frequent kept successor (smallest id among equals).
 * Synchronous: allocates device memory, runs on `stream` and waits for it.  *out is owned by the
 * library until tasc_ngram_destroy.
 */
tasc_status tasc_ngram_build(const int32_t* tokens, const int64_t* doc_offsets, int64_t n_docs,
                             int32_t vocab, int32_t n_max, int32_t p_min, tasc_mem where,
                             void* stream, tasc_ngram** out);
void tasc_ngram_destroy(tasc_ngram* ng);

/*
 * Canonical dump of M_order for parity checks: the kept n-grams sorted by their tokens.
 *   ctx_next  HOST int32[cap, order] (context tokens then the successor), counts HOST uint32[cap].
 *   n_inout   in: cap (rows available); out: number of kept n-grams.  With NULL arrays only the
 *             count is returned.  TASC_ENOMEM if cap is too small (count still returned).
 */
tasc_status tasc_ngram_export(const tasc_ngram* ng, int32_t order, int32_t* ctx_next,
                              uint32_t* counts, int64_t* n_inout);
/* Same for the per-context aggregates: ctx HOST int32[cap, order-1], total/top/top_count HOST [cap]. */
tasc_status tasc_ngram_export_contexts(const tasc_ngram* ng, int32_t order, int32_t* ctx,
                                       uint32_t* total, int32_t* top, uint32_t* top_count,
                                       int64_t* n_inout);
/* Most frequent corpus token (smallest id among equals) and, if non-NULL, HOST uint32[vocab] counts. */
tasc_status tasc_ngram_unigram(const tasc_ngram* ng, int32_t* fallback, uint32_t* counts);

typedef struct {
    int64_t n_tokens;
    int64_t windows[TASC_MAX_ORDER + 1];   /* windows counted per order                 */
    int64_t distinct[TASC_MAX_ORDER + 1];  /* distinct n-grams before pruning           */
    int64_t kept[TASC_MAX_ORDER + 1];      /* n-grams kept after pruning                */
    int64_t contexts[TASC_MAX_ORDER + 1];  /* kept contexts                             */
    double build_ms;                       /* device time of the whole build            */
    double count_ms;                       /* device time of the counting kernels alone */
} tasc_ngram_stats;
tasc_status tasc_ngram_get_stats(const tasc_ngram* ng, tasc_ngram_stats* out);

/*
 * Size and dominance of the typical set of one table (paper, "Task-Induced n-Grams Concentration":
 * the n-gram entropy and the number of unique n-grams that attain 80 % of the n-gram CDF; Appendix,
 * "Predicting Model Speedup ... from the Data": Renyi entropy H_alpha(p) = log(sum p^alpha) / (1 - alpha),
 * used there with alpha = 2).  The distribution is p(x) = count(x) / total over the entries x of the
 * table of n-grams of length `order` that the build kept (build with p_min = 1 for the corpus' full
 * distribution); order 1 is the token (unigram) distribution, which is never pruned.
 *   coverage_ppm  share of the total count to reach, in parts per million, in [0, 1000000]
 *                 (800000 = the paper's 80 %).
 *   out           HOST; written only on success.
 *     n_entries   entries with a non-zero count
 *     total       sum of their counts
 *     n_cover     fewest entries, most frequent first, whose counts sum to >= total * coverage_ppm / 1e6
 *                 (exact integer arithmetic)
 *     shannon     -sum p ln p, nats (fp64)
 *     renyi2      -ln sum p^2, nats (fp64)
 * Runs its kernels on `stream` and synchronises it before returning (an analysis call, not part of
 * the decode loop); allocates and frees a few KB of device scratch.  An empty table gives all zeros.
 * Errors: TASC_EINVAL (null, order outside [1, n_max], coverage out of range), TASC_EHIP.
 */
typedef struct {
    int64_t n_entries;
    int64_t total;
    int64_t n_cover;
    double shannon;
    double renyi2;
} tasc_table_entropy;
tasc_status tasc_ngram_entropy(const tasc_ngram* ng, int32_t order, int32_t coverage_ppm,
                               tasc_table_entropy* out, void* stream);

/*
 * tasc_ngram_entropy for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same kernels in the same order, with their scratch (the
 * per-workgroup partial sums, the two select histograms, the select state: 37 KB) in a fixed array inside the
 * library instead of a hipMalloc'ed buffer.  Calls no hipMalloc / hipFree and does not synchronise: it only
 * enqueues kernels on `stream` (the scratch is cleared by a kernel, not a memset).
 *   out_device  DEVICE tasc_table_entropy, written by the last kernel; valid once `stream` has been synchronised.
 * Every call on one device shares that device's array: calls that overlap on one device (different streams)
 * race; calls on one stream are ordered and independent (each clears the scratch first).
 * Limit: tables of at most TASC_ENTROPY_NOALLOC_MAX_SLOTS hash slots (order 1: vocabulary entries); beyond it
 * TASC_ENOMEM and nothing is enqueued.  Other errors as tasc_ngram_entropy.
 */
#define TASC_ENTROPY_NOALLOC_MAX_SLOTS (1ull << 32)
tasc_status tasc_ngram_entropy_noalloc(const tasc_ngram* ng, int32_t order, int32_t coverage_ppm,
                                       tasc_table_entropy* out_device, void* stream);

/* ------------------------------------------------------------------------------------------
 * Target model.  The paper uses the target as a black box; the architecture (pre-norm RMSNorm,
 * RoPE with rotate-half pairing, grouped-query attention, SwiGLU, untied LM head, sparse additive
 * bigram bias on the logits) is that of the benchmark configurations.
 * ---------------------------------------------------------------------------------------- */
typedef struct {
    int32_t dtype;      /* tasc_dtype of the matrices and of the KV cache                  */
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t max_pos;    /* RoPE table length: largest position + 1                         */
    float rope_theta;   /* angle of pair i at position p: p * theta^(-2i/head_dim)         */
    float rms_eps;      /* RMSNorm: x * g / sqrt(mean(x^2) + eps)                          */
} tasc_model_desc;

/*
 * All matrices are [out_features, in_features] row-major in `dtype` (bf16 as raw 16-bit
 * patterns); gains are fp32.  Per-layer entries are HOST arrays of n_layers pointers.  The
 * pointed-to data may be host or device memory (`where`); it is copied, the caller may free it
 * after the call.
 *   embed, lm_head [vocab, d_model];  wq [n_heads*head_dim, d_model];  wk, wv [n_kv_heads*head_dim,
 *   d_model];  wo [d_model, n_heads*head_dim];  wg, wu [d_ffn, d_model];  wd [d_model, d_ffn];
 *   g1, g2, gf fp32 [d_model].
 * LM-head bias (all four NULL for none): logits[v] = h . lm_head[v] + bias(u, v), u = the input
 * token of the row; bias(u, v) = bias_val[j] if v = bias_col[j] for some j in
 * [bias_rowptr[u], bias_rowptr[u+1]) (columns ascending within a row), else bias_base[u].
 */
typedef struct {
    tasc_mem where;
    const void* embed;
    const void* lm_head;
    const float* gf;
    const void* const* wq;
    const void* const* wk;
    const void* const* wv;
    const void* const* wo;
    const void* const* wg;
    const void* const* wu;
    const void* const* wd;
    const float* const* g1;
    const float* const* g2;
    const int64_t* bias_rowptr; /* [vocab + 1] */
    const int32_t* bias_col;    /* [nnz]       */
    const float* bias_val;      /* [nnz]       */
    const float* bias_base;     /* [vocab]     */
} tasc_weight_ptrs;

/* Synchronous (copies and repacks the weights into library-owned device memory). */
tasc_status tasc_model_create(const tasc_model_desc* desc, const tasc_weight_ptrs* w, tasc_model** out);
void tasc_model_destroy(tasc_model* m);

/* ------------------------------------------------------------------------------------------
 * Session: `batch` sequences decoded in lock-step.
 *   max_len   most tokens (prompt + generated + drafts in flight) a sequence may hold
 *   max_rows  most rows per sequence in one forward: >= k + 1, also the prefill chunk length
 * KV cache: pages of 16 positions, [page][K|V][kv_head][...], one pool per layer, all inside the
 * caller's kv_pool; a block table maps (sequence, position / 16) to a page.  Positions whose
 * drafts were rejected stay allocated and are overwritten by the next step ("rollback" only
 * shortens the sequence's cached length).
 * ---------------------------------------------------------------------------------------- */
size_t tasc_session_kv_bytes(const tasc_model* m, int32_t batch, int32_t max_len);
size_t tasc_session_workspace_bytes(const tasc_model* m, int32_t batch, int32_t max_len, int32_t max_rows);
/* kv_pool and workspace: DEVICE memory, 256-byte aligned, at least the sizes above; owned by the
 * caller and must outlive the session.  Synchronous (initialises the block table). */
tasc_status tasc_session_create(const tasc_model* m, int32_t batch, int32_t max_len, int32_t max_rows,
                                void* kv_pool, size_t kv_bytes, void* workspace, size_t ws_bytes,
                                tasc_session** out);
void tasc_session_destroy(tasc_session* s);

/*
 * Resets the session and runs the prompt forward: fills the KV cache for all prompt positions and
 * commits, as generated token #1, the argmax at the last prompt position (the "pending" token,
 * whose own KV is not cached yet).
 *   prompts         int32, concatenated, host or device per `where`
 *   prompt_offsets  HOST int64[batch + 1]; every prompt has 1..max_len tokens
 *   max_new         tokens to generate per sequence (>= 1); a sequence that has them is frozen
 */
tasc_status tasc_session_prefill(const tasc_model* m, tasc_session* s, const int32_t* prompts,
                                 const int64_t* prompt_offsets, tasc_mem where, int32_t max_new,
                                 void* stream);

typedef struct {
    int32_t k;                       /* draft tokens per step, 0..TASC_MAX_K (0 = plain greedy)   */
    int32_t lambda_q16;              /* round(lambda * 65536) in [0, 65536]; 49152 = 0.75         */
    int32_t p_min_ctx;               /* pruning threshold of the context drafter (>= 1)           */
    int32_t ctx_includes_generated;  /* 1: context = prompt + committed output; 0: prompt only    */
} tasc_spec_params;

/*
 * Proposes k tokens for every sequence (section "Proposed Method: TASC-spec"): k times in a row,
 * each source (corpus tables; n-gram counts of the sequence's own committed tokens) backs off from
 * order n_max to 2 to its first matching context, the proposal is
 *     argmax_x  q C_corp(x) T_ctx + (65536 - q) C_ctx(x) T_corp        (q = lambda_q16)
 * i.e. the argmax of p_mixed, ties to the smallest token id; with one source matching, that
 * source's most frequent successor; with none, the corpus' most frequent token.  A source whose
 * weight is 0 is not consulted.  Each proposal is appended to the running context of the next.
 *   drafts  DEVICE int32[batch, k]
 * Limit: the kernel keeps a sequence's committed tokens in LDS, so the session's max_len (which includes the
 * 2 * max_rows slack tasc_session_create asks for) must not exceed 4096 tokens; TASC_EINVAL otherwise.
 */
tasc_status tasc_draft(const tasc_ngram* ng, tasc_session* s, const tasc_spec_params* p,
                       int32_t* drafts, void* stream);

/*
 * One target forward over the rows [pending, d_1..d_k] of every sequence (subsection "Speculative
 * Decoding": the drafted tokens are verified in parallel via a single forward pass), then greedy
 * acceptance: a_i = argmax of row i (lowest index among equals), m = the longest prefix with
 * d_i = a_{i-1}; the sequence commits d_1..d_m and the bonus token a_m, its cached length grows by
 * 1 + m, the new pending token is a_m.
 *   drafts      DEVICE int32[batch, k] (ignored if k = 0)
 *   accept_len  DEVICE int32[batch], nullable
 *   emitted     DEVICE int32[batch, k + 1], nullable: d_1..d_m, a_m, then -1 padding
 *   logits_dbg  DEVICE fp32[batch, k + 1, vocab], nullable: the full logits of every row
 * A sequence that already has its max_new tokens is frozen (accept_len 0, emitted all -1).
 */
tasc_status tasc_verify_step(const tasc_model* m, tasc_session* s, const int32_t* drafts, int32_t k,
                             int32_t* accept_len, int32_t* emitted, float* logits_dbg, void* stream);

typedef struct {
    int64_t steps;                       /* verify steps executed                                  */
    int64_t emitted;                     /* tokens delivered (batch * max_new)                     */
    int64_t accepted;                    /* draft tokens accepted over all steps and sequences     */
    int64_t proposed;                    /* draft tokens proposed to live sequences                */
    int64_t accept_hist[TASC_MAX_K + 1]; /* number of (step, sequence) pairs per accept length     */
    double prefill_ms, decode_ms;        /* device time (HIP events on `stream`)                   */
    int64_t xcd_local_steps;             /* steps whose layer phases synchronised through one XCD's L2 */
} tasc_gen_stats;

/*
 * Prefill, then draft + verify until every sequence has max_new tokens (plain greedy if p->k = 0,
 * `ng` may then be NULL).  Synchronous.
 *   out_tokens  DEVICE int32[batch, max_new]
 *   trace       DEVICE int32, nullable, capacity trace_steps steps of
 *               [batch][1 + k + (k+1) + 1] = (committed length before the step, drafts, argmax
 *               ids, accept length) for step-by-step replay against a reference
 *   stats       HOST, nullable
 */
tasc_status tasc_generate(const tasc_model* m, const tasc_ngram* ng, tasc_session* s,
                          const int32_t* prompts, const int64_t* prompt_offsets, tasc_mem where,
                          int32_t max_new, const tasc_spec_params* p, int32_t* out_tokens,
                          int32_t* trace, int32_t trace_steps, tasc_gen_stats* stats, void* stream);

/* Health of a session whose decode steps run on the persistent small-batch kernels (forwards of at most 16 rows on a
 * bf16 model: one launch per step whose workgroups wait for each other's results).  Those kernels need all their
 * workgroups resident at once, one per compute unit: the session must have the device to itself while a step runs (a
 * kernel of another stream, session or process that occupies compute units can keep a workgroup from starting).  Every
 * wait is bounded; a wait that runs out sets a flag in the session and the step's outputs (tokens, accept_len, emitted,
 * the cache) are then undefined.  tasc_verify_step and tasc_draft do not read the flag (that would cost a host round trip
 * per step); tasc_generate checks it at its end, and this call reads it on demand:
 *   *timed_out (HOST) = 1 if a step of this session ran into a time-out since the last tasc_session_prefill (which
 *   clears the flag and makes the session usable again), else 0.  Synchronises `stream`.  Errors: TASC_EINVAL, TASC_EHIP. */
tasc_status tasc_session_status(tasc_session* s, int32_t* timed_out, void* stream);

/* Copies sequence b's committed tokens (prompt + generated) to HOST int32[cap]; *n = how many.
 * Synchronises `stream`. */
tasc_status tasc_session_get_tokens(const tasc_session* s, int32_t b, int32_t* tokens, int32_t cap,
                                    int32_t* n, void* stream);

/* ------------------------------------------------------------------------------------------
 * Library-wide options (for tests and tuning; the defaults are what the benchmarks run).
 *   TASC_CFG_SMALL_PATH  how a bf16 forward of at most 16 rows runs: 2 (default) = one persistent
 *                        kernel for the whole step, 1 = the same kernel launched once per phase,
 *                        0 = the type-generic kernels.  Results of 1 and 2 are bit-identical.
 *   TASC_CFG_SMALL_GRID  workgroups of the persistent kernel; 0 (default) = one per compute unit.
 *   TASC_CFG_SMALL_LAYER_WGS, TASC_CFG_SMALL_LAYER_STRIDE
 *                        the layer phases run on the workgroups stride * j, j < wgs, of that grid
 *                        (0 = defaults); the LM head always uses the whole grid.  Results do not
 *                        depend on these.
 *   TASC_CFG_TILED_PATH  bf16 forwards of more than 16 rows: 1 (default) = LDS-tiled MFMA kernels,
 *                        0 = the type-generic kernels.
 *   TASC_CFG_SMALL_XCD_LOCAL
 *                        1 (default) = when the layer phases' workgroups all run on one XCD (the
 *                        kernel checks), their barriers exchange data through that XCD's L2 and
 *                        skip the L2 write-back and invalidate; 0 = agent-scope barriers always.
 *                        Results do not depend on it.
 *   TASC_CFG_SMALL_LAYER_WORKERS
 *                        in that XCD-local mode, how many of the layer workgroups compute; the
 *                        others prefetch the next phase's weights into the XCD's L2 (0 = default:
 *                        all compute).  Results do not depend on it.
 *   TASC_CFG_SMALL_KERNEL
 *                        which kernel TASC_CFG_SMALL_PATH 1 and 2 run: 1 (default) = the spatial pipeline (every workgroup
 *                        keeps one kind of work for all layers, weights requested a layer ahead, activations handed
 *                        over through polled buffers) where the model fits it, 0 = the barrier kernel (phases separated
 *                        by barriers among a group of workgroups).  Results are bit-identical.
 *   TASC_CFG_PIPE_SHARE  output tiles (of 16 features) a workgroup of the spatial pipeline takes per layer at least, 1..3
 *                        (default 1): larger values put fewer workgroups on every role.  Results do not depend on it.
 *   TASC_CFG_CHAINS      forwards of more than 16 rows: into how many ranges of sequences the batch is cut for the
 *                        layers, each range on a stream of its own beside the caller's (0 = the library's rule, 1..4).
 *                        A row's kernels and summation order do not depend on it, so neither does any result; with few
 *                        rows per sequence range the layer kernels of one range leave compute units idle that another
 *                        range's kernels fill.  The caller's stream waits for every range before the LM head.
 *   TASC_CFG_STEP_GRAPH  1 (default): a verify step of the tiled kernels (forwards of more than 16 rows) is recorded
 *                        into a HIP graph the second time it is called with the same k and the same draft / result
 *                        pointers, and replayed as one graph launch from then on (a step is a few hundred launches
 *                        with step-invariant arguments); 0: every kernel is launched on its own.  Same kernels, same
 *                        results.  Steps that ask for logits or a trace, run under the per-class timers, or are
 *                        called on a stream that is itself being captured are always launched one by one.
 */
enum {
    TASC_CFG_SMALL_PATH = 0, TASC_CFG_SMALL_GRID = 1, TASC_CFG_SMALL_LAYER_WGS = 2, TASC_CFG_SMALL_LAYER_STRIDE = 3,
    TASC_CFG_TILED_PATH = 4, TASC_CFG_SMALL_XCD_LOCAL = 5, TASC_CFG_SMALL_LAYER_WORKERS = 6, TASC_CFG_SMALL_KERNEL = 7,
    TASC_CFG_PIPE_SHARE = 8, TASC_CFG_CHAINS = 9, TASC_CFG_STEP_GRAPH = 10
};
tasc_status tasc_config_set(int32_t key, int32_t value);

/* ------------------------------------------------------------------------------------------
 * The model-derived bigram drafter of the paper's comparison (Related Work; Results, "TASC-spec":
 * a bigram model that assigns each token its most probable next token under the given model, from
 * the model's conditional distribution for every vocabulary element; evaluated alone and mixed with
 * the context drafter).
 * ---------------------------------------------------------------------------------------- */
/*
 * next_tok[x] = the target's greedy next token (lowest index on ties) after the one-token sequence
 * [x], for every x in [0, vocab): ceil(vocab / batch) prefill passes of `batch` one-token prompts
 * through the session's ordinary forward path.
 *   s         any session of `m` with max_len >= 2 + 2 * max_rows (max_rows = 1 wastes no rows); its
 *             sequences are overwritten, so call tasc_session_prefill again before decoding with it.
 *   next_tok  DEVICE int32[vocab], written.
 * Synchronises `stream` before returning.  Errors: TASC_EINVAL, TASC_EHIP.
 */
tasc_status tasc_model_bigram(const tasc_model* m, tasc_session* s, int32_t* next_tok, void* stream);
/*
 * The drafter as tables, usable wherever tasc_ngram_build's result is (tasc_draft, tasc_generate,
 * the exports): order 2 holds, for every token x, the single successor next_tok[x] with count 1
 * (T(x) = 1, a point mass: lambda weighs it against the context statistics exactly as it weighs the
 * corpus tables), orders 3..n_max are empty, so only the context source uses them.  The fallback
 * token is the most frequent token of the V pairs [x, next_tok[x]].
 *   next_tok  HOST or DEVICE (`where`) int32[vocab], every value in [0, vocab).
 *   n_max     in [2, TASC_MAX_ORDER], n_max * ceil(log2(vocab)) <= 128.
 * Errors as tasc_ngram_build (TASC_EINVAL for a successor outside the vocabulary).
 */
tasc_status tasc_ngram_from_bigram(const int32_t* next_tok, tasc_mem where, int32_t vocab, int32_t n_max,
                                   void* stream, tasc_ngram** out);

/* ------------------------------------------------------------------------------------------
 * Counting core of the paper's tokenizer enrichment ("Enriching the Tokenizer": the merge reward
 * f_merge(t^n) = freq(t^n) * (n - 1) and the loop of the algorithm "Tokenizer Enrichment"), WITHOUT
 * the prefix-collision filter (it needs token strings; every candidate passes).  Starting from the
 * base vocabulary [0, vocab), step i counts the token n-grams, 2 <= n <= n_max, of the corpus as
 * tokenised so far (windows inside one output, as in tasc_ngram_build), takes the n-gram with the
 * largest reward (ties: the shorter n-gram, then the lexicographically smallest token tuple), names it
 * token vocab + i and re-tokenises the corpus: its occurrences are replaced left to right, without
 * overlap, inside each output.  Ends after `budget` merges or when no n-gram is left.
 *   tokens, out_tokens  HOST or DEVICE (`where`, both alike) int32; out_tokens has room for the input
 *                       length and receives the final corpus (corpus_len[*n_merges] tokens).
 *   doc_offsets         HOST int64[n_docs + 1]; out_offsets HOST int64[n_docs + 1] (final boundaries).
 *   merges              HOST int32[budget][1 + TASC_MAX_ORDER]: n, then the n tokens (over the vocabulary
 *                       of that step), then -1 padding; merge_freq HOST int64[budget]: freq of the pick.
 *   corpus_len          HOST int64[budget + 1]: corpus length before merge i; entry *n_merges = final.
 *   n_merges            HOST: merges performed (<= budget).
 * Limits: n_max in [2, TASC_MAX_ORDER], n_max * ceil(log2(vocab + budget)) <= 128, corpus < 2^32 - 1
 * tokens.  Synchronous (one host round trip per merge); allocates about 20 bytes of device scratch per
 * corpus token plus the tables of one tasc_ngram_build.  Errors: TASC_EINVAL, TASC_ENOMEM, TASC_EHIP.
 * ---------------------------------------------------------------------------------------- */
tasc_status tasc_tok_enrich(const int32_t* tokens, const int64_t* doc_offsets, int64_t n_docs, int32_t vocab,
                            int32_t n_max, int32_t budget, tasc_mem where, void* stream, int32_t* merges,
                            int64_t* merge_freq, int64_t* corpus_len, int32_t* out_tokens,
                            int64_t* out_offsets, int32_t* n_merges);

/* ------------------------------------------------------------------------------------------
 * Measurement: per-kernel-class device time, taken with HIP event pairs recorded on the stream
 * each kernel is launched on.  Off by default (no events are recorded).  The classes follow the
 * steps of the hot path: table build is timed by tasc_ngram_get_stats, the rest here.
 * ---------------------------------------------------------------------------------------- */
enum {
    TASC_KC_DRAFT = 0,    /* draft proposal kernel                                            */
    TASC_KC_PREPARE = 1,  /* row metadata + embedding gather                                  */
    TASC_KC_NORM = 2,     /* RMSNorm                                                          */
    TASC_KC_GEMM_QKV = 3, /* fused q/k/v projection                                           */
    TASC_KC_ROPE_KV = 4,  /* RoPE + KV append                                                 */
    TASC_KC_ATTN = 5,     /* attention over the paged cache                                   */
    TASC_KC_GEMM_O = 6,   /* output projection + residual                                     */
    TASC_KC_GEMM_GU = 7,  /* gate/up projection + SwiGLU                                      */
    TASC_KC_GEMM_D = 8,   /* down projection + residual                                       */
    TASC_KC_LMHEAD = 9,   /* LM head + bias + partial argmax                                  */
    TASC_KC_ACCEPT = 10,  /* argmax reduce, draft compare, accept length, KV rollback         */
    TASC_KC_VERIFY = 11,  /* one whole verify step (all of the above but the draft)           */
    TASC_KC_LAYERS = 12,  /* the fused decoder-layer kernel of the small-batch verify step     */
    TASC_N_KERNEL_CLASSES = 13
};
/* class_mask: bit c enables class c; 0 disables.  Applies to later calls of this process. */
tasc_status tasc_profile_enable(uint32_t class_mask);
/* Waits for the device, then returns and clears the time and launch count recorded per class.
 * total_ms, launches: HOST arrays of TASC_N_KERNEL_CLASSES entries. */
tasc_status tasc_profile_read(double* total_ms, int64_t* launches);
/* The single durations behind tasc_profile_read, for medians: waits for the device, then writes the time of every recorded
 * launch of class `cls`, in launch order, to ms[0 .. min(*n, cap)) (HOST) and their number to *n; clears nothing (call it
 * before tasc_profile_read). */
tasc_status tasc_profile_durations(int32_t cls, double* ms, int64_t cap, int64_t* n);

/* Per-phase timing of the persistent small-batch kernel: while device_buf is non-NULL every launch
 * writes, for workgroup w < capacity / (2 * phases) and phase p (phases = 3 + 5 * n_layers: embedding,
 * five per layer, LM head, accept), the 100 MHz wall-clock ticks at which w began and ended p into
 * device_buf[(w * phases + p) * 2 + {0, 1}].  device_buf: DEVICE uint64[capacity]; NULL turns it off. */
tasc_status tasc_profile_phases(uint64_t* device_buf, int64_t capacity);

/* A plain device-to-device copy kernel (reads `bytes`, writes `bytes`; DEVICE pointers, 16-byte aligned,
 * bytes a multiple of 16): the known-size reference against which rocprofv3's FETCH_SIZE / WRITE_SIZE
 * counters of the other kernels are scaled. */
tasc_status tasc_calibration_copy(void* dst, const void* src, size_t bytes, void* stream);

/* Attainable bf16 MFMA rate of the device: one workgroup of 8 waves per compute unit issues `iters` x 32
 * independent v_mfma_f32_32x32x16_bf16 per wave on register operands (no memory traffic in the loop);
 * *tflops (HOST) = the rate of the second of two launches, timed with HIP events on `stream`.  The
 * reference beside the published peak for the GEMM kernels' utilisation.  Synchronises the stream. */
tasc_status tasc_calibration_mfma(int32_t iters, void* stream, double* tflops);

/* Attainable read rate of the device for a stream of independent 16-byte loads: one workgroup of 512 threads per
 * compute unit takes 64 KB blocks of src (DEVICE pointer, 16-byte aligned, bytes a multiple of 65536) round-robin,
 * 8 loads in flight per lane, `passes` times over the buffer, and stores nothing.  *gbps (HOST) = bytes read / time of
 * the second of two launches (HIP events on `stream`).  A buffer of a few MB stays in the L2 of every XCD and gives
 * the L2-to-compute-unit rate, one beyond the memory-side cache (> 256 MB) the HBM read rate: the references beside
 * the published 8 TB/s for the kernels that stream weights and the KV cache.  Synchronises the stream. */
tasc_status tasc_calibration_read(const void* src, size_t bytes, int32_t passes, void* stream, double* gbps);

/* Latency of one hand-over of `bytes` among `n_workgroups` resident workgroups (ids stride * j of a grid of one workgroup
 * per compute unit; the dispatcher deals ids to the 8 XCDs in turn, so stride 8 keeps them on one XCD and stride 1
 * spreads them): every participant writes its share of the bytes, then reads all of them, 200 times in a row.
 *   with_flags = 0  "flag in data": readers poll the data words themselves (agent-scope loads) until none holds the
 *                   sentinel -- how the small-batch pipeline kernel hands activations from phase to phase;
 *   with_flags = 1  stores, a wait for them, one arrival flag per participant polled by one wave, then the loads.
 * *us_per_handover (HOST) = the best of three runs, from the device's 100 MHz clock.  The reference for how short a chain
 * of dependent phases spread over many compute units can be.  Allocates and frees its buffers; synchronises the stream.
 * Errors: TASC_EINVAL, TASC_EHIP (also when a wait times out or a reader sees stale data). */
tasc_status tasc_calibration_handover(int32_t n_workgroups, int32_t stride, int32_t bytes, int32_t with_flags, void* stream,
                                      double* us_per_handover);

/* Duration of one launch of the tiled bf16 GEMM out[M, N] = epilogue(A[M, K] W[N, K]^T) at a given shape, with the tile
 * shape the forward would choose for it: the measuring stick for the projections of a verify step (Speculative Decoding:
 * one forward over the k + 1 candidate rows of every sequence).  epilogue: 0 plain fp32 store, 1 residual add, 2 SwiGLU
 * (bf16 out, N = 2 x d_ffn with gate and up rows interleaved), 4 fp32 partial sums of `slices` k-slices (1..8).  The operands
 * are constant fills the call allocates and frees; *us_per_launch (HOST) = the mean of `iters` back-to-back launches after 3
 * warm-up launches, from HIP events on `stream`.  Synchronises the stream.  Errors: TASC_EINVAL (shape), TASC_EHIP. */
tasc_status tasc_calibration_gemm(int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t slices, int32_t iters, void* stream,
                                  double* us_per_launch);

#ifdef __cplusplus
}
#endif
#endif /* TASC_H */
