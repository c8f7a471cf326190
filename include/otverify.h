/*
 * otverify: target-side verification step of cross-vocabulary speculative decoding on one MI355X (gfx950).
 *
 * The operation is the verification half of OmniDraft's Algorithm 1 (Cross-vocabulary Speculative Decoding):
 * given the target model's final hidden states for the k+1 verified positions of each sequence, the drafter's
 * logits and drafted ids, a direct draft->target id map and an n-gram cache (Section "Cross-vocabulary N-gram
 * Cache"), it
 *   - projects the hidden states through the LM head and forms softmax statistics of the target rows and of
 *     the draft rows (the parallel target pass of Algorithm 1);
 *   - translates the drafted ids into target-vocabulary tokens t_j with probabilities q'(t_j) (Eq. 1): direct
 *     id lookup, or one target token for several consecutive draft tokens that hit the cache, whose
 *     probability is the product of the sub-token probabilities;
 *   - accepts t_j while u_j < min(1, p(t_j)/q'(t_j)) (Algorithm 1, rejection sampling step);
 *   - draws the final token from norm(max(0, p - q')) at the first rejected position, with q' extended to the
 *     whole target vocabulary by Eq. 2, or a free token from p when everything was accepted (Algorithm 1).
 *
 * Conventions
 *   - Every function returns OT_OK (0) or a negative OT_ERR_*; nothing throws, aborts or prints.
 *     ot_last_error() returns a thread-local, NUL-terminated description of the last failure on this thread.
 *   - Pointers are marked HOST or DEVICE.  The library never frees or reallocates caller memory.
 *   - Device work is enqueued on the stream given at init and is asynchronous: the caller synchronises that
 *     stream before reading outputs.  One context must not be used from two threads at once.
 *   - Uniform random numbers are Philox4x32-10 (Salmon et al., SC'11) with key = (seed low, seed high) and
 *     counter = (mapped position j, step, seq_id low, seq_id high).  Output word 0 gives the acceptance
 *     uniform of position j, word 1 the uniform of the final-token draw at row j; a uniform is the word's top
 *     24 bits times 2^-24.
 */
#ifndef OTVERIFY_H_
#define OTVERIFY_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ------------------------------------------------------------------------------------- */
#define OT_OK                 0
#define OT_ERR_NULL          -1   /* a required pointer is NULL                                              */
#define OT_ERR_SHAPE         -2   /* a size is out of range, over capacity, or row offsets are not monotone  */
#define OT_ERR_DTYPE         -3   /* dtype is neither OT_BF16 nor OT_F32                                     */
#define OT_ERR_MAP           -4   /* direct map entry out of range, or two draft ids share a target id       */
#define OT_ERR_NGRAM         -5   /* n-gram entry length or id out of range                                  */
#define OT_ERR_CTX_MISMATCH  -6   /* the n-gram cache was built for another context                          */
#define OT_ERR_HIP           -7   /* a HIP call failed; ot_last_error() carries hipGetErrorString            */
#define OT_ERR_NOMEM         -8   /* host or device allocation failed                                        */

/* ---- storage types of hidden states, LM-head weights and draft logits --------------------------------- */
/* OT_BF16 is the production type: the LM head runs on the matrix cores, bound by the weight stream.
 * OT_F32 exists for small problems that want fp32 arithmetic end to end (checks against an fp32 model, toy
 * vocabularies): its LM head is a vector-ALU kernel that re-reads W once per 8 rows and never hosts the draft side,
 * so a step costs several times the bf16 one at the same shape (measured: about 6x at d = 4096, V_t = 128256,
 * 144 rows).  Nothing is refused for size; it is simply slow there.                                          */
#define OT_BF16 0
#define OT_F32  1

/* ---- per-sequence output flags ------------------------------------------------------------------------ */
#define OT_FLAG_UNMAPPABLE 1      /* a drafted id had neither a cache hit nor a direct image: proposal cut   */
#define OT_FLAG_RESID_ZERO 2      /* the residual had zero mass: final token drawn from p instead            */
#define OT_FLAG_BAD_ID     4      /* a drafted id was outside [0, V_d): the sequence emits nothing           */

#define OT_MAX_NGRAM_LEN   8      /* largest supported key length of a cache entry                           */
#define OT_MAX_K          63      /* largest supported number of drafted tokens per sequence                 */

typedef struct ot_ctx ot_ctx;                 /* owns the packed LM head, maps and workspace                  */
typedef struct ot_ngram_cache ot_ngram_cache; /* owns the device hash table of one n-gram cache               */

/* ---- ot_verify_init ----------------------------------------------------------------------------------- */
/* The draft rows' softmax statistics and what the drafted ids look up for the translation (Eq. 1: the drafted logit,
 * the direct image, the n-gram cache probes) need nothing from the LM head.  Where the bf16 LM-head kernel supports it
 * (more than 16 rows, at most 255 sequences) the LM-head launch itself can do that work: with up to 176 rows, where the
 * launch is bound by the weight stream, every multiplying workgroup takes a piece of a draft row while its first loads
 * are in flight; with more rows a few workgroups at the front of the launch take all of it.  The launch then also
 * leaves the target rows' softmax partials, and one launch follows it (window walk, acceptance test, final draw)
 * instead of three. */
/* Capacity edges (all shapes inside max_batch / max_k are served; what changes is the launch structure):
 *   - 16 rows or fewer, OT_F32, or a step entered through ot_verify_step_from_logits: the draft side always runs
 *     after the LM head (the softmax statistics of all rows and the lookups as a launch of their own, then the launch
 *     that walks, tests and draws: one launch more, a few microseconds);
 *   - more than 255 sequences in a step: the same, and the translation with the acceptance test gets a launch of its
 *     own as well (two launches more, about 25 us at 256 sequences with a 32000-id draft vocabulary);
 *   - OT_DRAFT_SIDE_AUTO also chooses the first of these when hosting would lengthen the LM-head launch: more than two
 *     draft rows per multiplying workgroup (up to 176 rows), or front workgroups that would need more than half
 *     of the launch (above).                                                                                     */
#define OT_DRAFT_SIDE_AUTO        0   /* decide per step from its shape (estimate of both durations)               */
#define OT_DRAFT_SIDE_IN_LM_HEAD  1   /* inside the LM-head launch whenever the kernel supports the shape          */
#define OT_DRAFT_SIDE_SEPARATE    2   /* always as launches of their own after the LM head                         */

typedef struct ot_verify_config {
  int32_t d;               /* hidden size; for OT_BF16 a multiple of 8                                        */
  int32_t V_t;             /* target vocabulary size                                                          */
  int32_t V_d;             /* draft vocabulary size                                                           */
  int32_t max_batch;       /* capacity: B <= max_batch                                                        */
  int32_t max_k;           /* capacity: k_b <= max_k <= OT_MAX_K; rows <= max_batch * (max_k + 1)             */
  int32_t dtype;           /* OT_BF16 or OT_F32: type of W, hidden and draft_logits                           */
  int32_t max_ngram_len;   /* 2..OT_MAX_NGRAM_LEN: longest key any cache used with this context may hold      */
  int32_t draft_side;      /* OT_DRAFT_SIDE_*: where the part of a step that needs no target logits runs          */
  const void*    W;        /* DEVICE [d, V_t] row-major LM-head weights (z = h . W).  Read during init only:
                              OT_BF16 weights are re-tiled into a private copy, OT_F32 weights are copied.    */
  const int32_t* direct_map; /* HOST [V_d]: target id of each draft id, or -1.  Must be one-to-one on the
                              mapped part (the paper's t_i <-> d_i), else OT_ERR_MAP.                         */
  void*          stream;   /* hipStream_t on which all device work of this context is enqueued (NULL = the
                              default stream)                                                                 */
} ot_verify_config;

/* Creates a context on the current HIP device.  Allocates the private LM-head copy (d * V_t elements), the
 * two map tables and a workspace sized for max_batch * (max_k + 1) rows of fp32 logits.  Synchronises the
 * stream before returning.  *out is NULL on failure.                                                         */
int  ot_verify_init(const ot_verify_config* cfg, ot_ctx** out);
void ot_verify_destroy(ot_ctx* ctx);          /* synchronises the stream, frees everything; NULL is a no-op   */

/* ---- the n-gram cache ---------------------------------------------------------------------------------- */
/* The cache C = {(t_i, [d_j]_{j=1:n})} (Section "Cross-vocabulary N-gram Cache") lives on the device as an
 * open-addressing hash table that the translation step probes.  Entries are given in CSR form on the HOST: entry e
 * maps draft ids key_ids[key_off[e] .. key_off[e+1]) (2 <= length <= cfg.max_ngram_len, ids in [0, V_d)) to
 * target_ids[e] in [0, V_t); the arrays are not referenced after a call returns.  Of pairs with equal keys the last
 * one wins.  A cache may be used only with the context it was made for and must be destroyed before it.  The calls
 * below synchronise the context's stream: cache maintenance happens between steps.
 *
 * Every verification step that is handed a cache advances the cache's logical clock by one and, for each entry
 * the translation scan uses (the entry becomes a mapped token of a proposal, accepted or not), adds one to the
 * entry's use count and stamps it with the clock.  Every insert call that adds at least one pair advances the clock
 * by one and stamps the entries it adds or overwrites (a call with n_entries == 0 changes nothing).  The cost of a
 * maintenance call follows the number of entries it touches, not the size of the cache: the device reports the
 * entries it used through a small log in pinned host memory and receives the changed slots as one packed patch
 * (measured: about 45 us for an insert that evicts one entry of a full 100 000-entry cache, once the stream is
 * idle).  A cache holds about 80 KB of pinned host memory for that log and patch.                            */
#define OT_EVICT_NONE 0   /* an insert call whose new keys do not fit fails as a whole (OT_ERR_SHAPE)             */
#define OT_EVICT_LRU  1   /* evict the entry not used for the longest time        (Appendix "N-gram Cache        */
#define OT_EVICT_LFU  2   /* evict the entry with the fewest uses                  Scalability")                 */

/* Bulk build: a cache of capacity n_entries without eviction holding the given entries.  n_entries may be 0.  */
int  ot_ngram_cache_build(ot_ctx* ctx, int32_t n_entries, const int32_t* key_off, const int32_t* key_ids,
                          const int32_t* target_ids, ot_ngram_cache** out);
/* An empty cache for at most `capacity` entries (0 .. 2^26) with the given eviction policy.                    */
int  ot_ngram_cache_create(ot_ctx* ctx, int32_t capacity, int32_t policy, ot_ngram_cache** out);
/* Online update (the cache-update step that closes an iteration of Algorithm 1): adds the pairs in order.  A known key gets the new target and a fresh time stamp and keeps its use count.  A new key that finds
 * the cache full first evicts one entry: LRU the smallest (last use, insertion number), LFU the smallest (uses,
 * last use, insertion number).  *n_evicted (may be NULL) receives the number of evictions.                     */
int  ot_ngram_cache_insert(ot_ngram_cache* cache, int32_t n_entries, const int32_t* key_off, const int32_t* key_ids,
                           const int32_t* target_ids, int32_t* n_evicted);
/* Number of entries and (if n_key_ids is not NULL) total number of key ids, i.e. the sizes ot_ngram_cache_export
 * needs.                                                                                                       */
int  ot_ngram_cache_size(const ot_ngram_cache* cache, int32_t* n_entries, int32_t* n_key_ids);
/* Copies the entries out in insertion order: HOST key_off [n+1], key_ids, target_ids [n], and, if not NULL, the
 * use counts and last-use clocks [n].  OT_ERR_SHAPE if max_entries / max_key_ids are too small.                */
int  ot_ngram_cache_export(ot_ngram_cache* cache, int32_t max_entries, int32_t max_key_ids, int32_t* key_off,
                           int32_t* key_ids, int32_t* target_ids, int64_t* uses, int64_t* last_used);
/* Brings saved entries back with their statistics (the arrays ot_ngram_cache_export fills, all HOST, all required):
 * the pairs are added in order like an insert, but each keeps its use count and last-use clock, nothing is evicted
 * (OT_ERR_SHAPE if they do not fit) and the cache's clock becomes at least the largest last-use clock.  Exporting a
 * cache and importing the result into an empty cache of the same capacity and policy therefore continues with the
 * same eviction order as the original.  A key the cache already holds gets the given target and statistics.     */
int  ot_ngram_cache_import(ot_ngram_cache* cache, int32_t n_entries, const int32_t* key_off, const int32_t* key_ids,
                           const int32_t* target_ids, const int64_t* uses, const int64_t* last_used);
void ot_ngram_cache_destroy(ot_ngram_cache* cache);

/* ---- ot_verify_step ------------------------------------------------------------------------------------ */
/* Ragged batch: sequence b drafted k_b tokens and owns the k_b + 1 rows row_off[b] .. row_off[b+1]-1; row j of
 * a sequence is the target's hidden state that predicts mapped token t_j (Algorithm 1: p(t_t) .. p(t_{t+m})).
 * M = row_off[B] rows in total, K = M - B drafted positions; the k_b draft rows of sequence b start at draft
 * row row_off[b] - b.                                                                                         */
typedef struct ot_step_in {
  int32_t         B;                  /* number of sequences, 0 <= B <= max_batch                             */
  uint32_t        step;               /* Philox counter word 1                                                */
  const int32_t*  row_off;            /* DEVICE [B+1]                                                         */
  const int32_t*  row_off_host;       /* HOST   [B+1], same values; used for validation and launch sizes      */
  const void*     hidden;             /* DEVICE [M, d] row-major, cfg.dtype                                   */
  const void*     draft_logits;       /* DEVICE [K, V_d] row-major, cfg.dtype                                 */
  const int32_t*  draft_ids;          /* DEVICE [K] drafted ids d_i                                           */
  const float*    temperature;        /* DEVICE [B]; 0 selects the greedy rule for that sequence              */
  const float*    draft_temperature;  /* DEVICE [B], or NULL: the drafter used `temperature`                  */
  const uint64_t* seq_id;             /* DEVICE [B] Philox stream id of each sequence                         */
  uint64_t        seed;               /* Philox key                                                           */
} ot_step_in;

/* Caller-allocated DEVICE buffers, all required.  Per sequence ([B]):
 *   n_mapped        m_b, number of target-vocabulary tokens the proposal translated into
 *   n_accept        n_b <= m_b, accepted mapped tokens (the correction / free token is not counted)
 *   n_accept_draft  the same in draft-token units, sum of the accepted spans' lengths
 *   n_emit          tokens written to out_tokens: n_b + 1, or 0 with OT_FLAG_BAD_ID
 *   hits_proposed   mapped tokens that came from the n-gram cache; hits_accepted: those among the accepted
 *   flags           OR of OT_FLAG_*
 * Per row ([M], entry row_off[b] + j belongs to mapped position j of sequence b):
 *   out_tokens      j < n_b: accepted t_j; j == n_b: the correction or free token; other entries -1
 *   mapped_ids      t_j for j < m_b, else -1;  span_start / span_len: the draft positions t_j covers (else -1/0)
 *   p_tok, q_tok, ratio  p_j(t_j), q'(t_j), min(1, p/q') for j < m_b, else 0.  For a greedy sequence p_tok is
 *                   1 or 0 (argmax match) and ratio equals it.                                                */
typedef struct ot_step_out {
  int32_t *n_mapped, *n_accept, *n_accept_draft, *n_emit, *hits_proposed, *hits_accepted, *flags;
  int32_t *out_tokens, *mapped_ids, *span_start, *span_len;
  float   *p_tok, *q_tok, *ratio;
} ot_step_out;

/* Enqueues one verification step.  `cache` may be NULL (direct map only).  Returns OT_ERR_SHAPE if B or any
 * k_b exceeds the capacity or row_off_host is not increasing by at least 1 per sequence.  B == 0 is a no-op. */
int ot_verify_step(ot_ctx* ctx, ot_ngram_cache* cache_or_null, const ot_step_in* in, ot_step_out* out);

/* Same, but the LM-head projection is skipped and `target_logits` (DEVICE [M, V_t] row-major fp32, the z_j of
 * Algorithm 1's target pass) is used instead; in->hidden is ignored.                                          */
int ot_verify_step_from_logits(ot_ctx* ctx, ot_ngram_cache* cache_or_null, const ot_step_in* in,
                               const float* target_logits, ot_step_out* out);

/* ---- hybrid distillation loss, forward values --------------------------------------------------------- */
/* Section "Cross-vocabulary Distillation", the loss equation: L = L_DM + lambda * L_N-gram, the expectation over
 * drafted tokens d_i of  D_KL(q' || p)(t_i) * I_DM(d_i)  -  lambda * log q(d_i) * I_N-gram(d_i).
 *   - a mapped token that came through the direct map carries the reverse KL between q', the draft distribution
 *     of its position lifted into the target vocabulary (Eq. 2, not renormalised; the sum runs over q'(v) > 0),
 *     and the target distribution p of its row;
 *   - a mapped token that came from the n-gram cache carries NLL = -sum over its sub-tokens of ln q(d), or (
 *     OT_NGRAM_TERM_APPROX_KL) the KL with Eq. 2's two overrides, times lambda: the constant `lambda`, or
 *     (OT_LAMBDA_TARGET_PROB) the verified target probability p(t_i);
 *   - p and q are the step's distributions (its temperatures); sequences with a target or draft temperature of 0
 *     contribute nothing; with accepted_only != 0 only n-grams the target accepted count.
 * Must be called after ot_verify_step / ot_verify_step_from_logits on this context with the same `in`, and with
 * that step's output buffers: it reads the translation from them and the logits and row statistics from the
 * context's workspace (`target_logits`: the pointer given to ot_verify_step_from_logits, or NULL after
 * ot_verify_step).  Work is enqueued on the context's stream.                                                  */
#define OT_LAMBDA_FIXED          0
#define OT_LAMBDA_TARGET_PROB    1
#define OT_NGRAM_TERM_NLL        0
#define OT_NGRAM_TERM_APPROX_KL  1
typedef struct ot_loss_config {
  float   lambda;         /* used with OT_LAMBDA_FIXED (0.2 in the paper's experiments)                          */
  int32_t lambda_mode;    /* OT_LAMBDA_*                                                                         */
  int32_t ngram_term;     /* OT_NGRAM_TERM_*                                                                     */
  int32_t accepted_only;  /* != 0: n-gram tokens at mapped positions j >= n_accept[b] are left out               */
} ot_loss_config;
/* Caller-allocated DEVICE buffers.  Per row ([M], entry row_off[b] + j is mapped token j of sequence b):
 *   kind    0 no term, 1 direct-mapping token (KL term), 2 n-gram token
 *   kl      the KL term of a direct-mapping token, or of an n-gram token with OT_NGRAM_TERM_APPROX_KL, else 0
 *   nll     -sum ln q(d) over the sub-tokens of an n-gram token, else 0
 *   weight  lambda of an n-gram token, else 0
 *   totals  [5]: sum of the KL terms of direct-mapping tokens; sum of weight * (nll or kl) of n-gram tokens; number
 *           of direct-mapping tokens; number of n-gram sub-tokens; loss = (sum 1 + sum 2) / max(1, count 1 + count 2)
 *   qprime  optional (may be NULL): [M, V_t] fp32, row row_off[b] + j = q' of Eq. 2 over the whole target vocabulary
 *           at mapped position j (with the overrides of the n-gram matched there), zeros for rows without a term   */
typedef struct ot_loss_out {
  int32_t* kind;
  double  *kl, *nll, *weight, *totals;
  float*   qprime;
} ot_loss_out;
int ot_distill_loss(ot_ctx* ctx, const ot_step_in* in, const ot_step_out* step_out, const float* target_logits_or_null,
                    const ot_loss_config* cfg, ot_loss_out* out);

/* ---- adaptive drafting: stop rule and the acceptance head's loss value -------------------------------- */
/* Section "Online Adaptive Drafting": a head f_phi gives, for proposed token i, the logit of
 * P(y_i accepted | y_<i accepted) = sigmoid(f_phi(e_i)); drafting exits once
 * P(some y_i', i' <= i, rejected) = 1 - prod_{i' <= i} sigmoid(f_phi(e_i')) exceeds gamma.  The head is trained
 * with a weighted binary cross-entropy against the labels min(1, p/q), which ot_verify_step outputs as `ratio`.
 * The head's layers are the drafter's business: its logits are the input.  Arrays are laid out like the step's
 * per-row outputs: entry row_off[b] + i belongs to proposed token i of sequence b (the last row of a sequence
 * is unused).  Only the first n_valid[b] tokens of sequence b are considered (NULL: all k_b).
 *   p_accept      sigmoid(head_logits), 0 for unused entries
 *   p_any_reject  1 - running product of p_accept within the sequence
 *   n_keep        [B] min{i >= 1 : p_any_reject at token i-1 > gamma}, the token that tips the rule is kept; or
 *                 the number of tokens considered if the rule never fires
 *   bce           optional (may be NULL, needs `labels`): [3] = sum over the tokens considered of
 *                 -(w_accept * l * ln sigmoid(a) + w_reject * (1 - l) * ln(1 - sigmoid(a))), their number, the mean
 * All buffers are DEVICE memory except row_off_host; work is enqueued on the context's stream.                 */
typedef struct ot_adapt_in {
  int32_t        B;
  float          gamma;          /* stopping threshold (0.3 / 0.7 in the paper's experiments)                    */
  float          w_accept, w_reject;
  int32_t        reserved;       /* must be 0                                                                    */
  const int32_t* row_off;        /* DEVICE [B+1]                                                                 */
  const int32_t* row_off_host;   /* HOST   [B+1]                                                                 */
  const float*   head_logits;    /* DEVICE [M] f_phi(e_i)                                                        */
  const float*   labels;         /* DEVICE [M] acceptance ratios in [0, 1], or NULL                              */
  const int32_t* n_valid;        /* DEVICE [B], or NULL                                                          */
} ot_adapt_in;
typedef struct ot_adapt_out {
  float   *p_accept, *p_any_reject;   /* [M]                                                                     */
  int32_t *n_keep;                    /* [B]                                                                     */
  double  *bce;                       /* [3] or NULL                                                             */
} ot_adapt_out;
int ot_adaptive_drafting(ot_ctx* ctx, const ot_adapt_in* in, ot_adapt_out* out);

/* The same operation for callers that cannot allocate device memory or hold a context: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  It takes no context and allocates nothing: its only scratch
 * (two binary64 loss partials per sequence, 64 KB) is an array inside the library's code object, one copy per GPU,
 * held until the process ends.  Work is enqueued on `stream` (a hipStream_t, NULL = the default stream) of the current
 * device.  Limits: B <= OT_STATIC_MAX_BATCH (else OT_ERR_SHAPE), k_b <= OT_MAX_K.  Results are identical to
 * ot_adaptive_drafting.  All calls on one GPU share the scratch: calls whose device work overlaps on one GPU (two
 * streams, two threads) race on it; calls on one stream do not.  The array's device address is looked up on the
 * first call per device and by every ot_verify_init.                                                            */
#define OT_STATIC_MAX_BATCH 4096
int ot_adaptive_drafting_static(const ot_adapt_in* in, ot_adapt_out* out, void* stream);

/* ---- diagnostics ---------------------------------------------------------------------------------------- */
/* Device pointers into the context's workspace, valid until ot_verify_destroy and overwritten by every step.
 * Row statistics are those of the softmax of the Notation paragraph: p_j(v) = exp((z_v - row_max)/T) / row_sumexp. */
typedef struct ot_workspace_view {
  const float*   logits;        /* [rows, ld_logits] fp32 target logits of the last ot_verify_step            */
  int64_t        ld_logits;
  const float*   row_max;       /* [M]                                                                        */
  const double*  row_sumexp;    /* [M] sum_v exp((z_v - row_max)/T_b); T_b == 0 rows use T = 1                */
  const int32_t* row_argmax;    /* [M] lowest index of the maximum                                            */
  const float*   draft_row_max; /* [K] the same three statistics of the draft rows at the draft temperature   */
  const double*  draft_row_sumexp;
  const int32_t* draft_row_argmax;
} ot_workspace_view;
int ot_verify_workspace(ot_ctx* ctx, ot_workspace_view* view);

/* Kernel timing.  While enabled, every step records HIP events between its kernels on the context's stream.
 * ot_verify_profile_read synchronises the stream, adds the elapsed milliseconds of the steps run since the
 * last read into ms[0 .. OT_N_STAGES) (overwriting it), stores the number of steps in *n_steps and resets.    */
#define OT_STAGE_LM_HEAD          0   /* z = h . W                                                            */
#define OT_STAGE_SOFTMAX_STATS    1   /* softmax statistics of the target and draft rows; 0 when the LM-head
                                         launch computes them itself                                          */
#define OT_STAGE_TRANSLATE_ACCEPT 2   /* translation scan + n-gram probes (Eq. 1), acceptance ratios, Philox  */
#define OT_STAGE_RESIDUAL_DRAW    3   /* masses of max(0, p - q') (Eq. 2) at the final row, inverse-CDF draw  */
#define OT_N_STAGES               4
int ot_verify_profile(ot_ctx* ctx, int32_t enable);
int ot_verify_profile_read(ot_ctx* ctx, float* ms, int32_t* n_steps);

const char* ot_last_error(void);
const char* ot_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OTVERIFY_H_ */
