/*
 * disco.h -- C boundary of the MI355X (gfx950) hot path of one DISCO speculative-decoding iteration
 * (arXiv 2405.04304, "Dynamic Speculation Lookahead Accelerates Speculative Decoding of LLMs").
 *
 * One iteration (paper Sec. 2 and Fig. 1; Sec. 3 "Dynamic Speculation Lookahead Optimization"):
 *   the draft model decodes tokens one at a time (disco_draft_step); after every draft token a
 *   small classifier over [top-10 draft probabilities, entropy, position] decides whether to draft
 *   another token (disco_classify, Eq. 2); the target model then checks the whole block of
 *   SL + 1 tokens in one forward against its KV cache (disco_verify); the longest draft prefix that
 *   equals the target's arg-max tokens is accepted (disco_accept; rejection sampling at temperature
 *   0) and the rejected suffix is dropped from both KV caches (disco_kv_rollback).
 *
 * Conventions
 *   - "dev" pointers are DEVICE memory, "host" pointers are HOST memory.  The caller owns every
 *     device buffer (weights, KV pages, workspace, logits, outputs); the library allocates no
 *     device memory and keeps borrowed pointers only.  Handles are small host objects.
 *   - Every call validates its arguments on the host BEFORE any launch and returns 0 on success or
 *     a negative DISCO_E* code; it never aborts, throws or prints.  disco_last_error() gives the
 *     message of the calling thread's last failure.
 *   - All launches are asynchronous on the caller's HIP stream (disco_stream is a hipStream_t).
 *     KV lengths are host-side metadata updated at enqueue time.
 *   - Weight matrices are bf16.  A "packed" matrix W[N x K] (N % 16 == 0, K % 32 == 0) is stored
 *     as 1 KiB tiles of 16 rows x 32 columns, tile (rt, kt) at element offset (rt * K/32 + kt) * 512,
 *     and inside a tile the element of row r, column c at  ((c / 8) * 16 + r) * 8 + c % 8  -- the
 *     operand order of the 16x16x32 bf16 matrix instruction, so a wavefront streams a tile with one
 *     fully coalesced 128-bit load per lane.  disco_pack_weight converts from row-major.
 *   - At most DISCO_MAX_BLOCK tokens are fed per forward.
 */
#ifndef DISCO_H
#define DISCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DISCO_MAX_BLOCK 16
#define DISCO_TOPK 10          /* k of Eq. 2 (the paper's footnote: k = 10 in all experiments) */
#define DISCO_N_FEAT 12        /* top-10 probabilities, entropy, position                       */
#define DISCO_CLF_HIDDEN_MAX 256
#define DISCO_CLASSIFY_SCRATCH_BYTES 4352   /* optional scratch of disco_classify */

enum {
  DISCO_OK = 0,
  DISCO_EINVAL = -1,  /* null / misaligned pointer, bad enum, shape the kernels do not support   */
  DISCO_ECAP = -2,    /* block length or KV capacity exceeded                                    */
  DISCO_ESTATE = -3,  /* rollback outside [0, len], handle mismatch                               */
  DISCO_EHIP = -4     /* a HIP runtime call failed                                                */
};

enum { DISCO_FAMILY_A = 0,   /* pre-LN LayerNorm, exact-erf GELU MLP, learned position table     */
       DISCO_FAMILY_B = 1 }; /* RMSNorm, rotary (pairs c, c + d_head/2), SwiGLU MLP               */

typedef void* disco_stream;  /* a hipStream_t (0 = the null stream) */

typedef struct disco_model_desc {
  int32_t family, n_layers, d_model, n_heads, d_head, n_kv_heads, d_ff, vocab;
  int32_t max_pos;           /* rows of the position table (family A), ignored for family B      */
  float norm_eps;            /* LayerNorm / RMSNorm epsilon                                       */
  float rope_base;           /* rotary base (family B)                                            */
} disco_model_desc;

/* Device pointers of one layer.  Vectors are fp32; matrices are packed bf16 (see above).
 * w_in: family A = W1 [d_ff x d_model]; family B = gate and up matrices interleaved by 16-row
 * tiles (disco_pack_gate_up), [2 d_ff x d_model].  w_out: W2 / down [d_model x d_ff].
 * wqkv: rows ordered [q heads | k heads | v heads], [(n_heads + 2 n_kv_heads) d_head x d_model]. */
typedef struct disco_layer_weights {
  const float* norm1_g; const float* norm1_b;   /* *_b NULL for family B */
  const void* wqkv; const void* wo;
  const float* norm2_g; const float* norm2_b;
  const void* w_in; const void* w_out;
} disco_layer_weights;

typedef struct disco_model_weights {
  const void* tok_emb;        /* bf16 row-major [vocab x tok_emb_stride], first d_model columns used */
  int64_t tok_emb_stride;     /* elements between rows (>= d_model)                                 */
  const void* pos_emb;        /* bf16 row-major [max_pos x d_model], family A; else NULL            */
  const disco_layer_weights* layers;  /* HOST array of n_layers entries (copied by the library)    */
  const float* normf_g; const float* normf_b;
  const void* wlm;            /* packed [vocab x d_model]                                           */
} disco_model_weights;

typedef struct disco_model disco_model;  /* immutable: desc + borrowed device weight pointers       */
typedef struct disco_kv disco_kv;        /* one sequence's paged KV cache: page order + length      */

/* Halting classifier of Eq. 2: C = sigmoid(w2 . relu(W1 f + b1) + b2), f = 12 features.
 * dev_params: fp32 [W1 (hidden x 12, row-major) | b1 (hidden) | w2 (hidden) | b2 (1)].             */
typedef struct disco_clf {
  const float* dev_params;
  int32_t hidden;             /* 1 .. DISCO_CLF_HIDDEN_MAX */
} disco_clf;

/* Result of one disco_classify call (device memory, 16-byte aligned). */
typedef struct disco_clf_out {
  int32_t token;              /* arg-max of the draft logits, lowest id on ties                     */
  float feats[DISCO_N_FEAT];  /* top-10 probabilities (descending), entropy (nats), position        */
  float score;                /* C_i                                                                */
  uint32_t halt;              /* bit 0: stop drafting after this token; bit 1 (reference lookahead    */
                              /* only): the token differs from the reference and is not in the block  */
  uint32_t executed;          /* 1 if the call ran, 0 if it was gated off                            */
} disco_clf_out;

typedef struct disco_accept_out {
  int32_t n;                        /* number of accepted draft tokens                              */
  int32_t n_emit;                   /* n + 1                                                        */
  int32_t emit[DISCO_MAX_BLOCK];    /* accepted draft tokens followed by the target's token         */
} disco_accept_out;

const char* disco_last_error(void);

/* ---- layout helpers ------------------------------------------------------------------------- */

/* Row-major bf16 [n x k] -> packed.  n % 16 == 0, k % 32 == 0; src and dst must not overlap.       */
int disco_pack_weight(const void* dev_src, int64_t n, int64_t k, void* dev_dst, disco_stream s);
/* Gate [d_ff x k] and up [d_ff x k] (row-major) -> one packed [2 d_ff x k] matrix whose 16-row
 * tiles alternate gate tile i, up tile i, so the SwiGLU product is formed inside one workgroup.   */
int disco_pack_gate_up(const void* dev_gate, const void* dev_up, int64_t d_ff, int64_t k,
                       void* dev_dst, disco_stream s);

/* ---- handles --------------------------------------------------------------------------------- */

int disco_model_create(const disco_model_desc* desc, const disco_model_weights* w, disco_model** out);
void disco_model_destroy(disco_model* m);

/* Bytes of KV storage for capacity_tokens positions (rounded up to whole pages): the page order, for
 * family B the rotary table (cos, sin per position and channel pair, fp32), and the pages.          */
size_t disco_kv_bytes(const disco_model* m, int capacity_tokens, int page_tokens);
/* dev_pages: caller's buffer of at least disco_kv_bytes(...), 256-byte aligned.  Logical page i of
 * the sequence lives in physical page host_page_order[i] (a permutation of 0..n_pages-1), or in
 * page i when host_page_order is NULL.  page_tokens must be a multiple of 4.  Page layout:
 * [layer][physical page][K | V][kv head] blocks of page_tokens x d_head bf16; K blocks are
 * [token][d_head], V blocks are stored transposed, [d_head][token].  The rotary table of a family B
 * cache is written by the first forward that uses the cache, on that call's stream.               */
int disco_kv_create(const disco_model* m, void* dev_pages, size_t bytes, int capacity_tokens,
                    int page_tokens, const int32_t* host_page_order, disco_kv** out);
void disco_kv_destroy(disco_kv* kv);
int disco_kv_len(const disco_kv* kv);
int disco_kv_pages_in_use(const disco_kv* kv);
/* Install given keys/values, bf16 [n_layers][2][ctx][n_kv_heads][d_head], as positions [0, ctx);
 * sets len = ctx.  (Synthetic workloads pre-fill the cache this way.)                              */
int disco_kv_fill(disco_kv* kv, const void* dev_src, int ctx, disco_stream s);

/* Workspace bytes for forwards of up to max_block tokens against up to max_ctx cached positions.   */
size_t disco_workspace_bytes(const disco_model* m, int max_block, int max_ctx);
/* Must run once on a fresh workspace before its first use (and again if a launch that used it was
 * aborted): zeroes the small ticket counters with which the workgroups of a split reduction find
 * out which of them finishes last (kernels leave the counters at zero), and, for a LayerNorm model,
 * computes the two correction vectors of every matrix that reads a normalised row (W . gain and
 * W . bias of the norm in front of it: 4 one-token products per layer and 2 for the LM head, a few
 * ms for a 15B-class model) into the workspace: the forwards apply LayerNorm inside those matrices'
 * kernels.  The model's weights must therefore be in place when this runs, and it must run again if
 * they change.  A workspace belongs to the model it was initialised for and serves one stream at a time. */
int disco_workspace_init(const disco_model* m, void* dev_ws, size_t ws_bytes, int max_block, int max_ctx,
                         disco_stream s);

/* ---- the five calls of the iteration --------------------------------------------------------- */

/* Draft decode step (Sec. 2: the draft model generates autoregressively).  Feeds n_in tokens
 * (1, or 2 when the previous block was fully accepted and the draft has not yet seen its own last
 * token) from dev_tokens_in at positions kv->len .., appends their keys/values, and writes the fp32
 * logits [vocab] of the LAST fed token to dev_logits.  kv->len += n_in.
 * dev_gate (may be NULL): if *dev_gate != 0 when the kernels run, the step does nothing on the
 * device (the host still advances kv->len; roll it back with disco_kv_rollback).  The word must not
 * change while the step's launches are in flight (a step that is gated off half way leaves the
 * workspace's ticket counters non-zero: initialise the workspace again).
 * Errors: EINVAL (null/misaligned, n_in not in [1, DISCO_MAX_BLOCK]), ECAP (KV capacity).          */
int disco_draft_step(const disco_model* draft, disco_kv* kv, const int32_t* dev_tokens_in, int n_in,
                     float* dev_logits, void* dev_ws, size_t ws_bytes, const uint32_t* dev_gate,
                     disco_stream s);

/* Features and halting decision of Eq. 2 in one launch.  Reads logits [vocab]; computes the
 * soft-max's top-10 probabilities (descending), its entropy in nats, the arg-max token; evaluates
 * the classifier on [top-10, entropy, pos_feature]; halt = (score < tau) || force_halt.
 * Writes *dev_out; if dev_token_next != NULL stores the token there (input of the next draft step);
 * if dev_block_slot != NULL stores the token there too (slot of the draft block);
 * if dev_gate != NULL: the call is skipped when *dev_gate != 0, and sets *dev_gate = 1 on halt;
 * if dev_sl_count != NULL it is incremented when the call executes;
 * if dev_force_token != NULL and *dev_force_token >= 0, the logit of that token is first raised to
 * max + 4 (in dev_logits too): the synthetic-workload hook that makes the draft agree with a known
 * target token at chosen positions.  clf may be NULL (score = NaN, halt = force_halt).
 * dev_scratch (may be NULL): DISCO_CLASSIFY_SCRATCH_BYTES of device memory, 256-byte aligned,
 * prepared once by disco_classify_scratch_init and used by one stream at a time; with it the
 * reduction over the vocabulary is spread over many workgroups, without it one workgroup does it
 * all (same results up to fp32 summation order).  vocab <= 65536; dev_logits 16-byte aligned.       */
int disco_classify(const disco_clf* clf, float* dev_logits, int vocab, float pos_feature, float tau,
                   int force_halt, disco_clf_out* dev_out, int32_t* dev_token_next,
                   int32_t* dev_block_slot, uint32_t* dev_gate, int32_t* dev_sl_count,
                   const int32_t* dev_force_token, void* dev_scratch, disco_stream s);
/* Zeroes the ticket word of a classify scratch buffer (kernels leave it at zero afterwards).        */
int disco_classify_scratch_init(void* dev_scratch, disco_stream s);

/* disco_classify for callers that cannot allocate device memory or pass a scratch buffer of their own
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the many-
 * workgroup reduction uses an array inside the library's code object instead of dev_scratch
 * (DISCO_CLASSIFY_SCRATCH_BYTES per GPU, held until the process ends).  Same arguments, same results
 * and the same kernels as disco_classify with a scratch buffer; the call allocates nothing, enqueues a
 * small fill kernel that zeroes the array's ticket word and then the classify kernel.  vocab above
 * DISCO_CLASSIFY_STATIC_MAX_VOCAB is refused with DISCO_ECAP.  Every call on one GPU shares that GPU's
 * array: calls that overlap on one GPU (different streams, or replays of graphs that hold it) race;
 * serialise them.  The first call on a device looks the array's address up (make it before a capture). */
#define DISCO_CLASSIFY_STATIC_MAX_VOCAB 65536
int disco_classify_static(const disco_clf* clf, float* dev_logits, int vocab, float pos_feature, float tau,
                          int force_halt, disco_clf_out* dev_out, int32_t* dev_token_next,
                          int32_t* dev_block_slot, uint32_t* dev_gate, int32_t* dev_sl_count,
                          const int32_t* dev_force_token, disco_stream s);

/* Target verification forward (Fig. 1: the target validates all draft tokens in parallel).
 * dev_block = [last emitted token, d_1 .. d_SL], n_block = SL + 1 in [1, DISCO_MAX_BLOCK]; token j
 * sits at position kv->len + j and attends to positions <= its own (causal inside the block).
 * Appends n_block KV entries (kv->len += n_block); writes the arg-max token of every row to
 * dev_argmax[n_block] (lowest id on ties) and, if dev_logits != NULL, the fp32 logits
 * [n_block x vocab].  Errors as disco_draft_step.                                                   */
int disco_verify(const disco_model* target, disco_kv* kv, const int32_t* dev_block, int n_block,
                 int32_t* dev_argmax, float* dev_logits, void* dev_ws, size_t ws_bytes,
                 disco_stream s);

/* Greedy acceptance (Sec. 3: rejection sampling at zero temperature; Fig. 1).
 * n = the largest j <= n_block - 1 with block[i] == argmax[i-1] for all 1 <= i <= j;
 * emit = block[1..n] followed by argmax[n].  Writes *dev_out and, if host_out != NULL (pinned,
 * device-accessible host memory), the same record there.
 * dev_n_block (may be NULL) overrides n_block with a device-resident value in [1, n_block].         */
int disco_accept(const int32_t* dev_block, const int32_t* dev_argmax, int n_block,
                 const int32_t* dev_n_block, disco_accept_out* dev_out, disco_accept_out* host_out,
                 disco_stream s);

/* KV rollback of the rejected suffix (implied by Fig. 1: rejected tokens leave no state).
 * Sets len = new_len, 0 <= new_len <= len (else ESTATE); whole pages beyond it are released.  Host
 * metadata only: entries >= new_len are dead and are overwritten by the next append; work already
 * enqueued on any stream is unaffected.  new_len == len is a no-op.                                */
int disco_kv_rollback(disco_kv* kv, int new_len);

/* ---- fused draft loop (Sec. 3: draft, classify, repeat until halt or SL_max) ------------------ */

typedef struct disco_loop_out {
  int32_t sl;                         /* number of drafted tokens                                   */
  int32_t block[DISCO_MAX_BLOCK];     /* block[0] = last emitted token, block[1..sl] = draft tokens */
  int32_t halted;                     /* 1 if a step's decision (or the forced halt of the last step) ended the drafting */
} disco_loop_out;

/* Enqueues up to `cap` (draft step, classify) pairs with no host round trip: a device flag set by
 * the first halting classify turns the remaining steps into no-ops.  dev_tokens_in/n_in as in
 * disco_draft_step for the first step; pos_feature0 is the position feature of the first drafted
 * token and grows by 1 per step; static_sl > 0 forces "halt exactly at step static_sl" (static
 * lookahead) and ignores the classifier's verdict.  dev_force_tokens (may be NULL): cap entries,
 * one per step, as dev_force_token of disco_classify.  dev_steps: cap records of disco_clf_out.
 * On return the host's kv->len has advanced by n_in + steps - 1 (steps = static_sl if > 0, else
 * cap); after synchronising, the caller reads sl from host_out (pinned) or dev_out and calls
 * disco_kv_rollback(kv, len0 + n_in + sl - 1).
 * dev_logits: fp32 [vocab] scratch for the draft logits.  cap in [1, DISCO_MAX_BLOCK - 1].
 * If a launch fails (DISCO_EHIP) the host's kv->len is what it was on entry; the device-side loop state
 * (gate, counters, dev_out) is undefined and the workspace must be initialised again before its next use. */
int disco_draft_loop(const disco_model* draft, disco_kv* kv, const disco_clf* clf,
                     const int32_t* dev_tokens_in, int n_in, int cap, int static_sl,
                     float pos_feature0, float tau, const int32_t* dev_force_tokens,
                     float* dev_logits, disco_clf_out* dev_steps, disco_loop_out* dev_out,
                     disco_loop_out* host_out, void* dev_ws, size_t ws_bytes, disco_stream s);

/* Options of disco_draft_loop_ex (any pointer may be NULL; a NULL opts means none).
 *   dev_force_tokens: as in disco_draft_loop.
 *   dev_ref_tokens: cap entries, the known continuation (the target's greedy tokens at the positions
 *     being drafted; entries < 0 are ignored).  Drafting stops at the first draft token that differs
 *     from it, and that token is NOT part of the block: the "oracle" lookahead of Sec. 3 ("Finding the
 *     optimal SL per iteration"), an upper bound that needs the target's text in advance.  Then sl counts
 *     the matching tokens and sl + 1 draft steps have run (sl == cap: cap steps).
 *   dev_u_draft / dev_draft_probs / temperature: as in disco_draft_loop_sampled (not with the two above).
 *   ppl_threshold: > 0 selects the perplexity rule, the rule-based baseline of App. F (the paper names
 *     it and gives no formula; this is the usual definition): after draft token j of the block,
 *     ppl_j = exp(-(1/j) sum_{i<=j} ln p_i) with p_i the draft's probability of its own token i, and
 *     drafting stops after the first token with ppl_j > ppl_threshold (that token stays in the block)
 *     or at cap.  The step records then carry ppl_j in their score field.  Needs clf == NULL and
 *     static_sl == 0; not with dev_ref_tokens or sampling.  0 = off.                                    */
typedef struct disco_loop_opts {
  const int32_t* dev_force_tokens;
  const int32_t* dev_ref_tokens;
  float temperature;
  const float* dev_u_draft;
  float* dev_draft_probs;
  float ppl_threshold;
  /* A block drafted in several calls (the host looks at `halted` between them and enqueues more steps only
   * if drafting goes on: steps enqueued after a halt are empty launches that still cost time).
   * block_offset = k > 0: dev_out already holds k draft tokens of this block from the calls before, on the same
   * workspace; nothing is reset, step j writes block[k + j] and dev_steps[k + j - 1], dev_tokens_in points at
   * block[k] (n_in = 1), pos_feature0 and the per-step option arrays are those of step k + 1.
   * open_end != 0: the call's last step does not force a halt.  k + cap <= DISCO_MAX_BLOCK - 1.                  */
  int32_t block_offset;
  int32_t open_end;
} disco_loop_opts;

int disco_draft_loop_ex(const disco_model* draft, disco_kv* kv, const disco_clf* clf,
                        const int32_t* dev_tokens_in, int n_in, int cap, int static_sl,
                        float pos_feature0, float tau, const disco_loop_opts* opts, float* dev_logits,
                        disco_clf_out* dev_steps, disco_loop_out* dev_out, disco_loop_out* host_out,
                        void* dev_ws, size_t ws_bytes, disco_stream s);

/* ---- one speculative iteration driven from the host side of the library (Fig. 1) ------------- */

/* Device and pinned buffers one iteration works in; the caller owns them all and may reuse them for
 * every iteration of a sequence.                                                                     */
typedef struct disco_iter_buffers {
  int32_t* dev_tokens_in;          /* 2 entries: the tokens the draft model has not seen yet           */
  float* dev_logits_draft;         /* [draft vocab] fp32                                               */
  disco_clf_out* dev_steps;        /* DISCO_MAX_BLOCK - 1 step records                                 */
  disco_loop_out* dev_loop_out;
  disco_loop_out* host_loop_out;   /* pinned, device-accessible                                        */
  int32_t* dev_argmax;             /* DISCO_MAX_BLOCK entries                                          */
  disco_accept_out* dev_accept_out;
  disco_accept_out* host_accept_out;  /* pinned, device-accessible                                     */
} disco_iter_buffers;

typedef struct disco_iter_result {
  int32_t sl;                      /* draft tokens in the block                                        */
  int32_t n;                       /* accepted ones                                                    */
  int32_t draft_forwards;          /* draft steps whose result was used (sl, plus the leaving step of a reference run) */
  int32_t draft_steps_enqueued;    /* steps launched, empty ones after a halt included                 */
  int32_t block[DISCO_MAX_BLOCK];  /* block[0..sl]                                                     */
  int32_t emit[DISCO_MAX_BLOCK];   /* emit[0..n]: accepted draft tokens, then the target's token       */
} disco_iter_result;

/* One iteration of Fig. 1: draft until the policy halts or `cap` tokens are drafted, verify the block
 * with the target, accept greedily, drop the rejected suffix from both caches.  The call blocks: it
 * synchronises stream s after each chunk of draft steps and after the acceptance, and returns the
 * outcome in *host_result (ordinary host memory).
 * host_pending[n_pending] (1 or 2 host values): the tokens of the sequence that the draft cache does not
 * hold yet; the last one is the last emitted token, block[0].  cap = 0 (or draft == NULL): no drafting,
 * the target decodes one token.  static_sl, pos_feature0, tau, opts (sampling excluded; block_offset and
 * open_end are set by this call and must be 0) as in disco_draft_loop_ex.
 * chunk: draft steps enqueued between two looks at the halt flag (0 = library default; >= cap: the whole
 * loop at once, as disco_draft_loop does).  Steps enqueued after a halt are empty launches, a look at the
 * flag is a stream synchronisation: the chunk trades one for the other and does not change the result.
 * A static lookahead (static_sl > 0) is enqueued whole.
 * On return kv_target holds len0_t + n + 1 entries and kv_draft at most as many (it lacks the tokens the
 * next call passes as pending).  Errors as the calls it is made of; after an error the cache lengths are
 * those of the failing call's contract and the iteration must not be resumed.                          */
int disco_iterate(const disco_model* target, disco_kv* kv_target, void* dev_ws_target, size_t ws_target_bytes,
                  const disco_model* draft, disco_kv* kv_draft, void* dev_ws_draft, size_t ws_draft_bytes,
                  const disco_clf* clf, const int32_t* host_pending, int n_pending, int cap, int static_sl,
                  int chunk, float pos_feature0, float tau, const disco_loop_opts* opts,
                  const disco_iter_buffers* buf, disco_iter_result* host_result, disco_stream s);

/* ---- sampling at temperature > 0 (Sec. 3, last sentence; App. F) ----------------------------- */
/* The method keeps the rejection-sampling scheme of speculative decoding, which preserves the target
 * model's distribution, and is reported at temperature 1 as well.  Distributions are
 * softmax(logits / temperature); a token is drawn from a distribution by inverting its cumulative sum
 * in vocabulary order at u * total, with u uniform on [0, 1) SUPPLIED BY THE CALLER (device memory),
 * so that a run is a function of its inputs.  vocab % 4 == 0, vocab <= 65536, temperature > 0.       */

/* Draw one token per row from softmax(dev_logits[row] / temperature), rows n_rows x vocab with row
 * stride ld_logits floats (a multiple of 4).  dev_u: n_rows uniforms.  dev_probs (may be NULL)
 * receives the fp32 probability rows [n_rows x vocab]; dev_tokens the drawn ids [n_rows].             */
int disco_sample(const float* dev_logits, int n_rows, int vocab, int64_t ld_logits, float temperature,
                 const float* dev_u, float* dev_probs, int32_t* dev_tokens, disco_stream s);

/* Speculative sampling over one block.  dev_block = [last emitted token, d_1 .. d_SL];
 * dev_draft_probs[j - 1] = the distribution d_j was drawn from (rows of vocab floats);
 * dev_target_logits[j] = the target's logits after block[0..j] (n_block rows).  d_j is kept while
 * u_accept[j - 1] * q(d_j) < p(d_j); at the first rejection (after n kept tokens) the iteration's
 * last token is drawn from norm(max(0, p_n - q_n)), and from p_SL when all are kept, with
 * dev_u_resample[n] (n_block entries).  Writes n and the emitted tokens as disco_accept does.
 * dev_n_block (may be NULL) overrides n_block with a device-resident value in [1, n_block].          */
int disco_accept_sample(const int32_t* dev_block, int n_block, const int32_t* dev_n_block,
                        const float* dev_draft_probs, const float* dev_target_logits, int vocab,
                        float temperature, const float* dev_u_accept, const float* dev_u_resample,
                        disco_accept_out* dev_out, disco_accept_out* host_out, disco_stream s);

/* disco_draft_loop with sampled draft tokens: step j draws its token from
 * softmax(draft logits / temperature) with dev_u_draft[j - 1] and stores the probability row in
 * dev_draft_probs[j - 1] (cap rows of vocab floats); the classifier's features stay those of the
 * temperature-1 softmax of the raw logits.  No forced tokens.  Other arguments as disco_draft_loop.  */
int disco_draft_loop_sampled(const disco_model* draft, disco_kv* kv, const disco_clf* clf,
                             const int32_t* dev_tokens_in, int n_in, int cap, int static_sl,
                             float pos_feature0, float tau, float temperature, const float* dev_u_draft,
                             float* dev_draft_probs, float* dev_logits, disco_clf_out* dev_steps,
                             disco_loop_out* dev_out, disco_loop_out* host_out, void* dev_ws,
                             size_t ws_bytes, disco_stream s);

/* ---- classifier training and evaluation (Sec. 4 "SL classifier training", App. D.1 / D.2) ----- */
/* The paper trains the shallow FFN of Eq. 2 with a cross-entropy loss on (features, accepted /
 * rejected) pairs from a labelling run and reports F1; it names no optimiser.  Here: features are
 * standardised per component over the training set, the loss is the mean binary cross-entropy, and
 * `epochs` full-batch gradient steps of size lr are taken from the initial parameters.
 * dev_feats: [n x 12] fp32 (records of disco_classify, position feature included); dev_labels: [n]
 * int32 in {0, 1}; n <= DISCO_TRAIN_MAX_N.  dev_params: layout of disco_clf.dev_params; on entry the
 * initial parameters (read in the standardised feature space), on return the trained parameters with
 * the standardisation folded into W1 and b1, so that they apply to raw features.  dev_loss (may be
 * NULL): [epochs], the mean loss before each step.  One workgroup; results are reproducible.          */
#define DISCO_TRAIN_MAX_N 2560
int disco_clf_train(const float* dev_feats, const int32_t* dev_labels, int n, int hidden, int epochs,
                    float lr, float* dev_params, float* dev_loss, disco_stream s);

/* Scores C of n feature vectors and, if dev_labels and dev_counts are given, the confusion counts of
 * "accepted iff C >= tau" added to dev_counts[4] = {true pos., false pos., false neg., true neg.}
 * (the caller zeroes them; F1 = 2 TP / (2 TP + FP + FN)).  dev_scores may be NULL.                    */
int disco_clf_eval(const disco_clf* clf, const float* dev_feats, const int32_t* dev_labels, int n,
                   float tau, float* dev_scores, int32_t* dev_counts, disco_stream s);

/* Training examples from a labelling run (App. D.1: at every generated position the draft predicts one token
 * from the prompt plus the target's own continuation; the example is the Eq. 2 feature vector of the draft's
 * distribution, labelled by whether the draft's token equals the target's).  dev_records: the n records that
 * disco_classify wrote, one per position; dev_ref_tokens: the target's n tokens.  Writes dev_feats [n x 12],
 * dev_labels [n] (1 = equal) and, if dev_tokens != NULL, the draft's tokens [n].                          */
int disco_clf_examples(const disco_clf_out* dev_records, int n, const int32_t* dev_ref_tokens, float* dev_feats,
                       int32_t* dev_labels, int32_t* dev_tokens, disco_stream s);

/* ---- rule-based lookahead baseline (Sec. 2 footnote, Table 1 "dynHeur") ------------------------------ */

/* The heuristic the paper compares with changes the lookahead "according to the acceptance of the previous
 * iterations" and gives no constants; this is the usual rule: after an iteration whose `drafted` tokens were
 * all accepted the next lookahead is lookahead + up, otherwise lookahead - down, kept inside [1, cap]; an
 * iteration that drafted nothing leaves it unchanged.  Host arithmetic only.  Returns the next lookahead, or
 * DISCO_EINVAL (lookahead < 1, cap < 1, accepted outside [0, drafted], negative steps).                   */
int disco_heuristic_next(int lookahead, int drafted, int accepted, int up, int down, int cap);

/* ---- prompt pass (Sec. 2: both models are given the prompt before the first iteration) ----------- */

/* Processes n_tokens prompt tokens in one dense pass instead of n_tokens / DISCO_MAX_BLOCK skinny
 * forwards: the same arithmetic per token (bf16 weights, fp32-grade activations, bf16 KV entries) with
 * the GEMMs tiled for the matrix unit.  Token i sits at position kv->len + i and attends to positions
 * <= its own.  Appends n_tokens KV entries (kv->len += n_tokens).  dev_logits_last (may be NULL):
 * fp32 [vocab], the logits after the last prompt token.  The pass works on groups of 16 tokens: the
 * cache needs capacity for kv->len + 16 * ceil(n_tokens / 16) positions (entries beyond the new
 * kv->len are scratch, as always); the projection widths (d_q + 2 d_kv, and 2 d_ff or d_ff) must be
 * multiples of 64 (DISCO_EINVAL otherwise: feed such a model's prompt through disco_verify in blocks
 * instead).  dev_ws: device buffer of at least
 * disco_prefill_workspace_bytes(m, n_tokens, max_ctx >= kv->len + 16 * ceil(n_tokens / 16)) bytes,
 * 256-byte aligned, initialised once with disco_workspace_init (which zeroes the ticket counters at
 * its start; they sit at the offsets of an ordinary workspace).  Errors: EINVAL, ECAP, ESTATE, EHIP. */
#define DISCO_PREFILL_MAX 8192
size_t disco_prefill_workspace_bytes(const disco_model* m, int n_tokens, int max_ctx);
int disco_prefill(const disco_model* m, disco_kv* kv, const int32_t* dev_tokens, int n_tokens,
                  float* dev_logits_last, void* dev_ws, size_t ws_bytes, disco_stream s);

/* The prompt pass with options.  flags = 0 is disco_prefill.
 * DISCO_PREFILL_BF16_ACTIVATIONS: the matrix-unit inputs of the pass (normalised residual rows, attention output,
 * MLP activations, and inside the attention the queries and the soft-max probabilities) are rounded to bf16,
 * the usual mixed-precision arithmetic of bf16 inference, instead of being carried as a bf16 hi + lo pair
 * (fp32 grade).  Half the matrix-unit work and each weight tile fetched for twice as many tokens;
 * accumulation, residual stream, norms, soft-max statistics and the KV entries are unchanged.
 * Each GEMM then carries a relative input rounding error of up to 2^-9 per element (the weights already carry
 * one of that size), so logits and KV entries differ from those of the fp32-grade pass by a few 1e-3 of their
 * row's scale per layer pair: a pass for throughput, outside the parity statement of the decode path.       */
#define DISCO_PREFILL_BF16_ACTIVATIONS 1u
int disco_prefill_ex(const disco_model* m, disco_kv* kv, const int32_t* dev_tokens, int n_tokens,
                     float* dev_logits_last, unsigned flags, void* dev_ws, size_t ws_bytes, disco_stream s);

/* ---- launch structure ------------------------------------------------------------------------------ */

/* How a forward is cut into launches.  Process-wide; returns the previous mode, or DISCO_EINVAL.  Not to be
 * changed while calls are in flight on other threads.
 * mode 0 (default): one launch per phase (QKV projection, attention, O-projection, MLP input, MLP output per
 *   layer; LM head), except that the QKV projection and the attention of a layer share ONE launch in models of
 *   the RMSNorm / rotary / SwiGLU family whose query heads all have their own K / V head: the attention of a head
 *   needs only that head's rows of the projection, so its workgroups wait for those alone (a counter per head)
 *   instead of for the whole grid.  Every such wait is bounded; if one ever runs out (about a second; it needs the
 *   launch's workgroups not to be resident together for that long) the launch still ends, the workspace is
 *   marked, and every later result of that workspace says so -- NaN logits, -1 in disco_verify's arg-max and in
 *   disco_loop_out.sl, DISCO_EHIP from disco_iterate -- until disco_workspace_init is called again.
 * mode 1: a forward (and a whole draft loop) of that family as ONE cooperative launch of persistent workgroups
 *   with a grid barrier between the phases (in a draft loop also the features / classifier and the next token's
 *   embedding, the kernel leaving at the first halting step), where the model's shapes allow it (else mode 0 is
 *   used silently); results agree with mode 0 to fp32 summation order.
 * mode 2: one launch per phase, nothing shared; results agree with mode 0 to fp32 summation order (the context
 *   is dealt to the attention's workgroups differently).
 * On MI355X mode 0 is the fastest (a 13B-class verification block: 4.97 ms, against 5.03 ms in mode 2 and
 * 5.8 ms in mode 1; a 68M-class draft step: 76 us against 78 us and 139 us): a phase boundary inside a
 * launch costs more than a kernel boundary there, a per-head hand-off a little less.                     */
int disco_set_launch_mode(int mode);

#ifdef __cplusplus
}
#endif
#endif /* DISCO_H */
