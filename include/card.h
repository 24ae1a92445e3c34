/*
 * card.h - C ABI of libcard: the target model's multi-token verification step of CARD
 * (query-and-correct speculative decoding) on one MI355X (gfx950), plus the shared
 * candidate cache the target queries and corrects.
 *
 * What one verification step is (CARD Design, overview figure and its caption; Cache
 * Correction, last paragraph; Comparing with Tree-Verified Methods): the target model
 * forwards the chain of r candidate tokens picked from the shared cache in a single
 * plain-causal pass against its existing KV cache, compares its own arg-max prediction
 * with each candidate, keeps the longest matching prefix and emits its own next token,
 * which corrects the draft side.  At temperature 0 this reproduces plain greedy decoding
 * of the target exactly (lossless).
 *
 * Conventions for every function
 *   - returns CARD_OK (0) or a negative card_status; never throws, aborts or prints;
 *   - "dev" pointers are device memory of the current HIP device, "host" pointers are
 *     ordinary host memory; every device buffer is owned by the caller and must stay
 *     alive until the stream has finished the call;
 *   - device work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and is asynchronous; no function synchronises unless it says so;
 *   - argument errors are detected on the host before anything is enqueued.
 *   - the library allocates no device memory.
 */
#ifndef CARD_H
#define CARD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum card_status {
    CARD_OK = 0,
    CARD_EINVAL = -1,    /* null pointer, non-positive size, unsupported shape            */
    CARD_ERANGE = -2,    /* r outside [1, max_r], level / index outside the cache         */
    CARD_ECAPACITY = -3, /* ctx_len + r exceeds max_ctx or the block table                 */
    CARD_EDEVICE = -4,   /* a HIP call failed (launch error, wrong device architecture)    */
    CARD_ESTALE = -5,    /* cache write refers to an epoch that a correction has ended     */
    CARD_ETOOBIG = -6    /* card_verify_static: the model's workspace exceeds the scratch   */
} card_status;

const char* card_strerror(int status);

/* ------------------------------------------------------------------------------------------
 * Model description.  Decoder-only, pre-norm: RMSNorm, rotary embedding with half-split
 * pairing, grouped-query attention, SwiGLU feed-forward, untied vocabulary head, no biases
 * (the LLaMA / Qwen families named in Experimental Setup, "Models and Datasets").
 * Constraints: head_dim in {64, 128}; d_model a multiple of 64; d_ffn a multiple of 8;
 * n_q_heads a multiple of n_kv_heads; kv_block == 16; max_ctx a positive multiple of 16;
 * 1 <= max_r <= 32; every packed matrix below 4 GiB; 0 <= grid_wgs <= 256.
 * ---------------------------------------------------------------------------------------- */
typedef struct card_model_cfg {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rope_theta, rms_eps;
    int32_t kv_block; /* tokens per KV page: 16                                             */
    int32_t max_ctx;  /* capacity of the block table in tokens (multiple of kv_block)       */
    int32_t max_r;    /* largest r a call may pass (<= 32)                                  */
    int32_t grid_wgs; /* workgroups of the verify kernel: 0 = one per compute unit (at most
                         256); a smaller number leaves the other compute units to kernels the
                         caller runs beside it (the draft model of the paper runs in parallel
                         with the target: CARD Design, first paragraph).  The packed weight
                         order depends on it: pack and verify with the same value.            */
} card_model_cfg;

/* Tensors of the canonical (caller-side) weight set. Matrices are bf16, row-major
 * [out_features][in_features]; gains are fp32 vectors of d_model entries. */
typedef enum card_tensor {
    CARD_T_EMBED = 0,  /* [vocab][d_model]                      layer ignored */
    CARD_T_WQ = 1,     /* [n_q_heads*head_dim][d_model]                       */
    CARD_T_WK = 2,     /* [n_kv_heads*head_dim][d_model]                      */
    CARD_T_WV = 3,     /* [n_kv_heads*head_dim][d_model]                      */
    CARD_T_WO = 4,     /* [d_model][n_q_heads*head_dim]                       */
    CARD_T_WG = 5,     /* [d_ffn][d_model]   gate                             */
    CARD_T_WU = 6,     /* [d_ffn][d_model]   up                               */
    CARD_T_WD = 7,     /* [d_model][d_ffn]   down                             */
    CARD_T_LM_HEAD = 8,/* [vocab][d_model]                      layer ignored */
    CARD_T_G_ATTN = 9, /* fp32 [d_model]  gain of the norm before attention   */
    CARD_T_G_FFN = 10, /* fp32 [d_model]  gain of the norm before the FFN     */
    CARD_T_G_FINAL = 11/* fp32 [d_model]                        layer ignored */
} card_tensor;

/* Sizes of the caller-allocated device buffers (bytes; 0 if cfg is invalid). */
size_t card_packed_weight_bytes(const card_model_cfg* cfg);
size_t card_workspace_bytes(const card_model_cfg* cfg);
/* bytes of ONE of the two page pools (K or V) holding n_pages pages for all layers */
size_t card_kv_pool_bytes(const card_model_cfg* cfg, int32_t n_pages);

/* Where fragment (n-tile t, k-step s) of a packed matrix with n_tiles x k_steps fragments lives:
 * its index (in units of 1 KiB) from the start of the matrix, for batch width `batch`
 * (2 for the fused QKV matrix, 1 for the O and down projections, 8 for gate/up and the
 * vocabulary head) on a grid of `grid` workgroups.  A pure host function: it is the single
 * definition of the stream order that card_weights_pack_tensor writes and card_verify reads
 * (tile t belongs to grid position t % grid; k-step s to wavefront pair floor(4 s / k_steps);
 * inside a pair: batch of tiles, then k-step, then tile).  Returns -1 on invalid arguments. */
int64_t card_stream_frag_index(int32_t n_tiles, int32_t k_steps, int32_t batch, int32_t grid, int32_t t,
                               int32_t s);

/* Re-lays one canonical tensor (src_dev, device memory, layout above) into its place inside
 * the packed weight blob (packed_dev, card_packed_weight_bytes(cfg) bytes).  The packed
 * layout stores every matrix as 1 KiB fragments (16 rows x 32 columns in the register order of
 * the gfx950 bf16 matrix instruction), in the order in which the verify kernel's wavefronts
 * consume them, so each of them streams one contiguous run per matrix; values are moved,
 * never changed.  That order depends on the number of compute units of the CURRENT device:
 * pack on the device (or an identical one) that will verify.  The blob records the grid size;
 * card_verify on a grid of another size reports accepted_len = -1.
 * Call once per tensor (per layer for layer tensors). */
int card_weights_pack_tensor(const card_model_cfg* cfg, int32_t tensor, int32_t layer,
                             const void* src_dev, void* packed_dev, void* stream);

/* ------------------------------------------------------------------------------------------
 * Paged KV cache of the target model (bf16).  k_pages / v_pages each hold
 * card_kv_pool_bytes(cfg, n_pages) bytes; page p of layer l starts at
 * ((l * n_pages + p) * n_kv_heads) * 16 * head_dim elements.  Token position t lives in page
 * block_table[t / 16], slot t % 16.  Inside a page both K (after rotation) and V are stored in
 * the operand order of the gfx950 matrix instructions that consume them (use card_kv_gather to
 * read them back in plain order).  K and V are rounded to bf16 (nearest even) from their fp32
 * values when they are written; later rows of the same call and all later calls read the rounded
 * values.  The pools need no initialisation: positions [0, ctx_len) must have been written by
 * earlier calls, and a call that writes the first slot of a page also clears that page's slots
 * behind the ones it writes, so no step ever multiplies a zero probability with bits it did not
 * store.  One layer of a pool (n_pages * n_kv_heads * 16 * head_dim * 2 bytes) must stay below
 * 4 GiB.
 * ---------------------------------------------------------------------------------------- */
typedef struct card_kv {
    void* k_pages;              /* dev */
    void* v_pages;              /* dev */
    const int32_t* block_table; /* dev, max_ctx/16 entries, each in [0, n_pages)            */
    int32_t n_pages;
    int32_t pending_token;      /* the target's own prediction for position ctx_len (the last
                                   call's correction_token, or the arg-max after prefill);
                                   -1 = none: the first candidate is taken as given          */
} card_kv;

typedef struct card_verify_result {
    int32_t accepted_len;     /* 0..r: length of the longest prefix of the candidates that
                                 equals the target's own greedy tokens                       */
    int32_t correction_token; /* the target's token for position ctx_len + accepted_len      */
    int32_t kv_first_slot;    /* == ctx_len                                                  */
    int32_t kv_count;         /* == accepted_len: positions [first, first+count) of the KV
                                 cache now hold verified tokens; later ones are stale and
                                 are overwritten by the next call                            */
} card_verify_result;

/* One verification step (overview figure, steps 1-3: forward the queried path, accept the
 * matching prefix, emit the next token).  Forwards the r candidates at positions
 * ctx_len .. ctx_len+r-1 against kv[0, ctx_len), causal among themselves; writes K and V of
 * all r rows into the cache; candidate i is accepted iff every earlier one was and it equals
 * pred[i], where pred[0] = kv->pending_token and pred[i] = arg-max (lowest index on ties) of
 * row i-1's vocabulary logits.  Logits are never written to memory.  Every sum of the step is
 * taken per row in an order that does not depend on r (within r <= 8, r <= 16 and r <= 32 each,
 * on one grid, as long as ctx_len + r stays inside the same stretch of 512 tokens): row i of a
 * step has bit for bit the logits of the plain decode step (r = 1) at its position, so what is
 * accepted never depends on how the text is cut into steps.
 *   packed_weights_dev : blob filled by card_weights_pack_tensor
 *   kv                 : host struct (read during the call only)
 *   cand_tokens_dev    : dev (or device-visible pinned host memory, as card_step_begin uses:
 *                        the kernel reads the ids itself), r int32 token ids in [0, vocab)
 *   workspace_dev      : dev, card_workspace_bytes(cfg) bytes, prepared by card_workspace_init
 *                        once after allocation (and again after a call reported CARD_EDEVICE or
 *                        accepted_len < 0); calls sharing a workspace must not overlap
 *   out_dev            : dev (or device-visible pinned host) card_verify_result
 *   row_argmax_dev     : dev, optional (may be NULL): r int32, arg-max of each row
 * The step runs as one persistent kernel, one workgroup per compute unit (or cfg->grid_wgs of
 * them), whose workgroups meet at flag barriers in the workspace; every wait is bounded.  The
 * step ends normally and reports accepted_len = -1, correction_token = -1, kv_count = 0 when
 *   - the grid failed to meet (other work held compute units for longer than the waits last:
 *     run nothing else on the compute units this kernel is to use),
 *   - the weights were packed for another grid size,
 *   - the workspace was never prepared by card_workspace_init,
 *   - a candidate token id lies outside [0, vocab) (ids live in device memory, so the host
 *     cannot check them; the forward then ran on a clamped id and its result is void).
 * Errors: CARD_EINVAL, CARD_ERANGE (r), CARD_ECAPACITY (ctx_len + r > max_ctx), CARD_EDEVICE
 * (the device cannot hold one workgroup of the kernel per compute unit, or the launch failed);
 * nothing is enqueued on error.  Calls from several threads are fine as long as calls that
 * share a workspace do not overlap; all calls of a thread go to the thread's current device. */
int card_verify(const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv,
                int32_t ctx_len, const int32_t* cand_tokens_dev, int32_t r, void* workspace_dev,
                void* stream, card_verify_result* out_dev, int32_t* row_argmax_dev);

/* Verification at a sampling temperature (Experimental Setup: temperature 1.0 columns of the main
 * results; CARD Design: the target keeps the sampling mechanism of speculative decoding, so the
 * output is distributed as the target's own sampling).  The paper gives no formula; the reading
 * taken here: the path the cache returns is a deterministic proposal (a point mass on each
 * candidate), for which speculative sampling accepts candidate c with probability p(c) and on a
 * rejection emits a draw from p restricted to the other tokens.  Both come from ONE draw x ~ p per
 * position: accept iff x == c, else emit x.  The draw is arg-max_v (logit_v / T + G(seed, pos, v))
 * with G standard Gumbel noise from a counter-based generator keyed by the seed, the absolute
 * position of the token being drawn and the token id v:
 *     mix(x): x ^= x>>16; x *= 0x7feb352d; x ^= x>>15; x *= 0x846ca68b; x ^= x>>16   (32-bit)
 *     key = mix(mix(mix(seed_lo ^ 0x243f6a88) ^ seed_hi) ^ pos);  h = mix(key + v * 0x9e3779b9)
 *     u = ((h >> 8) + 0.5) / 2^24;  G = -ln(-ln(u))
 * so a position's token does not depend on which call computes its row: a chain of these steps
 * emits exactly the text that token-by-token sampling with the same seed emits, whatever the
 * candidates were.  temperature == 0 is card_verify.  pred[0] = kv->pending_token as before (the
 * previous call's correction token, itself such a draw).  row_token_dev receives the r draws;
 * logits_dev (optional, may be NULL; test use) the fp32 logits [r][vocab] before temperature and
 * noise. */
typedef struct card_sampling {
    float temperature; /* >= 0 */
    uint64_t seed;
} card_sampling;

int card_verify_sampled(const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv,
                        int32_t ctx_len, const int32_t* cand_tokens_dev, int32_t r,
                        const card_sampling* sampling, void* workspace_dev, void* stream,
                        card_verify_result* out_dev, int32_t* row_token_dev, float* logits_dev);

/* card_verify for callers that cannot allocate device memory or hand a workspace over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same step, same
 * results; the workspace is a 32 MiB array that lives in the library's code object (each GPU the
 * library runs on holds its own copy until the process ends), so the call allocates nothing and
 * takes no workspace argument.  Limits and rules:
 *   - card_workspace_bytes(cfg) must not exceed card_static_scratch_bytes() (32 MiB: models up to
 *     a few layers of width 512 at max_r 32), else CARD_ETOOBIG and nothing is enqueued;
 *   - every call on a GPU shares that GPU's array, which keeps the last call's contents: the
 *     first call, and a call for another cfg than the previous one, clear the part they use
 *     (a small kernel on `stream`, in front of the step); calls that overlap on one GPU race;
 *   - after a call that reported accepted_len < 0 call card_static_scratch_reset(): the next
 *     call on the current device then clears the array again before it runs.
 * Inputs and outputs are the caller's, as for card_verify. */
int card_verify_static(const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv,
                       int32_t ctx_len, const int32_t* cand_tokens_dev, int32_t r, void* stream,
                       card_verify_result* out_dev, int32_t* row_argmax_dev);
size_t card_static_scratch_bytes(void);
int card_static_scratch_reset(void);

/* Test entry point, not on the timed path: the same forward, additionally storing the fp32
 * logits [r][vocab] (dev) so that tests can bound the error of the final-layer logits. */
int card_verify_debug_logits(const card_model_cfg* cfg, const void* packed_weights_dev,
                             const card_kv* kv, int32_t ctx_len, const int32_t* cand_tokens_dev,
                             int32_t r, void* workspace_dev, void* stream,
                             card_verify_result* out_dev, int32_t* row_argmax_dev,
                             float* logits_dev);

/* Prepares a freshly allocated workspace (card_workspace_bytes(cfg) bytes, dev, 16-byte aligned):
 * clears all of it (barrier words, flags and arrival counters start at zero; hand-over bytes
 * that a step never writes must be finite) and marks it as prepared.  Asynchronous on `stream`;
 * allocates nothing. */
int card_workspace_init(const card_model_cfg* cfg, void* workspace_dev, void* stream);

/* Measurement hooks (benchmark only; one user at a time; allocate no device memory).
 * card_profile_enable: while enabled, card_verify brackets its kernel with a pair of HIP
 * events recorded on the call's stream, up to max_launches pairs; card_profile_collect waits
 * for them, writes each launch's duration in milliseconds to ms_host (host array of
 * max_launches floats), returns the count in *n_host and disables the hook.
 * card_profile_disable switches the hook off and destroys its events: call it before the process
 * ends (the library never touches the HIP runtime from a static destructor).
 * card_profile_timeline: buf_dev = device array of 32 uint64 per workgroup (256 workgroups), or
 * NULL to switch off; while set, the verify kernel stores 100 MHz timestamps of the phase
 * boundaries of decoder layer `layer` there.  Slots per workgroup (consumer wavefront 0):
 * 0 start, 1 QKV done, 2 barrier, 3 attention done, 4 barrier, 5 O-proj done, 6 barrier,
 * 7 gate/up done, 8 barrier, 9 down done, 10 barrier; 11 end of the QKV k-loop, 16 page
 * preload issued, 12 QKV stores acknowledged; attention workgroups: 13 page loop entered,
 * 14 left, 15 wavefronts merged, 29 partial stored, 30 arrival counted, 31 cuts merged;
 * 17-20 the producer of wavefront pair 0 starts streaming the QKV / O / gate-up / down matrix;
 * 21-23 / 24-26 / 27-28 QKV / O-projection / down phase: first activations arrived, k-loop left,
 * ticks the k-loop spent waiting for weight fragments (a duration, not a time stamp; the down
 * phase has no such slot). */
int card_profile_enable(int32_t max_launches);
int card_profile_collect(float* ms_host, int32_t* n_host);
int card_profile_disable(void);
int card_profile_timeline(void* buf_dev, int32_t layer);

/* Test helper: copies K (rotated) and V of positions [first_slot, first_slot+count) of one
 * layer out of the paged cache into plain fp32 arrays [count][n_kv_heads][head_dim] (dev). */
int card_kv_gather(const card_model_cfg* cfg, const card_kv* kv, int32_t layer,
                   int32_t first_slot, int32_t count, float* k_out_dev, float* v_out_dev,
                   void* stream);

/* ------------------------------------------------------------------------------------------
 * Shared candidate cache (Cache Construction, eqs. (1)-(9); Cache Correction).  A host object:
 * a tree whose level l is the primary cache C^(l) - at most K nodes (token, path score w of
 * eq. (3), index of the parent in level l-1, i.e. the tuples of the secondary cache, eq. (5),
 * that survived the top-K selection of eqs. (6)-(7)).  Level 0 holds the candidates for the
 * next position the target has not verified.  One writer (draft side) and one reader (target
 * side) may call concurrently: every function takes the object's lock.
 * ---------------------------------------------------------------------------------------- */
typedef struct card_cache card_cache;

int card_cache_create(int32_t K, int32_t max_depth, card_cache** out);
void card_cache_destroy(card_cache* c);

/* Draft side: store level `level` (<= current depth; an existing level is replaced and deeper
 * ones dropped).  tokens / parent_idx / path_score: host arrays of n <= K entries; parents
 * index level-1 and are -1 at level 0.  `epoch` must equal card_cache_epoch() as read when
 * the writer last synchronised with the corrections, else CARD_ESTALE and nothing changes. */
int card_cache_write(card_cache* c, int64_t epoch, int32_t level, int32_t n, const int32_t* tokens,
                     const int32_t* parent_idx, const float* path_score);

/* Target side, before a step: look the just-verified token up among the level-0 nodes (the
 * best-scored one on duplicates).  On a hit writes the best path below it - starting with the
 * verified token itself, following parent links down to the highest-scored descendant on the
 * deepest reachable level, at most max_len tokens - and returns 1; returns 0 on a miss. */
int card_cache_query(const card_cache* c, int32_t verified_token, int32_t max_len,
                     int32_t* out_tokens, int32_t* out_len, float* out_score);

/* Target side, after a step: walk the n verified tokens down from level 0, make the children of
 * the last matched node the new level 0 and drop everything outside its subtree (a rejected
 * path's siblings stay available).  A token without a node empties the cache.  Increments the
 * epoch.  Returns 1 if the chain was found, 0 if the cache was emptied. */
int card_cache_correct(card_cache* c, const int32_t* verified_tokens, int32_t n);

int64_t card_cache_epoch(const card_cache* c);
int32_t card_cache_depth(const card_cache* c);
/* copies level `level` out (host arrays of at least K entries; any may be NULL); returns the
 * node count or a negative status */
int card_cache_read_level(const card_cache* c, int32_t level, int32_t* tokens, int32_t* parent_idx,
                          float* path_score);

/* ------------------------------------------------------------------------------------------
 * Draft side: construction of one cache level on the device (Cache Construction, eqs. (1)-(9);
 * Mask Construction for Draft Model).  The draft model - any model in the same packed format -
 * forwards the nodes of the primary cache's current level in one pass and expands each into its
 * k most probable next tokens; the K best-scored extensions form the next level.
 *
 * card_draft_level, eqs. (1)-(2): forwards n_rows <= max_r tree nodes.  Row i carries token
 * tokens_dev[i] at sequence position positions_dev[i] (context length + depth of the node); its
 * key and value are stored in cache slot first_slot + i (slots of tree nodes lie behind the
 * committed context: first_slot >= ctx_len).  Visibility (the mask rules: a node inherits its
 * parent's causal history and sees itself, never its peers): every slot below mask_base is
 * visible; slot mask_base + j is visible to row i iff bit j % 32 of mask_dev[i * mask_words + j / 32]
 * is set.  mask_base is a multiple of 16, at most ctx_len (bits of context slots at or above
 * mask_base must be set by the caller); first_slot + n_rows <= mask_base + 32 * mask_words;
 * mask_words <= 32 (1024 tree slots).  A level wider than max_r rows is forwarded in several
 * calls (peers do not see each other, so the calls are independent).  Results, without the
 * logits ever being stored: per row the k <= 16 most probable tokens (most probable first, equal
 * logits by ascending token id) and their probabilities under softmax over the whole vocabulary.
 * logits_dev (optional, test use): fp32 [n_rows][vocab].  Errors as card_verify.
 *
 * card_cache_select, eqs. (3)-(7): scores every (parent i, its j-th token) pair
 * w = prob[i][j] * sigma[i] (sigma: cumulative probability of parent i's sequence, eq. (4)),
 * pools the n_parents * k tuples (eq. (5)), sorts them by score (eq. (6)) and keeps the K best
 * (eq. (7)): out_tokens / out_scores / out_parents [K], best first, equal scores by (parent, rank).
 * n_parents * k <= 2048.  Entries of topk_tokens_dev that are negative are skipped; if fewer than
 * the returned count remain, the outputs behind them are marked empty (token -1, score 0, parent
 * -1).  Returns the number of entries written, min(K, n_parents * k), or a negative status.  Appending token m to
 * parent m's sequence (eqs. (8)-(9)) is what card_cache_write stores from these arrays.
 * ---------------------------------------------------------------------------------------- */
/* Host helper, Mask Construction for Draft Model: the mask rows of one level from the rows of
 * the level above.  Row i = row parent_idx_host[i] of parent_mask_host (inherited causal history;
 * parent -1: a root, which sees only the context slots in [mask_base, ctx_len)) plus the bit of
 * its own slot first_slot + i.  Arrays are host memory, [rows][mask_words]. */
int card_tree_mask_level(const uint32_t* parent_mask_host, const int32_t* parent_idx_host,
                         int32_t n_rows, int32_t first_slot, int32_t ctx_len, int32_t mask_base,
                         int32_t mask_words, uint32_t* out_mask_host);

typedef struct card_tree_rows {
    const int32_t* tokens_dev;     /* [n_rows] */
    const int32_t* positions_dev;  /* [n_rows] */
    int32_t first_slot;
    const uint32_t* mask_dev;      /* [n_rows][mask_words] */
    int32_t mask_words;
    int32_t mask_base;
} card_tree_rows;

int card_draft_level(const card_model_cfg* cfg, const void* packed_weights_dev, const card_kv* kv,
                     int32_t ctx_len, const card_tree_rows* rows, int32_t n_rows, int32_t k,
                     void* workspace_dev, void* stream, int32_t* topk_tokens_dev,
                     float* topk_probs_dev, float* logits_dev);
int card_cache_select(const float* sigma_dev, const int32_t* topk_tokens_dev,
                      const float* topk_probs_dev, int32_t n_parents, int32_t k, int32_t K,
                      int32_t* out_tokens_dev, float* out_scores_dev, int32_t* out_parents_dev,
                      void* stream);

/* ------------------------------------------------------------------------------------------
 * One target step of the query-and-correct loop in two calls (overview figure: query the cache
 * with the token just verified, verify the returned path, correct the cache with what was
 * verified; Comparing with Tree-Verified Methods: the number of verified tokens varies from step
 * to step with what the cache holds).
 * card_step_begin: looks kv->pending_token (>= 0: the token verified last) up in the cache; on a
 * hit the candidates are the returned path, 1..max_len tokens starting with that token; on a miss
 * the step falls back to a plain decode step, r = 1, on the token itself.  The candidates are
 * written to cand_staging (int32[max_len], host memory the device can read: pinned, allocated
 * with hipHostMalloc) and the step is enqueued on `stream` like card_verify; `out` must be
 * readable by the host after the stream has finished (pinned host memory, or copy it back).
 * step_host (host) records the candidates for card_step_end.
 * card_step_end, after the stream has finished: writes the tokens the step emitted (the accepted
 * path tokens behind the query key, then the target's own token: out->accepted_len of them) to
 * emitted_host (int32[max_len]) and re-roots the cache (card_cache_correct with the accepted
 * candidates: level 0 then holds the children of the last accepted node, among which the next
 * step looks the target's own token up).  flags = CARD_STEP_NO_CORRECT skips the
 * correction: the "query without correct" variant of the ablation study, in which the cache is
 * queried but never re-rooted by the target.  Returns CARD_EDEVICE if out reports a failed step.
 * ---------------------------------------------------------------------------------------- */
typedef struct card_step {
    int32_t r;          /* candidates forwarded by this step                     */
    int32_t hit;        /* 1: the cache had a path for the token, 0: plain decode */
    float path_score;   /* score of the returned path (0 on a miss)              */
    int32_t cand[32];
} card_step;

enum { CARD_STEP_NO_CORRECT = 1 };

int card_step_begin(card_cache* cache, const card_model_cfg* cfg, const void* packed_weights_dev,
                    const card_kv* kv, int32_t ctx_len, int32_t max_len, int32_t* cand_staging,
                    void* workspace_dev, void* stream, card_verify_result* out,
                    int32_t* row_argmax_dev, card_step* step_host);
/* card_step_begin at a sampling temperature (card_verify_sampled in place of card_verify: the
 * loop then emits the text of token-by-token sampling with the same seed; the T = 1 columns of
 * the main results).  row_token_dev receives the draws.  card_step_end is the same. */
int card_step_begin_sampled(card_cache* cache, const card_model_cfg* cfg, const void* packed_weights_dev,
                            const card_kv* kv, int32_t ctx_len, int32_t max_len, int32_t* cand_staging,
                            void* workspace_dev, void* stream, card_verify_result* out,
                            int32_t* row_token_dev, card_step* step_host, const card_sampling* sampling);
int card_step_end(card_cache* cache, const card_step* step_host, const card_verify_result* out_host,
                  int32_t flags, int32_t* emitted_host, int32_t* n_emitted_host);

#ifdef __cplusplus
}
#endif
#endif /* CARD_H */
