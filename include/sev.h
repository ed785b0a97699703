/*
 * sev — batched speculative verification on one MI355X (gfx950).
 *
 * The library implements the server half of the disaggregated draft/verify
 * cycle (paper section 4.1): edges send candidate tokens, the server scores all
 * candidates of all batched requests in ONE target-model forward pass with
 * per-sequence masking over heterogeneous cache lengths (section 4.3,
 * "Processing heterogeneous requests"), returns the accepted tokens plus one
 * additional token from its own forward pass, and brings its KV cache in line
 * with the accepted tokens (section 4.2, "Post-verification update").
 *
 * Conventions
 *   - Plain C ABI.  Every function returns 0 (SEV_OK) or a negative sev_status;
 *     sev_last_error() gives a thread-local message for the last failure.
 *     No exception crosses the boundary.
 *   - Pointers are marked [host] or [device].  The caller owns every buffer it
 *     passes; the library owns only the opaque handles and the activation
 *     workspace it allocates inside sev_kv_create.
 *   - Calls that take a `stream` (a hipStream_t passed as void*, NULL = default
 *     stream) only enqueue work and return; outputs are valid once the caller
 *     has synchronised that stream.  Argument validation is done on the host
 *     before anything is launched; a failed call launches nothing.
 *   - Target model: decoder-only pre-norm transformer, RMSNorm, rotary embedding
 *     on half-split pairs (element i with i+head_dim/2, angle pos*base^(-2i/hd)),
 *     grouped-query attention, SwiGLU feed-forward, untied output head, no biases.
 *   - Acceptance is greedy exact match (temperature 0): a candidate is accepted
 *     iff it equals the target's arg-max prediction given its accepted
 *     ancestors; arg-max ties go to the lowest token id.
 */
#ifndef SEV_H
#define SEV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SEV_OK = 0,
    SEV_EINVAL = -1,    /* bad pointer, shape, index or unsupported configuration       */
    SEV_ESTATE = -2,    /* call not valid in the handle's current state                 */
    SEV_ENOSPACE = -3,  /* pages / workspace / arena do not cover the request           */
    SEV_EHIP = -4       /* the HIP runtime reported an error                            */
} sev_status;

enum { SEV_F32 = 0, SEV_BF16 = 1 };

/* Weight tensor kinds for sev_model_load_tensor.  Matrices are given in canonical
 * [out_features][in_features] row-major layout (y = x * W^T), in the model dtype:
 *   EMBED, LM_HEAD [vocab][d];  WQ [Hq*hd][d];  WK, WV [Hkv*hd][d];  WO [d][Hq*hd];
 *   WG, WU [d_ffn][d];  WD [d][d_ffn].
 * Norm gains are float32 vectors [d] (always float32) and default to 1. */
enum {
    SEV_W_EMBED = 0, SEV_W_WQ = 1, SEV_W_WK = 2, SEV_W_WV = 3, SEV_W_WO = 4,
    SEV_W_WG = 5, SEV_W_WU = 6, SEV_W_WD = 7, SEV_W_LM_HEAD = 8,
    SEV_W_NORM_ATTN = 9, SEV_W_NORM_FFN = 10, SEV_W_NORM_FINAL = 11
};

#define SEV_MAX_DRAFT 64   /* draft nodes per request and per call (ancestor sets are 64-bit masks) */
#define SEV_MAX_BATCH 256  /* requests per call */

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rope_base, rms_eps;
    int32_t dtype;          /* SEV_F32 or SEV_BF16: storage type of weights and KV cache */
} sev_model_desc;

typedef struct sev_model sev_model;   /* shape + the weight arena (borrowed device memory)            */
typedef struct sev_kv sev_kv;         /* page pools, page tables, per-slot length / next token / pending block */

/* ---------------------------------------------------------------- model ---- */

/* Bytes of device memory the model's weights occupy in the library's own
 * layout (bf16 matrices are re-tiled for the matrix cores at load time).
 * Returns 0 for an unsupported description. */
size_t sev_model_arena_bytes(const sev_model_desc *desc);

/* Creates a model over a caller-allocated, 256-byte aligned [device] arena of at least
 * sev_model_arena_bytes(desc) bytes; the arena must outlive the model.  Norm
 * gains are set to 1 (enqueued on the default stream); all matrices must then
 * be loaded with sev_model_load_tensor before the first verify.
 * SEV_F32 supports any even head_dim <= 256; SEV_BF16 requires head_dim 128,
 * d_model, d_ffn, n_q_heads*head_dim multiples of 64 and vocab a multiple of 32. */
int sev_model_create(const sev_model_desc *desc, void *arena /*[device]*/, size_t arena_bytes,
                     sev_model **out);
int sev_model_destroy(sev_model *m);

/* Converts one tensor from the canonical layout (src, [device], model dtype;
 * float32 for norm gains) into its place in the arena.  `layer` is ignored for
 * EMBED, LM_HEAD and NORM_FINAL.  src may be reused once `stream` has passed
 * this call.  Enqueues only. */
int sev_model_load_tensor(sev_model *m, int kind, int layer, const void *src /*[device]*/,
                          void *stream);

/* ------------------------------------------------------------- KV cache ---- */

/* Bytes of one page pool covering n_pages pages of page_size tokens for all
 * layers, K and V together. */
size_t sev_kv_pool_bytes(const sev_model *m, int64_t n_pages, int page_size);

/* Creates the cache state for up to max_requests request slots over a caller-
 * allocated [device] pool (256-byte aligned, >= sev_kv_pool_bytes).  Also allocates the
 * activation workspace for up to max_rows draft tokens per call (sum over the
 * batch) — the only device allocation the library makes.  page_size must be 16.
 * Every slot starts empty (length 0, no pages, next token -1).
 * The pool must be cleared (all zero bytes) before its first use: cache slots that a mask hides
 * (the tail of a request's last page, padding) still enter the attention products with weight 0,
 * so they must not hold NaN or infinity bit patterns. */
int sev_kv_create(const sev_model *m, int max_requests, int max_rows, int64_t n_pages,
                  int page_size, void *pool /*[device]*/, size_t pool_bytes, sev_kv **out);
int sev_kv_destroy(sev_kv *kv);

/* Assigns physical pages to a slot: page_ids [host] int32[n_pages], each in
 * [0, n_pages of the pool); logical token t of the slot lives in page
 * page_ids[t / page_size].  Pages may be non-contiguous and in any order; the
 * caller keeps slots' page sets disjoint.  Enqueues the table upload on `stream`. */
int sev_kv_set_pages(sev_kv *kv, int slot, const int32_t *page_ids /*[host]*/, int n_pages,
                     void *stream);

/* Sets the committed length and the target's prediction for the next position of B
 * slots at once (used after importing cache contents, and to rewind a slot to an
 * earlier committed state).  slots, seq_lens, next_toks are [host] int32[B]
 * (slots NULL = 0..B-1; next_tok -1 = unknown).  Clears any pending block.  One
 * kernel launch; the arrays are copied at call time. */
int sev_kv_set_state(sev_kv *kv, const int32_t *slots /*[host]*/, const int32_t *seq_lens /*[host]*/,
                     const int32_t *next_toks /*[host]*/, int B, void *stream);

/* Copies n_tokens positions starting at logical position `start` of one layer
 * of a slot between the paged cache and a plain [n_tokens][n_kv_heads][head_dim]
 * array in the model dtype ([device]); `to_cache` != 0 writes the cache.  Does
 * not change the slot's length.  For cache import/export and for tests. */
int sev_kv_copy_tokens(sev_kv *kv, int slot, int layer, int start, int n_tokens,
                       void *k /*[device]*/, void *v /*[device]*/, int to_cache, void *stream);

/* Reads back a slot's committed length, next-token prediction and the sticky
 * device-side error flags of the handle (synchronises `stream`).  Flags:
 * bit 0 = a verify saw prefix_lens != committed length, bit 1 = malformed parent
 * array (parent index not smaller than the child's), bit 2 = token id out of range. */
int sev_kv_get_state(sev_kv *kv, int slot, int32_t *seq_len, int32_t *next_tok,
                     uint32_t *error_flags, void *stream);

/* ---------------------------------------------------------------- verify --- */

/* The batched verification step (paper sections 4.1 and 4.3).
 *
 * Request b (b = 0..B-1) uses cache slot b, whose committed prefix has length
 * prefix_lens[b] ([host] int32[B]; must equal the slot's length — checked on the
 * device, see error flag bit 0).  draft_tokens is [device] int32[B][k]: the k
 * candidate tokens of each request.  draft_mask selects the attention mask among
 * candidates: NULL = chain (candidate i follows candidate i-1: causal mask);
 * otherwise [device] int32[B][k] parent indices (-1 = child of the committed
 * prefix, else the index of an earlier candidate), which the library expands to
 * the ancestor-or-self mask; candidate i sits at position prefix_len+depth(i).
 *
 * One forward pass of the target model scores all B*k candidates; candidate
 * K/V are written to cache positions prefix_len + i (pending).  Then, per request,
 * greedy acceptance walks from the prefix: the first candidate (a child of the
 * prefix) is compared with the slot's next-token prediction, each further one
 * with the arg-max at its accepted parent.
 *   accept_len[b]  [device] int32: number of accepted candidates (0..k)
 *   bonus_token[b] [device] int32: the target's prediction after the last accepted
 *                  candidate (the slot's own next-token prediction if none).
 * The slot is left PENDING: sev_kv_commit keeps the accepted candidates' K/V,
 * sev_kv_rollback drops the block; a new verify on a pending slot implies rollback.
 * Requires k <= SEV_MAX_DRAFT, B <= SEV_MAX_BATCH, B*k <= max_rows, and pages
 * covering prefix_lens[b] + k tokens in every slot (SEV_ENOSPACE otherwise). */
int sev_verify(const sev_model *weights, sev_kv *kv_cache, const int32_t *prefix_lens /*[host]*/,
               const int32_t *draft_tokens /*[device]*/, const int32_t *draft_mask /*[device]*/,
               int B, int k, int32_t *accept_len /*[device]*/, int32_t *bonus_token /*[device]*/,
               void *stream);

/* Extended form: arbitrary slot mapping, ragged draft lengths, debug outputs and
 * the forced-accept mode used to fill caches. */
typedef struct {
    int32_t B;                    /* requests in this call                                              */
    int32_t k_max;                /* row stride of draft_tokens / parents / accept_path                 */
    const int32_t *slots;         /* [host] int32[B] cache slot of each request; NULL = 0..B-1; distinct */
    const int32_t *prefix_lens;   /* [host] int32[B]                                                    */
    const int32_t *draft_lens;    /* [host] int32[B] candidates per request (1..k_max); NULL = k_max    */
    const int32_t *draft_tokens;  /* [device] int32[B][k_max]; entries beyond draft_lens[b] are ignored */
    const int32_t *parents;       /* [device] int32[B][k_max] or NULL for chains                        */
    int32_t mode;                 /* 0 = verify; 1 = append: accept every candidate of a chain          */
                                  /*     (cache fill / teacher forcing), bonus = arg-max after the last */
                                  /* | 2 = padded-KV comparison variant (bfloat16 path): the paper's     */
                                  /*     handling of heterogeneous batches (section 4.3: every sequence  */
                                  /*     padded to the longest of the batch under a per-sequence mask):  */
                                  /*     attention walks max_b(prefix_len + draft_len) cache slots of    */
                                  /*     EVERY request, the ones past its own end masked.  Same results, */
                                  /*     the longest sequence's cost; every slot's pages must cover that */
                                  /*     length (SEV_ENOSPACE otherwise)                                 */
    int32_t *accept_len;          /* [device] int32[B]                                                  */
    int32_t *bonus_token;         /* [device] int32[B]                                                  */
    int32_t *accept_path;         /* [device] int32[B][k_max] accepted candidate indices in order, -1 padded; may be NULL */
    int32_t *row_argmax;          /* [device] int32[sum of draft_lens] target arg-max at every candidate, packed by request; may be NULL */
    float *logits;                /* [device] float32[sum of draft_lens][vocab], debugging/parity only; may be NULL */
} sev_verify_args;

int sev_verify_ex(const sev_model *weights, sev_kv *kv_cache, const sev_verify_args *args,
                  void *stream);

/* Stochastic verification: the rule the paper's method inherits from speculative sampling
 * (section 4.1: the cycle preserves the server model's output distribution exactly; section 5:
 * all models run at temperature 0.7), in its multi-step form for trees (section 2, tree-based
 * speculative decoding).  One forward over the draft block as in sev_verify_ex; then, per
 * request: the block's root must be the token the server emitted in the previous step (a node
 * with parent -1 whose token is the slot's next token, lowest index first; no random number is
 * spent on it; without one nothing is accepted and that token is returned).  At the current
 * node, p = softmax(logits computed there / temperature); its children are tried in index
 * order: child c (token x, drawn by the edge from q_c) is accepted iff u_accept[b][c] * q_c(x) <
 * p(x); a rejection replaces p by the normalised residual max(0, p - q_c); an acceptance moves
 * to c.  When no child is left, the emitted token is drawn from the current p by inverse CDF in
 * token-id order with u_emit[b].  A chain is the tree whose node i has parent i - 1 (parents =
 * NULL).  All random numbers are inputs.  The slot is left pending exactly as after sev_verify_ex
 * (accepted path, emitted token as the next token): sev_kv_commit / sev_kv_rollback apply.
 * More than 16 rejected siblings at one node set error flag bit 3 (the rest are ignored).
 *   draft_probs   [device] float32[sum of draft lengths][vocab], rows packed like the GEMM rows
 *                 (request 0's candidates, then request 1's, ...); row of candidate 0 is unused
 *   u_accept      [device] float32[B][k_max], u_emit [device] float32[B], all in [0, 1)
 *   logits_ws     [device] float32[sum of draft lengths][vocab]: caller-provided workspace; holds
 *                 the block's logits on return
 *   accept_len, emitted_token [device] int32[B]
 * Errors as sev_verify_ex (trees: k_max <= 64 nodes, parents precede children). */
typedef struct {
    int32_t B, k_max;
    const int32_t *slots;         /* [host] or NULL */
    const int32_t *prefix_lens;   /* [host] */
    const int32_t *draft_lens;    /* [host] or NULL */
    const int32_t *draft_tokens;  /* [device] int32[B][k_max] */
    const int32_t *parents;       /* [device] int32[B][k_max] or NULL (chains), as in sev_verify_args */
    const float *draft_probs;
    const float *u_accept;
    const float *u_emit;
    float temperature;
    float *logits_ws;
    int32_t *accept_len;
    int32_t *emitted_token;
    int32_t *accept_path;         /* [device] int32[B][k_max] accepted node indices, -1 padded; may be NULL */
} sev_sample_args;

int sev_verify_sample(const sev_model *weights, sev_kv *kv_cache, const sev_sample_args *args, void *stream);

/* sev_verify_sample for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same step, but the block's logits -- the one scratch buffer
 * sev_verify_sample takes from its caller -- live in a static device array of SEV_STATIC_SCRATCH_BYTES inside the
 * library (one copy per GPU, held until the process ends).  args->logits_ws must be NULL; everything else is as in
 * sev_verify_sample, outputs included (the logits themselves are not returned).  The call makes no hipMalloc /
 * hipFree and uses no allocating library routine; it needs sev_profile_enable to be off (SEV_ESTATE otherwise).
 * SEV_ENOSPACE if (sum of draft lengths) * vocab * 4 bytes exceeds SEV_STATIC_SCRATCH_BYTES.
 * All calls on one GPU share the array: calls that overlap on one GPU (different streams, different handles) race;
 * the array keeps the previous call's contents, and every row a call reads it has written first. */
#define SEV_STATIC_SCRATCH_BYTES (64u << 20)
int sev_verify_sample_static(const sev_model *weights, sev_kv *kv_cache, const sev_sample_args *args, void *stream);

/* Prefill: the step before verification (appendix "Additional Details on
 * Evaluation Setup": the prompt is prefilled on the server before decoding starts
 * and is excluded from the reported metrics).  Appends n_tokens[b] tokens to the
 * cache of each listed slot under a causal mask: token i of the block sits at
 * position start_lens[b] + i and attends every position up to its own.  Nothing is
 * accepted or rejected.  Blocks longer than the cache's row budget are processed
 * in chunks; every chunk is committed before the next one starts.  On completion
 * (stream order) the slot's length is start_lens[b] + n_tokens[b] and its
 * next-token prediction is the arg-max after the last token.
 *   slots       [host]   int32[B] or NULL (= 0..B-1)
 *   start_lens  [host]   int32[B]; must equal the slots' current lengths (checked on the
 *                        device: error flag bit 0 of sev_kv_get_state)
 *   n_tokens    [host]   int32[B], each 1..t_max
 *   tokens      [device] int32[B][t_max]; entries beyond n_tokens[b] are ignored
 * Errors: SEV_EINVAL (null pointers, B, lengths, slots), SEV_ENOSPACE (pages of a slot do not
 * cover start + n), SEV_EHIP.  Any pending verify of a listed slot is dropped. */
int sev_prefill(const sev_model *weights, sev_kv *kv_cache, const int32_t *slots /*[host]*/,
                const int32_t *start_lens /*[host]*/, const int32_t *n_tokens /*[host]*/,
                const int32_t *tokens /*[device]*/, int B, int t_max, void *stream);

/* Applies the last verify of each listed slot (paper section 4.2: the cache is
 * updated according to the accepted tokens): the accepted candidates' K/V are
 * moved to positions len..len+a-1 (chains: already in place), the slot's length
 * grows by accept_len and its next-token prediction becomes bonus_token.
 * slots is [host] int32[B] (NULL = 0..B-1).  The accepted lengths are read on the
 * device; no host round trip.  A slot without a pending block is left unchanged. */
int sev_kv_commit(sev_kv *kv, const int32_t *slots /*[host]*/, int B, void *stream);

/* Drops the pending block of each listed slot: length and next-token prediction
 * stay as before the verify. */
int sev_kv_rollback(sev_kv *kv, const int32_t *slots /*[host]*/, int B, void *stream);

/* ------------------------------------------------------------------ misc --- */

const char *sev_last_error(void);

/* Per-kernel-class device time, measured with HIP events recorded on the launch
 * stream around every launch of the selected classes.  sev_profile_enable resets
 * the totals and selects classes by bit mask (bit i = class i, 0 = off; off by
 * default).  sev_profile_read waits for the recorded events and returns the total
 * milliseconds and the number of timed spans of class `which` since the reset.
 * See sev_profile_name for the classes. */
int sev_profile_enable(sev_kv *kv, unsigned class_mask);
int sev_profile_read(sev_kv *kv, int which, double *total_ms, int64_t *launches);
const char *sev_profile_name(int which);   /* NULL beyond the last class */

#ifdef __cplusplus
}
#endif
#endif /* SEV_H */
