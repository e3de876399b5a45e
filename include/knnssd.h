/*
 * knnssd.h - C ABI of the MI355X-native KNN-SSD decode path.
 *
 * KNN-SSD (paper Sec. 4): a decoder-only LLM M with L = 2*n_blocks skippable
 * sublayers (attention and MLP counted separately, Sec. 3.1) drafts tokens with
 * a subset of its own sublayers, M(z), and verifies them with the full model in
 * one forward pass (Sec. 4.2). Which skip set z is used is decided per sample
 * by a nearest-neighbour search of the prompt's last hidden vector among stored
 * anchor vectors (Sec. 4.2, Eq. 4-6). Decoding is greedy, so the emitted tokens
 * are exactly the full model's own greedy continuation (Sec. 3.1).
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses, "host" pointers host addresses.
 *   - The caller owns every device buffer (weights, KV cache, workspace, anchor
 *     table) and the HIP stream; the library allocates no device memory. All
 *     buffers must stay valid until knnssd_destroy.
 *   - Every matrix is given row-major [out_features][in_features]; weight_dtype says
 *     whether matrices hold fp32 or bf16 values. RMSNorm gains are always fp32. For the
 *     tuned bf16 kernels the caller repacks each matrix once into stream order
 *     (knnssd_pack_matrix) and sets cfg.weights_packed.
 *   - Skip mask layout: mask[2*b] = 1 skips the attention sublayer of block b,
 *     mask[2*b+1] = 1 skips its MLP sublayer (z_i = 1 means "skip", Sec. 3.1).
 *   - Activations, residual stream, RoPE, softmax and all accumulators are fp32;
 *     keys/values are rounded to kv_dtype (nearest-even) when they are cached.
 *   - Every call returns KNNSSD_OK (0) or a negative error code. Arguments are
 *     validated before anything is launched. Calls are synchronous with respect
 *     to their host outputs (the stream is drained before scalars are returned).
 *     A context is not thread-safe.
 */
#ifndef KNNSSD_H
#define KNNSSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KNNSSD_OK 0
#define KNNSSD_EINVAL (-1)      /* null pointer or malformed argument                     */
#define KNNSSD_ESHAPE (-2)      /* shape not supported by the kernels                     */
#define KNNSSD_ERANGE (-3)      /* position / length / token id outside the valid range   */
#define KNNSSD_EDEGENERATE (-4) /* zero-norm or non-finite query / anchor (cosine undefined) */
#define KNNSSD_ESTATE (-5)      /* call made in the wrong order                           */
#define KNNSSD_EHIP (-6)        /* a HIP runtime call failed                              */

#define KNNSSD_FP32 0
#define KNNSSD_BF16 1

#define KNNSSD_PREFILL_AUTO 0
#define KNNSSD_PREFILL_CHUNKED 1
#define KNNSSD_ATTN_MFMA 0
#define KNNSSD_ATTN_VALU 1
#define KNNSSD_MERGE_FUSED 0
#define KNNSSD_MERGE_SEPARATE 1

#define KNNSSD_MAX_ROWS 16  /* rows one verification pass can carry: max_draft + 1 <= 16 */

typedef struct knnssd_model_cfg {
    int32_t n_blocks, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t max_seq;      /* KV-cache capacity in positions                          */
    int32_t max_anchors;  /* largest anchor table knnssd_set_anchors will be given   */
    float rope_base;      /* RoPE: rotate-half pairs (i, i+head_dim/2), angle pos*base^(-2i/head_dim) */
    float rms_eps;
    int32_t weight_dtype; /* KNNSSD_FP32 | KNNSSD_BF16 */
    int32_t kv_dtype;     /* KNNSSD_FP32 | KNNSSD_BF16 */
    int32_t weights_packed; /* 1: wqkv/wo/wgu/wdown/lm_head are in stream order (knnssd_pack_matrix) and the
                               tuned bf16 kernels run; 0: row-major, generic kernels. embed is always row-major. */
    int32_t prefill_mode;   /* KNNSSD_PREFILL_AUTO: prompts go through the many-row prefill kernels where the shape
                               fits them; KNNSSD_PREFILL_CHUNKED: through 16-row passes of the verification kernels.
                               Only read with weights_packed = 1. */
    int32_t verify_attn;    /* which split-KV attention kernel verification passes (and the draft steps of
                               grouped-query models, and of any model once the context brings more (kv head,
                               256-position chunk) items than 512) use: KNNSSD_ATTN_MFMA (matrix cores, the default) or
                               KNNSSD_ATTN_VALU (vector ALUs). One kernel per context, never chosen per pass, so a
                               row's result does not depend on how many rows share its pass. Only read with
                               weights_packed = 1. Results stay within the stated tolerances either way. */
    int32_t attn_merge;     /* where the chunks of the split-KV attention are merged: KNNSSD_MERGE_FUSED (the default:
                               inside the attention launch, by the workgroup that finishes a group's last chunk, while
                               a kv head has at most four (row, head) pairs and the context at most 2048 positions
                               (6144 on the matrix-core kernel); in a launch of its own beyond) or
                               KNNSSD_MERGE_SEPARATE (always in a launch of its own). Same arithmetic, same bits.
                               Only read with weights_packed = 1. */
} knnssd_model_cfg;

/* Device pointers to the model. The four per-block members are HOST arrays of
 * n_blocks DEVICE pointers (the arrays are copied by knnssd_create).
 *   wqkv[b]  : [(n_heads + 2*n_kv_heads)*head_dim][d_model]  rows: all q heads, then k heads, then v heads
 *   wo[b]    : [d_model][n_heads*head_dim]
 *   wgu[b]   : [2*d_ffn][d_model]                            rows: gate rows, then up rows
 *   wdown[b] : [d_model][d_ffn]                                                            */
typedef struct knnssd_weights {
    const void *embed;          /* [vocab][d_model] */
    const void *lm_head;        /* [vocab][d_model] */
    const float *final_norm;    /* [d_model] */
    const float *const *attn_norm;
    const void *const *wqkv;
    const void *const *wo;
    const float *const *mlp_norm;
    const void *const *wgu;
    const void *const *wdown;
} knnssd_weights;

typedef struct knnssd_gen_cfg {
    int32_t max_new;       /* tokens to emit after the prompt (the prefill's own token included) */
    int32_t max_draft;     /* K: draft tokens per round, 0 = plain autoregressive decoding, <= 15 */
    float conf_threshold;  /* > 0: stop drafting after the first draft whose top-1 probability is
                              below it (that token is still verified); <= 0 disables the rule    */
    int32_t keep_mask;     /* 1: do not route this sample, draft with the mask already installed (the
                              fixed-configuration Self-SD baseline of Sec. 5.1 on a task stream); 0: route */
} knnssd_gen_cfg;

/* Counters of one knnssd_generate call. Mean generated length M = (emitted-1)/rounds and
 * acceptance rate alpha = accepted/drafted are the paper's App. C.2 metrics. Times are GPU
 * time from HIP events on the context's stream. */
typedef struct knnssd_stats {
    int64_t rounds, drafted, accepted, emitted;
    int64_t ns_prefill, ns_knn, ns_draft, ns_verify, ns_total;
    int64_t draft_passes, verify_passes;
} knnssd_stats;

typedef struct knnssd_ctx knnssd_ctx;

/* Stream order. The tuned kernels read each weight matrix once per pass, front to back, in the
 * order their wavefronts consume it; knnssd_pack_matrix rewrites a row-major bf16 matrix into
 * that order (same size, out of place, one kernel on hip_stream; src and dst are device
 * pointers, 16-byte aligned, and must not overlap). knnssd_pack_supported says whether a shape
 * can use it (bf16 weights and cache, d_model, d_ffn and n_heads*head_dim multiples of 32). */
#define KNNSSD_W_QKV 0      /* [(n_heads+2*n_kv_heads)*head_dim][d_model] */
#define KNNSSD_W_O 1        /* [d_model][n_heads*head_dim]                */
#define KNNSSD_W_GATE_UP 2  /* [2*d_ffn][d_model]                         */
#define KNNSSD_W_DOWN 3     /* [d_model][d_ffn]                           */
#define KNNSSD_W_LM_HEAD 4  /* [vocab][d_model]                           */
int32_t knnssd_pack_supported(const knnssd_model_cfg *cfg);
int32_t knnssd_pack_matrix(const knnssd_model_cfg *cfg, int32_t which, const void *src_dev, void *dst_dev,
                           void *hip_stream);

/* Bytes of device workspace / KV cache a context of this shape needs (0 if cfg is invalid). */
size_t knnssd_workspace_bytes(const knnssd_model_cfg *cfg);
size_t knnssd_kvcache_bytes(const knnssd_model_cfg *cfg);

/* Create a context over caller-owned device memory. kv_dev and ws_dev must be 256-byte
 * aligned; kv_bytes and ws_bytes are the sizes of the two buffers, and the call fails with
 * KNNSSD_EINVAL when either is smaller than the size queries above say for THIS cfg (the queries
 * depend on every field, weights_packed included). hip_stream is a hipStream_t (NULL = the null
 * stream). Launches a few set-up kernels (RoPE table, the workgroups' shares of each matrix) on the stream.
 * The library reads no environment variable: every switch is a cfg field. */
int32_t knnssd_create(const knnssd_model_cfg *cfg, const knnssd_weights *w, void *kv_dev, size_t kv_bytes,
                      void *ws_dev, size_t ws_bytes, void *hip_stream, knnssd_ctx **out);
int32_t knnssd_destroy(knnssd_ctx *ctx);

/* Anchor table for the KNN routing step (Sec. 4.1: anchors a_ij with their domain label i and
 * one stored skip set z*_i per domain). anchors_dev: [n_anchors][dim] in anchor_dtype (KNNSSD_FP32, or
 * KNNSSD_BF16: half the bytes to scan; the values the caller stored ARE the anchors, products and sums stay
 * fp32), 16-byte aligned, dim must equal d_model; labels_dev: int32 [n_anchors] in [0, n_domains); masks_host:
 * uint8 [n_domains][mask_len], copied; mask_len must be 2*n_blocks (KNNSSD_ESHAPE otherwise: the table is read
 * with that row length). n_anchors <= cfg.max_anchors. */
int32_t knnssd_set_anchors(knnssd_ctx *ctx, const void *anchors_dev, int32_t anchor_dtype, const int32_t *labels_dev,
                           int32_t n_anchors, int32_t dim, const uint8_t *masks_host, int32_t n_domains,
                           int32_t mask_len);

/* Prefill (Sec. 4.2: the routing query is the prompt's last hidden vector): the full model over
 * n prompt tokens at positions 0..n-1. Resets the KV cache length to n. Outputs: the first
 * generated token (host) and, if last_hidden_dev is not NULL, the final-RMSNorm hidden state of
 * the last prompt token (fp32 [d_model], device) - the vector the KNN step is queried with. */
int32_t knnssd_prefill(knnssd_ctx *ctx, const int32_t *tokens_host, int32_t n, float *last_hidden_dev,
                       int32_t *first_token_out);

/* Eq. 4-6: cosine-similarity arg-max of query_dev (fp32 [d_model], device) over all anchors
 * (lowest index wins a tie), domain = that anchor's label, and the domain's stored skip set
 * becomes the context's draft mask. Host outputs may be NULL. mask_out: 2*n_blocks bytes. */
int32_t knnssd_select_skipset(knnssd_ctx *ctx, const float *query_dev, int32_t *anchor_idx_out,
                              int32_t *domain_out, uint8_t *mask_out);

/* Install a draft mask directly (2*n_blocks bytes on the host; NULL = skip nothing). */
int32_t knnssd_set_skipset(knnssd_ctx *ctx, const uint8_t *mask_host);

/* K nearest anchors (cosine similarity: Eq. 4 generalised from the arg-max to the K best, lowest index first among
 * equal scores) of each of n_queries query vectors against the installed anchor table, and the majority domain
 * among the K (a tie between domains goes to the tied domain whose best anchor ranks first; K = 1 is Eq. 4-5).
 * Batched: up to 4 queries share one pass over the table. queries_dev: fp32 [n_queries][d_model], 16-byte aligned
 * (device). anchor_idx_out: int32 [n_queries][k] (host). cosine_out: fp32 [n_queries][k] (host, may be NULL).
 * domain_out: int32 [n_queries] (host). 1 <= k <= 16 and k <= number of anchors. Installs no mask.
 * KNNSSD_EDEGENERATE for a zero-norm or non-finite query or anchor, KNNSSD_ESTATE without an anchor table,
 * KNNSSD_ERANGE for k or n_queries out of range or a table of more than 2^24 anchors. */
#define KNNSSD_KNN_KMAX 16
int32_t knnssd_knn_topk(knnssd_ctx *ctx, const float *queries_dev, int32_t n_queries, int32_t k,
                        int32_t *anchor_idx_out, float *cosine_out, int32_t *domain_out);

/* The routing step for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. Same scan and arg-max kernels as
 * knnssd_select_skipset, no context: the per-anchor scores (the kernels' scratch buffer) live in a device array
 * inside the library (KNNSSD_ROUTE_MAX_ANCHORS floats = 256 KB on every GPU the library runs on, held until the
 * process ends); the call allocates and frees nothing and never waits for the GPU. Everything is enqueued on
 * hip_stream (a hipStream_t of the CURRENT device); result_dev (device, int32[4]) receives, in stream order:
 * [0] the arg-max anchor n* (lowest index on ties), [1] its label, [2] 1 if a zero-norm or non-finite query or
 * anchor was met (then [0] = [1] = -1), [3] the bits of the fp32 score (v . a) / |a|. query_dev: fp32 [dim];
 * anchors_dev: fp32 [n_anchors][dim]; labels_dev: int32 [n_anchors]; all device pointers, query and anchors 16-byte
 * aligned; dim a multiple of 4. KNNSSD_ERANGE when n_anchors is not in [1, KNNSSD_ROUTE_MAX_ANCHORS], KNNSSD_ESHAPE
 * for a bad dim, KNNSSD_EINVAL for null or misaligned pointers; nothing is enqueued on an error. All calls on one
 * GPU share that GPU's array: calls whose kernels may overlap on one GPU (different streams, no ordering between
 * them) race on it. */
#define KNNSSD_ROUTE_MAX_ANCHORS 65536
int32_t knnssd_route_static(const float *query_dev, const float *anchors_dev, const int32_t *labels_dev,
                            int32_t n_anchors, int32_t dim, void *hip_stream, int32_t *result_dev);

/* Anchor index n* and domain (Eq. 4-5) of the most recent routing on this context, whether it was made by
 * knnssd_select_skipset or inside knnssd_generate; both are -1 before the first routing. Either output
 * pointer may be NULL. Host-only, no device work. */
int32_t knnssd_last_selection(const knnssd_ctx *ctx, int32_t *anchor_idx_out, int32_t *domain_out);

/* One draft step (Eq. 7): token_in at position pos through M(z) with the installed mask; only
 * retained attention sublayers read and write the KV cache. Returns the arg-max token (lowest
 * index on ties) and its softmax probability at temperature 1. pos must be < max_seq and at most one past the
 * last position written so far (the prefill's and the accepted rows', plus the draft steps made since the last
 * verification): KNNSSD_ERANGE otherwise, since attention would read entries nobody wrote. */
int32_t knnssd_draft_step(knnssd_ctx *ctx, int32_t token_in, int32_t pos, int32_t *token_out,
                          float *top1_prob_out);

/* Verification (Sec. 4.2): the full model over n rows tokens_host = [x_last, d_1..d_k]
 * (n = k+1 <= KNNSSD_MAX_ROWS) at positions start_pos..start_pos+k in ONE pass; every block
 * overwrites its KV entries at those positions; row i attends to positions 0..start_pos+i.
 * Greedy acceptance: *n_accepted_out = j, the number of leading drafts equal to the model's own
 * token; *next_token_out = the model's token after the accepted prefix; *new_cache_len_out =
 * start_pos + j + 1 (cache entries beyond it are dead: rollback is this counter). start_pos must not exceed the
 * current cache length (KNNSSD_ERANGE): draft steps fill only the retained blocks' entries, so the full model
 * can only continue from positions that a prefill or a verification wrote. */
int32_t knnssd_verify(knnssd_ctx *ctx, const int32_t *tokens_host, int32_t n, int32_t start_pos,
                      int32_t *n_accepted_out, int32_t *next_token_out, int32_t *new_cache_len_out);

/* The whole per-sample path: prefill, KNN routing (query_dev, or the prompt's own last hidden
 * vector when query_dev is NULL; skipped when no anchor table is set or max_draft = 0, in which
 * case the installed mask is used), then draft/verify rounds until max_new tokens are out.
 * out_tokens_host must hold max_new entries; *n_out receives the count. n_prompt + max_new +
 * max_draft must not exceed max_seq. stats may be NULL. */
int32_t knnssd_generate(knnssd_ctx *ctx, const int32_t *prompt_host, int32_t n_prompt,
                        const float *query_dev, const knnssd_gen_cfg *gen, int32_t *out_tokens_host,
                        int32_t *n_out, knnssd_stats *stats);

/* Measurement aid: enqueues ONLY the launches of the weight-streaming kernel of one draft step
 * (kind 0, n = 1, the installed mask: gemv_kernel) or of one verification pass (kind 1,
 * n <= KNNSSD_MAX_ROWS rows: gemm_mfma_kernel), back to back on the context's stream between two
 * HIP events. Outputs: the number of launches, the GPU time between the events (ns, in both
 * gemm_ns and pass_ns) and the weight bytes the launches streamed, so bytes / time is the
 * kernel's achieved bandwidth and time / launches its average duration. The pass's other
 * kernels are skipped, so its numerical outputs are meaningless and the cache entries at
 * start_pos.. are overwritten: prefill again before decoding. KNNSSD_ESHAPE if the shape runs on
 * the generic kernels. */
int32_t knnssd_profile_pass(knnssd_ctx *ctx, int32_t kind, const int32_t *tokens_host, int32_t n, int32_t start_pos,
                            int64_t *n_launches, int64_t *gemm_ns, int64_t *gemm_bytes, int64_t *pass_ns);

/* Parity/debug: fp32 logits of row `row` of the most recent pass (draft: row 0). */
int32_t knnssd_get_logits(knnssd_ctx *ctx, int32_t row, float *logits_host);

/* Parity/debug: cached key and value (as fp32) of one block at one position,
 * each [n_kv_heads*head_dim] on the host. */
int32_t knnssd_read_kv(knnssd_ctx *ctx, int32_t block, int32_t pos, float *k_host, float *v_host);

/* One transition of the task stream of Sec. 4.2, Eq. 8 (host only, no device work): the next sample stays in domain
 * `current` unless u_switch < mix_ratio; on a switch it lands on one of the other n_domains - 1 domains, taken in
 * increasing order, chosen by u_pick. u_switch and u_pick are uniform draws on [0, 1) the caller supplies (the library
 * draws no random numbers). Returns the next domain, or KNNSSD_EINVAL / KNNSSD_ERANGE (negative) for n_domains < 1, a
 * current domain outside [0, n_domains), a mix ratio outside [0, 1] or a draw outside [0, 1). */
int32_t knnssd_stream_next_domain(int32_t current, int32_t n_domains, double mix_ratio, double u_switch, double u_pick);

/* Message for an error code; for KNNSSD_EHIP the text of the last HIP error of this thread. */
const char *knnssd_strerror(int32_t code);

#ifdef __cplusplus
}
#endif
#endif /* KNNSSD_H */
