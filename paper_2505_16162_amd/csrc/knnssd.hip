// Host side of the KNN-SSD C ABI: argument checks, workspace layout, and the order in which the
// kernels of a draft step, a verification pass and a generation are put on the stream.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/knnssd.h"
#include "device_types.h"
#include "kernels_generic.h"
#include "kernels_bf16.h"
#include "kernels_prefill.h"
#include "kernels_vattn.h"

using namespace ks;

static thread_local char g_hip_err[256] = "no HIP error recorded";

#define HIP_TRY(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) {                                                                    \
            snprintf(g_hip_err, sizeof(g_hip_err), "%s at %s:%d", hipGetErrorString(e_), __FILE__, __LINE__); \
            return KNNSSD_EHIP;                                                                    \
        }                                                                                          \
    } while (0)

#define KS_TRY(expr)                    \
    do {                                \
        int32_t rc_ = (expr);           \
        if (rc_ != KNNSSD_OK) return rc_; \
    } while (0)

static const size_t KS_MAX_DYN_LDS = 160 * 1024;  // dynamic LDS the tuned kernels may ask for (one workgroup per compute unit)

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Workspace layout (byte offsets, all 256-byte aligned).
struct WsLayout {
    size_t draft_ctl, ver_ctl, gen, head, knn, out3;
    size_t x, xn, qkv, att, u, logits, hidden_last, rope_cos, rope_sin, knn_scores, knn_topk, knn_cand_idx, knn_cand_val, knn_bad, out_tokens;
    // tuned bf16 path
    size_t act_d, qrot, ss, head_part, attn_part, attn_arrivals, split_tab;
    // tuned prompt prefill (stream-order weights only): all prompt rows at once
    size_t pf_tokens, pf_x, pf_q, pf_frag_d, pf_frag_att, pf_frag_u, pf_ss, pf_rstd;
    int pf_tt;          // token tiles the fragment buffers are laid out for
    size_t total;
};

static bool cfg_valid(const knnssd_model_cfg *c) {
    if (!c) return false;
    if (c->n_blocks < 0 || c->d_model <= 0 || c->n_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 ||
        c->d_ffn <= 0 || c->vocab <= 0 || c->max_seq <= 0 || c->max_anchors < 0)
        return false;
    if (c->weight_dtype != KNNSSD_FP32 && c->weight_dtype != KNNSSD_BF16) return false;
    if (c->kv_dtype != KNNSSD_FP32 && c->kv_dtype != KNNSSD_BF16) return false;
    if (!(c->rope_base > 0.f) || !(c->rms_eps >= 0.f)) return false;
    if (c->prefill_mode != KNNSSD_PREFILL_AUTO && c->prefill_mode != KNNSSD_PREFILL_CHUNKED) return false;
    if (c->verify_attn != KNNSSD_ATTN_MFMA && c->verify_attn != KNNSSD_ATTN_VALU) return false;
    if (c->attn_merge != KNNSSD_MERGE_FUSED && c->attn_merge != KNNSSD_MERGE_SEPARATE) return false;
    return true;
}

static bool cfg_supported(const knnssd_model_cfg *c) {
    if (c->head_dim != 64 && c->head_dim != 128) return false;
    if (c->n_heads % c->n_kv_heads) return false;
    if (c->d_model % 8 || c->d_ffn % 8) return false;
    if (c->max_seq > 15360) return false;  // attention scores of one row are kept in LDS (60 KB)
    return true;
}

static WsLayout ws_layout(const knnssd_model_cfg *c) {
    WsLayout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t R = KS_MAX_ROWS;
    const size_t qkv_dim = (size_t)(c->n_heads + 2 * c->n_kv_heads) * c->head_dim;
    L.draft_ctl = take(sizeof(PassCtl));
    L.ver_ctl = take(sizeof(PassCtl));
    L.gen = take(sizeof(GenState));
    L.head = take(sizeof(HeadResult));
    L.knn = take(sizeof(KnnResult));
    L.out3 = take(4 * sizeof(int32_t));
    L.x = take(R * c->d_model * 4);
    L.xn = take(R * c->d_model * 4);
    L.qkv = take(R * qkv_dim * 4);
    L.att = take(R * (size_t)c->n_heads * c->head_dim * 4);
    L.u = take(R * (size_t)c->d_ffn * 4);
    L.logits = take(R * (size_t)c->vocab * 4);
    L.hidden_last = take((size_t)c->d_model * 4);
    L.rope_cos = take((size_t)c->max_seq * (c->head_dim / 2) * 4);
    L.rope_sin = take((size_t)c->max_seq * (c->head_dim / 2) * 4);
    L.knn_scores = take((size_t)(c->max_anchors > 0 ? c->max_anchors : 1) * 4 * KNN_QMAX);
    L.knn_topk = take(sizeof(KnnTopk) * KNN_QMAX);
    L.knn_cand_idx = take((size_t)KNN_QMAX * KNN_SLICES_MAX * KNN_KMAX * 4);
    L.knn_cand_val = take((size_t)KNN_QMAX * KNN_SLICES_MAX * KNN_KMAX * 4);
    L.knn_bad = take((size_t)KNN_QMAX * KNN_SLICES_MAX * 4);
    L.out_tokens = take((size_t)c->max_seq * 4);
    {
        const size_t qd = (size_t)c->n_heads * c->head_dim;
        const size_t max_chunks = ((size_t)c->max_seq + ATT_CHUNK - 1) / ATT_CHUNK;
        L.act_d = take(R * c->d_model * 4);
        L.qrot = take(R * qd * 4);
        L.ss = take((size_t)KS_NWG * R * 4);
        L.head_part = take(R * (size_t)KS_NWG * sizeof(HeadPartial));
        L.attn_part = take(R * c->n_heads * max_chunks * (c->head_dim + ATT_PAD) * 4);
        L.attn_arrivals = take(R * (size_t)c->n_heads * 4);
        L.split_tab = take((size_t)5 * KS_NWG * sizeof(WgSplit));
        if (c->weights_packed) {
            const size_t tt = (((size_t)c->max_seq + 15) / 16 + 15) / 16 * 16, rows = tt * 16;
            L.pf_tt = (int)tt;
            L.pf_tokens = take(rows * 4);
            L.pf_x = take(rows * c->d_model * 4);
            L.pf_q = take(rows * qd * 4);
            L.pf_frag_d = take(3 * rows * (size_t)c->d_model * 2);
            L.pf_frag_att = take(3 * rows * qd * 2);
            L.pf_frag_u = take(3 * rows * (size_t)c->d_ffn * 2);
            L.pf_ss = take((size_t)KS_NWG * rows * 4);
            L.pf_rstd = take(rows * 4);
        }
    }
    L.total = off;
    return L;
}

static bool tuned_ok(const knnssd_model_cfg &g);
static bool prefill_tuned_ok(const knnssd_model_cfg &g);

struct knnssd_ctx {
    knnssd_model_cfg cfg;
    WsLayout L;
    hipStream_t stream;
    char *ws;
    char *kv;
    size_t kv_block_bytes;
    const void *embed, *lm_head;
    const float *final_norm;
    std::vector<const float *> attn_norm, mlp_norm;
    std::vector<const void *> wqkv, wo, wgu, wdown;
    // anchors
    const void *anchors;
    int32_t anchor_dtype;             // KNNSSD_FP32 | KNNSSD_BF16
    const int32_t *labels;
    int32_t n_anchors, n_domains;
    std::vector<uint8_t> masks;       // [n_domains][2*n_blocks]
    std::vector<uint8_t> draft_mask;  // installed mask
    bool prefilled;
    bool tuned;         // shape fits the tuned bf16 draft kernels
    bool tuned_verify;  // ... and the matrix-core verification kernels (every K a multiple of 32)
    bool tuned_prefill; // ... and the many-row prefill kernels (a row group fits 16 tile slots)
    bool verify_attn_mfma;  // verification passes run their split-KV attention on the matrix cores
    // tabulated workgroup splits of the five matrix shapes (tuned kernels)
    const WgSplit *split_qkv = nullptr, *split_o = nullptr, *split_gu = nullptr, *split_down = nullptr, *split_head = nullptr;
    int32_t cache_len;        // positions whose K/V every block holds (prefill + accepted rows)
    int32_t draft_len;        // positions a draft step may attend to: cache_len plus the drafts made since
    int32_t last_anchor = -1, last_domain = -1;   // most recent routing
    // pinned host staging for small read-backs
    int32_t *h_stage;
    int32_t *d_flags;   // device view of h_stage + 512: words the round-control kernels write for the host
    std::vector<hipEvent_t> events;
    // knnssd_profile_pass: enqueue only the weight-streaming launches of a pass and count them
    bool gemm_only = false;
    int64_t prof_launches = 0, prof_bytes = 0;
    bool in_prefill = false;   // the pass being enqueued belongs to a prompt prefill

    template <typename T> T *wsp(size_t off) { return reinterpret_cast<T *>(ws + off); }
};

extern "C" size_t knnssd_workspace_bytes(const knnssd_model_cfg *cfg) {
    if (!cfg_valid(cfg) || !cfg_supported(cfg)) return 0;
    return ws_layout(cfg).total;
}

extern "C" size_t knnssd_kvcache_bytes(const knnssd_model_cfg *cfg) {
    if (!cfg_valid(cfg)) return 0;
    size_t elt = cfg->kv_dtype == KNNSSD_BF16 ? 2 : 4;
    size_t per_block = align_up((size_t)2 * cfg->n_kv_heads * cfg->max_seq * cfg->head_dim * elt, 256);
    return per_block * (size_t)(cfg->n_blocks > 0 ? cfg->n_blocks : 1);
}

extern "C" const char *knnssd_strerror(int32_t code) {
    switch (code) {
        case KNNSSD_OK: return "ok";
        case KNNSSD_EINVAL: return "invalid argument";
        case KNNSSD_ESHAPE: return "shape not supported";
        case KNNSSD_ERANGE: return "position, length or token id out of range";
        case KNNSSD_EDEGENERATE: return "zero-norm or non-finite vector: cosine similarity undefined";
        case KNNSSD_ESTATE: return "call made in the wrong order";
        case KNNSSD_EHIP: return g_hip_err;
        default: return "unknown error code";
    }
}

extern "C" int32_t knnssd_create(const knnssd_model_cfg *cfg, const knnssd_weights *w, void *kv_dev, size_t kv_bytes,
                                 void *ws_dev, size_t ws_bytes, void *hip_stream, knnssd_ctx **out) {
    if (!out) return KNNSSD_EINVAL;
    *out = nullptr;
    if (!cfg_valid(cfg) || !w || !kv_dev || !ws_dev) return KNNSSD_EINVAL;
    if (!cfg_supported(cfg)) return KNNSSD_ESHAPE;
    // the kernels index these buffers by the layout of THIS cfg: a buffer sized for another one must not get through
    if (ws_bytes < ws_layout(cfg).total || kv_bytes < knnssd_kvcache_bytes(cfg)) return KNNSSD_EINVAL;
    if (cfg->weights_packed && !tuned_ok(*cfg)) return KNNSSD_ESHAPE;
    if (((uintptr_t)kv_dev & 255) || ((uintptr_t)ws_dev & 255)) return KNNSSD_EINVAL;
    if (!w->embed || !w->lm_head || !w->final_norm) return KNNSSD_EINVAL;
    const int nb = cfg->n_blocks;
    if (nb > 0 && (!w->attn_norm || !w->wqkv || !w->wo || !w->mlp_norm || !w->wgu || !w->wdown)) return KNNSSD_EINVAL;
    for (int b = 0; b < nb; ++b) {
        if (!w->attn_norm[b] || !w->wqkv[b] || !w->wo[b] || !w->mlp_norm[b] || !w->wgu[b] || !w->wdown[b])
            return KNNSSD_EINVAL;
        // 16-byte loads of weight rows
        if (((uintptr_t)w->wqkv[b] | (uintptr_t)w->wo[b] | (uintptr_t)w->wgu[b] | (uintptr_t)w->wdown[b]) & 15)
            return KNNSSD_EINVAL;
    }
    if (((uintptr_t)w->embed | (uintptr_t)w->lm_head) & 15) return KNNSSD_EINVAL;

    knnssd_ctx *c = new (std::nothrow) knnssd_ctx();
    if (!c) return KNNSSD_EINVAL;
    c->cfg = *cfg;
    c->L = ws_layout(cfg);
    c->stream = (hipStream_t)hip_stream;
    c->ws = (char *)ws_dev;
    c->kv = (char *)kv_dev;
    c->kv_block_bytes = knnssd_kvcache_bytes(cfg) / (size_t)(nb > 0 ? nb : 1);
    c->embed = w->embed; c->lm_head = w->lm_head; c->final_norm = w->final_norm;
    for (int b = 0; b < nb; ++b) {
        c->attn_norm.push_back(w->attn_norm[b]); c->mlp_norm.push_back(w->mlp_norm[b]);
        c->wqkv.push_back(w->wqkv[b]); c->wo.push_back(w->wo[b]);
        c->wgu.push_back(w->wgu[b]); c->wdown.push_back(w->wdown[b]);
    }
    c->anchors = nullptr; c->anchor_dtype = KNNSSD_FP32; c->labels = nullptr; c->n_anchors = 0; c->n_domains = 0;
    c->draft_mask.assign((size_t)2 * nb, 0);
    c->prefilled = false; c->cache_len = 0; c->draft_len = 0;
    c->tuned = cfg->weights_packed != 0;     // stream-order weights <=> tuned kernels (checked above)
    c->tuned_verify = c->tuned;
    c->tuned_prefill = c->tuned && prefill_tuned_ok(*cfg) && cfg->prefill_mode == KNNSSD_PREFILL_AUTO;
    // Attention of the verification passes: the vector-ALU kernel walks a work item's (row, head) pairs one by one,
    // the matrix-core kernel takes 16 at a time. The latter is faster from two pairs on and 10 % slower at one; the
    // choice is per context (never per pass), so a row's result does not depend on how many rows share its pass.
    c->verify_attn_mfma = cfg->verify_attn == KNNSSD_ATTN_MFMA;
    if (c->tuned) {
        hipError_t ea = hipFuncSetAttribute((const void *)gemv_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, KS_MAX_DYN_LDS);
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute((const void *)gemm_mfma_kernel<false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, KS_MAX_DYN_LDS);
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute((const void *)gemm_mfma_kernel<false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, KS_MAX_DYN_LDS);
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute((const void *)gemm_mfma_kernel<true, false>, hipFuncAttributeMaxDynamicSharedMemorySize, KS_MAX_DYN_LDS);
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute((const void *)gemm_mfma_kernel<true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, KS_MAX_DYN_LDS);
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute((const void *)attn_partial_mfma_kernel<128, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)vattn_lds_bytes<128>());
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute((const void *)attn_partial_mfma_kernel<64, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)vattn_lds_bytes<64>());
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute((const void *)attn_partial_mfma_kernel<128, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)vattn_lds_bytes<128>());
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute((const void *)attn_partial_mfma_kernel<64, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)vattn_lds_bytes<64>());
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute((const void *)prefill_gemm_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pf_gemm_lds_bytes(4));
        if (ea == hipSuccess)
            ea = hipFuncSetAttribute((const void *)prefill_gemm_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pf_gemm_lds_bytes(2));
        if (ea != hipSuccess) {
            snprintf(g_hip_err, sizeof(g_hip_err), "%s (hipFuncSetAttribute)", hipGetErrorString(ea));
            delete c;
            return KNNSSD_EHIP;
        }
    }
    if (c->tuned) {
        // the five matrix shapes' workgroup splits, computed by the same device code that packs and reads the matrices
        WgSplit *tab = c->wsp<WgSplit>(c->L.split_tab);
        const int d = cfg->d_model, H = cfg->n_heads, Hkv = cfg->n_kv_heads, hd = cfg->head_dim;
        GemmOp shape{};
        shape.H = H; shape.Hkv = Hkv; shape.hd = hd;
        auto tabulate = [&](int slot, int type, int N, int K) {
            GemmOp o = shape;
            o.type = type; o.N = N; o.K = K;
            hipLaunchKernelGGL(split_table_kernel, dim3(1), dim3(KS_NWG), 0, c->stream, o, tab + (size_t)slot * KS_NWG);
            return (const WgSplit *)(tab + (size_t)slot * KS_NWG);
        };
        c->split_qkv = tabulate(0, OP_QKV, (H + 2 * Hkv) * hd, d);
        c->split_o = tabulate(1, OP_RESID, d, H * hd);
        c->split_gu = tabulate(2, OP_SWIGLU, cfg->d_ffn, d);
        c->split_down = tabulate(3, OP_RESID, d, cfg->d_ffn);
        c->split_head = tabulate(4, OP_HEAD, cfg->vocab, d);
        // arrival counters of the attention kernel that merges its own chunks: zero between launches
        hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, c->stream, c->wsp<int>(c->L.attn_arrivals), KS_MAX_ROWS * cfg->n_heads);
        hipError_t et = hipGetLastError();
        if (et != hipSuccess) {
            snprintf(g_hip_err, sizeof(g_hip_err), "%s (split_table_kernel)", hipGetErrorString(et));
            delete c;
            return KNNSSD_EHIP;
        }
    }
    c->h_stage = nullptr;
    hipError_t e = hipHostMalloc((void **)&c->h_stage, 4096, hipHostMallocDefault);
    if (e != hipSuccess) {
        snprintf(g_hip_err, sizeof(g_hip_err), "%s (hipHostMalloc)", hipGetErrorString(e));
        delete c;
        return KNNSSD_EHIP;
    }
    c->d_flags = nullptr;
    e = hipHostGetDevicePointer((void **)&c->d_flags, c->h_stage + 512, 0);
    if (e != hipSuccess) {
        snprintf(g_hip_err, sizeof(g_hip_err), "%s (hipHostGetDevicePointer)", hipGetErrorString(e));
        (void)hipHostFree(c->h_stage);
        delete c;
        return KNNSSD_EHIP;
    }
    const int half = cfg->head_dim / 2;
    const int n = cfg->max_seq * half;
    hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, c->stream, c->wsp<float>(c->L.rope_cos),
                       c->wsp<float>(c->L.rope_sin), cfg->max_seq, half, cfg->head_dim, (double)cfg->rope_base);
    e = hipGetLastError();
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) {
        snprintf(g_hip_err, sizeof(g_hip_err), "%s (rope table)", hipGetErrorString(e));
        (void)hipHostFree(c->h_stage);
        delete c;
        return KNNSSD_EHIP;
    }
    *out = c;
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_pack_supported(const knnssd_model_cfg *cfg) {
    return (cfg_valid(cfg) && cfg_supported(cfg) && tuned_ok(*cfg)) ? 1 : 0;
}

extern "C" int32_t knnssd_pack_matrix(const knnssd_model_cfg *cfg, int32_t which, const void *src_dev, void *dst_dev,
                                      void *hip_stream) {
    if (!cfg || !src_dev || !dst_dev || src_dev == dst_dev) return KNNSSD_EINVAL;
    if (!cfg_valid(cfg)) return KNNSSD_EINVAL;
    if (!cfg_supported(cfg) || !tuned_ok(*cfg)) return KNNSSD_ESHAPE;
    if (((uintptr_t)src_dev | (uintptr_t)dst_dev) & 15) return KNNSSD_EINVAL;
    const int d = cfg->d_model, qd = cfg->n_heads * cfg->head_dim;
    GemmOp op{};
    op.H = cfg->n_heads; op.Hkv = cfg->n_kv_heads; op.hd = cfg->head_dim;
    switch (which) {
        case KNNSSD_W_QKV: op.type = OP_QKV; op.N = (cfg->n_heads + 2 * cfg->n_kv_heads) * cfg->head_dim; op.K = d; break;
        case KNNSSD_W_O: op.type = OP_RESID; op.N = d; op.K = qd; break;
        case KNNSSD_W_GATE_UP: op.type = OP_SWIGLU; op.N = cfg->d_ffn; op.K = d; break;
        case KNNSSD_W_DOWN: op.type = OP_RESID; op.N = d; op.K = cfg->d_ffn; break;
        case KNNSSD_W_LM_HEAD: op.type = OP_HEAD; op.N = cfg->vocab; op.K = d; break;
        default: return KNNSSD_EINVAL;
    }
    hipLaunchKernelGGL(pack_matrix_kernel, dim3(KS_NWG), dim3(NT), 0, (hipStream_t)hip_stream, op, (const bf16_t *)src_dev,
                       (bf16_t *)dst_dev);
    HIP_TRY(hipGetLastError());
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_destroy(knnssd_ctx *ctx) {
    if (!ctx) return KNNSSD_EINVAL;
    (void)hipStreamSynchronize(ctx->stream);
    for (hipEvent_t ev : ctx->events) (void)hipEventDestroy(ev);
    if (ctx->h_stage) (void)hipHostFree(ctx->h_stage);
    delete ctx;
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_set_anchors(knnssd_ctx *ctx, const void *anchors_dev, int32_t anchor_dtype, const int32_t *labels_dev,
                                      int32_t n_anchors, int32_t dim, const uint8_t *masks_host, int32_t n_domains,
                                      int32_t mask_len) {
    if (!ctx || !anchors_dev || !labels_dev || !masks_host) return KNNSSD_EINVAL;
    if (anchor_dtype != KNNSSD_FP32 && anchor_dtype != KNNSSD_BF16) return KNNSSD_EINVAL;
    if (n_anchors <= 0 || n_domains <= 0) return KNNSSD_EINVAL;
    if (dim != ctx->cfg.d_model) return KNNSSD_ESHAPE;
    if (mask_len != 2 * ctx->cfg.n_blocks) return KNNSSD_ESHAPE;     // one entry per sublayer
    if (n_anchors > ctx->cfg.max_anchors) return KNNSSD_ERANGE;
    if ((uintptr_t)anchors_dev & 15) return KNNSSD_EINVAL;
    const size_t ml = (size_t)mask_len;
    for (size_t i = 0; i < ml * n_domains; ++i)
        if (masks_host[i] > 1) return KNNSSD_EINVAL;
    ctx->anchors = anchors_dev; ctx->anchor_dtype = anchor_dtype; ctx->labels = labels_dev;
    ctx->n_anchors = n_anchors; ctx->n_domains = n_domains;
    ctx->masks.assign(masks_host, masks_host + ml * n_domains);
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_set_skipset(knnssd_ctx *ctx, const uint8_t *mask_host) {
    if (!ctx) return KNNSSD_EINVAL;
    const size_t ml = (size_t)2 * ctx->cfg.n_blocks;
    if (!mask_host) { ctx->draft_mask.assign(ml, 0); return KNNSSD_OK; }
    for (size_t i = 0; i < ml; ++i)
        if (mask_host[i] > 1) return KNNSSD_EINVAL;
    ctx->draft_mask.assign(mask_host, mask_host + ml);
    return KNNSSD_OK;
}

// ------------------------------------------------------------------------------------------
// one forward pass: every retained sublayer in order, then the head
// ------------------------------------------------------------------------------------------
template <typename WT, int MR>
static void launch_gemm(knnssd_ctx *c, const PassCtl *ctl, int epi, const void *W, const void *W2, const float *X, int ldx,
                        float *Y, int ldy, int N, int K, int use_head_from) {
    int wgs = (N + 3) / 4;
    if (wgs > 2048) wgs = 2048;
    const WT *w = (const WT *)W, *w2 = (const WT *)W2;
    if (epi == EPI_STORE)
        hipLaunchKernelGGL((gemm_rows_kernel<WT, MR, EPI_STORE>), dim3(wgs), dim3(256), 0, c->stream, ctl, w, w2, X, ldx, Y, ldy, N, K, use_head_from);
    else if (epi == EPI_RESID)
        hipLaunchKernelGGL((gemm_rows_kernel<WT, MR, EPI_RESID>), dim3(wgs), dim3(256), 0, c->stream, ctl, w, w2, X, ldx, Y, ldy, N, K, use_head_from);
    else
        hipLaunchKernelGGL((gemm_rows_kernel<WT, MR, EPI_SWIGLU>), dim3(wgs), dim3(256), 0, c->stream, ctl, w, w2, X, ldx, Y, ldy, N, K, use_head_from);
}

template <typename WT, typename KT, int MR>
static int32_t run_pass_t(knnssd_ctx *c, PassCtl *ctl, const uint8_t *mask) {
    const knnssd_model_cfg &g = c->cfg;
    const int d = g.d_model, H = g.n_heads, Hkv = g.n_kv_heads, hd = g.head_dim, F = g.d_ffn;
    const int qd = H * hd, qkvd = (H + 2 * Hkv) * hd;
    float *x = c->wsp<float>(c->L.x), *xn = c->wsp<float>(c->L.xn), *qkv = c->wsp<float>(c->L.qkv);
    float *att = c->wsp<float>(c->L.att), *u = c->wsp<float>(c->L.u), *logits = c->wsp<float>(c->L.logits);
    const float *cos_t = c->wsp<float>(c->L.rope_cos), *sin_t = c->wsp<float>(c->L.rope_sin);
    hipStream_t s = c->stream;
    const int rows = MR;  // grid rows; kernels drop rows >= n_rows

    hipLaunchKernelGGL((embed_kernel<WT>), dim3(rows), dim3(256), 0, s, ctl, (const WT *)c->embed, x, d);
    for (int b = 0; b < g.n_blocks; ++b) {
        KT *kvb = (KT *)(c->kv + (size_t)b * c->kv_block_bytes);
        if (!(mask && mask[2 * b])) {
            hipLaunchKernelGGL(rmsnorm_kernel, dim3(rows), dim3(256), 0, s, ctl, x, c->attn_norm[b], xn, d, g.rms_eps);
            launch_gemm<WT, MR>(c, ctl, EPI_STORE, c->wqkv[b], nullptr, xn, d, qkv, qkvd, qkvd, d, 0);
            hipLaunchKernelGGL((rope_kv_kernel<KT>), dim3(rows), dim3(256), 0, s, ctl, qkv, kvb, cos_t, sin_t, H, Hkv, hd, g.max_seq);
            hipLaunchKernelGGL((attention_kernel<KT>), dim3(H, rows), dim3(256), (size_t)g.max_seq * 4, s, ctl, qkv, kvb, att, H, Hkv, hd, g.max_seq);
            launch_gemm<WT, MR>(c, ctl, EPI_RESID, c->wo[b], nullptr, att, qd, x, d, d, qd, 0);
        }
        if (!(mask && mask[2 * b + 1])) {
            hipLaunchKernelGGL(rmsnorm_kernel, dim3(rows), dim3(256), 0, s, ctl, x, c->mlp_norm[b], xn, d, g.rms_eps);
            const WT *wg = (const WT *)c->wgu[b];
            launch_gemm<WT, MR>(c, ctl, EPI_SWIGLU, wg, wg + (size_t)F * d, xn, d, u, F, F, d, 0);
            launch_gemm<WT, MR>(c, ctl, EPI_RESID, c->wdown[b], nullptr, u, F, x, d, d, F, 0);
        }
    }
    hipLaunchKernelGGL(rmsnorm_kernel, dim3(rows), dim3(256), 0, s, ctl, x, c->final_norm, xn, d, g.rms_eps);
    launch_gemm<WT, MR>(c, ctl, EPI_STORE, c->lm_head, nullptr, xn, d, logits, g.vocab, g.vocab, d, 1);
    hipLaunchKernelGGL(argmax_kernel, dim3(rows), dim3(1024), 0, s, ctl, logits, g.vocab, c->wsp<HeadResult>(c->L.head));
    HIP_TRY(hipGetLastError());
    return KNNSSD_OK;
}

// ------------------------------------------------------------------------------------------
// tuned bf16 passes
// ------------------------------------------------------------------------------------------
static bool tuned_ok(const knnssd_model_cfg &g) {
    if (g.weight_dtype != KNNSSD_BF16 || g.kv_dtype != KNNSSD_BF16) return false;
    const int nwg = KS_NWG;
    auto per = [&](long long n) { return (int)((n + nwg - 1) / nwg); };
    if (per(g.vocab) > MAX_LROWS || 2 * per(g.d_ffn) > MAX_LROWS) return false;
    if (2 * per((long long)(g.n_heads + g.n_kv_heads) * g.head_dim / 2) + per((long long)g.n_kv_heads * g.head_dim) > MAX_LROWS) return false;
    if (per(g.d_model) > MAX_LROWS) return false;
    // the verification GEMM's staging buffers hold the shortest chunk of 16 rows for every matrix
    {
        const int mr[4] = {per(g.vocab), 2 * per(g.d_ffn), per(g.d_model),
                           2 * per((long long)(g.n_heads + g.n_kv_heads) * g.head_dim / 2) + per((long long)g.n_kv_heads * g.head_dim)};
        for (int i = 0; i < 4; ++i)
            if (mfma_bbuf_bytes(KS_MAX_DYN_LDS, mr[i]) < MFMA_MIN_BBUF) return false;
    }
    // every reduction length is a whole number of 32-column MFMA steps
    if (g.d_model % 32 || g.d_ffn % 32 || (g.n_heads * g.head_dim) % 32) return false;
    if (gemv_lds_bytes(g.d_ffn) > KS_MAX_DYN_LDS || gemv_lds_bytes(g.n_heads * g.head_dim) > KS_MAX_DYN_LDS ||
        gemv_lds_bytes(g.d_model) > KS_MAX_DYN_LDS)
        return false;
    return true;
}

// gain of the norm that reads the residual stream after sublayer index `after` (-1: after the embedding)
static const float *next_gain(const knnssd_ctx *c, const uint8_t *mask, int after) {
    for (int s = after + 1; s < 2 * c->cfg.n_blocks; ++s)
        if (!(mask && mask[s])) return (s & 1) ? c->mlp_norm[s >> 1] : c->attn_norm[s >> 1];
    return c->final_norm;
}

// One pass with the tuned bf16 kernels. rows1 = true: a draft step (one row, vector-ALU GEMV, fp32
// activations); false: verification / prefill (up to 16 rows on the matrix cores, activations as
// three bf16 planes). want_head = false skips the LM head (prefill chunks before the last).
// start: the position of the pass's first row as the host knows it (the control block will hold the same number).
static int32_t run_pass_bf16(knnssd_ctx *c, PassCtl *ctl, const uint8_t *mask, bool rows1, bool want_head, int n_rows, int start) {
    const knnssd_model_cfg &g = c->cfg;
    const int d = g.d_model, H = g.n_heads, Hkv = g.n_kv_heads, hd = g.head_dim, F = g.d_ffn;
    const int qd = H * hd, qkvd = (H + 2 * Hkv) * hd;
    float *x = c->wsp<float>(c->L.x), *act_d = c->wsp<float>(c->L.act_d), *qrot = c->wsp<float>(c->L.qrot);
    float *att = c->wsp<float>(c->L.att), *u = c->wsp<float>(c->L.u), *ss = c->wsp<float>(c->L.ss);
    hipStream_t s = c->stream;
    // most rows of one matrix a workgroup owns (fixes the verification GEMM's LDS plan), and the chunk length that
    // GEMM stages its activations in: the producer of those activations writes them as that GEMM's chunk images
    auto max_rows_of = [&](int type, int N) {
        auto per = [&](long long n) { return (int)((n + KS_NWG - 1) / KS_NWG); };
        if (type == OP_QKV) return 2 * per((long long)(H + Hkv) * hd / 2) + per((long long)Hkv * hd);
        if (type == OP_SWIGLU) return 2 * per(N);
        return per(N);
    };
    auto kc_of = [&](int type, int N, int K) {
        int kc = 0, nc = 0;
        mfma_chunking(KS_MAX_DYN_LDS, max_rows_of(type, N), n_rows, K, &kc, &nc);
        return kc;
    };
    // chunk length of the GEMM that reads the residual stream's operands after sublayer index `after`
    auto kc_next = [&](int after) {
        for (int sl = after + 1; sl < 2 * g.n_blocks; ++sl)
            if (!(mask && mask[sl])) return (sl & 1) ? kc_of(OP_SWIGLU, F, d) : kc_of(OP_QKV, qkvd, d);
        return kc_of(OP_HEAD, g.vocab, d);
    };
    auto launch = [&](const GemmOp &op) {
        if (rows1) hipLaunchKernelGGL(gemv_kernel, dim3(KS_NWG), dim3(NT), gemv_lds_bytes(op.K), s, op, ctl);
        else {
            GemmOp v = op;
            v.max_rows = max_rows_of(v.type, v.N);
            v.lds_bytes = (int)KS_MAX_DYN_LDS;
            v.n_rows = n_rows;
            mfma_chunking(KS_MAX_DYN_LDS, v.max_rows, n_rows, v.K, &v.kc, &v.nc);
            v.bbuf_bytes = mfma_bbuf_bytes(KS_MAX_DYN_LDS, v.max_rows);
            v.fixed_lds = (int)mfma_fixed_lds(KS_MAX_DYN_LDS, v.max_rows);
            v.red_bufs = mfma_red_bufs(KS_MAX_DYN_LDS, v.max_rows);
            // many activation chunks (many token rows, long K): the variant whose weight stream rolls on across the
            // chunk boundaries; few chunks: the leaner per-chunk loops, which drain the stream at a boundary. A drain
            // is cheap against a chunk of two batches or more per wavefront and dear against less (measured: the down
            // projection in three chunks is 1 % faster per-chunk at 18 units per wavefront and chunk, K = 13824 with
            // 20 rows per workgroup, and 6 % faster rolling at 9, K = 11008 with 16 rows per workgroup).
            const int tiles = (v.max_rows + 15) / 16, ksplit = NWV / (tiles >= 3 ? 4 : (tiles >= 2 ? 2 : 1));   // as make_split deals the tile lanes
            const bool ring = v.nc >= 4 || (v.nc >= 2 && (v.kc >> 5) / ksplit < 16);
            if (c->in_prefill) {
                if (ring) hipLaunchKernelGGL((gemm_mfma_kernel<true, true>), dim3(KS_NWG), dim3(NT), KS_MAX_DYN_LDS, s, v, ctl);
                else hipLaunchKernelGGL((gemm_mfma_kernel<true, false>), dim3(KS_NWG), dim3(NT), KS_MAX_DYN_LDS, s, v, ctl);
            } else {
                if (ring) hipLaunchKernelGGL((gemm_mfma_kernel<false, true>), dim3(KS_NWG), dim3(NT), KS_MAX_DYN_LDS, s, v, ctl);
                else hipLaunchKernelGGL((gemm_mfma_kernel<false, false>), dim3(KS_NWG), dim3(NT), KS_MAX_DYN_LDS, s, v, ctl);
            }
        }
        if (c->gemm_only) {    // measurement aid: count what this launch streams
            c->prof_launches += 1;
            c->prof_bytes += ((op.type == OP_SWIGLU) ? 2 * (int64_t)op.N : (int64_t)op.N) * op.K * 2;
        }
    };
    const bool others = !c->gemm_only;   // measurement aid: only the weight-streaming launches are enqueued
    GemmOp base{};
    base.n_ss = KS_NWG; base.inv_dim = 1.0f / (float)d; base.eps = g.rms_eps;
    base.H = H; base.Hkv = Hkv; base.hd = hd; base.max_seq = g.max_seq;
    base.cos_t = c->wsp<float>(c->L.rope_cos); base.sin_t = c->wsp<float>(c->L.rope_sin);

    GemmOp e = base;
    e.type = OP_EMBED; e.N = d; e.embed = (const bf16_t *)c->embed; e.x = x; e.gain_next = next_gain(c, mask, -1);
    e.act_out = act_d; e.ss_out = ss; e.n_rows = n_rows; e.out_kc = kc_next(-1);
    if (!others) {
    } else if (rows1) hipLaunchKernelGGL((embed_producer_kernel<false>), dim3(KS_NWG), dim3(NT), 0, s, e, ctl);
    else hipLaunchKernelGGL((embed_producer_kernel<true>), dim3(KS_NWG), dim3(NT), 0, s, e, ctl);

    AttnArgs aa{};
    aa.q = qrot; aa.partial = c->wsp<float>(c->L.attn_part); aa.H = H; aa.Hkv = Hkv; aa.hd = hd; aa.max_seq = g.max_seq; aa.group = H / Hkv;
    aa.max_chunks = (g.max_seq + ATT_CHUNK - 1) / ATT_CHUNK; aa.act_out = att;
    aa.n_rows = n_rows; aa.out_kc = kc_of(OP_RESID, d, qd);
    // Where the chunks of the split-KV attention are merged (the arithmetic is the same everywhere, so a value does not
    // depend on the choice). Few (row, head) pairs per kv head: the workgroup that finishes a group's last chunk merges
    // the group inside the attention launch (13B-shaped: -2.7 us per block at 2 rows, -2.4 us per draft step, against
    // the merge launch). Many pairs (Qwen-shaped 9 rows: 45 per kv head): the one workgroup's serial merge costs 5 us per
    // block MORE than the launch that spreads it over the chip, so that launch stays.
    // Draft steps of models without grouped heads bring one pair per kv head and take the vector-ALU kernel, until the
    // context is so long that its one workgroup per unit needs three rounds for the items: then the matrix-core
    // kernel's three workgroups per unit finish first (13B-shaped, context 4096: 19.8 against 23.1 us per block).
    const int n_chunks_now = (start + n_rows + ATT_CHUNK - 1) / ATT_CHUNK;
    const bool mfma_attn = (!rows1 || aa.group >= 2 || Hkv * n_chunks_now > 2 * KS_NWG) && c->verify_attn_mfma;
    // Contexts whose chunks do not fit one batch of the merge's loads keep the launch as well (every batch is a
    // dependent round trip of the one workgroup): eight chunks on the vector-ALU kernel, 24 on the matrix-core one.
    const bool self_merge = c->cfg.attn_merge == KNNSSD_MERGE_FUSED && n_rows * aa.group <= ATT_SELF_MERGE_PAIRS &&
                            start + n_rows <= (mfma_attn ? ATT_SELF_MERGE_CHUNKS_MFMA : ATT_SELF_MERGE_CHUNKS) * ATT_CHUNK;
    // More than eight chunks, or more (pair tile, kv head, chunk) items than two workgroups per compute unit take in
    // one round: the variant compiled for three per unit, whose merge fetches up to 24 chunks together
    const int va_items = (n_rows * aa.group + 15) / 16 * ((Hkv * n_chunks_now + 7) & ~7);
    const bool va_long = n_chunks_now > ATT_SELF_MERGE_CHUNKS || va_items > 2 * KS_NWG;
    const int va_grid = va_items > 2 * KS_NWG ? 3 * KS_NWG : 2 * KS_NWG;
    for (int b = 0; b < g.n_blocks; ++b) {
        bf16_t *kvb = (bf16_t *)(c->kv + (size_t)b * c->kv_block_bytes);
        if (!(mask && mask[2 * b])) {
            GemmOp o = base;
            o.type = OP_QKV; o.W = (const bf16_t *)c->wqkv[b]; o.N = qkvd; o.K = d; o.act_in = act_d;
            o.ss_in = ss; o.q_out = qrot; o.kv_block = kvb; o.split = c->split_qkv;
            launch(o);
            aa.kv_block = kvb;
            aa.arrivals = self_merge ? c->wsp<int>(c->L.attn_arrivals) : nullptr;
            if (!others) {
            } else if (mfma_attn) {
                // verification, and draft steps of grouped-query models (one row still brings H / Hkv pairs per kv
                // head): the pairs of a work item side by side on the matrix cores
                if (va_long) {
                    if (hd == 128) hipLaunchKernelGGL((attn_partial_mfma_kernel<128, true>), dim3(va_grid), dim3(VA_NT), vattn_lds_bytes<128>(), s, aa, ctl);
                    else hipLaunchKernelGGL((attn_partial_mfma_kernel<64, true>), dim3(va_grid), dim3(VA_NT), vattn_lds_bytes<64>(), s, aa, ctl);
                } else if (hd == 128) hipLaunchKernelGGL((attn_partial_mfma_kernel<128, false>), dim3(2 * KS_NWG), dim3(VA_NT), vattn_lds_bytes<128>(), s, aa, ctl);
                else hipLaunchKernelGGL((attn_partial_mfma_kernel<64, false>), dim3(2 * KS_NWG), dim3(VA_NT), vattn_lds_bytes<64>(), s, aa, ctl);
            } else if (hd == 128) hipLaunchKernelGGL((attn_partial_kernel<128>), dim3(KS_NWG), dim3(NT), attn_lds_bytes(128), s, aa, ctl);
            else hipLaunchKernelGGL((attn_partial_kernel<64>), dim3(KS_NWG), dim3(NT), attn_lds_bytes(64), s, aa, ctl);
            if (!others || self_merge) {
            } else if (rows1) hipLaunchKernelGGL((attn_combine_kernel<false>), dim3(16), dim3(NT), 0, s, aa, ctl);
            else hipLaunchKernelGGL((attn_combine_kernel<true>), dim3(64), dim3(NT), 0, s, aa, ctl);
            GemmOp r = base;
            r.type = OP_RESID; r.W = (const bf16_t *)c->wo[b]; r.N = d; r.K = qd; r.act_in = att;
            r.ss_in = nullptr; r.x = x; r.gain_next = next_gain(c, mask, 2 * b); r.act_out = act_d;
            r.ss_out = ss; r.split = c->split_o; r.out_kc = kc_next(2 * b);
            launch(r);
        }
        if (!(mask && mask[2 * b + 1])) {
            GemmOp o = base;
            o.type = OP_SWIGLU; o.W = (const bf16_t *)c->wgu[b]; o.N = F; o.K = d; o.act_in = act_d;
            o.ss_in = ss; o.act_out = u; o.split = c->split_gu; o.out_kc = kc_of(OP_RESID, d, F);
            launch(o);
            GemmOp r = base;
            r.type = OP_RESID; r.W = (const bf16_t *)c->wdown[b]; r.N = d; r.K = F; r.act_in = u;
            r.ss_in = nullptr; r.x = x; r.gain_next = next_gain(c, mask, 2 * b + 1); r.act_out = act_d;
            r.ss_out = ss; r.split = c->split_down; r.out_kc = kc_next(2 * b + 1);
            launch(r);
        }
    }
    if (want_head) {
        GemmOp h = base;
        h.type = OP_HEAD; h.W = (const bf16_t *)c->lm_head; h.N = g.vocab; h.K = d; h.act_in = act_d;
        h.ss_in = ss; h.logits = c->wsp<float>(c->L.logits); h.head_part = c->wsp<HeadPartial>(c->L.head_part);
        h.split = c->split_head;
        launch(h);
        if (others) hipLaunchKernelGGL(head_final_kernel, dim3(KS_MAX_ROWS), dim3(NT), 0, s, c->wsp<HeadPartial>(c->L.head_part), KS_NWG,
                           ctl, c->wsp<HeadResult>(c->L.head));
    }
    HIP_TRY(hipGetLastError());
    return KNNSSD_OK;
}

// mr: 1 for a draft step, KS_MAX_ROWS for verification / prefill; n_rows: the rows the control block will hold when
// the pass runs (the host always knows the count, the device fills in the contents)
static int32_t run_pass(knnssd_ctx *c, PassCtl *ctl, const uint8_t *mask, int mr, int n_rows, int start, bool want_head = true) {
    const bool wb = c->cfg.weight_dtype == KNNSSD_BF16, kb = c->cfg.kv_dtype == KNNSSD_BF16;
    if (n_rows < 1 || n_rows > mr) return KNNSSD_ERANGE;
    if (mr == 1 && c->tuned) return run_pass_bf16(c, ctl, mask, true, true, 1, start);
    if (mr != 1 && c->tuned_verify) return run_pass_bf16(c, ctl, mask, false, want_head, n_rows, start);
    if (mr == 1) {
        if (wb && kb) return run_pass_t<bf16_t, bf16_t, 1>(c, ctl, mask);
        if (wb && !kb) return run_pass_t<bf16_t, float, 1>(c, ctl, mask);
        if (!wb && kb) return run_pass_t<float, bf16_t, 1>(c, ctl, mask);
        return run_pass_t<float, float, 1>(c, ctl, mask);
    }
    if (wb && kb) return run_pass_t<bf16_t, bf16_t, KS_MAX_ROWS>(c, ctl, mask);
    if (wb && !kb) return run_pass_t<bf16_t, float, KS_MAX_ROWS>(c, ctl, mask);
    if (!wb && kb) return run_pass_t<float, bf16_t, KS_MAX_ROWS>(c, ctl, mask);
    return run_pass_t<float, float, KS_MAX_ROWS>(c, ctl, mask);
}

static int32_t set_pass(knnssd_ctx *c, PassCtl *ctl, int active, int n_rows, int start, int head_from, const int32_t *toks) {
    TokArgs ta;
    for (int i = 0; i < KS_MAX_ROWS; ++i) ta.t[i] = (i < n_rows) ? toks[i] : 0;
    hipLaunchKernelGGL(set_pass_kernel, dim3(1), dim3(64), 0, c->stream, ctl, active, n_rows, start, head_from, ta);
    HIP_TRY(hipGetLastError());
    return KNNSSD_OK;
}

// copy `bytes` from device to the pinned staging area and wait for it
static int32_t read_back(knnssd_ctx *c, const void *dev, size_t bytes) {
    HIP_TRY(hipMemcpyAsync(c->h_stage, dev, bytes, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    return KNNSSD_OK;
}

// Tile slots a row group of each matrix needs in the prefill GEMM (<= 0: the shape does not fit its 16 slots)
static int pf_slots(const knnssd_model_cfg &g, int type) {
    auto per = [&](long long n) { return (int)((n + KS_NWG - 1) / KS_NWG); };
    int rows;
    if (type == OP_QKV) rows = 2 * per((long long)(g.n_heads + g.n_kv_heads) * g.head_dim / 2) + per((long long)g.n_kv_heads * g.head_dim);
    else if (type == OP_SWIGLU) rows = 2 * per(g.d_ffn);
    else rows = per(g.d_model);
    const int t = (rows + 15) / 16;
    return t <= PF_SLOTS ? t : 0;
}

static bool prefill_tuned_ok(const knnssd_model_cfg &g) {
    return pf_slots(g, OP_QKV) > 0 && pf_slots(g, OP_SWIGLU) > 0 && pf_slots(g, OP_RESID) > 0;
}

// The full model over the first n_tok prompt rows (a multiple of 16) with the matrix-core prefill kernels: fills the
// KV cache at positions 0..n_tok-1. The last rows of the prompt go through an ordinary 16-row pass afterwards,
// which also produces the first token and the routing query.
static int32_t prefill_tuned(knnssd_ctx *c, const int32_t *tokens_host, int n_tok) {
    const knnssd_model_cfg &g = c->cfg;
    const int d = g.d_model, H = g.n_heads, Hkv = g.n_kv_heads, hd = g.head_dim, F = g.d_ffn;
    const int qd = H * hd, qkvd = (H + 2 * Hkv) * hd, TT = c->L.pf_tt, TTL = n_tok / 16;
    hipStream_t s = c->stream;
    int32_t *toks = c->wsp<int32_t>(c->L.pf_tokens);
    float *x = c->wsp<float>(c->L.pf_x), *q = c->wsp<float>(c->L.pf_q), *ss = c->wsp<float>(c->L.pf_ss);
    float *rstd = c->wsp<float>(c->L.pf_rstd);
    bf16_t *frag_d = c->wsp<bf16_t>(c->L.pf_frag_d), *frag_att = c->wsp<bf16_t>(c->L.pf_frag_att);
    bf16_t *frag_u = c->wsp<bf16_t>(c->L.pf_frag_u);
    HIP_TRY(hipMemcpyAsync(toks, tokens_host, (size_t)n_tok * 4, hipMemcpyHostToDevice, s));
    hipLaunchKernelGGL(prefill_embed_kernel, dim3(n_tok), dim3(PF_NT), 0, s, toks, (const bf16_t *)c->embed,
                       next_gain(c, nullptr, -1), d, g.rms_eps, TT, x, frag_d, rstd);

    GemmOp base{};
    base.H = H; base.Hkv = Hkv; base.hd = hd; base.max_seq = g.max_seq;
    base.cos_t = c->wsp<float>(c->L.rope_cos); base.sin_t = c->wsp<float>(c->L.rope_sin);
    auto gemm = [&](const GemmOp &op, const bf16_t *fin, bf16_t *fout, const float *rs, float *ss_out, int *n_shares) {
        PfArgs a{};
        a.op = op; a.frag_in = fin; a.frag_out = fout; a.rstd = rs; a.ss_out = ss_out; a.TT = TT; a.n_tok = n_tok;
        a.T = pf_slots(g, op.type); a.G = PF_SLOTS / a.T;
        const int gx = (KS_NWG + a.G - 1) / a.G;
        // enough workgroups to fill the chip with 16 token tiles each? otherwise 8 per workgroup
        const bool wide = (long long)gx * ((TTL + 15) / 16) >= 200;
        if (n_shares) *n_shares = gx;
        if (wide) hipLaunchKernelGGL(prefill_gemm_kernel<4>, dim3(gx, (TTL + 15) / 16), dim3(PF_NT), pf_gemm_lds_bytes(4), s, a);
        else hipLaunchKernelGGL(prefill_gemm_kernel<2>, dim3(gx, (TTL + 7) / 8), dim3(PF_NT), pf_gemm_lds_bytes(2), s, a);
    };
    auto norm = [&](int n_shares) {
        hipLaunchKernelGGL(prefill_rstd_kernel, dim3((n_tok + 255) / 256), dim3(256), 0, s, ss, n_shares, TT * 16, n_tok,
                           1.0f / (float)d, g.rms_eps, rstd);
    };
    for (int b = 0; b < g.n_blocks; ++b) {
        bf16_t *kvb = (bf16_t *)(c->kv + (size_t)b * c->kv_block_bytes);
        int shares = 0;
        GemmOp o = base;
        o.type = OP_QKV; o.W = (const bf16_t *)c->wqkv[b]; o.N = qkvd; o.K = d; o.q_out = q; o.kv_block = kvb;
        gemm(o, frag_d, nullptr, rstd, nullptr, nullptr);
        PfAttn at{};
        at.q = q; at.kv_block = kvb; at.frag_out = frag_att; at.H = H; at.Hkv = Hkv; at.max_seq = g.max_seq; at.TT = TT; at.n_tok = n_tok;
        if (hd == 128) hipLaunchKernelGGL(prefill_attn_kernel<128>, dim3(((TTL + 3) / 4) * H), dim3(256), 0, s, at);
        else hipLaunchKernelGGL(prefill_attn_kernel<64>, dim3(((TTL + 3) / 4) * H), dim3(256), 0, s, at);
        GemmOp r = base;
        r.type = OP_RESID; r.W = (const bf16_t *)c->wo[b]; r.N = d; r.K = qd; r.x = x; r.gain_next = next_gain(c, nullptr, 2 * b);
        gemm(r, frag_att, frag_d, nullptr, ss, &shares);
        norm(shares);
        GemmOp u = base;
        u.type = OP_SWIGLU; u.W = (const bf16_t *)c->wgu[b]; u.N = F; u.K = d;
        gemm(u, frag_d, frag_u, rstd, nullptr, nullptr);
        GemmOp dn = base;
        dn.type = OP_RESID; dn.W = (const bf16_t *)c->wdown[b]; dn.N = d; dn.K = F; dn.x = x; dn.gain_next = next_gain(c, nullptr, 2 * b + 1);
        gemm(dn, frag_u, frag_d, nullptr, ss, &shares);
        norm(shares);
    }
    HIP_TRY(hipGetLastError());
    return KNNSSD_OK;
}

static int32_t prefill_impl(knnssd_ctx *c, const int32_t *tokens, int32_t n, float *last_hidden_dev, int32_t *first_token) {
    PassCtl *ver = c->wsp<PassCtl>(c->L.ver_ctl);
    int s0 = 0;
    if (c->tuned_prefill) {
        // every complete 16-row tile before the prompt's last rows goes through the matrix-core prefill
        const int n_main = (n - 1) / KS_MAX_ROWS * KS_MAX_ROWS;
        if (n_main >= 2 * KS_MAX_ROWS) {
            KS_TRY(prefill_tuned(c, tokens, n_main));
            s0 = n_main;
        }
    }
    for (int s = s0; s < n; s += KS_MAX_ROWS) {
        int rows = n - s < KS_MAX_ROWS ? n - s : KS_MAX_ROWS;
        bool last = s + rows >= n;
        KS_TRY(set_pass(c, ver, 1, rows, s, last ? rows - 1 : rows, tokens + s));
        c->in_prefill = true;
        int32_t rc_pass = run_pass(c, ver, nullptr, KS_MAX_ROWS, rows, s, last);
        c->in_prefill = false;
        KS_TRY(rc_pass);
        if (last) {
            if (c->tuned_verify) {
                // the last pass left the final norm's operands as the LM head's chunk images
                int head_kc = 0, head_nc = 0;
                mfma_chunking(KS_MAX_DYN_LDS, (c->cfg.vocab + KS_NWG - 1) / KS_NWG, rows, c->cfg.d_model, &head_kc, &head_nc);
                hipLaunchKernelGGL(hidden_from_image_kernel, dim3(8), dim3(NT), 0, c->stream, c->wsp<float>(c->L.act_d),
                                   head_kc, rows, c->wsp<float>(c->L.ss), KS_NWG, c->cfg.d_model, c->cfg.rms_eps, ver,
                                   c->wsp<float>(c->L.hidden_last), last_hidden_dev);
                HIP_TRY(hipGetLastError());
            } else {
                const float *xn_last = c->wsp<float>(c->L.xn) + (size_t)(rows - 1) * c->cfg.d_model;
                HIP_TRY(hipMemcpyAsync(c->wsp<float>(c->L.hidden_last), xn_last, (size_t)c->cfg.d_model * 4,
                                       hipMemcpyDeviceToDevice, c->stream));
                if (last_hidden_dev)
                    HIP_TRY(hipMemcpyAsync(last_hidden_dev, xn_last, (size_t)c->cfg.d_model * 4, hipMemcpyDeviceToDevice, c->stream));
            }
            KS_TRY(read_back(c, &c->wsp<HeadResult>(c->L.head)->tok[rows - 1], 4));
            *first_token = c->h_stage[0];
        }
    }
    c->prefilled = true;
    c->cache_len = n;
    c->draft_len = n;
    return KNNSSD_OK;
}

static int32_t check_tokens(const knnssd_ctx *c, const int32_t *t, int32_t n) {
    for (int i = 0; i < n; ++i)
        if (t[i] < 0 || t[i] >= c->cfg.vocab) return KNNSSD_ERANGE;
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_prefill(knnssd_ctx *ctx, const int32_t *tokens_host, int32_t n, float *last_hidden_dev,
                                  int32_t *first_token_out) {
    if (!ctx || !tokens_host || !first_token_out) return KNNSSD_EINVAL;
    if (n <= 0 || n > ctx->cfg.max_seq) return KNNSSD_ERANGE;
    KS_TRY(check_tokens(ctx, tokens_host, n));
    return prefill_impl(ctx, tokens_host, n, last_hidden_dev, first_token_out);
}

// the scan of the anchor table for nq <= KNN_QMAX queries at once, in the table's storage type
static void launch_scan(knnssd_ctx *c, const float *queries, int nq, float *scores) {
    const int N = c->n_anchors, D = c->cfg.d_model;
    int wgs = (N + 3) / 4;
    if (wgs > 4096) wgs = 4096;
    const dim3 g(wgs), b(256);
    if (c->anchor_dtype == KNNSSD_BF16) {
        const bf16_t *a = (const bf16_t *)c->anchors;
        if (nq == 1) hipLaunchKernelGGL((knn_scores_multi_kernel<1, bf16_t>), g, b, 0, c->stream, queries, a, N, D, scores);
        else if (nq == 2) hipLaunchKernelGGL((knn_scores_multi_kernel<2, bf16_t>), g, b, 0, c->stream, queries, a, N, D, scores);
        else if (nq == 3) hipLaunchKernelGGL((knn_scores_multi_kernel<3, bf16_t>), g, b, 0, c->stream, queries, a, N, D, scores);
        else hipLaunchKernelGGL((knn_scores_multi_kernel<4, bf16_t>), g, b, 0, c->stream, queries, a, N, D, scores);
    } else {
        const float *a = (const float *)c->anchors;
        if (nq == 1) hipLaunchKernelGGL((knn_scores_multi_kernel<1, float>), g, b, 0, c->stream, queries, a, N, D, scores);
        else if (nq == 2) hipLaunchKernelGGL((knn_scores_multi_kernel<2, float>), g, b, 0, c->stream, queries, a, N, D, scores);
        else if (nq == 3) hipLaunchKernelGGL((knn_scores_multi_kernel<3, float>), g, b, 0, c->stream, queries, a, N, D, scores);
        else hipLaunchKernelGGL((knn_scores_multi_kernel<4, float>), g, b, 0, c->stream, queries, a, N, D, scores);
    }
}

static int32_t select_impl(knnssd_ctx *c, const float *query_dev, int32_t *idx_out, int32_t *dom_out) {
    const int N = c->n_anchors, D = c->cfg.d_model;
    float *scores = c->wsp<float>(c->L.knn_scores);
    KnnResult *res = c->wsp<KnnResult>(c->L.knn);
    launch_scan(c, query_dev, 1, scores);
    hipLaunchKernelGGL(knn_argmax_kernel, dim3(1), dim3(1024), 0, c->stream, scores, query_dev, c->labels, N, D, res);
    HIP_TRY(hipGetLastError());
    KS_TRY(read_back(c, res, sizeof(KnnResult)));
    KnnResult r;
    memcpy(&r, c->h_stage, sizeof(r));
    if (r.degenerate) return KNNSSD_EDEGENERATE;
    if (r.label < 0 || r.label >= c->n_domains) return KNNSSD_ERANGE;
    const size_t ml = (size_t)2 * c->cfg.n_blocks;
    c->draft_mask.assign(c->masks.begin() + ml * r.label, c->masks.begin() + ml * (r.label + 1));
    *idx_out = r.idx;
    *dom_out = r.label;
    c->last_anchor = r.idx; c->last_domain = r.label;
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_knn_topk(knnssd_ctx *ctx, const float *queries_dev, int32_t n_queries, int32_t k,
                                   int32_t *anchor_idx_out, float *cosine_out, int32_t *domain_out) {
    if (!ctx || !queries_dev || !anchor_idx_out || !domain_out) return KNNSSD_EINVAL;
    if (!ctx->anchors) return KNNSSD_ESTATE;
    if ((uintptr_t)queries_dev & 15) return KNNSSD_EINVAL;
    if (n_queries <= 0 || k < 1 || k > KNN_KMAX || k > ctx->n_anchors) return KNNSSD_ERANGE;
    const int N = ctx->n_anchors, D = ctx->cfg.d_model;
    float *scores = ctx->wsp<float>(ctx->L.knn_scores);
    KnnTopk *res = ctx->wsp<KnnTopk>(ctx->L.knn_topk);
    for (int q0 = 0; q0 < n_queries; q0 += KNN_QMAX) {
        const int nq = n_queries - q0 < KNN_QMAX ? n_queries - q0 : KNN_QMAX;
        const float *qp = queries_dev + (size_t)q0 * D;
        launch_scan(ctx, qp, nq, scores);
        int n_slices = N / 2048;                      // stage 1 slices per query: a few thousand scores each
        if (n_slices < 1) n_slices = 1;
        if (n_slices > KNN_SLICES_MAX) n_slices = KNN_SLICES_MAX;
        // a slice is ranked by one workgroup, whose lanes keep one mask bit per entry they look at
        if ((N + n_slices - 1) / n_slices > KNN_ROUNDS_MAX_N) n_slices = (N + KNN_ROUNDS_MAX_N - 1) / KNN_ROUNDS_MAX_N;
        if (n_slices > KNN_SLICES_MAX) return KNNSSD_ERANGE;       // more than 16.7 million anchors
        int32_t *cand_idx = ctx->wsp<int32_t>(ctx->L.knn_cand_idx);
        float *cand_val = ctx->wsp<float>(ctx->L.knn_cand_val);
        int *bad = ctx->wsp<int>(ctx->L.knn_bad);
        hipLaunchKernelGGL(knn_topk_part_kernel, dim3(nq, n_slices), dim3(1024), 0, ctx->stream, scores, N, k, n_slices, cand_idx, cand_val, bad);
        hipLaunchKernelGGL(knn_topk_kernel, dim3(nq), dim3(1024), 0, ctx->stream, cand_idx, cand_val, n_slices, bad, qp, ctx->labels, D, k, res);
        HIP_TRY(hipGetLastError());
        KS_TRY(read_back(ctx, res, sizeof(KnnTopk) * nq));
        const KnnTopk *h = reinterpret_cast<const KnnTopk *>(ctx->h_stage);
        for (int q = 0; q < nq; ++q) {
            if (h[q].degenerate) return KNNSSD_EDEGENERATE;
            if (h[q].domain < 0 || h[q].domain >= ctx->n_domains) return KNNSSD_ERANGE;
            for (int r = 0; r < k; ++r) {
                anchor_idx_out[(size_t)(q0 + q) * k + r] = h[q].idx[r];
                if (cosine_out) cosine_out[(size_t)(q0 + q) * k + r] = h[q].cosine[r];
            }
            domain_out[q0 + q] = h[q].domain;
        }
    }
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_last_selection(const knnssd_ctx *ctx, int32_t *anchor_idx_out, int32_t *domain_out) {
    if (!ctx) return KNNSSD_EINVAL;
    if (anchor_idx_out) *anchor_idx_out = ctx->last_anchor;
    if (domain_out) *domain_out = ctx->last_domain;
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_select_skipset(knnssd_ctx *ctx, const float *query_dev, int32_t *anchor_idx_out,
                                         int32_t *domain_out, uint8_t *mask_out) {
    if (!ctx || !query_dev) return KNNSSD_EINVAL;
    if (!ctx->anchors) return KNNSSD_ESTATE;
    if ((uintptr_t)query_dev & 15) return KNNSSD_EINVAL;
    int32_t idx = -1, dom = -1;
    KS_TRY(select_impl(ctx, query_dev, &idx, &dom));
    if (anchor_idx_out) *anchor_idx_out = idx;
    if (domain_out) *domain_out = dom;
    if (mask_out) memcpy(mask_out, ctx->draft_mask.data(), ctx->draft_mask.size());
    return KNNSSD_OK;
}

// ------------------------------------------------------------------------------------------
// Routing for callers that cannot allocate. The scan's per-anchor scores (the one scratch buffer of the routing
// kernels) live in a file-scope device array instead of the caller's workspace. `route_scratch` below is only the
// host-side stand-in of that array: the device address comes from hipGetSymbolAddress, once per device, and host
// code uses that address (never the array's name) wherever it needs the memory.
// ------------------------------------------------------------------------------------------
static __device__ __align__(256) float route_scratch[KNNSSD_ROUTE_MAX_ANCHORS];

static const int ROUTE_MAX_DEVICES = 64;
static float *g_route_scratch_dev[ROUTE_MAX_DEVICES];      // per device: its own copy of the array, at its own address

// Address of the current device's copy of the scratch array (looked up on the first call made with that device
// current; allocates nothing).
static int32_t route_scratch_ptr(float **out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= ROUTE_MAX_DEVICES) return KNNSSD_ERANGE;
    if (!g_route_scratch_dev[dev]) {
        float *p = nullptr;
        HIP_TRY(hipGetSymbolAddress((void **)&p, HIP_SYMBOL(route_scratch)));
        if (!p) return KNNSSD_EHIP;
        g_route_scratch_dev[dev] = p;
    }
    *out = g_route_scratch_dev[dev];
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_route_static(const float *query_dev, const float *anchors_dev, const int32_t *labels_dev,
                                       int32_t n_anchors, int32_t dim, void *hip_stream, int32_t *result_dev) {
    if (!query_dev || !anchors_dev || !labels_dev || !result_dev) return KNNSSD_EINVAL;
    if (((uintptr_t)query_dev | (uintptr_t)anchors_dev) & 15) return KNNSSD_EINVAL;
    if ((uintptr_t)result_dev & 3) return KNNSSD_EINVAL;
    if (dim < 4 || (dim & 3)) return KNNSSD_ESHAPE;                 // the scan reads anchors in 16-byte pieces
    if (n_anchors <= 0 || n_anchors > KNNSSD_ROUTE_MAX_ANCHORS) return KNNSSD_ERANGE;
    float *scores = nullptr;
    KS_TRY(route_scratch_ptr(&scores));
    hipStream_t s = (hipStream_t)hip_stream;
    int wgs = (n_anchors + 3) / 4;
    if (wgs > 4096) wgs = 4096;
    // every score the arg-max reads is written by the scan of the same call, so nothing has to start at zero
    hipLaunchKernelGGL((knn_scores_multi_kernel<1, float>), dim3(wgs), dim3(256), 0, s, query_dev, anchors_dev, n_anchors, dim, scores);
    hipLaunchKernelGGL(knn_argmax_kernel, dim3(1), dim3(1024), 0, s, (const float *)scores, query_dev, labels_dev, n_anchors, dim,
                       reinterpret_cast<KnnResult *>(result_dev));
    HIP_TRY(hipGetLastError());
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_draft_step(knnssd_ctx *ctx, int32_t token_in, int32_t pos, int32_t *token_out,
                                     float *top1_prob_out) {
    if (!ctx || !token_out) return KNNSSD_EINVAL;
    if (!ctx->prefilled) return KNNSSD_ESTATE;
    if (pos < 0 || pos >= ctx->cfg.max_seq) return KNNSSD_ERANGE;
    if (pos > ctx->draft_len) return KNNSSD_ERANGE;       // positions in between were never written
    if (token_in < 0 || token_in >= ctx->cfg.vocab) return KNNSSD_ERANGE;
    PassCtl *dr = ctx->wsp<PassCtl>(ctx->L.draft_ctl);
    KS_TRY(set_pass(ctx, dr, 1, 1, pos, 0, &token_in));
    KS_TRY(run_pass(ctx, dr, ctx->draft_mask.data(), 1, 1, pos));
    KS_TRY(read_back(ctx, ctx->wsp<HeadResult>(ctx->L.head), sizeof(HeadResult)));
    HeadResult hr;
    memcpy(&hr, ctx->h_stage, sizeof(hr));
    *token_out = hr.tok[0];
    if (top1_prob_out) *top1_prob_out = hr.prob[0];
    ctx->draft_len = pos + 1;
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_verify(knnssd_ctx *ctx, const int32_t *tokens_host, int32_t n, int32_t start_pos,
                                 int32_t *n_accepted_out, int32_t *next_token_out, int32_t *new_cache_len_out) {
    if (!ctx || !tokens_host || !n_accepted_out || !next_token_out) return KNNSSD_EINVAL;
    if (!ctx->prefilled) return KNNSSD_ESTATE;
    if (n <= 0 || n > KS_MAX_ROWS) return KNNSSD_ERANGE;
    if (start_pos < 0 || start_pos + n > ctx->cfg.max_seq) return KNNSSD_ERANGE;
    if (start_pos > ctx->cache_len) return KNNSSD_ERANGE;  // the full model's K/V in between were never written (drafts fill only retained blocks)
    KS_TRY(check_tokens(ctx, tokens_host, n));
    PassCtl *ver = ctx->wsp<PassCtl>(ctx->L.ver_ctl);
    KS_TRY(set_pass(ctx, ver, 1, n, start_pos, 0, tokens_host));
    KS_TRY(run_pass(ctx, ver, nullptr, KS_MAX_ROWS, n, start_pos));
    int32_t *out3 = ctx->wsp<int32_t>(ctx->L.out3);
    hipLaunchKernelGGL(verify_accept_kernel, dim3(1), dim3(1), 0, ctx->stream, ver, ctx->wsp<HeadResult>(ctx->L.head), out3);
    HIP_TRY(hipGetLastError());
    KS_TRY(read_back(ctx, out3, 12));
    *n_accepted_out = ctx->h_stage[0];
    *next_token_out = ctx->h_stage[1];
    if (new_cache_len_out) *new_cache_len_out = ctx->h_stage[2];
    ctx->cache_len = ctx->h_stage[2];
    ctx->draft_len = ctx->cache_len;
    return KNNSSD_OK;
}

static int32_t get_event(knnssd_ctx *c, size_t i, hipEvent_t *ev) {
    while (c->events.size() <= i) {
        hipEvent_t e;
        HIP_TRY(hipEventCreate(&e));
        c->events.push_back(e);
    }
    *ev = c->events[i];
    return KNNSSD_OK;
}

static int32_t mark(knnssd_ctx *c, size_t i) {
    hipEvent_t ev;
    KS_TRY(get_event(c, i, &ev));
    HIP_TRY(hipEventRecord(ev, c->stream));
    return KNNSSD_OK;
}

static int64_t elapsed_ns(knnssd_ctx *c, size_t a, size_t b) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->events[a], c->events[b]) != hipSuccess) return 0;
    return (int64_t)((double)ms * 1e6);
}

extern "C" int32_t knnssd_generate(knnssd_ctx *ctx, const int32_t *prompt_host, int32_t n_prompt, const float *query_dev,
                                   const knnssd_gen_cfg *gen, int32_t *out_tokens_host, int32_t *n_out, knnssd_stats *stats) {
    if (!ctx || !prompt_host || !gen || !out_tokens_host || !n_out) return KNNSSD_EINVAL;
    if (n_prompt <= 0 || gen->max_new <= 0) return KNNSSD_ERANGE;
    if (gen->max_draft < 0 || gen->max_draft > KS_MAX_ROWS - 1) return KNNSSD_ERANGE;
    if ((int64_t)n_prompt + gen->max_new + gen->max_draft > ctx->cfg.max_seq) return KNNSSD_ERANGE;
    if (query_dev && ((uintptr_t)query_dev & 15)) return KNNSSD_EINVAL;
    KS_TRY(check_tokens(ctx, prompt_host, n_prompt));

    size_t ev = 0;
    KS_TRY(mark(ctx, ev++));  // 0
    int32_t first = 0;
    KS_TRY(prefill_impl(ctx, prompt_host, n_prompt, nullptr, &first));
    KS_TRY(mark(ctx, ev++));  // 1
    if (ctx->anchors && gen->max_draft > 0 && !gen->keep_mask) {
        int32_t idx, dom;
        KS_TRY(select_impl(ctx, query_dev ? query_dev : ctx->wsp<float>(ctx->L.hidden_last), &idx, &dom));
    }
    KS_TRY(mark(ctx, ev++));  // 2

    GenState *st = ctx->wsp<GenState>(ctx->L.gen);
    PassCtl *dr = ctx->wsp<PassCtl>(ctx->L.draft_ctl), *ver = ctx->wsp<PassCtl>(ctx->L.ver_ctl);
    HeadResult *head = ctx->wsp<HeadResult>(ctx->L.head);
    int32_t *out_dev = ctx->wsp<int32_t>(ctx->L.out_tokens);
    hipStream_t s = ctx->stream;
    hipLaunchKernelGGL(gen_init_kernel, dim3(1), dim3(1), 0, s, st, n_prompt, first, gen->max_new, gen->max_draft,
                       gen->conf_threshold, out_dev);
    int64_t n_draft_passes = 0, n_verify_passes = 0;
    std::vector<size_t> round_ev;  // triples of event indices
    bool done = gen->max_new <= 1;
    int32_t emitted_host = 1;     // the host mirrors the round control far enough to know each pass's row count
    // Where the draft count of a round is decided on the device (confidence stop), the host would have to wait after
    // every draft step before it can enqueue the next pass, and the GPU idles meanwhile. Instead it predicts that the
    // round stops where the last one did and enqueues the verification pass for that count right behind the draft
    // step; the pass runs only if the prediction came true (verify_begin_kernel), otherwise its kernels return at
    // once and the host carries on step by step. Without a threshold the count is known and nothing is waited for.
    int pred_k = 1;
    volatile int32_t *flags = (volatile int32_t *)ctx->h_stage + 512;   // [0] draft goes on, [1] emitted, [2] drafts made
    while (!done) {
        hipLaunchKernelGGL(round_begin_kernel, dim3(1), dim3(1), 0, s, st, dr);
        size_t ea = ev++, eb = ev++, ec = ev++;
        KS_TRY(mark(ctx, ea));
        int kmax = gen->max_new - emitted_host - 1;
        if (kmax > gen->max_draft) kmax = gen->max_draft;
        int k_host = 0;
        const int cache_len_host = n_prompt + emitted_host - 1;     // every emitted token but the last is in the cache
        bool verified = false;        // the round's verification pass has been enqueued for the right draft count
        bool stepwise = false;        // a prediction failed in this round: wait after every step from here on
        auto enqueue_verify = [&](int k, int expect_k) -> int32_t {
            hipLaunchKernelGGL(verify_begin_kernel, dim3(1), dim3(1), 0, s, st, dr, ver, expect_k);
            KS_TRY(run_pass(ctx, ver, nullptr, KS_MAX_ROWS, k + 1, cache_len_host));
            hipLaunchKernelGGL(accept_kernel, dim3(1), dim3(1), 0, s, st, ver, head, out_dev, ctx->d_flags + 1);
            KS_TRY(mark(ctx, ec));
            return KNNSSD_OK;
        };
        for (int i = 0; i < kmax; ++i) {
            KS_TRY(run_pass(ctx, dr, ctx->draft_mask.data(), 1, 1, cache_len_host + i));
            hipLaunchKernelGGL(draft_end_kernel, dim3(1), dim3(1), 0, s, st, dr, head, ctx->d_flags);
            ++n_draft_passes; ++k_host;
            const bool last = k_host == kmax;                  // the round ends here whatever the confidence is
            if (!(gen->conf_threshold > 0.f)) continue;        // no stop rule: kmax drafts, nothing to wait for
            if (stepwise && last) break;                       // every earlier step was seen to go on: the count is known
            if (!stepwise && k_host < pred_k && !last) continue;   // predicted to go on; a pass enqueued in vain returns at once
            const int expected = k_host;
            if (!stepwise) {                                   // predicted (or bound) to stop here: verification goes out ahead
                KS_TRY(mark(ctx, eb));
                KS_TRY(enqueue_verify(expected, expected));
            }
            HIP_TRY(hipStreamSynchronize(s));
            if (!flags[0]) {                                   // the draft has stopped, after flags[2] steps
                const int made = flags[2];
                n_draft_passes -= k_host - made;               // steps enqueued beyond the stop did not run
                k_host = made;
                verified = !stepwise && made == expected;
                break;
            }
            stepwise = true;                                   // it goes on: the pass enqueued ahead did not run
        }
        pred_k = k_host > 0 ? k_host : 1;
        if (!verified) {
            KS_TRY(mark(ctx, eb));
            KS_TRY(enqueue_verify(k_host, -1));
        }
        ++n_verify_passes;
        round_ev.push_back(ea); round_ev.push_back(eb); round_ev.push_back(ec);
        HIP_TRY(hipStreamSynchronize(s));
        emitted_host = flags[1];
        done = emitted_host >= gen->max_new;
    }
    size_t e_end = ev++;
    KS_TRY(mark(ctx, e_end));
    KS_TRY(read_back(ctx, st, sizeof(GenState)));
    GenState hs;
    memcpy(&hs, ctx->h_stage, sizeof(hs));
    const int32_t emitted = hs.emitted < gen->max_new ? hs.emitted : gen->max_new;
    HIP_TRY(hipMemcpyAsync(out_tokens_host, out_dev, (size_t)emitted * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    *n_out = emitted;
    ctx->cache_len = hs.cache_len;
    ctx->draft_len = hs.cache_len;
    if (stats) {
        memset(stats, 0, sizeof(*stats));
        stats->rounds = hs.rounds; stats->drafted = hs.drafted; stats->accepted = hs.accepted; stats->emitted = emitted;
        stats->ns_prefill = elapsed_ns(ctx, 0, 1);
        stats->ns_knn = elapsed_ns(ctx, 1, 2);
        for (size_t i = 0; i + 3 <= round_ev.size(); i += 3) {
            stats->ns_draft += elapsed_ns(ctx, round_ev[i], round_ev[i + 1]);
            stats->ns_verify += elapsed_ns(ctx, round_ev[i + 1], round_ev[i + 2]);
        }
        stats->ns_total = elapsed_ns(ctx, 0, e_end);
        stats->draft_passes = n_draft_passes; stats->verify_passes = n_verify_passes;
    }
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_profile_pass(knnssd_ctx *ctx, int32_t kind, const int32_t *tokens_host, int32_t n, int32_t start_pos,
                                       int64_t *n_launches, int64_t *gemm_ns, int64_t *gemm_bytes, int64_t *pass_ns) {
    if (!ctx || !tokens_host || !n_launches || !gemm_ns || !gemm_bytes || !pass_ns) return KNNSSD_EINVAL;
    if (!ctx->prefilled) return KNNSSD_ESTATE;
    if (kind != 0 && kind != 1) return KNNSSD_EINVAL;
    if (n <= 0 || n > (kind == 0 ? 1 : KS_MAX_ROWS)) return KNNSSD_ERANGE;
    if (start_pos < 0 || start_pos + n > ctx->cfg.max_seq) return KNNSSD_ERANGE;
    KS_TRY(check_tokens(ctx, tokens_host, n));
    if (!(kind == 0 ? ctx->tuned : ctx->tuned_verify)) return KNNSSD_ESHAPE;   // only the tuned kernels are instrumented
    PassCtl *ctl = ctx->wsp<PassCtl>(kind == 0 ? ctx->L.draft_ctl : ctx->L.ver_ctl);
    KS_TRY(set_pass(ctx, ctl, 1, n, start_pos, 0, tokens_host));
    hipEvent_t p0, p1;
    HIP_TRY(hipEventCreate(&p0));
    {
        const hipError_t e1 = hipEventCreate(&p1);
        if (e1 != hipSuccess) { (void)hipEventDestroy(p0); HIP_TRY(e1); }
    }
    ctx->prof_launches = 0; ctx->prof_bytes = 0;
    ctx->gemm_only = true;
    (void)hipEventRecord(p0, ctx->stream);
    int32_t rc = run_pass(ctx, ctl, kind == 0 ? ctx->draft_mask.data() : nullptr, kind == 0 ? 1 : KS_MAX_ROWS, n, start_pos);
    (void)hipEventRecord(p1, ctx->stream);
    ctx->gemm_only = false;
    hipError_t es = hipStreamSynchronize(ctx->stream);
    float pms = 0.f;
    (void)hipEventElapsedTime(&pms, p0, p1);
    (void)hipEventDestroy(p0);
    (void)hipEventDestroy(p1);
    *n_launches = ctx->prof_launches; *gemm_bytes = ctx->prof_bytes;
    *gemm_ns = (int64_t)((double)pms * 1e6); *pass_ns = *gemm_ns;
    if (rc != KNNSSD_OK) return rc;
    HIP_TRY(es);
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_stream_next_domain(int32_t current, int32_t n_domains, double mix_ratio, double u_switch, double u_pick) {
    if (n_domains < 1) return KNNSSD_EINVAL;
    if (current < 0 || current >= n_domains) return KNNSSD_ERANGE;
    if (!(mix_ratio >= 0.0 && mix_ratio <= 1.0) || !(u_switch >= 0.0 && u_switch < 1.0) || !(u_pick >= 0.0 && u_pick < 1.0))
        return KNNSSD_ERANGE;
    if (n_domains == 1 || !(u_switch < mix_ratio)) return current;
    int32_t slot = (int32_t)(u_pick * (double)(n_domains - 1));       // one of the other N-1 domains, equally likely
    if (slot > n_domains - 2) slot = n_domains - 2;
    return slot < current ? slot : slot + 1;
}

extern "C" int32_t knnssd_get_logits(knnssd_ctx *ctx, int32_t row, float *logits_host) {
    if (!ctx || !logits_host) return KNNSSD_EINVAL;
    if (row < 0 || row >= KS_MAX_ROWS) return KNNSSD_ERANGE;
    const float *src = ctx->wsp<float>(ctx->L.logits) + (size_t)row * ctx->cfg.vocab;
    HIP_TRY(hipMemcpyAsync(logits_host, src, (size_t)ctx->cfg.vocab * 4, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(hipStreamSynchronize(ctx->stream));
    return KNNSSD_OK;
}

extern "C" int32_t knnssd_read_kv(knnssd_ctx *ctx, int32_t block, int32_t pos, float *k_host, float *v_host) {
    if (!ctx || !k_host || !v_host) return KNNSSD_EINVAL;
    const knnssd_model_cfg &g = ctx->cfg;
    if (block < 0 || block >= g.n_blocks || pos < 0 || pos >= g.max_seq) return KNNSSD_ERANGE;
    const size_t elt = g.kv_dtype == KNNSSD_BF16 ? 2 : 4;
    std::vector<char> tmp((size_t)g.head_dim * elt);
    HIP_TRY(hipStreamSynchronize(ctx->stream));
    for (int kv = 0; kv < 2; ++kv) {
        float *dst = kv ? v_host : k_host;
        for (int h = 0; h < g.n_kv_heads; ++h) {
            const char *src = ctx->kv + (size_t)block * ctx->kv_block_bytes +
                              ((((size_t)kv * g.n_kv_heads + h) * g.max_seq + pos) * g.head_dim) * elt;
            HIP_TRY(hipMemcpy(tmp.data(), src, tmp.size(), hipMemcpyDeviceToHost));
            for (int i = 0; i < g.head_dim; ++i) {
                if (elt == 4) {
                    memcpy(&dst[h * g.head_dim + i], tmp.data() + 4 * i, 4);
                } else {
                    uint16_t b;
                    memcpy(&b, tmp.data() + 2 * i, 2);
                    uint32_t u = (uint32_t)b << 16;
                    memcpy(&dst[h * g.head_dim + i], &u, 4);
                }
            }
        }
    }
    return KNNSSD_OK;
}
