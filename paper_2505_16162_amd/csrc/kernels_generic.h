// Generic (any shape, fp32 or bf16 storage) kernels of the decode path, written for gfx950:
// 64-wide wavefronts, 16-byte coalesced weight loads, wavefront reductions.
// These are the kernels of the fp32 path and the building blocks the tuned bf16 kernels
// fall back to when a shape does not fit their tiling.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_types.h"

namespace ks {

typedef uint16_t bf16_t;  // raw bit pattern

__device__ __forceinline__ float bf16_to_float(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round to nearest even (inf/nan pass through with the payload truncated)
__device__ __forceinline__ bf16_t float_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) return (bf16_t)(u >> 16);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float load_as_float(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_as_float(const bf16_t *p, size_t i) { return bf16_to_float(p[i]); }
__device__ __forceinline__ void store_rounded(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_rounded(bf16_t *p, size_t i, float v) { p[i] = float_to_bf16_rne(v); }

// One 16-byte chunk of a weight row as floats.
template <typename WT> struct WChunk;
template <> struct WChunk<float> {
    static constexpr int N = 4;
    float v[4];
    __device__ __forceinline__ void load(const float *p) {
        float4 t = *reinterpret_cast<const float4 *>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
};
template <> struct WChunk<bf16_t> {
    static constexpr int N = 8;
    float v[8];
    __device__ __forceinline__ void load(const bf16_t *p) {
        uint4 t = *reinterpret_cast<const uint4 *>(p);
        v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
        v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
        v[4] = __uint_as_float(t.z << 16); v[5] = __uint_as_float(t.z & 0xffff0000u);
        v[6] = __uint_as_float(t.w << 16); v[7] = __uint_as_float(t.w & 0xffff0000u);
    }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// ------------------------------------------------------------------------------------------
// pass control
// ------------------------------------------------------------------------------------------
struct TokArgs { int32_t t[KS_MAX_ROWS]; };

__global__ void set_pass_kernel(PassCtl *ctl, int active, int n_rows, int start, int head_from, TokArgs toks) {
    if (threadIdx.x == 0) {
        ctl->active = active; ctl->n_rows = n_rows; ctl->start = start; ctl->head_from = head_from;
    }
    if (threadIdx.x < KS_MAX_ROWS) ctl->tok[threadIdx.x] = toks.t[threadIdx.x];
}

// ------------------------------------------------------------------------------------------
// RoPE table: cos/sin of pos * base^(-2i/head_dim), evaluated in double, stored fp32
// ------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(float *cos_t, float *sin_t, int max_seq, int half, int head_dim, double base) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= max_seq * half) return;
    int pos = idx / half, i = idx % half;
    double ang = (double)pos * pow(base, -2.0 * (double)i / (double)head_dim);
    cos_t[idx] = (float)cos(ang);
    sin_t[idx] = (float)sin(ang);
}

// ------------------------------------------------------------------------------------------
// embedding gather: x[r][:] = E[tok[r]][:]
// ------------------------------------------------------------------------------------------
template <typename WT>
__global__ void embed_kernel(const PassCtl *ctl, const WT *E, float *x, int d) {
    if (!ctl->active) return;
    int r = blockIdx.x;
    if (r >= ctl->n_rows) return;
    const WT *row = E + (size_t)ctl->tok[r] * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) x[(size_t)r * d + i] = load_as_float(row, i);
}

// ------------------------------------------------------------------------------------------
// RMSNorm: out[r][:] = x[r][:] * rsqrt(mean(x^2) + eps) * gain       (one workgroup per row)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rmsnorm_kernel(const PassCtl *ctl, const float *x, const float *gain,
                                                      float *out, int d, float eps) {
    if (!ctl->active) return;
    int r = blockIdx.x;
    if (r >= ctl->n_rows) return;
    __shared__ float part[4];
    const float *xr = x + (size_t)r * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) { float v = xr[i]; ss = fmaf(v, v, ss); }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = (part[0] + part[1]) + (part[2] + part[3]);
    float rs = 1.0f / sqrtf(tot / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += 256) out[(size_t)r * d + i] = xr[i] * rs * gain[i];
}

// ------------------------------------------------------------------------------------------
// Y = X W^T for up to MR rows of X, one output feature per wavefront (lanes stride over K in
// 16-byte chunks of the weight row), with the epilogues the decoder needs.
// ------------------------------------------------------------------------------------------
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };

template <typename WT, int MR, int EPI>
__global__ __launch_bounds__(256) void gemm_rows_kernel(const PassCtl *ctl, const WT *__restrict__ W,
                                                        const WT *__restrict__ W2, const float *__restrict__ X,
                                                        int ldx, float *Y, int ldy, int N, int K, int use_head_from) {
    if (!ctl->active) return;
    const int n_rows = min(ctl->n_rows, MR);
    const int row_lo = use_head_from ? ctl->head_from : 0;
    if (row_lo >= n_rows) return;
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    constexpr int VEC = WChunk<WT>::N;

    for (int o = wave; o < N; o += n_waves) {
        float acc[MR], acc2[MR];
#pragma unroll
        for (int r = 0; r < MR; ++r) { acc[r] = 0.f; acc2[r] = 0.f; }
        const WT *wrow = W + (size_t)o * K;
        const WT *wrow2 = (EPI == EPI_SWIGLU) ? (W2 + (size_t)o * K) : nullptr;
        for (int k = lane * VEC; k < K; k += 64 * VEC) {
            WChunk<WT> w, w2;
            w.load(wrow + k);
            if (EPI == EPI_SWIGLU) w2.load(wrow2 + k);
#pragma unroll
            for (int r = 0; r < MR; ++r) {
                if (r >= row_lo && r < n_rows) {
                    const float *xp = X + (size_t)r * ldx + k;
#pragma unroll
                    for (int j = 0; j < VEC; j += 4) {
                        float4 xv = *reinterpret_cast<const float4 *>(xp + j);
                        acc[r] = fmaf(w.v[j + 0], xv.x, acc[r]);
                        acc[r] = fmaf(w.v[j + 1], xv.y, acc[r]);
                        acc[r] = fmaf(w.v[j + 2], xv.z, acc[r]);
                        acc[r] = fmaf(w.v[j + 3], xv.w, acc[r]);
                        if (EPI == EPI_SWIGLU) {
                            acc2[r] = fmaf(w2.v[j + 0], xv.x, acc2[r]);
                            acc2[r] = fmaf(w2.v[j + 1], xv.y, acc2[r]);
                            acc2[r] = fmaf(w2.v[j + 2], xv.z, acc2[r]);
                            acc2[r] = fmaf(w2.v[j + 3], xv.w, acc2[r]);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < MR; ++r) {
            if (r >= row_lo && r < n_rows) {
                float a = wave_sum(acc[r]);
                float b = (EPI == EPI_SWIGLU) ? wave_sum(acc2[r]) : 0.f;
                if (lane == 0) {
                    float *yp = Y + (size_t)r * ldy + o;
                    if (EPI == EPI_STORE) *yp = a;
                    if (EPI == EPI_RESID) *yp = *yp + a;
                    if (EPI == EPI_SWIGLU) *yp = (a / (1.0f + expf(-a))) * b;
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// RoPE on q (in place) and k, then k and v into the cache (rounded to the cache type).
// qkv: [rows][(H + 2 Hkv) * hd] fp32.  cache layout: [2 (k,v)][Hkv][max_seq][hd]
// ------------------------------------------------------------------------------------------
template <typename KT>
__global__ __launch_bounds__(256) void rope_kv_kernel(const PassCtl *ctl, float *qkv, KT *kv_block,
                                                      const float *cos_t, const float *sin_t, int H, int Hkv,
                                                      int hd, int max_seq) {
    if (!ctl->active) return;
    const int r = blockIdx.x;
    if (r >= ctl->n_rows) return;
    const int pos = ctl->start + r;
    const int half = hd >> 1;
    const int ld = (H + 2 * Hkv) * hd;
    float *row = qkv + (size_t)r * ld;
    const float *cs = cos_t + (size_t)pos * half, *sn = sin_t + (size_t)pos * half;
    KT *kc = kv_block;
    KT *vc = kv_block + (size_t)Hkv * max_seq * hd;
    for (int idx = threadIdx.x; idx < (H + Hkv) * half; idx += blockDim.x) {
        int h = idx / half, i = idx % half;
        float c = cs[i], s = sn[i];
        float a = row[h * hd + i], b = row[h * hd + i + half];
        float ra = a * c - b * s, rb = b * c + a * s;
        if (h < H) {
            row[h * hd + i] = ra; row[h * hd + i + half] = rb;
        } else {
            size_t base = ((size_t)(h - H) * max_seq + pos) * hd;
            store_rounded(kc, base + i, ra);
            store_rounded(kc, base + i + half, rb);
        }
    }
    const float *vrow = row + (size_t)(H + Hkv) * hd;
    for (int idx = threadIdx.x; idx < Hkv * hd; idx += blockDim.x) {
        int h = idx / hd, i = idx % hd;
        store_rounded(vc, ((size_t)h * max_seq + pos) * hd + i, vrow[idx]);
    }
}

// ------------------------------------------------------------------------------------------
// Attention of one (row, head): softmax(q K^T / sqrt(hd)) V over positions 0..start+r.
// One workgroup per (head, row); scores are kept in LDS (max_seq floats of dynamic LDS).
// ------------------------------------------------------------------------------------------
template <typename KT>
__global__ __launch_bounds__(256) void attention_kernel(const PassCtl *ctl, const float *qkv, const KT *kv_block,
                                                        float *att, int H, int Hkv, int hd, int max_seq) {
    if (!ctl->active) return;
    const int h = blockIdx.x, r = blockIdx.y;
    if (r >= ctl->n_rows) return;
    extern __shared__ float score_lds[];
    float *scores = score_lds;           // [len]
    __shared__ float red[8];
    __shared__ float outp[4][128];
    const int len = ctl->start + r + 1;
    const int kvh = h / (H / Hkv);
    const int ld = (H + 2 * Hkv) * hd;
    const float *q = qkv + (size_t)r * ld + h * hd;
    const KT *kc = kv_block + (size_t)kvh * max_seq * hd;
    const KT *vc = kv_block + ((size_t)Hkv + kvh) * max_seq * hd;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float scale = 1.0f / sqrtf((float)hd);

    float q0 = (lane < hd) ? q[lane] : 0.f;
    float q1 = (lane + 64 < hd) ? q[lane + 64] : 0.f;
    float lmax = -INFINITY;
    for (int t = wave; t < len; t += 4) {
        const KT *kt = kc + (size_t)t * hd;
        float p = 0.f;
        if (lane < hd) p = q0 * load_as_float(kt, lane);
        if (lane + 64 < hd) p = fmaf(q1, load_as_float(kt, lane + 64), p);
        p = wave_sum(p) * scale;
        if (lane == 0) scores[t] = p;
        lmax = fmaxf(lmax, p);
    }
    if (lane == 0) red[wave] = lmax;
    __syncthreads();
    const float mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float lsum = 0.f;
    for (int t = threadIdx.x; t < len; t += 256) {
        float e = expf(scores[t] - mx);
        scores[t] = e;
        lsum += e;
    }
    lsum = wave_sum(lsum);
    if (lane == 0) red[4 + wave] = lsum;
    __syncthreads();
    const float den = (red[4] + red[5]) + (red[6] + red[7]);
    // output: thread (part, i) sums its share of positions for dimension i
    const int nparts = 256 / hd;   // hd 64 -> 4 parts, hd 128 -> 2 parts
    const int i = threadIdx.x % hd, part = threadIdx.x / hd;
    float acc = 0.f;
    if (part < nparts)
        for (int t = part; t < len; t += nparts) acc = fmaf(scores[t], load_as_float(vc, (size_t)t * hd + i), acc);
    if (part < 4) outp[part][i] = acc;
    __syncthreads();
    if ((int)threadIdx.x < hd) {
        float s = 0.f;
        for (int p = 0; p < nparts; ++p) s += outp[p][threadIdx.x];
        att[(size_t)r * (H * hd) + h * hd + threadIdx.x] = s / den;
    }
}

// ------------------------------------------------------------------------------------------
// arg-max (lowest index on ties) and top-1 softmax probability of each logits row
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

__global__ __launch_bounds__(1024) void argmax_kernel(const PassCtl *ctl, const float *logits, int V, HeadResult *res) {
    if (!ctl->active) return;
    const int r = blockIdx.x;
    if (r >= ctl->n_rows || r < ctl->head_from) return;
    __shared__ float sv[16];
    __shared__ int si[16];
    __shared__ float ssum[16];
    const float *row = logits + (size_t)r * V;
    float bv = -INFINITY; int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < V; i += 1024) { float v = row[i]; if (better(v, i, bv, bi)) { bv = v; bi = i; } }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        float ov = __shfl_xor(bv, off, 64); int oi = __shfl_xor(bi, off, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    bv = sv[0]; bi = si[0];
    for (int w = 1; w < 16; ++w) if (better(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
    float s = 0.f;
    for (int i = threadIdx.x; i < V; i += 1024) s += expf(row[i] - bv);
    s = wave_sum(s);
    if (lane == 0) ssum[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float tot = 0.f;
        for (int w = 0; w < 16; ++w) tot += ssum[w];
        res->tok[r] = bi;
        res->prob[r] = 1.0f / tot;
    }
}

// ------------------------------------------------------------------------------------------
// KNN routing, Eq. 4: score_n = (v . a_n) / |a_n|  (|v| is a common positive factor), then arg-max
// ------------------------------------------------------------------------------------------
template <int Q, typename AT>
__global__ __launch_bounds__(256) void knn_scores_multi_kernel(const float *__restrict__ queries, const AT *__restrict__ anchors,
                                                               int N, int D, float *scores);

__global__ __launch_bounds__(1024) void knn_argmax_kernel(const float *scores, const float *query, const int32_t *labels,
                                                          int N, int D, KnnResult *res) {
    __shared__ float sv[16];
    __shared__ int si[16];
    __shared__ int bad;
    __shared__ float qn[16];
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    float bv = -INFINITY; int bi = 0x7fffffff; int mybad = 0;
    for (int i = threadIdx.x; i < N; i += 1024) {
        float v = scores[i];
        if (!isfinite(v)) mybad = 1;
        else if (better(v, i, bv, bi)) { bv = v; bi = i; }
    }
    float q2 = 0.f;
    for (int i = threadIdx.x; i < D; i += 1024) { float v = query[i]; q2 = fmaf(v, v, q2); }
    q2 = wave_sum(q2);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        float ov = __shfl_xor(bv, off, 64); int oi = __shfl_xor(bi, off, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (mybad) atomicOr(&bad, 1);
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; qn[wave] = q2; }
    __syncthreads();
    if (threadIdx.x == 0) {
        bv = sv[0]; bi = si[0];
        float qtot = qn[0];
        for (int w = 1; w < 16; ++w) { if (better(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; } qtot += qn[w]; }
        int degenerate = bad || !(qtot > 0.f) || !isfinite(qtot) || bi == 0x7fffffff;
        res->degenerate = degenerate;
        res->idx = degenerate ? -1 : bi;
        res->label = degenerate ? -1 : labels[bi];
        res->score = bv;
    }
}

// ------------------------------------------------------------------------------------------
// K nearest anchors for a few queries at once (Eq. 4 generalised from the arg-max to the K best), then the
// majority domain among them. One pass over the anchor table serves up to KNN_QMAX queries: a wavefront
// streams one anchor (16-byte nontemporal loads, all of a block in flight before the first is used) and
// forms its dot product with every query (the queries are small and stay in cache) and its own norm.
// ------------------------------------------------------------------------------------------
#define KNN_QMAX 4
#define KNN_KMAX 16

__global__ void fill_zero_kernel(int *p, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

struct KnnTopk {
    int32_t idx[KNN_KMAX];
    float cosine[KNN_KMAX];
    int32_t domain;       // majority label among the K; ties go to the tied label whose best anchor ranks first
    int32_t degenerate;   // 1: zero-norm / non-finite query or anchor met
};

// AT = float or bf16_t: the type the anchor table is stored in (queries, products and sums are fp32 either way). A lane's
// 16-byte load covers EPL = 4 or 8 consecutive elements of an anchor. A wavefront takes A consecutive anchors at a
// time and L loads per lane of each, so 8 loads per lane are in flight whatever the storage type and query count, a
// query value fetched from the cache serves A anchors (with four queries the query reads would otherwise be four
// times the table's bytes), and 5120 elements are whole blocks in every variant. An anchor's sums are formed in the
// same order whatever A is: a lane adds its elements in column order, then the 64 lanes are summed.
template <int Q, typename AT>
struct KnnTile {
    static constexpr int EPL = 16 / (int)sizeof(AT);
    static constexpr int A = (Q >= 3 || EPL == 8) ? 4 : 2;
    static constexpr int L = 8 / A;
};

template <int Q, typename AT>
__global__ __launch_bounds__(256) void knn_scores_multi_kernel(const float *__restrict__ queries, const AT *__restrict__ anchors,
                                                               int N, int D, float *scores /*[Q][N]*/) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    constexpr int EPL = KnnTile<Q, AT>::EPL;          // elements per lane and load
    constexpr int A = KnnTile<Q, AT>::A, L = KnnTile<Q, AT>::L;
    constexpr int BLK = L * 64 * EPL;                 // elements of an anchor per block of L loads per lane
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int n_waves = (gridDim.x * blockDim.x) >> 6;
    for (int n0 = wave * A; n0 < N; n0 += n_waves * A) {
        const AT *a[A];
#pragma unroll
        for (int t = 0; t < A; ++t) a[t] = anchors + (size_t)min(n0 + t, N - 1) * D;      // past the table: the last anchor again, not stored
        float dot[A][Q], nn[A];
#pragma unroll
        for (int t = 0; t < A; ++t) {
            nn[t] = 0.f;
#pragma unroll
            for (int q = 0; q < Q; ++q) dot[t][q] = 0.f;
        }
        for (int k0 = 0; k0 < D; k0 += BLK) {            // blocks of A x L 16-byte loads per lane, issued together
            f4 av[A][L];
#pragma unroll
            for (int j = 0; j < L; ++j) {
                const int k = min(k0 + (j * 64 + lane) * EPL, D - EPL);           // clamped, masked below
#pragma unroll
                for (int t = 0; t < A; ++t) av[t][j] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(a[t] + k));
            }
#pragma unroll
            for (int j = 0; j < L; ++j) {
                const int k = k0 + (j * 64 + lane) * EPL;
                if (k < D) {
                    float4 qv[Q][EPL / 4];
#pragma unroll
                    for (int q = 0; q < Q; ++q)
#pragma unroll
                        for (int i4 = 0; i4 < EPL / 4; ++i4)
                            qv[q][i4] = *reinterpret_cast<const float4 *>(queries + (size_t)q * D + k + 4 * i4);
#pragma unroll
                    for (int t = 0; t < A; ++t) {
                        float e[EPL];
                        if constexpr (EPL == 4) {
                            e[0] = av[t][j].x; e[1] = av[t][j].y; e[2] = av[t][j].z; e[3] = av[t][j].w;
                        } else {
#pragma unroll
                            for (int w = 0; w < 4; ++w) {
                                const unsigned int u = __float_as_uint(av[t][j][w]);
                                e[2 * w] = __uint_as_float(u << 16); e[2 * w + 1] = __uint_as_float(u & 0xffff0000u);
                            }
                        }
#pragma unroll
                        for (int i = 0; i < EPL; ++i) nn[t] = fmaf(e[i], e[i], nn[t]);
#pragma unroll
                        for (int q = 0; q < Q; ++q) {
#pragma unroll
                            for (int i4 = 0; i4 < EPL / 4; ++i4) {
                                dot[t][q] = fmaf(e[4 * i4], qv[q][i4].x, dot[t][q]); dot[t][q] = fmaf(e[4 * i4 + 1], qv[q][i4].y, dot[t][q]);
                                dot[t][q] = fmaf(e[4 * i4 + 2], qv[q][i4].z, dot[t][q]); dot[t][q] = fmaf(e[4 * i4 + 3], qv[q][i4].w, dot[t][q]);
                            }
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < A; ++t) {
            const float nt = wave_sum(nn[t]);
            const bool ok = nt > 0.f && isfinite(nt);
            const float inv = ok ? 1.0f / sqrtf(nt) : 0.f;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const float d = wave_sum(dot[t][q]);
                if (lane == 0 && n0 + t < N) scores[(size_t)q * N + n0 + t] = ok ? d * inv : NAN;
            }
        }
    }
}

// The K best (largest value, lowest anchor index on ties) of n entries, in rank order, by one workgroup of 1024
// threads. Entry i has value val[i] and anchor index (map ? map[i] : first + i); entries with a negative index are
// dead. Two levels of K rounds of arg-max, both inside single wavefronts (registers and cross-lane moves, no
// meeting per round): every wavefront ranks the K best of its sixteenth of the entries (a lane looks at entries 64
// apart and marks the ones it has given away in a 64-bit mask, hence n <= KNN_ROUNDS_MAX_N), the workgroup meets once,
// and the first wavefront ranks the K best of the 16 x K survivors. taken_idx / taken_val receive the winners
// (0x7fffffff / -inf once the entries run out); returns nonzero in the threads that met a non-finite value.
#define KNN_ROUNDS_MAX_N (16 * 64 * 64)
#define KNN_SLICES_MAX 256       // stage-1 slices per query: 256 x KNN_ROUNDS_MAX_N anchors at most
struct KnnRoundsLds {
    float val[16][KNN_KMAX];
    int idx[16][KNN_KMAX];
};

__device__ __forceinline__ void knn_wave_best(float &bv, int &bi, int &bp) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(bv, off, 64); const int oi = __shfl_xor(bi, off, 64), op = __shfl_xor(bp, off, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; bp = op; }
    }
}

__device__ __forceinline__ int knn_rounds(const float *val, const int32_t *map, int first, int n, int K, int *taken_idx,
                                          float *taken_val, KnnRoundsLds *wl) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int anybad = 0;
    {
        const int w0 = (int)((long long)n * wave / 16), w1 = (int)((long long)n * (wave + 1) / 16);
        const int M = (w1 - w0 + 63) >> 6;                 // <= 64
        unsigned long long given = 0;                       // bit m: this lane's entry w0 + 64 m + lane is among the winners
        // the lane's first MR entries stay in registers over the rounds (slices of a few thousand scores and the
        // candidate lists have no more); entries beyond are read again in every round
        constexpr int MR = 4;
        float rv[MR]; int rg[MR];
#pragma unroll
        for (int m = 0; m < MR; ++m) {
            const int i = w0 + (m << 6) + lane;
            rv[m] = -INFINITY; rg[m] = -1;                  // a dead entry
            if (i < w1) {
                const float v = val[i];
                if (!isfinite(v)) anybad = 1;
                else { rv[m] = v; rg[m] = map ? map[i] : first + i; }
            }
        }
        for (int r = 0; r < K; ++r) {
            float bv = -INFINITY; int bi = 0x7fffffff, bp = -1;
#pragma unroll
            for (int m = 0; m < MR; ++m)
                if (!((given >> m) & 1ull) && rg[m] >= 0 && better(rv[m], rg[m], bv, bi)) { bv = rv[m]; bi = rg[m]; bp = w0 + (m << 6) + lane; }
            for (int m = MR; m < M; ++m) {
                const int i = w0 + (m << 6) + lane;
                if (i >= w1 || ((given >> m) & 1ull)) continue;
                const float v = val[i];
                if (!isfinite(v)) { anybad = 1; continue; }
                const int gi = map ? map[i] : first + i;
                if (gi >= 0 && better(v, gi, bv, bi)) { bv = v; bi = gi; bp = i; }
            }
            knn_wave_best(bv, bi, bp);                      // every lane holds the winner
            if (bp >= 0 && ((bp - w0) & 63) == lane) given |= 1ull << ((bp - w0) >> 6);
            if (lane == 0) { wl->val[wave][r] = bv; wl->idx[wave][r] = bi; }
        }
    }
    __syncthreads();
    if (wave == 0) {
        // 16 x KNN_KMAX slots, four per lane; slots of rounds that were not played are dead
        float cv[4]; int ci[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int c = (m << 6) + lane, w = c / KNN_KMAX, r = c % KNN_KMAX;
            const bool live = r < K;
            cv[m] = live ? wl->val[w][r] : -INFINITY;
            ci[m] = live ? wl->idx[w][r] : 0x7fffffff;
        }
        unsigned int given = 0;
        for (int r = 0; r < K; ++r) {
            float bv = -INFINITY; int bi = 0x7fffffff, bp = -1;
#pragma unroll
            for (int m = 0; m < 4; ++m)
                if (!((given >> m) & 1u) && ci[m] != 0x7fffffff && better(cv[m], ci[m], bv, bi)) { bv = cv[m]; bi = ci[m]; bp = (m << 6) + lane; }
            knn_wave_best(bv, bi, bp);
            if (bp >= 0 && (bp & 63) == lane) given |= 1u << (bp >> 6);
            if (lane == 0) { taken_idx[r] = bi; taken_val[r] = bv; }
        }
    }
    __syncthreads();
    return anybad;
}

// Stage 1 of the top-K: workgroup (query q, slice b) leaves the K best of its slice of the scores as candidates.
__global__ __launch_bounds__(1024) void knn_topk_part_kernel(const float *scores /*[Q][N]*/, int N, int K, int n_slices,
                                                             int32_t *cand_idx /*[Q][n_slices][KNN_KMAX]*/, float *cand_val,
                                                             int *bad_flag /*[Q][n_slices]*/) {
    __shared__ KnnRoundsLds wl;
    __shared__ int tidx[KNN_KMAX];
    __shared__ float tval[KNN_KMAX];
    const int q = blockIdx.x, b = blockIdx.y;
    const int i0 = (int)((long long)N * b / n_slices), i1 = (int)((long long)N * (b + 1) / n_slices);
    const int kk = min(K, i1 - i0);
    const int anybad = knn_rounds(scores + (size_t)q * N + i0, nullptr, i0, i1 - i0, kk, tidx, tval, &wl);
    const int slice_bad = __syncthreads_or(anybad);           // every slice writes its own flag: nothing to clear beforehand
    if (threadIdx.x == 0) bad_flag[q * n_slices + b] = slice_bad ? 1 : 0;
    if (threadIdx.x < KNN_KMAX) {
        const size_t o = ((size_t)q * n_slices + b) * KNN_KMAX + threadIdx.x;
        const bool live = (int)threadIdx.x < kk && tidx[threadIdx.x] != 0x7fffffff;
        cand_idx[o] = live ? tidx[threadIdx.x] : -1;
        cand_val[o] = live ? tval[threadIdx.x] : -INFINITY;
    }
}

// Stage 2: one workgroup per query merges the slices' candidates (K rounds again), then the vote.
__global__ __launch_bounds__(1024) void knn_topk_kernel(const int32_t *cand_idx, const float *cand_val, int n_slices, const int *bad_flag,
                                                        const float *queries, const int32_t *labels, int D, int K, KnnTopk *res) {
    __shared__ KnnRoundsLds wl;
    __shared__ int taken[KNN_KMAX];
    __shared__ float tval[KNN_KMAX];
    __shared__ float qn[16];
    const int q = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float *qv = queries + (size_t)q * D;
    float q2 = 0.f;
    for (int i = threadIdx.x; i < D; i += 1024) { const float v = qv[i]; q2 = fmaf(v, v, q2); }
    q2 = wave_sum(q2);
    if (lane == 0) qn[wave] = q2;
    __syncthreads();
    const size_t o = (size_t)q * n_slices * KNN_KMAX;
    knn_rounds(cand_val + o, cand_idx + o, 0, n_slices * KNN_KMAX, K, taken, tval, &wl);
    int mybad = 0;
    for (int b = threadIdx.x; b < n_slices; b += 1024) mybad |= bad_flag[q * n_slices + b];
    const int bad = __syncthreads_or(mybad);
    // the winners' labels, fetched side by side (the vote below walks them many times)
    __shared__ int lab_of[KNN_KMAX];
    if (threadIdx.x < KNN_KMAX) {
        const int t = taken[threadIdx.x];
        lab_of[threadIdx.x] = ((int)threadIdx.x < K && t != 0x7fffffff && t >= 0) ? labels[t] : -1;
    }
    __syncthreads();
    // (no per-thread arrays below: they would live in scratch memory, one memory round trip per access)
    float qtot = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) qtot += qn[w];
    const bool degenerate = bad || !(qtot > 0.f) || !isfinite(qtot) || taken[0] == 0x7fffffff;
    const float invq = degenerate ? 0.f : 1.0f / sqrtf(qtot);
    if (threadIdx.x < KNN_KMAX) {
        const int r = threadIdx.x;
        const bool live = r < K && !degenerate && taken[r] != 0x7fffffff;
        res[q].idx[r] = live ? taken[r] : -1;
        res[q].cosine[r] = live ? tval[r] * invq : 0.f;
        if (!live) lab_of[r] = -1;                    // only this thread touches entry r here
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        // ranked order: the first label to reach the highest count wins a tie only if its best anchor ranks first,
        // i.e. count every label, then take the best-ranked label among those with the highest count
        int best_label = -1, best_count = 0;
        for (int r = 0; r < K && !degenerate; ++r) {
            const int lab = lab_of[r];
            if (lab < 0) break;                       // the winners ran out
            bool seen = false;
            for (int t = 0; t < r; ++t) seen = seen || (lab_of[t] == lab);
            if (seen) continue;                       // counted when first met
            int cnt = 0;
            for (int t = r; t < K; ++t) if (lab_of[t] == lab) ++cnt;
            if (cnt > best_count) { best_count = cnt; best_label = lab; }
        }
        res[q].domain = degenerate ? -1 : best_label;
        res[q].degenerate = degenerate ? 1 : 0;
    }
}

// ------------------------------------------------------------------------------------------
// draft / verify round control (Sec. 4.2), advanced on the device
// ------------------------------------------------------------------------------------------
__global__ void gen_init_kernel(GenState *st, int cache_len, int x_last, int max_new, int max_draft, float thr,
                                int32_t *out_tokens) {
    st->cache_len = cache_len; st->x_last = x_last; st->emitted = 1; st->max_new = max_new;
    st->max_draft = max_draft; st->conf_thr = thr; st->kmax = 0; st->k = 0; st->done = (max_new <= 1);
    st->n_accepted = 0; st->rounds = 0; st->drafted = 0; st->accepted = 0; st->draft_passes = 0;
    out_tokens[0] = x_last;
}

__global__ void round_begin_kernel(GenState *st, PassCtl *draft) {
    int remaining = st->max_new - st->emitted;
    int kmax = st->done ? 0 : min(st->max_draft, remaining - 1);
    if (kmax < 0) kmax = 0;
    st->kmax = kmax; st->k = 0;
    draft->active = kmax > 0; draft->n_rows = 1; draft->start = st->cache_len; draft->head_from = 0;
    draft->tok[0] = st->x_last;
}

// host_flag (may be null): two pinned host words: [0] receives the pass's new `active` value, so the host can decide on
// the next draft step after a plain stream synchronisation, without a copy; [2] the drafts made so far in the round
__global__ void draft_end_kernel(GenState *st, PassCtl *draft, const HeadResult *res, int32_t *host_flag) {
    if (!draft->active) { if (host_flag) { host_flag[0] = 0; host_flag[2] = st->k; } return; }
    int k = st->k;
    int d = res->tok[0]; float p = res->prob[0];
    st->drafts[k] = d; st->draft_p[k] = p;
    k += 1; st->k = k; st->draft_passes += 1;
    bool stop = (k >= st->kmax) || (st->conf_thr > 0.f && p < st->conf_thr);
    draft->active = stop ? 0 : 1;
    if (host_flag) { host_flag[0] = stop ? 0 : 1; host_flag[2] = k; }
    draft->tok[0] = d;
    draft->start = st->cache_len + k;
}

// expect_k >= 0: the pass was enqueued ahead of the host's knowledge, for a round of exactly expect_k drafts (its
// launch arguments and activation layout are those of expect_k + 1 rows); it runs only if the draft did stop there
__global__ void verify_begin_kernel(const GenState *st, const PassCtl *draft, PassCtl *ver, int expect_k) {
    const bool as_expected = expect_k < 0 || (draft->active == 0 && st->k == expect_k);
    ver->active = (st->done || !as_expected) ? 0 : 1;
    ver->n_rows = st->k + 1; ver->start = st->cache_len; ver->head_from = 0;
    ver->tok[0] = st->x_last;
    for (int i = 0; i < st->k; ++i) ver->tok[i + 1] = st->drafts[i];
}

// Greedy acceptance and rollback: keep the leading drafts that equal the full model's own
// token, emit the model's next token after them, move the cache length behind the last kept row.
// host_emitted (may be null): pinned host word that receives the new count of emitted tokens
// ver: the pass whose result this is; a pass that did not run (enqueued ahead for a draft count that did not come
// true) leaves the state alone
__global__ void accept_kernel(GenState *st, const PassCtl *ver, const HeadResult *res, int32_t *out_tokens, int32_t *host_emitted) {
    if (st->done || !ver->active) { if (host_emitted) *host_emitted = st->emitted; return; }
    int k = st->k, j = 0;
    while (j < k && st->drafts[j] == res->tok[j]) ++j;
    int e = st->emitted;
    for (int i = 0; i < j; ++i) out_tokens[e + i] = st->drafts[i];
    out_tokens[e + j] = res->tok[j];
    st->emitted = e + j + 1;
    st->cache_len += j + 1;
    st->x_last = res->tok[j];
    st->n_accepted = j;
    st->rounds += 1; st->drafted += k; st->accepted += j;
    if (st->emitted >= st->max_new) st->done = 1;
    if (host_emitted) *host_emitted = st->emitted;
}

// Acceptance for a stand-alone verification call: rows tok[0..n-1] = [x_last, d_1..d_k].
__global__ void verify_accept_kernel(const PassCtl *ver, const HeadResult *res, int32_t *out3) {
    int k = ver->n_rows - 1, j = 0;
    while (j < k && ver->tok[j + 1] == res->tok[j]) ++j;
    out3[0] = j; out3[1] = res->tok[j]; out3[2] = ver->start + j + 1;
}

}  // namespace ks
