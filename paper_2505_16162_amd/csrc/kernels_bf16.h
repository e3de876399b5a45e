// Tuned bf16 kernels of the decode path for gfx950 (MI355X).
//
// Everything here is bound by HBM bandwidth: a pass streams every retained weight matrix once.
// The kernels therefore share one structure: a fixed grid of workgroups, each owning a balanced
// share of every matrix's rows; the weights are stored in the order the wavefronts stream them
// (units of <= 16 rows x 32 columns, the MFMA A operand), so every wavefront reads one contiguous
// region with several 16-byte loads per lane in flight; the wavefronts meet once in LDS for the
// reduction and the fused epilogue (RoPE + KV-cache write, residual add + next RMSNorm's
// operands, SwiGLU, LM-head arg-max partials).
//
// RMSNorm is folded in without a pass of its own: the producer of a residual row writes
// gain (.) x (the next norm's gain applied) plus its share of sum(x^2); the consumer adds the
// shares up in a fixed order and scales its dot products by rsqrt(mean + eps).
#pragma once
#include <type_traits>

#include "kernels_generic.h"

namespace ks {

constexpr int NT = 1024;       // threads per workgroup
constexpr int NWV = NT / 64;   // wavefronts per workgroup
constexpr int MAX_LROWS = 640; // most rows of one matrix a workgroup may own
constexpr int ATT_CHUNK = NWV * 16;  // positions per split-KV work item (fixed: results do not depend on context length)
constexpr int ATT_PG = 4;      // (row, head) pairs per attention work item
constexpr int ATT_SELF_MERGE_PAIRS = 4;   // most (row, head) pairs per kv head for which the attention launch merges its own chunks
constexpr int ATT_SELF_MERGE_CHUNKS = 8;  // ... and most chunks (one batch of the merge's loads: context <= 2048)
constexpr int ATT_SELF_MERGE_CHUNKS_MFMA = 24;  // the matrix-core kernel's 256-thread workgroups can hold a batch of 24 (context <= 6144)
constexpr int ATT_PAD = 4;     // a chunk's partial is [head_dim] weighted values, its maximum, its sum, 2 spare floats (16-byte rows)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

enum { OP_QKV = 0, OP_RESID = 1, OP_SWIGLU = 2, OP_HEAD = 3, OP_EMBED = 4 };

struct HeadPartial { float maxv; int idx; float sumexp; int pad; };

// One matrix-vector / small-M matrix product with its epilogue.
struct WgSplit;
struct GemmOp {
    int type;
    const bf16_t *W;  // [N][K] row-major; OP_SWIGLU: [2N][K], gate rows then up rows
    int N, K;
    const float *act_in;      // fp32, the next norm's gain already applied. Draft: [K]. Verify: the live rows as this GEMM's
                              // chunk images (image_offset; with one row that is the plain vector again)
    const float *ss_in;       // [KS_MAX_ROWS][KS_NWG] the workgroups' shares of sum(x^2) per token row; nullptr: input is not normalised
    int n_ss;                 // = KS_NWG (the tuned kernels rely on it)
    float inv_dim, eps;
    // OP_RESID / OP_EMBED: residual stream and the operands of the next norm
    float *x;                 // [KS_MAX_ROWS][N]
    const float *gain_next;   // [N]
    float *act_out;           // fp32 (also OP_SWIGLU's output). Draft: [N]. Verify: the chunk images of the GEMM that reads
                              // them (image_offset with out_kc and n_rows)
    float *ss_out;            // [KS_MAX_ROWS][KS_NWG] (a row's shares are contiguous: its reader fetches them with four loads)
    // OP_QKV
    float *q_out;             // [KS_MAX_ROWS][H*hd], rotated
    bf16_t *kv_block;         // this block's cache: [2][Hkv][max_seq][hd]
    const float *cos_t, *sin_t;
    int H, Hkv, hd, max_seq;
    // OP_HEAD
    float *logits;            // [KS_MAX_ROWS][N]
    HeadPartial *head_part;   // [KS_MAX_ROWS][gridDim]
    // OP_EMBED
    const bf16_t *embed;
    // verification GEMM: LDS plan (dynamic LDS bytes of the launch, most rows any workgroup owns of this matrix)
    int lds_bytes, max_rows;
    int kc, nc;               // activation chunk length in columns and chunk count (mfma_chunking, set by the host)
    int bbuf_bytes, fixed_lds, red_bufs;   // the rest of that kernel's LDS plan (mfma_bbuf_bytes, mfma_fixed_lds, mfma_red_bufs)
    int out_kc;               // chunk length of the GEMM that reads act_out (the same call for its shape and row count)
    int n_rows;               // token rows of the pass as the host counts them (the same number the control block holds)
    // [KS_NWG] this matrix shape's workgroup splits, tabulated once (split_table_kernel): a kernel reads its entry
    // with one scalar load instead of recomputing it in every wavefront of every launch
    const WgSplit *split;
};

__device__ __forceinline__ float bf_lo(unsigned int u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(unsigned int u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ float dot8(u32x4 w, float4 x0, float4 x1, float acc) {
    acc = fmaf(bf_lo(w.x), x0.x, acc); acc = fmaf(bf_hi(w.x), x0.y, acc);
    acc = fmaf(bf_lo(w.y), x0.z, acc); acc = fmaf(bf_hi(w.y), x0.w, acc);
    acc = fmaf(bf_lo(w.z), x1.x, acc); acc = fmaf(bf_hi(w.z), x1.y, acc);
    acc = fmaf(bf_lo(w.w), x1.z, acc); acc = fmaf(bf_hi(w.w), x1.w, acc);
    return acc;
}

// Hand-placed streaming loads: the compiler's own wait insertion drains the whole queue wherever a load sits under
// a loop-carried or conditional path, which leaves gaps in a wavefront's request stream. These two helpers issue a
// nontemporal 16-byte load the compiler does not count, and wait until at most KEEP younger loads are still in
// flight before the register may be used (loads return in order).
__device__ __forceinline__ u32x4 stream_load(const bf16_t *p) {
    u32x4 v;
    asm volatile("global_load_dwordx4 %0, %1, off nt" : "=v"(v) : "v"(p) : "memory");
    return v;
}
template <int KEEP>
__device__ __forceinline__ void stream_wait(u32x4 &r) {
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(r) : "n"(KEEP) : "memory");
}
// the same for small operands that are expected in cache (no nontemporal hint)
__device__ __forceinline__ u32x4 stream_load_x4(const void *p) {
    u32x4 v;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(p) : "memory");
    return v;
}
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float stream_load_f32(const float *p) {
    float v;
    asm volatile("global_load_dword %0, %1, off" : "=v"(v) : "v"(p) : "memory");
    return v;
}
// waits that name several registers at once (a kernel's small first operands, issued before the KEEP loads that may
// stay in flight): N 16-byte pieces, or four norm shares and two epilogue values
template <int KEEP, int N>
__device__ __forceinline__ void stream_wait_pieces(u32x4 *x) {
    static_assert(N == 3 || N == 4 || N == 5, "piece count");
    if constexpr (N == 3)
        asm volatile("s_waitcnt vmcnt(%3)" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]) : "n"(KEEP) : "memory");
    else if constexpr (N == 4)
        asm volatile("s_waitcnt vmcnt(%4)" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]) : "n"(KEEP) : "memory");
    else
        asm volatile("s_waitcnt vmcnt(%5)" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]) : "n"(KEEP) : "memory");
}
template <int KEEP>
__device__ __forceinline__ void stream_wait_scalars(float *sh, float &a, float &b) {
    asm volatile("s_waitcnt vmcnt(%6)" : "+v"(sh[0]), "+v"(sh[1]), "+v"(sh[2]), "+v"(sh[3]), "+v"(a), "+v"(b) : "n"(KEEP) : "memory");
}
// drain: every register of the batch is named, so that no use of any of them can be moved above the wait
__device__ __forceinline__ void stream_drain8(u32x4 *r) {
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7]) : : "memory");
}

// First of the n items that workgroup wg owns when n items are dealt to the KS_NWG workgroups in balanced contiguous
// shares: floor(n * wg / KS_NWG), as a multiply and a shift (a 64-bit division costs a wavefront hundreds of cycles,
// and every wavefront runs several of these before it can issue its first load).
static_assert(KS_NWG == 256, "wg_share assumes 256 workgroups");
__device__ __forceinline__ int wg_share(int n, int wg) { return (int)(((unsigned int)n * (unsigned int)wg) >> 8); }

// A uniform value the optimiser must treat as defined here: arithmetic on it cannot be hoisted above this point.
__device__ __forceinline__ int pinned_here(int v) {
    asm volatile("" : "+s"(v));
    return v;
}

// Rows of W a workgroup owns, as a table of global row indices in LDS. Returns the count.
// OP_QKV orders them [first halves of np rotary pairs][their second halves][nv value rows],
// OP_SWIGLU [nf gate rows][the matching nf up rows].
// FILL = false only counts (scalar work): the GEMM kernels need the counts to place their first weight loads and
// fill the table afterwards, while those loads are in flight.
template <bool FILL>
__device__ __forceinline__ int build_row_table(const GemmOp &op, int wg, int *rowidx, int *n_first) {
    int R = 0;
    if (op.type == OP_QKV) {
        const int half = op.hd >> 1;
        const int P = (op.H + op.Hkv) * half, VR = op.Hkv * op.hd;
        const int p0 = wg_share(P, wg), p1 = wg_share(P, wg + 1);
        const int v0 = wg_share(VR, wg), v1 = wg_share(VR, wg + 1);
        const int np = p1 - p0, nv = v1 - v0;
        R = 2 * np + nv;
        if constexpr (FILL) {
            for (int t = threadIdx.x; t < R; t += NT) {
                int row;
                if (t < 2 * np) {
                    int p = p0 + (t < np ? t : t - np);
                    int head = p / half, i = p - head * half;
                    row = head * op.hd + i + (t < np ? 0 : half);
                } else {
                    row = (op.H + op.Hkv) * op.hd + v0 + (t - 2 * np);
                }
                rowidx[t] = row;
            }
        }
        *n_first = np;
    } else if (op.type == OP_SWIGLU) {
        const int f0 = wg_share(op.N, wg), f1 = wg_share(op.N, wg + 1);
        const int nf = f1 - f0;
        R = 2 * nf;
        if constexpr (FILL)
            for (int t = threadIdx.x; t < R; t += NT) rowidx[t] = (t < nf) ? f0 + t : op.N + f0 + (t - nf);
        *n_first = nf;
    } else {
        const int r0 = wg_share(op.N, wg), r1 = wg_share(op.N, wg + 1);
        R = r1 - r0;
        if constexpr (FILL)
            for (int t = threadIdx.x; t < R; t += NT) rowidx[t] = r0 + t;
        *n_first = R;
    }
    return R;
}

// workgroup sum of one float per thread (NT threads); scratch: NWV floats of LDS
__device__ __forceinline__ float block_sum(float v, float *scratch) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < NWV; ++w) t += scratch[w];
    return t;
}

// ------------------------------------------------------------------------------------------
// Epilogue shared by the draft (1 row) and verify (n_rows) kernels. vals[lr * ld + m] holds the
// finished dot product of local row lr and token row m (LDS).
// ------------------------------------------------------------------------------------------
// i / n for 0 <= i < 2^20 and n >= 1 from a float product (inv = an approximation of 1/n within a few ulp): the
// quotient is corrected by one step either way, so the result is exact; an integer division costs ten times as much
__device__ __forceinline__ int div_small(int i, int n, float inv) {
    int q = (int)(((float)i + 0.5f) * inv);
    const int r = i - q * n;
    q += (r >= n) - (r < 0);
    return q;
}

// Where the verification GEMM's activations live ("chunk images"). The GEMM stages its token rows through LDS in
// chunks of kc columns (mfma_chunking); the producer of those activations writes them so that a chunk is one contiguous
// range of fp32 values: chunk c holds columns [c*kc, c*kc + cols_c) of the n_rows live rows, row after row. All chunks
// before the last are full, so chunk c starts at c * n_rows * kc. The consumer fetches a chunk as 16-byte pieces with
// straight indexing (4 bytes per element cross the L2, not the 6 of ready-made bf16 planes) and splits every value into
// its three bf16 planes on the way into LDS. With one live row the image is the plain vector.
// Returns the element offset of (row m, column n).
__device__ __forceinline__ int image_offset(int m, int n, int ldn, int kc, int n_rows, float inv_kc) {
    const int c = div_small(n, kc, inv_kc);
    const int cols_c = min(kc, ldn - c * kc);
    return c * (n_rows * kc) + m * cols_c + (n - c * kc);
}

// IMAGE = false: the draft step's plain vector (row 0); true: the chunk image of the GEMM that reads the value
template <bool IMAGE>
__device__ __forceinline__ void store_act(const GemmOp &op, int m, int n, int ldn, float v, float inv_kc) {
    if (!IMAGE) op.act_out[(size_t)m * ldn + n] = v;
    else op.act_out[image_offset(m, n, ldn, op.out_kc, op.n_rows, inv_kc)] = v;
}

template <bool PLANES>
__device__ __forceinline__ void gemm_epilogue(const GemmOp &op, const PassCtl *ctl, int wg, int nwg, int R, int n_first,
                                              const int *rowidx, const float *vals, int ld, const float *rstd,
                                              int row_lo, int n_rows, float *scratch, float xpre, float gpre) {
    // xpre / gpre: OP_RESID only, the residual value and the next norm's gain of element i = tid (fetched early by
    // the caller so that the tail of the kernel does not wait on memory)
    const int tid = threadIdx.x;
    const float inv_kc = PLANES ? __builtin_amdgcn_rcpf((float)op.out_kc) : 0.f;
    if (op.type == OP_RESID) {
        // one thread per (row of W, token row): residual add, operands of the next norm, x^2 left in vals
        float *vw = const_cast<float *>(vals);
        for (int i = tid; i < R * ld; i += NT) {
            const int t = i / ld, m = i - t * ld;
            float sq = 0.f;
            if (m < n_rows) {
                const int n = rowidx[t];
                const bool pre = i == tid;
                const float xn = (pre ? xpre : op.x[(size_t)m * op.N + n]) + vals[i];
                op.x[(size_t)m * op.N + n] = xn;
                store_act<PLANES>(op, m, n, op.N, (pre ? gpre : op.gain_next[n]) * xn, inv_kc);
                sq = xn * xn;
            }
            vw[i] = sq;
        }
        __syncthreads();
        // this workgroup's share of sum(x^2) per token row: one wavefront per row, fixed order
        const int lane = tid & 63;
        for (int m = tid >> 6; m < n_rows; m += NWV) {
            float sacc = 0.f;
            for (int t = lane; t < R; t += 64) sacc += vals[t * ld + m];
            sacc = wave_sum(sacc);
            if (lane == 0) op.ss_out[(size_t)m * KS_NWG + wg] = sacc;
        }
    } else if (op.type == OP_SWIGLU) {
        const float inv_rows = __builtin_amdgcn_rcpf((float)n_rows);
        for (int i = tid; i < n_first * n_rows; i += NT) {       // one thread per (gate row, token row)
            const int t = div_small(i, n_rows, inv_rows), m = i - t * n_rows;
            const int n = rowidx[t];
            const float a = vals[t * ld + m] * rstd[m], b = vals[(t + n_first) * ld + m] * rstd[m];
            store_act<PLANES>(op, m, n, op.N, (a / (1.0f + expf(-a))) * b, inv_kc);
        }
    } else if (op.type == OP_QKV) {
        const int half = op.hd >> 1, qd = op.H * op.hd;
        const int np = n_first;
        bf16_t *kc = op.kv_block;
        bf16_t *vc = op.kv_block + (size_t)op.Hkv * op.max_seq * op.hd;
        const int start = ctl->start;
        const float inv_rows = __builtin_amdgcn_rcpf((float)n_rows);
        const int hd_shift = 31 - __builtin_clz(op.hd), hd_mask = op.hd - 1;      // head_dim is 64 or 128
        for (int it = tid; it < (R - np) * n_rows; it += NT) {    // one thread per (pair or value row, token row)
            // t < np: rotary pair (row, row + half);  t >= np: value row (local index t + np)
            const int t = div_small(it, n_rows, inv_rows), m = it - t * n_rows;
            const bool is_pair = t < np;
            const int lr = is_pair ? t : t + np;
            const int n = rowidx[lr];
            {
                const int pos = start + m;
                if (is_pair) {
                    const int head = n >> hd_shift, i = n & hd_mask;
                    const float c = op.cos_t[(size_t)pos * half + i], s = op.sin_t[(size_t)pos * half + i];
                    const float a = vals[lr * ld + m] * rstd[m], b = vals[(lr + np) * ld + m] * rstd[m];
                    const float ra = a * c - b * s, rb = b * c + a * s;
                    if (head < op.H) {
                        op.q_out[(size_t)m * qd + n] = ra;
                        op.q_out[(size_t)m * qd + n + half] = rb;
                    } else {
                        const size_t base = ((size_t)(head - op.H) * op.max_seq + pos) * op.hd + i;
                        kc[base] = float_to_bf16_rne(ra);
                        kc[base + half] = float_to_bf16_rne(rb);
                    }
                } else {
                    const int vr = n - (op.H + op.Hkv) * op.hd;
                    const int head = vr >> hd_shift, i = vr & hd_mask;
                    vc[((size_t)head * op.max_seq + pos) * op.hd + i] = float_to_bf16_rne(vals[lr * ld + m] * rstd[m]);
                }
            }
        }
    } else if (op.type == OP_HEAD) {
        // logits of this workgroup's rows, plus (max, lowest arg-max, sum exp(l - max)) over them: one wavefront per
        // token row, so the rows of a pass are handled side by side and the workgroup never meets
        const int lane = tid & 63;
        for (int m = row_lo + (tid >> 6); m < n_rows; m += NWV) {
            float bv = -INFINITY; int bi = 0x7fffffff;
            for (int t = lane; t < R; t += 64) {
                const int n = rowidx[t];
                const float l = vals[t * ld + m] * rstd[m];
                op.logits[(size_t)m * op.N + n] = l;
                if (better(l, n, bv, bi)) { bv = l; bi = n; }
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                float ov = __shfl_xor(bv, off, 64); int oi = __shfl_xor(bi, off, 64);
                if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
            }
            float se = 0.f;
            for (int t = lane; t < R; t += 64) se += expf(vals[t * ld + m] * rstd[m] - bv);
            se = wave_sum(se);
            if (lane == 0) {
                HeadPartial hp; hp.maxv = bv; hp.idx = bi; hp.sumexp = (R > 0) ? se : 0.f; hp.pad = 0;
                op.head_part[(size_t)m * nwg + wg] = hp;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Stream order. The weight matrices are not read in row-major order: knnssd_pack_matrix rewrites
// each of them once into the exact order the kernels stream it, so that every wavefront reads one
// contiguous region of HBM with fully coalesced loads (row-major operand tiles, 16 rows x 64
// bytes per load, measure about 30 % slower on MI355X). The order is:
//
//   workgroup (256 of them, balanced row shares, rows in build_row_table order)
//     tile (T = ceil(R/16) tiles of rpt = ceil(R/T) <= 16 rows; the last one may be shorter)
//       wavefront of the tile's lane: tl = 4, 2 or 1 tile lanes work on different tiles at once,
//       the ksplit = 16 / tl wavefronts of a lane deal the columns among themselves in fixed
//       512-column blocks (wavefront kpart owns the g = 16 / ksplit 32-column steps
//       [kpart*g, kpart*g+g) of every block)
//         unit = one 32-column step of the tile: rows_t x 64 bytes, stored as 4 column groups of
//         rows_t 16-byte pieces (piece (kg, r) = 8 columns at 8*kg of row r), which is the A operand
//         of v_mfma_f32_16x16x32_bf16 with lane = 16*kg + r.
//
// The draft GEMV and the verification GEMM read the same units; they differ only in the
// arithmetic applied to a unit. The packed matrix has the size of the original.
// ------------------------------------------------------------------------------------------
struct alignas(64) WgSplit {
    int R, n_first;   // rows of this workgroup, rows of the first kind (rotary pairs / gate rows)
    int T, rpt, tl, ksplit, ksshift, g, gshift;
    int KS, nfull, rem;   // 32-column steps in K, full 16-step blocks, steps of the last partial block
    size_t wg_base;       // element offset of the workgroup's region in the packed matrix
};
static_assert(sizeof(WgSplit) == 64, "one 64-byte scalar load per workgroup");
static_assert(KS_NWG * sizeof(WgSplit) >= (size_t)KS_NWG * KS_MAX_ROWS * sizeof(float),
              "a split table doubles as a dummy share array (a GEMM without a norm in front reads it and drops the result)");

template <bool FILL = true>
__device__ __forceinline__ WgSplit make_split(const GemmOp &op, int wg, int nwg, int *rowidx) {
    WgSplit s;
    s.R = build_row_table<FILL>(op, wg, rowidx, &s.n_first);
    size_t rows_before;
    if (op.type == OP_QKV) {
        const int half = op.hd >> 1;
        const long long P = (long long)(op.H + op.Hkv) * half, VR = (long long)op.Hkv * op.hd;
        rows_before = (size_t)(2 * wg_share((int)P, wg) + wg_share((int)VR, wg));
    } else if (op.type == OP_SWIGLU) {
        rows_before = (size_t)(2 * wg_share(op.N, wg));
    } else {
        rows_before = (size_t)wg_share(op.N, wg);
    }
    s.wg_base = rows_before * op.K;
    s.T = (s.R + 15) >> 4;
    s.rpt = s.T ? (s.R + s.T - 1) / s.T : 0;
    s.tl = s.T >= 3 ? 4 : (s.T >= 2 ? 2 : 1);   // three tiles: one round on three of four lanes, not two rounds on two
    s.ksplit = NWV / s.tl;                      // NWV = 16: 4, 8 or 16
    s.ksshift = (s.tl == 4) ? 2 : (s.tl == 2 ? 3 : 4);
    s.g = 16 >> s.ksshift;
    s.gshift = (s.g == 4) ? 2 : (s.g == 2 ? 1 : 0);
    s.KS = op.K >> 5;
    s.nfull = s.KS >> 4;
    s.rem = s.KS & 15;
    return s;
}

// One wavefront's share of one tile.
struct WaveTile {
    bool have;          // this wavefront has a tile in this round
    int t, rows_t;      // tile index, its row count
    int cnt;            // 32-column steps this wavefront owns (over all of K)
    int unit;           // elements per unit = rows_t * 32
    size_t base;        // element offset of the wavefront's first unit in the packed matrix
};

__device__ __forceinline__ WaveTile wave_tile(const WgSplit &s, int K, int round, int tlane, int kpart) {
    WaveTile w;
    w.t = round * s.tl + tlane;
    w.have = w.t < s.T;
    w.rows_t = w.have ? min(s.rpt, s.R - w.t * s.rpt) : 1;
    w.unit = w.rows_t * 32;
    w.cnt = w.have ? s.nfull * s.g + min(max(s.rem - kpart * s.g, 0), s.g) : 0;
    const int steps_before = s.nfull * s.g * kpart + min(s.rem, kpart * s.g);
    w.base = s.wg_base + (size_t)(w.t * s.rpt) * K + (size_t)steps_before * w.unit;
    return w;
}

// 32-column step (index within K) of a wavefront's u-th unit
__device__ __forceinline__ int step_of_unit(const WgSplit &s, int kpart, int u) {
    return ((u >> s.gshift) << 4) + kpart * s.g + (u & (s.g - 1));
}

// Tabulates the splits of one matrix shape (type, N, K and the head counts of op): table[wg], KS_NWG entries.
__global__ void split_table_kernel(GemmOp op, WgSplit *table) {
    const int wg = blockIdx.x * blockDim.x + threadIdx.x;
    if (wg < KS_NWG) table[wg] = make_split<false>(op, wg, KS_NWG, nullptr);
}

// Rewrites a row-major matrix into stream order (run once per matrix when the model is loaded).
__global__ __launch_bounds__(NT, 1) void pack_matrix_kernel(GemmOp op, const bf16_t *__restrict__ src, bf16_t *__restrict__ dst) {
    __shared__ int rowidx[MAX_LROWS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const WgSplit s = make_split(op, blockIdx.x, gridDim.x, rowidx);
    __syncthreads();
    const int tlane = wave >> s.ksshift, kpart = wave & (s.ksplit - 1);
    const int r16 = lane & 15, kg = lane >> 4;
    for (int round = 0; round * s.tl < s.T; ++round) {
        const WaveTile w = wave_tile(s, op.K, round, tlane, kpart);
        if (!w.have || r16 >= w.rows_t) continue;
        const bf16_t *srow = src + (size_t)rowidx[w.t * s.rpt + r16] * op.K + kg * 8;
        bf16_t *d = dst + w.base + (size_t)(kg * w.rows_t + r16) * 8;
        for (int u = 0; u < w.cnt; ++u) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(srow + (size_t)step_of_unit(s, kpart, u) * 32);
            *reinterpret_cast<u32x4 *>(d + (size_t)u * w.unit) = v;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Draft step (one row): y = W x on the vector ALUs. Each wavefront streams its units (eight 16-byte
// loads per lane in flight), lane (kg, r) multiplies its 8 weights with x[32*step + 8*kg ..] from
// LDS and keeps a private sum for row r; a tile ends with a 4-lane reduction over kg.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void gemv_device(const GemmOp &op, const PassCtl *ctl, int wg, int nwg, char *lds) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = op.K;
    float *xs = reinterpret_cast<float *>(lds);                 // [K]
    float *part = xs + K;                                       // [MAX_LROWS][NWV]
    int *rowidx = reinterpret_cast<int *>(part + MAX_LROWS * NWV);
    float *vals = reinterpret_cast<float *>(rowidx + MAX_LROWS);     // [MAX_LROWS]
    float *scratch = vals + MAX_LROWS;                               // [4*NWV + KS_MAX_ROWS]
    float *rstd_s = scratch + 4 * NWV;

    // read through the scalar cache while that is still possible: after the first hand-placed load (whose memory
    // clobber the compiler must honour) this would become a vector load queued behind the whole weight batch
    const int active = ctl->active;
    const WgSplit s = op.split[wg];                // tabulated; the row table is filled below
    const int R = s.R;
    const int tlane = wave >> s.ksshift, kpart = wave & (s.ksplit - 1);
    const int r16 = lane & 15, kg = lane >> 4;

    // Order of the first loads: the input vector and the norm's shares (small, cache hits) go out first and the
    // first weight batch right behind them; the vector is in LDS and the workgroup has met long before the
    // weights arrive, so no wavefront sits on a full batch. Every load of this prologue is a hand-placed one and
    // unconditional (addresses are clamped instead), and one wait that leaves the weight batch in flight covers
    // all the small ones: the compiler's own counting would charge the weight loads to them.
    constexpr int XQ = 4;
    u32x4 xr[XQ];
#pragma unroll
    for (int q = 0; q < XQ; ++q) xr[q] = stream_load_x4(op.act_in + min((tid + q * NT) * 4, K - 4));
    float sh[4];
    {
        // KS_NWG = 4 x 64 shares per token row; without a norm in front of this GEMM the loads read the split table
        // instead (as large as the share array) and their result is dropped
        const float *sp = op.ss_in ? op.ss_in : reinterpret_cast<const float *>(op.split);
#pragma unroll
        for (int j = 0; j < 4; ++j) sh[j] = stream_load_f32(sp + lane + 64 * j);
    }
    float xpre, gpre;
    {
        const bool resid = op.type == OP_RESID;
        const int n = resid ? min(wg_share(op.N, wg) + tid, op.N - 1) : 0;
        xpre = stream_load_f32((resid ? op.x : op.act_in) + n);
        gpre = stream_load_f32((resid ? op.gain_next : op.act_in) + n);
    }
    // Weight loads are hand-placed streaming loads the compiler does not track (see stream_load): all of them, so
    // that none of the compiler's own waits is ever aimed at a weight register. Each batch is eight unconditional
    // loads (a wavefront with fewer units re-reads its last one; one without units reads the matrix's first bytes).
    // A round's batch is issued at ONE place in the code, the first round's included: with two places the compiler
    // gives them different registers and joins them with copies, which would read registers whose loads are still
    // in flight. (Round 0 therefore also runs for a workgroup without rows; it then owns no unit.)
    u32x4 wa[8];
    if (!active) return;           // uniform (read long ago, so no wait here); loads in flight are dropped with the wavefront
    for (int round = 0; round == 0 || round * s.tl < s.T; ++round) {
        const WaveTile w = wave_tile(s, K, round, tlane, kpart);
        const bf16_t *wp = op.W + w.base + (size_t)(kg * w.rows_t + min(r16, w.rows_t - 1)) * 8;
        {
            const bf16_t *p0 = w.cnt > 0 ? wp : op.W;
            const int last = max(w.cnt - 1, 0);
#pragma unroll
            for (int i = 0; i < 8; ++i) wa[i] = stream_load(p0 + (size_t)min(i, last) * w.unit);
        }
        if (round == 0) {
            // the row table is read after the next meeting at the earliest; its index arithmetic is pinned behind
            // the weight loads just issued (it is loop invariant and would otherwise be hoisted in front of them)
            GemmOp shape;
            shape.type = pinned_here(op.type); shape.N = pinned_here(op.N);
            shape.H = pinned_here(op.H); shape.Hkv = pinned_here(op.Hkv); shape.hd = pinned_here(op.hd);
            int n_first_unused;
            build_row_table<true>(shape, pinned_here(wg), rowidx, &n_first_unused);
            stream_wait_pieces<8 + 6, XQ>(xr);          // the six small loads and the eight weight loads stay in flight
            // (stores clamped like the loads: a duplicate writes the same value to the same place)
#pragma unroll
            for (int q = 0; q < XQ; ++q) *reinterpret_cast<u32x4 *>(xs + min((tid + q * NT) * 4, K - 4)) = xr[q];
            for (int i = (tid + XQ * NT) * 4; i < K; i += NT * 4) *reinterpret_cast<float4 *>(xs + i) = *reinterpret_cast<const float4 *>(op.act_in + i);
            __syncthreads();
        }
        float acc = 0.f;
        int u0 = 0;
        // steady state: every unit has a successor eight units on; its register is refilled the moment it has been
        // used and the wait before a unit leaves the seven younger loads in flight, so the stream never drains.
        // (The loop sits under its own condition so that it has one way in: a second, empty way in would make the
        // compiler treat the registers as results of loads it tracks and drain the stream at the loop's head.)
        if (w.cnt >= 16) {
            do {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float *xp = xs + step_of_unit(s, kpart, u0 + i) * 32 + kg * 8;
                    const float4 x0 = *reinterpret_cast<const float4 *>(xp), x1 = *reinterpret_cast<const float4 *>(xp + 4);
                    stream_wait<7>(wa[i]);
                    acc = dot8(wa[i], x0, x1, acc);
                    wa[i] = stream_load(wp + (size_t)(u0 + i + 8) * w.unit);
                }
                u0 += 8;
            } while (u0 + 16 <= w.cnt);
        }
        // tail: at most 15 units left, drained batch by batch (at least one drain: no load of this round may be
        // in flight when the next round's batch is issued into the same registers)
        do {
            stream_drain8(wa);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (u0 + i < w.cnt) {
                    const float *xp = xs + step_of_unit(s, kpart, u0 + i) * 32 + kg * 8;
                    const float4 x0 = *reinterpret_cast<const float4 *>(xp), x1 = *reinterpret_cast<const float4 *>(xp + 4);
                    acc = dot8(wa[i], x0, x1, acc);
                }
            }
            u0 += 8;
            if (u0 >= w.cnt) break;        // left with nothing in flight; any load below is followed by a drain
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (u0 + i < w.cnt) wa[i] = stream_load(wp + (size_t)(u0 + i) * w.unit);
        } while (true);
        acc += __shfl_xor(acc, 16, 64);
        acc += __shfl_xor(acc, 32, 64);
        if (w.have && kg == 0 && r16 < w.rows_t) part[(w.t * s.rpt + r16) * NWV + kpart] = acc;
    }
    // the norm's shares and the epilogue's two values were issued before the first weight batch and are long here
    // (every round ends drained); the wait only ties their registers to this point
    stream_wait_scalars<0>(sh, xpre, gpre);
    if (wave == 0) {
        float share = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) share += sh[j];
        const float r = op.ss_in ? 1.0f / sqrtf(wave_sum(share) * op.inv_dim + op.eps) : 1.0f;
        if (lane == 0) rstd_s[0] = r;
    }
    __syncthreads();
    // finished dot products: fixed-order sum over the wavefronts that shared the tile's columns
    for (int t = tid; t < R; t += NT) {
        float sum = 0.f;
        for (int k = 0; k < s.ksplit; ++k) sum += part[t * NWV + k];
        vals[t] = sum;
    }
    __syncthreads();
    gemm_epilogue<false>(op, ctl, wg, nwg, R, s.n_first, rowidx, vals, 1, rstd_s, ctl->head_from, 1, scratch, xpre, gpre);
}

__host__ __device__ inline size_t gemv_lds_bytes(int K) {
    return (size_t)K * 4 + (size_t)MAX_LROWS * NWV * 4 + MAX_LROWS * 4 + MAX_LROWS * 4 + (4 * NWV + KS_MAX_ROWS) * 4;
}

__global__ __launch_bounds__(NT, 1) void gemv_kernel(GemmOp op, const PassCtl *ctl) {
    extern __shared__ __align__(16) char lds[];
    gemv_device(op, ctl, blockIdx.x, gridDim.x, lds);
}

// ------------------------------------------------------------------------------------------
// Verification (up to 16 rows): Y = W X on the matrix cores. A unit is the A operand of
// v_mfma_f32_16x16x32_bf16 as stored (lane = 16*kg + r), the token rows are the B operand.
// Activations stay fp32-exact: each value is the sum of three bf16 planes (hi + mid + lo), so a
// unit takes three MFMAs whose bf16 x bf16 products are exact in the fp32 accumulator. The path is
// HBM-bound (<= 16 flop per weight byte against a ridge of ~300), so the two extra MFMAs cost
// nothing. A token row's result never depends on how many other rows are live.
// ------------------------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int MFMA_BQ = 3;          // 16-byte pieces (four fp32 values) of an activation chunk a thread may carry: 72 KB of planes in LDS

// LDS plan of the verification GEMM: [vals: max_rows x 16 floats][red: 1 or 2 x NWV x 256 floats][row table][scratch]
// and two activation staging buffers sharing what is left of the dynamic LDS the launch asked for. A staging buffer
// must hold the shortest chunk (512 columns) of 16 rows; where a workgroup owns so many rows of the matrix that
// two partial-tile buffers leave less than that, there is one (and one more meeting per round).
constexpr int MFMA_MIN_BBUF = 3 * KS_MAX_ROWS * (512 * 2 + 16);
__host__ __device__ inline size_t mfma_fixed_lds_rb(int max_rows, int red_bufs) {
    return ((size_t)max_rows * KS_MAX_ROWS * 4 + (size_t)red_bufs * NWV * 256 * 4 + (size_t)max_rows * 4 + (4 * NWV + KS_MAX_ROWS) * 4 + 255) / 256 * 256;
}
__host__ __device__ inline int mfma_red_bufs(size_t lds_total, int max_rows) {
    return ((long long)lds_total - (long long)mfma_fixed_lds_rb(max_rows, 2)) / 2 / 256 * 256 >= MFMA_MIN_BBUF ? 2 : 1;
}
__host__ __device__ inline size_t mfma_fixed_lds(size_t lds_total, int max_rows) {
    return mfma_fixed_lds_rb(max_rows, mfma_red_bufs(lds_total, max_rows));
}
__host__ __device__ inline int mfma_bbuf_bytes(size_t lds_total, int max_rows) {
    long long b = ((long long)lds_total - (long long)mfma_fixed_lds(lds_total, max_rows)) / 2 / 256 * 256;
    const long long cap = (long long)MFMA_BQ * NT * 24;     // a fetched piece becomes 3 x 8 bytes of planes
    return (int)(b > cap ? cap : b);
}
// The token rows (B operand) are staged through LDS in column chunks shared by all wavefronts: only the live rows
// are staged, so few rows mean long chunks (often the whole of K). A chunk is a multiple of 512 columns, i.e. whole
// blocks of the column deal; the deal itself does not depend on the chunk length, so a row's sum is grouped the
// same way however many rows are live.
__host__ __device__ inline void mfma_chunking(size_t lds_total, int max_rows, int n_rows, int K, int *kc, int *nc) {
    const int bbuf = mfma_bbuf_bytes(lds_total, max_rows);
    int KC = (bbuf / (3 * n_rows) - 16) / 2;
    KC = KC / 512 * 512;
    if (KC < 512) KC = 512;
    if (KC > K) KC = (K + 511) / 512 * 512;
    *kc = KC;
    *nc = (K + KC - 1) / KC;
}

// RING: the weight stream rolls on across the boundaries of the activation chunks (launches with many chunks)
template <bool RING>
__device__ __forceinline__ void gemm_mfma_device(const GemmOp &op, const PassCtl *ctl, int wg, int nwg, char *lds) {
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = op.K;
    float *vals = reinterpret_cast<float *>(lds);                       // [max_rows][16]
    float *red = vals + (size_t)op.max_rows * KS_MAX_ROWS;              // [1 or 2][NWV][256]
    const int RB = op.red_bufs;
    int *rowidx = reinterpret_cast<int *>(red + RB * NWV * 256);
    float *scratch = reinterpret_cast<float *>(rowidx + op.max_rows);
    float *rstd_s = scratch + 4 * NWV;
    const int BBUF = op.bbuf_bytes;
    char *bbuf = lds + op.fixed_lds;                                    // [2][BBUF] activation chunks
    const int n_rows = op.n_rows;                                       // the host's count; equals ctl->n_rows

    const int active = ctl->active;     // both through the scalar cache, which only works before the first hand-placed load
    const WgSplit s = op.split[wg];     // tabulated; the row table is filled below, behind the first loads
    const int R = s.R;

    const int tlane = wave >> s.ksshift, kpart = wave & (s.ksplit - 1);
    const int r16 = lane & 15, kg = lane >> 4;
    const int KC = op.kc, NC = op.nc;                                    // see mfma_chunking
    const int brow = min(r16, n_rows - 1);                               // dead token lanes re-read the last live row
    u32x4 breg[MFMA_BQ];
    // The activations arrive as chunk images (image_offset): chunk c is one contiguous range of n_rows * cols_c fp32
    // values, row after row. Piece i of the range (four values of row i / (cols_c/4)) is split into its three exact
    // bf16 planes (hi + mid + lo by truncation) and lands in the LDS stage, whose 3 * n_rows rows (plane-major) have
    // cols_c + 8 elements each (the 16 spare bytes spread the rows over the banks and are never read).
    auto chunk_pieces = [&](int c) { return n_rows * (min(KC, K - c * KC) >> 2); };
    // (t = the thread's index, passed in so that a caller inside the unit loop can hand over a copy the optimiser
    // cannot see through: the piece offsets are then recomputed on the spot instead of living in registers)
    auto bchunk_load = [&](int c, int t) {   // global -> registers (hand-placed loads)
        const float *src = op.act_in + c * (n_rows * KC);
        const int last = chunk_pieces(c) - 1;
#pragma unroll
        for (int q = 0; q < MFMA_BQ; ++q)        // unconditional (clamped): the waits below count on exactly MFMA_BQ loads
            breg[q] = stream_load_x4(src + min(t + q * NT, last) * 4);
    };
    auto bchunk_store = [&](int c, int t) {  // registers -> planes in LDS buffer c & 1
        char *dst = bbuf + (c & 1) * BBUF;
        const int cols = min(KC, K - c * KC), ppr = cols >> 2;      // pieces per row
        const int last = n_rows * ppr - 1, bstride = (cols + 8) * 2, pstep = n_rows * bstride;
        const float inv_ppr = __builtin_amdgcn_rcpf((float)ppr);
#pragma unroll
        for (int q = 0; q < MFMA_BQ; ++q) {      // clamped like the loads: a duplicate writes the same value to the same place
            const int i = min(t + q * NT, last);
            const int row = div_small(i, ppr, inv_ppr), c4 = i - row * ppr;
            unsigned int hi[4], mid[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned int u = breg[q][e];
                const float r1 = __uint_as_float(u) - __uint_as_float(u & 0xffff0000u);
                const unsigned int um = __float_as_uint(r1);
                hi[e] = u; mid[e] = um;
                lo[e] = __float_as_uint(r1 - __uint_as_float(um & 0xffff0000u));
            }
            char *d = dst + row * bstride + c4 * 8;
            // the upper halves of two neighbouring values make one register of a plane
            *reinterpret_cast<u32x2 *>(d) = u32x2{__builtin_amdgcn_perm(hi[1], hi[0], 0x07060302u), __builtin_amdgcn_perm(hi[3], hi[2], 0x07060302u)};
            *reinterpret_cast<u32x2 *>(d + pstep) = u32x2{__builtin_amdgcn_perm(mid[1], mid[0], 0x07060302u), __builtin_amdgcn_perm(mid[3], mid[2], 0x07060302u)};
            *reinterpret_cast<u32x2 *>(d + 2 * pstep) = u32x2{__builtin_amdgcn_perm(lo[1], lo[0], 0x07060302u), __builtin_amdgcn_perm(lo[3], lo[2], 0x07060302u)};
        }
    };

    // units of chunk c this wavefront owns (they are consecutive in its stream)
    auto chunk_count = [&](int c, bool have) {
        const int cs = min(KC, K - c * KC) >> 5, nfull = cs >> 4, rem = cs & 15;
        return have ? nfull * s.g + min(max(rem - kpart * s.g, 0), s.g) : 0;
    };

    // Order of the first loads: activations, norm shares and residual values (small, cache hits) go out first and
    // the first weight batch right behind them. The activations are in LDS and the workgroup has met long before
    // the weights arrive. Every load of the main part is a hand-placed one (see stream_load) and unconditional
    // (addresses are clamped instead), so the number of loads in flight is known at every wait; the compiler's
    // own counting would charge the weight stream to the small loads and the other way round.
    bchunk_load(0, tid);
    float sh[4];
    {
        // KS_NWG = 4 x 64 shares per token row, wavefront m sums row m's; without a norm in front of this GEMM the
        // loads read the split table instead (as large as the share array) and their result is dropped
        const float *sp = (op.ss_in ? op.ss_in : reinterpret_cast<const float *>(op.split)) + min(wave, n_rows - 1) * KS_NWG;
#pragma unroll
        for (int j = 0; j < 4; ++j) sh[j] = stream_load_f32(sp + lane + 64 * j);
    }
    float xpre, gpre;
    {
        const bool resid = op.type == OP_RESID;
        const int n = resid ? min(wg_share(op.N, wg) + (tid >> 4), op.N - 1) : 0;
        const float *fallback = op.act_in;
        xpre = stream_load_f32((resid ? op.x : fallback) + (resid ? (size_t)min(tid & 15, n_rows - 1) * op.N + n : 0));
        gpre = stream_load_f32((resid ? op.gain_next : fallback) + n);
    }
    if (!active) return;                 // uniform (read long ago, so no wait here); loads in flight are dropped with the wavefront

    constexpr int DA = 8;                        // weight loads in flight per wavefront
    u32x4 a[DA];
    const bool defer = RB == 2 && NC == 1 && s.T > s.tl && 2 * (s.T - s.tl) <= s.tl;    // see the end of the round loop
    // fixed-order sum of a round's partial tiles over the wavefronts that shared each tile's columns
    auto sum_round = [&](int rnd) {
        const float *rr = red + (size_t)(rnd & (RB - 1)) * NWV * 256;
        for (int i = tid; i < s.tl * 256; i += NT) {
            const int l = i >> 8, e = i & 255, tt = rnd * s.tl + l, rit = e >> 4;
            if (tt < s.T && rit < s.rpt && tt * s.rpt + rit < R) {
                float sum = 0.f;
                for (int k = 0; k < s.ksplit; ++k) sum += rr[(size_t)(l * s.ksplit + k) * 256 + e];
                vals[(tt * s.rpt + rit) * KS_MAX_ROWS + (e & 15)] = sum;
            }
        }
    };
    for (int round = 0; round * s.tl < s.T; ++round) {   // T = 0 when this workgroup owns no rows
        const WaveTile w = wave_tile(s, K, round, tlane, kpart);
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
        // lane = (row of the tile, 8-column group); dead rows re-read the tile's last live row: their products land
        // in accumulator rows that are never stored
        const bf16_t *ap = op.W + w.base + (size_t)(kg * w.rows_t + min(r16, w.rows_t - 1)) * 8;
        if constexpr (!RING) {
            // few chunks: one loop nest per chunk, the weight stream drained at each boundary
            int cnt = chunk_count(0, w.have);
            const bool stage = round == 0 || NC > 1;     // a single chunk stays in LDS for every round
            // a batch: eight unconditional loads (a wavefront with fewer units re-reads its last one; one without units
            // reads the matrix's first bytes). No load of an earlier batch is in flight when one is issued.
            auto a_batch = [&](const bf16_t *p, int n) {
                const bf16_t *p0 = n > 0 ? p : op.W;
                const int last = max(n - 1, 0);
    #pragma unroll
                for (int j = 0; j < DA; ++j) a[j] = stream_load(p0 + (size_t)min(j, last) * w.unit);
            };
            if (stage && round > 0) bchunk_load(0, tid);
            a_batch(ap, cnt);
            if (round == 0) {
                // the row table is read after the next meeting at the earliest; its index arithmetic is pinned behind
                // the weight loads just issued (it is loop invariant and would otherwise be hoisted in front of them)
                GemmOp shape;
                shape.type = pinned_here(op.type); shape.N = pinned_here(op.N);
                shape.H = pinned_here(op.H); shape.Hkv = pinned_here(op.Hkv); shape.hd = pinned_here(op.hd);
                int n_first_unused;
                build_row_table<true>(shape, pinned_here(wg), rowidx, &n_first_unused);
            }
            if (stage) {
                stream_wait_pieces<DA, MFMA_BQ>(breg);
                bchunk_store(0, tid);
                __syncthreads();
            }
            int c = 0;
            do {                                     // NC >= 1
                if (c + 1 < NC) bchunk_load(c + 1, tid);
                const int bstride = (min(KC, K - c * KC) + 8) * 2;                  // bytes per staged row of this chunk
                const char *bsrc = bbuf + (c & 1) * BBUF + brow * bstride + kg * 16;
                auto unit_mfma = [&](int u, const u32x4 &a4) {
                    const int ls = step_of_unit(s, kpart, u);     // step within the chunk
                    const bf16x8 av = __builtin_bit_cast(bf16x8, a4);
    #pragma unroll
                    for (int p = 0; p < 3; ++p) {
                        const u32x4 bv = *reinterpret_cast<const u32x4 *>(bsrc + p * n_rows * bstride + ls * 64);
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bv), acc, 0, 0, 0);
                    }
                };
                int u0 = 0;
                // steady state: a unit's register is refilled the moment the unit has been used, and the wait before a
                // unit leaves the seven younger weight loads in flight (loads of the next activation chunk, issued
                // after the batch, only make that wait stricter). One way into the loop: see the draft GEMV.
                if (cnt >= 2 * DA) {
                    do {
    #pragma unroll
                        for (int j = 0; j < DA; ++j) {
                            stream_wait<DA - 1>(a[j]);
                            unit_mfma(u0 + j, a[j]);
                            a[j] = stream_load(ap + (size_t)(u0 + j + DA) * w.unit);
                        }
                        u0 += DA;
                    } while (u0 + 2 * DA <= cnt);
                }
                // tail: at most 15 units left, drained batch by batch; at least one drain, so that no load (of weights or
                // of the next activation chunk) is in flight afterwards
                do {
                    stream_drain8(a);
    #pragma unroll
                    for (int j = 0; j < DA; ++j)
                        if (u0 + j < cnt) unit_mfma(u0 + j, a[j]);
    #pragma unroll
                    for (int j = 0; j < DA; ++j)
                        if (u0 + DA + j < cnt) a[j] = stream_load(ap + (size_t)(u0 + DA + j) * w.unit);
                    u0 += DA;
                } while (u0 < cnt);        // a load was issued above only if this holds: every load is followed by a drain
                ap += (size_t)cnt * w.unit;
                if (c + 1 >= NC) break;                // nothing in flight here
                // next chunk's first weight loads go out before the workgroup meets
                ++c;
                cnt = chunk_count(c, w.have);
                a_batch(ap, cnt);
                stream_wait_pieces<DA, MFMA_BQ>(breg);     // long complete (drained above); orders the stores after it
                bchunk_store(c, tid);
                __syncthreads();
            } while (true);
            stream_drain8(a);      // nothing is in flight here (every way out of the loop passes a drain); costs nothing
        } else {
            // The wavefront's units of this round form ONE stream over all activation chunks: unit U belongs to chunk
            // U / CU (CU units per full chunk), and the weight loads roll on across chunk boundaries. Only the arithmetic
            // has to stop at a boundary until the next chunk is staged.
            const int total = w.cnt;
            const int CU = (KC >> 9) * s.g;
            const bool stage = round == 0 || NC > 1;     // a single chunk stays in LDS for every round
            // a batch: eight unconditional loads (a wavefront with fewer units re-reads its last one; one without units
            // reads the matrix's first bytes). No load of an earlier batch is in flight when one is issued.
            if (stage && round > 0) bchunk_load(0, tid);
            {
                const bf16_t *p0 = total > 0 ? ap : op.W;
                const int last = max(total - 1, 0);
    #pragma unroll
                for (int j = 0; j < DA; ++j) a[j] = stream_load(p0 + (size_t)min(j, last) * w.unit);
            }
            if (round == 0) {
                // the row table is read after the next meeting at the earliest; its index arithmetic is pinned behind
                // the weight loads just issued (it is loop invariant and would otherwise be hoisted in front of them)
                GemmOp shape;
                shape.type = pinned_here(op.type); shape.N = pinned_here(op.N);
                shape.H = pinned_here(op.H); shape.Hkv = pinned_here(op.Hkv); shape.hd = pinned_here(op.hd);
                int n_first_unused;
                build_row_table<true>(shape, pinned_here(wg), rowidx, &n_first_unused);
            }
            if (stage) {
                stream_wait_pieces<DA, MFMA_BQ>(breg);
                bchunk_store(0, tid);
                __syncthreads();
            }
            // state of the chunk being consumed
            int c = 0;                                   // its index
            int bnd = NC > 1 ? CU : 0x7fffffff;          // first unit of the next chunk
            int young = 0;                               // weight loads issued since the next chunk's pieces were requested
            int ls0 = 0;                                 // 32-column steps in front of the chunk
            int bstride = (min(KC, K) + 8) * 2;          // bytes per staged row of the chunk
            const char *bsrc = bbuf + brow * bstride + kg * 16;
            if (NC > 1) bchunk_load(1, tid);
            // A boundary: the next chunk's pieces (requested one chunk ago) go to LDS, the workgroup meets, the chunk
            // after that is requested. DRAINED = false: the weight stream stays in flight, so the wait for the pieces
            // leaves as many loads in flight as were issued after them (at most eight are ever outstanding).
            auto boundary = [&](auto drained) {
                // (the waits that depend on the count name no register: a wait that names the pieces in several
                // alternative branches would make the compiler join the alternatives with register copies, placed
                // in front of the wait; the one wait that names them comes last and is satisfied by then)
                if constexpr (decltype(drained)::value) {
                    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                } else {
                    switch (min(young, DA)) {
                        case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
                        case 1: asm volatile("s_waitcnt vmcnt(1)" ::: "memory"); break;
                        case 2: asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); break;
                        case 3: asm volatile("s_waitcnt vmcnt(3)" ::: "memory"); break;
                        case 4: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
                        case 5: asm volatile("s_waitcnt vmcnt(5)" ::: "memory"); break;
                        case 6: asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); break;
                        case 7: asm volatile("s_waitcnt vmcnt(7)" ::: "memory"); break;
                        default: break;
                    }
                }
                stream_wait_pieces<DA, MFMA_BQ>(breg);
                int t = tid;
                asm volatile("" : "+v"(t));
                ++c;
                bchunk_store(c, t);
                __syncthreads();
                if (c + 1 < NC) { bchunk_load(c + 1, t); young = 0; bnd += CU; }
                else bnd = 0x7fffffff;
                ls0 = c * (KC >> 5);
                bstride = (min(KC, K - c * KC) + 8) * 2;
                bsrc = bbuf + (c & 1) * BBUF + brow * bstride + kg * 16;
            };
            auto unit_mfma = [&](int u, const u32x4 &a4) {
                const int ls = step_of_unit(s, kpart, u) - ls0;     // step within the chunk
                const bf16x8 av = __builtin_bit_cast(bf16x8, a4);
    #pragma unroll
                for (int p = 0; p < 3; ++p) {
                    const u32x4 bv = *reinterpret_cast<const u32x4 *>(bsrc + p * n_rows * bstride + ls * 64);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, bv), acc, 0, 0, 0);
                }
            };
            int u0 = 0;
            // steady state: a unit's register is refilled the moment the unit has been used, and the wait before a
            // unit leaves the seven younger weight loads in flight (loads of activation pieces, issued in between,
            // only make that wait stricter). One way into the loop: see the draft GEMV.
            if (total >= 2 * DA) {
                do {
    #pragma unroll
                    for (int j = 0; j < DA; ++j) {
                        if (u0 + j == bnd) boundary(std::false_type{});
                        stream_wait<DA - 1>(a[j]);
                        unit_mfma(u0 + j, a[j]);
                        a[j] = stream_load(ap + (size_t)(u0 + j + DA) * w.unit);
                        ++young;
                    }
                    u0 += DA;
                } while (u0 + 2 * DA <= total);
            }
            // tail: at most 15 units left, drained batch by batch; at least one drain, so that no load is in flight
            // afterwards
            do {
                stream_drain8(a);
    #pragma unroll
                for (int j = 0; j < DA; ++j)
                    if (u0 + j < total) {
                        if (u0 + j == bnd) boundary(std::true_type{});
                        unit_mfma(u0 + j, a[j]);
                    }
    #pragma unroll
                for (int j = 0; j < DA; ++j)
                    if (u0 + DA + j < total) a[j] = stream_load(ap + (size_t)(u0 + DA + j) * w.unit);
                u0 += DA;
            } while (u0 < total);          // a load was issued above only if this holds: every load is followed by a drain
            // boundaries this wavefront's stream did not reach (it ended earlier, or the wavefront owns no unit): every
            // wavefront stages its pieces of every chunk and meets the others
            while (c + 1 < NC) {
                stream_drain8(a);
                boundary(std::true_type{});
            }
            stream_drain8(a);      // nothing is in flight here (every way out of the loops passes a drain); costs nothing
        }
        // partial tile of this wavefront -> LDS; lane holds D[row 4*kg + q][token r16]. The partials of
        // consecutive rounds alternate between two buffers, so one meeting per round is enough: a buffer is
        // written again only after every wavefront has passed the next round's meeting, i.e. finished summing it.
        // With two rounds over activations that stay staged (one chunk) every round has a buffer of its own and
        // nothing is restaged, so the wavefronts need not meet between the rounds: a wavefront that is done with its
        // first tile goes straight on to its second, and both rounds are summed after the loop. That pays where the
        // second round keeps at most half of the tile lanes busy (3 tiles on 2 lanes, 6 on 4: the wavefronts with a
        // second tile fill what would be a half-idle round; measured -0.7 % per verification pass on the 7B shapes)
        // and costs 0.3 % where it is nearly full (7 or 8 tiles on 4 lanes), so only the former do it.
        float *redr = red + (size_t)(round & (RB - 1)) * NWV * 256;
        {
            float *rp = redr + (size_t)wave * 256;
#pragma unroll
            for (int q = 0; q < 4; ++q) rp[(4 * kg + q) * 16 + r16] = acc[q];
        }
        if (!defer) {
            __syncthreads();    // also: every wavefront is done with the staging buffers of this round
            sum_round(round);
            if (RB == 1) __syncthreads();   // the one buffer is written again in the next round
        }
    }
    if (defer) {
        __syncthreads();
        sum_round(0);
        if (s.tl < s.T) sum_round(1);
    }
    // the norm's shares and the epilogue's two values were issued before the first weight batch and are long here
    // (every round ends drained); the wait only ties their registers to this point
    stream_wait_scalars<0>(sh, xpre, gpre);
    if (wave < KS_MAX_ROWS) {
        float share = 0.f;
#pragma unroll
        for (int j = 0; j < 4; ++j) share += sh[j];
        const float r = (op.ss_in && wave < n_rows) ? 1.0f / sqrtf(wave_sum(share) * op.inv_dim + op.eps) : 1.0f;
        if (lane == 0) rstd_s[wave] = r;
    }
    __syncthreads();
    gemm_epilogue<true>(op, ctl, wg, nwg, R, s.n_first, rowidx, vals, KS_MAX_ROWS, rstd_s,
                        op.type == OP_HEAD ? ctl->head_from : 0, n_rows, scratch, xpre, gpre);
}

// PREFILL only names the launch site (prompt chunks vs verification passes) so that a profile keeps the two apart
template <bool PREFILL, bool RING>
__global__ __launch_bounds__(NT, 1) void gemm_mfma_kernel(GemmOp op, const PassCtl *ctl) {
    extern __shared__ __align__(16) char lds[];
    gemm_mfma_device<RING>(op, ctl, blockIdx.x, gridDim.x, lds);
}

// final-RMSNorm hidden state of one row from the head's operands: gain (.) x times rstd
__global__ __launch_bounds__(NT) void hidden_from_image_kernel(const float *image, int kc, int n_rows, const float *ss, int n_ss,
                                                               int d, float eps, const PassCtl *ctl, float *out0, float *out1) {
    // image: the LM head's chunk images (chunk length kc, n_rows live rows as the host counts them)
    if (!ctl->active) return;
    __shared__ float rs;
    const int m = min(ctl->n_rows, n_rows) - 1;
    if (threadIdx.x < 64) {
        float s = 0.f;
        for (int i = threadIdx.x; i < n_ss; i += 64) s += ss[(size_t)m * n_ss + i];
        s = wave_sum(s);
        if (threadIdx.x == 0) rs = 1.0f / sqrtf(s / (float)d + eps);
    }
    __syncthreads();
    const float inv_kc = __builtin_amdgcn_rcpf((float)kc);
    for (int i = blockIdx.x * NT + threadIdx.x; i < d; i += gridDim.x * NT) {
        const float v = image[image_offset(m, i, d, kc, n_rows, inv_kc)] * rs;
        out0[i] = v;
        if (out1) out1[i] = v;
    }
}

// ------------------------------------------------------------------------------------------
// Embedding as the first producer: x = E[tok], gain (.) x and the shares of sum(x^2)
// ------------------------------------------------------------------------------------------
template <bool PLANES>
__global__ __launch_bounds__(NT) void embed_producer_kernel(GemmOp op, const PassCtl *ctl) {
    __shared__ float scratch[NWV];
    if (!ctl->active) return;
    // the image layout is the one the host computed for op.n_rows rows: never more rows than that
    const int n_rows = min(min(ctl->n_rows, KS_MAX_ROWS), PLANES ? op.n_rows : KS_MAX_ROWS);
    const float inv_kc = PLANES ? __builtin_amdgcn_rcpf((float)op.out_kc) : 0.f;
    const int wg = blockIdx.x;         // launched with KS_NWG workgroups (wg_share)
    const int r0 = wg_share(op.N, wg), r1 = wg_share(op.N, wg + 1);
    for (int m = 0; m < n_rows; ++m) {
        const bf16_t *row = op.embed + (size_t)ctl->tok[m] * op.N;
        float ssq = 0.f;
        for (int n = r0 + threadIdx.x; n < r1; n += NT) {
            float v = bf16_to_float(row[n]);
            op.x[(size_t)m * op.N + n] = v;
            store_act<PLANES>(op, m, n, op.N, op.gain_next[n] * v, inv_kc);
            ssq = fmaf(v, v, ssq);
        }
        float s = block_sum(ssq, scratch);
        if (threadIdx.x == 0) op.ss_out[(size_t)m * KS_NWG + wg] = s;
    }
}

// ------------------------------------------------------------------------------------------
// Split-KV attention over the contiguous bf16 cache. Work item = (kv head, ATT_CHUNK = 256-position
// chunk, group of ATT_PG (row, q-head) pairs). Wavefront w of the workgroup's 16 owns 16 positions of
// the chunk and keeps their K and V fragments in registers (lane = (position, 8-dim slice)); the
// sixteen wavefronts' (max, sum, weighted V) are merged in LDS and written as the chunk's partial.
// ------------------------------------------------------------------------------------------
struct AttnArgs {
    const float *q;          // [KS_MAX_ROWS][H*hd] rotated queries
    const bf16_t *kv_block;  // [2][Hkv][max_seq][hd]
    float *partial;          // [KS_MAX_ROWS*H][max_chunks][hd + ATT_PAD]
    int H, Hkv, hd, max_seq, max_chunks;
    int group;               // H / Hkv
    // combine
    float *act_out;          // fp32: draft [H*hd]; verify: chunk images
    int out_kc, n_rows;      // PLANES: act_out holds the O projection's chunk images: that GEMM's chunk length and the pass's
                             // row count as the host counts them
    int *arrivals;           // attn_partial_mfma_kernel: [pair tiles][Hkv] arrival counters (zero between launches) when the
                             // last workgroup of a group merges the chunks itself; nullptr: attn_combine_kernel follows
};

// ------------------------------------------------------------------------------------------
// Merging the chunks inside the attention launch. The workgroup that finishes the last chunk of a group of (row, head)
// pairs merges the group's chunks and hands the result to the O projection, so no merge launch follows. Nobody waits:
// every workgroup writes its partial through to memory (agent-scope stores), waits for the writes to be acknowledged
// and counts itself in; the one that draws the last number reads the group's partials back from memory (agent-scope
// loads: another compute die's L2 may hold older lines of the buffer) and runs the arithmetic of attn_combine_device,
// operation for operation, so a value does not depend on where it was merged. The counter is left at zero.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void store_agent(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void load2_agent(const float *p, float &a, float &b) {      // p 8-byte aligned
    const unsigned long long v = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    a = __uint_as_float((unsigned int)v); b = __uint_as_float((unsigned int)(v >> 32));
}

// Called by every thread of the workgroup after its partial's stores: true in the workgroup that arrives last of the
// group's n_expected (uniform). ticket: one int of LDS; the caller's next workgroup meeting orders its reuse.
__device__ __forceinline__ bool last_arrival(int *counter, int n_expected, int *ticket) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // this thread's partial stores have been acknowledged
    __syncthreads();
    if (threadIdx.x == 0) {
        const int t = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (t == n_expected - 1) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *ticket = t;
    }
    __syncthreads();
    return *ticket == n_expected - 1;
}

struct AttnArgs;
template <int HD, int CB>
__device__ __forceinline__ void merge_pairs_device(const AttnArgs &a, int kvh, int p_base, int n_p, int group, float inv_group,
                                                   int start, int tid, int nt);

template <int HD>
__device__ __forceinline__ void attn_partial_device(const AttnArgs &a, const PassCtl *ctl, int wg, int nwg, char *lds) {
    constexpr int LPP = HD / 8;        // lanes per position
    constexpr int PPS = 64 / LPP;      // positions per step
    constexpr int STEPS = 16 / PPS;    // steps per wavefront (16 positions)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ps = lane / LPP, dg = lane % LPP;
    const int n_rows = min(ctl->n_rows, KS_MAX_ROWS), start = ctl->start;
    const int group = a.group;                          // H / Hkv, from the host
    const float inv_group = __builtin_amdgcn_rcpf((float)group);
    const int P = n_rows * group;                       // (row, head-in-group) pairs per kv head
    const int n_pg = (P + ATT_PG - 1) / ATT_PG;
    const int n_chunks = (start + n_rows + ATT_CHUNK - 1) / ATT_CHUNK;
    const int n_items = a.Hkv * n_chunks * n_pg;
    float *qs = reinterpret_cast<float *>(lds);                         // [ATT_PG][HD]
    float *red = qs + ATT_PG * HD;                                      // [NWV][ATT_PG][HD + 2]
    int *ticket = reinterpret_cast<int *>(red + NWV * ATT_PG * (HD + 2));
    const float scale = 1.0f / sqrtf((float)HD);
    const size_t kv_head_stride = (size_t)a.max_seq * HD;

    for (int item = wg; item < n_items; item += nwg) {
        // item -> (kv head, chunk, pair group), pair group fastest (float-product divisions, see div_small)
        const int per_head = n_pg * n_chunks;
        const int kvh = div_small(item, per_head, __builtin_amdgcn_rcpf((float)per_head));
        const int in_head = item - kvh * per_head;
        const int chunk = div_small(in_head, n_pg, __builtin_amdgcn_rcpf((float)n_pg));
        const int pg = in_head - chunk * n_pg;
        const int p_base = pg * ATT_PG;
        const int n_p = min(ATT_PG, P - p_base);
        __syncthreads();   // previous item's LDS reads are done
        // this wavefront's 16 positions of K and V (issued before the queries are staged)
        const int pos0 = chunk * ATT_CHUNK + wave * 16;
        const bf16_t *kc = a.kv_block + (size_t)kvh * kv_head_stride;
        const bf16_t *vc = a.kv_block + ((size_t)a.Hkv + kvh) * kv_head_stride;
        u32x4 kf[STEPS], vf[STEPS];
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            // unconditional loads (a position past the end re-reads the last live one; its score is masked below):
            // a load under a divergent branch would be waited for on the spot, one round trip after the other
            const int pos = min(pos0 + s * PPS + ps, start + n_rows - 1);
            kf[s] = *reinterpret_cast<const u32x4 *>(kc + (size_t)pos * HD + dg * 8);
            vf[s] = *reinterpret_cast<const u32x4 *>(vc + (size_t)pos * HD + dg * 8);
        }
        for (int i = tid; i < n_p * HD; i += NT) {
            const int pl = i / HD, dim = i - pl * HD, p = p_base + pl;
            const int m = div_small(p, group, inv_group), h = kvh * group + (p - m * group);
            qs[pl * HD + dim] = a.q[(size_t)m * a.H * HD + h * HD + dim];
        }
        __syncthreads();
        for (int pl = 0; pl < n_p; ++pl) {
            const int p = p_base + pl;
            const int m = div_small(p, group, inv_group);
            const int len = start + m + 1;          // row m attends positions [0, len)
            const float *qp = qs + pl * HD + dg * 8;
            const float4 q0 = *reinterpret_cast<const float4 *>(qp), q1 = *reinterpret_cast<const float4 *>(qp + 4);
            float sc[STEPS];
            float mx = -INFINITY;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                float d = dot8(kf[s], q0, q1, 0.f);
#pragma unroll
                for (int off = 1; off < LPP; off <<= 1) d += __shfl_xor(d, off, 64);
                const int pos = pos0 + s * PPS + ps;
                sc[s] = (pos < len) ? d * scale : -INFINITY;
                mx = fmaxf(mx, sc[s]);
            }
#pragma unroll
            for (int off = LPP; off < 64; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
            float l = 0.f;
            float o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = 0.f;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const float e = (sc[s] > -INFINITY) ? expf(sc[s] - mx) : 0.f;
                l += e;
                o[0] = fmaf(e, bf_lo(vf[s].x), o[0]); o[1] = fmaf(e, bf_hi(vf[s].x), o[1]);
                o[2] = fmaf(e, bf_lo(vf[s].y), o[2]); o[3] = fmaf(e, bf_hi(vf[s].y), o[3]);
                o[4] = fmaf(e, bf_lo(vf[s].z), o[4]); o[5] = fmaf(e, bf_hi(vf[s].z), o[5]);
                o[6] = fmaf(e, bf_lo(vf[s].w), o[6]); o[7] = fmaf(e, bf_hi(vf[s].w), o[7]);
            }
#pragma unroll
            for (int off = LPP; off < 64; off <<= 1) {
                l += __shfl_xor(l, off, 64);
#pragma unroll
                for (int j = 0; j < 8; ++j) o[j] += __shfl_xor(o[j], off, 64);
            }
            // l counted every lane of a position LPP times over? no: each lane group of LPP lanes holds the same
            // score, and the xor-sum above runs over the position groups only, so l is the sum over positions.
            float *rp = red + ((size_t)wave * ATT_PG + pl) * (HD + 2);
            if (ps == 0) {
#pragma unroll
                for (int j = 0; j < 8; ++j) rp[dg * 8 + j] = o[j];
            }
            if (lane == 0) { rp[HD] = mx; rp[HD + 1] = l; }
        }
        __syncthreads();
        // merge the wavefronts' partials: thread (pl, dim)
        for (int i = tid; i < n_p * HD; i += NT) {
            const int pl = i / HD, dim = i - pl * HD, p = p_base + pl;
            const int m = div_small(p, group, inv_group), h = kvh * group + (p - m * group);
            float M = -INFINITY;
#pragma unroll
            for (int w = 0; w < NWV; ++w) M = fmaxf(M, red[((size_t)w * ATT_PG + pl) * (HD + 2) + HD]);
            float L = 0.f, O = 0.f;
#pragma unroll
            for (int w = 0; w < NWV; ++w) {
                const float *rp = red + ((size_t)w * ATT_PG + pl) * (HD + 2);
                const float f = (rp[HD] > -INFINITY) ? expf(rp[HD] - M) : 0.f;
                L = fmaf(rp[HD + 1], f, L);
                O = fmaf(rp[dim], f, O);
            }
            float *out = a.partial + (((size_t)m * a.H + h) * a.max_chunks + chunk) * (HD + ATT_PAD);
            if (a.arrivals) {
                store_agent(out + dim, O);
                if (dim == 0) { store_agent(out + HD, M); store_agent(out + HD + 1, L); }
            } else {
                out[dim] = O;
                if (dim == 0) { out[HD] = M; out[HD + 1] = L; }
            }
        }
        if (a.arrivals && last_arrival(a.arrivals + pg * a.Hkv + kvh, n_chunks, ticket))
            merge_pairs_device<HD, ATT_SELF_MERGE_CHUNKS>(a, kvh, p_base, n_p, group, inv_group, start, tid, NT);
    }
}

// The merge itself, by the nt threads of the calling workgroup: pairs [p_base, p_base + n_p) of kv head kvh, two
// neighbouring dimensions per thread and step (8-byte agent-scope loads), the partials of CB chunks fetched together.
template <int HD, int CB>
__device__ __forceinline__ void merge_pairs_device(const AttnArgs &a, int kvh, int p_base, int n_p, int group, float inv_group,
                                                   int start, int tid, int nt) {
    constexpr int PSTR = HD + ATT_PAD, H2 = HD / 2;
    const int qd = a.H * HD;
    const float inv_kc = __builtin_amdgcn_rcpf((float)a.out_kc);
    GemmOp st{};   // only the fields store_act uses
    st.act_out = a.act_out; st.out_kc = a.out_kc; st.n_rows = a.n_rows;
    for (int i = tid; i < n_p * H2; i += nt) {
        const int pl = i / H2, dim = (i - pl * H2) * 2, p = p_base + pl;
        const int m = div_small(p, group, inv_group), h = kvh * group + (p - m * group);
        const int nc_m = (start + m + 1 + ATT_CHUNK - 1) / ATT_CHUNK;   // chunks row m can see
        const float *pp = a.partial + ((size_t)m * a.H + h) * a.max_chunks * PSTR;
        float mv0[CB], lv0[CB], oa0[CB], ob0[CB];
#pragma unroll
        for (int k = 0; k < CB; ++k) {
            const float *cp = pp + (size_t)min(k, nc_m - 1) * PSTR;
            load2_agent(cp + HD, mv0[k], lv0[k]);
            load2_agent(cp + dim, oa0[k], ob0[k]);
        }
        float M = -INFINITY;
#pragma unroll
        for (int k = 0; k < CB; ++k) M = fmaxf(M, mv0[k]);
        for (int base = CB; base < nc_m; base += CB) {
#pragma unroll
            for (int k = 0; k < CB; ++k) {
                float mk, lk;
                load2_agent(pp + (size_t)min(base + k, nc_m - 1) * PSTR + HD, mk, lk);
                M = fmaxf(M, mk);
            }
        }
        float L = 0.f, Oa = 0.f, Ob = 0.f;
#pragma unroll
        for (int k = 0; k < CB; ++k) {
            const float f = (k < nc_m && mv0[k] > -INFINITY) ? expf(mv0[k] - M) : 0.f;
            L = fmaf(lv0[k], f, L);
            Oa = fmaf(oa0[k], f, Oa);
            Ob = fmaf(ob0[k], f, Ob);
        }
        for (int base = CB; base < nc_m; base += CB) {
            float mv[CB], lv[CB], oa[CB], ob[CB];
#pragma unroll
            for (int k = 0; k < CB; ++k) {
                const float *cp = pp + (size_t)min(base + k, nc_m - 1) * PSTR;
                load2_agent(cp + HD, mv[k], lv[k]);
                load2_agent(cp + dim, oa[k], ob[k]);
            }
#pragma unroll
            for (int k = 0; k < CB; ++k) {
                const float f = (base + k < nc_m && mv[k] > -INFINITY) ? expf(mv[k] - M) : 0.f;
                L = fmaf(lv[k], f, L);
                Oa = fmaf(oa[k], f, Oa);
                Ob = fmaf(ob[k], f, Ob);
            }
        }
        store_act<true>(st, m, h * HD + dim, qd, Oa / L, inv_kc);
        store_act<true>(st, m, h * HD + dim + 1, qd, Ob / L, inv_kc);
    }
}

__host__ __device__ inline size_t attn_lds_bytes(int hd) { return (size_t)(ATT_PG * hd + NWV * ATT_PG * (hd + 2) + 4) * 4; }

template <int HD>
__global__ __launch_bounds__(NT) void attn_partial_kernel(AttnArgs a, const PassCtl *ctl) {
    extern __shared__ __align__(16) char lds[];
    if (!ctl->active) return;
    attn_partial_device<HD>(a, ctl, blockIdx.x, gridDim.x, lds);
}

// merge the chunks of every (row, head) in chunk order and hand the result to the O projection
template <bool PLANES>
__device__ __forceinline__ void attn_combine_device(const AttnArgs &a, const PassCtl *ctl, int wg, int nwg) {
    // (the plane layout is the one the host computed for a.n_rows rows: never more rows than that)
    const int n_rows = min(min(ctl->n_rows, KS_MAX_ROWS), PLANES ? a.n_rows : KS_MAX_ROWS), start = ctl->start;
    const int hd = a.hd, qd = a.H * hd;
    const int total = n_rows * qd;
    GemmOp st{};   // only the fields store_act uses
    st.act_out = a.act_out; st.out_kc = a.out_kc; st.n_rows = a.n_rows;
    const float inv_kc = PLANES ? __builtin_amdgcn_rcpf((float)a.out_kc) : 0.f;
    const float inv_qd = __builtin_amdgcn_rcpf((float)qd);
    const int hd_shift = 31 - __builtin_clz(hd);                           // head_dim is 64 or 128
    constexpr int CB = 8;                                                  // chunks whose partials are fetched together
    for (int i = wg * NT + threadIdx.x; i < total; i += nwg * NT) {
        const int m = div_small(i, qd, inv_qd), c = i - m * qd, h = c >> hd_shift, dim = c & (hd - 1);
        const int n_chunks = (start + m + 1 + ATT_CHUNK - 1) / ATT_CHUNK;   // chunks row m can see
        const int pstr = hd + ATT_PAD;
        const float *pp = a.partial + ((size_t)m * a.H + h) * a.max_chunks * pstr;
        // Two passes in chunk order (largest maximum, then the weighted sums) over partials fetched CB chunks at a
        // time with unconditional loads before any of them is used: a load per loop iteration would cost one memory
        // round trip per chunk. The first CB chunks (all of them up to 2048 positions) are fetched once, for both
        // passes. Entries past the last chunk re-read it and enter the sums with weight zero, which leaves the sums
        // bit for bit as if they had been skipped.
        float mv0[CB], lv0[CB], ov0[CB];
#pragma unroll
        for (int k = 0; k < CB; ++k) {
            const float *cp = pp + (size_t)min(k, n_chunks - 1) * pstr;
            mv0[k] = cp[hd]; lv0[k] = cp[hd + 1]; ov0[k] = cp[dim];
        }
        float M = -INFINITY;
#pragma unroll
        for (int k = 0; k < CB; ++k) M = fmaxf(M, mv0[k]);
        for (int base = CB; base < n_chunks; base += CB) {
            float mv[CB];
#pragma unroll
            for (int k = 0; k < CB; ++k) mv[k] = pp[(size_t)min(base + k, n_chunks - 1) * pstr + hd];
#pragma unroll
            for (int k = 0; k < CB; ++k) M = fmaxf(M, mv[k]);
        }
        float L = 0.f, O = 0.f;
#pragma unroll
        for (int k = 0; k < CB; ++k) {
            const float f = (k < n_chunks && mv0[k] > -INFINITY) ? expf(mv0[k] - M) : 0.f;
            L = fmaf(lv0[k], f, L);
            O = fmaf(ov0[k], f, O);
        }
        for (int base = CB; base < n_chunks; base += CB) {
            float mv[CB], lv[CB], ov[CB];
#pragma unroll
            for (int k = 0; k < CB; ++k) {
                const float *cp = pp + (size_t)min(base + k, n_chunks - 1) * pstr;
                mv[k] = cp[hd]; lv[k] = cp[hd + 1]; ov[k] = cp[dim];
            }
#pragma unroll
            for (int k = 0; k < CB; ++k) {
                const float f = (base + k < n_chunks && mv[k] > -INFINITY) ? expf(mv[k] - M) : 0.f;
                L = fmaf(lv[k], f, L);
                O = fmaf(ov[k], f, O);
            }
        }
        store_act<PLANES>(st, m, c, qd, O / L, inv_kc);
    }
}

template <bool PLANES>
__global__ __launch_bounds__(NT) void attn_combine_kernel(AttnArgs a, const PassCtl *ctl) {
    if (!ctl->active) return;
    attn_combine_device<PLANES>(a, ctl, blockIdx.x, gridDim.x);
}

// ------------------------------------------------------------------------------------------
// LM-head final step: merge the workgroups' (max, arg-max, sum-exp) per row in workgroup order
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(NT) void head_final_kernel(const HeadPartial *parts, int n_parts, const PassCtl *ctl,
                                                        HeadResult *res) {
    if (!ctl->active) return;
    __shared__ float sv[NWV];
    __shared__ int si[NWV];
    __shared__ float ss[NWV];
    const int m = blockIdx.x;
    if (m >= ctl->n_rows || m < ctl->head_from) return;
    const HeadPartial *pp = parts + (size_t)m * n_parts;
    float bv = -INFINITY; int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < n_parts; i += NT) {
        HeadPartial hp = pp[i];
        if (hp.idx != 0x7fffffff && better(hp.maxv, hp.idx, bv, bi)) { bv = hp.maxv; bi = hp.idx; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        float ov = __shfl_xor(bv, off, 64); int oi = __shfl_xor(bi, off, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sv[wave] = bv; si[wave] = bi; }
    __syncthreads();
    bv = sv[0]; bi = si[0];
    for (int w = 1; w < NWV; ++w) if (better(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
    float s = 0.f;
    for (int i = threadIdx.x; i < n_parts; i += NT) {
        HeadPartial hp = pp[i];
        if (hp.idx != 0x7fffffff) s += hp.sumexp * expf(hp.maxv - bv);
    }
    s = wave_sum(s);
    if (lane == 0) ss[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float tot = 0.f;
        for (int w = 0; w < NWV; ++w) tot += ss[w];
        res->tok[m] = bi;
        res->prob[m] = 1.0f / tot;
    }
}

}  // namespace ks
