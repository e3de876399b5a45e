// Prompt prefill for the tuned bf16 path (gfx950): the full model over hundreds to thousands of rows.
//
// Unlike a decode pass this is bound by the matrix cores, so it has kernels of its own. They read the
// SAME stream-order weights as the decode kernels (a unit = <= 16 rows x 32 columns is one MFMA A
// operand) and keep the same arithmetic: activations stay fp32-exact as three bf16 planes, so an
// output takes three MFMAs per 32 columns and the products are exact in the fp32 accumulator.
//
// Activations of all rows live in "fragment order": [plane][32-column step][16-row tile][lane][8],
// lane = 16*kg + r holding row r of the tile and columns 8*kg..8*kg+7 of the step, i.e. the MFMA B
// operand of v_mfma_f32_16x16x32_bf16 as stored, so staging a tile is a linear copy.
//
// prefill_gemm_kernel: a workgroup owns up to 16 weight tiles (G consecutive row groups of the decode
// layout, T tile slots each) and 4*TBW token tiles; per 32-column step it stages the 16 weight units
// and the 3 x 4*TBW token fragments through LDS (double buffered, one meeting per step); its 8
// wavefronts form a 2 x 4 grid, each holding 8 x TBW accumulator tiles. Epilogues are the decode
// ones (RoPE + KV write, residual + next norm's operands, SwiGLU) applied to 16 rows at a time.
#pragma once
#include "kernels_bf16.h"

namespace ks {

constexpr int PF_NT = 512;             // threads per workgroup of the prefill GEMM (8 wavefronts)
constexpr int PF_SLOTS = 16;           // weight tiles per workgroup
constexpr int PF_LR = PF_SLOTS * 16;   // local rows (slot, row in tile)
constexpr int PF_VLD = PF_LR + 1;      // leading dimension of the epilogue's staging array

struct PfArgs {
    GemmOp op;              // type, W, N, K, x, gain_next, q_out, kv_block, cos_t, sin_t, H, Hkv, hd, max_seq
    const bf16_t *frag_in;  // [3][K/32][TT][512] fragment order
    bf16_t *frag_out;       // same layout over the output features (OP_RESID / OP_SWIGLU)
    const float *rstd;      // [n_tok] rsqrt(mean(x^2) + eps) of the input rows; nullptr: input is not normalised
    float *ss_out;          // OP_RESID: [gridDim.x][TT*16] this workgroup's share of sum(x^2) per row
    int TT;                 // token tiles the fragment buffers are laid out for
    int n_tok;              // live rows (a multiple of 16)
    int G, T;               // row groups per workgroup, tile slots per row group (G*T <= PF_SLOTS)
};

__device__ __forceinline__ size_t frag_off(int KS, int TT, int pl, int ks, int tt) {
    return (((size_t)pl * KS + ks) * TT + tt) * 512;
}

// the three bf16 planes of v at feature n of row (tt, m), fragment order
__device__ __forceinline__ void store_frag(bf16_t *frag, int KS, int TT, int tt, int m, int n, float v) {
    const unsigned int u = __float_as_uint(v);
    const float hi = __uint_as_float(u & 0xffff0000u);
    const float r1 = v - hi;
    const float mid = __uint_as_float(__float_as_uint(r1) & 0xffff0000u);
    const float lo = r1 - mid;
    const size_t in_tile = (size_t)((((n & 31) >> 3) * 16 + m) * 8 + (n & 7));
    frag[frag_off(KS, TT, 0, n >> 5, tt) + in_tile] = (bf16_t)(u >> 16);
    frag[frag_off(KS, TT, 1, n >> 5, tt) + in_tile] = (bf16_t)(__float_as_uint(mid) >> 16);
    frag[frag_off(KS, TT, 2, n >> 5, tt) + in_tile] = (bf16_t)(__float_as_uint(lo) >> 16);
}

// Row-group tables of one workgroup (LDS)
struct PfTables {
    int grp_R[PF_SLOTS], grp_nfirst[PF_SLOTS], grp_rpt[PF_SLOTS];
    int rowidx[PF_LR];          // [G][16*T] global row of local row lr of group gi
};

// Epilogue for the 16 rows of token tile tt: vals[m*PF_VLD + slot*16 + row_in_tile] holds the finished dot products.
// Thread (m = tid / 32, jj = tid % 32) walks the local rows jj, jj+32, ... of every row group of the workgroup.
__device__ __forceinline__ void pf_epilogue(const PfArgs &a, const PfTables *tb, const float *vals, int tt, int n_groups) {
    const GemmOp &op = a.op;
    const int tid = threadIdx.x, m = tid >> 5, jj = tid & 31;
    const int tok = tt * 16 + m;
    const float rs = a.rstd ? a.rstd[tok] : 1.0f;
    const float *vrow = vals + (size_t)m * PF_VLD;
    float sq = 0.f;
    for (int gi = 0; gi < n_groups; ++gi) {
        const int R = tb->grp_R[gi], nf = tb->grp_nfirst[gi], rpt = tb->grp_rpt[gi];
        const int *rowidx = tb->rowidx + gi * 16 * a.T;
        const int slot0 = gi * a.T;
        auto col = [&](int lr) { const int t = lr / rpt; return (slot0 + t) * 16 + (lr - t * rpt); };
        if (op.type == OP_RESID) {
            for (int lr = jj; lr < R; lr += 32) {
                const int n = rowidx[lr];
                const size_t xi = (size_t)tok * op.N + n;
                const float xn = op.x[xi] + vrow[col(lr)];
                op.x[xi] = xn;
                store_frag(a.frag_out, op.N >> 5, a.TT, tt, m, n, op.gain_next[n] * xn);
                sq = fmaf(xn, xn, sq);
            }
        } else if (op.type == OP_SWIGLU) {
            for (int t = jj; t < nf; t += 32) {
                const int n = rowidx[t];
                const float g = vrow[col(t)] * rs, u = vrow[col(t + nf)] * rs;
                store_frag(a.frag_out, op.N >> 5, a.TT, tt, m, n, (g / (1.0f + expf(-g))) * u);
            }
        } else {   // OP_QKV
            const int half = op.hd >> 1, qd = op.H * op.hd, np = nf;
            bf16_t *kc = op.kv_block;
            bf16_t *vc = op.kv_block + (size_t)op.Hkv * op.max_seq * op.hd;
            const int pos = tok;                                   // the prompt starts at position 0
            for (int t = jj; t < R - np; t += 32) {
                const bool is_pair = t < np;
                const int lr = is_pair ? t : t + np;
                const int n = rowidx[lr];
                if (is_pair) {
                    const int head = n / op.hd, i = n - head * op.hd;
                    const float c = op.cos_t[(size_t)pos * half + i], s = op.sin_t[(size_t)pos * half + i];
                    const float x0 = vrow[col(lr)] * rs, x1 = vrow[col(lr + np)] * rs;
                    const float ra = x0 * c - x1 * s, rb = x1 * c + x0 * s;
                    if (head < op.H) {
                        op.q_out[(size_t)tok * qd + n] = ra;
                        op.q_out[(size_t)tok * qd + n + half] = rb;
                    } else {
                        const size_t base = ((size_t)(head - op.H) * op.max_seq + pos) * op.hd + i;
                        kc[base] = float_to_bf16_rne(ra);
                        kc[base + half] = float_to_bf16_rne(rb);
                    }
                } else {
                    const int vr = n - (op.H + op.Hkv) * op.hd;
                    const int head = vr / op.hd, i = vr - head * op.hd;
                    vc[((size_t)head * op.max_seq + pos) * op.hd + i] = float_to_bf16_rne(vrow[col(lr)] * rs);
                }
            }
        }
    }
    if (op.type == OP_RESID) {
        // this workgroup's share of sum(x^2) of row tok: the 32 threads of the row sit in one wavefront
#pragma unroll
        for (int off = 1; off < 32; off <<= 1) sq += __shfl_xor(sq, off, 64);
        if (jj == 0) a.ss_out[(size_t)blockIdx.x * a.TT * 16 + tok] = sq;
    }
}

template <int TBW>
__global__ __launch_bounds__(PF_NT, 1) void prefill_gemm_kernel(PfArgs a) {
    extern __shared__ __align__(16) char lds[];
    constexpr int TB = 4 * TBW;                       // token tiles of the workgroup
    constexpr int NB = 3 * TB * 64 / PF_NT;           // 16-byte pieces of token fragments per thread and step
    constexpr int A_BYTES = PF_SLOTS * 1024, B_BYTES = 3 * TB * 1024;
    char *abuf = lds;                                 // [2][A_BYTES]
    char *bbuf = lds + 2 * A_BYTES;                   // [2][B_BYTES]
    PfTables *tb = reinterpret_cast<PfTables *>(lds + 2 * A_BYTES + 2 * B_BYTES);
    __shared__ size_t slot_base[PF_SLOTS];            // element offset of the slot's tile in the packed matrix
    __shared__ int slot_rows[PF_SLOTS], slot_g[PF_SLOTS], slot_gshift[PF_SLOTS];

    const GemmOp &op = a.op;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wa = wave >> 2, wb = wave & 3, kg = lane >> 4, r16 = lane & 15;
    const int K = op.K, KS = K >> 5, nfull = KS >> 4, rem = KS & 15;
    const int tt0 = blockIdx.y * TB;
    const int TTL = a.n_tok >> 4;                     // live token tiles

    // row groups of this workgroup and their tile slots
    int n_groups = 0;
    if (tid < PF_SLOTS) { slot_rows[tid] = 0; slot_base[tid] = 0; slot_g[tid] = 1; slot_gshift[tid] = 0; }
    __syncthreads();
    for (int gi = 0; gi < a.G; ++gi) {
        const int wgid = blockIdx.x * a.G + gi;
        if (wgid >= KS_NWG) break;
        const WgSplit s = make_split(op, wgid, KS_NWG, tb->rowidx + gi * 16 * a.T);
        if (tid == 0) { tb->grp_R[gi] = s.R; tb->grp_nfirst[gi] = s.n_first; tb->grp_rpt[gi] = s.rpt > 0 ? s.rpt : 1; }
        if (tid < s.T) {
            const int slot = gi * a.T + tid;
            slot_rows[slot] = min(s.rpt, s.R - tid * s.rpt);
            slot_base[slot] = s.wg_base + (size_t)(tid * s.rpt) * K;
            slot_g[slot] = s.g; slot_gshift[slot] = s.gshift;
        }
        n_groups = gi + 1;
    }
    __syncthreads();
    // empty slots borrow slot 0's geometry and data: their products land in accumulators that are never stored
    if (tid < PF_SLOTS && slot_rows[tid] == 0) {
        slot_rows[tid] = max(slot_rows[0], 1); slot_base[tid] = slot_base[0]; slot_g[tid] = slot_g[0]; slot_gshift[tid] = slot_gshift[0];
    }
    __syncthreads();

    // what this thread stages per step: two pieces of weight units, NB pieces of token fragments (kept as element
    // offsets from the kernel's own pointers, so that the loads stay global loads)
    size_t a_off[2]; int a_unit[2], a_g[2], a_gshift[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int i = tid + q * PF_NT, slot = i >> 6, piece = i & 63, rows = slot_rows[slot];
        a_off[q] = slot_base[slot] + (size_t)min(piece, rows * 4 - 1) * 8;
        a_unit[q] = rows * 32; a_g[q] = slot_g[slot]; a_gshift[q] = slot_gshift[slot];
    }
    size_t b_off[NB];
#pragma unroll
    for (int q = 0; q < NB; ++q) {
        const int i = tid + q * PF_NT, pl = i / (TB * 64), ttl = (i >> 6) % TB, ln = i & 63;
        b_off[q] = frag_off(KS, a.TT, pl, 0, min(tt0 + ttl, a.TT - 1)) + ln * 8;
    }
    const size_t b_step = (size_t)a.TT * 512;          // elements between consecutive steps of one plane
    const bf16_t *__restrict__ Wg = op.W;
    const bf16_t *__restrict__ Fg = a.frag_in;
    u32x4 ra[2], rb[NB];
    auto stage_load = [&](int st) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int w16 = st & 15, kpart = w16 >> a_gshift[q], u = (st >> 4) * a_g[q] + (w16 & (a_g[q] - 1));
            const int before = nfull * a_g[q] * kpart + min(rem, kpart * a_g[q]);
            ra[q] = *reinterpret_cast<const u32x4 *>(Wg + a_off[q] + (size_t)(before + u) * a_unit[q]);
        }
#pragma unroll
        for (int q = 0; q < NB; ++q) rb[q] = *reinterpret_cast<const u32x4 *>(Fg + b_off[q] + (size_t)st * b_step);
        __builtin_amdgcn_sched_barrier(0);             // the loads stay at the top of the step, ahead of the MFMAs that hide them
    };
    auto stage_store = [&](int buf) {
#pragma unroll
        for (int q = 0; q < 2; ++q) *reinterpret_cast<u32x4 *>(abuf + buf * A_BYTES + (tid + q * PF_NT) * 16) = ra[q];
#pragma unroll
        for (int q = 0; q < NB; ++q) *reinterpret_cast<u32x4 *>(bbuf + buf * B_BYTES + (tid + q * PF_NT) * 16) = rb[q];
    };

    // this wavefront's operand addresses inside a staged step
    int aoff[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int slot = wa * 8 + i, rows = slot_rows[slot];
        aoff[i] = slot * 1024 + (kg * rows + min(r16, rows - 1)) * 16;
    }
    const int boff = (wb * TBW) * 1024 + lane * 16;

    f32x4 acc[8][TBW];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < TBW; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    stage_load(0);
    stage_store(0);
    __syncthreads();
    for (int st = 0; st < KS; ++st) {
        const int buf = st & 1;
        stage_load(min(st + 1, KS - 1));               // the last step re-reads itself: harmless, keeps the loads unconditional
        bf16x8 av[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) av[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(abuf + buf * A_BYTES + aoff[i]));
#pragma unroll
        for (int j = 0; j < TBW; ++j) {
            bf16x8 bv[3];
#pragma unroll
            for (int p = 0; p < 3; ++p)
                bv[p] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(bbuf + buf * B_BYTES + p * TB * 1024 + boff + j * 1024));
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int p = 0; p < 3; ++p) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[i], bv[p], acc[i][j], 0, 0, 0);
        }
        stage_store(buf ^ 1);
        __syncthreads();
    }

    // epilogue, one token tile at a time through a staging array that reuses the operand buffers
    float *vals = reinterpret_cast<float *>(lds);      // [16][PF_VLD]
#pragma unroll
    for (int j = 0; j < TBW; ++j) {
        for (int wq = 0; wq < 4; ++wq) {
            const int tt = tt0 + wq * TBW + j;
            if (tt >= TTL) continue;                   // uniform over the workgroup
            __syncthreads();
            if (wb == wq) {
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int q = 0; q < 4; ++q) vals[r16 * PF_VLD + (wa * 8 + i) * 16 + 4 * kg + q] = acc[i][j][q];
            }
            __syncthreads();
            pf_epilogue(a, tb, vals, tt, n_groups);
        }
    }
}

__host__ __device__ inline size_t pf_gemm_lds_bytes(int tbw) {
    return (size_t)2 * PF_SLOTS * 1024 + (size_t)2 * 3 * 4 * tbw * 1024 + sizeof(PfTables);
}

// ------------------------------------------------------------------------------------------
// Embedding of the prompt rows: x = E[tok], the first norm's operands gain (.) x in fragment order
// and the row's rsqrt(mean(x^2) + eps). One workgroup per row.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(PF_NT) void prefill_embed_kernel(const int32_t *toks, const bf16_t *embed, const float *gain, int d,
                                                              float eps, int TT, float *x, bf16_t *frag, float *rstd) {
    __shared__ float part[PF_NT / 64];
    const int tok = blockIdx.x, tt = tok >> 4, m = tok & 15;
    const bf16_t *row = embed + (size_t)toks[tok] * d;
    float sq = 0.f;
    for (int n = threadIdx.x; n < d; n += PF_NT) {
        const float v = bf16_to_float(row[n]);
        x[(size_t)tok * d + n] = v;
        store_frag(frag, d >> 5, TT, tt, m, n, gain[n] * v);
        sq = fmaf(v, v, sq);
    }
    sq = wave_sum(sq);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = sq;
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int w = 0; w < PF_NT / 64; ++w) s += part[w];
        rstd[tok] = 1.0f / sqrtf(s / (float)d + eps);
    }
}

// rsqrt(mean(x^2) + eps) per row from the producers' shares, summed in share order
__global__ void prefill_rstd_kernel(const float *ss, int n_shares, int stride, int n_tok, float inv_dim, float eps, float *rstd) {
    const int tok = blockIdx.x * blockDim.x + threadIdx.x;
    if (tok >= n_tok) return;
    float s = 0.f;
    for (int i = 0; i < n_shares; ++i) s += ss[(size_t)i * stride + tok];
    rstd[tok] = 1.0f / sqrtf(s * inv_dim + eps);
}

// ------------------------------------------------------------------------------------------
// Causal attention of the prompt rows over the bf16 cache, on the matrix cores. A workgroup = one query
// head x four consecutive 16-row tiles (one wavefront each); keys and values go through LDS in chunks
// of 64 positions shared by the four wavefronts (values transposed on the way in, so that both are
// MFMA B operands as stored). Per chunk a wavefront computes S = Q K^T (Q exact as three bf16 planes),
// the running softmax in fp32 on the vector ALUs, and O += P V with P exact as three bf16 planes;
// P changes from accumulator layout to operand layout through a wavefront-private LDS tile.
// ------------------------------------------------------------------------------------------
struct PfAttn {
    const float *q;          // [n_tok][H*hd] rotated queries
    const bf16_t *kv_block;  // [2][Hkv][max_seq][hd]
    bf16_t *frag_out;        // attention output in fragment order over H*hd features
    int H, Hkv, max_seq, TT, n_tok;
};

// eight fp32 values -> the three bf16 planes of an MFMA operand fragment (exact: hi + mid + lo = value)
__device__ __forceinline__ void split_planes8(const float *v, bf16x8 *out3) {
    unsigned int w[3][4];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const unsigned int u = __float_as_uint(v[e]);
        const float hi = __uint_as_float(u & 0xffff0000u);
        const float r1 = v[e] - hi;
        const unsigned int um = __float_as_uint(r1);
        const float mid = __uint_as_float(um & 0xffff0000u);
        const unsigned int ul = __float_as_uint(r1 - mid);
        const unsigned int h16 = u >> 16, m16 = um >> 16, l16 = ul >> 16;
        if (e & 1) { w[0][e >> 1] |= h16 << 16; w[1][e >> 1] |= m16 << 16; w[2][e >> 1] |= l16 << 16; }
        else { w[0][e >> 1] = h16; w[1][e >> 1] = m16; w[2][e >> 1] = l16; }
    }
#pragma unroll
    for (int p = 0; p < 3; ++p) out3[p] = __builtin_bit_cast(bf16x8, u32x4{w[p][0], w[p][1], w[p][2], w[p][3]});
}

template <int HD>
__global__ __launch_bounds__(256) void prefill_attn_kernel(PfAttn a) {
    constexpr int CH = 64, LPP = HD / 8, QS = HD / 32, DT = HD / 16;
    constexpr int KSTR = HD * 2 + 16;      // bytes per staged key row (+16: the 16 rows of an operand read spread over the banks)
    constexpr int VSTR = CH * 2 + 16;      // bytes per staged (transposed) value row
    constexpr int PSTR = CH + 4;           // floats per row of the P tile
    constexpr int PIECES = CH * LPP, PQ = PIECES / 256;
    __shared__ __align__(16) char kl[CH * KSTR];
    __shared__ __align__(16) char vl[HD * VSTR];
    __shared__ __align__(16) float pb[4][16 * PSTR];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = lane >> 4, r16 = lane & 15;
    const int n_rt = a.n_tok >> 4, n_b = (n_rt + 3) >> 2;
    const int b = n_b - 1 - (int)(blockIdx.x / a.H);          // long blocks first
    const int h = blockIdx.x % a.H, kvh = h / (a.H / a.Hkv);
    const int rt = min(b * 4 + wave, n_rt - 1);               // a wavefront past the last tile repeats it and stores nothing
    const bool live = b * 4 + wave < n_rt;
    const int n_chunks = b + 1;                               // positions 0 .. 64b+63 cover every row of the block
    const int last_pos = a.n_tok - 1, qd = a.H * HD;
    const float scale = 1.0f / sqrtf((float)HD);
    const bf16_t *kg_ = a.kv_block + (size_t)kvh * a.max_seq * HD;
    const bf16_t *vg_ = a.kv_block + ((size_t)a.Hkv + kvh) * a.max_seq * HD;

    // the wavefront's 16 query rows as operand fragments: lane (kg, i) holds row i, dims 32*ks + 8*kg .. +7
    bf16x8 qa[QS][3];
    {
        const float *qp = a.q + (size_t)(rt * 16 + r16) * qd + h * HD + kg * 8;
#pragma unroll
        for (int ks = 0; ks < QS; ++ks) {
            float v[8];
            const float4 v0 = *reinterpret_cast<const float4 *>(qp + ks * 32), v1 = *reinterpret_cast<const float4 *>(qp + ks * 32 + 4);
            v[0] = v0.x; v[1] = v0.y; v[2] = v0.z; v[3] = v0.w; v[4] = v1.x; v[5] = v1.y; v[6] = v1.z; v[7] = v1.w;
            split_planes8(v, qa[ks]);
        }
    }

    u32x4 kr[PQ], vr[PQ];
    auto chunk_load = [&](int c) {
#pragma unroll
        for (int q = 0; q < PQ; ++q) {
            const int i = tid + q * 256;
            const int pos = min(c * CH + i / LPP, last_pos);
            kr[q] = *reinterpret_cast<const u32x4 *>(kg_ + (size_t)pos * HD + (i % LPP) * 8);
            vr[q] = *reinterpret_cast<const u32x4 *>(vg_ + (size_t)pos * HD + (i % LPP) * 8);
        }
    };
    auto chunk_store = [&]() {
#pragma unroll
        for (int q = 0; q < PQ; ++q) {
            const int i = tid + q * 256, pos = i / LPP, d0 = (i % LPP) * 8;
            *reinterpret_cast<u32x4 *>(kl + pos * KSTR + d0 * 2) = kr[q];
            const unsigned int w[4] = {vr[q].x, vr[q].y, vr[q].z, vr[q].w};
#pragma unroll
            for (int e = 0; e < 8; ++e)        // transpose: value of dim d0+e at position pos
                *reinterpret_cast<bf16_t *>(vl + (d0 + e) * VSTR + pos * 2) = (bf16_t)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffffu));
        }
    };

    float mrun[4], lsum[4];
    f32x4 o[DT];
#pragma unroll
    for (int q = 0; q < 4; ++q) { mrun[q] = -INFINITY; lsum[q] = 0.f; }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float *pw = pb[wave];
    const int row_tok = rt * 16 + 4 * kg;                     // position of accumulator row q of this lane: row_tok + q

    chunk_load(0);
    for (int c = 0; c < n_chunks; ++c) {
        __syncthreads();                                      // the previous chunk has been consumed by every wavefront
        chunk_store();
        __syncthreads();
        chunk_load(min(c + 1, n_chunks - 1));
        // S = Q K^T for the chunk's four position tiles: lane (kg, j) holds rows 4*kg..4*kg+3 at position 16*pt + j
        float sc[4][4];
#pragma unroll
        for (int pt = 0; pt < 4; ++pt) {
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < QS; ++ks) {
                const bf16x8 kb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(kl + (pt * 16 + r16) * KSTR + (ks * 32 + kg * 8) * 2));
#pragma unroll
                for (int p = 0; p < 3; ++p) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[ks][p], kb, acc, 0, 0, 0);
            }
            const int pos = c * CH + pt * 16 + r16;
#pragma unroll
            for (int q = 0; q < 4; ++q) sc[pt][q] = (pos <= row_tok + q) ? acc[q] * scale : -INFINITY;
        }
        // running softmax per row (rows are replicated over the 16 lanes of a kg group)
        float f[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float cm = fmaxf(fmaxf(sc[0][q], sc[1][q]), fmaxf(sc[2][q], sc[3][q]));
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) cm = fmaxf(cm, __shfl_xor(cm, off, 64));
            const float mnew = fmaxf(mrun[q], cm);            // finite: position 0 is visible to every row
            f[q] = (mrun[q] > -INFINITY) ? expf(mrun[q] - mnew) : 0.f;
            mrun[q] = mnew;
            float ps = 0.f;
#pragma unroll
            for (int pt = 0; pt < 4; ++pt) {
                const float e = (sc[pt][q] > -INFINITY) ? expf(sc[pt][q] - mnew) : 0.f;
                pw[(4 * kg + q) * PSTR + pt * 16 + r16] = e;
                ps += e;
            }
            lsum[q] = lsum[q] * f[q] + ps;
        }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int q = 0; q < 4; ++q) o[dt][q] *= f[q];
        // O += P V: P back from LDS in operand layout (lane (kg, i): row i, positions 32*ks2 + 8*kg .. +7)
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
            float pv[8];
            const float4 p0 = *reinterpret_cast<const float4 *>(pw + r16 * PSTR + ks2 * 32 + kg * 8);
            const float4 p1 = *reinterpret_cast<const float4 *>(pw + r16 * PSTR + ks2 * 32 + kg * 8 + 4);
            pv[0] = p0.x; pv[1] = p0.y; pv[2] = p0.z; pv[3] = p0.w; pv[4] = p1.x; pv[5] = p1.y; pv[6] = p1.z; pv[7] = p1.w;
            bf16x8 pa[3];
            split_planes8(pv, pa);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const bf16x8 vb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(vl + (dt * 16 + r16) * VSTR + (ks2 * 32 + kg * 8) * 2));
#pragma unroll
                for (int p = 0; p < 3; ++p) o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa[p], vb, o[dt], 0, 0, 0);
            }
        }
    }
    // row sums over the 16 lanes of a kg group, then the rows' outputs in fragment order
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) lsum[q] += __shfl_xor(lsum[q], off, 64);
    }
    if (live) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float inv = 1.0f / lsum[q];
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                store_frag(a.frag_out, qd >> 5, a.TT, rt, 4 * kg + q, h * HD + dt * 16 + r16, o[dt][q] * inv);
        }
    }
}

}  // namespace ks
