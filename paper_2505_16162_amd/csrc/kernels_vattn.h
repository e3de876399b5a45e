// Split-KV attention of a verification pass on the matrix cores.
//
// The vector-ALU kernel (attn_partial_kernel, kernels_bf16.h) walks the (row, head) pairs of a work item one
// after the other; a verification pass of k+1 rows has (k+1) x group pairs per kv head, and at 9 rows the walk
// costs three times the draft step's attention. Here a work item is (kv head, 256-position chunk, tile of up to
// 16 pairs) and its four wavefronts take 64 positions each (eight wavefronts of 32 positions measure the same:
// the kernel is bound by its chain of memory round trips, not by instruction issue):
//   S = Q K^T  scores of the 16 pairs against the wavefront's 64 positions: Q as three exact bf16 planes (A
//              operand, from the rotated fp32 queries), K straight from the cache (a lane's 16-byte load of one
//              position IS its B-operand fragment),
//   softmax    partial over the 64 positions in fp32 on the vector ALUs (max, exp, sum),
//   O = P V    P back through a wavefront-private LDS tile into operand layout as three exact planes; V needs no
//              transposition through memory: a lane loads DT consecutive dimensions of its 8 positions and regroups
//              them in registers (one byte permute per operand register), so that matrix instruction t produces
//              dimensions {DT * n + t} in its 16 columns n,
// then the four wavefronts' (max, sum, O) are merged in LDS and written as the chunk's partial, in the format
// attn_combine_kernel reads. A pair's result does not depend on which other pairs share its tile, nor on the
// number of rows in the pass.
#pragma once
#include "kernels_prefill.h"

namespace ks {

constexpr int VA_NW = 4;                   // wavefronts per workgroup
constexpr int VA_NT = 64 * VA_NW;          // threads per workgroup
constexpr int VA_WP = ATT_CHUNK / VA_NW;   // positions per wavefront
constexpr int VA_TP = VA_WP / 16;          // position tiles of the score product
constexpr int VA_KS = VA_WP / 32;          // summation steps of the value product
static_assert(VA_WP % 32 == 0 && VA_WP * VA_NW == ATT_CHUNK, "whole summation steps, whole chunk");

typedef unsigned int va_u32x2 __attribute__((ext_vector_type(2)));

template <int HD>
__host__ __device__ constexpr size_t vattn_lds_bytes() {
    // per wavefront: the P tile [16][positions + 4] fp32 and its share [16][HD + 4] fp32 of the merge buffer
    return (size_t)VA_NW * 16 * (VA_WP + 4) * 4 + (size_t)VA_NW * 16 * (HD + 4) * 4;
}

// LONG = false: contexts of up to eight chunks. LONG = true: compiled for three workgroups per compute unit (168
// registers per lane), so that a launch with more work items than 2 x 256 workgroups runs in one round instead of
// two, and with a merge that fetches the partials of up to 24 chunks together.
template <int HD, bool LONG>
__global__ __launch_bounds__(VA_NT, LONG ? 3 : 1) void attn_partial_mfma_kernel(AttnArgs a, const PassCtl *ctl) {
    constexpr int QS = HD / 32, DT = HD / 16;
    constexpr int PSTR = VA_WP + 4;            // floats per row of the P tile
    constexpr int MSTR = HD + 4;               // floats per row of the merge buffer (16-byte aligned rows)
    static_assert(DT == 8 || DT == 4, "a lane loads 16 or 8 bytes of a value row");
    extern __shared__ __align__(16) char lds[];
    __shared__ int tickets[1];
    if (!ctl->active) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = lane >> 4, r16 = lane & 15;
    float *pw = reinterpret_cast<float *>(lds) + wave * 16 * PSTR;                        // this wavefront's P tile
    float *mb = reinterpret_cast<float *>(lds + (size_t)VA_NW * 16 * PSTR * 4);           // [VA_NW][16][MSTR] merge buffer

    const int n_rows = min(ctl->n_rows, KS_MAX_ROWS), start = ctl->start;
    const int group = a.group;
    const float inv_group = __builtin_amdgcn_rcpf((float)group);
    const int P = n_rows * group;                       // (row, head-in-group) pairs per kv head
    const int n_pt = (P + 15) >> 4;
    const int n_chunks = (start + n_rows + ATT_CHUNK - 1) / ATT_CHUNK;
    // Work items in launch order: pair tile slowest, and a tile's (kv head, chunk) items padded to a multiple of 8,
    // so that the tiles of one (kv head, chunk) run on workgroups 8k apart, i.e. (workgroups are dealt round-robin
    // over the 8 XCDs) behind the same L2, which then fetches that chunk's keys and values from HBM once
    const int per_tile = a.Hkv * n_chunks, tile_stride = (per_tile + 7) & ~7;
    const int n_items = n_pt * tile_stride;
    const int last_pos = start + n_rows - 1, qd = a.H * HD;
    const float scale = 1.0f / sqrtf((float)HD);
    const size_t kv_head_stride = (size_t)a.max_seq * HD;

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int pt = div_small(item, tile_stride, __builtin_amdgcn_rcpf((float)tile_stride));
        const int in_tile = item - pt * tile_stride;
        if (in_tile >= per_tile) continue;              // padding (the whole workgroup skips it together)
        const int kvh = div_small(in_tile, n_chunks, __builtin_amdgcn_rcpf((float)n_chunks));
        const int chunk = in_tile - kvh * n_chunks;
        const int wp0 = chunk * ATT_CHUNK + wave * VA_WP;          // this wavefront's first position
        const bf16_t *kc = a.kv_block + (size_t)kvh * kv_head_stride;
        const bf16_t *vc = a.kv_block + ((size_t)a.Hkv + kvh) * kv_head_stride;

        // queries of the tile's pairs as operand fragments: lane (kg, i) holds pair 16*pt + i, dims 32*ks + 8*kg .. +7
        // (a lane past the last pair repeats it; its accumulator row is never stored)
        f32x4 qf[QS][2];
        {
            const int p = min(pt * 16 + r16, P - 1);
            const int m = div_small(p, group, inv_group), h = kvh * group + (p - m * group);
            const float *qp = a.q + (size_t)m * qd + h * HD + kg * 8;
#pragma unroll
            for (int ks = 0; ks < QS; ++ks) {
                qf[ks][0] = *reinterpret_cast<const f32x4 *>(qp + ks * 32);
                qf[ks][1] = *reinterpret_cast<const f32x4 *>(qp + ks * 32 + 4);
            }
        }
        // keys: position tile t4, lane (kg, j) loads position 16*t4 + j, dims 32*ks + 8*kg .. +7 = its B fragment.
        // Positions past the last live one re-read it; their scores are masked below.
        u32x4 kf[VA_TP][QS];
#pragma unroll
        for (int t4 = 0; t4 < VA_TP; ++t4) {
            const int pos = min(wp0 + t4 * 16 + r16, last_pos);
#pragma unroll
            for (int ks = 0; ks < QS; ++ks)
                kf[t4][ks] = *reinterpret_cast<const u32x4 *>(kc + (size_t)pos * HD + ks * 32 + kg * 8);
        }
        // values: lane (kg, n) loads dims DT*n .. DT*n + DT-1 of positions 32*ks2 + 8*kg + j, j = 0..7 (the eight
        // summation slots it owns in step ks2); vw[ks2][j][w] holds dims DT*n + 2w, +1 of slot j
        unsigned int vw[VA_KS][8][DT / 2];
#pragma unroll
        for (int ks2 = 0; ks2 < VA_KS; ++ks2)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int pos = min(wp0 + ks2 * 32 + kg * 8 + j, last_pos);
                const bf16_t *vp = vc + (size_t)pos * HD + r16 * DT;
                if constexpr (DT == 8) {
                    const u32x4 t = *reinterpret_cast<const u32x4 *>(vp);
                    vw[ks2][j][0] = t.x; vw[ks2][j][1] = t.y; vw[ks2][j][2] = t.z; vw[ks2][j][3] = t.w;
                } else {
                    const va_u32x2 t = *reinterpret_cast<const va_u32x2 *>(vp);
                    vw[ks2][j][0] = t.x; vw[ks2][j][1] = t.y;
                }
            }
        bf16x8 qa[QS][3];
#pragma unroll
        for (int ks = 0; ks < QS; ++ks) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[e] = qf[ks][0][e]; v[4 + e] = qf[ks][1][e]; }
            split_planes8(v, qa[ks]);
        }
        // accumulator row q of this lane is pair 16*pt + 4*kg + q; it sees positions <= start + its token row
        int vis[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int p = min(pt * 16 + 4 * kg + q, P - 1);
            vis[q] = start + div_small(p, group, inv_group);
        }
        // S = Q K^T: lane (kg, j) holds pairs 4*kg .. 4*kg+3 at position 16*t4 + j
        float sc[VA_TP][4];
#pragma unroll
        for (int t4 = 0; t4 < VA_TP; ++t4) {
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < QS; ++ks) {
                const bf16x8 kb = __builtin_bit_cast(bf16x8, kf[t4][ks]);
#pragma unroll
                for (int p = 0; p < 3; ++p) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[ks][p], kb, acc, 0, 0, 0);
            }
            const int pos = wp0 + t4 * 16 + r16;
#pragma unroll
            for (int q = 0; q < 4; ++q) sc[t4][q] = (pos <= vis[q]) ? acc[q] * scale : -INFINITY;
        }
        // softmax over the wavefront's positions, per pair (a pair's values sit in the 16 lanes of a kg group)
        float mx[4], ls[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float cm = sc[0][q];
#pragma unroll
            for (int t4 = 1; t4 < VA_TP; ++t4) cm = fmaxf(cm, sc[t4][q]);
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) cm = fmaxf(cm, __shfl_xor(cm, off, 64));
            mx[q] = cm;                                       // -inf when none of the positions is visible
            float ps = 0.f;
#pragma unroll
            for (int t4 = 0; t4 < VA_TP; ++t4) {
                const float e = (sc[t4][q] > -INFINITY) ? expf(sc[t4][q] - cm) : 0.f;
                pw[(4 * kg + q) * PSTR + t4 * 16 + r16] = e;
                ps += e;
            }
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) ps += __shfl_xor(ps, off, 64);
            ls[q] = ps;
        }
        // (the P tile is private to this wavefront: its stores above and its loads below are ordered by the in-order
        // LDS pipeline of one wavefront; the barrier keeps the compiler from moving a load above a store of another
        // lane's element and costs no instruction)
        __builtin_amdgcn_wave_barrier();
        // O = P V: P back from LDS in operand layout (lane (kg, i): pair i, positions 32*ks2 + 8*kg .. +7); the value
        // operand of instruction t takes dimension DT*n + t of the lane's eight positions: the low (t even) or high
        // (t odd) halves of word t/2 of two neighbouring slots make one operand register
        f32x4 o[DT];
#pragma unroll
        for (int t = 0; t < DT; ++t) o[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks2 = 0; ks2 < VA_KS; ++ks2) {
            float pv[8];
            const float4 p0 = *reinterpret_cast<const float4 *>(pw + r16 * PSTR + ks2 * 32 + kg * 8);
            const float4 p1 = *reinterpret_cast<const float4 *>(pw + r16 * PSTR + ks2 * 32 + kg * 8 + 4);
            pv[0] = p0.x; pv[1] = p0.y; pv[2] = p0.z; pv[3] = p0.w; pv[4] = p1.x; pv[5] = p1.y; pv[6] = p1.z; pv[7] = p1.w;
            bf16x8 pa[3];
            split_planes8(pv, pa);
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                u32x4 vb;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    // bytes 0-3 of the selector's source are the second operand, 4-7 the first
                    vb[jj] = __builtin_amdgcn_perm(vw[ks2][2 * jj + 1][t >> 1], vw[ks2][2 * jj][t >> 1],
                                                   (t & 1) ? 0x07060302u : 0x05040100u);
                }
                const bf16x8 vbf = __builtin_bit_cast(bf16x8, vb);
#pragma unroll
                for (int p = 0; p < 3; ++p) o[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa[p], vbf, o[t], 0, 0, 0);
            }
        }
        __syncthreads();        // the previous item's merge buffer has been read by every wavefront
        {
            float *mw = mb + (size_t)wave * 16 * MSTR;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float *row = mw + (4 * kg + q) * MSTR;
#pragma unroll
                for (int t4 = 0; t4 < DT / 4; ++t4)
                    *reinterpret_cast<float4 *>(row + r16 * DT + 4 * t4) =
                        make_float4(o[4 * t4][q], o[4 * t4 + 1][q], o[4 * t4 + 2][q], o[4 * t4 + 3][q]);
                if (r16 == 0) { row[HD] = mx[q]; row[HD + 1] = ls[q]; }
            }
        }
        __syncthreads();
        // merge the wavefronts in position order: thread (pair, dim)
        const int n_p = min(16, P - pt * 16);
        const bool last_merges = a.arrivals != nullptr;       // uniform: see below
        for (int i = tid; i < n_p * HD; i += VA_NT) {
            const int pl = i / HD, dim = i - pl * HD, p = pt * 16 + pl;
            const int m = div_small(p, group, inv_group), h = kvh * group + (p - m * group);
            float M = -INFINITY;
#pragma unroll
            for (int w = 0; w < VA_NW; ++w) M = fmaxf(M, mb[((size_t)w * 16 + pl) * MSTR + HD]);
            float L = 0.f, O = 0.f;
#pragma unroll
            for (int w = 0; w < VA_NW; ++w) {
                const float *rp = mb + ((size_t)w * 16 + pl) * MSTR;
                const float f = (rp[HD] > -INFINITY) ? expf(rp[HD] - M) : 0.f;
                L = fmaf(rp[HD + 1], f, L);
                O = fmaf(rp[dim], f, O);
            }
            float *out = a.partial + (((size_t)m * a.H + h) * a.max_chunks + chunk) * (HD + ATT_PAD);
            if (last_merges) {
                store_agent(out + dim, O);
                if (dim == 0) { store_agent(out + HD, M); store_agent(out + HD + 1, L); }
            } else {
                out[dim] = O;
                if (dim == 0) { out[HD] = M; out[HD + 1] = L; }
            }
        }
        if (!last_merges) continue;
        if (!last_arrival(a.arrivals + pt * a.Hkv + kvh, n_chunks, tickets)) continue;
        merge_pairs_device<HD, LONG ? ATT_SELF_MERGE_CHUNKS_MFMA : ATT_SELF_MERGE_CHUNKS>(a, kvh, pt * 16, n_p, group, inv_group, start, tid, VA_NT);
    }
}

}  // namespace ks
