// Split-KV attention of a verification pass on the matrix cores.
//
// The vector-ALU kernel (attn_partial_kernel, kernels_bf16.h) walks the (row, head) pairs of a work item one
// after the other; a verification pass of k+1 rows has (k+1) x group pairs per kv head, and at 9 rows the walk
// costs three times the draft step's attention. Here a work item is (kv head, 256-position chunk, tile of up to
// 16 pairs) and its four wavefronts take 64 positions each:
//   S = Q K^T  scores of the 16 pairs against the wavefront's 64 positions: Q as three exact bf16 planes (A
//              operand, from the rotated fp32 queries), K straight from the cache (a lane's 16-byte load of one
//              position IS its B-operand fragment),
//   softmax    partial over the 64 positions in fp32 on the vector ALUs (max, exp, sum),
//   O = P V    P back through a wavefront-private LDS tile into operand layout as three exact planes, V transposed
//              through LDS on the way in,
// then the four wavefronts' (max, sum, O) are merged in LDS and written as the chunk's partial, in the format
// attn_combine_kernel reads. A pair's result does not depend on which other pairs share its tile, nor on the
// number of rows in the pass.
#pragma once
#include "kernels_prefill.h"

namespace ks {

constexpr int VA_NT = 256;                 // threads per workgroup (four wavefronts)
constexpr int VA_WP = ATT_CHUNK / 4;       // positions per wavefront
static_assert(VA_WP == 64, "four position tiles of 16 per wavefront");

template <int HD>
__host__ __device__ constexpr size_t vattn_lds_bytes() {
    // per wavefront: transposed values [HD][64 positions + 8] bf16 and the P tile [16][64 + 4] fp32; the merge
    // buffer [4][16][HD + 2] fp32 reuses the value area once every wavefront is done with it
    return (size_t)4 * HD * (VA_WP * 2 + 16) + (size_t)4 * 16 * (VA_WP + 4) * 4;
}

template <int HD>
__global__ __launch_bounds__(VA_NT) void attn_partial_mfma_kernel(AttnArgs a, const PassCtl *ctl) {
    constexpr int QS = HD / 32, DT = HD / 16, LPP = HD / 8;
    constexpr int VSTR = VA_WP * 2 + 16;       // bytes per transposed value row (one dimension, 64 positions)
    constexpr int PSTR = VA_WP + 4;            // floats per row of the P tile
    constexpr int VQ = VA_WP * LPP / 64;       // 16-byte value pieces per lane
    static_assert(4 * 16 * (HD + 2) * 4 <= 4 * HD * VSTR, "the merge buffer fits the value area");
    extern __shared__ __align__(16) char lds[];
    if (!ctl->active) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = lane >> 4, r16 = lane & 15;
    char *vt = lds + (size_t)wave * HD * VSTR;                                            // this wavefront's V^T
    float *pw = reinterpret_cast<float *>(lds + (size_t)4 * HD * VSTR) + wave * 16 * PSTR; // this wavefront's P tile
    float *mb = reinterpret_cast<float *>(lds);                                           // [4][16][HD + 2] merge buffer

    const int n_rows = min(ctl->n_rows, KS_MAX_ROWS), start = ctl->start;
    const int group = a.group;
    const float inv_group = __builtin_amdgcn_rcpf((float)group);
    const int P = n_rows * group;                       // (row, head-in-group) pairs per kv head
    const int n_pt = (P + 15) >> 4;
    const int n_chunks = (start + n_rows + ATT_CHUNK - 1) / ATT_CHUNK;
    const int n_items = a.Hkv * n_chunks * n_pt;
    const int last_pos = start + n_rows - 1, qd = a.H * HD;
    const float scale = 1.0f / sqrtf((float)HD);
    const size_t kv_head_stride = (size_t)a.max_seq * HD;

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        // item -> (kv head, chunk, pair tile), pair tile fastest
        const int per_head = n_pt * n_chunks;
        const int kvh = div_small(item, per_head, __builtin_amdgcn_rcpf((float)per_head));
        const int in_head = item - kvh * per_head;
        const int chunk = div_small(in_head, n_pt, __builtin_amdgcn_rcpf((float)n_pt));
        const int pt = in_head - chunk * n_pt;
        const int wp0 = chunk * ATT_CHUNK + wave * VA_WP;          // this wavefront's first position
        const bf16_t *kc = a.kv_block + (size_t)kvh * kv_head_stride;
        const bf16_t *vc = a.kv_block + ((size_t)a.Hkv + kvh) * kv_head_stride;

        // keys: position tile t4, lane (kg, j) loads position 16*t4 + j, dims 32*ks + 8*kg .. +7 = its B fragment.
        // Positions past the last live one re-read it; their scores are masked below.
        u32x4 kf[4][QS];
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
            const int pos = min(wp0 + t4 * 16 + r16, last_pos);
#pragma unroll
            for (int ks = 0; ks < QS; ++ks)
                kf[t4][ks] = *reinterpret_cast<const u32x4 *>(kc + (size_t)pos * HD + ks * 32 + kg * 8);
        }
        // values: 64 positions x HD as 16-byte pieces, piece i = (position i / LPP, dims 8 * (i % LPP) .. +7)
        u32x4 vr[VQ];
#pragma unroll
        for (int q = 0; q < VQ; ++q) {
            const int i = lane + 64 * q;
            const int pos = min(wp0 + i / LPP, last_pos);
            vr[q] = *reinterpret_cast<const u32x4 *>(vc + (size_t)pos * HD + (i % LPP) * 8);
        }
        // queries of the tile's pairs as operand fragments: lane (kg, i) holds pair 16*pt + i, dims 32*ks + 8*kg .. +7
        // (a lane past the last pair repeats it; its accumulator row is never stored)
        bf16x8 qa[QS][3];
        {
            const int p = min(pt * 16 + r16, P - 1);
            const int m = div_small(p, group, inv_group), h = kvh * group + (p - m * group);
            const float *qp = a.q + (size_t)m * qd + h * HD + kg * 8;
#pragma unroll
            for (int ks = 0; ks < QS; ++ks) {
                float v[8];
                const float4 v0 = *reinterpret_cast<const float4 *>(qp + ks * 32), v1 = *reinterpret_cast<const float4 *>(qp + ks * 32 + 4);
                v[0] = v0.x; v[1] = v0.y; v[2] = v0.z; v[3] = v0.w; v[4] = v1.x; v[5] = v1.y; v[6] = v1.z; v[7] = v1.w;
                split_planes8(v, qa[ks]);
            }
        }
        __syncthreads();        // the previous item's merge buffer (which overlays the value areas) has been read
        // values into LDS, transposed: row = dimension, column = position within the wavefront's 64
#pragma unroll
        for (int q = 0; q < VQ; ++q) {
            const int i = lane + 64 * q, pos = i / LPP, d0 = (i % LPP) * 8;
            const unsigned int w[4] = {vr[q].x, vr[q].y, vr[q].z, vr[q].w};
#pragma unroll
            for (int e = 0; e < 8; ++e)
                *reinterpret_cast<bf16_t *>(vt + (d0 + e) * VSTR + pos * 2) = (bf16_t)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffffu));
        }
        // accumulator row q of this lane is pair 16*pt + 4*kg + q; it sees positions <= start + its token row
        int vis[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int p = min(pt * 16 + 4 * kg + q, P - 1);
            vis[q] = start + div_small(p, group, inv_group);
        }
        // S = Q K^T: lane (kg, j) holds pairs 4*kg .. 4*kg+3 at position 16*t4 + j
        float sc[4][4];
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
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
        // softmax over the wavefront's 64 positions, per pair (a pair's values sit in the 16 lanes of a kg group)
        float mx[4], ls[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float cm = fmaxf(fmaxf(sc[0][q], sc[1][q]), fmaxf(sc[2][q], sc[3][q]));
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) cm = fmaxf(cm, __shfl_xor(cm, off, 64));
            mx[q] = cm;                                       // -inf when none of the 64 positions is visible
            float ps = 0.f;
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                const float e = (sc[t4][q] > -INFINITY) ? expf(sc[t4][q] - cm) : 0.f;
                pw[(4 * kg + q) * PSTR + t4 * 16 + r16] = e;
                ps += e;
            }
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) ps += __shfl_xor(ps, off, 64);
            ls[q] = ps;
        }
        // O = P V: P back from LDS in operand layout (lane (kg, i): pair i, positions 32*ks2 + 8*kg .. +7)
        f32x4 o[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
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
                const bf16x8 vb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(vt + (dt * 16 + r16) * VSTR + (ks2 * 32 + kg * 8) * 2));
#pragma unroll
                for (int p = 0; p < 3; ++p) o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa[p], vb, o[dt], 0, 0, 0);
            }
        }
        __syncthreads();        // every wavefront is done with its value area: the merge buffer may overlay them
        {
            float *mw = mb + (size_t)wave * 16 * (HD + 2);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float *row = mw + (4 * kg + q) * (HD + 2);
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) row[dt * 16 + r16] = o[dt][q];
                if (r16 == 0) { row[HD] = mx[q]; row[HD + 1] = ls[q]; }
            }
        }
        __syncthreads();
        // merge the four wavefronts in position order: thread (pair, dim)
        for (int i = tid; i < 16 * HD; i += VA_NT) {
            const int pl = i / HD, dim = i - pl * HD, p = pt * 16 + pl;
            if (p < P) {
                const int m = div_small(p, group, inv_group), h = kvh * group + (p - m * group);
                float M = -INFINITY;
#pragma unroll
                for (int w = 0; w < 4; ++w) M = fmaxf(M, mb[((size_t)w * 16 + pl) * (HD + 2) + HD]);
                float L = 0.f, O = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float *rp = mb + ((size_t)w * 16 + pl) * (HD + 2);
                    const float f = (rp[HD] > -INFINITY) ? expf(rp[HD] - M) : 0.f;
                    L = fmaf(rp[HD + 1], f, L);
                    O = fmaf(rp[dim], f, O);
                }
                float *out = a.partial + (((size_t)m * a.H + h) * a.max_chunks + chunk) * (HD + 2);
                out[dim] = O;
                if (dim == 0) { out[HD] = M; out[HD + 1] = L; }
            }
        }
    }
}

}  // namespace ks
