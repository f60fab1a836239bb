// Partial attention of one item on the vector ALUs, for GQA groups G = Hq/Hkv up to 8.
// A second, selectable implementation (FD_OPT_PATH = 1) and a cross-check: the MFMA kernel
// is the default at every group size, because its K/V stream needs no registers and the
// HBM bound hides the padding of its matrix tiles.
//
// Steps a2-a6 of the hot path (paper Section 4.2.1: partial attention of the
// query against a KV shard, with online-softmax statistics; Algorithm 4 Part 1).
//
// Data flow per wave (64 lanes = 4 rows of 16 lanes):
//   * one 128-bit load instruction covers 4 consecutive keys: row r of the wave
//     reads key (4*i + r), lane c of the row reads dims 8c..8c+7 of it, so a
//     wave always touches whole, consecutive 256-byte K/V rows;
//   * QK^T: 4 packed-bf16 dot2 per (head, key) per lane, then a 16-lane DPP
//     row sum; scale*log2(e) is applied to the fp32 sum;
//   * each 16-lane row keeps its OWN running max / sum / accumulator over the
//     keys it owns (no cross-row traffic in the loop); the 16 row states of the
//     workgroup are merged once per item (shuffles inside a wave, LDS across
//     waves);
//   * K of the next 32-key tile is in flight while this tile's softmax and PV run,
//     V of the next tile while the next scores run.
#pragma once

#include "fd_device.hpp"

namespace fd {

constexpr int kValuTileKeys = 32;   // keys per wave tile (8 loads x 4 rows)
constexpr int kValuLoads = kValuTileKeys / 4;

// Loads keys kb + 4*i + r (i = 0..7) of K or of V.  MASKED: rows at or past j1
// re-read row j1-1 (always a live row); their scores are forced to -inf later.
template <bool MASKED>
__device__ __forceinline__ void valu_load_rows(uint4 (&dst)[kValuLoads], const uint4* base, int kb, int j1, int r, int c)
{
#pragma unroll
    for (int i = 0; i < kValuLoads; ++i) {
        int key = kb + 4 * i + r;
        if (MASKED) key = key < j1 ? key : j1 - 1;
        dst[i] = load_stream(base + (size_t)key * kRowU4 + c);
    }
}

template <int G>
struct ValuState {
    float m[G];
    float l[G];
    float acc[G][8];
};

// a3: s[g][i] = scale*log2(e) * <q_g, K[kb + 4i + r]> for the 8 keys of this row
template <int G, bool MASKED>
__device__ __forceinline__ void valu_scores(const uint4 (&kt)[kValuLoads], const uint32_t (&qr)[G][4],
                                            float (&s)[G][kValuLoads], float scale_log2, int kb, int j1, int r)
{
#pragma unroll
    for (int i = 0; i < kValuLoads; ++i) {
        const uint4 kk = kt[i];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float a = dot2_bf16(kk.x, qr[g][0], 0.f);
            a = dot2_bf16(kk.y, qr[g][1], a);
            a = dot2_bf16(kk.z, qr[g][2], a);
            a = dot2_bf16(kk.w, qr[g][3], a);
            a = row16_sum(a) * scale_log2;
            if (MASKED) a = (kb + 4 * i + r) < j1 ? a : -INFINITY;
            s[g][i] = a;
        }
    }
}

// a4: online softmax in base 2.  The running max is raised and the accumulators
// rescaled only when some row of the wave needs it; s becomes p = 2^(s - m).
template <int G>
__device__ __forceinline__ void valu_softmax(float (&s)[G][kValuLoads], ValuState<G>& st)
{
    float mnew[G];
    bool raise = false;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float tm = s[g][0];
#pragma unroll
        for (int i = 1; i < kValuLoads; ++i) tm = fmaxf(tm, s[g][i]);
        mnew[g] = fmaxf(st.m[g], tm);
        raise |= mnew[g] > st.m[g];
    }
    if (__any(raise)) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float alpha = fast_exp2(st.m[g] - mnew[g]);
            st.m[g] = mnew[g];
            st.l[g] *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) st.acc[g][e] *= alpha;
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int i = 0; i < kValuLoads; ++i) {
            s[g][i] = fast_exp2(s[g][i] - st.m[g]);
            st.l[g] += s[g][i];
        }
    }
}

// a5: acc[g][e] += p[g][key] * V[key][8c + e]
template <int G>
__device__ __forceinline__ void valu_pv(const uint4 (&vt)[kValuLoads], const float (&s)[G][kValuLoads],
                                        ValuState<G>& st)
{
#pragma unroll
    for (int i = 0; i < kValuLoads; ++i) {
        const uint4 vv = vt[i];
        const float v0 = bf16_lo(vv.x), v1 = bf16_hi(vv.x), v2 = bf16_lo(vv.y), v3 = bf16_hi(vv.y);
        const float v4 = bf16_lo(vv.z), v5 = bf16_hi(vv.z), v6 = bf16_lo(vv.w), v7 = bf16_hi(vv.w);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float pw = s[g][i];
            st.acc[g][0] = fmaf(pw, v0, st.acc[g][0]);
            st.acc[g][1] = fmaf(pw, v1, st.acc[g][1]);
            st.acc[g][2] = fmaf(pw, v2, st.acc[g][2]);
            st.acc[g][3] = fmaf(pw, v3, st.acc[g][3]);
            st.acc[g][4] = fmaf(pw, v4, st.acc[g][4]);
            st.acc[g][5] = fmaf(pw, v5, st.acc[g][5]);
            st.acc[g][6] = fmaf(pw, v6, st.acc[g][6]);
            st.acc[g][7] = fmaf(pw, v7, st.acc[g][7]);
        }
    }
}

// Attends keys [j0, j1) (j0 < j1) of tile (b, kvh) for its G query heads and
// writes the normalised result to dst_o[G][D] and (if non-null) the log-sum-exp
// times lse_mul to dst_lse[G].  SHARED: the destination is a partial that another
// workgroup may read within this launch (coherent stores).  Leaves LDS free for
// reuse on return.
template <int G, bool SHARED>
__device__ inline void valu_item(const Params& p, int b, int kvh, int j0, int j1, float* dst_o, float* dst_lse,
                                 float lse_mul, ItemSmem<G>& sm)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int r = lane >> 4, c = lane & 15;

    // a2: the group's queries, 8 dims per lane as 4 packed bf16 pairs
    uint32_t qr[G][4];
    {
        const uint4* qp = reinterpret_cast<const uint4*>(p.q) + ((size_t)b * p.Hq + (size_t)kvh * G) * kRowU4 + c;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint4 t = qp[g * kRowU4];
            qr[g][0] = t.x; qr[g][1] = t.y; qr[g][2] = t.z; qr[g][3] = t.w;
        }
    }
    const size_t row0 = ((size_t)b * p.Hkv + kvh) * (size_t)p.S_max;
    const uint4* kp = reinterpret_cast<const uint4*>(p.k) + row0 * kRowU4;
    const uint4* vp = reinterpret_cast<const uint4*>(p.v) + row0 * kRowU4;

    ValuState<G> st;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        st.m[g] = kNegBig;
        st.l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[g][e] = 0.f;
    }

    // a3-a5: wave w owns the 32-key tiles w, w+4, w+8, ... of the item
    const int n_tiles = (j1 - j0 + kValuTileKeys - 1) / kValuTileKeys;
    const int n_full = (j1 - j0) / kValuTileKeys;       // tiles below n_full need no mask
    const float sl2 = p.scale_log2;
    // One K buffer and one V buffer: K of the next tile is requested as soon as the
    // scores of this tile are done (it flies during softmax + PV), V of the next
    // tile as soon as PV is done (it flies during the next tile's scores).
    uint4 kt[kValuLoads], vt[kValuLoads];
    auto load = [&](uint4 (&dst)[kValuLoads], const uint4* base, int tt) {
        const int kb = j0 + tt * kValuTileKeys;
        if (tt < n_full) valu_load_rows<false>(dst, base, kb, j1, r, c);
        else valu_load_rows<true>(dst, base, kb, j1, r, c);
    };
    int t = wave;
    if (t < n_tiles) {
        load(kt, kp, t);
        load(vt, vp, t);
    }
    while (t < n_tiles) {
        const int kb = j0 + t * kValuTileKeys;
        const int tn = t + kWaves;
        float s[G][kValuLoads];
        if (t < n_full) valu_scores<G, false>(kt, qr, s, sl2, kb, j1, r);
        else valu_scores<G, true>(kt, qr, s, sl2, kb, j1, r);
        if (tn < n_tiles) load(kt, kp, tn);
        valu_softmax<G>(s, st);
        valu_pv<G>(vt, s, st);
        if (tn < n_tiles) load(vt, vp, tn);
        t = tn;
    }

    trace_event(p, kEvLoopEnd);
    // a6: merge the 4 row states of the wave (lanes c, c+16, c+32, c+48 hold the same dims)
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float M = fmaxf(st.m[g], __shfl_xor(st.m[g], 16));
        M = fmaxf(M, __shfl_xor(M, 32));
        const float f = fast_exp2(st.m[g] - M);
        float lw = st.l[g] * f;
        lw += __shfl_xor(lw, 16);
        lw += __shfl_xor(lw, 32);
        st.m[g] = M;
        st.l[g] = lw;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float a = st.acc[g][e] * f;
            a += __shfl_xor(a, 16);
            a += __shfl_xor(a, 32);
            st.acc[g][e] = a;
        }
    }
    if (r == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float4* d = reinterpret_cast<float4*>(&sm.acc[wave][g][c * 8]);
            d[0] = make_float4(st.acc[g][0], st.acc[g][1], st.acc[g][2], st.acc[g][3]);
            d[1] = make_float4(st.acc[g][4], st.acc[g][5], st.acc[g][6], st.acc[g][7]);
            if (c == 0) {
                sm.m[g][wave] = st.m[g];
                sm.l[g][wave] = st.l[g];
            }
        }
    }
    __syncthreads();

    item_finish<G, SHARED>(sm, G, dst_o, dst_lse, lse_mul);
}

}  // namespace fd
