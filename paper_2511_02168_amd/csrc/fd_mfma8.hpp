// Flash Decode over an FP8 (OCP E4M3) KV cache -- the MFMA kernel's stream at half the bytes.
//
// q stays bf16; K and V are one byte per element, a stored byte standing for
// value * k_scale (v_scale).  Every E4M3 value is a bf16 value, so a stage is converted
// exactly to bf16 on its way from LDS to the matrix cores and the arithmetic is the bf16
// kernel's: k_scale is folded into the score scale, v_scale into the final normalisation.
//
// A wave stage is 32 keys (4 KB of K + 4 KB of V: the byte size of the bf16 kernel's
// 16-key stage, so ring, DMA count per stage and wait counts are shared with it).
//   * QK^T: two 16-key blocks x 4 steps of v_mfma_f32_16x16x32_bf16; a lane reads the 8
//     bytes (8 dims) of its key with one ds_read_b64.
//   * PV: v_mfma_f32_16x16x32_f16 with K = 32 keys: V is widened to IEEE half (every E4M3 value
//     is a half value too) and P goes in as ONE half (11 significant bits, 2^-12 relative:
//     an eighth of the output tolerance) instead of the bf16 kernel's hi + lo pair, which
//     halves the PV matrix work and drops the split arithmetic; the weights carry a factor
//     2^kM8PShift so that small ones stay clear of half's underflow, and the sum l carries it
//     too, so it cancels in o = acc / l and moves into the reference maximum for the lse.
//     The B operand (P) of lane
//     (head, kg) is exactly the 8 scores that lane holds after QK^T (keys 4kg..4kg+3 of
//     both blocks), so P still never moves between lanes; the A operand (V^T: 8 keys
//     of one dim per lane) comes from ds_read_b64_tr_b8, whose 16-lane groups each
//     transpose an 8-row x 16-byte tile: lanes 2j, 2j+1 of a group point at the two
//     halves of row j, lane i receives byte column i of the 8 rows (probed on gfx950).
//     Row j of group kg is pointed at key 16*(j>>2) + 4kg + (j&3): P's key order.
// LDS layout of a half stage: key row r (0..31) at r*128, its 16-byte chunk c at position
// c ^ swz(r), swz(r) = (r ^ (r >> 2)) & 7: conflict-free for both access patterns.
#pragma once

#include "fd_mfma.hpp"

namespace fd {

constexpr int kM8BlockKeys = 32;                            // keys per wave stage
constexpr int kM8RowBytes = kD;                             // one byte per element
constexpr int kM8HalfBytes = kM8BlockKeys * kM8RowBytes;    // K (or V) of a stage: 4 KB
static_assert(2 * kM8HalfBytes == kMfStageBytes, "the FP8 stage reuses the bf16 kernel's ring");

typedef int i32x2_t __attribute__((ext_vector_type(2)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) i32x2_t* lds_i32x2_ptr;

__device__ __forceinline__ int swz8(int r) { return (r ^ (r >> 2)) & 7; }

// 8 E4M3 bytes (w.x = bytes 0..3, w.y = 4..7) -> 8 bf16, exactly: every E4M3 value is a bf16
// value, and v_cvt_scalef32_pk_bf16_fp8 with scale 1 converts two bytes per instruction.
__device__ __forceinline__ bf16x8_t fp8x8_to_bf16(i32x2_t w)
{
    typedef __bf16 bf16x2_v __attribute__((ext_vector_type(2)));
    const bf16x2_v a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.x, 1.0f, false);
    const bf16x2_v b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.x, 1.0f, true);
    const bf16x2_v c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.y, 1.0f, false);
    const bf16x2_v d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.y, 1.0f, true);
    bf16x8_t r;
    r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
    r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
    return r;
}

// 8 E4M3 bytes -> 8 IEEE halves, exactly (v_cvt_scalef32_pk_f16_fp8 with scale 1)
__device__ __forceinline__ f16x8_t fp8x8_to_f16(i32x2_t w)
{
    typedef _Float16 f16x2_v __attribute__((ext_vector_type(2)));
    const f16x2_v a = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w.x, 1.0f, false);
    const f16x2_v b = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w.x, 1.0f, true);
    const f16x2_v c = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w.y, 1.0f, false);
    const f16x2_v d = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w.y, 1.0f, true);
    f16x8_t r;
    r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
    r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
    return r;
}

// Weights are computed as 2^(score - reference + kM8PShift): at most 2^(kRescaleSlack + kM8PShift)
// = 2^14, far below half's largest value, and a weight 2^-32 of the largest still is a half.
constexpr float kM8PShift = 8.0f;

// Requests the 32 keys [kb, kb+32) of K and V (rows of 128 bytes starting at kp / vp,
// wave-uniform) into one stage: 4 + 4 transfers of 8 rows.  Rows at or past j1 re-read
// row j1-1; their scores are masked later.
__device__ __forceinline__ void mfma8_issue_stage(uint32_t lds_stage, const uint8_t* kp, const uint8_t* vp, int kb,
                                                  int j1, int lane)
{
    const int rsub = lane >> 3, pos = lane & 7;
    const int last = j1 - 1 - kb;                         // last live row of the block (>= 0)
    kp = scalar_ptr(kp);
    vp = scalar_ptr(vp);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 8 * i + rsub;
        const uint32_t voff = (uint32_t)(min(r, last) * kM8RowBytes + ((pos ^ swz8(r)) << 4));
        dma_row4(lds_stage + i * 1024, kp, voff);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 8 * i + rsub;
        const uint32_t voff = (uint32_t)(min(r, last) * kM8RowBytes + ((pos ^ swz8(r)) << 4));
        dma_row4(lds_stage + kM8HalfBytes + i * 1024, vp, voff);
    }
}

// One landed stage of 32 keys: scores, online softmax, PV.
template <bool MASKED>
__device__ __forceinline__ void mfma8_consume_stage(const char* stage, const bf16x8_t (&qb)[4], MfmaState& st,
                                                    float scale_log2, int kb, int j1, int lane)
{
    const int i16 = lane & 15, kg = lane >> 4;

    // a3: S^T[key][head] for the two 16-key blocks; lane (key i16, kg) feeds dims 32t + 8kg .. +7
    f32x4_t s[2];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
        s[blk] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        const int row = 16 * blk + i16;
        const char* rowp = stage + row * kM8RowBytes + ((kg & 1) << 3);
        const int sw = swz8(row);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int chunk = 2 * t + (kg >> 1);
            const i32x2_t w = *reinterpret_cast<const i32x2_t*>(rowp + ((chunk ^ sw) << 4));
            s[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fp8x8_to_bf16(w), qb[t], s[blk], 0, 0, 0);
        }
    }
    // now s[blk][e] = <q_head, K[kb + 16 blk + 4kg + e]> for head = lane & 15

    // a4: online softmax in base 2 over the lane's 8 keys
    float p[8];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float x = s[blk][e] * scale_log2;
            if (MASKED) x = (kb + 16 * blk + 4 * kg + e) < j1 ? x : -INFINITY;
            p[4 * blk + e] = x;
        }
    float tm = fmaxf(fmaxf(fmaxf(p[0], p[1]), fmaxf(p[2], p[3])), fmaxf(fmaxf(p[4], p[5]), fmaxf(p[6], p[7])));
    tm = head_lanes_max(tm);
    // lazy reference maximum as in mfma_consume_stage
    if (__any(tm > st.m + kRescaleSlack)) {
        const float mnew = fmaxf(st.m, tm);
        const float alpha = fast_exp2(st.m - mnew);
        st.m = mnew;
        st.l *= alpha;
#pragma unroll
        for (int db = 0; db < 8; ++db) st.acc[db] *= alpha;
    }
    f16x8_t ph;
    const float mref = st.m - kM8PShift;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        p[e] = fast_exp2(p[e] - mref);
        st.l += p[e];
        ph[e] = (_Float16)p[e];
    }

    // a5: O^T[dim][head] += V^T . P^T over the 32 keys, 16 dims at a time
    const char* vstage = stage + kM8HalfBytes;
    const int j = i16 >> 1;                                    // row of this lane pair inside the transposed tile
    const int vrow = 16 * (j >> 2) + 4 * kg + (j & 3);         // = the key P's element j stands for
    const char* vrowp = vstage + vrow * kM8RowBytes + ((i16 & 1) << 3);
    const int vsw = swz8(vrow);
#pragma unroll
    for (int db = 0; db < 8; ++db) {
        const i32x2_t w = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_i32x2_ptr)(vrowp + ((db ^ vsw) << 4)));
        st.acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fp8x8_to_f16(w), ph, st.acc[db], 0, 0, 0);
    }
}

// mfma_prefetch for an FP8 cache: q and each wave's first NST - 1 32-key blocks.
template <int NST>
__device__ __forceinline__ void mfma8_prefetch(const Params& p, int b, int kvh, int j0, int j1_max, char* ring,
                                               MfmaPrefetch& pf)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    mfma_load_q(p, b, kvh, lane, pf.qb);
    pf.j0 = j0;
    pf.j1_max = j1_max;
    const size_t row0 = ((size_t)b * p.Hkv + kvh) * (size_t)p.S_max;
#pragma unroll
    for (int s = 0; s < NST - 1; ++s) {
        const int kb = j0 + (wave + kWaves * s) * kM8BlockKeys;
        if (kb < j1_max)
            mfma8_issue_stage(lds_address(ring + (wave * NST + s) * kMfStageBytes),
                              reinterpret_cast<const uint8_t*>(p.k) + (row0 + kb) * kM8RowBytes,
                              reinterpret_cast<const uint8_t*>(p.v) + (row0 + kb) * kM8RowBytes, kb, j1_max, lane);
    }
}

// Attends keys [j0, j1) (j0 < j1) of tile (b, kvh) of an FP8 cache; contract as mfma_item,
// PAGED as there (a 32-key block never straddles a page of 32 keys or more).
template <int NST, bool PAGED, bool SHARED, class Hook>
__device__ __forceinline__ void mfma8_item(const Params& p, int b, int kvh, int j0, int j1, float* dst_o, float* dst_lse,
                                  float lse_mul, char* ring, MfmaPrefetch& pf, const Hook& hook)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int G = p.G;
    const int head = lane & 15, kg = lane >> 4;

    const size_t row0 = PAGED ? 0 : ((size_t)b * p.Hkv + kvh) * (size_t)p.S_max;
    const uint8_t* kbase = reinterpret_cast<const uint8_t*>(p.k) + row0 * kM8RowBytes;
    const uint8_t* vbase = reinterpret_cast<const uint8_t*>(p.v) + row0 * kM8RowBytes;

    MfmaState st;
    st.m = kNegBig;
    st.l = 0.f;
#pragma unroll
    for (int db = 0; db < 8; ++db) st.acc[db] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const int n_blocks = (j1 - j0 + kM8BlockKeys - 1) / kM8BlockKeys;
    const int mine = wave < n_blocks ? (n_blocks - wave + kWaves - 1) / kWaves : 0;
    char* my_ring = ring + wave * (NST * kMfStageBytes);
    const uint32_t my_ring_lds = lds_address(my_ring);
    int* my_pages = reinterpret_cast<int*>(ring + mfma_ring_bytes(NST)) + wave * kMfPageSlots;
    const float sl2 = p.scale_log2;
    constexpr int P = NST - 1;

    // q and this wave's stage 0: from the prefetch if it aimed at this range (see mfma_item)
    bf16x8_t qb[4];
    int n_requested = 0;                  // leading stages of this wave that are already on their way (or landed)
    if (!PAGED && pf.any()) {
#pragma unroll
        for (int t = 0; t < 4; ++t) qb[t] = pf.qb[t];
        // a prefetched block counts if it was aimed at this range and lies wholly inside it;
        // if any block the prefetch requested does not, wait for all of them before the ring
        // slots are requested again
        int n_issued = NST - 1, n_valid = 0;
        if (pf.j0 == j0) {
            n_issued = 0;
#pragma unroll
            for (int s = 0; s < NST - 1; ++s) {
                const int kb = j0 + (wave + kWaves * s) * kM8BlockKeys;
                n_issued += kb < pf.j1_max;
                n_valid += kb + kM8BlockKeys <= j1;
            }
        }
        if (n_valid != n_issued) wait_loads_landed();
        n_requested = n_valid;
        pf.reset();
    } else {
        mfma_load_q(p, b, kvh, lane, qb);
    }
    // chunks of blocks as in mfma_item: one for a contiguous cache, kMfPageSlots blocks at a
    // time for a paged one, page numbers fetched into LDS while the pipeline is empty
    const int chunk_blocks = PAGED ? kMfPageSlots : max(mine, 1);
    for (int c0 = 0; c0 < mine; c0 += chunk_blocks) {
        const int cmine = min(chunk_blocks, mine - c0);
        if (PAGED) {
            const int32_t* row = p.block_table + (size_t)b * p.pages_per_seq;
            for (int i = lane; i < cmine; i += 64) {
                const int kb = j0 + (wave + kWaves * (c0 + i)) * kM8BlockKeys;
                const int pg = row[kb >> p.page_shift];
                my_pages[i] = min(max(pg, 0), p.num_pages - 1);
            }
        }
        const auto issue = [&](int s) {
            const int kb = j0 + (wave + kWaves * (c0 + s)) * kM8BlockKeys;
            const uint8_t *kp, *vp;
            if (PAGED) {
                const int pg = __builtin_amdgcn_readfirstlane(my_pages[s]);
                const size_t first_row = (((size_t)pg * p.Hkv + kvh) << p.page_shift) + (kb & ((1 << p.page_shift) - 1));
                kp = kbase + first_row * kM8RowBytes;
                vp = vbase + first_row * kM8RowBytes;
            } else {
                kp = kbase + (size_t)kb * kM8RowBytes;
                vp = vbase + (size_t)kb * kM8RowBytes;
            }
            mfma8_issue_stage(my_ring_lds + (s % NST) * kMfStageBytes, kp, vp, kb, j1, lane);
        };
        // NST - 1 stages go out up front (measured: requesting the whole ring at once and
        // waiting for all of it starts the first consume later and loses half a microsecond)
        for (int s = (c0 == 0 ? n_requested : 0); s < P && s < cmine; ++s) issue(s);
        // the caller's side job before, the compiler's wait for the q loads here, outside the loop (see mfma_item)
        if (c0 == 0 && wave == 0) hook();
        asm volatile("" ::"v"(qb[0]), "v"(qb[1]), "v"(qb[2]), "v"(qb[3]));
        // the range's last block, if ragged, after the loop (see mfma_item)
        const int kb_last = j0 + (wave + kWaves * (c0 + cmine - 1)) * kM8BlockKeys;
        const int full = kb_last + kM8BlockKeys <= j1 ? cmine : cmine - 1;
        for (int s = 0; s < full; ++s) {
            if (s + P < cmine) issue(s + P);
            wait_stages_in_flight(min(P, cmine - 1 - s));
            if (c0 + s == 0) trace_event(p, kEvFirstStage);
            const int kb = j0 + (wave + kWaves * (c0 + s)) * kM8BlockKeys;
            mfma8_consume_stage<false>(my_ring + (s % NST) * kMfStageBytes, qb, st, sl2, kb, j1, lane);
        }
        if (full < cmine) {
            wait_stages_in_flight(0);
            if (c0 + full == 0) trace_event(p, kEvFirstStage);
            mfma8_consume_stage<true>(my_ring + (full % NST) * kMfStageBytes, qb, st, sl2, kb_last, j1, lane);
        }
    }

    trace_event(p, kEvLoopEnd);
    st.l = head_lanes_sum(st.l);
    st.m -= kM8PShift;                                    // l and acc carry 2^kM8PShift: lse = (m - shift) + log2(l)
    __syncthreads();                                      // all waves are done reading their rings
    ItemSmem<kMfRows>& sm = *reinterpret_cast<ItemSmem<kMfRows>*>(ring);
    if (head < G) {
        if (kg == 0) {
            sm.m[head][wave] = st.m;
            sm.l[head][wave] = st.l;
        }
#pragma unroll
        for (int db = 0; db < 8; ++db)
            *reinterpret_cast<float4*>(&sm.acc[wave][head][16 * db + 4 * kg]) =
                make_float4(st.acc[db][0], st.acc[db][1], st.acc[db][2], st.acc[db][3]);
    }
    __syncthreads();
    item_finish<kMfRows, SHARED>(sm, G, dst_o, dst_lse, lse_mul, p.out_mul);
}

}  // namespace fd
