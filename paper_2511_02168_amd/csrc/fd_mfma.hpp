// Partial attention of one key range on the matrix cores: the default kernel for every
// GQA group size up to 16 (the group's query rows are the columns of a 16-wide MFMA tile;
// below 16 the rest is padding, which the HBM bound hides).
//
// Steps a2-a6 of the hot path (paper Section 4.2.1, Algorithm 4 Part 1) for up
// to 16 query heads that share one KV head.
//
// Data flow, per wave (the 4 waves of a workgroup are independent pipelines):
//   * K and V rows go global -> LDS directly (global_load_lds_dwordx4, no
//     registers in between).  The wave owns a private ring of NST stages in LDS,
//     one stage = 16 keys of K (4 KB) + the same 16 keys of V (4 KB), and keeps
//     NST-1 stages in flight while it computes on the oldest.  A wave only reads
//     what it loaded itself, so the loop needs no workgroup barrier: the wave's
//     own vmcnt tells it when a stage has landed.
//   * wave w takes the 16-key blocks w, w+4, w+8, ... of the range, so the
//     workgroup streams the range front to back.
//   * QK^T: S^T[16 keys x 16 heads] = K_blk . q^T with 4 v_mfma_f32_16x16x32_bf16
//     (contraction over D = 128).  K is the A operand, read from LDS as 16-byte
//     chunks (one chunk = 8 dims); rows are XOR-swizzled so the 16 rows of a
//     block hit 16 different chunk positions.
//   * the result layout (lane = head, 4 keys per lane) is exactly the B operand
//     layout of v_mfma_f32_16x16x16_bf16, so P never moves between lanes.
//   * P is split into bf16 hi + lo parts (p = hi + lo to 2^-16 relative), two
//     MFMAs per 16-dim block, so the result carries fp32-grade weights.
//   * PV: O^T[16 dims x 16 heads] += V^T_blk . P^T; the transposed V operand comes
//     from ds_read_b64_tr_b16, which hands each lane 4 keys of one dim.
#pragma once

#include "fd_device.hpp"

namespace fd {

constexpr int kMfBlockKeys = 16;                            // keys per wave stage
constexpr int kMfHalfBytes = kMfBlockKeys * kD * 2;         // K (or V) of a stage: 4 KB
constexpr int kMfStageBytes = 2 * kMfHalfBytes;             // 8 KB
constexpr int kMfRows = 16;                                 // MFMA tile rows = max heads per KV head

__host__ __device__ constexpr int mfma_ring_bytes(int nst) { return kWaves * nst * kMfStageBytes; }
// Paged cache: page numbers of a wave's next blocks, fetched kMfPageSlots blocks at a time
// into LDS behind the ring, so that the streaming loop itself never touches the block table.
constexpr int kMfPageSlots = 256;    // 16K keys per workgroup between refills; 4 KB of LDS
__host__ __device__ constexpr int mfma_lds_bytes(int nst) { return mfma_ring_bytes(nst) + kWaves * kMfPageSlots * 4; }

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;

// 64 lanes x 16 bytes, global -> LDS.  Lane l's 16 bytes come from gbase + voff(l)
// and land at LDS byte address lds_addr + 16*l.  lds_addr and gbase are
// wave-uniform.  Completion is tracked by vmcnt like any vector load.  The data is
// used once: the non-temporal hint raises streaming read bandwidth measurably.
__device__ __forceinline__ void dma_row4(uint32_t lds_addr, const void* gbase, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(gbase)
                 : "memory", "m0");
}

// The same pointer, held in scalar registers (the value must already be wave-uniform).  Free where
// the compiler knows the value to be uniform; where it cannot tell (a value that came through
// LDS or a call it did not inline), this is what puts it into the scalar registers dma_row4 needs.
template <class T>
__device__ __forceinline__ const T* scalar_ptr(const T* p)
{
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const T*>((uintptr_t)(((uint64_t)hi << 32) | lo));
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// waits until at most `stages` later stages (8 loads each) are still in flight
__device__ __forceinline__ void wait_stages_in_flight(int stages)
{
    switch (stages) {
        case 0: wait_vmcnt<0>(); break;
        case 1: wait_vmcnt<8>(); break;
        case 2: wait_vmcnt<16>(); break;
        case 3: wait_vmcnt<24>(); break;
        case 4: wait_vmcnt<32>(); break;
        case 5: wait_vmcnt<40>(); break;
        case 6: wait_vmcnt<48>(); break;
        default: wait_vmcnt<56>(); break;
    }
}

__device__ __forceinline__ uint32_t lds_address(const void* p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// How far (base-2 units) a score may exceed the running reference maximum before the
// accumulators are rescaled.
constexpr float kRescaleSlack = 6.0f;

struct MfmaState {
    float m;            // reference maximum of head (lane & 15), base-2 units, same in the 4 lanes of a head:
                        // at least (largest score seen) - kRescaleSlack
    float l;            // this lane's share of the running sum (its 4 keys per block)
    f32x4_t acc[8];     // O^T: block db, element e = dim 16*db + 4*(lane>>4) + e of head (lane & 15)
};

// Requests the 16 keys [kb, kb+16) of K and V, whose rows start at kp / vp (wave-uniform),
// into one stage.  Rows at or past j1 re-read row j1-1 (a live row of the same block);
// their scores are masked later.
// LDS layout of a half stage: row r (0..15) at r*256, its 16-byte chunk c stored at
// position c ^ r.
__device__ __forceinline__ void mfma_issue_stage(uint32_t lds_stage, const uint16_t* kp, const uint16_t* vp,
                                                 int kb, int j1, int lane)
{
    const int rsub = lane >> 4, pos = lane & 15;
    const bool full = kb + kMfBlockKeys <= j1;
    kp = scalar_ptr(kp);
    vp = scalar_ptr(vp);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 4 * i + rsub;                       // row of the block this lane fills
        int src_row = r;
        if (!full) src_row = min(r, j1 - 1 - kb);
        const uint32_t voff = (uint32_t)(src_row * 256 + ((pos ^ r) << 4));
        dma_row4(lds_stage + i * 1024, kp, voff);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 4 * i + rsub;
        int src_row = r;
        if (!full) src_row = min(r, j1 - 1 - kb);
        const uint32_t voff = (uint32_t)(src_row * 256 + ((pos ^ r) << 4));
        dma_row4(lds_stage + kMfHalfBytes + i * 1024, vp, voff);
    }
}

// One landed stage: scores, online softmax, PV.
// F16: q, K, V hold IEEE half instead of bf16; the same tiles through the f16 MFMAs, P split
// into half hi + lo (p in [0, 1]: the lo part keeps it to ~2^-21, flushing below 6e-8).
template <bool MASKED, bool F16>
__device__ __forceinline__ void mfma_consume_stage(const char* stage, const bf16x8_t (&qb)[4], MfmaState& st,
                                                   float scale_log2, int kb, int j1, int lane)
{
    const int i16 = lane & 15, kg = lane >> 4;

    // a3: S^T[key i16][head] over D = 4 steps of 32 dims; step t, lane group kg uses chunk 4t + kg
    f32x4_t s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int chunk = 4 * t + kg;
        const uint4 kk = *reinterpret_cast<const uint4*>(stage + i16 * 256 + ((chunk ^ i16) << 4));
        if (F16)
            s = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, kk), __builtin_bit_cast(f16x8_t, qb[t]), s,
                                                       0, 0, 0);
        else
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kk), qb[t], s, 0, 0, 0);
    }
    // now s[e] = <q_head, K[kb + 4kg + e]> for head = lane & 15

    // a4: online softmax in base 2
    float p[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        p[e] = s[e] * scale_log2;
        if (MASKED) p[e] = (kb + 4 * kg + e) < j1 ? p[e] : -INFINITY;
    }
    float tm = fmaxf(fmaxf(p[0], p[1]), fmaxf(p[2], p[3]));
    tm = head_lanes_max(tm);
    // The reference maximum st.m only moves when some head's scores exceed it by more than
    // kRescaleSlack (then every head moves to its current maximum): weights stay below
    // 2^kRescaleSlack, which fp32 sums and the hi + lo split below carry without loss, and the
    // rescale of the accumulators becomes a rare event instead of one per new maximum.
    if (__any(tm > st.m + kRescaleSlack)) {
        const float mnew = fmaxf(st.m, tm);
        const float alpha = fast_exp2(st.m - mnew);
        st.m = mnew;
        st.l *= alpha;
#pragma unroll
        for (int db = 0; db < 8; ++db) st.acc[db] *= alpha;
    }
    s16x4_t phi, plo;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        p[e] = fast_exp2(p[e] - st.m);
        st.l += p[e];
        if (F16) {
            const _Float16 hi = (_Float16)p[e];
            const _Float16 lo = (_Float16)(p[e] - (float)hi);
            phi[e] = __builtin_bit_cast(short, hi);
            plo[e] = __builtin_bit_cast(short, lo);
        } else {
            // hi = p cut to its upper 16 bits (a bf16 value), lo = the exact rest, rounded to bf16
            const uint32_t bits = __builtin_bit_cast(uint32_t, p[e]);
            const __bf16 lo = (__bf16)(p[e] - __builtin_bit_cast(float, bits & 0xffff0000u));
            phi[e] = (short)(bits >> 16);
            plo[e] = __builtin_bit_cast(short, lo);
        }
    }

    // a5: O^T[dim][head] += V^T . P^T, 16 dims at a time.  Lane t of a 16-lane group
    // points at row 4kg + t/4, dims 16db + 4(t%4) .. +3; the transposing read then
    // gives lane i the 4 keys 4kg..4kg+3 of dim 16db + i.
    const char* vstage = stage + kMfHalfBytes;
    const int vrow = 4 * kg + (i16 >> 2);
    const int vsub = i16 & 3;
#pragma unroll
    for (int db = 0; db < 8; ++db) {
        const int chunk = 2 * db + (vsub >> 1);
        const char* src = vstage + vrow * 256 + ((chunk ^ vrow) << 4) + ((vsub & 1) << 3);
        const s16x4_t vt = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)src);
        if (F16) {
            const f16x4_t vh = __builtin_bit_cast(f16x4_t, vt);
            st.acc[db] = __builtin_amdgcn_mfma_f32_16x16x16f16(vh, __builtin_bit_cast(f16x4_t, phi), st.acc[db], 0, 0, 0);
            st.acc[db] = __builtin_amdgcn_mfma_f32_16x16x16f16(vh, __builtin_bit_cast(f16x4_t, plo), st.acc[db], 0, 0, 0);
        } else {
            st.acc[db] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vt, phi, st.acc[db], 0, 0, 0);
            st.acc[db] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vt, plo, st.acc[db], 0, 0, 0);
        }
    }
}

// What a workgroup requested for its first key range before the range's end was known (the
// sequence length still on its way): the query group, and stage 0 of every wave, aimed at the
// split's nominal start.  Consumed by the first mfma_item call, which checks it against the range.
struct MfmaPrefetch {
    bf16x8_t qb[4];
    int j0;          // start of the range the stages were aimed at; -1 = nothing requested
    int j1_max;      // no block at or past this key was requested
    __device__ __forceinline__ void reset() { j0 = -1; }
    __device__ __forceinline__ bool any() const { return j0 >= 0; }
};

// a2: B operand of QK^T: lane (head, kg) holds dims 8*(4t + kg) .. +7 of its head; rows >= G are zero.
__device__ __forceinline__ void mfma_load_q(const Params& p, int b, int kvh, int lane, bf16x8_t (&qb)[4])
{
    const int head = lane & 15, kg = lane >> 4;
    const uint4* qp = reinterpret_cast<const uint4*>(p.q) + ((size_t)b * p.Hq + (size_t)kvh * p.G + head) * kRowU4;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (head < p.G) v = qp[4 * t + kg];
        qb[t] = __builtin_bit_cast(bf16x8_t, v);
    }
}

// Requests q and each wave's first NST - 1 16-key blocks (the stages the loop keeps in flight) of the range starting at j0
// of tile (b, kvh), knowing only that the range ends at or before j1_max <= S_max (contiguous
// cache).  Rows up to j1_max - 1 may be read: inside the cache, possibly past the sequence's end;
// a block that turns out not to lie wholly inside the real range is requested again by
// mfma_item, so what was read past the end is never used.
template <int NST>
__device__ __forceinline__ void mfma_prefetch(const Params& p, int b, int kvh, int j0, int j1_max, char* ring,
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
        const int kb = j0 + (wave + kWaves * s) * kMfBlockKeys;
        if (kb < j1_max)
            mfma_issue_stage(lds_address(ring + (wave * NST + s) * kMfStageBytes), p.k + (row0 + kb) * kD, p.v + (row0 + kb) * kD,
                             kb, j1_max, lane);
    }
}

// Attends keys [j0, j1) (j0 < j1) of tile (b, kvh) for its G <= 16 query heads.
// ring: this workgroup's LDS ring (mfma_ring_bytes(NST) bytes, 16-byte aligned);
// it doubles as the ItemSmem<16> staging at the end of the range.
// Writes the normalised result to dst_o[G][D] and the log-sum-exp times lse_mul to
// dst_lse[G] (SHARED as in item_finish).  Leaves LDS free for reuse on return.
// pf: what mfma_prefetch requested for this range, if anything (reset here).  hook: a side job
// of the caller that touches no global memory; wave 0 runs it once, right after its first
// requests of the loop have gone out, in time the wave would spend waiting for them.
template <int NST, bool PAGED, bool F16, bool SHARED, class Hook>
__device__ __forceinline__ void mfma_item(const Params& p, int b, int kvh, int j0, int j1, float* dst_o, float* dst_lse,
                                 float lse_mul, char* ring, MfmaPrefetch& pf, const Hook& hook)
{
    static_assert(NST >= 2 && NST <= 8, "ring depth");
    static_assert(sizeof(ItemSmem<kMfRows>) <= (size_t)mfma_ring_bytes(2), "staging must fit the ring");
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int G = p.G;
    const int head = lane & 15, kg = lane >> 4;

    // contiguous cache: the tile's rows; paged cache: looked up per block, see below
    constexpr bool paged = PAGED;                         // compile-time: the contiguous loop pays nothing for it
    const size_t row0 = paged ? 0 : ((size_t)b * p.Hkv + kvh) * (size_t)p.S_max;
    const uint16_t* kbase = p.k + row0 * kD;
    const uint16_t* vbase = p.v + row0 * kD;

    MfmaState st;
    st.m = kNegBig;
    st.l = 0.f;
#pragma unroll
    for (int db = 0; db < 8; ++db) st.acc[db] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // a3-a5: this wave's blocks are wave, wave + 4, ...; `mine` of them
    const int n_blocks = (j1 - j0 + kMfBlockKeys - 1) / kMfBlockKeys;
    const int mine = wave < n_blocks ? (n_blocks - wave + kWaves - 1) / kWaves : 0;
    char* my_ring = ring + wave * (NST * kMfStageBytes);
    const uint32_t my_ring_lds = lds_address(my_ring);
    int* my_pages = reinterpret_cast<int*>(ring + mfma_ring_bytes(NST)) + wave * kMfPageSlots;
    const float sl2 = p.scale_log2;
    constexpr int P = NST - 1;                            // stages in flight ahead of the one being consumed

    // a2: the query group, requested first (the round trip overlaps the issue of the first stages),
    // unless the prefetch already did.  This wave's stage 0 counts as requested if the prefetch
    // aimed at this range and the block lies wholly inside it; a prefetched block that does not
    // is waited for and requested again below.
    bf16x8_t qb[4];
    int n_requested = 0;                  // leading stages of this wave that are already on their way (or landed)
    if (!paged && pf.any()) {
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
                const int kb = j0 + (wave + kWaves * s) * kMfBlockKeys;
                n_issued += kb < pf.j1_max;
                n_valid += kb + kMfBlockKeys <= j1;
            }
        }
        if (n_valid != n_issued) wait_loads_landed();
        n_requested = n_valid;
        pf.reset();
    } else {
        mfma_load_q(p, b, kvh, lane, qb);
    }

    // The wave's blocks are streamed in chunks: the whole range at once for a contiguous
    // cache; kMfPageSlots blocks at a time for a paged one, whose page numbers are fetched
    // into LDS before the chunk starts (the pipeline is empty then, so these ordinary
    // loads disturb nothing).  The softmax state carries across chunks.
    const int chunk_blocks = paged ? kMfPageSlots : max(mine, 1);
    for (int c0 = 0; c0 < mine; c0 += chunk_blocks) {
        const int cmine = min(chunk_blocks, mine - c0);
        if (paged) {
            const int32_t* row = p.block_table + (size_t)b * p.pages_per_seq;
            for (int i = lane; i < cmine; i += 64) {
                const int kb = j0 + (wave + kWaves * (c0 + i)) * kMfBlockKeys;
                const int pg = row[kb >> p.page_shift];
                my_pages[i] = min(max(pg, 0), p.num_pages - 1);      // never leave the pool
            }
        }
        // requests stage `s` of this chunk into its ring slot
        const auto issue = [&](int s) {
            const int kb = j0 + (wave + kWaves * (c0 + s)) * kMfBlockKeys;
            const uint16_t *kp, *vp;
            if (paged) {
                const int pg = __builtin_amdgcn_readfirstlane(my_pages[s]);
                const size_t first_row = (((size_t)pg * p.Hkv + kvh) << p.page_shift) + (kb & ((1 << p.page_shift) - 1));
                kp = p.k + first_row * kD;
                vp = p.v + first_row * kD;
            } else {
                kp = kbase + (size_t)kb * kD;
                vp = vbase + (size_t)kb * kD;
            }
            mfma_issue_stage(my_ring_lds + (s % NST) * kMfStageBytes, kp, vp, kb, j1, lane);
        };
        // NST - 1 stages go out up front (measured: requesting the whole ring at once and
        // waiting for all of it starts the first consume later and loses half a microsecond)
        for (int s = (c0 == 0 ? n_requested : 0); s < P && s < cmine; ++s) issue(s);
        // The caller's side job (LDS and arithmetic only), once, by wave 0, with its first requests
        // on their way and BEFORE the compiler's wait for q below: that wait is "every vector load
        // of this wave has returned", the stage requests included, so whatever stands behind it
        // runs after the first stage has landed instead of beside its flight.
        if (c0 == 0 && wave == 0) hook();
        // Make the compiler wait for the q loads HERE: the loop below must contain no
        // compiler-generated vmcnt wait, which would also drain the stage loads the loop
        // keeps in flight (they are issued from inline asm, invisible to its counter).
        asm volatile("" ::"v"(qb[0]), "v"(qb[1]), "v"(qb[2]), "v"(qb[3]));
        // Only the range's last block can be ragged; it is the last block of the wave that owns it
        // and is handled after the loop, which therefore holds the unmasked code alone.
        const int kb_last = j0 + (wave + kWaves * (c0 + cmine - 1)) * kMfBlockKeys;
        const int full = kb_last + kMfBlockKeys <= j1 ? cmine : cmine - 1;
        for (int s = 0; s < full; ++s) {
            if (s + P < cmine) issue(s + P);
            wait_stages_in_flight(min(P, cmine - 1 - s));
            if (c0 + s == 0) trace_event(p, kEvFirstStage);
            const int kb = j0 + (wave + kWaves * (c0 + s)) * kMfBlockKeys;
            mfma_consume_stage<false, F16>(my_ring + (s % NST) * kMfStageBytes, qb, st, sl2, kb, j1, lane);
        }
        if (full < cmine) {
            wait_stages_in_flight(0);
            if (c0 + full == 0) trace_event(p, kEvFirstStage);
            mfma_consume_stage<true, F16>(my_ring + (full % NST) * kMfStageBytes, qb, st, sl2, kb_last, j1, lane);
        }
    }

    trace_event(p, kEvLoopEnd);
    // a6: every lane of a head gets the head's sum; then the wave leaves its state in LDS
    st.l = head_lanes_sum(st.l);
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
    item_finish<kMfRows, SHARED>(sm, G, dst_o, dst_lse, lse_mul);
}

}  // namespace fd
