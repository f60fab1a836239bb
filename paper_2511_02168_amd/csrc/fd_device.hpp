// Device-side building blocks shared by the Flash Decode kernels (gfx950 only).
//
// Vocabulary (paper, Section 4.2 and Algorithm 4, mapped onto one GPU):
//   tile   = one (sequence b, KV head kvh): the G = Hq/Hkv query heads that
//            share a KV head are processed together.
//   split  = a contiguous key range of a tile (the role of a rank's KV shard).
//   item   = (tile, split): the unit of work a workgroup takes.
//   partial= normalised output o_i[G][D] and log-sum-exp lse_i[G] of an item
//            (the "inbox" content of Algorithm 4).
//   counter= arrivals per tile (the "signal flags" of Algorithm 4).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fd_fastdiv.hpp"

namespace fd {

constexpr int kD = 128;            // head dimension
constexpr int kRowU4 = kD * 2 / 16; // 16-byte chunks per K/V row (16)
constexpr int kWgThreads = 256;
constexpr int kWaves = kWgThreads / 64;
constexpr int kSplitAlign = 64;    // split lengths are multiples of this many keys
constexpr int kAdaptiveKeys = 512; // default keys per split when the library chooses
constexpr int kMaxGroupTiles = 2048;  // tiles one XCD group can index in adaptive mode
constexpr int kLseStride = 32;        // floats per slot of part_lse: one 128-byte line per slot (G <= 16 used)
constexpr float kNegBig = -3.0e38f;   // finite stand-in for "no key seen yet"
constexpr float kLn2 = 0.6931471805599453f;

// Kernel arguments.  The fields a workgroup needs before its first K/V request come first, within
// the first two 64-byte lines of the argument block, so that they arrive with the first scalar loads.
struct Params {
    const uint16_t* k;        // [B, Hkv, S_max, D] bf16, or the page pool [num_pages, Hkv, page_size, D]
    const uint16_t* v;        // like k
    const uint16_t* q;        // [B, Hq, D] bf16
    const int32_t* seq_lens;  // [B]
    int32_t B, Hq, Hkv, G, S_max;
    int32_t n_splits;         // 0 = adaptive
    int32_t xcd_groups;       // 1 or 8
    int32_t xcd_shift;        // log2(xcd_groups)
    int32_t grid;             // workgroups of the persistent launch
    // Fixed n_splits: what the host can work out before the launch, so that a workgroup reaches
    // its first K/V request after a few dozen instructions.
    int32_t split_keys;       // keys per split (from S_max, a multiple of kSplitAlign); 0 in adaptive mode
    int32_t sched_uniform;    // 1: every XCD group has the same tiles, members and item blocks (the three below)
    int32_t sched_members, sched_base, sched_rem;
    FastDiv div_n_splits;     // division by n_splits (fixed mode)
    FastDiv div_hkv;          // division by Hkv
    int32_t max_splits;
    int32_t adaptive_keys;    // adaptive mode: keys per split the split count is derived from
    float scale_log2;         // softmax scale * log2(e) (FP8 cache: times k_scale)
    float out_mul;            // factor on every normalised output row: 1, or v_scale of an FP8 cache
    unsigned long long* trace;  // optional [grid][kTraceEvents] timestamps (100 MHz), or null
    float* out;               // [B, Hq, D]
    float* lse;               // [B, Hq] or null
    float* part_o;            // [B*Hkv, max_splits, G, D]
    float* part_lse;          // [B*Hkv, max_splits, kLseStride], heads 0..G-1 used (log2 units)
    uint32_t* counters;       // [B*Hkv]
    uint32_t* status;         // [1] set non-zero by a waiting combine kernel that gave up
    uint32_t spin_limit;      // polls a waiting combine workgroup makes before it gives up
    const int32_t* block_table;  // paged cache: [B, pages_per_seq], pool page of each logical page; null = contiguous
    int32_t page_shift;       // log2(page_size)
    int32_t pages_per_seq;
    int32_t num_pages;
    // two-level combine (tiles with more than tree_rows partials, see tree_arrive)
    int32_t tree_rows;        // a tile with more live partials than this is merged in two levels; INT32_MAX = never
    float* part2_o;           // [B*Hkv, group_cap, G, D] results of the first level
    float* part2_lse;         // [B*Hkv, group_cap, kLseStride]
    uint32_t* group_counters; // [B*Hkv, kMaxGroups] arrivals per first-level group
    int32_t group_cap;        // first-level groups the workspace has room for per tile
    uint32_t* bsp_direct;     // [B*Hkv] bulk-synchronous mode: 1 = kernel 1 wrote the tile's final result itself
    int32_t bsp_groups;       // bulk-synchronous mode: workgroups per tile of kernel 2 (its gridDim.y)
};

// ---- optional in-kernel timeline (for tuning; off unless a buffer is attached) --
constexpr int kTraceEvents = 12;
enum { kEvStart = 0, kEvFirstStage = 1, kEvLoopEnd = 2, kEvPartialOut = 3, kEvStoresAcked = 4, kEvCounted = 5,
       kEvCombined = 6, kEvEnd = 7, kEvCombA = 8, kEvCombB = 9, kEvCombC = 10, kEvCombD = 11 };
__device__ __forceinline__ void trace_event(const Params& p, int ev)
{
    if (p.trace && threadIdx.x == 0) p.trace[(size_t)blockIdx.x * kTraceEvents + ev] = wall_clock64();
}
// the same with a time taken earlier (the kernel's entry is stamped after the prologue's requests
// have gone out: looking at p.trace first would put a dependent branch in front of them)
__device__ __forceinline__ void trace_event_at(const Params& p, int ev, unsigned long long t)
{
    if (p.trace && threadIdx.x == 0) p.trace[(size_t)blockIdx.x * kTraceEvents + ev] = t;
}

// Sequence length as the kernels use it: clamped into [0, S_max] so that a bad
// entry can never index outside the cache.
__device__ __forceinline__ int seq_len_of(const Params& p, int b)
{
    const int s = p.seq_lens[b];
    return s < 0 ? 0 : (s > p.S_max ? p.S_max : s);
}

// ---- split geometry (a split never starts inside a 64-key block) -----------
__device__ __forceinline__ int num_splits_of(const Params& p, int S)
{
    if (p.n_splits > 0) return p.n_splits;
    int n = (S + p.adaptive_keys - 1) / p.adaptive_keys;
    n = n < 1 ? 1 : n;
    return n > p.max_splits ? p.max_splits : n;
}

__host__ __device__ __forceinline__ int split_keys_of(int S, int n)
{
    int c = (S + n - 1) / n;
    c = (c + kSplitAlign - 1) / kSplitAlign * kSplitAlign;
    return c < kSplitAlign ? kSplitAlign : c;
}

// ---- persistent-grid work list ---------------------------------------------
// Workgroup w belongs to XCD group x = w % X (the hardware deals workgroups to
// the 8 XCDs round-robin, so with X = 8 a group is one XCD and its L2).  Group x
// owns tiles t = x, x+X, x+2X, ...; its items are those tiles' splits in order.
// Member wl = w / X of the group takes the contiguous block of items
// [wl*E/members, (wl+1)*E/members): consecutive splits of one tile become ONE
// longer key range (one partial, one arrival), and a workgroup streams long
// contiguous stretches of the cache.
struct WorkList {
    int x, wl, members, n_tiles, n_items;
    int base, rem;        // block w = [block_first(w), block_first(w + 1)): base items, one more in the first rem blocks
    int first, last;      // this workgroup's block of items [first, last)
};

// First item of block w when n_items items are dealt to `members` blocks as evenly as
// possible (32-bit arithmetic only: this is evaluated on latency-critical paths).
__device__ __forceinline__ int block_first(int w, int base, int rem) { return w * base + min(w, rem); }


struct Item {
    int tile, b, kvh, split, n, S;
};

// pre[] : exclusive prefix of split counts over the group's tiles (adaptive mode).
__device__ inline void worklist_init(const Params& p, WorkList& wlst, int* pre, int* scan_tmp)
{
    const int X = p.xcd_groups;
    const int T = p.B * p.Hkv;
    wlst.x = blockIdx.x & (X - 1);
    wlst.wl = blockIdx.x >> p.xcd_shift;
    if (p.n_splits > 0 && p.sched_uniform) {            // the usual case: nothing left to divide
        wlst.members = p.sched_members;
        wlst.n_tiles = T >> p.xcd_shift;
        wlst.n_items = wlst.n_tiles * p.n_splits;
        wlst.base = p.sched_base;
        wlst.rem = p.sched_rem;
        wlst.first = block_first(wlst.wl, wlst.base, wlst.rem);
        wlst.last = block_first(wlst.wl + 1, wlst.base, wlst.rem);
        return;
    }
    wlst.members = (p.grid - wlst.x + X - 1) >> p.xcd_shift;
    wlst.n_tiles = wlst.x < T ? (T - wlst.x + X - 1) >> p.xcd_shift : 0;
    if (p.n_splits > 0) {
        wlst.n_items = wlst.n_tiles * p.n_splits;
        wlst.base = wlst.n_items / wlst.members;
        wlst.rem = wlst.n_items - wlst.base * wlst.members;
        wlst.first = block_first(wlst.wl, wlst.base, wlst.rem);
        wlst.last = block_first(wlst.wl + 1, wlst.base, wlst.rem);
        return;
    }
    // adaptive: block-wide exclusive scan of n_b over the group's tiles
    const int tid = threadIdx.x;
    const int per = (wlst.n_tiles + kWgThreads - 1) / kWgThreads;
    const int lo = tid * per;
    int sum = 0;
    for (int k = lo; k < lo + per && k < wlst.n_tiles; ++k) {
        const int t = wlst.x + X * k;
        sum += num_splits_of(p, seq_len_of(p, (int)fast_div((uint32_t)t, p.div_hkv)));
    }
    scan_tmp[tid] = sum;
    __syncthreads();
    for (int off = 1; off < kWgThreads; off <<= 1) {
        const int add = tid >= off ? scan_tmp[tid - off] : 0;
        __syncthreads();
        scan_tmp[tid] += add;
        __syncthreads();
    }
    int run = scan_tmp[tid] - sum;
    for (int k = lo; k < lo + per && k < wlst.n_tiles; ++k) {
        pre[k] = run;
        const int t = wlst.x + X * k;
        run += num_splits_of(p, seq_len_of(p, (int)fast_div((uint32_t)t, p.div_hkv)));
    }
    if (tid == kWgThreads - 1) pre[wlst.n_tiles] = scan_tmp[tid];
    __syncthreads();
    wlst.n_items = pre[wlst.n_tiles];
    wlst.base = wlst.n_items / wlst.members;
    wlst.rem = wlst.n_items - wlst.base * wlst.members;
    wlst.first = block_first(wlst.wl, wlst.base, wlst.rem);
    wlst.last = block_first(wlst.wl + 1, wlst.base, wlst.rem);
}

// Which tile and split item e of a fixed-n_splits work list is: needs no sequence length, so a
// workgroup can aim its first K/V request before seq_lens has arrived.
__device__ __forceinline__ void fixed_item_place(const Params& p, const WorkList& wlst, int e, Item& it)
{
    const int k = (int)fast_div((uint32_t)e, p.div_n_splits);
    it.split = e - k * p.n_splits;
    it.tile = wlst.x + (k << p.xcd_shift);
    it.b = (int)fast_div((uint32_t)it.tile, p.div_hkv);
    it.kvh = it.tile - it.b * p.Hkv;
    it.n = p.n_splits;
}

// sl_first: seq_lens[lane] of the first 64 sequences, requested when the kernel starts, so
// that for B <= 64 the first item's length is not a load that the whole prologue waits for.
__device__ __forceinline__ Item worklist_item(const Params& p, const WorkList& wlst, const int* pre, int e, int sl_first)
{
    Item it;
    if (p.n_splits > 0) {
        fixed_item_place(p, wlst, e, it);
    } else {
        int lo = 0, hi = wlst.n_tiles;      // largest k with pre[k] <= e
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (pre[mid] <= e) lo = mid; else hi = mid;
        }
        it.split = e - pre[lo];
        it.tile = wlst.x + (lo << p.xcd_shift);
        it.b = (int)fast_div((uint32_t)it.tile, p.div_hkv);
        it.kvh = it.tile - it.b * p.Hkv;
    }
    if (p.B <= 64) {
        const int s = __builtin_amdgcn_readlane(sl_first, __builtin_amdgcn_readfirstlane(it.b));
        it.S = s < 0 ? 0 : (s > p.S_max ? p.S_max : s);
    } else {
        it.S = seq_len_of(p, it.b);
    }
    it.n = num_splits_of(p, it.S);
    return it;
}

// ---- small arithmetic helpers ------------------------------------------------
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// acc + a.lo*b.lo + a.hi*b.hi on packed bf16 pairs, fp32 accumulate (v_dot2c_f32_bf16)
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), acc, false);
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// 128-bit load of K/V data that is used once: the non-temporal hint keeps the
// stream from displacing useful lines and measurably raises read bandwidth.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream(const uint4* p)
{
    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// ---- exchange of partials between workgroups ----------------------------------
// A gfx950 device has 8 XCDs, each with its own L2 that is not kept coherent with the
// others.  An agent-scope release FENCE writes back a whole L2, far too heavy to run once
// per item.  A workgroup therefore WRITES its partial with agent-scope stores (sc1: written
// through to the device-coherent level) and keeps the order "partial, then counter" by
// waiting for the stores' acknowledgements (s_waitcnt vmcnt(0)) before the workgroup
// barrier that precedes the counter increment.
// The one workgroup that READS a tile's partials does so after it has seen the complete count,
// with ordinary loads and WITHOUT an acquire fence (an L2 invalidate costs 0.5-0.8 us on the
// critical tail of every call).  That is safe because no cache on the reader's side can hold
// a stale copy of what it reads:
//   * every slot owns whole 128-byte lines (a partial's o block is G x 512 bytes, its lse one
//     padded line of kLseStride floats), so no line is shared between two writers and a
//     local writer never pulls a neighbour's not-yet-written data into the local L2;
//   * a line of the partial buffer is read by nobody but its tile's combiner, once per
//     launch, after the last arrival: nothing can have fetched it earlier in this launch;
//   * what an earlier launch left in L1 / L2 is dropped at the launch boundary, as for any
//     kernel that reads what the previous kernel wrote from another XCD.
// No other data travels between workgroups in a launch.
__device__ __forceinline__ void store_agent(float* p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 16 bytes (16-byte aligned) in one coherent store
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_agent4(float* p, f32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ float load_agent(const float* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// the same wait, where it stands for "every K/V transfer this wave requested has landed in LDS"
__device__ __forceinline__ void wait_loads_landed() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}

// Sum over each row of 16 lanes (DPP only, every lane of the row gets the total).
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_f32<0xB1>(x);    // quad_perm [1,0,3,2]
    x += dpp_f32<0x4E>(x);    // quad_perm [2,3,0,1]
    x += dpp_f32<0x141>(x);   // row_half_mirror
    x += dpp_f32<0x140>(x);   // row_mirror
    return x;
}

// Maximum over each row of 16 lanes (DPP only, every lane of the row gets it).
__device__ __forceinline__ float row16_max(float x)
{
    x = fmaxf(x, dpp_f32<0xB1>(x));
    x = fmaxf(x, dpp_f32<0x4E>(x));
    x = fmaxf(x, dpp_f32<0x141>(x));
    x = fmaxf(x, dpp_f32<0x140>(x));
    return x;
}

// Maximum / sum over the 4 lanes {i, i ^ 16, i ^ 32, i ^ 48} (in the MFMA kernels: the 4 key
// groups of one query head), every one of them gets the result, with no trip through LDS.
// v_permlane16_swap exchanges the odd 16-lane rows of its first operand with the even rows of
// its second, v_permlane32_swap the upper half of the first with the lower half of the second;
// fed the same value twice they return the two partners of every pair side by side.
// Written as asm: through the compiler's builtins the max of the two results is folded away
// (it takes them for equal).  The s_nop covers the wait states these instructions need after a
// VALU write of their operands.
__device__ __forceinline__ void rows_swap16(float& a, float& b)
{
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void rows_swap32(float& a, float& b)
{
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float head_lanes_max(float x)
{
    float a = x, b = x;
    rows_swap16(a, b);
    a = b = fmaxf(a, b);
    rows_swap32(a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ float head_lanes_sum(float x)
{
    float a = x, b = x;
    rows_swap16(a, b);
    a = b = a + b;
    rows_swap32(a, b);
    return a + b;
}

// ---- end of an item: merge the workgroup's 4 wave states, normalise, store ------
// Each wave leaves its running max m, sum l and unnormalised accumulator for the
// ROWS query heads of the tile here; all in base-2 units.
template <int ROWS>
struct ItemSmem {
    float m[ROWS][kWaves];
    float l[ROWS][kWaves];
    float acc[kWaves][ROWS][kD];
};

// a6: o = sum_w acc_w 2^(m_w - M) / sum_w l_w 2^(m_w - M), lse = M + log2(sum).
// SHARED: the destination is a partial another workgroup may read in this launch
// (coherent stores).  Call with the wave states written and a barrier passed;
// returns with every thread past its last read of sm.  A thread produces 4 dims of
// one head: this tail runs with one wave per SIMD, where every instruction counts.
template <int ROWS, bool SHARED>
__device__ inline void item_finish(const ItemSmem<ROWS>& sm, int G, float* dst_o, float* dst_lse, float lse_mul,
                                   float out_mul = 1.0f)
{
    static_assert(kWaves == 4, "the wave states of a head are read as one float4");
#pragma nounroll
    for (int idx = threadIdx.x; idx < G * (kD / 4); idx += kWgThreads) {
        const int g = idx >> 5, d4 = idx & 31;
        const float4 mv = *reinterpret_cast<const float4*>(sm.m[g]);
        const float4 lv = *reinterpret_cast<const float4*>(sm.l[g]);
        const float M = fmaxf(fmaxf(mv.x, mv.y), fmaxf(mv.z, mv.w));
        const float f[4] = {fast_exp2(mv.x - M), fast_exp2(mv.y - M), fast_exp2(mv.z - M), fast_exp2(mv.w - M)};
        const float L = (lv.x * f[0] + lv.y * f[1]) + (lv.z * f[2] + lv.w * f[3]);
        f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float4 a = *reinterpret_cast<const float4*>(&sm.acc[w][g][4 * d4]);
            o[0] += a.x * f[w];
            o[1] += a.y * f[w];
            o[2] += a.z * f[w];
            o[3] += a.w * f[w];
        }
        o *= __builtin_amdgcn_rcpf(L) * out_mul;
        const float res_lse = (M + fast_log2(L)) * lse_mul;
        if (SHARED) {
            store_agent4(&dst_o[4 * idx], o);
            if (d4 == 0) store_agent(&dst_lse[g], res_lse);
        } else {
            *reinterpret_cast<f32x4*>(&dst_o[4 * idx]) = o;
            if (d4 == 0 && dst_lse) dst_lse[g] = res_lse;
        }
    }
    __syncthreads();
}

// ---- Combine (Algorithm 4, Part 2), one workgroup per tile -------------------
// Merges the partials of tile (b, kvh) into out / lse.  Of the tile's n slots only
// the "live" ones hold a partial: a workgroup that attended several consecutive
// splits in one go wrote a single partial into the first slot and lse = -inf
// into the others (as it does for splits with no keys).  Rows are merged in
// ascending slot order within fixed row slices, so the result does not depend
// on which workgroup runs this.
constexpr int kMaxSplits = 1024;

constexpr int kCombineWCap = 4096;     // weights staged in LDS: heads x (live rows, padded)
constexpr int kCombineGroup = 8;       // rows are loaded and padded in groups of this many
constexpr int kTreeGroup = 16;         // two-level combine: partials merged by one first-level combine
constexpr int kMaxGroups = 64;         // first-level groups per tile (kMaxSplits / kTreeGroup)
constexpr int kTreeRowsDefault = 64;   // tiles with more live partials than this are merged in two levels

// The slots of a tile that hold a partial, in ascending order: row k at
// [(k % R) * stride + k / R] (R row slices, see combine_tile).  Kept apart from the combine's
// scratch: the fused kernel fills it while its K/V ring (which the scratch overlays) is in use.
struct LiveList {
    int live[kMaxSplits + 8 * 32];
    int n_live;
    int my_rank;        // position of this workgroup's own partial in the list (combine_live_from_schedule), -1 if it has none
};

struct CombineSmem {
    float w[kCombineWCap];      // exp2(lse - max) of row k of head g at [((g * R) + k % R) * KJ + k / R], 0 in the padding
    float invL[16];             // per head
    float4 red[kWgThreads];     // cross-slice reduction
};

// Fallback of combine_tile for a tile whose weights do not fit the LDS staging area
// (roughly more than kCombineWCap / G live partials): same formulas, every lse re-read
// from memory.  Correct and slow; kept out of line of the fast path.
__device__ inline void combine_tile_unstaged(const float* plse, const float* po, float* out_rows, float* lse_rows,
                                                   int G, int n_live, const int* live, int log_r, int stride)
{
    const float4* po4 = reinterpret_cast<const float4*>(po);
    const auto slot = [&](int k) { return live[(k & ((1 << log_r) - 1)) * stride + (k >> log_r)]; };
    for (int pair = threadIdx.x; pair < G * (kD / 4); pair += kWgThreads) {
        const int g = pair / (kD / 4), d4 = pair % (kD / 4);
        float M = -INFINITY, L = 0.f;
#pragma nounroll
        for (int k = 0; k < n_live; ++k) M = fmaxf(M, plse[slot(k) * kLseStride + g]);
#pragma nounroll
        for (int k = 0; k < n_live; ++k) L += fast_exp2(plse[slot(k) * kLseStride + g] - M);
        const float invL = __builtin_amdgcn_rcpf(L);
        float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma nounroll
        for (int k = 0; k < n_live; ++k) {
            const float w = fast_exp2(plse[slot(k) * kLseStride + g] - M);
            const float4 x = po4[(size_t)(slot(k) * G + g) * (kD / 4) + d4];
            o.x += w * x.x; o.y += w * x.y; o.z += w * x.z; o.w += w * x.w;
        }
        o.x *= invL; o.y *= invL; o.z *= invL; o.w *= invL;
        reinterpret_cast<float4*>(out_rows)[pair] = o;
        if (d4 == 0 && lse_rows) lse_rows[g] = (M + fast_log2(L)) * kLn2;
    }
}

// Combine of one tile (Algorithm 4 Part 2: the log-sum-exp merge of the partials) by the workgroup
// that saw the last arrival.  BATCH = rows whose loads a thread keeps in flight (a
// multiple of kCombineGroup).
//
// This runs once per tile on the critical path of the call's tail, on ONE workgroup with
// one wave per SIMD.  Two things cost time there: dependent memory round trips (0.4-1 us
// each while the rest of the chip is still streaming) and instructions (a lone wave
// retires only ~250 of them per microsecond).  Hence:
//   1. the list of live slots is there already (fused kernel: derived from the schedule
//      while the K/V stream ran) or wave 0 reads head 0's lse of every slot, up to 4 slots
//      per lane in flight, and lists the live ones in ascending order;
//   2. no acquire fence (see "exchange of partials" above): ordinary loads, which pull rows
//      ~1.7x faster than coherent ones;
//   3. one round trip: each thread requests its first BATCH rows of o; meanwhile 16 lanes
//      per head fetch that head's lse values, reduce max and sum with DPP, and leave the
//      rows' weights in LDS (zero in the padding, so the row loop needs no bounds logic);
//   4. the row loop is a load, a 64-bit multiply-add for the address and four FMAs per row.
// A thread owns 4 output dims of one head.  With fewer than 256 such pairs (G < 8), R
// threads share a pair, thread slice s taking rows s, s+R, ...; the slices are summed
// through LDS.  Rows are taken in ascending order within a slice and slices in ascending
// order, so for a given partition the result does not depend on which workgroup runs this.
// What the combining workgroup of the fused kernel knows about who wrote the tile's
// partials: the tile's items are [t0, t0 + n) of a work list cut into `members` contiguous
// blocks (see WorkList, block_first); block w wrote one partial, into the slot of its first
// item of this tile, if it holds any of the tile's items and that item's key range is not
// empty.
struct TileSchedule {
    int t0, base, rem, members, split_keys, S;
};

// Row slices of a combine: R = 2^log_r threads share one (head, 4 dims) pair, R the largest
// power of two with R * G * 32 <= 256.
__device__ __forceinline__ int combine_log_r(int G) { return G >= 5 ? 0 : G >= 3 ? 1 : G == 2 ? 2 : 3; }
__device__ __forceinline__ int combine_live_stride(int log_r) { return (kMaxSplits >> log_r) + 32; }

// Pads the live list to whole row groups (the padding re-reads the first live row with weight 0)
// and publishes the count.  Wave 0 only.
__device__ __forceinline__ void combine_live_finish(LiveList& sm, int count, int live0, int log_r, int lane)
{
    const int R = 1 << log_r, stride = combine_live_stride(log_r);
    for (int k = count + lane; k < count + R * (kCombineGroup + 1); k += 64)
        sm.live[(k & (R - 1)) * stride + (k >> log_r)] = live0;
    if (lane == 0) sm.n_live = count;
}

// The live slots of a tile of the fused kernel follow from the schedule: no memory access.
// Wave 0 only (all 64 lanes).  It depends on nothing another workgroup does, so the fused kernel
// runs it early, while the wave would otherwise wait for K/V data in flight.
__device__ inline void combine_live_from_schedule(LiveList& sm, const TileSchedule& sch, int n, int G, int my_block)
{
    const int lane = threadIdx.x & 63;
    const int log_r = combine_log_r(G), R = 1 << log_r, stride = combine_live_stride(log_r);
    int count = 0, live0 = 0;
    if (lane == 0) sm.my_rank = -1;
    // Candidate blocks: a range that surely contains every block holding an item of [t0, t0 + n)
    // (block w starts at or after w * base and before (w + 1) * (base + 1))
    const int t0 = sch.t0, members = sch.members;
    int w_first = 0, w_end = members;
    if (sch.base > 0) {
        w_first = max(0, (int)((float)t0 * __builtin_amdgcn_rcpf((float)(sch.base + 1))) - 1);
        w_end = min(members, (int)((float)(t0 + n) * __builtin_amdgcn_rcpf((float)sch.base)) + 2);
    }
#pragma nounroll
    for (int w0 = w_first; w0 < w_end; w0 += 64) {
        const int w = w0 + lane;
        const int lo = max(block_first(w, sch.base, sch.rem), t0);
        const int hi = min(block_first(w + 1, sch.base, sch.rem), t0 + n);
        const bool live = w < w_end && lo < hi && (long long)(lo - t0) * sch.split_keys < sch.S;
        const unsigned long long mask = __ballot(live);
        const int k = count + __popcll(mask & ((1ull << lane) - 1ull));
        if (live) sm.live[(k & (R - 1)) * stride + (k >> log_r)] = lo - t0;
        if (live && w == my_block) sm.my_rank = k;
        if (count == 0 && mask != 0) live0 = __builtin_amdgcn_readlane(lo - t0, __builtin_ctzll(mask));
        count += __popcll(mask);
    }
    combine_live_finish(sm, count, live0, log_r, lane);
}

struct CombineArgs {
    const float* plse;      // lse lines of the rows to merge
    const float* po;        // their o blocks
    float* out_rows;
    float* lse_rows;        // or null
    int G, n_live, KJ, log_r, stride;
    bool to_partial;        // the result is itself a partial another workgroup will merge: coherent stores,
                            // lse left in base-2 units (two-level combine, first level)
};

// Stores of a combine's result.
__device__ __forceinline__ void combine_store_o(const CombineArgs& a, int pair, float4 o)
{
    if (a.to_partial) store_agent4(a.out_rows + 4 * pair, f32x4{o.x, o.y, o.z, o.w});
    else reinterpret_cast<float4*>(a.out_rows)[pair] = o;
}

// Second half of combine_tile: weights, row loop, output.  NR0 = rows in a thread's first batch
// = min(BATCH, KJ), a template parameter so that every thread issues exactly NL lse loads and then
// exactly NR0 row loads, unconditionally: the compiler can then wait for the lse values alone
// (vmcnt = the number of younger row loads) and the weights are computed while the rows are still
// arriving.  Every load costs the compute unit's one address unit some tens of cycles whether it
// brings a live row or padding, so the padding is kept small (KJ = 1, 2, 4 or a multiple of 8).
// Threads with no (head, dims) pair of their own load the rows of pair 0 and drop them.
template <int BATCH, int NR0>
__device__ __forceinline__ void combine_rows(const Params& p, const CombineArgs& a, CombineSmem& sm, const LiveList& ll, int tid)
{
    static_assert(NR0 >= 1 && NR0 <= BATCH, "first batch");
    // lse loads per statistics lane (16 rows each): with at most 2 rows per slice there are at
    // most 8 * 2 = 16 live rows
    constexpr int NL = NR0 <= 2 ? 1 : 4;
    const int G = a.G, n_live = a.n_live, KJ = a.KJ, log_r = a.log_r, stride = a.stride;
    const int R = 1 << log_r;
    const int kPairs = G * (kD / 4);
    // thread -> (pair, slice) without an integer division
    const int slice = (int)(((tid >> 5) + 0.5f) * __builtin_amdgcn_rcpf((float)G));
    const int pair0 = tid - slice * kPairs;
    const size_t row_f4 = (size_t)G * (kD / 4);          // float4 per slot
    const float4* po4 = reinterpret_cast<const float4*>(a.po);
    const bool active0 = slice < R && pair0 < kPairs;
    const int* my_live = &ll.live[(active0 ? slice : 0) * stride];

    // weights: 16 lanes per head, lane j takes rows j, j+16, ...; the lse loads go out first
    const bool stat_lane = (tid >> 4) < G;
    const int sg = stat_lane ? tid >> 4 : 0, sj = tid & 15;
    const auto live_at = [&](int k) { return ll.live[(k & (R - 1)) * stride + (k >> log_r)]; };
    if (n_live > 64 && stat_lane) {                      // rows past the first 64: rare, staged through LDS
        float* wg = &sm.w[sg * R * KJ];
#pragma nounroll
        for (int k = sj + 64; k < n_live; k += 16) wg[(k & (R - 1)) * KJ + (k >> log_r)] = a.plse[live_at(k) * kLseStride + sg];
    }
    float v[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int k = sj + 16 * i;
        v[i] = a.plse[live_at(k < n_live ? k : 0) * kLseStride + sg];
    }

    float4 x[BATCH];
    {
        const int pair = active0 ? pair0 : 0;
#pragma unroll
        for (int j = 0; j < NR0; ++j) x[j] = po4[my_live[j] * row_f4 + pair];
    }
    const auto load_rows = [&](int j0, int pair) {       // groups of rows [j0, j0 + BATCH) below KJ
#pragma unroll
        for (int grp = 0; grp < BATCH / kCombineGroup; ++grp) {
            if (j0 + grp * kCombineGroup < KJ) {
#pragma unroll
                for (int u = 0; u < kCombineGroup; ++u) {
                    const int j = grp * kCombineGroup + u;
                    x[j] = po4[my_live[j0 + j] * row_f4 + pair];
                }
            }
        }
    };

    if (stat_lane) {
        float* wg = &sm.w[sg * R * KJ];
        const auto at = [&](int k) { return (k & (R - 1)) * KJ + (k >> log_r); };
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (sj + 16 * i >= n_live) v[i] = -INFINITY;
        float m = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
#pragma nounroll
        for (int k = sj + 64; k < n_live; k += 16) m = fmaxf(m, wg[at(k)]);
        const float M = row16_max(m);
        float l = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = sj + 16 * i;
            if (k < R * KJ) {
                const float e = fast_exp2(v[i] - M);     // 0 for the padding (v = -inf)
                wg[at(k)] = e;
                l += e;
            }
        }
#pragma nounroll
        for (int k = sj + 64; k < R * KJ; k += 16) {
            const float e = k < n_live ? fast_exp2(wg[at(k)] - M) : 0.f;
            wg[at(k)] = e;
            l += e;
        }
        const float L = row16_sum(l);
        if (sj == 0) {
            sm.invL[sg] = __builtin_amdgcn_rcpf(L);
            if (a.to_partial) store_agent(&a.lse_rows[sg], M + fast_log2(L));
            else if (a.lse_rows) a.lse_rows[sg] = (M + fast_log2(L)) * kLn2;
        }
    }
    __syncthreads();
    trace_event(p, kEvCombC);

#pragma nounroll
    for (int pbase = 0; pbase < kPairs; pbase += kWgThreads) {
        const int pair = pbase + pair0;
        const bool active = slice < R && pair < kPairs;
        float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
        if (active) {
            const int g = pair >> 5;
            const float* my_w = &sm.w[(g * R + slice) * KJ];
            if (pbase > 0) load_rows(0, pair);
            // first batch: NR0 rows, known to lie below KJ
#pragma unroll
            for (int j = 0; j < NR0; ++j) {
                const float w = my_w[j];
                o.x += w * x[j].x;
                o.y += w * x[j].y;
                o.z += w * x[j].z;
                o.w += w * x[j].w;
            }
            // further batches (more than BATCH rows per slice: rare)
#pragma nounroll
            for (int j0 = BATCH; j0 < KJ; j0 += BATCH) {
                load_rows(j0, pair);
#pragma unroll
                for (int grp = 0; grp < BATCH / kCombineGroup; ++grp) {
                    if (j0 + grp * kCombineGroup < KJ) {
#pragma unroll
                        for (int u = 0; u < kCombineGroup; ++u) {
                            const int j = grp * kCombineGroup + u;
                            const float w = my_w[j0 + j];
                            o.x += w * x[j].x;
                            o.y += w * x[j].y;
                            o.z += w * x[j].z;
                            o.w += w * x[j].w;
                        }
                    }
                }
            }
            const float invL = sm.invL[g];
            o.x *= invL; o.y *= invL; o.z *= invL; o.w *= invL;
        }
        trace_event(p, kEvCombD);
        if (R > 1) {
            sm.red[tid] = o;
            __syncthreads();
            if (active && slice == 0) {
#pragma nounroll
                for (int r = 1; r < R; ++r) {
                    const float4 t = sm.red[r * kPairs + pair];
                    o.x += t.x; o.y += t.y; o.z += t.z; o.w += t.w;
                }
                combine_store_o(a, pair, o);
            }
        } else if (active) {
            combine_store_o(a, pair, o);
        }
    }
}

// The live rows among n candidates, found by reading head 0's lse of each (a row without a partial
// holds -inf there).  Wave 0 only (all 64 lanes).
__device__ __forceinline__ void combine_live_from_memory(LiveList& ll, const float* plse, int n, int G)
{
    const int lane = threadIdx.x & 63;
    const int log_r = combine_log_r(G), R = 1 << log_r, stride = combine_live_stride(log_r);
    int count = 0, live0 = 0;
#pragma nounroll
    for (int base = 0; base < n; base += 256) {          // one trip up to 256 slots
        float first[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = base + j * 64 + lane;
            first[j] = load_agent(&plse[min(i, n - 1) * kLseStride]);     // unconditional: the 4 loads fly together
            if (i >= n) first[j] = -INFINITY;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (base + j * 64 < n) {
                const bool live = first[j] != -INFINITY;
                const unsigned long long mask = __ballot(live);
                const int k = count + __popcll(mask & ((1ull << lane) - 1ull));
                if (live) ll.live[(k & (R - 1)) * stride + (k >> log_r)] = base + j * 64 + lane;
                if (count == 0 && mask != 0) live0 = base + j * 64 + __builtin_ctzll(mask);
                count += __popcll(mask);
            }
        }
    }
    combine_live_finish(ll, count, live0, log_r, lane);
}

// What a combine merges and where the result goes.
struct CombineJob {
    const float* plse;      // lse lines of the candidate rows (row i at plse + i * kLseStride)
    const float* po;        // their o blocks (row i at po + i * G * kD)
    float* out_rows;        // [G][kD]
    float* lse_rows;        // [G] or null (never null with to_partial)
    int n;                  // candidate rows (slots) to scan when the live list is not there yet
    bool to_partial;        // see CombineArgs
};

// live_ready: the live list is already in ll (combine_live_from_schedule, or a caller's own
// list); otherwise wave 0 finds the live rows by reading head 0's lse of every candidate.
template <int BATCH>
__device__ __forceinline__ void combine_core(const Params& p, const CombineJob& job, CombineSmem& sm, LiveList& ll,
                                             bool live_ready)
{
    static_assert(BATCH % kCombineGroup == 0 && BATCH <= 32, "row batch");
    const int G = p.G;          // <= 16
    // Opaque to the optimiser: everything below that depends on the thread index is then
    // computed here, not hoisted out of the caller's loop into registers that would stay
    // occupied during the K/V streaming.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const float* plse = job.plse;
    const float* po = job.po;
    float* out_rows = job.out_rows;
    float* lse_rows = job.lse_rows;
    const int n = job.n;

    const int log_r = combine_log_r(G);
    const int R = 1 << log_r;
    const int stride = combine_live_stride(log_r);       // of one slice's live list

    if (tid < 64 && !live_ready) combine_live_from_memory(ll, plse, n, G);
    trace_event(p, kEvCombA);
    __syncthreads();
    const int n_live = ll.n_live;
    trace_event(p, kEvCombB);
    if (n_live == 0) {                                   // no key anywhere in the tile
        for (int i = tid; i < G * kD; i += kWgThreads) out_rows[i] = 0.f;
        if (tid < G && lse_rows) lse_rows[tid] = -INFINITY;
        __syncthreads();
        return;
    }
    // rows per slice, padded to 1, 2, 4 or whole groups
    const int per_slice = (n_live + R - 1) >> log_r;
    const int KJ = per_slice <= 2 ? per_slice : per_slice <= 4 ? 4 : (per_slice + kCombineGroup - 1) & ~(kCombineGroup - 1);
    if (G * R * KJ > kCombineWCap) {
        combine_tile_unstaged(plse, po, out_rows, lse_rows, G, n_live, ll.live, log_r, stride);
        __syncthreads();
        return;
    }

    // the rest is compiled once per number of rows in a thread's first batch, so that the
    // number of row loads between the lse loads and their first use is a compile-time constant
    const CombineArgs a = {plse, po, out_rows, lse_rows, G, n_live, KJ, log_r, stride, job.to_partial};
    switch (min(BATCH, KJ)) {
        case 1: combine_rows<BATCH, 1>(p, a, sm, ll, tid); break;
        case 2: combine_rows<BATCH, 2>(p, a, sm, ll, tid); break;
        case 4: combine_rows<BATCH, 4>(p, a, sm, ll, tid); break;
        case 8: combine_rows<BATCH, 8>(p, a, sm, ll, tid); break;
        case 16: combine_rows<BATCH, (BATCH >= 16 ? 16 : 8)>(p, a, sm, ll, tid); break;
        case 24: combine_rows<BATCH, (BATCH >= 24 ? 24 : 8)>(p, a, sm, ll, tid); break;
        default: combine_rows<BATCH, (BATCH >= 32 ? 32 : 8)>(p, a, sm, ll, tid); break;
    }
    __syncthreads();
}

// The flat combine of tile (b, kvh): its n slots' partials into out / lse.
template <int BATCH>
__device__ __forceinline__ void combine_tile(const Params& p, int tile, int b, int kvh, int n, CombineSmem& sm, LiveList& ll,
                                             bool live_ready = false)
{
    const int G = p.G;
    const CombineJob job = {p.part_lse + (size_t)tile * p.max_splits * kLseStride,
                            p.part_o + (size_t)tile * p.max_splits * G * kD,
                            p.out + ((size_t)b * p.Hq + (size_t)kvh * G) * kD,
                            p.lse ? p.lse + (size_t)b * p.Hq + (size_t)kvh * G : nullptr,
                            n, false};
    combine_core<BATCH>(p, job, sm, ll, live_ready);
}

// ---- Two-level combine -------------------------------------------------------------------
// One compute unit pulls partial rows at some 50 GB/s, so a tile with hundreds of partials (one
// long sequence on one or two KV heads, cut over the whole chip) would spend longer in its
// combine than in the K/V stream.  Such a tile is merged in two levels, still without anybody
// waiting: its live partials, in ascending slot order, form groups of kTreeGroup; a group has an
// arrival counter of its own; the workgroup that completes a group's count merges the group's
// rows into ONE partial of a second buffer (coherent stores, base-2 lse, like any partial) and
// then counts the group as arrived at the tile's counter; whoever completes that count merges the
// groups' results into out / lse.  Groups follow from the schedule alone and every merge takes
// its rows in ascending order, so the result does not depend on who merges, and the
// bulk-synchronous kernel 2 (one workgroup per group) computes the same bits.

// Wave 0: the live list becomes its own rows [first, first + count), count <= 64.
__device__ __forceinline__ void tree_sublist(LiveList& ll, int first, int count, int G)
{
    const int lane = threadIdx.x & 63;
    const int log_r = combine_log_r(G), R = 1 << log_r, stride = combine_live_stride(log_r);
    const int k = first + lane;
    // every lane reads its entry before any lane writes (one instruction each, in order)
    const int slot = lane < count ? ll.live[(k & (R - 1)) * stride + (k >> log_r)] : 0;
    const int slot0 = __builtin_amdgcn_readfirstlane(slot);
    if (lane < count) ll.live[(lane & (R - 1)) * stride + (lane >> log_r)] = slot;
    combine_live_finish(ll, count, slot0, log_r, lane);
}

// Wave 0: the live list 0, 1, ..., count - 1 (the groups' results, all live).
__device__ __forceinline__ void tree_identity_list(LiveList& ll, int count, int G)
{
    const int lane = threadIdx.x & 63;
    const int log_r = combine_log_r(G), R = 1 << log_r, stride = combine_live_stride(log_r);
#pragma nounroll
    for (int k = lane; k < count; k += 64) ll.live[(k & (R - 1)) * stride + (k >> log_r)] = k;
    combine_live_finish(ll, count, 0, log_r, lane);
}

// The whole workgroup: merges first-level group `grp` of tile (b, kvh), whose m > kTreeGroup live
// partials are listed in ll and all written, counts the group at the tile's counter and, if
// that completes the tile, merges the groups' results into out / lse.  `flag`: a word of LDS.
template <int BATCH>
__device__ __forceinline__ void tree_merge_group(const Params& p, int tile, int b, int kvh, int grp, int m,
                                                 CombineSmem& sm, LiveList& ll, int* flag)
{
    const int G = p.G;
    const int first = grp * kTreeGroup;
    const int gsize = min(kTreeGroup, m - first);
    const int n_groups = (m + kTreeGroup - 1) / kTreeGroup;
    const size_t base2 = (size_t)tile * p.group_cap;
    // level 0: the group's rows into the second buffer; level 1 (only for the workgroup that
    // completes the tile's count of groups): the groups' results into out / lse.  One loop, so
    // that the combine is compiled into the kernel once for both.
#pragma nounroll
    for (int level = 0; level < 2; ++level) {
        if (threadIdx.x < 64) {
            if (level == 0) tree_sublist(ll, first, gsize, G);
            else tree_identity_list(ll, n_groups, G);
        }
        CombineJob job;
        if (level == 0) {
            job = {p.part_lse + (size_t)tile * p.max_splits * kLseStride, p.part_o + (size_t)tile * p.max_splits * G * kD,
                   p.part2_o + (base2 + grp) * G * kD, p.part2_lse + (base2 + grp) * kLseStride, 0, true};
        } else {
            job = {p.part2_lse + base2 * kLseStride, p.part2_o + base2 * G * kD,
                   p.out + ((size_t)b * p.Hq + (size_t)kvh * G) * kD,
                   p.lse ? p.lse + (size_t)b * p.Hq + (size_t)kvh * G : nullptr, 0, false};
        }
        combine_core<BATCH>(p, job, sm, ll, true);
        if (level == 1) {
            if (threadIdx.x == 0)                               // re-arm for the next call
                __hip_atomic_store(&p.counters[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
        }
        // the group's result went out with coherent stores: acknowledged, then counted
        wait_stores_done();
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t old = __hip_atomic_fetch_add(&p.counters[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = old + 1u == (uint32_t)n_groups;
        }
        __syncthreads();
        if (!*flag) break;
    }
    __syncthreads();
}

// Fused kernel: this workgroup's partial, number `rank` of the tile's m live ones, is written and
// acknowledged and the workgroup has passed a barrier.  Counts it at its group; the workgroup
// that completes the group goes on with tree_merge_group.
template <int BATCH>
__device__ __forceinline__ void tree_arrive(const Params& p, int tile, int b, int kvh, int rank, int m,
                                            CombineSmem& sm, LiveList& ll, int* flag)
{
    const int grp = rank / kTreeGroup;
    const int gsize = min(kTreeGroup, m - grp * kTreeGroup);
    uint32_t* gc = &p.group_counters[(size_t)tile * kMaxGroups + grp];
    if (threadIdx.x == 0) {
        const uint32_t old = __hip_atomic_fetch_add(gc, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = old + 1u == (uint32_t)gsize;
        if (last) __hip_atomic_store(gc, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);     // re-arm for the next call
        *flag = last;
    }
    __syncthreads();
    if (*flag) tree_merge_group<BATCH>(p, tile, b, kvh, grp, m, sm, ll, flag);
    else __syncthreads();
}

}  // namespace fd
