// libfd.so: kernels' entry points and the C ABI declared in include/fd.h.
// gfx950 (MI355X) only.

#include "../../include/fd.h"

#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <chrono>
#include <mutex>
#include <new>

#include "fd_device.hpp"
#include "fd_valu.hpp"
#include "fd_mfma.hpp"
#include "fd_mfma8.hpp"

// Workspace of fd_decode_static (the entry point for callers that cannot allocate): partials,
// their log-sum-exps and the arrival counters of ONE call at a time, laid out as a handle's
// workspace.  Each GPU the library runs on holds its own copy at its own address until the
// process ends.  Host code never uses this name as an address: it asks the runtime for the
// copy's device address once per device (static_device_state) and passes that pointer on.
static __device__ __align__(256) unsigned char scratch[FD_STATIC_SCRATCH_BYTES];

namespace fd {

// ---------------------------------------------------------------------------
// Kernels
// ---------------------------------------------------------------------------

// Sets n 32-bit words (arrival counters and status word to zero; the partial buffers to a NaN
// pattern for the debug call).  A kernel, not a memset: a caller may be recording the stream
// into a graph.
__global__ __launch_bounds__(kWgThreads) void fd_fill_words_kernel(uint32_t* dst, size_t n, uint32_t value)
{
    for (size_t i = (size_t)blockIdx.x * kWgThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kWgThreads) dst[i] = value;
}

// How a workgroup attends one key range: on the vector ALUs ...
template <int G>
struct ValuPath {
    static constexpr bool kPrefetch = false;
    ItemSmem<G>* sm;
    __device__ __forceinline__ void prefetch(const Params&, int, int, int, int, MfmaPrefetch&) const {}
    template <bool SHARED, class Hook>
    __device__ __forceinline__ void item(const Params& p, int b, int kvh, int j0, int j1, float* o, float* l,
                                         float mul, MfmaPrefetch&, const Hook& hook) const
    {
        if (threadIdx.x < 64) hook();
        valu_item<G, SHARED>(p, b, kvh, j0, j1, o, l, mul, *sm);
    }
};

// ... or on the matrix cores, through an LDS ring of NST stages per wave.  With a contiguous
// cache the first key range's first stages can be requested before the range's end is known.
template <int NST, bool PAGED, bool F16>
struct MfmaPath {
    static constexpr bool kPrefetch = !PAGED;
    char* ring;
    __device__ __forceinline__ void prefetch(const Params& p, int b, int kvh, int j0, int j1_max, MfmaPrefetch& pf) const
    {
        mfma_prefetch<NST>(p, b, kvh, j0, j1_max, ring, pf);
    }
    template <bool SHARED, class Hook>
    __device__ __forceinline__ void item(const Params& p, int b, int kvh, int j0, int j1, float* o, float* l,
                                         float mul, MfmaPrefetch& pf, const Hook& hook) const
    {
        mfma_item<NST, PAGED, F16, SHARED>(p, b, kvh, j0, j1, o, l, mul, ring, pf, hook);
    }
};

template <int NST, bool PAGED>
struct Mfma8Path {
    static constexpr bool kPrefetch = !PAGED;
    char* ring;
    __device__ __forceinline__ void prefetch(const Params& p, int b, int kvh, int j0, int j1_max, MfmaPrefetch& pf) const
    {
        mfma8_prefetch<NST>(p, b, kvh, j0, j1_max, ring, pf);
    }
    template <bool SHARED, class Hook>
    __device__ __forceinline__ void item(const Params& p, int b, int kvh, int j0, int j1, float* o, float* l,
                                         float mul, MfmaPrefetch& pf, const Hook& hook) const
    {
        mfma8_item<NST, PAGED, SHARED>(p, b, kvh, j0, j1, o, l, mul, ring, pf, hook);
    }
};

struct SchedSmem {
    int pre[kMaxGroupTiles + 1];
    int scan_tmp[kWgThreads];
    int is_last;
    LiveList live;
};

// What a workgroup does after a partial: nothing (kernel 1 of the bulk-synchronous
// baseline), count and combine if last (the fused kernel), or count only (kernel 1 of the
// fine-grained-waits variant, whose combine kernel waits for the counts).
constexpr int kModeBsp = 0, kModeFused = 1, kModeSignal = 2;
// Counter value of a tile whose result kernel 1 wrote itself (fine-grained waits).
constexpr uint32_t kTileDirect = 0x80000000u;

// The persistent loop of a workgroup.  kModeFused: work decomposition to combine in one
// launch (the workgroup that completes a tile's split count merges the tile: paper Section
// 4.2.5 / Algorithm 4 without the barrier and without the second launch).  kModeBsp: up to
// the partial only (kernel 1 of the bulk-synchronous baseline, Section 4.2.2).  kModeSignal:
// partial and arrival count (kernel 1 of the fine-grained-waits variant, Section 4.2.4).
template <int MODE, int COMB_BATCH, class Path>
__device__ __forceinline__ void persistent_loop(const Params& p, const Path& path, SchedSmem& ss, CombineSmem& comb)
{
    const unsigned long long t_entry = wall_clock64();
    // Ask for every line of the argument block at once: left alone, the compiler fetches each
    // field at its first use, three dependent scalar-cache misses in a row (0.25 us each)
    // before the first K/V request can go out.
    asm volatile("" ::"s"(p.trace), "s"(p.part_o), "s"(p.block_table), "s"(p.num_pages), "s"(p.tree_rows));
    const int G = p.G;
    const int lane = threadIdx.x & 63;
    const int sl_first = lane < p.B ? p.seq_lens[lane] : 0;     // in flight during the work-list arithmetic
    WorkList wl;
    worklist_init(p, wl, ss.pre, ss.scan_tmp);

    int e = wl.first;
    // Fixed n_splits: where the first key range starts does not depend on the sequence length
    // (splits are cut from S_max), so q and the first stage of every wave are requested now,
    // while seq_lens is still on its way; the range's end is settled when it arrives.
    MfmaPrefetch pf;
    pf.reset();
    if (Path::kPrefetch && p.n_splits > 0 && e < wl.last) {
        Item it0;
        fixed_item_place(p, wl, e, it0);
        const int s1 = min(p.n_splits, it0.split + (wl.last - e));
        const int j0 = it0.split * p.split_keys;
        const int j1_max = min(s1 * p.split_keys, p.S_max);
        if (j0 < j1_max)
            path.prefetch(p, __builtin_amdgcn_readfirstlane(it0.b), __builtin_amdgcn_readfirstlane(it0.kvh), j0, j1_max, pf);
    }
    trace_event_at(p, kEvStart, t_entry);

    while (e < wl.last) {
        // a run = the splits [split, s1) of one tile that fall into this workgroup's block
        Item it = worklist_item(p, wl, ss.pre, e, sl_first);
        it.tile = __builtin_amdgcn_readfirstlane(it.tile);      // all of these are workgroup-uniform
        it.b = __builtin_amdgcn_readfirstlane(it.b);
        it.kvh = __builtin_amdgcn_readfirstlane(it.kvh);
        it.split = __builtin_amdgcn_readfirstlane(it.split);
        it.n = __builtin_amdgcn_readfirstlane(it.n);
        it.S = __builtin_amdgcn_readfirstlane(it.S);
        const int s1 = min(it.n, it.split + (wl.last - e));
        const int run = s1 - it.split;
        const int t0 = e - it.split;         // the tile's first item in this work list
        e += run;
        // keys per split: from S_max for a fixed split count (known before the launch), from the
        // sequence's own length when the library chose the count
        const int c = p.n_splits > 0 ? p.split_keys : split_keys_of(it.S, it.n);
        const int j0 = min(it.split * c, it.S);
        const int j1 = min(s1 * c, it.S);
        const size_t slot = (size_t)it.tile * p.max_splits + it.split;
        const bool direct = run == it.n;     // the whole tile in one go: this is the final result
        if (Path::kPrefetch && pf.any() && j0 >= j1) {           // the prefetched range turned out empty
            wait_loads_landed();
            pf.reset();
        }

        if (direct) {
            float* o = p.out + ((size_t)it.b * p.Hq + (size_t)it.kvh * G) * kD;
            float* l = p.lse ? p.lse + (size_t)it.b * p.Hq + it.kvh * G : nullptr;
            if (j0 < j1) {
                path.template item<false>(p, it.b, it.kvh, j0, j1, o, l, kLn2, pf, [] {});
            } else {                         // empty sequence: out = 0, lse = -inf
                for (int i = threadIdx.x; i < G * kD; i += kWgThreads) o[i] = 0.f;
                if (l && threadIdx.x < G) l[threadIdx.x] = -INFINITY;
            }
            // bulk-synchronous mode: tell kernel 2 that this tile needs no combine
            if (MODE == kModeBsp && threadIdx.x == 0) {
                if (p.bsp_groups == 1) p.counters[it.tile] = 1u;
                else p.bsp_direct[it.tile] = 1u;
            }
            // fine-grained waits: tell the waiting combine workgroup that there is nothing to merge
            if (MODE == kModeSignal) {
                __syncthreads();
                if (threadIdx.x == 0)
                    __hip_atomic_store(&p.counters[it.tile], kTileDirect, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            continue;
        }

        // a6: one partial for the run in its first slot; the run's other slots (and
        // the first one too if the run has no keys) are marked empty
        // a8, first part: which of the tile's slots will hold a partial follows from the schedule;
        // wave 0 lists them while it would otherwise wait for its first K/V stages (in case this
        // workgroup turns out to be the tile's last arriver).
        const auto list_live = [&] {
            if (MODE == kModeFused) {
                const TileSchedule sch = {t0, wl.base, wl.rem, wl.members, c, it.S};
                combine_live_from_schedule(ss.live, sch, it.n, G, wl.wl);
            }
        };
        if (j0 < j1)
            path.template item<true>(p, it.b, it.kvh, j0, j1, p.part_o + slot * G * kD, p.part_lse + slot * kLseStride, 1.0f, pf, list_live);
        else if (threadIdx.x < 64)
            list_live();
        // (head 0's lse is what a combine that scans memory for live slots looks at)
        for (int r = (j0 < j1 ? 1 : 0) + threadIdx.x; r < run; r += kWgThreads)
            store_agent(&p.part_lse[(slot + r) * kLseStride], -INFINITY);

        trace_event(p, kEvPartialOut);
        // bulk-synchronous mode with several workgroups of kernel 2 per tile: this tile does need
        // them (every workgroup that holds a part of it says so)
        if (MODE == kModeBsp && p.bsp_groups > 1 && threadIdx.x == 0) p.bsp_direct[it.tile] = 0u;
        if (MODE != kModeBsp) {
            // a7: the partial went out with coherent stores; once they are acknowledged
            // and every wave has reached the barrier, one thread counts the run's splits
            // as arrived (Algorithm 4: push, then atomic increment of the flag).
            // a8: whoever completes the tile's count combines it.
            wait_stores_done();
            trace_event(p, kEvStoresAcked);
            __syncthreads();
            if (MODE == kModeFused && p.tree_rows != INT32_MAX) {      // (the host rules it out for most launches)
                // a tile with very many partials is merged in two levels (tree_arrive); a run
                // without keys holds no partial and is not counted there
                const int m = __builtin_amdgcn_readfirstlane(ss.live.n_live);
                if (m > p.tree_rows) {
                    const int rank = __builtin_amdgcn_readfirstlane(ss.live.my_rank);
                    if (j0 < j1) tree_arrive<COMB_BATCH>(p, it.tile, it.b, it.kvh, rank, m, comb, ss.live, &ss.is_last);
                    __syncthreads();
                    continue;
                }
            }
            uint32_t old = 0;
            if (threadIdx.x == 0)
                old = __hip_atomic_fetch_add(&p.counters[it.tile], (uint32_t)run, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (threadIdx.x == 0) ss.is_last = old + (uint32_t)run == (uint32_t)it.n;
            __syncthreads();
            trace_event(p, kEvCounted);
            if (MODE == kModeFused && ss.is_last) {
                combine_tile<COMB_BATCH>(p, it.tile, it.b, it.kvh, it.n, comb, ss.live, true);
                if (threadIdx.x == 0)                               // re-arm for the next call
                    __hip_atomic_store(&p.counters[it.tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                trace_event(p, kEvCombined);
            }
            __syncthreads();
        }
    }
    trace_event(p, kEvEnd);
}

template <int G>
union __attribute__((aligned(16))) ValuWgSmem {
    ItemSmem<G> item;
    CombineSmem comb;
};

template <int G, bool FUSED>
__global__ __launch_bounds__(kWgThreads, (G <= 3 ? 2 : 1)) void fd_valu_kernel(Params p)
{
    __shared__ ValuWgSmem<G> sm;
    __shared__ SchedSmem ss;
    persistent_loop<(FUSED ? kModeFused : kModeBsp), (G <= 2 ? 16 : 8)>(p, ValuPath<G>{&sm.item}, ss, sm.comb);
}

extern __shared__ __attribute__((aligned(16))) char fd_dyn_smem[];

// CB = rows a combining thread keeps in flight: 32 when the workgroup has the CU to itself
// (512 registers per lane), 8 when two workgroups share it.
// PAGED: K/V rows are found through p.block_table (built for NST = 2 only).
// F16: IEEE half q/K/V instead of bf16 (built for NST = 2 only).
template <int NST, bool FUSED, int CB, bool PAGED, bool F16>
__global__ __launch_bounds__(kWgThreads, 1) void fd_mfma_kernel(Params p)
{
    static_assert(sizeof(CombineSmem) <= (size_t)mfma_ring_bytes(NST), "combine scratch must fit the ring");
    __shared__ SchedSmem ss;
    persistent_loop<(FUSED ? kModeFused : kModeBsp), CB>(p, MfmaPath<NST, PAGED, F16>{fd_dyn_smem}, ss,
                                                        *reinterpret_cast<CombineSmem*>(fd_dyn_smem));
}

// The MFMA kernel over an FP8 (E4M3) KV cache: 32-key stages converted to bf16 between LDS and the matrix cores.
template <int NST, bool FUSED, int CB, bool PAGED>
__global__ __launch_bounds__(kWgThreads, 1) void fd_mfma8_kernel(Params p)
{
    __shared__ SchedSmem ss;
    persistent_loop<(FUSED ? kModeFused : kModeBsp), CB>(p, Mfma8Path<NST, PAGED>{fd_dyn_smem}, ss,
                                                        *reinterpret_cast<CombineSmem*>(fd_dyn_smem));
}

// Kernel 1 of the fine-grained-waits variant (Section 4.2.4): partials and arrival counts, no combine.
__global__ __launch_bounds__(kWgThreads, 1) void fd_mfma_signal_kernel(Params p)
{
    __shared__ SchedSmem ss;
    persistent_loop<kModeSignal, 8>(p, MfmaPath<2, false, false>{fd_dyn_smem}, ss, *reinterpret_cast<CombineSmem*>(fd_dyn_smem));
}

// Kernel 2 of the bulk-synchronous baseline: one workgroup per tile.
__global__ __launch_bounds__(kWgThreads) void fd_combine_kernel(Params p)
{
    __shared__ CombineSmem sm;
    __shared__ LiveList ll;
    __shared__ uint32_t done;
    const int tile = blockIdx.x;
    const int b = tile / p.Hkv, kvh = tile - b * p.Hkv;
    const int n = num_splits_of(p, seq_len_of(p, b));
    // kernel 1 marks tiles it wrote as final results (all splits in one block)
    if (threadIdx.x == 0) {
        done = p.counters[tile];
        if (done) p.counters[tile] = 0u;
    }
    __syncthreads();
    if (done) return;
    trace_event(p, kEvStart);
    combine_tile<32>(p, tile, b, kvh, n, sm, ll);
    trace_event(p, kEvEnd);
}

// Kernel 2 of the bulk-synchronous baseline for launches in which a tile may hold more than
// p.tree_rows partials: workgroup (x, y) = (tile, first-level group), p.bsp_groups per tile.
// Workgroup (tile, g) merges group g of a tile that does hold that many (the last of them to finish
// merges the groups' results), workgroup (tile, 0) merges a tile that does not, and the rest leave.
// Tiles that kernel 1 wrote as final results are marked in p.bsp_direct, which kernel 1 writes for
// every tile and nobody clears (several workgroups look at the mark).
__global__ __launch_bounds__(kWgThreads) void fd_combine_tree_kernel(Params p)
{
    __shared__ CombineSmem sm;
    __shared__ LiveList ll;
    __shared__ int flag;
    const int tile = blockIdx.x, grp = blockIdx.y;
    const int b = tile / p.Hkv, kvh = tile - b * p.Hkv;
    const uint32_t direct = p.bsp_direct[tile];
    const int n = num_splits_of(p, seq_len_of(p, b));
    if (direct) return;
    if (threadIdx.x < 64) combine_live_from_memory(ll, p.part_lse + (size_t)tile * p.max_splits * kLseStride, n, p.G);
    __syncthreads();
    const int m = ll.n_live;
    __syncthreads();                       // everybody has m before wave 0 rewrites the list
    if (m > p.tree_rows) {
        if (grp * kTreeGroup < m) tree_merge_group<32>(p, tile, b, kvh, grp, m, sm, ll, &flag);
        return;
    }
    if (grp == 0) combine_tile<32>(p, tile, b, kvh, n, sm, ll, true);
}


// Kernel 2 of the fine-grained-waits variant (Section 4.2.4; Algorithm 4 Part 2 as the paper
// writes it: the consumer waits on the tile's flag, then combines).  Launched on a second
// stream next to kernel 1.  A workgroup takes tiles blockIdx.x, + gridDim.x, ...; thread 0
// polls the tile's arrival counter with coherent loads until the count is complete, the
// other waves sleep at the barrier.  Kernel 1 never waits for anything, so the counts always
// complete; the poll is bounded all the same (p.spin_limit): a workgroup that gives up sets
// *p.status and leaves its remaining tiles alone.
// Sharing a CU with kernel 1: the waiting workgroup is capped at 128 registers per lane (kernel 1
// needs at most 360 of a SIMD's 512) and is launched with kWaitPadLds bytes of LDS it never
// touches: with them one waiter (its own 22 KB + the padding) fits beside a workgroup of
// kernel 1 (83 KB) in the CU's 160 KB, two waiters do not, so a compute unit never hosts more
// than one of them while kernel 1 is resident.  Correctness does not depend on it (kernel 1
// never waits); it keeps the waiters from crowding kernel 1 out of LDS.
constexpr int kWaitPadLds = 24 * 1024;
static_assert(sizeof(CombineSmem) + sizeof(LiveList) + kWaitPadLds + 85 * 1024 <= 160 * 1024, "one waiter beside kernel 1");
static_assert(2 * (sizeof(CombineSmem) + sizeof(LiveList) + kWaitPadLds) + 80 * 1024 > 160 * 1024, "never two waiters beside kernel 1");
__global__ __launch_bounds__(kWgThreads, 4) void fd_combine_wait_kernel(Params p)
{
    __shared__ CombineSmem sm;
    __shared__ LiveList ll;
    __shared__ uint32_t seen;
    const int tiles = p.B * p.Hkv;
    for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const int b = tile / p.Hkv, kvh = tile - b * p.Hkv;
        const uint32_t n = (uint32_t)num_splits_of(p, seq_len_of(p, b));
        if (threadIdx.x == 0) {
            uint32_t c = 0, polls = 0;
            while (true) {
                c = __hip_atomic_load(&p.counters[tile], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (c >= n || ++polls >= p.spin_limit) break;
                __builtin_amdgcn_s_sleep(32);       // ~1 us between polls: hundreds of pollers must not load the memory system
            }
            seen = c;
        }
        __syncthreads();
        const uint32_t c = seen;
        __syncthreads();
        if (c < n) {                       // gave up: report, touch nothing else
            if (threadIdx.x == 0) __hip_atomic_store(p.status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        if (c != kTileDirect) combine_tile<8>(p, tile, b, kvh, (int)n, sm, ll);
        if (threadIdx.x == 0)              // re-arm for the next call
            __hip_atomic_store(&p.counters[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Measurement aid: reads `n_vec` 16-byte vectors once with the loads the K/V stream uses
// (128-bit, non-temporal), one contiguous block per workgroup, and folds them into a
// checksum that is practically never stored.  Its bandwidth is what a kernel that does
// nothing but read can reach on this chip: the "achievable" line next to the 8 TB/s peak.
__global__ __launch_bounds__(kWgThreads) void fd_stream_read_kernel(const uint4* __restrict__ src, size_t n_vec,
                                                                    uint32_t* sink)
{
    constexpr int kUnroll = 16;                                // 64 KB per workgroup step
    const size_t chunk = (size_t)kWgThreads * kUnroll;
    const size_t n_chunks = n_vec / chunk;
    const size_t first = blockIdx.x * n_chunks / gridDim.x, last = (blockIdx.x + 1) * n_chunks / gridDim.x;
    uint32_t acc = 0;
    for (size_t c = first; c < last; ++c) {
        const uint4* p = src + c * chunk + threadIdx.x;
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = load_stream(p + u * kWgThreads);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    // the tail that does not fill a chunk
    for (size_t i = n_chunks * chunk + (size_t)blockIdx.x * kWgThreads + threadIdx.x; i < n_vec;
         i += (size_t)gridDim.x * kWgThreads) {
        const uint4 v = load_stream(src + i);
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u) *sink = acc;
}

}  // namespace fd

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

#define FD_HIP(call)                                                                               \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) return fail(FD_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_));     \
    } while (0)

constexpr uint32_t kMagic = 0x46444831u;

struct Layout {
    size_t part_o_off, part_lse_off, part2_o_off, part2_lse_off;
    size_t counters_off, group_counters_off, bsp_direct_off, status_off, total;     // zeroed from counters_off on
    int group_cap;
};

}  // namespace

struct fd_handle_s {
    uint32_t magic;
    fd_config cfg;
    int G;
    int device;
    int num_cus;
    void* workspace;
    Layout lay;
    int opt_path, opt_xcd, opt_wgs_per_cu, opt_ring, opt_spin_limit, opt_split_keys, opt_tree_rows;
    hipStream_t side_stream;      // fine-grained waits: the waiting combine kernel runs here
    hipEvent_t ev_fork, ev_join;
    int last_grid, last_path;
    unsigned long long* trace;
    int trace_capacity;      // workgroups the trace buffer has room for
};

namespace {

int check_config(const fd_config* c)
{
    if (!c) return fail(FD_ERR_INVALID_ARG, "config is NULL");
    if (c->B <= 0 || c->Hq <= 0 || c->Hkv <= 0 || c->S_max <= 0)
        return fail(FD_ERR_INVALID_ARG, "B, Hq, Hkv, S_max must be positive (got %d, %d, %d, %d)", c->B, c->Hq,
                    c->Hkv, c->S_max);
    if (c->Hq % c->Hkv) return fail(FD_ERR_INVALID_ARG, "Hq (%d) must be a multiple of Hkv (%d)", c->Hq, c->Hkv);
    if (c->max_splits < 1 || c->max_splits > FD_MAX_SPLITS)
        return fail(FD_ERR_INVALID_ARG, "max_splits must be in 1..%d (got %d)", FD_MAX_SPLITS, c->max_splits);
    if (!(c->scale >= 0.0f) || std::isinf(c->scale)) return fail(FD_ERR_INVALID_ARG, "scale must be finite and >= 0");
    if (c->D != fd::kD) return fail(FD_ERR_UNSUPPORTED, "only D = 128 is built (got %d)", c->D);
    if (c->kv_layout != 0) return fail(FD_ERR_UNSUPPORTED, "only kv_layout 0 ([B,Hkv,S_max,D]) is built");
    if (c->dtype != FD_DTYPE_BF16 && c->dtype != FD_DTYPE_FP16 && c->dtype != FD_DTYPE_FP8_KV)
        return fail(FD_ERR_UNSUPPORTED, "dtype must be FD_DTYPE_BF16 (0), FD_DTYPE_FP16 (1) or FD_DTYPE_FP8_KV (2), got %d", c->dtype);
    if (!(c->k_scale >= 0.0f) || !(c->v_scale >= 0.0f) || std::isinf(c->k_scale) || std::isinf(c->v_scale))
        return fail(FD_ERR_INVALID_ARG, "k_scale and v_scale must be finite and >= 0");
    const int G = c->Hq / c->Hkv;
    if (G > 16) return fail(FD_ERR_UNSUPPORTED, "GQA group Hq/Hkv = %d is not built (1..16)", G);
    if ((long long)c->B * c->Hkv > (1ll << 24)) return fail(FD_ERR_UNSUPPORTED, "B*Hkv too large");
    // work items are counted in 32 bits
    if ((long long)c->B * c->Hkv * c->max_splits >= (1ll << 31))
        return fail(FD_ERR_UNSUPPORTED, "B*Hkv*max_splits = %lld does not fit 31 bits", (long long)c->B * c->Hkv * c->max_splits);
    return FD_OK;
}

Layout make_layout(const fd_config& c)
{
    const size_t tiles = (size_t)c.B * c.Hkv, G = (size_t)(c.Hq / c.Hkv);
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    Layout l;
    // first-level groups of the two-level combine: a tile has at most max_splits partials
    l.group_cap = (c.max_splits + fd::kTreeGroup - 1) / fd::kTreeGroup;
    if (l.group_cap > fd::kMaxGroups) l.group_cap = fd::kMaxGroups;
    l.part_o_off = 0;
    l.part_lse_off = up(tiles * c.max_splits * G * fd::kD * sizeof(float));
    l.part2_o_off = l.part_lse_off + up(tiles * c.max_splits * fd::kLseStride * sizeof(float));
    l.part2_lse_off = l.part2_o_off + up(tiles * l.group_cap * G * fd::kD * sizeof(float));
    l.counters_off = l.part2_lse_off + up(tiles * l.group_cap * fd::kLseStride * sizeof(float));
    l.group_counters_off = l.counters_off + up(tiles * sizeof(uint32_t));
    l.bsp_direct_off = l.group_counters_off + up(tiles * fd::kMaxGroups * sizeof(uint32_t));
    l.status_off = l.bsp_direct_off + up(tiles * sizeof(uint32_t));
    l.total = l.status_off + 256;
    return l;
}

void release_sync_objects(fd_handle_t h)
{
    if (h->ev_fork) (void)hipEventDestroy(h->ev_fork);
    if (h->ev_join) (void)hipEventDestroy(h->ev_join);
    if (h->side_stream) (void)hipStreamDestroy(h->side_stream);
    h->ev_fork = h->ev_join = nullptr;
    h->side_stream = nullptr;
}

int check_handle(fd_handle_t h)
{
    if (!h || h->magic != kMagic) return fail(FD_ERR_INVALID_ARG, "invalid handle");
    return FD_OK;
}

int launch_fill(void* dst, size_t bytes, uint32_t value, hipStream_t st)
{
    const size_t words = bytes / sizeof(uint32_t);
    if (words == 0) return FD_OK;
    const size_t wgs = (words + fd::kWgThreads - 1) / fd::kWgThreads;
    hipLaunchKernelGGL(fd::fd_fill_words_kernel, dim3((unsigned)(wgs < 1024 ? wgs : 1024)), dim3(fd::kWgThreads), 0, st,
                       (uint32_t*)dst, words, value);
    FD_HIP(hipGetLastError());
    return FD_OK;
}

// p.bsp_groups workgroups per tile: 1, or the first-level groups a tile of this launch may have
int launch_combine(const fd::Params& p, hipStream_t st)
{
    if (p.bsp_groups > 1)
        hipLaunchKernelGGL(fd::fd_combine_tree_kernel, dim3(p.B * p.Hkv, p.bsp_groups), dim3(fd::kWgThreads), 0, st, p);
    else
        hipLaunchKernelGGL(fd::fd_combine_kernel, dim3(p.B * p.Hkv), dim3(fd::kWgThreads), 0, st, p);
    FD_HIP(hipGetLastError());
    return FD_OK;
}

template <int G>
int launch_valu(const fd::Params& p, bool fused, int grid, hipStream_t st)
{
    if (fused) {
        hipLaunchKernelGGL((fd::fd_valu_kernel<G, true>), dim3(grid), dim3(fd::kWgThreads), 0, st, p);
        FD_HIP(hipGetLastError());
        return FD_OK;
    }
    hipLaunchKernelGGL((fd::fd_valu_kernel<G, false>), dim3(grid), dim3(fd::kWgThreads), 0, st, p);
    FD_HIP(hipGetLastError());
    return launch_combine(p, st);
}

template <int NST, int CB, bool PAGED, bool F16>
int launch_mfma(const fd::Params& p, bool fused, int grid, hipStream_t st)
{
    // more than 64 KB of dynamic LDS has to be granted once per kernel and device
    static thread_local int granted_device[2] = {-1, -1};
    int dev = 0;
    FD_HIP(hipGetDevice(&dev));
    const size_t ring = (size_t)fd::mfma_lds_bytes(NST);      // ring + page-number slots
    if (granted_device[fused] != dev) {
        if (fused)
            FD_HIP(hipFuncSetAttribute((const void*)fd::fd_mfma_kernel<NST, true, CB, PAGED, F16>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)ring));
        else
            FD_HIP(hipFuncSetAttribute((const void*)fd::fd_mfma_kernel<NST, false, CB, PAGED, F16>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)ring));
        granted_device[fused] = dev;
    }
    if (fused) {
        hipLaunchKernelGGL((fd::fd_mfma_kernel<NST, true, CB, PAGED, F16>), dim3(grid), dim3(fd::kWgThreads), ring, st, p);
        FD_HIP(hipGetLastError());
        return FD_OK;
    }
    hipLaunchKernelGGL((fd::fd_mfma_kernel<NST, false, CB, PAGED, F16>), dim3(grid), dim3(fd::kWgThreads), ring, st, p);
    FD_HIP(hipGetLastError());
    return launch_combine(p, st);
}

template <int NST, int CB, bool PAGED>
int launch_mfma8(const fd::Params& p, bool fused, int grid, hipStream_t st)
{
    static thread_local int granted_device[2] = {-1, -1};
    int dev = 0;
    FD_HIP(hipGetDevice(&dev));
    const size_t lds = (size_t)fd::mfma_lds_bytes(NST);
    if (granted_device[fused] != dev) {
        if (fused)
            FD_HIP(hipFuncSetAttribute((const void*)fd::fd_mfma8_kernel<NST, true, CB, PAGED>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        else
            FD_HIP(hipFuncSetAttribute((const void*)fd::fd_mfma8_kernel<NST, false, CB, PAGED>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        granted_device[fused] = dev;
    }
    if (fused) {
        hipLaunchKernelGGL((fd::fd_mfma8_kernel<NST, true, CB, PAGED>), dim3(grid), dim3(fd::kWgThreads), lds, st, p);
        FD_HIP(hipGetLastError());
        return FD_OK;
    }
    hipLaunchKernelGGL((fd::fd_mfma8_kernel<NST, false, CB, PAGED>), dim3(grid), dim3(fd::kWgThreads), lds, st, p);
    FD_HIP(hipGetLastError());
    return launch_combine(p, st);
}

// Fine-grained waits (Section 4.2.4): kernel 1 (partials + arrival counts) on the caller's
// stream, the waiting combine kernel on the handle's second stream, forked and joined with
// events so that the caller's stream sees one operation.  Kernel 1 goes first: if the
// hardware ever ran the two one after the other, the combine kernel would find every count
// complete instead of waiting for a kernel that cannot start.
int launch_waits(fd_handle_t h, const fd::Params& p, int grid, hipStream_t st)
{
    static thread_local int granted_device = -1;
    int dev = 0;
    FD_HIP(hipGetDevice(&dev));
    const size_t lds = (size_t)fd::mfma_lds_bytes(2);
    if (granted_device != dev) {
        FD_HIP(hipFuncSetAttribute((const void*)fd::fd_mfma_signal_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        granted_device = dev;
    }
    const int tiles = p.B * p.Hkv;
    const int waiters = tiles < h->num_cus ? tiles : h->num_cus;
    FD_HIP(hipEventRecord(h->ev_fork, st));
    FD_HIP(hipStreamWaitEvent(h->side_stream, h->ev_fork, 0));
    hipLaunchKernelGGL(fd::fd_mfma_signal_kernel, dim3(grid), dim3(fd::kWgThreads), lds, st, p);
    FD_HIP(hipGetLastError());
    hipLaunchKernelGGL(fd::fd_combine_wait_kernel, dim3(waiters), dim3(fd::kWgThreads), fd::kWaitPadLds, h->side_stream, p);
    FD_HIP(hipGetLastError());
    FD_HIP(hipEventRecord(h->ev_join, h->side_stream));
    FD_HIP(hipStreamWaitEvent(st, h->ev_join, 0));
    return FD_OK;
}

// Paged-cache arguments of a call; table == nullptr for the contiguous layout.
struct PagedArgs {
    const int32_t* table;
    int32_t page_size, pages_per_seq, num_pages;
};

int decode_common(fd_handle_t h, const void* q, const void* k, const void* v, const int32_t* seq_lens, float* out,
                  float* lse, int32_t n_splits, void* stream, int mode, const PagedArgs& pg = PagedArgs{nullptr, 0, 0, 0})
{
    const bool fused = mode == fd::kModeFused;
    int rc = check_handle(h);
    if (rc) return rc;
    if (!q || !k || !v || !seq_lens || !out) return fail(FD_ERR_INVALID_ARG, "q, k_cache, v_cache, seq_lens, out must be non-NULL");
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15)
        return fail(FD_ERR_INVALID_ARG, "q, k_cache, v_cache and out must be 16-byte aligned");
    if (n_splits < 0 || n_splits > h->cfg.max_splits)
        return fail(FD_ERR_INVALID_ARG, "n_splits must be in 0..max_splits=%d (got %d)", h->cfg.max_splits, n_splits);
    int cur_dev = 0;
    FD_HIP(hipGetDevice(&cur_dev));
    if (cur_dev != h->device)
        return fail(FD_ERR_INVALID_ARG, "the handle belongs to device %d, the current device is %d", h->device, cur_dev);
    const fd_config& c = h->cfg;
    const int tiles = c.B * c.Hkv;
    int page_shift = 0;
    if (pg.table) {
        if (pg.page_size < 16 || pg.page_size > 65536 || (pg.page_size & (pg.page_size - 1)))
            return fail(FD_ERR_INVALID_ARG, "page_size must be a power of two in 16..65536 (got %d)", pg.page_size);
        if (pg.num_pages <= 0 || pg.pages_per_seq <= 0)
            return fail(FD_ERR_INVALID_ARG, "num_pages and pages_per_seq must be positive");
        if ((long long)pg.pages_per_seq * pg.page_size < c.S_max)
            return fail(FD_ERR_INVALID_ARG, "block table rows cover %lld keys, fewer than S_max = %d",
                        (long long)pg.pages_per_seq * pg.page_size, c.S_max);
        while ((1 << page_shift) < pg.page_size) ++page_shift;
    }

    // which kernel: the MFMA kernel by default for every group size.  Its K/V stream goes
    // global -> LDS and needs no registers; measured on MI355X it is as fast as the VALU
    // kernel or faster at every G (1 % slower on a 1K-key call, 2-20 % faster elsewhere,
    // 5 % at G = 1 on 128K keys), although at G = 1 fifteen of its sixteen matrix rows are
    // padding: the bound is HBM, not the matrix pipe.  The VALU kernel stays selectable.
    const int G = h->G;
    int path = h->opt_path;
    if (pg.table) {
        // only the MFMA kernel follows a block table; it handles every group size
        if (path == 1) return fail(FD_ERR_UNSUPPORTED, "the VALU kernel does not read paged caches");
        path = 2;
    }
    if (c.dtype == FD_DTYPE_FP8_KV) {
        if (path == 1 || mode == fd::kModeSignal)
            return fail(FD_ERR_UNSUPPORTED, "an FP8 cache is read by the MFMA kernel, fused or BSP only");
        if (pg.table && pg.page_size < 32)
            return fail(FD_ERR_UNSUPPORTED, "an FP8 cache is paged in pages of at least 32 keys (got %d)", pg.page_size);
        path = 2;
    }
    if (c.dtype == FD_DTYPE_FP16) {
        if (path == 1) return fail(FD_ERR_UNSUPPORTED, "the VALU kernel is built for bf16 only");
        if (mode == fd::kModeSignal) return fail(FD_ERR_UNSUPPORTED, "the fine-grained-waits variant is built for bf16 only");
        path = 2;
    }
    if (path == 0) path = 2;
    if (mode == fd::kModeSignal) {
        if (path != 2 || pg.table) return fail(FD_ERR_UNSUPPORTED, "the fine-grained-waits variant exists for the MFMA kernel on a contiguous cache only");
        if (!h->side_stream) return fail(FD_ERR_HIP, "the handle has no second stream");
    }
    if (path == 1 && G > 8) return fail(FD_ERR_UNSUPPORTED, "the VALU kernel is built for Hq/Hkv <= 8 (got %d)", G);

    // persistent grid: a fixed number of workgroups per CU, never more than there are items.
    // MFMA kernel: one workgroup per CU and a ring of 2 stages per wave (ONE 8 KB stage in
    // flight per wave, 8 MB on the whole chip) measured fastest: deeper rings only lengthen
    // the queues in front of memory, which every dependent access of the tail then waits in.
    const long long items_max = (long long)tiles * (n_splits > 0 ? n_splits : c.max_splits);
    int per_cu = h->opt_wgs_per_cu > 0 ? h->opt_wgs_per_cu : ((path == 2 || G >= 4) ? 1 : 2);
    if (mode == fd::kModeSignal) per_cu = 1;
    if (path == 2 && per_cu > 2)
        return fail(FD_ERR_INVALID_ARG, "the MFMA kernel runs 1 or 2 workgroups per CU (FD_OPT_WGS_PER_CU = %d)", per_cu);
    long long grid = (long long)h->num_cus * per_cu;
    if (grid > items_max) grid = items_max;
    int X = h->opt_xcd;
    // Work lists: one per XCD (the workgroups that exchange a tile's partials share an L2 and
    // finish together, which keeps the tail short) or one for the chip (every XCD streams
    // from all over the cache).  Measured over 8..256 tiles of 2K..128K keys: with a fixed
    // split count the lists per XCD win 0.5-2 % up to 8K keys per sequence, lose 1-8 % from 32K
    // keys on (an XCD then streams few, large contiguous regions) and at 16K keys lose 2-3 % with
    // 32 tiles or fewer; with adaptive splits over ragged lengths they win except for few, long
    // sequences.
    if (X == 0) {
        const bool per_xcd = n_splits > 0 ? (c.S_max <= 8192 || (c.S_max <= 16384 && tiles >= 64))
                                          : !(tiles <= 32 && c.S_max > 16384);
        X = (tiles % 8 == 0 && per_xcd) ? 8 : 1;
    }
    if (grid < 8) X = 1;
    if (X == 8) grid -= grid % 8;
    if (n_splits == 0 && (tiles + X - 1) / X > fd::kMaxGroupTiles)
        return fail(FD_ERR_UNSUPPORTED, "adaptive splits support at most %d tiles per XCD group", fd::kMaxGroupTiles);

    fd::Params p;
    p.q = (const uint16_t*)q;
    p.k = (const uint16_t*)k;
    p.v = (const uint16_t*)v;
    p.block_table = pg.table;
    p.page_shift = page_shift;
    p.pages_per_seq = pg.pages_per_seq;
    p.num_pages = pg.num_pages;
    p.seq_lens = seq_lens;
    p.out = out;
    p.lse = lse;
    char* ws = (char*)h->workspace;
    p.part_o = (float*)(ws + h->lay.part_o_off);
    p.part_lse = (float*)(ws + h->lay.part_lse_off);
    p.counters = (uint32_t*)(ws + h->lay.counters_off);
    p.status = (uint32_t*)(ws + h->lay.status_off);
    p.part2_o = (float*)(ws + h->lay.part2_o_off);
    p.part2_lse = (float*)(ws + h->lay.part2_lse_off);
    p.group_counters = (uint32_t*)(ws + h->lay.group_counters_off);
    p.bsp_direct = (uint32_t*)(ws + h->lay.bsp_direct_off);
    p.group_cap = h->lay.group_cap;
    // Two-level combine: only where a tile can hold more partials than the threshold.  A tile's
    // partials are at most its splits, at most the workgroups of its list, and, with a fixed split
    // count, about one per block of items that overlaps it.
    {
        const int tree_rows = h->opt_tree_rows > 0 ? h->opt_tree_rows : fd::kTreeRowsDefault;
        const long long n_eff = n_splits > 0 ? n_splits : c.max_splits;
        const long long members = (grid + X - 1) / X;
        long long rows_bound = n_eff < members ? n_eff : members;
        if (n_splits > 0 && tiles / X > 0) {
            const long long base = (long long)(tiles / X) * n_splits / members;     // items per block (the shortest list)
            if (base >= 1 && n_splits / base + 2 < rows_bound) rows_bound = n_splits / base + 2;
        }
        const bool tree = mode != fd::kModeSignal && rows_bound > tree_rows;
        p.tree_rows = tree ? tree_rows : INT32_MAX;
        p.bsp_groups = 1;
        if (tree) {
            p.bsp_groups = (int)((rows_bound + fd::kTreeGroup - 1) / fd::kTreeGroup);
            if (p.bsp_groups > h->lay.group_cap) p.bsp_groups = h->lay.group_cap;
        }
    }
    p.spin_limit = h->opt_spin_limit > 0 ? (uint32_t)h->opt_spin_limit : (1u << 20);
    p.B = c.B; p.Hq = c.Hq; p.Hkv = c.Hkv; p.G = h->G; p.S_max = c.S_max;
    p.n_splits = n_splits;
    p.max_splits = c.max_splits;
    p.xcd_groups = X;
    p.xcd_shift = X == 8 ? 3 : 0;
    p.grid = (int32_t)grid;
    // Adaptive splits: 512 keys each, unless even sequences of S_max keys would leave three
    // quarters of the compute units without an item; then 256 (measured on such shapes: 6-15 %
    // faster; with half the units busy at 512 keys the finer cut already loses, its partials cost
    // more than the idle units gain).
    p.adaptive_keys = h->opt_split_keys > 0 ? h->opt_split_keys : fd::kAdaptiveKeys;
    if (h->opt_split_keys == 0 && (long long)tiles * ((c.S_max + fd::kAdaptiveKeys - 1) / fd::kAdaptiveKeys) <= h->num_cus / 4)
        p.adaptive_keys = fd::kAdaptiveKeys / 2;
    p.split_keys = n_splits > 0 ? fd::split_keys_of(c.S_max, n_splits) : 0;
    p.div_n_splits = fd::make_fastdiv((uint32_t)(n_splits > 0 ? n_splits : 1));
    p.div_hkv = fd::make_fastdiv((uint32_t)c.Hkv);
    p.sched_uniform = n_splits > 0 && tiles % X == 0 && grid % X == 0;
    p.sched_members = p.sched_base = p.sched_rem = 0;
    if (p.sched_uniform) {
        const long long members = grid / X, n_items = (long long)(tiles / X) * n_splits;
        p.sched_members = (int32_t)members;
        p.sched_base = (int32_t)(n_items / members);
        p.sched_rem = (int32_t)(n_items % members);
    }
    const float scale = c.scale > 0.f ? c.scale : 1.0f / std::sqrt((float)c.D);
    p.scale_log2 = scale * 1.4426950408889634f;
    p.out_mul = 1.0f;
    if (c.dtype == FD_DTYPE_FP8_KV) {
        p.scale_log2 *= c.k_scale > 0.f ? c.k_scale : 1.0f;
        p.out_mul = c.v_scale > 0.f ? c.v_scale : 1.0f;
    }
    p.trace = (h->trace && grid <= h->trace_capacity) ? h->trace : nullptr;

    hipStream_t st = (hipStream_t)stream;
    h->last_grid = (int)grid;
    h->last_path = path;
    if (mode == fd::kModeSignal) return launch_waits(h, p, (int)grid, st);
    if (path == 2) {
        int nst = h->opt_ring > 0 ? h->opt_ring : 2;
        if (per_cu > 1) nst = 2;                       // two workgroups per CU share the LDS
        const bool two = per_cu > 1;
        if (h->cfg.dtype == FD_DTYPE_FP8_KV)
        {
            if (pg.table)
                return two ? launch_mfma8<2, 8, true>(p, fused, (int)grid, st) : launch_mfma8<2, 32, true>(p, fused, (int)grid, st);
            if (two) return launch_mfma8<2, 8, false>(p, fused, (int)grid, st);
            if (nst == 4) return launch_mfma8<4, 32, false>(p, fused, (int)grid, st);
            if (nst == 3) return launch_mfma8<3, 32, false>(p, fused, (int)grid, st);
            return launch_mfma8<2, 32, false>(p, fused, (int)grid, st);
        }
        if (h->cfg.dtype == FD_DTYPE_FP16) {           // the half and the paged kernels are built for the default ring depth
            if (pg.table)
                return two ? launch_mfma<2, 8, true, true>(p, fused, (int)grid, st)
                           : launch_mfma<2, 32, true, true>(p, fused, (int)grid, st);
            return two ? launch_mfma<2, 8, false, true>(p, fused, (int)grid, st)
                       : launch_mfma<2, 32, false, true>(p, fused, (int)grid, st);
        }
        if (pg.table)
            return two ? launch_mfma<2, 8, true, false>(p, fused, (int)grid, st)
                       : launch_mfma<2, 32, true, false>(p, fused, (int)grid, st);
        if (two) return launch_mfma<2, 8, false, false>(p, fused, (int)grid, st);
        if (nst == 4) return launch_mfma<4, 32, false, false>(p, fused, (int)grid, st);
        if (nst == 3) return launch_mfma<3, 32, false, false>(p, fused, (int)grid, st);
        return launch_mfma<2, 32, false, false>(p, fused, (int)grid, st);
    }
    switch (G) {
        case 1: return launch_valu<1>(p, fused, (int)grid, st);
        case 2: return launch_valu<2>(p, fused, (int)grid, st);
        case 3: return launch_valu<3>(p, fused, (int)grid, st);
        case 4: return launch_valu<4>(p, fused, (int)grid, st);
        case 5: return launch_valu<5>(p, fused, (int)grid, st);
        case 6: return launch_valu<6>(p, fused, (int)grid, st);
        case 7: return launch_valu<7>(p, fused, (int)grid, st);
        case 8: return launch_valu<8>(p, fused, (int)grid, st);
        default: return fail(FD_ERR_UNSUPPORTED, "GQA group %d is not built", G);
    }
}

}  // namespace

namespace {

// Per-device set-up of fd_decode_static, done on the first call on a device (with that device
// current): the device address of this GPU's copy of `scratch`, and the device's CU count.
struct StaticDeviceState {
    bool ready;
    void* ptr;
    int num_cus;
};
constexpr int kMaxStaticDevices = 64;
StaticDeviceState g_static_dev[kMaxStaticDevices];
std::mutex g_static_mutex;

int static_device_state(int dev, StaticDeviceState* out)
{
    if (dev < 0 || dev >= kMaxStaticDevices) return fail(FD_ERR_UNSUPPORTED, "device index %d is out of range", dev);
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticDeviceState& s = g_static_dev[dev];
    if (!s.ready) {
        hipDeviceProp_t prop;
        FD_HIP(hipGetDeviceProperties(&prop, dev));
        if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
            return fail(FD_ERR_UNSUPPORTED, "device is %s; this library is built for gfx950 only", prop.gcnArchName);
        void* ptr = nullptr;
        FD_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || ((uintptr_t)ptr & 255)) return fail(FD_ERR_HIP, "the static workspace has no usable device address");
        s.ptr = ptr;
        s.num_cus = prop.multiProcessorCount;
        s.ready = true;
    }
    *out = s;
    return FD_OK;
}

}  // namespace

extern "C" {

size_t fd_workspace_bytes(const fd_config* cfg)
{
    if (check_config(cfg) != FD_OK) return 0;
    return make_layout(*cfg).total;
}

int fd_create(const fd_config* cfg, fd_handle_t* out)
{
    if (!out) return fail(FD_ERR_INVALID_ARG, "out handle pointer is NULL");
    *out = nullptr;
    int rc = check_config(cfg);
    if (rc) return rc;
    int dev = 0;
    FD_HIP(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    FD_HIP(hipGetDeviceProperties(&prop, dev));
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return fail(FD_ERR_UNSUPPORTED, "device is %s; this library is built for gfx950 only", prop.gcnArchName);
    fd_handle_s* h = new (std::nothrow) fd_handle_s();
    if (!h) return fail(FD_ERR_WORKSPACE, "out of host memory");
    h->magic = kMagic;
    h->cfg = *cfg;
    h->G = cfg->Hq / cfg->Hkv;
    h->device = dev;
    h->num_cus = prop.multiProcessorCount;
    h->lay = make_layout(*cfg);
    h->opt_path = h->opt_xcd = h->opt_wgs_per_cu = h->opt_ring = h->opt_spin_limit = h->opt_split_keys = h->opt_tree_rows = 0;
    h->side_stream = nullptr;
    h->ev_fork = h->ev_join = nullptr;
    h->last_grid = h->last_path = 0;
    h->trace = nullptr;
    h->trace_capacity = 0;
    // second stream (default priority) and fork/join events for the fine-grained-waits variant
    if (hipStreamCreateWithFlags(&h->side_stream, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&h->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&h->ev_join, hipEventDisableTiming) != hipSuccess) {
        release_sync_objects(h);
        delete h;
        return fail(FD_ERR_HIP, "creating the handle's stream and events failed");
    }
    hipError_t e = hipMalloc(&h->workspace, h->lay.total);
    if (e != hipSuccess) {
        const size_t want = h->lay.total;
        release_sync_objects(h);
        delete h;
        return fail(FD_ERR_WORKSPACE, "hipMalloc of %zu workspace bytes failed: %s", want, hipGetErrorString(e));
    }
    e = hipMemset((char*)h->workspace + h->lay.counters_off, 0, h->lay.total - h->lay.counters_off);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipFree(h->workspace);
        release_sync_objects(h);
        delete h;
        return fail(FD_ERR_HIP, "zeroing the counters failed: %s", hipGetErrorString(e));
    }
    *out = h;
    return FD_OK;
}

int fd_destroy(fd_handle_t h)
{
    int rc = check_handle(h);
    if (rc) return rc;
    h->magic = 0;
    hipError_t e = hipFree(h->workspace);
    release_sync_objects(h);
    delete h;
    if (e != hipSuccess) return fail(FD_ERR_HIP, "hipFree: %s", hipGetErrorString(e));
    return FD_OK;
}

int fd_reset(fd_handle_t h, void* stream)
{
    int rc = check_handle(h);
    if (rc) return rc;
    return launch_fill((char*)h->workspace + h->lay.counters_off, h->lay.total - h->lay.counters_off, 0u, (hipStream_t)stream);
}

int fd_decode(fd_handle_t h, const void* q, const void* k_cache, const void* v_cache, const int32_t* seq_lens,
              float* out, float* lse, int32_t n_splits, void* stream)
{
    return decode_common(h, q, k_cache, v_cache, seq_lens, out, lse, n_splits, stream, fd::kModeFused);
}

int fd_decode_bsp(fd_handle_t h, const void* q, const void* k_cache, const void* v_cache, const int32_t* seq_lens,
                  float* out, float* lse, int32_t n_splits, void* stream)
{
    return decode_common(h, q, k_cache, v_cache, seq_lens, out, lse, n_splits, stream, fd::kModeBsp);
}

int fd_decode_waits(fd_handle_t h, const void* q, const void* k_cache, const void* v_cache, const int32_t* seq_lens,
                    float* out, float* lse, int32_t n_splits, void* stream)
{
    return decode_common(h, q, k_cache, v_cache, seq_lens, out, lse, n_splits, stream, fd::kModeSignal);
}

int fd_decode_static(const fd_config* cfg, const void* q, const void* k_cache, const void* v_cache,
                                const int32_t* seq_lens, float* out, float* lse, int32_t n_splits, void* stream)
{
    int rc = check_config(cfg);
    if (rc) return rc;
    const Layout lay = make_layout(*cfg);
    if (lay.total > (size_t)FD_STATIC_SCRATCH_BYTES)
        return fail(FD_ERR_WORKSPACE,
                    "this shape needs %zu workspace bytes, the static workspace holds %zu: lower max_splits or use a handle",
                    lay.total, (size_t)FD_STATIC_SCRATCH_BYTES);
    int dev = 0;
    FD_HIP(hipGetDevice(&dev));
    StaticDeviceState sd;
    rc = static_device_state(dev, &sd);
    if (rc) return rc;

    // a handle that lives on this stack frame and owns nothing
    fd_handle_s h = {};
    h.magic = kMagic;
    h.cfg = *cfg;
    h.G = cfg->Hq / cfg->Hkv;
    h.device = dev;
    h.num_cus = sd.num_cus;
    h.workspace = sd.ptr;
    h.lay = lay;

    // The workspace keeps what the last call on this GPU left (possibly of another shape, possibly
    // cut short): the counters and the status word must start at zero.
    rc = launch_fill((char*)sd.ptr + lay.counters_off, lay.total - lay.counters_off, 0u, (hipStream_t)stream);
    if (rc) return rc;
    return decode_common(&h, q, k_cache, v_cache, seq_lens, out, lse, n_splits, stream, fd::kModeFused);
}

int fd_autotune(fd_handle_t h, const void* q, const void* k_cache, const void* v_cache, const int32_t* seq_lens,
                float* out, float* lse, int32_t n_splits, void* stream, int32_t reps, float* best_us)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (reps <= 0 || reps > 10000) return fail(FD_ERR_INVALID_ARG, "reps must be in 1..10000");
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0, e1;
    FD_HIP(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return fail(FD_ERR_HIP, "hipEventCreate failed");
    }
    const int tiles = h->cfg.B * h->cfg.Hkv;
    const bool bf16 = h->cfg.dtype == FD_DTYPE_BF16;
    // The joint search space (the one-GPU counterpart of tuning the transfer granularity together
    // with the kernel's tiling, paper Section 6.3): how finely a tile is cut when the library picks
    // the split count x the work-list shape x (workgroups per CU, ring stages) of the MFMA kernel,
    // plus the VALU kernel; only what this handle's dtype is built for.
    struct Cand { int path, xcd, per_cu, ring, split_keys; };
    Cand cands[97];
    int n_cand = 0;
    // candidate 0: the options as they stand (the defaults' rules, unless the caller set some)
    const Cand saved = {h->opt_path, h->opt_xcd, h->opt_wgs_per_cu, h->opt_ring, h->opt_split_keys};
    cands[n_cand++] = saved;
    const int xcds[2] = {1, 8};
    const int shapes[4][2] = {{1, 2}, {2, 2}, {1, 3}, {1, 4}};
    const int n_shapes = bf16 ? 4 : 2;                        // deeper rings are built for bf16 only
    const int grains[4] = {512, 256, 1024, 2048};
    const int n_grains = n_splits == 0 ? 4 : 1;               // a fixed split count is the caller's choice
    for (int gi = 0; gi < n_grains; ++gi) {
        const int grain = n_splits == 0 ? grains[gi] : 0;
        for (int xi = 0; xi < 2; ++xi) {
            if (xcds[xi] == 8 && tiles % 8 != 0) continue;
            for (int si = 0; si < n_shapes; ++si) cands[n_cand++] = Cand{2, xcds[xi], shapes[si][0], shapes[si][1], grain};
            if (bf16 && h->G <= 8) cands[n_cand++] = Cand{1, xcds[xi], 0, 0, grain};
        }
    }
    const auto apply = [&](const Cand& c) {
        h->opt_path = c.path; h->opt_xcd = c.xcd; h->opt_wgs_per_cu = c.per_cu; h->opt_ring = c.ring; h->opt_split_keys = c.split_keys;
    };
    const auto call = [&]() { return decode_common(h, q, k_cache, v_cache, seq_lens, out, lse, n_splits, stream, fd::kModeFused); };
    // mean time of `reps` calls of the options in force; FD_ERR_UNSUPPORTED = not built for this shape
    const auto measure = [&](float* us) -> int {
        int r = FD_OK;
        for (int w = 0; w < 3 && r == FD_OK; ++w) r = call();
        if (r != FD_OK) return r;
        if (hipEventRecord(e0, st) != hipSuccess) return fail(FD_ERR_HIP, "hipEventRecord failed");
        for (int i = 0; i < reps && r == FD_OK; ++i) r = call();
        if (r != FD_OK) return r;
        float ms = 0.f;
        if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
            return fail(FD_ERR_HIP, "timing a candidate failed");
        *us = ms * 1000.f / (float)reps;
        return FD_OK;
    };

    // Settle: the first tens of milliseconds of work after an idle period run a few per cent
    // slower whatever is launched, which would handicap the candidates measured first.
    rc = FD_OK;
    const auto t0 = std::chrono::steady_clock::now();
    bool settling = true;
    while (settling && rc == FD_OK && std::chrono::steady_clock::now() - t0 < std::chrono::milliseconds(100)) {
        for (int i = 0; i < 20 && rc == FD_OK; ++i) {
            rc = call();
            if (rc == FD_ERR_UNSUPPORTED) {                    // the options in force are not built for this shape:
                rc = FD_OK;                                    // the candidates below decide
                settling = false;
                break;
            }
        }
        if (rc == FD_OK && hipStreamSynchronize(st) != hipSuccess) rc = fail(FD_ERR_HIP, "hipStreamSynchronize failed");
    }

    float best = 0.f;
    int best_i = -1;
    bool saved_ok = false;
    for (int i = 0; i < n_cand && rc == FD_OK; ++i) {
        apply(cands[i]);
        float us = 0.f;
        const int r1 = measure(&us);
        if (r1 == FD_ERR_UNSUPPORTED) continue;                // a combination this shape does not allow: not a failure
        if (r1 != FD_OK) { rc = r1; break; }
        if (i == 0) saved_ok = true;
        if (best_i < 0 || us < best) { best = us; best_i = i; }
    }
    // Confirm: differences of a per cent are inside the spread of one pass, so a winner other
    // than the options the handle came with has to beat them again, twice, by 0.5 %.
    if (rc == FD_OK && best_i > 0 && saved_ok) {
        float us_new[2] = {0.f, 0.f}, us_old[2] = {0.f, 0.f};
        for (int pass = 0; pass < 2 && rc == FD_OK; ++pass) {
            apply(saved);
            rc = measure(&us_old[pass]);
            if (rc != FD_OK) break;
            apply(cands[best_i]);
            rc = measure(&us_new[pass]);
        }
        if (rc == FD_OK) {
            const float o = us_old[0] < us_old[1] ? us_old[0] : us_old[1];
            const float n = us_new[0] > us_new[1] ? us_new[0] : us_new[1];
            if (n < 0.995f * o) best = n;
            else { best_i = 0; best = o; }
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc != FD_OK || best_i < 0) {
        apply(saved);
        return rc != FD_OK ? rc : fail(FD_ERR_UNSUPPORTED, "no option combination is built for this shape");
    }
    apply(cands[best_i]);
    // leave out / lse holding a result of the chosen combination
    rc = call();
    if (rc == FD_OK && hipStreamSynchronize(st) != hipSuccess) rc = fail(FD_ERR_HIP, "hipStreamSynchronize failed");
    if (rc != FD_OK) {
        apply(saved);
        return rc;
    }
    if (best_us) *best_us = best;
    return FD_OK;
}

int fd_decode_paged(fd_handle_t h, const void* q, const void* k_pages, const void* v_pages, const int32_t* block_table,
                    int32_t page_size, int32_t pages_per_seq, int32_t num_pages, const int32_t* seq_lens, float* out,
                    float* lse, int32_t n_splits, void* stream)
{
    if (!block_table) return fail(FD_ERR_INVALID_ARG, "block_table must be non-NULL");
    return decode_common(h, q, k_pages, v_pages, seq_lens, out, lse, n_splits, stream, fd::kModeFused,
                         PagedArgs{block_table, page_size, pages_per_seq, num_pages});
}

int fd_decode_paged_bsp(fd_handle_t h, const void* q, const void* k_pages, const void* v_pages,
                        const int32_t* block_table, int32_t page_size, int32_t pages_per_seq, int32_t num_pages,
                        const int32_t* seq_lens, float* out, float* lse, int32_t n_splits, void* stream)
{
    if (!block_table) return fail(FD_ERR_INVALID_ARG, "block_table must be non-NULL");
    return decode_common(h, q, k_pages, v_pages, seq_lens, out, lse, n_splits, stream, fd::kModeBsp,
                         PagedArgs{block_table, page_size, pages_per_seq, num_pages});
}

int fd_set_option(fd_handle_t h, int32_t key, int32_t value)
{
    int rc = check_handle(h);
    if (rc) return rc;
    switch (key) {
        case FD_OPT_PATH:
            if (value < 0 || value > 2) return fail(FD_ERR_INVALID_ARG, "FD_OPT_PATH must be 0, 1 or 2");
            h->opt_path = value;
            return FD_OK;
        case FD_OPT_XCD_GROUPS:
            if (value != 0 && value != 1 && value != 8) return fail(FD_ERR_INVALID_ARG, "FD_OPT_XCD_GROUPS must be 0, 1 or 8");
            h->opt_xcd = value;
            return FD_OK;
        case FD_OPT_WGS_PER_CU:
            if (value < 0 || value > 16) return fail(FD_ERR_INVALID_ARG, "FD_OPT_WGS_PER_CU must be in 0..16");
            h->opt_wgs_per_cu = value;
            return FD_OK;
        case FD_OPT_SPIN_LIMIT:
            if (value < 0) return fail(FD_ERR_INVALID_ARG, "FD_OPT_SPIN_LIMIT must be >= 0");
            h->opt_spin_limit = value;
            return FD_OK;
        case FD_OPT_RING_STAGES:
            if (value != 0 && (value < 2 || value > 4)) return fail(FD_ERR_INVALID_ARG, "FD_OPT_RING_STAGES must be 0, 2, 3 or 4");
            h->opt_ring = value;
            return FD_OK;
        case FD_OPT_TREE_ROWS:
            if (value < 0 || (value > 0 && value < 2)) return fail(FD_ERR_INVALID_ARG, "FD_OPT_TREE_ROWS must be 0 or at least 2");
            h->opt_tree_rows = value;
            return FD_OK;
        case FD_OPT_SPLIT_KEYS:
            if (value != 0 && (value < fd::kSplitAlign || value > 65536 || value % fd::kSplitAlign))
                return fail(FD_ERR_INVALID_ARG, "FD_OPT_SPLIT_KEYS must be 0 or a multiple of %d in %d..65536", fd::kSplitAlign, fd::kSplitAlign);
            h->opt_split_keys = value;
            return FD_OK;
        default:
            return fail(FD_ERR_INVALID_ARG, "unknown or read-only option %d", key);
    }
}

int fd_get_option(fd_handle_t h, int32_t key, int32_t* value)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (!value) return fail(FD_ERR_INVALID_ARG, "value pointer is NULL");
    switch (key) {
        case FD_OPT_PATH: *value = h->opt_path; return FD_OK;
        case FD_OPT_XCD_GROUPS: *value = h->opt_xcd; return FD_OK;
        case FD_OPT_WGS_PER_CU: *value = h->opt_wgs_per_cu; return FD_OK;
        case FD_OPT_RING_STAGES: *value = h->opt_ring; return FD_OK;
        case FD_OPT_SPIN_LIMIT: *value = h->opt_spin_limit; return FD_OK;
        case FD_OPT_SPLIT_KEYS: *value = h->opt_split_keys; return FD_OK;
        case FD_OPT_TREE_ROWS: *value = h->opt_tree_rows; return FD_OK;
        case FD_INFO_WAIT_GAVE_UP: {
            uint32_t flag = 0;
            FD_HIP(hipDeviceSynchronize());
            FD_HIP(hipMemcpy(&flag, (char*)h->workspace + h->lay.status_off, sizeof(flag), hipMemcpyDeviceToHost));
            *value = (int32_t)flag;
            return FD_OK;
        }
        case FD_INFO_NUM_CUS: *value = h->num_cus; return FD_OK;
        case FD_INFO_LAST_GRID: *value = h->last_grid; return FD_OK;
        case FD_INFO_LAST_PATH: *value = h->last_path; return FD_OK;
        default: return fail(FD_ERR_INVALID_ARG, "unknown option %d", key);
    }
}

int fd_debug_poison_workspace(fd_handle_t h, void* stream)
{
    int rc = check_handle(h);
    if (rc) return rc;
    return launch_fill(h->workspace, h->lay.counters_off, 0xFFFFFFFFu, (hipStream_t)stream);
}

int fd_debug_read_counters(fd_handle_t h, uint32_t* host_dst, int32_t n)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (!host_dst || n != h->cfg.B * h->cfg.Hkv) return fail(FD_ERR_INVALID_ARG, "host_dst NULL or n != B*Hkv");
    FD_HIP(hipDeviceSynchronize());
    FD_HIP(hipMemcpy(host_dst, (char*)h->workspace + h->lay.counters_off, (size_t)n * sizeof(uint32_t),
                     hipMemcpyDeviceToHost));
    return FD_OK;
}

int fd_debug_set_trace(fd_handle_t h, void* device_buffer, int32_t capacity_workgroups)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (device_buffer && capacity_workgroups <= 0) return fail(FD_ERR_INVALID_ARG, "trace capacity must be positive");
    if ((uintptr_t)device_buffer & 7) return fail(FD_ERR_INVALID_ARG, "trace buffer must be 8-byte aligned");
    h->trace = (unsigned long long*)device_buffer;
    h->trace_capacity = device_buffer ? capacity_workgroups : 0;
    return FD_OK;
}

int fd_debug_stream_read(const void* src, size_t bytes, uint32_t* sink, void* stream)
{
    if (!src || !sink || bytes < 16) return fail(FD_ERR_INVALID_ARG, "src, sink must be non-NULL and bytes >= 16");
    if ((uintptr_t)src & 15) return fail(FD_ERR_INVALID_ARG, "src must be 16-byte aligned");
    int dev = 0, cus = 0;
    FD_HIP(hipGetDevice(&dev));
    FD_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    hipLaunchKernelGGL(fd::fd_stream_read_kernel, dim3(cus), dim3(fd::kWgThreads), 0, (hipStream_t)stream,
                       (const uint4*)src, bytes / 16, sink);
    FD_HIP(hipGetLastError());
    return FD_OK;
}

const char* fd_last_error(void) { return g_err; }

int fd_version(void) { return FD_VERSION; }

}  // extern "C"
