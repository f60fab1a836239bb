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

namespace fd {

constexpr int kD = 128;            // head dimension
constexpr int kRowU4 = kD * 2 / 16; // 16-byte chunks per K/V row (16)
constexpr int kWgThreads = 256;
constexpr int kWaves = kWgThreads / 64;
constexpr int kSplitAlign = 64;    // split lengths are multiples of this many keys
constexpr int kAdaptiveKeys = 512; // keys per split when the library chooses
constexpr int kMaxGroupTiles = 2048;  // tiles one XCD group can index in adaptive mode
constexpr float kNegBig = -3.0e38f;   // finite stand-in for "no key seen yet"
constexpr float kLn2 = 0.6931471805599453f;

struct Params {
    const uint16_t* q;        // [B, Hq, D] bf16
    const uint16_t* k;        // [B, Hkv, S_max, D] bf16
    const uint16_t* v;        // [B, Hkv, S_max, D] bf16
    const int32_t* seq_lens;  // [B]
    float* out;               // [B, Hq, D]
    float* lse;               // [B, Hq] or null
    float* part_o;            // [B*Hkv, max_splits, G, D]
    float* part_lse;          // [B*Hkv, max_splits, G]   (log2 units)
    uint32_t* counters;       // [B*Hkv]
    int32_t B, Hq, Hkv, G, S_max;
    int32_t n_splits;         // 0 = adaptive
    int32_t max_splits;
    int32_t xcd_groups;       // 1 or 8
    float scale_log2;         // softmax scale * log2(e)
};

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
    int n = (S + kAdaptiveKeys - 1) / kAdaptiveKeys;
    n = n < 1 ? 1 : n;
    return n > p.max_splits ? p.max_splits : n;
}

__device__ __forceinline__ int split_keys_of(int S, int n)
{
    int c = (S + n - 1) / n;
    c = (c + kSplitAlign - 1) / kSplitAlign * kSplitAlign;
    return c < kSplitAlign ? kSplitAlign : c;
}

// ---- persistent-grid work list ---------------------------------------------
// Workgroup w belongs to XCD group x = w % X (the hardware deals workgroups to
// the 8 XCDs round-robin, so with X = 8 a group is one XCD and its L2).  Group x
// owns tiles t = x, x+X, x+2X, ...; its items are those tiles' splits in order.
// Member wl = w / X of the group takes items wl, wl + members, ...
struct WorkList {
    int x, wl, members, n_tiles, n_items;
};

struct Item {
    int tile, b, kvh, split, n, S;
};

// pre[] : exclusive prefix of split counts over the group's tiles (adaptive mode).
__device__ inline void worklist_init(const Params& p, WorkList& wlst, int* pre, int* scan_tmp)
{
    const int X = p.xcd_groups;
    const int T = p.B * p.Hkv;
    wlst.x = blockIdx.x % X;
    wlst.wl = blockIdx.x / X;
    wlst.members = (gridDim.x - wlst.x + X - 1) / X;
    wlst.n_tiles = wlst.x < T ? (T - wlst.x + X - 1) / X : 0;
    if (p.n_splits > 0) {
        wlst.n_items = wlst.n_tiles * p.n_splits;
        return;
    }
    // adaptive: block-wide exclusive scan of n_b over the group's tiles
    const int tid = threadIdx.x;
    const int per = (wlst.n_tiles + kWgThreads - 1) / kWgThreads;
    const int lo = tid * per;
    int sum = 0;
    for (int k = lo; k < lo + per && k < wlst.n_tiles; ++k) {
        const int t = wlst.x + X * k;
        sum += num_splits_of(p, seq_len_of(p, t / p.Hkv));
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
        run += num_splits_of(p, seq_len_of(p, t / p.Hkv));
    }
    if (tid == kWgThreads - 1) pre[wlst.n_tiles] = scan_tmp[tid];
    __syncthreads();
    wlst.n_items = pre[wlst.n_tiles];
}

__device__ __forceinline__ Item worklist_item(const Params& p, const WorkList& wlst, const int* pre, int e)
{
    Item it;
    int k;
    if (p.n_splits > 0) {
        k = e / p.n_splits;
        it.split = e - k * p.n_splits;
    } else {
        int lo = 0, hi = wlst.n_tiles;      // largest k with pre[k] <= e
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (pre[mid] <= e) lo = mid; else hi = mid;
        }
        k = lo;
        it.split = e - pre[k];
    }
    it.tile = wlst.x + p.xcd_groups * k;
    it.b = it.tile / p.Hkv;
    it.kvh = it.tile - it.b * p.Hkv;
    it.S = seq_len_of(p, it.b);
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

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

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

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// ---- Combine (Algorithm 4, Part 2), one workgroup per tile -------------------
// Merges the n partials of tile (b, kvh) into out / lse, in split order
// i = 0..n-1 (fixed order: results do not depend on which workgroup runs this).
// Partials with lse = -inf (empty key range) have weight 0 and their o rows,
// which nobody wrote, are ignored.
// sm: 2*G floats of LDS.  Ends with every thread past its last read of sm.
template <int G>
__device__ inline void combine_tile(const Params& p, int tile, int b, int kvh, int n, float* sm)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const float* plse = p.part_lse + (size_t)tile * p.max_splits * G;
    const float4* po = reinterpret_cast<const float4*>(p.part_o + (size_t)tile * p.max_splits * G * kD);

    for (int g = wave; g < G; g += kWaves) {
        float mx = -INFINITY;
        for (int i = lane; i < n; i += 64) mx = fmaxf(mx, plse[i * G + g]);
        mx = wave_max(mx);
        float sum = 0.f;
        for (int i = lane; i < n; i += 64) {
            const float v = plse[i * G + g];
            sum += (v == -INFINITY) ? 0.f : fast_exp2(v - mx);
        }
        sum = wave_sum(sum);
        if (lane == 0) {
            sm[g] = mx;
            sm[G + g] = sum > 0.f ? 1.0f / sum : 0.f;
            if (p.lse) p.lse[(size_t)b * p.Hq + kvh * G + g] = sum > 0.f ? (mx + fast_log2(sum)) * kLn2 : -INFINITY;
        }
    }
    __syncthreads();

    float4* dst = reinterpret_cast<float4*>(p.out + ((size_t)b * p.Hq + (size_t)kvh * G) * kD);
    for (int vi = tid; vi < G * (kD / 4); vi += kWgThreads) {
        const int g = vi / (kD / 4), d4 = vi % (kD / 4);
        const float M = sm[g], invL = sm[G + g];
        float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 8
        for (int i = 0; i < n; ++i) {
            const float lw = plse[i * G + g];
            const bool live = lw != -INFINITY;
            const float w = live ? fast_exp2(lw - M) * invL : 0.f;
            float4 x = po[(size_t)(i * G + g) * (kD / 4) + d4];
            o.x += live ? w * x.x : 0.f;
            o.y += live ? w * x.y : 0.f;
            o.z += live ? w * x.z : 0.f;
            o.w += live ? w * x.w : 0.f;
        }
        dst[vi] = o;
    }
    __syncthreads();
}

}  // namespace fd
