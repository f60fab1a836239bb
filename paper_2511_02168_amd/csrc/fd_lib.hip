// libfd.so: kernels' entry points and the C ABI declared in include/fd.h.
// gfx950 (MI355X) only.

#include "../../include/fd.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "fd_device.hpp"
#include "fd_valu.hpp"

namespace fd {

// ---------------------------------------------------------------------------
// Kernels
// ---------------------------------------------------------------------------

template <int G>
union __attribute__((aligned(16))) WgSmem {
    ValuSmem<G> valu;
    float comb[2 * G];
};

// Persistent split-KV kernel.  FUSED: steps a1-a8 in one launch (the workgroup
// that completes a tile's last split merges the tile, paper Section 4.2.5 /
// Algorithm 4 without barrier or second launch).  !FUSED: steps a1-a6 only
// (kernel 1 of the bulk-synchronous baseline, Section 4.2.2).
template <int G, bool FUSED>
__global__ __launch_bounds__(kWgThreads, (G <= 5 ? 2 : 1)) void fd_valu_kernel(Params p)
{
    __shared__ WgSmem<G> sm;
    __shared__ int pre[kMaxGroupTiles + 1];
    __shared__ int scan_tmp[kWgThreads];
    __shared__ int is_last;

    WorkList wl;
    worklist_init(p, wl, pre, scan_tmp);

    for (int e = wl.wl; e < wl.n_items; e += wl.members) {
        const Item it = worklist_item(p, wl, pre, e);
        const int c = split_keys_of(it.S, it.n);
        const int j0 = it.split * c;
        const int j1 = min(j0 + c, it.S);
        const size_t slot = (size_t)it.tile * p.max_splits + it.split;
        const bool direct = it.n == 1;       // a single split is already the final result

        if (j0 < j1) {
            if (direct) {
                float* o = p.out + ((size_t)it.b * p.Hq + (size_t)it.kvh * G) * kD;
                float* l = p.lse ? p.lse + (size_t)it.b * p.Hq + it.kvh * G : nullptr;
                valu_item<G>(p, it.b, it.kvh, j0, j1, o, l, kLn2, sm.valu);
            } else {
                valu_item<G>(p, it.b, it.kvh, j0, j1, p.part_o + slot * G * kD, p.part_lse + slot * G, 1.0f,
                             sm.valu);
            }
        } else if (direct) {                 // empty sequence: out = 0, lse = -inf
            float* o = p.out + ((size_t)it.b * p.Hq + (size_t)it.kvh * G) * kD;
            for (int i = threadIdx.x; i < G * kD; i += kWgThreads) o[i] = 0.f;
            if (p.lse && threadIdx.x < G) p.lse[(size_t)it.b * p.Hq + it.kvh * G + threadIdx.x] = -INFINITY;
        } else {                             // empty split: weight zero in the combine
            if (threadIdx.x < G) p.part_lse[slot * G + threadIdx.x] = -INFINITY;
        }

        if (FUSED && !direct) {
            // a7: publish the partial, then count the arrival (Algorithm 4: push, then
            // atomic increment of the flag).  a8: the last arriver of the tile combines.
            __threadfence();
            __syncthreads();
            if (threadIdx.x == 0) {
                const uint32_t old = atomicAdd(&p.counters[it.tile], 1u);
                is_last = old == (uint32_t)(it.n - 1);
            }
            __syncthreads();
            if (is_last) {
                __threadfence();
                combine_tile<G>(p, it.tile, it.b, it.kvh, it.n, sm.comb);
                if (threadIdx.x == 0) p.counters[it.tile] = 0;     // re-arm for the next call
            }
            __syncthreads();
        }
    }
}

// Kernel 2 of the bulk-synchronous baseline: one workgroup per tile with more
// than one split.
template <int G>
__global__ __launch_bounds__(kWgThreads) void fd_combine_kernel(Params p)
{
    __shared__ float sm[2 * G];
    const int tile = blockIdx.x;
    const int b = tile / p.Hkv, kvh = tile - b * p.Hkv;
    const int n = num_splits_of(p, seq_len_of(p, b));
    if (n == 1) return;
    combine_tile<G>(p, tile, b, kvh, n, sm);
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
    size_t part_o_off, part_lse_off, counters_off, total;
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
    int opt_path, opt_xcd, opt_wgs_per_cu;
    int last_grid, last_path;
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
    const int G = c->Hq / c->Hkv;
    if (G > 8) return fail(FD_ERR_UNSUPPORTED, "GQA group Hq/Hkv = %d is not built (1..8)", G);
    if ((long long)c->B * c->Hkv > (1ll << 24)) return fail(FD_ERR_UNSUPPORTED, "B*Hkv too large");
    return FD_OK;
}

Layout make_layout(const fd_config& c)
{
    const size_t tiles = (size_t)c.B * c.Hkv, G = (size_t)(c.Hq / c.Hkv);
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    Layout l;
    l.part_o_off = 0;
    l.part_lse_off = up(tiles * c.max_splits * G * fd::kD * sizeof(float));
    l.counters_off = l.part_lse_off + up(tiles * c.max_splits * G * sizeof(float));
    l.total = l.counters_off + up(tiles * sizeof(uint32_t));
    return l;
}

int check_handle(fd_handle_t h)
{
    if (!h || h->magic != kMagic) return fail(FD_ERR_INVALID_ARG, "invalid handle");
    return FD_OK;
}

template <int G>
int launch_g(fd_handle_t h, const fd::Params& p, bool fused, int grid, hipStream_t st)
{
    if (fused) {
        hipLaunchKernelGGL((fd::fd_valu_kernel<G, true>), dim3(grid), dim3(fd::kWgThreads), 0, st, p);
        FD_HIP(hipGetLastError());
    } else {
        hipLaunchKernelGGL((fd::fd_valu_kernel<G, false>), dim3(grid), dim3(fd::kWgThreads), 0, st, p);
        FD_HIP(hipGetLastError());
        if (p.n_splits != 1) {
            hipLaunchKernelGGL((fd::fd_combine_kernel<G>), dim3(p.B * p.Hkv), dim3(fd::kWgThreads), 0, st, p);
            FD_HIP(hipGetLastError());
        }
    }
    h->last_path = 1;
    return FD_OK;
}

int decode_common(fd_handle_t h, const void* q, const void* k, const void* v, const int32_t* seq_lens, float* out,
                  float* lse, int32_t n_splits, void* stream, bool fused)
{
    int rc = check_handle(h);
    if (rc) return rc;
    if (!q || !k || !v || !seq_lens || !out) return fail(FD_ERR_INVALID_ARG, "q, k_cache, v_cache, seq_lens, out must be non-NULL");
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15)
        return fail(FD_ERR_INVALID_ARG, "q, k_cache, v_cache and out must be 16-byte aligned");
    if (n_splits < 0 || n_splits > h->cfg.max_splits)
        return fail(FD_ERR_INVALID_ARG, "n_splits must be in 0..max_splits=%d (got %d)", h->cfg.max_splits, n_splits);
    const fd_config& c = h->cfg;
    const int tiles = c.B * c.Hkv;

    // persistent grid: a fixed number of workgroups per CU, never more than there are items
    const long long items_max = (long long)tiles * (n_splits > 0 ? n_splits : c.max_splits);
    const int per_cu = h->opt_wgs_per_cu > 0 ? h->opt_wgs_per_cu : 2;
    long long grid = (long long)h->num_cus * per_cu;
    if (grid > items_max) grid = items_max;
    int X = h->opt_xcd;
    if (X == 0) X = (tiles % 8 == 0) ? 8 : 1;
    if (grid < 8) X = 1;
    if (X == 8) grid -= grid % 8;
    if (n_splits == 0 && (tiles + X - 1) / X > fd::kMaxGroupTiles)
        return fail(FD_ERR_UNSUPPORTED, "adaptive splits support at most %d tiles per XCD group", fd::kMaxGroupTiles);

    fd::Params p;
    p.q = (const uint16_t*)q;
    p.k = (const uint16_t*)k;
    p.v = (const uint16_t*)v;
    p.seq_lens = seq_lens;
    p.out = out;
    p.lse = lse;
    char* ws = (char*)h->workspace;
    p.part_o = (float*)(ws + h->lay.part_o_off);
    p.part_lse = (float*)(ws + h->lay.part_lse_off);
    p.counters = (uint32_t*)(ws + h->lay.counters_off);
    p.B = c.B; p.Hq = c.Hq; p.Hkv = c.Hkv; p.G = h->G; p.S_max = c.S_max;
    p.n_splits = n_splits;
    p.max_splits = c.max_splits;
    p.xcd_groups = X;
    const float scale = c.scale > 0.f ? c.scale : 1.0f / std::sqrt((float)c.D);
    p.scale_log2 = scale * 1.4426950408889634f;

    hipStream_t st = (hipStream_t)stream;
    h->last_grid = (int)grid;
    switch (h->G) {
        case 1: return launch_g<1>(h, p, fused, (int)grid, st);
        case 2: return launch_g<2>(h, p, fused, (int)grid, st);
        case 3: return launch_g<3>(h, p, fused, (int)grid, st);
        case 4: return launch_g<4>(h, p, fused, (int)grid, st);
        case 5: return launch_g<5>(h, p, fused, (int)grid, st);
        case 6: return launch_g<6>(h, p, fused, (int)grid, st);
        case 7: return launch_g<7>(h, p, fused, (int)grid, st);
        case 8: return launch_g<8>(h, p, fused, (int)grid, st);
        default: return fail(FD_ERR_UNSUPPORTED, "GQA group %d is not built", h->G);
    }
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
    h->opt_path = h->opt_xcd = h->opt_wgs_per_cu = 0;
    h->last_grid = h->last_path = 0;
    hipError_t e = hipMalloc(&h->workspace, h->lay.total);
    if (e != hipSuccess) {
        const size_t want = h->lay.total;
        delete h;
        return fail(FD_ERR_WORKSPACE, "hipMalloc of %zu workspace bytes failed: %s", want, hipGetErrorString(e));
    }
    e = hipMemset((char*)h->workspace + h->lay.counters_off, 0, h->lay.total - h->lay.counters_off);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipFree(h->workspace);
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
    delete h;
    if (e != hipSuccess) return fail(FD_ERR_HIP, "hipFree: %s", hipGetErrorString(e));
    return FD_OK;
}

int fd_reset(fd_handle_t h, void* stream)
{
    int rc = check_handle(h);
    if (rc) return rc;
    FD_HIP(hipMemsetAsync((char*)h->workspace + h->lay.counters_off, 0, h->lay.total - h->lay.counters_off,
                          (hipStream_t)stream));
    return FD_OK;
}

int fd_decode(fd_handle_t h, const void* q, const void* k_cache, const void* v_cache, const int32_t* seq_lens,
              float* out, float* lse, int32_t n_splits, void* stream)
{
    return decode_common(h, q, k_cache, v_cache, seq_lens, out, lse, n_splits, stream, true);
}

int fd_decode_bsp(fd_handle_t h, const void* q, const void* k_cache, const void* v_cache, const int32_t* seq_lens,
                  float* out, float* lse, int32_t n_splits, void* stream)
{
    return decode_common(h, q, k_cache, v_cache, seq_lens, out, lse, n_splits, stream, false);
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
    FD_HIP(hipMemsetAsync(h->workspace, 0xFF, h->lay.counters_off, (hipStream_t)stream));
    return FD_OK;
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

const char* fd_last_error(void) { return g_err; }

int fd_version(void) { return FD_VERSION; }

}  // extern "C"
