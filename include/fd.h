/*
 * fd.h -- C ABI of the MI355X (gfx950) Flash Decode library, libfd.so.
 *
 * Flash Decode = attention of ONE query token per sequence against a bf16 KV
 * cache.  The KV range of each sequence is cut into splits; every split is
 * attended independently (partial output + log-sum-exp), and the partials are
 * merged by the online-softmax Combine.  This is the single-GPU form of the
 * paper's Distributed Flash Decode (Section 4.2, Algorithm 4): a KV split plays
 * the role of a rank's KV shard, the partial buffer the role of the inbox, and
 * a per-(batch, KV head) arrival counter the role of the signal flags.
 *
 *   fd_decode      "fused": ONE persistent kernel.  The workgroup that finishes
 *                  the last split of a (batch, KV head) tile, detected with an
 *                  atomic counter, merges that tile's partials on the spot
 *                  (Section 4.2.5 "Fused Kernels"; Algorithm 4 Part 1 + Part 2
 *                  without the global barrier and without the second launch).
 *   fd_decode_bsp  bulk-synchronous baseline (Section 4.2.2): kernel 1 writes
 *                  all partials, kernel 2 merges them; stream order is the
 *                  global barrier.  Same arithmetic, bitwise-identical results.
 *
 * All tensor pointers are DEVICE pointers owned by the caller; the library
 * owns only the handle's workspace.  Calls are asynchronous on the caller's
 * stream: they never synchronise and never allocate.  Calls that share a
 * handle must be issued on one stream (they share the workspace).
 *
 * Every function returns FD_OK (0) or a negative FD_ERR_* code; the text of the
 * last error of the calling thread is available from fd_last_error().  No
 * exception crosses this boundary.  Argument checks happen on the host before
 * anything is launched.
 */
#ifndef FD_H_
#define FD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FD_VERSION 150

enum {
    FD_OK = 0,
    FD_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, n_splits out of range ...   */
    FD_ERR_UNSUPPORTED = -2, /* a shape the kernels are not built for (D != 128, G > 16 ...) */
    FD_ERR_WORKSPACE = -3,   /* workspace allocation failed / too small for this call        */
    FD_ERR_HIP = -4          /* a HIP runtime call failed (no device, launch error)          */
};

/* Keys per split used when the library picks the split count itself (FD_OPT_SPLIT_KEYS = 0); half
 * of it for shapes with very few items, see fd_decode. */
#define FD_ADAPTIVE_SPLIT_KEYS 512
/* Upper bound accepted for fd_config.max_splits. */
#define FD_MAX_SPLITS 1024

typedef struct fd_handle_s* fd_handle_t;

/*
 * Problem shape, fixed per handle.
 *   B           sequences in the batch (each contributes one query token)
 *   Hq, Hkv     query heads and KV heads; Hq % Hkv == 0; query head h reads KV
 *               head h / (Hq/Hkv) (consecutive query heads share a KV head)
 *   D           head dimension; only 128 is built
 *   S_max       row capacity of the KV cache per (sequence, KV head)
 *   max_splits  largest split count any call on this handle may use
 *               (1 .. FD_MAX_SPLITS); sizes the partial workspace
 *   kv_layout   0 = contiguous [B, Hkv, S_max, D] (the only layout)
 *   scale       softmax scale; 0 means 1/sqrt(D).  Applied in fp32 to the
 *               fp32 dot product (never folded into a re-rounded bf16 q).
 *   dtype       FD_DTYPE_BF16 (the benchmark's format) or FD_DTYPE_FP16 (IEEE half, the
 *               paper's format, Section 5.1): wherever the comments below say bf16, read
 *               "dtype".  Half inputs run on the MFMA kernel only (FD_OPT_PATH = 1 and
 *               fd_decode_waits are FD_ERR_UNSUPPORTED); sums are fp32 either way.
 *               FD_DTYPE_FP8_KV: q is bf16, k_cache and v_cache hold ONE BYTE per element,
 *               OCP FP8 E4M3 (largest value 448, 0x7f / 0xff = NaN), same [B, Hkv, S_max, D]
 *               shape; a byte stands for value * k_scale (v_scale):
 *               out = v_scale * softmax(scale * k_scale * q K8^T) V8.  Half the cache
 *               bytes per key.  MFMA kernel; fd_decode / fd_decode_bsp, and the paged entry
 *               points with pages of at least 32 keys (pool of bytes, same shape).
 *   k_scale,    per-tensor dequantisation factors of an FP8 cache (0 means 1); ignored for
 *   v_scale     the other dtypes
 */
typedef struct {
    int32_t B, Hq, Hkv, D, S_max;
    int32_t max_splits;
    int32_t kv_layout;
    float scale;
    int32_t dtype;
    float k_scale, v_scale;
} fd_config;

/* fd_config.dtype: element type of q, k_cache, v_cache (out and lse are always fp32). */
#define FD_DTYPE_BF16 0
#define FD_DTYPE_FP16 1
#define FD_DTYPE_FP8_KV 2

/* Bytes of device workspace (Algorithm 4's inbox and flags for this shape) fd_create() allocates
 * for cfg (0 if cfg is invalid). */
size_t fd_workspace_bytes(const fd_config* cfg);

/*
 * Validates cfg, allocates the workspace on the current HIP device (partials
 * [B,Hkv,max_splits,G,D] fp32, their LSEs, one arrival counter per tile; for the two-level
 * merge of tiles with very many partials, FD_OPT_TREE_ROWS, a second partial buffer of
 * ceil(max_splits/16) rows per tile and 64 group counters per tile), zeroes
 * the counters, and creates the stream and two events fd_decode_waits uses.
 * Synchronous.  *out receives the handle.
 * The workspace stands for Algorithm 4's inbox and signal flags.  The paper gives the problem
 * only as the inputs of Algorithm 4 (query, KV shard) and has no interface; a handle that fixes
 * the shape and owns inbox and flags is this library's reading.  The paper is also silent on how
 * the flags are re-armed between the calls of its timing loop (Section 5.1); here they start at
 * zero (this call) and the workgroup that merges a tile stores zero back, so that every
 * completed call leaves them ready for the next.
 */
int fd_create(const fd_config* cfg, fd_handle_t* out);

/* Frees the workspace and the handle.  NULL is FD_ERR_INVALID_ARG.  The caller makes sure no
 * call on the handle is still running. */
int fd_destroy(fd_handle_t h);

/*
 * Re-zeroes the arrival counters (Algorithm 4's flags) on `stream` (a hipStream_t, NULL =
 * default stream).  Only needed after a call was aborted mid-kernel or a fd_decode_waits call
 * gave up waiting: every completed call leaves the counters at zero by itself (see fd_create).
 * The clearing is a small kernel launch, not a memset, so the call may be recorded into a
 * HIP graph with the rest of the stream.
 */
int fd_reset(fd_handle_t h, void* stream);

/*
 * Fused Flash Decode (Algorithm 4 with Part 1 and Part 2 in one kernel).
 *
 *   q        [B, Hq, D]          bf16, device
 *   k_cache  [B, Hkv, S_max, D]  bf16, device; 16-byte aligned
 *   v_cache  [B, Hkv, S_max, D]  bf16, device; 16-byte aligned
 *   seq_lens [B] int32, device; 0 <= seq_lens[b] <= S_max.  Read on the device:
 *            the host never waits for it.  Rows >= seq_lens[b] never influence a result
 *            (they may hold anything, NaN included).  With n_splits > 0 a workgroup
 *            requests the first rows of its first split (up to 256, or 512 of an FP8
 *            cache) before seq_lens has arrived: rows below S_max of the
 *            [B, Hkv, S_max, D] arrays may therefore be read and dropped; nothing outside
 *            the arrays is touched.
 *   out      [B, Hq, D] fp32, device:  softmax(scale * q K^T) V
 *   lse      [B, Hq]    fp32, device, natural log of sum_j exp(score_j);
 *            may be NULL (then it is not written)
 *   n_splits > 0: the key axis [0, S_max) is cut into n_splits equal ranges of
 *                 ceil(S_max / n_splits) keys, rounded up to 64; a sequence uses the
 *                 ranges below seq_lens[b] (the last one cut short, the rest empty);
 *                 n_splits <= max_splits.
 *            = 0: adaptive, n_b = clamp(ceil(seq_lens[b]/512), 1, max_splits) ranges of
 *                 the sequence's own length, computed on the device (FD_OPT_SPLIT_KEYS
 *                 replaces the 512; left at 0, the library takes 256 instead when even
 *                 B*Hkv sequences of S_max keys would give no more items than a quarter
 *                 of the GPU's compute units).
 *   stream   hipStream_t (NULL = default stream)
 *
 * seq_lens[b] == 0 gives out = 0 and lse = -inf for that sequence.
 * The device that is current when the handle was created must be current for every call
 * on it (otherwise FD_ERR_INVALID_ARG, nothing is launched).
 * Accumulation is fp32; results match an fp64 evaluation of the definition to
 * about 1e-5 relative on N(0,1) data.
 */
int fd_decode(fd_handle_t h, const void* q, const void* k_cache, const void* v_cache,
              const int32_t* seq_lens, float* out, float* lse, int32_t n_splits, void* stream);

/*
 * Bulk-synchronous baseline (Section 4.2.2): same arguments, same results bit
 * for bit; two launches (partials, then combine) on `stream`.
 */
int fd_decode_bsp(fd_handle_t h, const void* q, const void* k_cache, const void* v_cache,
                  const int32_t* seq_lens, float* out, float* lse, int32_t n_splits,
                  void* stream);

/*
 * Fine-grained waits (Section 4.2.4), the paper's step between the bulk-synchronous baseline
 * and the fused kernel: same arguments and results (bitwise) as fd_decode.  Two kernels run
 * SIDE BY SIDE: kernel 1 (on `stream`) writes partials and bumps a tile's arrival counter;
 * the combine kernel (on a second stream the handle owns, forked from and joined to `stream`
 * with events, so that `stream` sees one operation) waits per tile until the counter is
 * complete, then merges that tile, while other tiles are still being attended.  Kernel 1
 * never waits, so the counts always complete; the combine kernel's wait is bounded all the
 * same (FD_OPT_SPIN_LIMIT polls, ~1 us each): if it ever gives up, FD_INFO_WAIT_GAVE_UP
 * reads 1, out / lse of that call are undefined, and fd_reset is needed before the next
 * call.  MFMA kernel, contiguous cache only (else FD_ERR_UNSUPPORTED).
 */
int fd_decode_waits(fd_handle_t h, const void* q, const void* k_cache, const void* v_cache,
                    const int32_t* seq_lens, float* out, float* lse, int32_t n_splits, void* stream);

/*
 * The same computation over a PAGED KV cache (the layout decode servers use).
 *
 *   k_pages, v_pages  [num_pages, Hkv, page_size, D] bf16, device, 16-byte aligned: the
 *                     page pool; the page_size rows of one (page, KV head) are contiguous
 *   block_table       [B, pages_per_seq] int32, device: key j of sequence b is row
 *                     j % page_size of pool page block_table[b][j / page_size].  Only
 *                     entries of pages below ceil(seq_lens[b] / page_size) are looked at;
 *                     entries outside [0, num_pages) are clamped into that range, so that
 *                     no access ever leaves the pool (the result is then meaningless)
 *   page_size         power of two, 16 .. 65536 keys
 *   pages_per_seq     row length of block_table; pages_per_seq * page_size >= S_max
 *   everything else   as for fd_decode (S_max of the handle bounds seq_lens[b])
 *
 * Rows at or past seq_lens[b] are never read here (no early request: the page must be looked
 * up first).  The MFMA kernel
 * serves every group size here (FD_OPT_PATH = 1 is FD_ERR_UNSUPPORTED): each wave looks up
 * the page of each of its 16-key blocks; page numbers are staged in LDS 256 blocks ahead,
 * so the streaming loop is the contiguous one plus one LDS read per block.
 * fd_decode_paged_bsp is the two-kernel baseline, bitwise equal as above.
 */
int fd_decode_paged(fd_handle_t h, const void* q, const void* k_pages, const void* v_pages,
                    const int32_t* block_table, int32_t page_size, int32_t pages_per_seq, int32_t num_pages,
                    const int32_t* seq_lens, float* out, float* lse, int32_t n_splits, void* stream);
int fd_decode_paged_bsp(fd_handle_t h, const void* q, const void* k_pages, const void* v_pages,
                        const int32_t* block_table, int32_t page_size, int32_t pages_per_seq,
                        int32_t num_pages, const int32_t* seq_lens, float* out, float* lse, int32_t n_splits,
                        void* stream);

/*
 * For callers that cannot allocate device memory or hold a handle (code recorded into a HIP
 * graph, tight serving loops, harnesses that forbid allocation): fd_decode with the shape passed
 * by value and the workspace in a static device array of FD_STATIC_SCRATCH_BYTES that the
 * library's code object carries (each GPU holds it from the first use of the library until the
 * process ends).  Arguments and results as for fd_decode on a handle made from *cfg with the
 * default options (bitwise the same results).  The call allocates nothing on the host or the
 * device and never synchronises; it launches one small kernel that clears the arrival counters
 * and then the fused kernel, both on `stream`.  The first call on a device looks up the array's
 * device address and the device's properties (make that call outside a graph capture).
 * A shape whose workspace (fd_workspace_bytes) exceeds FD_STATIC_SCRATCH_BYTES is refused with
 * FD_ERR_WORKSPACE: lower max_splits, or use a handle.
 * All calls on one GPU share the one array, which keeps what the last call left: calls that
 * overlap on one GPU (two streams, two threads) race and give undefined results; calls in
 * stream order on one stream are safe.
 */
#define FD_STATIC_SCRATCH_BYTES (32u << 20)
int fd_decode_static(const fd_config* cfg, const void* q, const void* k_cache, const void* v_cache,
                     const int32_t* seq_lens, float* out, float* lse, int32_t n_splits, void* stream);

/*
 * Picks the handle's options by measurement: SYNCHRONOUS, unlike every other call here.
 * The one-GPU counterpart of the paper's joint tuning of transfer granularity and kernel tiling
 * (Section 6.3).  Runs fd_decode on the given arguments (after 0.1 s of untimed calls: 3 untimed +
 * `reps` timed calls, HIP events on `stream`) for the options as they stand and for every
 * combination of
 *   - the split granularity FD_OPT_SPLIT_KEYS in {256, 512, 1024, 2048} when n_splits = 0
 *     (a fixed n_splits is the caller's choice and is left alone),
 *   - FD_OPT_XCD_GROUPS in {1, 8 where B*Hkv is a multiple of 8},
 *   - (FD_OPT_WGS_PER_CU, FD_OPT_RING_STAGES) in {(1,2), (2,2), (1,3), (1,4)} of the MFMA kernel
 *     (the deeper rings for bf16 only), plus the VALU kernel for bf16 with Hq/Hkv <= 8;
 * combinations the shape does not allow are skipped.  A winner other than the options the handle
 * came with is measured against them twice more and kept only if it is at least 0.5 % faster
 * both times (a per cent is inside the spread of one pass).  Leaves the handle set to the choice (read
 * it back with fd_get_option); *best_us (host, may be NULL) receives its mean time per
 * call in microseconds.  out / lse hold a result of the chosen combination afterwards.  On
 * error the options are left as they were.  The defaults are rules fitted to measurements
 * on a few shapes; this call replaces the rule by the measurement for the shape and the
 * data placement at hand (the rules miss by up to 10 % on shapes between their samples).
 * Results of later calls differ from the defaults' only in rounding (another partition).
 * What is measured is repeated calls on the caller's buffers: a cache that fits the 256 MB
 * Infinity Cache is then read from there, and the choice is the best for THAT (it can lose by a
 * few per cent where every call reads another cache from HBM, as the layers of a model do: the
 * defaults' rules were fitted to that case).
 */
int fd_autotune(fd_handle_t h, const void* q, const void* k_cache, const void* v_cache,
                const int32_t* seq_lens, float* out, float* lse, int32_t n_splits, void* stream,
                int32_t reps, float* best_us);

/*
 * Tuning / introspection knobs (per handle).  Unknown keys: FD_ERR_INVALID_ARG.
 *   FD_OPT_PATH          0 auto (the MFMA kernel), 1 VALU kernel (Hq/Hkv <= 8 only),
 *                        2 MFMA kernel
 *   FD_OPT_XCD_GROUPS    0 auto (by measurement: 8 when B*Hkv is a multiple of 8 and, for a
 *                        fixed split count, S_max <= 8192, or S_max <= 16384 with at least 64
 *                        tiles; for adaptive splits unless there are at most 32 tiles with
 *                        S_max > 16384; else 1), 1 = one global item list,
 *                        8 = items of a tile stay on one XCD (tile t -> workgroups with
 *                        id % 8 == t % 8)
 *   FD_OPT_WGS_PER_CU    persistent workgroups launched per compute unit (0 auto: 1 for the MFMA
 *                        kernel).  The MFMA kernel runs 1 or 2: a call with a larger value set
 *                        fails with FD_ERR_INVALID_ARG
 *   FD_OPT_RING_STAGES   MFMA kernel: stages (16 keys of K and V, 8 KB) in each wave's
 *                        LDS ring: 0 auto (2), 2, 3 or 4; always 2 with 2 workgroups per CU,
 *                        half inputs or a paged cache
 *   FD_OPT_SPIN_LIMIT    fd_decode_waits: polls before a waiting workgroup gives up (0 = 1048576, about a second)
 *   FD_OPT_TREE_ROWS     a tile with more partials than this is merged in two levels: groups of 16
 *                        partials by the workgroup that completes a group's arrival count, the
 *                        groups' results by the one that completes the tile's (one compute unit
 *                        pulling hundreds of partials would take longer than the K/V stream: one
 *                        long sequence on one or two KV heads).  0 auto (64), else >= 2.
 *                        fd_decode and fd_decode_bsp agree bitwise for any value; fd_decode_waits
 *                        always merges in one level and then differs from them in rounding
 *   FD_OPT_SPLIT_KEYS    n_splits = 0: keys per split the split count is derived from (0 = 512, or 256 for very few items, see fd_decode;
 *                        else a multiple of 64 in 64..65536)
 *   FD_INFO_*            read-only, through fd_get_option; FD_INFO_WAIT_GAVE_UP synchronises the device
 */
enum {
    FD_OPT_PATH = 1,
    FD_OPT_XCD_GROUPS = 2,
    FD_OPT_WGS_PER_CU = 3,
    FD_OPT_RING_STAGES = 4,
    FD_OPT_SPIN_LIMIT = 5,
    FD_OPT_SPLIT_KEYS = 6,
    FD_OPT_TREE_ROWS = 7,
    FD_INFO_NUM_CUS = 100,
    FD_INFO_LAST_GRID = 101,   /* workgroups of the last fused / split launch */
    FD_INFO_LAST_PATH = 102,   /* 1 VALU, 2 MFMA */
    FD_INFO_WAIT_GAVE_UP = 103 /* 1 after a fd_decode_waits call whose combine kernel gave up waiting */
};
int fd_set_option(fd_handle_t h, int32_t key, int32_t value);
int fd_get_option(fd_handle_t h, int32_t key, int32_t* value);

/*
 * Test aid: fills the partial workspace with NaN on `stream` (counters are left
 * alone), so that a combine that reads a partial nobody wrote shows up.
 */
int fd_debug_poison_workspace(fd_handle_t h, void* stream);
/* Test aid: copies the arrival counters to host memory (synchronous); n = B*Hkv. */
int fd_debug_read_counters(fd_handle_t h, uint32_t* host_dst, int32_t n);

/*
 * Tuning aid: attaches (or, with NULL, detaches) a device buffer of
 * capacity_workgroups * FD_TRACE_EVENTS uint64 in which every workgroup of later
 * fused / split launches records 100 MHz timestamps of its milestones: 0 start,
 * 1 first stage landed, 2 loop end, 3 partial stored, 4 stores acknowledged,
 * 5 counted, 6 combined, 7 end, and inside a combine 8 entered, 9 fence
 * passed, 10 weights ready, 11 rows accumulated (the last key range of the
 * workgroup wins; 0 = not reached).  Launches with more workgroups than the
 * capacity record nothing.  The caller owns the buffer.
 */
#define FD_TRACE_EVENTS 12
int fd_debug_set_trace(fd_handle_t h, void* device_buffer, int32_t capacity_workgroups);

/*
 * Measurement aid, no handle needed: one pass of 128-bit non-temporal loads (the loads of
 * the K/V stream) over `bytes` bytes (rounded down to 16) at src (device, 16-byte aligned),
 * one contiguous block per workgroup, one workgroup per compute unit; nothing is written
 * (sink, device, 4 bytes, only keeps the loads alive).  Asynchronous on `stream`.  Timing
 * it gives the bandwidth a read-only kernel reaches on this chip, the practical ceiling
 * for fd_decode.
 */
int fd_debug_stream_read(const void* src, size_t bytes, uint32_t* sink, void* stream);

/* Text of the calling thread's last error ("" if none). Never NULL. */
const char* fd_last_error(void);
int fd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FD_H_ */
