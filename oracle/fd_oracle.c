/*
 * fd_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain fp64 CPU definition of what the Flash Decode hot path computes:
 * single-query softmax attention over a bf16 KV cache, plus the log-sum-exp
 * (LSE) of the scores, and the online-softmax "Combine" of partial results.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may load
 * this file.  It shares no code, header, table or helper with the HIP library;
 * the product never calls it.
 *
 * What it follows (paper: "Eliminating Multi-GPU Performance Taxes"):
 *   - Section 4.2.1 (Flash Decode overview): attention of one query against a
 *     KV shard, normalised partial values per shard, then a combine that gives
 *     the globally correct output.  The split + combine is an exact
 *     reformulation of plain softmax attention, so fd_oracle_decode() is the
 *     textbook definition written out: two passes, no tiling, no online update.
 *   - Algorithm 4, Part 2 ("Combine ... reduce via online softmax"):
 *     fd_oracle_merge() merges normalised partials (o_i, lse_i).
 *   The paper never prints the formulas (it cites Flash-Decoding and the
 *   online-softmax paper); the readings taken here (scale 1/sqrt(D), natural-log
 *   LSE, query head h uses KV head h / (Hq/Hkv), empty range -> out 0 and
 *   lse -inf) are listed in the design notes of the repository.
 *
 * Parity pins (tests/test_oracle_pins.py): closed forms (one key, identical
 * keys, zero keys, two keys = logistic weights, one dominant key), invariants
 * (merge of any partition == unsplit, key permutation, score shift, convex
 * hull), fp64 library softmax-attention / logsumexp, and a pure-Python brute
 * force on tiny shapes.
 *
 * Layouts (all host pointers, row-major, caller owns everything):
 *   q        [B, Hq, D]           uint16 = raw bf16 bit patterns
 *   k, v     [B, Hkv, S_max, D]   uint16 = raw bf16 bit patterns
 *   seq_lens [B]                  int32, 0 <= seq_lens[b] <= S_max
 *   out      [B, Hq, D]           double
 *   lse      [B, Hq]              double, natural log
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* bf16 is the upper half of an IEEE binary32: widen exactly. */
static double bf16_bits_to_double(uint16_t bits)
{
    uint32_t w = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/*
 * IEEE binary16 (1 sign, 5 exponent, 10 fraction bits) widened exactly: the paper's own
 * precision (Section 5.1 runs its kernels in FP16).  Subnormals are f * 2^-24, exponent 31
 * is infinity / NaN.
 */
static double fp16_bits_to_double(uint16_t bits)
{
    const int sign = bits >> 15, e = (bits >> 10) & 31, f = bits & 1023;
    double mag;
    if (e == 0) mag = ldexp((double)f, -24);
    else if (e == 31) mag = f ? NAN : INFINITY;
    else mag = ldexp((double)(1024 + f), e - 25);
    return sign ? -mag : mag;
}

/* fmt 0: bf16 bit patterns, 1: fp16 bit patterns */
static double elem_to_double(uint16_t bits, int fmt)
{
    return fmt == 1 ? fp16_bits_to_double(bits) : bf16_bits_to_double(bits);
}

/*
 * Attention of query row (b, h) over keys j in [j0, j1) of its KV head.
 * scores: caller-provided scratch of at least (j1 - j0) doubles.
 * Writes out_row[D] and *lse_row.  Empty range: zeros and -inf.
 */
static void attend_range(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                         int Hq, int Hkv, int D, int64_t S_max, double scale,
                         int b, int h, int64_t j0, int64_t j1,
                         double* scores, double* out_row, double* lse_row, int fmt)
{
    const int G = Hq / Hkv;
    const int kvh = h / G;
    const uint16_t* qrow = q + ((int64_t)b * Hq + h) * D;
    const uint16_t* kbase = k + ((int64_t)b * Hkv + kvh) * S_max * D;
    const uint16_t* vbase = v + ((int64_t)b * Hkv + kvh) * S_max * D;

    for (int d = 0; d < D; ++d) out_row[d] = 0.0;
    if (j1 <= j0) {
        *lse_row = -INFINITY;
        return;
    }

    /* pass 1: s_j = scale * <q, k_j>, and the maximum */
    double m = -INFINITY;
    for (int64_t j = j0; j < j1; ++j) {
        const uint16_t* krow = kbase + j * D;
        double dot = 0.0;
        for (int d = 0; d < D; ++d)
            dot += elem_to_double(qrow[d], fmt) * elem_to_double(krow[d], fmt);
        double s = scale * dot;
        scores[j - j0] = s;
        if (s > m) m = s;
    }

    /* pass 2: l = sum exp(s_j - m); out = sum (exp(s_j - m) / l) v_j */
    double l = 0.0;
    for (int64_t j = j0; j < j1; ++j) l += exp(scores[j - j0] - m);
    for (int64_t j = j0; j < j1; ++j) {
        const double w = exp(scores[j - j0] - m) / l;
        const uint16_t* vrow = vbase + j * D;
        for (int d = 0; d < D; ++d) out_row[d] += w * elem_to_double(vrow[d], fmt);
    }
    *lse_row = m + log(l);
}

/*
 * Full decode attention for every (b, h).  scale <= 0 means 1/sqrt(D).
 * n_threads <= 0 means the OpenMP default.  Returns 0, or -1 on bad arguments
 * or allocation failure.
 */
int fd_oracle_decode_fmt(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                         const int32_t* seq_lens, int B, int Hq, int Hkv, int D,
                         int64_t S_max, double scale, int n_threads,
                         double* out, double* lse, int fmt)
{
    if (!q || !k || !v || !seq_lens || !out || !lse || fmt < 0 || fmt > 1) return -1;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || S_max <= 0 || Hq % Hkv) return -1;
    for (int b = 0; b < B; ++b)
        if (seq_lens[b] < 0 || seq_lens[b] > S_max) return -1;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)D);

    int failed = 0;
    const int rows = B * Hq;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif
#pragma omp parallel
    {
        double* scores = (double*)malloc(sizeof(double) * (size_t)S_max);
        if (!scores) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < rows; ++r) {
            if (!scores) continue;
            const int b = r / Hq, h = r % Hq;
            attend_range(q, k, v, Hq, Hkv, D, S_max, scale, b, h, 0, seq_lens[b],
                         scores, out + (int64_t)r * D, lse + r, fmt);
        }
        free(scores);
    }
    return failed ? -1 : 0;
}

/*
 * OCP FP8 E4M3 (the "fn" variant: 1 sign, 4 exponent bits with bias 7, 3 fraction bits; no
 * infinities, 0x7f / 0xff are NaN, largest finite value 448) widened exactly.
 */
static double fp8_e4m3_to_double(uint8_t bits)
{
    const int sign = bits >> 7, e = (bits >> 3) & 15, f = bits & 7;
    double mag;
    if (e == 15 && f == 7) mag = NAN;
    else if (e == 0) mag = ldexp((double)f, -9);
    else mag = ldexp((double)(8 + f), e - 10);
    return sign ? -mag : mag;
}

double fd_oracle_element_fp8(uint8_t bits) { return fp8_e4m3_to_double(bits); }

/*
 * Decode attention over an FP8 KV cache: q holds bf16 bit patterns, k and v hold E4M3
 * bytes; a stored byte stands for value * k_scale (resp. v_scale), i.e.
 *     s_j = scale * k_scale * <q, K8_j>,   out = v_scale * sum_j softmax(s)_j V8_j.
 * Same two passes as attend_range, written out again because the element types differ.
 */
int fd_oracle_decode_fp8kv(const uint16_t* q, const uint8_t* k, const uint8_t* v,
                           const int32_t* seq_lens, int B, int Hq, int Hkv, int D,
                           int64_t S_max, double scale, double k_scale, double v_scale,
                           int n_threads, double* out, double* lse)
{
    if (!q || !k || !v || !seq_lens || !out || !lse) return -1;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || S_max <= 0 || Hq % Hkv) return -1;
    if (!(k_scale > 0.0) || !(v_scale > 0.0)) return -1;
    for (int b = 0; b < B; ++b)
        if (seq_lens[b] < 0 || seq_lens[b] > S_max) return -1;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)D);
    const int G = Hq / Hkv;
    int failed = 0;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif
#pragma omp parallel
    {
        double* scores = (double*)malloc(sizeof(double) * (size_t)S_max);
        if (!scores) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < B * Hq; ++r) {
            if (!scores) continue;
            const int b = r / Hq, h = r % Hq, kvh = h / G;
            const uint16_t* qrow = q + (int64_t)r * D;
            const uint8_t* kbase = k + ((int64_t)b * Hkv + kvh) * S_max * D;
            const uint8_t* vbase = v + ((int64_t)b * Hkv + kvh) * S_max * D;
            double* out_row = out + (int64_t)r * D;
            const int64_t S = seq_lens[b];
            for (int d = 0; d < D; ++d) out_row[d] = 0.0;
            if (S == 0) {
                lse[r] = -INFINITY;
                continue;
            }
            double m = -INFINITY;
            for (int64_t j = 0; j < S; ++j) {
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += bf16_bits_to_double(qrow[d]) * fp8_e4m3_to_double(kbase[j * D + d]);
                scores[j] = scale * k_scale * dot;
                if (scores[j] > m) m = scores[j];
            }
            double l = 0.0;
            for (int64_t j = 0; j < S; ++j) l += exp(scores[j] - m);
            for (int64_t j = 0; j < S; ++j) {
                const double w = exp(scores[j] - m) / l;
                for (int d = 0; d < D; ++d) out_row[d] += w * fp8_e4m3_to_double(vbase[j * D + d]);
            }
            for (int d = 0; d < D; ++d) out_row[d] *= v_scale;
            lse[r] = m + log(l);
        }
        free(scores);
    }
    return failed ? -1 : 0;
}

/* The same for bf16 bit patterns (the benchmark's format). */
int fd_oracle_decode(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                     const int32_t* seq_lens, int B, int Hq, int Hkv, int D,
                     int64_t S_max, double scale, int n_threads,
                     double* out, double* lse)
{
    return fd_oracle_decode_fmt(q, k, v, seq_lens, B, Hq, Hkv, D, S_max, scale, n_threads, out, lse, 0);
}

/* Exact value of one stored element (for tests of the two formats). */
double fd_oracle_element(uint16_t bits, int fmt) { return elem_to_double(bits, fmt); }

/*
 * Attention of one query row (b, h) restricted to keys [j0, j1): the
 * "partial attention over a shard" of Section 4.2.1.  Used to build partials
 * for merge tests and to check sampled rows of large problems one by one.
 */
int fd_oracle_partial(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                      int Hq, int Hkv, int D, int64_t S_max, double scale,
                      int b, int h, int64_t j0, int64_t j1,
                      double* out_row, double* lse_row)
{
    if (!q || !k || !v || !out_row || !lse_row) return -1;
    if (Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv || b < 0 || h < 0 || h >= Hq) return -1;
    if (j0 < 0 || j1 > S_max) return -1;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)D);
    double* scores = (double*)malloc(sizeof(double) * (size_t)(j1 > j0 ? j1 - j0 : 1));
    if (!scores) return -1;
    attend_range(q, k, v, Hq, Hkv, D, S_max, scale, b, h, j0, j1, scores, out_row, lse_row, 0);
    free(scores);
    return 0;
}

/*
 * Combine of Algorithm 4, Part 2: n normalised partials (o_i[D], lse_i) of
 * disjoint key sets give
 *     L   = max_i lse_i + ln sum_i exp(lse_i - max)
 *     out = sum_i exp(lse_i - L) * o_i
 * Partials with lse_i = -inf (empty key set) carry weight zero and are
 * skipped.  All empty: out = 0, L = -inf.
 */
int fd_oracle_merge(const double* part_o, const double* part_lse, int n, int D,
                    double* out_row, double* lse_row)
{
    if (!part_o || !part_lse || !out_row || !lse_row || n < 0 || D <= 0) return -1;
    for (int d = 0; d < D; ++d) out_row[d] = 0.0;
    double mx = -INFINITY;
    for (int i = 0; i < n; ++i)
        if (part_lse[i] > mx) mx = part_lse[i];
    if (mx == -INFINITY) {
        *lse_row = -INFINITY;
        return 0;
    }
    double sum = 0.0;
    for (int i = 0; i < n; ++i)
        if (part_lse[i] != -INFINITY) sum += exp(part_lse[i] - mx);
    const double L = mx + log(sum);
    for (int i = 0; i < n; ++i) {
        if (part_lse[i] == -INFINITY) continue;
        const double w = exp(part_lse[i] - L);
        for (int d = 0; d < D; ++d) out_row[d] += w * part_o[(int64_t)i * D + d];
    }
    *lse_row = L;
    return 0;
}

int fd_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
