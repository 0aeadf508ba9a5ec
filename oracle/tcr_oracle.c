/*
 * CPU oracle for segmented / full sum-reduction and inclusive scan of binary16 data.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP library is checked
 * against; nothing in the product path may call it.  It shares no code, header,
 * table or helper with the HIP sources.
 *
 * What it computes is the plain definition given at the start of Section 3 of the
 * paper ("Reduction and Scan on GPUs"):
 *   - the reduction of a vector is the sum of its elements;
 *   - the scan (prefix sum) of a vector is the vector of running sums, the first
 *     entry being the first element and the last entry being the total, i.e. the
 *     scan is inclusive;
 *   - the regular segmented forms apply the same operation independently to
 *     consecutive, equally sized pieces of the input;
 * plus the exclusive variant of the scan (each output leaves out its own element), irregular segments
 * given by an offsets array, and the first two moments of every segment.
 * The matrix-product algorithms of Sections 4 and 5 reach exactly these results (up
 * to the order of floating-point additions), so the oracle is the definition written
 * out: one left-to-right loop per segment, accumulating in binary64.  Each binary16
 * input is widened exactly (every binary16 value is representable in binary64) by a
 * bit-level decoder written here; no half-precision library type is used.
 *
 * All pointers are host pointers.  Functions return 0 on success, 1 on a bad argument
 * (null pointer with n > 0, seg_len == 0, or n not a multiple of seg_len).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

/* binary16 bit pattern -> binary64 value: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
double oracle_half_to_double(uint16_t h)
{
    const int sign = (h >> 15) & 1;
    const int expo = (h >> 10) & 0x1f;
    const int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);                 /* zero and subnormals: frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), expo - 25);  /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

static int bad_args(const void *in, const void *out, uint64_t n, uint64_t seg_len)
{
    if (seg_len == 0) return 1;
    if (n % seg_len != 0) return 1;
    if (n > 0 && (in == NULL || out == NULL)) return 1;
    return 0;
}

#ifdef _OPENMP
/*
 * The timed multi-core build only (never the yardstick): a segment longer than kOmpChunk elements is cut into
 * chunks of that fixed size, whatever the number of threads, so that the additions always come in the same
 * order.  Reduce: chunk sums side by side, then added in chunk order.  Scan: chunk totals, their running sums
 * in chunk order, then every chunk scanned from the sum in front of it (the chunked two-pass scan).  The results
 * differ from the left-to-right loops only in the order of binary64 additions: not at all for integer-valued
 * data, by parts in 10^12 otherwise.
 */
#include <stdlib.h>
enum { kOmpChunk = 1 << 16 };

static double chunk_sum(const uint16_t *in, uint64_t from, uint64_t to)
{
    double acc = 0.0;
    for (uint64_t k = from; k < to; ++k) acc += oracle_half_to_double(in[k]);
    return acc;
}

/* totals[c] = sum of chunk c of the segment [begin, begin + len), c = 0 .. chunks - 1 */
static double *chunk_totals(const uint16_t *in, uint64_t begin, uint64_t len, uint64_t chunks)
{
    double *totals = (double *)malloc(chunks * sizeof(double));
    if (totals == NULL) return NULL;
#pragma omp parallel for schedule(static)
    for (uint64_t c = 0; c < chunks; ++c) {
        const uint64_t from = begin + c * kOmpChunk;
        const uint64_t to = (c + 1) * kOmpChunk < len ? from + kOmpChunk : begin + len;
        totals[c] = chunk_sum(in, from, to);
    }
    return totals;
}
#endif

/* out[s] = sum_{k=0}^{seg_len-1} in[s*seg_len + k],   s = 0 .. n/seg_len - 1. */
int oracle_segmented_reduce(const uint16_t *in, double *out, uint64_t n, uint64_t seg_len)
{
    if (bad_args(in, out, n, seg_len)) return 1;
    const uint64_t segs = n / seg_len;
#ifdef _OPENMP                      /* the timed multi-core build: the same loop, segments shared among threads */
    if (seg_len > 2 * (uint64_t)kOmpChunk) {        /* few long segments: the chunks of one segment side by side */
        const uint64_t chunks = (seg_len + kOmpChunk - 1) / kOmpChunk;
        for (uint64_t s = 0; s < segs; ++s) {
            double *totals = chunk_totals(in, s * seg_len, seg_len, chunks);
            if (totals == NULL) return 1;
            double acc = 0.0;
            for (uint64_t c = 0; c < chunks; ++c) acc += totals[c];
            out[s] = acc;
            free(totals);
        }
        return 0;
    }
#pragma omp parallel for schedule(static)
#endif
    for (uint64_t s = 0; s < segs; ++s) {
        double acc = 0.0;
        for (uint64_t k = 0; k < seg_len; ++k)
            acc += oracle_half_to_double(in[s * seg_len + k]);
        out[s] = acc;
    }
    return 0;
}

/* out[s*seg_len + k] = sum_{j=0}^{k} in[s*seg_len + j]   (inclusive). */
int oracle_segmented_scan(const uint16_t *in, double *out, uint64_t n, uint64_t seg_len)
{
    if (bad_args(in, out, n, seg_len)) return 1;
    const uint64_t segs = n / seg_len;
#ifdef _OPENMP
    if (seg_len > 2 * (uint64_t)kOmpChunk) {        /* few long segments: the chunked two-pass scan */
        const uint64_t chunks = (seg_len + kOmpChunk - 1) / kOmpChunk;
        for (uint64_t s = 0; s < segs; ++s) {
            const uint64_t begin = s * seg_len;
            double *totals = chunk_totals(in, begin, seg_len, chunks);
            if (totals == NULL) return 1;
            double run = 0.0;                       /* totals[c] becomes the sum in front of chunk c */
            for (uint64_t c = 0; c < chunks; ++c) {
                const double t = totals[c];
                totals[c] = run;
                run += t;
            }
#pragma omp parallel for schedule(static)
            for (uint64_t c = 0; c < chunks; ++c) {
                const uint64_t from = begin + c * kOmpChunk;
                const uint64_t to = (c + 1) * kOmpChunk < seg_len ? from + kOmpChunk : begin + seg_len;
                double acc = totals[c];
                for (uint64_t k = from; k < to; ++k) {
                    acc += oracle_half_to_double(in[k]);
                    out[k] = acc;
                }
            }
            free(totals);
        }
        return 0;
    }
#pragma omp parallel for schedule(static)
#endif
    for (uint64_t s = 0; s < segs; ++s) {
        double acc = 0.0;
        for (uint64_t k = 0; k < seg_len; ++k) {
            acc += oracle_half_to_double(in[s * seg_len + k]);
            out[s * seg_len + k] = acc;
        }
    }
    return 0;
}

/*
 * Exclusive form: out[s*seg_len + k] = sum_{j=0}^{k-1} in[s*seg_len + j]; the first output of a
 * segment is 0.  (Section 5 of the paper uses exclusive scans of tile columns internally; as a
 * user-facing variant it is the inclusive scan of Section 3 with each output leaving out its own
 * element.)
 */
int oracle_segmented_scan_exclusive(const uint16_t *in, double *out, uint64_t n, uint64_t seg_len)
{
    if (bad_args(in, out, n, seg_len)) return 1;
    const uint64_t segs = n / seg_len;
    for (uint64_t s = 0; s < segs; ++s) {
        double acc = 0.0;
        for (uint64_t k = 0; k < seg_len; ++k) {
            out[s * seg_len + k] = acc;
            acc += oracle_half_to_double(in[s * seg_len + k]);
        }
    }
    return 0;
}

/*
 * Irregular segments (the paper mentions them in a footnote of Section 3 and reduces them to the
 * regular case by padding; the result is the same as applying the definition to each piece):
 * segment s is in[offsets[s] .. offsets[s+1]), offsets has nseg + 1 non-decreasing entries.
 *   reduce: out[s] = sum of segment s (0 if empty).
 *   scan:   out[k] = sum of in[offsets[s] .. k] for every k in segment s (out indexed like in;
 *           entries outside the segments are left untouched).
 */
int oracle_irregular_reduce(const uint16_t *in, const uint64_t *offsets, double *out, uint64_t nseg)
{
    if (nseg > 0 && (in == NULL || offsets == NULL || out == NULL)) return 1;
    for (uint64_t s = 0; s < nseg; ++s) {
        if (offsets[s + 1] < offsets[s]) return 1;
        double acc = 0.0;
        for (uint64_t k = offsets[s]; k < offsets[s + 1]; ++k)
            acc += oracle_half_to_double(in[k]);
        out[s] = acc;
    }
    return 0;
}

int oracle_irregular_scan(const uint16_t *in, const uint64_t *offsets, double *out, uint64_t nseg)
{
    if (nseg > 0 && (in == NULL || offsets == NULL || out == NULL)) return 1;
    for (uint64_t s = 0; s < nseg; ++s) {
        if (offsets[s + 1] < offsets[s]) return 1;
        double acc = 0.0;
        for (uint64_t k = offsets[s]; k < offsets[s + 1]; ++k) {
            acc += oracle_half_to_double(in[k]);
            out[k] = acc;
        }
    }
    return 0;
}

/* Exclusive form of the irregular scan: out[k] = sum of the elements of k's segment in front of k. */
int oracle_irregular_scan_exclusive(const uint16_t *in, const uint64_t *offsets, double *out, uint64_t nseg)
{
    if (nseg > 0 && (in == NULL || offsets == NULL || out == NULL)) return 1;
    for (uint64_t s = 0; s < nseg; ++s) {
        if (offsets[s + 1] < offsets[s]) return 1;
        double acc = 0.0;
        for (uint64_t k = offsets[s]; k < offsets[s + 1]; ++k) {
            out[k] = acc;
            acc += oracle_half_to_double(in[k]);
        }
    }
    return 0;
}

/*
 * First two moments of every segment -- the reduction the paper's conclusion points at as the next use of
 * the method (mean and variance for batch normalisation):
 *   sum[s]   = sum_{k < seg_len} x[s*seg_len + k]
 *   sumsq[s] = sum_{k < seg_len} x[s*seg_len + k]^2
 * The square of a binary16 value has at most 22 significant bits, so every product is exact in binary64.
 */
int oracle_segmented_moments(const uint16_t *in, double *sum, double *sumsq, uint64_t n, uint64_t seg_len)
{
    if (bad_args(in, sum, n, seg_len)) return 1;
    if (n > 0 && sumsq == NULL) return 1;
    const uint64_t segs = n / seg_len;
    for (uint64_t s = 0; s < segs; ++s) {
        double a = 0.0, q = 0.0;
        for (uint64_t k = 0; k < seg_len; ++k) {
            const double v = oracle_half_to_double(in[s * seg_len + k]);
            a += v;
            q += v * v;
        }
        sum[s] = a;
        sumsq[s] = q;
    }
    return 0;
}

/* The two moments of irregular segments: segment s is in[offsets[s] .. offsets[s+1]); empty segments give 0, 0. */
int oracle_irregular_moments(const uint16_t *in, const uint64_t *offsets, double *sum, double *sumsq, uint64_t nseg)
{
    if (nseg > 0 && (in == NULL || offsets == NULL || sum == NULL || sumsq == NULL)) return 1;
    for (uint64_t s = 0; s < nseg; ++s) {
        if (offsets[s + 1] < offsets[s]) return 1;
        double a = 0.0, q = 0.0;
        for (uint64_t k = offsets[s]; k < offsets[s + 1]; ++k) {
            const double v = oracle_half_to_double(in[k]);
            a += v;
            q += v * v;
        }
        sum[s] = a;
        sumsq[s] = q;
    }
    return 0;
}

/*
 * binary64 value -> nearest binary16 bit pattern, ties to the even significand, magnitudes from 65520 on to
 * infinity, results below 2^-14 as subnormals (multiples of 2^-24).  Written out on the integer significand; no
 * half-precision library type or conversion instruction is used.
 */
uint16_t oracle_double_to_half(double v)
{
    const uint16_t sign = signbit(v) ? 0x8000u : 0u;
    if (isnan(v)) return (uint16_t)(sign | 0x7e00u);
    double a = fabs(v);
    if (isinf(a)) return (uint16_t)(sign | 0x7c00u);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                            /* a = m * 2^e with 0.5 <= m < 1: a lies in [2^(e-1), 2^e) */
    int ulp_exp = e - 1 - 10;                      /* a normal binary16 number near a is a multiple of 2^(e-11) */
    if (ulp_exp < -24) ulp_exp = -24;              /* subnormal range: multiples of 2^-24 */
    const double scaled = ldexp(a, -ulp_exp);      /* exact: a in units of the spacing; < 2048 */
    double whole = floor(scaled);
    const double rest = scaled - whole;            /* exact */
    if (rest > 0.5 || (rest == 0.5 && fmod(whole, 2.0) == 1.0)) whole += 1.0;
    const double r = ldexp(whole, ulp_exp);        /* the rounded magnitude, exact in binary64 */
    if (r >= 65536.0) return (uint16_t)(sign | 0x7c00u);
    if (r == 0.0) return sign;
    /* encode r: it is a binary16 value now */
    int re;
    (void)frexp(r, &re);
    if (re - 1 < -14) return (uint16_t)(sign | (uint16_t)ldexp(r, 24));         /* subnormal: fraction = r / 2^-24 */
    const int biased = re - 1 + 15;
    const uint16_t frac = (uint16_t)(ldexp(r, 10 - (re - 1)) - 1024.0);
    return (uint16_t)(sign | (uint16_t)(biased << 10) | frac);
}

/*
 * The scan with a binary16 accumulator, the precision of the paper's half-precision mode (Section 2.2: the
 * matrix units take binary16 inputs and accumulate in binary16 or binary32; Section 6 counts 2 bytes per
 * scanned output).  The definition of Section 3 is taken in its own order, left to right, and every addition
 * is rounded to binary16 at once:
 *     acc_0 = 0,   acc_{k+1} = round16(acc_k + x_k),   inclusive: out[k] = acc_{k+1},   exclusive: out[k] = acc_k.
 * The sum of two binary16 values is exact in binary64 (their bits span less than 53 positions), so each step
 * rounds exactly once.  out receives binary16 bit patterns.
 */
int oracle_segmented_scan_half_acc(const uint16_t *in, uint16_t *out, uint64_t n, uint64_t seg_len, int exclusive)
{
    if (bad_args(in, out, n, seg_len)) return 1;
    const uint64_t segs = n / seg_len;
    for (uint64_t s = 0; s < segs; ++s) {
        uint16_t acc = 0;
        for (uint64_t k = 0; k < seg_len; ++k) {
            const uint16_t next = oracle_double_to_half(oracle_half_to_double(acc) + oracle_half_to_double(in[s * seg_len + k]));
            out[s * seg_len + k] = exclusive ? acc : next;
            acc = next;
        }
    }
    return 0;
}

/* Full (unsegmented) forms: one segment that spans the whole input. */
int oracle_reduce(const uint16_t *in, double *out, uint64_t n)
{
    if (n == 0) {
        if (out) out[0] = 0.0;
        return out ? 0 : 1;
    }
    return oracle_segmented_reduce(in, out, n, n);
}

int oracle_scan(const uint16_t *in, double *out, uint64_t n)
{
    if (n == 0) return 0;
    return oracle_segmented_scan(in, out, n, n);
}

/*
 * Sampled inclusive-scan outputs, one by one: out[q] = sum of in[first .. idx[q]] where
 * first is the start of the segment containing idx[q].  Used to check a few outputs of
 * an input too large to scan and hold on the host in binary64.
 */
int oracle_segmented_scan_at(const uint16_t *in, uint64_t n, uint64_t seg_len,
                             const uint64_t *idx, uint64_t count, double *out)
{
    if (seg_len == 0 || n % seg_len != 0) return 1;
    if (count > 0 && (in == NULL || idx == NULL || out == NULL)) return 1;
    for (uint64_t q = 0; q < count; ++q) {
        if (idx[q] >= n) return 1;
        const uint64_t first = idx[q] - idx[q] % seg_len;
        double acc = 0.0;
        for (uint64_t k = first; k <= idx[q]; ++k)
            acc += oracle_half_to_double(in[k]);
        out[q] = acc;
    }
    return 0;
}
