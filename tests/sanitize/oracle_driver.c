/* Runs every function of the CPU oracle on small inputs, edge cases included, so that a build with
 * -fsanitize=address,undefined can watch it: out-of-bounds accesses, signed overflow, bad shifts.
 * Prints "ok" and exits 0 when every call returned what its contract says.  Test infrastructure only. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double oracle_half_to_double(uint16_t h);
uint16_t oracle_double_to_half(double v);
int oracle_segmented_reduce(const uint16_t *in, double *out, uint64_t n, uint64_t seg_len);
int oracle_segmented_scan(const uint16_t *in, double *out, uint64_t n, uint64_t seg_len);
int oracle_segmented_scan_exclusive(const uint16_t *in, double *out, uint64_t n, uint64_t seg_len);
int oracle_segmented_scan_half_acc(const uint16_t *in, uint16_t *out, uint64_t n, uint64_t seg_len, int exclusive);
int oracle_irregular_reduce(const uint16_t *in, const uint64_t *offsets, double *out, uint64_t nseg);
int oracle_irregular_scan(const uint16_t *in, const uint64_t *offsets, double *out, uint64_t nseg);
int oracle_irregular_scan_exclusive(const uint16_t *in, const uint64_t *offsets, double *out, uint64_t nseg);
int oracle_segmented_moments(const uint16_t *in, double *sum, double *sumsq, uint64_t n, uint64_t seg_len);
int oracle_irregular_moments(const uint16_t *in, const uint64_t *offsets, double *sum, double *sumsq, uint64_t nseg);
int oracle_reduce(const uint16_t *in, double *out, uint64_t n);
int oracle_scan(const uint16_t *in, double *out, uint64_t n);
int oracle_segmented_scan_at(const uint16_t *in, uint64_t n, uint64_t seg_len, const uint64_t *idx, uint64_t count, double *out);

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void)
{
    /* every bit pattern through the decoder and back */
    for (uint32_t b = 0; b < 65536; ++b) {
        const double v = oracle_half_to_double((uint16_t)b);
        if (!isnan(v)) CHECK(oracle_double_to_half(v) == (uint16_t)b);
    }
    CHECK(oracle_double_to_half(1e300) == 0x7c00 && oracle_double_to_half(-1e300) == 0xfc00);
    CHECK(oracle_double_to_half(1e-300) == 0 && oracle_double_to_half(NAN) == 0x7e00);

    enum { N = 3 * 5 * 7 * 8 };
    uint16_t *x = malloc(N * sizeof *x);            /* exactly N elements: one read past the end is caught */
    double *out = malloc(N * sizeof *out), *out2 = malloc(N * sizeof *out2);
    uint16_t *hout = malloc(N * sizeof *hout);
    CHECK(x && out && out2 && hout);
    for (int i = 0; i < N; ++i) x[i] = oracle_double_to_half((double)((i * 37) % 17 - 8));
    const uint64_t lens[] = {1, 2, 3, 5, 7, 8, 15, 24, 105, 840};
    for (unsigned i = 0; i < sizeof lens / sizeof lens[0]; ++i) {
        const uint64_t L = lens[i];
        CHECK(oracle_segmented_reduce(x, out, N, L) == 0);
        CHECK(oracle_segmented_scan(x, out, N, L) == 0);
        CHECK(oracle_segmented_scan_exclusive(x, out, N, L) == 0);
        CHECK(oracle_segmented_scan_half_acc(x, hout, N, L, 0) == 0);
        CHECK(oracle_segmented_scan_half_acc(x, hout, N, L, 1) == 0);
        CHECK(oracle_segmented_moments(x, out, out2, N, L) == 0);
    }
    CHECK(oracle_reduce(x, out, N) == 0 && oracle_scan(x, out, N) == 0);
    CHECK(oracle_reduce(x, out, 0) == 0 && out[0] == 0.0 && oracle_scan(NULL, NULL, 0) == 0);
    CHECK(oracle_segmented_reduce(x, out, N, 0) == 1 && oracle_segmented_scan(x, out, N, 11) == 1);
    CHECK(oracle_segmented_reduce(NULL, out, N, 8) == 1 && oracle_segmented_scan_half_acc(x, NULL, N, 8, 0) == 1);
    CHECK(oracle_segmented_reduce(NULL, NULL, 0, 8) == 0);

    const uint64_t off[] = {3, 3, 10, 10, 10, 500, N};   /* empty segments, a partial cover, the last element */
    const uint64_t nseg = sizeof off / sizeof off[0] - 1;
    double red[6], sq[6];
    CHECK(oracle_irregular_reduce(x, off, red, nseg) == 0 && red[0] == 0.0 && red[2] == 0.0);
    CHECK(oracle_irregular_scan(x, off, out, nseg) == 0 && oracle_irregular_scan_exclusive(x, off, out, nseg) == 0);
    CHECK(oracle_irregular_moments(x, off, red, sq, nseg) == 0);
    const uint64_t bad[] = {5, 4};
    CHECK(oracle_irregular_reduce(x, bad, red, 1) == 1 && oracle_irregular_reduce(NULL, NULL, NULL, 0) == 0);
    const uint64_t idx[] = {0, 7, 8, N - 1};
    double at[4];
    CHECK(oracle_segmented_scan_at(x, N, 8, idx, 4, at) == 0);
    const uint64_t beyond[] = {N};
    CHECK(oracle_segmented_scan_at(x, N, 8, beyond, 1, at) == 1);
    free(x); free(out); free(out2); free(hout);
    puts("ok");
    return 0;
}
