/* Exercises the host side of libtcr.so that needs no GPU -- argument validation, the tuning table's text form,
 * the dispatch names, the workspace bound, the variant switch -- against a build whose host code carries
 * -fsanitize=address,undefined.  Prints "ok" and exits 0.  Test infrastructure only. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/tcr.h"

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void)
{
    char *buf = malloc(8192);
    CHECK(buf != NULL);
    void *in = buf, *out = buf + 4096;                 /* host addresses, never followed: every call below fails validation */
    CHECK(tcr_segmented_reduce(in, (float *)out, 64, 0, NULL) == TCR_ERR_INVALID_ARG);
    CHECK(tcr_segmented_scan(in, (float *)out, 65, 16, NULL) == TCR_ERR_INVALID_ARG);
    CHECK(tcr_segmented_scan_ex(in, out, 64, 16, 8, NULL) == TCR_ERR_INVALID_ARG);
    CHECK(tcr_segmented_scan_ex(in, out, 64, 16, TCR_ACC_F16, NULL) == TCR_ERR_INVALID_ARG);
    CHECK(tcr_segmented_scan_noalloc(in, (float *)out, (1ull << 30) + 16, 16, NULL) == TCR_ERR_UNSUPPORTED);
    CHECK(tcr_scan(NULL, NULL, 0, NULL) == TCR_OK && tcr_segmented_reduce(NULL, NULL, 0, 16, NULL) == TCR_OK);
    CHECK(tcr_irregular_reduce(in, NULL, (float *)out, 64, 3, NULL) == TCR_ERR_INVALID_ARG);
    CHECK(tcr_segmented_moments(in, (float *)out, NULL, 64, 7, NULL) == TCR_ERR_INVALID_ARG);
    CHECK(tcr_autotune(9, in, (float *)out, 64, 16, NULL) == TCR_ERR_INVALID_ARG);
    CHECK(tcr_autotune_irregular(3, in, NULL, (float *)out, 64, 2, NULL) == TCR_ERR_INVALID_ARG);

    /* the tuning table as text: a buffer of exactly the reported size, truncation, rejected texts */
    const char *text = "scan:8=33;scan:41=13;reduce:20=1;scan_any:6=1;reduce_any:9=3;irregular:0=2;irregular:1=1;";
    CHECK(tcr_tuning_import(text) == TCR_OK);
    const uint64_t need = tcr_tuning_export(NULL, 0);
    CHECK(need == strlen(text) + 1);
    char *exact = malloc(need);
    CHECK(exact != NULL && tcr_tuning_export(exact, need) == need && strcmp(exact, text) == 0);
    char tiny[5];
    CHECK(tcr_tuning_export(tiny, sizeof tiny) == need && strcmp(tiny, "scan") == 0);
    char one[1];
    CHECK(tcr_tuning_export(one, 1) == need && one[0] == '\0');
    const char *rejected[] = {"scan", "scan:", "scan:1", "scan:1=", "scan:1=2", "scan:99=1;", "scan:-1=1;", "scan:1=-1;",
                              "scan:1=99999999999999999999;", "sc:1=1;", ";", "irregular:5=0;", "reduce_any:3=32;"};
    for (unsigned i = 0; i < sizeof rejected / sizeof rejected[0]; ++i) CHECK(tcr_tuning_import(rejected[i]) == TCR_ERR_INVALID_ARG);
    CHECK(tcr_tuning_import(NULL) == TCR_ERR_INVALID_ARG);
    CHECK(tcr_tuning_export(exact, need) == need && strcmp(exact, text) == 0);      /* untouched by the rejected ones */
    free(exact);

    /* dispatch names and the workspace bound over many sizes, with and without the table above */
    for (int round = 0; round < 2; ++round) {
        for (int op = -1; op <= 8; ++op) {
            for (int e = 0; e <= 38; e += 2) {
                const uint64_t lens[] = {0, 1, 3, 8, 16, 24, 100, 512, 1000, 4096, 8160, 8168, 65536, 100003, 1ull << 20, 3ull << 20, 1ull << 24};
                for (unsigned i = 0; i < sizeof lens / sizeof lens[0]; ++i) {
                    const uint64_t n = lens[i] ? ((1ull << e) / lens[i] + 1) * lens[i] : (1ull << e);
                    CHECK(tcr_kernel_name(op, n, lens[i]) != NULL);
                    (void)tcr_workspace_bytes(op, n, lens[i]);
                }
            }
        }
        CHECK(tcr_tuning_import("") == TCR_OK);
    }
    CHECK(tcr_set_variant("formulation", "dpp") == TCR_OK && tcr_set_variant("formulation", "x") == TCR_ERR_INVALID_ARG);
    CHECK(tcr_set_variant(NULL, "x") == TCR_ERR_INVALID_ARG && tcr_set_variant("untuned_reduce", "tiles") == TCR_OK);
    CHECK(tcr_set_variant("reset", "") == TCR_OK);
    for (int s = -1; s <= 6; ++s) CHECK(tcr_status_string(s) != NULL);
    CHECK(tcr_last_hip_error() != NULL);
    tcr_release();
    free(buf);
    puts("ok");
    return 0;
}
