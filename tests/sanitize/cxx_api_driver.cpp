// Compiles include/tcr.hpp as C++11 and calls every wrapper with arguments that the library rejects before it
// touches a device (null pointers, n == 0): the wrappers must hand their arguments on unchanged.
#include <cstdio>
#include <cstring>

#include "tcr.hpp"

#define CHECK(cond)                                               \
    do {                                                          \
        if (!(cond)) {                                            \
            std::printf("failed: %s (line %d)\n", #cond, __LINE__); \
            return 1;                                             \
        }                                                         \
    } while (0)

int main() {
    float out[4] = {0};
    const uint64_t offsets[2] = {0, 0};
    CHECK(tcr::SegmentedReduce(nullptr, out, 16, 16) == TCR_ERR_INVALID_ARG);
    CHECK(tcr::SegmentedScan(nullptr, out, 16, 16) == TCR_ERR_INVALID_ARG);
    CHECK(tcr::Reduce(nullptr, out, 16) == TCR_ERR_INVALID_ARG);
    CHECK(tcr::Scan(nullptr, out, 16) == TCR_ERR_INVALID_ARG);
    CHECK(tcr::SegmentedScan(nullptr, static_cast<void*>(out), 16, 16, tcr::kExclusive | tcr::kOutF16) == TCR_ERR_INVALID_ARG);
    CHECK(tcr::Scan(nullptr, static_cast<void*>(out), 16, tcr::kExclusive) == TCR_ERR_INVALID_ARG);
    CHECK(tcr::SegmentedScan(out, out, 16, 16, 8u) == TCR_ERR_INVALID_ARG);                    // an unknown flag
    CHECK(tcr::SegmentedScan(out, out, 16, 16, tcr::kAccF16) == TCR_ERR_INVALID_ARG);          // needs kOutF16
    CHECK(tcr::SegmentedReduce(nullptr, offsets, out, 16, 1) == TCR_ERR_INVALID_ARG);
    CHECK(tcr::SegmentedScan(nullptr, offsets, out, 16, 1) == TCR_ERR_INVALID_ARG);
    CHECK(tcr::SegmentedScan(nullptr, offsets, static_cast<void*>(out), 16, 1, tcr::kExclusive) == TCR_ERR_INVALID_ARG);
    CHECK(tcr::SegmentedMoments(nullptr, out, out + 1, 16, 16) == TCR_ERR_INVALID_ARG);
    CHECK(tcr::SegmentedMoments(nullptr, offsets, out, out + 1, 16, 1) == TCR_ERR_INVALID_ARG);
    CHECK(tcr::SegmentedReduce(out, out + 1, 15, 4) == TCR_ERR_INVALID_ARG);                   // seg_len does not divide n
    CHECK(tcr::SegmentedReduce(out, out, 0, 16) == TCR_OK);                                     // n == 0: nothing to do
    CHECK(tcr::SegmentedScan(out, out, 0, 16) == TCR_OK);
    CHECK(std::strcmp(tcr::status_string(TCR_ERR_INVALID_ARG), tcr_status_string(TCR_ERR_INVALID_ARG)) == 0);
    std::printf("ok\n");
    return 0;
}
