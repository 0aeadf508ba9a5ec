/*
 * tcr.hpp -- the C ABI of tcr.h under the names the paper gives its library (Section 6: "an API similar to CUB's,
 * providing functions such as SegmentedReduce, Reduce, SegmentedScan and Scan").  Header only: every function is an
 * inline call of the extern "C" entry point named beside it, with the same arguments, alignment rules, ownership
 * and error behaviour (see tcr.h); nothing is computed here.
 *
 *   in      device pointer to n binary16 values          out   device pointer, caller owned
 *   stream  a hipStream_t (passed on as void*; nullptr = the default stream)
 *   Every call returns a tcr_status; tcr::status_string gives its text.
 */
#ifndef TCR_HPP
#define TCR_HPP

#include "tcr.h"

namespace tcr {

/* Scan modes (Section 5 computes inclusive scans and, for the column carries, exclusive ones; Section 2.2 names
 * binary16 and binary32 accumulators): combine with |. */
enum ScanFlags : uint32_t {
    kInclusive = 0u,
    kExclusive = TCR_SCAN_EXCLUSIVE,
    kOutF16 = TCR_OUT_F16,                 /* results as binary16 (binary32 accumulation) */
    kAccF16 = TCR_ACC_F16                  /* binary16 accumulator; needs kOutF16 */
};

/* out[s] = sum of in[s * seg_len .. (s + 1) * seg_len): tcr_segmented_reduce. */
inline tcr_status SegmentedReduce(const void* in, float* out, uint64_t n, uint64_t seg_len, void* stream = nullptr) {
    return tcr_segmented_reduce(in, out, n, seg_len, stream);
}
/* out[0] = sum of in[0 .. n): tcr_reduce. */
inline tcr_status Reduce(const void* in, float* out, uint64_t n, void* stream = nullptr) { return tcr_reduce(in, out, n, stream); }
/* Inclusive running sums that restart every seg_len elements: tcr_segmented_scan. */
inline tcr_status SegmentedScan(const void* in, float* out, uint64_t n, uint64_t seg_len, void* stream = nullptr) {
    return tcr_segmented_scan(in, out, n, seg_len, stream);
}
/* Inclusive running sums of the whole array: tcr_scan. */
inline tcr_status Scan(const void* in, float* out, uint64_t n, void* stream = nullptr) { return tcr_scan(in, out, n, stream); }
/* The scans with ScanFlags; out holds binary16 values with kOutF16, binary32 otherwise: tcr_segmented_scan_ex,
 * tcr_scan_ex. */
inline tcr_status SegmentedScan(const void* in, void* out, uint64_t n, uint64_t seg_len, uint32_t flags, void* stream = nullptr) {
    return tcr_segmented_scan_ex(in, out, n, seg_len, flags, stream);
}
inline tcr_status Scan(const void* in, void* out, uint64_t n, uint32_t flags, void* stream = nullptr) {
    return tcr_scan_ex(in, out, n, flags, stream);
}

/* Irregular segments: segment s is in[offsets[s] .. offsets[s + 1]), offsets a device array of nseg + 1
 * non-decreasing positions: tcr_irregular_reduce, tcr_irregular_scan, tcr_irregular_scan_ex. */
inline tcr_status SegmentedReduce(const void* in, const uint64_t* offsets, float* out, uint64_t n, uint64_t nseg, void* stream = nullptr) {
    return tcr_irregular_reduce(in, offsets, out, n, nseg, stream);
}
inline tcr_status SegmentedScan(const void* in, const uint64_t* offsets, float* out, uint64_t n, uint64_t nseg, void* stream = nullptr) {
    return tcr_irregular_scan(in, offsets, out, n, nseg, stream);
}
inline tcr_status SegmentedScan(const void* in, const uint64_t* offsets, void* out, uint64_t n, uint64_t nseg, uint32_t flags,
                                void* stream = nullptr) {
    return tcr_irregular_scan_ex(in, offsets, out, n, nseg, flags, stream);
}

/* Sum and sum of squares of every segment (the use that Section 7 points at): tcr_segmented_moments,
 * tcr_irregular_moments. */
inline tcr_status SegmentedMoments(const void* in, float* sum, float* sumsq, uint64_t n, uint64_t seg_len, void* stream = nullptr) {
    return tcr_segmented_moments(in, sum, sumsq, n, seg_len, stream);
}
inline tcr_status SegmentedMoments(const void* in, const uint64_t* offsets, float* sum, float* sumsq, uint64_t n, uint64_t nseg,
                                   void* stream = nullptr) {
    return tcr_irregular_moments(in, offsets, sum, sumsq, n, nseg, stream);
}

inline const char* status_string(tcr_status status) { return tcr_status_string((int)status); }

}  /* namespace tcr */

#endif
