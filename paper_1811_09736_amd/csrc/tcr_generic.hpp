// Kernels for what the tiled kernels do not take: reductions of regular segments whose length is no power
// of two (long ones; short ones run on the fixed tiles of tcr_irregular.hpp), the shortest segments and the
// moments.  The paper handles such sizes by zero padding
// or by masking (Section 4, "Support for arbitrary segment sizes ...").  Padding in place is not possible
// behind this interface, so:
//   masked_*        one wavefront per segment (or per 65536-element piece of one) walks the 512-element
//                   tiles of the ARRAY (aligned to the array, not to the segment) that the segment
//                   touches; elements of a tile outside the segment are read as zero -- the paper's
//                   zero padding, applied to the operand registers -- and the matrix-core products,
//                   the running sums through the accumulator and the 128-bit loads of the tuned
//                   kernels apply unchanged; only the 8-element groups cut by a segment end are read
//                   element by element.
//   generic_*       one thread per segment: 16-bit loads, binary32 adds.
// They are correct for every seg_len >= 1; none of them is tuned.
#pragma once
#include "tcr_device.hpp"
#include "tcr_scan.hpp"

namespace tcr {

constexpr int kGenericThreads = 256;

// One thread per segment (short segments).
__device__ __forceinline__ void put(void* out, uint64_t i, float v, bool f16) {
    if (f16) static_cast<_Float16*>(out)[i] = (_Float16)v;
    else static_cast<float*>(out)[i] = v;
}

// exclusive: each output leaves out its own element; f16: outputs rounded to binary16.
template <bool SCAN>
__global__ __launch_bounds__(kGenericThreads) void generic_thread_kernel(const _Float16* __restrict__ in,
                                                                         void* __restrict__ out, uint64_t nseg,
                                                                         uint64_t seg_len, bool exclusive, bool f16) {
    const uint64_t s = (uint64_t)blockIdx.x * kGenericThreads + threadIdx.x;
    if (s >= nseg) return;
    const _Float16* p = in + s * seg_len;
    float acc = 0.0f;
    for (uint64_t k = 0; k < seg_len; ++k) {
        const float v = (float)p[k];
        if (SCAN) put(out, s * seg_len + k, exclusive ? acc : acc + v, f16);
        acc += v;
    }
    if (!SCAN) put(out, s, acc, f16);
}

// Segments of 1, 2, 4 or 8 elements: a lane adds up the whole segments inside its 8 consecutive elements and
// stores the 8 >> LOG2L results side by side (seg_len 1 is the conversion to binary32, also the inclusive scan).
template <int LOG2L>
__global__ __launch_bounds__(kGenericThreads) void tiny_reduce_kernel(const _Float16* __restrict__ in,
                                                                      float* __restrict__ out, uint64_t n) {
    static_assert(LOG2L >= 0 && LOG2L <= 3, "");
    constexpr int kResults = 8 >> LOG2L;
    const uint64_t g = ((uint64_t)blockIdx.x * kGenericThreads + threadIdx.x) * 8;
    if (g >= n) return;
    const half8 x = load8_guarded<true>(in, g, n);
    float r[kResults];
#pragma unroll
    for (int i = 0; i < kResults; ++i) {
        float acc = 0.0f;
#pragma unroll
        for (int e = 0; e < (1 << LOG2L); ++e) acc += (float)x[(i << LOG2L) + e];
        r[i] = acc;
    }
    float* dst = out + (g >> LOG2L);
    if (g + 8 <= n) {
        if constexpr (kResults == 8) {
            store4(dst, 0, (float4v){r[0], r[1], r[2], r[3]});
            store4(dst, 4, (float4v){r[4], r[5], r[6], r[7]});
        } else if constexpr (kResults == 4) {
            store4(dst, 0, (float4v){r[0], r[1], r[2], r[3]});
        } else {
#pragma unroll
            for (int i = 0; i < kResults; ++i) dst[i] = r[i];
        }
    } else {
#pragma unroll
        for (int i = 0; i < kResults; ++i)
            if (g + (uint64_t)((i + 1) << LOG2L) <= n) dst[i] = r[i];
    }
}

// The inclusive scan of segments of 1, 2, 4 or 8 elements: running sums inside a lane's 8 elements, restarted
// every 1 << LOG2L of them (seg_len 1: the conversion again).
template <int LOG2L>
__global__ __launch_bounds__(kGenericThreads) void tiny_scan_kernel(const _Float16* __restrict__ in,
                                                                    float* __restrict__ out, uint64_t n) {
    static_assert(LOG2L >= 0 && LOG2L <= 3, "");
    const uint64_t g = ((uint64_t)blockIdx.x * kGenericThreads + threadIdx.x) * 8;
    if (g >= n) return;
    const half8 x = load8_guarded(in, g, n);
    float r[8];
    float acc = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if ((e & ((1 << LOG2L) - 1)) == 0) acc = 0.0f;
        acc += (float)x[e];
        r[e] = acc;
    }
    store4_guarded(out, g, n, (float4v){r[0], r[1], r[2], r[3]});
    store4_guarded(out, g + 4, n, (float4v){r[4], r[5], r[6], r[7]});
}

// ---------------------------------------------------------------------------------------- masked tiles
// 8 inputs at element g (a multiple of 8), those outside [begin, end) read as zero.
template <bool STREAM = false>
__device__ __forceinline__ half8 load8_masked(const _Float16* __restrict__ in, uint64_t g, uint64_t begin, uint64_t end) {
    if (g >= begin && g + 8 <= end) return load8<STREAM>(in, g);
    half8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (g + e >= begin && g + e < end) ? in[g + e] : (_Float16)0.0f;
    return v;
}

// One wavefront adds up the segment [begin, end); the result is uniform.  `in` is 16-byte aligned.
__device__ __forceinline__ float masked_wave_reduce(const _Float16* __restrict__ in, uint64_t begin, uint64_t end,
                                                    const LaneId& id) {
    constexpr int kSteps = 4;
    float4v acc = splat(0.0f);                           // running row sums (the accumulator matrix V of Reduction_256N)
    for (uint64_t t0 = begin & ~(uint64_t)(kTile - 1); t0 < end; t0 += (uint64_t)(kTile * kSteps)) {
        half8 x[kSteps];
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            const uint64_t tile = t0 + (uint64_t)(kTile * i);
            x[i] = (tile < end) ? load8_masked<true>(in, tile + (uint64_t)(kRow * id.j + 8 * id.g), begin, end)
                                : __builtin_bit_cast(half8, splat(0.0f));
        }
#pragma unroll
        for (int i = 0; i < kSteps; ++i) acc = mfma(const_ones(), x[i], acc);
    }
    return read_lane(row_sum_to_last<16>(acc[0]), 15);
}

constexpr int kMaskedWaves = 4;                          // wavefronts (segments) per workgroup

__global__ __launch_bounds__(kMaskedWaves * kWave) void masked_wave_reduce_kernel(const _Float16* __restrict__ in,
                                                                                  float* __restrict__ out, uint64_t nseg,
                                                                                  uint64_t seg_len) {
    const LaneId id;
    const uint64_t s = (uint64_t)blockIdx.x * kMaskedWaves + (uint64_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (s >= nseg) return;
    const float total = masked_wave_reduce(in, s * seg_len, (s + 1) * seg_len, id);
    if (id.lane == 0) out[s] = total;
}

// Long segments of any length: wavefront w adds up piece w % per of segment w / per (pieces of `span` elements
// counted from the segment's start, the last one shorter) into dst[w]; reduce_final_kernel adds the pieces.
__global__ __launch_bounds__(kMaskedWaves * kWave) void masked_span_reduce_kernel(const _Float16* __restrict__ in,
                                                                                  float* __restrict__ dst, uint64_t nseg,
                                                                                  uint64_t seg_len, uint64_t span,
                                                                                  uint64_t per) {
    const LaneId id;
    const uint64_t w = (uint64_t)blockIdx.x * kMaskedWaves + (uint64_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (w >= nseg * per) return;
    const uint64_t s = w / per, piece = w - s * per;
    const uint64_t begin = s * seg_len + piece * span;
    const uint64_t seg_end = (s + 1) * seg_len;
    const uint64_t end = begin + span < seg_end ? begin + span : seg_end;
    const float total = masked_wave_reduce(in, begin, end, id);
    if (id.lane == 0) dst[w] = total;
}

// ---------------------------------------------------------------------------------------- first two moments
// Sum and sum of squares of a segment -- the statistics of a normalisation layer, which the paper's conclusion
// names as the next use of reductions on matrix cores.  The sum is Reduction_256N (V <- ones . X^T + V).  The
// sum of squares takes the data as BOTH operands: entry (i, j) of X . X^T is the inner product of data rows i
// and j, so the DIAGONAL of W <- X . X^T + W accumulates the sums of squares of the 16 rows (the other entries
// are not used).  A product of two binary16 values is exact in the binary32 accumulator.
// One wavefront, segment [begin, end) over zero-masked tiles of the array; both results are uniform.
__device__ __forceinline__ void masked_wave_moments(const _Float16* __restrict__ in, uint64_t begin, uint64_t end,
                                                    const LaneId& id, float& sum, float& sumsq) {
    constexpr int kSteps = 4;
    float4v acc = splat(0.0f), sq = splat(0.0f);
    for (uint64_t t0 = begin & ~(uint64_t)(kTile - 1); t0 < end; t0 += (uint64_t)(kTile * kSteps)) {
        half8 x[kSteps];
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            const uint64_t tile = t0 + (uint64_t)(kTile * i);
            x[i] = (tile < end) ? load8_masked<true>(in, tile + (uint64_t)(kRow * id.j + 8 * id.g), begin, end)
                                : __builtin_bit_cast(half8, splat(0.0f));
        }
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            acc = mfma(const_ones(), x[i], acc);
            sq = __builtin_amdgcn_mfma_f32_16x16x32_f16(x[i], x[i], sq, 0, 0, 0);
        }
    }
    sum = read_lane(row_sum_to_last<16>(acc[0]), 15);
    // lane (j, g) holds rows 4g .. 4g+3 of column j: the diagonal entry of column j sits in lane (j, j / 4), register j % 4
    const int r = id.j & 3;
    const float d = r == 0 ? sq[0] : (r == 1 ? sq[1] : (r == 2 ? sq[2] : sq[3]));
    sumsq = wave_sum(id.g == (id.j >> 2) ? d : 0.0f);
}

// One wavefront per piece: piece w % per of segment w / per (pieces of `span` elements from the segment's
// start; per == 1: whole segments).  sum[w], sumsq[w] receive the piece's moments.
__global__ __launch_bounds__(kMaskedWaves * kWave) void masked_moments_kernel(const _Float16* __restrict__ in,
                                                                              float* __restrict__ sum,
                                                                              float* __restrict__ sumsq, uint64_t nseg,
                                                                              uint64_t seg_len, uint64_t span, uint64_t per) {
    const LaneId id;
    const uint64_t w = (uint64_t)blockIdx.x * kMaskedWaves + (uint64_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (w >= nseg * per) return;
    const uint64_t s = w / per, piece = w - s * per;
    const uint64_t begin = s * seg_len + piece * span;
    const uint64_t seg_end = (s + 1) * seg_len;
    const uint64_t end = begin + span < seg_end ? begin + span : seg_end;
    float a, q;
    masked_wave_moments(in, begin, end, id, a, q);
    if (id.lane == 0) {
        sum[w] = a;
        sumsq[w] = q;
    }
}

// Short segments: one thread per segment, binary32 adds and fused multiply-adds.
__global__ __launch_bounds__(kGenericThreads) void generic_moments_kernel(const _Float16* __restrict__ in,
                                                                          float* __restrict__ sum,
                                                                          float* __restrict__ sumsq, uint64_t nseg,
                                                                          uint64_t seg_len) {
    const uint64_t s = (uint64_t)blockIdx.x * kGenericThreads + threadIdx.x;
    if (s >= nseg) return;
    const _Float16* p = in + s * seg_len;
    float a = 0.0f, q = 0.0f;
    for (uint64_t k = 0; k < seg_len; ++k) {
        const float v = (float)p[k];
        a += v;
        q = __builtin_fmaf(v, v, q);
    }
    sum[s] = a;
    sumsq[s] = q;
}

}  // namespace tcr
