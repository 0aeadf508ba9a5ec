// Kernels for segment lengths without a tuned path (not a power of two, or shorter than 16).
// The paper handles such sizes by zero padding or by masking the constant matrix (Section 4,
// "Support for arbitrary segment sizes ..."); padding in place is not possible behind this
// interface and segments that start at odd element offsets rule out 128-bit operand loads, so
// these kernels read 16-bit elements and do the arithmetic with binary32 adds and the
// wavefront scan primitive.  They are correct for every seg_len >= 1 and make no claim on
// bandwidth.
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

// One wavefront per segment: 64 elements per step, four steps in flight.
template <bool SCAN>
__global__ __launch_bounds__(kGenericThreads) void generic_wave_kernel(const _Float16* __restrict__ in,
                                                                       void* __restrict__ out, uint64_t nseg,
                                                                       uint64_t seg_len, bool exclusive, bool f16) {
    constexpr int kSteps = 4;
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t s = (uint64_t)blockIdx.x * (kGenericThreads / kWave) +
                       (uint64_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (s >= nseg) return;
    const _Float16* p = in + s * seg_len;
    const uint64_t q = s * seg_len;
    float carry = 0.0f;      // SCAN: total of the steps already done (uniform)
    float acc = 0.0f;        // REDUCE: this lane's running sum
    for (uint64_t k0 = 0; k0 < seg_len; k0 += (uint64_t)(kWave * kSteps)) {
        float v[kSteps];
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            const uint64_t k = k0 + (uint64_t)(kWave * i + lane);
            v[i] = (k < seg_len) ? (float)p[k] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            if (SCAN) {
                const uint64_t k = k0 + (uint64_t)(kWave * i + lane);
                const float incl = wave_scan_inclusive(v[i]);
                const float excl = wave_shr1(incl);          // sum of the lower lanes only (no subtraction)
                if (k < seg_len) put(out, q + k, (exclusive ? excl : incl) + carry, f16);
                carry += read_lane(incl, 63);
            } else {
                acc += v[i];
            }
        }
    }
    if (!SCAN) {
        const float total = wave_sum(acc);
        if (lane == 0) put(out, s, total, f16);
    }
}

// Irregular segments: segment s is [offsets[s], offsets[s+1]).  One wavefront per segment, same
// arithmetic as generic_wave_kernel.  (The paper reduces the irregular case to the regular one by
// padding the input, Section 3 footnote; reading the offsets directly needs no padded copy.)
template <bool SCAN>
__global__ __launch_bounds__(kGenericThreads) void irregular_wave_kernel(const _Float16* __restrict__ in,
                                                                         const uint64_t* __restrict__ offsets,
                                                                         float* __restrict__ out, uint64_t nseg) {
    constexpr int kSteps = 4;
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t s = (uint64_t)blockIdx.x * (kGenericThreads / kWave) +
                       (uint64_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (s >= nseg) return;
    const uint64_t begin = offsets[s], end = offsets[s + 1];
    float carry = 0.0f, acc = 0.0f;
    for (uint64_t k0 = begin; k0 < end; k0 += (uint64_t)(kWave * kSteps)) {
        float v[kSteps];
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            const uint64_t k = k0 + (uint64_t)(kWave * i + lane);
            v[i] = (k < end) ? (float)in[k] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            if (SCAN) {
                const uint64_t k = k0 + (uint64_t)(kWave * i + lane);
                const float incl = wave_scan_inclusive(v[i]);
                if (k < end) out[k] = incl + carry;
                carry += read_lane(incl, 63);
            } else {
                acc += v[i];
            }
        }
    }
    if (!SCAN) {
        const float total = wave_sum(acc);
        if (lane == 0) out[s] = total;
    }
}

}  // namespace tcr
