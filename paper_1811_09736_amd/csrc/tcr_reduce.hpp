// Segmented / full sum-reduction kernels (Section 4 of the paper, re-derived for MFMA).
//
//   reduce_small_kernel   seg_len in {16, 32, ..., 512}: a segment is part of one wavefront tile.
//                         One "ones" product per tile gives the 16 row sums (the paper's
//                         Reduction_16: P.A, here with every row of the constant equal to P's
//                         first row); rows of one segment are folded with binary32 cross-lane
//                         adds (where Reduction_256 uses a second product with P^T).
//   reduce_span_kernel    seg_len >= 1024 and the full reduction: each wavefront walks a span of
//                         consecutive tiles and keeps the 16 running row sums in the accumulator,
//                         V_i = ones.A_i + V_{i-1} (the work-efficient Reduction_256N), folding
//                         the 16 sums once at the end; optionally the wavefronts of a workgroup
//                         combine their sums through LDS (block-level Reduction_256N).
//   reduce_final_kernel   device level: binary32 partials of one segment -> its result (the
//                         second kernel of the paper's grid-level reduction).
//
// FORM selects the arithmetic inside a tile: kMfma (matrix cores) or kDpp (convert, add in
// binary32, cross-lane DPP adds) -- the wavefront-primitive alternative kept for measurement.
#pragma once
#include "tcr_device.hpp"

namespace tcr {

enum Formulation { kMfma = 0, kDpp = 1 };

// Sum over aligned groups of GROUP lanes (GROUP up to 64); valid in the last lane of a group.
template <int GROUP>
__device__ __forceinline__ float lanes_sum_to_last(float x) {
    x = row_sum_to_last<(GROUP < 16 ? GROUP : 16)>(x);
    if constexpr (GROUP > 16)
        x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x142, 0xa, 0xf, false));
    if constexpr (GROUP > 32)
        x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x143, 0xc, 0xf, false));
    return x;
}

__device__ __forceinline__ float sum8(half8 v) {
    float a = (float)v[0] + (float)v[1];
    float b = (float)v[2] + (float)v[3];
    float c = (float)v[4] + (float)v[5];
    float d = (float)v[6] + (float)v[7];
    return (a + b) + (c + d);
}

// ------------------------------------------------------------------------------ small segments
// Grid: one workgroup (WAVES wavefronts) per WAVES*U tiles.  n is a multiple of seg_len = 1 << LOG2L.
// LOAD: how the tiles reach the operand registers (TileLoad; matrix-core formulation, full tiles).
template <int FORM, int LOG2L, int U, int WAVES, int LOAD = kLoadDirect>
__global__ __launch_bounds__(WAVES * kWave) void reduce_small_kernel(const _Float16* __restrict__ in,
                                                                     float* __restrict__ out, uint64_t n) {
    static_assert(LOG2L >= 4 && LOG2L <= 9, "");
    const LaneId id;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keeps per-wave branches and addresses scalar
    const uint64_t base = ((uint64_t)blockIdx.x * WAVES + wave) * (uint64_t)(kTile * U);
    if (base >= n) return;
    const uint64_t nseg = n >> LOG2L;
    // element offset of this lane's 8 values inside a tile
    const int lane_off = (FORM == kMfma) ? (kRow * id.j + 8 * id.g) : (8 * id.lane);

    half8 x[U];
    if (base + (uint64_t)(kTile * U) <= n) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if constexpr (FORM == kMfma && LOAD != kLoadDirect) x[u] = load_tile_operand<LOAD, true>(in, base + (uint64_t)(kTile * u), id.j, id.g, id.lane, wave);
            else x[u] = load8<true>(in, base + (uint64_t)(kTile * u + lane_off));
        }
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8_guarded<true>(in, base + (uint64_t)(kTile * u + lane_off), n);
    }

    // Per tile, the segment sums sit in scattered lanes (the last lane of each row group).  They are
    // gathered with one cross-lane read per tile so that the wavefront's U * 512 / seg_len results leave
    // as one run of consecutive 32-bit stores in lane order.
    constexpr int RT = kTile >> LOG2L;                   // results per tile
    static_assert(RT * U <= kWave, "one result per lane at most");
    float t[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (FORM == kMfma) {
            if constexpr (LOG2L == 4) {
                // two segments per row: rows 0..7 of the product carry the first, 8..15 the second;
                // segment 2j + h of the tile ends up in lane (j, g = 2h)
                t[u] = mfma(const_half_rows(id), x[u], splat(0.0f))[0];
            } else {
                constexpr int ROWS = 1 << (LOG2L - 5);   // tile rows per segment; sum valid in the group's last row
                t[u] = row_sum_to_last<ROWS>(mfma(const_ones(), x[u], splat(0.0f))[0]);
            }
        } else {
            constexpr int LANES = 1 << (LOG2L - 3);      // lanes per segment; sum valid in the group's last lane
            t[u] = lanes_sum_to_last<LANES>(sum8(x[u]));
        }
    }
    const int slot = id.lane;                            // this lane stores result `slot` of the wavefront
    const int slot_tile = slot / RT, slot_seg = slot % RT;
    int src;                                             // lane that holds segment slot_seg of a tile
    if constexpr (FORM == kMfma) {
        if constexpr (LOG2L == 4) src = (slot_seg >> 1) + 32 * (slot_seg & 1);
        else src = ((slot_seg + 1) << (LOG2L - 5)) - 1;
    } else {
        src = ((slot_seg + 1) << (LOG2L - 3)) - 1;
    }
    float v = 0.0f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float got = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src << 2, __builtin_bit_cast(int, t[u])));
        if (u == slot_tile) v = got;
    }
    const uint64_t s = (base >> LOG2L) + (uint64_t)slot;
    if (slot < RT * U && s < nseg) out[s] = v;
}

// First two moments of small segments (seg_len in {16, ..., 512}): reduce_small_kernel's sums, and the sums of
// squares from the diagonal of X . X^T -- the tile multiplied with itself on the matrix cores, whose entry
// (j, j) is the sum of the squares of tile row j (products of two binary16 values are exact in the binary32
// accumulator).  Lane (j, g) holds rows 4g .. 4g+3 of column j of the product, so the diagonal entry of row j
// sits in lane (j, j / 4), register j % 4, and one cross-lane read brings it to every lane of column j.
__device__ __forceinline__ float row_squares(half8 a, const LaneId& id) {
    const float4v d = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, a, splat(0.0f), 0, 0, 0);
    const int r = id.j & 3;
    const float c = r == 0 ? d[0] : (r == 1 ? d[1] : (r == 2 ? d[2] : d[3]));
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((id.j + 16 * (id.j >> 2)) << 2, __builtin_bit_cast(int, c)));
}

template <int LOG2L, int U, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void moments_small_kernel(const _Float16* __restrict__ in,
                                                                      float* __restrict__ sum, float* __restrict__ sumsq,
                                                                      uint64_t n) {
    static_assert(LOG2L >= 4 && LOG2L <= 9, "");
    const LaneId id;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t base = ((uint64_t)blockIdx.x * WAVES + wave) * (uint64_t)(kTile * U);
    if (base >= n) return;
    const uint64_t nseg = n >> LOG2L;
    const int lane_off = kRow * id.j + 8 * id.g;
    half8 x[U];
    if (base + (uint64_t)(kTile * U) <= n) {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8<true>(in, base + (uint64_t)(kTile * u + lane_off));
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8_guarded<true>(in, base + (uint64_t)(kTile * u + lane_off), n);
    }
    constexpr int RT = kTile >> LOG2L;                   // results per tile
    static_assert(RT * U <= kWave, "one result per lane at most");
    float t[U], q[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (LOG2L == 4) {
            // two segments per row, as in reduce_small_kernel: segment 2j + h of the tile in lane (j, g = 2h);
            // the squares of each half row come from the tile with the other half's columns zeroed
            t[u] = mfma(const_half_rows(id), x[u], splat(0.0f))[0];
            const half8 zero = __builtin_bit_cast(half8, splat(0.0f));
            const float first = row_squares(id.g < 2 ? x[u] : zero, id);
            const float second = row_squares(id.g < 2 ? zero : x[u], id);
            q[u] = id.g < 2 ? first : second;
        } else {
            constexpr int ROWS = 1 << (LOG2L - 5);       // tile rows per segment; sums valid in the group's last row
            t[u] = row_sum_to_last<ROWS>(mfma(const_ones(), x[u], splat(0.0f))[0]);
            q[u] = row_sum_to_last<ROWS>(row_squares(x[u], id));
        }
    }
    const int slot = id.lane;                            // this lane stores results `slot` of the wavefront
    const int slot_tile = slot / RT, slot_seg = slot % RT;
    int src;                                             // lane that holds segment slot_seg of a tile
    if constexpr (LOG2L == 4) src = (slot_seg >> 1) + 32 * (slot_seg & 1);
    else src = ((slot_seg + 1) << (LOG2L - 5)) - 1;
    float a = 0.0f, b = 0.0f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float ga = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src << 2, __builtin_bit_cast(int, t[u])));
        const float gb = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src << 2, __builtin_bit_cast(int, q[u])));
        if (u == slot_tile) {
            a = ga;
            b = gb;
        }
    }
    const uint64_t s = (base >> LOG2L) + (uint64_t)slot;
    if (slot < RT * U && s < nseg) {
        sum[s] = a;
        sumsq[s] = b;
    }
}

// ------------------------------------------------------------------------------ long spans
// Wavefront w (global index) reduces elements [w*span, min((w+1)*span, n)); span is a multiple
// of the tile size.  COMBINE == false: dst[w] receives that sum (one wavefront per segment or per
// partial).  COMBINE == true: the WAVES sums of a workgroup are added through LDS in wavefront
// order and dst[blockIdx.x] receives the result (block-level Reduction_256N: one workgroup per
// segment or per partial).
// FINAL == true (device level, Section 4, as one kernel instead of the paper's two): dst holds `per`
// partials per segment; every workgroup counts itself on a running counter after its partial is
// visible, and the workgroup that counts last adds up the partials of every segment, in a fixed
// order, into fin.out.  The counter is never reset: the host passes its value at launch.
struct ReduceFinish {
    float* out;            // [nseg]
    uint32_t* counter;     // running count of finished workgroups
    uint32_t base;         // value of *counter when this launch starts
    uint32_t nseg, per;    // dst holds nseg * per partials
};

template <int FORM, int U, int WAVES, bool COMBINE, bool FINAL = false>
__global__ __launch_bounds__(WAVES * kWave) void reduce_span_kernel(const _Float16* __restrict__ in,
                                                                    float* __restrict__ dst, uint64_t n,
                                                                    uint64_t span, uint64_t nspans, ReduceFinish fin) {
    __shared__ float s_total[WAVES];
    __shared__ uint32_t s_count;
    const LaneId id;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keeps per-wave branches and addresses scalar
    const uint64_t w = (uint64_t)blockIdx.x * WAVES + wave;
    float total = 0.0f;
    if (w < nspans) {
        const uint64_t begin = w * span;
        const uint64_t end = (begin + span < n) ? begin + span : n;
        const int lane_off = (FORM == kMfma) ? (kRow * id.j + 8 * id.g) : (8 * id.lane);
        float4v acc = splat(0.0f);          // MFMA: running row sums (the accumulator matrix V)
        float s0 = 0.0f, s1 = 0.0f;         // DPP: per-lane running sums
        uint64_t t = begin;
        for (; t + (uint64_t)(kTile * U) <= end; t += (uint64_t)(kTile * U)) {
            half8 x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) x[u] = load8<true>(in, t + (uint64_t)(kTile * u + lane_off));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if constexpr (FORM == kMfma) acc = mfma(const_ones(), x[u], acc);
                else if (u & 1) s1 += sum8(x[u]);
                else s0 += sum8(x[u]);
            }
        }
        for (; t < end; t += kTile) {
            const half8 x = load8_guarded<true>(in, t + (uint64_t)lane_off, end);
            if constexpr (FORM == kMfma) acc = mfma(const_ones(), x, acc);
            else s0 += sum8(x);
        }
        if constexpr (FORM == kMfma) total = read_lane(row_sum_to_last<16>(acc[0]), 15);   // fold the 16 row sums
        else total = read_lane(lanes_sum_to_last<64>(s0 + s1), 63);
    }
    if constexpr (!FINAL) {
        if constexpr (!COMBINE) {
            if (w < nspans && id.lane == 0) dst[w] = total;
        } else {
            if (id.lane == 0) s_total[wave] = total;
            __syncthreads();
            if (threadIdx.x == 0) {
                float sum = 0.0f;
#pragma unroll
                for (int k = 0; k < WAVES; ++k) sum += s_total[k];
                dst[blockIdx.x] = sum;
            }
        }
    } else {
        static_assert(!FINAL || COMBINE || WAVES == 1, "one partial per workgroup");
        if (id.lane == 0) s_total[wave] = total;
        __syncthreads();
        if (threadIdx.x == 0) {
            float sum = 0.0f;
#pragma unroll
            for (int k = 0; k < WAVES; ++k) sum += s_total[k];
            // The partial is written through to device scope and its acknowledgement is waited for before the
            // count is issued; the last workgroup reads the partials with device-scope loads that bypass its
            // caches.  (A device-scope release / acquire pair instead would write back and invalidate the L2
            // once per workgroup: measured, it costs a third of the bandwidth.)
            __hip_atomic_store(&dst[blockIdx.x], sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");       // compiler ordering
            __builtin_amdgcn_s_waitcnt(0x0F70);                          // vmcnt(0): the store has been acknowledged
            s_count = __hip_atomic_fetch_add(fin.counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - fin.base;
        }
        __syncthreads();
        if (s_count == gridDim.x - 1u) {
            for (uint32_t seg = (uint32_t)wave; seg < fin.nseg; seg += WAVES) {
                const float* p = dst + (uint64_t)seg * fin.per;
                float a = 0.0f;
                for (uint32_t i = (uint32_t)id.lane; i < fin.per; i += kWave)
                    a += __hip_atomic_load(&p[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const float t = wave_sum(a);
                if (id.lane == 0) fin.out[seg] = t;
            }
        }
    }
}

// ------------------------------------------------------------------------------ partials -> result
// Workgroup s adds the `per` binary32 partials of segment s in a fixed order.
constexpr int kFinalThreads = 256;
__global__ __launch_bounds__(kFinalThreads) void reduce_final_kernel(const float* __restrict__ partials,
                                                                     float* __restrict__ out, uint64_t per) {
    constexpr int kBlockThreads = kFinalThreads;
    __shared__ float wave_tot[kFinalThreads / kWave];
    const float* p = partials + (uint64_t)blockIdx.x * per;
    float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
    uint64_t i = threadIdx.x;
    for (; i + 3 * kBlockThreads < per; i += 4 * kBlockThreads) {
        a0 += p[i];
        a1 += p[i + kBlockThreads];
        a2 += p[i + 2 * kBlockThreads];
        a3 += p[i + 3 * kBlockThreads];
    }
    for (; i < per; i += kBlockThreads) a0 += p[i];
    const float t = wave_sum((a0 + a1) + (a2 + a3));
    if ((threadIdx.x & 63) == 0) wave_tot[threadIdx.x >> 6] = t;
    __syncthreads();
    if (threadIdx.x == 0) out[blockIdx.x] = (wave_tot[0] + wave_tot[1]) + (wave_tot[2] + wave_tot[3]);
}

}  // namespace tcr
