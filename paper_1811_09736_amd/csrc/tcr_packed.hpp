// Regular segments of 3 to 30 elements (no power of two, or 4 or 8): sums (and sums of squares) as ONE product
// per 16 rows with a masked constant matrix, the rows laid out by the segments instead of by the array.
//
// The paper reduces segments that do not fill a tile row by masking the constant matrix P (Section 4, "Support for
// arbitrary segment sizes").  A mask on the constant operand is shared by the 16 data rows of a product, so it
// serves only if every row is cut in the same places -- which the rows of the ARRAY (32 elements each) are not
// when 32 is no multiple of seg_len.  Here a row is W = m * seg_len consecutive elements, m whole segments
// (W <= 32, even): lane (j, g) loads X[j][8g .. 8g+7] from element j * W + 8g of the tile, a 4-byte-aligned
// 128-bit load, and
//     D[i][j] = sum_k P[i][k] X[j][k],        P[i][k] = 1 iff i < m and i * seg_len <= k < (i + 1) * seg_len,
// is the sum of segment i of row j: m * 16 results from one product, no masks on the data, no running sums across
// lanes, no carries.  The columns from W on hold the next row's elements and meet zeros of P (inputs are finite by
// the library's contract); they cost matrix-core and cache bandwidth, of which there is plenty, not memory traffic.
// (Rows of an odd number of elements start on 2-byte boundaries; the hardware takes such 128-bit loads, but at
// n = 2^28 the kernel then needs 127-151 us where rows of an even width need 93-106, so odd lengths pack an even
// number of segments per row and those from 17 on are left to the masked rows of the array, 103-105 us.)
// Sums of squares: the row's elements of segment i kept, the others cleared (the mask on the data operand),
// multiplied with the row itself; the diagonal of that product (exact: binary16 products in binary32) is the
// segment's sum of squares -- m products per tile, the masks built once per wavefront.
// Results are staged in LDS per wavefront in segment order and written as consecutive stores.
#pragma once
#include "tcr_device.hpp"
#include "tcr_irregular.hpp"

namespace tcr {

struct PackedGrid {
    uint64_t n;          // elements
    uint64_t nseg;
    uint32_t seg_len;    // 3 .. 30
    uint32_t per_row;    // m: segments per row; m * seg_len is even and at most 32
};

// Segments per row for seg_len, 0 if no row width fits: the largest m with m * seg_len <= 32 and m * seg_len even
// (rows then start on 4-byte boundaries of a 4-byte-aligned array).  3 elements: 10; 5: 6; 6: 5; 7: 4; 9: 2; 10: 3;
// 11 to 15: 2; even lengths from 18 on: 1.
__host__ __device__ inline uint32_t packed_per_row(uint64_t seg_len) {
    if (seg_len < 3 || seg_len > 30) return 0;
    uint32_t m = 32u / (uint32_t)seg_len;
    if ((seg_len & 1u) && (m & 1u)) --m;
    return m;
}

// KIND: kSum (out) or kBoth (out: sums, out2: sums of squares).  in: 4-byte aligned.
// A wavefront takes U tiles of 16 rows; nothing is shared between wavefronts.
template <int KIND, int U, int WAVES>
__global__ __launch_bounds__(WAVES * kWave) void packed_rows_reduce_kernel(const _Float16* __restrict__ in,
                                                                           float* __restrict__ out, float* __restrict__ out2,
                                                                           PackedGrid grid) {
    static_assert(KIND == kSum || KIND == kBoth, "");
    constexpr int CH = channels<KIND>();
    // 16 U m results per wavefront and channel (dynamic: the launch passes WAVES * CH * 16 * U * m * 4 bytes)
    extern __shared__ __attribute__((aligned(16))) float s_stage[];

    const LaneId id;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t L = grid.seg_len, m = grid.per_row, W = L * m;
    const uint64_t rows = (grid.nseg + m - 1) / m;
    const uint64_t row0 = ((uint64_t)blockIdx.x * WAVES + (uint64_t)wave) * (uint64_t)(16 * U);
    if (row0 >= rows) return;
    const uint64_t first_elem = row0 * W;
    const uint64_t avail = grid.n - first_elem;
    const uint32_t span = avail < (uint64_t)(16u * U * W) ? (uint32_t)avail : 16u * U * W;     // elements of the wavefront's rows that exist
    const __amdgpu_buffer_rsrc_t src = make_rsrc(in + first_elem, span * 2u);

    // P's entries of lane (i, g): ones on columns [i L, (i + 1) L) for i < m
    const int lo = (int)(L * (uint32_t)id.j) - 8 * id.g;
    const half8 p = id.j < (int)m ? drop_leading(leading_ones(lo + (int)L), lo) : splat_half(0.0f);
    const int cols = (int)W - 8 * id.g;          // of this lane's eight columns, those that belong to the row

    float* const stage = s_stage + (uint32_t)(wave * CH) * (16u * U * m);
    float* const stage2 = stage + (uint32_t)(CH - 1) * (16u * U * m);
    // (all loads are requested before the first is used)
    half8 xs_in[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t at = (uint32_t)(16 * u + id.j) * W + 8u * (uint32_t)id.g;
        xs_in[u] = cols > 0 ? buffer_load8<true>(src, at * 2u) : splat_half(0.0f);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t at = (uint32_t)(16 * u + id.j) * W + 8u * (uint32_t)id.g;
        half8 x = xs_in[u];
        // (the one lane that the end of the array cuts reads element by element -- whatever the range check made of
        // its 128 bits)
        if (cols > 0 && at < span && at + 8u > span) {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = at + (uint32_t)e < span ? in[first_elem + at + (uint32_t)e] : (_Float16)0.0f;
        }
        xs_in[u] = x;
        const float4v d = mfma(p, x, splat(0.0f));
        const uint32_t slot = (uint32_t)(16 * u + id.j) * m;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if ((uint32_t)(4 * id.g + r) < m) stage[slot + (uint32_t)(4 * id.g + r)] = d[r];
    }
    if constexpr (CH == 2) {
        const int r = id.j & 3;
        const bool on_diagonal = id.g == (id.j >> 2);          // lane (j, g) holds D[4g .. 4g+3][j]
        for (uint32_t i = 0; i < m; ++i) {
            // this lane's columns of segment i, as a mask on its eight values
            const int from = (int)(L * i) - 8 * id.g;
            const u64x2 keep = __builtin_bit_cast(u64x2, keep_leading(drop_leading(__builtin_bit_cast(half8, (u64x2){~0ull, ~0ull}), from), from + (int)L));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const half8 xs = __builtin_bit_cast(half8, __builtin_bit_cast(u64x2, xs_in[u]) & keep);
                const float4v q = mfma(xs, xs_in[u], splat(0.0f));
                const float diag = r == 0 ? q[0] : (r == 1 ? q[1] : (r == 2 ? q[2] : q[3]));
                if (on_diagonal) stage2[(uint32_t)(16 * u + id.j) * m + i] = diag;
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint64_t seg0 = row0 * m;
    const uint64_t left = grid.nseg - seg0;
    const uint32_t count = left < (uint64_t)(16u * U * m) ? (uint32_t)left : 16u * U * m;
    // (seg0 is a multiple of 16: 128-bit stores wherever the result arrays are 16-byte aligned)
    const bool wide = ((reinterpret_cast<uintptr_t>(out) | (CH == 2 ? reinterpret_cast<uintptr_t>(out2) : 0)) & 15u) == 0;
    const uint32_t whole = wide ? count & ~3u : 0u;
    for (uint32_t k = 4u * (uint32_t)id.lane; k < whole; k += 4u * (uint32_t)kWave) {
        *reinterpret_cast<float4v*>(out + seg0 + k) = *reinterpret_cast<const float4v*>(stage + k);
        if constexpr (CH == 2) *reinterpret_cast<float4v*>(out2 + seg0 + k) = *reinterpret_cast<const float4v*>(stage2 + k);
    }
    for (uint32_t k = whole + (uint32_t)id.lane; k < count; k += (uint32_t)kWave) {
        out[seg0 + k] = stage[k];
        if constexpr (CH == 2) out2[seg0 + k] = stage2[k];
    }
}

}  // namespace tcr
