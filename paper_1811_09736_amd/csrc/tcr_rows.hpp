// Regular segments whose length is no power of two, from 17 elements up to a few thousand: sums (and sums of
// squares) with every addition of the data itself on the matrix cores.
//
// The paper handles such lengths by padding the data or by masking the constant matrix P (Section 4, "Support
// for arbitrary segment sizes").  A mask on the CONSTANT operand is shared by the 16 data rows of a product,
// but a segment boundary falls on a different column in every row; so here the mask goes onto the DATA operand
// instead.  A tile row of 32 elements holds at most one boundary when seg_len >= 32: the row splits into a head
// (in front of the boundary: the end of one segment) and a tail (from the boundary on: the start of the next).
// Two products with the all-ones constant,
//     head_j = sum_k 1 . (X[j][k] if k <  c_j else 0)        tail_j = sum_k 1 . (X[j][k] if k >= c_j else 0)
// give both pieces of every row (a row without a boundary is all head), as plain sums of exactly the elements
// that belong together -- no prefix differences, nothing cancels.  For the sums of squares the two masked
// operands are multiplied with themselves and the diagonal of each product is read off, as in the moments of
// the power-of-two lengths.  What remains is one value per ROW, not per element: a segmented running sum over
// the 16 rows of a sub-tile (four cross-lane steps on (flag, value) pairs), chained through the sub-tiles of a
// wavefront in registers and through the wavefronts of a workgroup in LDS.  A row that holds the end of a
// segment writes that segment's result: what arrives from the rows in front plus its own head.
// With seg_len < 32 a row holds several boundaries, and between two of them lies a whole segment: one more masked
// product each, whose row sum is that segment's result as it stands (dispatched from 17 elements on: one whole
// segment per row at most; with two or three, 9 to 15 elements, the kernel is no faster than the fixed tiles).
//
// A workgroup owns WHOLE segments (as many as fit into 16320 elements), so no sum crosses workgroups: one
// launch, no workspace, the same order of additions in every run.  Its rows are rows of the ARRAY (aligned 64-byte
// pieces from the 16-byte boundary at or below `in`), so every load is an aligned 128-bit load in the operand
// layout; the pieces of its first and last row that belong to a neighbour's segments are masked away like any
// other head or tail.
#pragma once
#include "tcr_device.hpp"
#include "tcr_reduce.hpp"
#include "tcr_irregular.hpp"

namespace tcr {

struct RowsGrid {
    uint64_t seg_len;       // 32 <= seg_len <= kRowsMaxSegLen
    uint64_t nseg;
    uint64_t n;             // elements of the array counted from the aligned base: the caller's n + shift
    uint32_t shift;         // elements between the aligned base and the caller's first element (0 .. 7)
    uint32_t per_group;     // segments per workgroup
    uint32_t magic;         // ceil(2^32 / seg_len): x / seg_len == umulhi(x, magic) for x * seg_len < 2^32
};

constexpr uint32_t kRowsGroupElems = 16320;       // a workgroup's segments span at most 512 rows of 32 elements
constexpr uint64_t kRowsMaxSegLen = 8160;         // at least two segments per workgroup

// Inclusive segmented scan over the 16 lanes of each row of lanes (the 16 data rows of a sub-tile, held
// redundantly by the four lane rows).
template <int CH>
__device__ __forceinline__ void rows_seg_scan_inclusive(uint32_t& f, float (&v)[CH]) {
    seg_combine_left<0x111, 0xf, true>(f, v);
    seg_combine_left<0x112, 0xf, true>(f, v);
    seg_combine_left<0x114, 0xf, true>(f, v);
    seg_combine_left<0x118, 0xf, true>(f, v);
}

// KIND: kSum (out) or kBoth (out: sums, out2: sums of squares).
// WHOLES > 0: seg_len < 32.  A row then holds up to WHOLES + 1 boundaries, seg_len apart (one more than 32 /
// seg_len rounded down): its head, up to WHOLES whole segments between neighbouring boundaries -- one more masked
// product each, whose row sum is that segment's result as it stands -- and its tail behind the last boundary.
template <int KIND, int U, int WAVES, int WHOLES = 0>
__global__ __launch_bounds__(WAVES * kWave) void rows_reduce_kernel(const _Float16* __restrict__ in,
                                                                    float* __restrict__ out, float* __restrict__ out2,
                                                                    RowsGrid grid) {
    static_assert(KIND == kSum || KIND == kBoth, "");
    static_assert(U * WAVES * 16 >= 512, "a workgroup's rows must fit its sub-tiles");
    constexpr int CH = channels<KIND>();
    __shared__ float s_wave_value[CH][WAVES];
    __shared__ uint32_t s_wave_flag[WAVES];

    const LaneId id;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t L = (uint32_t)grid.seg_len;
    const uint64_t s0 = (uint64_t)blockIdx.x * grid.per_group;                  // first segment of the workgroup
    const uint64_t left = grid.nseg - s0;
    const uint32_t count = left < grid.per_group ? (uint32_t)left : grid.per_group;
    const uint64_t begin = s0 * grid.seg_len + grid.shift;                       // positions count from the aligned base
    const uint64_t end = begin + (uint64_t)count * L;
    const uint64_t row_lo = begin >> 5;
    const uint32_t nrows = (uint32_t)(((end + 31) >> 5) - row_lo);               // <= 512
    const int d0 = (int)(begin & 31);                                            // the first segment starts at column d0 of row 0

    // the workgroup's rows as a buffer: rows beyond them (and elements beyond the array) read as zero
    const uint64_t first_elem = row_lo << 5;
    const uint64_t avail = grid.n - first_elem;
    const uint32_t span = (uint64_t)nrows * 32 < avail ? nrows * 32 : (uint32_t)avail;
    // (the range check takes or drops a lane's 128 bits as a whole: the buffer ends with the last whole group of
    // 8 elements, and the one group that the end of the array cuts is read element by element)
    const __amdgpu_buffer_rsrc_t src = make_rsrc(in + first_elem, (span & ~7u) * 2u);

    half8 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t row = (uint32_t)(16 * (wave * U + u) + id.j);
        const uint32_t at = row * 32u + 8u * (uint32_t)id.g;
        x[u] = buffer_load8<true>(src, at * 2u);
        if (at < span && at + 8u > span) {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[u][e] = at + (uint32_t)e < span ? in[first_elem + at + (uint32_t)e] : (_Float16)0.0f;
        }
    }

    float head[CH][U], carry_in[CH][U];      // per row: its head piece; the sum arriving from the rows in front (this sub-tile only)
    constexpr int kWholes = WHOLES > 0 ? WHOLES : 1;
    float whole[CH][kWholes][U];             // WHOLES > 0: the segments between the row's boundaries
    uint32_t whole_which[kWholes][U];        // ... and which they are (counted inside the workgroup, from 1; 0: none)
    uint32_t flag_in[U];                     // a boundary lies in an earlier row of the sub-tile
    uint32_t which[U];                       // the segment (counted inside the workgroup, from 1) that ends in this row; 0: none
    uint32_t seen_before[U];                 // a boundary lies in an earlier sub-tile of this wavefront
    float before[CH][U];                     // sum since the last boundary when the sub-tile starts (this wavefront only)
    float run[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) run[c] = 0.0f;
    uint32_t seen = 0u;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        // row r of the workgroup starts t elements behind the start of its first segment; the first boundary
        // at or behind the row's start is number k = ceil(t / L), c columns into the row
        const int r = 16 * (wave * U + u) + id.j;
        const int t = 32 * r - d0;
        const uint32_t k = t <= 0 ? 0u : __umulhi((uint32_t)t + L - 1u, grid.magic);
        const uint32_t c = k * L - (uint32_t)t;                 // t <= 0: d0 - 32 r, which is d0 for row 0
        const bool has = c < 32u;
        which[u] = (has && k >= 1u && k <= count) ? k : 0u;
        const int lead = (int)c - 8 * id.g;                     // of this lane's eight elements, those in front of the boundary
        const half8 xh = keep_leading(x[u], has ? lead : 8);
        half8 xt = drop_leading(x[u], has ? lead : 8);
        if constexpr (WHOLES > 0) {
            // further boundaries, seg_len apart: the elements between boundary w and w + 1 of the row are segment
            // k + w + 1 (from 1), whole.  (c < seg_len < 32: the row always has the first boundary.)
#pragma unroll
            for (int w = 0; w < WHOLES; ++w) {
                const bool present = c + (uint32_t)(w + 1) * L < 32u;
                whole_which[w][u] = (present && k + (uint32_t)w < count) ? k + (uint32_t)w + 1u : 0u;
                // (not there: nothing is kept for it and the tail stays as it is)
                const int upto = present ? lead + (w + 1) * (int)L : 0;
                const half8 xm = keep_leading(xt, upto);
                xt = drop_leading(xt, upto);
                whole[0][w][u] = mfma(const_ones(), xm, splat(0.0f))[0];
                if constexpr (CH == 2) whole[CH - 1][w][u] = row_squares(xm, id);
            }
        }
        float v[CH];
        head[0][u] = mfma(const_ones(), xh, splat(0.0f))[0];
        const float tail = mfma(const_ones(), xt, splat(0.0f))[0];
        v[0] = has ? tail : head[0][u];
        if constexpr (CH == 2) {
            head[CH - 1][u] = row_squares(xh, id);
            const float tail2 = row_squares(xt, id);
            v[CH - 1] = has ? tail2 : head[CH - 1][u];
        }
        uint32_t f = has ? 1u : 0u;
        rows_seg_scan_inclusive<CH>(f, v);
        flag_in[u] = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)f, 0x111, 0xf, 0xf, true);
        const uint32_t sub_flag = (uint32_t)__builtin_amdgcn_readlane((int)f, 15);
        seen_before[u] = seen;
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) {
            carry_in[ch][u] = row_shr<1>(v[ch]);
            const float sub_value = read_lane(v[ch], 15);
            before[ch][u] = run[ch];
            run[ch] = sub_flag ? sub_value : run[ch] + sub_value;
        }
        seen |= sub_flag;
    }
    if (id.lane == 0) {
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) s_wave_value[ch][wave] = run[ch];
        s_wave_flag[wave] = seen;
    }
    __syncthreads();
    float ext[CH];                            // from the wavefronts in front, back to the nearest one with a boundary
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) ext[ch] = 0.0f;
    for (int w = wave - 1; w >= 0; --w) {
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) ext[ch] += s_wave_value[ch][w];
        if (s_wave_flag[w]) break;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (which[u] != 0u && id.g == 0) {
            const uint64_t s = s0 + (uint64_t)(which[u] - 1u);
            {
                const float into_sub = seen_before[u] ? before[0][u] : before[0][u] + ext[0];
                out[s] = (flag_in[u] ? carry_in[0][u] : carry_in[0][u] + into_sub) + head[0][u];
            }
            if constexpr (CH == 2) {
                const float into_sub = seen_before[u] ? before[CH - 1][u] : before[CH - 1][u] + ext[CH - 1];
                out2[s] = (flag_in[u] ? carry_in[CH - 1][u] : carry_in[CH - 1][u] + into_sub) + head[CH - 1][u];
            }
        }
        if constexpr (WHOLES > 0) {
#pragma unroll
            for (int w = 0; w < WHOLES; ++w) {
                if (whole_which[w][u] != 0u && id.g == 0) {
                    const uint64_t s = s0 + (uint64_t)(whole_which[w][u] - 1u);
                    out[s] = whole[0][w][u];
                    if constexpr (CH == 2) out2[s] = whole[CH - 1][w][u];
                }
            }
        }
    }
}

}  // namespace tcr
