// Device-side building blocks: 64-lane cross-lane (DPP) primitives, the constant operand
// matrices, and the 16x16x32 MFMA tile operations on which every kernel is built.
//
// Tile convention (the "operand map").  One wavefront owns a tile of 512 consecutive
// elements, viewed as a row-major 16 x 32 matrix X (row j = elements 32j .. 32j+31).
// Lane l = j + 16 g (j = l % 16, g = l / 16) loads the 8 binary16 values X[j][8g .. 8g+7]
// with one 128-bit load; that register quadruple is exactly the B operand of
// v_mfma_f32_16x16x32_f16 for the product  D = C_const . X^T + Acc,
//     D[i][j] = sum_k C_const[i][k] * X[j][k] + Acc[i][j],
// and lane (j, g) receives D[4g .. 4g+3][j] in its four accumulator registers.
// This is the transposed form of the paper's products (Section 4: P.A reduces columns of a
// column-major tile; Section 5: A.U scans rows of a row-major tile): the constant sits on
// the left so that a lane's four results are four *consecutive* elements of the output and
// go out as one 128-bit store.
//
// Only raw input ever enters an MFMA A/B operand (those are binary16).  Every derived
// quantity -- row totals, carries, running sums -- travels through the binary32 accumulator
// or through binary32 cross-lane adds, which is what keeps integer-valued results exact.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tcr {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr int kTile = 512;          // elements per wavefront tile (16 rows x 32)
constexpr int kRow = 32;            // elements per tile row

// ---------------------------------------------------------------- cross-lane primitives

// Value of the lane `N` places lower inside the same row of 16 lanes; 0 where that lane
// would fall outside the row.
template <int N>
__device__ __forceinline__ float row_shr(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x110 + N, 0xf, 0xf, true));
}

// Inclusive scan over the 16 lanes of each row, restricted to aligned groups of GROUP lanes.
template <int GROUP>
__device__ __forceinline__ float row_scan_inclusive(float x, int j) {
    static_assert(GROUP == 1 || GROUP == 2 || GROUP == 4 || GROUP == 8 || GROUP == 16, "");
    if constexpr (GROUP == 16) {
        // (the row is the group: what row_shr delivers from outside it is already 0)
        x += row_shr<1>(x);
        x += row_shr<2>(x);
        x += row_shr<4>(x);
        x += row_shr<8>(x);
        return x;
    }
    const int p = j & (GROUP - 1);
    if constexpr (GROUP > 1) { float v = row_shr<1>(x); x += (p >= 1) ? v : 0.0f; }
    if constexpr (GROUP > 2) { float v = row_shr<2>(x); x += (p >= 2) ? v : 0.0f; }
    if constexpr (GROUP > 4) { float v = row_shr<4>(x); x += (p >= 4) ? v : 0.0f; }
    if constexpr (GROUP > 8) { float v = row_shr<8>(x); x += (p >= 8) ? v : 0.0f; }
    return x;
}

// Sum over aligned groups of GROUP lanes of a row; valid in the last lane of each group.
template <int GROUP>
__device__ __forceinline__ float row_sum_to_last(float x) {
    if constexpr (GROUP > 1) x += row_shr<1>(x);
    if constexpr (GROUP > 2) x += row_shr<2>(x);
    if constexpr (GROUP > 4) x += row_shr<4>(x);
    if constexpr (GROUP > 8) x += row_shr<8>(x);
    return x;
}

// Inclusive scan over all 64 lanes (rows chained through row-broadcast steps).
__device__ __forceinline__ float wave_scan_inclusive(float x) {
    x += row_shr<1>(x);
    x += row_shr<2>(x);
    x += row_shr<4>(x);
    x += row_shr<8>(x);
    // lane 15 of rows 0 and 2 -> every lane of rows 1 and 3
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x142, 0xa, 0xf, false));
    // lane 31 -> every lane of rows 2 and 3
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x143, 0xc, 0xf, false));
    return x;
}

__device__ __forceinline__ float read_lane(float x, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), lane));
}

// Sum over all 64 lanes, returned uniformly.
__device__ __forceinline__ float wave_sum(float x) { return read_lane(wave_scan_inclusive(x), 63); }

// A workgroup barrier that orders LDS accesses only: unlike __syncthreads() it does not wait for the wavefront's
// outstanding loads from memory, so data requested before it keeps arriving while the workgroup works on LDS.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---------------------------------------------------------------- constant operand matrices

// A-operand registers of lane (i, g): entries C[i][8g .. 8g+7] of a 16 x 32 constant matrix.
struct LaneId {
    int lane, j, g;
    __device__ __forceinline__ LaneId() {
        lane = threadIdx.x & (kWave - 1);
        j = lane & 15;
        g = lane >> 4;
    }
};

// All-ones matrix (the paper's underlined 1; every row plays the role of P's first row, so
// every accumulator row ends up holding the sums).
__device__ __forceinline__ half8 const_ones() {
    half8 c;
#pragma unroll
    for (int e = 0; e < 8; ++e) c[e] = (_Float16)1.0f;
    return c;
}

__device__ __forceinline__ half8 splat_half(float v) {
    const _Float16 h = (_Float16)v;
    return (half8){h, h, h, h, h, h, h, h};
}

// Eight binary16 values of which the first `count` (clamped to 0..8) are 1 and the rest 0: one
// register quadruple of a triangular constant.  Built with two 64-bit shifts instead of eight
// compares so that a one-tile wavefront spends few VALU instructions on its constants.
typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ half8 leading_ones(int count) {
    const unsigned long long ones = 0x3C003C003C003C00ull;          // four binary16 ones
    const int c = count < 0 ? 0 : (count > 8 ? 8 : count);
    const int clo = c < 4 ? c : 4, chi = c - clo;
    u64x2 v;
    v[0] = clo ? ones >> (16 * (4 - clo)) : 0ull;
    v[1] = chi ? ones >> (16 * (4 - chi)) : 0ull;
    return __builtin_bit_cast(half8, v);
}

// Lower-triangular-with-diagonal pieces of U^T (Section 5's U, transposed because the constant
// is on the left here).  Output row i of the first product is position i of a tile row,
// output row i of the second product is position 16 + i:
//   tri_lo[i][k] = 1  iff  k <= i            tri_hi[i][k] = 1  iff  k <= 16 + i
// Lane (i, g) holds k = 8g .. 8g+7, so its registers are a run of ones followed by zeros.
// EXCL = 1 drops the diagonal (k < i): the exclusive scan, the strict triangle that Section 5
// uses for its column scans.
// All three constants are one pattern -- the run of ones that lanes (i, 0) and (i, 1) hold of tri_lo -- placed in
// the lower or the upper pair of lane rows, with zeros or ones in the other pair: tri_lo is zero for k >= 16
// (lane rows 2 and 3), tri_hi is all ones for k < 16 and repeats tri_lo's pattern 16 positions on.  Written this
// way the pattern is computed once per wavefront however many of the constants a kernel uses.
template <int EXCL>
__device__ __forceinline__ half8 tri_pattern(const LaneId& id) { return leading_ones(id.j - 8 * (id.g & 1) + 1 - EXCL); }
__device__ __forceinline__ half8 select8(bool take, half8 a, half8 b) {
    const u64x2 x = __builtin_bit_cast(u64x2, a), y = __builtin_bit_cast(u64x2, b);
    u64x2 r;
    r[0] = take ? x[0] : y[0];
    r[1] = take ? x[1] : y[1];
    return __builtin_bit_cast(half8, r);
}
template <int EXCL = 0>
__device__ __forceinline__ half8 const_tri_lo(const LaneId& id) { return select8(id.g < 2, tri_pattern<EXCL>(id), splat_half(0.0f)); }
template <int EXCL = 0>
__device__ __forceinline__ half8 const_tri_hi(const LaneId& id) { return select8(id.g < 2, splat_half(1.0f), tri_pattern<EXCL>(id)); }
// Same, for rows that hold two independent segments of 16: the second half starts afresh
// (1 iff 16 <= k <= 16 + i).
template <int EXCL = 0>
__device__ __forceinline__ half8 const_tri_hi_seg16(const LaneId& id) { return select8(id.g < 2, splat_half(0.0f), tri_pattern<EXCL>(id)); }
// Two half-row sums at once: output rows 0..7 add up k < 16, rows 8..15 add up k >= 16.
__device__ __forceinline__ half8 const_half_rows(const LaneId& id) {
    const bool one = (id.g >= 2) == (id.j >= 8);
    half8 c;
#pragma unroll
    for (int e = 0; e < 8; ++e) c[e] = one ? (_Float16)1.0f : (_Float16)0.0f;
    return c;
}

// The first `count` (0 .. 8) of a lane's eight binary16 values kept, the others cleared.
__device__ __forceinline__ half8 keep_leading(half8 x, int count) {
    const int c = count < 0 ? 0 : (count > 8 ? 8 : count);
    const int clo = c < 4 ? c : 4, chi = c - clo;
    u64x2 m;
    m[0] = clo ? ~0ull >> (16 * (4 - clo)) : 0ull;
    m[1] = chi ? ~0ull >> (16 * (4 - chi)) : 0ull;
    return __builtin_bit_cast(half8, __builtin_bit_cast(u64x2, x) & m);
}
__device__ __forceinline__ half8 drop_leading(half8 x, int count) {
    const int c = count < 0 ? 0 : (count > 8 ? 8 : count);
    const int clo = c < 4 ? c : 4, chi = c - clo;
    u64x2 m;
    m[0] = clo ? ~0ull >> (16 * (4 - clo)) : 0ull;
    m[1] = chi ? ~0ull >> (16 * (4 - chi)) : 0ull;
    return __builtin_bit_cast(half8, __builtin_bit_cast(u64x2, x) & ~m);
}

__device__ __forceinline__ float4v mfma(half8 constant, half8 data, float4v acc) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(constant, data, acc, 0, 0, 0);
}

__device__ __forceinline__ float4v splat(float v) { return (float4v){v, v, v, v}; }


// ---------------------------------------------------------------- loads and stores

// 8 consecutive binary16 values starting at element `off` (a multiple of 8).  STREAM = true marks the load
// non-temporal: the reductions read every input once and write next to nothing, and without cache allocation
// for those reads they run 8-28 % faster (and no longer pay for the dirty lines a preceding scan left behind);
// the scans, whose loads compete with twice as many bytes of stores, are SLOWER with it and keep plain loads.
template <bool STREAM = false>
__device__ __forceinline__ half8 load8(const _Float16* __restrict__ in, uint64_t off) {
    if constexpr (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const half8*>(in + off));
    else return *reinterpret_cast<const half8*>(in + off);
}
// The same with elements at or beyond n read as zero (the paper's zero padding of a short last tile, Section 4).
template <bool STREAM = false>
__device__ __forceinline__ half8 load8_guarded(const _Float16* __restrict__ in, uint64_t off, uint64_t n) {
    half8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (_Float16)0.0f;
    if (off + 8 <= n) {
        v = load8<STREAM>(in, off);
    } else if (off < n) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (off + e < n) v[e] = in[off + e];
    }
    return v;
}

// How a tile reaches the MFMA operand registers (kept switchable for the measurement that chose kLoadDirect):
//   kLoadDirect   every lane loads its operand -- X[j][8g .. 8g+7] for lane (j, g) -- straight from memory; the 64
//                 loads of a wavefront still cover one contiguous KiB, only the order of the lanes inside it differs;
//   kLoadStaged   lanes load in lane order (lane l: elements 8l .. 8l+7), write to LDS, and read their operand back
//                 from there (the staging through shared memory of the paper's WMMA kernels);
//   kLoadLdsDma   the same staging without the trip through registers: gfx950's 128-bit load from memory into LDS.
// Full tiles only (tile_base + 512 <= n).
enum TileLoad { kLoadDirect = 0, kLoadStaged = 1, kLoadLdsDma = 2 };
template <int LOAD, bool STREAM>
__device__ __forceinline__ half8 load_tile_operand(const _Float16* __restrict__ in, uint64_t tile_base, int j, int g, int lane, int wave) {
    if constexpr (LOAD == kLoadDirect) {
        return load8<STREAM>(in, tile_base + (uint64_t)(kRow * j + 8 * g));
    } else {
        __shared__ half8 s_stage[16][kWave];              // one KiB per wavefront, touched by that wavefront only
        if constexpr (LOAD == kLoadStaged) {
            s_stage[wave][lane] = load8<STREAM>(in, tile_base + (uint64_t)(8 * lane));
        } else {
            // lane l's 16 bytes land at the wavefront's LDS base + 16 l
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(in + tile_base + (uint64_t)(8 * lane)),
                                             (void __attribute__((address_space(3)))*)&s_stage[wave][0], 16, 0, 0);
            __builtin_amdgcn_s_waitcnt(0x0F70);           // vmcnt(0): the data has arrived in LDS
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        return s_stage[wave][4 * j + g];                  // element 32 j + 8 g of the tile
    }
}

__device__ __forceinline__ void store4_guarded(float* __restrict__ out, uint64_t off, uint64_t n, float4v v) {
    if (off + 4 <= n) {
        *reinterpret_cast<float4v*>(out + off) = v;
    } else if (off < n) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (off + e < n) out[off + e] = v[e];
    }
}
__device__ __forceinline__ void store4(float* __restrict__ out, uint64_t off, float4v v) {
    *reinterpret_cast<float4v*>(out + off) = v;
}

// Raw buffer resource over [ptr, ptr + bytes).  The hardware range check makes loads beyond `bytes`
// return zero and drops stores beyond it, so a ragged tile needs no branch around its memory
// instructions (a branch there would also defeat the compiler's counting of outstanding loads and
// stores, which the pipelined scan relies on).  Offsets are in bytes; `bytes` < 2^32.
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* ptr, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(ptr), 0, (int)bytes, 0x00020000);
}
// STREAM = true: non-temporal, as for load8.
template <bool STREAM = false>
__device__ __forceinline__ half8 buffer_load8(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
    return __builtin_bit_cast(half8, __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, STREAM ? 2 : 0));
}
// Four consecutive results of one lane at element `elem` of the resource, binary32 or binary16.
template <int F16>
__device__ __forceinline__ void buffer_store4_t(__amdgpu_buffer_rsrc_t r, uint32_t elem, float4v v) {
    if constexpr (F16) {
        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
        const h4 h = {(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(uint2v, h), r, (int)(elem * 2u), 0, 0);
    } else {
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uint4v, v), r, (int)(elem * 4u), 0, 0);
    }
}

// Binary16 output in the operand map: lane (j, g) holds positions 4g .. 4g+3 (lo) and 16+4g .. 16+4g+3 (hi) of tile
// row j, two 64-bit pieces.  Lane rows g and g+1 (g even) exchange one piece each (v_permlane16_swap: the odd
// lane rows of one register against the even lane rows of another), after which every lane holds 8 CONSECUTIVE
// results -- g even: positions 16+4g .. 16+4g+7, g odd: 4(g-1) .. 4(g-1)+7 -- and stores them as 128 bits like
// the binary32 results.  (With 64-bit stores the binary16 scans ran at 64-70 % of the HBM peak against 72-77 %
// for binary32 output.)  Returns the 8 values; `elem` receives their position inside the tile.
typedef unsigned int uint2w __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4v pair_rows_f16(float4v lo, float4v hi, int j, int g, uint32_t& elem) {
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    const uint2w l = __builtin_bit_cast(uint2w, (h4){(_Float16)lo[0], (_Float16)lo[1], (_Float16)lo[2], (_Float16)lo[3]});
    const uint2w h = __builtin_bit_cast(uint2w, (h4){(_Float16)hi[0], (_Float16)hi[1], (_Float16)hi[2], (_Float16)hi[3]});
    const uint2w a = __builtin_amdgcn_permlane16_swap(h[0], l[0], false, false);
    const uint2w b = __builtin_amdgcn_permlane16_swap(h[1], l[1], false, false);
    elem = (uint32_t)(kRow * j + ((g & 1) ? 4 * (g - 1) : 16 + 4 * g));
    return (uint4v){a[0], b[0], a[1], b[1]};
}
// Both pieces of a lane's results for one tile: binary32 as two 128-bit stores, binary16 as one.
template <int F16>
__device__ __forceinline__ void store_tile_rows_t(void* __restrict__ out, uint64_t tile_base, int j, int g, float4v lo, float4v hi) {
    if constexpr (F16) {
        uint32_t elem;
        const uint4v v = pair_rows_f16(lo, hi, j, g, elem);
        *reinterpret_cast<uint4v*>(static_cast<_Float16*>(out) + tile_base + elem) = v;
    } else {
        float* o = static_cast<float*>(out) + tile_base + (uint64_t)(kRow * j + 4 * g);
        *reinterpret_cast<float4v*>(o) = lo;
        *reinterpret_cast<float4v*>(o + 16) = hi;
    }
}
// The same through a buffer resource; tile_elem: first element of the tile inside the resource.
template <int F16>
__device__ __forceinline__ void buffer_store_tile_rows_t(__amdgpu_buffer_rsrc_t r, uint32_t tile_elem, int j, int g, float4v lo, float4v hi) {
    if constexpr (F16) {
        uint32_t elem;
        const uint4v v = pair_rows_f16(lo, hi, j, g, elem);
        __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)((tile_elem + elem) * 2u), 0, 0);
    } else {
        const uint32_t elem = tile_elem + (uint32_t)(kRow * j + 4 * g);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uint4v, lo), r, (int)(elem * 4u), 0, 0);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uint4v, hi), r, (int)((elem + 16u) * 4u), 0, 0);
    }
}
// Eight consecutive results of one lane (the lane-ordered tile), binary32 or binary16.
template <int F16>
__device__ __forceinline__ void store8_t(void* __restrict__ out, uint64_t off, float4v a, float4v b) {
    if constexpr (F16) {
        const half8 h = {(_Float16)a[0], (_Float16)a[1], (_Float16)a[2], (_Float16)a[3], (_Float16)b[0], (_Float16)b[1], (_Float16)b[2], (_Float16)b[3]};
        *reinterpret_cast<half8*>(static_cast<_Float16*>(out) + off) = h;
    } else {
        *reinterpret_cast<float4v*>(static_cast<float*>(out) + off) = a;
        *reinterpret_cast<float4v*>(static_cast<float*>(out) + off + 4) = b;
    }
}
template <int F16>
__device__ __forceinline__ void buffer_store8_t(__amdgpu_buffer_rsrc_t r, uint32_t elem, float4v a, float4v b) {
    if constexpr (F16) {
        const half8 h = {(_Float16)a[0], (_Float16)a[1], (_Float16)a[2], (_Float16)a[3], (_Float16)b[0], (_Float16)b[1], (_Float16)b[2], (_Float16)b[3]};
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uint4v, h), r, (int)(elem * 2u), 0, 0);
    } else {
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uint4v, a), r, (int)(elem * 4u), 0, 0);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uint4v, b), r, (int)((elem + 4u) * 4u), 0, 0);
    }
}

// Output in binary32 (F16 = 0) or rounded to binary16 (F16 = 1, the paper's own output precision):
// four consecutive results of one lane, `off` counted in elements.
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
template <int F16>
__device__ __forceinline__ void store4_t(void* __restrict__ out, uint64_t off, float4v v) {
    if constexpr (F16) {
        const half4 h = {(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
        *reinterpret_cast<half4*>(static_cast<_Float16*>(out) + off) = h;
    } else {
        *reinterpret_cast<float4v*>(static_cast<float*>(out) + off) = v;
    }
}
template <int F16>
__device__ __forceinline__ void store4_guarded_t(void* __restrict__ out, uint64_t off, uint64_t n, float4v v) {
    if (off + 4 <= n) {
        store4_t<F16>(out, off, v);
    } else if (off < n) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (off + e < n) {
                if constexpr (F16) static_cast<_Float16*>(out)[off + e] = (_Float16)v[e];
                else static_cast<float*>(out)[off + e] = v[e];
            }
        }
    }
}

}  // namespace tcr
