// The scan with a binary16 ACCUMULATOR: the precision of the paper's half-precision mode (Section 2.2: the
// matrix units accumulate in binary16 or binary32; Section 6 counts 2 bytes per scanned output).  The
// 16x16x32 binary16 MFMA of gfx950 accumulates in binary32 only, so this variant cannot run on the matrix
// cores: it is the cross-lane formulation with every addition a binary16 add -- a lane's 8 elements in
// sequence, lane totals across the wavefront with DPP, tile totals through registers, wavefront totals through
// LDS and workgroup totals through the descriptor chain of the binary32 scans (the totals travel as binary32
// words that hold binary16 values).
//
// The order of the additions is a tree, not the left-to-right order of the definition, so a result differs
// from the left-to-right binary16 scan wherever an addition rounds.  It is equal bit for bit when no addition
// rounds (every sum of consecutive elements of a segment is a binary16 value: integers within +-2048, say).
// Otherwise each output has gone through at most kHalfRoundings additions, each with a relative error of at
// most 2^-11:  |out - exact| <= kHalfRoundings * 2^-11 * (sum of |x| over the elements it adds up), plus overflow to
// infinity beyond 65504 like any binary16 sum.
#pragma once
#include "tcr_device.hpp"
#include "tcr_scan.hpp"

namespace tcr {

// 7 inside a lane, 6 across the lanes, U - 1 tiles of a wavefront, 15 wavefronts, 1 for the chain's carry
// (added up in binary32 and rounded once), 3 to combine these, 1 for the element itself.
constexpr int kHalfRoundings = 7 + 6 + 7 + 15 + 1 + 3 + 1;

template <int CTRL, int ROW_MASK, bool BOUND>
__device__ __forceinline__ _Float16 half_dpp(_Float16 x) {
    const int v = (int)__builtin_bit_cast(unsigned short, x);
    return __builtin_bit_cast(_Float16, (unsigned short)__builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, BOUND));
}

// Inclusive binary16 scan over aligned groups of `group` lanes (a power of two, 1 .. 64).
__device__ __forceinline__ _Float16 half_lanes_scan_inclusive(_Float16 x, int lane, int group) {
    const int p = lane & (group - 1);
    const _Float16 zero = (_Float16)0.0f;
    { const _Float16 v = half_dpp<0x111, 0xf, true>(x); x += (p >= 1) ? v : zero; }
    { const _Float16 v = half_dpp<0x112, 0xf, true>(x); x += (p >= 2) ? v : zero; }
    { const _Float16 v = half_dpp<0x114, 0xf, true>(x); x += (p >= 4) ? v : zero; }
    { const _Float16 v = half_dpp<0x118, 0xf, true>(x); x += (p >= 8) ? v : zero; }
    if (group > 16) x += half_dpp<0x142, 0xa, false>(x);      // lane 15 of rows 0 and 2 -> every lane of rows 1 and 3
    if (group > 32) x += half_dpp<0x143, 0xc, false>(x);      // lane 31 -> every lane of rows 2 and 3
    return x;
}

// seg_mask = seg_len - 1 for a power-of-two seg_len, all ones for the one-segment scan; seg_len is only compared
// against a lane's, a tile's, a wavefront's and a workgroup's share (saturated for the one-segment scan).
// Grid: one workgroup per WAVES * U tiles of 512 elements (lane l of a tile holds elements 8l .. 8l+7).
template <int U, int WAVES, int CARRY, int EXCL>
__global__ __launch_bounds__(WAVES * kWave) void scan_half_kernel(const _Float16* __restrict__ in,
                                                                  _Float16* __restrict__ out, uint64_t n,
                                                                  uint64_t seg_mask, uint64_t seg_len,
                                                                  ScanWorkspace ws_arg) {
    static_assert(CARRY == kNoCarry || CARRY == kLookback, "");
    const ScanWorkspace ws = resolve_workspace(ws_arg);
    constexpr uint64_t kChunk = (uint64_t)kTile * U;
    constexpr uint64_t kBlockTile = kChunk * WAVES;
    __shared__ float s_wave_total[WAVES];         // binary16 values
    __shared__ float s_prefix;
    __shared__ uint32_t s_tile;
    const _Float16 zero = (_Float16)0.0f;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t tile = blockIdx.x;
    if constexpr (CARRY == kLookback) {
        if (threadIdx.x == 0)
            s_tile = __hip_atomic_fetch_add(ws.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - ws.ticket_base;
        __syncthreads();
        tile = s_tile;
        if (tile == 0 && threadIdx.x == 0 && ws.state != nullptr && !ws.device_managed) ws.state[0] = ws.epoch;
    }
    const uint64_t block_base = (uint64_t)tile * kBlockTile;
    const uint64_t base = block_base + (uint64_t)wave * kChunk;
    const bool full = base + kChunk <= n;

    half8 x[U];
    if (full) {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8(in, base + (uint64_t)(kTile * u + 8 * lane));
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8_guarded(in, base + (uint64_t)(kTile * u + 8 * lane), n);
    }

    // inside a lane: running binary16 sums, restarting every seg_len elements when segments are shorter than 8
    const int restart = seg_len < 8 ? (int)seg_len - 1 : 7;            // a segment starts where (e & restart) == 0 ...
    half8 p[U];
    _Float16 carry_lane[U], tile_total[U];
    const int group = seg_len >= (uint64_t)kTile ? kWave : (seg_len >= 8 ? (int)(seg_len >> 3) : 1);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        _Float16 run = zero;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (seg_len < 8 && (e & restart) == 0) run = zero;           // ... (for seg_len >= 8: only at e == 0, where run is 0)
            if constexpr (EXCL) p[u][e] = run;
            run += x[u][e];
            if constexpr (!EXCL) p[u][e] = run;
        }
        // across the lanes of a segment (or of the tile)
        const _Float16 incl = half_lanes_scan_inclusive(run, lane, group);
        const _Float16 prev = half_dpp<0x138, 0xf, true>(incl);          // the previous lane's (0 for lane 0)
        carry_lane[u] = (seg_len > 8 && (lane & (group - 1)) != 0) ? prev : zero;
        tile_total[u] = __builtin_bit_cast(_Float16, (unsigned short)__builtin_amdgcn_readlane(
            (int)__builtin_bit_cast(unsigned short, incl), 63));
    }
    // across the tiles of this wavefront; restarts where a segment starts
    _Float16 before[U];
    _Float16 run = zero;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (((base + (uint64_t)(kTile * u)) & seg_mask) == 0) run = zero;
        before[u] = run;
        run += tile_total[u];
    }
    // across wavefronts and workgroups (only when a segment is longer than a wavefront's share)
    _Float16 ext = zero;
    if (seg_len > kChunk) {
        if (lane == 0) s_wave_total[wave] = (float)run;
        __syncthreads();
        const int first_wave = (seg_len >= kBlockTile) ? 0 : (wave & ~((int)(seg_len / kChunk) - 1));
        for (int w = first_wave; w < wave; ++w) ext += (_Float16)s_wave_total[w];
        if constexpr (CARRY == kLookback) {
            if (seg_len > kBlockTile) {
                if (wave == 0) {
                    _Float16 total = zero;
#pragma unroll
                    for (int w = 0; w < WAVES; ++w) total += (_Float16)s_wave_total[w];
                    const uint32_t pos = (uint32_t)((block_base & seg_mask) / kBlockTile);
                    // (the totals of earlier workgroups are added up in binary32 and rounded once)
                    const float pre = lookback_exclusive_prefix<64>(ws, tile, pos, (float)total, lane);
                    if (lane == 0) s_prefix = (float)(_Float16)pre;
                }
                __syncthreads();
                ext += (_Float16)s_prefix;
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const _Float16 carry = (seg_len > (uint64_t)kTile ? (carry_lane[u] + before[u]) : carry_lane[u]) + ext;
        half8 r;
#pragma unroll
        for (int e = 0; e < 8; ++e) r[e] = p[u][e] + carry;
        const uint64_t off = base + (uint64_t)(kTile * u + 8 * lane);
        if (full) {
            *reinterpret_cast<half8*>(out + off) = r;
        } else if (off < n) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (off + e < n) out[off + e] = r[e];
        }
    }
}

}  // namespace tcr
