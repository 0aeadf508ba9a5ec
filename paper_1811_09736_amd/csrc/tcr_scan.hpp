// Segmented / full inclusive-scan kernels (Section 5 of the paper, re-derived for MFMA).
//
// Inside a tile (16 rows of 32 elements) the scan is the paper's  Scan(V) = G + A.U :
//   * A.U, the inclusive scan of every row, is two products with the triangular constants
//     (positions 0..15 and 16..31 of a row);
//   * G, "everything before this row", starts from a product with the all-ones matrix, which
//     leaves every row's total in every lane of that row's column; the exclusive scan of those
//     16 totals is done with binary32 cross-lane adds (the paper multiplies L.A by the ones
//     matrix instead, which would push binary32 sums through a binary16 operand);
//   * G plus the running carry of earlier tiles (the paper's S matrix) enters the triangular
//     products through the accumulator, so adding the carry costs nothing.
//
//   scan_small_kernel     seg_len in {16, ..., 512}: segments never leave a tile (Scan_16 and
//                         Scan_16N / Scan_256 territory).
//   scan_block_kernel     seg_len >= 1024 and the full scan: a workgroup scans WAVES*U consecutive
//                         tiles (Scan_256N per wavefront, the block-level combination through
//                         LDS), and a segment longer than a workgroup's share gets its carry
//                         from earlier workgroups either by single-pass decoupled look-back
//                         (CARRY == kLookback) or from a precomputed table of exclusive prefixes
//                         (CARRY == kTable, the reduce-then-scan alternative).
//   scan_chain_kernel     the same single pass for segments of 32768 elements and more as a
//                         persistent three-stage pipeline (the dispatched device-level scan,
//                         Section 5, for the matrix-core formulation).
//   scan_partials_kernel, gather_totals_kernel, uniform_add_kernel
//                         the small kernels of the multi-kernel strategies (reduce-then-scan, and
//                         the paper's scan-then-propagate).
#pragma once
#include "tcr_device.hpp"
#include "tcr_reduce.hpp"

namespace tcr {

enum CarryMode { kNoCarry = 0, kLookback = 1, kTable = 2 };
// Host-side choice of how a carry crosses workgroups: a single pass (default: scan_chain_kernel or
// look-back), reduce-then-scan (kTable kernels), or the paper's own three-kernel scan-then-propagate.
enum CarryStrategy { kStrategyLookback = 0, kStrategyReduceThenScan = 1, kStrategyScanThenPropagate = 2 };

// Inclusive scan over aligned groups of GROUP lanes (GROUP up to 64).
template <int GROUP>
__device__ __forceinline__ float lanes_scan_inclusive(float x, int lane) {
    if constexpr (GROUP <= 16) return row_scan_inclusive<GROUP>(x, lane & 15);
    x = row_scan_inclusive<16>(x, lane & 15);
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x142, 0xa, 0xf, false));
    if constexpr (GROUP > 32)
        x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x143, 0xc, 0xf, false));
    return x;
}

// Value of the previous lane of the wavefront (0 for lane 0).
__device__ __forceinline__ float wave_shr1(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x138, 0xf, 0xf, true));
}

// In-lane scan of 8 values, binary32: inclusive (EXCL = 0) or exclusive (EXCL = 1).  Returns the
// sum of all eight.
template <int EXCL = 0>
__device__ __forceinline__ float scan8(half8 v, float (&p)[8]) {
    float run = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if constexpr (EXCL) p[e] = run;
        run += (float)v[e];
        if constexpr (!EXCL) p[e] = run;
    }
    return run;
}

// ------------------------------------------------------------------------------ small segments
// MODE bit 0: exclusive scan; bit 1: binary16 output.
// LOAD: how the tiles reach the operand registers (TileLoad; matrix-core formulation, full tiles).
template <int FORM, int LOG2L, int U, int WAVES, int MODE = 0, int LOAD = kLoadDirect>
__global__ __launch_bounds__(WAVES * kWave) void scan_small_kernel(const _Float16* __restrict__ in,
                                                                   void* __restrict__ out, uint64_t n) {
    constexpr int EXCL = MODE & 1, F16 = MODE >> 1;
    static_assert(LOG2L >= 4 && LOG2L <= 9, "");
    const LaneId id;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keeps per-wave branches and addresses scalar
    const uint64_t base = ((uint64_t)blockIdx.x * WAVES + wave) * (uint64_t)(kTile * U);
    if (base >= n) return;
    const bool full = base + (uint64_t)(kTile * U) <= n;
    const int lane_off = (FORM == kMfma) ? (kRow * id.j + 8 * id.g) : (8 * id.lane);

    half8 x[U];
    if (full) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if constexpr (FORM == kMfma && LOAD != kLoadDirect) x[u] = load_tile_operand<LOAD, false>(in, base + (uint64_t)(kTile * u), id.j, id.g, id.lane, wave);
            else x[u] = load8(in, base + (uint64_t)(kTile * u + lane_off));
        }
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8_guarded(in, base + (uint64_t)(kTile * u + lane_off), n);
    }

#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t tbase = base + (uint64_t)(kTile * u);
        float4v lo, hi;
        uint64_t off_lo, off_hi;
        if constexpr (FORM == kMfma) {
            if constexpr (LOG2L == 4) {
                lo = mfma(const_tri_lo<EXCL>(id), x[u], splat(0.0f));
                hi = mfma(const_tri_hi_seg16<EXCL>(id), x[u], splat(0.0f));
            } else if constexpr (LOG2L == 5) {
                lo = mfma(const_tri_lo<EXCL>(id), x[u], splat(0.0f));
                hi = mfma(const_tri_hi<EXCL>(id), x[u], splat(0.0f));
            } else {
                constexpr int ROWS = 1 << (LOG2L - 5);
                const float4v tot = mfma(const_ones(), x[u], splat(0.0f));
                const float incl = row_scan_inclusive<ROWS>(tot[0], id.j);
                const float prev = row_shr<1>(incl);
                const float g = ((id.j & (ROWS - 1)) == 0) ? 0.0f : prev;     // rows before mine, same segment
                lo = mfma(const_tri_lo<EXCL>(id), x[u], splat(g));
                hi = mfma(const_tri_hi<EXCL>(id), x[u], splat(g));
            }
            off_lo = tbase + (uint64_t)(kRow * id.j + 4 * id.g);
            off_hi = off_lo + 16;
        } else {
            constexpr int LANES = 1 << (LOG2L - 3);
            float p[8];
            const float lane_total = scan8<EXCL>(x[u], p);
            const float incl = lanes_scan_inclusive<LANES>(lane_total, id.lane);
            const float prev = wave_shr1(incl);
            const float g = ((id.lane & (LANES - 1)) == 0) ? 0.0f : prev;
            lo = (float4v){p[0] + g, p[1] + g, p[2] + g, p[3] + g};
            hi = (float4v){p[4] + g, p[5] + g, p[6] + g, p[7] + g};
            off_lo = tbase + (uint64_t)(8 * id.lane);
            off_hi = off_lo + 4;
        }
        if (full) {
            if constexpr (FORM == kMfma) store_tile_rows_t<F16>(out, tbase, id.j, id.g, lo, hi);
            else store8_t<F16>(out, off_lo, lo, hi);
        } else {
            store4_guarded_t<F16>(out, off_lo, n, lo);
            store4_guarded_t<F16>(out, off_hi, n, hi);
        }
    }
}

// ------------------------------------------------------------------------------ look-back state
// One 64-bit word per workgroup tile: high half = tag, low half = binary32 value.
// tag = epoch * 4 + status; a word whose epoch differs from the launch's is "not yet written",
// so the table never needs clearing between launches.
constexpr uint32_t kStatusAggregate = 1;   // value = total of this tile only
constexpr uint32_t kStatusPrefix = 2;      // value = total of this tile and all earlier tiles of its segment
constexpr int kSpinLimit = 1 << 20;        // polls of one look-back window before giving up

struct ScanWorkspace {
    unsigned long long* desc;   // [tiles]
    uint32_t* ticket;           // running count of tiles handed out since the workspace was created
    uint32_t* gave_up;          // set to 1 if a bounded wait expired
    uint32_t ticket_base;       // value of *ticket when this launch starts
    uint32_t epoch;
    // state[0]: epoch of the latest launch, state[1]: *ticket at its start.  Host-managed workspaces
    // (device_managed == 0) pass epoch and ticket_base above and the launch only records its epoch in
    // state[0]; device-managed ones (launches recorded into HIP graphs, whose arguments are frozen)
    // take both from state[], which chain_begin_kernel advances in front of every launch.
    uint32_t* state;
    uint32_t device_managed;
};

__device__ __forceinline__ ScanWorkspace resolve_workspace(ScanWorkspace w) {
    if (w.state != nullptr && w.device_managed) {
        w.epoch = w.state[0];
        w.ticket_base = w.state[1];
    }
    return w;
}

// Device-managed workspaces: one workgroup, enqueued in front of every launch that chains tiles.  Starts a
// new epoch (clearing the descriptor table when the 30-bit epoch wraps) and records the ticket count the
// launch starts from -- every earlier launch on the stream has finished drawing by now.
constexpr int kBeginThreads = 256;
__global__ __launch_bounds__(kBeginThreads) void chain_begin_kernel(uint32_t* __restrict__ counters,
                                                                    unsigned long long* __restrict__ desc,
                                                                    uint64_t desc_capacity) {
    uint32_t epoch = counters[2] + 1u;
    if (epoch >= (1u << 30) - 2u) {
        for (uint64_t i = threadIdx.x; i < desc_capacity; i += kBeginThreads) desc[i] = 0ull;
        epoch = 1u;
    }
    __syncthreads();                                  // every thread has read the old epoch
    if (threadIdx.x == 0) {
        counters[2] = epoch;
        counters[3] = counters[0];
    }
}

// Host-managed workspaces that must not be cleared from the host (no synchronisation, no runtime call that may
// allocate): every descriptor and the running counters back to zero, in stream order.  The give-up flag
// (counters[1]) survives unless keep_flag == 0.
constexpr int kClearThreads = 256;
__global__ __launch_bounds__(kClearThreads) void workspace_clear_kernel(uint32_t* __restrict__ counters,
                                                                        unsigned long long* __restrict__ desc,
                                                                        uint64_t desc_capacity, uint32_t keep_flag) {
    const uint64_t stride = (uint64_t)gridDim.x * kClearThreads;
    for (uint64_t i = (uint64_t)blockIdx.x * kClearThreads + threadIdx.x; i < desc_capacity; i += stride) desc[i] = 0ull;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        counters[0] = 0u;
        if (!keep_flag) counters[1] = 0u;
        counters[2] = 0u;
        counters[3] = 0u;
    }
}

__device__ __forceinline__ unsigned long long pack_desc(uint32_t epoch, uint32_t status, float v) {
    return ((unsigned long long)(epoch * 4u + status) << 32) | (unsigned long long)__builtin_bit_cast(uint32_t, v);
}

// Descriptor words live in uncached device memory and are read with agent scope: the tiles of
// one chain run on different XCDs, whose L2 caches are not coherent with each other.  (A read
// that only bypasses the first-level cache was tried and does see stale words.)
__device__ __forceinline__ unsigned long long load_descriptor(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Executed by one whole wavefront.  Returns (uniformly) the sum of the totals of all earlier
// tiles of this tile's segment and publishes this tile's own state.
//   pos     number of earlier tiles that may belong to this tile's segment (0 = none: nothing to look up)
//   closed  a segment starts inside this tile: `total` is then the sum since the last such start, which is
//           all a later tile can need of this one, so it is published as a finished prefix at once and
//           the carry found here (for the elements in front of the first start) is not added to it
//   WIN     descriptors inspected per round (the WIN nearest predecessors, one per lane).
// Every agent-scope read costs a slice of a resource shared by the whole chip (measured: one
// 64-wide read per tile adds ~6 ns per tile to the launch, and wider windows only add to it), so
// the window is kept as narrow as the distance to the nearest finished prefix allows.
template <int WIN>
__device__ __forceinline__ float lookback_carry(const ScanWorkspace& ws, uint32_t tile, uint32_t pos, bool closed,
                                                float total, int lane) {
    static_assert(WIN >= 1 && WIN <= kWave, "");
    const bool final_now = closed || pos == 0;
    if (lane == 0)
        __hip_atomic_store(&ws.desc[tile], pack_desc(ws.epoch, final_now ? kStatusPrefix : kStatusAggregate, total),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (pos == 0) return 0.0f;
    constexpr int kNone = 1 << 30;
    float acc = 0.0f;
    uint32_t base = 0;                           // this round inspects distances base+1 .. base+WIN
    while (true) {
        const bool in_window = lane < WIN;
        const bool valid = in_window && base + 1u + (uint32_t)lane <= pos;   // not past the segment's first tile
        // slots past the segment start act as "prefix 0"; lanes outside the window as "aggregate 0"
        uint32_t status = in_window ? kStatusPrefix : kStatusAggregate;
        float value = 0.0f;
        bool ready = !valid;
        int nearest = kNone;                     // lane of the nearest finished prefix
        int polls = 0;
        while (true) {
            if (!ready) {
                const uint32_t dist = base + 1u + (uint32_t)lane;
                const unsigned long long d = load_descriptor(&ws.desc[tile - dist]);
                const uint32_t tag = (uint32_t)(d >> 32);
                if ((tag >> 2) == ws.epoch && (tag & 3u) != 0u) {
                    status = tag & 3u;
                    value = __builtin_bit_cast(float, (uint32_t)d);
                    ready = true;
                }
            }
            const unsigned long long m = __ballot(ready && status == kStatusPrefix);
            nearest = (m != 0ull) ? __builtin_ctzll(m) : kNone;
            // done once every slot nearer than the nearest finished prefix has been written
            if (__ballot(!ready && lane < nearest) == 0ull) break;
            if (++polls > kSpinLimit) {          // should be unreachable: predecessors hold earlier tickets
                if (lane == 0) __hip_atomic_store(ws.gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        acc += wave_sum((ready && lane <= nearest) ? value : 0.0f);
        if (nearest != kNone) break;
        base += (uint32_t)WIN;
    }
    if (lane == 0 && !final_now)
        __hip_atomic_store(&ws.desc[tile], pack_desc(ws.epoch, kStatusPrefix, acc + total), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    return acc;
}

// Regular segments: tile number `pos` of its segment has exactly `pos` predecessors and no start inside.
template <int WIN>
__device__ __forceinline__ float lookback_exclusive_prefix(const ScanWorkspace& ws, uint32_t tile, uint32_t pos,
                                                           float total, int lane) {
    return lookback_carry<WIN>(ws, tile, pos, false, total, lane);
}

// ------------------------------------------------------------------------------ long segments
// seg_mask  = seg_len - 1 for a power-of-two seg_len, all ones for the full scan (one segment).
// seg_len   only compared against the wavefront / workgroup share (saturated for the full scan).
// Grid: one workgroup (WAVES wavefronts) per WAVES*U tiles.
// MODE bit 0: exclusive scan; bit 1: binary16 output.
template <int FORM, int U, int WAVES, int CARRY, int MODE = 0>
__global__ __launch_bounds__(WAVES * kWave) void scan_block_kernel(const _Float16* __restrict__ in,
                                                                   void* __restrict__ out, uint64_t n,
                                                                   uint64_t seg_mask, uint64_t seg_len,
                                                                   ScanWorkspace ws_arg,
                                                                   const float* __restrict__ tile_prefix) {
    constexpr int EXCL = MODE & 1, F16 = MODE >> 1;
    const ScanWorkspace ws = resolve_workspace(ws_arg);
    constexpr uint64_t kChunk = (uint64_t)kTile * U;             // one wavefront's share
    constexpr uint64_t kBlockTile = kChunk * WAVES;              // one workgroup's share
    __shared__ float s_wave_total[WAVES];
    __shared__ float s_prefix;
    __shared__ uint32_t s_tile;

    const LaneId id;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: keeps per-wave branches and addresses scalar
    uint32_t tile = blockIdx.x;
    if constexpr (CARRY == kLookback) {
        // tiles are handed out in launch order, so every predecessor of a waiting tile is
        // already running or finished
        if (threadIdx.x == 0)
            s_tile = __hip_atomic_fetch_add(ws.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - ws.ticket_base;
        __syncthreads();
        tile = s_tile;
    }
    if constexpr (CARRY == kLookback) {
        if (tile == 0 && threadIdx.x == 0 && ws.state != nullptr && !ws.device_managed) ws.state[0] = ws.epoch;
    }
    const uint64_t block_base = (uint64_t)tile * kBlockTile;
    const uint64_t base = block_base + (uint64_t)wave * kChunk;
    const bool full = base + kChunk <= n;
    const int lane_off = (FORM == kMfma) ? (kRow * id.j + 8 * id.g) : (8 * id.lane);

    half8 x[U];
    if (full) {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8(in, base + (uint64_t)(kTile * u + lane_off));
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8_guarded(in, base + (uint64_t)(kTile * u + lane_off), n);
    }

    // per tile: exclusive carry of this lane's row (MFMA) or lane (DPP) inside the tile, and the tile total
    float inner[U], tile_total[U];
    float p[(FORM == kDpp) ? U : 1][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (FORM == kMfma) {
            const float4v tot = mfma(const_ones(), x[u], splat(0.0f));
            const float incl = row_scan_inclusive<16>(tot[0], id.j);
            inner[u] = row_shr<1>(incl);
            tile_total[u] = read_lane(incl, 15);
        } else {
            const float lane_total = scan8<EXCL>(x[u], p[u]);
            const float incl = wave_scan_inclusive(lane_total);
            inner[u] = wave_shr1(incl);
            tile_total[u] = read_lane(incl, 63);
        }
    }
    // running carry over this wavefront's tiles (the S matrix of Scan_256N); restarts where a segment starts
    float before[U];
    float run = 0.0f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (((base + (uint64_t)(kTile * u)) & seg_mask) == 0) run = 0.0f;
        before[u] = run;
        run += tile_total[u];
    }
    // carry from earlier wavefronts / workgroups of the same segment (only when a segment is
    // longer than one wavefront's share; then the share lies inside a single segment)
    float ext = 0.0f;
    if (seg_len > kChunk) {
        if (id.lane == 0) s_wave_total[wave] = run;
        __syncthreads();
        const int first_wave = (seg_len >= kBlockTile) ? 0 : (wave & ~((int)(seg_len / kChunk) - 1));
        for (int w = first_wave; w < wave; ++w) ext += s_wave_total[w];
        if (CARRY != kNoCarry && seg_len > kBlockTile) {
            if constexpr (CARRY == kLookback) {
                if (wave == 0) {
                    float total = 0.0f;
#pragma unroll
                    for (int w = 0; w < WAVES; ++w) total += s_wave_total[w];
                    const uint32_t pos = (uint32_t)((block_base & seg_mask) / kBlockTile);
                    const float pre = lookback_exclusive_prefix<64>(ws, tile, pos, total, id.lane);
                    if (id.lane == 0) s_prefix = pre;
                }
                __syncthreads();
                ext += s_prefix;
            } else {
                ext += tile_prefix[tile];
            }
        }
    }

#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t tbase = base + (uint64_t)(kTile * u);
        const float carry = inner[u] + (before[u] + ext);
        float4v lo, hi;
        uint64_t off_lo, off_hi;
        if constexpr (FORM == kMfma) {
            lo = mfma(const_tri_lo<EXCL>(id), x[u], splat(carry));
            hi = mfma(const_tri_hi<EXCL>(id), x[u], splat(carry));
            off_lo = tbase + (uint64_t)(kRow * id.j + 4 * id.g);
            off_hi = off_lo + 16;
        } else {
            const float* q = p[(FORM == kDpp) ? u : 0];
            lo = (float4v){q[0] + carry, q[1] + carry, q[2] + carry, q[3] + carry};
            hi = (float4v){q[4] + carry, q[5] + carry, q[6] + carry, q[7] + carry};
            off_lo = tbase + (uint64_t)(8 * id.lane);
            off_hi = off_lo + 4;
        }
        if (full) {
            if constexpr (FORM == kMfma) store_tile_rows_t<F16>(out, tbase, id.j, id.g, lo, hi);
            else store8_t<F16>(out, off_lo, lo, hi);
        } else {
            store4_guarded_t<F16>(out, off_lo, n, lo);
            store4_guarded_t<F16>(out, off_hi, n, hi);
        }
    }
}

// ------------------------------------------------------------------------------ long segments, pipelined
// scan_chain_kernel: the single-pass chained scan as a persistent, software-pipelined loop (either
// formulation of the tile arithmetic).  One workgroup per compute unit draws tiles by ticket and holds three at a time, each in
// registers of its own:
//     C  just drawn: its loads are issued first thing in a step,
//     B  loaded a step ago: its totals are computed and its aggregate PUBLISHED next,
//     A  published a step ago: its carry is looked up, its results are computed and stored.
// Why three stages.  scan_block_kernel leaves a compute unit with nothing in flight while a tile waits for
// its carry (one descriptor round trip per tile).  Persistent workgroups move in step, one tile each per
// "generation", so with two stages every tile would wait for the slowest aggregate of its whole
// generation in every step.  Publishing a tile's aggregate a full step before its carry is looked up
// removes the wait: by then the aggregates of all lower tiles have been visible for a step.
// The carry of a tile is the inclusive prefix of the workgroup's OWN previous tile plus the aggregates of
// the tiles in between (about one per workgroup, read in one round trip, see chain_sum_totals); no tile
// waits for another tile's prefix, and only aggregates are published.
// Loads are always issued before the stores of the same step: a wavefront's memory operations complete
// in issue order, so data requested after stores could not be used before those stores have drained.
// All bulk loads and stores go through range-checked buffer resources and are unconditional, which lets
// the compiler count outstanding operations exactly instead of draining them at every branch.
// Tickets: three draws at the start of a workgroup (spaced out, see the kernel) and one per finished
// tile, so a launch of G workgroups over T tiles draws exactly T + 3G tickets.
// Progress: a tile waits only for aggregates of lower tickets.  Each of those is held by a running
// workgroup, which publishes it after finishing at most two tiles with still lower tickets; so the
// lowest unfinished ticket can always complete.
// seg_len: any multiple of 8 that is at least one workgroup's share, or seg_len == n with n % 8 == 0.

// Executed by one whole wavefront: the sum of the published totals of tiles lo .. tile-1, read up to
// four per lane per round trip.
__device__ __forceinline__ float chain_sum_totals(const ScanWorkspace& ws, uint32_t lo, uint32_t tile, int lane) {
    float acc = 0.0f;
    uint32_t hi = tile;                                  // tiles lo .. hi-1 are still to be added
    while (hi > lo) {
        const uint32_t span = (hi - lo > 256u) ? 256u : hi - lo;
        float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        bool need[4];
        uint32_t idx[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            need[q] = (uint32_t)(lane + 64 * q) < span;
            // slots beyond the span read this tile's own word, so all four reads are issued
            // unconditionally, travel together and are waited for once
            idx[q] = need[q] ? hi - 1u - (uint32_t)(lane + 64 * q) : tile;
        }
        const uint32_t want = ws.epoch * 4u + kStatusAggregate;
        int polls = 0;
        while (true) {
            unsigned long long d[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) d[q] = load_descriptor(&ws.desc[idx[q]]);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (need[q] && (uint32_t)(d[q] >> 32) == want) {
                    v[q] = __builtin_bit_cast(float, (uint32_t)d[q]);
                    need[q] = false;
                }
            }
            if (__ballot(need[0] || need[1] || need[2] || need[3]) == 0ull) break;
            if (++polls > kSpinLimit) {                  // should be unreachable: predecessors hold earlier tickets
                if (lane == 0) __hip_atomic_store(ws.gave_up, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        acc += wave_sum((v[0] + v[1]) + (v[2] + v[3]));
        hi -= span;
    }
    return acc;
}

// What the chain needs to know of a tile of an IRREGULAR scan without reading the offsets: where the tile's
// last segment start lies (kNoHead: it has none; kOutside: it has none and lies outside [offsets[0],
// offsets[nseg]), so nothing of it is stored), and which tile in front of it holds the nearest segment start
// (kNoHead: none does).  Written by irregular_bounds_kernel.
struct TileLink {
    uint32_t last_head;
    uint32_t prev_head_tile;
};
constexpr uint32_t kNoHead = 0xffffffffu, kOutside = 0xfffffffeu;

struct ChainShared {
    float wave_total[16];
    float prefix;
    uint32_t ticket;
};

// One held tile, as seen by one wavefront.
template <int U>
struct ChainTile {
    half8 x[U];          // the wavefront's share of the tile
    float pre[U];        // per lane: carry inside the wavefront's share in front of the lane's row of tile u
    float ext;           // total of the lower wavefronts of the workgroup
    float total;         // wavefront 0: total of the tile
    uint32_t tile;       // ticket; >= tiles: nothing to do
    uint32_t pos;        // index of the tile inside its segment
    uint32_t count;      // elements of the wavefront's share that exist (the last tile of a segment is ragged)
    uint64_t base;       // first element of the wavefront's share
    uint32_t last_head, prev_head_tile;      // irregular segments only: the tile's TileLink (the same in every lane)
};

// Tiles are laid out per segment: segment s owns tiles s * per_segment .. (s + 1) * per_segment - 1, which
// start at s * seg_len and may overhang its end (the overhang is cut off by the buffer range check).  seg_len
// is any multiple of 8 that is at least one tile; the one-segment scan has seg_len = n and per_segment = tiles.
// Irregular segments (IRREG, a table of TileLinks): one grid over the whole array (seg_len = n, per_segment =
// tiles); the kernel scans and stores only the tiles WITHOUT a segment start that lie inside the covered part of
// the array -- such a tile continues the segment of the tiles in front of it, back to the nearest tile with a
// start -- and publishes for every tile the sum behind its last start (all of it if it has none), which is
// exactly what the tiles behind it need of it, and the running sum at its end in a second table behind the
// first.  The tiles with starts are left to a second kernel.
struct ChainGrid {
    uint64_t seg_len;
    uint32_t per_segment;
    uint32_t tiles;
};

// Stage C: request the data of ticket `tile`.
template <int FORM, int U, int WAVES, bool IRREG = false>
__device__ __forceinline__ void chain_load(ChainTile<U>& t, uint32_t tile, const _Float16* __restrict__ in,
                                           const ChainGrid& grid, const LaneId& id, int wave,
                                           const TileLink* __restrict__ links = nullptr) {
    constexpr uint32_t kChunk = (uint32_t)kTile * U;
    constexpr uint64_t kBlockTile = (uint64_t)kChunk * WAVES;
    const uint32_t seg = tile / grid.per_segment;
    t.tile = tile;
    t.pos = tile - seg * grid.per_segment;
    const uint64_t seg_begin = (uint64_t)seg * grid.seg_len;
    t.base = seg_begin + (uint64_t)t.pos * kBlockTile + (uint64_t)wave * kChunk;
    // elements of the wavefront's share inside the segment (none for a ticket past the last tile)
    const uint64_t seg_end = seg_begin + grid.seg_len;
    const uint64_t left = (tile < grid.tiles && t.base < seg_end) ? seg_end - t.base : 0;
    t.count = left < kChunk ? (uint32_t)left : kChunk;
    const __amdgpu_buffer_rsrc_t src = make_rsrc(in + (t.count ? t.base : 0), t.count * 2u);
#pragma unroll
    for (int u = 0; u < U; ++u)
        t.x[u] = buffer_load8(src, (uint32_t)(kTile * u + (FORM == kMfma ? kRow * id.j + 8 * id.g : 8 * id.lane)) * 2u);
    if constexpr (IRREG) {
        // the same address in every lane: a scalar load, its two words in scalar registers until the next step
        const TileLink link = links[tile < grid.tiles ? tile : 0u];
        t.last_head = link.last_head;
        t.prev_head_tile = link.prev_head_tile;
    }
}

// Stage B: totals of the tile, carries inside the workgroup, aggregate published.  Contains one barrier,
// executed also for a ticket past the last tile.
template <int FORM, int U, int WAVES, bool IRREG = false>
__device__ __forceinline__ void chain_publish(ChainTile<U>& t, const ScanWorkspace& ws, uint32_t tiles, ChainShared& sh,
                                              const LaneId& id, int wave) {
    if constexpr (IRREG) {
        static_assert(!IRREG || FORM == kMfma, "");
        // a tile with a segment start is not scanned here: only the sum behind its last start is wanted of it,
        // so everything in front of that start is cleared (the masking of Section 4, on the data operand)
        if (t.last_head < kOutside) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int at = (int)((uint32_t)wave * (uint32_t)(kTile * U) + (uint32_t)(kTile * u + kRow * id.j + 8 * id.g));
                t.x[u] = drop_leading(t.x[u], (int)t.last_head - at);
            }
        }
    }
    float run = 0.0f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (FORM == kMfma) {
            const float4v tot = mfma(const_ones(), t.x[u], splat(0.0f));
            const float incl = row_scan_inclusive<16>(tot[0], id.j);
            t.pre[u] = row_shr<1>(incl) + run;
            run += read_lane(incl, 15);
        } else {
            const float incl = wave_scan_inclusive(sum8(t.x[u]));
            t.pre[u] = wave_shr1(incl) + run;
            run += read_lane(incl, 63);
        }
        asm volatile("" : "+v"(t.pre[u]));        // keep the sum here: sunk to its use it costs a second register per tile
    }
    if (id.lane == 0) sh.wave_total[wave] = run;
    __syncthreads();
    float ext = 0.0f;
    for (int w = 0; w < wave; ++w) ext += sh.wave_total[w];
    t.ext = ext;
    if (wave == 0) {
        float total = 0.0f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) total += sh.wave_total[w];
        t.total = total;
        if (id.lane == 0 && t.tile < tiles)
            __hip_atomic_store(&ws.desc[t.tile], pack_desc(ws.epoch, kStatusAggregate, total), __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Stage A: carry from the earlier tiles of the segment, results, stores.  Returns a freshly drawn ticket.
// own_end / own_incl (wavefront 0): index after the tile this workgroup finished last (0: none yet) and
// that tile's inclusive prefix.
template <int FORM, int U, int WAVES, int MODE, bool IRREG = false>
__device__ __forceinline__ uint32_t chain_finish(ChainTile<U>& t, void* __restrict__ out,
                                                 const ScanWorkspace& ws, ChainShared& sh, const LaneId& id, int wave,
                                                 uint32_t& own_end, float& own_incl, uint32_t tiles) {
    constexpr int EXCL = MODE & 1, F16 = MODE >> 1;
    if (wave == 0) {
        uint32_t drawn = 0u;                      // used only after the reads below, so the draw rides along with them
        if (id.lane == 0) drawn = __hip_atomic_fetch_add(ws.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t seg_first = t.tile - t.pos;                        // first tile of the segment
        bool closed = false;                                        // irregular: the tile holds a segment start
        if constexpr (IRREG) {
            // the segment reaches back to the nearest tile with a start, whose published sum begins at that start
            closed = t.last_head < kOutside;
            seg_first = (closed || t.prev_head_tile >= t.tile) ? t.tile : t.prev_head_tile;
        }
        const bool resume = own_end > seg_first;  // the workgroup's previous tile lies in the same segment
        float before = chain_sum_totals(ws, resume ? own_end : seg_first, t.tile, id.lane);
        if (resume) before += own_incl;
        own_end = t.tile + 1u;
        own_incl = closed ? t.total : before + t.total;
        // The reads above have drained this wavefront's memory operations (or, with nothing to read, this
        // does); saying so explicitly keeps the pending ticket draw from counting, after the branch
        // rejoins, as a pending write to a register in all wavefronts.
        __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0)
        if constexpr (IRREG) {
            // the running sum at the end of this tile (since the last start), for the second kernel: one read
            // there instead of a sum over all the tiles back to that start.  (Behind the wait: nothing in this
            // kernel reads it, so nobody waits for the store's way to memory either.)
            if (id.lane == 0)
                __hip_atomic_store(&ws.desc[tiles + t.tile], pack_desc(ws.epoch, kStatusPrefix, own_incl), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
        if (id.lane == 0) {
            sh.prefix = before;
            sh.ticket = drawn - ws.ticket_base;
        }
    }
    __syncthreads();
    const float ext = t.ext + sh.prefix;
    const uint32_t fresh = __builtin_amdgcn_readfirstlane(sh.ticket);

    uint32_t store = t.count;
    if constexpr (IRREG) {
        // only tiles without a start, inside the covered part of the array (everything else: an empty range)
        if (t.last_head != kNoHead) store = 0u;
    }
    const __amdgpu_buffer_rsrc_t dst =
        make_rsrc(static_cast<char*>(out) + (store ? t.base : 0) * (F16 ? 2u : 4u), store * (F16 ? 2u : 4u));
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float carry = t.pre[u] + ext;
        if constexpr (FORM == kMfma) {
            const float4v lo = mfma(const_tri_lo<EXCL>(id), t.x[u], splat(carry));
            const float4v hi = mfma(const_tri_hi<EXCL>(id), t.x[u], splat(carry));
            buffer_store_tile_rows_t<F16>(dst, (uint32_t)(kTile * u), id.j, id.g, lo, hi);
        } else {
            float p[8];                           // the in-lane scan is recomputed here rather than kept for a step
            scan8<EXCL>(t.x[u], p);
            buffer_store8_t<F16>(dst, (uint32_t)(kTile * u + 8 * id.lane), (float4v){p[0] + carry, p[1] + carry, p[2] + carry, p[3] + carry},
                                 (float4v){p[4] + carry, p[5] + carry, p[6] + carry, p[7] + carry});
        }
    }
    return fresh;
}

template <int FORM, int U, int WAVES, int MODE, bool IRREG = false>
__global__ __launch_bounds__(WAVES * kWave) void scan_chain_kernel(const _Float16* __restrict__ in,
                                                                   void* __restrict__ out, ChainGrid grid,
                                                                   ScanWorkspace ws_arg, const TileLink* __restrict__ links) {
    static_assert(WAVES <= 16, "");
    const uint32_t tiles = grid.tiles;
    const ScanWorkspace ws = resolve_workspace(ws_arg);
    __shared__ ChainShared sh;
    __shared__ uint32_t s_draw;

    const LaneId id;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // The three start-up draws are spaced out (each follows work on the previous ticket): drawn back to
    // back, workgroup i would hold tiles 3i .. 3i+2 and every workgroup's first tile would wait for
    // aggregates its neighbour publishes two steps later -- the launch would start as a chain of
    // workgroups a step apart.  Spaced out, the first draws of all workgroups come before the second ones.
    if (threadIdx.x == 0)
        s_draw = __hip_atomic_fetch_add(ws.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - ws.ticket_base;
    __syncthreads();
    const uint32_t first = __builtin_amdgcn_readfirstlane(s_draw);
    if (first == 0 && threadIdx.x == 0 && ws.state != nullptr && !ws.device_managed) ws.state[0] = ws.epoch;
    if (first >= tiles) {
        // keeps the number of tickets drawn per launch fixed: three per workgroup plus one per tile
        if (threadIdx.x == 0) {
            __hip_atomic_fetch_add(ws.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_fetch_add(ws.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        return;
    }
    ChainTile<U> a, b, c;
    chain_load<FORM, U, WAVES, IRREG>(a, first, in, grid, id, wave, links);
    __syncthreads();                              // s_draw has been read by everyone
    if (threadIdx.x == 0)
        s_draw = __hip_atomic_fetch_add(ws.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - ws.ticket_base;
    __syncthreads();
    const uint32_t second = __builtin_amdgcn_readfirstlane(s_draw);
    chain_load<FORM, U, WAVES, IRREG>(b, second, in, grid, id, wave, links);
    chain_publish<FORM, U, WAVES, IRREG>(a, ws, tiles, sh, id, wave);          // (its barrier also orders the reads of s_draw)
    if (threadIdx.x == 0)
        s_draw = __hip_atomic_fetch_add(ws.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - ws.ticket_base;
    __syncthreads();
    uint32_t fresh = __builtin_amdgcn_readfirstlane(s_draw);
    // Everything requested so far is waited for here, once: entering the loop with loads pending would make
    // the compiler assume, on every trip, that nothing was issued after them and wait for the stores as well.
    __builtin_amdgcn_s_waitcnt(0x0F70);           // vmcnt(0), other counters untouched

    uint32_t own_end = 0u;
    float own_incl = 0.0f;
    // three tiles per trip, the register sets rotating through the stages, so no tile is ever copied between
    // registers (a copy would have to wait for the loads it copies, and with them for the stores before)
    while (true) {
        chain_load<FORM, U, WAVES, IRREG>(c, fresh, in, grid, id, wave, links);
        chain_publish<FORM, U, WAVES, IRREG>(b, ws, tiles, sh, id, wave);
        fresh = chain_finish<FORM, U, WAVES, MODE, IRREG>(a, out, ws, sh, id, wave, own_end, own_incl, tiles);
        if (b.tile >= tiles) break;
        chain_load<FORM, U, WAVES, IRREG>(a, fresh, in, grid, id, wave, links);
        chain_publish<FORM, U, WAVES, IRREG>(c, ws, tiles, sh, id, wave);
        fresh = chain_finish<FORM, U, WAVES, MODE, IRREG>(b, out, ws, sh, id, wave, own_end, own_incl, tiles);
        if (c.tile >= tiles) break;
        chain_load<FORM, U, WAVES, IRREG>(b, fresh, in, grid, id, wave, links);
        chain_publish<FORM, U, WAVES, IRREG>(a, ws, tiles, sh, id, wave);
        fresh = chain_finish<FORM, U, WAVES, MODE, IRREG>(c, out, ws, sh, id, wave, own_end, own_incl, tiles);
        if (a.tile >= tiles) break;
    }
}

// The last n - n8 (1 .. 7) elements of a one-segment scan whose n is no multiple of 8, after scan_chain_kernel has
// scanned the first n8 = n - n % 8 (the chain's tiles end with whole groups of 8 elements).  One workgroup: the
// sum of everything in front is the sum of the chain's tile totals, which all lie in its descriptor table once it
// has finished (eight reads per thread on their way at a time: the table is uncached); one thread then runs over
// the remaining elements.  MODE as for the chain.
constexpr int kTailThreads = 1024;
template <int MODE>
__global__ __launch_bounds__(kTailThreads) void scan_tail_kernel(const _Float16* __restrict__ in, void* __restrict__ out,
                                                                 uint64_t n8, uint64_t n, ScanWorkspace ws_arg, uint32_t tiles) {
    constexpr int EXCL = MODE & 1, F16 = MODE >> 1;
    __shared__ float s_part[kTailThreads / kWave];
    const ScanWorkspace ws = resolve_workspace(ws_arg);
    float part = 0.0f;
    for (uint32_t t0 = threadIdx.x; t0 < tiles; t0 += 8u * kTailThreads) {
        unsigned long long d[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t t = t0 + (uint32_t)(q * kTailThreads);
            d[q] = load_descriptor(&ws.desc[t < tiles ? t : t0]);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (t0 + (uint32_t)(q * kTailThreads) < tiles) part += __builtin_bit_cast(float, (uint32_t)d[q]);
    }
    part = wave_sum(part);
    if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x >> 6] = part;
    __syncthreads();
    if (threadIdx.x != 0) return;
    float acc = 0.0f;
#pragma unroll
    for (int w = 0; w < kTailThreads / kWave; ++w) acc += s_part[w];
    for (uint64_t k = n8; k < n; ++k) {
        const float x = (float)in[k];
        const float r = EXCL ? acc : acc + x;
        acc += x;
        if constexpr (F16) static_cast<_Float16*>(out)[k] = (_Float16)r;
        else static_cast<float*>(out)[k] = r;
    }
}

// ------------------------------------------------------------------------------ one workgroup per segment, any length
// Segment lengths that are no power of two (the paper pads such segments, Section 4): workgroup s scans
// segment s, whose length is a multiple of 8 and at most WAVES * U tiles.  The tiles are laid out from the
// segment's start, so no tile holds two segments; the part of the workgroup's share beyond the segment's end
// is cut off by the buffer range check -- zero padding that costs no memory traffic.  Matrix cores only.
template <int U, int WAVES, int MODE>
__global__ __launch_bounds__(WAVES * kWave) void scan_segment_kernel(const _Float16* __restrict__ in,
                                                                     void* __restrict__ out, uint64_t seg_len) {
    constexpr int EXCL = MODE & 1, F16 = MODE >> 1;
    constexpr uint32_t kChunk = (uint32_t)kTile * U;
    __shared__ float s_wave_total[WAVES];
    const LaneId id;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint64_t offset = (uint64_t)wave * kChunk;                      // of the wavefront's share inside the segment
    const uint64_t left = offset < seg_len ? seg_len - offset : 0;
    const uint32_t count = left < kChunk ? (uint32_t)left : kChunk;
    const uint64_t base = (uint64_t)blockIdx.x * seg_len + (count ? offset : 0);
    const __amdgpu_buffer_rsrc_t src = make_rsrc(in + base, count * 2u);
    half8 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) x[u] = buffer_load8(src, (uint32_t)(kTile * u + kRow * id.j + 8 * id.g) * 2u);
    float pre[U];
    float run = 0.0f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float4v tot = mfma(const_ones(), x[u], splat(0.0f));
        const float incl = row_scan_inclusive<16>(tot[0], id.j);
        pre[u] = row_shr<1>(incl) + run;
        run += read_lane(incl, 15);
    }
    float ext = 0.0f;
    if constexpr (WAVES > 1) {
        if (id.lane == 0) s_wave_total[wave] = run;
        __syncthreads();
        for (int w = 0; w < wave; ++w) ext += s_wave_total[w];
    }
    const __amdgpu_buffer_rsrc_t dst = make_rsrc(static_cast<char*>(out) + base * (F16 ? 2u : 4u), count * (F16 ? 2u : 4u));
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float carry = pre[u] + ext;
        const float4v lo = mfma(const_tri_lo<EXCL>(id), x[u], splat(carry));
        const float4v hi = mfma(const_tri_hi<EXCL>(id), x[u], splat(carry));
        buffer_store_tile_rows_t<F16>(dst, (uint32_t)(kTile * u), id.j, id.g, lo, hi);
    }
}

// ------------------------------------------------------------------------------ reduce-then-scan helper
// Workgroup s turns the `per` workgroup totals of segment s into exclusive prefixes, in place.
constexpr int kPartialsThreads = 256;
__global__ __launch_bounds__(kPartialsThreads) void scan_partials_kernel(float* __restrict__ totals, uint64_t per) {
    constexpr int kBlockThreads = kPartialsThreads;
    __shared__ float s_wave[kPartialsThreads / kWave];
    float* p = totals + (uint64_t)blockIdx.x * per;
    const uint64_t run_len = (per + kBlockThreads - 1) / kBlockThreads;
    const uint64_t lo = (uint64_t)threadIdx.x * run_len;
    const uint64_t hi = (lo + run_len < per) ? lo + run_len : per;
    float sum = 0.0f;
    for (uint64_t i = lo; i < hi; ++i) sum += p[i];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float incl = wave_scan_inclusive(sum);
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    float carry = wave_shr1(incl);
    for (int w = 0; w < wave; ++w) carry += s_wave[w];
    for (uint64_t i = lo; i < hi; ++i) {
        const float v = p[i];
        p[i] = carry;
        carry += v;
    }
}

// ------------------------------------------------------------------------------ scan-then-propagate helpers
// The paper's device-level scan (Section 5): kernel 1 scans every workgroup share on its own,
// kernel 2 scans the shares' totals, kernel 3 adds the preceding total to every element of a
// share.  gather_totals_kernel reads the totals off the end of each share after kernel 1;
// scan_partials_kernel is kernel 2; uniform_add_kernel is kernel 3.
__global__ __launch_bounds__(256) void gather_totals_kernel(const float* __restrict__ out, float* __restrict__ totals,
                                                            uint64_t share, uint64_t shares, uint64_t n) {
    const uint64_t t = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= shares) return;
    const uint64_t end = ((t + 1) * share < n) ? (t + 1) * share : n;
    totals[t] = out[end - 1];
}

__global__ __launch_bounds__(256) void uniform_add_kernel(float* __restrict__ out, const float* __restrict__ offsets,
                                                          uint64_t share, uint64_t n) {
    // one workgroup per 4096 elements; share is a multiple of 4096
    const uint64_t base = (uint64_t)blockIdx.x * 4096 + (uint64_t)threadIdx.x * 4;
    const float add = offsets[((uint64_t)blockIdx.x * 4096) / share];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const uint64_t off = base + (uint64_t)r * 1024;
        if (off + 4 <= n) {
            float4v v = *reinterpret_cast<float4v*>(out + off);
            v += splat(add);
            *reinterpret_cast<float4v*>(out + off) = v;
        } else {
            for (int e = 0; e < 4; ++e)
                if (off + e < n) out[off + e] += add;
        }
    }
}

}  // namespace tcr
