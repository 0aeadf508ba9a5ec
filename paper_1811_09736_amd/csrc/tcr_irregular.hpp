// Irregular segments given by an offsets array, load-balanced: the work is cut by ELEMENTS, not by
// segments.  A workgroup owns a fixed tile of the flat array whatever the segments look like, so sixteen
// million segments of a few elements, a handful of segments of a hundred million elements and any mix
// of the two all run as the same stream of aligned 128-bit loads and stores.
//
// The paper treats the irregular case by padding the input to regular segments (Section 3, footnote);
// reading the offsets needs no padded copy.  Segment starts inside a tile make the scan operator
// "restart here", which no constant operand matrix expresses (the triangular matrix would have to differ
// from tile row to tile row), so the tile arithmetic is the cross-lane formulation throughout: a lane
// scans its 8 consecutive elements, (flag, value) pairs are combined across lanes with DPP under
//     (fl, vl) . (fr, vr) = (fl | fr,  fr ? vr : vl + vr),
// across a wavefront's sub-tiles in registers and across wavefronts through LDS.  Across tiles the scan
// uses the descriptor chain of the regular scans -- a tile that contains a segment start publishes the
// sum since its last start as a finished prefix at once, because no later tile can need more of it --
// while the reduction, where at most one result per tile depends on earlier tiles, leaves the tiles
// independent and adds that one carry afterwards (two small kernels over the per-tile sums).
//
// What a tile needs from the offsets is found before it starts: irregular_bounds_kernel writes, per
// tile boundary, how many offsets lie below it, so a tile reads its range of entries with one look-up
// instead of searching while its data waits in registers.
#pragma once
#include "tcr_scan.hpp"

namespace tcr {

__device__ __forceinline__ uint32_t wave_shr1_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x138, 0xf, 0xf, true);
}

// One step of the segmented scan: the pair CTRL places to the left (or the identity (0, 0) where the
// DPP pattern delivers nothing) is combined in front of this lane's pair.  CH values may share one flag.
template <int CTRL, int ROW_MASK, bool BOUND, int CH>
__device__ __forceinline__ void seg_combine_left(uint32_t& f, float (&v)[CH]) {
    const uint32_t fl = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)f, CTRL, ROW_MASK, 0xf, BOUND);
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const float vl = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v[c]), CTRL, ROW_MASK, 0xf, BOUND));
        v[c] = f ? v[c] : v[c] + vl;
    }
    f |= fl;
}

// Inclusive segmented scan over the 64 lanes: on return (f, v) of lane l is the combination of the
// pairs of lanes 0 .. l.
template <int CH>
__device__ __forceinline__ void wave_seg_scan_inclusive(uint32_t& f, float (&v)[CH]) {
    seg_combine_left<0x111, 0xf, true>(f, v);
    seg_combine_left<0x112, 0xf, true>(f, v);
    seg_combine_left<0x114, 0xf, true>(f, v);
    seg_combine_left<0x118, 0xf, true>(f, v);
    seg_combine_left<0x142, 0xa, false>(f, v);     // lane 15 of rows 0 and 2 -> rows 1 and 3
    seg_combine_left<0x143, 0xc, false>(f, v);     // lane 31 -> rows 2 and 3
}
__device__ __forceinline__ void wave_seg_scan_inclusive(uint32_t& f, float& v) {
    float one[1] = {v};
    wave_seg_scan_inclusive<1>(f, one);
    v = one[0];
}

// The same scan with the flags as one bit per lane in a scalar register pair: the shifts of the flags are then
// scalar instructions and a step costs the vector unit one cross-lane addition and one select.  Returns the
// inclusive flags (bit l: a flag in lanes 0 .. l).
template <int CH>
__device__ __forceinline__ uint64_t wave_seg_scan_inclusive_bits(uint64_t flags, float (&v)[CH]) {
    auto step = [&](auto ctrl, auto row_mask, auto bound, uint64_t from_left) {
        const bool f = __builtin_amdgcn_inverse_ballot_w64(flags);
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const float vl = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v[c]), decltype(ctrl)::value,
                                                                                   decltype(row_mask)::value, 0xf, decltype(bound)::value));
            v[c] = f ? v[c] : v[c] + vl;
        }
        flags |= from_left;
    };
    using std::integral_constant;
    step(integral_constant<int, 0x111>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{}, (flags << 1) & 0xfffefffefffefffeull);
    step(integral_constant<int, 0x112>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{}, (flags << 2) & 0xfffcfffcfffcfffcull);
    step(integral_constant<int, 0x114>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{}, (flags << 4) & 0xfff0fff0fff0fff0ull);
    step(integral_constant<int, 0x118>{}, integral_constant<int, 0xf>{}, integral_constant<bool, true>{}, (flags << 8) & 0xff00ff00ff00ff00ull);
    // lane 15 of rows 0 and 2 -> every lane of rows 1 and 3; lane 31 -> every lane of rows 2 and 3
    step(integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{}, integral_constant<bool, false>{},
         ((flags >> 15) & 1ull ? 0x00000000ffff0000ull : 0ull) | ((flags >> 47) & 1ull ? 0xffff000000000000ull : 0ull));
    step(integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{}, integral_constant<bool, false>{},
         (flags >> 31) & 1ull ? 0xffffffff00000000ull : 0ull);
    return flags;
}

// What is summed (KIND): 0 the elements, 1 their squares (exact in binary32), 2 both at once, as two
// channels that share the segment starts.
constexpr int kSum = 0, kSquares = 1, kBoth = 2;
template <int KIND>
constexpr int channels() { return KIND == kBoth ? 2 : 1; }
template <int KIND, int C>
__device__ __forceinline__ float term(_Float16 h) {
    const float v = (float)h;
    return (KIND == kSquares || (KIND == kBoth && C == 1)) ? v * v : v;
}

// Running sums (channel C) of a lane's 8 elements that restart at heads, one fused multiply-add per element:
// keep[e] is 0 where element e is a head and 1 elsewhere, so q * keep + x either continues the sum or restarts
// it (products with 0 and 1 are exact, so this rounds like the additions alone).
template <int KIND, int C>
__device__ __forceinline__ void lane_keep_scan(half8 x, half8 keep, float (&p)[8]) {
    float q = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        q = __builtin_fmaf(q, (float)keep[e], term<KIND, C>(x[e]));
        p[e] = q;
    }
}

// Number of entries of the sorted array a[0 .. count) that are smaller than key, found by an aligned group of G
// lanes with G probes per round; every group has a key of its own (the same in all of its lanes), so a round of
// the whole wavefront is one load instruction shared by 64 / G searches.  (A probe is a memory request of its own
// until the last rounds, and requests are what the search costs: 64 probes per round need the fewest rounds and
// the most requests.  32769 boundaries among 16.8 million entries: 25 us with G = 64, 13 with 16, 10 with 8, 11
// with 4.)
template <int G>
__device__ __forceinline__ uint64_t group_lower_bound(const uint64_t* __restrict__ a, uint64_t count, uint64_t key, int lane) {
    static_assert(G >= 2 && G < kWave && (G & (G - 1)) == 0, "");
    const int member = lane & (G - 1), first_lane = lane & ~(G - 1);
    uint64_t lo = 0, hi = count;             // a[i] < key for i < lo;  a[i] >= key for i >= hi
    while (__ballot(lo < hi) != 0) {
        const bool open = lo < hi;
        const uint64_t step = (hi - lo + (uint64_t)(G - 1)) / (uint64_t)G;
        const uint64_t idx = lo + step * (uint64_t)(member + 1) - 1;
        const bool below = open && idx < hi && a[idx] < key;
        const uint64_t c = (uint64_t)__builtin_popcountll((__ballot(below) >> first_lane) & ((1ull << G) - 1ull));
        if (open) {
            const uint64_t first_not_below = lo + step * (c + 1) - 1;                  // member c's probe, if it made one
            hi = first_not_below < hi ? first_not_below : hi;
            lo = lo + step * c;
        }
    }
    return lo;
}

// starts_below[i] = number of entries of offsets[0 .. count) below i * tile_elems, i = 0 .. boundaries - 1;
// ends_below[i] (optional) = the same for i * tile_elems + 1, i.e. with the entries ON the boundary added,
// which turns "segment starts in [begin, end)" into "segment ends in (begin, end]".  kBoundsGroup lanes per boundary.
constexpr int kBoundsWaves = 4;
constexpr int kBoundsGroup = 8;
constexpr int kBoundsPerWave = kWave / kBoundsGroup;
// shift: the tiles are laid out from `shift` elements in front of the array (see irregular_scan_kernel), so
// entry s lies on tile position offsets[s] + shift.
__global__ __launch_bounds__(kBoundsWaves * kWave) void irregular_bounds_kernel(const uint64_t* __restrict__ offsets,
                                                                                uint64_t count, uint64_t tile_elems,
                                                                                uint64_t boundaries, uint32_t shift,
                                                                                uint64_t* __restrict__ starts_below,
                                                                                uint64_t* __restrict__ ends_below,
                                                                                TileLink* __restrict__ links = nullptr) {
    constexpr int G = kBoundsGroup;
    const int lane = threadIdx.x & (kWave - 1);
    const int member = lane & (G - 1), first_lane = lane & ~(G - 1);
    const uint64_t wave_first = ((uint64_t)blockIdx.x * kBoundsWaves + (uint64_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)) * kBoundsPerWave;
    if (wave_first >= boundaries) return;
    // (a group beyond the last boundary repeats the last one's search and writes nothing)
    const uint64_t wanted = wave_first + (uint64_t)(lane / G);
    const bool mine = wanted < boundaries && member == 0;          // this lane writes the group's results
    const uint64_t i = wanted < boundaries ? wanted : boundaries - 1;
    const bool reachable = i * tile_elems >= (uint64_t)shift;       // no entry lies in front of position `shift`
    const uint64_t key = reachable ? i * tile_elems - shift : 0;
    const uint64_t below = group_lower_bound<G>(offsets, count, key, lane);
    if (mine) starts_below[i] = below;
    if (links != nullptr && mine) {
        // the last entry in front of boundary i: the nearest start for tile i, and the last start of tile i - 1
        // if it lies there (boundaries = tiles + 1: tile i exists for i < boundaries - 1)
        // (a tile without a start is covered by a segment iff some entry lies in front of it, but not all of them)
        const int tile_log2 = __builtin_ctzll(tile_elems);        // (every tile size is a power of two)
        const bool any = below > 0;
        const uint64_t at = any ? offsets[below - 1] + shift : 0;
        const uint64_t in_tile = at >> tile_log2;
        if (i + 1 < boundaries) links[i].prev_head_tile = (any && in_tile < i) ? (uint32_t)in_tile : kNoHead;
        if (i >= 1)
            links[i - 1].last_head = (any && in_tile == i - 1) ? (uint32_t)(at - (in_tile << tile_log2))
                                                               : ((any && below < count) ? kNoHead : kOutside);
    }
    if (ends_below == nullptr) return;
    uint64_t on = 0;                          // entries equal to key follow directly
    bool more = reachable;
    while (__ballot(more) != 0) {
        const uint64_t idx = below + on + (uint64_t)member;
        const bool equal = more && idx < count && offsets[idx] == key;
        const int c = __builtin_popcountll((__ballot(equal) >> first_lane) & ((1ull << G) - 1ull));
        if (more) {
            on += (uint64_t)c;
            more = c == G;
        }
    }
    if (mine) ends_below[i] = below + on;
}

// Tile geometry of both kernels: WAVES wavefronts, each with U consecutive 512-element sub-tiles; a lane holds
// elements 8 lane .. 8 lane + 7 of a sub-tile.  Heads are the positions offsets[0 .. nseg]; a bit per head in
// an LDS bitmap tells every lane where its running sums restart.  offsets must be non-decreasing and at
// most n.
//
// Scan: out[k] = running sum of the segment that contains k, offsets[0] <= k < offsets[nseg].
// REGULAR: the heads are the multiples of seg_len instead (offsets and starts_below are not read): regular
// segments of a length no other kernel is tuned for -- odd lengths above all, which leave no 8-element group
// aligned with the segments.  MODE bit 0: exclusive scan; bit 1: binary16 output.
// Arrays that are not 16-byte aligned: `in` and `out` point `shift` (0..7) elements in front of the caller's
// arrays, where `in` is 16-byte aligned, n counts from there and entry s lies on position offsets[s] + shift;
// the elements in front of offsets[0] + shift belong to no segment like any others outside the segments.
// vector_stores == 0: `out` is not 16-byte aligned there and every result is stored on its own.
// SECOND == true: the second kernel of the two-kernel scan of long segments.  scan_chain_kernel has scanned every
// tile without a segment start and published, for EVERY tile, the sum behind its last start; this kernel takes
// the tiles WITH starts.  Nothing is waited for and nothing published: the carry of the elements in front of
// the tile's first start is the sum of the published values from the nearest tile with a start on.
// One tile; `given` is the tile's number for SECOND (otherwise it is drawn by ticket).
template <int U, int WAVES, bool REGULAR, int MODE, bool SECOND>
__device__ __forceinline__ void irregular_scan_tile(const _Float16* __restrict__ in, const uint64_t* __restrict__ offsets,
                                                    void* __restrict__ out, uint64_t n, uint64_t nseg,
                                                    const uint64_t* __restrict__ starts_below, uint64_t seg_len, uint32_t shift,
                                                    uint32_t vector_stores, const ScanWorkspace& ws_arg,
                                                    const TileLink* __restrict__ links, uint32_t given) {
    constexpr int EXCL = MODE & 1, F16 = MODE >> 1;
    constexpr uint32_t kChunk = (uint32_t)kTile * U;          // one wavefront's share
    constexpr uint32_t kBlockTile = kChunk * WAVES;           // one workgroup's share
    __shared__ uint32_t s_heads[kBlockTile / 32];
    __shared__ float s_wave_value[WAVES];
    __shared__ uint32_t s_wave_flag[WAVES];
    __shared__ float s_prefix;
    __shared__ uint32_t s_ready;              // set once s_prefix holds the carry from earlier tiles
    __shared__ uint32_t s_tile;
    __shared__ uint64_t s_bound[2];
    // the eight factors of a lane by the byte of its head bits: binary16 0 where the bit is set, 1 elsewhere
    __shared__ __attribute__((aligned(16))) uint32_t s_factors[256][4];

    const ScanWorkspace ws = resolve_workspace(ws_arg);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // tiles are handed out in launch order, so every predecessor of a waiting tile is running or finished
    if (threadIdx.x == 0) {
        s_ready = 0u;
        const uint32_t t = SECOND ? given
                                  : __hip_atomic_fetch_add(ws.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - ws.ticket_base;
        s_tile = t;
        if constexpr (REGULAR) {
            // heads in [tb, tb + tile) are the multiples head_lo .. head_hi - 1 of seg_len; one thread divides for
            // the whole workgroup (64-bit divisions are long instruction sequences)
            // (entry s lies on position s * seg_len + shift; the tile's range is taken relative to `shift`)
            const uint64_t tile_b = (uint64_t)t * kBlockTile, tile_e = tile_b + kBlockTile;
            const uint64_t b = tile_b > shift ? tile_b - shift : 0, e = tile_e - shift;
            const uint64_t q0 = b / seg_len, q1 = e / seg_len;
            s_bound[0] = q0 + (q0 * seg_len != b ? 1u : 0u);
            s_bound[1] = q1 + (q1 * seg_len != e ? 1u : 0u);
        }
    }
    for (uint32_t i = threadIdx.x; i < kBlockTile / 32; i += WAVES * kWave) s_heads[i] = 0u;
    for (uint32_t b = threadIdx.x; b < 256u; b += WAVES * kWave) {
#pragma unroll
        for (int k = 0; k < 4; ++k)
            s_factors[b][k] = ((b >> (2 * k)) & 1u ? 0u : 0x3c00u) | ((b >> (2 * k + 1)) & 1u ? 0u : 0x3c000000u);
    }
    __syncthreads();
    const uint32_t tile = s_tile;
    if (!SECOND && tile == 0 && threadIdx.x == 0 && ws.state != nullptr && !ws.device_managed) ws.state[0] = ws.epoch;

    const uint64_t tb = (uint64_t)tile * kBlockTile;
    const uint64_t base = tb + (uint64_t)wave * kChunk;
    const bool full = base + kChunk <= n;
    half8 x[U];
    if (full) {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8(in, base + (uint64_t)(kTile * u + 8 * lane));
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8_guarded(in, base + (uint64_t)(kTile * u + 8 * lane), n);
    }
    // everything else that depends on the tile's number alone is asked for now as well: the covered part of the
    // array and, for the second kernel, the running sum at the end of the tile in front (used only if a segment
    // reaches in from there) -- a tile's work is a chain of loads, and these need not be links of it
    const uint64_t first = (REGULAR ? 0 : offsets[0]) + shift;
    const uint64_t last = REGULAR || offsets[nseg] + shift > n ? n : offsets[nseg] + shift;
    float second_pre = 0.0f;
    if constexpr (SECOND) {
        if (wave == 0 && tile != 0u && links[tile].prev_head_tile < tile) {
            const uint32_t tiles = (uint32_t)((n + kBlockTile - 1) / kBlockTile);
            second_pre = __builtin_bit_cast(float, (uint32_t)load_descriptor(&ws.desc[tiles + tile - 1u]));
        }
    }

    // heads in [tb, tb + tile): entries head_lo .. head_hi - 1
    const uint64_t head_lo = REGULAR ? s_bound[0] : starts_below[tile];
    const uint64_t head_hi = REGULAR ? s_bound[1] : starts_below[tile + 1];
    const bool has_heads = head_lo < head_hi;
    if (has_heads) {
        for (uint64_t s = head_lo + threadIdx.x; s < head_hi; s += (uint64_t)(WAVES * kWave)) {
            const uint64_t pos = (REGULAR ? s * seg_len : offsets[s]) + shift - tb;
            if (pos < (uint64_t)kBlockTile) atomicOr(&s_heads[pos >> 5], 1u << (pos & 31u));
        }
        __syncthreads();
    }

    // Running sums inside a lane as fused multiply-adds with the factors (sum * factor + element restarts where
    // the factor is 0): here for the sum behind the lane's last head, below once more from the sum that reaches
    // the lane.  The pairs (head in the lane, that sum) are combined across the lanes with the flags as a lane
    // mask in scalar registers, and across the wavefront's sub-tiles in registers.
    uint32_t bits[U];                             // the lane's head bits (its factors are looked up again for the second pass)
    uint64_t flag_before[U];                      // bit l: a head in a lane in front of lane l inside the sub-tile
    uint32_t seen_before[U];                      // a head in a sub-tile in front
    float lane_value[U], before[U], run = 0.0f;
    uint32_t chunk_flag = 0u;
    const uint8_t* head_bytes = reinterpret_cast<const uint8_t*>(s_heads) + wave * (kChunk / 8);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        bits[u] = has_heads ? (uint32_t)head_bytes[(kTile / 8) * u + lane] : 0u;
        const uint64_t heads_in = __ballot(bits[u] != 0u);
        uint64_t flags = heads_in;
        const half8 keep = *reinterpret_cast<const half8*>(s_factors[bits[u]]);
        float v[1] = {0.0f};
#pragma unroll
        for (int e = 0; e < 8; ++e) v[0] = __builtin_fmaf(v[0], (float)keep[e], (float)x[u][e]);
        flags = wave_seg_scan_inclusive_bits<1>(flags, v);
        flag_before[u] = flags << 1;
        const uint32_t sub_flag = (uint32_t)(flags >> 63);
        seen_before[u] = chunk_flag;
        lane_value[u] = wave_shr1(v[0]);
        const float sub_value = read_lane(v[0], 63);
        before[u] = run;
        run = sub_flag ? sub_value : run + sub_value;
        chunk_flag |= sub_flag;
    }
    if (lane == 0) {
        s_wave_value[wave] = run;
        s_wave_flag[wave] = chunk_flag;
    }
    __syncthreads();

    // carry from the wavefronts in front, back to the nearest one that holds a head
    float ext = 0.0f;
    bool open = true;                         // no head between the tile's start and this wavefront's share
    for (int v = wave - 1; v >= 0; --v) {
        ext += s_wave_value[v];
        if (s_wave_flag[v]) {
            open = false;
            break;
        }
    }
    // the part [valid_lo, valid_hi) of this wavefront's share lies in a segment (all of it, nearly always)
    // (an offsets array that reaches beyond n is the caller's error; nothing is stored beyond n all the same)
    const uint32_t valid_lo = first > base ? (uint32_t)(first - base < kChunk ? first - base : kChunk) : 0u;
    const uint32_t valid_hi = last > base ? (uint32_t)(last - base < kChunk ? last - base : kChunk) : 0u;
    const bool inside = valid_lo == 0u && valid_hi == kChunk && vector_stores != 0u;
    // A wavefront behind a head needs nothing from earlier tiles and goes straight to its stores.  The others
    // wait for the carry that wavefront 0 (always open) looks up -- on a flag in LDS, not at a barrier: a barrier
    // that only some wavefronts of a workgroup execute is outside what the language defines, and one that all
    // execute would hold the closed wavefronts back until the look-up ends (measured: 337 -> 429 us with short
    // segments).  The wait ends: the look-up's own waits are bounded, so wavefront 0 always sets the flag.
    if (open) {
        if (wave == 0) {
            float total = 0.0f;
            bool closed = false;
            for (int v = WAVES - 1; v >= 0; --v) {
                total += s_wave_value[v];
                if (s_wave_flag[v]) {
                    closed = true;
                    break;
                }
            }
            // nothing in front of the tile can reach into it if it starts with a head (or is the first)
            const uint32_t reach = (has_heads && (s_heads[0] & 1u)) ? 0u : tile;
            // 8 descriptors per round: most tiles hold a head and finish their predecessor's wait at distance 1,
            // and chains of open tiles are short with two workgroups per compute unit (measured at n = 2^28:
            // 302 / 340 us for short / long segments with 4-8 per round, 303 / 396 with 1, 323 / 362 with 64)
            float pre = 0.0f;
            if constexpr (SECOND) {
                // the running sum at the end of the tile in front (the chain's second table: tiles .. 2 tiles - 1)
                if (reach != 0u) pre = second_pre;
            } else {
                pre = lookback_carry<8>(ws, tile, reach, closed, total, lane);
            }
            if (lane == 0) {
                s_prefix = pre;
                __hip_atomic_store(&s_ready, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        }
        while (__hip_atomic_load(&s_ready, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0u) __builtin_amdgcn_s_sleep(1);
        ext += s_prefix;
    }
    void* const dst = F16 ? static_cast<void*>(static_cast<_Float16*>(out) + base) : static_cast<void*>(static_cast<float*>(out) + base);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float into_sub = seen_before[u] ? before[u] : before[u] + ext;
        float q = __builtin_amdgcn_inverse_ballot_w64(flag_before[u]) ? lane_value[u] : lane_value[u] + into_sub;
        const half8 keep = *reinterpret_cast<const half8*>(s_factors[bits[u]]);
        float p[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if constexpr (EXCL) {
                p[e] = q * (float)keep[e];
                q = p[e] + (float)x[u][e];
            } else {
                q = __builtin_fmaf(q, (float)keep[e], (float)x[u][e]);
                p[e] = q;
            }
        }
        const uint32_t k = (uint32_t)(kTile * u + 8 * lane);
        if (inside) {
            store8_t<F16>(dst, k, (float4v){p[0], p[1], p[2], p[3]}, (float4v){p[4], p[5], p[6], p[7]});
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (k + e >= valid_lo && k + e < valid_hi) {
                    if constexpr (F16) static_cast<_Float16*>(dst)[k + e] = (_Float16)p[e];
                    else static_cast<float*>(dst)[k + e] = p[e];
                }
            }
        }
    }
}

template <int U, int WAVES, bool REGULAR, int MODE, bool SECOND = false>
__global__ __launch_bounds__(WAVES * kWave) __attribute__((amdgpu_waves_per_eu(SECOND ? 4 : 8, 8)))
void irregular_scan_kernel(const _Float16* __restrict__ in, const uint64_t* __restrict__ offsets, void* __restrict__ out,
                           uint64_t n, uint64_t nseg, const uint64_t* __restrict__ starts_below, uint64_t seg_len,
                           uint32_t shift, uint32_t vector_stores, ScanWorkspace ws_arg, const TileLink* __restrict__ links = nullptr) {
    if constexpr (!SECOND) {
        irregular_scan_tile<U, WAVES, REGULAR, MODE, false>(in, offsets, out, n, nseg, starts_below, seg_len, shift, vector_stores, ws_arg,
                                                            links, 0u);
    } else {
        // Workgroup b looks at tiles b, b + G, b + 2 G, ... (G workgroups, at most 64 tiles each: one per lane) and
        // takes those that hold a segment start -- a handful when segments are long.
        constexpr uint64_t kBlockTile = (uint64_t)kTile * U * WAVES;
        const uint64_t tiles = (n + kBlockTile - 1) / kBlockTile;
        const uint64_t mine = (uint64_t)blockIdx.x + (uint64_t)gridDim.x * (uint64_t)(threadIdx.x & (kWave - 1));
        unsigned long long todo = __ballot(mine < tiles && links[mine < tiles ? mine : 0].last_head < kOutside);
        while (todo != 0ull) {
            const uint32_t bit = (uint32_t)__builtin_ctzll(todo);
            todo &= todo - 1ull;
            irregular_scan_tile<U, WAVES, REGULAR, MODE, true>(in, offsets, out, n, nseg, starts_below, seg_len, shift, vector_stores,
                                                               ws_arg, links, blockIdx.x + gridDim.x * bit);
            __syncthreads();                  // the tile's LDS is free for the next one
        }
    }
}


// Sum of one tile since its last head (all of it if it has none) and whether it has one: the pair that later
// tiles may need of it.
struct TilePair {
    float value;
    uint32_t flag;
};
constexpr uint64_t kNoSegment = ~0ull;

__device__ __forceinline__ uint32_t wave_scan_inclusive_u32(uint32_t x) {
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, true);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);
    x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);
    return x;
}

// Reduction: out[s] = sum of segment s.  Tiles are independent.  While the heads are marked, the position of
// every entry of offsets that falls into the tile is kept in LDS (a tile with more entries than an eighth of its
// elements reads them from memory again), and every element gets a factor: 0 on a head, 1 elsewhere.  A lane's
// running sums are then one fused multiply-add per element (sum * factor + element: the sum restarts where the
// factor is 0), the sums behind the lanes' last heads are combined across the wavefront with the flags as a
// lane mask in scalar registers, and nothing is added to the eight running sums afterwards: a wavefront stages
// them in LDS as they are, next to the 64 sums that reach its lanes from in front, and its lanes walk the
// entries that end a segment inside the sub-tile -- the result is the staged sum plus, unless a head lies
// between the lane's first element and the segment's last, the sum from in front -- so consecutive lanes write
// consecutive results.  The one result per tile that belongs to a segment begun in an earlier tile is written
// without that earlier part; the tile records which segment it is (carried[tile], or none) and its own pair
// (pairs[tile]) for the carry kernels.
// REGULAR: entry s is s * seg_len, s = 0 .. nseg, instead of offsets[s] (offsets and the tables are not read).
// shift: as for irregular_scan_kernel (`in` points that many elements in front of the caller's array).
// KIND: sums of the elements, of their squares, or both (out2 and the pairs of the second channel, which
// follow the first channel's `tiles` pairs, are used for kBoth only).
template <int U, int WAVES, bool REGULAR, int KIND = kSum>
__global__ __launch_bounds__(WAVES * kWave) void irregular_reduce_kernel(const _Float16* __restrict__ in,
                                                                         const uint64_t* __restrict__ offsets,
                                                                         float* __restrict__ out, float* __restrict__ out2,
                                                                         uint64_t n,
                                                                         const uint64_t* __restrict__ starts_below,
                                                                         const uint64_t* __restrict__ ends_below,
                                                                         uint64_t seg_len, uint64_t nseg, uint32_t shift,
                                                                         TilePair* __restrict__ pairs,
                                                                         uint64_t* __restrict__ carried) {
    constexpr uint32_t kChunk = (uint32_t)kTile * U;
    constexpr uint32_t kBlockTile = kChunk * WAVES;
    constexpr int kSubs = U * WAVES;
    static_assert(kSubs <= kWave, "one lane per sub-tile count");
    __shared__ uint32_t s_heads[kBlockTile / 32];
    __shared__ uint32_t s_ends[kSubs];            // segment ends per sub-tile
    // entry head_lo + i lies on element tb + s_position[i + 1]; s_position[0] is no position
    constexpr uint32_t kPositions = kBlockTile / 8 + 62;
    __shared__ uint16_t s_position[kPositions + 2];
    __shared__ uint64_t s_bound[4];
    static_assert(kBlockTile <= 65535u, "positions are kept in 16 bits");
    constexpr int CH = channels<KIND>();
    __shared__ float s_wave_value[CH][WAVES];
    __shared__ uint32_t s_wave_flag[WAVES];
    // Per wavefront: first one binary16 value per element of its share, 0 on a head and 1 elsewhere (the factor
    // that continues or restarts a lane's running sum); later, sub-tile by sub-tile, the running sums of 512
    // elements and the 64 sums that reach the lanes from in front, per channel.
    constexpr uint32_t kStageFloats = (uint32_t)kTile + (uint32_t)kWave;
    constexpr uint32_t kRegionBytes = kChunk * 2u > CH * kStageFloats * 4u ? kChunk * 2u : CH * kStageFloats * 4u;
    __shared__ __attribute__((aligned(16))) unsigned char s_region[WAVES][kRegionBytes];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t tile = blockIdx.x;
    const uint64_t tb = (uint64_t)tile * kBlockTile;
    const uint64_t base = tb + (uint64_t)wave * kChunk;
    const bool full = base + kChunk <= n;
    // which offsets entries fall into the tile: asked for first, so that the entries themselves can be requested
    // while the tile's data is still on its way (the barriers below order LDS only and wait for neither)
    uint64_t head_lo = 0, head_hi = 0, end_lo = 0, end_hi = 0;
    if constexpr (!REGULAR) {
        head_lo = starts_below[tile];
        head_hi = starts_below[tile + 1];
        end_lo = ends_below[tile];
        end_hi = ends_below[tile + 1];
    }
    half8 x[U];
    if (full) {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8<true>(in, base + (uint64_t)(kTile * u + 8 * lane));
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = load8_guarded<true>(in, base + (uint64_t)(kTile * u + 8 * lane), n);
    }
    for (uint32_t i = threadIdx.x; i < kBlockTile / 32; i += WAVES * kWave) s_heads[i] = 0u;
    if (threadIdx.x < kSubs) s_ends[threadIdx.x] = 0u;
    if (threadIdx.x == 0) s_position[0] = 0xffffu;
    half8* const my_keep = reinterpret_cast<half8*>(s_region[wave]);
#pragma unroll
    for (int u = 0; u < U; ++u) my_keep[u * kWave + lane] = splat_half(1.0f);

    // entries [head_lo, head_hi) lie in [tb, tb + tile): heads; entries [end_lo, end_hi) lie in
    // (tb, tb + tile]: each closes the segment in front of it.  head_lo <= end_lo, head_hi <= end_hi.
    if constexpr (REGULAR) {
        // one thread divides for the whole workgroup (64-bit divisions are long instruction sequences)
        if (threadIdx.x == 0) {
            // entry s lies on position s * seg_len + shift: the tile's range relative to `shift` (for the first
            // tile with shift > 0 the values in front are not used: it takes every entry from 0 on)
            const uint64_t b = tb > shift ? tb - shift : 0, e = tb + kBlockTile - shift, entries = nseg + 1;
            const uint64_t q0 = b / seg_len, q1 = e / seg_len;
            const uint64_t h0 = q0 + (q0 * seg_len != b ? 1u : 0u), h1 = q1 + (q1 * seg_len != e ? 1u : 0u);
            s_bound[0] = h0;
            s_bound[1] = h1 < entries ? h1 : entries;
            s_bound[2] = q0 + 1;
            s_bound[3] = q1 + 1 < entries ? q1 + 1 : entries;
        }
    }
    // the first entries of every thread are requested in front of the barrier (a tile of segments of 16 elements
    // has two per thread), so that their way from memory overlaps the data's
    constexpr int kAhead = 2;
    uint64_t ahead[kAhead] = {};
    if constexpr (!REGULAR) {
#pragma unroll
        for (int k = 0; k < kAhead; ++k) {
            const uint64_t s = head_lo + threadIdx.x + (uint64_t)(k * WAVES * kWave);
            if (s < end_hi) ahead[k] = offsets[s];
        }
    }
    lds_barrier();
    if constexpr (REGULAR) {
        head_lo = s_bound[0];
        head_hi = s_bound[1];
        end_lo = s_bound[2];
        end_hi = s_bound[3];
    }
    // (the first tile also takes the entries on position 0, which close empty segments in front of everything)
    if (tile == 0) end_lo = 0;
    const bool has_entries = head_lo < end_hi;
    if (has_entries) {
        // Entry s: its position is kept, its bit and its factor are set, and it counts as a segment end for the
        // sub-tile of the element in front of it.  Consecutive lanes hold consecutive entries, which mostly end
        // segments in the same sub-tile: every run of lanes with the same sub-tile adds its length once (64
        // additions to one LDS word take 64 turns).
        auto mark = [&](uint64_t s, bool valid, uint64_t entry) {
            uint32_t sub = ~0u;
            if (valid) {
                const uint64_t pos = entry + shift - tb;
                if (s - head_lo < (uint64_t)kPositions) s_position[s - head_lo + 1] = (uint16_t)pos;
                if (pos < (uint64_t)kBlockTile) {
                    atomicOr(&s_heads[pos >> 5], 1u << (pos & 31u));
                    reinterpret_cast<_Float16*>(s_region[pos / kChunk])[pos % kChunk] = (_Float16)0.0f;
                }
                if (pos - 1 < (uint64_t)kBlockTile) sub = (uint32_t)(pos - 1) >> 9;
                else if (pos == 0 && tile == 0) sub = 0u;
            }
            const uint32_t left = (uint32_t)__builtin_amdgcn_update_dpp((int)~sub, (int)sub, 0x138, 0xf, 0xf, false);
            const bool first = lane == 0 || left != sub;                       // of a run of equal values
            const uint64_t later = (__ballot(first) >> 1) >> lane;             // bit k: lane + 1 + k starts a run
            const uint32_t length = later ? (uint32_t)__builtin_ctzll(later) + 1u : (uint32_t)(kWave - lane);
            if (first && sub != ~0u) atomicAdd(&s_ends[sub], length);
        };
        // (every wavefront makes whole trips: the lanes of a trip are asked about together)
        uint64_t s0 = head_lo + (uint64_t)(wave * kWave);
#pragma unroll
        for (int k = 0; k < kAhead; ++k, s0 += (uint64_t)(WAVES * kWave))
            if (s0 < end_hi) mark(s0 + lane, s0 + lane < end_hi, REGULAR ? (s0 + lane) * seg_len : ahead[k]);
        for (; s0 < end_hi; s0 += (uint64_t)(WAVES * kWave)) {
            const uint64_t s = s0 + lane;
            mark(s, s < end_hi, REGULAR ? s * seg_len : (s < end_hi ? offsets[s] : 0));
        }
        lds_barrier();
    }
    const bool has_heads = head_lo < head_hi;

    // Running sums inside every lane (restarting at heads, nothing carried in yet), then the pairs
    // (head in the lane, sum behind its last head) combined across the lanes and the wavefront's sub-tiles.
    float p[CH][U][8];
    uint64_t flag_before[U];                      // bit l: a head in a lane in front of lane l inside the sub-tile
    uint32_t seen_before[U];                      // a head in a sub-tile in front
    float lane_value[CH][U], before[CH][U], run[CH];
    uint32_t chunk_flag = 0u;
#pragma unroll
    for (int c = 0; c < CH; ++c) run[c] = 0.0f;
    const uint8_t* head_bytes = reinterpret_cast<const uint8_t*>(s_heads) + wave * (kChunk / 8);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint64_t flags = 0;
        half8 keep = splat_half(1.0f);
        if (has_heads) {
            flags = __ballot(head_bytes[(kTile / 8) * u + lane] != 0);
            keep = my_keep[u * kWave + lane];
        }
        lane_keep_scan<KIND, 0>(x[u], keep, p[0][u]);
        if constexpr (CH == 2) lane_keep_scan<KIND, 1>(x[u], keep, p[CH - 1][u]);
        float v[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) v[c] = p[c][u][7];
        flags = wave_seg_scan_inclusive_bits<CH>(flags, v);
        flag_before[u] = flags << 1;
        const uint32_t sub_flag = (uint32_t)(flags >> 63);
        seen_before[u] = chunk_flag;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            lane_value[c][u] = wave_shr1(v[c]);
            const float sub_value = read_lane(v[c], 63);
            before[c][u] = run[c];
            run[c] = sub_flag ? sub_value : run[c] + sub_value;
        }
        chunk_flag |= sub_flag;
    }
    if (lane == 0) {
#pragma unroll
        for (int c = 0; c < CH; ++c) s_wave_value[c][wave] = run[c];
        s_wave_flag[wave] = chunk_flag;
    }
    lds_barrier();

    if (wave == 0 && lane == 0) {
        float total[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) total[c] = 0.0f;
        uint32_t closed = 0u;
        for (int v = WAVES - 1; v >= 0; --v) {
#pragma unroll
            for (int c = 0; c < CH; ++c) total[c] += s_wave_value[c][v];
            if (s_wave_flag[v]) {
                closed = 1u;
                break;
            }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) pairs[(uint64_t)c * gridDim.x + tile] = TilePair{total[c], closed};
        // the first segment end of the tile closes a segment begun earlier unless an entry sits on tb itself
        carried[tile] = (end_lo < end_hi && end_lo == head_lo && end_lo >= 1) ? end_lo - 1 : kNoSegment;
    }
    if (end_lo == end_hi) return;             // no segment ends here: nothing to write

    float ext[CH];                            // carry from the wavefronts in front, inside this tile only
#pragma unroll
    for (int c = 0; c < CH; ++c) ext[c] = 0.0f;
    for (int v = wave - 1; v >= 0; --v) {
#pragma unroll
        for (int c = 0; c < CH; ++c) ext[c] += s_wave_value[c][v];
        if (s_wave_flag[v]) break;
    }
    // entries that end a segment in each of this wavefront's sub-tiles
    const uint32_t mine = lane < kSubs ? s_ends[lane] : 0u;
    const uint32_t upto = wave_scan_inclusive_u32(mine);
    // (this wavefront has read all of its keep values: the region now stages running sums.  Per channel: a
    // lane's sums 0..3 at 16 bytes per lane, its sums 4..7 likewise in a second plane -- 128-bit stores without
    // bank conflicts -- then the 64 sums that reach the lanes from in front)
    float* const stage = reinterpret_cast<float*>(my_keep);
    // the entries as 32-bit numbers counted from head_lo: entry head_lo + i closes segment head_lo + i - 1
    const bool listed = end_hi - head_lo <= (uint64_t)kPositions;      // every position of the tile is in LDS
    const uint64_t room = nseg >= head_lo ? nseg - head_lo : 0;         // (beyond it: offsets not sorted)
    const uint32_t i_limit = room < 0xfffffffeull ? (uint32_t)room : 0xfffffffeu;
    const uint32_t i_first = head_lo == 0 ? 1u : 0u;                    // offsets[0] closes nothing
    float* const out_from = out + head_lo;                              // (out_from[i - 1] is never touched for head_lo + i == 0)
    float* const out2_from = CH == 2 ? out2 + head_lo : nullptr;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int sub = wave * U + u;
        const uint32_t count = (uint32_t)__builtin_amdgcn_readlane((int)mine, sub);
        if (count == 0u) continue;
        const uint32_t i0 = (uint32_t)(end_lo - head_lo) + ((uint32_t)__builtin_amdgcn_readlane((int)upto, sub) - count);
        // the sub-tile's running sums without what reaches the lane from in front of it, and that sum per lane
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float* const mine_at = stage + c * kStageFloats;
            *reinterpret_cast<float4v*>(mine_at + 4 * lane) = (float4v){p[c][u][0], p[c][u][1], p[c][u][2], p[c][u][3]};
            *reinterpret_cast<float4v*>(mine_at + kTile / 2 + 4 * lane) = (float4v){p[c][u][4], p[c][u][5], p[c][u][6], p[c][u][7]};
            const float into_sub = seen_before[u] ? before[c][u] : before[c][u] + ext[c];
            mine_at[kTile + lane] = __builtin_amdgcn_inverse_ballot_w64(flag_before[u]) ? lane_value[c][u] : lane_value[c][u] + into_sub;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (uint32_t r = (uint32_t)lane; r < count; r += (uint32_t)kWave) {
            const uint32_t i = i0 + r;
            if (i < i_first || i > i_limit) continue;
            // positions of this entry and the one before it (no position if that one lies in front of the tile)
            uint32_t end, begin;
            if (listed) {
                end = s_position[i + 1];
                begin = s_position[i];
            } else {
                const uint64_t s = head_lo + i;
                end = (uint32_t)((REGULAR ? s * seg_len : offsets[s]) + shift - tb);
                begin = i > 0 ? (uint32_t)((REGULAR ? (s - 1) * seg_len : offsets[s - 1]) + shift - tb) : 0xffffu;
            }
            const uint32_t last = end - 1u - (uint32_t)(sub * kTile);   // the segment's last element
            const bool take = end != begin && last < (uint32_t)kTile;   // not an empty segment
            const uint32_t at = last & (uint32_t)(kTile - 1);
            const uint32_t at_lane = at >> 3, e = at & 7u;
            // the sum from in front of the lane belongs to the result unless a head lies between the lane's
            // first element and this one
            const uint32_t heads_upto = (uint32_t)head_bytes[(kTile / 8) * u + at_lane] & ((2u << e) - 1u);
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const float* const mine_at = stage + c * kStageFloats;
                const float from_front = mine_at[kTile + at_lane];
                const float value = mine_at[(e >> 2) * (kTile / 2) + 4 * at_lane + (e & 3u)] + (heads_upto ? 0.0f : from_front);
                (c == 0 ? out_from : out2_from)[(int64_t)i - 1] = take ? value : 0.0f;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// The pairs of 64 consecutive tiles combined into one (one wavefront per group).  blockIdx.y is the channel:
// channel c has its `tiles` pairs behind those of channel c - 1, likewise its groups.
constexpr int kCarryWaves = 4;
__global__ __launch_bounds__(kCarryWaves * kWave) void irregular_groups_kernel(const TilePair* __restrict__ pairs,
                                                                               uint64_t tiles,
                                                                               TilePair* __restrict__ groups) {
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t g = (uint64_t)blockIdx.x * kCarryWaves + (uint64_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (g * kWave >= tiles) return;
    pairs += (uint64_t)blockIdx.y * tiles;
    groups += (uint64_t)blockIdx.y * ((tiles + kWave - 1) / kWave);
    const uint64_t t = g * kWave + (uint64_t)lane;
    TilePair mine = {0.0f, 0u};
    if (t < tiles) mine = pairs[t];
    wave_seg_scan_inclusive(mine.flag, mine.value);
    if (lane == kWave - 1) groups[g] = mine;
}

// Adds to the one carried result of every tile the sum that reaches the tile from the tiles in front of
// it: the groups back to the nearest one with a head, then the tiles of its own group.  Plain loads, fixed
// order: the results do not vary from run to run.  blockIdx.y is the channel (results: out, then out2).
__global__ __launch_bounds__(kCarryWaves * kWave) void irregular_carry_kernel(const TilePair* __restrict__ pairs,
                                                                              const TilePair* __restrict__ groups,
                                                                              const uint64_t* __restrict__ carried,
                                                                              uint64_t tiles, float* __restrict__ out,
                                                                              float* __restrict__ out2) {
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t g = (uint64_t)blockIdx.x * kCarryWaves + (uint64_t)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (g * kWave >= tiles) return;
    pairs += (uint64_t)blockIdx.y * tiles;
    groups += (uint64_t)blockIdx.y * ((tiles + kWave - 1) / kWave);
    if (blockIdx.y) out = out2;
    const uint64_t t = g * kWave + (uint64_t)lane;
    const uint64_t seg = t < tiles ? carried[t] : kNoSegment;
    if (__ballot(seg != kNoSegment) == 0ull) return;
    float into_group = 0.0f;
    for (uint64_t reach = g; reach > 0; reach = reach > (uint64_t)kWave ? reach - kWave : 0) {
        const bool valid = (uint64_t)lane < reach;
        TilePair q = {0.0f, 0u};
        if (valid) q = groups[reach - 1 - (uint64_t)lane];          // lane 0 reads the nearest group
        const unsigned long long closed = __ballot(valid && q.flag != 0u);
        const int nearest = closed != 0ull ? __builtin_ctzll(closed) : kWave;
        into_group += wave_sum((valid && lane <= nearest) ? q.value : 0.0f);
        if (closed != 0ull) break;
    }
    TilePair mine = {0.0f, 0u};
    if (t < tiles) mine = pairs[t];
    wave_seg_scan_inclusive(mine.flag, mine.value);
    const uint32_t flag_before = wave_shr1_u32(mine.flag);
    const float value_before = wave_shr1(mine.value);
    if (seg != kNoSegment) out[seg] += flag_before ? value_before : value_before + into_group;
}

}  // namespace tcr
