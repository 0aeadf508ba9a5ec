// Host side of the library, part 2 of 3 (included by tcr_api.hip only): the dispatch from segment length
// to kernel and launch shape -- the role the paper gives its auto-tuner (Section 6) -- with the tuning
// table that tcr_autotune fills.
#pragma once
#include "tcr_workspace.hpp"

namespace tcr {
namespace host {

// ---------------------------------------------------------------------------- helpers
__global__ void fill_zero_kernel(float* out, uint64_t count) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) out[i] = 0.0f;
}

inline bool is_pow2(uint64_t v) { return v != 0 && (v & (v - 1)) == 0; }
inline int log2u(uint64_t v) {
    int l = 0;
    while ((1ull << l) < v) ++l;
    return l;
}
inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

inline tcr_status check_launch(const char* what) {
    if (hip_failed(hipGetLastError(), what)) return TCR_ERR_HIP;
    return TCR_OK;
}


// ---------------------------------------------------------------------------- tuning table
// The paper selects algorithm, wavefronts per workgroup and coarsening per segment size with an
// auto-tuner (Section 6).  Here the defaults are frozen from sweeps on MI355X; tcr_autotune can
// re-time the candidates on the machine at hand and override the default for one class of
// segment lengths (index log2(seg_len), or kWholeClass for the one-segment operations).
constexpr int kWholeClass = 41;
// One table per kind of choice; an entry is -1 (the frozen default) or  id + 32 * formulation:
//   kTuneScan, kTuneReduce      powers of two from 16 and the one-segment operations, class = log2(seg_len) or
//                               kWholeClass.  id: a launch shape (small segments: kSmallScanShapes /
//                               kSmallReduceShapes; longer: kScanShapes incl. the two multi-kernel carry
//                               strategies / reduce_candidates); formulation 1 forces the cross-lane (DPP)
//                               arithmetic for the class (0: whatever tcr_set_variant says, matrix cores by default).
//   kTuneScanAny, kTuneReduceAny  every other seg_len, class = floor(log2(seg_len)).  id: which kernel takes the
//                               length (see scan_any_candidates / reduce_any_candidates).
//   kTuneIrregular              class 0: tile shape of tcr_irregular_reduce / _moments, class 1: of tcr_irregular_scan.
enum TuneTable { kTuneScan = 0, kTuneReduce = 1, kTuneScanAny = 2, kTuneReduceAny = 3, kTuneIrregular = 4, kTuneTables = 5 };
constexpr const char* kTuneTableNames[kTuneTables] = {"scan", "reduce", "scan_any", "reduce_any", "irregular"};
constexpr int kTuneFormBit = 32;
inline signed char g_tuned[kTuneTables][kWholeClass + 1];
inline bool g_tuning_initialised = false;
inline void init_tuning() {
    if (g_tuning_initialised) return;
    std::memset(g_tuned, -1, sizeof(g_tuned));
    g_tuning_initialised = true;
}
inline int tuning_class(uint64_t seg_len, bool whole) { return whole ? kWholeClass : log2u(seg_len); }
inline int floor_log2(uint64_t v) {
    int l = 0;
    while ((v >> (l + 1)) != 0) ++l;
    return l;
}
// The shape id chosen for a class (-1: none) and the formulation its kernels run.
inline int tuned_id(int table, int cls) {
    init_tuning();
    const int v = g_tuned[table][cls];
    return v < 0 ? -1 : (v & (kTuneFormBit - 1));
}
inline int tuned_formulation(int table, int cls) {
    init_tuning();
    const int v = g_tuned[table][cls];
    return (v >= 0 && (v & kTuneFormBit)) ? kDpp : g_variant.formulation;
}


// ---------------------------------------------------------------------------- reduce dispatch
// Launch shapes of the small-segment kernels (U tiles per wavefront, W wavefronts per workgroup); id 0 is the
// frozen default of each.
struct SmallShape { int u, w; };
constexpr SmallShape kSmallReduceShapes[] = {{kSmallReduceU, kSmallReduceW}, {1, 4}, {1, 8}, {4, 4}};
constexpr SmallShape kSmallScanShapes[] = {{1, kSmallScanW}, {1, 4}, {2, 2}, {2, 4}};
constexpr int kSmallShapeCount = 4;
// reduce_small keeps one result per lane: U * 512 / seg_len <= 64
inline bool small_reduce_shape_valid(int id, int log2l) {
    return id >= 0 && id < kSmallShapeCount && ((kTile >> log2l) * kSmallReduceShapes[id].u <= kWave);
}

template <int FORM, int U, int W>
inline void launch_reduce_small_shape(const _Float16* in, float* out, uint64_t n, int log2l, hipStream_t s) {
    const uint64_t blocks = ceil_div(n, (uint64_t)kTile * U * W);
    const dim3 grid((unsigned)blocks), block(W * kWave);
    switch (log2l) {
        case 4: if constexpr (U <= 2) reduce_small_kernel<FORM, 4, U, W><<<grid, block, 0, s>>>(in, out, n); break;
        case 5: reduce_small_kernel<FORM, 5, U, W><<<grid, block, 0, s>>>(in, out, n); break;
        case 6: reduce_small_kernel<FORM, 6, U, W><<<grid, block, 0, s>>>(in, out, n); break;
        case 7: reduce_small_kernel<FORM, 7, U, W><<<grid, block, 0, s>>>(in, out, n); break;
        case 8: reduce_small_kernel<FORM, 8, U, W><<<grid, block, 0, s>>>(in, out, n); break;
        default: reduce_small_kernel<FORM, 9, U, W><<<grid, block, 0, s>>>(in, out, n); break;
    }
}

template <int FORM>
inline tcr_status launch_reduce_small(const _Float16* in, float* out, uint64_t n, int log2l, hipStream_t s) {
    if (log2l < 4 || log2l > 9) return TCR_ERR_UNSUPPORTED;
    int shape = tuned_id(kTuneReduce, log2l);
    if (!small_reduce_shape_valid(shape, log2l)) shape = 0;
    if (FORM == kMfma && shape == 0 && g_variant.tile_load != kLoadDirect) {
        // the measured alternatives to loading operands directly (default shape only)
        constexpr int U = kSmallReduceU, W = kSmallReduceW;
        const dim3 grid((unsigned)ceil_div(n, (uint64_t)kTile * U * W)), block(W * kWave);
        const bool dma = g_variant.tile_load == kLoadLdsDma;
        switch (log2l) {
#define TCR_CASE(L) case L: if (dma) reduce_small_kernel<kMfma, L, U, W, kLoadLdsDma><<<grid, block, 0, s>>>(in, out, n); \
                            else reduce_small_kernel<kMfma, L, U, W, kLoadStaged><<<grid, block, 0, s>>>(in, out, n); break;
            TCR_CASE(4) TCR_CASE(5) TCR_CASE(6) TCR_CASE(7) TCR_CASE(8) TCR_CASE(9)
#undef TCR_CASE
        }
        return check_launch("reduce_small_kernel");
    }
    switch (shape) {
        case 1: launch_reduce_small_shape<FORM, 1, 4>(in, out, n, log2l, s); break;
        case 2: launch_reduce_small_shape<FORM, 1, 8>(in, out, n, log2l, s); break;
        case 3: launch_reduce_small_shape<FORM, 4, 4>(in, out, n, log2l, s); break;
        default: launch_reduce_small_shape<FORM, kSmallReduceU, kSmallReduceW>(in, out, n, log2l, s); break;
    }
    return check_launch("reduce_small_kernel");
}

template <int FORM>
inline tcr_status launch_reduce_span(const _Float16* in, float* dst, uint64_t n, uint64_t span, uint64_t nspans,
                              int combine_waves, hipStream_t s, const ReduceFinish* finish = nullptr) {
    const ReduceFinish none = {};
    if (finish != nullptr) {          // one partial per workgroup; the last workgroup adds them up
        if (combine_waves == 4) {
            reduce_span_kernel<FORM, 8, 4, true, true><<<dim3((unsigned)ceil_div(nspans, 4)), dim3(4 * kWave), 0, s>>>(
                in, dst, n, span, nspans, *finish);
        } else if (combine_waves == 2) {
            reduce_span_kernel<FORM, 8, 2, true, true><<<dim3((unsigned)ceil_div(nspans, 2)), dim3(2 * kWave), 0, s>>>(
                in, dst, n, span, nspans, *finish);
        } else {
            reduce_span_kernel<FORM, 8, 1, false, true><<<dim3((unsigned)nspans), dim3(kWave), 0, s>>>(in, dst, n, span, nspans,
                                                                                                       *finish);
        }
        return check_launch("reduce_span_kernel");
    }
    if (combine_waves == 4) {
        reduce_span_kernel<FORM, 8, 4, true><<<dim3((unsigned)ceil_div(nspans, 4)), dim3(4 * kWave), 0, s>>>(
            in, dst, n, span, nspans, none);
    } else if (combine_waves == 2) {
        reduce_span_kernel<FORM, 8, 2, true><<<dim3((unsigned)ceil_div(nspans, 2)), dim3(2 * kWave), 0, s>>>(
            in, dst, n, span, nspans, none);
    } else {
        const dim3 grid((unsigned)nspans), block(kWave);
        if (span >= 8 * kTile) reduce_span_kernel<FORM, 8, 1, false><<<grid, block, 0, s>>>(in, dst, n, span, nspans, none);
        else if (span >= 4 * kTile) reduce_span_kernel<FORM, 4, 1, false><<<grid, block, 0, s>>>(in, dst, n, span, nspans, none);
        else reduce_span_kernel<FORM, 2, 1, false><<<grid, block, 0, s>>>(in, dst, n, span, nspans, none);
    }
    return check_launch("reduce_span_kernel");
}

struct ReducePlan {
    uint64_t span;      // elements per wavefront
    int combine;        // wavefronts per workgroup whose sums are added through LDS (1: none)
    uint64_t per;       // partials per segment left for reduce_final_kernel (1: results go straight to out)
    uint64_t nspans;    // wavefronts in total
};


// Reduce candidates for seg_len >= 1024 (power of two) or one segment: (span, combine) pairs.
struct ReduceShape { uint64_t span; int combine; };
inline int reduce_candidates(uint64_t n, uint64_t seg_len, bool whole, ReduceShape* c) {
    int k = 0;
    if (!whole && seg_len <= kWaveSpanMax) {
        c[k++] = {seg_len, 1};                                   // one wavefront per segment
        if (seg_len >= 8192) c[k++] = {seg_len / 2, 2};
        if (seg_len >= 16384) c[k++] = {seg_len / 4, 4};
        return k;
    }
    if (whole) {
        uint64_t span = 4096;
        while (span < kWaveSpanMax && n / span > 4096) span <<= 1;
        if (ceil_div(n, span) == 1) {
            c[k++] = {ceil_div(n, kTile) * kTile, 1};
            return k;
        }
        c[k++] = {span, kReduceBlockW};                          // default
        c[k++] = {span, 1};
        if (span > 16384) c[k++] = {span / 4, kReduceBlockW};
        if (span > 32768) c[k++] = {span / 2, kReduceBlockW};
        return k;
    }
    c[k++] = {kWaveSpanMax, (seg_len / kWaveSpanMax >= (uint64_t)kReduceBlockW) ? kReduceBlockW : 2};   // default
    c[k++] = {kWaveSpanMax, 1};
    c[k++] = {16384, 4};
    c[k++] = {32768, 4};
    return k;
}

// seg_len >= 1024 (a power of two), or one segment of any length (whole).
inline ReducePlan plan_reduce(uint64_t n, uint64_t seg_len, bool whole) {
    ReduceShape cand[4];
    const int count = reduce_candidates(n, seg_len, whole, cand);
    int pick = tuned_id(kTuneReduce, tuning_class(seg_len, whole));
    if (pick < 0 || pick >= count) {
        // frozen defaults: segments of 8192 .. 32768 elements are split over 2 or 4 wavefronts; from 2^18 elements
        // on (and for one segment) every wavefront leaves a partial of its own for the second kernel -- combining
        // the wavefronts of a workgroup first holds each back to the slowest (n = 2^28: 81.5-81.9 us against
        // 83.9-86.1 us with 4 combined; 8 or 16 combined, which make a segment of 2^19 or 2^20 elements one
        // workgroup's and the second kernel unnecessary, 84.1 and 90.8 us)
        if (whole || seg_len >= (1ull << 18)) pick = count > 1 ? 1 : 0;
        else pick = (seg_len < 8192 || seg_len > 32768) ? 0 : (seg_len == 8192 ? 1 : 2);
    }
    ReducePlan p;
    p.span = cand[pick].span;
    p.combine = cand[pick].combine;
    const uint64_t len = whole ? n : seg_len;
    p.per = ceil_div(len, p.span * (uint64_t)p.combine);
    p.nspans = whole ? ceil_div(n, p.span) : n / p.span;
    return p;
}

inline tcr_status reduce_long(const _Float16* in, float* out, uint64_t n, uint64_t seg_len, bool whole, hipStream_t s) {
    const ReducePlan p = plan_reduce(n, seg_len, whole);
    const int form = tuned_formulation(kTuneReduce, tuning_class(seg_len, whole));
    const uint64_t nseg = whole ? 1 : n / seg_len;
    float* dst = out;
    Workspace* ws = nullptr;
    bool capturing = false;
    if (p.per > 1) {
        tcr_status st = get_workspace(s, &ws, &capturing);
        if (st != TCR_OK) return st;
        st = ensure_partials(ws, s, nseg * p.per, capturing);
        if (st != TCR_OK) return st;
        dst = ws->partials;
    }
    if (p.per > 1 && g_variant.reduce_fused && nseg * p.per <= kFusedPartialsMax) {
        // one kernel: the workgroup that finishes last adds up the partials
        if (capturing || ws->device_managed) return TCR_ERR_UNSUPPORTED;     // its count base is a kernel argument
        ScanWorkspace dev = {};
        tcr_status st = begin_lookback(ws, s, 0, &dev, false);   // the running counter that also hands out scan tiles
        if (st != TCR_OK) return st;
        const ReduceFinish fin = {out, dev.ticket, dev.ticket_base, (uint32_t)nseg, (uint32_t)p.per};
        st = form == kMfma ? launch_reduce_span<kMfma>(in, dst, n, p.span, p.nspans, p.combine, s, &fin)
                                            : launch_reduce_span<kDpp>(in, dst, n, p.span, p.nspans, p.combine, s, &fin);
        if (st != TCR_OK) {
            ws->dirty = true;
            return st;
        }
        ws->tickets_issued += (uint32_t)(nseg * p.per);   // one count per workgroup
        return TCR_OK;
    }
    tcr_status st = form == kMfma ? launch_reduce_span<kMfma>(in, dst, n, p.span, p.nspans, p.combine, s)
                                                   : launch_reduce_span<kDpp>(in, dst, n, p.span, p.nspans, p.combine, s);
    if (st != TCR_OK) return st;
    if (p.per > 1) {
        reduce_final_kernel<<<dim3((unsigned)nseg), dim3(kFinalThreads), 0, s>>>(dst, out, p.per);
        st = check_launch("reduce_final_kernel");
    }
    return st;
}


// ---------------------------------------------------------------------------- scan dispatch
// MODE bit 0: exclusive, bit 1: binary16 output (TCR_SCAN_EXCLUSIVE, TCR_OUT_F16).
template <int FORM, int MODE, int U, int W>
inline void launch_scan_small_shape(const _Float16* in, void* out, uint64_t n, int log2l, hipStream_t s) {
    const uint64_t blocks = ceil_div(n, (uint64_t)kTile * U * W);
    const dim3 grid((unsigned)blocks), block(W * kWave);
    switch (log2l) {
        case 4: scan_small_kernel<FORM, 4, U, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
        case 5: scan_small_kernel<FORM, 5, U, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
        case 6: scan_small_kernel<FORM, 6, U, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
        case 7: scan_small_kernel<FORM, 7, U, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
        case 8: scan_small_kernel<FORM, 8, U, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
        default: scan_small_kernel<FORM, 9, U, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
    }
}

template <int FORM, int MODE>
inline tcr_status launch_scan_small(const _Float16* in, void* out, uint64_t n, int log2l, hipStream_t s) {
    if (log2l < 4 || log2l > 9) return TCR_ERR_UNSUPPORTED;
    int shape = tuned_id(kTuneScan, log2l);
    if (shape < 0 || shape >= kSmallShapeCount) shape = 0;
    if constexpr (FORM == kMfma && MODE == 0) {
        if (shape == 0 && g_variant.tile_load != kLoadDirect) {
            // the measured alternatives to loading operands directly (default shape, plain mode only)
            constexpr int W = kSmallScanW;
            const dim3 grid((unsigned)ceil_div(n, (uint64_t)kTile * W)), block(W * kWave);
            const bool dma = g_variant.tile_load == kLoadLdsDma;
            switch (log2l) {
#define TCR_CASE(L) case L: if (dma) scan_small_kernel<kMfma, L, 1, W, 0, kLoadLdsDma><<<grid, block, 0, s>>>(in, out, n); \
                            else scan_small_kernel<kMfma, L, 1, W, 0, kLoadStaged><<<grid, block, 0, s>>>(in, out, n); break;
                TCR_CASE(4) TCR_CASE(5) TCR_CASE(6) TCR_CASE(7) TCR_CASE(8) TCR_CASE(9)
#undef TCR_CASE
            }
            return check_launch("scan_small_kernel");
        }
    }
    switch (shape) {
        case 1: launch_scan_small_shape<FORM, MODE, 1, 4>(in, out, n, log2l, s); break;
        case 2: launch_scan_small_shape<FORM, MODE, 2, 2>(in, out, n, log2l, s); break;
        case 3: launch_scan_small_shape<FORM, MODE, 2, 4>(in, out, n, log2l, s); break;
        default: launch_scan_small_shape<FORM, MODE, 1, kSmallScanW>(in, out, n, log2l, s); break;
    }
    return check_launch("scan_small_kernel");
}

template <int FORM, int U, int W, int CARRY, int MODE>
inline void launch_scan_block(const _Float16* in, void* out, uint64_t n, uint64_t seg_mask, uint64_t seg_len,
                       const ScanWorkspace& dev, const float* prefix, hipStream_t s) {
    const unsigned blocks = (unsigned)ceil_div(n, (uint64_t)kTile * U * W);
    scan_block_kernel<FORM, U, W, CARRY, MODE><<<dim3(blocks), dim3(W * kWave), 0, s>>>(
        in, out, n, seg_mask, seg_len, dev, prefix);
}

// Launch shapes of scan_block_kernel.  Ids 0..6 take tiles in blockIdx order and need a whole
// segment inside one workgroup share; ids 7..9 hand tiles out by ticket (tiles are then processed
// in the order workgroups actually start, which keeps the tiles in flight contiguous in memory and
// measured 5-9 % faster for 1024-thread workgroups even without a carry) and chain workgroups
// through the look-back when a segment is longer than the share.  One ticket costs about 12 ns of
// a chip-wide serial resource, so ticketed shares start at 16384 elements.
// Ids 10 and 11 are scan_chain_kernel: persistent workgroups (one per compute unit) that take
// 32768-element tiles by ticket in a loop and keep three in flight (loading, aggregate published,
// carry looked up and stored); for segments of at least one tile and the one-segment scan,
// matrix-core formulation only, n a multiple of 8.
struct ScanShape { int u, w; bool ticket; int persistent; };      // persistent: workgroups per compute unit (0: one per tile)
constexpr ScanShape kScanShapes[] = {{1, 2, false, 0}, {1, 4, false, 0}, {1, 8, false, 0}, {1, 16, false, 0},
                                     {2, 16, false, 0}, {4, 16, false, 0}, {8, 16, false, 0}, {2, 16, true, 0},
                                     {4, 16, true, 0}, {8, 16, true, 0}, {4, 16, true, 1}, {8, 8, true, 1}};
constexpr int kScanShapeCount = 12;
// Two more ids choose a multi-kernel carry strategy instead of a single-pass shape (segments longer than one
// 65536-element share only): the paper's three-kernel scan-then-propagate (Section 5) and reduce-then-scan.
// (14: one segment whose n is no multiple of 8 -- the chain over the whole groups of 8, then scan_tail_kernel)
constexpr int kScanIdReduceThenScan = 12, kScanIdScanThenPropagate = 13, kScanIdChainTail = 14, kScanIdCount = 15;
inline uint64_t scan_shape_tile(int id) { return (uint64_t)kTile * kScanShapes[id].u * kScanShapes[id].w; }

inline bool scan_shape_valid(int id, uint64_t len, bool whole) {      // len: seg_len, or n for the one-segment scan
    if (id == kScanIdReduceThenScan || id == kScanIdScanThenPropagate) return len > kCarryTile;
    if (id == kScanIdChainTail) return whole && len % 8 != 0 && len >= 2 * scan_shape_tile(10) && g_variant.scan_carry == kStrategyLookback;
    if (id < 0 || id >= kScanShapeCount) return false;
    if (kScanShapes[id].persistent)                             // (whole: len == n, which must be a multiple of 8)
        return whole ? len % 8 == 0 : len >= scan_shape_tile(id);
    return kScanShapes[id].ticket || scan_shape_tile(id) >= len;
}

// Compute units of the current device (cached per device id).
inline int compute_units() {
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int cu = 0;
        if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0) cu = 256;
        cached[dev] = cu;
    }
    return cached[dev];
}

inline int default_scan_shape(uint64_t len, bool whole, int form) {
    if (len <= 1024) return 0;
    if (len <= 2048) return 1;
    if (len <= 4096) return 2;
    if (len < 8192 || (whole && len == 8192)) return 3;
    if (!whole && len <= 16384) return 7;          // one ticketed share per segment (two segments of 8192)
    // the pipelined chain: segments of 32768 and more, one segment with n % 8 == 0.  (16 wavefronts of 4 tiles
    // for the matrix cores; the DPP arithmetic needs more registers and takes 8 wavefronts of 8 tiles.)
    if (scan_shape_valid(10, len, whole)) return form == kMfma ? 10 : 11;
    // n not a multiple of 8: the chain over the whole groups of 8 and a second, tiny kernel for the rest (measured
    // at n = 2^28 - 3: 297 us against 307-323 us for scan_block_kernel with decoupled look-back, which short arrays keep)
    if (scan_shape_valid(kScanIdChainTail, len, whole)) return kScanIdChainTail;
    return (whole || len >= (1u << 20)) ? 9 : 8;
}

inline int pick_scan_shape(uint64_t len, bool whole) {
    const int cls = tuning_class(len, whole);
    const int tuned = tuned_id(kTuneScan, cls);
    return scan_shape_valid(tuned, len, whole) ? tuned : default_scan_shape(len, whole, tuned_formulation(kTuneScan, cls));
}

template <int FORM, int CARRY, int MODE>
inline void launch_scan_shape(int id, const _Float16* in, void* out, uint64_t n, uint64_t seg_mask, uint64_t seg_len,
                       const ScanWorkspace& dev, const float* prefix, hipStream_t s) {
    // CARRY is kNoCarry for ids 0..6 and kLookback for ids 7..9
    if constexpr (CARRY == kNoCarry) {
        switch (id) {
            case 0: launch_scan_block<FORM, 1, 2, kNoCarry, MODE>(in, out, n, seg_mask, seg_len, dev, prefix, s); break;
            case 1: launch_scan_block<FORM, 1, 4, kNoCarry, MODE>(in, out, n, seg_mask, seg_len, dev, prefix, s); break;
            case 2: launch_scan_block<FORM, 1, 8, kNoCarry, MODE>(in, out, n, seg_mask, seg_len, dev, prefix, s); break;
            case 3: launch_scan_block<FORM, 1, 16, kNoCarry, MODE>(in, out, n, seg_mask, seg_len, dev, prefix, s); break;
            case 4: launch_scan_block<FORM, 2, 16, kNoCarry, MODE>(in, out, n, seg_mask, seg_len, dev, prefix, s); break;
            case 5: launch_scan_block<FORM, 4, 16, kNoCarry, MODE>(in, out, n, seg_mask, seg_len, dev, prefix, s); break;
            default: launch_scan_block<FORM, 8, 16, kNoCarry, MODE>(in, out, n, seg_mask, seg_len, dev, prefix, s); break;
        }
    } else {
        switch (id) {
            case 7: launch_scan_block<FORM, 2, 16, kLookback, MODE>(in, out, n, seg_mask, seg_len, dev, prefix, s); break;
            case 8: launch_scan_block<FORM, 4, 16, kLookback, MODE>(in, out, n, seg_mask, seg_len, dev, prefix, s); break;
            default: launch_scan_block<FORM, 8, 16, kLookback, MODE>(in, out, n, seg_mask, seg_len, dev, prefix, s); break;
        }
    }
}

// Smallest blockIdx-ordered shape that holds `fit` elements (used by the multi-kernel strategies).
inline int nocarry_shape_for(uint64_t fit) {
    for (int id = 0; id < 7; ++id)
        if (scan_shape_tile(id) >= fit) return id;
    return 6;
}

// The persistent chain (shape 10 or 11) over segments of `seg_len` elements: any multiple of 8 that is at
// least one tile, or one segment of n elements (n a multiple of 8).
template <int FORM, int MODE>
tcr_status launch_chain(int shape, const _Float16* in, void* out, uint64_t n, uint64_t seg_len, hipStream_t s,
                        ScanWorkspace* used = nullptr, uint32_t* used_tiles = nullptr) {
    const uint64_t tile = scan_shape_tile(shape);
    const uint64_t per_segment = ceil_div(seg_len, tile);
    const uint64_t tiles = (n / seg_len) * per_segment;
    ScanWorkspace dev = {};
    Workspace* ws = nullptr;
    bool capturing = false;
    tcr_status st = get_workspace(s, &ws, &capturing);
    if (st != TCR_OK) return st;
    st = begin_lookback(ws, s, tiles, &dev, capturing);
    if (st != TCR_OK) return st;
    const uint64_t resident = (uint64_t)compute_units() * (uint64_t)kScanShapes[shape].persistent;
    const uint64_t groups = tiles < resident ? tiles : resident;
    const ChainGrid grid = {seg_len, (uint32_t)per_segment, (uint32_t)tiles};
    if (shape == 10) scan_chain_kernel<FORM, 4, 16, MODE><<<dim3((unsigned)groups), dim3(16 * kWave), 0, s>>>(in, out, grid, dev, nullptr);
    else scan_chain_kernel<FORM, 8, 8, MODE><<<dim3((unsigned)groups), dim3(8 * kWave), 0, s>>>(in, out, grid, dev, nullptr);
    st = check_launch("scan_chain_kernel");
    if (st != TCR_OK) {
        ws->dirty = true;
        return st;
    }
    ws->tickets_issued += (uint32_t)(tiles + 3 * groups);   // three drawn at the start of every workgroup, one per tile
    if (used != nullptr) *used = dev;
    if (used_tiles != nullptr) *used_tiles = (uint32_t)tiles;
    return TCR_OK;
}

// One segment of n elements, n no multiple of 8: the chain over the first n - n % 8, then the rest.
template <int FORM, int MODE>
tcr_status launch_chain_tail(const _Float16* in, void* out, uint64_t n, hipStream_t s) {
    const uint64_t n8 = n & ~7ull;
    ScanWorkspace dev = {};
    uint32_t tiles = 0;
    tcr_status st = launch_chain<FORM, MODE>(FORM == kMfma ? 10 : 11, in, out, n8, n8, s, &dev, &tiles);
    if (st != TCR_OK) return st;
    scan_tail_kernel<MODE><<<dim3(1), dim3(kTailThreads), 0, s>>>(in, out, n8, n, dev, tiles);
    return check_launch("scan_tail_kernel");
}

// seg_len >= 1024 (power of two), or the full scan (seg_len == n, any n).
template <int FORM, int MODE>
inline tcr_status scan_long(const _Float16* in, void* out, uint64_t n, uint64_t seg_len, bool whole, hipStream_t s) {
    const uint64_t seg_mask = whole ? ~0ull : seg_len - 1;
    const uint64_t host_seg_len = seg_len;            // decides the launch; the kernels see a saturated
    if (whole) seg_len = ~0ull;                       // length for the one-segment case (n need not be a power of two)
    // the carry strategy: forced by tcr_set_variant, else the class's tuned choice, else the single pass
    int strategy = g_variant.scan_carry;
    int shape = strategy == kStrategyLookback ? pick_scan_shape(host_seg_len, whole) : -1;
    if (shape == kScanIdReduceThenScan) strategy = kStrategyReduceThenScan;
    if (shape == kScanIdScanThenPropagate) strategy = MODE == 0 ? kStrategyScanThenPropagate : kStrategyLookback;
    if (shape == kScanIdChainTail) return launch_chain_tail<FORM, MODE>(in, out, n, s);
    if (shape >= kScanShapeCount) shape = default_scan_shape(host_seg_len, whole, FORM);    // (the strategies have fixed shapes)
    if (shape == kScanIdChainTail) shape = 9;             // (a forced multi-kernel strategy: its no-carry shares do not use it)
    const bool table = strategy != kStrategyLookback;     // the two multi-kernel strategies
    if (table && host_seg_len <= kCarryTile) {
        const ScanWorkspace none = {};
        launch_scan_shape<FORM, kNoCarry, MODE>(nocarry_shape_for(host_seg_len), in, out, n, seg_mask, seg_len, none, nullptr, s);
        return check_launch("scan_block_kernel");
    }
    if (!table) {
        if (!kScanShapes[shape].ticket) {
            const ScanWorkspace none = {};
            launch_scan_shape<FORM, kNoCarry, MODE>(shape, in, out, n, seg_mask, seg_len, none, nullptr, s);
            return check_launch("scan_block_kernel");
        }
        if (kScanShapes[shape].persistent) return launch_chain<FORM, MODE>(shape, in, out, n, host_seg_len, s);
        const uint64_t tiles = ceil_div(n, scan_shape_tile(shape));
        ScanWorkspace dev = {};
        Workspace* ws = nullptr;
        bool capturing = false;
        tcr_status st = get_workspace(s, &ws, &capturing);
        if (st != TCR_OK) return st;
        st = begin_lookback(ws, s, tiles, &dev, capturing);
        if (st != TCR_OK) return st;
        launch_scan_shape<FORM, kLookback, MODE>(shape, in, out, n, seg_mask, seg_len, dev, nullptr, s);
        st = check_launch("scan_block_kernel");
        if (st != TCR_OK) {
            ws->dirty = true;
            return st;
        }
        ws->tickets_issued += (uint32_t)tiles;      // one per workgroup; wraps modulo 2^32 like the device counter
        return TCR_OK;
    }
    if (strategy == kStrategyScanThenPropagate) {
        // the paper's three kernels; totals are read back from the binary32 inclusive output
        if (MODE != 0) return TCR_ERR_UNSUPPORTED;
        const uint64_t shares = ceil_div(n, kCarryTile);
        Workspace* w = nullptr;
        bool capturing = false;
        tcr_status st = get_workspace(s, &w, &capturing);
        if (st != TCR_OK) return st;
        st = ensure_partials(w, s, shares, capturing);
        if (st != TCR_OK) return st;
        const ScanWorkspace none = {};
        float* o = static_cast<float*>(out);
        launch_scan_block<FORM, kCarryU, kCarryW, kNoCarry, 0>(in, out, n, kCarryTile - 1, kCarryTile, none, nullptr, s);
        st = check_launch("scan_block_kernel");
        if (st != TCR_OK) return st;
        gather_totals_kernel<<<dim3((unsigned)ceil_div(shares, 256)), dim3(256), 0, s>>>(o, w->partials, kCarryTile, shares, n);
        st = check_launch("gather_totals_kernel");
        if (st != TCR_OK) return st;
        const uint64_t per = whole ? shares : host_seg_len / kCarryTile;
        scan_partials_kernel<<<dim3((unsigned)(whole ? 1 : n / host_seg_len)), dim3(kPartialsThreads), 0, s>>>(w->partials, per);
        st = check_launch("scan_partials_kernel");
        if (st != TCR_OK) return st;
        uniform_add_kernel<<<dim3((unsigned)ceil_div(n, 4096)), dim3(256), 0, s>>>(o, w->partials, kCarryTile, n);
        return check_launch("uniform_add_kernel");
    }
    const uint64_t tiles = ceil_div(n, kCarryTile);
    ScanWorkspace dev = {};
    Workspace* ws = nullptr;
    bool capturing = false;
    tcr_status st = get_workspace(s, &ws, &capturing);
    if (st != TCR_OK) return st;
    // reduce-then-scan: workgroup totals, their exclusive scan per segment, then the scan proper
    st = ensure_partials(ws, s, tiles, capturing);
    if (st != TCR_OK) return st;
    // one wavefront span per workgroup tile; spans are uniform because seg_len is a multiple of the tile (or one segment)
    st = launch_reduce_span<FORM>(in, ws->partials, n, kCarryTile, tiles, 1, s);
    if (st != TCR_OK) return st;
    const uint64_t per = whole ? tiles : host_seg_len / kCarryTile;
    const uint64_t groups = whole ? 1 : n / host_seg_len;
    scan_partials_kernel<<<dim3((unsigned)groups), dim3(kPartialsThreads), 0, s>>>(ws->partials, per);
    st = check_launch("scan_partials_kernel");
    if (st != TCR_OK) return st;
    launch_scan_block<FORM, kCarryU, kCarryW, kTable, MODE>(in, out, n, seg_mask, seg_len, dev, ws->partials, s);
    return check_launch("scan_block_kernel");
}

// Irregular segments: fixed tiles of the flat array, whatever the segments.  Tile shapes (U sub-tiles of 512
// elements per wavefront, W wavefronts); id 0 is the frozen default: 32768-element tiles for the chained scan,
// 8192-element tiles of four wavefronts for the reduction, whose tiles are independent (measured at n = 2^28:
// 90 us against 92 us with eight wavefronts of four sub-tiles on log-normal lengths, 143 against 153 us on
// segments of 16 elements on average: a tile's work is a chain of dependent steps -- its range of offsets
// entries, the entries, the marks, the sums -- and small workgroups keep more tiles in flight per compute unit).
constexpr SmallShape kIrregularScanShapes[] = {{4, 16}, {2, 16}};
constexpr SmallShape kIrregularReduceShapes[] = {{4, 4}, {4, 8}, {2, 8}};
constexpr int kIrregularScanShapeCount = 2, kIrregularReduceShapeCount = 3;
inline int irregular_shape(bool scan) {
    const int id = tuned_id(kTuneIrregular, scan ? 1 : 0);
    return (id >= 0 && id < (scan ? kIrregularScanShapeCount : kIrregularReduceShapeCount)) ? id : 0;
}
inline uint64_t irregular_tile_elems(bool scan, int shape) {
    const SmallShape t = scan ? kIrregularScanShapes[shape] : kIrregularReduceShapes[shape];
    return (uint64_t)kTile * t.u * t.w;
}
inline uint64_t irregular_tiles(bool scan, uint64_t n, int shape) { return ceil_div(n, irregular_tile_elems(scan, shape)); }
// 8-byte words of the partials area: the look-up table(s) of the tile boundaries, and for the reduction one
// carried-segment index and one pair per tile and one pair per group of 64 tiles.
inline uint64_t irregular_words(bool scan, uint64_t n, int shape) {
    const uint64_t tiles = irregular_tiles(scan, n, shape);
    // (scan: the look-up table and one TileLink per tile)
    return scan ? 2 * tiles + 1 : 2 * (tiles + 1) + 2 * tiles + ceil_div(tiles, kWave);
}
// The largest of these over the tile shapes (the smallest tiles): what tcr_workspace_bytes reports.
inline uint64_t irregular_tiles_max(bool scan, uint64_t n) {
    uint64_t m = 0;
    for (int id = 0; id < (scan ? kIrregularScanShapeCount : kIrregularReduceShapeCount); ++id)
        if (irregular_tiles(scan, n, id) > m) m = irregular_tiles(scan, n, id);
    return m;
}
inline uint64_t irregular_words_max(bool scan, uint64_t n) {
    uint64_t m = 0;
    for (int id = 0; id < (scan ? kIrregularScanShapeCount : kIrregularReduceShapeCount); ++id)
        if (irregular_words(scan, n, id) > m) m = irregular_words(scan, n, id);
    return m;
}

// The tiles start at the 16-byte boundary at or below `in`: `shift` elements in front of it (0 for aligned arrays).
inline uint32_t alignment_shift(const _Float16* in) { return (uint32_t)((reinterpret_cast<uintptr_t>(in) & 15u) / 2u); }

// offsets == nullptr: regular segments of seg_len elements (no look-up table; MODE as for the other scans).
// in: 2-byte aligned; out: aligned to its element size.  shape: an id of kIrregularScanShapes.
template <int MODE, int U, int W>
inline void launch_irregular_scan_shape(bool regular, const _Float16* in, const uint64_t* offsets, void* out, uint64_t n, uint64_t nseg,
                                        const uint64_t* starts, uint64_t seg_len, uint32_t shift, uint32_t vector_stores,
                                        const ScanWorkspace& dev, uint64_t tiles, hipStream_t s) {
    const dim3 grid((unsigned)tiles), block(W * kWave);
    if (regular) irregular_scan_kernel<U, W, true, MODE><<<grid, block, 0, s>>>(in, nullptr, out, n, nseg, nullptr, seg_len, shift, vector_stores, dev);
    else irregular_scan_kernel<U, W, false, MODE><<<grid, block, 0, s>>>(in, offsets, out, n, nseg, starts, 0, shift, vector_stores, dev);
}

template <int MODE>
inline tcr_status launch_irregular_scan(const _Float16* in, const uint64_t* offsets, void* out, uint64_t n, uint64_t nseg,
                                        uint64_t seg_len, hipStream_t s, int shape = -1) {
    if (shape < 0) shape = irregular_shape(true);
    const uint64_t elems = irregular_tile_elems(true, shape);
    const uint32_t shift = alignment_shift(in);
    in -= shift;
    out = static_cast<char*>(out) - (size_t)shift * ((MODE & 2) ? 2 : 4);
    n += shift;
    const uint32_t vector_stores = aligned(out, 16) ? 1u : 0u;
    const uint64_t tiles = irregular_tiles(true, n, shape);
    const bool regular = offsets == nullptr;
    Workspace* ws = nullptr;
    bool capturing = false;
    tcr_status st = get_workspace(s, &ws, &capturing);
    if (st != TCR_OK) return st;
    if (!regular) {
        st = ensure_partials(ws, s, 2 * irregular_words(true, n, shape), capturing);
        if (st != TCR_OK) return st;
    }
    // Long segments -- fewer segments than a quarter of the tiles, so most tiles hold no segment start: the
    // pipelined chain scans the tiles without a start, a second kernel the others.  (Default tile shape, 16-byte
    // aligned arrays.)
    const bool two_kernels = !regular && shape == 0 && shift == 0 && vector_stores != 0 && g_variant.formulation == kMfma &&
                             g_variant.irregular_scan != 1 && (g_variant.irregular_scan == 2 || nseg <= tiles / 4);
    ScanWorkspace dev = {};
    st = begin_lookback(ws, s, two_kernels ? 2 * tiles : tiles, &dev, capturing);      // (two kernels: a second table behind the first)
    if (st != TCR_OK) return st;
    uint64_t* starts = reinterpret_cast<uint64_t*>(ws->partials);
    TileLink* links = reinterpret_cast<TileLink*>(starts + (tiles + 1));
    if (!regular) {
        irregular_bounds_kernel<<<dim3((unsigned)ceil_div(tiles + 1, kBoundsWaves * kBoundsPerWave)), dim3(kBoundsWaves * kWave), 0, s>>>(
            offsets, nseg + 1, elems, tiles + 1, shift, starts, nullptr, two_kernels ? links : nullptr);
        st = check_launch("irregular_bounds_kernel");
        if (st != TCR_OK) return st;
    }
    if (two_kernels) {
        const uint64_t resident = (uint64_t)compute_units();
        const uint64_t groups = tiles < resident ? tiles : resident;
        scan_chain_kernel<kMfma, 4, 16, MODE, true><<<dim3((unsigned)groups), dim3(16 * kWave), 0, s>>>(
            in, out, ChainGrid{n, (uint32_t)tiles, (uint32_t)tiles}, dev, links);
        st = check_launch("scan_chain_kernel");
        if (st != TCR_OK) {
            ws->dirty = true;
            return st;
        }
        ws->tickets_issued += (uint32_t)(tiles + 3 * groups);
        // (every workgroup of the second kernel looks at up to 64 tiles)
        const uint64_t second = ceil_div(tiles, kWave) > resident ? ceil_div(tiles, kWave) : (tiles < resident ? tiles : resident);
        irregular_scan_kernel<4, 16, false, MODE, true><<<dim3((unsigned)second), dim3(16 * kWave), 0, s>>>(
            in, offsets, out, n, nseg, starts, 0, shift, vector_stores, dev, links);
        return check_launch("irregular_scan_kernel");
    }
    if (shape == 1) launch_irregular_scan_shape<MODE, 2, 16>(regular, in, offsets, out, n, nseg, starts, seg_len, shift, vector_stores, dev, tiles, s);
    else launch_irregular_scan_shape<MODE, 4, 16>(regular, in, offsets, out, n, nseg, starts, seg_len, shift, vector_stores, dev, tiles, s);
    st = check_launch("irregular_scan_kernel");
    if (st != TCR_OK) {
        ws->dirty = true;
        return st;
    }
    ws->tickets_issued += (uint32_t)tiles;
    return TCR_OK;
}

// offsets == nullptr: regular segments of seg_len elements (no look-up tables).
// kind: kSum, kSquares (regular segments only), or kBoth with the sums of squares in out2.  shape: an id of
// kIrregularReduceShapes.
template <int U, int W>
inline void launch_irregular_reduce_shape(bool regular, int kind, const _Float16* in, const uint64_t* offsets, float* out, float* out2,
                                          uint64_t n, const uint64_t* starts, const uint64_t* ends, uint64_t seg_len, uint64_t nseg,
                                          uint32_t shift, TilePair* pairs, uint64_t* carried, uint64_t tiles, hipStream_t s) {
    const dim3 grid((unsigned)tiles), block(W * kWave);
    if (regular) {
        if (kind == kBoth) irregular_reduce_kernel<U, W, true, kBoth><<<grid, block, 0, s>>>(in, nullptr, out, out2, n, nullptr, nullptr, seg_len, nseg, shift, pairs, carried);
        else if (kind == kSquares) irregular_reduce_kernel<U, W, true, kSquares><<<grid, block, 0, s>>>(in, nullptr, out, out2, n, nullptr, nullptr, seg_len, nseg, shift, pairs, carried);
        else irregular_reduce_kernel<U, W, true, kSum><<<grid, block, 0, s>>>(in, nullptr, out, out2, n, nullptr, nullptr, seg_len, nseg, shift, pairs, carried);
    } else {
        if (kind == kBoth) irregular_reduce_kernel<U, W, false, kBoth><<<grid, block, 0, s>>>(in, offsets, out, out2, n, starts, ends, 0, nseg, shift, pairs, carried);
        else irregular_reduce_kernel<U, W, false, kSum><<<grid, block, 0, s>>>(in, offsets, out, nullptr, n, starts, ends, 0, nseg, shift, pairs, carried);
    }
}

inline tcr_status launch_irregular_reduce(const _Float16* in, const uint64_t* offsets, float* out, uint64_t n, uint64_t nseg,
                                          uint64_t seg_len, hipStream_t s, int kind = kSum, float* out2 = nullptr, int shape = -1) {
    if (shape < 0) shape = irregular_shape(false);
    const uint64_t elems = irregular_tile_elems(false, shape);
    const uint32_t shift = alignment_shift(in);
    in -= shift;
    n += shift;
    const uint64_t tiles = irregular_tiles(false, n, shape);
    const uint64_t groups = ceil_div(tiles, kWave);
    const bool regular = offsets == nullptr;
    const unsigned ch = kind == kBoth ? 2u : 1u;
    Workspace* ws = nullptr;
    bool capturing = false;
    tcr_status st = get_workspace(s, &ws, &capturing);
    if (st != TCR_OK) return st;
    st = ensure_partials(ws, s, 2 * (irregular_words(false, n, shape) + (ch - 1) * (tiles + groups)), capturing);
    if (st != TCR_OK) return st;
    uint64_t* starts = reinterpret_cast<uint64_t*>(ws->partials);
    uint64_t* ends = starts + (tiles + 1);
    uint64_t* carried = ends + (tiles + 1);
    TilePair* pairs = reinterpret_cast<TilePair*>(carried + tiles);              // ch * tiles
    TilePair* group_pairs = pairs + ch * tiles;                                   // ch * groups
    if (!regular) {
        irregular_bounds_kernel<<<dim3((unsigned)ceil_div(tiles + 1, kBoundsWaves * kBoundsPerWave)), dim3(kBoundsWaves * kWave), 0, s>>>(
            offsets, nseg + 1, elems, tiles + 1, shift, starts, ends);
        st = check_launch("irregular_bounds_kernel");
        if (st != TCR_OK) return st;
    }
    if (shape == 1) launch_irregular_reduce_shape<4, 8>(regular, kind, in, offsets, out, out2, n, starts, ends, seg_len, nseg, shift, pairs, carried, tiles, s);
    else if (shape == 2) launch_irregular_reduce_shape<2, 8>(regular, kind, in, offsets, out, out2, n, starts, ends, seg_len, nseg, shift, pairs, carried, tiles, s);
    else launch_irregular_reduce_shape<4, 4>(regular, kind, in, offsets, out, out2, n, starts, ends, seg_len, nseg, shift, pairs, carried, tiles, s);
    st = check_launch("irregular_reduce_kernel");
    if (st != TCR_OK || tiles == 1) return st;          // a single tile has nothing in front of it
    const dim3 carry_grid((unsigned)ceil_div(groups, kCarryWaves), ch);
    irregular_groups_kernel<<<carry_grid, dim3(kCarryWaves * kWave), 0, s>>>(pairs, tiles, group_pairs);
    st = check_launch("irregular_groups_kernel");
    if (st != TCR_OK) return st;
    irregular_carry_kernel<<<carry_grid, dim3(kCarryWaves * kWave), 0, s>>>(pairs, group_pairs, carried, tiles, out, out2);
    return check_launch("irregular_carry_kernel");
}

// Regular segments from 17 elements on, no power of two: whole segments per workgroup, masked row products
// (tcr_rows.hpp).  `in` needs only 2-byte alignment.  kind: kSum, or kBoth with the sums of squares in out2.
// Measured at n = 2^28 against the kernels that took these lengths before: sums 77-98 us from 33 to 8000
// elements (fixed tiles with marked starts: 114-157 us below 1000; one wavefront per segment over masked tiles:
// 114 us at 1000, 89 at 2000, 80 from 3000 on); both moments 88-108 us (fixed tiles 184-249 us; masked tiles 119 us
// at 1000, 93 at 2000, 82 from 3000 on, where they stay).  From 17 to 31 elements (two boundaries per row): sums
// 102-110 us (fixed tiles 117-150 us), both moments 140-170 us (177-217 us).
// (Below 17 -- two or three whole segments per row -- it only equals the fixed tiles at 11-15 elements, 123-130 us
// either way, and loses to them at 9 and 10, 170 against 144-168 us.)
constexpr uint64_t kRowsReduceMin = 17, kRowsMomentsMin = 17, kRowsReduceMax = kRowsMaxSegLen, kRowsMomentsMax = 2999;
inline bool rows_reduce_takes(uint64_t seg_len, int kind = kSum) {
    return g_variant.rows_reduce && seg_len >= (kind == kBoth ? kRowsMomentsMin : kRowsReduceMin) &&
           seg_len <= (kind == kBoth ? kRowsMomentsMax : kRowsReduceMax);
}
inline tcr_status launch_rows_reduce(const _Float16* in, float* out, float* out2, uint64_t n, uint64_t seg_len, int kind,
                                     hipStream_t s) {
    constexpr int U = 4, W = 8;
    const uint32_t shift = alignment_shift(in);
    RowsGrid grid;
    grid.seg_len = seg_len;
    grid.nseg = n / seg_len;
    grid.n = n + shift;
    grid.shift = shift;
    grid.per_group = (uint32_t)(kRowsGroupElems / seg_len);
    grid.magic = (uint32_t)(((1ull << 32) + seg_len - 1) / seg_len);
    const dim3 blocks((unsigned)ceil_div(grid.nseg, grid.per_group)), block(W * kWave);
    if (seg_len < 32) {              // 17 .. 31: two boundaries per row and a whole segment between them
        if (kind == kBoth) rows_reduce_kernel<kBoth, U, W, 1><<<blocks, block, 0, s>>>(in - shift, out, out2, grid);
        else rows_reduce_kernel<kSum, U, W, 1><<<blocks, block, 0, s>>>(in - shift, out, nullptr, grid);
    } else {
        if (kind == kBoth) rows_reduce_kernel<kBoth, U, W><<<blocks, block, 0, s>>>(in - shift, out, out2, grid);
        else rows_reduce_kernel<kSum, U, W><<<blocks, block, 0, s>>>(in - shift, out, nullptr, grid);
    }
    return check_launch("rows_reduce_kernel");
}

// Regular segments of 3 to 30 elements that pack into rows of an even number of at most 32 elements (every even
// length that is no power of two, odd lengths up to 15): one product per 16 rows with a masked constant matrix
// (tcr_packed.hpp).  `in` 4-byte aligned.  kind: kSum, or kBoth with the sums of squares in out2.
// Measured at n = 2^28 against the kernels that took these lengths before -- sums: 3 elements 162 us (one thread per
// segment: 274), 5 to 7 107-116 (fixed tiles with marked starts 162-183), 9 to 15 98-104 (125-148), even lengths
// from 18 to 30 91-99 (masked rows of the array 102-106); both moments: 3 elements 310 (one thread per segment
// 320-345), 5 to 7 153-190 (213-250), 9 to 15 110-134 (180-216), 18 to 30 100-110 (140-170).
// Two launch shapes: eight tiles per wavefront where a row's width is no multiple of 8 (rows of 18 elements: 99
// against 113 us; 22: 97 against 105; 26 to 30: 94-96 against 97-99), four where it is (24: 90 against 96 us); twelve
// or sixteen tiles, or two or eight wavefronts, change nothing.  (U, W) = (8, 4) and (4, 4).
// (4 and 8 elements as well: sums 117 and 102 us against 125 and 110 for the kernel with whole segments inside a
// lane's eight elements, both moments 208 and 128 against 272 and 219 with one thread per segment; 2 elements: 178
// against 167 us, and 16 rows of P for the squares -- left where they are)
inline bool packed_reduce_takes(uint64_t seg_len) {
    return g_variant.rows_reduce && packed_per_row(seg_len) != 0 && (!is_pow2(seg_len) || seg_len == 4 || seg_len == 8);
}
template <int KIND, int U, int W>
inline void launch_packed_shape(const _Float16* in, float* out, float* out2, const PackedGrid& grid, hipStream_t s) {
    const uint64_t rows = ceil_div(grid.nseg, (uint64_t)grid.per_row);
    const size_t staging = (size_t)W * channels<KIND>() * 16 * U * grid.per_row * sizeof(float);      // at most 40 KiB
    packed_rows_reduce_kernel<KIND, U, W><<<dim3((unsigned)ceil_div(rows, (uint64_t)(16 * U * W))), dim3(W * kWave), staging, s>>>(in, out, out2, grid);
}
// alt: the other launch shape than the one the row width calls for.
inline tcr_status launch_packed_reduce(const _Float16* in, float* out, float* out2, uint64_t n, uint64_t seg_len, int kind,
                                       hipStream_t s, bool alt = false) {
    const PackedGrid grid = {n, n / seg_len, (uint32_t)seg_len, packed_per_row(seg_len)};
    const bool four = ((grid.seg_len * grid.per_row) % 8u == 0) != alt;
    if (kind == kBoth) {
        if (four) launch_packed_shape<kBoth, 4, 4>(in, out, out2, grid, s);
        else launch_packed_shape<kBoth, 8, 4>(in, out, out2, grid, s);
    } else {
        if (four) launch_packed_shape<kSum, 4, 4>(in, out, nullptr, grid, s);
        else launch_packed_shape<kSum, 8, 4>(in, out, nullptr, grid, s);
    }
    return check_launch("packed_rows_reduce_kernel");
}

// Any other seg_len >= 1 (no power of two, or below 16): no kernel is tuned for it.
// Scans from 2 elements on and reductions of 8 to 999 elements run on the fixed tiles of the irregular
// kernels with the multiples of seg_len as segment starts.  Measured at n = 2^28: scans 300-325 us
// whatever the length (one thread or one wavefront per segment took 440-5600 us below 256 elements,
// 350-400 us above, and 13 ms for 15 segments of 2^24 + 1 elements); reductions 146-231 us (against
// 230-1060 us).  Longer reductions keep one wavefront per segment over zero-masked tiles (116 us at
// 1000 elements, 85 us at 3001), the shortest segments one thread each.
constexpr uint64_t kTiledScanMin = 2;
// (sums from 5 elements on: 161-183 us at 5..7 against 193-210 us with one thread per segment, 274 either way at 3;
// both moments from 8 on: below, one thread per segment is faster, 213-232 against 231-259 us)
constexpr uint64_t kTiledReduceMin = 5, kTiledMomentsMin = 8, kTiledReduceMax = 1000;

// Which kernel takes a reduction whose seg_len is no power of two (or below 16); class = floor(log2(seg_len)).
// The default is the first valid one of: rows, tiles, the rest (one wavefront per segment over masked tiles from
// 1000 elements, one thread per segment below 5).
enum ReduceAny { kReduceAnyRows = 0, kReduceAnyTiles = 1, kReduceAnyTilesAlt = 2, kReduceAnyMasked = 3, kReduceAnyPacked = 4, kReduceAnyPackedAlt = 5, kReduceAnyCount = 6 };
constexpr uint64_t kMaskedReduceMin = 256;              // (valid for any length; pointless for short segments)
inline bool reduce_any_valid(int id, uint64_t seg_len) {
    switch (id) {
        case kReduceAnyRows: return rows_reduce_takes(seg_len);
        case kReduceAnyTiles:
        case kReduceAnyTilesAlt: return seg_len >= kTiledReduceMin && seg_len < kTiledReduceMax;
        case kReduceAnyMasked: return seg_len >= kMaskedReduceMin;
        case kReduceAnyPacked:
        case kReduceAnyPackedAlt: return packed_reduce_takes(seg_len);
        default: return false;
    }
}
// packed_ok: the array is 4-byte aligned (the packed rows need that; kernel names are given for aligned arrays)
inline int pick_reduce_any(uint64_t seg_len, bool packed_ok = true) {
    const int tuned = tuned_id(kTuneReduceAny, floor_log2(seg_len));
    if (reduce_any_valid(tuned, seg_len) && ((tuned != kReduceAnyPacked && tuned != kReduceAnyPackedAlt) || packed_ok)) return tuned;
    if (packed_ok && reduce_any_valid(kReduceAnyPacked, seg_len)) return kReduceAnyPacked;
    if (reduce_any_valid(kReduceAnyRows, seg_len)) return kReduceAnyRows;
    if (reduce_any_valid(kReduceAnyTiles, seg_len)) return kReduceAnyTiles;
    return kReduceAnyMasked;                            // (or one thread per segment, below 8 elements)
}

template <bool SCAN>
inline tcr_status launch_generic(const _Float16* in, void* out, uint64_t n, uint64_t seg_len, uint32_t flags, hipStream_t s,
                                 int tiles_shape = 0) {
    const uint64_t nseg = n / seg_len;
    const bool excl = (flags & TCR_SCAN_EXCLUSIVE) != 0, f16 = (flags & TCR_OUT_F16) != 0;
    // 1, 2, 4 or 8 elements (scans: the plain binary32 inclusive one): whole segments inside a lane's 8 elements.
    // `out` is 16-byte aligned for scans; reductions need it for their 128-bit stores.
    // 4 and 8 elements: reductions on rows of whole segments unless the tuning table or the variant says otherwise
    const bool packed_first = !SCAN && (seg_len == 4 || seg_len == 8) && packed_reduce_takes(seg_len) && aligned(in, 4) &&
                              (pick_reduce_any(seg_len) == kReduceAnyPacked || pick_reduce_any(seg_len) == kReduceAnyPackedAlt);
    if (is_pow2(seg_len) && seg_len <= 8 && !packed_first && (SCAN ? flags == 0 : aligned(out, 16))) {
        const dim3 grid((unsigned)ceil_div(n, (uint64_t)kGenericThreads * 8)), block(kGenericThreads);
        float* o = static_cast<float*>(out);
        if constexpr (SCAN) {
            switch (seg_len) {
                case 1: tiny_scan_kernel<0><<<grid, block, 0, s>>>(in, o, n); break;
                case 2: tiny_scan_kernel<1><<<grid, block, 0, s>>>(in, o, n); break;
                case 4: tiny_scan_kernel<2><<<grid, block, 0, s>>>(in, o, n); break;
                default: tiny_scan_kernel<3><<<grid, block, 0, s>>>(in, o, n); break;
            }
            return check_launch("tiny_scan_kernel");
        }
        switch (seg_len) {
            case 1: tiny_reduce_kernel<0><<<grid, block, 0, s>>>(in, o, n); break;
            case 2: tiny_reduce_kernel<1><<<grid, block, 0, s>>>(in, o, n); break;
            case 4: tiny_reduce_kernel<2><<<grid, block, 0, s>>>(in, o, n); break;
            default: tiny_reduce_kernel<3><<<grid, block, 0, s>>>(in, o, n); break;
        }
        return check_launch("tiny_reduce_kernel");
    }
    if constexpr (SCAN) {
        if (seg_len >= kTiledScanMin) {
            switch (flags & 3u) {
                case 0: return launch_irregular_scan<0>(in, nullptr, out, n, nseg, seg_len, s, tiles_shape);
                case 1: return launch_irregular_scan<1>(in, nullptr, out, n, nseg, seg_len, s, tiles_shape);
                case 2: return launch_irregular_scan<2>(in, nullptr, out, n, nseg, seg_len, s, tiles_shape);
                default: return launch_irregular_scan<3>(in, nullptr, out, n, nseg, seg_len, s, tiles_shape);
            }
        }
    } else {
        const int pick = pick_reduce_any(seg_len, aligned(in, 4));
        if (pick == kReduceAnyPacked || pick == kReduceAnyPackedAlt)
            return launch_packed_reduce(in, static_cast<float*>(out), nullptr, n, seg_len, kSum, s, pick == kReduceAnyPackedAlt);
        if (pick == kReduceAnyRows) return launch_rows_reduce(in, static_cast<float*>(out), nullptr, n, seg_len, kSum, s);
        if (pick == kReduceAnyTiles || pick == kReduceAnyTilesAlt)
            return launch_irregular_reduce(in, nullptr, static_cast<float*>(out), n, nseg, seg_len, s, kSum, nullptr,
                                           pick == kReduceAnyTilesAlt ? 1 : 0);
    }
    if (SCAN || seg_len < kTiledReduceMin) {         // (also reductions of 3 elements from an array that is not 4-byte aligned)
        generic_thread_kernel<SCAN><<<dim3((unsigned)ceil_div(nseg, kGenericThreads)), dim3(kGenericThreads), 0, s>>>(
            in, out, nseg, seg_len, excl, f16);
        return check_launch("generic_thread_kernel");
    }
    // reductions from 1000 elements on: masked 512-element tiles of the array, one wavefront per segment
    const dim3 grid((unsigned)ceil_div(nseg, kMaskedWaves)), block(kMaskedWaves * kWave);
    if (seg_len <= 2 * kWaveSpanMax) {
        masked_wave_reduce_kernel<<<grid, block, 0, s>>>(in, static_cast<float*>(out), nseg, seg_len);
        return check_launch("masked_wave_reduce_kernel");
    }
    // long segments: pieces of 65536 elements per wavefront, then the paper's second kernel over the pieces
    const uint64_t per = ceil_div(seg_len, kWaveSpanMax);
    Workspace* ws = nullptr;
    bool capturing = false;
    tcr_status st = get_workspace(s, &ws, &capturing);
    if (st != TCR_OK) return st;
    st = ensure_partials(ws, s, nseg * per, capturing);
    if (st != TCR_OK) return st;
    masked_span_reduce_kernel<<<dim3((unsigned)ceil_div(nseg * per, kMaskedWaves)), block, 0, s>>>(
        in, ws->partials, nseg, seg_len, kWaveSpanMax, per);
    st = check_launch("masked_span_reduce_kernel");
    if (st != TCR_OK) return st;
    reduce_final_kernel<<<dim3((unsigned)nseg), dim3(kFinalThreads), 0, s>>>(ws->partials, static_cast<float*>(out), per);
    return check_launch("reduce_final_kernel");
}

// The tuned scan paths for one (formulation, mode) pair.
template <int FORM, int MODE>
inline tcr_status scan_tuned(const _Float16* x, void* out, uint64_t n, uint64_t seg_len, hipStream_t s) {
    if (seg_len == n) return scan_long<FORM, MODE>(x, out, n, n, true, s);
    if (seg_len <= kTile) return launch_scan_small<FORM, MODE>(x, out, n, log2u(seg_len), s);
    return scan_long<FORM, MODE>(x, out, n, seg_len, false, s);
}

// First two moments of every segment, any seg_len >= 1 that divides n.
template <int LOG2L>
inline void launch_moments_small(const _Float16* in, float* sum, float* sumsq, uint64_t n, hipStream_t s) {
    const uint64_t per_group = (uint64_t)kTile * kSmallReduceU * kSmallReduceW;
    moments_small_kernel<LOG2L, kSmallReduceU, kSmallReduceW><<<dim3((unsigned)ceil_div(n, per_group)), dim3(kSmallReduceW * kWave), 0, s>>>(
        in, sum, sumsq, n);
}

inline tcr_status launch_moments(const _Float16* in, float* sum, float* sumsq, uint64_t n, uint64_t seg_len, hipStream_t s) {
    const uint64_t nseg = n / seg_len;
    if (is_pow2(seg_len) && seg_len >= 16 && seg_len <= kTile) {
        switch (log2u(seg_len)) {
            case 4: launch_moments_small<4>(in, sum, sumsq, n, s); break;
            case 5: launch_moments_small<5>(in, sum, sumsq, n, s); break;
            case 6: launch_moments_small<6>(in, sum, sumsq, n, s); break;
            case 7: launch_moments_small<7>(in, sum, sumsq, n, s); break;
            case 8: launch_moments_small<8>(in, sum, sumsq, n, s); break;
            default: launch_moments_small<9>(in, sum, sumsq, n, s); break;
        }
        return check_launch("moments_small_kernel");
    }
    if (packed_reduce_takes(seg_len) && aligned(in, 4)) return launch_packed_reduce(in, sum, sumsq, n, seg_len, kBoth, s);
    if (rows_reduce_takes(seg_len, kBoth)) return launch_rows_reduce(in, sum, sumsq, n, seg_len, kBoth, s);
    if (seg_len >= kTiledMomentsMin && seg_len < kTiledReduceMax) {
        // fixed tiles with the segment starts marked, both moments as two channels of one pass
        return launch_irregular_reduce(in, nullptr, sum, n, nseg, seg_len, s, kBoth, sumsq);
    }
    if (seg_len < kTiledMomentsMin) {        // under 8 elements: one thread per segment
        generic_moments_kernel<<<dim3((unsigned)ceil_div(nseg, kGenericThreads)), dim3(kGenericThreads), 0, s>>>(
            in, sum, sumsq, nseg, seg_len);
        return check_launch("generic_moments_kernel");
    }
    const dim3 block(kMaskedWaves * kWave);
    if (seg_len <= 2 * kWaveSpanMax) {
        masked_moments_kernel<<<dim3((unsigned)ceil_div(nseg, kMaskedWaves)), block, 0, s>>>(in, sum, sumsq, nseg, seg_len,
                                                                                             seg_len, 1);
        return check_launch("masked_moments_kernel");
    }
    // long segments: 65536-element pieces, then the second kernel of the device-level reduction for each moment
    const uint64_t per = ceil_div(seg_len, kWaveSpanMax), pieces = nseg * per;
    Workspace* ws = nullptr;
    bool capturing = false;
    tcr_status st = get_workspace(s, &ws, &capturing);
    if (st != TCR_OK) return st;
    st = ensure_partials(ws, s, 2 * pieces, capturing);
    if (st != TCR_OK) return st;
    masked_moments_kernel<<<dim3((unsigned)ceil_div(pieces, kMaskedWaves)), block, 0, s>>>(
        in, ws->partials, ws->partials + pieces, nseg, seg_len, kWaveSpanMax, per);
    st = check_launch("masked_moments_kernel");
    if (st != TCR_OK) return st;
    reduce_final_kernel<<<dim3((unsigned)nseg), dim3(kFinalThreads), 0, s>>>(ws->partials, sum, per);
    reduce_final_kernel<<<dim3((unsigned)nseg), dim3(kFinalThreads), 0, s>>>(ws->partials + pieces, sumsq, per);
    return check_launch("reduce_final_kernel");
}

// Segment lengths that are no power of two, a multiple of 8, and fit one workgroup: scan_segment_kernel with the
// smallest share that holds a segment.
inline bool segment_kernel_takes(uint64_t seg_len) {
    return g_variant.formulation == kMfma && seg_len % 8 == 0 && seg_len > kTile && seg_len < 2 * scan_shape_tile(10);
}

template <int U, int W, int MODE>
void launch_scan_segment_shape(const _Float16* in, void* out, uint64_t n, uint64_t seg_len, hipStream_t s) {
    scan_segment_kernel<U, W, MODE><<<dim3((unsigned)(n / seg_len)), dim3(W * kWave), 0, s>>>(in, out, seg_len);
}

// Shares in steps of at most a third, so that few wavefronts of a workgroup lie beyond the segment's end.
template <int MODE>
tcr_status launch_scan_segment(const _Float16* in, void* out, uint64_t n, uint64_t seg_len, hipStream_t s) {
    const uint64_t t = ceil_div(seg_len, kTile);           // tiles per segment
    if (t <= 2) launch_scan_segment_shape<1, 2, MODE>(in, out, n, seg_len, s);
    else if (t <= 3) launch_scan_segment_shape<1, 3, MODE>(in, out, n, seg_len, s);
    else if (t <= 4) launch_scan_segment_shape<1, 4, MODE>(in, out, n, seg_len, s);
    else if (t <= 6) launch_scan_segment_shape<1, 6, MODE>(in, out, n, seg_len, s);
    else if (t <= 8) launch_scan_segment_shape<1, 8, MODE>(in, out, n, seg_len, s);
    else if (t <= 12) launch_scan_segment_shape<1, 12, MODE>(in, out, n, seg_len, s);
    else if (t <= 16) launch_scan_segment_shape<1, 16, MODE>(in, out, n, seg_len, s);
    else if (t <= 24) launch_scan_segment_shape<2, 12, MODE>(in, out, n, seg_len, s);
    else if (t <= 32) launch_scan_segment_shape<2, 16, MODE>(in, out, n, seg_len, s);
    else if (t <= 48) launch_scan_segment_shape<4, 12, MODE>(in, out, n, seg_len, s);
    else if (t <= 64) launch_scan_segment_shape<4, 16, MODE>(in, out, n, seg_len, s);
    else if (t <= 96) launch_scan_segment_shape<8, 12, MODE>(in, out, n, seg_len, s);
    else launch_scan_segment_shape<8, 16, MODE>(in, out, n, seg_len, s);
    return check_launch("scan_segment_kernel");
}

// Segment lengths that are no power of two but long enough for the persistent chain (its ragged last tile per
// segment is cut off by the buffer range check, which works on whole 8-element groups).
inline bool chain_takes_any_length(uint64_t seg_len) {
    return g_variant.formulation == kMfma && g_variant.scan_carry == kStrategyLookback && seg_len % 8 == 0 &&
           seg_len >= 2 * scan_shape_tile(10);
}

// Which kernel takes a scan whose seg_len is no power of two (or below 16); class = floor(log2(seg_len)).  The
// default: the chain where it is valid, one workgroup per segment where that is known to win, else the tiles.
enum ScanAny { kScanAnyTiles = 0, kScanAnyTilesAlt = 1, kScanAnySegment = 2, kScanAnyChain = 3, kScanAnyCount = 4 };
inline bool scan_any_valid(int id, uint64_t seg_len) {
    switch (id) {
        case kScanAnyTiles:
        case kScanAnyTilesAlt: return seg_len >= kTiledScanMin;
        case kScanAnySegment: return segment_kernel_takes(seg_len);
        case kScanAnyChain: return chain_takes_any_length(seg_len);
        default: return false;
    }
}
// One workgroup per segment beats the fixed tiles (284-291 us at n = 2^28 whatever the length) where the segments
// start on 128-byte boundaries and fill at least four fifths of the workgroup's share of one tile per wavefront:
// 270-282 us at 1280, 1536, 2560, 3584, 7168 and 8000 elements; 293-372 us at 520, 1000, 2056, 3000, 4088, 4104
// (short of the share, or rows of the tiles that straddle cache lines), 300-315 us from 12000 elements on (two
// tiles per wavefront).
inline bool segment_kernel_preferred(uint64_t seg_len) {
    if (!segment_kernel_takes(seg_len) || seg_len % 64 != 0 || seg_len > 16 * (uint64_t)kTile) return false;
    const uint64_t t = ceil_div(seg_len, kTile);
    const uint64_t share = t <= 4 ? t : (t <= 6 ? 6 : (t <= 8 ? 8 : (t <= 12 ? 12 : 16)));     // as launch_scan_segment picks it
    return 5 * seg_len >= 4 * share * kTile;
}
inline int pick_scan_any(uint64_t seg_len) {
    const int tuned = tuned_id(kTuneScanAny, floor_log2(seg_len));
    if (scan_any_valid(tuned, seg_len)) return tuned;
    if (scan_any_valid(kScanAnyChain, seg_len)) return kScanAnyChain;
    if (segment_kernel_preferred(seg_len)) return kScanAnySegment;
    return kScanAnyTiles;
}

inline tcr_status scan_any(const void* in, void* out, uint64_t n, uint64_t seg_len, uint32_t flags, hipStream_t s) {
    const _Float16* x = static_cast<const _Float16*>(in);
    const int mode = (int)(flags & 3u);
    if (seg_len != n && (!is_pow2(seg_len) || seg_len < 16)) {
        const int pick = pick_scan_any(seg_len);
        if (pick == kScanAnyChain) {
            // long segments of any length that keeps 8-element groups whole: the chain on a per-segment tile grid
            switch (mode) {
                case 0: return launch_chain<kMfma, 0>(10, x, out, n, seg_len, s);
                case 1: return launch_chain<kMfma, 1>(10, x, out, n, seg_len, s);
                case 2: return launch_chain<kMfma, 2>(10, x, out, n, seg_len, s);
                default: return launch_chain<kMfma, 3>(10, x, out, n, seg_len, s);
            }
        }
        if (pick == kScanAnySegment) {
            switch (mode) {
                case 0: return launch_scan_segment<0>(x, out, n, seg_len, s);
                case 1: return launch_scan_segment<1>(x, out, n, seg_len, s);
                case 2: return launch_scan_segment<2>(x, out, n, seg_len, s);
                default: return launch_scan_segment<3>(x, out, n, seg_len, s);
            }
        }
        return launch_generic<true>(x, out, n, seg_len, flags, s, pick == kScanAnyTilesAlt ? 1 : 0);
    }
    // the cross-lane alternative is kept for the default mode only
    const int form = tuned_formulation(kTuneScan, tuning_class(seg_len, seg_len == n));
    if (form == kDpp && mode == 0) return scan_tuned<kDpp, 0>(x, out, n, seg_len, s);
    if (g_variant.formulation == kDpp) return TCR_ERR_UNSUPPORTED;        // forced for every class: the other modes have no kernels
    switch (mode) {
        case 0: return scan_tuned<kMfma, 0>(x, out, n, seg_len, s);
        case 1: return scan_tuned<kMfma, 1>(x, out, n, seg_len, s);
        case 2: return scan_tuned<kMfma, 2>(x, out, n, seg_len, s);
        default: return scan_tuned<kMfma, 3>(x, out, n, seg_len, s);
    }
}

// The scan with a binary16 accumulator (TCR_ACC_F16): powers of two and the one-segment scan, 16-byte aligned arrays.
template <int U, int W, int CARRY, int EXCL>
inline void launch_scan_half_shape(const _Float16* in, _Float16* out, uint64_t n, uint64_t seg_mask, uint64_t seg_len,
                                   const ScanWorkspace& dev, hipStream_t s) {
    const unsigned blocks = (unsigned)ceil_div(n, (uint64_t)kTile * U * W);
    scan_half_kernel<U, W, CARRY, EXCL><<<dim3(blocks), dim3(W * kWave), 0, s>>>(in, out, n, seg_mask, seg_len, dev);
}

template <int EXCL>
inline tcr_status scan_half(const _Float16* in, _Float16* out, uint64_t n, uint64_t seg_len, hipStream_t s) {
    const bool whole = seg_len == n;
    if (!whole && !is_pow2(seg_len)) return TCR_ERR_UNSUPPORTED;
    if (!aligned(in, 16) || !aligned(out, 16)) return TCR_ERR_UNSUPPORTED;
    const uint64_t len = seg_len;                                  // decides the launch shape
    const uint64_t seg_mask = (whole && !is_pow2(n)) ? ~0ull : seg_len - 1;
    if (whole && !is_pow2(n)) seg_len = ~0ull;                     // one segment of any length: never restarts
    const ScanWorkspace none = {};
    if (len <= 1024) launch_scan_half_shape<1, 2, kNoCarry, EXCL>(in, out, n, seg_mask, seg_len, none, s);
    else if (len <= 4096) launch_scan_half_shape<1, 8, kNoCarry, EXCL>(in, out, n, seg_mask, seg_len, none, s);
    else if (len <= 16384) launch_scan_half_shape<2, 16, kNoCarry, EXCL>(in, out, n, seg_mask, seg_len, none, s);
    else if (len <= 65536) launch_scan_half_shape<8, 16, kNoCarry, EXCL>(in, out, n, seg_mask, seg_len, none, s);
    else {
        const uint64_t tiles = ceil_div(n, (uint64_t)kTile * 8 * 16);
        ScanWorkspace dev = {};
        Workspace* ws = nullptr;
        bool capturing = false;
        tcr_status st = get_workspace(s, &ws, &capturing);
        if (st != TCR_OK) return st;
        st = begin_lookback(ws, s, tiles, &dev, capturing);
        if (st != TCR_OK) return st;
        launch_scan_half_shape<8, 16, kLookback, EXCL>(in, out, n, seg_mask, seg_len, dev, s);
        st = check_launch("scan_half_kernel");
        if (st != TCR_OK) {
            ws->dirty = true;
            return st;
        }
        ws->tickets_issued += (uint32_t)tiles;
        return TCR_OK;
    }
    return check_launch("scan_half_kernel");
}

// out_align: the natural alignment of the output's elements.
inline tcr_status validate(const void* in, const void* out, uint64_t n, uint64_t seg_len, uintptr_t out_align) {
    if (seg_len == 0) return TCR_ERR_INVALID_ARG;
    if (n % seg_len != 0) return TCR_ERR_INVALID_ARG;
    if (n == 0) return TCR_OK;
    if (in == nullptr || out == nullptr) return TCR_ERR_INVALID_ARG;
    if (!aligned(in, 2) || !aligned(out, out_align)) return TCR_ERR_INVALID_ARG;
    if (n > kMaxElements) return TCR_ERR_UNSUPPORTED;
    return TCR_OK;
}


}  // namespace host
}  // namespace tcr
