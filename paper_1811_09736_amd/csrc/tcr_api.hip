// C ABI of the library (declared in include/tcr.h): argument validation, the dispatch from
// segment length to kernel and launch shape (the role the paper gives its auto-tuner,
// Section 6), and the per-(device, stream) workspace for cross-workgroup carries.
#include "../../include/tcr.h"

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "tcr_reduce.hpp"
#include "tcr_scan.hpp"
#include "tcr_generic.hpp"

namespace {

using namespace tcr;

thread_local std::string g_hip_error;

bool hip_failed(hipError_t e, const char* what) {
    if (e == hipSuccess) return false;
    g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return true;
}
#define TCR_HIP(call)                                   \
    do {                                                \
        if (hip_failed((call), #call)) return TCR_ERR_HIP; \
    } while (0)

// ---------------------------------------------------------------------------- variant settings
struct Variant {
    int formulation = kMfma;
    int scan_carry = kStrategyLookback;
    bool reduce_fused = false;      // long reductions: a second kernel adds the partials (true: the last workgroup does)
};
Variant g_variant;

// Launch shapes (U = tiles of 512 elements per wavefront, W = wavefronts per workgroup) come from
// timing sweeps at n = 2^28 on MI355X: short-lived wavefronts with one tile each stream best, so
// segments up to 16384 elements take the smallest workgroup share that still contains a whole
// segment; longer ones (and the full scan) run the persistent chain, whose tiles pass carries
// between workgroups.
constexpr int kSmallScanW = 2;                       // scan_small: U = 1
constexpr int kSmallReduceU = 2, kSmallReduceW = 4;  // reduce_small
constexpr uint64_t kWaveSpanMax = 65536;             // reduce: longest span one wavefront folds
constexpr int kReduceBlockW = 4;                     // reduce: wavefronts combined through LDS for longer segments
constexpr int kCarryU = 8, kCarryW = 16;             // the multi-kernel scan strategies: 65536 elements per workgroup
constexpr uint64_t kCarryTile = (uint64_t)kTile * kCarryU * kCarryW;
constexpr uint64_t kMaxElements = 1ull << 38;        // keeps every grid below 2^31 workgroups
constexpr uint64_t kFusedPartialsMax = 4096;         // partials one workgroup adds up at the end of a fused long reduction

// ---------------------------------------------------------------------------- workspace
struct Workspace {
    unsigned long long* desc = nullptr;
    uint64_t desc_capacity = 0;     // tiles
    float* partials = nullptr;
    uint64_t partials_capacity = 0; // floats
    uint32_t* counters = nullptr;   // [0] = ticket, [1] = gave_up flag, [2] = latest epoch, [3] = ticket base (device-managed)
    uint32_t tickets_issued = 0;    // host mirror of counters[0] once all enqueued launches finish
    uint32_t epoch = 0;
    // Once a launch that chains tiles has been recorded into a HIP graph, epoch and ticket base live on the
    // device (advanced by chain_begin_kernel in front of every launch) and the two host mirrors above are
    // no longer used: a replayed graph repeats its kernel arguments.
    bool device_managed = false;
    bool dirty = true;              // counters / descriptors must be re-zeroed before use
    bool caller_owned = false;      // memory supplied through tcr_set_workspace: never grown, never freed
    bool flag_valid = true;         // false until the first clean-up has written the caller's (uninitialised) flag word
};

std::mutex g_mutex;
std::map<std::pair<int, hipStream_t>, Workspace> g_workspaces;
// Caller-supplied workspaces, one per device: [256-byte header: ticket, flag | descriptors | partials],
// the two areas of equal size.  While one is set, every call on that device uses it, whatever its stream.
std::map<int, Workspace> g_caller_workspaces;
constexpr uint64_t kWorkspaceHeader = 256;

// Look-back descriptor tables are allocated uncached (polling them through the L2 path measured
// ~5 % slower on the full scan).  Uncached allocations are never handed back to the runtime:
// a table that is outgrown or released is parked here and reused by the next request it fits.
struct ParkedTable {
    int device;
    unsigned long long* ptr;
    uint64_t capacity;
};
std::vector<ParkedTable> g_parked_tables;

tcr_status acquire_table(int device, uint64_t tiles, unsigned long long** ptr, uint64_t* capacity) {
    for (size_t i = 0; i < g_parked_tables.size(); ++i) {
        if (g_parked_tables[i].device == device && g_parked_tables[i].capacity >= tiles) {
            *ptr = g_parked_tables[i].ptr;
            *capacity = g_parked_tables[i].capacity;
            g_parked_tables.erase(g_parked_tables.begin() + (long)i);
            return TCR_OK;
        }
    }
    uint64_t cap = 1024;
    while (cap < tiles) cap <<= 1;
    void* p = nullptr;
    if (hipExtMallocWithFlags(&p, cap * sizeof(unsigned long long), hipDeviceMallocUncached) != hipSuccess) {
        (void)hipGetLastError();
        return TCR_ERR_WORKSPACE;
    }
    *ptr = static_cast<unsigned long long*>(p);
    *capacity = cap;
    return TCR_OK;
}

// Every call that needs workspace memory comes through here.  *capturing tells the caller that the stream
// is recording a HIP graph: nothing may then be allocated, cleared or synchronised, so a workspace that is
// too small or not yet initialised makes the call return TCR_ERR_UNSUPPORTED.
tcr_status get_workspace(hipStream_t stream, Workspace** out, bool* capturing) {
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    TCR_HIP(hipStreamIsCapturing(stream, &capture));
    *capturing = capture != hipStreamCaptureStatusNone;
    int dev = 0;
    TCR_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_mutex);
    auto own = g_caller_workspaces.find(dev);
    *out = own != g_caller_workspaces.end() ? &own->second : &g_workspaces[std::make_pair(dev, stream)];
    return TCR_OK;
}

tcr_status ensure_partials(Workspace* ws, hipStream_t stream, uint64_t floats, bool capturing) {
    if (floats <= ws->partials_capacity) return TCR_OK;
    if (ws->caller_owned) return TCR_ERR_WORKSPACE;
    if (capturing) return TCR_ERR_UNSUPPORTED;
    TCR_HIP(hipStreamSynchronize(stream));
    if (ws->partials) TCR_HIP(hipFree(ws->partials));
    ws->partials = nullptr;
    ws->partials_capacity = 0;
    uint64_t cap = 1;
    while (cap < floats) cap <<= 1;
    if (hipMalloc(&ws->partials, cap * sizeof(float)) != hipSuccess) {
        (void)hipGetLastError();
        return TCR_ERR_WORKSPACE;
    }
    ws->partials_capacity = cap;
    return TCR_OK;
}

// Makes room for `tiles` descriptors and starts a new epoch (tiles == 0: only the running counter is wanted).
tcr_status begin_lookback(Workspace* ws, hipStream_t stream, uint64_t tiles, ScanWorkspace* dev, bool capturing) {
    if (ws->caller_owned && tiles > ws->desc_capacity) return TCR_ERR_WORKSPACE;
    if (capturing && (ws->counters == nullptr || tiles > ws->desc_capacity || ws->dirty)) return TCR_ERR_UNSUPPORTED;
    if (ws->counters == nullptr) {
        if (hipMalloc(&ws->counters, 4 * sizeof(uint32_t)) != hipSuccess) {
            (void)hipGetLastError();
            return TCR_ERR_WORKSPACE;
        }
        TCR_HIP(hipMemset(ws->counters, 0, 4 * sizeof(uint32_t)));
        ws->tickets_issued = 0;
        ws->dirty = true;
    }
    if (tiles > ws->desc_capacity) {
        TCR_HIP(hipStreamSynchronize(stream));
        int dev_id = 0;
        TCR_HIP(hipGetDevice(&dev_id));
        std::lock_guard<std::mutex> lock(g_mutex);
        if (ws->desc) g_parked_tables.push_back({dev_id, ws->desc, ws->desc_capacity});
        ws->desc = nullptr;
        ws->desc_capacity = 0;
        const tcr_status st = acquire_table(dev_id, tiles, &ws->desc, &ws->desc_capacity);
        if (st != TCR_OK) return st;
        ws->dirty = true;
    }
    if (ws->dirty || (!ws->device_managed && ws->epoch >= (1u << 30) - 2u)) {
        // first use, growth, a failed launch, or epoch wrap: start from a clean slate
        TCR_HIP(hipStreamSynchronize(stream));
        if (ws->desc_capacity) TCR_HIP(hipMemset(ws->desc, 0, ws->desc_capacity * sizeof(unsigned long long)));
        uint32_t keep_flag = 0;
        if (ws->flag_valid) TCR_HIP(hipMemcpy(&keep_flag, ws->counters + 1, sizeof(uint32_t), hipMemcpyDeviceToHost));
        ws->flag_valid = true;
        uint32_t init[4] = {0u, keep_flag, 0u, 0u};
        TCR_HIP(hipMemcpy(ws->counters, init, sizeof(init), hipMemcpyHostToDevice));
        ws->tickets_issued = 0;
        ws->epoch = 0;
        ws->dirty = false;
    }
    if (capturing) ws->device_managed = true;         // for good: the host can no longer follow the counters
    dev->desc = ws->desc;
    dev->ticket = ws->counters;
    dev->gave_up = ws->counters + 1;
    dev->state = ws->counters + 2;
    dev->device_managed = ws->device_managed ? 1u : 0u;
    if (ws->device_managed) {
        chain_begin_kernel<<<dim3(1), dim3(kBeginThreads), 0, stream>>>(ws->counters, ws->desc, ws->desc_capacity);
        if (hip_failed(hipGetLastError(), "chain_begin_kernel")) return TCR_ERR_HIP;
        dev->ticket_base = 0;
        dev->epoch = 0;
        return TCR_OK;
    }
    ws->epoch += 1;
    dev->ticket_base = ws->tickets_issued;
    dev->epoch = ws->epoch;
    return TCR_OK;
}

// ---------------------------------------------------------------------------- helpers
__global__ void fill_zero_kernel(float* out, uint64_t count) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) out[i] = 0.0f;
}

bool is_pow2(uint64_t v) { return v != 0 && (v & (v - 1)) == 0; }
int log2u(uint64_t v) {
    int l = 0;
    while ((1ull << l) < v) ++l;
    return l;
}
bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

tcr_status check_launch(const char* what) {
    if (hip_failed(hipGetLastError(), what)) return TCR_ERR_HIP;
    return TCR_OK;
}

// ---------------------------------------------------------------------------- reduce dispatch
template <int FORM>
tcr_status launch_reduce_small(const _Float16* in, float* out, uint64_t n, int log2l, hipStream_t s) {
    constexpr int U = kSmallReduceU, W = kSmallReduceW;
    const uint64_t blocks = ceil_div(n, (uint64_t)kTile * U * W);
    const dim3 grid((unsigned)blocks), block(W * kWave);
    switch (log2l) {
        case 4: reduce_small_kernel<FORM, 4, U, W><<<grid, block, 0, s>>>(in, out, n); break;
        case 5: reduce_small_kernel<FORM, 5, U, W><<<grid, block, 0, s>>>(in, out, n); break;
        case 6: reduce_small_kernel<FORM, 6, U, W><<<grid, block, 0, s>>>(in, out, n); break;
        case 7: reduce_small_kernel<FORM, 7, U, W><<<grid, block, 0, s>>>(in, out, n); break;
        case 8: reduce_small_kernel<FORM, 8, U, W><<<grid, block, 0, s>>>(in, out, n); break;
        case 9: reduce_small_kernel<FORM, 9, U, W><<<grid, block, 0, s>>>(in, out, n); break;
        default: return TCR_ERR_UNSUPPORTED;
    }
    return check_launch("reduce_small_kernel");
}

template <int FORM>
tcr_status launch_reduce_span(const _Float16* in, float* dst, uint64_t n, uint64_t span, uint64_t nspans,
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

// ---------------------------------------------------------------------------- tuning table
// The paper selects algorithm, wavefronts per workgroup and coarsening per segment size with an
// auto-tuner (Section 6).  Here the defaults are frozen from sweeps on MI355X; tcr_autotune can
// re-time the candidates on the machine at hand and override the default for one class of
// segment lengths (index log2(seg_len), or kWholeClass for the one-segment operations).
constexpr int kWholeClass = 41;
signed char g_tuned_scan[kWholeClass + 1];
signed char g_tuned_reduce[kWholeClass + 1];
bool g_tuning_initialised = false;
void init_tuning() {
    if (g_tuning_initialised) return;
    std::memset(g_tuned_scan, -1, sizeof(g_tuned_scan));
    std::memset(g_tuned_reduce, -1, sizeof(g_tuned_reduce));
    g_tuning_initialised = true;
}
int tuning_class(uint64_t seg_len, bool whole) { return whole ? kWholeClass : log2u(seg_len); }

// Reduce candidates for seg_len >= 1024 (power of two) or one segment: (span, combine) pairs.
struct ReduceShape { uint64_t span; int combine; };
int reduce_candidates(uint64_t n, uint64_t seg_len, bool whole, ReduceShape* c) {
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
ReducePlan plan_reduce(uint64_t n, uint64_t seg_len, bool whole) {
    init_tuning();
    ReduceShape cand[4];
    const int count = reduce_candidates(n, seg_len, whole, cand);
    int pick = g_tuned_reduce[tuning_class(seg_len, whole)];
    if (pick < 0 || pick >= count) {
        // frozen defaults: segments of 8192 .. 32768 elements are split over 2 or 4 wavefronts
        pick = (whole || seg_len < 8192 || seg_len > 32768) ? 0 : (seg_len == 8192 ? 1 : 2);
    }
    ReducePlan p;
    p.span = cand[pick].span;
    p.combine = cand[pick].combine;
    const uint64_t len = whole ? n : seg_len;
    p.per = ceil_div(len, p.span * (uint64_t)p.combine);
    p.nspans = whole ? ceil_div(n, p.span) : n / p.span;
    return p;
}

tcr_status reduce_long(const _Float16* in, float* out, uint64_t n, uint64_t seg_len, bool whole, hipStream_t s) {
    const ReducePlan p = plan_reduce(n, seg_len, whole);
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
        st = g_variant.formulation == kMfma ? launch_reduce_span<kMfma>(in, dst, n, p.span, p.nspans, p.combine, s, &fin)
                                            : launch_reduce_span<kDpp>(in, dst, n, p.span, p.nspans, p.combine, s, &fin);
        if (st != TCR_OK) {
            ws->dirty = true;
            return st;
        }
        ws->tickets_issued += (uint32_t)(nseg * p.per);   // one count per workgroup
        return TCR_OK;
    }
    tcr_status st = g_variant.formulation == kMfma ? launch_reduce_span<kMfma>(in, dst, n, p.span, p.nspans, p.combine, s)
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
template <int FORM, int MODE>
tcr_status launch_scan_small(const _Float16* in, void* out, uint64_t n, int log2l, hipStream_t s) {
    constexpr int W = kSmallScanW;
    const uint64_t blocks = ceil_div(n, (uint64_t)kTile * W);
    const dim3 grid((unsigned)blocks), block(W * kWave);
    switch (log2l) {
        case 4: scan_small_kernel<FORM, 4, 1, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
        case 5: scan_small_kernel<FORM, 5, 1, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
        case 6: scan_small_kernel<FORM, 6, 1, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
        case 7: scan_small_kernel<FORM, 7, 1, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
        case 8: scan_small_kernel<FORM, 8, 1, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
        case 9: scan_small_kernel<FORM, 9, 1, W, MODE><<<grid, block, 0, s>>>(in, out, n); break;
        default: return TCR_ERR_UNSUPPORTED;
    }
    return check_launch("scan_small_kernel");
}

template <int FORM, int U, int W, int CARRY, int MODE>
void launch_scan_block(const _Float16* in, void* out, uint64_t n, uint64_t seg_mask, uint64_t seg_len,
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
uint64_t scan_shape_tile(int id) { return (uint64_t)kTile * kScanShapes[id].u * kScanShapes[id].w; }

bool scan_shape_valid(int id, uint64_t len, bool whole) {      // len: seg_len, or n for the one-segment scan
    if (id < 0 || id >= kScanShapeCount) return false;
    if (kScanShapes[id].persistent)                             // (whole: len == n, which must be a multiple of 8)
        return g_variant.formulation == kMfma && (whole ? len % 8 == 0 : len >= scan_shape_tile(id));
    return kScanShapes[id].ticket || scan_shape_tile(id) >= len;
}

// Compute units of the current device (cached per device id).
int compute_units() {
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

int default_scan_shape(uint64_t len, bool whole) {
    if (len <= 1024) return 0;
    if (len <= 2048) return 1;
    if (len <= 4096) return 2;
    if (len < 8192 || (whole && len == 8192)) return 3;
    if (!whole && len <= 16384) return 7;          // one ticketed share per segment (two segments of 8192)
    if (scan_shape_valid(10, len, whole)) return 10;   // the pipelined chain: segments of 32768 and more, one segment
    // another formulation, or n not a multiple of 8: scan_block_kernel shares of 65536 / 32768 elements
    return (whole || len >= (1u << 20)) ? 9 : 8;
}

int pick_scan_shape(uint64_t len, bool whole) {
    init_tuning();
    const int tuned = g_tuned_scan[tuning_class(len, whole)];
    return scan_shape_valid(tuned, len, whole) ? tuned : default_scan_shape(len, whole);
}

template <int FORM, int CARRY, int MODE>
void launch_scan_shape(int id, const _Float16* in, void* out, uint64_t n, uint64_t seg_mask, uint64_t seg_len,
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
int nocarry_shape_for(uint64_t fit) {
    for (int id = 0; id < 7; ++id)
        if (scan_shape_tile(id) >= fit) return id;
    return 6;
}

// seg_len >= 1024 (power of two), or the full scan (seg_len == n, any n).
template <int FORM, int MODE>
tcr_status scan_long(const _Float16* in, void* out, uint64_t n, uint64_t seg_len, bool whole, hipStream_t s) {
    const uint64_t seg_mask = whole ? ~0ull : seg_len - 1;
    const uint64_t host_seg_len = seg_len;            // decides the launch; the kernels see a saturated
    if (whole) seg_len = ~0ull;                       // length for the one-segment case (n need not be a power of two)
    const bool table = g_variant.scan_carry != kStrategyLookback;     // the two multi-kernel strategies
    if (table && host_seg_len <= kCarryTile) {
        const ScanWorkspace none = {};
        launch_scan_shape<FORM, kNoCarry, MODE>(nocarry_shape_for(host_seg_len), in, out, n, seg_mask, seg_len, none, nullptr, s);
        return check_launch("scan_block_kernel");
    }
    if (!table) {
        const int shape = pick_scan_shape(host_seg_len, whole);
        if (!kScanShapes[shape].ticket) {
            const ScanWorkspace none = {};
            launch_scan_shape<FORM, kNoCarry, MODE>(shape, in, out, n, seg_mask, seg_len, none, nullptr, s);
            return check_launch("scan_block_kernel");
        }
        const uint64_t tiles = ceil_div(n, scan_shape_tile(shape));
        ScanWorkspace dev = {};
        Workspace* ws = nullptr;
        bool capturing = false;
        tcr_status st = get_workspace(s, &ws, &capturing);
        if (st != TCR_OK) return st;
        st = begin_lookback(ws, s, tiles, &dev, capturing);
        if (st != TCR_OK) return st;
        uint64_t tickets = tiles;                       // scan_block_kernel: one per workgroup
        bool chain = false;
        if constexpr (FORM == kMfma) {
            if (kScanShapes[shape].persistent) {
                const uint64_t resident = (uint64_t)compute_units() * (uint64_t)kScanShapes[shape].persistent;
                const uint64_t groups = tiles < resident ? tiles : resident;
                const dim3 grid((unsigned)groups);
                if (shape == 10)
                    scan_chain_kernel<4, 16, MODE><<<grid, dim3(16 * kWave), 0, s>>>(in, out, n, seg_mask, dev, (uint32_t)tiles);
                else
                    scan_chain_kernel<8, 8, MODE><<<grid, dim3(8 * kWave), 0, s>>>(in, out, n, seg_mask, dev, (uint32_t)tiles);
                tickets = tiles + 3 * groups;           // three drawn at the start of every workgroup, one per tile
                chain = true;
            }
        }
        if (!chain) launch_scan_shape<FORM, kLookback, MODE>(shape, in, out, n, seg_mask, seg_len, dev, nullptr, s);
        st = check_launch(chain ? "scan_chain_kernel" : "scan_block_kernel");
        if (st != TCR_OK) {
            ws->dirty = true;
            return st;
        }
        ws->tickets_issued += (uint32_t)tickets;    // wraps modulo 2^32 like the device counter
        return TCR_OK;
    }
    if (g_variant.scan_carry == kStrategyScanThenPropagate) {
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

// Any other seg_len >= 1: the untuned kernels.
constexpr uint64_t kGenericThreadMax = 96;           // up to here one thread walks a segment, beyond a wavefront does
constexpr uint64_t kMaskedMin = 256;                 // from here on the wavefront walks masked 512-element tiles of the array

template <bool SCAN>
tcr_status launch_generic(const _Float16* in, void* out, uint64_t n, uint64_t seg_len, uint32_t flags, hipStream_t s) {
    const uint64_t nseg = n / seg_len;
    const bool excl = (flags & TCR_SCAN_EXCLUSIVE) != 0, f16 = (flags & TCR_OUT_F16) != 0;
    if (seg_len <= kGenericThreadMax) {
        generic_thread_kernel<SCAN><<<dim3((unsigned)ceil_div(nseg, kGenericThreads)), dim3(kGenericThreads), 0, s>>>(
            in, out, nseg, seg_len, excl, f16);
        return check_launch("generic_thread_kernel");
    }
    if (seg_len < kMaskedMin) {
        generic_wave_kernel<SCAN><<<dim3((unsigned)ceil_div(nseg, kGenericThreads / kWave)), dim3(kGenericThreads), 0, s>>>(
            in, out, nseg, seg_len, excl, f16);
        return check_launch("generic_wave_kernel");
    }
    // masked 512-element tiles of the array, one wavefront per segment
    const dim3 grid((unsigned)ceil_div(nseg, kMaskedWaves)), block(kMaskedWaves * kWave);
    if constexpr (SCAN) {
        switch (flags & 3u) {
            case 0: masked_wave_scan_kernel<0><<<grid, block, 0, s>>>(in, out, nseg, seg_len); break;
            case 1: masked_wave_scan_kernel<1><<<grid, block, 0, s>>>(in, out, nseg, seg_len); break;
            case 2: masked_wave_scan_kernel<2><<<grid, block, 0, s>>>(in, out, nseg, seg_len); break;
            default: masked_wave_scan_kernel<3><<<grid, block, 0, s>>>(in, out, nseg, seg_len); break;
        }
        return check_launch("masked_wave_scan_kernel");
    } else {
        masked_wave_reduce_kernel<<<grid, block, 0, s>>>(in, static_cast<float*>(out), nseg, seg_len);
        return check_launch("masked_wave_reduce_kernel");
    }
}

// The tuned scan paths for one (formulation, mode) pair.
template <int FORM, int MODE>
tcr_status scan_tuned(const _Float16* x, void* out, uint64_t n, uint64_t seg_len, hipStream_t s) {
    if (seg_len == n) return scan_long<FORM, MODE>(x, out, n, n, true, s);
    if (seg_len <= kTile) return launch_scan_small<FORM, MODE>(x, out, n, log2u(seg_len), s);
    return scan_long<FORM, MODE>(x, out, n, seg_len, false, s);
}

tcr_status scan_any(const void* in, void* out, uint64_t n, uint64_t seg_len, uint32_t flags, hipStream_t s) {
    const _Float16* x = static_cast<const _Float16*>(in);
    if (seg_len != n && (!is_pow2(seg_len) || seg_len < 16)) return launch_generic<true>(x, out, n, seg_len, flags, s);
    const int mode = (int)(flags & 3u);
    if (g_variant.formulation == kDpp) {
        // the wavefront-primitive alternative is kept for the default mode only
        if (mode != 0) return TCR_ERR_UNSUPPORTED;
        return scan_tuned<kDpp, 0>(x, out, n, seg_len, s);
    }
    switch (mode) {
        case 0: return scan_tuned<kMfma, 0>(x, out, n, seg_len, s);
        case 1: return scan_tuned<kMfma, 1>(x, out, n, seg_len, s);
        case 2: return scan_tuned<kMfma, 2>(x, out, n, seg_len, s);
        default: return scan_tuned<kMfma, 3>(x, out, n, seg_len, s);
    }
}

tcr_status validate(const void* in, const void* out, uint64_t n, uint64_t seg_len, uintptr_t out_align) {
    if (seg_len == 0) return TCR_ERR_INVALID_ARG;
    if (n % seg_len != 0) return TCR_ERR_INVALID_ARG;
    if (n == 0) return TCR_OK;
    if (in == nullptr || out == nullptr) return TCR_ERR_INVALID_ARG;
    if (!aligned(in, 16) || !aligned(out, out_align)) return TCR_ERR_INVALID_ARG;
    if (n > kMaxElements) return TCR_ERR_UNSUPPORTED;
    return TCR_OK;
}

}  // namespace

// ================================================================================ C ABI

extern "C" tcr_status tcr_segmented_reduce(const void* in, float* out, uint64_t n, uint64_t seg_len, void* stream) {
    tcr_status st = validate(in, out, n, seg_len, 4);
    if (st != TCR_OK || n == 0) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const _Float16* x = static_cast<const _Float16*>(in);
    if (seg_len == n) return reduce_long(x, out, n, n, true, s);
    if (!is_pow2(seg_len) || seg_len < 16) return launch_generic<false>(x, out, n, seg_len, 0u, s);
    if (seg_len <= kTile)
        return g_variant.formulation == kMfma ? launch_reduce_small<kMfma>(x, out, n, log2u(seg_len), s)
                                              : launch_reduce_small<kDpp>(x, out, n, log2u(seg_len), s);
    return reduce_long(x, out, n, seg_len, false, s);
}

extern "C" tcr_status tcr_segmented_scan_ex(const void* in, void* out, uint64_t n, uint64_t seg_len, uint32_t flags,
                                            void* stream) {
    if ((flags & ~(uint32_t)(TCR_SCAN_EXCLUSIVE | TCR_OUT_F16)) != 0) return TCR_ERR_INVALID_ARG;
    tcr_status st = validate(in, out, n, seg_len, 16);
    if (st != TCR_OK || n == 0) return st;
    return scan_any(in, out, n, seg_len, flags, static_cast<hipStream_t>(stream));
}

extern "C" tcr_status tcr_segmented_scan(const void* in, float* out, uint64_t n, uint64_t seg_len, void* stream) {
    return tcr_segmented_scan_ex(in, out, n, seg_len, 0u, stream);
}

extern "C" tcr_status tcr_scan_ex(const void* in, void* out, uint64_t n, uint32_t flags, void* stream) {
    if (n == 0) return (flags & ~(uint32_t)(TCR_SCAN_EXCLUSIVE | TCR_OUT_F16)) ? TCR_ERR_INVALID_ARG : TCR_OK;
    return tcr_segmented_scan_ex(in, out, n, n, flags, stream);
}

extern "C" tcr_status tcr_irregular_reduce(const void* in, const uint64_t* offsets, float* out, uint64_t nseg,
                                           void* stream) {
    if (nseg == 0) return TCR_OK;
    if (in == nullptr || offsets == nullptr || out == nullptr) return TCR_ERR_INVALID_ARG;
    if (!aligned(in, 2) || !aligned(offsets, 8) || !aligned(out, 4)) return TCR_ERR_INVALID_ARG;
    if (nseg > kMaxElements) return TCR_ERR_UNSUPPORTED;
    if (aligned(in, 16)) {                   // 128-bit loads of whole 8-element groups of the array
        masked_irregular_kernel<false><<<dim3((unsigned)ceil_div(nseg, kMaskedWaves)), dim3(kMaskedWaves * kWave), 0,
                                         static_cast<hipStream_t>(stream)>>>(static_cast<const _Float16*>(in), offsets, out, nseg);
        return check_launch("masked_irregular_kernel");
    }
    irregular_wave_kernel<false><<<dim3((unsigned)ceil_div(nseg, kGenericThreads / kWave)), dim3(kGenericThreads), 0,
                                   static_cast<hipStream_t>(stream)>>>(static_cast<const _Float16*>(in), offsets, out, nseg);
    return check_launch("irregular_wave_kernel");
}

extern "C" tcr_status tcr_irregular_scan(const void* in, const uint64_t* offsets, float* out, uint64_t nseg,
                                         void* stream) {
    if (nseg == 0) return TCR_OK;
    if (in == nullptr || offsets == nullptr || out == nullptr) return TCR_ERR_INVALID_ARG;
    if (!aligned(in, 2) || !aligned(offsets, 8) || !aligned(out, 4)) return TCR_ERR_INVALID_ARG;
    if (nseg > kMaxElements) return TCR_ERR_UNSUPPORTED;
    if (aligned(in, 16) && aligned(out, 16)) {
        masked_irregular_kernel<true><<<dim3((unsigned)ceil_div(nseg, kMaskedWaves)), dim3(kMaskedWaves * kWave), 0,
                                        static_cast<hipStream_t>(stream)>>>(static_cast<const _Float16*>(in), offsets, out, nseg);
        return check_launch("masked_irregular_kernel");
    }
    irregular_wave_kernel<true><<<dim3((unsigned)ceil_div(nseg, kGenericThreads / kWave)), dim3(kGenericThreads), 0,
                                  static_cast<hipStream_t>(stream)>>>(static_cast<const _Float16*>(in), offsets, out, nseg);
    return check_launch("irregular_wave_kernel");
}

extern "C" tcr_status tcr_reduce(const void* in, float* out, uint64_t n, void* stream) {
    if (out == nullptr) return TCR_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n == 0) {
        fill_zero_kernel<<<dim3(1), dim3(64), 0, s>>>(out, 1);
        return check_launch("fill_zero_kernel");
    }
    tcr_status st = validate(in, out, n, n, 4);
    if (st != TCR_OK) return st;
    return reduce_long(static_cast<const _Float16*>(in), out, n, n, true, s);
}

extern "C" tcr_status tcr_scan(const void* in, float* out, uint64_t n, void* stream) {
    return tcr_scan_ex(in, out, n, 0u, stream);
}

extern "C" tcr_status tcr_set_variant(const char* key, const char* value) {
    if (key == nullptr || value == nullptr) return TCR_ERR_INVALID_ARG;
    if (std::strcmp(key, "reset") == 0) {
        g_variant = Variant();
        return TCR_OK;
    }
    if (std::strcmp(key, "formulation") == 0) {
        if (std::strcmp(value, "mfma") == 0) g_variant.formulation = kMfma;
        else if (std::strcmp(value, "dpp") == 0) g_variant.formulation = kDpp;
        else return TCR_ERR_INVALID_ARG;
        return TCR_OK;
    }
    if (std::strcmp(key, "scan_carry") == 0) {
        if (std::strcmp(value, "lookback") == 0) g_variant.scan_carry = kStrategyLookback;
        else if (std::strcmp(value, "reduce_then_scan") == 0) g_variant.scan_carry = kStrategyReduceThenScan;
        else if (std::strcmp(value, "scan_then_propagate") == 0) g_variant.scan_carry = kStrategyScanThenPropagate;
        else return TCR_ERR_INVALID_ARG;
        return TCR_OK;
    }
    if (std::strcmp(key, "reduce_finish") == 0) {
        if (std::strcmp(value, "fused") == 0) g_variant.reduce_fused = true;
        else if (std::strcmp(value, "second_kernel") == 0) g_variant.reduce_fused = false;
        else return TCR_ERR_INVALID_ARG;
        return TCR_OK;
    }
    return TCR_ERR_INVALID_ARG;
}

namespace {

// Average time of `reps` back-to-back calls of f on stream s, in microseconds (negative on a HIP error).
template <typename F>
float time_calls(F f, hipStream_t s, int reps) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1.0f;
    float us = -1.0f;
    if (f() == TCR_OK && hipStreamSynchronize(s) == hipSuccess && hipEventRecord(e0, s) == hipSuccess) {
        bool ok = true;
        for (int r = 0; r < reps && ok; ++r) ok = f() == TCR_OK;
        float ms = 0.0f;
        if (ok && hipEventRecord(e1, s) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
            hipEventElapsedTime(&ms, e0, e1) == hipSuccess)
            us = ms * 1000.0f / (float)reps;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return us;
}

}  // namespace

extern "C" tcr_status tcr_autotune(int op, const void* in, float* out, uint64_t n, uint64_t seg_len, void* stream) {
    if (op < 0 || op > 3) return TCR_ERR_INVALID_ARG;
    if (op >= 2) seg_len = n;
    const bool is_scan = (op == 1 || op == 3);
    tcr_status st = validate(in, out, n, seg_len, is_scan ? 16 : 4);
    if (st != TCR_OK) return st;
    if (n == 0) return TCR_OK;
    const bool whole = seg_len == n;
    if (!whole && (!is_pow2(seg_len) || seg_len < 1024)) return TCR_OK;       // a single shape: nothing to choose
    if (whole && n < 1024) return TCR_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    init_tuning();
    const int cls = tuning_class(seg_len, whole);
    signed char* slot = is_scan ? &g_tuned_scan[cls] : &g_tuned_reduce[cls];
    ReduceShape cand[4];
    const int count = is_scan ? kScanShapeCount : reduce_candidates(n, seg_len, whole, cand);
    int best = -1;
    float best_us = 0.0f;
    for (int id = 0; id < count; ++id) {
        if (is_scan && !scan_shape_valid(id, seg_len, whole)) continue;
        if (is_scan && !kScanShapes[id].ticket && scan_shape_tile(id) > 8 * seg_len && !whole) continue;   // far oversized shares
        *slot = (signed char)id;
        const float us = time_calls([&]() -> tcr_status {
            return is_scan ? tcr_segmented_scan(in, out, n, seg_len, stream) : tcr_segmented_reduce(in, out, n, seg_len, stream);
        }, s, 5);
        if (us < 0.0f) {
            *slot = -1;
            return TCR_ERR_HIP;
        }
        if (best < 0 || us < best_us) {
            best = id;
            best_us = us;
        }
    }
    *slot = (signed char)best;
    return TCR_OK;
}

extern "C" uint64_t tcr_tuning_export(char* buffer, uint64_t capacity) {
    init_tuning();
    std::string text;
    for (int c = 0; c <= kWholeClass; ++c) {
        if (g_tuned_scan[c] >= 0) text += "scan:" + std::to_string(c) + "=" + std::to_string((int)g_tuned_scan[c]) + ";";
        if (g_tuned_reduce[c] >= 0) text += "reduce:" + std::to_string(c) + "=" + std::to_string((int)g_tuned_reduce[c]) + ";";
    }
    if (buffer != nullptr && capacity > 0) {
        const uint64_t m = text.size() < capacity - 1 ? text.size() : capacity - 1;
        std::memcpy(buffer, text.data(), m);
        buffer[m] = '\0';
    }
    return text.size() + 1;
}

extern "C" tcr_status tcr_tuning_import(const char* text) {
    if (text == nullptr) return TCR_ERR_INVALID_ARG;
    signed char scan[kWholeClass + 1], reduce[kWholeClass + 1];
    std::memset(scan, -1, sizeof(scan));
    std::memset(reduce, -1, sizeof(reduce));
    const char* p = text;
    while (*p != '\0') {
        const bool is_scan = std::strncmp(p, "scan:", 5) == 0;
        const bool is_reduce = std::strncmp(p, "reduce:", 7) == 0;
        if (!is_scan && !is_reduce) return TCR_ERR_INVALID_ARG;
        p += is_scan ? 5 : 7;
        char* end = nullptr;
        const long cls = std::strtol(p, &end, 10);
        if (end == p || *end != '=' || cls < 0 || cls > kWholeClass) return TCR_ERR_INVALID_ARG;
        p = end + 1;
        const long id = std::strtol(p, &end, 10);
        if (end == p || *end != ';' || id < 0 || id >= (is_scan ? kScanShapeCount : 4)) return TCR_ERR_INVALID_ARG;
        p = end + 1;
        (is_scan ? scan : reduce)[cls] = (signed char)id;
    }
    init_tuning();
    std::memcpy(g_tuned_scan, scan, sizeof(scan));
    std::memcpy(g_tuned_reduce, reduce, sizeof(reduce));
    return TCR_OK;
}

extern "C" const char* tcr_kernel_name(int op, uint64_t n, uint64_t seg_len) {
    if (op == 2 || op == 3) seg_len = n;
    if (n == 0 || seg_len == 0 || n % seg_len != 0) return "";
    const bool mf = g_variant.formulation == kMfma;
    const bool whole = seg_len == n;
    if (!whole && (!is_pow2(seg_len) || seg_len < 16)) {
        if (op != 0 && op != 1) return "";
        if (seg_len <= kGenericThreadMax) return "generic_thread_kernel";
        if (seg_len < kMaskedMin) return "generic_wave_kernel";
        return op == 0 ? "masked_wave_reduce_kernel" : "masked_wave_scan_kernel";
    }
    if (op == 0 || op == 2) {
        if (!whole && seg_len <= kTile) return mf ? "reduce_small_kernel<mfma>" : "reduce_small_kernel<dpp>";
        const ReducePlan p = plan_reduce(n, seg_len, whole);
        if (p.combine == 1) return mf ? "reduce_span_kernel<mfma,wave>" : "reduce_span_kernel<dpp,wave>";
        if (p.per == 1) return mf ? "reduce_span_kernel<mfma,block>" : "reduce_span_kernel<dpp,block>";
        const uint64_t nseg = whole ? 1 : n / seg_len;
        if (g_variant.reduce_fused && nseg * p.per <= kFusedPartialsMax)
            return mf ? "reduce_span_kernel<mfma,block,finish>" : "reduce_span_kernel<dpp,block,finish>";
        return mf ? "reduce_span_kernel<mfma,block>+reduce_final_kernel" : "reduce_span_kernel<dpp,block>+reduce_final_kernel";
    }
    if (op == 1 || op == 3) {
        if (!whole && seg_len <= kTile) return mf ? "scan_small_kernel<mfma>" : "scan_small_kernel<dpp>";
        const bool table = g_variant.scan_carry != kStrategyLookback;
        if (table && seg_len <= kCarryTile)
            return mf ? "scan_block_kernel<mfma,nocarry>" : "scan_block_kernel<dpp,nocarry>";
        if (g_variant.scan_carry == kStrategyScanThenPropagate)
            return mf ? "scan_block_kernel<mfma,nocarry>+gather_totals_kernel+scan_partials_kernel+uniform_add_kernel"
                      : "scan_block_kernel<dpp,nocarry>+gather_totals_kernel+scan_partials_kernel+uniform_add_kernel";
        if (!table) {
            const int shape = pick_scan_shape(seg_len, whole);
            if (kScanShapes[shape].persistent) return "scan_chain_kernel<mfma>";
            if (!kScanShapes[shape].ticket) return mf ? "scan_block_kernel<mfma,nocarry>" : "scan_block_kernel<dpp,nocarry>";
            if (scan_shape_tile(shape) >= seg_len) return mf ? "scan_block_kernel<mfma,ticket>" : "scan_block_kernel<dpp,ticket>";
            return mf ? "scan_block_kernel<mfma,lookback>" : "scan_block_kernel<dpp,lookback>";
        }
        return mf ? "reduce_span_kernel+scan_partials_kernel+scan_block_kernel<mfma,table>"
                  : "reduce_span_kernel+scan_partials_kernel+scan_block_kernel<dpp,table>";
    }
    return "";
}

extern "C" tcr_status tcr_check_device_flags(void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    TCR_HIP(hipStreamSynchronize(s));
    int dev = 0;
    TCR_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_mutex);
    for (auto& kv : g_workspaces) {
        if (kv.first.first != dev || kv.second.counters == nullptr) continue;
        uint32_t flag = 0;
        TCR_HIP(hipMemcpy(&flag, kv.second.counters + 1, sizeof(flag), hipMemcpyDeviceToHost));
        if (flag != 0) {
            g_hip_error = "a look-back wait expired";
            return TCR_ERR_HIP;
        }
    }
    return TCR_OK;
}

extern "C" uint64_t tcr_workspace_bytes(int op, uint64_t n, uint64_t seg_len) {
    if (op < 0 || op > 3 || n == 0) return 0;
    if (op >= 2) seg_len = n;
    if (seg_len == 0 || n % seg_len != 0) return 0;
    // Upper bounds over every variant and launch shape: one 8-byte descriptor per 16384-element share (the
    // smallest share handed out by ticket), one binary32 partial per 16384 elements (the smallest span a
    // reduction leaves a partial for is 65536, as is the share of the multi-kernel scans).
    const uint64_t shares = ceil_div(n, 16384);
    const uint64_t area = (shares * 8 + 255) / 256 * 256;
    return kWorkspaceHeader + 2 * area;
}

extern "C" tcr_status tcr_set_workspace(void* dev_ptr, uint64_t bytes) {
    int dev = 0;
    TCR_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_mutex);
    if (dev_ptr == nullptr) {
        g_caller_workspaces.erase(dev);
        return TCR_OK;
    }
    if (!aligned(dev_ptr, 256) || bytes < kWorkspaceHeader + 512) return TCR_ERR_INVALID_ARG;
    const uint64_t area = (bytes - kWorkspaceHeader) / 2 / 256 * 256;
    Workspace w;
    w.caller_owned = true;
    w.counters = static_cast<uint32_t*>(dev_ptr);
    w.desc = reinterpret_cast<unsigned long long*>(static_cast<char*>(dev_ptr) + kWorkspaceHeader);
    w.desc_capacity = area / 8;
    w.partials = reinterpret_cast<float*>(static_cast<char*>(dev_ptr) + kWorkspaceHeader + area);
    w.partials_capacity = area / 4;
    w.dirty = true;                                   // zeroed by the first call that chains tiles
    w.flag_valid = false;
    g_caller_workspaces[dev] = w;
    return TCR_OK;
}

extern "C" void tcr_release(void) {
    std::lock_guard<std::mutex> lock(g_mutex);
    for (auto& kv : g_workspaces) {
        Workspace& w = kv.second;
        if (w.desc) g_parked_tables.push_back({kv.first.first, w.desc, w.desc_capacity});   // uncached: parked, not freed
        if (w.partials) (void)hipFree(w.partials);
        if (w.counters) (void)hipFree(w.counters);
    }
    g_workspaces.clear();
}

extern "C" const char* tcr_status_string(tcr_status s) {
    switch (s) {
        case TCR_OK: return "ok";
        case TCR_ERR_INVALID_ARG: return "invalid argument";
        case TCR_ERR_UNSUPPORTED: return "unsupported size or variant";
        case TCR_ERR_WORKSPACE: return "workspace allocation failed or caller workspace too small";
        case TCR_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" const char* tcr_last_hip_error(void) { return g_hip_error.c_str(); }
