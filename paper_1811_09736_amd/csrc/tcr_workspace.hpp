// Host side of the library, part 1 of 3 (included by tcr_api.hip only): error bookkeeping, the variant
// settings, and the per-(device, stream) workspace for cross-workgroup carries.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "../../include/tcr.h"
#include "tcr_reduce.hpp"
#include "tcr_scan.hpp"
#include "tcr_generic.hpp"
#include "tcr_irregular.hpp"
#include "tcr_rows.hpp"
#include "tcr_packed.hpp"
#include "tcr_half.hpp"

namespace tcr {
namespace host {

using namespace tcr;

inline thread_local std::string g_hip_error;

inline bool hip_failed(hipError_t e, const char* what) {
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
    int tile_load = kLoadDirect;    // small power-of-two segments, default shape and mode: how tiles reach the operand registers
    int irregular_scan = 0;         // 0: one kernel or two by the number of segments; 1: always one; 2: always two (where possible)
    bool rows_reduce = true;        // untuned lengths: the row-product kernels (false: the fixed tiles with marked starts)
};
inline Variant g_variant;

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
    bool clear_in_stream = false;   // clean-ups run as a kernel on the call's stream instead of host-side memsets
};

inline std::mutex g_mutex;
inline std::map<std::pair<int, hipStream_t>, Workspace> g_workspaces;
// Caller-supplied workspaces, one per device: [256-byte header: ticket, flag | descriptors | partials],
// the two areas of equal size.  While one is set, every call on that device uses it, whatever its stream.
inline std::map<int, Workspace> g_caller_workspaces;
constexpr uint64_t kWorkspaceHeader = 256;
// Set by an entry point for the duration of one call: the workspace that call must use, whatever the maps hold.
inline thread_local Workspace* g_forced_workspace = nullptr;

// Look-back descriptor tables are allocated uncached (polling them through the L2 path measured
// ~5 % slower on the full scan).  Uncached allocations are never handed back to the runtime:
// a table that is outgrown or released is parked here and reused by the next request it fits.
struct ParkedTable {
    int device;
    unsigned long long* ptr;
    uint64_t capacity;
};
inline std::vector<ParkedTable> g_parked_tables;

inline tcr_status acquire_table(int device, uint64_t tiles, unsigned long long** ptr, uint64_t* capacity) {
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
inline tcr_status get_workspace(hipStream_t stream, Workspace** out, bool* capturing) {
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    TCR_HIP(hipStreamIsCapturing(stream, &capture));
    *capturing = capture != hipStreamCaptureStatusNone;
    if (g_forced_workspace != nullptr) {
        *out = g_forced_workspace;
        return TCR_OK;
    }
    int dev = 0;
    TCR_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_mutex);
    auto own = g_caller_workspaces.find(dev);
    *out = own != g_caller_workspaces.end() ? &own->second : &g_workspaces[std::make_pair(dev, stream)];
    return TCR_OK;
}

inline tcr_status ensure_partials(Workspace* ws, hipStream_t stream, uint64_t floats, bool capturing) {
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
inline tcr_status begin_lookback(Workspace* ws, hipStream_t stream, uint64_t tiles, ScanWorkspace* dev, bool capturing) {
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
        if (ws->clear_in_stream) {
            // a kernel in front of the launch, ordered by the stream: no synchronisation, no runtime memset
            const uint64_t want = (ws->desc_capacity + kClearThreads - 1) / kClearThreads;
            const unsigned blocks = want < 1 ? 1u : (want > 1024 ? 1024u : (unsigned)want);
            workspace_clear_kernel<<<dim3(blocks), dim3(kClearThreads), 0, stream>>>(ws->counters, ws->desc, ws->desc_capacity,
                                                                                     ws->flag_valid ? 1u : 0u);
            if (hip_failed(hipGetLastError(), "workspace_clear_kernel")) return TCR_ERR_HIP;
        } else {
            TCR_HIP(hipStreamSynchronize(stream));
            if (ws->desc_capacity) TCR_HIP(hipMemset(ws->desc, 0, ws->desc_capacity * sizeof(unsigned long long)));
            uint32_t keep_flag = 0;
            if (ws->flag_valid) TCR_HIP(hipMemcpy(&keep_flag, ws->counters + 1, sizeof(uint32_t), hipMemcpyDeviceToHost));
            uint32_t init[4] = {0u, keep_flag, 0u, 0u};
            TCR_HIP(hipMemcpy(ws->counters, init, sizeof(init), hipMemcpyHostToDevice));
        }
        ws->flag_valid = true;
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


}  // namespace host
}  // namespace tcr
