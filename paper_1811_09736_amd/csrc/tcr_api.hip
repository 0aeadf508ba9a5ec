// C ABI of the library (declared in include/tcr.h), part 3 of 3 of the host side: argument validation and
// the exported entry points.  The workspace lives in tcr_workspace.hpp, the dispatch in tcr_dispatch.hpp.
#include "tcr_dispatch.hpp"

using namespace tcr;
using namespace tcr::host;

// ================================================================================ C ABI
// ================================================================================ C ABI

extern "C" tcr_status tcr_segmented_reduce(const void* in, float* out, uint64_t n, uint64_t seg_len, void* stream) {
    tcr_status st = validate(in, out, n, seg_len, 4);
    if (st != TCR_OK || n == 0) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const _Float16* x = static_cast<const _Float16*>(in);
    // the tuned kernels load 128 bits at a time; an input that is not aligned for that takes the fixed tiles laid
    // out from the 16-byte boundary below it
    if (!aligned(in, 16)) {
        if (aligned(in, 4) && packed_reduce_takes(seg_len)) return launch_packed_reduce(x, out, nullptr, n, seg_len, kSum, s);
        if (rows_reduce_takes(seg_len)) return launch_rows_reduce(x, out, nullptr, n, seg_len, kSum, s);    // (any length it fits)
        return launch_irregular_reduce(x, nullptr, out, n, n / seg_len, seg_len, s);
    }
    if (seg_len == n) return reduce_long(x, out, n, n, true, s);
    if (!is_pow2(seg_len) || seg_len < 16) return launch_generic<false>(x, out, n, seg_len, 0u, s);
    if (seg_len <= kTile)
        return tuned_formulation(kTuneReduce, log2u(seg_len)) == kMfma ? launch_reduce_small<kMfma>(x, out, n, log2u(seg_len), s)
                                                                       : launch_reduce_small<kDpp>(x, out, n, log2u(seg_len), s);
    return reduce_long(x, out, n, seg_len, false, s);
}

extern "C" tcr_status tcr_segmented_scan_ex(const void* in, void* out, uint64_t n, uint64_t seg_len, uint32_t flags,
                                            void* stream) {
    if ((flags & ~(uint32_t)(TCR_SCAN_EXCLUSIVE | TCR_OUT_F16 | TCR_ACC_F16)) != 0) return TCR_ERR_INVALID_ARG;
    if ((flags & TCR_ACC_F16) && !(flags & TCR_OUT_F16)) return TCR_ERR_INVALID_ARG;     // a binary16 accumulator has binary16 results
    tcr_status st = validate(in, out, n, seg_len, (flags & TCR_OUT_F16) ? 2 : 4);
    if (st != TCR_OK || n == 0) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (flags & TCR_ACC_F16) {
        const _Float16* x = static_cast<const _Float16*>(in);
        _Float16* y = static_cast<_Float16*>(out);
        return (flags & TCR_SCAN_EXCLUSIVE) ? scan_half<1>(x, y, n, seg_len, s) : scan_half<0>(x, y, n, seg_len, s);
    }
    if (!aligned(in, 16) || !aligned(out, 16)) {
        // arrays that are not aligned for 128-bit accesses: the fixed tiles, laid out from the boundary below `in`
        const _Float16* x = static_cast<const _Float16*>(in);
        switch (flags & 3u) {
            case 0: return launch_irregular_scan<0>(x, nullptr, out, n, n / seg_len, seg_len, s);
            case 1: return launch_irregular_scan<1>(x, nullptr, out, n, n / seg_len, seg_len, s);
            case 2: return launch_irregular_scan<2>(x, nullptr, out, n, n / seg_len, seg_len, s);
            default: return launch_irregular_scan<3>(x, nullptr, out, n, n / seg_len, seg_len, s);
        }
    }
    return scan_any(in, out, n, seg_len, flags, s);
}

extern "C" tcr_status tcr_segmented_scan(const void* in, float* out, uint64_t n, uint64_t seg_len, void* stream) {
    return tcr_segmented_scan_ex(in, out, n, seg_len, 0u, stream);
}

// ------------------------------------------------------------------------------ the call that allocates nothing
// Device memory of the allocation-free scan: a workspace laid out like a caller-supplied one -- a 256-byte header
// (ticket counter, give-up flag, two state words), a descriptor area and a partials area -- in a file-scope
// array, one copy per GPU, held until the process ends.  Host code never uses the array's name as an address:
// the address on each device comes from hipGetSymbolAddress, once, with that device current.
constexpr uint64_t kStaticMaxElements = 1ull << 30;
constexpr uint64_t kStaticDescriptors = kStaticMaxElements / 16384;       // the smallest share handed out by ticket
constexpr uint64_t kStaticPartials = kStaticMaxElements / kCarryTile;     // binary32 totals of the multi-kernel strategies
constexpr uint64_t kStaticBytes = kWorkspaceHeader + kStaticDescriptors * 8 + kStaticPartials * 4;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {
constexpr int kMaxDevices = 64;
Workspace g_static_workspace[kMaxDevices];        // host-side bookkeeping of each device's copy of `scratch`
bool g_static_ready[kMaxDevices] = {};

// The workspace over the current device's copy of `scratch`; its address is looked up on the first call there.
tcr_status static_workspace(Workspace** out) {
    int dev = 0;
    TCR_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return TCR_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    Workspace& w = g_static_workspace[dev];
    if (!g_static_ready[dev]) {
        unsigned char* ptr = nullptr;
        TCR_HIP(hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)));
        if (ptr == nullptr || !aligned(ptr, 256)) return TCR_ERR_HIP;
        w = Workspace();
        w.caller_owned = true;                        // never grown, never freed
        w.clear_in_stream = true;                     // cleared by a kernel on the call's stream, not from the host
        w.counters = reinterpret_cast<uint32_t*>(ptr);
        w.desc = reinterpret_cast<unsigned long long*>(ptr + kWorkspaceHeader);
        w.desc_capacity = kStaticDescriptors;
        w.partials = reinterpret_cast<float*>(ptr + kWorkspaceHeader + kStaticDescriptors * 8);
        w.partials_capacity = kStaticPartials;
        w.dirty = true;                               // the first call that chains tiles clears it
        w.flag_valid = false;
        g_static_ready[dev] = true;
    }
    *out = &w;
    return TCR_OK;
}
}  // namespace

extern "C" tcr_status tcr_segmented_scan_noalloc(const void* in, float* out, uint64_t n, uint64_t seg_len, void* stream) {
    const tcr_status valid = validate(in, out, n, seg_len, 4);
    if (valid != TCR_OK || n == 0) return valid;
    if (n > kStaticMaxElements) {
        g_hip_error = "tcr_segmented_scan_noalloc: n exceeds 2^30 elements, the size its fixed device scratch is laid out for";
        return TCR_ERR_UNSUPPORTED;
    }
    Workspace* ws = nullptr;
    const tcr_status st = static_workspace(&ws);
    if (st != TCR_OK) return st;
    g_forced_workspace = ws;
    const tcr_status result = tcr_segmented_scan_ex(in, out, n, seg_len, 0u, stream);
    g_forced_workspace = nullptr;
    return result;
}

extern "C" tcr_status tcr_scan_ex(const void* in, void* out, uint64_t n, uint32_t flags, void* stream) {
    if (n == 0) {
        if (flags & ~(uint32_t)(TCR_SCAN_EXCLUSIVE | TCR_OUT_F16 | TCR_ACC_F16)) return TCR_ERR_INVALID_ARG;
        return ((flags & TCR_ACC_F16) && !(flags & TCR_OUT_F16)) ? TCR_ERR_INVALID_ARG : TCR_OK;
    }
    return tcr_segmented_scan_ex(in, out, n, n, flags, stream);
}

static tcr_status validate_irregular(const void* in, const uint64_t* offsets, const void* out, uint64_t n, uint64_t nseg,
                                     uintptr_t out_align = 4) {
    if (in == nullptr && n != 0) return TCR_ERR_INVALID_ARG;
    if (offsets == nullptr || out == nullptr) return TCR_ERR_INVALID_ARG;
    if (!aligned(in, 2) || !aligned(offsets, 8) || !aligned(out, out_align)) return TCR_ERR_INVALID_ARG;
    if (nseg > kMaxElements || n > kMaxElements) return TCR_ERR_UNSUPPORTED;
    return TCR_OK;
}

extern "C" tcr_status tcr_irregular_reduce(const void* in, const uint64_t* offsets, float* out, uint64_t n, uint64_t nseg,
                                           void* stream) {
    if (nseg == 0) return TCR_OK;
    const tcr_status st = validate_irregular(in, offsets, out, n, nseg);
    if (st != TCR_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n == 0) {                            // every segment is empty
        fill_zero_kernel<<<dim3((unsigned)ceil_div(nseg, 256)), dim3(256), 0, s>>>(out, nseg);
        return check_launch("fill_zero_kernel");
    }
    return launch_irregular_reduce(static_cast<const _Float16*>(in), offsets, out, n, nseg, 0, s);
}

extern "C" tcr_status tcr_irregular_moments(const void* in, const uint64_t* offsets, float* sum, float* sumsq, uint64_t n,
                                            uint64_t nseg, void* stream) {
    if (nseg == 0) return TCR_OK;
    const tcr_status st = validate_irregular(in, offsets, sum, n, nseg);
    if (st != TCR_OK) return st;
    if (sumsq == nullptr || !aligned(sumsq, 4) || sumsq == sum) return TCR_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (n == 0) {                            // every segment is empty
        fill_zero_kernel<<<dim3((unsigned)ceil_div(nseg, 256)), dim3(256), 0, s>>>(sum, nseg);
        fill_zero_kernel<<<dim3((unsigned)ceil_div(nseg, 256)), dim3(256), 0, s>>>(sumsq, nseg);
        return check_launch("fill_zero_kernel");
    }
    return launch_irregular_reduce(static_cast<const _Float16*>(in), offsets, sum, n, nseg, 0, s, kBoth, sumsq);
}

extern "C" tcr_status tcr_irregular_scan_ex(const void* in, const uint64_t* offsets, void* out, uint64_t n, uint64_t nseg,
                                            uint32_t flags, void* stream) {
    if ((flags & ~(uint32_t)(TCR_SCAN_EXCLUSIVE | TCR_OUT_F16)) != 0) return TCR_ERR_INVALID_ARG;
    if (nseg == 0 || n == 0) return TCR_OK;
    const tcr_status st = validate_irregular(in, offsets, out, n, nseg, (flags & TCR_OUT_F16) ? 2 : 4);
    if (st != TCR_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const _Float16* x = static_cast<const _Float16*>(in);
    switch (flags & 3u) {
        case 0: return launch_irregular_scan<0>(x, offsets, out, n, nseg, 0, s);
        case 1: return launch_irregular_scan<1>(x, offsets, out, n, nseg, 0, s);
        case 2: return launch_irregular_scan<2>(x, offsets, out, n, nseg, 0, s);
        default: return launch_irregular_scan<3>(x, offsets, out, n, nseg, 0, s);
    }
}

extern "C" tcr_status tcr_irregular_scan(const void* in, const uint64_t* offsets, float* out, uint64_t n, uint64_t nseg,
                                         void* stream) {
    return tcr_irregular_scan_ex(in, offsets, out, n, nseg, 0u, stream);
}

extern "C" tcr_status tcr_segmented_moments(const void* in, float* sum, float* sumsq, uint64_t n, uint64_t seg_len,
                                             void* stream) {
    tcr_status st = validate(in, sum, n, seg_len, 4);
    if (st != TCR_OK || n == 0) return st;
    if (sumsq == nullptr || !aligned(sumsq, 4)) return TCR_ERR_INVALID_ARG;
    if (!aligned(in, 16) && aligned(in, 4) && packed_reduce_takes(seg_len))
        return launch_packed_reduce(static_cast<const _Float16*>(in), sum, sumsq, n, seg_len, kBoth, static_cast<hipStream_t>(stream));
    if (!aligned(in, 16) && rows_reduce_takes(seg_len, kBoth))
        return launch_rows_reduce(static_cast<const _Float16*>(in), sum, sumsq, n, seg_len, kBoth, static_cast<hipStream_t>(stream));
    if (!aligned(in, 16))                    // the tiled reduction with both moments as its two channels
        return launch_irregular_reduce(static_cast<const _Float16*>(in), nullptr, sum, n, n / seg_len, seg_len,
                                       static_cast<hipStream_t>(stream), kBoth, sumsq);
    return launch_moments(static_cast<const _Float16*>(in), sum, sumsq, n, seg_len, static_cast<hipStream_t>(stream));
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
    if (!aligned(in, 16)) return launch_irregular_reduce(static_cast<const _Float16*>(in), nullptr, out, n, 1, n, s);
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
    if (std::strcmp(key, "tile_load") == 0) {
        if (std::strcmp(value, "direct") == 0) g_variant.tile_load = kLoadDirect;
        else if (std::strcmp(value, "lds") == 0) g_variant.tile_load = kLoadStaged;
        else if (std::strcmp(value, "lds_dma") == 0) g_variant.tile_load = kLoadLdsDma;
        else return TCR_ERR_INVALID_ARG;
        return TCR_OK;
    }
    if (std::strcmp(key, "irregular_scan") == 0) {
        if (std::strcmp(value, "auto") == 0) g_variant.irregular_scan = 0;
        else if (std::strcmp(value, "single") == 0) g_variant.irregular_scan = 1;
        else if (std::strcmp(value, "chain") == 0) g_variant.irregular_scan = 2;
        else return TCR_ERR_INVALID_ARG;
        return TCR_OK;
    }
    if (std::strcmp(key, "untuned_reduce") == 0) {
        if (std::strcmp(value, "rows") == 0) g_variant.rows_reduce = true;
        else if (std::strcmp(value, "tiles") == 0) g_variant.rows_reduce = false;
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

namespace {

// Times every candidate value of one table entry with `call` and leaves the fastest one there.
// candidates: values (id + 32 * formulation) that are valid for the call at hand.
template <typename F>
tcr_status tune_entry(int table, int cls, const std::vector<int>& candidates, F call, hipStream_t s) {
    init_tuning();
    if (candidates.size() < 2) return TCR_OK;                    // nothing to choose
    signed char* slot = &g_tuned[table][cls];
    int best = -1;
    float best_us = 0.0f;
    for (int v : candidates) {
        *slot = (signed char)v;
        const float us = time_calls(call, s, 5);
        if (us < 0.0f) {
            *slot = -1;
            return TCR_ERR_HIP;
        }
        if (best < 0 || us < best_us) {
            best = v;
            best_us = us;
        }
    }
    *slot = (signed char)best;
    return TCR_OK;
}

}  // namespace

extern "C" tcr_status tcr_autotune(int op, const void* in, float* out, uint64_t n, uint64_t seg_len, void* stream) {
    if (op < 0 || op > 3) return TCR_ERR_INVALID_ARG;
    if (op >= 2) seg_len = n;
    const bool is_scan = (op == 1 || op == 3);
    tcr_status st = validate(in, out, n, seg_len, 4);
    if (st != TCR_OK) return st;
    if (n == 0) return TCR_OK;
    if (!aligned(in, 16) || (is_scan && !aligned(out, 16))) return TCR_ERR_INVALID_ARG;     // the tuned kernels' alignment
    const bool whole = seg_len == n;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const auto call = [&]() -> tcr_status {
        return is_scan ? tcr_segmented_scan(in, out, n, seg_len, stream) : tcr_segmented_reduce(in, out, n, seg_len, stream);
    };
    std::vector<int> cand;
    if (!whole && (!is_pow2(seg_len) || seg_len < 16)) {
        // lengths without a tuned path: which kernel takes them
        if (is_pow2(seg_len) && seg_len <= 8 && (is_scan || seg_len < 4)) return TCR_OK;     // (a single kernel)
        for (int id = 0; id < (is_scan ? (int)kScanAnyCount : (int)kReduceAnyCount); ++id)
            if (is_scan ? scan_any_valid(id, seg_len) : reduce_any_valid(id, seg_len)) cand.push_back(id);
        return tune_entry(is_scan ? kTuneScanAny : kTuneReduceAny, floor_log2(seg_len), cand, call, s);
    }
    const int cls = tuning_class(seg_len, whole);
    // both formulations of the tile arithmetic, unless tcr_set_variant has forced the cross-lane one everywhere
    const int forms = g_variant.formulation == kMfma ? 2 : 1;
    for (int form = 0; form < forms; ++form) {
        const int bit = form ? kTuneFormBit : 0;
        if (!whole && seg_len <= (uint64_t)kTile) {
            for (int id = 0; id < kSmallShapeCount; ++id)
                if (is_scan || small_reduce_shape_valid(id, log2u(seg_len))) cand.push_back(id + bit);
        } else if (is_scan) {
            for (int id = 0; id < kScanIdCount; ++id) {
                if (!scan_shape_valid(id, seg_len, whole)) continue;
                if (id < kScanShapeCount && !kScanShapes[id].ticket && scan_shape_tile(id) > 8 * seg_len && !whole) continue;   // far oversized shares
                cand.push_back(id + bit);
            }
        } else {
            ReduceShape shapes[4];
            const int count = reduce_candidates(n, seg_len, whole, shapes);
            for (int id = 0; id < count; ++id) cand.push_back(id + bit);
        }
    }
    return tune_entry(is_scan ? kTuneScan : kTuneReduce, cls, cand, call, s);
}

extern "C" tcr_status tcr_autotune_irregular(int op, const void* in, const uint64_t* offsets, float* out, uint64_t n, uint64_t nseg,
                                             void* stream) {
    if (op != 4 && op != 5) return TCR_ERR_INVALID_ARG;
    if (nseg == 0 || n == 0) return TCR_OK;
    const tcr_status st = validate_irregular(in, offsets, out, n, nseg);
    if (st != TCR_OK) return st;
    const bool is_scan = op == 5;
    std::vector<int> cand;
    for (int id = 0; id < (is_scan ? kIrregularScanShapeCount : kIrregularReduceShapeCount); ++id) cand.push_back(id);
    return tune_entry(kTuneIrregular, is_scan ? 1 : 0, cand, [&]() -> tcr_status {
        return is_scan ? tcr_irregular_scan(in, offsets, out, n, nseg, stream) : tcr_irregular_reduce(in, offsets, out, n, nseg, stream);
    }, static_cast<hipStream_t>(stream));
}

extern "C" uint64_t tcr_tuning_export(char* buffer, uint64_t capacity) {
    init_tuning();
    std::string text;
    for (int t = 0; t < kTuneTables; ++t)
        for (int c = 0; c <= kWholeClass; ++c)
            if (g_tuned[t][c] >= 0)
                text += std::string(kTuneTableNames[t]) + ":" + std::to_string(c) + "=" + std::to_string((int)g_tuned[t][c]) + ";";
    if (buffer != nullptr && capacity > 0) {
        const uint64_t m = text.size() < capacity - 1 ? text.size() : capacity - 1;
        std::memcpy(buffer, text.data(), m);
        buffer[m] = '\0';
    }
    return text.size() + 1;
}

extern "C" tcr_status tcr_tuning_import(const char* text) {
    if (text == nullptr) return TCR_ERR_INVALID_ARG;
    signed char fresh[kTuneTables][kWholeClass + 1];
    std::memset(fresh, -1, sizeof(fresh));
    // ids a table accepts (a formulation bit on top for the first two); whether an id fits a given length is
    // decided when the class is used, and an id that does not fit falls back to the default
    const int id_limit[kTuneTables] = {kScanIdCount, 4, kScanAnyCount, kReduceAnyCount, 3};
    const char* p = text;
    while (*p != '\0') {
        int table = -1;
        size_t len = 0;
        for (int t = 0; t < kTuneTables; ++t) {
            const size_t l = std::strlen(kTuneTableNames[t]);
            if (std::strncmp(p, kTuneTableNames[t], l) == 0 && p[l] == ':' && l > len) {
                table = t;
                len = l;
            }
        }
        if (table < 0) return TCR_ERR_INVALID_ARG;
        p += len + 1;
        char* end = nullptr;
        const long cls = std::strtol(p, &end, 10);
        if (end == p || *end != '=' || cls < 0 || cls > kWholeClass) return TCR_ERR_INVALID_ARG;
        p = end + 1;
        const long v = std::strtol(p, &end, 10);
        if (end == p || *end != ';' || v < 0 || v >= 2 * kTuneFormBit) return TCR_ERR_INVALID_ARG;
        const bool has_form = table == kTuneScan || table == kTuneReduce;
        if ((v & (kTuneFormBit - 1)) >= id_limit[table] || (!has_form && v >= kTuneFormBit)) return TCR_ERR_INVALID_ARG;
        if (table == kTuneIrregular && cls > 1) return TCR_ERR_INVALID_ARG;
        p = end + 1;
        fresh[table][cls] = (signed char)v;
    }
    init_tuning();
    std::memcpy(g_tuned, fresh, sizeof(fresh));
    return TCR_OK;
}

extern "C" const char* tcr_kernel_name(int op, uint64_t n, uint64_t seg_len) {
    if (op == 4) return n ? "irregular_bounds_kernel+irregular_reduce_kernel+irregular_groups_kernel+irregular_carry_kernel" : "fill_zero_kernel";
    if (op == 5) return n ? "irregular_bounds_kernel+irregular_scan_kernel" : "";
    if (op == 2 || op == 3) seg_len = n;
    if (n == 0 || seg_len == 0 || n % seg_len != 0) return "";
    const bool whole = seg_len == n;
    if (!whole && (!is_pow2(seg_len) || seg_len < 16)) {
        if (op != 0 && op != 1) return "";
        if (op == 0) {
            const int pick = pick_reduce_any(seg_len);
            if (is_pow2(seg_len) && seg_len <= 8 && pick != kReduceAnyPacked && pick != kReduceAnyPackedAlt)
                return "tiny_reduce_kernel";                                         // (16-byte aligned results)
            if (pick == kReduceAnyPacked || pick == kReduceAnyPackedAlt) return "packed_rows_reduce_kernel";
            if (seg_len < kTiledReduceMin) return "generic_thread_kernel";
            if (pick == kReduceAnyRows) return "rows_reduce_kernel";
            if (pick == kReduceAnyTiles || pick == kReduceAnyTilesAlt) return "irregular_reduce_kernel<regular>+irregular_groups_kernel+irregular_carry_kernel";
            return seg_len <= 2 * kWaveSpanMax ? "masked_wave_reduce_kernel" : "masked_span_reduce_kernel+reduce_final_kernel";
        }
        if (is_pow2(seg_len) && seg_len <= 8) return "tiny_scan_kernel";            // (the plain scan; other modes: the tiles)
        const int pick = pick_scan_any(seg_len);
        if (pick == kScanAnyChain) return "scan_chain_kernel<mfma>";
        return pick == kScanAnySegment ? "scan_segment_kernel" : "irregular_scan_kernel<regular>";
    }
    const int cls = tuning_class(seg_len, whole);
    if (op == 0 || op == 2) {
        const bool mf = tuned_formulation(kTuneReduce, cls) == kMfma;
        if (!whole && seg_len <= kTile) return mf ? "reduce_small_kernel<mfma>" : "reduce_small_kernel<dpp>";
        const ReducePlan p = plan_reduce(n, seg_len, whole);
        // <formulation, wave | block (wavefronts of a workgroup combined)>, and what adds up the partials, if any are left
        const uint64_t nseg = whole ? 1 : n / seg_len;
        const bool fused = p.per > 1 && g_variant.reduce_fused && nseg * p.per <= kFusedPartialsMax;
        if (p.combine == 1) {
            if (p.per == 1) return mf ? "reduce_span_kernel<mfma,wave>" : "reduce_span_kernel<dpp,wave>";
            if (fused) return mf ? "reduce_span_kernel<mfma,wave,finish>" : "reduce_span_kernel<dpp,wave,finish>";
            return mf ? "reduce_span_kernel<mfma,wave>+reduce_final_kernel" : "reduce_span_kernel<dpp,wave>+reduce_final_kernel";
        }
        if (p.per == 1) return mf ? "reduce_span_kernel<mfma,block>" : "reduce_span_kernel<dpp,block>";
        if (fused) return mf ? "reduce_span_kernel<mfma,block,finish>" : "reduce_span_kernel<dpp,block,finish>";
        return mf ? "reduce_span_kernel<mfma,block>+reduce_final_kernel" : "reduce_span_kernel<dpp,block>+reduce_final_kernel";
    }
    if (op == 1 || op == 3) {
        const bool mf = tuned_formulation(kTuneScan, cls) == kMfma;
        if (!whole && seg_len <= kTile) return mf ? "scan_small_kernel<mfma>" : "scan_small_kernel<dpp>";
        // the carry strategy as scan_long resolves it
        int strategy = g_variant.scan_carry;
        int shape = strategy == kStrategyLookback ? pick_scan_shape(seg_len, whole) : -1;
        if (shape == kScanIdReduceThenScan) strategy = kStrategyReduceThenScan;
        if (shape == kScanIdScanThenPropagate) strategy = kStrategyScanThenPropagate;
        if (shape == kScanIdChainTail) return mf ? "scan_chain_kernel<mfma>+scan_tail_kernel" : "scan_chain_kernel<dpp>+scan_tail_kernel";
        if (shape >= kScanShapeCount) shape = default_scan_shape(seg_len, whole, mf ? kMfma : kDpp);
        if (shape == kScanIdChainTail) shape = 9;
        const bool table = strategy != kStrategyLookback;
        if (table && seg_len <= kCarryTile)
            return mf ? "scan_block_kernel<mfma,nocarry>" : "scan_block_kernel<dpp,nocarry>";
        if (strategy == kStrategyScanThenPropagate)
            return mf ? "scan_block_kernel<mfma,nocarry>+gather_totals_kernel+scan_partials_kernel+uniform_add_kernel"
                      : "scan_block_kernel<dpp,nocarry>+gather_totals_kernel+scan_partials_kernel+uniform_add_kernel";
        if (!table) {
            if (kScanShapes[shape].persistent) return mf ? "scan_chain_kernel<mfma>" : "scan_chain_kernel<dpp>";
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
    // every workspace of this device whose flag word has been initialised: library-owned, the caller's, the static one
    std::vector<const Workspace*> all;
    for (auto& kv : g_workspaces)
        if (kv.first.first == dev) all.push_back(&kv.second);
    auto own = g_caller_workspaces.find(dev);
    if (own != g_caller_workspaces.end()) all.push_back(&own->second);
    if (dev >= 0 && dev < kMaxDevices && g_static_ready[dev]) all.push_back(&g_static_workspace[dev]);
    for (const Workspace* w : all) {
        if (w->counters == nullptr || !w->flag_valid) continue;
        uint32_t flag = 0;
        TCR_HIP(hipMemcpy(&flag, w->counters + 1, sizeof(flag), hipMemcpyDeviceToHost));
        if (flag != 0) {
            g_hip_error = "a look-back wait expired";
            return TCR_ERR_HIP;
        }
    }
    return TCR_OK;
}

extern "C" uint64_t tcr_workspace_bytes(int op, uint64_t n, uint64_t seg_len) {
    if (op < 0 || op > 7 || n == 0) return 0;
    const bool irregular = op == 4 || op == 5 || op == 7;
    if (op == 2 || op == 3) seg_len = n;
    if (!irregular && (seg_len == 0 || n % seg_len != 0)) return 0;
    const bool scan = op == 1 || op == 3 || op == 5;
    const bool moments = op == 6 || op == 7;
    // A workspace has two areas of equal size: 8-byte tile descriptors, and binary32 partials (which the tiled
    // kernels of the irregular calls use as 8-byte words: look-up tables, carried-segment indices, pairs).
    // The tiled kernels lay their tiles out from the 16-byte boundary below `in`: up to 7 elements more.
    const uint64_t padded = n + 7;
    uint64_t desc = 0, words = 0;
    if (scan) {
        // chained tiles (of the smallest tile shape); two tables of them for the two-kernel scan of irregular segments
        desc = (irregular ? 2 : 1) * irregular_tiles_max(true, padded);
        if (irregular) words = irregular_words_max(true, padded); // where the tile boundaries fall among the offsets
    } else {
        // tables, one carried-segment index and one pair per tile and per group of 64 tiles; the sums of squares
        // add a second set of pairs
        const uint64_t tiles = irregular_tiles_max(false, padded);
        words = irregular_words_max(false, padded) + (moments ? tiles + ceil_div(tiles, kWave) : 0);
    }
    if (!irregular) {
        // Regular calls run the tiled kernels above for some lengths and alignments; otherwise, over every variant
        // and launch shape: one descriptor per 16384-element share (the smallest share handed out by ticket),
        // and at most one binary32 partial per 4096 elements (the smallest span a wavefront of the one-segment
        // reduction leaves a partial for; segmented reductions and the multi-kernel scans leave one per 65536, the
        // moments two).
        const uint64_t shares = ceil_div(n, 16384);
        if (scan && shares > desc) desc = shares;
        const uint64_t partials = ceil_div(n, 4096);
        if (ceil_div(partials, 2) > words) words = ceil_div(partials, 2);
    }
    const uint64_t bytes = 8 * (desc > words ? desc : words);
    return kWorkspaceHeader + 2 * ((bytes + 255) / 256 * 256);
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

extern "C" tcr_status tcr_release_stream(void* stream) {
    int dev = 0;
    TCR_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_workspaces.find(std::make_pair(dev, static_cast<hipStream_t>(stream)));
    if (it == g_workspaces.end()) return TCR_OK;
    Workspace& w = it->second;
    if (w.desc) g_parked_tables.push_back({dev, w.desc, w.desc_capacity});       // uncached: parked, not freed
    if (w.partials) (void)hipFree(w.partials);
    if (w.counters) (void)hipFree(w.counters);
    g_workspaces.erase(it);
    return TCR_OK;
}

extern "C" const char* tcr_status_string(int status) {
    switch (status) {
        case TCR_OK: return "ok";
        case TCR_ERR_INVALID_ARG: return "invalid argument";
        case TCR_ERR_UNSUPPORTED: return "unsupported size or variant";
        case TCR_ERR_WORKSPACE: return "workspace allocation failed or caller workspace too small";
        case TCR_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" const char* tcr_last_hip_error(void) { return g_hip_error.c_str(); }

