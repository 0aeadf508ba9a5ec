/*
 * tcr -- segmented and full sum-reduction and inclusive prefix scan of IEEE binary16 data
 * with binary32 accumulation and output, for AMD MI355X (gfx950).
 *
 * The operations are the ones defined at the start of Section 3 of "Accelerating Reduction
 * and Scan Using Tensor Core Units" (ICS'19): reduction is the sum of a vector, scan is its
 * vector of running sums (inclusive: first entry = first element, last entry = total), and
 * the regular segmented forms apply them to consecutive pieces of equal length.  They are
 * evaluated the way Sections 4 and 5 describe -- as small matrix products of the data with
 * constant ones / triangular matrices on the matrix cores -- re-derived for CDNA4 MFMA.
 *
 * Conventions common to every call
 *   in      DEVICE pointer to n binary16 values, contiguous, read only.  16-byte aligned for the tuned kernels;
 *           with less (2 bytes at least) the call runs on the fixed tiles of the irregular calls, laid out from
 *           the 16-byte boundary below `in`: up to 7 elements in front of `in` are read and ignored.
 *   out     DEVICE pointer, caller owned, must not overlap `in`.  Scans: 16-byte aligned for the tuned kernels,
 *           at least the alignment of an element otherwise; reductions: 4-byte aligned.
 *   stream  a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *           and return.  They do not wait for the work; the exceptions are the calls that set up or grow a
 *           library-owned workspace (the first chained call on a stream, a larger n, the call after a failed
 *           launch, and one call in 2^30 per workspace), which synchronise the stream once while they allocate
 *           and clear it.  With a caller-supplied workspace only the clearing remains; tcr_segmented_scan_noalloc
 *           never synchronises.
 *   Inputs must be finite.  (A zero entry of a constant matrix times an infinity is NaN, so
 *   non-finite inputs poison outputs that the plain definition would leave finite.)
 *   Results for integer-valued inputs whose partial sums stay below 2^24 in magnitude are
 *   exact.  For other inputs the order of the binary32 additions is unspecified and, for
 *   operations that need a cross-workgroup carry, may differ from run to run.
 *   Argument errors are reported synchronously and nothing is enqueued.  Device-side faults
 *   surface at the caller's next synchronisation.
 *   The library keeps one small workspace per (device, stream), grown on demand by the first
 *   call that needs it; calls issued on one stream are ordered by the stream.  Calls that
 *   share a stream from several host threads must be serialised by the caller.
 *   HIP graphs: every call may be recorded into a graph, provided the workspace it needs exists already: a
 *   call that would have to allocate, grow or initialise workspace while its stream is capturing returns
 *   TCR_ERR_UNSUPPORTED and records nothing (run the same call once outside the capture, or supply a workspace
 *   and run one chained scan on it first).  Calls that use no workspace (scans with seg_len <= 4096, reduces
 *   with seg_len <= 262144 -- powers of two from 16 on; default variant and tuning) never do.
 *   From the first recorded chained scan on, the workspace keeps its launch counters on the device and every
 *   chained scan on it, recorded or not, is preceded by one small bookkeeping kernel.  The "fused"
 *   reduce_finish variant cannot be recorded.
 *   There is no CPU fallback: without a usable HIP device every call returns TCR_ERR_HIP.
 */
#ifndef TCR_H
#define TCR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TCR_OK = 0,
    TCR_ERR_INVALID_ARG = 1,   /* null / misaligned pointer, seg_len == 0, n % seg_len != 0 */
    TCR_ERR_UNSUPPORTED = 2,   /* a size or variant this build has no kernel for */
    TCR_ERR_WORKSPACE = 3,     /* workspace allocation failed, or the caller's workspace is too small */
    TCR_ERR_HIP = 4            /* a HIP runtime call failed (see tcr_last_hip_error) */
} tcr_status;

/*
 * Regular segmented sum reduction (Section 3; algorithms of Section 4).
 *   out[s] = sum_{k < seg_len} in[s*seg_len + k],  s = 0 .. n/seg_len - 1.
 * out: n/seg_len floats, 4-byte aligned.  n == 0 is a no-op.  seg_len must divide n.
 * Every seg_len >= 1 is accepted; the tuned paths are the powers of two from 16 upwards and
 * seg_len == n.  Other lengths: reductions of 3 to 30 elements that pack into rows of an even number of at most 32
 * elements (every even length that is no power of two, 4 and 8, odd ones up to 15) take one product per 16 such rows with a masked constant matrix
 * (the masking that Section 4 proposes for arbitrary segment sizes; `in` 4-byte aligned, no workspace);
 * reductions of 17 to 8160 elements otherwise take whole segments per workgroup and mask the data operand of the
 * products row by row where a segment ends (the same masking moved from the constant matrix to the data; no
 * workspace); reductions of 5 to 15 elements from arrays that are not 4-byte aligned and all scans run on fixed
 * tiles of the array with the segment starts marked (the kernels of the
 * irregular calls below; they use the workspace), except scans of a multiple of 8 elements from 65536 on (the
 * chained scan) and of a multiple of 64 elements up to 8192 that fills a workgroup's tiles to four fifths (one
 * workgroup per segment; the tuning table can give it every multiple of 8 between 520 and 65528); longer
 * reductions run one wavefront per
 * segment (per 65536-element piece of one, from 131072 elements) over zero-masked tiles of the array, the
 * paper's padding of such segments (Section 4) applied in registers.
 */
tcr_status tcr_segmented_reduce(const void *in, float *out, uint64_t n, uint64_t seg_len, void *stream);

/*
 * Regular segmented inclusive scan (Section 3; algorithms of Section 5).
 *   out[s*seg_len + k] = sum_{j <= k} in[s*seg_len + j].
 * out: n floats.  n == 0 is a no-op.  seg_len must divide n.
 * Every seg_len >= 1 is accepted, as for tcr_segmented_reduce.
 */
tcr_status tcr_segmented_scan(const void *in, float *out, uint64_t n, uint64_t seg_len, void *stream);

/*
 * tcr_segmented_scan for callers that cannot allocate device memory: code under HIP graph capture set-ups, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same results (binary32 inclusive scan, every
 * seg_len >= 1 that divides n, seg_len == n for the full scan), same kernels -- but the workspace of the chained
 * kernels (ticket counter, per-tile descriptors, totals of the multi-kernel variants) is a fixed array in the
 * library's own device image: 256 + 2^16 * 8 + 2^14 * 4 bytes (about 0.56 MiB), present on every GPU the library
 * runs on until the process ends.  The call never calls hipMalloc / hipFree or a routine that allocates, and
 * never synchronises: what must start from zero is cleared by a small kernel on `stream` in front of the first
 * launch that needs it (and again after a failed launch or 2^30 launches).
 *   n <= 2^30 elements; more returns TCR_ERR_UNSUPPORTED and enqueues nothing.
 *   All calls on one GPU share that GPU's array, which keeps the last call's counters: calls on one GPU must be
 *   ordered (one stream, or events between streams); calls that overlap on one GPU race.  Not for use by several
 *   host threads at once on one GPU.  tcr_set_workspace does not affect it.
 */
tcr_status tcr_segmented_scan_noalloc(const void *in, float *out, uint64_t n, uint64_t seg_len, void *stream);

/*
 * Scan variants.  flags is a combination of
 *   TCR_SCAN_EXCLUSIVE  out[s*seg_len + k] = sum_{j < k} in[s*seg_len + j] (the first output of a segment
 *                       is 0): the exclusive scan that Section 5 uses for its column scans;
 *   TCR_OUT_F16         results are rounded (to nearest even) to binary16 and `out` points to n binary16
 *                       values -- the paper's own output precision (Section 6 counts 4 bytes per scanned
 *                       element).  Accumulation stays binary32; sums beyond 65504 become infinities.
 *   TCR_ACC_F16         (with TCR_OUT_F16 only) the ACCUMULATOR is binary16 as well, the half-precision mode of
 *                       the paper's matrix units (Section 2.2): every addition rounds to binary16.  The gfx950
 *                       binary16 MFMA accumulates in binary32 only, so this mode runs on cross-lane adds; the
 *                       additions form a tree, so a result equals the left-to-right binary16 scan bit for bit
 *                       only while no addition rounds (all sums of consecutive elements of a segment are
 *                       binary16 values, e.g. integers within +-2048); otherwise each output has gone through
 *                       at most 40 roundings of relative size 2^-11 (a running count of ones stalls at 2048, as
 *                       it does for any binary16 accumulator).  Powers of two and seg_len == n, 16-byte aligned
 *                       arrays; TCR_ERR_UNSUPPORTED otherwise.
 * flags == 0 is tcr_segmented_scan / tcr_scan.  out: n elements.  Unknown flag bits (and TCR_ACC_F16 without
 * TCR_OUT_F16)
 * return TCR_ERR_INVALID_ARG.  Under the "dpp" formulation only flags == 0 has tuned kernels
 * (TCR_ERR_UNSUPPORTED otherwise); segment lengths without a tuned path accept every flag.
 */
#define TCR_SCAN_EXCLUSIVE 1u
#define TCR_OUT_F16 2u
#define TCR_ACC_F16 4u
tcr_status tcr_segmented_scan_ex(const void *in, void *out, uint64_t n, uint64_t seg_len, uint32_t flags, void *stream);
tcr_status tcr_scan_ex(const void *in, void *out, uint64_t n, uint32_t flags, void *stream);

/*
 * Irregular segments (the paper pads them to regular ones, footnote in Section 3; here the segment
 * boundaries are read directly).  Segment s is in[offsets[s] .. offsets[s+1]); offsets is a DEVICE pointer to
 * nseg + 1 non-decreasing element indices, 8-byte aligned, none larger than n; empty segments are allowed.
 * n is the number of elements of `in` (and of `out` for the scan): the launch is sized by it, the segments
 * may cover any part [offsets[0], offsets[nseg]) of it.
 *   tcr_irregular_reduce  out[s] = sum of segment s (0 for an empty one); out: nseg floats.
 *   tcr_irregular_scan    out[k] = sum of in[offsets[s] .. k] for k in segment s; out is indexed like `in`
 *                         (positions outside [offsets[0], offsets[nseg]) are not written).
 * The work is divided by elements, not by segments: fixed tiles of the array at a speed that hardly depends on
 * the mix of segment lengths.  Both use the workspace (tcr_workspace_bytes, op 4 and 5): one small kernel looks
 * up where the tile boundaries fall among the offsets; the scan chains its tiles like the long regular scans
 * (with fewer segments than a quarter of the tiles it runs as two kernels: the pipelined chain of the long
 * regular scans takes the tiles without a segment start, a second kernel the others);
 * the reduction keeps its tiles independent and two small kernels add the one sum per tile that reaches in
 * from earlier tiles -- plain loads in a fixed order, so the reduction's results are the same from run to run.
 * in and out need only their natural alignment (2 and 4 bytes): the tiles start at the 16-byte boundary at or
 * below `in` (up to 7 elements in front of it are read and ignored), and a scan whose `out` does not sit at the
 * same distance from a 16-byte boundary stores its results one by one (slower).
 * The offsets are not validated (they live on the device): entries that decrease or exceed n give wrong
 * results for the segments they bound, never an access outside in[0 .. n), beyond those leading elements,
 * and the outputs.  nseg == 0 is a no-op.
 */
tcr_status tcr_irregular_reduce(const void *in, const uint64_t *offsets, float *out, uint64_t n, uint64_t nseg, void *stream);
tcr_status tcr_irregular_scan(const void *in, const uint64_t *offsets, float *out, uint64_t n, uint64_t nseg, void *stream);
/* The scan with the flags of tcr_segmented_scan_ex (exclusive, binary16 output; out: n elements, aligned to
 * their size). */
tcr_status tcr_irregular_scan_ex(const void *in, const uint64_t *offsets, void *out, uint64_t n, uint64_t nseg, uint32_t flags,
                                 void *stream);

/*
 * First two moments of every segment: the statistics of a normalisation layer, which the paper's conclusion
 * (Section 7) names as the next use of reductions on matrix cores.
 *   sum[s] = sum_{k < seg_len} x,   sumsq[s] = sum_{k < seg_len} x^2,   x = in[s*seg_len + k].
 * sum, sumsq: n/seg_len floats each, 4-byte aligned, distinct.  Every seg_len >= 1 that divides n, including
 * seg_len == n.  The sums of squares come from products of the data with itself on the matrix cores (exact
 * products, binary32 accumulation); both are exact for integer-valued inputs while the sums stay below 2^24.
 * Powers of two up to 512: a tile per wavefront like the reductions; 3 to 30 elements that pack into rows of an
 * even number of at most 32 elements: the masked constant matrix of tcr_segmented_reduce for the sums, and for the
 * squares one product per segment of a row, of the row's elements of that segment with the row; other lengths
 * from 17 to 2999: whole segments per workgroup with the data operand masked row by row, the squares from the
 * masked operand times itself; 8 to 15 elements from arrays that are not 4-byte aligned: the fixed tiles of the
 * irregular kernels with both moments in one pass (they use the workspace); longer ones: one wavefront per segment
 * (per 65536-element piece of a long one).
 */
tcr_status tcr_segmented_moments(const void *in, float *sum, float *sumsq, uint64_t n, uint64_t seg_len, void *stream);
/* The same for irregular segments (offsets, n, nseg as for tcr_irregular_reduce; empty segments give 0 and 0):
 * both moments in one pass over the fixed tiles. */
tcr_status tcr_irregular_moments(const void *in, const uint64_t *offsets, float *sum, float *sumsq, uint64_t n, uint64_t nseg,
                                 void *stream);

/*
 * Full reduction (device level, Section 4): out[0] = sum of all n inputs (0 for n == 0).
 * Any n is accepted.  out: 1 float.
 */
tcr_status tcr_reduce(const void *in, float *out, uint64_t n, void *stream);

/*
 * Full inclusive scan (device level, Section 5): out[k] = sum_{j <= k} in[j].
 * Any n is accepted.  out: n floats.
 */
tcr_status tcr_scan(const void *in, float *out, uint64_t n, void *stream);

/*
 * Bench / test hook: choose among measured alternatives.  Keys and values:
 *   "formulation"  "mfma" (default: matrix-core products) | "dpp" (cross-lane wavefront primitives)
 *   "scan_carry"   "lookback" (default: single pass, decoupled look-back) | "reduce_then_scan" |
 *                  "scan_then_propagate" (the paper's three-kernel device-level scan, Section 5;
 *                  plain binary32 inclusive scan only)
 *   "tile_load"    "direct" (default: every lane loads its matrix-core operand straight from memory) | "lds" (lanes
 *                  load in lane order, stage the tile in LDS and read their operand back: the staging of the
 *                  paper's own kernels) | "lds_dma" (the same with gfx950's load from memory into LDS).  Applies
 *                  to tcr_segmented_reduce / tcr_segmented_scan with seg_len 16 .. 512 in their default launch
 *                  shape; kept for the measurement that chose "direct"
 *   "untuned_reduce" "rows" (default: reductions and moments of 3 .. 8160 elements, no power of two, as products
 *                  over rows of whole segments or masked rows of the array) | "tiles" (the fixed tiles with marked
 *                  segment starts / one thread or one wavefront per segment that took these lengths before; kept
 *                  as the measured alternative)
 *   "irregular_scan" "auto" (default: one kernel or two by the number of segments) | "single" (always the one
 *                  kernel of chained tiles) | "chain" (always two, where the launch allows it: default tile shape,
 *                  16-byte aligned arrays, matrix-core formulation)
 *   "reduce_finish" "second_kernel" (default: the paper's two-kernel device-level reduction, Section 4) |
 *                  "fused" (one kernel: the workgroup that finishes last adds up the partials)
 *   "reset"        any value: back to the defaults
 * Returns TCR_ERR_INVALID_ARG for an unknown key or value.  Process-wide; not thread safe.
 */
tcr_status tcr_set_variant(const char *key, const char *value);

/*
 * Auto-tuning (the paper picks algorithm, wavefronts per workgroup and coarsening per segment size with an
 * auto-tuner, Section 6).  The library ships with choices frozen from sweeps on MI355X; tcr_autotune re-times
 * every candidate for this (op, n, seg_len) on the caller's buffers -- op: 0 segmented_reduce, 1 segmented_scan,
 * 2 reduce, 3 scan (seg_len ignored) -- and makes the fastest one the choice for that class of segment lengths
 * for the rest of the process.  What is searched, per class:
 *   powers of two from 16 to 512 (class log2(seg_len)): tiles per wavefront and wavefronts per workgroup of the
 *     small-segment kernels, and the formulation (matrix cores or cross-lane adds);
 *   longer powers of two and the one-segment operations (class 41): the launch shape -- scans: 12 shapes of
 *     share size, ticketed or not, persistent chain or not, plus the two multi-kernel carry strategies of
 *     tcr_set_variant("scan_carry"); reductions: span per wavefront and wavefronts combined -- and the formulation;
 *   every other length (class floor(log2(seg_len))): which kernel takes it -- scans: fixed tiles with marked
 *     starts (two tile shapes), one workgroup per segment, the chain on a per-segment tile grid; reductions: rows
 *     of whole segments (two launch shapes), masked row products, fixed tiles (two shapes), one wavefront per
 *     segment over masked tiles.
 * tcr_autotune_irregular does the same for the tile shape of tcr_irregular_reduce (op 4; also used by
 * tcr_irregular_moments) and tcr_irregular_scan (op 5) on the caller's offsets.
 * Both SYNCHRONISE the stream and overwrite `out` with (correct) results several times; they are no-ops where
 * there is a single candidate.  Every candidate gives the same results up to the order of binary32 additions.
 * tcr_tuning_export writes the current choices as text -- "table:class=value;" items, tables scan, reduce,
 * scan_any, reduce_any, irregular (class 0 reduce, 1 scan); value = candidate id, plus 32 in the first two tables
 * when the class runs the cross-lane formulation -- NUL terminated, truncated to `capacity`, and returns the
 * size needed; tcr_tuning_import replaces the choices with such a text (TCR_ERR_INVALID_ARG if it does not
 * parse; the empty string restores the defaults; an id that does not fit a length falls back to the default
 * when that length is used).  Not thread safe.
 */
tcr_status tcr_autotune(int op, const void *in, float *out, uint64_t n, uint64_t seg_len, void *stream);
tcr_status tcr_autotune_irregular(int op, const void *in, const uint64_t *offsets, float *out, uint64_t n, uint64_t nseg,
                                  void *stream);
uint64_t tcr_tuning_export(char *buffer, uint64_t capacity);
tcr_status tcr_tuning_import(const char *text);

/*
 * Name of the kernel the dispatcher would launch for (op, n, seg_len) under the current
 * variant settings; op is 0 = segmented_reduce, 1 = segmented_scan, 2 = reduce, 3 = scan,
 * 4 = irregular_reduce, 5 = irregular_scan (seg_len is ignored).  The arrays are taken to be 16-byte aligned
 * (regular calls on arrays that are not run irregular_reduce_kernel<regular> / irregular_scan_kernel<regular>).
 * Returns a static string ("" when nothing would be launched); never NULL.
 */
const char *tcr_kernel_name(int op, uint64_t n, uint64_t seg_len);

/*
 * Waits for `stream` and reports whether any scan kernel issued so far on the current
 * device gave up waiting for a predecessor tile's carry (a bounded wait of 2^20 polls that should never
 * expire: every predecessor holds an earlier ticket and is running).  A kernel that gives up leaves wrong
 * results behind and the call that launched it has long returned TCR_OK; this is the only place where it
 * shows.  Covers library-owned workspaces, the caller's and the fixed one of tcr_segmented_scan_noalloc.
 * Returns TCR_OK if none did, TCR_ERR_HIP otherwise.  Synchronises; for tests.
 */
tcr_status tcr_check_device_flags(void *stream);

/*
 * Caller-supplied workspace, for callers that manage device memory themselves.
 * tcr_workspace_bytes: an upper bound, over every variant, launch shape and pointer alignment, of the workspace a
 *   call with these arguments can need (op as for tcr_kernel_name, and 6 = segmented_moments,
 *   7 = irregular_moments; 0 for arguments no call accepts).
 * tcr_set_workspace: from now on every call on the CURRENT device uses [dev_ptr, dev_ptr + bytes) instead of
 *   library-owned memory, whatever its stream, and allocates nothing; a call that needs more returns
 *   TCR_ERR_WORKSPACE.  dev_ptr: device memory, 256-byte aligned, at least 768 bytes, contents arbitrary (the
 *   first call that chains tiles synchronises its stream once and clears it); it stays the caller's and must
 *   outlive the calls that use it.  One buffer serves one stream at a time: calls that use it must be ordered
 *   by their streams or by the caller.  dev_ptr == NULL returns the device to library-owned workspaces.
 *   TCR_ERR_INVALID_ARG for a misaligned or too small buffer.
 */
uint64_t tcr_workspace_bytes(int op, uint64_t n, uint64_t seg_len);
tcr_status tcr_set_workspace(void *dev_ptr, uint64_t bytes);

/* Releases every library-owned workspace.  The caller must have synchronised all streams.
 * The (small, uncached) look-back tables are kept for reuse until the process ends. */
void tcr_release(void);
/* Releases the library-owned workspace of `stream` on the current device (a no-op if it has none): the library
 * keeps one per (device, stream) until told otherwise, so a caller that creates and destroys streams freely calls
 * this before destroying one.  The caller must have synchronised the stream. */
tcr_status tcr_release_stream(void *stream);

/* Text for a status code (any int: values that are no tcr_status give "unknown status"). */
const char *tcr_status_string(int status);

/* Text of the last HIP error seen by this library on the calling thread ("" if none). */
const char *tcr_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TCR_H */
