/*
 * okt.h - C ABI of the Ok-Topk one-GPU hot path for AMD MI355X (gfx950).
 *
 * The library implements, as hand-written HIP kernels, the per-iteration
 * gradient sparsification of Ok-Topk SGD and the local sparse reduction a
 * worker performs on the pieces it receives for its own region of the index
 * space (Li & Hoefler, "Near-Optimal Sparse Allreduce for Distributed Deep
 * Learning", PPoPP'22; Algorithm 1 "O(k) sparse allreduce", Algorithm 2
 * "Ok-Topk SGD").
 *
 * Conventions common to every call
 *   - Pointers named d_* are DEVICE pointers owned by the caller.  The library
 *     allocates and frees nothing, ever; scratch memory comes in through the
 *     d_ws / ws_bytes pair (size it with okt_workspace_bytes; 256-byte aligned;
 *     its contents on entry do not matter and are garbage on exit).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Every call only enqueues work on that stream and returns; no call
 *     synchronises with the host.  Scalar results (threshold, counts) are
 *     written to device memory so that the next call consumes them without a
 *     host round trip.  Two calls that share one workspace must be ordered on
 *     one stream.
 *   - fp32 is IEEE binary32; an index is a uint32; vectors are contiguous.
 *     Dense fp32 vectors must be 16-byte aligned, uint64 outputs 8-byte aligned.
 *   - "Magnitude" order is the order of key(x) = bits(x) & 0x7fffffff, i.e. the
 *     order of |x| for finite x (+-0 lowest; Inf above finite; NaN above Inf).
 *   - Return value: OKT_OK, or a negative okt_status.  Argument errors are found
 *     on the host before anything is launched; then no output is touched.
 *     OKT_ERR_HIP means the HIP runtime refused a launch; okt_last_hip_error
 *     gives its reason.
 *   - Host threads may call the library at the same time as long as the calls
 *     share no workspace and no output buffer; the library keeps no state
 *     between calls.  okt_time_next_kernel and okt_last_hip_error act per
 *     thread, okt_debug_spin_limit and okt_debug_slot_min_n on the whole
 *     process.
 *   - The kernels that place their output through a scan across workgroups
 *     (the select family, the reduce family, the index intersection) wait for
 *     one another through device memory.  Every such wait ends by construction
 *     and is bounded all the same; should one run out, the kernel still exits
 *     normally, every count the call writes (d_nnz_out, d_count_out) is set to
 *     UINT64_MAX and the other outputs are unspecified (all stores stay inside
 *     the buffers).
 */
#ifndef OKT_H
#define OKT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum okt_status {
    OKT_OK = 0,
    OKT_ERR_INVALID_ARG = -1, /* null/misaligned pointer, size out of range    */
    OKT_ERR_WORKSPACE = -2,   /* d_ws missing, misaligned or too small         */
    OKT_ERR_HIP = -3          /* the HIP runtime refused a launch              */
} okt_status;

/* Text for a status code; never NULL; static storage. */
const char* okt_status_string(int status);

/*
 * The HIP runtime's text for the error behind the calling thread's most recent
 * OKT_ERR_HIP ("no error" if there was none); never NULL; static storage.
 */
const char* okt_last_hip_error(void);

/*
 * Test hook: the number of polls a wait between workgroups may take before it
 * gives up, for every call made after this one, process-wide (0 = the built-in
 * limit, about 2^24).  With a limit of 1 a call either completes as usual or
 * reports UINT64_MAX counts as described above; it never hangs or faults.
 */
void okt_debug_spin_limit(uint32_t polls);

/*
 * Test hook: the shortest vector for which the select calls take their
 * three-pass form (per-tile slots in the workspace; see okt_threshold_select),
 * for every call made after this one, process-wide (0 = the built-in lengths).
 * Both forms give the same output; with a length of 1 small test vectors
 * exercise the three-pass form.
 */
void okt_debug_slot_min_n(uint64_t n);

/*
 * The length in force: vectors at least this long take the three-pass form, in
 * the plain selects (accumulating = 0) or in the calls that form the accumulator
 * on the way (okt_accumulate_select, okt_accumulate_topk_select; nonzero).
 */
uint64_t okt_slot_min_n(int accumulating);

/*
 * Measurement hook.  The next call this thread makes records `start_event` right
 * before and `stop_event` right after the launch of its main kernel (hipEvent_t
 * passed as void*; either may be NULL), on the stream of that call - the kernel
 * that moves the data, not the small launches around it (clearing of scan state,
 * slice table, histogram bookkeeping): okt_residual_accumulate, the select
 * family, okt_accumulate_select, the pass of okt_accumulate_topk_select that
 * forms the accumulator, okt_region_partition, the tile kernel of the reduce
 * family, the collect pass of okt_topk_threshold_exact (not recorded when that
 * call takes its unsampled path), the intersect kernel.  The pair is used
 * once and forgotten; a call that launches no such kernel (an argument error, an
 * empty input) leaves it armed for the next one.  For benchmarks: so that an
 * event time can be compared with a profiler's kernel duration.
 */
void okt_time_next_kernel(void* start_event, void* stop_event);

/*
 * Measurement only: two kernels that do none of the method's work and show what
 * plain streaming reaches on the GPU at hand, to be timed beside the hot path
 * (okt_time_next_kernel brackets them like the others).
 *   okt_stream_copy  d_dst[i] = d_src[i], i < n: 4 B read + 4 B written per element.
 *   okt_stream_sum   reads d_src[0..n) once and writes OKT_STREAM_SUM_PARTIALS
 *                    partial sums (fp32, summation order unspecified) to
 *                    d_partials_out: 4 B read per element.
 * Device pointers, 16-byte aligned (d_partials_out: 4); the buffers must not
 * overlap; n < 2^32; n == 0 is a no-op for the copy and writes zeros for the sum.
 * Returns OKT_ERR_INVALID_ARG before any launch otherwise.
 */
#define OKT_STREAM_SUM_PARTIALS 2048
int okt_stream_copy(const float* d_src, float* d_dst, uint64_t n, void* stream);
int okt_stream_sum(const float* d_src, uint64_t n, float* d_partials_out, void* stream);

/*
 * Measurement only: the memory traffic of okt_sparse_reduce_batch without its
 * arithmetic.  Arguments as okt_sparse_reduce_batch (no counts, no dense copy):
 * the region is cut into the same tiles, the same kernel builds the same table of
 * slice boundaries, and then one workgroup per tile reads every entry of the
 * tile's slices once - short sorted runs of (index, value) pairs scattered over
 * d_idx_cat / d_val_cat - and writes it to d_idx_out / d_val_out[j * capacity + p],
 * p being the entry's position among region j's input entries (entries beyond
 * `capacity` are dropped).  Nothing is summed, ranked or scanned: the time of this
 * call is what the reduce's access pattern alone costs on the GPU at hand.
 * okt_time_next_kernel brackets the tile kernel, as for the reduce.
 */
int okt_stream_gather(const uint32_t* d_idx_cat, const float* d_val_cat,
                      const uint64_t* d_chunk_off, const uint32_t* d_lo_hi, uint32_t B, uint32_t P,
                      uint32_t max_width, uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                      void* d_ws, size_t ws_bytes, void* stream);

/* Library version, major * 10000 + minor * 100 + patch. */
int okt_version(void);

/*
 * Bytes of workspace that suffice for every call below on vectors of at most
 * n_max elements, reductions over regions at most n_max wide and at most P_max
 * contributions: about 2 bytes per element of n_max (candidates of the exact
 * threshold with their indices, and the per-tile slots of the three-pass
 * selects), plus the reduce's slice table.  Pure host arithmetic.
 */
size_t okt_workspace_bytes(uint64_t n_max, uint32_t P_max);

/*
 * Accumulate residuals (Algorithm 2, line 4):  acc[i] = eps[i] + lr * G[i].
 *   d_grad            in   fp32[n]  the stochastic gradient G
 *   d_residual_inout  in   fp32[n]  the residual eps of the previous iteration
 *                     out  fp32[n]  the accumulator acc, in place
 *   lr                the learning rate alpha
 * Arithmetic: fp32 multiply rounded, then fp32 add rounded (never fused);
 * subnormals kept.  n = 0 is a no-op.  n must be below 2^32.
 */
int okt_residual_accumulate(const float* d_grad, float* d_residual_inout, float lr,
                            uint64_t n, void* stream);

/*
 * Exact local top-k threshold (Algorithm 1, lines 2-4, th_re_evaluate; Sec.
 * 3.1.3: the k-th largest value, which the paper obtains by sorting; here an
 * exact radix select on the magnitude keys).
 *   d_acc            in   fp32[n]
 *   k                1 <= k <= n < 2^32
 *   d_threshold_out  out  fp32[1]   th >= 0 whose key is the k-th largest key,
 *                                   counted with multiplicity
 *   d_count_ge_out   out  uint64[1] #{i : key(acc[i]) >= key(th)}  (>= k; > k
 *                                   only when values tie with the k-th)
 * Integer work only: the result is exact and run-to-run identical.
 * Workspace: okt_workspace_bytes(n, 0); a smaller one (>= 64 KiB) still gives
 * the same result, with more passes over d_acc.
 */
int okt_topk_threshold_exact(const float* d_acc, uint64_t n, uint64_t k,
                             float* d_threshold_out, uint64_t* d_count_ge_out,
                             void* d_ws, size_t ws_bytes, void* stream);

/*
 * Threshold top-k selection, packaging into one consecutive COO buffer and
 * residual update (Sec. 3.1.3: with a threshold at hand the selection is one
 * comparison per element; Sec. 3.1.2 packaging; Algorithm 2, line 6, with
 * `indexes` taken as all locally selected entries).
 *   S = {i : key(acc[i]) >= key(*d_threshold)} in ascending i.
 *   d_acc_inout  in   fp32[n] acc;  out  the residual: +0.0f at the emitted
 *                entries, untouched elsewhere
 *   d_threshold  in   fp32[1] on the device (its sign is ignored)
 *   d_idx_out    out  uint32[capacity]  ascending indices of the emitted entries
 *   d_val_out    out  fp32[capacity]    their values, bit copies of acc
 *   capacity     entries the two output buffers can hold.  If |S| > capacity
 *                only the first `capacity` members of S (in index order) are
 *                emitted and zeroed; the others stay in the residual.
 *   d_nnz_out    out  uint64[2]  {emitted = min(|S|, capacity), |S|}
 * A single pass over acc.  n = 0 gives {0, 0}.  n must be below 2^32.
 * Workspace: okt_workspace_bytes(n, 0).  Two forms give the same output.  One
 * kernel that places its entries through a scan across its workgroups needs
 * only some KiB of it (a descriptor per workgroup) and is what a short vector,
 * or a call with less than the full workspace, gets.  For a long vector (okt_slot_min_n and up) with the full workspace the
 * call makes three passes: a streaming one with no scan in it, which sets what
 * every 1024 elements select aside in the workspace, a scan over the counts, and
 * a short one that moves the entries to their places; only the first touches
 * the vector as a whole.  okt_threshold_select_copy, okt_accumulate_select and
 * okt_accumulate_topk_select have the same two forms.
 */
int okt_threshold_select(float* d_acc_inout, uint64_t n, const float* d_threshold,
                         uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                         uint64_t* d_nnz_out, void* d_ws, size_t ws_bytes, void* stream);

/*
 * okt_threshold_select for callers that cannot allocate or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments without d_ws / ws_bytes, same results bit for bit;
 * always the one-kernel form of okt_threshold_select (a fill kernel that clears
 * the scan state, then the select kernel), whatever the length.  The scan state
 * lives in an array of
 * OKT_SELECT_NOALLOC_SCRATCH_BYTES of device memory that is part of the library
 * (every GPU the library runs on holds its own copy until the process ends);
 * the call allocates and frees nothing.
 *   - The device current on the calling thread must be the one `stream` and the
 *     buffers belong to.  The first call on a device asks the runtime where the
 *     array lives there, so make it outside any stream capture.
 *   - The array suffices for every n the interface allows on GPUs with up to 1024
 *     compute units; a vector that would need more scan state than it holds is
 *     refused with OKT_ERR_WORKSPACE before anything is launched.
 *   - All calls on one GPU share the array (each call clears the part it uses
 *     with a fill kernel first): calls that overlap in time on one GPU - two
 *     streams, two host threads - race.  Order them on one stream.
 */
#define OKT_SELECT_NOALLOC_SCRATCH_BYTES (144 * 1024)
int okt_threshold_select_noalloc(float* d_acc_inout, uint64_t n, const float* d_threshold,
                                 uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                                 uint64_t* d_nnz_out, void* stream);

/*
 * The same selection and packaging without the residual update: d_acc is only
 * read.  For callers that follow Algorithm 2, line 6 to the letter and zero the
 * entries of `indexes` (the locally selected entries that reached the global
 * top-k) after the allreduce, with okt_index_intersect_zero; the pass then has
 * no scattered store into the dense vector.  Outputs as okt_threshold_select.
 */
int okt_threshold_select_copy(const float* d_acc, uint64_t n, const float* d_threshold,
                              uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                              uint64_t* d_nnz_out, void* d_ws, size_t ws_bytes, void* stream);

/*
 * The accumulate and the threshold selection of one iteration in a single pass,
 * for the iterations that reuse a threshold (Sec. 3.1.3: the threshold is
 * re-evaluated only every tau' iterations, so in between it is known before the
 * accumulator is).  Same result, bit for bit, as okt_residual_accumulate
 * followed by okt_threshold_select with the same arguments:
 *   acc = eps + lr * G (two roundings); S = {i : key(acc[i]) >= key(*d_threshold)};
 *   outputs as in okt_threshold_select; d_residual_inout ends as acc with +0.0f
 *   at the emitted entries.
 * d_grad and d_residual_inout must not overlap.  Moves 12 B per element and 8 B
 * per selected entry; the residual is written once, densely.
 */
int okt_accumulate_select(const float* d_grad, float* d_residual_inout, float lr, uint64_t n,
                          const float* d_threshold, uint32_t* d_idx_out, float* d_val_out,
                          uint64_t capacity, uint64_t* d_nnz_out, void* d_ws, size_t ws_bytes,
                          void* stream);

/*
 * A whole iteration that re-evaluates the threshold (Algorithm 1, lines 2-4;
 * Algorithm 2, lines 4-6) while reading the gradient and the residual once.
 * Same results, bit for bit, as okt_residual_accumulate, okt_topk_threshold_exact
 * on the accumulator with the same k, and okt_threshold_select with that
 * threshold and the same capacity:
 *   d_threshold_out, d_count_ge_out   as in okt_topk_threshold_exact
 *   d_idx_out, d_val_out, d_nnz_out   as in okt_threshold_select
 *   d_residual_inout                  ends as acc with +0.0f at the emitted entries
 * 1 <= k <= n < 2^32; d_grad and d_residual_inout must not overlap.
 * With a workspace of okt_workspace_bytes(n, .) and n of four million or more,
 * the pass that forms the accumulator also sets aside, in index order, every
 * element above a bound read off a sample; the exact selection and the final
 * select then run over those candidates (a few percent of the vector), and only
 * the emitted entries are zeroed in the residual with scattered stores: 12 B per
 * element instead of 20.  A shorter vector, a smaller workspace (the minimum is
 * what the three calls need), or a sample that misled take the three steps over
 * the whole vector: the results are the same.
 */
int okt_accumulate_topk_select(const float* d_grad, float* d_residual_inout, float lr, uint64_t n,
                               uint64_t k, float* d_threshold_out, uint64_t* d_count_ge_out,
                               uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                               uint64_t* d_nnz_out, void* d_ws, size_t ws_bytes, void* stream);

/*
 * Balanced split of the index space [0, n) into R regions by the local top-k
 * entries (Algorithm 1, lines 5-7, space_repartition; Sec. 3.1.1: every worker
 * derives region boundaries that give each region an equal share of its own
 * top-k entries), and the split of the sorted COO buffer by those boundaries.
 *   d_idx         in   uint32[*d_nnz] ascending (the output of
 *                      okt_threshold_select)
 *   d_nnz         in   uint64[1] on the device (d_nnz_out of the select works).
 *                      A count above n - the all-ones word of a select whose
 *                      bounded wait gave up - is never used to address d_idx: the
 *                      call then writes the equal split b[r] = floor(r * n / R)
 *                      and sets every offset to UINT64_MAX
 *   R             number of regions, >= 1
 *   d_bounds_out  out  uint32[R+1]  b[0] = 0, b[R] = n,
 *                      b[r] = idx[floor(r * nnz / R)]; if nnz = 0 the equal
 *                      split b[r] = floor(r * n / R)
 *   d_offsets_out out  uint64[R+1]  off[r] = first COO position whose index is
 *                      >= b[r]; off[R] = nnz.  Region r owns COO entries
 *                      [off[r], off[r+1]); the counts differ by at most one.
 * Averaging the boundary vectors over workers is a collective and not part of
 * this library.  1 <= n < 2^32.
 */
int okt_region_partition(const uint32_t* d_idx, const uint64_t* d_nnz, uint64_t n,
                         uint32_t R, uint32_t* d_bounds_out, uint64_t* d_offsets_out,
                         void* stream);

/*
 * Local reduction over one region (Algorithm 1, line 8, the "reduce" of
 * split_and_reduce; Sec. 3.1.1: worker i sums the sparse pieces it receives for
 * region i).  Plain sum, no 1/P.
 *   d_idx_cat, d_val_cat  in  the P contributions back to back; contribution p is
 *                         the slice [d_chunk_off[p], d_chunk_off[p+1]); inside a
 *                         contribution indices are strictly ascending (anything
 *                         else is undefined behaviour); entries outside [lo, hi)
 *                         are skipped, so whole-space COO buffers may be passed
 *   d_chunk_off           in  uint64[P+1] on the device, non-decreasing
 *   P                     1 <= P <= 65535
 *   lo, hi                the region, lo <= hi
 *   d_idx_out, d_val_out  out uint32/fp32[capacity]: every index present in any
 *                         contribution inside the region (also when the sum is
 *                         zero), ascending, with the sum of its values.  Sums are
 *                         accumulated in fp64 and rounded once to fp32; the order
 *                         of the fp64 additions is not fixed.
 *   capacity              entries the output can hold; the union is truncated to
 *                         its first `capacity` members.  It is also taken as the
 *                         estimate of the union's size from which the kernel's
 *                         tile width is chosen: a capacity far from the real size
 *                         costs speed, never correctness
 *   d_nnz_out             out uint64[2] {emitted, size of the union}
 *   d_dense_out_or_null   out fp32[hi-lo] the region densified (absent = +0.0f),
 *                         or NULL
 */
int okt_sparse_reduce(const uint32_t* d_idx_cat, const float* d_val_cat,
                      const uint64_t* d_chunk_off, uint32_t P, uint32_t lo, uint32_t hi,
                      uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                      uint64_t* d_nnz_out, float* d_dense_out_or_null,
                      void* d_ws, size_t ws_bytes, void* stream);

/*
 * The same reduction with the contributions given as P arbitrary slices
 * [d_seg_begin[p], d_seg_end[p]) of d_idx_cat / d_val_cat (both uint64[P] on the
 * device; an end below its begin reads as an empty slice).  This is the shape of
 * a reduction that takes its contributions in buckets and overlaps with the
 * exchange (Sec. 3.1.1, bucketing): the partial result of the buckets so far is
 * one more slice of the next call.  With two buffers in turn nothing is copied:
 * a call writes its output to the front of the other buffer, where the pieces of
 * the next bucket are received behind it, and its d_nnz_out points at the end
 * word of that slice (begin 0, so the emitted count is the end; the word after it
 * takes the total, so the partial result is listed last and the vector has one
 * spare word).  Each call rounds its sums to fp32 once; over K buckets a value is
 * rounded K times.
 */
int okt_sparse_reduce_segments(const uint32_t* d_idx_cat, const float* d_val_cat,
                               const uint64_t* d_seg_begin, const uint64_t* d_seg_end,
                               uint32_t P, uint32_t lo, uint32_t hi, uint32_t* d_idx_out,
                               float* d_val_out, uint64_t capacity, uint64_t* d_nnz_out,
                               float* d_dense_out_or_null, void* d_ws, size_t ws_bytes,
                               void* stream);

/*
 * The same reduction for B independent regions in one launch (all regions a
 * worker owns in one bucket, or the regions of several simulated workers).
 * Region j has P contributions described by d_chunk_off[j*(P+1) .. j*(P+1)+P]
 * (absolute positions in d_idx_cat / d_val_cat), bounds d_lo_hi[2j], d_lo_hi[2j+1]
 * (uint32 on the device) and writes its output at position j * capacity of
 * d_idx_out / d_val_out, its counts at d_nnz_out[2j..2j+1], and, if
 * d_dense_out_or_null is given, its densified region at element j * max_width.
 * Every region must be at most max_width wide (wider is an invalid argument the
 * kernel reports by setting both counts of that region to UINT64_MAX).
 * 1 <= B <= 65535.  Workspace: okt_sparse_reduce_batch_workspace_bytes(B, P, max_width).
 */
size_t okt_sparse_reduce_batch_workspace_bytes(uint32_t B, uint32_t P, uint32_t max_width);

int okt_sparse_reduce_batch(const uint32_t* d_idx_cat, const float* d_val_cat,
                            const uint64_t* d_chunk_off, const uint32_t* d_lo_hi,
                            uint32_t B, uint32_t P, uint32_t max_width,
                            uint32_t* d_idx_out, float* d_val_out, uint64_t capacity,
                            uint64_t* d_nnz_out, float* d_dense_out_or_null,
                            void* d_ws, size_t ws_bytes, void* stream);

/*
 * Global top-k selection on the reduced sparse values of the own region
 * (Sec. 3.1.2, "balance and allgatherv": each worker selects the global top-k
 * values from the reduced top-k values of its region by the global threshold and
 * packages them, with their indexes, into a consecutive buffer; Algorithm 1,
 * line 13, the local part).  The threshold comparison of okt_threshold_select
 * over a sorted COO list instead of a dense vector; the input is not modified.
 *   d_idx_in, d_val_in  in  uint32/fp32[max_nnz]  the reduced region (the output
 *                       of okt_sparse_reduce); d_val_in 16-byte aligned
 *   d_nnz_in            in  uint64[1] on the device: entries present; more than
 *                       max_nnz is read as max_nnz
 *   max_nnz             host-side bound of *d_nnz_in (sizes the launch), < 2^32
 *   d_threshold         in  fp32[1] the global threshold (its sign is ignored)
 *   d_idx_out, d_val_out out uint32/fp32[capacity]  the entries j, in order, with
 *                       key(val[j]) >= key(*d_threshold); bit copies
 *   d_nnz_out           out uint64[2] {emitted = min(selected, capacity), selected}
 * Workspace: okt_workspace_bytes(max_nnz, 0).  max_nnz = 0 gives {0, 0}.
 * The global threshold itself (Algorithm 1, lines 9-12) is
 * okt_topk_threshold_exact applied to the value array of the gathered reduced
 * entries; the gather is a collective and not part of this library.
 */
int okt_coo_threshold_select(const uint32_t* d_idx_in, const float* d_val_in,
                             const uint64_t* d_nnz_in, uint64_t max_nnz,
                             const float* d_threshold, uint32_t* d_idx_out, float* d_val_out,
                             uint64_t capacity, uint64_t* d_nnz_out, void* d_ws,
                             size_t ws_bytes, void* stream);

/*
 * indexes = local top-k indexes intersected with the global top-k indexes
 * (Algorithm 1, line 14), and the residual update eps = acc - acc(indexes)
 * (Algorithm 2, line 6) completed on a residual that okt_threshold_select or
 * okt_accumulate_select left with ALL locally selected entries zeroed: a locally
 * selected entry whose index is not among the global top-k indexes did not
 * contribute to the applied update, so its value is written back.
 *   d_residual_inout  in/out fp32[n]  on exit +0.0f exactly at `indexes`
 *   d_local_idx, d_local_val  in  the sorted COO the select emitted
 *   d_local_nnz       in  uint64[1] on the device (d_nnz_out of the select);
 *                     more than max_local is read as max_local
 *   d_global_idx      in  uint32[...] ascending: the indexes of the global top-k
 *                     values u_t (all regions, as the allgatherv returns them)
 *   d_global_nnz      in  uint64[1] on the device, clamped to max_global
 *   max_local, max_global  host-side bounds (< 2^32) of the two counts
 *   d_indexes_out_or_null  out uint32[max_local] the intersection, ascending;
 *                     NULL if only the residual is wanted
 *   d_count_out       out uint64[1] the size of the intersection
 * Local indices must be strictly ascending and below n, global indices ascending
 * (anything else is undefined, except that an index >= n is never written to).
 * Workspace: okt_workspace_bytes(max_local, 0).
 */
int okt_index_intersect_restore(float* d_residual_inout, uint64_t n,
                                const uint32_t* d_local_idx, const float* d_local_val,
                                const uint64_t* d_local_nnz, uint64_t max_local,
                                const uint32_t* d_global_idx, const uint64_t* d_global_nnz,
                                uint64_t max_global, uint32_t* d_indexes_out_or_null,
                                uint64_t* d_count_out, void* d_ws, size_t ws_bytes,
                                void* stream);

/*
 * The same `indexes`, applied to an accumulator that was left untouched by
 * okt_threshold_select_copy: eps = acc with +0.0f written at `indexes`
 * (Algorithm 2, line 6, literally).  Arguments as okt_index_intersect_restore,
 * without the local values.  Ends in the same residual, bit for bit, as
 * okt_threshold_select followed by okt_index_intersect_restore.
 */
int okt_index_intersect_zero(float* d_acc_inout, uint64_t n, const uint32_t* d_local_idx,
                             const uint64_t* d_local_nnz, uint64_t max_local,
                             const uint32_t* d_global_idx, const uint64_t* d_global_nnz,
                             uint64_t max_global, uint32_t* d_indexes_out_or_null,
                             uint64_t* d_count_out, void* d_ws, size_t ws_bytes, void* stream);

/*
 * The communication scheme of the data-balancing step before the allgatherv of
 * the global top-k values (Sec. 3.1.2, "balance and allgatherv": each worker uses
 * the gathered buffer sizes to generate which chunk is sent to which worker), and
 * the rule for taking the step at all (Sec. 5.3: when the largest buffer is more
 * than four times the average).  HOST pointers; pure host arithmetic, no GPU.
 *   h_sizes          in   uint64[P]  entries in each worker's packed buffer (< 2^32)
 *   h_triggered_out  out  1 if max(sizes) * P > 4 * sum(sizes), else 0
 *   h_plan_out       out  the chunks, in list order, if triggered (else none):
 *                         the P buffers in worker order are one list of T entries,
 *                         which is re-cut into consecutive pieces of floor or ceil
 *                         T / P entries, worker j getting list positions
 *                         [floor(j T / P), floor((j+1) T / P)).  A chunk says that
 *                         `count` entries from position src_offset of worker src's
 *                         old buffer become the entries from position dst_offset of
 *                         worker dst's new buffer; src == dst is the part a worker
 *                         keeps (possibly shifted).  The order of the list, hence
 *                         of the indexes, is kept.
 *   plan_capacity    chunks h_plan_out can hold; 2 P - 1 always suffice, fewer is
 *                    OKT_ERR_INVALID_ARG if the plan does not fit
 *   h_plan_len_out   out  number of chunks written
 * Moving the chunks is communication and not part of this library.
 */
typedef struct okt_chunk {
    uint32_t src, dst;
    uint64_t src_offset, dst_offset, count;
} okt_chunk;

int okt_balance_plan(const uint64_t* h_sizes, uint32_t P, okt_chunk* h_plan_out,
                     uint32_t plan_capacity, uint32_t* h_plan_len_out, int* h_triggered_out);

#ifdef __cplusplus
}
#endif
#endif /* OKT_H */
