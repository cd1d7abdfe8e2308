/*
 * gtopk.h - C ABI of the gTop-k S-SGD data-parallel hot path for MI355X (gfx950).
 *
 * The library computes, for P simulated workers whose gradient buffers all
 * live on one GPU, the three parts of one gTop-k S-SGD iteration
 * (paper: Algorithm 4, "gTopKAllReduce based S-SGD"):
 *
 *   1. local selection        Algorithm 4 lines 4-8
 *   2. gTopKAllReduce         Algorithm 3 lines 1-18, built from the Top-k
 *                             operation of Definition 1, then the average of Eq. 3
 *   3. extra residual         Algorithm 3 lines 19-23 (broadcast and gMask, which
 *                             on one GPU reduce to "all workers read one global
 *                             index set") and Algorithm 4 line 10
 *
 * Conventions, for every entry point:
 *   - Every pointer argument is a DEVICE pointer owned by the caller.  The
 *     library never allocates, frees or keeps device memory; temporary storage
 *     comes from the caller's workspace `ws` (size from the *_workspace_bytes
 *     query; contents need no initialisation and are clobbered).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     A call only enqueues kernels on `stream` and returns; it never
 *     synchronises with the host.  Two calls that share a workspace must be
 *     ordered (same stream, or an event between them).
 *   - Values are IEEE-754 binary32 (the paper trains in fp32: note under
 *     Table III).  Every add is one round-to-nearest fp32
 *     add; denormals are not flushed.  Magnitude |v| is compared on the integer
 *     `bits(v) & 0x7fffffff`.  "Top k" means: the first k entries under the
 *     total order (|v| descending, index ascending) - exactly k entries, the
 *     lower index winning among equal magnitudes.
 *   - A sparse k-set is two arrays, indices (uint32, ascending, distinct) and
 *     values (float), k entries each.
 *   - Return value: GTOPK_OK (0) when the work was enqueued, a negative
 *     gtopk_status otherwise; on an argument error nothing is enqueued.
 *     Argument errors are found on the host, without touching the GPU.
 *   - Not checked (results unspecified, but no access outside the given sizes):
 *     NaN/Inf inputs; unsorted, duplicate or out-of-range indices in
 *     caller-provided k-sets (an entry whose index is >= m is skipped where it
 *     would be written to a row).  Buffers must not overlap each other.
 */
#ifndef GTOPK_H_
#define GTOPK_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GTOPK_OK = 0,
    GTOPK_EINVAL = -1,     /* null pointer; m < 1 or m > 2^31; k < 1 or k > m; k > 2^30 where
                              sets are merged (gtopk_merge, gtopk_tree, and the step calls
                              with P > 1: a merged pair has 2k slots); P < 1, P > 32768 or not
                              a power of two (the paper assumes a power of two, Section III);
                              stride < m; batch < 1 or batch > 32767; k-set stride < k;
                              copies < 1 or > 65535 (gtopk_apply_update); P > 1024
                              (gtopk_topk_allreduce, which takes any P from 1 on)            */
    GTOPK_EWORKSPACE = -2, /* ws_bytes smaller than the matching *_workspace_bytes query   */
    GTOPK_EALIGN = -3,     /* a pointer is not 16-byte aligned                              */
    GTOPK_EHIP = -4        /* a kernel launch failed (hipGetLastError)                      */
} gtopk_status;

/* Human-readable name of a status code (static string, never NULL). */
const char* gtopk_status_string(int status);

/* Bytes of workspace that gtopk_local_select, gtopk_tree, gtopk_residual_restore
 * and gtopk_step need for these sizes.  Returns 0 if the sizes are invalid. */
size_t gtopk_workspace_bytes(int64_t m, int32_t k, int32_t P);

/* Bytes of workspace gtopk_merge needs for `batch` pairs of k-sets (0 if invalid). */
size_t gtopk_merge_workspace_bytes(int32_t k, int32_t batch);

/*
 * Local selection, Algorithm 4 lines 4-8, for P workers at once.
 *
 *   grad      [P rows] in : fresh gradients; row w starts at grad + w*stride, m floats
 *   residual  [P rows] i/o: G_{i-1} on entry.  On return row w holds
 *                           acc = residual + grad (line 4) with the k selected
 *                           entries replaced by +0.0 (line 8)
 *   m, stride             : elements per worker and distance between rows (>= m)
 *   out_idx   [P][k] out  : indices of the k selected entries of each worker, ascending
 *   out_val   [P][k] out  : acc at those indices, bit for bit (line 7)
 *   m : 1 .. 2^31;  k : 1 .. m;  P : a power of two, 1 .. 32768 (the limit of the step
 *   calls, whose workspace this call shares);  ws : gtopk_workspace_bytes(m, k, P) bytes
 */
int gtopk_local_select(const float* grad, float* residual, int64_t m, int64_t stride,
                       int32_t P, int32_t k, uint32_t* out_idx, float* out_val,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * The Top-k operation of Definition 1 on `batch` independent pairs of k-sets:
 * out[b] = a[b] TOP b[b].  The candidates are the union of the two index sets;
 * at an index held by both operands the two values are added (one fp32 add), at
 * an index held by one its value is kept unchanged; the top k of the union are
 * written index-ascending.  Always exactly k entries.
 *
 *   a_idx/a_val, b_idx/b_val : set b of each operand starts at + b*in_stride (elements)
 *   out_idx/out_val          : result b starts at + b*out_stride
 *   in_stride, out_stride    : >= k
 */
int gtopk_merge(const uint32_t* a_idx, const float* a_val,
                const uint32_t* b_idx, const float* b_val,
                int32_t k, int32_t batch, int64_t in_stride,
                uint32_t* out_idx, float* out_val, int64_t out_stride,
                void* ws, size_t ws_bytes, void* stream);

/*
 * gTopKAllReduce, Algorithm 3 lines 1-18, over the P workers' k-sets, followed
 * by the division by P of Eq. 3.  Round j (j = 0 .. log2 P - 1) merges worker i
 * with worker i + 2^j for every i that is a multiple of 2^(j+1); the result of
 * the last round is what rank 0 would broadcast (line 19).
 *
 *   loc_idx, loc_val [P][k] in : the workers' local k-sets (not modified)
 *   g_idx, g_val     [k]   out : the global k-set; values are the tree's sums / P
 *   P : a power of two, 1 .. 32768;  k : 1 .. 2^30;  ws : gtopk_workspace_bytes(k, k, P) bytes
 *       or more (any m >= k gives enough)
 */
int gtopk_tree(const uint32_t* loc_idx, const float* loc_val, int32_t P, int32_t k,
               uint32_t* g_idx, float* g_val, void* ws, size_t ws_bytes, void* stream);

/*
 * Extra residual, Algorithm 4 line 10, for P workers at once: every locally
 * selected entry whose INDEX is not in the global set (gMask, Algorithm 3 lines
 * 21-22) is added back: residual[w][loc_idx[w][t]] += loc_val[w][t].
 * Needs no workspace.
 */
int gtopk_residual_restore(float* residual, int64_t m, int64_t stride, int32_t P, int32_t k,
                           const uint32_t* loc_idx, const float* loc_val,
                           const uint32_t* g_idx, void* stream);

/*
 * One whole iteration of the hot path: gtopk_local_select, gtopk_tree and
 * gtopk_residual_restore in sequence, with bit-identical results.
 * loc_idx / loc_val may be NULL (then the local k-sets stay in the workspace).
 * Small problems (P <= 64, k <= 512, P*k <= 4096, m <= 2^20 - 3) run as four kernels: the
 * speculative threshold of a worker in one block, the streaming pass, the exact local
 * selection of a worker in one block, the whole tree with the average and the extra
 * residual in one block.
 *   m : 1 .. 2^31;  k : 1 .. m (and <= 2^30 if P > 1);  P : a power of two, 1 .. 32768;
 *   stride >= m;  ws : gtopk_workspace_bytes(m, k, P) bytes
 */
int gtopk_step(const float* grad, float* residual, int64_t m, int64_t stride,
               int32_t P, int32_t k, uint32_t* g_idx, float* g_val,
               uint32_t* loc_idx, float* loc_val,
               void* ws, size_t ws_bytes, void* stream);

/*
 * gtopk_step with every worker's speculative threshold carried from one call to the next.
 * The local selection (Algorithm 4 lines 5-7) first filters each row with a threshold
 * that is only a guess of the k-th largest magnitude, then selects exactly among what
 * passed; gtopk_step takes that guess from a sample of the row on every call.  In training
 * the k-th largest magnitude of a worker moves little from one iteration to the next, so
 * here the exact value found by one call, extrapolated and lowered by a margin, serves the
 * next call, and the sampling kernels have nothing to do for that worker.  Results are
 * bit-identical to gtopk_step whatever the carried threshold is worth: a worker whose
 * guess left fewer than k entries, or more than its candidate list holds, is selected
 * from its dense row (slower), and samples again on the following call.
 *
 *   thr_state [P][4] uint32 i/o : caller-owned device memory (16-byte aligned), one entry
 *       per worker; all zero before the first call and whenever the caller wants every
 *       worker to start from a sample again (a new model, a different k).  Its contents
 *       are otherwise opaque.
 * All other arguments, and all errors, as gtopk_step; GTOPK_EINVAL if thr_state is NULL.
 */
int gtopk_step_carry(const float* grad, float* residual, int64_t m, int64_t stride,
                     int32_t P, int32_t k, uint32_t* g_idx, float* g_val,
                     uint32_t* loc_idx, float* loc_val, uint32_t* thr_state,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * gtopk_step for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace
 * is a device array of GTOPK_STATIC_WORKSPACE_BYTES that is part of the library's code
 * object (every GPU the process uses holds one copy until the process ends); the call
 * allocates and frees nothing.  Arguments and results are those of gtopk_step.
 *   - GTOPK_EWORKSPACE if gtopk_workspace_bytes(m, k, P) exceeds
 *     GTOPK_STATIC_WORKSPACE_BYTES (nothing is enqueued); the two small configurations
 *     of the benchmark set (m = 65,536 / P = 4 / k = 66 and m = 269,722 / P = 8 / k = 270)
 *     fit, the large ones do not - use gtopk_step with a caller-owned workspace there.
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one
 *     GPU (different streams without an event between them, or different threads) race.
 *     Calls on one stream are ordered and safe; the array needs no clearing between them.
 *   - The array's address is looked up on the first call on each device, with that device
 *     current; GTOPK_EHIP if the lookup fails.
 */
#define GTOPK_STATIC_WORKSPACE_BYTES (16u << 20)
int gtopk_step_static(const float* grad, float* residual, int64_t m, int64_t stride,
                      int32_t P, int32_t k, uint32_t* g_idx, float* g_val,
                      uint32_t* loc_idx, float* loc_val, void* stream);

/*
 * Model update, Algorithm 4 line 11: W_i = W_{i-1} - eta * G~_i, applied at the k entries
 * of the global set (every other entry of G~_i is zero): for each of `copies` replicas
 * of the weights (row c starts at weights + c*stride, m floats; in the paper every
 * worker holds one replica, on one GPU one is enough),
 *     weights[c][g_idx[t]] = weights[c][g_idx[t]] - lr * g_val[t]
 * as one fp32 multiply followed by one fp32 subtract.  g_idx must be distinct and < m.
 * Needs no workspace.
 */
int gtopk_apply_update(float* weights, int64_t m, int64_t stride, int32_t copies, int32_t k,
                       const uint32_t* g_idx, const float* g_val, float lr, void* stream);

/*
 * The dense gMask that gTopKAllReduce returns (Algorithm 3 lines 20-22): mask[i] = 1 for
 * every i in g_idx, 0 elsewhere; mask has m bytes (16-byte aligned).  Needs no workspace.
 */
int gtopk_dense_mask(const uint32_t* g_idx, int32_t k, int64_t m, uint8_t* mask, void* stream);

/*
 * The aggregation of Top-k S-SGD, Algorithm 1 procedure TopKAllReduce, with all P workers'
 * k-sets on this GPU (the procedure's AllGather is then a no-op): dense[i] = s_i / P, where
 * s_i starts at +0.0 and receives worker g's value at index i (if worker g holds i) for
 * g = 0 .. P-1 IN THAT ORDER, one fp32 add each; the division is one fp32 divide.  (As
 * printed the procedure starts the sum from the caller's own sparse gradient and would
 * count it twice; the zero start gives the average that the call site's comment states.)
 * An index held by nobody gets +0.0.  This is the comparison workload for gtopk_tree: it
 * moves P*k entries in and a dense m-vector out.
 *
 *   loc_idx, loc_val [P][k] in : the workers' k-sets (index-ascending, indices < m)
 *   P                          : 1 .. 1024, any value (not only powers of two)
 *   dense            [m]   out : the averaged dense gradient G_i
 *   ws                         : gtopk_allreduce_workspace_bytes(m, P) bytes
 */
size_t gtopk_allreduce_workspace_bytes(int64_t m, int32_t P);
int gtopk_topk_allreduce(const uint32_t* loc_idx, const float* loc_val, int32_t P, int32_t k,
                         int64_t m, float* dense, void* ws, size_t ws_bytes, void* stream);

/*
 * Second sparsification of the naive gTop-k, Algorithm 2 lines 11-13: the k entries of a
 * dense m-vector with the largest |v| (same rule as everywhere: exactly k, lower index
 * first among equal magnitudes), as an index-ascending k-set with the values copied bit
 * for bit.  Algorithm 2's remaining lines are gtopk_topk_allreduce before it (line 9),
 * gtopk_residual_restore (line 14) and gtopk_apply_update (line 15) after it.
 *
 *   dense [m] in : not modified
 *   ws           : gtopk_workspace_bytes(m, k, 1) bytes
 */
int gtopk_dense_topk(const float* dense, int64_t m, int32_t k, uint32_t* g_idx, float* g_val,
                     void* ws, size_t ws_bytes, void* stream);

/*
 * Instrumentation for benchmarks (not part of the method): gtopk_step with HIP event
 * records at its stage boundaries.  `events` holds the HOST handles of six hipEvent_t
 * (created by the caller, passed as void*), recorded on `stream`:
 *   [0] start  [1] after the speculative-threshold kernels  [2] after the streaming
 *   accumulate/filter kernel  [3] after the exact local selection
 *   [4] after the tree  [5] after the residual restore.
 * The handles belong to this one call: the library keeps nothing between calls, so
 * concurrent callers (each with its own workspace, stream and events) do not interfere.
 * thr_state: NULL (then the call is gtopk_step) or as in gtopk_step_carry.
 * Results are those of gtopk_step.  GTOPK_EINVAL if events or one of the handles is NULL.
 */
#define GTOPK_STAGE_EVENTS 6
int gtopk_step_timed(const float* grad, float* residual, int64_t m, int64_t stride,
                     int32_t P, int32_t k, uint32_t* g_idx, float* g_val,
                     uint32_t* loc_idx, float* loc_val, uint32_t* thr_state,
                     void* ws, size_t ws_bytes, void* stream, void* const* events);

/*
 * Instrumentation for benchmarks (not part of the method): the streaming pass of the local
 * selection with everything but its memory traffic taken out (same block shape, same
 * number of 16-byte accesses in flight, same cache policy), to put on record what the
 * memory system gives to that access pattern.
 *   mode 0: b[i] = b[i] + a[i] for i < n  (8 bytes read and 4 written per element, as the pass)
 *   mode 1: a and b are only read; one float per 32768 elements is written to sink
 *           (sink holds n / 32768 floats; it may be NULL in every other mode)
 * Modes 2 to 7 are mode 0 with ONE of the pass's choices changed, so that the choice is
 * measured rather than asserted:
 *   mode 2: ordinary (temporal) loads      mode 3: ordinary stores      mode 4: both ordinary
 *   mode 5: 256 threads x 32 accesses per lane and array   mode 6: 1024 threads x 8
 *           (the pass: 512 x 16; all three cover 32768 elements per block)
 *   mode 7: 512 threads x 4: blocks of 8192 elements
 * n must be a positive multiple of 32768.
 */
#define GTOPK_PROBE_MODES 8
int gtopk_probe_stream(const float* a, float* b, int64_t n, int32_t mode, float* sink,
                       void* stream);

/*
 * Instrumentation for tests (not part of the method): after a gtopk_local_select or
 * gtopk_step on workspace `ws` with these sizes has COMPLETED, copy to the host how
 * many candidates the streaming pass kept for each worker (host_counts[P]) and the
 * capacity of a worker's candidate list (*host_capacity).  A worker whose count is
 * below k or above the capacity was selected from its dense row instead.
 * Synchronous (blocking device-to-host copy).
 */
int gtopk_debug_candidate_counts(const void* ws, int64_t m, int32_t k, int32_t P,
                                 uint32_t* host_counts, uint32_t* host_capacity);

/*
 * Instrumentation for tests (not part of the method): after a gtopk_merge on workspace `ws`
 * with these sizes has COMPLETED, copy to the host how many slots of each pair's union
 * reached the pair's speculative threshold (host_kept[batch]).  A pair with fewer than k
 * was merged and selected once more from its complete union.  GTOPK_EINVAL where merges
 * of this k do not go through a speculative threshold (gtopk_debug_plan, plan[11]).
 * Synchronous (blocking device-to-host copy).
 */
int gtopk_debug_merge_kept(const void* ws, int32_t k, int32_t batch, uint32_t* host_kept);

/*
 * Instrumentation for tests (not part of the method; host only, touches no GPU): how the
 * local selection of these sizes is laid out, so that a test can build rows that defeat
 * the speculative threshold and can tell which regime it exercises.
 *   plan[0] tile_stride  sample tile t of a row covers elements [t*tile_stride, +plan[2])
 *   plan[1] n_tiles      tiles per row (t = 0 .. n_tiles-1, the last one clipped to m)
 *   plan[2] tile_len     elements per tile
 *   plan[3] target       sample rank whose histogram-bucket edge becomes the threshold
 *   plan[4] capacity     entries a worker's candidate list holds
 *   plan[5] pass_histogram  1 if the streaming pass counts the first digits of its
 *                        candidates itself (the dense-row fallback then uses a histogram
 *                        of its own), 0 if the select's histogram kernel does
 *   plan[6] small_path   1 if gtopk_step takes the few-launch path for small problems at
 *                        these sizes (gtopk_step_carry, gtopk_step_timed and the stand-alone
 *                        calls always take the general kernels)
 *   plan[7] run_groups   1 if the local selection of the general kernels selects the candidates
 *                        where the streaming pass left them, one group per run (long runs),
 *                        0 if it first copies them into index order (short runs)
 *   plan[8] small_tile_stride, plan[9] small_n_tiles, plan[10] small_target: the sampler of
 *                        the few-launch path (same tile_len; all 0 where plan[6] is 0)
 *   plan[11] merge_filtered  1 if a merge of two k-sets of this k goes through a speculative
 *                        threshold (a sample of the union; only slots that reach it are kept)
 *   plan[12] merge_tile_stride, plan[13] merge_n_tiles, plan[14] merge_target: that sample -
 *                        tile t covers positions [t*merge_tile_stride, +plan[2]) of both
 *                        operands (all 0 where plan[11] is 0)
 *   plan[15] reserved (0)
 */
#define GTOPK_PLAN_WORDS 16
int gtopk_debug_plan(int64_t m, int32_t k, int32_t P, uint32_t* plan);

#ifdef __cplusplus
}
#endif
#endif /* GTOPK_H_ */
