// gTop-k S-SGD data-parallel hot path for MI355X (gfx950, wave64): the C ABI.
//
// Pipeline of one iteration (paper: Algorithm 4; Definition 1; Algorithm 3; Eq. 3):
//
//   local select   sample histogram -> speculative threshold -> ONE streaming pass
//                  (acc = residual + grad, written back; entries at or above the
//                  speculative threshold are compacted into a short candidate list)
//                  -> exact select of the k-th key among the candidates
//                  -> index-ordered emit of the k selected entries.
//                  The speculative threshold only decides how much work the exact
//                  part has; if it left a worker fewer than k candidates or more than
//                  the list holds, that worker's exact part reads its dense row
//                  instead (same kernels, decided on the device).
//   tree           per round: index-ordered union of the two k-sets of each pair
//                  (values at shared indices added) -> the same exact select
//                  -> ordered emit; the last round divides by P.  Very large sets are
//                  merged through a speculative threshold of their own (a sample of
//                  the union; only the slots that reach it are kept), with the
//                  complete union standing by for a pair whose threshold misses.
//   restore        membership test of each local entry in the global index set.
//
// Nothing here is a dense contraction, so there is no MFMA; the streaming pass is
// bound by HBM bandwidth and everything after it by launch latency.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "gtopk.h"
#include "common.hip.h"
#include "stream_pass.hip.h"
#include "select.hip.h"
#include "merge.hip.h"
#include "apply.hip.h"
#include "aggregate.hip.h"
#include "small.hip.h"

using namespace gtopk;

namespace {

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
inline uint32_t ceil_div(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }
inline bool is_pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

struct Carver {
    char* base;
    size_t off = 0;
    template <class T> T* take(size_t n) {
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off = align_up(off + n * sizeof(T));
        return p;
    }
};

// hist .. hist_dense are carved back to back so that one clear covers them
SelState carve_select(Carver& c, size_t sets, uint32_t list_cap, uint32_t maxgroups,
                      bool with_dense_hist = false) {
    SelState s;
    s.hist = c.take<uint32_t>(sets * kHistBins);
    s.list_cnt = c.take<uint32_t>(sets);
    s.grp_gt = c.take<uint32_t>(sets * maxgroups);
    s.grp_in = c.take<uint32_t>(sets * maxgroups);
    s.bin_hi = c.take<uint32_t>(sets);
    s.bin_lo_inv = c.take<uint32_t>(sets);
    s.hist_dense = with_dense_hist ? c.take<uint32_t>(sets * kHistBins) : nullptr;   // cleared as well
    s.d1 = c.take<uint32_t>(sets);
    s.krem = c.take<uint32_t>(sets);
    s.T = c.take<uint32_t>(sets);
    s.need = c.take<uint32_t>(sets);
    s.T_out = nullptr;
    s.list = c.take<uint2>(sets * list_cap);
    s.off_gt = c.take<uint32_t>(sets * maxgroups);
    s.off_eq = c.take<uint32_t>(sets * maxgroups);
    s.list_cap = list_cap;
    s.maxgroups = maxgroups;
    s.seg_list = 0u;
    return s;
}
// words from s.hist to the end of s.bin_lo_inv / s.hist_dense (padding included)
inline size_t select_clear_words(const SelState& s) { return (size_t)(s.d1 - s.hist); }

// A second copy of the arrays that must be zero when a select starts; everything
// else is shared with `base`.  Two such states alternate between the rounds of the tree,
// so that one can be cleared while the other is in use.
SelState carve_select_alt(Carver& c, const SelState& base, size_t sets, size_t* clear_words) {
    SelState s = base;
    s.hist = c.take<uint32_t>(sets * kHistBins);
    s.list_cnt = c.take<uint32_t>(sets);
    s.grp_gt = c.take<uint32_t>(sets * base.maxgroups);
    s.grp_in = c.take<uint32_t>(sets * base.maxgroups);
    s.bin_hi = c.take<uint32_t>(sets);
    s.bin_lo_inv = c.take<uint32_t>(sets);
    uint32_t* end = c.take<uint32_t>(1);
    *clear_words = base.hist ? (size_t)(end - s.hist) : 0;
    return s;
}

// slots per group of an array of n slots: a multiple of 256, at least min_slots, and large
// enough that there are at most max_groups (<= kMaxGroups) groups
uint32_t group_slots_for(uint64_t n, uint32_t max_groups, uint32_t min_slots = 1024) {
    uint32_t L = ceil_div(n, max_groups);
    L = (L + 255u) & ~255u;
    return L < min_slots ? min_slots : L;
}
constexpr uint32_t kMergeMinSlots = 512;        // merged sets: one round of a block (swept 512 / 1024)

// Groups per set when `sets` sets are selected from side by side.  Every block of k_bucket
// and k_emit pays a fixed price (it reads the set's 4096-bin histogram, or the list of
// in-bin keys), so a batch gets about kTargetBlocks blocks in total and no more (swept: 512 .. 4096;
// a tree of 32 sets of 255,570 entries: 268 / 291 / 307 us at 1024 / 2048 / 4096).
constexpr uint32_t kTargetBlocks = 1024;
constexpr uint32_t kLocalTargetBlocks = 8192;   // the same for the local selection's P sets
uint32_t groups_for(uint32_t sets) {
    const uint32_t g = kTargetBlocks / (sets ? sets : 1);
    return g < 32 ? 32 : (g > (uint32_t)kMaxGroups ? (uint32_t)kMaxGroups : g);
}

constexpr uint64_t kInlineFinishMax = 1u << 20;  // sets up to this many slots: no k_finish
constexpr uint32_t kUnionPathMinK = 131072;      // sets above this size take k_union_path
constexpr int kUnionPathEpt = 8;
constexpr int kUnionHistBlock = 1024;           // threads per block of the union that also histograms
constexpr uint32_t kUnionCutsMinK = 1u << 19;   // sets above this size: cut points in a kernel of their own

struct MergeWs {
    SelState sel;      // state of even rounds
    SelState sel_alt;  // state of odd rounds (own hist / list_cnt / grp_gt)
    size_t alt_clear_words;
    uint32_t* m_idx;   // [pairs][m_stride]: the 2k slots of a pair, padded to a multiple of 8
    float* m_val;
    uint32_t m_stride;
    uint32_t* tmin[2]; // [pairs] smallest key of each output set, alternating between rounds
    uint32_t* inv_min; // [2*pairs] 0x7fffffff - smallest key of each caller-supplied operand
    uint32_t* cuts;    // [pairs][tiles + 1] cut points of k_union_path's blocks (large sets)
    // the largest sets are merged through a speculative threshold (FiltSrc); all NULL otherwise
    uint32_t* f_samp_hist;  // [pairs][16384]  } cleared together at the start of every round
    uint32_t* f_set_cnt;    // [pairs]         }
    size_t f_clear_words;
    uint32_t* f_tspec;      // [pairs]
    uint32_t* f_tile_cnt;   // [pairs][tiles]
    SelState sel_rep;       // select state of the pairs that fall back to their complete union
    size_t rep_clear_words;
    uint32_t L;
    size_t bytes;
};

// Sets of more than 2^22 entries whose 8192-slot union tiles fit the select's group tables
// are merged through a speculative threshold.  Measured at C4 size: at k = 6.4 M the rounds of
// the tree take 3.4 instead of 3.6 ms; at k = 1.85 M the sample and the stand-by launches for a
// threshold that misses (about 65 us per round) cost more than the smaller select saves.
constexpr uint32_t kMergeFilterMinK = 1u << 22;
inline bool merge_filtered(uint32_t k) {
    return k > kMergeFilterMinK &&
           ceil_div(2ull * k, (uint64_t)kUnionHistBlock * kUnionPathEpt) <= (uint32_t)kMaxGroups;
}

MergeWs carve_merge(Carver& c, uint32_t k, size_t pairs) {
    MergeWs w;
    w.L = group_slots_for(2ull * k, kMaxGroups, kMergeMinSlots);
    w.sel = carve_select(c, pairs, 2 * k, ceil_div(2ull * k, w.L));
    w.sel_alt = carve_select_alt(c, w.sel, pairs, &w.alt_clear_words);
    w.m_stride = (2 * k + 7u) & ~7u;
    w.m_idx = c.take<uint32_t>(pairs * w.m_stride);
    w.m_val = c.take<float>(pairs * w.m_stride);
    w.tmin[0] = c.take<uint32_t>(pairs);
    w.tmin[1] = c.take<uint32_t>(pairs);
    w.inv_min = c.take<uint32_t>(2 * pairs);
    w.cuts = c.take<uint32_t>(k > kUnionCutsMinK
                                  ? pairs * ((size_t)ceil_div(2ull * k, kUnionHistBlock * kUnionPathEpt) + 1)
                                  : 0);
    w.f_samp_hist = w.f_set_cnt = w.f_tspec = w.f_tile_cnt = nullptr;
    w.f_clear_words = w.rep_clear_words = 0;
    w.sel_rep = w.sel;
    if (merge_filtered(k)) {
        const size_t ntiles = ceil_div(2ull * k, kUnionHistBlock * kUnionPathEpt);
        w.f_samp_hist = c.take<uint32_t>(pairs * kSampleBins);
        w.f_set_cnt = c.take<uint32_t>(pairs);
        uint32_t* end = c.take<uint32_t>(1);
        w.f_clear_words = w.f_samp_hist ? (size_t)(end - w.f_samp_hist) : 0;
        w.f_tspec = c.take<uint32_t>(pairs);
        w.f_tile_cnt = c.take<uint32_t>(pairs * ntiles);
        w.sel_rep = carve_select_alt(c, w.sel, pairs, &w.rep_clear_words);
    }
    w.bytes = c.off;
    return w;
}

struct StepWs {
    // local select
    uint32_t* samp_hist;   // [P][16384]    } cleared together
    uint32_t* cand_count;  // [P]           }
    uint32_t* tspec;       // [P] speculative threshold of the streaming pass
    uint32_t* cand_idx;    // [P][cap] candidates as the streaming pass left them (runs)
    float* cand_val;
    uint2* run_table;      // [P][nchunks]
    uint32_t* run_off;     // [P][nchunks]
    uint32_t* ord_idx;     // [P][cap] candidates in index order
    float* ord_val;
    SelState sel;          // P sets
    uint32_t cap, nchunks;
    uint32_t Lc, gcand;    // candidate list: slots per group, groups
    uint32_t Ld, gdense;   // dense row: slots per group, groups
    // tree
    MergeWs mrg;           // P/2 pairs
    uint32_t* x_idx;       // [P/2][k] ping
    float* x_val;
    uint32_t* y_idx;       // [P/4][k] pong
    float* y_val;
    // step
    uint32_t* gbits;       // [ceil(m/32)] one bit per gradient element: the global set
    size_t gbits_words;
    uint32_t* loc_idx;     // [P][k] when the caller does not want them
    float* loc_val;
    size_t bytes;
};

uint32_t cand_capacity(int64_t m, uint32_t k) {
    uint64_t cap = 3ull * k + 8192;
    if (cap > (uint64_t)m) cap = (uint64_t)m;
    return (uint32_t)cap;
}

// Small problems take the few-launch path: the local selection of a worker in one block,
// the whole tree with the average and the extra residual in one block.
static bool small_problem(int64_t m, int64_t k, int64_t P) {
    return P <= kSmallMaxP && k <= kSmallMaxK && P * k <= kSmallMaxEntries &&
           m + 3 <= (int64_t)kSmallMaxChunks * kSmallChunk;
}

struct SamplePlan { uint32_t tile_stride, n_tiles, target; };

// Long candidate lists are selected where the streaming pass left them, one group per run
// (RunSrc): from about 256 expected candidates per chunk of the row on, and while the runs
// of a row are no more than the select's group tables hold.
static bool run_groups(int64_t m, uint32_t k) {
    const double per_chunk = 1.4 * (double)k * (double)kChunk / (double)m;
    return per_chunk >= 256.0 && ceil_div((uint64_t)m + 3, kChunk) <= (uint64_t)kMaxGroups;
}
// (the few-launch path takes a smaller sample: one block per worker reads it)
constexpr double kSampleMean = 256.0, kSampleMinTiles = 4096.0;
constexpr double kSmallSampleMean = 16.0, kSmallSampleMinTiles = 128.0;
SamplePlan plan_sample(int64_t m, uint32_t k, double sample_mean = kSampleMean,
                       double min_tiles = kSampleMinTiles);

StepWs carve_step(void* ws, int64_t m, uint32_t k, uint32_t P) {
    Carver c{reinterpret_cast<char*>(ws)};
    StepWs s;
    s.cap = cand_capacity(m, k);
    s.nchunks = ceil_div((uint64_t)m + 3, kChunk);      // a row may start up to 3 elements into a chunk
    {
        uint32_t g = kLocalTargetBlocks / P;
        g = g < 32 ? 32 : (g > (uint32_t)kMaxGroups ? (uint32_t)kMaxGroups : g);
        s.Lc = group_slots_for(s.cap, g);
        const uint32_t lmin = group_slots_for(s.cap, kMaxGroups);
        if (s.Lc > 8192u) s.Lc = lmin > 8192u ? lmin : 8192u;
        s.gcand = ceil_div(s.cap, s.Lc);
    }
    // dense rows (a worker whose candidate list cannot be used; the dense top-k)
    s.gdense = P == 1 ? (uint32_t)kMaxGroups : 1024u;
    s.Ld = group_slots_for((uint64_t)m, s.gdense);
    s.gdense = ceil_div((uint64_t)m, s.Ld);
    s.samp_hist = c.take<uint32_t>((size_t)P * kSampleBins);
    s.cand_count = c.take<uint32_t>(P);
    s.tspec = c.take<uint32_t>(P);
    s.cand_idx = c.take<uint32_t>((size_t)P * s.cap);
    s.cand_val = c.take<float>((size_t)P * s.cap);
    // (the few-launch path for small problems cuts a row into runs of 4096 elements)
    const uint32_t nruns_small = small_problem(m, k, P) ? ceil_div((uint64_t)m + 3, kSmallChunk) : 0u;
    s.run_table = c.take<uint2>((size_t)P * (s.nchunks > nruns_small ? s.nchunks : nruns_small));
    s.run_off = c.take<uint32_t>((size_t)P * s.nchunks);
    s.ord_idx = c.take<uint32_t>((size_t)P * s.cap);
    s.ord_val = c.take<float>((size_t)P * s.cap);
    {
        uint32_t g = s.gcand > s.gdense ? s.gcand : s.gdense;
        if (run_groups(m, k) && s.nchunks > g) g = s.nchunks;      // one group per run
        s.sel = carve_select(c, P, s.cap, g, /*with_dense_hist=*/true);
    }
    const size_t pairs = P > 1 ? P / 2 : 1;
    s.mrg = carve_merge(c, k, pairs);
    s.x_idx = c.take<uint32_t>(pairs * k);
    s.x_val = c.take<float>(pairs * k);
    const size_t quarter = P > 3 ? P / 4 : 1;
    s.y_idx = c.take<uint32_t>(quarter * k);
    s.y_val = c.take<float>(quarter * k);
    s.gbits_words = (size_t)((m + 31) / 32);
    s.gbits = c.take<uint32_t>(s.gbits_words);
    s.loc_idx = c.take<uint32_t>((size_t)P * k);
    s.loc_val = c.take<float>((size_t)P * k);
    s.bytes = c.off;
    return s;
}

constexpr int64_t kMaxMergeK = (int64_t)1 << 30;     // a merged pair has 2k slots, a uint32

bool sizes_ok(int64_t m, int64_t k, int64_t P) {
    return m >= 1 && m <= ((int64_t)1 << 31) && k >= 1 && k <= m && is_pow2(P) && P <= 65535 &&
           (P == 1 || k <= kMaxMergeK);
}

int launch_status() { return hipGetLastError() == hipSuccess ? GTOPK_OK : GTOPK_EHIP; }

// Instrumentation: the caller's events of one gtopk_step_timed call (NULL: none).
void mark_stage(int i, void* const* events, hipStream_t st) {
    if (events) (void)hipEventRecord((hipEvent_t)events[i], st);
}

ZeroJob zero_job(uint32_t* p0 = nullptr, size_t n0 = 0, uint32_t* p1 = nullptr, size_t n1 = 0,
                 uint32_t* p2 = nullptr, size_t n2 = 0, uint32_t* p3 = nullptr, size_t n3 = 0,
                 uint32_t* p4 = nullptr, size_t n4 = 0) {
    return ZeroJob{{p0, p1, p2, p3, p4, nullptr}, {n0, n1, n2, n3, n4, 0}};
}

void zero_async(hipStream_t st, const ZeroJob& job) {
    size_t n = 0;
    for (int a = 0; a < kZeroSlots; ++a) n = job.n[a] > n ? job.n[a] : n;
    if (n == 0) return;
    uint32_t blocks = (uint32_t)((n + 1023) / 1024 > 1024 ? 1024 : (n + 1023) / 1024);
    hipLaunchKernelGGL(k_zero_u32, dim3(blocks ? blocks : 1), dim3(256), 0, st, job);
}

// how a batch of sets is walked and emitted
struct SelGrid {
    uint32_t sets;
    uint32_t walk_blocks;   // blocks per set of k_bucket
    uint32_t groups;        // blocks per set of k_emit (= emit groups, at most)
    uint64_t nphys_max;     // slots of a set's list, at most (sizes k_hist)
    bool own_finish;        // k_finish once per set instead of a finish in every emit block
};

// histogram + bucket + emit
template <class Src, bool DIVIDE>
void run_select(const Src& src, const SelState& ss0, const SelGrid& gr, uint32_t k, uint32_t* out_idx,
                float* out_val, int64_t out_stride, float divisor, uint32_t* gbits, hipStream_t st,
                bool with_hist = true) {
    // large merged sets, finished once per set: the in-bin keys stay with their groups (no shared counter)
    SelState ss = ss0;
    ss.seg_list = (Src::kSegList && gr.own_finish) ? 1u : 0u;
    // few blocks per set (a popular bin takes one same-address atomic per block): 4 slots per
    // thread up to 32 blocks, then 32 blocks with more slots per thread, then 32 slots per
    // thread up to 256 blocks (swept at k = 255,570 .. 6.4 M)
    uint32_t hb = ceil_div(gr.nphys_max, 4 * kHistBlock);
    if (hb > 32) {
        hb = ceil_div(gr.nphys_max, 32 * kHistBlock);
        hb = hb < 32 ? 32 : (hb > 256 ? 256 : hb);
    }
    if (hb < 1) hb = 1;
    if (with_hist)
        hipLaunchKernelGGL((k_hist<Src>), dim3(hb + (Src::kRunScan ? 1 : 0), gr.sets), dim3(kHistBlock), 0,
                           st, src, ss, hb);
    hipLaunchKernelGGL((k_bucket<Src>), dim3(gr.walk_blocks, gr.sets), dim3(kBlock), 0, st, src, ss, k);
    // small sets: every block of the emit finishes the select itself (the list of keys it
    // needs for that is short); large sets: once per set, in a kernel of its own
    if (!gr.own_finish) {
        hipLaunchKernelGGL((k_emit<Src, DIVIDE, true>), dim3(gr.groups, gr.sets), dim3(kBlock), 0, st,
                           src, ss, k, out_idx, out_val, out_stride, divisor, gbits);
    } else {
        hipLaunchKernelGGL((k_finish<Src>), dim3(gr.sets), dim3(1024), 0, st, src, ss);
        hipLaunchKernelGGL((k_emit<Src, DIVIDE, false>), dim3(gr.groups, gr.sets), dim3(kBlock), 0, st,
                           src, ss, k, out_idx, out_val, out_stride, divisor, gbits);
    }
}

// Sample plan for the speculative threshold: tiles of 64 contiguous elements, evenly
// spaced, about kSampleMean / rho elements per worker but at least 4096 tiles (all
// elements if the row is short).  `target` is the rank in the sample whose bucket edge is taken: the
// expected sample rank of the k-th key plus 5.5 standard deviations, so that the
// candidate list holds at least k entries except with probability ~1e-8 per worker
// (and then that worker is merely selected from its dense row).
// sample_mean: expected sample rank of the k-th key, at least.  min_tiles: spread (with
// 4096, a layer of 1 % of the row still gets ~40 tiles).
SamplePlan plan_sample(int64_t m, uint32_t k, double sample_mean, double min_tiles) {
    SamplePlan p;
    double want = sample_mean * (double)m / (double)k;
    if (want < min_tiles * kSampleTile) want = min_tiles * kSampleTile;
    if (want >= (double)m) {
        p.tile_stride = kSampleTile;
    } else {
        const uint64_t tiles = (uint64_t)(want / kSampleTile) + 1;
        const uint64_t ts = (uint64_t)m / tiles;
        p.tile_stride = (uint32_t)(ts < (uint64_t)kSampleTile ? kSampleTile : ts);
    }
    p.n_tiles = ceil_div((uint64_t)m, p.tile_stride);
    const uint64_t last = (uint64_t)m - (uint64_t)(p.n_tiles - 1) * p.tile_stride;
    const uint64_t sampled = (uint64_t)(p.n_tiles - 1) * kSampleTile +
                             (last < (uint64_t)kSampleTile ? last : (uint64_t)kSampleTile);
    if (sampled >= (uint64_t)m) {
        p.target = k;                        // the "sample" is the whole row: exact count
    } else {
        // 5.5 standard deviations of the count, plus 3 % for the tiles' placement error
        const double mean = (double)k * (double)sampled / (double)m;
        double t = 1.03 * mean + 5.5 * __builtin_sqrt(mean) + 2.0;
        if (t > (double)sampled) t = (double)sampled;
        p.target = (uint32_t)t;
        if (p.target < 1) p.target = 1;
    }
    return p;
}

// The pass can also histogram the candidates it keeps; the select's own histogram kernel
// then only serves workers that fall back to their dense row.  That costs LDS atomics and,
// per block and non-empty bin, a global atomic in the pass.  Measured against the
// histogram kernel it saves: at rho = 0.001 (45 candidates per 32768-element block) the
// pass does not change and the select gains 6-8 us; at rho = 0.01 (460 per block) the pass
// loses 55 us and the select gains 13 us; at rho = 0.0725 (3,300 per block) the pass loses
// 120 us and the select gains 85 us; at rho = 0.25 (11,500 per block) the pass loses
// 80 us and the select gains 230 us.  So at both ends, not in between.
bool pass_histograms(int64_t m, uint32_t k) {
    const double per_block = 1.4 * (double)k * (double)kChunk / (double)m;
    return per_block <= 128.0 || per_block >= 4096.0;
}

// the candidate lists (or dense rows) of the P workers as the select kernels' source
CandSrc cand_source(const float* rows, int64_t stride, int64_t m, uint32_t k, const StepWs& w,
                    bool producer_hist, bool no_bounds, uint32_t* thr_state = nullptr) {
    return CandSrc{rows, stride, (uint32_t)m, k, w.cap, w.nchunks, w.Lc, w.Ld,
                   w.cand_idx, w.cand_val, w.cand_count, w.tspec, w.run_table, w.run_off,
                   w.ord_idx, w.ord_val, producer_hist, no_bounds, reinterpret_cast<uint4*>(thr_state)};
}

// The grids are sized for the candidate lists.  A worker that is selected from its dense
// row has more groups than that; its blocks take several each.  Every emit block finishes
// the select itself: the list of in-bin keys is short.
SelGrid local_grid(const StepWs& w, uint32_t P) {
    const uint32_t gd = w.gdense < 256u ? w.gdense : 256u;
    const uint32_t gx = w.gcand > gd ? w.gcand : gd;
    return SelGrid{P, gx, gx, (uint64_t)w.cap, false};
}

// `zero_rows`: store +0.0 at the selected entries (the stand-alone call); gtopk_step
// passes false and settles the rows in k_restore_fused.  `pre_cleared`: the caller has
// already cleared this call's counters and histograms.
int do_local_select(const float* grad, float* residual, int64_t m, int64_t stride, uint32_t P,
                    uint32_t k, uint32_t* out_idx, float* out_val, const StepWs& w, bool zero_rows,
                    bool pre_cleared, hipStream_t st, void* const* events = nullptr,
                    uint32_t* thr_state = nullptr) {
    // workers whose threshold is carried over from the previous call skip the sampling (both
    // kernels are launched all the same: who samples is decided on the device)
    const uint4* carry = reinterpret_cast<const uint4*>(thr_state);
    if (!pre_cleared)
        zero_async(st, zero_job(w.samp_hist, (size_t)(w.tspec - w.samp_hist), w.sel.hist,
                                select_clear_words(w.sel)));

    const SamplePlan sp = plan_sample(m, k);
    uint32_t sblocks = ceil_div(sp.n_tiles, (kSampleBlock / kSampleTile) * 8);
    // about 256 blocks in all: every block flushes its own 16384-bin histogram with atomics
    const uint32_t sb_max = P >= 64 ? 4u : (P <= 16 ? 16u : 256u / P);
    if (sblocks > sb_max) sblocks = sb_max;
    if (sblocks < 1) sblocks = 1;
    hipLaunchKernelGGL(k_sample, dim3(sblocks, P), dim3(kSampleBlock), 0, st, grad, residual,
                       (uint32_t)m, stride, sp.tile_stride, sp.n_tiles, w.samp_hist, carry);
    hipLaunchKernelGGL(k_sample_pick, dim3(P), dim3(kSampleBlock), 0, st, w.samp_hist, sp.target,
                       w.tspec, carry);
    mark_stage(1, events, st);

    const bool producer_hist = pass_histograms(m, k);
    if (producer_hist)
        hipLaunchKernelGGL(k_accum_filter<true>, dim3(w.nchunks, P), dim3(kSBlock), 0, st, grad,
                           residual, (uint32_t)m, stride, w.tspec, w.cand_idx, w.cand_val, w.cap,
                           w.cand_count, w.run_table, w.nchunks, w.sel.hist);
    else
        hipLaunchKernelGGL(k_accum_filter<false>, dim3(w.nchunks, P), dim3(kSBlock), 0, st, grad,
                           residual, (uint32_t)m, stride, w.tspec, w.cand_idx, w.cand_val, w.cap,
                           w.cand_count, w.run_table, w.nchunks, w.sel.hist);
    mark_stage(2, events, st);

    const CandSrc src = cand_source(residual, stride, m, k, w, producer_hist, false, thr_state);
    // the histogram kernel always runs: where the pass has counted its candidates it serves
    // only the workers that came back with fewer than k of them
    if (run_groups(m, k)) {
        RunSrc rs;
        static_cast<CandSrc&>(rs) = src;
        // k_bucket: every wave of a block takes a run; k_emit: a block per run; a worker on its
        // dense row uses the blocks there are
        SelGrid gr = local_grid(w, P);
        const uint32_t rb = ceil_div(w.nchunks, kBlock / kWave);
        if (gr.walk_blocks < rb) gr.walk_blocks = rb;
        if (gr.groups < w.nchunks) gr.groups = w.nchunks;
        run_select<RunSrc, false>(rs, w.sel, gr, k, out_idx, out_val, (int64_t)k, 1.0f, nullptr, st);
    } else {
        run_select<CandSrc, false>(src, w.sel, local_grid(w, P), k, out_idx, out_val, (int64_t)k, 1.0f,
                                   nullptr, st);
    }
    // a kernel of its own: while the select runs, a dense row may still be read as a whole
    if (zero_rows)
        hipLaunchKernelGGL(k_zero_selected, dim3(ceil_div(k, kBlock), P), dim3(kBlock), 0, st, out_idx,
                           k, residual, stride);
    return launch_status();
}

// Sample of a union for its speculative threshold: 256 tiles of 64 positions of either
// operand.  Every slot of the union is sampled with probability f = sampled / k, so the
// k-th key of the union has expected sample rank `sampled`; the target adds 5.5 standard
// deviations and 3 % for the tiles' placement error, as for a row (plan_sample).
struct MergeSamplePlan { uint32_t tile_stride, n_tiles, target, blocks; };
inline MergeSamplePlan plan_merge_sample(uint32_t k) {
    MergeSamplePlan p;
    const uint32_t want_tiles = 256;
    p.tile_stride = k / want_tiles;                          // k > 2^19: at least 2048
    if (p.tile_stride < (uint32_t)kSampleTile) p.tile_stride = kSampleTile;
    p.n_tiles = ceil_div(k, p.tile_stride);
    const uint64_t last = (uint64_t)k - (uint64_t)(p.n_tiles - 1) * p.tile_stride;
    const double sampled = (double)(p.n_tiles - 1) * kSampleTile + (double)(last < (uint64_t)kSampleTile ? last : kSampleTile);
    double t = 1.03 * sampled + 5.5 * __builtin_sqrt(sampled) + 2.0;
    if (t > 2.0 * sampled) t = 2.0 * sampled;
    p.target = (uint32_t)t;
    p.blocks = ceil_div(p.n_tiles, kSampleBlock / kSampleTile);
    if (p.blocks > 16) p.blocks = 16;
    if (p.blocks < 1) p.blocks = 1;
    return p;
}

inline uint32_t min_key_blocks(uint32_t k) {
    const uint32_t b = ceil_div(k, 8192);
    return b < 1 ? 1 : (b > 64 ? 64 : b);
}

// Lanes per cut point by the number of cut points of the launch (see k_union_cuts).  Measured
// for sets of 1.9 M and 6.4 M entries, in us for (25 k, 12.5 k, 6.2 k, 3.1 k, 1.6 k) and
// (7.3 k, 3.6 k, 1.8 k, 0.9 k, 0.45 k) cut points:
//    2 lanes: 35 31 24 21 14 | 26 22 18 13 16      4 lanes: 41 22 16 13  9 | 17 13 11  8  7
//   16 lanes: 79 40 20 10  7 | 21 10  8  6  5     64 lanes: 131 73 36 18 9 | 41 19 11  6  5
inline void launch_union_cuts(const uint32_t* a_idx, const uint32_t* b_idx, uint32_t k, int64_t in_stride,
                              uint32_t tile, uint32_t ntiles, uint32_t batch, uint32_t* cuts, hipStream_t st) {
    const uint64_t total = (uint64_t)(ntiles + 1) * batch;
    const uint32_t L = total > 20000 ? 2u : (total > 5000 ? 4u : 16u);
    const dim3 grid(ceil_div((ntiles + 1) * L, kBlock), batch);
    if (L == 2)
        hipLaunchKernelGGL(k_union_cuts<2>, grid, dim3(kBlock), 0, st, a_idx, b_idx, k, in_stride, tile, ntiles, cuts);
    else if (L == 4)
        hipLaunchKernelGGL(k_union_cuts<4>, grid, dim3(kBlock), 0, st, a_idx, b_idx, k, in_stride, tile, ntiles, cuts);
    else
        hipLaunchKernelGGL(k_union_cuts<16>, grid, dim3(kBlock), 0, st, a_idx, b_idx, k, in_stride, tile, ntiles, cuts);
}

// one batch of merges: union + exact select + ordered emit.  `round` picks which of the
// two select states is used (it must be clear on entry); the other one is cleared on the
// side for the next round.
template <bool DIVIDE>
void do_merge_batch(const uint32_t* a_idx, const float* a_val, const uint32_t* b_idx,
                    const float* b_val, uint32_t k, uint32_t batch, int64_t in_stride,
                    uint32_t* out_idx, float* out_val, int64_t out_stride, const MergeWs& w,
                    int round, const uint32_t* in_min, bool in_min_inverted, uint32_t* out_min,
                    float divisor, uint32_t* gbits, hipStream_t st) {
    const bool odd = (round & 1) != 0;
    uint32_t* zp = odd ? w.sel.hist : w.sel_alt.hist;
    const uint32_t zw = (uint32_t)(odd ? select_clear_words(w.sel) : w.alt_clear_words);
    // w.L is the smallest group the workspace was sized for; a batch of many pairs takes larger ones
    uint32_t L = group_slots_for(2ull * k, groups_for(batch), kMergeMinSlots);
    if (L > 8192u) L = 8192u;
    if (L < w.L) L = w.L;
    const uint32_t groups = ceil_div(2ull * k, L);
    MergedSrc src{w.m_idx, w.m_val, 2 * k, w.m_stride, L, in_min, in_min_inverted};
    SelState ss = odd ? w.sel_alt : w.sel;
    ss.T_out = out_min;
    // The union runs in blocks as large as the histogram kernel's and counts the first digits
    // of the keys it produces, so the select below starts at its second kernel.
    // small sets: one entry of either operand per thread (latency);
    // large sets: cut by output position, eight slots per thread (throughput); for the
    // largest the blocks' cut points come from a kernel of their own
    if (k <= kUnionPathMinK)
        hipLaunchKernelGGL((k_union<1, kUnionHistBlock, true>), dim3(ceil_div(k, kUnionHistBlock), batch),
                           dim3(kUnionHistBlock), 0, st, a_idx, a_val, b_idx, b_val, k, in_stride, w.m_idx,
                           w.m_val, w.m_stride, zp, zw, src, ss);
    else if (k <= kUnionCutsMinK)
        hipLaunchKernelGGL((k_union_path<kUnionPathEpt, false, kUnionHistBlock, true>),
                           dim3(ceil_div(2 * k, kUnionHistBlock * kUnionPathEpt), batch),
                           dim3(kUnionHistBlock), 0, st, a_idx, a_val, b_idx, b_val, k, in_stride, w.m_idx,
                           w.m_val, w.m_stride, (const uint32_t*)nullptr, zp, zw, src, ss);
    else if (!w.f_samp_hist) {
        const uint32_t tile = kUnionHistBlock * kUnionPathEpt, ntiles = ceil_div(2 * k, tile);
        launch_union_cuts(a_idx, b_idx, k, in_stride, tile, ntiles, batch, w.cuts, st);
        hipLaunchKernelGGL((k_union_path<kUnionPathEpt, true, kUnionHistBlock, true>), dim3(ntiles, batch),
                           dim3(kUnionHistBlock), 0, st, a_idx, a_val, b_idx, b_val, k, in_stride, w.m_idx,
                           w.m_val, w.m_stride, (const uint32_t*)w.cuts, zp, zw, src, ss);
    } else {
        // The largest sets.  A sample of the union gives a threshold that a little more than k
        // of its slots are expected to reach; the union keeps only those, tile by tile, and the
        // select works on what is left (FiltSrc).  A pair whose union kept fewer than k slots is
        // then merged and selected once more, from its complete union; for every other pair
        // those launches return at once.
        const uint32_t tile = kUnionHistBlock * kUnionPathEpt, ntiles = ceil_div(2 * k, tile);
        zero_async(st, zero_job(w.f_samp_hist, w.f_clear_words, w.sel_rep.hist, w.rep_clear_words));
        const MergeSamplePlan mp = plan_merge_sample(k);
        hipLaunchKernelGGL(k_merge_sample, dim3(mp.blocks, batch), dim3(kSampleBlock), 0, st, a_idx, a_val,
                           b_idx, b_val, k, in_stride, mp.tile_stride, mp.n_tiles, w.f_samp_hist);
        hipLaunchKernelGGL(k_sample_pick, dim3(batch), dim3(kSampleBlock), 0, st,
                           (const uint32_t*)w.f_samp_hist, mp.target, w.f_tspec, (const uint4*)nullptr);
        launch_union_cuts(a_idx, b_idx, k, in_stride, tile, ntiles, batch, w.cuts, st);
        hipLaunchKernelGGL((k_union_path<kUnionPathEpt, true, kUnionHistBlock, true, true>), dim3(ntiles, batch),
                           dim3(kUnionHistBlock), 0, st, a_idx, a_val, b_idx, b_val, k, in_stride, w.m_idx,
                           w.m_val, w.m_stride, (const uint32_t*)w.cuts, zp, zw, src, ss,
                           UnionFilter{w.f_tspec, w.f_tile_cnt, w.f_set_cnt}, (const uint32_t*)nullptr);
        static_assert(kUnionHistBlock * kUnionPathEpt == 8192, "FiltSrc's tiles are the union's: 2^13 slots");
        const FiltSrc fs{w.m_idx, w.m_val, k, w.m_stride, 13u, ntiles, w.f_tile_cnt, w.f_set_cnt, w.f_tspec};
        run_select<FiltSrc, DIVIDE>(fs, ss, SelGrid{batch, ntiles, ntiles, 2ull * k, true}, k, out_idx, out_val,
                                    out_stride, divisor, gbits, st, /*with_hist=*/false);
        // the pairs that came out short
        MergedSrc rsrc = src;
        rsrc.gate_cnt = w.f_set_cnt;
        rsrc.gate_k = k;
        SelState rs = w.sel_rep;
        rs.T_out = out_min;
        hipLaunchKernelGGL((k_union_path<kUnionPathEpt, true, kUnionHistBlock, true>), dim3(ntiles, batch),
                           dim3(kUnionHistBlock), 0, st, a_idx, a_val, b_idx, b_val, k, in_stride, w.m_idx,
                           w.m_val, w.m_stride, (const uint32_t*)w.cuts, (uint32_t*)nullptr, 0u, rsrc, rs,
                           UnionFilter{nullptr, nullptr, nullptr}, (const uint32_t*)w.f_set_cnt);
        run_select<MergedSrc, DIVIDE>(rsrc, rs, SelGrid{batch, groups, groups, 2ull * k, true}, k, out_idx,
                                      out_val, out_stride, divisor, gbits, st, /*with_hist=*/false);
        return;
    }
    run_select<MergedSrc, DIVIDE>(src, ss, SelGrid{batch, groups, groups, 2ull * k, 2ull * k > kInlineFinishMax},
                                  k, out_idx, out_val, out_stride, divisor, gbits, st,
                                  /*with_hist=*/false);
}

// loc_min: the smallest key of each of the P input sets (the local selection's T), or NULL
// when the caller supplied the sets
int do_tree(const uint32_t* loc_idx, const float* loc_val, const uint32_t* loc_min, uint32_t P,
            uint32_t k, uint32_t* g_idx, float* g_val, const StepWs& w, uint32_t* gbits,
            bool pre_cleared, hipStream_t st) {
    const float divisor = (float)P;
    if (P == 1) {
        hipLaunchKernelGGL(k_copy_set, dim3(ceil_div(k, 256)), dim3(256), 0, st, loc_idx, loc_val, k,
                           g_idx, g_val, divisor, gbits);
        return launch_status();
    }
    if (!pre_cleared)
        zero_async(st, zero_job(w.mrg.sel.hist, select_clear_words(w.mrg.sel), w.mrg.sel_alt.hist,
                                w.mrg.alt_clear_words, w.mrg.inv_min, P));
    bool inverted = false;
    if (!loc_min) {
        // sets from the caller: find their smallest keys, the first round's lower bounds
        hipLaunchKernelGGL(k_set_min_key, dim3(min_key_blocks(k), P), dim3(kBlock), 0, st, loc_val,
                           (const float*)nullptr, (int64_t)k, k, w.mrg.inv_min);
        loc_min = w.mrg.inv_min;
        inverted = true;
    }
    // After every round the surviving sets are stored compactly, so round j always
    // merges set 2p with set 2p+1 of its input: exactly worker p*2^(j+1) with worker
    // p*2^(j+1) + 2^j of the original numbering.
    const uint32_t* in_idx = loc_idx;
    const float* in_val = loc_val;
    uint32_t* ping_i = w.x_idx; float* ping_v = w.x_val;
    uint32_t* pong_i = w.y_idx; float* pong_v = w.y_val;
    const uint32_t* in_min = loc_min;
    int round = 0;
    for (uint32_t pairs = P / 2; pairs >= 1; pairs /= 2, ++round) {
        const bool last = pairs == 1;
        uint32_t* out_min = w.mrg.tmin[round & 1];
        if (last) {
            do_merge_batch<true>(in_idx, in_val, in_idx + k, in_val + k, k, 1, 2 * (int64_t)k, g_idx,
                                 g_val, k, w.mrg, round, in_min, inverted, out_min, divisor, gbits,
                                 st);
        } else {
            do_merge_batch<false>(in_idx, in_val, in_idx + k, in_val + k, k, pairs, 2 * (int64_t)k,
                                  ping_i, ping_v, k, w.mrg, round, in_min, inverted, out_min, 1.0f,
                                  nullptr, st);
            in_min = out_min;
            inverted = false;
            in_idx = ping_i; in_val = ping_v;
            uint32_t* ti = ping_i; ping_i = pong_i; pong_i = ti;
            float* tv = ping_v; ping_v = pong_v; pong_v = tv;
        }
    }
    return launch_status();
}

}  // namespace

extern "C" {

const char* gtopk_status_string(int status) {
    switch (status) {
        case GTOPK_OK: return "GTOPK_OK";
        case GTOPK_EINVAL: return "GTOPK_EINVAL: invalid argument";
        case GTOPK_EWORKSPACE: return "GTOPK_EWORKSPACE: workspace too small";
        case GTOPK_EALIGN: return "GTOPK_EALIGN: pointer not 16-byte aligned";
        case GTOPK_EHIP: return "GTOPK_EHIP: kernel launch failed";
        default: return "GTOPK: unknown status";
    }
}

size_t gtopk_workspace_bytes(int64_t m, int32_t k, int32_t P) {
    if (!sizes_ok(m, k, P)) return 0;
    return carve_step(nullptr, m, (uint32_t)k, (uint32_t)P).bytes;
}

size_t gtopk_merge_workspace_bytes(int32_t k, int32_t batch) {
    if (k < 1 || k > kMaxMergeK || batch < 1 || batch > 32767) return 0;
    Carver c{nullptr};
    return carve_merge(c, (uint32_t)k, (size_t)batch).bytes;
}

int gtopk_local_select(const float* grad, float* residual, int64_t m, int64_t stride, int32_t P,
                       int32_t k, uint32_t* out_idx, float* out_val, void* ws, size_t ws_bytes,
                       void* stream) {
    if (!grad || !residual || !out_idx || !out_val || !ws) return GTOPK_EINVAL;
    if (!sizes_ok(m, k, P) || stride < m) return GTOPK_EINVAL;
    if (!aligned16(grad) || !aligned16(residual) || !aligned16(out_idx) || !aligned16(out_val) ||
        !aligned16(ws))
        return GTOPK_EALIGN;
    const StepWs w = carve_step(ws, m, (uint32_t)k, (uint32_t)P);
    if (ws_bytes < w.bytes) return GTOPK_EWORKSPACE;
    return do_local_select(grad, residual, m, stride, (uint32_t)P, (uint32_t)k, out_idx, out_val, w,
                           true, false, (hipStream_t)stream);
}

int gtopk_merge(const uint32_t* a_idx, const float* a_val, const uint32_t* b_idx, const float* b_val,
                int32_t k, int32_t batch, int64_t in_stride, uint32_t* out_idx, float* out_val,
                int64_t out_stride, void* ws, size_t ws_bytes, void* stream) {
    if (!a_idx || !a_val || !b_idx || !b_val || !out_idx || !out_val || !ws) return GTOPK_EINVAL;
    if (k < 1 || k > kMaxMergeK || batch < 1 || batch > 32767 || in_stride < k || out_stride < k)
        return GTOPK_EINVAL;
    if (!aligned16(a_idx) || !aligned16(a_val) || !aligned16(b_idx) || !aligned16(b_val) ||
        !aligned16(out_idx) || !aligned16(out_val) || !aligned16(ws))
        return GTOPK_EALIGN;
    Carver c{reinterpret_cast<char*>(ws)};
    const MergeWs w = carve_merge(c, (uint32_t)k, (size_t)batch);
    if (ws_bytes < w.bytes) return GTOPK_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    zero_async(st, zero_job(w.sel.hist, select_clear_words(w.sel), w.inv_min, 2 * (size_t)batch));
    hipLaunchKernelGGL(k_set_min_key, dim3(min_key_blocks((uint32_t)k), 2 * (uint32_t)batch),
                       dim3(kBlock), 0, st, a_val, b_val, in_stride, (uint32_t)k, w.inv_min);
    do_merge_batch<false>(a_idx, a_val, b_idx, b_val, (uint32_t)k, (uint32_t)batch, in_stride,
                          out_idx, out_val, out_stride, w, 0, w.inv_min, true, nullptr, 1.0f, nullptr,
                          st);
    return launch_status();
}

int gtopk_tree(const uint32_t* loc_idx, const float* loc_val, int32_t P, int32_t k, uint32_t* g_idx,
               float* g_val, void* ws, size_t ws_bytes, void* stream) {
    if (!loc_idx || !loc_val || !g_idx || !g_val || !ws) return GTOPK_EINVAL;
    if (k < 1 || k > kMaxMergeK || !is_pow2(P) || P > 65535) return GTOPK_EINVAL;
    if (!aligned16(loc_idx) || !aligned16(loc_val) || !aligned16(g_idx) || !aligned16(g_val) ||
        !aligned16(ws))
        return GTOPK_EALIGN;
    // the tree's scratch sits inside the step workspace; m only sizes the parts it does not use
    const StepWs w = carve_step(ws, (int64_t)k, (uint32_t)k, (uint32_t)P);
    if (ws_bytes < w.bytes) return GTOPK_EWORKSPACE;
    return do_tree(loc_idx, loc_val, nullptr, (uint32_t)P, (uint32_t)k, g_idx, g_val, w, nullptr,
                   false, (hipStream_t)stream);
}

int gtopk_residual_restore(float* residual, int64_t m, int64_t stride, int32_t P, int32_t k,
                           const uint32_t* loc_idx, const float* loc_val, const uint32_t* g_idx,
                           void* stream) {
    if (!residual || !loc_idx || !loc_val || !g_idx) return GTOPK_EINVAL;
    if (!sizes_ok(m, k, P) || stride < m) return GTOPK_EINVAL;
    if (!aligned16(residual) || !aligned16(loc_idx) || !aligned16(loc_val) || !aligned16(g_idx))
        return GTOPK_EALIGN;
    hipLaunchKernelGGL(k_restore, dim3(ceil_div((uint32_t)k, kBlock), (uint32_t)P), dim3(kBlock), 0,
                       (hipStream_t)stream, residual, (uint32_t)m, stride, (uint32_t)k, loc_idx, loc_val,
                       g_idx);
    return launch_status();
}

static int step_impl(const float* grad, float* residual, int64_t m, int64_t stride, int32_t P,
                     int32_t k, uint32_t* g_idx, float* g_val, uint32_t* loc_idx, float* loc_val,
                     void* ws, size_t ws_bytes, void* stream, void* const* events,
                     uint32_t* thr_state = nullptr) {
    if (!grad || !residual || !g_idx || !g_val || !ws) return GTOPK_EINVAL;
    if (!aligned16(thr_state)) return GTOPK_EALIGN;
    if ((loc_idx == nullptr) != (loc_val == nullptr)) return GTOPK_EINVAL;
    if (!sizes_ok(m, k, P) || stride < m) return GTOPK_EINVAL;
    if (!aligned16(grad) || !aligned16(residual) || !aligned16(g_idx) || !aligned16(g_val) ||
        !aligned16(loc_idx) || !aligned16(loc_val) || !aligned16(ws))
        return GTOPK_EALIGN;
    const StepWs w = carve_step(ws, m, (uint32_t)k, (uint32_t)P);
    if (ws_bytes < w.bytes) return GTOPK_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    uint32_t* li = loc_idx ? loc_idx : w.loc_idx;
    float* lv = loc_val ? loc_val : w.loc_val;
    if (!events && !thr_state && small_problem(m, k, P)) {
        // one block per worker samples, picks the threshold and clears the candidate counter
        const SamplePlan sp = plan_sample(m, (uint32_t)k, kSmallSampleMean, kSmallSampleMinTiles);
        hipLaunchKernelGGL(k_small_sample, dim3(P), dim3(kSmallBlock), 0, st, grad, residual,
                           (uint32_t)m, stride, sp.tile_stride, sp.n_tiles, sp.target, w.tspec,
                           w.cand_count);
        // small blocks: one run per 4096 elements (the run table was carved for that many)
        const uint32_t nruns = ceil_div((uint64_t)m + 3, kSmallChunk);
        hipLaunchKernelGGL((k_accum_filter<false, kSmallIters>), dim3(nruns, P), dim3(kSBlock), 0, st,
                           grad, residual, (uint32_t)m, stride, w.tspec, w.cand_idx, w.cand_val, w.cap,
                           w.cand_count, w.run_table, nruns, w.sel.hist);
        CandSrc src = cand_source(residual, stride, m, (uint32_t)k, w, false, false);
        src.nchunks = nruns;
        hipLaunchKernelGGL(k_small_select, dim3(P), dim3(kSmallBlock), 0, st, src, (uint32_t)k, li, lv);
        hipLaunchKernelGGL(k_small_tree, dim3(1), dim3(kSmallBlock), 0, st, li, lv, (uint32_t)P,
                           (uint32_t)k, g_idx, g_val, (float)P, residual, stride);
        return launch_status();
    }
    mark_stage(0, events, st);
    // one clear for everything this step needs zeroed: the sampler's histograms and the
    // candidate counters; both selects' histograms and tickets; the global-set bitmap
    zero_async(st, zero_job(w.samp_hist, (size_t)(w.tspec - w.samp_hist), w.sel.hist,
                            select_clear_words(w.sel), w.mrg.sel.hist, select_clear_words(w.mrg.sel),
                            w.mrg.sel_alt.hist, w.mrg.alt_clear_words, w.gbits, w.gbits_words));
    int rc = do_local_select(grad, residual, m, stride, (uint32_t)P, (uint32_t)k, li, lv, w, false,
                             true, st, events, thr_state);
    if (rc != GTOPK_OK) return rc;
    mark_stage(3, events, st);
    rc = do_tree(li, lv, w.sel.T, (uint32_t)P, (uint32_t)k, g_idx, g_val, w, w.gbits, true, st);
    if (rc != GTOPK_OK) return rc;
    mark_stage(4, events, st);
    hipLaunchKernelGGL(k_restore_fused, dim3(ceil_div((uint32_t)k, kBlock), (uint32_t)P), dim3(kBlock),
                       0, st, residual, stride, (uint32_t)k, li, lv, w.gbits, (const uint32_t*)w.sel.T);
    rc = launch_status();
    mark_stage(5, events, st);
    return rc;
}

int gtopk_step(const float* grad, float* residual, int64_t m, int64_t stride, int32_t P, int32_t k,
               uint32_t* g_idx, float* g_val, uint32_t* loc_idx, float* loc_val, void* ws,
               size_t ws_bytes, void* stream) {
    return step_impl(grad, residual, m, stride, P, k, g_idx, g_val, loc_idx, loc_val, ws, ws_bytes,
                     stream, nullptr);
}

// ---------------------------------------------------------------------------------
// gtopk_step for callers that cannot allocate: the workspace is a file-scope device array
// ---------------------------------------------------------------------------------
}  // extern "C"

// Every GPU the library runs on holds its own copy of this array until the process ends.
// In host code the name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[GTOPK_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};     // device address of `scratch` on each device, once known

// device address of `scratch` on the current device (looked up once per device), or NULL
void* scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" {

int gtopk_step_static(const float* grad, float* residual, int64_t m, int64_t stride, int32_t P,
                      int32_t k, uint32_t* g_idx, float* g_val, uint32_t* loc_idx, float* loc_val,
                      void* stream) {
    if (!sizes_ok(m, k, P)) return GTOPK_EINVAL;
    const size_t need = carve_step(nullptr, m, (uint32_t)k, (uint32_t)P).bytes;
    if (need > (size_t)GTOPK_STATIC_WORKSPACE_BYTES) return GTOPK_EWORKSPACE;
    void* ws = scratch_on_current_device();
    if (!ws) return GTOPK_EHIP;
    // everything the step needs zeroed is cleared by its first kernel, so what the
    // previous call left in the array does not matter
    return step_impl(grad, residual, m, stride, P, k, g_idx, g_val, loc_idx, loc_val, ws,
                     (size_t)GTOPK_STATIC_WORKSPACE_BYTES, stream, nullptr);
}

int gtopk_step_carry(const float* grad, float* residual, int64_t m, int64_t stride, int32_t P,
                     int32_t k, uint32_t* g_idx, float* g_val, uint32_t* loc_idx, float* loc_val,
                     uint32_t* thr_state, void* ws, size_t ws_bytes, void* stream) {
    if (!thr_state) return GTOPK_EINVAL;
    return step_impl(grad, residual, m, stride, P, k, g_idx, g_val, loc_idx, loc_val, ws, ws_bytes,
                     stream, nullptr, thr_state);
}

int gtopk_step_timed(const float* grad, float* residual, int64_t m, int64_t stride, int32_t P,
                     int32_t k, uint32_t* g_idx, float* g_val, uint32_t* loc_idx, float* loc_val,
                     uint32_t* thr_state, void* ws, size_t ws_bytes, void* stream,
                     void* const* events) {
    if (!events) return GTOPK_EINVAL;
    for (int i = 0; i < GTOPK_STAGE_EVENTS; ++i)
        if (!events[i]) return GTOPK_EINVAL;
    return step_impl(grad, residual, m, stride, P, k, g_idx, g_val, loc_idx, loc_val, ws, ws_bytes,
                     stream, events, thr_state);
}

int gtopk_apply_update(float* weights, int64_t m, int64_t stride, int32_t copies, int32_t k,
                       const uint32_t* g_idx, const float* g_val, float lr, void* stream) {
    if (!weights || !g_idx || !g_val) return GTOPK_EINVAL;
    if (m < 1 || m > ((int64_t)1 << 31) || k < 1 || k > m || stride < m || copies < 1 ||
        copies > 65535)
        return GTOPK_EINVAL;
    if (!aligned16(weights) || !aligned16(g_idx) || !aligned16(g_val)) return GTOPK_EALIGN;
    hipLaunchKernelGGL(k_apply_update, dim3(ceil_div((uint32_t)k, kBlock), (uint32_t)copies),
                       dim3(kBlock), 0, (hipStream_t)stream, weights, (uint32_t)m, stride, (uint32_t)k, g_idx,
                       g_val, lr);
    return launch_status();
}

int gtopk_dense_mask(const uint32_t* g_idx, int32_t k, int64_t m, uint8_t* mask, void* stream) {
    if (!g_idx || !mask) return GTOPK_EINVAL;
    if (m < 1 || m > ((int64_t)1 << 31) || k < 1 || k > m) return GTOPK_EINVAL;
    if (!aligned16(g_idx) || !aligned16(mask)) return GTOPK_EALIGN;
    hipStream_t st = (hipStream_t)stream;
    uint32_t blocks = ceil_div((uint64_t)m, 256 * 16);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(k_mask_clear, dim3(blocks), dim3(256), 0, st, mask, (uint64_t)m);
    hipLaunchKernelGGL(k_mask_set, dim3(ceil_div((uint32_t)k, kBlock)), dim3(kBlock), 0, st, mask,
                       (uint32_t)m, (uint32_t)k, g_idx);
    return launch_status();
}

size_t gtopk_allreduce_workspace_bytes(int64_t m, int32_t P) {
    if (m < 1 || m > ((int64_t)1 << 31) || P < 1 || P > kAggMaxP) return 0;
    const uint64_t nranges = ceil_div((uint64_t)m, kAggRange);
    return (size_t)(((uint64_t)P * (nranges + 1) * sizeof(uint32_t) + 255) & ~(uint64_t)255);
}

int gtopk_topk_allreduce(const uint32_t* loc_idx, const float* loc_val, int32_t P, int32_t k,
                         int64_t m, float* dense, void* ws, size_t ws_bytes, void* stream) {
    if (!loc_idx || !loc_val || !dense || !ws) return GTOPK_EINVAL;
    if (m < 1 || m > ((int64_t)1 << 31) || k < 1 || k > m || P < 1 || P > kAggMaxP)
        return GTOPK_EINVAL;
    if (!aligned16(loc_idx) || !aligned16(loc_val) || !aligned16(dense) || !aligned16(ws))
        return GTOPK_EALIGN;
    if (ws_bytes < gtopk_allreduce_workspace_bytes(m, P)) return GTOPK_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const uint32_t nranges = ceil_div((uint64_t)m, kAggRange);
    uint32_t* bounds = reinterpret_cast<uint32_t*>(ws);
    hipLaunchKernelGGL(k_slice_bounds, dim3(ceil_div(nranges + 1, kBlock), (uint32_t)P), dim3(kBlock),
                       0, st, loc_idx, (uint32_t)k, nranges, bounds);
    hipLaunchKernelGGL(k_scatter_mean, dim3(nranges), dim3(kBlock), 0, st, loc_idx, loc_val,
                       (uint32_t)P, (uint32_t)k, (uint32_t)m, bounds, nranges, (float)P, dense);
    return launch_status();
}

int gtopk_dense_topk(const float* dense, int64_t m, int32_t k, uint32_t* g_idx, float* g_val,
                     void* ws, size_t ws_bytes, void* stream) {
    if (!dense || !g_idx || !g_val || !ws) return GTOPK_EINVAL;
    if (!sizes_ok(m, k, 1)) return GTOPK_EINVAL;
    if (!aligned16(dense) || !aligned16(g_idx) || !aligned16(g_val) || !aligned16(ws))
        return GTOPK_EALIGN;
    const StepWs w = carve_step(ws, m, (uint32_t)k, 1);
    if (ws_bytes < w.bytes) return GTOPK_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    // a candidate count of zero makes the select read the dense row itself
    zero_async(st, zero_job(w.samp_hist, (size_t)(w.tspec - w.samp_hist), w.sel.hist, select_clear_words(w.sel)));
    const CandSrc src = cand_source(dense, m, m, (uint32_t)k, w, false, /*no_bounds=*/true);
    // one set, always read as a dense row: the grids follow the row's groups; without a
    // lower bound of the k-th key the list can be long, so large rows are finished once
    const SelGrid gr{1, w.gdense, w.gdense, (uint64_t)m, m > ((int64_t)1 << 20)};
    run_select<CandSrc, false>(src, w.sel, gr, (uint32_t)k, g_idx, g_val, (int64_t)k, 1.0f, nullptr, st);
    return launch_status();
}

int gtopk_debug_candidate_counts(const void* ws, int64_t m, int32_t k, int32_t P,
                                 uint32_t* host_counts, uint32_t* host_capacity) {
    if (!ws || !host_counts || !host_capacity || !sizes_ok(m, k, P)) return GTOPK_EINVAL;
    const StepWs w = carve_step(const_cast<void*>(ws), m, (uint32_t)k, (uint32_t)P);
    *host_capacity = w.cap;
    if (hipMemcpy(host_counts, w.cand_count, sizeof(uint32_t) * (size_t)P, hipMemcpyDeviceToHost) !=
        hipSuccess)
        return GTOPK_EHIP;
    return GTOPK_OK;
}

int gtopk_debug_merge_kept(const void* ws, int32_t k, int32_t batch, uint32_t* host_kept) {
    if (!ws || !host_kept || k < 1 || k > kMaxMergeK || batch < 1 || batch > 32767) return GTOPK_EINVAL;
    Carver c{reinterpret_cast<char*>(const_cast<void*>(ws))};
    const MergeWs w = carve_merge(c, (uint32_t)k, (size_t)batch);
    if (!w.f_set_cnt) return GTOPK_EINVAL;               // merges of this k are not filtered
    if (hipMemcpy(host_kept, w.f_set_cnt, sizeof(uint32_t) * (size_t)batch, hipMemcpyDeviceToHost) !=
        hipSuccess)
        return GTOPK_EHIP;
    return GTOPK_OK;
}

int gtopk_probe_stream(const float* a, float* b, int64_t n, int32_t mode, float* sink,
                       void* stream) {
    if (!a || !b || n < 1 || n % kChunk != 0 || n / kChunk > 0x7fffffff) return GTOPK_EINVAL;
    if (mode < 0 || mode >= GTOPK_PROBE_MODES) return GTOPK_EINVAL;
    if (mode == 1 && !sink) return GTOPK_EINVAL;
    if (!aligned16(a) || !aligned16(b) || !aligned16(sink)) return GTOPK_EALIGN;
    const uint32_t blocks = (uint32_t)(n / kChunk);      // of the pass's shape: 32768 elements each
    hipStream_t st = (hipStream_t)stream;
    switch (mode) {
        case 0: hipLaunchKernelGGL(k_probe_stream<true>, dim3(blocks), dim3(kSBlock), 0, st, a, b, sink); break;
        case 1: hipLaunchKernelGGL(k_probe_stream<false>, dim3(blocks), dim3(kSBlock), 0, st, a, b, sink); break;
        // cache policy
        case 2: hipLaunchKernelGGL((k_probe_stream<true, false, true>), dim3(blocks), dim3(kSBlock), 0, st, a, b, sink); break;
        case 3: hipLaunchKernelGGL((k_probe_stream<true, true, false>), dim3(blocks), dim3(kSBlock), 0, st, a, b, sink); break;
        case 4: hipLaunchKernelGGL((k_probe_stream<true, false, false>), dim3(blocks), dim3(kSBlock), 0, st, a, b, sink); break;
        // block shape (elements per block: 32768, 32768, 8192)
        case 5: hipLaunchKernelGGL((k_probe_stream<true, true, true, 256, 32>), dim3(blocks), dim3(256), 0, st, a, b, sink); break;
        case 6: hipLaunchKernelGGL((k_probe_stream<true, true, true, 1024, 8>), dim3(blocks), dim3(1024), 0, st, a, b, sink); break;
        default: hipLaunchKernelGGL((k_probe_stream<true, true, true, 512, 4>), dim3(blocks * 4), dim3(512), 0, st, a, b, sink); break;
    }
    return launch_status();
}

int gtopk_debug_plan(int64_t m, int32_t k, int32_t P, uint32_t* plan) {
    if (!plan || !sizes_ok(m, k, P)) return GTOPK_EINVAL;
    const SamplePlan sp = plan_sample(m, (uint32_t)k);
    plan[0] = sp.tile_stride;
    plan[1] = sp.n_tiles;
    plan[2] = (uint32_t)kSampleTile;
    plan[3] = sp.target;
    plan[4] = cand_capacity(m, (uint32_t)k);
    plan[5] = pass_histograms(m, (uint32_t)k) ? 1u : 0u;
    plan[6] = small_problem(m, k, P) ? 1u : 0u;
    plan[7] = run_groups(m, (uint32_t)k) ? 1u : 0u;
    for (int i = 8; i < GTOPK_PLAN_WORDS; ++i) plan[i] = 0u;
    if (P > 1 && merge_filtered((uint32_t)k)) {
        const MergeSamplePlan mp = plan_merge_sample((uint32_t)k);
        plan[11] = 1u;
        plan[12] = mp.tile_stride;
        plan[13] = mp.n_tiles;
        plan[14] = mp.target;
    }
    if (plan[6]) {
        const SamplePlan ss = plan_sample(m, (uint32_t)k, kSmallSampleMean, kSmallSampleMinTiles);
        plan[8] = ss.tile_stride;
        plan[9] = ss.n_tiles;
        plan[10] = ss.target;
    }
    return GTOPK_OK;
}

}  // extern "C"
