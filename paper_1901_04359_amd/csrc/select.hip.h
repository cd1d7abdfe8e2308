// Exact selection of the k entries with the largest keys out of a set, written out in
// index order: the common core of the local selection (Algorithm 4 lines 5-7) and of the
// Top-k operation between two sparse vectors (Definition 1).
//
// Three kernels per batch of sets:
//   k_hist    4096-bin histogram of the keys' first digit
//   k_bucket  every block picks, from that histogram, the bin d1 that holds the k-th
//             key; then, per group of slots: count of keys above the bin; keys inside
//             the bin are appended (with their group) to a short list.  For the local
//             selection of short runs this walk also copies the candidates, which the
//             streaming pass left as runs in arbitrary order, into index order (CandSrc);
//             long runs are selected where they lie, one group per run (RunSrc), a run per
//             wave of the walk's blocks.  Long groups of a merged set are walked four slots
//             per load.
//   k_emit    every block: LDS radix passes over the list give the exact key T and the
//             number of ties to take, and the block's output offsets; then, per group:
//             ordered compaction of the selected entries
// For large sets (long lists) the first half of k_emit runs once per set in a kernel of
// its own, k_finish, instead of once per block; the keys inside the bin then stay with their
// groups (SelState::seg_list) instead of going through one shared list counter.  Where the kernel that produces a set's
// entries has counted their first digits itself (the unions of the tree; the streaming
// pass at most densities), k_hist is not launched or has nothing to do for that set.
#pragma once
#include "common.hip.h"

namespace gtopk {

// per-set state of the exact select
struct SelState {
    // ---- must be zero when a select starts (cleared by the host side / the union) -------
    uint32_t* hist;       // [sets][4096]
    uint32_t* list_cnt;   // [sets]
    uint32_t* grp_gt;     // [sets][maxgroups] entries of the group above bin d1
    uint32_t* grp_in;     // [sets][maxgroups] entries of the group inside bin d1
    uint32_t* bin_hi;     // [sets] largest key seen inside bin d1
    uint32_t* bin_lo_inv; // [sets] 0x7fffffff - smallest key seen inside bin d1
    uint32_t* hist_dense; // [sets][4096] or NULL: the histogram of a set that is read as a dense
                          //   row although the producer of its candidates has already filled `hist`
    // --------------------------------------------------------------------------------
    uint32_t* d1;         // [sets] bin of the k-th key
    uint32_t* krem;       // [sets] rank of the k-th key inside bin d1 (1-based, from the top)
    uint32_t* T;          // [sets] the k-th largest key = the smallest key of the output set
    uint32_t* T_out;      // [sets] optional second copy of T that outlives the next select (or NULL)
    uint32_t* need;       // [sets] entries with key == T to take (>= 1)
    uint2* list;          // [sets][list_cap]  (key, group)
    uint32_t* off_gt;     // [sets][maxgroups] written by k_finish only: selected entries with
    uint32_t* off_eq;     //   key > T / entries with key == T in the groups before this one
    uint32_t list_cap, maxgroups;
    // seg_list != 0 (large merged sets, finished by k_finish): the in-bin keys of group g are not
    // appended to one list through a shared counter but stored from position (first slot of
    // group g) of `list` on, grp_in[g] of them - a block of k_bucket then waits for no atomic
    // (all blocks of a set reserving on one counter cost the walk a quarter of its time);
    // list_cnt stays 0
    uint32_t seg_list;
};

// ---------------------------------------------------------------------------------
// item sources
// ---------------------------------------------------------------------------------
// A source presents, per set s, nphys(s) "physical" slots in storage order and the same
// items in "logical" = index order, cut into groups of group_slots() consecutive logical
// positions.  k_hist and k_bucket walk the physical slots; logical() maps a physical slot
// to its logical position; kIdentity says the two orders coincide.  fetch_ord() reads an
// item by logical position (for the ordered emit).  fetch_*() return false for a slot that
// holds nothing.  group_range() hands a block the slots of a group of a set that is not
// read as a dense row; sources whose groups are not equal cuts of the logical order
// (kRunGroups: the runs of the streaming pass, the tiles of a filtered union) answer it
// from their own tables.  skip() takes a set out of a launch altogether.

// Local select: the candidate list of worker s, or - when the speculative threshold
// left fewer than k candidates or more than the list holds - the worker's dense row.
// The streaming pass leaves the candidates as one run per 32768-element chunk of the row,
// in index order inside a run, the runs in the order in which the blocks reserved them
// (run_table[w][chunk] = first slot, count); one extra block of k_hist scans the run
// counts (run_off[w][chunk] = first logical position of the run), and k_bucket's walk
// copies the candidates into index order on the side.
struct CandSrc {
    __device__ bool skip(int) const { return false; }     // every set of the launch is selected
    static constexpr bool kRunGroups = false;
    static constexpr bool kWaveGroups = false;
    static constexpr bool kVectorWalk = false;
    static constexpr bool kSegList = false;
    static constexpr bool kValueOnlyWalk = false;
    __device__ uint32_t fetch_bits(int, uint32_t) const { return 0u; }
    __device__ bool is_tomb(int, uint32_t) const { return false; }
    static constexpr bool kIdentity = false;
    static constexpr bool kRunScan = true;
    const float* res;
    int64_t stride;
    uint32_t m, k, cap, nchunks;
    uint32_t Lc, Ld;                      // slots per group: candidate list / dense row
    const uint32_t* cand_idx;             // [P][cap] runs in reservation order
    const float* cand_val;
    const uint32_t* cand_count;           // [P]
    const uint32_t* tspec;                // [P] speculative threshold = lower bound of all candidates
    const uint2* run_table;               // [P][nchunks] (first physical slot, count)
    uint32_t* run_off;                    // [P][nchunks] first logical position of the run
    uint32_t* ord_idx;                    // [P][cap] candidates in index order
    float* ord_val;
    bool producer_hist;                   // the streaming pass has histogrammed the candidates
    bool no_bounds;                       // dense rows without any threshold (the dense top-k)
    uint4* carry_state;                   // [P] or NULL: thresholds carried from call to call

    // Called once per set, by the thread that records the set's exact k-th key T: works out
    // the speculative threshold of the worker's NEXT call from what this call has seen.
    //   x  0: nothing known, 1: learning (the next call samples), 2: the next call filters
    //      with w instead of sampling
    //   y  T of this call          z  margin d between the predicted T and the threshold
    //   w  threshold for the next call = predicted T - d; the prediction is T + (T - previous T)
    // The margin follows the number of candidates the pass kept (aim: 1.25 k .. 2.2 k); the
    // next call may skip sampling once a prediction has come true to within half the
    // margin, and goes back to sampling when the list came close to either of its limits.
    // A wrong threshold costs time only: the select is exact whatever it filters with.
    __device__ void carry(int s, uint32_t T) const {
        if (!carry_state) return;
        uint4 c = carry_state[s];
        const uint32_t n = cand_count[s], ts = tspec[s];
        if (n < k || n > cap || no_bounds) {             // this call fell back to the dense row
            carry_state[s] = make_uint4(0u, T, c.z, 0u);
            return;
        }
        uint32_t d = c.z;
        uint32_t mode = 1;
        long long pred_next = (long long)T;
        if (c.x == 0) {
            d = T - ts;                                  // what the sampler chose
        } else {
            const long long pred = (long long)c.w + (long long)c.z;      // last call's prediction of T
            const long long err = pred > (long long)T ? pred - (long long)T : (long long)T - pred;
            if ((uint64_t)n * 100 > (uint64_t)k * 220) d -= d / 4;
            else if ((uint64_t)n * 100 < (uint64_t)k * 125) d += d / 2;
            const bool came_true = err * 2 <= (long long)d;
            const bool roomy = (uint64_t)n * 100 >= (uint64_t)k * 108 && (uint64_t)n * 100 <= (uint64_t)cap * 85;
            mode = (came_true && roomy) ? 2u : 1u;
            pred_next = 2ll * (long long)T - (long long)c.y;
        }
        if (d < 256u) d = 256u;
        if (d > T / 2 + 256u) d = T / 2 + 256u;
        if (pred_next < 0) pred_next = 0;
        if (pred_next > (long long)kAbs) pred_next = (long long)kAbs;
        const uint32_t next = pred_next > (long long)d ? (uint32_t)(pred_next - (long long)d) : 0u;
        carry_state[s] = make_uint4(mode, T, d, next);
    }

    __device__ bool dense(int s) const {
        const uint32_t c = cand_count[s];
        return c < k || c > cap;
    }
    // A dense row with MORE candidates than the list holds: the k-th key is at or above the
    // speculative threshold, and if the pass has histogrammed its candidates, that
    // histogram (which counts every candidate, stored or not) is the row's.
    __device__ bool overfull(int s) const { return !no_bounds && cand_count[s] > cap; }
    __device__ bool wants_hist(int s, bool dn) const {
        return !producer_hist || (dn && !overfull(s));
    }
    // Entries of such a row below the speculative threshold cannot be selected (more than k
    // others lie above it); the select ignores them, as if the row were a candidate list.
    __device__ uint32_t floor_key(int s, bool dn) const {
        return (dn && overfull(s)) ? tspec[s] : 0u;
    }
    __device__ uint32_t* hist_of(int s, bool dn, const SelState& st) const {
        return ((producer_hist && dn && !overfull(s)) ? st.hist_dense : st.hist) + (size_t)s * kHistBins;
    }
    __device__ uint32_t nphys(int s, bool dn) const { return dn ? m : cand_count[s]; }
    __device__ uint32_t group_slots(bool dn) const { return dn ? Ld : Lc; }
    __device__ uint32_t ngroups(int s, bool dn) const {
        return (uint32_t)(((uint64_t)nphys(s, dn) + group_slots(dn) - 1) / group_slots(dn));
    }
    // slots [first, end) that a block walks for group g of a set that is not a dense row
    // (false: none); and the group of the item at physical slot p
    __device__ bool group_range(int s, uint32_t g, uint32_t& first, uint32_t& end) const {
        const uint32_t n = cand_count[s];
        const uint64_t f = (uint64_t)g * Lc;
        if (f >= n) return false;
        first = (uint32_t)f;
        end = (uint32_t)(f + Lc < n ? f + Lc : n);
        return true;
    }
    __device__ uint32_t group_of(int s, bool dn, uint32_t p, uint32_t idx) const {
        return logical(s, dn, p, idx) / group_slots(dn);
    }
    // fetch_ord() for a position inside a range that group_range() has handed out
    __device__ bool fetch_emit(int s, bool dn, uint32_t lp, uint32_t& idx, uint32_t& bits) const {
        return fetch_ord(s, dn, lp, idx, bits);
    }
    // ... and of the item that fetch_ord() reads at position lp
    __device__ uint32_t group_of_ord(int, bool dn, uint32_t lp, uint32_t) const { return lp / group_slots(dn); }
    // Lower bound of the k-th key: the speculative threshold while at least k entries
    // reached it; for a worker with fewer the k-th key lies below it, and nothing bounds
    // it from below: plain coarse bins.
    __device__ Digit digit(int s, bool dn, const SelState&) const {
        if (dn && !overfull(s)) return Digit{0u, (uint32_t)kCoarseShift};
        return Digit{tspec[s], (uint32_t)kFineShift};
    }
    __device__ bool fetch_phys(int s, bool dn, uint32_t p, uint32_t& idx, uint32_t& bits) const {
        if (dn) {
            idx = p;
            bits = __float_as_uint(res[(int64_t)s * stride + p]);
        } else {
            idx = cand_idx[(size_t)s * cap + p];
            bits = __float_as_uint(cand_val[(size_t)s * cap + p]);
        }
        return true;
    }
    __device__ bool fetch_key_phys(int s, bool dn, uint32_t p, uint32_t& key) const {
        key = __float_as_uint(dn ? res[(int64_t)s * stride + p] : cand_val[(size_t)s * cap + p]) & kAbs;
        return true;
    }
    __device__ uint32_t logical(int s, bool dn, uint32_t p, uint32_t idx) const {
        if (dn) return p;
        // the streaming pass cuts a row into chunks at multiples of 32768 of idx + head
        const uint32_t head = (uint32_t)(((int64_t)s * stride) & 3);
        uint32_t chunk = (idx + head) >> kChunkLog2;
        if (chunk >= nchunks) chunk = nchunks - 1;       // never for a list the pass wrote
        const size_t r = (size_t)s * nchunks + chunk;
        const uint32_t lp = run_off[r] + (p - run_table[r].x);
        return lp < cap ? lp : cap - 1;                  // likewise
    }
    __device__ void store_ordered(int s, bool dn, uint32_t lp, uint32_t idx, uint32_t bits) const {
        if (!dn) {
            ord_idx[(size_t)s * cap + lp] = idx;
            ord_val[(size_t)s * cap + lp] = __uint_as_float(bits);
        }
    }
    __device__ bool fetch_ord(int s, bool dn, uint32_t lp, uint32_t& idx, uint32_t& bits) const {
        if (dn) {
            idx = lp;
            bits = __float_as_uint(res[(int64_t)s * stride + lp]);
        } else {
            idx = ord_idx[(size_t)s * cap + lp];
            bits = __float_as_uint(ord_val[(size_t)s * cap + lp]);
        }
        return true;
    }
    // exclusive scan of the run counts of worker s, by one block of kHistBlock threads
    __device__ void scan_runs(int s, uint32_t* s_wave) const {
        uint32_t carry = 0;
        for (uint32_t c0 = 0; c0 < nchunks; c0 += kHistBlock) {
            const uint32_t c = c0 + threadIdx.x;
            const uint32_t v = c < nchunks ? run_table[(size_t)s * nchunks + c].y : 0u;
            uint32_t tot;
            const uint32_t incl = block_incl_scan(v, s_wave, tot);
            if (c < nchunks) run_off[(size_t)s * nchunks + c] = carry + incl - v;
            carry += tot;
        }
    }
};

// The local select of LONG candidate lists (hundreds of candidates or more per chunk of the row):
// the groups are the runs themselves - group g of worker s is the run of chunk g, where the
// streaming pass left it - so nothing is copied into index order: the walk of k_bucket
// reads a run's values only, the emit reads the run's indices and values in place.  Runs
// differ in length (0 .. 32768 entries); with hundreds of runs per worker the blocks even
// out.  A worker that falls back to its dense row is handled as in CandSrc.
// kWaveGroups: every WAVE of a block of k_bucket / k_emit takes a run of its own (a block
// per run spends its time on the block's fixed chain of dependent loads, not on the run).
struct RunSrc : CandSrc {
    static constexpr bool kRunGroups = true;
    static constexpr bool kWaveGroups = true;
    static constexpr bool kValueOnlyWalk = true;
    static constexpr bool kRunScan = false;
    __device__ uint32_t fetch_bits(int s, uint32_t p) const { return __float_as_uint(cand_val[(size_t)s * cap + p]); }
    __device__ bool is_tomb(int, uint32_t) const { return false; }
    __device__ uint32_t ngroups(int s, bool dn) const { return dn ? CandSrc::ngroups(s, dn) : nchunks; }
    __device__ bool group_range(int s, uint32_t g, uint32_t& first, uint32_t& end) const {
        if (g >= nchunks) return false;
        const uint2 run = run_table[(size_t)s * nchunks + g];
        if (run.y == 0u || run.x >= cap) return false;
        first = run.x;
        end = run.y < cap - run.x ? run.x + run.y : cap;        // never cut for a list the pass wrote
        return true;
    }
    __device__ uint32_t group_of(int s, bool dn, uint32_t p, uint32_t idx) const {
        if (dn) return p / Ld;
        const uint32_t head = (uint32_t)(((int64_t)s * stride) & 3);
        const uint32_t chunk = (idx + head) >> kChunkLog2;
        return chunk < nchunks ? chunk : nchunks - 1;          // likewise
    }
    __device__ bool fetch_ord(int s, bool dn, uint32_t p, uint32_t& idx, uint32_t& bits) const {
        return fetch_phys(s, dn, p, idx, bits);
    }
    __device__ uint32_t group_of_ord(int s, bool dn, uint32_t p, uint32_t idx) const { return group_of(s, dn, p, idx); }
    __device__ bool fetch_emit(int s, bool dn, uint32_t p, uint32_t& idx, uint32_t& bits) const {
        return fetch_phys(s, dn, p, idx, bits);
    }
};

// Merge: n = 2k slots per pair (rows `stride` slots apart), index-ascending, a slot with
// index kTomb holds nothing.
// Every key of the union that is a plain copy of an operand's entry is at least that
// operand's smallest key, so the larger of the two smallest keys bounds the k-th key of
// the union from below (sums that cancel can fall under it; they land in bin 0).
// in_min[2s], in_min[2s+1] are those smallest keys (NULL: not known; inverted: stored as
// 0x7fffffff - key, the form in which k_set_min_key's atomic maximum leaves them).
struct MergedSrc {
    static constexpr bool kRunGroups = false;
    static constexpr bool kWaveGroups = false;
    // rows of values are 16-byte aligned and padded to whole vectors, groups start at
    // multiples of four slots: k_bucket walks them four slots per load
    static constexpr bool kVectorWalk = true;
    static constexpr bool kSegList = true;          // no set of this source is ever read as a dense row
    __device__ const uint32_t* value_row(int s) const { return reinterpret_cast<const uint32_t*>(val) + (size_t)s * stride; }
    static constexpr bool kIdentity = true;
    static constexpr bool kRunScan = false;
    // A tombstone's value is +0.0: its key falls into the lowest bin of either digit layout, so
    // a walk that only counts keys ABOVE a bin, and looks closer only at keys INSIDE it, can
    // read the values alone and ask is_tomb() for the few slots inside the bin.
    static constexpr bool kValueOnlyWalk = true;
    __device__ uint32_t fetch_bits(int s, uint32_t p) const { return __float_as_uint(val[(size_t)s * stride + p]); }
    __device__ bool is_tomb(int s, uint32_t p) const { return idx[(size_t)s * stride + p] == kTomb; }
    const uint32_t* idx;
    const float* val;
    uint32_t n, stride, L;       // L slots per group
    const uint32_t* in_min;
    bool inverted;
    // optional gate: set s is selected only if gate_cnt[s] < gate_k (the sets whose filtered
    // union came out short, see FiltSrc); NULL: every set
    const uint32_t* gate_cnt;
    uint32_t gate_k;
    __device__ bool skip(int s) const { return gate_cnt && gate_cnt[s] >= gate_k; }
    __device__ bool dense(int) const { return false; }
    __device__ void carry(int, uint32_t) const {}
    __device__ uint32_t floor_key(int, bool) const { return 0u; }
    __device__ bool wants_hist(int, bool) const { return true; }
    __device__ uint32_t* hist_of(int s, bool, const SelState& st) const {
        return st.hist + (size_t)s * kHistBins;
    }
    __device__ uint32_t nphys(int, bool) const { return n; }
    __device__ uint32_t group_slots(bool) const { return L; }
    __device__ uint32_t ngroups(int, bool) const { return (uint32_t)(((uint64_t)n + L - 1) / L); }
    __device__ bool group_range(int, uint32_t g, uint32_t& first, uint32_t& end) const {
        const uint64_t f = (uint64_t)g * L;
        if (f >= n) return false;
        first = (uint32_t)f;
        end = (uint32_t)(f + L < n ? f + L : n);
        return true;
    }
    __device__ uint32_t group_of(int, bool, uint32_t p, uint32_t) const { return p / L; }
    __device__ uint32_t group_of_ord(int, bool, uint32_t lp, uint32_t) const { return lp / L; }
    __device__ bool fetch_emit(int s, bool dn, uint32_t lp, uint32_t& i, uint32_t& bits) const {
        return fetch_phys(s, dn, lp, i, bits);
    }
    __device__ Digit digit(int s, bool, const SelState&) const {
        if (!in_min) return Digit{0u, (uint32_t)kCoarseShift};
        uint32_t ma = in_min[2 * s], mb = in_min[2 * s + 1];
        if (inverted) { ma = kAbs - ma; mb = kAbs - mb; }
        return Digit{ma > mb ? ma : mb, (uint32_t)kFineShift};
    }
    __device__ bool fetch_phys(int s, bool, uint32_t p, uint32_t& i, uint32_t& bits) const {
        i = idx[(size_t)s * stride + p];
        bits = __float_as_uint(val[(size_t)s * stride + p]);
        return i != kTomb;
    }
    __device__ bool fetch_key_phys(int s, bool, uint32_t p, uint32_t& key) const {
        key = __float_as_uint(val[(size_t)s * stride + p]) & kAbs;
        return idx[(size_t)s * stride + p] != kTomb;
    }
    __device__ uint32_t logical(int, bool, uint32_t p, uint32_t) const { return p; }
    __device__ void store_ordered(int, bool, uint32_t, uint32_t, uint32_t) const {}
    __device__ bool fetch_ord(int s, bool dn, uint32_t lp, uint32_t& i, uint32_t& bits) const {
        return fetch_phys(s, dn, lp, i, bits);
    }
    __device__ void scan_runs(int, uint32_t*) const {}
};

// Merge of LARGE sets through a speculative threshold: the union kernel has kept, of every
// tile of 8192 slots of the union, only the slots whose key reaches tspec[s] - a bucket
// edge taken from a sample of the union such that a little more than k slots are
// expected to reach it - packed at the start of the tile, in index order.  Group g of
// pair s is what is left of tile g: tile_cnt[s][g] slots from slot g * tile on.  A pair
// whose union kept fewer than k slots (set_cnt[s] < k: the sample misled) is skipped here
// and selected from its complete union instead (MergedSrc with the gate).
struct FiltSrc {
    static constexpr bool kRunGroups = true;
    static constexpr bool kWaveGroups = false;
    static constexpr bool kVectorWalk = true;
    static constexpr bool kSegList = true;          // no set of this source is ever read as a dense row
    __device__ const uint32_t* value_row(int s) const { return reinterpret_cast<const uint32_t*>(val) + (size_t)s * stride; }
    static constexpr bool kIdentity = false;
    static constexpr bool kRunScan = false;
    static constexpr bool kValueOnlyWalk = true;
    const uint32_t* idx;
    const float* val;
    uint32_t k, stride, tile_log2, ntiles;      // tiles of 2^tile_log2 slots
    const uint32_t* tile_cnt;     // [pairs][ntiles]
    const uint32_t* set_cnt;      // [pairs]
    const uint32_t* tspec;        // [pairs]
    __device__ bool skip(int s) const { return set_cnt[s] < k; }
    __device__ bool dense(int) const { return false; }
    __device__ void carry(int, uint32_t) const {}
    __device__ uint32_t floor_key(int, bool) const { return 0u; }
    __device__ bool wants_hist(int, bool) const { return true; }
    __device__ uint32_t* hist_of(int s, bool, const SelState& st) const { return st.hist + (size_t)s * kHistBins; }
    __device__ uint32_t nphys(int, bool) const { return ntiles << tile_log2; }      // <= 2^31 + 8192
    __device__ uint32_t group_slots(bool) const { return 1u << tile_log2; }
    __device__ uint32_t ngroups(int, bool) const { return ntiles; }
    __device__ Digit digit(int s, bool, const SelState&) const { return Digit{tspec[s], (uint32_t)kFineShift}; }
    __device__ uint32_t kept(int s, uint32_t g) const {
        const uint32_t c = tile_cnt[(size_t)s * ntiles + g];
        return c < (1u << tile_log2) ? c : (1u << tile_log2);
    }
    __device__ bool group_range(int s, uint32_t g, uint32_t& first, uint32_t& end) const {
        if (g >= ntiles) return false;
        const uint32_t c = kept(s, g);
        if (c == 0u) return false;
        first = g << tile_log2;
        end = first + c;
        return true;
    }
    __device__ uint32_t fetch_bits(int s, uint32_t p) const { return __float_as_uint(val[(size_t)s * stride + p]); }
    __device__ bool is_tomb(int, uint32_t) const { return false; }
    __device__ bool fetch_phys(int s, bool, uint32_t p, uint32_t& i, uint32_t& bits) const {
        const uint32_t g = p >> tile_log2;
        if (g >= ntiles || p - (g << tile_log2) >= kept(s, g)) return false;
        i = idx[(size_t)s * stride + p];
        bits = __float_as_uint(val[(size_t)s * stride + p]);
        return true;
    }
    __device__ bool fetch_key_phys(int s, bool dn, uint32_t p, uint32_t& key) const {
        uint32_t i, bits = 0;
        const bool ok = fetch_phys(s, dn, p, i, bits);
        key = bits & kAbs;
        return ok;
    }
    __device__ uint32_t logical(int, bool, uint32_t p, uint32_t) const { return p; }
    __device__ void store_ordered(int, bool, uint32_t, uint32_t, uint32_t) const {}
    __device__ bool fetch_ord(int s, bool dn, uint32_t lp, uint32_t& i, uint32_t& bits) const {
        return fetch_phys(s, dn, lp, i, bits);
    }
    // (inside a range from group_range() every slot is a kept one)
    __device__ bool fetch_emit(int s, bool, uint32_t p, uint32_t& i, uint32_t& bits) const {
        i = idx[(size_t)s * stride + p];
        bits = __float_as_uint(val[(size_t)s * stride + p]);
        return true;
    }
    __device__ uint32_t group_of(int, bool, uint32_t p, uint32_t) const { return p >> tile_log2; }
    __device__ uint32_t group_of_ord(int, bool, uint32_t lp, uint32_t) const { return lp >> tile_log2; }
    __device__ void scan_runs(int, uint32_t*) const {}
};

// ---------------------------------------------------------------------------------
// kernel 1: histogram of the first digit
// ---------------------------------------------------------------------------------

// Few, large blocks per set: a popular bin receives one global atomic per block.  The grid
// is sized for the sets' lists; a set that is read as a dense row (far longer) is walked
// by the same blocks with more loads in flight.
template <class Src, int BATCH>
__device__ __forceinline__ void hist_walk(const Src& src, int s, bool dn, const Digit& dg, uint32_t n,
                                          uint32_t fl, uint32_t hist_blocks, uint32_t* h) {
    const uint64_t step = (uint64_t)hist_blocks * kHistBlock;
    for (uint64_t p0 = (uint64_t)blockIdx.x * kHistBlock + threadIdx.x; p0 < n; p0 += step * BATCH) {
        uint32_t key[BATCH];
        bool ok[BATCH];
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            const uint64_t p = p0 + j * step;
            key[j] = 0;
            ok[j] = p < n && src.fetch_key_phys(s, dn, (uint32_t)p, key[j]) && key[j] >= fl;
        }
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            // a wave whose keys all fall into one bin (rows of zeros, equal values) adds once
            const uint32_t b = dg.bin(key[j]);
            const uint64_t act = __ballot(ok[j]);
            if (act == 0) continue;
            const uint32_t b0 = __shfl(b, __builtin_ctzll(act));
            if (__ballot(ok[j] && b == b0) == act) {
                if (lane_id() == (uint32_t)__builtin_ctzll(act)) atomicAdd(&h[b0], (uint32_t)__popcll(act));
            } else if (ok[j]) {
                atomicAdd(&h[b], 1u);
            }
        }
    }
}

// For a source whose runs need ordering, one extra block per set (the last one of the
// grid's x dimension) scans the run counts.
template <class Src>
__global__ __launch_bounds__(kHistBlock) void k_hist(Src src, SelState st, uint32_t hist_blocks) {
    __shared__ uint32_t h[kHistBins];
    __shared__ uint32_t s_wave[kHistBlock / kWave];
    const int s = blockIdx.y;
    if (Src::kRunScan && blockIdx.x == hist_blocks) {
        src.scan_runs(s, s_wave);
        return;
    }
    const bool dn = src.dense(s);
    if (!src.wants_hist(s, dn)) return;          // block-uniform: this set's histogram exists already
    for (int b = threadIdx.x; b < kHistBins; b += kHistBlock) h[b] = 0u;
    __syncthreads();
    const uint32_t n = src.nphys(s, dn);
    const Digit dg = src.digit(s, dn, st);
    const uint32_t fl = src.floor_key(s, dn);
    if (dn) hist_walk<Src, 8>(src, s, dn, dg, n, fl, hist_blocks, h);
    else hist_walk<Src, kHistBatch>(src, s, dn, dg, n, fl, hist_blocks, h);
    __syncthreads();
    uint32_t* out = src.hist_of(s, dn, st);
    for (int b = threadIdx.x; b < kHistBins; b += kHistBlock) {
        const uint32_t c = h[b];
        if (c) atomicAdd(&out[b], c);
    }
}

// ---------------------------------------------------------------------------------
// kernel 2: pick the bin; count keys above it per group, list keys inside it
// ---------------------------------------------------------------------------------

// Block b of set s walks the physical slots [b*L, (b+1)*L), L = group_slots(); a set with
// more such segments than the grid has blocks (a dense row) is walked in several turns.
// For a dense row, whose list can overflow, every group's count of in-bin keys and the
// row's smallest and largest in-bin key are recorded besides the list: if the list
// overflows although all in-bin keys are equal (rows of equal magnitudes), the finish needs
// nothing more than those.
// ---- the plain walk ----
// The walk of a set that is NOT read as a dense row: one segment per block, nothing that
// only a dense row needs.
template <class Src>
__device__ __forceinline__ void bucket_fast(const Src& src, const SelState& st, uint32_t k) {
    __shared__ uint32_t s_wave[kBlock / kWave];
    __shared__ uint32_t s_out[3];
    __shared__ uint32_t s_gt[kBlock / kWave];
    __shared__ uint32_t s_in[kBlock / kWave];
    __shared__ uint32_t s_base;
    constexpr int kStash = 1024;
    __shared__ uint2 s_stash[kStash];
    __shared__ uint32_t s_nstash;
    const int s = blockIdx.y;
    const uint32_t g = blockIdx.x;
    if (threadIdx.x == 0) s_nstash = 0u;       // visible after the barrier inside the pick
    constexpr bool dn = false;
    constexpr bool kOwnGroup = Src::kIdentity || Src::kRunGroups;     // every slot of the walk is of group g
    const uint32_t L = src.group_slots(dn);
    // (block 0 stays even when its group holds nothing: it records the bin)
    uint32_t first = 0, end = 0;
    if (!src.group_range(s, g, first, end)) {
        if (g != 0) return;
        first = end = 0;
    }
    const Digit dg = src.digit(s, dn, st);
    // one round of the walk: the block's next kBlock * kBatch slots, their items and logical positions
    uint32_t idx[kBatch], bits[kBatch], lp[kBatch];
    bool ok[kBatch];
    auto load_round = [&](uint32_t i0) {
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t p = i0 + j * kBlock + threadIdx.x;
            idx[j] = 0; bits[j] = 0;
            if (Src::kValueOnlyWalk) {
                ok[j] = p < end;
                if (ok[j]) bits[j] = src.fetch_bits(s, p);
            } else {
                ok[j] = p < end && src.fetch_phys(s, dn, p, idx[j], bits[j]);
            }
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t p = i0 + j * kBlock + threadIdx.x;
            lp[j] = (!kOwnGroup && p < end) ? src.logical(s, dn, p, idx[j]) : 0u;
        }
    };
    // the first round is fetched before the pick, so that its latency overlaps with it
    load_round((uint32_t)first);
    // every block picks the bin of the k-th key from the set's histogram
    {
        constexpr int kPer = kHistBins / kBlock;      // thread t owns 16 consecutive bins
        const uint32_t* hist = src.hist_of(s, dn, st);
        uint32_t loc[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) loc[j] = hist[threadIdx.x * kPer + j];
        suffix_pick<kPer>(loc, k, s_wave, s_out);
    }
    const uint32_t d1 = s_out[0];
    if (g == 0 && threadIdx.x == 0) {
        st.d1[s] = d1;
        st.krem[s] = k - s_out[1];
    }
    const uint32_t wave = threadIdx.x / kWave;
    uint32_t* ggt = st.grp_gt + (size_t)s * st.maxgroups;
    uint32_t gt = 0, in = 0;     // wave-uniform
    for (uint32_t i0 = (uint32_t)first; i0 < end; i0 += kBlock * kBatch) {
        if (i0 != (uint32_t)first) load_round(i0);
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t p = i0 + j * kBlock + threadIdx.x;
            if (!kOwnGroup && p < end) src.store_ordered(s, dn, lp[j], idx[j], bits[j]);
            const uint32_t key = bits[j] & kAbs;
            const uint32_t d = dg.bin(key);
            const bool above = ok[j] && d > d1;
            bool inside = ok[j] && d == d1;
            if (Src::kValueOnlyWalk && inside) inside = !src.is_tomb(s, p);
            const uint32_t lg = kOwnGroup ? g : lp[j] / L;
            if (kOwnGroup) gt += (uint32_t)__popcll(__ballot(above));
            else add_grouped(above, lg, ggt);
            // in-bin entries are parked in LDS (in any order) as long as they fit
            const uint64_t inm = __ballot(inside);
            if (inm) {
                const uint32_t cnt = (uint32_t)__popcll(inm);
                uint32_t base = 0;
                if (lane_id() == 0) base = atomicAdd(&s_nstash, cnt);
                base = __shfl(base, 0);
                const uint32_t pos = base + rank_in(inm);
                if (inside && pos < (uint32_t)kStash) s_stash[pos] = make_uint2(key, lg);
                in += cnt;
            }
        }
    }
    if (lane_id() == 0) { s_gt[wave] = gt; s_in[wave] = in; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t tg = 0, ti = 0;
        for (int v = 0; v < kBlock / kWave; ++v) { tg += s_gt[v]; ti += s_in[v]; }
        if (kOwnGroup) ggt[g] = tg;
        if (Src::kSegList && st.seg_list) {                    // the group's own range of the list
            st.grp_in[(size_t)s * st.maxgroups + g] = ti;
            s_base = (uint32_t)first;
        } else {
            s_base = ti ? atomicAdd(&st.list_cnt[s], ti) : 0u;     // one reservation per block
        }
    }
    __syncthreads();
    const uint32_t total = s_nstash;
    if (total == 0) return;
    uint2* list = st.list + (size_t)s * st.list_cap;
    if (total <= (uint32_t)kStash) {
        for (uint32_t i = threadIdx.x; i < total; i += kBlock)
            if (s_base + i < st.list_cap) list[s_base + i] = s_stash[i];
        return;
    }
    // more in-bin entries than the stash holds: walk the group again; this wave's entries
    // go to its slice of the block's reservation
    if (in == 0) return;
    uint32_t off = s_base;
    for (uint32_t v = 0; v < wave; ++v) off += s_in[v];
    for (uint32_t i0 = (uint32_t)first; i0 < end; i0 += kBlock * kBatch) {
        load_round(i0);
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t key = bits[j] & kAbs;
            bool inside = ok[j] && dg.bin(key) == d1;
            if (Src::kValueOnlyWalk && inside) inside = !src.is_tomb(s, i0 + j * kBlock + threadIdx.x);
            const uint64_t inm = __ballot(inside);
            if (inside) {
                const uint32_t pos = off + rank_in(inm);
                if (pos < st.list_cap) list[pos] = make_uint2(key, kOwnGroup ? g : lp[j] / L);
            }
            off += (uint32_t)__popcll(inm);
        }
    }
}

// ---- the plain walk, four slots per load ----
// For sources whose groups are ranges of slots of an aligned, padded row of values
// (kVectorWalk: the merged sets): the same walk as above with 16-byte loads, so that a
// thread has eight slots in flight instead of two.  (A group of thousands of slots is
// a chain of dependent rounds; what bounds the walk is how much each round carries.)
constexpr uint32_t kVectorWalkMinSlots = 4096;      // measured: 8192 -12 %, 4096 -6 %, 2048 even, 1024 +12 %
template <class Src>
__device__ __forceinline__ void bucket_vec(const Src& src, const SelState& st, uint32_t k) {
    static_assert(Src::kValueOnlyWalk && (Src::kIdentity || Src::kRunGroups), "every slot of the walk is of group g");
    constexpr int kWaves = kBlock / kWave;
    __shared__ uint32_t s_wave[kWaves];
    __shared__ uint32_t s_out[3];
    __shared__ uint32_t s_gt[kWaves];
    __shared__ uint32_t s_in[kWaves];
    __shared__ uint32_t s_base;
    constexpr int kStash = 1024;
    __shared__ uint2 s_stash[kStash];
    __shared__ uint32_t s_nstash;
    const int s = blockIdx.y;
    const uint32_t g = blockIdx.x;
    if (threadIdx.x == 0) s_nstash = 0u;       // visible after the barrier inside the pick
    constexpr bool dn = false;
    // (block 0 stays even when its group holds nothing: it records the bin)
    uint32_t first = 0, end = 0;               // first is a multiple of four
    if (!src.group_range(s, g, first, end)) {
        if (g != 0) return;
        first = end = 0;
    }
    const Digit dg = src.digit(s, dn, st);
    const uint32_t* vrow = src.value_row(s);
    constexpr uint32_t kRound = kBlock * kBatch * 4;          // slots per round of the block
    uint4 v[kBatch];
    auto load_round = [&](uint32_t i0) {
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t p = i0 + (j * kBlock + threadIdx.x) * 4;
            v[j] = p < end ? *reinterpret_cast<const uint4*>(vrow + p) : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    // the first round is fetched before the pick, so that its latency overlaps with it
    load_round(first);
    {
        constexpr int kPer = kHistBins / kBlock;      // thread t owns 16 consecutive bins
        const uint32_t* hist = src.hist_of(s, dn, st);
        uint32_t loc[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) loc[j] = hist[threadIdx.x * kPer + j];
        suffix_pick<kPer>(loc, k, s_wave, s_out);
    }
    const uint32_t d1 = s_out[0];
    if (g == 0 && threadIdx.x == 0) {
        st.d1[s] = d1;
        st.krem[s] = k - s_out[1];
    }
    const uint32_t wave = threadIdx.x / kWave;
    uint32_t gt = 0;             // this thread's count
    uint32_t in = 0;             // wave-uniform
    for (uint32_t i0 = first; i0 < end; i0 += kRound) {
        if (i0 != first) load_round(i0);
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t p = i0 + (j * kBlock + threadIdx.x) * 4;
            const uint32_t b4[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool ok = p + e < end;
                const uint32_t key = b4[e] & kAbs;
                const uint32_t d = dg.bin(key);
                gt += (ok && d > d1) ? 1u : 0u;
                bool inside = ok && d == d1;
                if (inside) inside = !src.is_tomb(s, p + e);
                // in-bin entries are parked in LDS (in any order) as long as they fit
                const uint64_t inm = __ballot(inside);
                if (inm) {
                    const uint32_t cnt = (uint32_t)__popcll(inm);
                    uint32_t base = 0;
                    if (lane_id() == 0) base = atomicAdd(&s_nstash, cnt);
                    base = __shfl(base, 0);
                    const uint32_t pos = base + rank_in(inm);
                    if (inside && pos < (uint32_t)kStash) s_stash[pos] = make_uint2(key, g);
                    in += cnt;
                }
            }
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) gt += __shfl_xor(gt, d);
    if (lane_id() == 0) { s_gt[wave] = gt; s_in[wave] = in; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t tg = 0, ti = 0;
        for (int w = 0; w < kWaves; ++w) { tg += s_gt[w]; ti += s_in[w]; }
        st.grp_gt[(size_t)s * st.maxgroups + g] = tg;
        if (Src::kSegList && st.seg_list) {                    // the group's own range of the list
            st.grp_in[(size_t)s * st.maxgroups + g] = ti;
            s_base = (uint32_t)first;
        } else {
            s_base = ti ? atomicAdd(&st.list_cnt[s], ti) : 0u;     // one reservation per block
        }
    }
    __syncthreads();
    const uint32_t total = s_nstash;
    if (total == 0) return;
    uint2* list = st.list + (size_t)s * st.list_cap;
    if (total <= (uint32_t)kStash) {
        for (uint32_t i = threadIdx.x; i < total; i += kBlock)
            if (s_base + i < st.list_cap) list[s_base + i] = s_stash[i];
        return;
    }
    // more in-bin entries than the stash holds: walk the group again; this wave's entries
    // go to its slice of the block's reservation
    if (in == 0) return;
    uint32_t off = s_base;
    for (uint32_t w = 0; w < wave; ++w) off += s_in[w];
    for (uint32_t i0 = first; i0 < end; i0 += kRound) {
        load_round(i0);
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t p = i0 + (j * kBlock + threadIdx.x) * 4;
            const uint32_t b4[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t key = b4[e] & kAbs;
                bool inside = p + e < end && dg.bin(key) == d1;
                if (inside) inside = !src.is_tomb(s, p + e);
                const uint64_t inm = __ballot(inside);
                if (inside) {
                    const uint32_t pos = off + rank_in(inm);
                    if (pos < st.list_cap) list[pos] = make_uint2(key, g);
                }
                off += (uint32_t)__popcll(inm);
            }
        }
    }
}

// ---- the walk of runs: one run per wave ----
// Wave v of block b walks group g = 4 b + v of a set that is not read as a dense row (the
// runs of the streaming pass: RunSrc).  The pick, the stash of in-bin keys and the one
// reservation per block are the plain walk's; the count of keys above the bin is the
// wave's own.
constexpr int kRunBatch = 8;                // loads a lane keeps in flight while it walks a run
template <class Src>
__device__ __forceinline__ void bucket_runs(const Src& src, const SelState& st, uint32_t k) {
    constexpr int kWaves = kBlock / kWave;
    __shared__ uint32_t s_wave[kWaves];
    __shared__ uint32_t s_out[3];
    __shared__ uint32_t s_in[kWaves];
    __shared__ uint32_t s_base;
    constexpr int kStash = 1024;
    __shared__ uint2 s_stash[kStash];
    __shared__ uint32_t s_nstash;
    const int s = blockIdx.y;
    const uint32_t wave = threadIdx.x / kWave, lane = lane_id();
    const uint32_t g = blockIdx.x * kWaves + wave;
    constexpr bool dn = false;
    // (block 0 stays even when its groups hold nothing: it records the bin)
    if (blockIdx.x != 0 && blockIdx.x * kWaves >= src.ngroups(s, dn)) return;
    if (threadIdx.x == 0) s_nstash = 0u;       // visible after the barrier inside the pick
    uint32_t first = 0, end = 0;               // wave-uniform
    if (!src.group_range(s, g, first, end)) first = end = 0;
    const Digit dg = src.digit(s, dn, st);
    uint32_t bits[kRunBatch];
    bool ok[kRunBatch];
    auto load_round = [&](uint32_t i0) {
#pragma unroll
        for (int j = 0; j < kRunBatch; ++j) {
            const uint32_t p = i0 + j * kWave + lane;
            ok[j] = p < end;
            bits[j] = ok[j] ? src.fetch_bits(s, p) : 0u;
        }
    };
    // the first round is fetched before the pick, so that its latency overlaps with it
    load_round(first);
    {
        constexpr int kPer = kHistBins / kBlock;      // thread t owns 16 consecutive bins
        const uint32_t* hist = src.hist_of(s, dn, st);
        uint32_t loc[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) loc[j] = hist[threadIdx.x * kPer + j];
        suffix_pick<kPer>(loc, k, s_wave, s_out);
    }
    const uint32_t d1 = s_out[0];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        st.d1[s] = d1;
        st.krem[s] = k - s_out[1];
    }
    uint32_t gt = 0, in = 0;     // wave-uniform
    for (uint32_t i0 = first; i0 < end; i0 += kWave * kRunBatch) {
        if (i0 != first) load_round(i0);
#pragma unroll
        for (int j = 0; j < kRunBatch; ++j) {
            const uint32_t key = bits[j] & kAbs;
            const uint32_t d = dg.bin(key);
            gt += (uint32_t)__popcll(__ballot(ok[j] && d > d1));
            const bool inside = ok[j] && d == d1;
            // in-bin entries are parked in LDS (in any order) as long as they fit
            const uint64_t inm = __ballot(inside);
            if (inm) {
                const uint32_t cnt = (uint32_t)__popcll(inm);
                uint32_t base = 0;
                if (lane == 0) base = atomicAdd(&s_nstash, cnt);
                base = __shfl(base, 0);
                const uint32_t pos = base + rank_in(inm);
                if (inside && pos < (uint32_t)kStash) s_stash[pos] = make_uint2(key, g);
                in += cnt;
            }
        }
    }
    if (lane == 0) {
        if (end != first) st.grp_gt[(size_t)s * st.maxgroups + g] = gt;
        s_in[wave] = in;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t ti = 0;
        for (int v = 0; v < kWaves; ++v) ti += s_in[v];
        s_base = ti ? atomicAdd(&st.list_cnt[s], ti) : 0u;     // one reservation per block
    }
    __syncthreads();
    const uint32_t total = s_nstash;
    if (total == 0) return;
    uint2* list = st.list + (size_t)s * st.list_cap;
    if (total <= (uint32_t)kStash) {
        for (uint32_t i = threadIdx.x; i < total; i += kBlock)
            if (s_base + i < st.list_cap) list[s_base + i] = s_stash[i];
        return;
    }
    // more in-bin entries than the stash holds: every wave walks its run again; its entries
    // go to its slice of the block's reservation
    if (in == 0) return;
    uint32_t off = s_base;
    for (uint32_t v = 0; v < wave; ++v) off += s_in[v];
    for (uint32_t i0 = first; i0 < end; i0 += kWave * kRunBatch) {
        load_round(i0);
#pragma unroll
        for (int j = 0; j < kRunBatch; ++j) {
            const uint32_t key = bits[j] & kAbs;
            const bool inside = ok[j] && dg.bin(key) == d1;
            const uint64_t inm = __ballot(inside);
            if (inside) {
                const uint32_t pos = off + rank_in(inm);
                if (pos < st.list_cap) list[pos] = make_uint2(key, g);
            }
            off += (uint32_t)__popcll(inm);
        }
    }
}

// ---- the general walk ----
template <class Src>
__device__ __forceinline__ void bucket_general(const Src& src, const SelState& st, uint32_t k) {
    __shared__ uint32_t s_wave[kBlock / kWave];
    __shared__ uint32_t s_out[3];
    __shared__ uint32_t s_gt[kBlock / kWave];
    __shared__ uint32_t s_in[kBlock / kWave];
    __shared__ uint32_t s_base;
    constexpr int kStash = 1024;
    __shared__ uint2 s_stash[kStash];
    __shared__ uint32_t s_nstash;
    __shared__ uint32_t s_hi, s_lo_inv;
    const int s = blockIdx.y;
    if (threadIdx.x == 0) { s_nstash = 0u; s_hi = 0u; s_lo_inv = 0u; }   // visible after the barrier inside the pick
    const bool dn = src.dense(s);
    const uint32_t n = src.nphys(s, dn);
    const uint32_t L = src.group_slots(dn);
    if ((uint64_t)blockIdx.x * L >= n) return;
    const Digit dg = src.digit(s, dn, st);
    const uint32_t fl = src.floor_key(s, dn);
    // one round of the walk: the block's next kBlock * kBatch slots, their items and groups
    uint32_t idx[kBatch], bits[kBatch], lp[kBatch], grp[kBatch];
    bool ok[kBatch];
    uint32_t g = blockIdx.x;                       // the segment being walked
    uint32_t end = 0;
    auto load_round = [&](uint32_t i0) {
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t p = i0 + j * kBlock + threadIdx.x;
            idx[j] = 0; bits[j] = 0;
            ok[j] = p < end && src.fetch_phys(s, dn, p, idx[j], bits[j]) && (bits[j] & kAbs) >= fl;
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t p = i0 + j * kBlock + threadIdx.x;
            lp[j] = p < end ? src.logical(s, dn, p, idx[j]) : 0u;
            grp[j] = Src::kIdentity ? g : lp[j] / L;
        }
    };
    // the first round is fetched before the pick, so that its latency overlaps with it
    {
        const uint64_t first = (uint64_t)g * L;
        end = (uint32_t)(first + L < n ? first + L : n);
        load_round((uint32_t)first);
    }
    // every block picks the bin of the k-th key from the set's histogram
    {
        constexpr int kPer = kHistBins / kBlock;      // thread t owns 16 consecutive bins
        const uint32_t* hist = src.hist_of(s, dn, st);
        uint32_t loc[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) loc[j] = hist[threadIdx.x * kPer + j];
        suffix_pick<kPer>(loc, k, s_wave, s_out);
    }
    const uint32_t d1 = s_out[0];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        st.d1[s] = d1;
        st.krem[s] = k - s_out[1];
    }
    const uint32_t wave = threadIdx.x / kWave;
    uint32_t* ggt = st.grp_gt + (size_t)s * st.maxgroups;
    uint32_t* gin = st.grp_in + (size_t)s * st.maxgroups;
    uint2* list = st.list + (size_t)s * st.list_cap;
    uint32_t hi = 0, lo_inv = 0;                   // this thread's in-bin extremes
    for (;;) {
        const uint32_t first = (uint32_t)((uint64_t)g * L);
        uint32_t gt = 0, in = 0;     // wave-uniform
        for (uint32_t i0 = first; i0 < end; i0 += kBlock * kBatch) {
            if (i0 != first || g != blockIdx.x) load_round(i0);
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                if (i0 + j * kBlock + threadIdx.x < end) src.store_ordered(s, dn, lp[j], idx[j], bits[j]);
                const uint32_t key = bits[j] & kAbs;
                const uint32_t d = dg.bin(key);
                const bool above = ok[j] && d > d1;
                const bool inside = ok[j] && d == d1;
                if (Src::kIdentity) {
                    gt += (uint32_t)__popcll(__ballot(above));
                } else {
                    add_grouped(above, grp[j], ggt);
                    if (dn) add_grouped(inside, grp[j], gin);
                }
                // in-bin entries are parked in LDS (in any order) as long as they fit
                const uint64_t inm = __ballot(inside);
                if (inm) {
                    const uint32_t cnt = (uint32_t)__popcll(inm);
                    uint32_t base = 0;
                    if (lane_id() == 0) base = atomicAdd(&s_nstash, cnt);
                    base = __shfl(base, 0);
                    const uint32_t pos = base + rank_in(inm);
                    if (inside) {
                        if (pos < (uint32_t)kStash) s_stash[pos] = make_uint2(key, grp[j]);
                        hi = key > hi ? key : hi;
                        lo_inv = kAbs - key > lo_inv ? kAbs - key : lo_inv;
                    }
                    in += cnt;
                }
            }
        }
        if (lane_id() == 0) { s_gt[wave] = gt; s_in[wave] = in; }
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t tg = 0, ti = 0;
            for (int v = 0; v < kBlock / kWave; ++v) { tg += s_gt[v]; ti += s_in[v]; }
            if (Src::kIdentity) ggt[g] = tg;
            s_base = ti ? atomicAdd(&st.list_cnt[s], ti) : 0u;     // one reservation per segment
        }
        __syncthreads();
        const uint32_t total = s_nstash;
        const uint32_t base = s_base;
        if (total != 0 && total <= (uint32_t)kStash) {
            for (uint32_t i = threadIdx.x; i < total; i += kBlock)
                if (base + i < st.list_cap) list[base + i] = s_stash[i];
        } else if (total != 0 && base < st.list_cap && in != 0) {
            // more in-bin entries than the stash holds: walk the segment again; this wave's
            // entries go to its slice of the reservation (nothing to do once the list is full)
            uint32_t off = base;
            for (uint32_t v = 0; v < wave; ++v) off += s_in[v];
            for (uint32_t i0 = first; i0 < end; i0 += kBlock * kBatch) {
                load_round(i0);
#pragma unroll
                for (int j = 0; j < kBatch; ++j) {
                    const uint32_t key = bits[j] & kAbs;
                    const bool inside = ok[j] && dg.bin(key) == d1;
                    const uint64_t inm = __ballot(inside);
                    if (inside) {
                        const uint32_t pos = off + rank_in(inm);
                        if (pos < st.list_cap) list[pos] = make_uint2(key, grp[j]);
                    }
                    off += (uint32_t)__popcll(inm);
                }
            }
        }
        // next segment of this block, if the set has more segments than the grid has blocks
        if ((uint64_t)(g + gridDim.x) * L >= n) break;
        g += gridDim.x;
        end = (uint32_t)((uint64_t)g * L + L < n ? (uint64_t)g * L + L : n);
        __syncthreads();                           // the stash and the counts have been read
        if (threadIdx.x == 0) s_nstash = 0u;
        __syncthreads();
    }
    // only a dense row's list can overflow (any other list holds the whole set)
    if (!dn) return;
    if (hi | lo_inv) {
        atomicMax(&s_hi, hi);
        atomicMax(&s_lo_inv, lo_inv);
    }
    __syncthreads();
    if (threadIdx.x == 0 && (s_hi | s_lo_inv)) {
        atomicMax(&st.bin_hi[s], s_hi);
        atomicMax(&st.bin_lo_inv[s], s_lo_inv);
    }
}

// Block b of set s walks the physical slots [b*L, (b+1)*L), L = group_slots().  A set
// that is read as a dense row takes the general walk (several segments per block, the
// bookkeeping for an overflowing list); every other set the plain one.
template <class Src>
__global__ __launch_bounds__(kBlock) void k_bucket(Src src, SelState st, uint32_t k) {
    if (src.skip(blockIdx.y)) return;
    if (src.dense(blockIdx.y)) bucket_general(src, st, k);
    else if constexpr (Src::kWaveGroups) bucket_runs(src, st, k);
    else if constexpr (Src::kVectorWalk) {
        // long groups four slots per load; short ones (a round or two) are faster the plain way
        if (src.group_slots(false) >= kVectorWalkMinSlots) bucket_vec(src, st, k);
        else bucket_fast(src, st, k);
    } else bucket_fast(src, st, k);
}

// ---------------------------------------------------------------------------------
// the finish: exact key, ties to take, per-group offsets
// ---------------------------------------------------------------------------------

// Calls f(key, group) for every entry of set s whose key lies in bin d1 - from the list
// that k_bucket wrote, or, if that list overflowed (more in-bin keys than it holds: rows
// of equal magnitudes), from the set's own slots.  Every thread of the block calls f the
// same number of times; key == kNoKey stands for "nothing".  T threads per block.
constexpr uint32_t kNoKey = 0xFFFFFFFFu;            // no key has bit 31 set

template <int T, class Src, class F>
__device__ __forceinline__ void for_each_in_bin(const Src& src, int s, bool dn, const Digit& dg,
                                                uint32_t d1, const uint2* list, uint32_t nlist,
                                                bool overflow, uint32_t nphys, uint32_t fl, F&& f) {
    const uint32_t t = threadIdx.x;
    if (!overflow) {
        for (uint32_t i0 = 0; i0 < nlist; i0 += T * kBatch) {
            uint2 e[kBatch];
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const uint32_t i = i0 + j * T + t;
                e[j] = i < nlist ? list[i] : make_uint2(kNoKey, 0u);
            }
#pragma unroll
            for (int j = 0; j < kBatch; ++j) f(e[j].x, e[j].y);
        }
    } else {
        constexpr int kWide = T >= 1024 ? 8 : kBatch;     // loads in flight per thread
        for (uint64_t p0 = 0; p0 < nphys; p0 += (uint64_t)T * kWide) {
            uint32_t key[kWide], grp[kWide];
#pragma unroll
            for (int j = 0; j < kWide; ++j) {
                const uint64_t p = p0 + (uint64_t)j * T + t;
                uint32_t idx = 0, bits = 0;
                const bool ok = p < nphys && src.fetch_phys(s, dn, (uint32_t)p, idx, bits) &&
                                (bits & kAbs) >= fl;
                key[j] = (ok && dg.bin(bits & kAbs) == d1) ? (bits & kAbs) : kNoKey;
                grp[j] = ok ? src.group_of(s, dn, (uint32_t)p, idx) : 0u;
            }
#pragma unroll
            for (int j = 0; j < kWide; ++j) f(key[j], grp[j]);
        }
    }
}

// ---------------------------------------------------------------------------------
// kernel 3 (large sets only): one block per set finishes the key and scans the groups
// ---------------------------------------------------------------------------------

// What every block of k_emit<.., INLINE = true> does for itself, done once per set: the
// exact key T, the number of ties to take, and for every group the counts of entries with
// key > T and with key == T in the groups before it.
template <class Src>
__global__ __launch_bounds__(1024) void k_finish(Src src, SelState st) {
    constexpr int kT = 1024;
    __shared__ uint32_t h[2048];
    __shared__ uint32_t g_gt[kMaxGroups];
    __shared__ uint32_t g_eq[kMaxGroups];
    __shared__ uint32_t s_wave[kT / kWave];
    __shared__ uint32_t s_out[3];
    // a segmented list (SelState::seg_list): where each group's entries start in the order of
    // the groups, and the entries themselves, gathered once, if they fit
    constexpr uint32_t kSegCache = 8192;
    __shared__ uint32_t g_off[Src::kSegList ? kMaxGroups : 1];
    __shared__ uint2 s_ent[Src::kSegList ? kSegCache : 1];
    const int s = blockIdx.x;
    const uint32_t t = threadIdx.x;
    if (src.skip(s)) return;
    const bool dn = src.dense(s);
    const uint32_t nphys = src.nphys(s, dn);
    const uint32_t ng = src.ngroups(s, dn);          // <= kMaxGroups
    const Digit dg = src.digit(s, dn, st);
    const uint32_t fl = src.floor_key(s, dn);
    const uint32_t d1 = st.d1[s];
    uint32_t krem = st.krem[s];
    const uint32_t nlist = st.list_cnt[s];
    const bool overflow = nlist > st.list_cap;       // the list is incomplete: read the set itself
    const uint2* list = st.list + (size_t)s * st.list_cap;
    const uint32_t lo = dg.lo(d1), width = dg.width(d1);    // bin d1 = [lo, lo + width)
    // per-group counts of keys above the bin (two groups per thread), loaded early
    const uint32_t ggt0 = 2 * t < ng ? st.grp_gt[(size_t)s * st.maxgroups + 2 * t] : 0u;
    const uint32_t ggt1 = 2 * t + 1 < ng ? st.grp_gt[(size_t)s * st.maxgroups + 2 * t + 1] : 0u;
    // an overflowed list whose in-bin keys are all one key (rows of equal magnitudes): that
    // key is T, and k_bucket's per-group in-bin counts are the tie counts
    const uint32_t bin_hi = st.bin_hi[s], bin_lo = kAbs - st.bin_lo_inv[s];
    const bool one_key = overflow && bin_hi == bin_lo;
    const uint32_t gin0 = (one_key && 2 * t < ng) ? st.grp_in[(size_t)s * st.maxgroups + 2 * t] : 0u;
    const uint32_t gin1 = (one_key && 2 * t + 1 < ng) ? st.grp_in[(size_t)s * st.maxgroups + 2 * t + 1] : 0u;
    const bool seg = Src::kSegList && st.seg_list != 0;      // uniform
    uint32_t nseg = 0;                                        // entries of a segmented list
    bool seg_cached = false;
    // entry i (< nseg) of a segmented list: it belongs to the last group whose entries start at or before i
    auto seg_fetch = [&](uint32_t i) -> uint2 {
        uint32_t glo = 0, ghi = ng;
        while (ghi - glo > 1) {
            const uint32_t mid = (glo + ghi) >> 1;
            if (g_off[mid] <= i) glo = mid; else ghi = mid;
        }
        uint32_t first = 0, end = 0;
        src.group_range(s, glo, first, end);
        const uint32_t p = first + (i - g_off[glo]);
        return p < st.list_cap ? list[p] : make_uint2(kNoKey, 0u);      // (always inside for a list k_bucket wrote)
    };
    if (seg) {
        const uint32_t c0 = 2 * t < ng ? st.grp_in[(size_t)s * st.maxgroups + 2 * t] : 0u;
        const uint32_t c1 = 2 * t + 1 < ng ? st.grp_in[(size_t)s * st.maxgroups + 2 * t + 1] : 0u;
        uint32_t tot;
        const uint32_t incl = block_incl_scan(c0 + c1, s_wave, tot);
        g_off[2 * t] = incl - c0 - c1;
        g_off[2 * t + 1] = incl - c1;
        __syncthreads();
        nseg = tot;
        seg_cached = nseg <= kSegCache;
        if (seg_cached) {
            // (all loads of a thread in flight together: each waits for a search in LDS and a load)
            uint2 e[kSegCache / kT];
#pragma unroll
            for (uint32_t j = 0; j < kSegCache / kT; ++j)
                if (j * kT + t < nseg) e[j] = seg_fetch(j * kT + t);
#pragma unroll
            for (uint32_t j = 0; j < kSegCache / kT; ++j)
                if (j * kT + t < nseg) s_ent[j * kT + t] = e[j];
            __syncthreads();
        }
    }
    // f(key, group) for every in-bin entry of the set; every thread calls f the same number of times
    auto each_entry = [&](auto&& f) {
        if (!seg) {
            for_each_in_bin<kT>(src, s, dn, dg, d1, list, nlist, overflow, nphys, fl, f);
        } else {
            for (uint32_t i0 = 0; i0 < nseg; i0 += kT * kBatch) {
                uint2 e[kBatch];
#pragma unroll
                for (int j = 0; j < kBatch; ++j) {
                    const uint32_t i = i0 + j * kT + t;
                    e[j] = i < nseg ? (seg_cached ? s_ent[i] : seg_fetch(i)) : make_uint2(kNoKey, 0u);
                }
#pragma unroll
                for (int j = 0; j < kBatch; ++j) f(e[j].x, e[j].y);
            }
        }
    };
    uint32_t T, need;
    if (one_key) {
        T = bin_hi;
        need = krem;
        g_gt[2 * t] = ggt0;
        g_gt[2 * t + 1] = ggt1;
        g_eq[2 * t] = gin0;
        g_eq[2 * t + 1] = gin1;
        __syncthreads();
    } else {
        // radix passes over rel = key - lo: bits 30..20, 19..10, 9..0; a pass whose bits are
        // zero for the whole bin is skipped
        uint32_t prefix = 0;          // value of the rel bits above the current pass
        for (int pass = 0; pass < 3; ++pass) {
            const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
            const int bits = pass == 0 ? 11 : 10;
            if (shift > 0 && width <= (1u << shift)) continue;       // uniform
            h[t] = 0u;
            h[t + kT] = 0u;
            __syncthreads();
            each_entry([&](uint32_t key, uint32_t) {
                const uint32_t rel = key - lo;
                const bool mine = key != kNoKey && (rel >> (shift + bits)) == prefix;
                const uint32_t b = (rel >> shift) & ((1u << bits) - 1u);
                // a wave whose keys all fall into one bin (masses of equal keys) adds once
                const uint64_t act = __ballot(mine);
                if (act) {
                    const uint32_t b0 = __shfl(b, __builtin_ctzll(act));
                    if (__ballot(mine && b == b0) == act) {
                        if (lane_id() == (uint32_t)__builtin_ctzll(act)) atomicAdd(&h[b0], (uint32_t)__popcll(act));
                    } else if (mine) {
                        atomicAdd(&h[b], 1u);
                    }
                }
            });
            __syncthreads();
            const uint32_t loc[2] = {h[2 * t], h[2 * t + 1]};
            suffix_pick<2>(loc, krem, s_wave, s_out);
            prefix = (prefix << bits) | s_out[0];
            krem -= s_out[1];
        }
        T = lo + prefix;
        need = krem;

        // per-group counts of selected-for-sure (key > T) and tied (key == T) entries
        g_gt[2 * t] = ggt0;
        g_gt[2 * t + 1] = ggt1;
        g_eq[2 * t] = 0u;
        g_eq[2 * t + 1] = 0u;
        __syncthreads();
        each_entry([&](uint32_t key, uint32_t g) {
            g &= (uint32_t)kMaxGroups - 1;
            add_grouped_lds(key != kNoKey && key > T, g, g_gt);
            add_grouped_lds(key != kNoKey && key == T, g, g_eq);
        });
        __syncthreads();
    }
    // exclusive scans over the groups (ng <= 2048: two per thread)
    {
        const uint32_t g0 = 2 * t, g1 = 2 * t + 1;
        const uint32_t a0 = g0 < ng ? g_gt[g0] : 0u, a1 = g1 < ng ? g_gt[g1] : 0u;
        const uint32_t e0 = g0 < ng ? g_eq[g0] : 0u, e1 = g1 < ng ? g_eq[g1] : 0u;
        uint32_t tot;
        const uint32_t ia = block_incl_scan(a0 + a1, s_wave, tot);
        const uint32_t ie = block_incl_scan(e0 + e1, s_wave, tot);
        uint32_t* og = st.off_gt + (size_t)s * st.maxgroups;
        uint32_t* oe = st.off_eq + (size_t)s * st.maxgroups;
        if (g0 < ng) { og[g0] = ia - a0 - a1; oe[g0] = ie - e0 - e1; }
        if (g1 < ng) { og[g1] = ia - a1; oe[g1] = ie - e1; }
    }
    if (t == 0) {
        st.T[s] = T;
        st.need[s] = need;
        if (st.T_out) st.T_out[s] = T;
        src.carry(s, T);
    }
}

// ---------------------------------------------------------------------------------
// kernel 4: finish the key (unless k_finish has), then ordered emit
// ---------------------------------------------------------------------------------

// One block per group.
//
// INLINE: every block first finishes the select of its set on its own - the list of keys
// inside bin d1 is short, so doing it per block is cheaper than a kernel in between: LDS
// radix passes over the list give the exact k-th key T and the number `need` of entries
// with key == T to take; the block's output offsets are the counts, over the groups before
// its own, of keys above the bin (grp_gt) plus list keys above T, and of list keys equal to
// T.  (If the list overflowed every block reads the whole set instead: correct, slow; the
// host side uses k_finish wherever such a set can be large.)
//
// Then the emit: an entry is selected if key > T, or key == T and fewer than `need`
// equal-key entries precede it in index order; its output slot is the number of selected
// entries before it.  DIVIDE: value / divisor (Eq. 3).  gbits != NULL: also set bit
// `index` of that bitmap (the dense gMask of Algorithm 3 lines 21-22, one bit per gradient
// element).  A block takes kBlock * kBatch items per round: their order inside a round is
// (sub-step j, wave, lane).
// The kernel writes nothing that a source reads.
// ---- the plain emit: one group per block ----
template <class Src, bool DIVIDE, bool INLINE>
__device__ __forceinline__ void emit_fast(
        const Src& src, const SelState& st, uint32_t k, uint32_t* __restrict__ out_idx,
        float* __restrict__ out_val, int64_t out_stride, float divisor,
        uint32_t* __restrict__ gbits) {
    constexpr int kWaves = kBlock / kWave;
    constexpr int kT = kBlock;
    __shared__ uint32_t h[2048];
    __shared__ uint32_t s_wave[kWaves];
    __shared__ uint32_t s_out[3];
    __shared__ uint32_t s_red[2][kWaves];
    __shared__ uint32_t s_eq[kBatch * kWaves];
    __shared__ uint32_t s_sel[kBatch * kWaves];
    __shared__ uint32_t s_cmp[kBlock];
    const int s = blockIdx.y;
    const uint32_t g = blockIdx.x;
    const uint32_t t = threadIdx.x;
    constexpr bool dn = false;
    const uint32_t n = src.nphys(s, dn);
    // (block 0 stays even when its group holds nothing: it records T)
    uint32_t first = 0, end = 0;
    if (!src.group_range(s, g, first, end)) {
        if (g != 0) return;
        first = end = 0;
    }
    const uint32_t wave = t / kWave;

    // the block's first round of items is fetched up front: its latency overlaps the finish
    uint32_t idx[kBatch], vb[kBatch];
    bool ok[kBatch];
    auto load_round = [&](uint32_t i0) {
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t p = i0 + j * kBlock + t;
            idx[j] = 0; vb[j] = 0;
            ok[j] = p < end && src.fetch_emit(s, dn, p, idx[j], vb[j]);
        }
    };
    load_round((uint32_t)first);

    // ---- finish -------------------------------------------------------------------------
    uint32_t T, need, off_gt, eq_before;
    if (!INLINE) {
        T = st.T[s];
        need = st.need[s];
        off_gt = st.off_gt[(size_t)s * st.maxgroups + g];
        eq_before = st.off_eq[(size_t)s * st.maxgroups + g];
    } else {
        const Digit dg = src.digit(s, dn, st);
        const uint32_t d1 = st.d1[s];
        uint32_t krem = st.krem[s];
        const uint32_t nlist = st.list_cnt[s];
        const bool overflow = nlist > st.list_cap;       // the list is incomplete: read the set itself
        const uint2* list = st.list + (size_t)s * st.list_cap;
        const uint32_t lo = dg.lo(d1), width = dg.width(d1);    // bin d1 = [lo, lo + width)
        // keys above the bin in the groups before this one
        uint32_t before_gt = 0;
        for (uint32_t gp = t; gp < g; gp += kT) before_gt += st.grp_gt[(size_t)s * st.maxgroups + gp];

        // a short list is read once and kept in registers
        constexpr int kCache = 4;
        constexpr uint32_t kNone = 0xFFFFFFFFu;            // no key has bit 31 set
        const bool cached = !overflow && nlist <= (uint32_t)(kCache * kT);
        uint2 ent[kCache];
#pragma unroll
        for (int j = 0; j < kCache; ++j) {
            const uint32_t i = t + (uint32_t)j * kT;
            ent[j] = (cached && i < nlist) ? list[i] : make_uint2(kNone, 0u);
        }
        // f(key, group): key == kNone = nothing
        auto for_each_entry = [&](auto&& f) {
            if (cached) {
#pragma unroll
                for (int j = 0; j < kCache; ++j) f(ent[j].x, ent[j].y);
            } else if (!overflow) {
                for (uint32_t i0 = 0; i0 < nlist; i0 += kT * kBatch) {
                    uint2 e[kBatch];
#pragma unroll
                    for (int j = 0; j < kBatch; ++j) {
                        const uint32_t i = i0 + j * kT + t;
                        e[j] = i < nlist ? list[i] : make_uint2(kNone, 0u);
                    }
#pragma unroll
                    for (int j = 0; j < kBatch; ++j) f(e[j].x, e[j].y);
                }
            } else {
                // every item of the set in logical order; items outside bin d1 are skipped
                for (uint64_t p0 = 0; p0 < n; p0 += (uint64_t)kT * kBatch) {
                    uint32_t key[kBatch], grp[kBatch];
#pragma unroll
                    for (int j = 0; j < kBatch; ++j) {
                        const uint64_t p = p0 + (uint64_t)j * kT + t;
                        uint32_t i2 = 0, b2 = 0;
                        const bool live = p < n && src.fetch_ord(s, dn, (uint32_t)p, i2, b2);
                        key[j] = (live && dg.bin(b2 & kAbs) == d1) ? (b2 & kAbs) : kNone;
                        grp[j] = live ? src.group_of_ord(s, dn, (uint32_t)p, i2) : 0u;
                    }
#pragma unroll
                    for (int j = 0; j < kBatch; ++j) f(key[j], grp[j]);
                }
            }
        };

        // radix passes over rel = key - lo: bits 30..20, 19..10, 9..0; a pass whose bits are
        // zero for the whole bin is skipped
        uint32_t prefix = 0;          // value of the rel bits above the current pass
        for (int pass = 0; pass < 3; ++pass) {
            const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
            const int bits = pass == 0 ? 11 : 10;
            if (shift > 0 && width <= (1u << shift)) continue;       // uniform
#pragma unroll
            for (int j = 0; j < 2048 / kT; ++j) h[t + j * kT] = 0u;
            __syncthreads();
            for_each_entry([&](uint32_t key, uint32_t) {
                if (key != kNone) {
                    const uint32_t rel = key - lo;
                    if ((rel >> (shift + bits)) == prefix)
                        atomicAdd(&h[(rel >> shift) & ((1u << bits) - 1u)], 1u);
                }
            });
            __syncthreads();
            constexpr int kPer = 2048 / kT;
            uint32_t loc[kPer];
#pragma unroll
            for (int j = 0; j < kPer; ++j) loc[j] = h[t * kPer + j];
            suffix_pick<kPer>(loc, krem, s_wave, s_out);
            prefix = (prefix << bits) | s_out[0];
            krem -= s_out[1];
        }
        T = lo + prefix;
        need = krem;

        // list keys of the groups before this one: above T, equal to T
        uint32_t c_gt = before_gt, c_eq = 0;
        for_each_entry([&](uint32_t key, uint32_t grp) {
            if (key != kNone && grp < g) {
                c_gt += key > T ? 1u : 0u;
                c_eq += key == T ? 1u : 0u;
            }
        });
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            c_gt += __shfl_xor(c_gt, d);
            c_eq += __shfl_xor(c_eq, d);
        }
        if (lane_id() == 0) { s_red[0][wave] = c_gt; s_red[1][wave] = c_eq; }
        __syncthreads();
        off_gt = 0;
        eq_before = 0;
#pragma unroll
        for (int v = 0; v < kWaves; ++v) { off_gt += s_red[0][v]; eq_before += s_red[1][v]; }
        if (g == 0 && t == 0) {
            st.T[s] = T;
            st.need[s] = need;
            if (st.T_out) st.T_out[s] = T;
            src.carry(s, T);
        }
    }

    // ---- emit ---------------------------------------------------------------------------
    uint32_t outp = off_gt + (eq_before < need ? eq_before : need);
    for (uint32_t i0 = (uint32_t)first; i0 < end; i0 += kBlock * kBatch) {
        if (i0 != (uint32_t)first) load_round(i0);
        bool is_gt[kBatch], is_eq[kBatch];
        uint64_t eqm[kBatch];
        __syncthreads();                  // the previous round's s_eq / s_sel are no longer read
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const uint32_t key = vb[j] & kAbs;
            is_gt[j] = ok[j] && key > T;
            is_eq[j] = ok[j] && key == T;
            eqm[j] = __ballot(is_eq[j]);
            if (lane_id() == 0) s_eq[j * kWaves + wave] = (uint32_t)__popcll(eqm[j]);
        }
        __syncthreads();
        bool sel[kBatch];
        uint64_t selm[kBatch];
        uint32_t eq_all = 0;
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            uint32_t eq_base = eq_before + eq_all;
            for (uint32_t v = 0; v < (uint32_t)kWaves; ++v) {
                const uint32_t c = s_eq[j * kWaves + v];
                if (v < wave) eq_base += c;
                eq_all += c;
            }
            sel[j] = is_gt[j] || (is_eq[j] && (eq_base + rank_in(eqm[j]) < need));
            selm[j] = __ballot(sel[j]);
            if (lane_id() == 0) s_sel[j * kWaves + wave] = (uint32_t)__popcll(selm[j]);
        }
        __syncthreads();
        uint32_t sel_all = 0;
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            uint32_t sel_base = outp + sel_all;
            for (uint32_t v = 0; v < (uint32_t)kWaves; ++v) {
                const uint32_t c = s_sel[j * kWaves + v];
                if (v < wave) sel_base += c;
                sel_all += c;
            }
            if (sel[j]) {
                const uint32_t pos = sel_base + rank_in(selm[j]);
                if (pos < k) {      // always true when the select state is consistent
                    out_idx[(int64_t)s * out_stride + pos] = idx[j];
                    float v = __uint_as_float(vb[j]);
                    if (DIVIDE) v = v / divisor;
                    out_val[(int64_t)s * out_stride + pos] = v;
                }
            }
        }
        outp += sel_all;
        eq_before += eq_all;
        if (gbits) {                      // block-uniform
            // a wave's selected indices, compacted, are ascending: the first of each run that
            // shares a bitmap word sets the bits of the whole run with one atomic
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const uint32_t nsel = (uint32_t)__popcll(selm[j]);
                if (sel[j]) s_cmp[wave * kWave + rank_in(selm[j])] = idx[j];
                __syncthreads();
                const uint32_t lane = lane_id();
                if (lane < nsel) {
                    const uint32_t* c = s_cmp + wave * kWave;
                    const uint32_t word = c[lane] >> 5;
                    if (lane == 0 || (c[lane - 1] >> 5) != word) {
                        uint32_t bits = 1u << (c[lane] & 31);
                        for (uint32_t q = lane + 1; q < nsel && (c[q] >> 5) == word; ++q)
                            bits |= 1u << (c[q] & 31);
                        atomicOr(&gbits[word], bits);
                    }
                }
                __syncthreads();
            }
        }
    }
}

// ---- the general emit: several groups per block, dense-row bookkeeping ----
template <class Src, bool DIVIDE, bool INLINE, int BLOCK>
__device__ __forceinline__ void emit_general(
        const Src& src, const SelState& st, uint32_t k, uint32_t* __restrict__ out_idx,
        float* __restrict__ out_val, int64_t out_stride, float divisor,
        uint32_t* __restrict__ gbits) {
    constexpr int kWaves = BLOCK / kWave;
    constexpr int kT = BLOCK;
    __shared__ uint32_t h[2048];
    __shared__ uint32_t s_wave[kWaves];
    __shared__ uint32_t s_out[3];
    __shared__ uint32_t s_red[2][kWaves];
    __shared__ uint32_t s_eq[kBatch * kWaves];
    __shared__ uint32_t s_sel[kBatch * kWaves];
    __shared__ uint32_t s_cmp[BLOCK];
    const int s = blockIdx.y;
    const uint32_t t = threadIdx.x;
    const bool dn = src.dense(s);
    const uint32_t nitems = src.nphys(s, dn);
    const uint32_t L = src.group_slots(dn);
    const uint32_t ngroups = (uint32_t)(((uint64_t)nitems + L - 1) / L);
    if (blockIdx.x >= ngroups) return;
    const uint32_t fl = src.floor_key(s, dn);
    const uint32_t wave = t / kWave;

    // what the INLINE finish keeps between the groups of this block
    constexpr int kCache = 4;
    uint2 ent[kCache];                   // a short list is read once and kept in registers
    bool cached = false, overflow = false, one_key = false, finished = false;
    uint32_t nlist = 0, d1 = 0, n = 0;
    Digit dg{0u, (uint32_t)kCoarseShift};
    const uint2* list = st.list + (size_t)s * st.list_cap;
    uint32_t T = 0, need = 0;
    if (!INLINE) {
        T = st.T[s];
        need = st.need[s];
    }

    // a set with more groups than the grid has blocks (a dense row) takes several turns
    for (uint32_t g = blockIdx.x; g < ngroups; g += gridDim.x) {
        if (g != blockIdx.x) __syncthreads();           // the previous group's LDS use is over
        const uint32_t first = g * L;                   // < nitems
        const uint32_t ng_items = nitems - first < L ? nitems - first : L;
        // the group's first round of items is fetched up front: its latency overlaps the finish
        uint32_t idx[kBatch], vb[kBatch];
        bool ok[kBatch];
        auto load_round = [&](uint32_t i0) {
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const uint32_t q = i0 + j * BLOCK + t;
                idx[j] = 0; vb[j] = 0;
                ok[j] = q < ng_items && src.fetch_ord(s, dn, first + q, idx[j], vb[j]) &&
                        (vb[j] & kAbs) >= fl;
            }
        };
        load_round(0u);

        // ---- finish ---------------------------------------------------------------------
        uint32_t off_gt, eq_before;
        if (!INLINE) {
            off_gt = st.off_gt[(size_t)s * st.maxgroups + g];
            eq_before = st.off_eq[(size_t)s * st.maxgroups + g];
        } else {
            // keys above the bin (and, for a one-key bin, keys inside it) in the groups before
            uint32_t before_gt = 0, before_in = 0;
            for (uint32_t gp = t; gp < g; gp += kT) before_gt += st.grp_gt[(size_t)s * st.maxgroups + gp];
            // f(key, group): key == kNoKey = nothing
            auto for_each_entry = [&](auto&& f) {
                if (cached) {
#pragma unroll
                    for (int j = 0; j < kCache; ++j) f(ent[j].x, ent[j].y);
                } else {
                    for_each_in_bin<kT>(src, s, dn, dg, d1, list, nlist, overflow, n, fl, f);
                }
            };
            if (!finished) {
                finished = true;
                dg = src.digit(s, dn, st);
                d1 = st.d1[s];
                uint32_t krem = st.krem[s];
                nlist = st.list_cnt[s];
                n = src.nphys(s, dn);
                overflow = nlist > st.list_cap;       // the list is incomplete
                // all in-bin keys are one key (rows of equal magnitudes): no pass over the set
                const uint32_t bin_hi = st.bin_hi[s], bin_lo = kAbs - st.bin_lo_inv[s];
                one_key = overflow && bin_hi == bin_lo;
                const uint32_t lo = dg.lo(d1), width = dg.width(d1);    // bin d1 = [lo, lo + width)
                cached = !overflow && nlist <= (uint32_t)(kCache * kT);
#pragma unroll
                for (int j = 0; j < kCache; ++j) {
                    const uint32_t i = t + (uint32_t)j * kT;
                    ent[j] = (cached && i < nlist) ? list[i] : make_uint2(kNoKey, 0u);
                }
                if (one_key) {
                    T = bin_hi;
                    need = krem;
                } else {
                    // radix passes over rel = key - lo: bits 30..20, 19..10, 9..0; a pass whose
                    // bits are zero for the whole bin is skipped
                    uint32_t prefix = 0;          // value of the rel bits above the current pass
                    for (int pass = 0; pass < 3; ++pass) {
                        const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
                        const int bits = pass == 0 ? 11 : 10;
                        if (shift > 0 && width <= (1u << shift)) continue;       // uniform
#pragma unroll
                        for (int j = 0; j < 2048 / kT; ++j) h[t + j * kT] = 0u;
                        __syncthreads();
                        for_each_entry([&](uint32_t key, uint32_t) {
                            if (key != kNoKey) {
                                const uint32_t rel = key - lo;
                                if ((rel >> (shift + bits)) == prefix)
                                    atomicAdd(&h[(rel >> shift) & ((1u << bits) - 1u)], 1u);
                            }
                        });
                        __syncthreads();
                        constexpr int kPer = 2048 / kT;
                        uint32_t loc[kPer];
#pragma unroll
                        for (int j = 0; j < kPer; ++j) loc[j] = h[t * kPer + j];
                        suffix_pick<kPer>(loc, krem, s_wave, s_out);
                        prefix = (prefix << bits) | s_out[0];
                        krem -= s_out[1];
                    }
                    T = lo + prefix;
                    need = krem;
                }
                if (g == 0 && t == 0) {
                    st.T[s] = T;
                    st.need[s] = need;
                    if (st.T_out) st.T_out[s] = T;
                    src.carry(s, T);
                }
            }
            // entries of the groups before this one: above T, equal to T
            uint32_t c_gt = before_gt, c_eq = 0;
            if (one_key) {
                for (uint32_t gp = t; gp < g; gp += kT) before_in += st.grp_in[(size_t)s * st.maxgroups + gp];
                c_eq = before_in;
            } else {
                for_each_entry([&](uint32_t key, uint32_t grp) {
                    if (key != kNoKey && grp < g) {
                        c_gt += key > T ? 1u : 0u;
                        c_eq += key == T ? 1u : 0u;
                    }
                });
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                c_gt += __shfl_xor(c_gt, d);
                c_eq += __shfl_xor(c_eq, d);
            }
            if (lane_id() == 0) { s_red[0][wave] = c_gt; s_red[1][wave] = c_eq; }
            __syncthreads();
            off_gt = 0;
            eq_before = 0;
#pragma unroll
            for (int v = 0; v < kWaves; ++v) { off_gt += s_red[0][v]; eq_before += s_red[1][v]; }
        }

        // ---- emit -----------------------------------------------------------------------
        uint32_t outp = off_gt + (eq_before < need ? eq_before : need);
        for (uint32_t i0 = 0; i0 < ng_items; i0 += BLOCK * kBatch) {
            if (i0 != 0) load_round(i0);
            bool is_gt[kBatch], is_eq[kBatch];
            uint64_t eqm[kBatch];
            __syncthreads();                  // the previous round's s_eq / s_sel are no longer read
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                const uint32_t key = vb[j] & kAbs;
                is_gt[j] = ok[j] && key > T;
                is_eq[j] = ok[j] && key == T;
                eqm[j] = __ballot(is_eq[j]);
                if (lane_id() == 0) s_eq[j * kWaves + wave] = (uint32_t)__popcll(eqm[j]);
            }
            __syncthreads();
            bool sel[kBatch];
            uint64_t selm[kBatch];
            uint32_t eq_all = 0;
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                uint32_t eq_base = eq_before + eq_all;
                for (uint32_t v = 0; v < (uint32_t)kWaves; ++v) {
                    const uint32_t c = s_eq[j * kWaves + v];
                    if (v < wave) eq_base += c;
                    eq_all += c;
                }
                sel[j] = is_gt[j] || (is_eq[j] && (eq_base + rank_in(eqm[j]) < need));
                selm[j] = __ballot(sel[j]);
                if (lane_id() == 0) s_sel[j * kWaves + wave] = (uint32_t)__popcll(selm[j]);
            }
            __syncthreads();
            uint32_t sel_all = 0;
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
                uint32_t sel_base = outp + sel_all;
                for (uint32_t v = 0; v < (uint32_t)kWaves; ++v) {
                    const uint32_t c = s_sel[j * kWaves + v];
                    if (v < wave) sel_base += c;
                    sel_all += c;
                }
                if (sel[j]) {
                    const uint32_t pos = sel_base + rank_in(selm[j]);
                    if (pos < k) {      // always true when the select state is consistent
                        out_idx[(int64_t)s * out_stride + pos] = idx[j];
                        float v = __uint_as_float(vb[j]);
                        if (DIVIDE) v = v / divisor;
                        out_val[(int64_t)s * out_stride + pos] = v;
                    }
                }
            }
            outp += sel_all;
            eq_before += eq_all;
            if (gbits) {                      // block-uniform
                // a wave's selected indices, compacted, are ascending: the first of each run that
                // shares a bitmap word sets the bits of the whole run with one atomic
#pragma unroll
                for (int j = 0; j < kBatch; ++j) {
                    const uint32_t nsel = (uint32_t)__popcll(selm[j]);
                    if (sel[j]) s_cmp[wave * kWave + rank_in(selm[j])] = idx[j];
                    __syncthreads();
                    const uint32_t lane = lane_id();
                    if (lane < nsel) {
                        const uint32_t* c = s_cmp + wave * kWave;
                        const uint32_t word = c[lane] >> 5;
                        if (lane == 0 || (c[lane - 1] >> 5) != word) {
                            uint32_t bits = 1u << (c[lane] & 31);
                            for (uint32_t q = lane + 1; q < nsel && (c[q] >> 5) == word; ++q)
                                bits |= 1u << (c[q] & 31);
                            atomicOr(&gbits[word], bits);
                        }
                    }
                    __syncthreads();
                }
            }
        }
    }
}

// (The register budget is the plain emit's: the general one, which runs for the rare dense
// row only, may spill.)
template <class Src, bool DIVIDE, bool INLINE>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(7, 8))) void k_emit(
        Src src, SelState st, uint32_t k, uint32_t* __restrict__ out_idx,
        float* __restrict__ out_val, int64_t out_stride, float divisor,
        uint32_t* __restrict__ gbits) {
    if (src.skip(blockIdx.y)) return;
    if (src.dense(blockIdx.y))
        emit_general<Src, DIVIDE, INLINE, kBlock>(src, st, k, out_idx, out_val, out_stride, divisor, gbits);
    else
        emit_fast<Src, DIVIDE, INLINE>(src, st, k, out_idx, out_val, out_stride, divisor, gbits);
}

// Algorithm 4 line 8 for the stand-alone local selection: +0.0 at the k selected entries of
// every worker's row.
__global__ __launch_bounds__(kBlock) void k_zero_selected(
        const uint32_t* __restrict__ sel_idx, uint32_t k, float* __restrict__ row,
        int64_t row_stride) {
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    const int s = blockIdx.y;
    if (t < k) row[(int64_t)s * row_stride + sel_idx[(size_t)s * k + t]] = 0.0f;
}

}  // namespace gtopk
