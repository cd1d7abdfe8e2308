// The Top-k operation between two sparse vectors (Definition 1): index-ordered union of
// two k-sets with the values at shared indices added.  Also the residual restore of
// Algorithm 4 line 10.
#pragma once
#include "common.hip.h"

namespace gtopk {

// Number of elements of the ascending array a[0..n) that are below x (UPPER: below or
// equal).  The whole wave calls it with the same arguments and gets the same result:
// each round the 64 lanes probe the last elements of 64 consecutive sub-ranges, so the
// dependent chain is log64(n) loads long.
template <bool UPPER>
__device__ inline uint32_t wave_count_below(const uint32_t* __restrict__ a, uint32_t n, uint32_t x) {
    uint32_t lo = 0, hi = n;              // the answer lies in [lo, hi]
    const uint32_t lane = lane_id();
    while (lo < hi) {
        const uint32_t len = hi - lo;
        const uint32_t step = (len + kWave - 1) / kWave;
        const uint32_t start = lo + lane * step;                     // this lane's sub-range
        const bool active = start < hi;
        const uint32_t last = (start + step < hi ? start + step : hi) - 1;
        bool below = false;
        if (active) {
            const uint32_t v = a[last];
            below = UPPER ? v <= x : v < x;
        }
        // sortedness makes the lanes with `below` a prefix of the active ones
        const uint32_t c = (uint32_t)__popcll(__ballot(below));
        const uint32_t nlo = lo + c * step < hi ? lo + c * step : hi;
        const uint32_t cstart = lo + c * step;                       // sub-range of lane c
        uint32_t nhi = hi;
        if (c < (uint32_t)kWave && cstart < hi)
            nhi = (cstart + step < hi ? cstart + step : hi) - 1;
        lo = nlo;
        hi = nhi;
    }
    return lo;
}

// Entry x of A goes to slot x + #{B < A[x]}, entry y of B to slot y + #{A <= B[y]}:
// a bijection onto [0, 2k) that lists the union in index order, A's copy first
// where both hold an index.  A's copy then carries the sum (one fp32 add) and B's
// slot becomes a tombstone.
// A block takes BLOCK*EPT consecutive entries of A and of B.  Four of its waves first
// find, each with one 64-ary search, the counts for the block's first and last entry of
// either side; every thread then searches only between those two counts, a short range
// that is staged in LDS.
// On the side, the grid clears zero_words words at zero_ptr: the select state that the
// NEXT round of the tree will use (this round's is in use, the other one is free).
// HIST: the block also counts the first digits of the keys it produces, which saves the
// select's histogram kernel; blocks are large then (BLOCK = 1024), as k_hist's are, so that
// a popular bin costs few global atomics.
template <int EPT, int BLOCK, bool HIST>
__global__ __launch_bounds__(BLOCK) void k_union(
        const uint32_t* __restrict__ a_idx, const float* __restrict__ a_val,
        const uint32_t* __restrict__ b_idx, const float* __restrict__ b_val, uint32_t k,
        int64_t in_stride, uint32_t* __restrict__ m_idx, float* __restrict__ m_val,
        uint32_t m_stride, uint32_t* __restrict__ zero_ptr, uint32_t zero_words, MergedSrc hsrc,
        SelState hst) {
    __shared__ uint32_t s_bound[4];
    __shared__ uint32_t s_hist[HIST ? kHistBins : 1];
    const int s = blockIdx.y;
    if (HIST)
        for (int b = threadIdx.x; b < kHistBins; b += BLOCK) s_hist[b] = 0u;   // barriers follow
    {
        const uint32_t nthreads = gridDim.x * gridDim.y * BLOCK;
        for (uint32_t i = (blockIdx.y * gridDim.x + blockIdx.x) * BLOCK + threadIdx.x; i < zero_words;
             i += nthreads)
            zero_ptr[i] = 0u;
    }
    const uint32_t x0 = blockIdx.x * (BLOCK * EPT);            // < k by the launch grid
    const uint32_t x1 = x0 + BLOCK * EPT - 1 < k ? x0 + BLOCK * EPT - 1 : k - 1;
    const uint32_t* ai = a_idx + (int64_t)s * in_stride;
    const float* av = a_val + (int64_t)s * in_stride;
    const uint32_t* bi = b_idx + (int64_t)s * in_stride;
    const float* bv = b_val + (int64_t)s * in_stride;
    uint32_t* mi = m_idx + (size_t)s * m_stride;
    float* mv = m_val + (size_t)s * m_stride;
    const uint32_t wave = threadIdx.x / kWave;
    // this thread's entries (loads overlap with the boundary searches)
    uint32_t ia[EPT], ib[EPT];
    float fa[EPT], fb[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const uint32_t x = x0 + j * BLOCK + threadIdx.x;
        const bool live = x < k;
        ia[j] = live ? ai[x] : 0u;
        ib[j] = live ? bi[x] : 0u;
        fa[j] = live ? av[x] : 0.0f;
        fb[j] = live ? bv[x] : 0.0f;
    }
    uint32_t bound = 0;
    if (wave == 0) bound = wave_count_below<false>(bi, k, ai[x0]);
    else if (wave == 1) bound = wave_count_below<false>(bi, k, ai[x1]);
    else if (wave == 2) bound = wave_count_below<true>(ai, k, bi[x0]);
    else if (wave == 3) bound = wave_count_below<true>(ai, k, bi[x1]);
    if (lane_id() == 0 && wave < 4) s_bound[wave] = bound;
    __syncthreads();
    // pa = #{B < ia} lies in [b_lo, b_hi], pb = #{A <= ib} in [a_lo, a_hi].  The searches
    // read bi[b_lo .. b_hi-1]; the match test reads bi/bv[pa] (pa <= b_hi) and the duplicate
    // test ai[pb-1] (pb-1 >= a_lo-1).  When those ranges fit, they are staged in LDS with
    // coalesced loads and searched there; otherwise the same code reads global memory.
    const uint32_t b_lo = s_bound[0], b_hi = s_bound[1], a_lo = s_bound[2], a_hi = s_bound[3];
    constexpr uint32_t kCap = 2u * BLOCK * EPT + 2u;
    __shared__ uint32_t s_bi[kCap];
    __shared__ float s_bv[kCap];
    __shared__ uint32_t s_ai[kCap];
    const uint32_t b_n = (b_hi < k ? b_hi + 1 : k) - b_lo;        // bi[b_lo .. min(b_hi, k-1)]
    const uint32_t a_first = a_lo > 0 ? a_lo - 1 : 0;
    const uint32_t a_n = a_hi - a_first;                          // ai[a_first .. a_hi-1]
    const bool staged = b_n <= kCap && a_n <= kCap;               // block-uniform
    if (staged) {
        // all loads first, then the LDS stores: one memory round trip for the whole stage
        constexpr int kRounds = (int)((kCap + BLOCK - 1) / BLOCK);
        uint32_t tb[kRounds], ta[kRounds];
        float tv[kRounds];
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const uint32_t i = r * BLOCK + threadIdx.x;
            tb[r] = i < b_n ? bi[b_lo + i] : 0u;
            tv[r] = i < b_n ? bv[b_lo + i] : 0.0f;
            ta[r] = i < a_n ? ai[a_first + i] : 0u;
        }
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const uint32_t i = r * BLOCK + threadIdx.x;
            if (i < b_n) { s_bi[i] = tb[r]; s_bv[i] = tv[r]; }
            if (i < a_n) s_ai[i] = ta[r];
        }
        __syncthreads();
    }
    auto B_idx = [&](uint32_t p) { return staged ? s_bi[p - b_lo] : bi[p]; };
    auto B_val = [&](uint32_t p) { return staged ? s_bv[p - b_lo] : bv[p]; };
    auto A_idx = [&](uint32_t p) { return staged ? s_ai[p - a_first] : ai[p]; };
    // all 2*EPT binary searches of a thread advance together, one load each per step
    uint32_t pa[EPT], pb[EPT], ha[EPT], hb[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        pa[j] = b_lo; ha[j] = b_hi;
        pb[j] = a_lo; hb[j] = a_hi;
    }
    const uint32_t ra = b_hi - b_lo, rb = a_hi - a_lo;
    const uint32_t rmax = ra > rb ? ra : rb;
    const int steps = rmax ? 32 - __builtin_clz(rmax) : 0;      // halvings until every range is empty
    for (int it = 0; it < steps; ++it) {
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            if (pa[j] < ha[j]) {
                const uint32_t mid = (pa[j] + ha[j]) >> 1;        // b_lo <= mid < b_hi
                if (B_idx(mid) < ia[j]) pa[j] = mid + 1; else ha[j] = mid;
            }
            if (pb[j] < hb[j]) {
                const uint32_t mid = (pb[j] + hb[j]) >> 1;        // a_lo <= mid < a_hi
                if (A_idx(mid) <= ib[j]) pb[j] = mid + 1; else hb[j] = mid;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const uint32_t x = x0 + j * BLOCK + threadIdx.x;
        if (x >= k) continue;
        float sum = fa[j];
        if (pa[j] < k && B_idx(pa[j]) == ia[j]) sum = sum + B_val(pa[j]);
        mi[x + pa[j]] = ia[j];
        mv[x + pa[j]] = sum;
        const bool dup = pb[j] > 0 && A_idx(pb[j] - 1) == ib[j];
        mi[x + pb[j]] = dup ? kTomb : ib[j];
        mv[x + pb[j]] = dup ? 0.0f : fb[j];         // a tombstone's value is +0.0 (see MergedSrc)
        if (HIST) {
            // the first digit of the keys this block has just produced (what k_hist would
            // read back): LDS counts now, one global add per bin and block below
            const Digit dg = hsrc.digit(s, false, hst);
            atomicAdd(&s_hist[dg.bin(__float_as_uint(sum) & kAbs)], 1u);
            if (!dup) atomicAdd(&s_hist[dg.bin(__float_as_uint(fb[j]) & kAbs)], 1u);
        }
    }
    if (HIST) {
        __syncthreads();
        uint32_t* out = hst.hist + (size_t)s * kHistBins;
        for (int b = threadIdx.x; b < kHistBins; b += BLOCK) {
            const uint32_t c = s_hist[b];
            if (c) atomicAdd(&out[b], c);
        }
    }
}

// First position of [lo, hi) at which pred is false (hi if there is none); pred must be
// true on a prefix of the range.  Wave-cooperative like wave_count_below: every lane
// calls it with the same arguments and gets the same result after log64(hi - lo) rounds.
template <class Pred>
__device__ inline uint32_t wave_first_false(uint32_t lo, uint32_t hi, Pred pred) {
    const uint32_t lane = lane_id();
    while (lo < hi) {
        const uint32_t len = hi - lo;
        const uint32_t step = (len + kWave - 1) / kWave;
        const uint32_t start = lo + lane * step;
        const bool active = start < hi;
        const uint32_t last = (start + step < hi ? start + step : hi) - 1;
        const bool t = active && pred(last);
        const uint32_t c = (uint32_t)__popcll(__ballot(t));
        const uint32_t cstart = lo + c * step;
        uint32_t nhi = hi;
        if (c < (uint32_t)kWave && cstart < hi) nhi = (cstart + step < hi ? cstart + step : hi) - 1;
        lo = cstart < hi ? cstart : hi;
        hi = nhi;
    }
    return lo;
}

// The same search by groups of L consecutive lanes (L a power of two), every group with a
// range and a predicate of its own (pred(x) may depend on the lane's group; the lanes of a
// group pass the same lo and hi, a group without work passes lo == hi): log_L rounds of one
// load per lane.  Fewer lanes per search mean more rounds but fewer loads per search, which
// is what counts once thousands of searches run side by side.  All 64 lanes must call it.
template <int L, class Pred>
__device__ inline uint32_t group_first_false(uint32_t lo, uint32_t hi, Pred pred) {
    static_assert(L >= 2 && L <= kWave && (L & (L - 1)) == 0, "a power of two, at most a wave");
    const uint32_t lane = lane_id(), gl = lane % L;
    const uint64_t gmask = (L == kWave ? ~0ull : ((1ull << (L % 64)) - 1ull)) << (lane - gl);
    while (__any(lo < hi)) {
        const bool busy = lo < hi;
        const uint32_t len = hi - lo;
        const uint32_t step = (len + L - 1) / L;
        const uint32_t start = lo + gl * step;
        const bool active = busy && start < hi;
        const uint32_t last = (start + step < hi ? start + step : hi) - 1;
        const bool t = active && pred(last);
        const uint32_t c = (uint32_t)__popcll(__ballot(t) & gmask);
        if (busy) {
            const uint32_t cstart = lo + c * step;
            uint32_t nhi = hi;
            if (c < (uint32_t)L && cstart < hi) nhi = (cstart + step < hi ? cstart + step : hi) - 1;
            lo = cstart < hi ? cstart : hi;
            hi = nhi;
        }
    }
    return lo;
}

// The same union, cut by OUTPUT position ("merge path"): for large sets.
// The 2k slots of a pair are the stable merge of A and B by index, A first among equals;
// the slot of an A entry that has an equal B entry right after it carries the sum, and
// that B entry's slot is a tombstone - exactly the layout k_union produces.
// A block owns kBlock*EPT consecutive slots.  Two of its waves find, each with one 64-ary
// search along a diagonal of the merge grid, how many A entries precede the block's
// first and last slot (CUTS: k_union_cuts has done that for all blocks beforehand, which
// pays for very large sets); the A and B entries in between (kBlock*EPT in total) are staged in
// LDS; every thread then finds the start of its own EPT slots with a binary search in LDS
// and merges EPT steps sequentially.  Rows of m_idx / m_val are m_stride apart (a multiple
// of EPT, 16-byte aligned), so every thread stores whole vectors; slots past 2k in the
// row's padding become tombstones.  HIST: as in k_union, with blocks as large as LDS allows.
// cuts[s][c] = number of A entries among the first c * tile slots of pair s (c = 0 .. ntiles;
// the last one is clamped to 2k slots): what k_union_path's blocks need, one search
// along a diagonal each, all side by side instead of one after the other in front of
// every block's work.
template <int L>
__global__ __launch_bounds__(kBlock) void k_union_cuts(
        const uint32_t* __restrict__ a_idx, const uint32_t* __restrict__ b_idx, uint32_t k,
        int64_t in_stride, uint32_t tile, uint32_t ntiles, uint32_t* __restrict__ cuts) {
    // L lanes per cut point: an L-ary search along the diagonal.  A binary search (L = 2)
    // waits for 23 dependent pairs of loads for sets of millions of entries, a 16-ary one
    // for 6 but issues four times as many; the host picks L by the number of cut points.
    const uint32_t c = (blockIdx.x * kBlock + threadIdx.x) / L;
    const int s = blockIdx.y;
    const bool work = c <= ntiles;
    const uint32_t* ai = a_idx + (int64_t)s * in_stride;
    const uint32_t* bi = b_idx + (int64_t)s * in_stride;
    const uint64_t pp = (uint64_t)c * tile;
    const uint32_t p = pp < 2ull * k ? (uint32_t)pp : 2 * k;
    const uint32_t lo = work ? (p > k ? p - k : 0u) : 0u, hi = work ? (p < k ? p : k) : 0u;
    // A[x] is among the first p slots iff A[x] <= B[p-1-x]
    const uint32_t x = group_first_false<L>(lo, hi, [&](uint32_t x) { return ai[x] <= bi[p - 1 - x]; });
    if (work && threadIdx.x % L == 0) cuts[(size_t)s * (ntiles + 1) + c] = x;
}

// FILTER (with HIST): of its tile the block keeps only the slots whose key reaches
// filt.tspec[s] (no tombstones either), packed at the start of the tile in index order;
// filt.tile_cnt[s][tile] = their number, which is also added to filt.set_cnt[s]; the first
// digits counted are those of the kept slots, in bins relative to the threshold (FiltSrc).
// gate_cnt != NULL: pair s is merged only if gate_cnt[s] < k (the complete union of a pair
// whose filtered union came out short).
struct UnionFilter {
    const uint32_t* tspec;
    uint32_t* tile_cnt;
    uint32_t* set_cnt;
};

template <int EPT, bool CUTS, int BLOCK, bool HIST, bool FILTER = false>
__global__ __launch_bounds__(BLOCK) void k_union_path(
        const uint32_t* __restrict__ a_idx, const float* __restrict__ a_val,
        const uint32_t* __restrict__ b_idx, const float* __restrict__ b_val, uint32_t k,
        int64_t in_stride, uint32_t* __restrict__ m_idx, float* __restrict__ m_val,
        uint32_t m_stride, const uint32_t* __restrict__ cuts, uint32_t* __restrict__ zero_ptr,
        uint32_t zero_words, MergedSrc hsrc, SelState hst, UnionFilter filt = UnionFilter{nullptr, nullptr, nullptr},
        const uint32_t* __restrict__ gate_cnt = nullptr) {
    static_assert(EPT % 4 == 0, "whole 16-byte vectors per thread");
    static_assert(!FILTER || HIST, "the filtered union counts its own first digits");
    if (gate_cnt && gate_cnt[blockIdx.y] >= k) return;       // block-uniform
    constexpr uint32_t kTile = BLOCK * EPT;
    constexpr uint32_t kStage = kTile + 3;         // A: previous + entries + sentinel; B: entries + next
    // EPT spare slots: with operands that are not sorted (unspecified results) a thread's
    // merge may run up to EPT entries past either staged range; it must stay inside LDS
    __shared__ uint32_t s_i[kStage + EPT];
    __shared__ float s_v[kStage + EPT];
    __shared__ uint32_t s_split[2];
    // two 16-bit counters per word: a tile holds kTile <= 65535 slots, so no count overflows, and
    // with the histogram at 8 KB two blocks fit the CU's LDS
    static_assert(kTile < 65536u, "16-bit counters");
    __shared__ uint32_t s_hist[HIST ? kHistBins / 2 : 1];
    auto count_bin = [&](uint32_t b) { atomicAdd(&s_hist[b >> 1], (b & 1u) ? 0x10000u : 1u); };
    __shared__ uint32_t s_scan[FILTER ? BLOCK / kWave : 1];
    const int s = blockIdx.y;
    if (HIST)
        for (int b = threadIdx.x; b < kHistBins / 2; b += BLOCK) s_hist[b] = 0u;   // barriers follow
    {
        const uint32_t nthreads = gridDim.x * gridDim.y * BLOCK;
        for (uint32_t i = (blockIdx.y * gridDim.x + blockIdx.x) * BLOCK + threadIdx.x; i < zero_words;
             i += nthreads)
            zero_ptr[i] = 0u;
    }
    const uint32_t n = 2 * k;
    const uint32_t p0 = blockIdx.x * kTile;                    // < n by the launch grid
    const uint32_t p1 = p0 + kTile < n ? p0 + kTile : n;
    const uint32_t* ai = a_idx + (int64_t)s * in_stride;
    const float* av = a_val + (int64_t)s * in_stride;
    const uint32_t* bi = b_idx + (int64_t)s * in_stride;
    const float* bv = b_val + (int64_t)s * in_stride;
    const uint32_t wave = threadIdx.x / kWave;
    if (CUTS) {
        if (threadIdx.x < 2) {
            uint32_t x = cuts[(size_t)s * (gridDim.x + 1) + blockIdx.x + threadIdx.x];
            if (x > k) x = k;             // only for operands that are not sorted
            s_split[threadIdx.x] = x;
        }
    } else if (wave < 2) {
        // number of A entries among the first p slots: A[x] is one of them iff A[x] <= B[p-1-x]
        const uint32_t p = wave == 0 ? p0 : p1;
        const uint32_t lo = p > k ? p - k : 0u, hi = p < k ? p : k;
        const uint32_t x = wave_first_false(lo, hi, [&](uint32_t x) { return ai[x] <= bi[p - 1 - x]; });
        if (lane_id() == 0) s_split[wave] = x;
    }
    __syncthreads();
    const uint32_t nout = p1 - p0;
    const uint32_t xa0 = s_split[0];
    uint32_t xa1 = s_split[1];
    // always true for sorted operands; keeps every access in bounds for any others
    if (xa1 < xa0) xa1 = xa0;
    if (xa1 > xa0 + nout) xa1 = xa0 + nout;
    const uint32_t yb0 = p0 - xa0, yb1 = p1 - xa1;
    const uint32_t na = xa1 - xa0, nb = yb1 - yb0;             // na + nb = p1 - p0
    // stage: s[0] = A[xa0-1] (or none), s[1 .. na] = A entries, s[na+1] = none (sentinel: above
    // every index); s[na+2 .. na+1+nb] = B entries, s[na+2+nb] = B[yb1] (or none)
    {
        constexpr int kRounds = (int)((kStage + BLOCK - 1) / BLOCK);
        uint32_t ti[kRounds];
        float tv[kRounds];
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const uint32_t c = r * BLOCK + threadIdx.x;
            ti[r] = kTomb;
            tv[r] = 0.0f;
            if (c < na + 1) {
                if (xa0 + c > 0) { ti[r] = ai[xa0 + c - 1]; tv[r] = av[xa0 + c - 1]; }
            } else if (c >= na + 2 && c < na + 3 + nb) {
                const uint32_t y = yb0 + (c - na - 2);
                if (y < k) { ti[r] = bi[y]; tv[r] = bv[y]; }
            }
        }
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            const uint32_t c = r * BLOCK + threadIdx.x;
            if (c < kStage) { s_i[c] = ti[r]; s_v[c] = tv[r]; }
        }
    }
    __syncthreads();
    const uint32_t* sa = s_i + 1;                  // sa[x], x in [-1, na]
    const uint32_t* sb = s_i + na + 2;             // sb[y], y in [0, nb]
    const float* sav = s_v + 1;
    const float* sbv = s_v + na + 2;
    const uint32_t d = threadIdx.x * EPT;          // first slot of this thread, relative to p0
    uint32_t oi[EPT];
    float ov[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) { oi[j] = kTomb; ov[j] = 0.0f; }
    if (d < nout) {                                // nout is a multiple of EPT except in the last block
        // A entries among the tile's first d slots
        uint32_t x = d > nb ? d - nb : 0u;
        {
            uint32_t hi = d < na ? d : na;
            while (x < hi) {
                const uint32_t mid = (x + hi) >> 1;
                if (sa[mid] <= sb[d - 1 - mid]) x = mid + 1; else hi = mid;
            }
        }
        uint32_t y = d - x;
        uint32_t a = sa[x], b = sb[y];
        uint32_t aprev = sa[(int)x - 1];
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            if (d + j >= nout) {                   // padding of the row
                oi[j] = kTomb;
                ov[j] = 0.0f;
            } else if (a <= b) {
                float v = sav[x];
                if (b == a) v = v + sbv[y];
                oi[j] = a;
                ov[j] = v;
                aprev = a;
                ++x;
                a = sa[x];
            } else {
                oi[j] = b == aprev ? kTomb : b;
                ov[j] = b == aprev ? 0.0f : sbv[y];  // a tombstone's value is +0.0 (see MergedSrc)
                ++y;
                b = sb[y];
            }
        }
    }
    if (!FILTER) {
        if (d < nout) {
            uint32_t* mi = m_idx + (size_t)s * m_stride + p0 + d;
            float* mv = m_val + (size_t)s * m_stride + p0 + d;
#pragma unroll
            for (int j = 0; j < EPT; j += 4) {
                *reinterpret_cast<uint4*>(mi + j) = make_uint4(oi[j], oi[j + 1], oi[j + 2], oi[j + 3]);
                *reinterpret_cast<float4*>(mv + j) = make_float4(ov[j], ov[j + 1], ov[j + 2], ov[j + 3]);
            }
            if (HIST) {
                // first digits of the keys just produced: what k_hist would read back
                const Digit dg = hsrc.digit(s, false, hst);
#pragma unroll
                for (int j = 0; j < EPT; ++j)
                    if (oi[j] != kTomb) count_bin(dg.bin(__float_as_uint(ov[j]) & kAbs));
            }
        }
    } else {
        // keep what reaches the threshold, packed at the start of the tile in slot order
        const uint32_t ts = filt.tspec[s];
        uint32_t keep = 0;
#pragma unroll
        for (int j = 0; j < EPT; ++j)
            if (oi[j] != kTomb && (__float_as_uint(ov[j]) & kAbs) >= ts) keep |= 1u << j;
        const uint32_t cnt = (uint32_t)__popc(keep);
        uint32_t total;
        const uint32_t incl = block_incl_scan(cnt, s_scan, total);      // total <= nout
        // (the scan's barriers lie behind every thread's merge: the staged operands are dead,
        // and their LDS collects the kept slots, which then leave in whole coalesced rows)
        uint32_t pos = incl - cnt;
        const Digit dg{ts, (uint32_t)kFineShift};
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            if ((keep >> j) & 1u) {
                s_i[pos] = oi[j];
                s_v[pos] = ov[j];
                ++pos;
                count_bin(dg.bin(__float_as_uint(ov[j]) & kAbs));
            }
        }
        __syncthreads();
        uint32_t* mi = m_idx + (size_t)s * m_stride + p0;
        float* mv = m_val + (size_t)s * m_stride + p0;
        for (uint32_t i = threadIdx.x; i < total; i += BLOCK) {
            mi[i] = s_i[i];
            mv[i] = s_v[i];
        }
        if (threadIdx.x == 0) {
            filt.tile_cnt[(size_t)s * gridDim.x + blockIdx.x] = total;
            if (total) atomicAdd(&filt.set_cnt[s], total);
        }
    }
    if (HIST) {
        __syncthreads();
        uint32_t* out = hst.hist + (size_t)s * kHistBins;
        for (int b = threadIdx.x; b < kHistBins; b += BLOCK) {
            const uint32_t c = (s_hist[b >> 1] >> ((b & 1) * 16)) & 0xFFFFu;
            if (c) atomicAdd(&out[b], c);
        }
    }
}

// Sample of the union of pair s for its speculative threshold: tile t covers positions
// [t * tile_stride, + 64) of BOTH operands (clipped to k), one wave per tile.  A sampled
// entry of A stands for its slot of the union: its value plus B's value at the same index,
// if B has one (binary search).  A sampled entry of B stands for its slot unless A holds
// the index too - that slot is A's.  So every slot of the union is sampled with the same
// probability, and the histogram of the sampled keys (16384 bins, added to samp_hist[s]
// with one atomic per non-empty bin and block) is read by k_sample_pick as for a row.
__global__ __launch_bounds__(kSampleBlock) void k_merge_sample(
        const uint32_t* __restrict__ a_idx, const float* __restrict__ a_val,
        const uint32_t* __restrict__ b_idx, const float* __restrict__ b_val, uint32_t k,
        int64_t in_stride, uint32_t tile_stride, uint32_t n_tiles, uint32_t* __restrict__ samp_hist) {
    __shared__ uint32_t h[kSampleBins];
    const int s = blockIdx.y;
    for (int b = threadIdx.x; b < kSampleBins; b += kSampleBlock) h[b] = 0u;
    __syncthreads();
    const uint32_t* ai = a_idx + (int64_t)s * in_stride;
    const float* av = a_val + (int64_t)s * in_stride;
    const uint32_t* bi = b_idx + (int64_t)s * in_stride;
    const float* bv = b_val + (int64_t)s * in_stride;
    static_assert(kSampleTile == kWave, "a tile is a wave's: the searches below are wave-cooperative");
    const uint32_t sub = threadIdx.x / kSampleTile, el = threadIdx.x % kSampleTile;
    const uint32_t tiles_per_round = (kSampleBlock / kSampleTile) * gridDim.x;
    for (uint64_t t = (uint64_t)blockIdx.x * (kSampleBlock / kSampleTile) + sub; t < n_tiles; t += tiles_per_round) {
        const uint64_t q0 = t * tile_stride;                       // wave-uniform
        if (q0 >= k) continue;
        const uint32_t cnt = k - q0 < (uint64_t)kSampleTile ? (uint32_t)(k - q0) : (uint32_t)kSampleTile;
        const bool act = el < cnt;
        const uint64_t q = q0 + (act ? el : cnt - 1);              // idle lanes repeat the tile's last entry
        const uint32_t ia = ai[q], ib = bi[q];
        const float va = av[q], vb = bv[q];
        // The tile's entries ascend, so the first B entry >= ia lies between those of the tile's
        // first and last index, and likewise for ib in A: sixteen lanes each find one of these
        // four bounds (6 rounds for millions of entries), then every lane finishes inside its
        // short ranges, both searches in step - a dozen dependent rounds instead of 46.
        const uint32_t ia_first = __shfl(ia, 0), ia_last = __shfl(ia, (int)cnt - 1);
        const uint32_t ib_first = __shfl(ib, 0), ib_last = __shfl(ib, (int)cnt - 1);
        const uint32_t j = el / 16;                                // which of the four bounds this lane helps with
        const uint32_t* arr = j < 2 ? bi : ai;
        const uint32_t want = j == 0 ? ia_first : j == 1 ? ia_last : j == 2 ? ib_first : ib_last;
        const uint32_t bound = group_first_false<16>(0u, k, [&](uint32_t x) { return arr[x] < want; });
        const uint32_t lo[4] = {__shfl(bound, 0), __shfl(bound, 16), __shfl(bound, 32), __shfl(bound, 48)};
        uint32_t lb = lo[0], hb = lo[1] > lo[0] ? lo[1] : lo[0];   // first B entry with index >= ia: in [lb, hb]
        uint32_t la = lo[2], ha = lo[3] > lo[2] ? lo[3] : lo[2];   // first A entry with index >= ib: in [la, ha]
        while (lb < hb || la < ha) {
            const uint32_t mb = (lb + hb) >> 1, ma = (la + ha) >> 1;
            const uint32_t xb = bi[mb < k ? mb : k - 1], xa = ai[ma < k ? ma : k - 1];
            if (lb < hb) { if (xb < ia) lb = mb + 1; else hb = mb; }
            if (la < ha) { if (xa < ib) la = ma + 1; else ha = ma; }
        }
        float v = va;
        if (lb < k && bi[lb] == ia) v = v + bv[lb];
        if (act) atomicAdd(&h[(__float_as_uint(v) & kAbs) >> kSampleShift], 1u);
        if (act && !(la < k && ai[la] == ib)) atomicAdd(&h[(__float_as_uint(vb) & kAbs) >> kSampleShift], 1u);
    }
    __syncthreads();
    uint32_t* out = samp_hist + (size_t)s * kSampleBins;
    for (int b = threadIdx.x; b < kSampleBins; b += kSampleBlock) {
        const uint32_t c = h[b];
        if (c) atomicAdd(&out[b], c);
    }
}

// Smallest key of each k-set, for sets that did not come out of a select of this library:
// out[s] = max over the set of (0x7fffffff - key), by atomic maximum onto a zeroed word.
// Set s is row s of v0 (v1 == NULL), or row s/2 of v0 (s even) / v1 (s odd).
__global__ __launch_bounds__(kBlock) void k_set_min_key(
        const float* __restrict__ v0, const float* __restrict__ v1, int64_t stride, uint32_t k,
        uint32_t* __restrict__ out) {
    __shared__ uint32_t s_wave[kBlock / kWave];
    const uint32_t s = blockIdx.y;
    const float* v = v1 ? ((s & 1) ? v1 : v0) + (int64_t)(s >> 1) * stride : v0 + (int64_t)s * stride;
    uint32_t best = 0;
    for (uint32_t i = blockIdx.x * kBlock + threadIdx.x; i < k; i += gridDim.x * kBlock) {
        const uint32_t inv = kAbs - (__float_as_uint(v[i]) & kAbs);
        best = inv > best ? inv : best;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const uint32_t o = __shfl_xor(best, d);
        best = o > best ? o : best;
    }
    if (lane_id() == 0) s_wave[threadIdx.x / kWave] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / kWave; ++w) best = s_wave[w] > best ? s_wave[w] : best;
        atomicMax(&out[s], best);
    }
}

// P == 1: the tree has no round; the global set is worker 0's set divided by 1.
__global__ void k_copy_set(const uint32_t* __restrict__ in_idx, const float* __restrict__ in_val,
                           uint32_t k, uint32_t* __restrict__ out_idx, float* __restrict__ out_val,
                           float divisor, uint32_t* __restrict__ gbits) {
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < k) {
        const uint32_t i = in_idx[t];
        out_idx[t] = i;
        out_val[t] = in_val[t] / divisor;
        if (gbits) atomicOr(&gbits[i >> 5], 1u << (i & 31));
    }
}

// ---------------------------------------------------------------------------------
// residual restore (Algorithm 4 line 10)
// ---------------------------------------------------------------------------------

__device__ __forceinline__ bool contains(const uint32_t* a, uint32_t n, uint32_t x) {
    uint32_t lo = 0, hi = n;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo < n && a[lo] == x;
}

// The literal form: the slots were zeroed by the local selection; add the value back
// where the index is not in the global set.
__global__ __launch_bounds__(kBlock) void k_restore(
        float* __restrict__ res, uint32_t m, int64_t stride, uint32_t k,
        const uint32_t* __restrict__ loc_idx, const float* __restrict__ loc_val,
        const uint32_t* __restrict__ g_idx) {
    const int w = blockIdx.y;
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    if (t >= k) return;
    const uint32_t i = loc_idx[(size_t)w * k + t];
    if (i >= m) return;                         // not a valid set: nothing is written outside the row
    if (contains(g_idx, k, i)) return;          // index is in the global set: stays zero
    float* slot = res + (int64_t)w * stride + i;
    *slot = *slot + loc_val[(size_t)w * k + t];
}

// The fused form used by gtopk_step, where the local selection did NOT zero its entries
// (the row still holds acc there).  Zero-then-add-back leaves acc unchanged except that
// +0.0 + (-0.0) = +0.0, so: an entry whose index is in the global set becomes +0.0, an
// entry that is -0.0 becomes +0.0, every other entry is already what the literal form
// produces.  gbits is the one-bit-per-element mask of the global set.  loc_min[w] is the
// smallest key of worker w's set: only a set that reaches down to key 0 can hold a -0.0, so
// the values of every other set are not read at all.
__global__ __launch_bounds__(kBlock) void k_restore_fused(
        float* __restrict__ res, int64_t stride, uint32_t k, const uint32_t* __restrict__ loc_idx,
        const float* __restrict__ loc_val, const uint32_t* __restrict__ gbits,
        const uint32_t* __restrict__ loc_min) {
    const int w = blockIdx.y;
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    if (t >= k) return;
    const uint32_t i = loc_idx[(size_t)w * k + t];
    const uint32_t vb = loc_min[w] == 0u ? __float_as_uint(loc_val[(size_t)w * k + t]) : 0u;   // block-uniform
    const bool in_g = (gbits[i >> 5] >> (i & 31)) & 1u;
    if (in_g || vb == 0x80000000u) res[(int64_t)w * stride + i] = 0.0f;
}

}  // namespace gtopk
