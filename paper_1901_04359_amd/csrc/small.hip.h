// The hot path for small problems (short rows, few workers, few selected entries), where a
// step is bound by the number of dependent kernel launches and not by bytes:
//   k_small_sample  the speculative threshold of one worker in ONE block (sample histogram
//                   in LDS and the pick), which also clears the worker's candidate counter;
//   k_small_select  the exact local selection (Algorithm 4 lines 5-7) of one worker in ONE
//                   block, with block-level synchronisation only: a short candidate list by
//                   one wave that holds all keys in registers, anything else by histogram,
//                   radix refinement and ordered emit;
//   k_small_tree    the whole gTopKAllReduce tree (Algorithm 3 lines 4-18: every round's
//                   Top-k operations of Definition 1), the division by P (Eq. 3) and the
//                   extra residual (Algorithm 4 line 10) in ONE block, all sets in LDS.
// The last two produce bit for bit what the general kernels produce; the threshold of the
// first only sizes the work.
#pragma once
#include "common.hip.h"
#include "select.hip.h"

namespace gtopk {

constexpr int kSmallBlock = 1024;
constexpr int kSmallIters = 2;               // float4 per lane of the streaming pass's blocks
constexpr int kSmallChunk = kSmallIters * 4 * kSBlock;      // 4096 elements per block = one run
constexpr int kSmallMaxChunks = 256;         // rows of at most 2^20 elements
constexpr int kSmallMaxEntries = 4096;       // P * k, at most
constexpr int kSmallMaxK = 512;
constexpr int kSmallMaxP = 64;
constexpr int kSmallRankList = 2048;         // candidate lists up to here: selection by one wave
constexpr int kSmallSampleUnroll = 16;       // tiles a wave of the sampler keeps in flight

// Sum / maximum / minimum of v over the 64 lanes of the wave (every lane takes part; the
// result is uniform): butterfly steps inside each row of 16 lanes, then the four row
// results on the scalar side.
#define GTOPK_ROW_BUTTERFLY(v, OP)                                                                  \
    do {                                                                                           \
        v = OP(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(v), 0xB1, 0xf, 0xf, true));  /* quad_perm [1,0,3,2] */ \
        v = OP(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(v), 0x4E, 0xf, 0xf, true));  /* quad_perm [2,3,0,1] */ \
        v = OP(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(v), 0x141, 0xf, 0xf, true)); /* row_half_mirror */     \
        v = OP(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(v), 0x140, 0xf, 0xf, true)); /* row_mirror */          \
    } while (0)
#define GTOPK_ROWS(v, OP)                                                                           \
    OP(OP((uint32_t)__builtin_amdgcn_readlane((int)(v), 0), (uint32_t)__builtin_amdgcn_readlane((int)(v), 16)), \
       OP((uint32_t)__builtin_amdgcn_readlane((int)(v), 32), (uint32_t)__builtin_amdgcn_readlane((int)(v), 48)))
__device__ __forceinline__ uint32_t op_add(uint32_t a, uint32_t b) { return a + b; }
__device__ __forceinline__ uint32_t op_max(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t op_min(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) { GTOPK_ROW_BUTTERFLY(v, op_add); return GTOPK_ROWS(v, op_add); }
__device__ __forceinline__ uint32_t wave_max(uint32_t v) { GTOPK_ROW_BUTTERFLY(v, op_max); return GTOPK_ROWS(v, op_max); }
__device__ __forceinline__ uint32_t wave_min(uint32_t v) { GTOPK_ROW_BUTTERFLY(v, op_min); return GTOPK_ROWS(v, op_min); }
#undef GTOPK_ROW_BUTTERFLY
#undef GTOPK_ROWS

// ONE wave selects the k largest of n <= 64 * NCH keys in LDS; keys[j] = key + 1 of position
// j, or 0 for a position that holds nothing and is never selected (at least k positions
// hold something).  Among equal keys the lower positions win.  The wave holds the keys in
// registers, 64 per register; no barrier and next to no LDS traffic inside the search.
//   1. T, the k-th largest key, is bracketed: count_ge(lo) >= k > count_ge(hi).  The bracket
//      starts at [smallest key, largest key + 1) and shrinks around a trial value placed
//      where a straight line through the two counts crosses k; after two moves of the same
//      end the next trial halves the bracket, so the loop ends on any input.
//   2. Once the bracket holds at most 64 keys they are gathered, one per lane, and T is
//      found bit by bit below the common prefix of the bracket's ends.
//   3. Positions above T are selected, and the lowest positions among those equal to T.
// Bit j of `selbits` (ceil(n / 32) words, all of them stored by this wave) tells whether
// position j is selected.  `gather`: 64 words of LDS of this wave's own.
template <int NCH>
__device__ __forceinline__ void wave_select(const uint32_t* keys, uint32_t n, uint32_t k,
                                            uint32_t* selbits, uint32_t* gather) {
    const uint32_t lane = lane_id();
    const uint64_t below = (1ull << lane) - 1ull;
    uint32_t K[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) K[c] = (uint32_t)c * kWave + lane < n ? keys[c * kWave + lane] : 0u;
    auto count_ge = [&](uint32_t v) {
        uint32_t mine = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c) mine += K[c] >= v ? 1u : 0u;
        return wave_sum(mine);
    };
    uint32_t mx = 0, mn = 0xFFFFFFFFu;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        mx = op_max(mx, K[c]);
        mn = op_min(mn, K[c] - 1u);                  // an empty position counts as the largest value
    }
    // ---- 1. bracket ---------------------------------------------------------------------
    uint32_t lo = wave_min(mn) + 1u, hi = wave_max(mx) + 1u;       // 1 <= lo < hi <= 2^31 + 1
    uint32_t c_lo = count_ge(lo), c_hi = 0u;                       // c_lo = positions that hold something
    int last = 0, run = 0;                                         // which end moved last, how often in a row
    while (hi - lo > 1u && c_lo - c_hi > (uint32_t)kWave) {
        const uint32_t w = hi - lo;
        uint32_t d = w >> 1;
        if (run < 2) {
            const float f = (float)w * (((float)(c_lo - k) + 0.5f) / (float)(c_lo - c_hi));
            d = (uint32_t)f;
            d = d < 1u ? 1u : (d > w - 1u ? w - 1u : d);
        } else {
            run = 0;
        }
        const uint32_t v = lo + d;                                 // lo < v < hi
        const uint32_t c = count_ge(v);
        const int side = c >= k ? 1 : 2;
        if (side == 1) { lo = v; c_lo = c; } else { hi = v; c_hi = c; }
        run = side == last ? run + 1 : 1;
        last = side;
    }
    // ---- 2. inside the bracket ------------------------------------------------------------
    uint32_t T = lo;
    if (hi - lo > 1u) {                              // wave-uniform; at most 64 keys in [lo, hi)
        uint32_t base = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const bool in = K[c] >= lo && K[c] < hi;
            const uint64_t m = __ballot(in);
            if (in) gather[base + (uint32_t)__popcll(m & below)] = K[c];
            base += (uint32_t)__popcll(m);
        }
        const uint32_t X = lane < base ? gather[lane] : 0u;        // the wave reads its own stores
        const uint32_t r = k - c_hi;                               // T is the r-th largest of them
        const int top = 31 - __builtin_clz(lo ^ (hi - 1u));        // the ends differ: lo < hi - 1
        T = top == 31 ? 0u : lo & ~((2u << top) - 1u);             // their common prefix
        for (int b = top; b >= 0; --b) {
            const uint32_t cand = T | (1u << b);
            if ((uint32_t)__popcll(__ballot(X >= cand)) >= r) T = cand;
        }
    }
    // ---- 3. mark --------------------------------------------------------------------------
    const uint32_t need = k - count_ge(T + 1u);      // positions with key == T to take (T <= 2^31)
    const uint32_t words = (n + 31) / 32;
    uint32_t eq_before = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        if ((uint32_t)c * kWave >= n) continue;      // wave-uniform
        const uint64_t eq = __ballot(K[c] == T);
        const bool sel = K[c] != 0u &&
                         (K[c] > T || (K[c] == T && eq_before + (uint32_t)__popcll(eq & below) < need));
        const uint64_t m = __ballot(sel);
        if (lane == 0) {
            selbits[2 * c] = (uint32_t)m;
            if ((uint32_t)(2 * c + 1) < words) selbits[2 * c + 1] = (uint32_t)(m >> 32);
        }
        eq_before += (uint32_t)__popcll(eq);
    }
}

// the same for a list length known at run time (n <= 64 * MAXCH, MAXCH = 16 or 32)
template <int MAXCH>
__device__ __forceinline__ void wave_select_any(const uint32_t* keys, uint32_t n, uint32_t k,
                                                uint32_t* selbits, uint32_t* gather) {
    if (n <= 128u) wave_select<2>(keys, n, k, selbits, gather);
    else if (n <= 192u) wave_select<3>(keys, n, k, selbits, gather);
    else if (n <= 256u) wave_select<4>(keys, n, k, selbits, gather);
    else if (n <= 384u) wave_select<6>(keys, n, k, selbits, gather);
    else if (n <= 512u) wave_select<8>(keys, n, k, selbits, gather);
    else if (n <= 640u) wave_select<10>(keys, n, k, selbits, gather);
    else if (n <= 768u) wave_select<12>(keys, n, k, selbits, gather);
    else if (MAXCH == 16 || n <= 1024u) wave_select<16>(keys, n, k, selbits, gather);
    else wave_select<32>(keys, n, k, selbits, gather);
}

// ---------------------------------------------------------------------------------
// speculative threshold of one worker in one block
// ---------------------------------------------------------------------------------

// Worker w = blockIdx.x.  Sample tile t covers [t*tile_stride, t*tile_stride + 64) of the
// accumulated row (clipped to m), one wave per tile; the block histograms the keys of all
// tiles in LDS and stores the lower edge of the bucket at which the count from the top
// reaches `target`.  It also clears the worker's candidate counter for the streaming pass
// that follows in stream order.
__global__ __launch_bounds__(kSmallBlock) void k_small_sample(
        const float* __restrict__ grad, const float* __restrict__ res, uint32_t m, int64_t stride,
        uint32_t tile_stride, uint32_t n_tiles, uint32_t target, uint32_t* __restrict__ tspec,
        uint32_t* __restrict__ cand_count) {
    constexpr int kT = kSmallBlock;
    __shared__ uint32_t h[kSampleBins];
    __shared__ uint32_t s_wave[kT / kWave];
    __shared__ uint32_t s_out[3];
    const int w = blockIdx.x;
    const uint32_t t = threadIdx.x;
    if (t == 0) cand_count[w] = 0u;
    for (int b = t; b < kSampleBins; b += kT) h[b] = 0u;
    __syncthreads();
    const float* g = grad + (int64_t)w * stride;
    const float* r = res + (int64_t)w * stride;
    const uint32_t wave = t / kWave, el = t % kWave;
    constexpr uint32_t kWaves = kT / kWave;
    for (uint32_t t0 = wave; t0 < n_tiles; t0 += kWaves * kSmallSampleUnroll) {
        float gv[kSmallSampleUnroll], rv[kSmallSampleUnroll];
        bool ok[kSmallSampleUnroll];
#pragma unroll
        for (int u = 0; u < kSmallSampleUnroll; ++u) {
            const uint32_t tile = t0 + (uint32_t)u * kWaves;
            const uint64_t q = (uint64_t)tile * tile_stride + el;
            ok[u] = tile < n_tiles && q < m;
            gv[u] = ok[u] ? g[q] : 0.0f;
            rv[u] = ok[u] ? r[q] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < kSmallSampleUnroll; ++u)
            if (ok[u]) atomicAdd(&h[(__float_as_uint(rv[u] + gv[u]) & kAbs) >> kSampleShift], 1u);
    }
    __syncthreads();
    constexpr int kPer = kSampleBins / kT;
    uint32_t loc[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) loc[j] = h[t * kPer + j];
    suffix_pick<kPer>(loc, target, s_wave, s_out);
    if (t == 0) tspec[w] = s_out[2] ? (s_out[0] << kSampleShift) : 0u;
}

// ---------------------------------------------------------------------------------
// local selection of one worker in one block
// ---------------------------------------------------------------------------------

// Worker s = blockIdx.x.  The items are the worker's candidate list (or, if the
// speculative threshold left fewer than k candidates or more than the list holds, its
// dense row; slow for a long row, but rows are short here).  A candidate list of at most
// 2048 entries goes to LDS and one wave selects from it (wave_select).  Anything else takes
// three stages, each a walk over the items:
//   1. LDS histogram of the first digit -> the bin d1 of the k-th key;
//   2. up to three LDS radix passes over the keys inside bin d1 -> the exact key T and the
//      number of ties to take;
//   3. the emit in index order (for a candidate list: run after run in chunk order).
__global__ __launch_bounds__(kSmallBlock) void k_small_select(
        CandSrc src, uint32_t k, uint32_t* __restrict__ out_idx, float* __restrict__ out_val) {
    constexpr int kT = kSmallBlock;
    __shared__ uint32_t h[kHistBins];
    __shared__ uint32_t s_wave[kT / kWave];
    __shared__ uint32_t s_out[3];
    __shared__ uint32_t s_rx[kSmallMaxChunks];
    __shared__ uint32_t s_roff[kSmallMaxChunks + 1];
    __shared__ uint32_t s_gather[kWave];
    const int s = blockIdx.x;
    const uint32_t t = threadIdx.x;
    const bool dn = src.dense(s);
    const uint32_t n = src.nphys(s, dn);
    if (!dn && n <= (uint32_t)kSmallRankList) {
        // ---- a short candidate list: the keys go to LDS in index order (run after run in
        // chunk order), one wave selects the k largest, ties to the lower index (Algorithm 4
        // line 5), and every thread writes out its selected entries
        uint32_t* keys = h;                                    // kSmallRankList <= kHistBins
        static_assert(kSmallRankList <= kHistBins && kSmallRankList / 32 <= kWave && kSmallRankList / 32 <= kSmallMaxChunks, "");
        const uint32_t nruns = src.nchunks;                    // <= kSmallMaxChunks <= kT
        uint2 run = make_uint2(0u, 0u);
        if (t < nruns) run = src.run_table[(size_t)s * src.nchunks + t];
        uint32_t tot;
        const uint32_t incl = block_incl_scan(run.y, s_wave, tot);
        if (t < nruns) { s_rx[t] = run.x; s_roff[t + 1] = incl; }
        if (t == 0) s_roff[0] = 0u;
        __syncthreads();
        constexpr int kPer = kSmallRankList / kT;
        uint32_t idx[kPer], bits[kPer];
#pragma unroll
        for (int c = 0; c < kPer; ++c) {
            const uint32_t lp = (uint32_t)c * kT + t;
            idx[c] = 0u; bits[c] = 0u;
            if (lp < n) {
                uint32_t r = 0, hi = nruns;             // the run r with roff[r] <= lp < roff[r+1]
                while (hi - r > 1) {
                    const uint32_t mid = (r + hi) >> 1;
                    if (s_roff[mid] <= lp) r = mid; else hi = mid;
                }
                src.fetch_phys(s, false, s_rx[r] + (lp - s_roff[r]), idx[c], bits[c]);
            }
            keys[lp] = lp < n ? (bits[c] & kAbs) + 1u : 0u;    // padding: beats nobody
        }
        __syncthreads();
        uint32_t* selbits = s_rx;                              // the run table has been used
        uint32_t* wpre = s_roff;
        if (t < (uint32_t)kWave) {                             // one wave selects
            wave_select_any<kSmallRankList / kWave>(keys, n, k, selbits, s_gather);
            // selected entries before each bitmap word (the wave reads its own stores)
            const uint32_t c = t < (n + 31) / 32 ? (uint32_t)__popc(selbits[t]) : 0u;
            wpre[t] = wave_incl_scan(c) - c;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < kPer; ++c) {
            const uint32_t lp = (uint32_t)c * kT + t;
            if (lp >= n) break;
            const uint32_t wd = selbits[lp >> 5];
            if ((wd >> (lp & 31)) & 1u) {
                // < k: exactly k entries are selected
                const uint32_t pos = wpre[lp >> 5] + (uint32_t)__popc(wd & ((1u << (lp & 31)) - 1u));
                out_idx[(size_t)s * k + pos] = idx[c];
                out_val[(size_t)s * k + pos] = __uint_as_float(bits[c]);
            }
        }
        return;
    }
    const Digit dg = src.digit(s, dn, SelState{});
    const uint32_t fl = src.floor_key(s, dn);

    // ---- 1. first digit --------------------------------------------------------------
    for (int b = t; b < kHistBins; b += kT) h[b] = 0u;
    __syncthreads();
    for (uint32_t p0 = 0; p0 < n; p0 += kT * 4) {
        uint32_t key[4];
        bool ok[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t p = p0 + j * kT + t;
            key[j] = 0;
            ok[j] = p < n && src.fetch_key_phys(s, dn, p, key[j]) && key[j] >= fl;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
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
    __syncthreads();
    uint32_t d1, krem;
    {
        constexpr int kPer = kHistBins / kT;
        uint32_t loc[kPer];
#pragma unroll
        for (int j = 0; j < kPer; ++j) loc[j] = h[t * kPer + j];
        suffix_pick<kPer>(loc, k, s_wave, s_out);
        d1 = s_out[0];
        krem = k - s_out[1];
    }
    // ---- 2. the exact key --------------------------------------------------------------
    const uint32_t lo = dg.lo(d1), width = dg.width(d1);    // bin d1 = [lo, lo + width)
    uint32_t prefix = 0;          // value of the rel bits above the current pass
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
        const int bits = pass == 0 ? 11 : 10;
        if (shift > 0 && width <= (1u << shift)) continue;       // uniform
        __syncthreads();                                         // the last pick has read h
        for (int b = t; b < 2048; b += kT) h[b] = 0u;
        __syncthreads();
        for (uint32_t p0 = 0; p0 < n; p0 += kT * 4) {
            uint32_t key[4];
            bool ok[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t p = p0 + j * kT + t;
                key[j] = 0;
                ok[j] = p < n && src.fetch_key_phys(s, dn, p, key[j]) && key[j] >= fl;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t rel = key[j] - lo;
                const bool mine = ok[j] && dg.bin(key[j]) == d1 && (rel >> (shift + bits)) == prefix;
                const uint32_t b = (rel >> shift) & ((1u << bits) - 1u);
                const uint64_t act = __ballot(mine);
                if (act == 0) continue;
                const uint32_t b0 = __shfl(b, __builtin_ctzll(act));
                if (__ballot(mine && b == b0) == act) {
                    if (lane_id() == (uint32_t)__builtin_ctzll(act)) atomicAdd(&h[b0], (uint32_t)__popcll(act));
                } else if (mine) {
                    atomicAdd(&h[b], 1u);
                }
            }
        }
        __syncthreads();
        const uint32_t loc[2] = {h[2 * t], h[2 * t + 1]};
        suffix_pick<2>(loc, krem, s_wave, s_out);
        prefix = (prefix << bits) | s_out[0];
        krem -= s_out[1];
    }
    const uint32_t T = lo + prefix;
    const uint32_t need = krem;

    // ---- 3. ordered emit ---------------------------------------------------------------
    // a candidate list is read run after run in chunk order: first slots and running counts
    uint32_t nruns = 1;
    if (!dn) {
        nruns = src.nchunks;                                   // <= kSmallMaxChunks <= kT
        uint2 run = make_uint2(0u, 0u);
        if (t < nruns) run = src.run_table[(size_t)s * src.nchunks + t];
        uint32_t tot;
        const uint32_t incl = block_incl_scan(run.y, s_wave, tot);
        if (t < nruns) { s_rx[t] = run.x; s_roff[t + 1] = incl; }
        if (t == 0) s_roff[0] = 0u;
    }
    __syncthreads();
    uint32_t outp = 0, eq_before = 0;
    for (uint32_t base = 0; base < n; base += kT) {
        const uint32_t lp = base + t;
        uint32_t idx = 0, bits = 0;
        bool ok = lp < n;
        if (ok) {
            uint32_t p = lp;
            if (!dn) {
                uint32_t r = 0, hi = nruns;             // the run r with roff[r] <= lp < roff[r+1]
                while (hi - r > 1) {
                    const uint32_t mid = (r + hi) >> 1;
                    if (s_roff[mid] <= lp) r = mid; else hi = mid;
                }
                p = s_rx[r] + (lp - s_roff[r]);
            }
            ok = src.fetch_phys(s, dn, p, idx, bits) && (bits & kAbs) >= fl;
        }
        const uint32_t key = bits & kAbs;
        const bool is_gt = ok && key > T;
        const bool is_eq = ok && key == T;
        uint32_t eq_tot, sel_tot;
        const uint32_t eq_incl = block_incl_scan(is_eq ? 1u : 0u, s_wave, eq_tot);
        const bool sel = is_gt || (is_eq && eq_before + eq_incl - 1u < need);
        const uint32_t sel_incl = block_incl_scan(sel ? 1u : 0u, s_wave, sel_tot);
        if (sel) {
            const uint32_t pos = outp + sel_incl - 1u;
            if (pos < k) {          // always true when the counts are consistent
                out_idx[(size_t)s * k + pos] = idx;
                out_val[(size_t)s * k + pos] = __uint_as_float(bits);
            }
        }
        outp += sel_tot;
        eq_before += eq_tot;
    }
}

// ---------------------------------------------------------------------------------
// the whole tree, the average and the extra residual in one block
// ---------------------------------------------------------------------------------

// All P k-sets sit in LDS (P * k <= 4096 entries).  Round j merges set 2p with set 2p+1 of
// the surviving sets for every pair p, the pairs side by side:
//   union      `team` = 1024 / pairs threads per pair: entry x of A goes to slot
//              x + #{B < A[x]}, entry y of B to y + #{A <= B[y]} (binary searches in LDS);
//              A's copy carries the sum at a shared index, B's slot there becomes a
//              tombstone: the union in index order in 2k slots;
//   select     one wave per pair (a wave takes two pairs in turn where there are 32) finds
//              the k largest keys of the pair's union in registers, ties to the lower slot
//              = lower index (Definition 1); see wave_select;
//   compact    selected slots, in slot (= index) order, become set p of the next round.
// After the last round set 0 is the global set: its values are divided by P and written
// out, and every worker's locally selected entries whose index is in it (or whose value is
// -0.0, which the literal zero-then-add-back would turn into +0.0) are stored as +0.0 in
// the worker's row - the rows still hold the accumulated values at the selected entries.
__global__ __launch_bounds__(kSmallBlock) void k_small_tree(
        const uint32_t* __restrict__ loc_idx, const float* __restrict__ loc_val, uint32_t P,
        uint32_t k, uint32_t* __restrict__ g_idx, float* __restrict__ g_val, float divisor,
        float* __restrict__ res, int64_t stride) {
    constexpr int kT = kSmallBlock;
    constexpr int kWaves = kT / kWave;
    constexpr int kMaxPairs = kSmallMaxP / 2;
    constexpr int kPer = kSmallMaxEntries / kT;       // entries of the input sets per thread
    __shared__ uint32_t a_idx[kSmallMaxEntries];      // the surviving sets, k entries each
    __shared__ uint32_t a_val[kSmallMaxEntries];
    __shared__ uint32_t m_idx[kSmallMaxEntries];      // per pair: the 2k slots of its union
    __shared__ uint32_t m_val[kSmallMaxEntries];
    __shared__ uint32_t m_key[kSmallMaxEntries];      // key + 1 of every slot (0: tombstone)
    __shared__ uint32_t selw[kSmallMaxEntries / 32 + kMaxPairs];   // per pair: one bit per slot
    __shared__ uint32_t wpre[kSmallMaxEntries / 32 + kMaxPairs];   // selected slots before each word
    __shared__ uint32_t s_gather[kT];                 // 64 words per wave
    const uint32_t t = threadIdx.x;
    const uint32_t total = P * k;
    uint32_t in_idx[kPer], in_val[kPer];              // kept for the extra residual
#pragma unroll
    for (int c = 0; c < kPer; ++c) {
        const uint32_t e = (uint32_t)c * kT + t;
        in_idx[c] = 0u; in_val[c] = 0u;
        if (e < total) {
            in_idx[c] = loc_idx[e];
            in_val[c] = __float_as_uint(loc_val[e]);
            a_idx[e] = in_idx[c];
            a_val[e] = in_val[c];
        }
    }
    __syncthreads();
    const uint32_t n2 = 2 * k;
    const uint32_t words = (n2 + 31) / 32;            // bitmap words per pair
    for (uint32_t nsets = P; nsets > 1; nsets >>= 1) {
        const uint32_t pairs = nsets >> 1;
        const uint32_t team = kT / pairs;             // threads per pair (pairs <= 32: >= 32)
        const uint32_t p = t / team, l = t % team;
        const uint32_t* ai = a_idx + (2 * p) * k;
        const uint32_t* av = a_val + (2 * p) * k;
        const uint32_t* bi = ai + k;
        const uint32_t* bv = av + k;
        uint32_t* mi = m_idx + p * n2;
        uint32_t* mv = m_val + p * n2;
        uint32_t* mk = m_key + p * n2;
        // ---- union ------------------------------------------------------------------
        // (one entry of A or of B per thread and turn: e < k is entry e of A, else entry e - k of B)
        for (uint32_t e = l; e < n2; e += team) {
            const bool of_b = e >= k;
            const uint32_t x = of_b ? e - k : e;
            const uint32_t* oi = of_b ? ai : bi;      // the other set
            const uint32_t mine = of_b ? bi[x] : ai[x];
            const uint32_t bound = mine + (of_b ? 1u : 0u);      // #{other < bound}; indices are < 2^31
            uint32_t lo = 0, hi = k;
            while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (oi[mid] < bound) lo = mid + 1; else hi = mid; }
            uint32_t idx = mine, val = of_b ? bv[x] : av[x];
            if (of_b) {
                if (lo > 0 && ai[lo - 1] == mine) idx = kTomb;                  // A's copy carries the sum
            } else if (lo < k && bi[lo] == mine) {
                val = __float_as_uint(__uint_as_float(val) + __uint_as_float(bv[lo]));     // one fp32 add
            }
            mi[x + lo] = idx;
            mv[x + lo] = val;
            mk[x + lo] = idx == kTomb ? 0u : (val & kAbs) + 1u;
        }
        __syncthreads();
        // ---- select: one wave per pair (pairs in turns where there are more than waves),
        // which then counts the selected slots before each bitmap word of the pair
        for (uint32_t q = t / kWave; q < pairs; q += kWaves) {
            wave_select_any<2 * kSmallMaxK / kWave>(m_key + q * n2, n2, k, selw + q * words,
                                                    s_gather + (t / kWave) * kWave);
            uint32_t before = 0;
            for (uint32_t v0 = 0; v0 < words; v0 += kWave) {
                const uint32_t v = v0 + lane_id();
                const uint32_t c = v < words ? (uint32_t)__popc(selw[q * words + v]) : 0u;
                const uint32_t incl = wave_incl_scan(c);
                if (v < words) wpre[q * words + v] = before + incl - c;
                before += __shfl(incl, kWave - 1);
            }
        }
        __syncthreads();
        // ---- compact into set p of the next round --------------------------------------
        // (every read of the current sets is over: they are overwritten in place)
        for (uint32_t i = l; i < n2; i += team) {
            const uint32_t wd = selw[p * words + (i >> 5)];
            if ((wd >> (i & 31)) & 1u) {
                // < k: exactly k slots are selected
                const uint32_t pos = wpre[p * words + (i >> 5)] + (uint32_t)__popc(wd & ((1u << (i & 31)) - 1u));
                a_idx[p * k + pos] = mi[i];
                a_val[p * k + pos] = mv[i];
            }
        }
        __syncthreads();
    }
    // ---- the global set: average, write out ------------------------------------------------
    for (uint32_t i = t; i < k; i += kT) {
        g_idx[i] = a_idx[i];
        g_val[i] = __uint_as_float(a_val[i]) / divisor;
    }
    // ---- extra residual ---------------------------------------------------------------------
    if (res) {
#pragma unroll
        for (int c = 0; c < kPer; ++c) {
            const uint32_t e = (uint32_t)c * kT + t;
            if (e >= total) break;
            const uint32_t w = e / k;
            const uint32_t i = in_idx[c];
            uint32_t lo = 0, hi = k;
            while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (a_idx[mid] < i) lo = mid + 1; else hi = mid; }
            const bool in_g = lo < k && a_idx[lo] == i;
            if (in_g || in_val[c] == 0x80000000u) res[(int64_t)w * stride + i] = 0.0f;
        }
    }
}

}  // namespace gtopk
