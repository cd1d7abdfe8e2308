// The hot path for small problems (short rows, few workers, few selected entries), where a
// step is bound by the number of dependent kernel launches and not by bytes:
//   k_small_select  the exact local selection (Algorithm 4 lines 5-7) of one worker in ONE
//                   block: histogram, radix refinement and ordered emit over the worker's
//                   candidate list, with block-level synchronisation only;
//   k_small_tree    the whole gTopKAllReduce tree (Algorithm 3 lines 4-18: every round's
//                   Top-k operations of Definition 1), the division by P (Eq. 3) and the
//                   extra residual (Algorithm 4 line 10) in ONE block, all sets in LDS.
// Both produce bit for bit what the general kernels produce.
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

// ---------------------------------------------------------------------------------
// local selection of one worker in one block
// ---------------------------------------------------------------------------------

// Worker s = blockIdx.x.  The items are the worker's candidate list (or, if the
// speculative threshold left fewer than k candidates or more than the list holds, its
// dense row; slow for a long row, but rows are short here).  Three stages, each a walk
// over the items:
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
    const int s = blockIdx.x;
    const uint32_t t = threadIdx.x;
    const bool dn = src.dense(s);
    const uint32_t n = src.nphys(s, dn);
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
// the surviving sets for every pair p, the pairs side by side, `team` = 1024 / pairs
// threads each:
//   union      entry x of A goes to slot x + #{B < A[x]}, entry y of B to y + #{A <= B[y]}
//              (binary searches in LDS); A's copy carries the sum at a shared index, B's
//              slot there becomes a tombstone: the union in index order in 2k slots;
//   select     the k-th largest key of the pair's union by four LDS radix passes of 8, 8, 8
//              and 7 bits (256 counters per pair), then the ties by index order;
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
    constexpr int kMaxPairs = kSmallMaxP / 2;
    __shared__ uint32_t a_idx[kSmallMaxEntries];      // the surviving sets, k entries each
    __shared__ uint32_t a_val[kSmallMaxEntries];
    __shared__ uint32_t m_idx[kSmallMaxEntries];      // per pair: the 2k slots of its union
    __shared__ uint32_t m_val[kSmallMaxEntries];
    __shared__ uint32_t cnt[kMaxPairs * 256];         // per pair: 256 radix counters
    __shared__ uint32_t p_prefix[kMaxPairs], p_rem[kMaxPairs];
    __shared__ uint32_t selw[kSmallMaxEntries / 32 + kMaxPairs];   // per pair: one bit per slot
    __shared__ uint32_t tiew[kSmallMaxEntries / 32 + kMaxPairs];   // likewise: slots with key == T
    const uint32_t t = threadIdx.x;
    const uint32_t total = P * k;
    for (uint32_t i = t; i < total; i += kT) {
        a_idx[i] = loc_idx[i];
        a_val[i] = __float_as_uint(loc_val[i]);
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
        // ---- union ------------------------------------------------------------------
        for (uint32_t x = l; x < k; x += team) {
            const uint32_t ia = ai[x], ib = bi[x];
            uint32_t lo = 0, hi = k;                  // #{B < ia}
            while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (bi[mid] < ia) lo = mid + 1; else hi = mid; }
            const uint32_t pa = lo;
            lo = 0; hi = k;                           // #{A <= ib}
            while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (ai[mid] <= ib) lo = mid + 1; else hi = mid; }
            const uint32_t pb = lo;
            float sum = __uint_as_float(av[x]);
            if (pa < k && bi[pa] == ia) sum = sum + __uint_as_float(bv[pa]);     // one fp32 add
            mi[x + pa] = ia;
            mv[x + pa] = __float_as_uint(sum);
            const bool dup = pb > 0 && ai[pb - 1] == ib;
            mi[x + pb] = dup ? kTomb : ib;
            mv[x + pb] = bv[x];
        }
        for (uint32_t i = t; i < pairs * words; i += kT) { selw[i] = 0u; tiew[i] = 0u; }
        if (t < pairs) { p_prefix[t] = 0u; p_rem[t] = k; }
        __syncthreads();
        // ---- the k-th largest key of every pair's union: radix passes ----------------
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = pass == 0 ? 23 : (pass == 1 ? 15 : (pass == 2 ? 7 : 0));
            const int bits = pass == 3 ? 7 : 8;
            for (uint32_t i = t; i < pairs * 256; i += kT) cnt[i] = 0u;
            __syncthreads();
            {
                const uint32_t pre = p_prefix[p];
                for (uint32_t i = l; i < n2; i += team) {
                    if (mi[i] == kTomb) continue;
                    const uint32_t key = mv[i] & kAbs;
                    if ((key >> (shift + bits)) == pre) atomicAdd(&cnt[p * 256 + ((key >> shift) & ((1u << bits) - 1u))], 1u);
                }
            }
            __syncthreads();
            // one wave per pair (pairs in turns) finds the digit at which the count from the
            // top reaches the pair's remaining rank
            for (uint32_t q = t / kWave; q < pairs; q += kT / kWave) {
                const uint32_t lane = lane_id();
                const uint32_t* c = cnt + q * 256;
                const uint32_t c0 = c[4 * lane], c1 = c[4 * lane + 1], c2 = c[4 * lane + 2], c3 = c[4 * lane + 3];
                const uint32_t mine = c0 + c1 + c2 + c3;
                // suffix sums over the lanes: above = counts in the lanes after this one
                uint32_t incl = mine;
#pragma unroll
                for (int d = 1; d < kWave; d <<= 1) {
                    const uint32_t o = __shfl_down(incl, d);
                    if (lane + d < (uint32_t)kWave) incl += o;
                }
                const uint32_t above = incl - mine;
                const uint32_t rem = p_rem[q];
                if (above < rem && above + mine >= rem) {          // exactly one lane owns the crossing
                    uint32_t run = above, dsel = 0, gt = 0;
                    const uint32_t cc[4] = {c0, c1, c2, c3};
#pragma unroll
                    for (int j = 3; j >= 0; --j) {
                        if (run < rem && run + cc[j] >= rem) { dsel = 4 * lane + j; gt = run; }
                        run += cc[j];
                    }
                    p_prefix[q] = (p_prefix[q] << bits) | dsel;
                    p_rem[q] = rem - gt;
                }
            }
            __syncthreads();
        }
        // now p_prefix[p] = T (all 31 bits), p_rem[p] = entries with key == T to take
        // ---- mark the selected slots ---------------------------------------------------
        // keys above T: selected; keys equal to T: marked in a second bitmap, of which one
        // thread per pair then takes the first p_rem bits (ties go by slot = index order)
        {
            const uint32_t T = p_prefix[p];
            for (uint32_t i = l; i < n2; i += team) {
                if (mi[i] == kTomb) continue;
                const uint32_t key = mv[i] & kAbs;
                if (key > T) atomicOr(&selw[p * words + (i >> 5)], 1u << (i & 31));
                else if (key == T) atomicOr(&tiew[p * words + (i >> 5)], 1u << (i & 31));
            }
        }
        __syncthreads();
        if (t < pairs) {
            uint32_t take = p_rem[t];
            for (uint32_t v = 0; v < words && take > 0; ++v) {
                uint32_t bits = tiew[t * words + v];
                const uint32_t have = (uint32_t)__popc(bits);
                if (have > take) {                    // keep the lowest `take` bits
                    uint32_t keep = 0;
                    for (uint32_t q = 0; q < take; ++q) { const uint32_t low = bits & (0u - bits); keep |= low; bits ^= low; }
                    bits = keep;
                    take = 0;
                } else {
                    take -= have;
                }
                selw[t * words + v] |= bits;
            }
        }
        __syncthreads();
        // ---- compact into set p of the next round --------------------------------------
        // (every read of the current sets is over: they are overwritten in place)
        for (uint32_t i = l; i < n2; i += team) {
            const uint32_t wd = selw[p * words + (i >> 5)];
            if ((wd >> (i & 31)) & 1u) {
                uint32_t pos = (uint32_t)__popc(wd & ((1u << (i & 31)) - 1u));
                for (uint32_t v = 0; v < (i >> 5); ++v) pos += (uint32_t)__popc(selw[p * words + v]);
                if (pos < k) {
                    a_idx[p * k + pos] = mi[i];
                    a_val[p * k + pos] = mv[i];
                }
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
        for (uint32_t e = t; e < total; e += kT) {
            const uint32_t w = e / k;
            const uint32_t i = loc_idx[e];
            const uint32_t vb = __float_as_uint(loc_val[e]);
            uint32_t lo = 0, hi = k;
            while (lo < hi) { const uint32_t mid = (lo + hi) >> 1; if (a_idx[mid] < i) lo = mid + 1; else hi = mid; }
            const bool in_g = lo < k && a_idx[lo] == i;
            if (in_g || vb == 0x80000000u) res[(int64_t)w * stride + i] = 0.0f;
        }
    }
}

}  // namespace gtopk
