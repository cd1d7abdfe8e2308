// gTop-k S-SGD data-parallel hot path for MI355X (gfx950, wave64).
//
// Pipeline of one iteration (paper: Algorithm 4; Definition 1; Algorithm 3; Eq. 3):
//
//   local select   sample histogram -> speculative threshold -> ONE streaming pass
//                  (acc = residual + grad, written back; entries at or above the
//                  speculative threshold are compacted into a short candidate list)
//                  -> exact radix select of the k-th key among the candidates
//                  -> index-ordered emit of the k selected entries (+ zeroing).
//                  The speculative threshold only decides how much work the exact
//                  part has; if it was too high or too low for a worker, that
//                  worker's exact part reads its dense row instead (same kernels).
//   tree           per round: index-ordered union of the two k-sets of each pair
//                  (values at shared indices added) -> the same exact radix select
//                  -> ordered emit; the last round divides by P.
//   restore        membership test of each local entry in the global index set,
//                  add back on a miss.
//
// Nothing here is a dense contraction, so there is no MFMA; the streaming pass is
// bound by HBM bandwidth and everything after it by launch latency.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gtopk.h"

namespace {

constexpr int kWave = 64;
constexpr int kBlock = 256;                 // threads per block in the streaming kernels
constexpr int kIters = 8;                   // float4 loads per lane in the streaming pass
constexpr int kWaveSpan = kIters * 4 * kWave;      // 2048 elements per wave
constexpr int kChunk = kWaveSpan * (kBlock / kWave);  // 8192 elements per block = one run
constexpr int kMergeRun = 256;              // merged-array slots per run
constexpr int kHistBins = 4096;             // 12-bit digits (the last pass uses 128 of them)
constexpr int kSampleBits = 14;             // sample histogram: exponent + 6 mantissa bits
constexpr int kSampleBins = 1 << kSampleBits;
constexpr int kSampleShift = 31 - kSampleBits;
constexpr int kSampleTile = 256;            // contiguous elements per sample tile
constexpr uint32_t kTomb = 0xFFFFFFFFu;     // index of a merged slot that holds nothing
constexpr uint32_t kAbs = 0x7FFFFFFFu;

// digit of a 31-bit key in select pass p: bits 30..19, 18..7, 6..0
__device__ __forceinline__ int pass_shift(int p) { return p == 0 ? 19 : (p == 1 ? 7 : 0); }
__device__ __forceinline__ int pass_bits(int p) { return p == 2 ? 7 : 12; }

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & (kWave - 1); }

// number of set bits of `mask` below the calling lane
__device__ __forceinline__ uint32_t rank_in(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// ---------------------------------------------------------------------------------
// small utilities
// ---------------------------------------------------------------------------------

typedef float floatx4 __attribute__((ext_vector_type(4)));

// clears up to three arrays in one launch (an array with n == 0 is skipped)
__global__ void k_zero_u32(uint32_t* p0, size_t n0, uint32_t* p1, size_t n1, uint32_t* p2, size_t n2) {
    const size_t step = (size_t)gridDim.x * blockDim.x;
    const size_t first = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (size_t i = first; i < n0; i += step) p0[i] = 0u;
    for (size_t i = first; i < n1; i += step) p1[i] = 0u;
    for (size_t i = first; i < n2; i += step) p2[i] = 0u;
}

// Largest digit d with sum_{b >= d} h[b] >= target, and above = sum_{b > d} h[b].
// All threads of the block call it; blockDim.x divides nbins and nbins / blockDim.x <= 16.
// Results land in s_out[0] (digit) and s_out[1] (above), valid after the call for all
// threads.  If the whole histogram holds fewer than `target` entries, digit = 0 and
// above = total - h[0] are NOT guaranteed; s_out[2] is 1 only when a digit was found.
__device__ void suffix_pick(const uint32_t* h, int nbins, uint32_t target,
                            uint32_t* s_tsum, uint32_t* s_out) {
    const int t = threadIdx.x;
    const int per = nbins / blockDim.x;
    uint32_t loc[16];
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        loc[j] = (j < per) ? h[t * per + j] : 0u;
        mine += loc[j];
    }
    s_tsum[t] = mine;
    if (t == 0) { s_out[0] = 0; s_out[1] = 0; s_out[2] = 0; }
    __syncthreads();
    uint32_t above = 0;
    for (int u = t + 1; u < (int)blockDim.x; ++u) above += s_tsum[u];
    if (above < target && above + mine >= target) {      // exactly one thread owns the crossing
        uint32_t run = above;
#pragma unroll
        for (int j = 15; j >= 0; --j) {
            if (j < per) {
                uint32_t c = loc[j];
                if (run < target && run + c >= target) {
                    s_out[0] = (uint32_t)(t * per + j);
                    s_out[1] = run;
                    s_out[2] = 1;
                }
                run += c;
            }
        }
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------
// local select, part 1: sampled histogram of |residual + grad| -> speculative threshold
// ---------------------------------------------------------------------------------

// Sample tile t of a row covers [t*tile_stride, t*tile_stride + 256) (clipped to m).
__global__ __launch_bounds__(kBlock) void k_sample_hist(
        const float* __restrict__ grad, const float* __restrict__ res, uint32_t m, int64_t stride,
        uint32_t tile_stride, uint32_t n_tiles, uint32_t* __restrict__ samp_hist) {
    __shared__ uint32_t h[kSampleBins];
    const int w = blockIdx.y;
    for (int b = threadIdx.x; b < kSampleBins; b += kBlock) h[b] = 0u;
    __syncthreads();
    const float* g = grad + (int64_t)w * stride;
    const float* r = res + (int64_t)w * stride;
    for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        uint64_t q = (uint64_t)t * tile_stride + threadIdx.x;
        if (q < m) {
            float a = r[q] + g[q];
            uint32_t key = __float_as_uint(a) & kAbs;
            atomicAdd(&h[key >> kSampleShift], 1u);
        }
    }
    __syncthreads();
    uint32_t* out = samp_hist + (size_t)w * kSampleBins;
    for (int b = threadIdx.x; b < kSampleBins; b += kBlock) {
        uint32_t c = h[b];
        if (c) atomicAdd(&out[b], c);
    }
}

// One block of 1024 threads per worker: the lower edge of the bucket at which the
// sample's suffix count reaches `target` becomes the worker's speculative threshold.
__global__ __launch_bounds__(1024) void k_sample_pick(const uint32_t* __restrict__ samp_hist,
                                                      uint32_t target, uint32_t* __restrict__ tspec) {
    __shared__ uint32_t s_tsum[1024];
    __shared__ uint32_t s_out[3];
    const int w = blockIdx.x;
    suffix_pick(samp_hist + (size_t)w * kSampleBins, kSampleBins, target, s_tsum, s_out);
    if (threadIdx.x == 0) tspec[w] = s_out[2] ? (s_out[0] << kSampleShift) : 0u;
}

// ---------------------------------------------------------------------------------
// local select, part 2: the streaming pass
// ---------------------------------------------------------------------------------

// Block (chunk, w) handles elements [chunk*8192, +8192) of worker w; each wave a
// contiguous 2048 of them, 8 float4 per lane, all held in registers.  Phase 1
// loads, adds, stores and counts the entries whose key reaches the speculative
// threshold; one atomicAdd per block reserves a contiguous range of the worker's
// candidate list; phase 2 writes the block's candidates there in index order.
// run_table[w][chunk] = (first slot, count) lets later kernels walk the list in
// index order although blocks reserve in any order.
template <bool ALIGNED>
__global__ __launch_bounds__(kBlock) void k_accum_filter(
        const float* __restrict__ grad, float* __restrict__ res, uint32_t m, int64_t stride,
        const uint32_t* __restrict__ tspec, uint32_t* __restrict__ cand_idx,
        float* __restrict__ cand_val, uint32_t cap, uint32_t* __restrict__ cand_count,
        uint2* __restrict__ run_table, uint32_t nchunks) {
    __shared__ uint32_t s_cnt[kBlock / kWave];
    __shared__ uint32_t s_base;
    const int w = blockIdx.y;
    const uint32_t chunk = blockIdx.x;
    const uint32_t lane = lane_id();
    const uint32_t wave = threadIdx.x / kWave;
    const float* g = grad + (int64_t)w * stride;
    float* r = res + (int64_t)w * stride;
    const uint32_t ts = tspec[w];
    const uint32_t wbase = chunk * (uint32_t)kChunk + wave * (uint32_t)kWaveSpan;  // <= m + 8191 < 2^32

    float a[kIters][4];
    const bool whole = ALIGNED && (wbase + (uint32_t)kWaveSpan <= m);   // wave-uniform
    if (whole) {
        floatx4 gv[kIters], rv[kIters];
#pragma unroll
        for (int i = 0; i < kIters; ++i) {
            const uint32_t q = wbase + i * 256 + lane * 4;
            gv[i] = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(g + q));
            rv[i] = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(r + q));
        }
#pragma unroll
        for (int i = 0; i < kIters; ++i) {
            const uint32_t q = wbase + i * 256 + lane * 4;
            const floatx4 s = rv[i] + gv[i];          // four independent fp32 adds
            *reinterpret_cast<floatx4*>(r + q) = s;
            a[i][0] = s.x; a[i][1] = s.y; a[i][2] = s.z; a[i][3] = s.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < kIters; ++i) {
            const uint32_t q = wbase + i * 256 + lane * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float s = 0.0f;
                if (q + e < m) {
                    s = r[q + e] + g[q + e];
                    r[q + e] = s;
                }
                a[i][e] = s;
            }
        }
    }

    uint32_t cnt = 0;   // wave-uniform
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
        const uint32_t q = wbase + i * 256 + lane * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool c = (q + e < m) && ((__float_as_uint(a[i][e]) & kAbs) >= ts);
            cnt += (uint32_t)__popcll(__ballot(c));
        }
    }
    if (lane == 0) s_cnt[wave] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t total = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
        uint32_t base = 0;
        if (total) base = atomicAdd(&cand_count[w], total);
        run_table[(size_t)w * nchunks + chunk] = make_uint2(base, total);
        s_base = base;
    }
    __syncthreads();
    if (cnt == 0) return;
    uint32_t off = s_base;
    for (uint32_t v = 0; v < wave; ++v) off += s_cnt[v];
    uint32_t* ci = cand_idx + (size_t)w * cap;
    float* cv = cand_val + (size_t)w * cap;
#pragma unroll
    for (int i = 0; i < kIters; ++i) {
        const uint32_t q = wbase + i * 256 + lane * 4;
        bool c[4];
        uint64_t b[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            c[e] = (q + e < m) && ((__float_as_uint(a[i][e]) & kAbs) >= ts);
            b[e] = __ballot(c[e]);
        }
        if ((b[0] | b[1] | b[2] | b[3]) == 0) continue;
        uint32_t pos = off + rank_in(b[0]) + rank_in(b[1]) + rank_in(b[2]) + rank_in(b[3]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (c[e]) {
                if (pos < cap) { ci[pos] = q + e; cv[pos] = a[i][e]; }
                ++pos;
            }
        }
        off += (uint32_t)(__popcll(b[0]) + __popcll(b[1]) + __popcll(b[2]) + __popcll(b[3]));
    }
}

// ---------------------------------------------------------------------------------
// item sources for the exact select (histogram passes, count, ordered emit)
// ---------------------------------------------------------------------------------
// A source presents, per set s, a flat array of nphys(s) slots (for histograms) and
// the same slots grouped into runs listed in index order (for the ordered emit).

// Local select: the candidate list of worker s, or - when the speculative threshold
// left fewer than k candidates or more than the list holds - the worker's dense row.
struct CandSrc {
    const float* res;
    int64_t stride;
    uint32_t m, k, cap, nchunks;
    const uint32_t* cand_idx;
    const float* cand_val;
    const uint32_t* cand_count;
    const uint2* run_table;

    __device__ bool dense(int s) const {
        const uint32_t c = cand_count[s];
        return c < k || c > cap;
    }
    __device__ uint32_t nphys(int s, bool dn) const { return dn ? m : cand_count[s]; }
    __device__ bool fetch(int s, bool dn, uint32_t p, uint32_t& idx, uint32_t& bits) const {
        if (dn) {
            idx = p;
            bits = __float_as_uint(res[(int64_t)s * stride + p]);
        } else {
            idx = cand_idx[(size_t)s * cap + p];
            bits = __float_as_uint(cand_val[(size_t)s * cap + p]);
        }
        return true;
    }
    __device__ uint32_t nruns(int, bool) const { return nchunks; }
    __device__ uint2 run(int s, bool dn, uint32_t r) const {
        if (dn) {
            const uint32_t base = r * (uint32_t)kChunk;
            const uint32_t left = m - base;
            return make_uint2(base, left < (uint32_t)kChunk ? left : (uint32_t)kChunk);
        }
        return run_table[(size_t)s * nchunks + r];
    }
};

// Merge: 2k slots per pair, index-ascending, a slot with index kTomb holds nothing.
struct MergedSrc {
    const uint32_t* idx;
    const float* val;
    uint32_t n;       // 2k
    __device__ bool dense(int) const { return false; }
    __device__ uint32_t nphys(int, bool) const { return n; }
    __device__ bool fetch(int s, bool, uint32_t p, uint32_t& i, uint32_t& bits) const {
        i = idx[(size_t)s * n + p];
        bits = __float_as_uint(val[(size_t)s * n + p]);
        return i != kTomb;
    }
    __device__ uint32_t nruns(int, bool) const { return (n + kMergeRun - 1) / kMergeRun; }
    __device__ uint2 run(int, bool, uint32_t r) const {
        const uint32_t base = r * (uint32_t)kMergeRun;
        const uint32_t left = n - base;
        return make_uint2(base, left < (uint32_t)kMergeRun ? left : (uint32_t)kMergeRun);
    }
};

// ---------------------------------------------------------------------------------
// exact select: three digit passes (12 + 12 + 7 bits of the 31-bit key)
// ---------------------------------------------------------------------------------

template <class Src>
__global__ __launch_bounds__(kBlock) void k_hist(Src src, int pass, uint32_t* __restrict__ hist,
                                                 const uint32_t* __restrict__ st_prefix) {
    __shared__ uint32_t h[kHistBins];
    const int s = blockIdx.y;
    const int shift = pass_shift(pass), bits = pass_bits(pass);
    const int nbins = 1 << bits;
    for (int b = threadIdx.x; b < nbins; b += kBlock) h[b] = 0u;
    __syncthreads();
    const bool dn = src.dense(s);
    const uint32_t n = src.nphys(s, dn);
    const uint32_t prefix = pass == 0 ? 0u : st_prefix[s];
    const uint32_t step = gridDim.x * kBlock;
    for (uint64_t p = (uint64_t)blockIdx.x * kBlock + threadIdx.x; p < n; p += step) {
        uint32_t idx, vb;
        if (src.fetch(s, dn, (uint32_t)p, idx, vb)) {
            const uint32_t key = vb & kAbs;
            // (key >> 31) is 0, so pass 0 matches the empty prefix
            if ((key >> (shift + bits)) == prefix) atomicAdd(&h[(key >> shift) & (nbins - 1)], 1u);
        }
    }
    __syncthreads();
    uint32_t* out = hist + (size_t)s * kHistBins;
    for (int b = threadIdx.x; b < nbins; b += kBlock) {
        const uint32_t c = h[b];
        if (c) atomicAdd(&out[b], c);
    }
}

// One block per set: pick the digit of this pass, extend the prefix, clear the histogram.
// After pass 2, st_prefix[s] is the k-th largest key T and st_krem[s] the number of
// entries with key == T to take (>= 1); k - st_krem[s] entries have key > T.
__global__ void k_pick(uint32_t* __restrict__ hist, int pass, uint32_t k,
                       uint32_t* __restrict__ st_prefix, uint32_t* __restrict__ st_krem) {
    __shared__ uint32_t s_tsum[kBlock];
    __shared__ uint32_t s_out[3];
    const int s = blockIdx.x;
    const int bits = pass_bits(pass);
    const int nbins = 1 << bits;
    uint32_t* h = hist + (size_t)s * kHistBins;
    const uint32_t target = pass == 0 ? k : st_krem[s];
    const uint32_t prefix = pass == 0 ? 0u : st_prefix[s];
    suffix_pick(h, nbins, target, s_tsum, s_out);
    const int per = nbins / blockDim.x;
    for (int j = 0; j < per; ++j) h[threadIdx.x * per + j] = 0u;
    if (threadIdx.x == 0) {
        st_prefix[s] = (prefix << bits) | s_out[0];
        st_krem[s] = target - s_out[1];
    }
}

// ---------------------------------------------------------------------------------
// ordered emit: per-run counts -> exclusive scan over runs -> write
// ---------------------------------------------------------------------------------

// One wave per run.
template <class Src>
__global__ __launch_bounds__(kBlock) void k_count(Src src, const uint32_t* __restrict__ st_T,
                                                  uint32_t* __restrict__ run_gt,
                                                  uint32_t* __restrict__ run_eq, uint32_t maxruns) {
    const int s = blockIdx.y;
    const uint32_t r = blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    const bool dn = src.dense(s);
    if (r >= src.nruns(s, dn)) return;
    const uint2 rn = src.run(s, dn, r);
    const uint32_t T = st_T[s];
    const uint32_t lane = lane_id();
    uint32_t gt = 0, eq = 0;
    for (uint32_t j0 = 0; j0 < rn.y; j0 += kWave) {
        const uint32_t j = j0 + lane;
        bool is_gt = false, is_eq = false;
        if (j < rn.y) {
            uint32_t idx, vb;
            if (src.fetch(s, dn, rn.x + j, idx, vb)) {
                const uint32_t key = vb & kAbs;
                is_gt = key > T;
                is_eq = key == T;
            }
        }
        gt += (uint32_t)__popcll(__ballot(is_gt));
        eq += (uint32_t)__popcll(__ballot(is_eq));
    }
    if (lane == 0) {
        run_gt[(size_t)s * maxruns + r] = gt;
        run_eq[(size_t)s * maxruns + r] = eq;
    }
}

// One block of 1024 threads per set: exclusive scans of run_gt and run_eq over the runs.
template <class Src>
__global__ __launch_bounds__(1024) void k_scan_runs(Src src, const uint32_t* __restrict__ run_gt,
                                                    const uint32_t* __restrict__ run_eq,
                                                    uint32_t* __restrict__ off_gt,
                                                    uint32_t* __restrict__ off_eq, uint32_t maxruns) {
    __shared__ uint32_t s_g[1024];
    __shared__ uint32_t s_e[1024];
    __shared__ uint32_t s_carry[2];
    const int s = blockIdx.x;
    const uint32_t n = src.nruns(s, src.dense(s));
    const int t = threadIdx.x;
    if (t == 0) { s_carry[0] = 0; s_carry[1] = 0; }
    __syncthreads();
    for (uint32_t base = 0; base < n; base += 1024) {
        const uint32_t r = base + t;
        const uint32_t g = r < n ? run_gt[(size_t)s * maxruns + r] : 0u;
        const uint32_t e = r < n ? run_eq[(size_t)s * maxruns + r] : 0u;
        s_g[t] = g;
        s_e[t] = e;
        __syncthreads();
        // Hillis-Steele inclusive scan over 1024 entries
        for (int d = 1; d < 1024; d <<= 1) {
            uint32_t ag = 0, ae = 0;
            if (t >= d) { ag = s_g[t - d]; ae = s_e[t - d]; }
            __syncthreads();
            s_g[t] += ag;
            s_e[t] += ae;
            __syncthreads();
        }
        const uint32_t cg = s_carry[0], ce = s_carry[1];
        if (r < n) {
            off_gt[(size_t)s * maxruns + r] = cg + s_g[t] - g;
            off_eq[(size_t)s * maxruns + r] = ce + s_e[t] - e;
        }
        __syncthreads();
        if (t == 1023) { s_carry[0] = cg + s_g[t]; s_carry[1] = ce + s_e[t]; }
        __syncthreads();
    }
}

// One wave per run.  An entry is selected if key > T, or key == T and fewer than
// `need` equal-key entries precede it in index order.  Its output slot is the
// number of selected entries before it.  ZERO: also store +0.0 at its index in
// the set's dense row (Algorithm 4 line 8).  DIVIDE: value / divisor (Eq. 3).
template <class Src, bool ZERO, bool DIVIDE>
__global__ __launch_bounds__(kBlock) void k_emit(
        Src src, const uint32_t* __restrict__ st_T, const uint32_t* __restrict__ st_need,
        const uint32_t* __restrict__ off_gt, const uint32_t* __restrict__ off_eq, uint32_t maxruns,
        uint32_t k, uint32_t* __restrict__ out_idx, float* __restrict__ out_val, int64_t out_stride,
        float* __restrict__ row, int64_t row_stride, float divisor) {
    const int s = blockIdx.y;
    const uint32_t r = blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    const bool dn = src.dense(s);
    if (r >= src.nruns(s, dn)) return;
    const uint2 rn = src.run(s, dn, r);
    const uint32_t T = st_T[s], need = st_need[s];
    const uint32_t lane = lane_id();
    uint32_t eq_before = off_eq[(size_t)s * maxruns + r];
    uint32_t outp = off_gt[(size_t)s * maxruns + r] + (eq_before < need ? eq_before : need);
    for (uint32_t j0 = 0; j0 < rn.y; j0 += kWave) {
        const uint32_t j = j0 + lane;
        bool is_gt = false, is_eq = false;
        uint32_t idx = 0, vb = 0;
        if (j < rn.y) {
            if (src.fetch(s, dn, rn.x + j, idx, vb)) {
                const uint32_t key = vb & kAbs;
                is_gt = key > T;
                is_eq = key == T;
            }
        }
        const uint64_t eqm = __ballot(is_eq);
        const bool sel = is_gt || (is_eq && (eq_before + rank_in(eqm) < need));
        const uint64_t selm = __ballot(sel);
        if (sel) {
            const uint32_t pos = outp + rank_in(selm);
            if (pos < k) {      // always true when the select state is consistent
                out_idx[(int64_t)s * out_stride + pos] = idx;
                float v = __uint_as_float(vb);
                if (DIVIDE) v = v / divisor;
                out_val[(int64_t)s * out_stride + pos] = v;
            }
            if (ZERO) row[(int64_t)s * row_stride + idx] = 0.0f;
        }
        outp += (uint32_t)__popcll(selm);
        eq_before += (uint32_t)__popcll(eqm);
    }
}

// ---------------------------------------------------------------------------------
// merge: index-ordered union of two k-sets into 2k slots
// ---------------------------------------------------------------------------------

// first position p in [0, n) with a[p] >= x (n if none)
__device__ __forceinline__ uint32_t lower_bound(const uint32_t* a, uint32_t n, uint32_t x) {
    uint32_t lo = 0, hi = n;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}
// first position p in [0, n) with a[p] > x (n if none)
__device__ __forceinline__ uint32_t upper_bound(const uint32_t* a, uint32_t n, uint32_t x) {
    uint32_t lo = 0, hi = n;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (a[mid] <= x) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Entry x of A goes to slot x + #{B < A[x]}, entry y of B to slot y + #{A <= B[y]}:
// a bijection onto [0, 2k) that lists the union in index order, A's copy first
// where both hold an index.  A's copy then carries the sum (one fp32 add) and B's
// slot becomes a tombstone.
__global__ __launch_bounds__(kBlock) void k_union(
        const uint32_t* __restrict__ a_idx, const float* __restrict__ a_val,
        const uint32_t* __restrict__ b_idx, const float* __restrict__ b_val, uint32_t k,
        int64_t in_stride, uint32_t* __restrict__ m_idx, float* __restrict__ m_val) {
    const int s = blockIdx.y;
    const uint32_t x = blockIdx.x * kBlock + threadIdx.x;
    if (x >= k) return;
    const uint32_t* ai = a_idx + (int64_t)s * in_stride;
    const float* av = a_val + (int64_t)s * in_stride;
    const uint32_t* bi = b_idx + (int64_t)s * in_stride;
    const float* bv = b_val + (int64_t)s * in_stride;
    uint32_t* mi = m_idx + (size_t)s * 2 * k;
    float* mv = m_val + (size_t)s * 2 * k;
    {
        const uint32_t i = ai[x];
        const uint32_t p = lower_bound(bi, k, i);
        float v = av[x];
        if (p < k && bi[p] == i) v = v + bv[p];
        mi[x + p] = i;
        mv[x + p] = v;
    }
    {
        const uint32_t i = bi[x];
        const uint32_t p = upper_bound(ai, k, i);
        const bool dup = p > 0 && ai[p - 1] == i;
        mi[x + p] = dup ? kTomb : i;
        mv[x + p] = bv[x];
    }
}

// P == 1: the tree has no round; the global set is worker 0's set divided by 1.
__global__ void k_copy_set(const uint32_t* __restrict__ in_idx, const float* __restrict__ in_val,
                           uint32_t k, uint32_t* __restrict__ out_idx, float* __restrict__ out_val,
                           float divisor) {
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < k) {
        out_idx[t] = in_idx[t];
        out_val[t] = in_val[t] / divisor;
    }
}

// ---------------------------------------------------------------------------------
// residual restore (Algorithm 4 line 10)
// ---------------------------------------------------------------------------------

__global__ __launch_bounds__(kBlock) void k_restore(
        float* __restrict__ res, int64_t stride, uint32_t k, const uint32_t* __restrict__ loc_idx,
        const float* __restrict__ loc_val, const uint32_t* __restrict__ g_idx) {
    const int w = blockIdx.y;
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    if (t >= k) return;
    const uint32_t i = loc_idx[(size_t)w * k + t];
    const uint32_t p = lower_bound(g_idx, k, i);
    if (p < k && g_idx[p] == i) return;          // index is in the global set: stays zero
    float* slot = res + (int64_t)w * stride + i;
    *slot = *slot + loc_val[(size_t)w * k + t];
}

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------

inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }
inline uint32_t ceil_div(uint64_t a, uint64_t b) { return (uint32_t)((a + b - 1) / b); }
inline bool is_pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

struct SelectWs {          // scratch of the exact select, for up to `sets` sets
    uint32_t* hist;        // [sets][4096]
    uint32_t* st_prefix;   // [sets]  -> T after the third pass
    uint32_t* st_krem;     // [sets]  -> number of key == T entries to take
    uint32_t* run_gt;      // [sets][maxruns]
    uint32_t* run_eq;
    uint32_t* off_gt;
    uint32_t* off_eq;
    uint32_t maxruns;
};

struct Carver {
    char* base;
    size_t off = 0;
    template <class T> T* take(size_t n) {
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off = align_up(off + n * sizeof(T));
        return p;
    }
};

SelectWs carve_select(Carver& c, size_t sets, uint32_t maxruns) {
    SelectWs s;
    s.hist = c.take<uint32_t>(sets * kHistBins);
    s.st_prefix = c.take<uint32_t>(sets);
    s.st_krem = c.take<uint32_t>(sets);
    s.run_gt = c.take<uint32_t>(sets * maxruns);
    s.run_eq = c.take<uint32_t>(sets * maxruns);
    s.off_gt = c.take<uint32_t>(sets * maxruns);
    s.off_eq = c.take<uint32_t>(sets * maxruns);
    s.maxruns = maxruns;
    return s;
}

struct MergeWs {
    SelectWs sel;
    uint32_t* m_idx;   // [pairs][2k]
    float* m_val;
    size_t bytes;
};

MergeWs carve_merge(Carver& c, uint32_t k, size_t pairs) {
    MergeWs w;
    w.sel = carve_select(c, pairs, ceil_div(2ull * k, kMergeRun));
    w.m_idx = c.take<uint32_t>(pairs * 2 * k);
    w.m_val = c.take<float>(pairs * 2 * k);
    w.bytes = c.off;
    return w;
}

struct StepWs {
    // local select
    uint32_t* samp_hist;   // [P][16384]
    uint32_t* cand_count;  // [P]      (kept right behind samp_hist: one clear covers both)
    uint32_t* tspec;       // [P]
    uint32_t* cand_idx;    // [P][cap]
    float* cand_val;
    uint2* run_table;      // [P][nchunks]
    SelectWs sel;          // [P] sets, maxruns = nchunks
    uint32_t cap, nchunks;
    // tree
    MergeWs mrg;           // P/2 pairs
    uint32_t* x_idx;       // [P/2][k] ping
    float* x_val;
    uint32_t* y_idx;       // [P/4][k] pong
    float* y_val;
    // step
    uint32_t* loc_idx;     // [P][k] when the caller does not want them
    float* loc_val;
    size_t bytes;
};

uint32_t cand_capacity(int64_t m, uint32_t k) {
    uint64_t cap = 3ull * k + 8192;
    if (cap > (uint64_t)m) cap = (uint64_t)m;
    return (uint32_t)cap;
}

StepWs carve_step(void* ws, int64_t m, uint32_t k, uint32_t P) {
    Carver c{reinterpret_cast<char*>(ws)};
    StepWs s;
    s.cap = cand_capacity(m, k);
    s.nchunks = ceil_div((uint64_t)m, kChunk);
    s.samp_hist = c.take<uint32_t>((size_t)P * kSampleBins);
    s.cand_count = c.take<uint32_t>(P);
    s.tspec = c.take<uint32_t>(P);
    s.cand_idx = c.take<uint32_t>((size_t)P * s.cap);
    s.cand_val = c.take<float>((size_t)P * s.cap);
    s.run_table = c.take<uint2>((size_t)P * s.nchunks);
    s.sel = carve_select(c, P, s.nchunks);
    const size_t pairs = P > 1 ? P / 2 : 1;
    s.mrg = carve_merge(c, k, pairs);
    s.x_idx = c.take<uint32_t>(pairs * k);
    s.x_val = c.take<float>(pairs * k);
    const size_t quarter = P > 3 ? P / 4 : 1;
    s.y_idx = c.take<uint32_t>(quarter * k);
    s.y_val = c.take<float>(quarter * k);
    s.loc_idx = c.take<uint32_t>((size_t)P * k);
    s.loc_val = c.take<float>((size_t)P * k);
    s.bytes = c.off;
    return s;
}

bool sizes_ok(int64_t m, int64_t k, int64_t P) {
    return m >= 1 && m <= ((int64_t)1 << 31) && k >= 1 && k <= m && is_pow2(P) && P <= 65535;
}

int launch_status() { return hipGetLastError() == hipSuccess ? GTOPK_OK : GTOPK_EHIP; }

void zero_async(hipStream_t st, uint32_t* p0, size_t n0, uint32_t* p1 = nullptr, size_t n1 = 0,
                uint32_t* p2 = nullptr, size_t n2 = 0) {
    size_t n = n0 > n1 ? n0 : n1;
    if (n2 > n) n = n2;
    uint32_t blocks = (uint32_t)((n + 1023) / 1024 > 1024 ? 1024 : (n + 1023) / 1024);
    hipLaunchKernelGGL(k_zero_u32, dim3(blocks ? blocks : 1), dim3(256), 0, st, p0, n0, p1, n1, p2, n2);
}

// exact select + ordered emit over `sets` sets of a source
template <class Src, bool ZERO, bool DIVIDE>
void run_select(const Src& src, const SelectWs& ws, uint32_t sets, uint32_t k, uint32_t hist_blocks,
                uint32_t* out_idx, float* out_val, int64_t out_stride, float* row,
                int64_t row_stride, float divisor, hipStream_t st) {
    for (int pass = 0; pass < 3; ++pass) {
        hipLaunchKernelGGL((k_hist<Src>), dim3(hist_blocks, sets), dim3(kBlock), 0, st, src, pass,
                           ws.hist, ws.st_prefix);
        const int nbins = pass == 2 ? 128 : kHistBins;
        hipLaunchKernelGGL(k_pick, dim3(sets), dim3(nbins < kBlock ? nbins : kBlock), 0, st, ws.hist,
                           pass, k, ws.st_prefix, ws.st_krem);
    }
    const uint32_t run_blocks = ceil_div(ws.maxruns, kBlock / kWave);
    hipLaunchKernelGGL((k_count<Src>), dim3(run_blocks, sets), dim3(kBlock), 0, st, src,
                       ws.st_prefix, ws.run_gt, ws.run_eq, ws.maxruns);
    hipLaunchKernelGGL((k_scan_runs<Src>), dim3(sets), dim3(1024), 0, st, src, ws.run_gt, ws.run_eq,
                       ws.off_gt, ws.off_eq, ws.maxruns);
    hipLaunchKernelGGL((k_emit<Src, ZERO, DIVIDE>), dim3(run_blocks, sets), dim3(kBlock), 0, st, src,
                       ws.st_prefix, ws.st_krem, ws.off_gt, ws.off_eq, ws.maxruns, k, out_idx,
                       out_val, out_stride, row, row_stride, divisor);
}

// Sample plan for the speculative threshold: tiles of 256 contiguous elements,
// evenly spaced, about kSampleMean / rho elements per worker (all of them if the row
// is short).  `target` is the rank in the sample whose bucket edge is taken: the
// expected sample rank of the k-th key plus 6.5 standard deviations, so that the
// candidate list holds at least k entries except with negligible probability.
struct SamplePlan { uint32_t tile_stride, n_tiles, target; };

SamplePlan plan_sample(int64_t m, uint32_t k) {
    const double kSampleMean = 448.0;
    SamplePlan p;
    double want = kSampleMean * (double)m / (double)k;
    if (want >= (double)m) {
        p.tile_stride = kSampleTile;
    } else {
        const uint64_t tiles = (uint64_t)(want / kSampleTile) + 1;
        uint64_t ts = ((uint64_t)m / tiles) & ~(uint64_t)3;
        p.tile_stride = (uint32_t)(ts < (uint64_t)kSampleTile ? kSampleTile : ts);
    }
    p.n_tiles = ceil_div((uint64_t)m, p.tile_stride);
    const uint64_t last = (uint64_t)m - (uint64_t)(p.n_tiles - 1) * p.tile_stride;
    const uint64_t sampled = (uint64_t)(p.n_tiles - 1) * kSampleTile +
                             (last < (uint64_t)kSampleTile ? last : (uint64_t)kSampleTile);
    if (sampled >= (uint64_t)m) {
        p.target = k;                        // the "sample" is the whole row: exact count
    } else {
        const double mean = (double)k * (double)sampled / (double)m;
        double t = mean + 6.5 * __builtin_sqrt(mean) + 2.0;
        if (t > (double)sampled) t = (double)sampled;
        p.target = (uint32_t)t;
        if (p.target < 1) p.target = 1;
    }
    return p;
}

int do_local_select(const float* grad, float* residual, int64_t m, int64_t stride, uint32_t P,
                    uint32_t k, uint32_t* out_idx, float* out_val, const StepWs& w, hipStream_t st) {
    // clear the sample histograms, the candidate counters and the select histograms
    zero_async(st, w.samp_hist, (size_t)P * kSampleBins, w.cand_count, P, w.sel.hist,
               (size_t)P * kHistBins);

    const SamplePlan sp = plan_sample(m, k);
    const uint32_t sblocks = sp.n_tiles < 64 ? sp.n_tiles : 64;
    hipLaunchKernelGGL(k_sample_hist, dim3(sblocks, P), dim3(kBlock), 0, st, grad, residual,
                       (uint32_t)m, stride, sp.tile_stride, sp.n_tiles, w.samp_hist);
    hipLaunchKernelGGL(k_sample_pick, dim3(P), dim3(1024), 0, st, w.samp_hist, sp.target, w.tspec);

    const bool vec = (stride % 4 == 0);
    if (vec)
        hipLaunchKernelGGL((k_accum_filter<true>), dim3(w.nchunks, P), dim3(kBlock), 0, st, grad,
                           residual, (uint32_t)m, stride, w.tspec, w.cand_idx, w.cand_val, w.cap,
                           w.cand_count, w.run_table, w.nchunks);
    else
        hipLaunchKernelGGL((k_accum_filter<false>), dim3(w.nchunks, P), dim3(kBlock), 0, st, grad,
                           residual, (uint32_t)m, stride, w.tspec, w.cand_idx, w.cand_val, w.cap,
                           w.cand_count, w.run_table, w.nchunks);

    CandSrc src{residual, stride, (uint32_t)m, k, w.cap, w.nchunks,
                w.cand_idx, w.cand_val, w.cand_count, w.run_table};
    uint32_t hb = ceil_div(w.cap, 2048);
    if (hb > 128) hb = 128;
    run_select<CandSrc, true, false>(src, w.sel, P, k, hb, out_idx, out_val, (int64_t)k, residual,
                                     stride, 1.0f, st);
    return launch_status();
}

// one batch of merges: union + exact select + ordered emit
template <bool DIVIDE>
void do_merge_batch(const uint32_t* a_idx, const float* a_val, const uint32_t* b_idx,
                    const float* b_val, uint32_t k, uint32_t batch, int64_t in_stride,
                    uint32_t* out_idx, float* out_val, int64_t out_stride, const MergeWs& w,
                    float divisor, hipStream_t st) {
    hipLaunchKernelGGL(k_union, dim3(ceil_div(k, kBlock), batch), dim3(kBlock), 0, st, a_idx, a_val,
                       b_idx, b_val, k, in_stride, w.m_idx, w.m_val);
    MergedSrc src{w.m_idx, w.m_val, 2 * k};
    uint32_t hb = ceil_div(2ull * k, 2048);
    if (hb > 128) hb = 128;
    run_select<MergedSrc, false, DIVIDE>(src, w.sel, batch, k, hb, out_idx, out_val, out_stride,
                                         nullptr, 0, divisor, st);
}

int do_tree(const uint32_t* loc_idx, const float* loc_val, uint32_t P, uint32_t k, uint32_t* g_idx,
            float* g_val, const StepWs& w, hipStream_t st) {
    const float divisor = (float)P;
    if (P == 1) {
        hipLaunchKernelGGL(k_copy_set, dim3(ceil_div(k, 256)), dim3(256), 0, st, loc_idx, loc_val, k,
                           g_idx, g_val, divisor);
        return launch_status();
    }
    zero_async(st, w.mrg.sel.hist, (size_t)(P / 2) * kHistBins);
    // After every round the surviving sets are stored compactly, so round j always
    // merges set 2p with set 2p+1 of its input: exactly worker p*2^(j+1) with worker
    // p*2^(j+1) + 2^j of the original numbering.
    const uint32_t* in_idx = loc_idx;
    const float* in_val = loc_val;
    uint32_t* ping_i = w.x_idx; float* ping_v = w.x_val;
    uint32_t* pong_i = w.y_idx; float* pong_v = w.y_val;
    for (uint32_t pairs = P / 2; pairs >= 1; pairs /= 2) {
        const bool last = pairs == 1;
        if (last) {
            do_merge_batch<true>(in_idx, in_val, in_idx + k, in_val + k, k, 1, 2 * (int64_t)k, g_idx,
                                 g_val, k, w.mrg, divisor, st);
        } else {
            do_merge_batch<false>(in_idx, in_val, in_idx + k, in_val + k, k, pairs, 2 * (int64_t)k,
                                  ping_i, ping_v, k, w.mrg, 1.0f, st);
            in_idx = ping_i; in_val = ping_v;
            uint32_t* ti = ping_i; ping_i = pong_i; pong_i = ti;
            float* tv = ping_v; ping_v = pong_v; pong_v = tv;
        }
    }
    return launch_status();
}

int do_restore(float* residual, int64_t stride, uint32_t P, uint32_t k, const uint32_t* loc_idx,
               const float* loc_val, const uint32_t* g_idx, hipStream_t st) {
    hipLaunchKernelGGL(k_restore, dim3(ceil_div(k, kBlock), P), dim3(kBlock), 0, st, residual, stride,
                       k, loc_idx, loc_val, g_idx);
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
    if (k < 1 || batch < 1 || batch > 65535) return 0;
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
                           (hipStream_t)stream);
}

int gtopk_merge(const uint32_t* a_idx, const float* a_val, const uint32_t* b_idx, const float* b_val,
                int32_t k, int32_t batch, int64_t in_stride, uint32_t* out_idx, float* out_val,
                int64_t out_stride, void* ws, size_t ws_bytes, void* stream) {
    if (!a_idx || !a_val || !b_idx || !b_val || !out_idx || !out_val || !ws) return GTOPK_EINVAL;
    if (k < 1 || batch < 1 || batch > 65535 || in_stride < k || out_stride < k) return GTOPK_EINVAL;
    if (!aligned16(a_idx) || !aligned16(a_val) || !aligned16(b_idx) || !aligned16(b_val) ||
        !aligned16(out_idx) || !aligned16(out_val) || !aligned16(ws))
        return GTOPK_EALIGN;
    Carver c{reinterpret_cast<char*>(ws)};
    const MergeWs w = carve_merge(c, (uint32_t)k, (size_t)batch);
    if (ws_bytes < w.bytes) return GTOPK_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    zero_async(st, w.sel.hist, (size_t)batch * kHistBins);
    do_merge_batch<false>(a_idx, a_val, b_idx, b_val, (uint32_t)k, (uint32_t)batch, in_stride,
                          out_idx, out_val, out_stride, w, 1.0f, st);
    return launch_status();
}

int gtopk_tree(const uint32_t* loc_idx, const float* loc_val, int32_t P, int32_t k, uint32_t* g_idx,
               float* g_val, void* ws, size_t ws_bytes, void* stream) {
    if (!loc_idx || !loc_val || !g_idx || !g_val || !ws) return GTOPK_EINVAL;
    if (k < 1 || !is_pow2(P) || P > 65535) return GTOPK_EINVAL;
    if (!aligned16(loc_idx) || !aligned16(loc_val) || !aligned16(g_idx) || !aligned16(g_val) ||
        !aligned16(ws))
        return GTOPK_EALIGN;
    // the tree's scratch sits inside the step workspace; m only sizes the parts it does not use
    const StepWs w = carve_step(ws, (int64_t)k, (uint32_t)k, (uint32_t)P);
    if (ws_bytes < w.bytes) return GTOPK_EWORKSPACE;
    return do_tree(loc_idx, loc_val, (uint32_t)P, (uint32_t)k, g_idx, g_val, w, (hipStream_t)stream);
}

int gtopk_residual_restore(float* residual, int64_t m, int64_t stride, int32_t P, int32_t k,
                           const uint32_t* loc_idx, const float* loc_val, const uint32_t* g_idx,
                           void* stream) {
    if (!residual || !loc_idx || !loc_val || !g_idx) return GTOPK_EINVAL;
    if (!sizes_ok(m, k, P) || stride < m) return GTOPK_EINVAL;
    if (!aligned16(residual) || !aligned16(loc_idx) || !aligned16(loc_val) || !aligned16(g_idx))
        return GTOPK_EALIGN;
    return do_restore(residual, stride, (uint32_t)P, (uint32_t)k, loc_idx, loc_val, g_idx,
                      (hipStream_t)stream);
}

int gtopk_step(const float* grad, float* residual, int64_t m, int64_t stride, int32_t P, int32_t k,
               uint32_t* g_idx, float* g_val, uint32_t* loc_idx, float* loc_val, void* ws,
               size_t ws_bytes, void* stream) {
    if (!grad || !residual || !g_idx || !g_val || !ws) return GTOPK_EINVAL;
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
    int rc = do_local_select(grad, residual, m, stride, (uint32_t)P, (uint32_t)k, li, lv, w, st);
    if (rc != GTOPK_OK) return rc;
    rc = do_tree(li, lv, (uint32_t)P, (uint32_t)k, g_idx, g_val, w, st);
    if (rc != GTOPK_OK) return rc;
    return do_restore(residual, stride, (uint32_t)P, (uint32_t)k, li, lv, g_idx, st);
}

}  // extern "C"
