// gTop-k S-SGD data-parallel hot path for MI355X (gfx950, wave64).
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
//                  -> ordered emit; the last round divides by P.
//   restore        membership test of each local entry in the global index set.
//
// Exact select of the k-th largest 31-bit key of a set, in four kernels:
//   hist    12-bit histogram of the top key bits
//   bucket  every block first picks, from that histogram, the bucket d1 that holds the
//           k-th key; then per group of items: count of keys above the bucket; keys
//           inside the bucket are appended (low 19 bits + group id) to a short list
//   finish  one block per set: two LDS radix passes over the list give the exact key
//           T and the number of ties to take; per-group counts are completed from the
//           list and scanned into output offsets
//   emit    per group: ordered compaction of the selected entries
//
// Nothing here is a dense contraction, so there is no MFMA; the streaming pass is
// bound by HBM bandwidth and everything after it by launch latency.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gtopk.h"

namespace {

constexpr int kWave = 64;
constexpr int kSBlock = 512;                // threads per block of the streaming pass
constexpr int kIters = 16;                  // float4 loads per lane and array in the streaming pass
constexpr int kWaveSpan = kIters * 4 * kWave;            // 4096 elements per wave
constexpr int kChunk = kWaveSpan * (kSBlock / kWave);    // 32768 elements per block = one run
constexpr int kBlock = 256;                 // threads per block of the select kernels
constexpr int kMaxSeg = 32;                 // runs per group, at most
constexpr int kMaxGroups = 2048;            // groups per set, at most (LDS arrays in k_finish)
constexpr int kHistBins = 4096;             // first digit: key bits 30..19
constexpr int kLowBits = 19;                // key bits below the first digit
constexpr uint32_t kLowMask = (1u << kLowBits) - 1;
constexpr int kSampleBits = 14;             // sample histogram: exponent + 6 mantissa bits
constexpr int kSampleBins = 1 << kSampleBits;
constexpr int kSampleShift = 31 - kSampleBits;
constexpr int kSampleTile = 256;            // contiguous elements per sample tile
constexpr int kSampleBlock = 1024;
constexpr uint32_t kTomb = 0xFFFFFFFFu;     // index of a merged slot that holds nothing
constexpr uint32_t kAbs = 0x7FFFFFFFu;

typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & (kWave - 1); }

// number of set bits of `mask` below the calling lane
__device__ __forceinline__ uint32_t rank_in(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// ---------------------------------------------------------------------------------
// block-wide primitives (every thread of the block must call them)
// ---------------------------------------------------------------------------------

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
    const uint32_t lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const uint32_t t = __shfl_up(v, d);
        if (lane >= (uint32_t)d) v += t;
    }
    return v;
}

// inclusive prefix sum over the block in thread order; s_wave: LDS, >= blockDim.x/64 words
__device__ uint32_t block_incl_scan(uint32_t v, uint32_t* s_wave, uint32_t& total) {
    const uint32_t wave = threadIdx.x / kWave;
    const uint32_t nw = blockDim.x / kWave;
    const uint32_t incl = wave_incl_scan(v);
    __syncthreads();                       // s_wave may still be read from an earlier call
    if (lane_id() == kWave - 1) s_wave[wave] = incl;
    __syncthreads();
    uint32_t base = 0, tot = 0;
    for (uint32_t i = 0; i < nw; ++i) {
        const uint32_t x = s_wave[i];
        if (i < wave) base += x;
        tot += x;
    }
    total = tot;
    return incl + base;
}

// Thread t owns the PER histogram bins [t*PER, (t+1)*PER), counts in loc[].  Finds the
// largest bin d with sum_{b >= d} >= target.  s_out[0] = d, s_out[1] = sum_{b > d},
// s_out[2] = 1 if such a bin exists (0 if the histogram holds fewer than target entries).
template <int PER>
__device__ void suffix_pick(const uint32_t (&loc)[PER], uint32_t target, uint32_t* s_wave,
                            uint32_t* s_out) {
    uint32_t mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) mine += loc[j];
    if (threadIdx.x == 0) { s_out[0] = 0; s_out[1] = 0; s_out[2] = 0; }
    uint32_t total;
    const uint32_t incl = block_incl_scan(mine, s_wave, total);
    const uint32_t above = total - incl;
    if (above < target && above + mine >= target) {       // exactly one thread owns the crossing
        uint32_t run = above;
#pragma unroll
        for (int j = PER - 1; j >= 0; --j) {
            const uint32_t c = loc[j];
            if (run < target && run + c >= target) {
                s_out[0] = (uint32_t)(threadIdx.x * PER + j);
                s_out[1] = run;
                s_out[2] = 1;
            }
            run += c;
        }
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------
// clearing
// ---------------------------------------------------------------------------------

struct ZeroJob { uint32_t* p[4]; size_t n[4]; };

// clears up to four arrays in one launch (an array with n == 0 is skipped)
__global__ void k_zero_u32(ZeroJob job) {
    const size_t step = (size_t)gridDim.x * blockDim.x;
    const size_t first = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
#pragma unroll
    for (int a = 0; a < 4; ++a)
        for (size_t i = first; i < job.n[a]; i += step) job.p[a][i] = 0u;
}

// ---------------------------------------------------------------------------------
// per-set state of the exact select
// ---------------------------------------------------------------------------------

struct SelState {
    uint32_t* hist;       // [sets][4096]   zero between uses
    uint32_t* list_cnt;   // [sets]         zero between uses
    uint32_t* d1;         // [sets] first digit of the k-th key
    uint32_t* krem;       // [sets] rank of the k-th key inside bucket d1 (1-based, from the top)
    uint32_t* T;          // [sets] the k-th largest key
    uint32_t* need;       // [sets] entries with key == T to take (>= 1)
    uint32_t* list;       // [sets][list_cap]  (low 19 key bits) | (group << 19)
    uint32_t* grp_gt;     // [sets][maxgroups] entries of the group above bucket d1
    uint32_t* off_gt;     // [sets][maxgroups] exclusive scans over groups
    uint32_t* off_eq;
    uint32_t list_cap, maxgroups;
};

// ---------------------------------------------------------------------------------
// local select, part 1: sampled histogram of |residual + grad| -> speculative threshold
// ---------------------------------------------------------------------------------

// Sample tile t of a row covers [t*tile_stride, t*tile_stride + 256) (clipped to m).  A
// block of 1024 threads takes four tiles per round.
__global__ __launch_bounds__(kSampleBlock) void k_sample(
        const float* __restrict__ grad, const float* __restrict__ res, uint32_t m, int64_t stride,
        uint32_t tile_stride, uint32_t n_tiles, uint32_t* __restrict__ samp_hist) {
    __shared__ uint32_t h[kSampleBins];
    const int w = blockIdx.y;
    for (int b = threadIdx.x; b < kSampleBins; b += kSampleBlock) h[b] = 0u;
    __syncthreads();
    const float* g = grad + (int64_t)w * stride;
    const float* r = res + (int64_t)w * stride;
    const uint32_t sub = threadIdx.x / kSampleTile, el = threadIdx.x % kSampleTile;
    constexpr int kUnroll = 8;
    const uint64_t tiles_per_round = (uint64_t)(kSampleBlock / kSampleTile) * gridDim.x;
    for (uint64_t t0 = (uint64_t)blockIdx.x * (kSampleBlock / kSampleTile) + sub; t0 < n_tiles;
         t0 += tiles_per_round * kUnroll) {
        float gv[kUnroll], rv[kUnroll];
        bool ok[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t t = t0 + (uint64_t)u * tiles_per_round;
            const uint64_t q = t * tile_stride + el;
            ok[u] = t < n_tiles && q < m;
            gv[u] = ok[u] ? g[q] : 0.0f;
            rv[u] = ok[u] ? r[q] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (ok[u]) {
                const uint32_t key = __float_as_uint(rv[u] + gv[u]) & kAbs;
                atomicAdd(&h[key >> kSampleShift], 1u);
            }
        }
    }
    __syncthreads();
    uint32_t* out = samp_hist + (size_t)w * kSampleBins;
    for (int b = threadIdx.x; b < kSampleBins; b += kSampleBlock) {
        const uint32_t c = h[b];
        if (c) atomicAdd(&out[b], c);
    }
}

// One block per worker turns the worker's sample histogram into the speculative
// threshold: the lower edge of the bucket at which the count from the top reaches
// `target`.
__global__ __launch_bounds__(kSampleBlock) void k_sample_pick(
        const uint32_t* __restrict__ samp_hist, uint32_t target, uint32_t* __restrict__ tspec) {
    __shared__ uint32_t s_wave[kSampleBlock / kWave];
    __shared__ uint32_t s_out[3];
    const int w = blockIdx.x;
    constexpr int kPer = kSampleBins / kSampleBlock;
    const uint32_t* hist = samp_hist + (size_t)w * kSampleBins;
    uint32_t loc[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) loc[j] = hist[threadIdx.x * kPer + j];
    suffix_pick<kPer>(loc, target, s_wave, s_out);
    if (threadIdx.x == 0) tspec[w] = s_out[2] ? (s_out[0] << kSampleShift) : 0u;
}

// ---------------------------------------------------------------------------------
// local select, part 2: the streaming pass
// ---------------------------------------------------------------------------------

// Block (chunk, w) handles elements [chunk*32768, +32768) of worker w; each of its 8
// waves a contiguous 4096 of them, 16 float4 per lane, all held in registers.  Phase 1
// loads, adds, stores and counts the entries whose key reaches the speculative
// threshold; one atomicAdd per block reserves a contiguous range of the worker's
// candidate list; phase 2 writes the block's candidates there in index order.
// run_table[w][chunk] = (first slot, count) lets later kernels walk the list in
// index order although blocks reserve in any order.
template <bool ALIGNED>
__global__ __launch_bounds__(kSBlock) void k_accum_filter(
        const float* __restrict__ grad, float* __restrict__ res, uint32_t m, int64_t stride,
        const uint32_t* __restrict__ tspec, uint32_t* __restrict__ cand_idx,
        float* __restrict__ cand_val, uint32_t cap, uint32_t* __restrict__ cand_count,
        uint2* __restrict__ run_table, uint32_t nchunks) {
    constexpr int kWaves = kSBlock / kWave;
    __shared__ uint32_t s_cnt[kWaves];
    __shared__ uint32_t s_base;
    const int w = blockIdx.y;
    const uint32_t chunk = blockIdx.x;
    const uint32_t lane = lane_id();
    const uint32_t wave = threadIdx.x / kWave;
    const float* g = grad + (int64_t)w * stride;
    float* r = res + (int64_t)w * stride;
    const uint32_t ts = tspec[w];
    // m <= 2^31 and chunk < ceil(m / 32768), so none of the offsets below wraps
    const uint32_t wbase = chunk * (uint32_t)kChunk + wave * (uint32_t)kWaveSpan;

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
            __builtin_nontemporal_store(s, reinterpret_cast<floatx4*>(r + q));
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
        uint32_t total = 0;
        for (int v = 0; v < kWaves; ++v) total += s_cnt[v];
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
// item sources for the exact select
// ---------------------------------------------------------------------------------
// A source presents, per set s, a flat array of nphys(s) slots (for the histogram) and
// the same slots as groups of segments; groups, and the segments inside a group, are
// listed in index order (for the ordered emit).

// Local select: the candidate list of worker s, or - when the speculative threshold
// left fewer than k candidates or more than the list holds - the worker's dense row.
struct CandSrc {
    const float* res;
    int64_t stride;
    uint32_t m, k, cap, nchunks, G;       // G runs per group
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
    __device__ uint32_t ngroups(int, bool) const { return (nchunks + G - 1) / G; }
    __device__ uint32_t nseg(int, bool, uint32_t g) const {
        const uint32_t left = nchunks - g * G;
        return left < G ? left : G;
    }
    __device__ uint2 segment(int s, bool dn, uint32_t g, uint32_t j) const {
        const uint32_t r = g * G + j;
        if (dn) {
            const uint32_t base = r * (uint32_t)kChunk;
            const uint32_t left = m - base;
            return make_uint2(base, left < (uint32_t)kChunk ? left : (uint32_t)kChunk);
        }
        return run_table[(size_t)s * nchunks + r];
    }
};

// Merge: n = 2k slots per pair, index-ascending, a slot with index kTomb holds nothing.
struct MergedSrc {
    const uint32_t* idx;
    const float* val;
    uint32_t n, L;       // L slots per group
    __device__ bool dense(int) const { return false; }
    __device__ uint32_t nphys(int, bool) const { return n; }
    __device__ bool fetch(int s, bool, uint32_t p, uint32_t& i, uint32_t& bits) const {
        i = idx[(size_t)s * n + p];
        bits = __float_as_uint(val[(size_t)s * n + p]);
        return i != kTomb;
    }
    __device__ uint32_t ngroups(int, bool) const { return (n + L - 1) / L; }
    __device__ uint32_t nseg(int, bool, uint32_t) const { return 1; }
    __device__ uint2 segment(int, bool, uint32_t g, uint32_t) const {
        const uint32_t base = g * L;
        const uint32_t left = n - base;
        return make_uint2(base, left < L ? left : L);
    }
};

// Segments of one group, in LDS; item i of the group is slot base[j] + i - start[j]
// of the segment j with start[j] <= i < start[j+1].
struct GroupSegs {
    uint32_t base[kMaxSeg];
    uint32_t start[kMaxSeg + 1];
    uint32_t n;
};

template <class Src>
__device__ uint32_t load_group(const Src& src, int s, bool dn, uint32_t g, GroupSegs* gs) {
    const uint32_t ns = src.nseg(s, dn, g);
    __syncthreads();                              // the previous group may still be in use
    if (threadIdx.x < ns) {
        const uint2 sg = src.segment(s, dn, g, threadIdx.x);
        gs->base[threadIdx.x] = sg.x;
        gs->start[threadIdx.x + 1] = sg.y;        // counts for now
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        gs->start[0] = 0;
        for (uint32_t j = 0; j < ns; ++j) {
            run += gs->start[j + 1];
            gs->start[j + 1] = run;
        }
        gs->n = ns;
    }
    __syncthreads();
    return gs->start[ns];
}

__device__ __forceinline__ uint32_t group_slot(const GroupSegs* gs, uint32_t i) {
    uint32_t j = 0;
    while (j + 1 < gs->n && i >= gs->start[j + 1]) ++j;
    return gs->base[j] + (i - gs->start[j]);
}

// ---------------------------------------------------------------------------------
// exact select, kernel 1: histogram of the first digit (key bits 30..19)
// ---------------------------------------------------------------------------------

constexpr int kHistBlock = 1024;

// adds the block's LDS histogram into the set's global one
__device__ void flush_hist(const uint32_t* h, uint32_t* out) {
    for (int b = threadIdx.x; b < kHistBins; b += blockDim.x) {
        const uint32_t c = h[b];
        if (c) atomicAdd(&out[b], c);
    }
}

// Few, large blocks per set: a popular bin receives one global atomic per block.
template <class Src>
__global__ __launch_bounds__(kHistBlock) void k_hist(Src src, SelState st) {
    __shared__ uint32_t h[kHistBins];
    const int s = blockIdx.y;
    for (int b = threadIdx.x; b < kHistBins; b += kHistBlock) h[b] = 0u;
    __syncthreads();
    const bool dn = src.dense(s);
    const uint32_t n = src.nphys(s, dn);
    const uint32_t step = gridDim.x * kHistBlock;
    for (uint64_t p = (uint64_t)blockIdx.x * kHistBlock + threadIdx.x; p < n; p += step) {
        uint32_t idx, vb;
        if (src.fetch(s, dn, (uint32_t)p, idx, vb)) atomicAdd(&h[(vb & kAbs) >> kLowBits], 1u);
    }
    __syncthreads();
    flush_hist(h, st.hist + (size_t)s * kHistBins);
}

// ---------------------------------------------------------------------------------
// exact select, kernel 2: per group, count keys above the bucket, list keys inside it
// ---------------------------------------------------------------------------------

template <class Src>
__global__ __launch_bounds__(kBlock) void k_bucket(Src src, SelState st, uint32_t k) {
    __shared__ GroupSegs gs;
    __shared__ uint32_t s_wave[kBlock / kWave];
    __shared__ uint32_t s_out[3];
    __shared__ uint32_t s_gt[kBlock / kWave];
    __shared__ uint32_t s_in[kBlock / kWave];
    __shared__ uint32_t s_base;
    const int s = blockIdx.y;
    const uint32_t g = blockIdx.x;
    const bool dn = src.dense(s);
    if (g >= src.ngroups(s, dn)) return;
    // every block picks the bucket of the k-th key from the set's histogram
    {
        constexpr int kPer = kHistBins / kBlock;      // thread t owns 16 consecutive bins
        const uint32_t* hist = st.hist + (size_t)s * kHistBins;
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
    const uint32_t total = load_group(src, s, dn, g, &gs);
    const uint32_t wave = threadIdx.x / kWave;
    uint32_t gt = 0, in = 0;     // wave-uniform
    for (uint32_t i0 = 0; i0 < total; i0 += kBlock) {
        const uint32_t i = i0 + threadIdx.x;
        bool above = false, inside = false;
        if (i < total) {
            uint32_t idx, vb;
            if (src.fetch(s, dn, group_slot(&gs, i), idx, vb)) {
                const uint32_t d = (vb & kAbs) >> kLowBits;
                above = d > d1;
                inside = d == d1;
            }
        }
        gt += (uint32_t)__popcll(__ballot(above));
        in += (uint32_t)__popcll(__ballot(inside));
    }
    if (lane_id() == 0) { s_gt[wave] = gt; s_in[wave] = in; }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t tg = 0, ti = 0;
        for (int v = 0; v < kBlock / kWave; ++v) { tg += s_gt[v]; ti += s_in[v]; }
        st.grp_gt[(size_t)s * st.maxgroups + g] = tg;
        s_base = ti ? atomicAdd(&st.list_cnt[s], ti) : 0u;     // one reservation per block
    }
    __syncthreads();
    if (in == 0) return;
    // second walk: this wave's bucket entries go to its slice of the block's reservation
    uint32_t off = s_base;
    for (uint32_t v = 0; v < wave; ++v) off += s_in[v];
    uint32_t* list = st.list + (size_t)s * st.list_cap;
    for (uint32_t i0 = 0; i0 < total; i0 += kBlock) {
        const uint32_t i = i0 + threadIdx.x;
        bool inside = false;
        uint32_t key = 0;
        if (i < total) {
            uint32_t idx, vb;
            if (src.fetch(s, dn, group_slot(&gs, i), idx, vb)) {
                key = vb & kAbs;
                inside = (key >> kLowBits) == d1;
            }
        }
        const uint64_t inm = __ballot(inside);
        if (inside) {
            const uint32_t pos = off + rank_in(inm);
            if (pos < st.list_cap) list[pos] = (key & kLowMask) | (g << kLowBits);
        }
        off += (uint32_t)__popcll(inm);
    }
}

// ---------------------------------------------------------------------------------
// exact select, kernel 3: one block per set finishes the key and scans the groups
// ---------------------------------------------------------------------------------

template <class Src>
__global__ __launch_bounds__(1024) void k_finish(Src src, SelState st) {
    constexpr int kT = 1024;
    __shared__ uint32_t h[kT];
    __shared__ uint32_t g_gt[kMaxGroups];
    __shared__ uint32_t g_eq[kMaxGroups];
    __shared__ uint32_t s_wave[kT / kWave];
    __shared__ uint32_t s_out[3];
    __shared__ GroupSegs gs;
    const int s = blockIdx.x;
    const uint32_t t = threadIdx.x;
    const bool dn = src.dense(s);
    const uint32_t ng = src.ngroups(s, dn);
    const uint32_t d1 = st.d1[s];
    uint32_t krem = st.krem[s];
    const uint32_t nlist = st.list_cnt[s];
    const bool overflow = nlist > st.list_cap;       // the list is incomplete: read the set itself
    const uint32_t* list = st.list + (size_t)s * st.list_cap;
    const uint32_t nphys = src.nphys(s, dn);

    // a short list is read once and kept in registers
    constexpr int kCache = 8;
    constexpr uint32_t kNone = 0xFFFFFFFFu;            // bit 31 is never set in a list entry
    const bool cached = !overflow && nlist <= (uint32_t)(kCache * kT);
    uint32_t ent[kCache];
#pragma unroll
    for (int j = 0; j < kCache; ++j) {
        const uint32_t i = t + (uint32_t)j * kT;
        ent[j] = (cached && i < nlist) ? list[i] : kNone;
    }
    auto for_each_entry = [&](auto&& f) {
        if (cached) {
#pragma unroll
            for (int j = 0; j < kCache; ++j)
                if (ent[j] != kNone) f(ent[j]);
        } else {
            for (uint32_t i = t; i < nlist; i += kT) f(list[i]);
        }
    };

    // two radix passes over the low 19 bits of the keys inside bucket d1: bits 18..9, 8..0
    uint32_t hi = 0;
    for (int pass = 0; pass < 2; ++pass) {
        h[t] = 0u;
        __syncthreads();
        if (!overflow) {
            for_each_entry([&](uint32_t e) {
                const uint32_t low = e & kLowMask;
                if (pass == 0) atomicAdd(&h[low >> 9], 1u);
                else if ((low >> 9) == hi) atomicAdd(&h[low & 511u], 1u);
            });
        } else {
            for (uint64_t p = t; p < nphys; p += kT) {
                uint32_t idx, vb;
                if (src.fetch(s, dn, (uint32_t)p, idx, vb)) {
                    const uint32_t key = vb & kAbs;
                    if ((key >> kLowBits) == d1) {
                        const uint32_t low = key & kLowMask;
                        if (pass == 0) atomicAdd(&h[low >> 9], 1u);
                        else if ((low >> 9) == hi) atomicAdd(&h[low & 511u], 1u);
                    }
                }
            }
        }
        __syncthreads();
        const uint32_t loc[1] = {h[t]};
        suffix_pick<1>(loc, krem, s_wave, s_out);
        if (pass == 0) hi = s_out[0];
        krem -= s_out[1];
    }
    const uint32_t tlow = (hi << 9) | s_out[0];
    const uint32_t T = (d1 << kLowBits) | tlow;
    const uint32_t need = krem;

    // per-group counts of selected-for-sure (key > T) and tied (key == T) entries
    for (uint32_t g = t; g < ng; g += kT) {
        g_gt[g] = overflow ? 0u : st.grp_gt[(size_t)s * st.maxgroups + g];
        g_eq[g] = 0u;
    }
    __syncthreads();
    if (!overflow) {
        for_each_entry([&](uint32_t e) {
            const uint32_t low = e & kLowMask, g = e >> kLowBits;
            if (low > tlow) atomicAdd(&g_gt[g], 1u);
            else if (low == tlow) atomicAdd(&g_eq[g], 1u);
        });
    } else {
        for (uint32_t g = 0; g < ng; ++g) {
            const uint32_t total = load_group(src, s, dn, g, &gs);
            uint32_t cg = 0, ce = 0;
            for (uint32_t i = t; i < total; i += kT) {
                uint32_t idx, vb;
                if (src.fetch(s, dn, group_slot(&gs, i), idx, vb)) {
                    const uint32_t key = vb & kAbs;
                    cg += key > T;
                    ce += key == T;
                }
            }
            if (cg) atomicAdd(&g_gt[g], cg);
            if (ce) atomicAdd(&g_eq[g], ce);
        }
    }
    __syncthreads();

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
    // leave the per-set scratch clear for the next select that uses it
    uint32_t* hg = st.hist + (size_t)s * kHistBins;
    for (uint32_t b = t; b < (uint32_t)kHistBins; b += kT) hg[b] = 0u;
    if (t == 0) {
        st.T[s] = T;
        st.need[s] = need;
        st.list_cnt[s] = 0u;
    }
}

// ---------------------------------------------------------------------------------
// exact select, kernel 4: ordered emit
// ---------------------------------------------------------------------------------

// One block per group.  An entry is selected if key > T, or key == T and fewer than
// `need` equal-key entries precede it in index order; its output slot is the number of
// selected entries before it.  ZERO: also store +0.0 at its index in the set's dense
// row (Algorithm 4 line 8).  DIVIDE: value / divisor (Eq. 3).  gbits != NULL: also set
// bit `index` of that bitmap (the dense gMask of Algorithm 3 lines 21-22, one bit per
// gradient element).
template <class Src, bool ZERO, bool DIVIDE>
__global__ __launch_bounds__(kBlock) void k_emit(
        Src src, SelState st, uint32_t k, uint32_t* __restrict__ out_idx,
        float* __restrict__ out_val, int64_t out_stride, float* __restrict__ row,
        int64_t row_stride, float divisor, uint32_t* __restrict__ gbits) {
    __shared__ GroupSegs gs;
    __shared__ uint32_t s_eq[kBlock / kWave];
    __shared__ uint32_t s_sel[kBlock / kWave];
    const int s = blockIdx.y;
    const uint32_t g = blockIdx.x;
    const bool dn = src.dense(s);
    if (g >= src.ngroups(s, dn)) return;
    const uint32_t T = st.T[s], need = st.need[s];
    uint32_t eq_before = st.off_eq[(size_t)s * st.maxgroups + g];
    uint32_t outp = st.off_gt[(size_t)s * st.maxgroups + g] + (eq_before < need ? eq_before : need);
    const uint32_t total = load_group(src, s, dn, g, &gs);
    const uint32_t wave = threadIdx.x / kWave;
    for (uint32_t i0 = 0; i0 < total; i0 += kBlock) {
        const uint32_t i = i0 + threadIdx.x;
        bool is_gt = false, is_eq = false;
        uint32_t idx = 0, vb = 0;
        if (i < total) {
            if (src.fetch(s, dn, group_slot(&gs, i), idx, vb)) {
                const uint32_t key = vb & kAbs;
                is_gt = key > T;
                is_eq = key == T;
            }
        }
        const uint64_t eqm = __ballot(is_eq);
        __syncthreads();                  // the previous step's s_eq / s_sel are no longer read
        if (lane_id() == 0) s_eq[wave] = (uint32_t)__popcll(eqm);
        __syncthreads();
        uint32_t eq_base = eq_before, eq_all = 0;
        for (uint32_t v = 0; v < kBlock / kWave; ++v) {
            if (v < wave) eq_base += s_eq[v];
            eq_all += s_eq[v];
        }
        const bool sel = is_gt || (is_eq && (eq_base + rank_in(eqm) < need));
        const uint64_t selm = __ballot(sel);
        if (lane_id() == 0) s_sel[wave] = (uint32_t)__popcll(selm);
        __syncthreads();
        uint32_t sel_base = outp, sel_all = 0;
        for (uint32_t v = 0; v < kBlock / kWave; ++v) {
            if (v < wave) sel_base += s_sel[v];
            sel_all += s_sel[v];
        }
        if (sel) {
            const uint32_t pos = sel_base + rank_in(selm);
            if (pos < k) {      // always true when the select state is consistent
                out_idx[(int64_t)s * out_stride + pos] = idx;
                float v = __uint_as_float(vb);
                if (DIVIDE) v = v / divisor;
                out_val[(int64_t)s * out_stride + pos] = v;
            }
            if (ZERO) row[(int64_t)s * row_stride + idx] = 0.0f;
            if (gbits) atomicOr(&gbits[idx >> 5], 1u << (idx & 31));
        }
        outp += sel_all;
        eq_before += eq_all;
    }
}

// ---------------------------------------------------------------------------------
// merge: index-ordered union of two k-sets into 2k slots
// ---------------------------------------------------------------------------------

// Entry x of A goes to slot x + #{B < A[x]}, entry y of B to slot y + #{A <= B[y]}:
// a bijection onto [0, 2k) that lists the union in index order, A's copy first
// where both hold an index.  A's copy then carries the sum (one fp32 add) and B's
// slot becomes a tombstone.  Both binary searches advance in the same loop.
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
    const uint32_t ia = ai[x], ib = bi[x];
    // lo_a -> #{B < ia} (lower bound), lo_b -> #{A <= ib} (upper bound)
    uint32_t lo_a = 0, hi_a = k, lo_b = 0, hi_b = k;
    while (lo_a < hi_a || lo_b < hi_b) {
        if (lo_a < hi_a) {
            const uint32_t mid = (lo_a + hi_a) >> 1;
            if (bi[mid] < ia) lo_a = mid + 1; else hi_a = mid;
        }
        if (lo_b < hi_b) {
            const uint32_t mid = (lo_b + hi_b) >> 1;
            if (ai[mid] <= ib) lo_b = mid + 1; else hi_b = mid;
        }
    }
    float va = av[x];
    if (lo_a < k && bi[lo_a] == ia) va = va + bv[lo_a];
    mi[x + lo_a] = ia;
    mv[x + lo_a] = va;
    const bool dup = lo_b > 0 && ai[lo_b - 1] == ib;
    mi[x + lo_b] = dup ? kTomb : ib;
    mv[x + lo_b] = bv[x];
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
        float* __restrict__ res, int64_t stride, uint32_t k, const uint32_t* __restrict__ loc_idx,
        const float* __restrict__ loc_val, const uint32_t* __restrict__ g_idx) {
    const int w = blockIdx.y;
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    if (t >= k) return;
    const uint32_t i = loc_idx[(size_t)w * k + t];
    if (contains(g_idx, k, i)) return;          // index is in the global set: stays zero
    float* slot = res + (int64_t)w * stride + i;
    *slot = *slot + loc_val[(size_t)w * k + t];
}

// The fused form used by gtopk_step, where the local selection did NOT zero its entries
// (the row still holds acc there).  Zero-then-add-back leaves acc unchanged except that
// +0.0 + (-0.0) = +0.0, so: an entry whose index is in the global set becomes +0.0, an
// entry that is -0.0 becomes +0.0, every other entry is already what the literal form
// produces.  gbits is the one-bit-per-element mask of the global set.
__global__ __launch_bounds__(kBlock) void k_restore_fused(
        float* __restrict__ res, int64_t stride, uint32_t k, const uint32_t* __restrict__ loc_idx,
        const float* __restrict__ loc_val, const uint32_t* __restrict__ gbits) {
    const int w = blockIdx.y;
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    if (t >= k) return;
    const uint32_t i = loc_idx[(size_t)w * k + t];
    const uint32_t vb = __float_as_uint(loc_val[(size_t)w * k + t]);
    const bool in_g = (gbits[i >> 5] >> (i & 31)) & 1u;
    if (in_g || vb == 0x80000000u) res[(int64_t)w * stride + i] = 0.0f;
}

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

// hist and list_cnt are carved back to back so that one clear covers them
SelState carve_select(Carver& c, size_t sets, uint32_t list_cap, uint32_t maxgroups) {
    SelState s;
    s.hist = c.take<uint32_t>(sets * kHistBins);
    s.list_cnt = c.take<uint32_t>(sets);
    s.d1 = c.take<uint32_t>(sets);
    s.krem = c.take<uint32_t>(sets);
    s.T = c.take<uint32_t>(sets);
    s.need = c.take<uint32_t>(sets);
    s.list = c.take<uint32_t>(sets * list_cap);
    s.grp_gt = c.take<uint32_t>(sets * maxgroups);
    s.off_gt = c.take<uint32_t>(sets * maxgroups);
    s.off_eq = c.take<uint32_t>(sets * maxgroups);
    s.list_cap = list_cap;
    s.maxgroups = maxgroups;
    return s;
}
// words from s.hist to the end of s.list_cnt (padding included)
inline size_t select_clear_words(const SelState& s) { return (size_t)(s.d1 - s.hist); }

// slots per group of a merged array of 2k slots: at least 1024, at most 2048 groups
uint32_t merged_group_slots(uint32_t k) {
    uint32_t L = ceil_div(2ull * k, kMaxGroups);
    L = (L + 255u) & ~255u;
    return L < 1024u ? 1024u : L;
}

struct MergeWs {
    SelState sel;
    uint32_t* m_idx;   // [pairs][2k]
    float* m_val;
    uint32_t L;
    size_t bytes;
};

MergeWs carve_merge(Carver& c, uint32_t k, size_t pairs) {
    MergeWs w;
    w.L = merged_group_slots(k);
    w.sel = carve_select(c, pairs, 2 * k, ceil_div(2ull * k, w.L));
    w.m_idx = c.take<uint32_t>(pairs * 2 * k);
    w.m_val = c.take<float>(pairs * 2 * k);
    w.bytes = c.off;
    return w;
}

struct StepWs {
    // local select
    uint32_t* samp_hist;   // [P][16384]   } cleared together
    uint32_t* cand_count;  // [P]          }
    uint32_t* tspec;       // [P]
    uint32_t* cand_idx;    // [P][cap]
    float* cand_val;
    uint2* run_table;      // [P][nchunks]
    SelState sel;          // P sets
    uint32_t cap, nchunks, G;
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

StepWs carve_step(void* ws, int64_t m, uint32_t k, uint32_t P) {
    Carver c{reinterpret_cast<char*>(ws)};
    StepWs s;
    s.cap = cand_capacity(m, k);
    s.nchunks = ceil_div((uint64_t)m, kChunk);
    s.G = ceil_div(s.nchunks, kMaxGroups);
    if (s.G < 16) s.G = 16;                       // <= 32 = kMaxSeg because m <= 2^31
    s.samp_hist = c.take<uint32_t>((size_t)P * kSampleBins);
    s.cand_count = c.take<uint32_t>(P);
    s.tspec = c.take<uint32_t>(P);
    s.cand_idx = c.take<uint32_t>((size_t)P * s.cap);
    s.cand_val = c.take<float>((size_t)P * s.cap);
    s.run_table = c.take<uint2>((size_t)P * s.nchunks);
    s.sel = carve_select(c, P, s.cap, ceil_div(s.nchunks, s.G));
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

bool sizes_ok(int64_t m, int64_t k, int64_t P) {
    return m >= 1 && m <= ((int64_t)1 << 31) && k >= 1 && k <= m && is_pow2(P) && P <= 65535;
}

int launch_status() { return hipGetLastError() == hipSuccess ? GTOPK_OK : GTOPK_EHIP; }

// Instrumentation: events the next gtopk_step records at its stage boundaries.
hipEvent_t g_stage_events[GTOPK_STAGE_EVENTS];
bool g_stage_armed = false;

void mark_stage(int i, bool armed, hipStream_t st) {
    if (armed) (void)hipEventRecord(g_stage_events[i], st);
}

void zero_async(hipStream_t st, uint32_t* p0, size_t n0, uint32_t* p1 = nullptr, size_t n1 = 0,
                uint32_t* p2 = nullptr, size_t n2 = 0, uint32_t* p3 = nullptr, size_t n3 = 0) {
    ZeroJob job{{p0, p1, p2, p3}, {n0, n1, n2, n3}};
    size_t n = 0;
    for (int a = 0; a < 4; ++a) n = job.n[a] > n ? job.n[a] : n;
    uint32_t blocks = (uint32_t)((n + 1023) / 1024 > 1024 ? 1024 : (n + 1023) / 1024);
    hipLaunchKernelGGL(k_zero_u32, dim3(blocks ? blocks : 1), dim3(256), 0, st, job);
}

// histogram + bucket + finish + emit over `sets` sets of at most nphys_max slots each
template <class Src, bool ZERO, bool DIVIDE>
void run_select(const Src& src, const SelState& ss, uint32_t sets, uint32_t k, uint64_t nphys_max,
                uint32_t* out_idx, float* out_val, int64_t out_stride, float* row,
                int64_t row_stride, float divisor, uint32_t* gbits, hipStream_t st) {
    uint32_t hb = ceil_div(nphys_max, 4 * kHistBlock);
    hb = hb < 1 ? 1 : (hb > 32 ? 32 : hb);
    hipLaunchKernelGGL((k_hist<Src>), dim3(hb, sets), dim3(kHistBlock), 0, st, src, ss);
    hipLaunchKernelGGL((k_bucket<Src>), dim3(ss.maxgroups, sets), dim3(kBlock), 0, st, src, ss, k);
    hipLaunchKernelGGL((k_finish<Src>), dim3(sets), dim3(1024), 0, st, src, ss);
    hipLaunchKernelGGL((k_emit<Src, ZERO, DIVIDE>), dim3(ss.maxgroups, sets), dim3(kBlock), 0, st, src,
                       ss, k, out_idx, out_val, out_stride, row, row_stride, divisor, gbits);
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

// `zero_rows`: store +0.0 at the selected entries (the stand-alone call); gtopk_step
// passes false and settles the rows in k_restore_fused.  `pre_cleared`: the caller has
// already cleared this call's counters and histograms.
int do_local_select(const float* grad, float* residual, int64_t m, int64_t stride, uint32_t P,
                    uint32_t k, uint32_t* out_idx, float* out_val, const StepWs& w, bool zero_rows,
                    bool pre_cleared, hipStream_t st, bool armed = false) {
    if (!pre_cleared)
        zero_async(st, w.samp_hist, (size_t)(w.tspec - w.samp_hist), w.sel.hist,
                   select_clear_words(w.sel));

    const SamplePlan sp = plan_sample(m, k);
    uint32_t sblocks = ceil_div(sp.n_tiles, (kSampleBlock / kSampleTile) * 8);
    if (sblocks > 16) sblocks = 16;
    if (sblocks < 1) sblocks = 1;
    hipLaunchKernelGGL(k_sample, dim3(sblocks, P), dim3(kSampleBlock), 0, st, grad, residual,
                       (uint32_t)m, stride, sp.tile_stride, sp.n_tiles, w.samp_hist);
    hipLaunchKernelGGL(k_sample_pick, dim3(P), dim3(kSampleBlock), 0, st, w.samp_hist, sp.target,
                       w.tspec);
    mark_stage(1, armed, st);

    const bool vec = (stride % 4 == 0);
    if (vec)
        hipLaunchKernelGGL((k_accum_filter<true>), dim3(w.nchunks, P), dim3(kSBlock), 0, st, grad,
                           residual, (uint32_t)m, stride, w.tspec, w.cand_idx, w.cand_val, w.cap,
                           w.cand_count, w.run_table, w.nchunks);
    else
        hipLaunchKernelGGL((k_accum_filter<false>), dim3(w.nchunks, P), dim3(kSBlock), 0, st, grad,
                           residual, (uint32_t)m, stride, w.tspec, w.cand_idx, w.cand_val, w.cap,
                           w.cand_count, w.run_table, w.nchunks);
    mark_stage(2, armed, st);

    CandSrc src{residual, stride, (uint32_t)m, k, w.cap, w.nchunks, w.G,
                w.cand_idx, w.cand_val, w.cand_count, w.run_table};
    if (zero_rows)
        run_select<CandSrc, true, false>(src, w.sel, P, k, w.cap, out_idx, out_val, (int64_t)k,
                                         residual, stride, 1.0f, nullptr, st);
    else
        run_select<CandSrc, false, false>(src, w.sel, P, k, w.cap, out_idx, out_val, (int64_t)k,
                                          residual, stride, 1.0f, nullptr, st);
    return launch_status();
}

// one batch of merges: union + exact select + ordered emit.
// w.sel's hist and list_cnt must be clear on entry and are left clear.
template <bool DIVIDE>
void do_merge_batch(const uint32_t* a_idx, const float* a_val, const uint32_t* b_idx,
                    const float* b_val, uint32_t k, uint32_t batch, int64_t in_stride,
                    uint32_t* out_idx, float* out_val, int64_t out_stride, const MergeWs& w,
                    float divisor, uint32_t* gbits, hipStream_t st) {
    hipLaunchKernelGGL(k_union, dim3(ceil_div(k, kBlock), batch), dim3(kBlock), 0, st, a_idx, a_val,
                       b_idx, b_val, k, in_stride, w.m_idx, w.m_val);
    MergedSrc src{w.m_idx, w.m_val, 2 * k, w.L};
    run_select<MergedSrc, false, DIVIDE>(src, w.sel, batch, k, 2ull * k, out_idx, out_val, out_stride,
                                         nullptr, 0, divisor, gbits, st);
}

int do_tree(const uint32_t* loc_idx, const float* loc_val, uint32_t P, uint32_t k, uint32_t* g_idx,
            float* g_val, const StepWs& w, uint32_t* gbits, bool pre_cleared, hipStream_t st) {
    const float divisor = (float)P;
    if (P == 1) {
        hipLaunchKernelGGL(k_copy_set, dim3(ceil_div(k, 256)), dim3(256), 0, st, loc_idx, loc_val, k,
                           g_idx, g_val, divisor, gbits);
        return launch_status();
    }
    if (!pre_cleared) zero_async(st, w.mrg.sel.hist, select_clear_words(w.mrg.sel));
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
                                 g_val, k, w.mrg, divisor, gbits, st);
        } else {
            do_merge_batch<false>(in_idx, in_val, in_idx + k, in_val + k, k, pairs, 2 * (int64_t)k,
                                  ping_i, ping_v, k, w.mrg, 1.0f, nullptr, st);
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
                           true, false, (hipStream_t)stream);
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
    zero_async(st, w.sel.hist, select_clear_words(w.sel));
    do_merge_batch<false>(a_idx, a_val, b_idx, b_val, (uint32_t)k, (uint32_t)batch, in_stride,
                          out_idx, out_val, out_stride, w, 1.0f, nullptr, st);
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
    return do_tree(loc_idx, loc_val, (uint32_t)P, (uint32_t)k, g_idx, g_val, w, nullptr, false,
                   (hipStream_t)stream);
}

int gtopk_residual_restore(float* residual, int64_t m, int64_t stride, int32_t P, int32_t k,
                           const uint32_t* loc_idx, const float* loc_val, const uint32_t* g_idx,
                           void* stream) {
    if (!residual || !loc_idx || !loc_val || !g_idx) return GTOPK_EINVAL;
    if (!sizes_ok(m, k, P) || stride < m) return GTOPK_EINVAL;
    if (!aligned16(residual) || !aligned16(loc_idx) || !aligned16(loc_val) || !aligned16(g_idx))
        return GTOPK_EALIGN;
    hipLaunchKernelGGL(k_restore, dim3(ceil_div((uint32_t)k, kBlock), (uint32_t)P), dim3(kBlock), 0,
                       (hipStream_t)stream, residual, stride, (uint32_t)k, loc_idx, loc_val, g_idx);
    return launch_status();
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
    const bool armed = g_stage_armed;
    g_stage_armed = false;
    mark_stage(0, armed, st);
    // one clear for everything this step needs zeroed: the sampler's histograms and the
    // candidate counters; both selects' histograms and tickets; the global-set bitmap
    zero_async(st, w.samp_hist, (size_t)(w.tspec - w.samp_hist), w.sel.hist,
               select_clear_words(w.sel), w.mrg.sel.hist, select_clear_words(w.mrg.sel), w.gbits,
               w.gbits_words);
    int rc = do_local_select(grad, residual, m, stride, (uint32_t)P, (uint32_t)k, li, lv, w, false,
                             true, st, armed);
    if (rc != GTOPK_OK) return rc;
    mark_stage(3, armed, st);
    rc = do_tree(li, lv, (uint32_t)P, (uint32_t)k, g_idx, g_val, w, w.gbits, true, st);
    if (rc != GTOPK_OK) return rc;
    mark_stage(4, armed, st);
    hipLaunchKernelGGL(k_restore_fused, dim3(ceil_div((uint32_t)k, kBlock), (uint32_t)P), dim3(kBlock),
                       0, st, residual, stride, (uint32_t)k, li, lv, w.gbits);
    rc = launch_status();
    mark_stage(5, armed, st);
    return rc;
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

int gtopk_arm_stage_events(void* const* events) {
    if (!events) { g_stage_armed = false; return GTOPK_OK; }
    for (int i = 0; i < GTOPK_STAGE_EVENTS; ++i) {
        if (!events[i]) return GTOPK_EINVAL;
        g_stage_events[i] = (hipEvent_t)events[i];
    }
    g_stage_armed = true;
    return GTOPK_OK;
}

}  // extern "C"
