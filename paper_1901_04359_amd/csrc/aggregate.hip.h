// The aggregation that Top-k S-SGD uses (Algorithm 1, procedure TopKAllReduce), as a
// comparison workload for the tree: the P workers' k-sets are summed into one dense
// vector in rank order and averaged.  With all sets already on one GPU the AllGather of the
// procedure is a no-op; what remains is the scatter-add loop and the division by P.
#pragma once
#include "common.hip.h"

namespace gtopk {

constexpr int kAggRange = 8192;        // dense elements per block (held in LDS)
constexpr int kAggStage = 2048;        // k-set entries staged in LDS at a time
constexpr int kAggMaxP = 1024;         // workers, at most

constexpr int kAggRangeLog2 = 13;
static_assert((1 << kAggRangeLog2) == kAggRange, "range size");

// bounds[g][b] = number of entries of worker g's (index-ascending) k-set with index below
// b * 8192, for b = 0 .. nranges: the slices that k_scatter_mean's blocks take.  Entry j
// writes the bounds that fall between its predecessor's range and its own; the last
// entry also writes those behind it.
__global__ __launch_bounds__(kBlock) void k_slice_bounds(
        const uint32_t* __restrict__ loc_idx, uint32_t k, uint32_t nranges,
        uint32_t* __restrict__ bounds) {
    const uint32_t j = blockIdx.x * kBlock + threadIdx.x;
    const int g = blockIdx.y;
    if (j >= k) return;
    const uint32_t* ig = loc_idx + (size_t)g * k;
    uint32_t* bg = bounds + (size_t)g * (nranges + 1);
    uint32_t cur = ig[j] >> kAggRangeLog2;
    if (cur > nranges) cur = nranges;                 // only for an index >= m (not a valid set)
    uint32_t b = 0;
    if (j > 0) {
        const uint32_t prev = ig[j - 1] >> kAggRangeLog2;
        b = prev + 1;                                 // bounds up to prev are the predecessors'
    }
    for (; b <= cur; ++b) bg[b] = j;
    if (j == k - 1)
        for (b = cur + 1; b <= nranges; ++b) bg[b] = k;
}

// Block b owns the dense elements [b*8192, (b+1)*8192).  It reads, for every worker, the
// slice of that worker's k-set that falls into its range, stages the slices' entries in
// LDS, all workers' loads in flight together, and adds them into an LDS copy of its range
// worker by worker: at one index the adds happen in the order g = 0 .. P-1, each one fp32
// add, the first onto +0.0.  Indices are distinct inside a worker's set, so the threads
// that apply one worker's slice never meet.  The range is written out once, divided by P.
__global__ __launch_bounds__(kBlock) void k_scatter_mean(
        const uint32_t* __restrict__ loc_idx, const float* __restrict__ loc_val, uint32_t P,
        uint32_t k, uint32_t m, const uint32_t* __restrict__ bounds, uint32_t nranges,
        float divisor, float* __restrict__ dense) {
    __shared__ float acc[kAggRange];
    __shared__ uint32_t st_i[kAggStage];
    __shared__ float st_v[kAggStage];
    __shared__ uint32_t s_lo[kAggMaxP];            // first entry of worker g inside the range
    __shared__ uint32_t s_off[kAggMaxP + 1];       // entries of workers < g inside the range
    __shared__ uint32_t s_wave[kBlock / kWave];
    const uint32_t t = threadIdx.x;
    const uint32_t base = blockIdx.x * (uint32_t)kAggRange;          // < m by the launch grid
    const uint32_t span = m - base < (uint32_t)kAggRange ? m - base : (uint32_t)kAggRange;
    for (uint32_t g = t; g < P; g += kBlock) {
        const uint32_t* bg = bounds + (size_t)g * (nranges + 1) + blockIdx.x;
        uint32_t lo = bg[0], hi = bg[1];
        // always lo <= hi <= k for a sorted set; keeps every access in bounds for any other
        if (hi > k) hi = k;
        if (lo > hi) lo = hi;
        s_lo[g] = lo;
        s_off[g + 1] = hi;                         // holds the end for now
    }
    for (uint32_t i = t; i < (uint32_t)kAggRange; i += kBlock) acc[i] = 0.0f;
    __syncthreads();
    // counts -> exclusive offsets (up to 4 workers per thread)
    {
        constexpr int kPer = kAggMaxP / kBlock;
        uint32_t c[kPer], sum = 0;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const uint32_t g = t * kPer + j;
            c[j] = g < P ? s_off[g + 1] - s_lo[g] : 0u;
            sum += c[j];
        }
        __syncthreads();                  // every end has been read before offsets overwrite them
        uint32_t total;
        uint32_t run = block_incl_scan(sum, s_wave, total) - sum;
        if (t == 0) s_off[0] = 0u;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const uint32_t g = t * kPer + j;
            run += c[j];
            if (g < P) s_off[g + 1] = run;
        }
    }
    __syncthreads();
    const uint32_t total = s_off[P];
    // worker that holds flat entry e: the last g with s_off[g] <= e (empty workers skipped)
    auto worker_of = [&](uint32_t e) {
        uint32_t lo = 0, hi = P;          // answer in [lo, hi)
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (s_off[mid] <= e) lo = mid; else hi = mid;
        }
        return lo;
    };
    for (uint32_t c0 = 0; c0 < total; c0 += (uint32_t)kAggStage) {
        const uint32_t c1 = c0 + (uint32_t)kAggStage < total ? c0 + (uint32_t)kAggStage : total;
        for (uint32_t e = c0 + t; e < c1; e += kBlock) {
            const uint32_t g = worker_of(e);
            const size_t j = (size_t)g * k + s_lo[g] + (e - s_off[g]);
            st_i[e - c0] = loc_idx[j] - base;
            st_v[e - c0] = loc_val[j];
        }
        __syncthreads();
        const uint32_t g_first = worker_of(c0), g_last = worker_of(c1 - 1);
        for (uint32_t g = g_first; g <= g_last; ++g) {
            const uint32_t b0 = s_off[g] > c0 ? s_off[g] : c0;
            const uint32_t b1 = s_off[g + 1] < c1 ? s_off[g + 1] : c1;
            if (b0 >= b1) continue;       // block-uniform
            for (uint32_t e = b0 + t; e < b1; e += kBlock) {
                const uint32_t i = st_i[e - c0];
                if (i < (uint32_t)kAggRange) acc[i] = acc[i] + st_v[e - c0];   // always true for sorted sets
            }
            __syncthreads();
        }
    }
    __syncthreads();
    float* out = dense + base;
    for (uint32_t i = t; i < span; i += kBlock) out[i] = acc[i] / divisor;
}

}  // namespace gtopk
