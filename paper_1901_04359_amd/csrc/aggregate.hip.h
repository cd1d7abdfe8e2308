// The aggregation that Top-k S-SGD uses (Algorithm 1, procedure TopKAllReduce), as a
// comparison workload for the tree: the P workers' k-sets are summed into one dense
// vector in rank order and averaged.  With all sets already on one GPU the AllGather of the
// procedure is a no-op; what remains is the scatter-add loop and the division by P.
#pragma once
#include "common.hip.h"

namespace gtopk {

constexpr int kAggRange = 8192;        // dense elements per block (held in LDS)
constexpr int kAggMaxP = 1024;         // workers, at most

constexpr int kAggRangeLog2 = 13;
static_assert((1 << kAggRangeLog2) == kAggRange, "range size");

// bounds[g][b] = number of entries of worker g's (index-ascending) k-set with index below
// b * kAggRange, for b = 0 .. nranges: the slices that k_scatter_mean's blocks take.  One
// binary search per bound; the searches of neighbouring bounds share their first probes.
__global__ __launch_bounds__(kBlock) void k_slice_bounds(
        const uint32_t* __restrict__ loc_idx, uint32_t k, uint32_t nranges,
        uint32_t* __restrict__ bounds) {
    const uint32_t b = blockIdx.x * kBlock + threadIdx.x;
    const int g = blockIdx.y;
    if (b > nranges) return;
    const uint32_t* ig = loc_idx + (size_t)g * k;
    const uint64_t target = (uint64_t)b << kAggRangeLog2;
    uint32_t lo = 0, hi = k;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if ((uint64_t)ig[mid] < target) lo = mid + 1; else hi = mid;
    }
    bounds[(size_t)g * (nranges + 1) + b] = lo;
}

// Block b owns the dense elements [b*R, (b+1)*R), R = kAggRange, and keeps them in LDS.
// It reads, for every worker, the slice of that worker's k-set that falls into its range
// and lays the slices end to end ("flat" order: by worker, then by index).  Threads take
// the flat entries 1024 at a time, four each, in registers.  At one index the adds must
// happen in worker order, each one fp32 add, the first onto +0.0; entries at different
// indices are independent.  So the entries of a batch are applied in rounds: every
// pending entry bids for its index with its flat position (LDS atomic minimum), the
// winners add their value and retire, until nothing is pending.  A round retires, for
// every index, the pending entry of the lowest worker; the number of rounds is the largest
// number of workers that share one index within the batch (1 to 3 for sparse sets).
// Batches follow each other in flat order, so the order holds across batches as well.
// The range is written out once, divided by P.
__global__ __launch_bounds__(kBlock) void k_scatter_mean(
        const uint32_t* __restrict__ loc_idx, const float* __restrict__ loc_val, uint32_t P,
        uint32_t k, uint32_t m, const uint32_t* __restrict__ bounds, uint32_t nranges,
        float divisor, float* __restrict__ dense) {
    constexpr int kEpt = 4;
    constexpr uint32_t kNoBid = 0xFFFFFFFFu;
    __shared__ __align__(16) float acc[kAggRange];
    __shared__ uint32_t bid[kAggRange];
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
    for (uint32_t i = t; i < (uint32_t)kAggRange; i += kBlock) { acc[i] = 0.0f; bid[i] = kNoBid; }
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
    for (uint32_t c0 = 0; c0 < total; c0 += kBlock * kEpt) {
        // thread t takes the flat entries c0 + 4t .. c0 + 4t + 3: its bids order them
        uint32_t ei[kEpt];
        float ev[kEpt];
        bool pending[kEpt];
#pragma unroll
        for (int u = 0; u < kEpt; ++u) {
            const uint32_t e = c0 + t * kEpt + u;
            pending[u] = e < total;
            ei[u] = 0;
            ev[u] = 0.0f;
            if (pending[u]) {
                const uint32_t g = worker_of(e);
                const size_t j = (size_t)g * k + s_lo[g] + (e - s_off[g]);
                ei[u] = loc_idx[j] - base;
                ev[u] = loc_val[j];
                pending[u] = ei[u] < (uint32_t)kAggRange;      // always true for sorted sets
            }
        }
        bool any = true;
        while (any) {                     // block-uniform: `any` comes from a block-wide vote
#pragma unroll
            for (int u = 0; u < kEpt; ++u)
                if (pending[u]) atomicMin(&bid[ei[u]], t * kEpt + u);
            __syncthreads();
            bool win[kEpt];
#pragma unroll
            for (int u = 0; u < kEpt; ++u) win[u] = pending[u] && bid[ei[u]] == t * kEpt + u;
            __syncthreads();
            bool left = false;
#pragma unroll
            for (int u = 0; u < kEpt; ++u) {
                if (win[u]) {
                    acc[ei[u]] = acc[ei[u]] + ev[u];
                    bid[ei[u]] = kNoBid;
                    pending[u] = false;
                }
                left = left || pending[u];
            }
            any = __syncthreads_or(left) != 0;
        }
    }
    __syncthreads();
    float* out = dense + base;                      // 16-byte aligned: base is a multiple of kAggRange
    if (span == (uint32_t)kAggRange) {
        for (uint32_t i = 4 * t; i < (uint32_t)kAggRange; i += 4 * kBlock) {
            const float4 a = *reinterpret_cast<const float4*>(&acc[i]);
            *reinterpret_cast<float4*>(out + i) =
                make_float4(a.x / divisor, a.y / divisor, a.z / divisor, a.w / divisor);
        }
    } else {
        for (uint32_t i = t; i < span; i += kBlock) out[i] = acc[i] / divisor;
    }
}

}  // namespace gtopk
