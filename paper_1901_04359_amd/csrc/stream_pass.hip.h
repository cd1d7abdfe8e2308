// Local selection, Algorithm 4 lines 4-8, the part that touches all P*m elements:
// a sampled histogram that yields a speculative threshold, and the one streaming pass
// that accumulates (line 4) and keeps the entries at or above that threshold.
#pragma once
#include "common.hip.h"

namespace gtopk {

// Sample tile t of a row covers [t*tile_stride, t*tile_stride + 64) (clipped to m): one
// wave per tile.  A block of 1024 threads takes sixteen tiles per round and keeps four
// rounds of loads in flight.
__global__ __launch_bounds__(kSampleBlock) void k_sample(
        const float* __restrict__ grad, const float* __restrict__ res, uint32_t m, int64_t stride,
        uint32_t tile_stride, uint32_t n_tiles, uint32_t* __restrict__ samp_hist,
        const uint4* __restrict__ carry) {
    __shared__ uint32_t h[kSampleBins];
    const int w = blockIdx.y;
    if (carry && carry[w].x == 2u) return;        // this worker filters with a carried threshold
    for (int b = threadIdx.x; b < kSampleBins; b += kSampleBlock) h[b] = 0u;
    __syncthreads();
    const float* g = grad + (int64_t)w * stride;
    const float* r = res + (int64_t)w * stride;
    const uint32_t sub = threadIdx.x / kSampleTile, el = threadIdx.x % kSampleTile;
    constexpr int kUnroll = 4;
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
        const uint32_t* __restrict__ samp_hist, uint32_t target, uint32_t* __restrict__ tspec,
        const uint4* __restrict__ carry) {
    __shared__ uint32_t s_wave[kSampleBlock / kWave];
    __shared__ uint32_t s_out[3];
    const int w = blockIdx.x;
    if (carry) {
        const uint4 c = carry[w];
        if (c.x == 2u) {                          // block-uniform
            if (threadIdx.x == 0) tspec[w] = c.w;
            return;
        }
    }
    constexpr int kPer = kSampleBins / kSampleBlock;
    const uint32_t* hist = samp_hist + (size_t)w * kSampleBins;
    uint32_t loc[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) loc[j] = hist[threadIdx.x * kPer + j];
    suffix_pick<kPer>(loc, target, s_wave, s_out);
    if (threadIdx.x == 0) tspec[w] = s_out[2] ? (s_out[0] << kSampleShift) : 0u;
}

// Rows need not start on a 16-byte boundary (stride and m are arbitrary).  With
// head = (w * stride) mod 4, element j of row w sits at "virtual" position v = j + head
// of a 16-byte aligned array that starts head elements before the row; chunks and
// float4 accesses are laid out on v, so every vector access is aligned and only the
// few lanes that straddle a row end fall back to scalar accesses.
//
// Block (chunk, w) handles virtual positions [chunk*32768, +32768) of worker w; each of
// its 8 waves a contiguous 4096 of them, 16 float4 per lane, all held in registers.
// (ITERS float4 per lane in general: 2048 * ITERS positions per block.  Short rows of few
// workers take small blocks, so that they spread over more than a handful of CUs.)
// Phase 1 loads, adds, stores and counts the entries whose key reaches the speculative
// threshold; one atomicAdd per block reserves a contiguous range ("run") of the worker's
// candidate list; phase 2 writes the block's candidates there in index order.
// Blocks reserve in any order, nobody waits for anybody; run_table[w][chunk] =
// (first slot, count) lets the select put the runs back into index order.
// HIST: the block also adds the first digits of its candidates to the worker's histogram
// (what the select's histogram kernel would read back), through an LDS histogram: one
// global atomic per non-empty bin.  (One global atomic per candidate is as good where the
// candidates are spread evenly, and far worse where they crowd into a few blocks.)
template <bool HIST, int ITERS = kIters>
__global__ __launch_bounds__(kSBlock) void k_accum_filter(
        const float* __restrict__ grad, float* __restrict__ res, uint32_t m, int64_t stride,
        const uint32_t* __restrict__ tspec, uint32_t* __restrict__ cand_idx,
        float* __restrict__ cand_val, uint32_t cap, uint32_t* __restrict__ cand_count,
        uint2* __restrict__ run_table, uint32_t nchunks, uint32_t* __restrict__ hist) {
    constexpr int kWaves = kSBlock / kWave;
    __shared__ uint32_t s_cnt[kWaves];
    __shared__ uint32_t s_base;
    __shared__ uint32_t s_total;
    __shared__ uint32_t s_h[HIST ? kHistBins : 1];
    if (HIST)
        for (int b = threadIdx.x; b < kHistBins; b += kSBlock) s_h[b] = 0u;     // a barrier follows
    const int w = blockIdx.y;
    const uint32_t chunk = blockIdx.x;
    const uint32_t lane = lane_id();
    const uint32_t wave = threadIdx.x / kWave;
    const uint32_t head = (uint32_t)(((int64_t)w * stride) & 3);
    // aligned array that holds the row at [head, head + m)
    const float* g = grad + (int64_t)w * stride - head;
    float* r = res + (int64_t)w * stride - head;
    const uint32_t vend = head + m;          // <= 2^31 + 3
    const uint32_t ts = tspec[w];
    // chunk < ceil((m + 3) / 32768), so none of the offsets below wraps
    constexpr uint32_t kSpan = ITERS * 4 * kWave;            // elements per wave
    const uint32_t wbase = chunk * (kSpan * (uint32_t)kWaves) + wave * kSpan;

    float a[ITERS][4];
    const bool whole = wbase >= head && wbase + kSpan <= vend;   // wave-uniform
    if (whole) {
        floatx4 gv[ITERS], rv[ITERS];
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const uint32_t v = wbase + i * 256 + lane * 4;
            gv[i] = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(g + v));
            rv[i] = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(r + v));
        }
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const uint32_t v = wbase + i * 256 + lane * 4;
            const floatx4 s = rv[i] + gv[i];          // four independent fp32 adds
            __builtin_nontemporal_store(s, reinterpret_cast<floatx4*>(r + v));
            a[i][0] = s.x; a[i][1] = s.y; a[i][2] = s.z; a[i][3] = s.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const uint32_t v = wbase + i * 256 + lane * 4;
            if (v >= head && v + 4 <= vend) {
                const floatx4 s = *reinterpret_cast<const floatx4*>(r + v) +
                                  *reinterpret_cast<const floatx4*>(g + v);
                *reinterpret_cast<floatx4*>(r + v) = s;
                a[i][0] = s.x; a[i][1] = s.y; a[i][2] = s.z; a[i][3] = s.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float s = 0.0f;
                    if (v + e >= head && v + e < vend) {
                        s = r[v + e] + g[v + e];
                        r[v + e] = s;
                    }
                    a[i][e] = s;
                }
            }
        }
    }

    uint32_t cnt = 0;   // wave-uniform
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
        const uint32_t v = wbase + i * 256 + lane * 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool c = (v + e >= head) && (v + e < vend) &&
                           ((__float_as_uint(a[i][e]) & kAbs) >= ts);
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
        s_total = total;
    }
    __syncthreads();
    if (HIST ? s_total == 0 : cnt == 0) return;      // HIST: block-uniform, a barrier follows
    const Digit dg{ts, (uint32_t)kFineShift};
    uint32_t off = s_base;
    for (uint32_t v = 0; v < wave; ++v) off += s_cnt[v];
    uint32_t* ci = cand_idx + (size_t)w * cap;
    float* cv = cand_val + (size_t)w * cap;
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
        const uint32_t v = wbase + i * 256 + lane * 4;
        bool c[4];
        uint64_t b[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            c[e] = (v + e >= head) && (v + e < vend) && ((__float_as_uint(a[i][e]) & kAbs) >= ts);
            b[e] = __ballot(c[e]);
        }
        if ((b[0] | b[1] | b[2] | b[3]) == 0) continue;
        uint32_t pos = off + rank_in(b[0]) + rank_in(b[1]) + rank_in(b[2]) + rank_in(b[3]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (c[e]) {
                if (pos < cap) { ci[pos] = v + e - head; cv[pos] = a[i][e]; }
                if (HIST) atomicAdd(&s_h[dg.bin(__float_as_uint(a[i][e]) & kAbs)], 1u);
                ++pos;
            }
        }
        off += (uint32_t)(__popcll(b[0]) + __popcll(b[1]) + __popcll(b[2]) + __popcll(b[3]));
    }
    if (HIST) {
        __syncthreads();
        uint32_t* out = hist + (size_t)w * kHistBins;
        for (int b = threadIdx.x; b < kHistBins; b += kSBlock) {
            const uint32_t n = s_h[b];
            if (n) atomicAdd(&out[b], n);
        }
    }
}

// ---------------------------------------------------------------------------------
// instrumentation: what the memory system gives to the pass's access pattern
// ---------------------------------------------------------------------------------

// The streaming pass with everything but its memory traffic taken out: same block shape,
// same 16 float4 per lane and array in flight, same non-temporal accesses.
//   ADD:  b[i] = b[i] + a[i]          (8 bytes read, 4 written per element, as the pass)
//   !ADD: both arrays read, one float per block written to `sink` (read-only ceiling)
// n is a multiple of kChunk (the caller checks).
// The other template arguments vary what the pass fixed, so that the choice stays on
// record: NTL / NTS = non-temporal loads / stores; THREADS x ITERS = threads per block x
// float4 per lane and array (a block covers THREADS * ITERS * 4 elements).
template <bool ADD, bool NTL = true, bool NTS = true, int THREADS = kSBlock, int ITERS = kIters>
__global__ __launch_bounds__(THREADS) void k_probe_stream(
        const float* __restrict__ a, float* __restrict__ b, float* __restrict__ sink) {
    constexpr int kSpan = ITERS * 4 * kWave;                 // elements per wave
    const uint32_t lane = lane_id();
    const uint32_t wave = threadIdx.x / kWave;
    const size_t base = (size_t)blockIdx.x * ((size_t)kSpan * (THREADS / kWave)) + (size_t)wave * kSpan;
    floatx4 av[ITERS], bv[ITERS];
#pragma unroll
    for (int i = 0; i < ITERS; ++i) {
        const size_t v = base + i * 256 + lane * 4;
        if (NTL) {
            av[i] = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(a + v));
            bv[i] = __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(b + v));
        } else {
            av[i] = *reinterpret_cast<const floatx4*>(a + v);
            bv[i] = *reinterpret_cast<const floatx4*>(b + v);
        }
    }
    if (ADD) {
#pragma unroll
        for (int i = 0; i < ITERS; ++i) {
            const size_t v = base + i * 256 + lane * 4;
            if (NTS) __builtin_nontemporal_store(bv[i] + av[i], reinterpret_cast<floatx4*>(b + v));
            else *reinterpret_cast<floatx4*>(b + v) = bv[i] + av[i];
        }
    } else {
        floatx4 acc = av[0] + bv[0];
#pragma unroll
        for (int i = 1; i < ITERS; ++i) acc = acc + av[i] + bv[i];
        float s = acc.x + acc.y + acc.z + acc.w;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d);
        if (lane == 0 && wave == 0) sink[blockIdx.x] = s;      // keeps the loads alive
    }
}

}  // namespace gtopk
