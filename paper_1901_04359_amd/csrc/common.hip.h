// Constants and wave/block primitives shared by the gTop-k kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gtopk {

constexpr int kWave = 64;
constexpr int kSBlock = 512;                // threads per block of the streaming pass
constexpr int kIters = 16;                  // float4 loads per lane and array in the streaming pass
constexpr int kWaveSpan = kIters * 4 * kWave;            // 4096 elements per wave
constexpr int kChunkLog2 = 15;
constexpr int kChunk = 1 << kChunkLog2;                  // 32768 elements per block = one run
static_assert(kChunk == kWaveSpan * (kSBlock / kWave), "a block covers exactly one chunk");
constexpr int kBlock = 256;                 // threads per block of the select kernels
constexpr int kBatch = 2;                   // items a thread loads before it processes any (swept: 1, 2, 4, 8)
constexpr int kHistBatch = 2;               // the same in the histogram kernel
constexpr int kMaxGroups = 2048;            // groups per set, at most
constexpr int kHistBins = 4096;             // bins of the first digit
constexpr int kFineShift = 10;              // narrowest bin: 2^10 keys, when a lower bound of T is known
constexpr int kCoarseShift = 19;            // bin width 2^19 keys (exponent + 4 mantissa bits) otherwise
constexpr int kSampleBits = 14;             // sample histogram: exponent + 6 mantissa bits
constexpr int kSampleBins = 1 << kSampleBits;
constexpr int kSampleShift = 31 - kSampleBits;
constexpr int kSampleTile = 64;             // contiguous elements per sample tile: one wave
constexpr int kSampleBlock = 1024;
constexpr int kHistBlock = 1024;
constexpr uint32_t kTomb = 0xFFFFFFFFu;     // index of a merged slot that holds nothing
constexpr uint32_t kAbs = 0x7FFFFFFFu;

typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & (kWave - 1); }

// number of set bits of `mask` below the calling lane
__device__ __forceinline__ uint32_t rank_in(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// ---- block-wide primitives: every thread of the block must call them ----------------

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
__device__ inline uint32_t block_incl_scan(uint32_t v, uint32_t* s_wave, uint32_t& total) {
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
__device__ inline void suffix_pick(const uint32_t (&loc)[PER], uint32_t target, uint32_t* s_wave,
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

// Adds 1 to arr[g] for every lane with pred.  Lanes of a wave that share g are combined
// into one atomic.  Every lane of the wave must call it.
__device__ __forceinline__ void add_grouped(bool pred, uint32_t g, uint32_t* arr) {
    uint64_t todo = __ballot(pred);
    while (todo) {
        const uint32_t leader = (uint32_t)__builtin_ctzll(todo);
        const uint32_t gl = __shfl(g, leader);
        const uint64_t same = __ballot(pred && g == gl);
        if (lane_id() == leader) atomicAdd(&arr[gl], (uint32_t)__popcll(same));
        todo &= ~same;
    }
}

// The same for an array in LDS whose lanes mostly differ in g (entries listed group by
// group, a few per group): one combined add if all lanes agree, else an LDS atomic per lane -
// the loop above would take one round per distinct group.
__device__ __forceinline__ void add_grouped_lds(bool pred, uint32_t g, uint32_t* arr) {
    const uint64_t todo = __ballot(pred);
    if (!todo) return;
    const uint32_t leader = (uint32_t)__builtin_ctzll(todo);
    const uint32_t gl = __shfl(g, leader);
    if (__ballot(pred && g == gl) == todo) {
        if (lane_id() == leader) atomicAdd(&arr[gl], (uint32_t)__popcll(todo));
    } else if (pred) {
        atomicAdd(&arr[g], 1u);
    }
}

// ---- first digit of a key ----------------------------------------------------------
// The 31-bit key space is cut into 4096 consecutive intervals ("bins").
//   coarse (base = 0, shift = 19): bin = the key's top 12 bits (exponent + 4 mantissa bits).
//   fine (shift = 10), for a known lower bound `base` of the k-th key; rel = key - base
//   (0 for keys below base):
//     bins 0 .. 2047     rel < 2^21, 1024 keys each (bin 0 also takes every key below base);
//     bins 2048 .. 4095  eight octaves [2^e, 2^(e+1)) of rel, e = 21 .. 28, 256 bins each:
//                        the resolution falls off with the distance from the bound, the way
//                        the keys themselves thin out; the last bin is open-ended.
// lo() / width() give a bin's key interval; both layouts tile [0, 2^31) without gaps.
struct Digit {
    uint32_t base, shift;
    static constexpr uint32_t kLinBins = 2048, kLinLog2 = 21, kSubLog2 = 8, kTopOctave = 28;
    __host__ __device__ __forceinline__ uint32_t bin(uint32_t key) const {
        const uint32_t rel = key > base ? key - base : 0u;
        if (shift != (uint32_t)kFineShift || rel < (1u << kLinLog2)) {
            const uint32_t d = rel >> shift;
            return d < (uint32_t)kHistBins - 1 ? d : (uint32_t)kHistBins - 1;
        }
        const uint32_t e = 31u - (uint32_t)__builtin_clz(rel);
        if (e > kTopOctave) return (uint32_t)kHistBins - 1;
        return kLinBins + ((e - kLinLog2) << kSubLog2) + ((rel >> (e - kSubLog2)) & ((1u << kSubLog2) - 1u));
    }
    // distance from base to the smallest key of bin d
    __host__ __device__ __forceinline__ unsigned long long edge(uint32_t d) const {
        if (shift != (uint32_t)kFineShift || d <= kLinBins) return (unsigned long long)d << shift;
        const uint32_t o = d - kLinBins, e = kLinLog2 + (o >> kSubLog2);
        return (1ull << e) + ((unsigned long long)(o & ((1u << kSubLog2) - 1u)) << (e - kSubLog2));
    }
    // smallest key of bin d
    __host__ __device__ __forceinline__ uint32_t lo(uint32_t d) const {
        if (d == 0) return 0u;
        const unsigned long long v = (unsigned long long)base + edge(d);
        return v > 0x80000000ull ? 0x80000000u : (uint32_t)v;      // bins past 2^31 hold no key
    }
    // number of keys of bin d (<= 2^31)
    __host__ __device__ __forceinline__ uint32_t width(uint32_t d) const {
        if (d == (uint32_t)kHistBins - 1) return 0x80000000u - lo(d);
        return lo(d + 1) - lo(d);
    }
};
static_assert(Digit::kLinBins + ((Digit::kTopOctave - Digit::kLinLog2 + 1) << Digit::kSubLog2) == kHistBins,
              "the fine layout has exactly kHistBins bins");

// ---- clearing ----------------------------------------------------------------------

constexpr int kZeroSlots = 6;
struct ZeroJob { uint32_t* p[kZeroSlots]; size_t n[kZeroSlots]; };

// clears up to six arrays in one launch (an array with n == 0 is skipped)
__global__ void k_zero_u32(ZeroJob job) {
    const size_t step = (size_t)gridDim.x * blockDim.x;
    const size_t first = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
#pragma unroll
    for (int a = 0; a < kZeroSlots; ++a)
        for (size_t i = first; i < job.n[a]; i += step) job.p[a][i] = 0u;
}

}  // namespace gtopk
