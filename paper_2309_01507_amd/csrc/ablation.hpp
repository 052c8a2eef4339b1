// Stand-alone compress / decompress with the quantizers that the paper ablates for the second moment (Sec. 4.1,
// Tab. 1): block-wise normalization with block size 128 or 2048 or rank-1 normalization, the 4-bit
// dynamic-exponent map (unsigned for non-negative input, signed for signed input), the same map without its zero
// ("DE-0", 15 points) or the Linear map, rounding to the nearest entry or stochastic rounding (App. D.3).  None of
// them is on an optimizer step's path except B128 / signed DE, B128 / Linear and rank-1 / Linear, which the step
// kernels implement themselves; these kernels are for studying the quantizers on real tensors, so they are plain:
// a lane owns 8 consecutive elements, IEEE division, a linear scan of the table.
#pragma once

#include "kernels.hpp"

namespace lpmm {

struct AblMap {
    float T[kCodes];          // increasing; n entries
    float thr[kCodes - 1];    // largest float not above the midpoint of neighbouring entries
    int n;
};

struct AblArgs {
    const float* x_in;        // compress: input
    float* x_out;             // decompress: output
    const uint32_t* q_in;
    uint32_t* q_out;
    float* sa;                // block scales, or row maxima
    float* sb;                // column maxima (rank-1)
    int64_t rows, cols, P;
    int stochastic;
    uint64_t seed;
};

// nearest entry, ties to the lower index: the number of thresholds below n
__device__ __forceinline__ uint32_t abl_nearest(const AblMap& m, float n) {
    uint32_t c = 0;
    for (int k = 0; k + 1 < m.n; ++k) c += n > m.thr[k] ? 1u : 0u;
    return c;
}

// Uniform number of element `idx`: the top 24 bits of output number idx + 1 of the SplitMix64 generator started at
// `seed`, scaled to [0, 1).
__device__ __forceinline__ float abl_uniform(uint64_t seed, uint64_t idx) {
    uint64_t z = seed + (idx + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return float(uint32_t(z >> 40)) * 0x1p-24f;
}

// App. D.3: the candidates are the entry at or below n and the entry at or above it (counted, the table being
// increasing); one candidate if n is an entry or outside the table's range; else the upper one with probability
// (n - T[q1]) / (T[q2] - T[q1]), in fp32 with IEEE division.
__device__ __forceinline__ uint32_t abl_stochastic(const AblMap& m, float n, float u) {
    int le = 0, lt = 0;
    for (int i = 0; i < m.n; ++i) {
        le += m.T[i] <= n ? 1 : 0;
        lt += m.T[i] < n ? 1 : 0;
    }
    const int q1 = le - 1, q2 = lt;
    if (q1 < 0) return uint32_t(q2 < m.n ? q2 : 0);
    if (q2 >= m.n || q1 == q2) return uint32_t(q1);
    const float p = (n - m.T[q1]) / (m.T[q2] - m.T[q1]);
    return uint32_t(u < p ? q2 : q1);
}

__device__ __forceinline__ uint32_t abl_code(const AblMap& m, const AblArgs& a, float x, float s, int64_t idx) {
    const float n = (s == 0.0f) ? 0.0f : x / s;
    return a.stochastic ? abl_stochastic(m, n, abl_uniform(a.seed, uint64_t(idx))) : abl_nearest(m, n);
}

__device__ __forceinline__ void abl_load_map(AblMap& s_map, const AblMap& m) {
    if (threadIdx.x < kCodes) s_map.T[threadIdx.x] = m.T[threadIdx.x];
    if (threadIdx.x < kCodes - 1) s_map.thr[threadIdx.x] = m.thr[threadIdx.x];
    if (threadIdx.x == 0) s_map.n = m.n;
    __syncthreads();
}

// Block-wise normalization: a workgroup takes 2048 consecutive elements (one block of 2048, or 16 blocks of 128).
template <int BLOCK>
__global__ __launch_bounds__(kThreads) void abl_quant_block_kernel(const AblArgs a, const AblMap m) {
    static_assert(BLOCK == 128 || BLOCK == 2048, "block sizes of Tab. 1");
    __shared__ AblMap s_map;
    __shared__ float s_part[kThreads / 64];
    abl_load_map(s_map, m);
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(a.P, a.P, t);                 // flat: one row of P columns
    float x[8], amax = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        x[e] = e < io.nv ? a.x_in[io.base + e] : 0.0f;
        amax = fmaxf(amax, fabsf(x[e]));
    }
    float sc = row16_allmax(amax);                          // 16 lanes x 8 elements = 128
    if constexpr (BLOCK == 2048) {
        sc = fmaxf(sc, __shfl_xor(sc, 16));
        sc = fmaxf(sc, __shfl_xor(sc, 32));
        if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = sc;
        __syncthreads();
        sc = fmaxf(fmaxf(s_part[0], s_part[1]), fmaxf(s_part[2], s_part[3]));
    }
    uint32_t w = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (e < io.nv) w |= abl_code(s_map, a, x[e], sc, io.base + e) << (4 * e);
    if (io.nv) store_codes(a.q_out, io, w);
    if constexpr (BLOCK == 2048) {
        if (threadIdx.x == 0) a.sa[blockIdx.x] = sc;
    } else {
        if ((threadIdx.x & 15) == 0 && (t >> 4) * 128 < a.P) a.sa[t >> 4] = sc;
    }
}

// Rank-1 normalization, second stage: codes against min(r_i, c_j) (the maxima are complete in sa / sb)
__global__ __launch_bounds__(kThreads) void abl_quant_rank1_kernel(const AblArgs a, const AblMap m) {
    __shared__ AblMap s_map;
    abl_load_map(s_map, m);
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(a.P, a.cols, t);
    if (!io.nv) return;
    uint32_t w = 0;
    int64_t i = io.i, j = io.j;
    for (int e = 0; e < io.nv; ++e) {
        w |= abl_code(s_map, a, a.x_in[io.base + e], fminf(a.sa[i], a.sb[j]), io.base + e) << (4 * e);
        if (++j == a.cols) { j = 0; ++i; }
    }
    store_codes(a.q_out, io, w);
}

// norm: 0 = block 128, 1 = block 2048, 2 = rank-1
__global__ __launch_bounds__(kThreads) void abl_dequant_kernel(const AblArgs a, const AblMap m, int norm) {
    __shared__ AblMap s_map;
    abl_load_map(s_map, m);
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(a.P, a.cols, t);
    if (!io.nv) return;
    const uint32_t w = load_codes(a.q_in, io);
    int64_t i = io.i, j = io.j;
    for (int e = 0; e < io.nv; ++e) {
        const int64_t idx = io.base + e;
        const float s = norm == 2 ? fminf(a.sa[i], a.sb[j]) : a.sa[norm == 0 ? idx >> 7 : idx >> 11];
        const uint32_t q = (w >> (4 * e)) & 15u;
        a.x_out[idx] = (int(q) < s_map.n ? s_map.T[q] : 0.0f) * s;
        if (++j == a.cols) { j = 0; ++i; }
    }
}

}  // namespace lpmm
