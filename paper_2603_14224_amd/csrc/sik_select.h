// Level-1 selection histogram shared by the scoring kernel and the stand-alone top-k kernels:
// every workgroup publishes the histogram of its token chunk as packed 16-bit counts, and the last
// workgroup of a query head to arrive adds the chunks up and locates the threshold bin.
#pragma once

#include "sik_device.h"

namespace sik {

static_assert(kBins == 2 * kBlock, "one thread owns two adjacent histogram bins");
constexpr int kHistWords = kBins / 2;  // 32-bit words per (query head, chunk): bins 2w | 2w+1 << 16
constexpr int kMaxChunks = 64;         // chunks per query head in the histogram-producing kernels
constexpr int kMaxChunkTokens = 65535; // a 16-bit count per bin must hold a whole chunk

// thr[row] = { threshold bin b* (-1: select everything), tokens in bins above b*, tokens in b*, 0 }
struct Threshold {
    int bstar, cgt, nb;
};

// Publish this workgroup's LDS histogram (kBins 32-bit counts) of one query head.
__device__ __forceinline__ void publish_hist(const uint32_t* lhist, uint32_t* part) {
    const int t = threadIdx.x;
    st_agent(&part[t], lhist[2 * t] | (lhist[2 * t + 1] << 16));
}

// Inclusive suffix sum over the 256 threads of the workgroup (thread t gets sum over u >= t).
__device__ __forceinline__ uint32_t block_suffix_sum(uint32_t v, uint32_t* lds4) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = static_cast<uint32_t>(__shfl_down(static_cast<int>(v), o, 64));
        if (lane + o < 64) v += up;
    }
    __syncthreads();  // lds4 may still be read from an earlier call
    if (lane == 0) lds4[wv] = v;
    __syncthreads();
#pragma unroll
    for (int w = 1; w < kBlock / kWave; ++w)
        if (wv + w < kBlock / kWave) v += lds4[wv + w];
    return v;
}

// Called by all threads of the last workgroup of a query head: add up the `nact` published chunk
// histograms and find the bin where the count from the top reaches kk = min(k, L).
__device__ __forceinline__ void find_threshold(const uint32_t* part_row, int nact, int kk, int L,
                                               int32_t* thr_row, uint32_t* lds4) {
    const int t = threadIdx.x;
    if (kk >= L) {  // uniform
        if (t == 0) {
            thr_row[0] = -1;
            thr_row[1] = L;
            thr_row[2] = 0;
        }
        return;
    }
    uint32_t c0 = 0, c1 = 0;
#pragma unroll 8
    for (int cc = 0; cc < nact; ++cc) {
        const uint32_t v = ld_agent(&part_row[cc * kHistWords + t]);
        c0 += v & 0xffffu;
        c1 += v >> 16;
    }
    const uint32_t own = c0 + c1;
    uint32_t cum = block_suffix_sum(own, lds4) - own;  // tokens in bins owned by higher threads
    const uint32_t ukk = static_cast<uint32_t>(kk);
    if (cum < ukk && ukk <= cum + c1) {
        thr_row[0] = 2 * t + 1;
        thr_row[1] = static_cast<int32_t>(cum);
        thr_row[2] = static_cast<int32_t>(c1);
    }
    cum += c1;
    if (cum < ukk && ukk <= cum + c0) {
        thr_row[0] = 2 * t;
        thr_row[1] = static_cast<int32_t>(cum);
        thr_row[2] = static_cast<int32_t>(c0);
    }
}

}  // namespace sik
