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
constexpr int kChunkCap = 64512;       // largest chunk the plans hand out: a multiple of 1024 below kMaxChunkTokens
constexpr int kMaxLen = kMaxChunks * kChunkCap;  // longest context the chunk plans cover (4 128 768 tokens)

struct Threshold {
    int bstar;  // threshold bin, -1: every token is selected
    int cgt;    // tokens in bins above bstar (all of them selected)
    int nb;     // tokens inside bstar (candidates)
};

// Publish this workgroup's LDS histogram (kBins 32-bit counts) of one query head; the kernel that
// follows in the stream reads it.
__device__ __forceinline__ void publish_hist(const uint32_t* lhist, uint32_t* part) {
    const int t = threadIdx.x;
    part[t] = lhist[2 * t] | (lhist[2 * t + 1] << 16);
}

// Inclusive suffix sum over the 256 threads of the workgroup (thread t gets sum over u >= t).
__device__ __forceinline__ uint32_t block_suffix_sum(uint32_t v, uint32_t* lds4) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = static_cast<uint32_t>(__shfl_down(static_cast<int>(v), o, 64));
        if (lane + o < 64) v += up;
    }
    if (lane == 0) lds4[wv] = v;
    __syncthreads();
#pragma unroll
    for (int w = 1; w < kBlock / kWave; ++w)
        if (wv + w < kBlock / kWave) v += lds4[wv + w];
    return v;
}

// The chunk histograms of one query head, as four 128-bit loads per lane in flight at a time:
// wavefront w takes chunks w, w+4, ...; lane l the words 4l .. 4l+3 (bins 8l .. 8l+7).
struct HistLoads {
    uint32_t cnt[8];
};
__device__ __forceinline__ HistLoads load_chunk_hists(const uint32_t* part_row, int nact) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    HistLoads h;
#pragma unroll
    for (int e = 0; e < 8; ++e) h.cnt[e] = 0u;
    const uint4* p4 = reinterpret_cast<const uint4*>(part_row);
#pragma unroll 8
    for (int cc = wv; cc < nact; cc += kBlock / kWave) {
        const uint4 v = p4[cc * (kHistWords / 4) + lane];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            h.cnt[2 * e] += w[e] & 0xffffu;
            h.cnt[2 * e + 1] += w[e] >> 16;
        }
    }
    return h;
}

// Called by all threads: add the chunk histograms up and find the bin where the count from the
// top reaches kk = min(k, L).  red: LDS [4][kBins] words, lds4: LDS [4], sthr: LDS [3].
__device__ __forceinline__ Threshold find_threshold(const HistLoads& h, int kk, int L, uint32_t* red,
                                                    uint32_t* lds4, int* sthr) {
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    Threshold r;
    if (kk >= L) {  // uniform: everything is selected
        r.bstar = -1;
        r.cgt = L;
        r.nb = 0;
        return r;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[wv * kBins + lane * 8 + e] = h.cnt[e];
    __syncthreads();
    uint32_t c0 = 0, c1 = 0;
#pragma unroll
    for (int w = 0; w < kBlock / kWave; ++w) {
        c0 += red[w * kBins + 2 * t];
        c1 += red[w * kBins + 2 * t + 1];
    }
    const uint32_t own = c0 + c1;
    uint32_t cum = block_suffix_sum(own, lds4) - own;  // tokens in bins owned by higher threads
    const uint32_t ukk = static_cast<uint32_t>(kk);
    if (cum < ukk && ukk <= cum + c1) {
        sthr[0] = 2 * t + 1;
        sthr[1] = static_cast<int>(cum);
        sthr[2] = static_cast<int>(c1);
    }
    cum += c1;
    if (cum < ukk && ukk <= cum + c0) {
        sthr[0] = 2 * t;
        sthr[1] = static_cast<int>(cum);
        sthr[2] = static_cast<int>(c0);
    }
    __syncthreads();
    r.bstar = sthr[0];
    r.cgt = sthr[1];
    r.nb = sthr[2];
    return r;
}

// ---- level 2 fallback: radix select inside the threshold bin, one workgroup -----------------
// Picks the `need` largest (score, then smaller index) among {i < L : bin(s_i) == bstar} and
// writes their indices to out[0 .. need).  NT = threads of the workgroup (all of them call); COHERENT: the
// scores were written by other workgroups of this launch and are read with agent-scope loads.
// h256: LDS, 256 words; sh: LDS, 4 words.
// radix_select_members: the same with the membership test handed in (member(v): does a token with score v compete).
template <int NT, bool COHERENT, class Member>
__device__ inline void radix_select_members(const float* __restrict__ s, int L, Member member, int need,
                                            int32_t* __restrict__ out, uint32_t* h256, uint32_t* sh) {
    const int tid = threadIdx.x;
    auto score = [&](int i) { return COHERENT ? ld_agent(&s[i]) : s[i]; };
    uint32_t prefix = 0, mask = 0;
    uint32_t remaining = static_cast<uint32_t>(need);
    for (int pass = 3; pass >= 0; --pass) {
        if (tid < 256) h256[tid] = 0u;
        __syncthreads();
#pragma unroll 8
        for (int i = tid; i < L; i += NT) {
            const float v = score(i);
            const uint32_t key = float_to_key(v);
            if (member(v) && (key & mask) == prefix)
                atomicAdd(&h256[(key >> (8 * pass)) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t cum = 0;
            int dsel = 0;
            for (int dgt = 255; dgt >= 0; --dgt) {
                const uint32_t cnt = h256[dgt];
                if (cum < remaining && remaining <= cum + cnt) {
                    dsel = dgt;
                    break;
                }
                cum += cnt;
            }
            sh[0] = static_cast<uint32_t>(dsel);
            sh[1] = remaining - cum;
        }
        __syncthreads();
        prefix |= sh[0] << (8 * pass);
        mask |= 255u << (8 * pass);
        remaining = sh[1];
        __syncthreads();
    }
    // prefix is now the key of the need-th largest member; `remaining` members equal to it are
    // taken in increasing index order, every larger member is taken.
    const uint32_t tau = prefix, need_eq = remaining;
    const uint32_t n_gt = static_cast<uint32_t>(need) - need_eq;
    if (tid == 0) {
        sh[2] = 0u;  // running count of larger members written
        sh[3] = 0u;  // running count of equal members seen
    }
    __syncthreads();
    // larger members: any order, one barrier-free sweep
#pragma unroll 8
    for (int i = tid; i < L; i += NT) {
        const float v = score(i);
        if (member(v) && float_to_key(v) > tau) out[atomicAdd(&sh[2], 1u)] = i;
    }
    // equal members: the first need_eq of them in index order; tiles of NT tokens, stop when served
    constexpr int kWaves = NT / kWave;
    for (int base = 0; base < L && need_eq > 0u; base += NT) {
        const int i = base + tid;
        bool eq = false;
        if (i < L) {
            const float v = score(i);
            eq = member(v) && float_to_key(v) == tau;
        }
        const uint64_t bal = __ballot(eq);
        const int lane = tid & 63, wv = tid >> 6;
        if (lane == 0) h256[wv] = static_cast<uint32_t>(__popcll(bal));
        __syncthreads();
        uint32_t before = sh[3], total = sh[3];
        for (int w = 0; w < kWaves; ++w) {
            if (w < wv) before += h256[w];
            total += h256[w];
        }
        const uint32_t ord = before + static_cast<uint32_t>(__popcll(bal & ((1ull << lane) - 1ull)));
        if (eq && ord < need_eq) out[n_gt + ord] = i;
        __syncthreads();
        if (tid == 0) sh[3] = total;
        if (total >= need_eq) break;  // uniform: every thread computed the same total
    }
    __syncthreads();
}

template <int NT = kBlock, bool COHERENT = false>
__device__ inline void radix_select_in_bin(const float* __restrict__ s, int L, float lo, float scale, int bstar,
                                           int need, int32_t* __restrict__ out, uint32_t* h256, uint32_t* sh) {
    radix_select_members<NT, COHERENT>(s, L, [=](float v) { return score_bin(v, lo, scale) == bstar; }, need, out,
                                       h256, sh);
}

}  // namespace sik
