// One decode step in ONE launch on gfx950: append -> lookup tables -> LUT-GEMV scores -> per-head top-k ->
// sparse attention ("Compressed-Domain Top-k Retrieval" followed by softmax(q K_S^T / sqrt(d)) V_S of "Background
// and Preliminaries"), with the scores never leaving the chip.
//
// Workgroup (1024 threads, one per compute unit) = (sequence, KV head, block of up to 4 query heads, token chunk
// of 1024 (T + TL) tokens).  A thread scores T + TL tokens for the block's heads and KEEPS the fp32 scores on the
// chip: T tokens' in registers, TL tokens' in LDS.
//   1. tables in LDS, scan of the chunk's codes, one 512-bin LDS histogram per head (as in the scoring kernel);
//   2. chunks of one head block exchange their histograms through memory: publish, arrive on a counter, wait
//      until all active chunks arrived (a BOUNDED spin: on give-up the status word of the workspace is set and the
//      workgroup leaves), read the others' histograms; with a single chunk per head block there is nothing to
//      exchange and no wait;
//   3. every workgroup derives the head's threshold bin, classifies its scores from the registers, compacts the
//      selected tokens of each head into an LDS list (deterministic order) and gathers them at once: 16
//      wavefronts = (head, slice of the list); with one chunk the threshold bin's candidates are ranked before
//      the gather and join the list;
//   4. several chunks: chunk partials (m, l, o[D]) and the threshold-bin candidates go to memory; the last
//      workgroup of a head to arrive ranks the candidates exactly (score desc, index asc), attends the winners,
//      merges the partials and writes the row.
// Variants: KVQ gathers 128-byte records of the 2-bit cache and dequantises them in registers; FX runs the scan in
// 16-bit fixed point and gives exact scores only to the tokens within a guard band of the threshold bin.
// The launch must be co-resident when a head block has more than one chunk (its workgroups wait for each other):
// the host only takes this path when the grid fits the compute units.  An appended row needs no wait: its new
// length is published by the last workgroup of the sequence to leave.  Every counter the kernel uses is left at
// zero by its last user, so the workspace's sync words need zeroing only once (sik_workspace_init).
#include <atomic>
#include <climits>
// (This header holds the kernel and its launch switch; sik_step_bf16.hip and sik_step_f16.hip instantiate it.  The
// including file defines SIK_STEP_TL_SETTER, the name of its export for the debug timeline.)
#pragma once

#include <atomic>
#include <climits>

#include "sik_attn_core.h"
#include "sik_device.h"
#include "sik_internal.h"
#include "sik_kvq.h"
#include "sik_scan.h"
#include "sik_select.h"
#include "sik_step_args.h"

namespace sik {

SIK_TL_DEFINE(SIK_STEP_TL_SETTER)


// 128-bit coherent load as two 64-bit ones (agent scope: bypasses this XCD's non-coherent cache lines)
__device__ __forceinline__ uint4 ld_agent4(const uint32_t* p) {
    const uint64_t a = ld_agent(reinterpret_cast<const uint64_t*>(p));
    const uint64_t b = ld_agent(reinterpret_cast<const uint64_t*>(p) + 1);
    return make_uint4(static_cast<uint32_t>(a), static_cast<uint32_t>(a >> 32), static_cast<uint32_t>(b),
                      static_cast<uint32_t>(b >> 32));
}
__device__ __forceinline__ void st_agent4(uint4* p, uint4 v) {
    st_agent(reinterpret_cast<uint64_t*>(p), static_cast<uint64_t>(v.y) << 32 | v.x);
    st_agent(reinterpret_cast<uint64_t*>(p) + 1, static_cast<uint64_t>(v.w) << 32 | v.z);
}

// Thread 0 polls *word (coherent loads) until it reaches `target` or `limit` polls have gone by; every thread
// gets the verdict.  A failed wait sets bit `bit` of the status word.
__device__ __forceinline__ bool bounded_wait(const uint32_t* word, uint32_t target, int limit, uint32_t* status,
                                             uint32_t bit, int* lds_flag) {
    if (threadIdx.x == 0) {
        int ok = 0;
        for (int n = 0; n < limit; ++n) {
            if (ld_agent(word) >= target) {
                ok = 1;
                break;
            }
            __builtin_amdgcn_s_sleep(2);
        }
        if (!ok) __hip_atomic_fetch_or(status, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *lds_flag = ok;
    }
    __syncthreads();
    const bool ok = *lds_flag != 0;
    __syncthreads();
    return ok;
}

// Exclusive prefix sum over the 256 threads of a group (thread t gets the sum over u > t: a SUFFIX sum, as the
// threshold search counts from the top bin down).  Called by all 1024 threads; lds4: this group's four words.
__device__ __forceinline__ uint32_t group_suffix_sum(uint32_t v, uint32_t* lds4) {
    const int lane = threadIdx.x & 63, wl = (threadIdx.x >> 6) & 3;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = static_cast<uint32_t>(__shfl_down(static_cast<int>(v), o, 64));
        if (lane + o < 64) v += up;
    }
    if (lane == 0) lds4[wl] = v;
    __syncthreads();
#pragma unroll
    for (int w = 1; w < 4; ++w)
        if (wl + w < 4) v += lds4[wl + w];
    return v;
}

template <int DT, int ODT, int T, int TL, bool FX = false, bool KVQ = false, bool FORCED = false>
__global__ __launch_bounds__(kStepThreads) void step_kernel(
    // (the first 14 dwords arrive in scalar registers with the wavefront: what the first loads need comes first;
    // dims0 = Hkv | Hq << 16, dims1 = R | nhb << 8 | nchunk << 16 | stream << 24)
    const uint16_t* __restrict__ q, const float* __restrict__ codebook, const uint8_t* __restrict__ codes,
    uint32_t dims0, uint32_t dims1, int Lmax, int32_t* __restrict__ seq_len, const uint16_t* K, const uint16_t* V,
    const StepArgs a) {
    constexpr int TT = T + TL;  // tokens per thread: T with their scores in registers, TL with their scores in LDS
    constexpr int kChunk = kStepThreads * TT;
    static_assert(TT <= 32, "one mask bit per token of a thread");
    static_assert(!FX || TL == 0, "the 16-bit sums of the first pass all stay in registers");
    const int Hkv = dims0 & 0xffffu, Hq = dims0 >> 16;
    const int R = dims1 & 0xffu, nhb = (dims1 >> 8) & 0xffu, nchunk = (dims1 >> 16) & 0xffu;
    const bool stream = (dims1 >> 24) & 1u;
    extern __shared__ __align__(16) unsigned char dyn[];  // selected-token lists, then the arrays of the last phase
    __shared__ __align__(16) float lut[kG * 16 * kHB];
    __shared__ float qs[kHB][kD];
    __shared__ float bp[kHB][2];
    // first pass in 16-bit fixed point (FX): entries at the float4 table's stride, bin base and band per head
    __shared__ __align__(16) uint16_t lutx[FX ? kG * 16 * 8 : 8];
    __shared__ int bpx[kHB][3], sband[kHB][2];
    __shared__ uint32_t lhist[kHB * kBins];  // this chunk's histograms, later the heads' totals
    __shared__ __align__(16) uint8_t newcode[kCodeBytes];
    __shared__ uint32_t wcnt[kHB][kStepWaves];
    __shared__ uint32_t s_nsel[kHB], s_ncand[kHB], lds4[kHB][4];
    __shared__ int sthr[kHB][3], s_last[kHB], s_flag;
    __shared__ float sm[kStepWaves], sl[kStepWaves];
    __shared__ float sacc[kStepWaves][kD];
    __shared__ float pml[kHB][2][kMaxChunks];
    __shared__ uint32_t fbits[FORCED ? 20 * kStepThreads / 32 : 1];  // forced tokens of this chunk, one bit per token
    __shared__ int32_t s_fidx[FORCED ? kMaxForced : 1];              // forced tokens of the KV head, -1: names no token
    __shared__ uint32_t s_fcnt;

    SIK_TL(36);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, p = lane & 15;
    const int g = tid >> 8, gt = tid & (kGroupThreads - 1), wl = wv & 3;  // group = head slot of the last phases
    const int c = blockIdx.x % nchunk;
    const int u = blockIdx.x / nchunk;
    const int hb = u % nhb;
    const int unit = u / nhb;
    const int h = unit % Hkv, b = unit / Hkv;
    const int start = c * kChunk;
    const int hq0 = h * R + hb * kHB;
    const int nh = min(kHB, R - hb * kHB);
    const size_t row0 = static_cast<size_t>(b) * Hq + hq0;
    uint32_t* const status = a.sync;
    uint32_t* const rsync = a.sync + kSyncHeader + row0 * kSyncPerRow;  // this block's first head
    uint32_t* const ssync = a.sync + kSyncHeader + static_cast<size_t>(gridDim.x / (nchunk * nhb * Hkv)) * Hq * kSyncPerRow +
                            static_cast<size_t>(b) * kSyncPerSeq;

    // ---- 0. every global load that does not depend on another goes out now -----------------------------------
    const uint4* cp = reinterpret_cast<const uint4*>(codes + static_cast<size_t>(unit) * Lmax * kCodeBytes);
    const int cap_end = min(Lmax, start + kChunk);
    uint4 cur[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int i = start + j * kStepThreads + tid;
        cur[j] = (j < TT && i < cap_end) ? cp[i] : make_uint4(0u, 0u, 0u, 0u);
    }
    const float4 cj = tid < kG * 16 ? reinterpret_cast<const float4*>(codebook)[static_cast<size_t>(unit) * kG * 16 + tid]
                                    : make_float4(0.f, 0.f, 0.f, 0.f);
    if (tid < kHB * 16) {  // 16 lanes x 16 B per query row
        const int s = tid >> 4;
        float f[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (s < nh) widen8<DT>(reinterpret_cast<const uint4*>(q + (row0 + s) * kD)[p], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) qs[s][8 * p + e] = f[e];
    }
    // gather role of this wavefront: head gs, slice gj of its list (see step 3)
    const int nslice = kStepWaves / nh;
    const int gs = wv % nh, gj = wv / nh;
    const uint4 qraw = reinterpret_cast<const uint4*>(q + (row0 + gs) * kD)[p];
    float4 al0 = make_float4(0.f, 0.f, 0.f, 0.f), al1 = al0;  // KVQ: alpha of this lane's 8 channels
    if constexpr (KVQ) {
        al0 = reinterpret_cast<const float4*>(a.alpha + static_cast<size_t>(unit) * kD)[2 * p];
        al1 = reinterpret_cast<const float4*>(a.alpha + static_cast<size_t>(unit) * kD)[2 * p + 1];
    }
    for (int e = tid; e < kHB * kBins; e += kStepThreads) lhist[e] = 0u;
    uint4 knew = make_uint4(0u, 0u, 0u, 0u), vnew = make_uint4(0u, 0u, 0u, 0u);
    float m8[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (a.k_new && tid < 16) {
        knew = reinterpret_cast<const uint4*>(a.k_new + static_cast<size_t>(unit) * kD)[tid];
        vnew = reinterpret_cast<const uint4*>(a.v_new + static_cast<size_t>(unit) * kD)[tid];
        const float4 m0 = reinterpret_cast<const float4*>(a.mu + static_cast<size_t>(unit) * kD)[2 * tid];
        const float4 m1 = reinterpret_cast<const float4*>(a.mu + static_cast<size_t>(unit) * kD)[2 * tid + 1];
        m8[0] = m0.x, m8[1] = m0.y, m8[2] = m0.z, m8[3] = m0.w;
        m8[4] = m1.x, m8[5] = m1.y, m8[6] = m1.z, m8[7] = m1.w;
    }
    const int n_forced = FORCED ? a.n_forced : 0;  // (a variant of its own: the plain step carries none of this)
    int fi = -1;  // forced token of this KV head that thread tid looks after
    if (tid < n_forced) fi = a.forced_idx[static_cast<size_t>(unit) * n_forced + tid];
    int L = seq_len[b];
    L = L < 0 ? 0 : (L > Lmax ? Lmax : L);
    const bool appended = a.k_new != nullptr;
    int t_new = -1;
    if (appended && L < Lmax) {
        t_new = L;
        L += 1;
    }
    // The new length is published by the LAST workgroup of the sequence to leave the kernel (a counter every
    // workgroup adds to on its way out, whichever way): by then each of them has read the old one, and nobody waits.
    auto leave = [&]() {
        if (appended && tid == 0 &&
            atomic_add_u32(&ssync[0], 1u) == static_cast<uint32_t>(Hkv) * nhb * nchunk - 1u) {
            seq_len[b] = L;
            st_agent(&ssync[0], 0u);
        }
    };
    const int nact = L > 0 ? (L + kChunk - 1) / kChunk : 1;
    if (c >= nact) {  // no token of this chunk is valid (chunk 0 always runs: it owns the outputs of L = 0)
        leave();
        return;
    }
    const int end = min(L, start + kChunk);
    const bool holds_new = t_new >= start && t_new < start + kChunk;
    if ((holds_new || (n_forced > 0 && c == 0 && t_new >= 0)) && tid < 16) {
        // Every head block whose chunk holds the new row stores it (identical bytes), so that the gather below
        // never waits for another workgroup's store; write-through, because the last workgroup of a head may
        // gather it from another XCD.  Chunk 0 stores it too when there is a forced set, which may name it.
        float f[8];
        widen8<DT>(knew, f);
        uint32_t byte = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) byte |= (f[e] >= m8[e] ? 1u : 0u) << (7 - e);
        newcode[tid] = static_cast<uint8_t>(byte);
        const size_t rowi = static_cast<size_t>(unit) * Lmax + t_new;
        if constexpr (KVQ) {  // the row is stored as one record (tid = p here: alpha of the same 8 channels)
            const float ra[8] = {alpha_reciprocal(al0.x), alpha_reciprocal(al0.y), alpha_reciprocal(al0.z),
                                 alpha_reciprocal(al0.w), alpha_reciprocal(al1.x), alpha_reciprocal(al1.y),
                                 alpha_reciprocal(al1.z), alpha_reciprocal(al1.w)};
            const uint2 slot = kvq_make_slot<DT>(knew, vnew, m8, ra, tid);
            st_agent(reinterpret_cast<uint64_t*>(a.kvq_w + rowi * kRecSlots + tid),
                     static_cast<uint64_t>(slot.y) << 32 | slot.x);
        } else {
            st_agent4(reinterpret_cast<uint4*>(a.Kw + rowi * kD) + tid, knew);
            st_agent4(reinterpret_cast<uint4*>(a.Vw + rowi * kD) + tid, vnew);
        }
        if (hb == 0) a.codes_w[rowi * kCodeBytes + tid] = static_cast<uint8_t>(byte);
    }
    // Forced tokens take part in the attention of every head of the KV head whatever their scores and do not
    // compete: they are left out of the histograms and of the classification (one LDS bit per token of the chunk),
    // the budget and the competing population shrink by their number, and chunk 0 attends them.
    int nfv = 0, fpos = 0;
    if (n_forced > 0) {  // uniform
        for (int e = tid; e < kChunk / 32; e += kStepThreads) fbits[e] = 0u;
        const bool fv = fi >= 0 && fi < L;
        fi = fv ? fi : -1;
        if (tid < kMaxForced) s_fidx[FORCED ? tid : 0] = fi;
        const uint64_t bf = __ballot(fv);
        if (tid == 0) s_fcnt = static_cast<uint32_t>(__popcll(bf));  // (the set spans the first two wavefronts)
        nfv = __syncthreads_count(fv ? 1 : 0);
        fpos = __popcll(bf & ((1ull << lane) - 1ull)) + (wv == 1 ? static_cast<int>(s_fcnt) : 0);
        if (fv && fi >= start && fi < end)
            atomicOr(&fbits[FORCED ? (fi - start) >> 5 : 0], 1u << ((fi - start) & 31));
    }
    __syncthreads();
    SIK_TL(37);

    // ---- 1. Table^(g)[j] for the block's heads, bin bounds, scan ------------------------------------------------
    if (tid < kG * 16) {
        const int gg = tid >> 4;
        float o[kHB];
#pragma unroll
        for (int s = 0; s < kHB; ++s) {
            const float* qq = &qs[s][4 * gg];
            float x = qq[0] * cj.x;
            x = fmaf(qq[1], cj.y, x);
            x = fmaf(qq[2], cj.z, x);
            x = fmaf(qq[3], cj.w, x);
            o[s] = x;
        }
        *reinterpret_cast<float4*>(&lut[tid * 4]) = make_float4(o[0], o[1], o[2], o[3]);
    }
    __syncthreads();
    if (tid < kHB * 32) {  // bins over mean +- 4.5 sigma of the score of a key with uniform independent codes
        const int s = tid >> 5, gg = tid & 31;
        const float* lf = &lut[gg * 16 * kHB + s];
        float sum = 0.0f, sq = 0.0f;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float x = lf[((j + gg) & 15) * kHB];
            sum += x;
            sq = fmaf(x, x, sq);
        }
        float mean = sum * (1.0f / 16.0f);
        float var = fmaxf(sq * (1.0f / 16.0f) - mean * mean, 0.0f);
#pragma unroll
        for (int o = 16; o >= 1; o >>= 1) {
            mean += __shfl_xor(mean, o, 32);
            var += __shfl_xor(var, o, 32);
        }
        if (gg == 0) {
            const float span = 9.0f * sqrtf(var);
            bp[s][0] = mean - 0.5f * span;
            bp[s][1] = (span > 1e-30f && span < 3.0e38f) ? static_cast<float>(kBins) / span : 0.0f;
        }
        if constexpr (FX) {
            // Fixed-point table of head s: E[g][j] = round((T[g][j] - min_j T[g]) / delta), delta chosen so that the
            // sum F of 32 entries fits 16 bits.  With S the exact sum of the looked-up T's and c = sum_g min_j T[g]:
            // |S - (delta F + c)| <= 32 x 0.52 delta (rounding of the entries, and of their binary32 evaluation),
            // and the binary32 score differs from S by at most gam = 31 x 2^-24 x sum_g max_j |T[g][j]| (1 + 1e-5).
            // Hence F_a - F_b >= D = 2 G implies score_a > score_b, with G = ceil(17 + 1.01 gam / delta) + 1.
            float mn = 3.4028235e38f, mx = -3.4028235e38f, ma = 0.0f;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float x = lf[((j + gg) & 15) * kHB];
                mn = fminf(mn, x);
                mx = fmaxf(mx, x);
                ma = fmaxf(ma, fabsf(x));
            }
            float R = mx - mn, A = ma;
#pragma unroll
            for (int o = 16; o >= 1; o >>= 1) {
                R += __shfl_xor(R, o, 32);
                A += __shfl_xor(A, o, 32);
            }
            const float inv = (R > 1e-30f && R < 3.0e38f) ? 65495.0f / R : 0.0f;  // 1 / delta
            float sumE = 0.0f, sqE = 0.0f;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int jj = (j + gg) & 15;
                const float e = rintf((lf[jj * kHB] - mn) * inv);
                lutx[(gg * 16 + jj) * 8 + s] = static_cast<uint16_t>(static_cast<int>(e));
                sumE += e;
                sqE = fmaf(e, e, sqE);
            }
            float meanE = sumE * (1.0f / 16.0f);
            float varE = fmaxf(sqE * (1.0f / 16.0f) - meanE * meanE, 0.0f);
#pragma unroll
            for (int o = 16; o >= 1; o >>= 1) {
                meanE += __shfl_xor(meanE, o, 32);
                varE += __shfl_xor(varE, o, 32);
            }
            if (gg == 0) {
                const float gam = 31.0f * 5.9604645e-8f * A;
                const float G = fminf(ceilf(17.0f + 1.01f * gam * inv) + 1.0f, 1.0e6f);
                const int D = 2 * static_cast<int>(G);
                // 512 bins of 2^sh units around the mean of F over uniform codes, wide enough for +- 4.5 sigma:
                // bin = (F >> sh) - base (any choice is correct, this one keeps the band small); a band of m bins on
                // either side of the threshold bin covers every F within D of it
                const int wreq = static_cast<int>(fminf(9.0f * sqrtf(varE) * (1.0f / kBins), 60000.0f));
                const int sh = wreq <= 1 ? 0 : 32 - __clz(wreq - 1);
                bpx[s][0] = (static_cast<int>(meanE) >> sh) - kBins / 2;
                bpx[s][1] = (D - 1 + (1 << sh) - 1) >> sh;
                bpx[s][2] = sh;
            }
        }
    }
    __syncthreads();
    float blo[kHB], bscale[kHB], bshift[kHB];
    int base6[kHB], shx[kHB];  // FX: bin = (F >> shx) - base6
#pragma unroll
    for (int s = 0; s < kHB; ++s) {
        blo[s] = bp[s][0];
        bscale[s] = bp[s][1];
        bshift[s] = bin_shift(bp[s][0], bp[s][1]);
        base6[s] = FX ? bpx[s][0] : 0;
        shx[s] = FX ? bpx[s][2] : 0;
    }
    SIK_TL(38);
    // The scores of this thread's tokens stay on the chip: the first T tokens' in registers, the other TL tokens'
    // in LDS (one float4 = four heads per token; large batches need more tokens per thread than the registers hold).
    // dyn: [lists][candidate stage][LDS scores]; the arrays of the last phase reuse it from the start.
    uint16_t* const lists = reinterpret_cast<uint16_t*>(dyn);
    const size_t lists_bytes = (static_cast<size_t>(kHB) * a.listcap * 2 + 15) & ~size_t(15);
    uint64_t* const cstage = reinterpret_cast<uint64_t*>(dyn + lists_bytes);
    float4* const lsc = reinterpret_cast<float4*>(dyn + lists_bytes + static_cast<size_t>(kHB) * kCandCap * 8);
    float sc[T][kHB];
    uint32_t fx[FX ? TT : 1][2];  // FX: the 16-bit sums of a token, heads 0 | 1 << 16 and 2 | 3 << 16
    uint32_t livemask = 0u;       // FX: token slots that hold a competing token
#pragma unroll
    for (int it = 0; it < TT; ++it) {
        const int tok = start + it * kStepThreads + tid;
        uint4 code = cur[it & 1];
        if (it + 2 < TT) {
            const int i = tok + 2 * kStepThreads;
            cur[it & 1] = i < end ? cp[i] : make_uint4(0u, 0u, 0u, 0u);
        }
        if (tok == t_new) code = *reinterpret_cast<const uint4*>(newcode);
        // (token slot it of thread tid is token it * 1024 + tid of the chunk)
        const bool live =
            tok < end && !(n_forced > 0 && ((fbits[FORCED ? it * 32 + (tid >> 5) : 0] >> (tid & 31)) & 1u));
        if constexpr (FX) {
            // 8-byte entries, two packed 16-bit adds per lookup: half the adds and half the LDS bytes of the
            // fp32 scan; the sums only place the token in a bin (exact scores follow for the band, below)
            typedef unsigned short us2 __attribute__((ext_vector_type(2)));
            us2 a01 = {0, 0}, a23 = {0, 0};
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const uint32_t word = dw == 0 ? code.x : (dw == 1 ? code.y : (dw == 2 ? code.z : code.w));
                uint2 v[8];
                lookup_batch_x(word, dw, lutx, v);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int n = 0; n < 8; ++n) {
                    a01 += __builtin_bit_cast(us2, v[n].x);
                    a23 += __builtin_bit_cast(us2, v[n].y);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            const uint32_t w01 = __builtin_bit_cast(uint32_t, a01), w23 = __builtin_bit_cast(uint32_t, a23);
            fx[it][0] = w01;
            fx[it][1] = w23;
            livemask |= (live ? 1u : 0u) << it;
            if (live) {
#pragma unroll
                for (int s = 0; s < kHB; ++s) {
                    const uint32_t w = s < 2 ? w01 : w23;
                    const int f6 = static_cast<int>(((s & 1) ? w >> 16 : w & 0xffffu) >> shx[s]);
                    if (s < nh) atomicAdd(&lhist[s * kBins + min(max(f6 - base6[s], 0), kBins - 1)], 1u);
                }
            }
            continue;
        }
        float acc[kHB];
        if constexpr (TT < 6) {
            // the lookups run one 8-group batch ahead of the adds (8 to 16 LDS reads in flight per wavefront)
            float4 v[2][8];
            lookup_batch<kHB>(code.x, 0, lut, v[0]);
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                if (dw < 3)
                    lookup_batch<kHB>(dw == 0 ? code.y : (dw == 1 ? code.z : code.w), dw + 1, lut, v[(dw + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                add_batch<kHB>(dw == 0, v[dw & 1], acc);
#pragma unroll
                for (int s = 0; s < kHB; ++s) asm volatile("" : "+v"(acc[s]));
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            // many tokens per thread: their scores take half the registers, so half a batch at a time (the 16
            // wavefronts of the workgroup hide the LDS latency between them)
            float4 v[4];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const uint32_t word = dw == 0 ? code.x : (dw == 1 ? code.y : (dw == 2 ? code.z : code.w));
                lookup_half<0>(word, dw, lut, v);
                __builtin_amdgcn_sched_barrier(0);
                add_half(dw == 0, v, acc);
#pragma unroll
                for (int s = 0; s < kHB; ++s) asm volatile("" : "+v"(acc[s]));
                __builtin_amdgcn_sched_barrier(0);
                lookup_half<1>(word, dw, lut, v);
                __builtin_amdgcn_sched_barrier(0);
                add_half(false, v, acc);
#pragma unroll
                for (int s = 0; s < kHB; ++s) asm volatile("" : "+v"(acc[s]));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int s = 0; s < kHB; ++s) {
            if (live && s < nh)
                atomicAdd(&lhist[s * kBins + bin_of_coord(bin_coord_shifted(acc[s], bscale[s], bshift[s]))], 1u);
            // slots at or beyond the sequence's end and forced tokens hold NaN: every comparison of the
            // classification fails
            acc[s] = live ? acc[s] : __builtin_nanf("");
            if (it < T) sc[it < T ? it : 0][s] = acc[s];
        }
        if (it >= T) lsc[(it - T) * kStepThreads + tid] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    }
    __syncthreads();

    SIK_TL(39);
    // ---- 2. histograms of the head block's chunks -----------------------------------------------------------------
    const int Lc = L - nfv;           // tokens that compete
    const int kb = a.k_per_mille > 0
                       ? min(a.k, max(1, static_cast<int>((static_cast<int64_t>(L) * a.k_per_mille + 999) / 1000)))
                       : a.k;
    const int kk = max(0, min(kb - nfv, Lc));  // dynamic picks per head (the forced tokens may use up the budget)
    bool alive = true;
    if (nact > 1) {
        if (tid < kHistWords)
            for (int s = 0; s < nh; ++s)
                st_agent(&a.parthist[((row0 + s) * nchunk + c) * kHistWords + tid],
                         lhist[s * kBins + 2 * tid] | (lhist[s * kBins + 2 * tid + 1] << 16));
        __builtin_amdgcn_s_waitcnt(0);  // every store of this lane (also the new row's) has been acknowledged
        __syncthreads();
        if (tid == 0) atomic_add_u32(&rsync[3], 1u);
        SIK_TL(40);
        for (int e = tid; e < kHB * kBins; e += kStepThreads) lhist[e] = 0u;
        alive = bounded_wait(&rsync[3], static_cast<uint32_t>(nact), a.spin_limit, status, 1u, &s_flag);
        if (!alive) {  // uniform: the launch is lost, the status word says so
            leave();
            return;
        }
        SIK_TL(41);
        if (g < nh) {
            const uint32_t* prow = a.parthist + (row0 + g) * nchunk * kHistWords;
            uint32_t cnt[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll 4
            for (int cc = wl; cc < nact; cc += 4) {
                const uint4 x = ld_agent4(prow + cc * kHistWords + lane * 4);
                const uint32_t w4[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    cnt[2 * e] += w4[e] & 0xffffu;
                    cnt[2 * e + 1] += w4[e] >> 16;
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (cnt[e]) atomicAdd(&lhist[g * kBins + lane * 8 + e], cnt[e]);
        }
        __syncthreads();
    }
    // threshold bin of head g: the bin where the count from the top reaches kk (every chunk finds the same)
    {
        int bstar = -1, cgt = Lc, nb = 0;
        uint32_t c0 = 0, c1 = 0;
        if (g < nh) {
            c0 = lhist[g * kBins + 2 * gt];
            c1 = lhist[g * kBins + 2 * gt + 1];
        }
        const uint32_t own = c0 + c1;
        uint32_t cum = group_suffix_sum(own, lds4[g]) - own;  // tokens in bins owned by higher threads
        const uint32_t ukk = static_cast<uint32_t>(kk);
        if (g < nh && kk > 0 && kk < Lc) {
            if (cum < ukk && ukk <= cum + c1) bstar = 2 * gt + 1, cgt = static_cast<int>(cum), nb = static_cast<int>(c1);
            cum += c1;
            if (cum < ukk && ukk <= cum + c0) bstar = 2 * gt, cgt = static_cast<int>(cum), nb = static_cast<int>(c0);
            if (bstar >= 0) {
                if constexpr (FX) {
                    // the band: m bins on either side of the threshold bin; bins above it are selected outright,
                    // the band's tokens are scored exactly and ranked
                    const int m = bpx[g][1];
                    const int lo_b = max(bstar - m, 0), hi_b = min(bstar + m, kBins - 1);
                    int above = 0, band = 0;
                    for (int bb = lo_b; bb <= hi_b; ++bb) {
                        const int cnt = static_cast<int>(lhist[g * kBins + bb]);
                        band += cnt;
                        above += bb > bstar ? cnt : 0;
                    }
                    cgt -= above;
                    nb = band;
                    sband[g][0] = lo_b;
                    sband[g][1] = hi_b;
                }
                sthr[g][0] = bstar, sthr[g][1] = cgt, sthr[g][2] = nb;
            }
        } else if (gt == 0) {  // everything is selected (or nothing exists)
            sthr[g][0] = kk > 0 ? -1 : kBins;
            sthr[g][1] = kk > 0 ? Lc : 0;
            sthr[g][2] = 0;
        }
        if (tid < kHB) s_nsel[tid] = 0u, s_ncand[tid] = 0u;
    }
    __syncthreads();

    SIK_TL(42);
    // ---- 3. classify from the registers, compact per head, gather ---------------------------------------------------
    float hi_f[kHB], lo_f[kHB];
    bool has_cand[kHB], crowded[kHB];
#pragma unroll
    for (int s = 0; s < kHB; ++s) {
        const int bstar = sthr[s][0];
        // bin(s) > b*  <=>  x >= b* + 1 and bin(s) == b*  <=>  b* <= x < b* + 1 with x = bin_coord(s), the clamped
        // end bins taking everything beyond them
        hi_f[s] = bstar < 0 ? -3.4028235e38f : (bstar >= kBins - 1 ? INFINITY : static_cast<float>(bstar + 1));
        lo_f[s] = bstar <= 0 ? -3.4028235e38f : (bstar >= kBins ? INFINITY : static_cast<float>(bstar));
        has_cand[s] = s < nh && bstar >= 0 && bstar < kBins && sthr[s][2] <= kCandCap;
        crowded[s] = s < nh && bstar >= 0 && bstar < kBins && sthr[s][2] > kCandCap;
    }
    // Stage A: one branch-free pass over the thread's tokens marks, per head, the selected ones and the ones at or
    // above the candidate bound in two bit masks (bit = token slot): a few instructions per score (a branch per
    // score for the rare candidates measured 3 us slower on 16 tokens per thread).  A threshold bin too crowded to
    // rank (e.g. all scores equal) sends the head's scores to memory for the radix selection of the last phase.
    uint32_t smask[kHB] = {0u, 0u, 0u, 0u}, gmask[kHB] = {0u, 0u, 0u, 0u};
    if constexpr (FX) {
        // the same two masks from the 16-bit sums: selected = a bin above the band, candidate = a bin of the band
        // (compared as F >> sh against the bins' lower edges; the clamped end bins take everything beyond them)
        int thr_s[kHB], thr_c[kHB];
#pragma unroll
        for (int s = 0; s < kHB; ++s) {
            const int bstar = sthr[s][0];
            const bool in = bstar >= 0 && bstar < kBins;
            thr_s[s] = bstar < 0 ? INT_MIN : ((!in || sband[s][1] >= kBins - 1) ? INT_MAX : sband[s][1] + 1 + base6[s]);
            thr_c[s] = !in ? INT_MAX : (sband[s][0] <= 0 ? INT_MIN : sband[s][0] + base6[s]);
        }
#pragma unroll
        for (int it = 0; it < TT; ++it) {
#pragma unroll
            for (int s = 0; s < kHB; ++s) {
                const uint32_t w = fx[it][s >> 1];
                const int f6 = static_cast<int>(((s & 1) ? w >> 16 : w & 0xffffu) >> shx[s]);
                smask[s] |= (f6 >= thr_s[s] ? 1u : 0u) << it;
                gmask[s] |= (f6 >= thr_c[s] ? 1u : 0u) << it;
            }
        }
        // token slots at or beyond the sequence's end, and forced tokens, are in no mask
#pragma unroll
        for (int s = 0; s < kHB; ++s) {
            smask[s] &= livemask;
            gmask[s] &= livemask;
        }
        // a band too crowded to rank: the exact scores of its members go to memory for the radix selection of the
        // last phase, minus infinity for everything else
        if (crowded[0] || crowded[1] || crowded[2] || crowded[3]) {  // uniform
            for (int it = 0; it < TT; ++it) {
                const int tok = start + it * kStepThreads + tid;
                if (tok < end) {
                    const uint4 code = tok == t_new ? *reinterpret_cast<const uint4*>(newcode) : cp[tok];
#pragma unroll
                    for (int s = 0; s < kHB; ++s) {
                        if (crowded[s]) {
                            const bool member = ((gmask[s] & ~smask[s]) >> it) & 1u;
                            st_agent(&a.scores[(row0 + s) * a.sstride + tok], member ? exact_score(lut, code, s) : -INFINITY);
                        }
                    }
                }
            }
        }
    } else {
#pragma unroll
    for (int it = 0; it < TT; ++it) {
        float v4[kHB];
        if (it < T) {
#pragma unroll
            for (int s = 0; s < kHB; ++s) v4[s] = sc[it < T ? it : 0][s];
        } else {
            const float4 f = lsc[(it - T) * kStepThreads + tid];
            v4[0] = f.x, v4[1] = f.y, v4[2] = f.z, v4[3] = f.w;
        }
        const int tok = start + it * kStepThreads + tid;
#pragma unroll
        for (int s = 0; s < kHB; ++s) {
            const float x = bin_coord(v4[s], blo[s], bscale[s]);
            smask[s] |= (x >= hi_f[s] ? 1u : 0u) << it;
            gmask[s] |= (x >= lo_f[s] ? 1u : 0u) << it;
            if (crowded[s] && tok < end)  // (a forced token's NaN goes out as minus infinity: it does not compete)
                st_agent(&a.scores[(row0 + s) * a.sstride + tok], v4[s] == v4[s] ? v4[s] : -INFINITY);
        }
    }
    }
    SIK_TL(8);
    // Stage B: selected tokens per wavefront, in rounds of "every lane pops one mask bit" (as many rounds as the
    // busiest lane has selected tokens): ballots and scalar counts only
    const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
    for (int s = 0; s < kHB; ++s) {
        if (s >= nh) smask[s] = 0u;
        uint32_t m = smask[s], tot = 0u;
        while (true) {
            const uint64_t bal = __ballot(m != 0u);
            if (bal == 0ull) break;
            tot += static_cast<uint32_t>(__popcll(bal));
            m &= m - 1u;
        }
        if (lane == 0) wcnt[s][wv] = tot;
        // candidates (about one token in a thousand): popped from the mask one by one (a wavefront-uniform loop
        // over the holders with scalar branches to the score's register was measured slower: the scalar unit is
        // shared by the 16 wavefronts)
        uint32_t cm = has_cand[s] ? (gmask[s] & ~smask[s]) : 0u;
        while (cm != 0u) {
            const int it = __ffs(static_cast<int>(cm)) - 1;
            cm &= cm - 1u;
            const uint32_t tok = static_cast<uint32_t>(start + it * kStepThreads + tid);
            if constexpr (FX) {  // only the token is staged: its exact score follows below
                const uint32_t at = atomicAdd(&s_ncand[s], 1u);
                if (at < static_cast<uint32_t>(kCandCap)) cstage[s * kCandCap + at] = tok;
            } else {
                float v = 0.0f;
                if (it < T) {
#pragma unroll
                    for (int j = 0; j < T; ++j) v = it == j ? sc[j][s] : v;
                } else {
                    v = reinterpret_cast<const float*>(&lsc[(it - T) * kStepThreads + tid])[s];
                }
                const uint32_t at = atomicAdd(&s_ncand[s], 1u);
                if (at < static_cast<uint32_t>(kCandCap))
                    cstage[s * kCandCap + at] = static_cast<uint64_t>(float_to_key(v)) << 32 | (~tok);
            }
        }
    }
    SIK_TL(9);
    __syncthreads();
    SIK_TL(10);
    // FX: the band's tokens get their binary32 scores, one thread per (head, token): the same sum, in the same
    // order, as the fp32 scan computes, so every path ranks by the same bits.  The code loads go out here and are
    // used after the lists have been written.
    const bool rescore = FX && g < nh && sthr[g][0] >= 0 && sthr[g][0] < kBins && sthr[g][2] <= kCandCap;
    const int nres = rescore ? static_cast<int>(min(s_ncand[g], static_cast<uint32_t>(kCandCap))) : 0;
    int rtok = -1;
    uint4 rcode = make_uint4(0u, 0u, 0u, 0u);
    if (gt < nres) {
        rtok = static_cast<int>(cstage[g * kCandCap + gt]);
        rcode = rtok == t_new ? *reinterpret_cast<const uint4*>(newcode) : cp[rtok];
    }
    if (tid < kHB * kStepWaves) {  // per head: offsets of the wavefronts (one 16-lane row per head)
        const int s = tid >> 4, w = tid & 15;
        const uint32_t cnt = wcnt[s][w];
        uint32_t incl = cnt;
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
            const uint32_t dn = static_cast<uint32_t>(__shfl_up(static_cast<int>(incl), o, 16));
            if (w >= o) incl += dn;
        }
        wcnt[s][w] = incl - cnt;
        if (w == 15) s_nsel[s] = incl;
    }
    __syncthreads();
    // Stage C: the same rounds again, now writing (order: wavefront, round, lane: deterministic)
#pragma unroll
    for (int s = 0; s < kHB; ++s) {
        uint32_t m = smask[s];
        uint32_t base = wcnt[s][wv];
        while (true) {
            const bool has = m != 0u;
            const uint64_t bal = __ballot(has);
            if (bal == 0ull) break;
            const uint32_t at = base + static_cast<uint32_t>(__popcll(bal & lt_mask));
            if (has && at < static_cast<uint32_t>(a.listcap))
                lists[s * a.listcap + at] = static_cast<uint16_t>((__ffs(static_cast<int>(m)) - 1) * kStepThreads + tid);
            base += static_cast<uint32_t>(__popcll(bal));
            m &= m - 1u;
        }
    }
    if constexpr (FX) {
        for (int j = gt; j < nres; j += kGroupThreads) {
            if (j != gt) {
                rtok = static_cast<int>(cstage[g * kCandCap + j]);
                rcode = rtok == t_new ? *reinterpret_cast<const uint4*>(newcode) : cp[rtok];
            }
            cstage[g * kCandCap + j] = static_cast<uint64_t>(float_to_key(exact_score(lut, rcode, g))) << 32 |
                                       (~static_cast<uint32_t>(rtok));
        }
    }
    __syncthreads();
    SIK_TL(11);
    // One active chunk: this workgroup owns its heads outright.  The threshold-bin candidates are ranked now (by
    // counting, keys are distinct) and the winners join the lists, so that one gather covers the head and the last
    // phase has nothing left to select.
    const bool sole = nact == 1;  // uniform
    const bool fast = sole && !(crowded[0] || crowded[1] || crowded[2] || crowded[3]);
    if (sole) {
        uint32_t add = 0u;
        if (g < nh) {
            const int bstar = sthr[g][0], need = kk - min(sthr[g][1], kk);
            if (bstar >= 0 && bstar < kBins && need > 0 && sthr[g][2] <= kCandCap) {
                const int ncand = static_cast<int>(min(s_ncand[g], static_cast<uint32_t>(kCandCap)));
                const uint64_t* const cg = cstage + g * kCandCap;
                const uint32_t nsel = s_nsel[g];
                for (int x0 = gt; x0 < ncand; x0 += kGroupThreads) {
                    const uint64_t me = cg[x0];
                    uint32_t rank = 0u;
                    for (int x = 0; x < ncand; x += 8) {  // (kCandCap is a multiple of 8: the reads stay inside cg)
                        uint64_t o8[8];
#pragma unroll
                        for (int y = 0; y < 8; ++y) o8[y] = cg[x + y];
#pragma unroll
                        for (int y = 0; y < 8; ++y) rank += (x + y < ncand && o8[y] > me) ? 1u : 0u;
                    }
                    if (rank < static_cast<uint32_t>(need) && nsel + rank < static_cast<uint32_t>(a.listcap))
                        lists[g * a.listcap + nsel + rank] =
                            static_cast<uint16_t>(static_cast<int>(~static_cast<uint32_t>(me)) - start);
                }
                add = static_cast<uint32_t>(min(need, ncand));
            }
        }
        __syncthreads();
        if (g < nh && gt == 0) s_nsel[g] += add;
        __syncthreads();
    }
    SIK_TL(43);
    // reservations in the head's index output and candidate area (several chunks only), issued before the gather
    // hides their round trip
    uint32_t my_res = 0u;
    if (nact > 1 && tid < 2 * nh) {
        const int s = tid >> 1;
        if ((tid & 1) == 0) {
            if (a.idx_out && s_nsel[s]) my_res = atomic_add_u32(&rsync[s * kSyncPerRow + 1], s_nsel[s]);
        } else {
            const uint32_t nc = min(s_ncand[s], static_cast<uint32_t>(kCandCap));
            if (nc) my_res = atomic_add_u32(&rsync[s * kSyncPerRow + 2], nc);
        }
    }
    const uint4* Kp = KVQ ? nullptr : reinterpret_cast<const uint4*>(K + static_cast<size_t>(unit) * Lmax * kD);
    const uint4* Vp = KVQ ? nullptr : reinterpret_cast<const uint4*>(V + static_cast<size_t>(unit) * Lmax * kD);
    const uint2* Rp = KVQ ? a.kvq + static_cast<size_t>(unit) * Lmax * kRecSlots : nullptr;
    const float al8[8] = {al0.x, al0.y, al0.z, al0.w, al1.x, al1.y, al1.z, al1.w};
    SoftmaxState st;
    init_state(st);
    if (gj < nslice) {
        const int n = min(static_cast<int>(s_nsel[gs]), a.listcap);
        const uint16_t* lst = lists + gs * a.listcap;
        auto fetch = [&](int j) { return start + static_cast<int>(lst[j]); };
        if constexpr (KVQ)  // records: 32 entries per wavefront step, dequantised in registers
            attend_list_q2(fetch, n, gj * 32, nslice * 32, Rp, q2_prepare<DT>(qraw, al8), a.scale_log2e, Lmax, st);
        else if (stream)
            attend_list<DT, true>(fetch, n, gj * 16, nslice * 16, Kp, Vp, qraw, a.scale_log2e, Lmax, st);
        else
            attend_list<DT, false>(fetch, n, gj * 16, nslice * 16, Kp, Vp, qraw, a.scale_log2e, Lmax, st);
        // chunk 0 also attends the forced tokens of the KV head: from the cache like any other row, or, given as
        // 16-bit side rows beside the 2-bit cache, with each logit shifted by -q . mu (the records they share the
        // softmax with hold the centred key)
        if (n_forced > 0 && c == 0) {
            if (KVQ && a.fK != nullptr) {
                float qf[8];
                widen8<DT>(qraw, qf);
                const float4 m0 = reinterpret_cast<const float4*>(a.mu + static_cast<size_t>(unit) * kD)[2 * p];
                const float4 m1 = reinterpret_cast<const float4*>(a.mu + static_cast<size_t>(unit) * kD)[2 * p + 1];
                const float mu_dot = qf[0] * m0.x + qf[1] * m0.y + qf[2] * m0.z + qf[3] * m0.w + qf[4] * m1.x +
                                     qf[5] * m1.y + qf[6] * m1.z + qf[7] * m1.w;
                const float zbias = -row16_sum(mu_dot) * a.scale_log2e;
                attend_list<DT, false>([&](int j) { return s_fidx[j] >= 0 ? j : -1; }, n_forced, gj * 16, nslice * 16,
                                       reinterpret_cast<const uint4*>(a.fK + static_cast<size_t>(unit) * n_forced * kD),
                                       reinterpret_cast<const uint4*>(a.fV + static_cast<size_t>(unit) * n_forced * kD),
                                       qraw, a.scale_log2e, n_forced, st, zbias);
            } else if constexpr (KVQ) {
                attend_list_q2([&](int j) { return s_fidx[j]; }, n_forced, gj * 32, nslice * 32, Rp,
                               q2_prepare<DT>(qraw, al8), a.scale_log2e, Lmax, st);
            } else {
                attend_list<DT, false>([&](int j) { return s_fidx[j]; }, n_forced, gj * 16, nslice * 16, Kp, Vp, qraw,
                                       a.scale_log2e, Lmax, st);
            }
        }
    }
    SIK_TL(44);
    // the four 16-lane rows of a wavefront hold four partial softmaxes; then the wavefronts of a head
    merge_from_lane(st, 16);
    merge_from_lane(st, 32);
    if ((lane >> 4) == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sacc[wv][8 * p + e] = st.acc[e];
        if (p == 0) {
            sm[wv] = st.m;
            sl[wv] = st.l;
        }
    }
    __syncthreads();
    if (nact > 1 && tid < 2 * nh) wcnt[tid >> 1][tid & 1] = my_res;  // [s][0] index-output base, [s][1] candidate base
    // partial of (head g, this chunk): thread gt < kD of group g holds o[gt]
    float M = kNegBig, Lsum = 0.0f, o = 0.0f;
    if (g < nh) {
        for (int w = g; w < nslice * nh; w += nh) M = fmaxf(M, sm[w]);
        for (int w = g; w < nslice * nh; w += nh) {
            const float f = fast_exp2(sm[w] - M);
            Lsum += sl[w] * f;
            if (gt < kD) o += sacc[w][gt] * f;
        }
    }
    __syncthreads();
    const int cgt_g = g < nh ? sthr[g][1] : 0, nb_g = g < nh ? sthr[g][2] : 0, bstar_g = g < nh ? sthr[g][0] : kBins;
    const bool ranked_g = nb_g <= kCandCap;
    const int need_g = g < nh ? kk - min(cgt_g, kk) : 0;
    // index row of head g: the forced tokens first (written by chunk 0), then the selected ones, then the winners
    // among the candidates; orow starts behind the forced ones and has kfree slots
    int32_t* const orow = (a.idx_out && g < nh) ? a.idx_out + (row0 + g) * a.k + nfv : nullptr;
    const int kfree = a.k - nfv;
    if (a.idx_out && c == 0 && tid < n_forced && fi >= 0)
        for (int s = 0; s < nh; ++s) a.idx_out[(row0 + s) * a.k + fpos] = fi;
    if (orow) {  // the selected tokens of this chunk (any order inside the row)
        const uint32_t base = nact > 1 ? wcnt[g][0] : 0u;
        const int n = min(static_cast<int>(s_nsel[g]), a.listcap);
        for (int j = gt; j < n; j += kGroupThreads)
            if (base + j < static_cast<uint32_t>(kfree)) orow[base + j] = start + static_cast<int>(lists[g * a.listcap + j]);
    }
    bool mine = g < nh;  // does this workgroup finish head g?
    float* const prow = a.partial + ((row0 + g) * kMaxChunks) * kPartStride;
    uint64_t* const pool = reinterpret_cast<uint64_t*>(a.pool) + (row0 + g) * kCandCap;
    if (nact > 1) {
        if (g < nh) {
            if (gt < kD) st_agent(&prow[static_cast<size_t>(c) * kPartStride + 2 + gt], o);
            if (gt == 0) {
                st_agent(&prow[static_cast<size_t>(c) * kPartStride], M);
                st_agent(&prow[static_cast<size_t>(c) * kPartStride + 1], Lsum);
            }
            if (ranked_g) {
                const uint32_t base = wcnt[g][1];
                const uint32_t nc = min(s_ncand[g], static_cast<uint32_t>(kCandCap));
                for (uint32_t j = gt; j < nc; j += kGroupThreads)
                    if (base + j < static_cast<uint32_t>(kCandCap)) st_agent(&pool[base + j], cstage[g * kCandCap + j]);
            }
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        SIK_TL(45);
        if (tid < nh) s_last[tid] = atomic_add_u32(&rsync[tid * kSyncPerRow], 1u) == static_cast<uint32_t>(nact) - 1u;
        __syncthreads();
        mine = g < nh && s_last[g] != 0;
        bool any = false;
        for (int s = 0; s < nh; ++s) any |= s_last[s] != 0;
        if (!any) {  // uniform
            leave();
            return;
        }
    }

    const size_t row = row0;  // (timeline marks of the workgroup that finishes the first head block)
    (void)row;
    if (fast) {  // uniform: everything selected has been gathered, the partial of step 3 is the result
        if (g < nh && gt < kD) store_out<ODT>(a.out, (row0 + g) * kD + gt, Lsum > 0.0f ? o / Lsum : 0.0f);
        if (orow)
            for (int j = kk + gt; j < kfree; j += kGroupThreads) orow[j] = -1;
        SIK_TL_ANY(47);
    } else {
    SIK_TL_ANY(46);
    // ---- 4. last workgroup of head g: candidates, merge, output (groups of 256 threads side by side; every
    // barrier below is reached by all 1024 threads) ---------------------------------------------------------------
    // LDS of this phase (the lists are dead): per group kCandCap + 8 sort keys, kCandCap ranks, kCandCap winners
    uint64_t* const lc = reinterpret_cast<uint64_t*>(dyn) + g * (kCandCap + 8);
    uint32_t* const rank_base = reinterpret_cast<uint32_t*>(reinterpret_cast<uint64_t*>(dyn) + kHB * (kCandCap + 8));
    uint32_t* const rank_of = rank_base + g * 2 * kCandCap;
    int32_t* const chosen = reinterpret_cast<int32_t*>(rank_of + kCandCap);
    const bool do_rank = !sole && mine && need_g > 0 && ranked_g && bstar_g >= 0 && bstar_g < kBins;
    const int ncand = do_rank ? min(nb_g, kCandCap) : 0;
    constexpr int kOPre = 8;
    float o_pre[kOPre], pm = kNegBig, pl = 0.0f;
    uint64_t cin[kCandCap / kGroupThreads];
    if (nact > 1) {
        if (mine && gt < nact) {
            pm = ld_agent(&prow[static_cast<size_t>(gt) * kPartStride]);
            pl = ld_agent(&prow[static_cast<size_t>(gt) * kPartStride + 1]);
        }
#pragma unroll
        for (int s2 = 0; s2 < kOPre; ++s2)
            o_pre[s2] = (mine && gt < kD && s2 < nact) ? ld_agent(&prow[static_cast<size_t>(s2) * kPartStride + 2 + gt]) : 0.0f;
#pragma unroll
        for (int e = 0; e < kCandCap / kGroupThreads; ++e) {
            const int j = gt + e * kGroupThreads;
            cin[e] = j < ncand ? ld_agent(&pool[j]) : 0ull;
        }
    } else {
#pragma unroll
        for (int e = 0; e < kCandCap / kGroupThreads; ++e) {
            const int j = gt + e * kGroupThreads;
            cin[e] = j < ncand ? cstage[g * kCandCap + j] : 0ull;
        }
    }
    __syncthreads();  // the candidate stage and the lists may be overwritten from here on
    if (nact > 1 && mine && gt < kMaxChunks) {
        pml[g][0][gt] = pm;
        pml[g][1][gt] = pl;
    }
    // ranking by counting, as many threads per candidate as the group has to spare
    const int Pn = ncand <= 64 ? 4 : (ncand <= 128 ? 2 : 1);
    const int slice = ((ncand + Pn - 1) / Pn + 7) & ~7;
#pragma unroll
    for (int e = 0; e < kCandCap / kGroupThreads; ++e) {
        const int j = gt + e * kGroupThreads;
        if (j < ncand) {
            lc[j] = cin[e];
            rank_of[j] = 0u;
        } else if (j < Pn * slice && j < kCandCap + 8) {
            lc[j] = 0ull;  // padding: the smallest key, outranks nothing
        }
    }
    __syncthreads();
    if (do_rank) {
        const int per = kGroupThreads / Pn, part = gt / per;
        for (int x0 = gt % per; x0 < ncand; x0 += per) {
            const uint64_t me = lc[x0];
            uint32_t rank = 0;
            for (int x = part * slice; x < min((part + 1) * slice, kCandCap + 8); x += 8) {
                uint64_t o8[8];
#pragma unroll
                for (int y = 0; y < 8; ++y) o8[y] = lc[x + y];
#pragma unroll
                for (int y = 0; y < 8; ++y) rank += o8[y] > me ? 1u : 0u;
            }
            if (Pn > 1) atomicAdd(&rank_of[x0], rank); else rank_of[x0] = rank;
        }
    }
    __syncthreads();
    if (do_rank) {
        for (int x0 = gt; x0 < ncand; x0 += kGroupThreads) {
            const int rank = static_cast<int>(rank_of[x0]);
            if (rank < need_g) {
                const int32_t ia = static_cast<int32_t>(~static_cast<uint32_t>(lc[x0]));
                chosen[rank] = ia;
                if (orow) orow[cgt_g + rank] = ia;
            }
        }
    }
    __syncthreads();
    // crowded bins: exact radix selection over the head's scores in memory, one head at a time, whole workgroup;
    // the winners go to the head's index row in memory (there may be more of them than the LDS list holds)
    for (int s = 0; s < nh; ++s) {
        const int need_s = kk - min(sthr[s][1], kk);
        const bool todo = (nact > 1 ? s_last[s] != 0 : true) && sthr[s][2] > kCandCap && sthr[s][0] >= 0 &&
                          sthr[s][0] < kBins && need_s > 0;
        if (todo) {  // uniform
            int32_t* dst = (a.idx_out ? a.idx_out : a.idx_ws) + (row0 + s) * a.k + nfv + sthr[s][1];
            __builtin_amdgcn_s_waitcnt(0);
            __syncthreads();
            if constexpr (FX)
                radix_select_members<kStepThreads, true>(a.scores + (row0 + s) * a.sstride, L,
                                                         [](float v) { return v > -INFINITY; }, need_s, dst, lhist,
                                                         &lds4[0][0]);
            else
                radix_select_members<kStepThreads, true>(
                    a.scores + (row0 + s) * a.sstride, L,
                    [lo = blo[s], sc_ = bscale[s], bst = sthr[s][0]](float v) {
                        return v > -INFINITY && score_bin(v, lo, sc_) == bst;
                    },
                    need_s, dst, lhist, &lds4[0][0]);
            __threadfence_block();
            __syncthreads();
        }
    }
    SoftmaxState st2;
    init_state(st2);
    const bool radix_g = mine && need_g > 0 && !ranked_g && bstar_g >= 0 && bstar_g < kBins;
    if (mine && need_g > 0) {
        const uint4 qg = reinterpret_cast<const uint4*>(q + (row0 + g) * kD)[p];
        const int32_t* gl = (a.idx_out ? a.idx_out : a.idx_ws) + (row0 + g) * a.k + nfv + cgt_g;
        if constexpr (KVQ) {
            const Q2Query qq = q2_prepare<DT>(qg, al8);
            if (do_rank)
                attend_list_q2([&](int j) { return chosen[j]; }, min(need_g, ncand), wl * 32, 128, Rp, qq,
                               a.scale_log2e, Lmax, st2);
            else if (radix_g)
                attend_list_q2([&](int j) { return gl[j]; }, need_g, wl * 32, 128, Rp, qq, a.scale_log2e, Lmax, st2);
        } else if (do_rank) {
            attend_list<DT, false>([&](int j) { return chosen[j]; }, min(need_g, ncand), wl * 16, 64, Kp, Vp, qg,
                                   a.scale_log2e, Lmax, st2);
        } else if (radix_g) {
            attend_list<DT, false>([&](int j) { return gl[j]; }, need_g, wl * 16, 64, Kp, Vp, qg, a.scale_log2e, Lmax,
                                   st2);
        }
    }
    merge_from_lane(st2, 16);
    merge_from_lane(st2, 32);
    __syncthreads();  // sacc / sm / sl of step 3 have been read
    if ((lane >> 4) == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sacc[wv][8 * p + e] = st2.acc[e];
        if (p == 0) {
            sm[wv] = st2.m;
            sl[wv] = st2.l;
        }
    }
    __syncthreads();
    if (mine && gt < kD) {
        float M2 = kNegBig, L2 = 0.0f, o2 = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) M2 = fmaxf(M2, sm[4 * g + w]);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float f = fast_exp2(sm[4 * g + w] - M2);
            L2 += sl[4 * g + w] * f;
            o2 += sacc[4 * g + w][gt] * f;
        }
        float Mg = M2, lt, ot;
        if (nact > 1) {  // chunk partials in chunk order: the result does not depend on the arrival order
#pragma unroll 8
            for (int s2 = 0; s2 < nact; ++s2) Mg = fmaxf(Mg, pml[g][0][s2]);
            const float a2 = fast_exp2(M2 - Mg);
            lt = L2 * a2, ot = o2 * a2;
#pragma unroll
            for (int s2 = 0; s2 < kOPre; ++s2) {
                if (s2 < nact) {
                    const float f = fast_exp2(pml[g][0][s2] - Mg);
                    lt += pml[g][1][s2] * f;
                    ot += o_pre[s2] * f;
                }
            }
#pragma unroll 8
            for (int s2 = kOPre; s2 < nact; ++s2) {
                const float f = fast_exp2(pml[g][0][s2] - Mg);
                lt += pml[g][1][s2] * f;
                ot += ld_agent(&prow[static_cast<size_t>(s2) * kPartStride + 2 + gt]) * f;
            }
        } else {  // one chunk: the partial of step 3 is in this thread's registers
            Mg = fmaxf(M2, M);
            const float a2 = fast_exp2(M2 - Mg), a1 = fast_exp2(M - Mg);
            lt = L2 * a2 + Lsum * a1;
            ot = o2 * a2 + o * a1;
        }
        store_out<ODT>(a.out, (row0 + g) * kD + gt, lt > 0.0f ? ot / lt : 0.0f);
    }
    if (mine && orow)
        for (int j = kk + gt; j < kfree; j += kGroupThreads) orow[j] = -1;
    SIK_TL_ANY(47);
    }
    // leave the head's counters at zero for the next call; the block's first head also clears the arrival counter
    if (mine && nact > 1 && gt == 0) {
        st_agent(&rsync[g * kSyncPerRow + 0], 0u);
        st_agent(&rsync[g * kSyncPerRow + 1], 0u);
        st_agent(&rsync[g * kSyncPerRow + 2], 0u);
        if (g == 0) st_agent(&rsync[3], 0u);
    }
    leave();
}


template <int DT, int ODT>
static hipError_t launch_step_t(const Dims& d, int T, int nchunk, size_t dyn, const void* q, const float* codebook,
                                const uint8_t* codes, int32_t* seq_len, const void* K, const void* V,
                                const StepArgs& a, hipStream_t s) {
    const int nhb = (d.R + kHB - 1) / kHB;
    const int grid = d.units() * nhb * nchunk;
    const uint32_t dims0 = static_cast<uint32_t>(d.Hkv) | static_cast<uint32_t>(d.Hq) << 16;
    const uint32_t dims1 = static_cast<uint32_t>(d.R) | static_cast<uint32_t>(nhb) << 8 |
                           static_cast<uint32_t>(nchunk) << 16 | (gather_streams(d, a.k) ? 1u << 24 : 0u);
    auto qp = static_cast<const uint16_t*>(q);
    auto Kp = static_cast<const uint16_t*>(K);
    auto Vp = static_cast<const uint16_t*>(V);
#define SIK_STEP(TV, TLV) SIK_STEP_(TV * 100 + TLV, TV, TLV, false, false, false)
#define SIK_STEP_Q2(TV, TLV) SIK_STEP_(kStepQ2Code + TV * 100 + TLV, TV, TLV, false, true, false)
#define SIK_STEP_F(TV, TLV)                                                 \
    SIK_STEP_(kStepFCode + TV * 100 + TLV, TV, TLV, false, false, true)     \
    SIK_STEP_(kStepFCode + kStepQ2Code + TV * 100 + TLV, TV, TLV, false, true, true)
#define SIK_STEP_FX(TV) SIK_STEP_(kStepFxCode + TV * 100, TV, 0, true, false, false)
#define SIK_STEP_(CODE, TV, TLV, FXV, Q2V, FV)                                                                  \
    case CODE: {                                                                                                \
        auto kern = step_kernel<DT, ODT, TV, TLV, FXV, Q2V, FV>;                                                  \
        static std::atomic<size_t> allowed{0};                                                                  \
        if (dyn > allowed.load(std::memory_order_relaxed)) {                                                    \
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                       \
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,                \
                                                     static_cast<int>(kStepLdsBudget));                         \
            if (e != hipSuccess) return e;                                                                      \
            allowed.store(kStepLdsBudget, std::memory_order_relaxed);                                           \
        }                                                                                                       \
        return launch_kernel(kern, grid, kStepThreads, s, qp, codebook, codes, dims0, dims1, d.Lmax, seq_len, Kp, Vp, \
                             a, dyn);                                                                           \
    }
    constexpr int kStepQ2Code = 200000, kStepFCode = 400000;
    switch ((a.kvq ? kStepQ2Code : 0) + (a.n_forced > 0 ? kStepFCode : 0) + T) {
        SIK_STEP(1, 0)
        SIK_STEP(2, 0)
        SIK_STEP(3, 0)
        SIK_STEP(4, 0)
        SIK_STEP(6, 0)
        SIK_STEP(8, 0)
        SIK_STEP(12, 0)
        SIK_STEP(12, 4)
        SIK_STEP(14, 4)
        SIK_STEP(16, 4)
        SIK_STEP_FX(4)
        SIK_STEP_FX(8)
        SIK_STEP_FX(12)
        SIK_STEP_FX(16)
        SIK_STEP_FX(20)
        SIK_STEP_Q2(1, 0)
        SIK_STEP_Q2(4, 0)
        SIK_STEP_Q2(12, 0)
        SIK_STEP_Q2(12, 4)
        SIK_STEP_Q2(14, 4)
        SIK_STEP_Q2(16, 4)
        SIK_STEP_F(1, 0)
        SIK_STEP_F(4, 0)
        SIK_STEP_F(12, 0)
        SIK_STEP_F(12, 4)
        SIK_STEP_F(14, 4)
        SIK_STEP_F(16, 4)
        default: return hipErrorInvalidValue;
    }
#undef SIK_STEP
#undef SIK_STEP_Q2
#undef SIK_STEP_F
#undef SIK_STEP_FX
#undef SIK_STEP_
}

}  // namespace sik
