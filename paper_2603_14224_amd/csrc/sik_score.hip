// LUT-GEMV retrieval over the packed sign codes for gfx950 (section "Compressed-Domain
// Top-k Retrieval"): Table^(g)[j] = q^(g) . c_j^(g), score_i = sum_g Table^(g)[Code_g(k_i)].
//
// One workgroup (512 threads, 1024 in small launches) serves one (batch, kv head) for a block of up to 4 query
// heads of its GQA group (a wider group is served by several head blocks that re-read the codes from L2: two float4
// tables in one workgroup were measured slower, 65 us against 2 x 18 us on the 8:1 workload)
// and a contiguous chunk of tokens.  The tables live in LDS as float4 entries holding the
// same (g, j) entry of four query heads: the 16 entries of a group span 256 B = all 64 LDS
// banks once, so the data-dependent ds_read_b128 of a wavefront (all lanes are at the same g)
// is bank-conflict free whatever the codes are.  Each lane owns one token per load: a single
// 128-bit load brings its 32 codes, i.e. a wavefront streams 1 KB of the code plane per load;
// the loads of the next 1024 tokens of the workgroup are in flight while the current ones are scored.
//
// What bounds the scan is vector-instruction issue, with the LDS reads close behind: 4 x 32 adds per token for
// a block of four heads cannot be avoided (no packed fp32 here), so everything around them is kept small - one
// instruction per table offset, four per histogram count - and the kernel stays under 128 registers, i.e. four
// wavefronts per SIMD, which hide the LDS latency (ds_read_b128 sustains over 200 B/clk per compute unit).
//
// A launch with one query head per KV head (no GQA, or the summed query of a group-shared selection) uses
// scalar table entries instead (HB = 1).
//
// With HIST the kernel also builds the first level of the selection: a histogram of a monotone
// map of each query head's scores, published per chunk for the select kernel.
#include "sik_device.h"
#include "sik_internal.h"
#include "sik_kvq.h"
#include "sik_scan.h"
#include "sik_select.h"

namespace sik {

SIK_TL_DEFINE(sik_dbg_tl_score)

constexpr int kIterTokens = 1024;  // tokens a workgroup scores per loop iteration: BLK threads x 1024 / BLK each

// FORCED: tokens named in forced_idx [B, Hkv, n_forced] (entries outside [0, L) ignored) always take part in
// the attention that follows and must not compete in the selection: their score is stored as -infinity and
// they are left out of the histogram ("Full Precision Sink Tokens": a fixed set that is always attended).
template <int DT, bool HIST, int BLK, bool FORCED, int HB>
__global__ __launch_bounds__(BLK) void score_kernel(
    // the first 14 dwords are preloaded into scalar registers with the wavefront: what the index arithmetic and
    // the first loads need comes first, so that they do not wait for a round trip to the argument block
    const uint16_t* __restrict__ q, const float* __restrict__ codebook, const uint8_t* __restrict__ codes, int Hkv,
    int Hq, int R, int Lmax, int nchunk, int chunk, int nhb, int q_sum, const int32_t* __restrict__ seq_len,
    float* __restrict__ scores, int sstride, uint32_t* __restrict__ parthist, float* __restrict__ binp,
    uint32_t* __restrict__ zero_counters, const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new,
    uint16_t* __restrict__ Kc, uint16_t* __restrict__ Vc, const float* __restrict__ mu,
    uint8_t* __restrict__ codes_w, const float* __restrict__ alpha, uint2* __restrict__ kvq,
    const int32_t* __restrict__ forced_idx, int n_forced, int32_t* __restrict__ lens_out) {
    static_assert(HB == 1 || HB == kHB, "scalar or float4 table entries");
    constexpr int kTokPerIter = kIterTokens / BLK;
    __shared__ __align__(16) float lut[kG * 16 * HB];  // entry (g, j): HB consecutive floats, one per query head
    __shared__ float qs[HB][kD];
    __shared__ float bp[HB][2];
    __shared__ uint32_t lhist[HIST ? HB * kBins : 1];
    __shared__ __align__(16) uint8_t newcode[kCodeBytes];
    __shared__ uint32_t fbits[FORCED ? (kMaxChunkTokens + 32) / 32 : 1];  // one bit per token of the chunk

    SIK_TL(0);
    const int tid = threadIdx.x;
    const int c = blockIdx.x % nchunk;
    const int u = blockIdx.x / nchunk;
    const int hb = u % nhb;
    const int unit = u / nhb;
    const int h = unit % Hkv, b = unit / Hkv;
    const int start = c * chunk;
    const int hq0 = h * R + hb * HB;
    const int nh = min(HB, R - hb * HB);
    const size_t row0 = static_cast<size_t>(b) * Hq + hq0;

    // every global load this workgroup needs before it can score goes out now, together; none of
    // them waits for seq_len (codes up to the capacity are readable, stale ones are never used)
    const uint4* cp = reinterpret_cast<const uint4*>(codes + static_cast<size_t>(unit) * Lmax * kCodeBytes);
    const int cap_end = min(Lmax, start + chunk);
    uint4 cur[kTokPerIter];
#pragma unroll
    for (int j = 0; j < kTokPerIter; ++j) {
        const int i = start + j * BLK + tid;
        cur[j] = i < cap_end ? cp[i] : make_uint4(0u, 0u, 0u, 0u);
    }
    int fi = -1;  // forced token of this KV head that thread tid looks after
    if constexpr (FORCED)
        if (tid < n_forced) fi = forced_idx[static_cast<size_t>(unit) * n_forced + tid];
    constexpr int kEntPerThread = kG * 16 / BLK < 1 ? 1 : kG * 16 / BLK;  // table entries (g, j) per thread
    float4 cj[kEntPerThread];
#pragma unroll
    for (int x = 0; x < kEntPerThread; ++x) {
        const int e = tid + x * BLK;
        cj[x] = e < kG * 16 ? reinterpret_cast<const float4*>(codebook)[static_cast<size_t>(unit) * kG * 16 + e]
                            : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (tid < HB * 16) {  // 16 lanes x 16 B per query row
        const int s = tid >> 4, p = tid & 15;
        float f[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (q_sum <= 1) {
            if (s < nh) widen8<DT>(reinterpret_cast<const uint4*>(q + (row0 + s) * kD)[p], f);
        } else if (s == 0) {
            // group-shared selection: the launch sees one "query head" per KV head whose query is the sum of the
            // q_sum real ones (the table is linear in the query, so its scores are the summed scores)
            for (int r = 0; r < q_sum; ++r) {
                float g[8];
                widen8<DT>(reinterpret_cast<const uint4*>(q + (row0 * q_sum + r) * kD)[p], g);
#pragma unroll
                for (int e = 0; e < 8; ++e) f[e] += g[e];
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) qs[s][8 * p + e] = f[e];
    }
    if constexpr (HIST) {
        for (int e = tid; e < HB * kBins; e += BLK) lhist[e] = 0u;
        if constexpr (FORCED)
            for (int e = tid; e < (chunk + 31) / 32; e += BLK) fbits[e] = 0u;
        // the kernels that follow count on zeroed per-head counters; when no prep launch precedes,
        // chunk 0 of each head block clears those of its heads
        // (a launch on the summed query of q_sum heads stands for q_sum rows of the kernel that follows)
        const int nrows = q_sum > 1 ? q_sum : nh;
        if (zero_counters && c == 0)
            for (int t = tid; t < nrows * 8; t += BLK) zero_counters[row0 * (q_sum > 1 ? q_sum : 1) * 8 + t] = 0u;
    }
    // decode-time append (k_new != nullptr): the new key/value row of this KV head goes to row t =
    // seq_len[b]; every workgroup counts it in (L = t + 1), the one whose chunk holds t encodes it
    // against the frozen mu and scores it from LDS, and head block 0 of that chunk also stores the row and
    // its code.  seq_len itself is incremented by the last workgroup of the kernel that follows.
    uint4 knew = make_uint4(0u, 0u, 0u, 0u), vnew = make_uint4(0u, 0u, 0u, 0u);
    float m8[8] = {0, 0, 0, 0, 0, 0, 0, 0}, a8[8] = {0, 0, 0, 0, 0, 0, 0, 0};  // mu, 1 / alpha
    if (k_new && tid < 16) {
        knew = reinterpret_cast<const uint4*>(k_new + static_cast<size_t>(unit) * kD)[tid];
        vnew = reinterpret_cast<const uint4*>(v_new + static_cast<size_t>(unit) * kD)[tid];
        const float4 m0 = reinterpret_cast<const float4*>(mu + static_cast<size_t>(unit) * kD)[2 * tid];
        const float4 m1 = reinterpret_cast<const float4*>(mu + static_cast<size_t>(unit) * kD)[2 * tid + 1];
        m8[0] = m0.x, m8[1] = m0.y, m8[2] = m0.z, m8[3] = m0.w;
        m8[4] = m1.x, m8[5] = m1.y, m8[6] = m1.z, m8[7] = m1.w;
        if (kvq) {  // 2-bit cache: the row is stored as a record, which also needs the frozen alpha
            const float4 a0 = reinterpret_cast<const float4*>(alpha + static_cast<size_t>(unit) * kD)[2 * tid];
            const float4 a1 = reinterpret_cast<const float4*>(alpha + static_cast<size_t>(unit) * kD)[2 * tid + 1];
            const float av[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) a8[e] = alpha_reciprocal(av[e]);
        }
    }
    int L = seq_len[b];
    L = L < 0 ? 0 : (L > Lmax ? Lmax : L);
    int t_new = -1;
    if (k_new && L < Lmax) {
        t_new = L;
        L += 1;
    }
    // The launch that follows takes the sequence's length (the appended token counted in) from this copy: it
    // publishes the new seq_len[b] itself and must not read a location it writes.
    if (HIST && lens_out != nullptr && c == 0 && hb == 0 && h == 0 && tid == 0) lens_out[b] = L;
    const bool holds_new = t_new >= start && t_new < start + chunk;
    if (holds_new && tid < 16) {
        float f[8];
        widen8<DT>(knew, f);
        uint32_t byte = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) byte |= (f[e] >= m8[e] ? 1u : 0u) << (7 - e);
        newcode[tid] = static_cast<uint8_t>(byte);
        if (hb == 0) {
            const size_t rowi = static_cast<size_t>(unit) * Lmax + t_new;
            if (kvq) {
                kvq[rowi * kRecSlots + tid] = kvq_make_slot<DT>(knew, vnew, m8, a8, tid);
            } else {
                reinterpret_cast<uint4*>(Kc + rowi * kD)[tid] = knew;
                reinterpret_cast<uint4*>(Vc + rowi * kD)[tid] = vnew;
            }
            codes_w[rowi * kCodeBytes + tid] = static_cast<uint8_t>(byte);
        }
    }
    if (start >= L && c != 0) {  // no valid token here (chunk 0 always runs: it owns the per-head outputs)
        if constexpr (HIST)      // consumers read every chunk's histogram: publish an empty one
            if (tid < kHistWords)
                for (int s = 0; s < nh; ++s) parthist[((row0 + s) * nchunk + c) * kHistWords + tid] = 0u;
        return;
    }
    const int end = min(L, start + chunk);
    __syncthreads();
    if constexpr (FORCED)  // the barriers below order these bits before the scoring loop reads them
        if (fi >= start && fi < end) atomicOr(&fbits[(fi - start) >> 5], 1u << ((fi - start) & 31));
    SIK_TL(1);

    // Table^(g)[j] for the HB query heads, fp32
#pragma unroll
    for (int x = 0; x < kEntPerThread; ++x) {
        const int e = tid + x * BLK;
        if (e < kG * 16) {
            const int g = e >> 4;
            float o[HB];
#pragma unroll
            for (int s = 0; s < HB; ++s) {
                const float* qq = &qs[s][4 * g];
                float a = qq[0] * cj[x].x;
                a = fmaf(qq[1], cj[x].y, a);
                a = fmaf(qq[2], cj[x].z, a);
                a = fmaf(qq[3], cj[x].w, a);
                o[s] = a;
            }
            if constexpr (HB == 4)
                *reinterpret_cast<float4*>(&lut[e * 4]) = make_float4(o[0], o[1], o[2], o[3]);
            else
                lut[e] = o[0];
        }
    }
    __syncthreads();

    if constexpr (HIST) {
        // Bins are spread over mean +- 4.5 sigma of the score of a key whose 32 codes are uniform
        // and independent (mean = sum_g mean_j T, var = sum_g var_j T); scores outside fall into the
        // end bins.  Any (lo, scale) is correct, this one keeps the threshold bin small.
        if (tid < HB * 32) {
            const int s = tid >> 5, g = tid & 31;
            // entry j of group g, head s: lanes start at different j so that they hit different banks
            const float* lf = &lut[g * 16 * HB + s];
            float sum = 0.0f, sq = 0.0f;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float x = lf[((j + g) & 15) * HB];
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
            if (g == 0) {
                const float span = 9.0f * sqrtf(var);
                const float lo = mean - 0.5f * span;
                const float scale = (span > 1e-30f && span < 3.0e38f) ? static_cast<float>(kBins) / span : 0.0f;
                bp[s][0] = lo;
                bp[s][1] = scale;
                if (c == 0 && s < nh) {
                    binp[(row0 + s) * 2] = lo;
                    binp[(row0 + s) * 2 + 1] = scale;
                }
            }
        }
        __syncthreads();
    }

    SIK_TL(2);
    // bin scale and shift of each head in registers (read from LDS inside the loop they would be fetched again
    // for every token: the histogram updates may alias them as far as the compiler knows)
    float bscale[HB], bshift[HB];
#pragma unroll
    for (int s = 0; s < HB; ++s) {
        bscale[s] = HIST ? bp[s][1] : 0.0f;
        bshift[s] = HIST ? bin_shift(bp[s][0], bp[s][1]) : 0.0f;
    }
    for (int base = start; base < end; base += kIterTokens) {
        uint4 code[kTokPerIter];
#pragma unroll
        for (int j = 0; j < kTokPerIter; ++j) code[j] = cur[j];
        const int nbase = base + kIterTokens;
        if (nbase < end) {
#pragma unroll
            for (int j = 0; j < kTokPerIter; ++j) {
                const int i = nbase + j * BLK + tid;
                if (i < end) cur[j] = cp[i];
            }
        }
        if (t_new >= base && t_new < nbase) {  // the appended token's code was written before the barriers above
#pragma unroll
            for (int j = 0; j < kTokPerIter; ++j)
                if (base + j * BLK + tid == t_new) code[j] = *reinterpret_cast<const uint4*>(newcode);
        }
        // Software pipeline over the 4 * kTokPerIter batches of this thread's tokens: the lookups of batch i + 1
        // are issued before the adds of batch i, so that 8 to 16 LDS reads are in flight per wavefront at under
        // 128 registers (left to itself the compiler either waits for each read or holds a whole token's 32).
        typename TableEntry<HB>::type v[2][8];
        auto word = [&](int i) {
            const uint4& cw = code[i >> 2];
            return (i & 3) == 0 ? cw.x : ((i & 3) == 1 ? cw.y : ((i & 3) == 2 ? cw.z : cw.w));
        };
        lookup_batch<HB>(word(0), 0, lut, v[0]);
#pragma unroll
        for (int j = 0; j < kTokPerIter; ++j) {
            const int tok = base + j * BLK + tid;
            float acc[HB];
#pragma unroll
            for (int dw = 0; dw < 4; ++dw) {
                const int i = 4 * j + dw;
                if (i + 1 < 4 * kTokPerIter) lookup_batch<HB>(word(i + 1), (i + 1) & 3, lut, v[(i + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                add_batch<HB>(dw == 0, v[i & 1], acc);
                // (keeps the adds here: as they are only used under "tok < end" they would move down there)
#pragma unroll
                for (int s = 0; s < HB; ++s) asm volatile("" : "+v"(acc[s]));
                __builtin_amdgcn_sched_barrier(0);
            }
            if (tok < end) {
                bool forced = false;
                if constexpr (FORCED) forced = (fbits[(tok - start) >> 5] >> ((tok - start) & 31)) & 1u;
#pragma unroll
                for (int s = 0; s < HB; ++s) {
                    if (s < nh) {
                        // streamed once, read by the next kernel: keep it out of the way of the end-of-kernel write-back
                        __builtin_nontemporal_store(forced ? -INFINITY : acc[s], &scores[(row0 + s) * sstride + tok]);
                        if constexpr (HIST)
                            if (!forced)
                                atomicAdd(&lhist[s * kBins + bin_of_coord(bin_coord_shifted(acc[s], bscale[s], bshift[s]))],
                                          1u);
                    }
                }
            }
        }
    }

    SIK_TL(3);
    if constexpr (HIST) {
        __syncthreads();
        if (tid < kHistWords)
            for (int s = 0; s < nh; ++s)
                publish_hist(&lhist[s * kBins], parthist + ((row0 + s) * nchunk + c) * kHistWords);
    }
    SIK_TL(4);
}

// Workgroup size: 512 threads (two wavefronts per SIMD share one table build; 256-thread workgroups were measured
// slower at every size: 37 against 33 us on 32 x 8 KV heads x 16K), and 1024 for small launches, which run one
// workgroup per compute unit: four wavefronts per SIMD hide the LDS latency there (128K context, one sequence:
// 10.5 against 11.3 us; no difference at 32K).
constexpr int kScoreBlock = 512;

// Tokens per workgroup: one workgroup per compute unit for small launches (latency-bound: fewest table builds),
// two (scalar tables: four) for large ones; whole loop iterations of 1024 tokens (so that the table build and
// the 2 KB histogram per head are amortised), at most kChunkCap tokens (the published histogram counts and the
// forced-token bitmap are sized for that) and at most kMaxChunks chunks per head: max_len <= kMaxLen.
void score_plan(const Dims& d, int* nhb_out, int* nchunk, int* chunk) {
    const int nhb = (d.R + kHB - 1) / kHB;
    const int units = d.units() * nhb;
    const bool small = static_cast<int64_t>(units) * d.Lmax <= (2 << 20);
    const int target = small ? 256 : (d.R == 1 ? 1024 : 512);
    int want = (target + units - 1) / units;
    if (want > kMaxChunks) want = kMaxChunks;
    int ch = (d.Lmax + want - 1) / want;
    ch = (ch + kIterTokens - 1) / kIterTokens * kIterTokens;
    if (ch > kChunkCap) ch = kChunkCap;  // more chunks instead
    *nhb_out = nhb;
    *chunk = ch;
    *nchunk = (d.Lmax + ch - 1) / ch;
}

bool score_plan_ok(const Dims& d) {
    int nhb, nchunk, chunk;
    score_plan(d, &nhb, &nchunk, &chunk);
    return chunk <= kChunkCap && nchunk <= kMaxChunks;
}

template <int DT>
static hipError_t launch_score_t(const Dims& d, const Workspace* w, bool zero, const Append& ap, const void* q,
                                 const float* codebook, const uint8_t* codes, const int32_t* seq_len,
                                 float* scores, const int32_t* forced_idx, int n_forced, int q_sum, hipStream_t s) {
    int nhb, nchunk, chunk;
    score_plan(d, &nhb, &nchunk, &chunk);
    const int grid = nchunk * nhb * d.units();
    const bool small_launch = static_cast<int64_t>(d.units()) * nhb * d.Lmax <= (2 << 20);
    auto qp = static_cast<const uint16_t*>(q);
#define SIK_SCORE2(HV, FV, HBV, BLKV)                                                                        \
    launch_kernel(score_kernel<DT, HV, BLKV, FV, HBV>, grid, BLKV, s, qp, codebook, codes, d.Hkv, d.Hq, d.R, d.Lmax, \
                  nchunk, chunk, nhb, q_sum, seq_len, scores, w ? w->sstride : d.Lmax, w ? w->parthist : nullptr, \
                  w ? w->binp : nullptr, zero ? w->counters : nullptr, ap.k_new, ap.v_new, ap.K, ap.V, ap.mu,   \
                  ap.codes, ap.alpha, static_cast<uint2*>(ap.kvq), forced_idx, n_forced, w ? w->lens : nullptr)
#define SIK_SCORE1(HV, FV, HBV) (small_launch ? SIK_SCORE2(HV, FV, HBV, 1024) : SIK_SCORE2(HV, FV, HBV, kScoreBlock))
#define SIK_SCORE(HV, FV) (d.R == 1 ? SIK_SCORE1(HV, FV, 1) : SIK_SCORE1(HV, FV, kHB))
    if (!w) return SIK_SCORE(false, false);
    if (n_forced > 0) return SIK_SCORE(true, true);
    return SIK_SCORE(true, false);
#undef SIK_SCORE
#undef SIK_SCORE1
#undef SIK_SCORE2
}

hipError_t launch_score(const Dims& d, const Workspace* w, bool zero_counters, const Append& ap, const void* q,
                        const float* codebook, const uint8_t* codes, const int32_t* seq_len, float* scores,
                        const int32_t* forced_idx, int n_forced, int q_sum, hipStream_t s) {
    if (!w) n_forced = 0;  // forced sets belong to the decode step (histogram-producing launches)
    return d.kv_dtype == kBF16 ? launch_score_t<kBF16>(d, w, zero_counters, ap, q, codebook, codes, seq_len, scores,
                                                       forced_idx, n_forced, q_sum, s)
                               : launch_score_t<kF16>(d, w, zero_counters, ap, q, codebook, codes, seq_len, scores,
                                                      forced_idx, n_forced, q_sum, s);
}

}  // namespace sik
