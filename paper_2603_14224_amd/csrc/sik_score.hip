// LUT-GEMV retrieval over the packed sign codes for gfx950 (section "Compressed-Domain
// Top-k Retrieval"): Table^(g)[j] = q^(g) . c_j^(g), score_i = sum_g Table^(g)[Code_g(k_i)].
//
// One workgroup serves one (batch, kv head) for a block of up to 4 query heads of its GQA group
// (a wider group is served by several head blocks that re-read the codes from L2: two float4
// tables in one workgroup were measured slower, 65 us against 2 x 18 us on the 8:1 workload)
// and a contiguous chunk of tokens.  The tables live in LDS as float4 entries holding the
// same (g, j) entry of four query heads: the 16 entries of a group span 256 B = all 64 LDS
// banks once, so the data-dependent ds_read_b128 of a wavefront (all lanes are at the same g)
// is bank-conflict free whatever the codes are.  Each lane owns one token per load: a single
// 128-bit load brings its 32 codes, i.e. a wavefront streams 1 KB of the code plane per load;
// four such loads per lane are in flight while the previous four tokens are scored.
//
// A launch with one query head per KV head (no GQA, or the summed query of a group-shared selection) uses
// scalar table entries instead (HB = 1).
//
// With HIST the kernel also builds the first level of the selection: a histogram of a monotone
// map of each query head's scores, published per chunk for the select kernel.
#include "sik_device.h"
#include "sik_internal.h"
#include "sik_kvq.h"
#include "sik_select.h"

namespace sik {

SIK_TL_DEFINE(sik_dbg_tl_score)

constexpr int kIterTokens = 1024;  // tokens a workgroup scores per loop iteration: BLK threads x 1024 / BLK each

constexpr int kHB = 4;  // query heads per workgroup = components of one float4 table entry

// Table lookups of one token.  HB = 4: float4 entries (four query heads at once), 256 B per group; HB = 1: scalar
// entries, 64 B per group (one query head per KV head: multi-head attention, or the summed query of a
// group-shared selection) - a quarter of the LDS traffic, the 16 entries of a group on 16 different banks.
template <int HB>
__device__ __forceinline__ void score_token(const uint4 code, const float* lut, float* acc) {
#pragma unroll
    for (int s = 0; s < HB; ++s) acc[s] = 0.0f;
    const uint32_t w[4] = {code.x, code.y, code.z, code.w};
    const char* base = reinterpret_cast<const char*>(lut);
#pragma unroll
    for (int dw = 0; dw < 4; ++dw) {
#pragma unroll
        for (int by = 0; by < 4; ++by) {
            // byte (4 dw + by) of the token: high nibble = Code of group g, low nibble = group g+1
            const int g = 8 * dw + 2 * by;
            const uint32_t bits = w[dw] >> (8 * by);
            if constexpr (HB == 4) {
                const uint32_t off_hi = bits & 0xf0u;  // Code * 16 B
                const uint32_t off_lo = (bits & 0x0fu) << 4;
                const float4 v0 = *reinterpret_cast<const float4*>(base + g * 256 + off_hi);
                acc[0] += v0.x;
                acc[1] += v0.y;
                acc[2] += v0.z;
                acc[3] += v0.w;
                const float4 v1 = *reinterpret_cast<const float4*>(base + (g + 1) * 256 + off_lo);
                acc[0] += v1.x;
                acc[1] += v1.y;
                acc[2] += v1.z;
                acc[3] += v1.w;
            } else {
                const uint32_t off_hi = (bits & 0xf0u) >> 2;  // Code * 4 B
                const uint32_t off_lo = (bits & 0x0fu) << 2;
                acc[0] += *reinterpret_cast<const float*>(base + g * 64 + off_hi);
                acc[0] += *reinterpret_cast<const float*>(base + (g + 1) * 64 + off_lo);
            }
        }
    }
}

// FORCED: tokens named in forced_idx [B, Hkv, n_forced] (entries outside [0, L) ignored) always take part in
// the attention that follows and must not compete in the selection: their score is stored as -infinity and
// they are left out of the histogram ("Full Precision Sink Tokens": a fixed set that is always attended).
template <int DT, bool HIST, int BLK, bool FORCED, int HB>
__global__ __launch_bounds__(BLK) void score_kernel(const uint16_t* __restrict__ q,
                                                       const float* __restrict__ codebook,
                                                       const uint8_t* __restrict__ codes,
                                                       const int32_t* __restrict__ seq_len,
                                                       float* __restrict__ scores, int sstride,
                                                       uint32_t* __restrict__ parthist,
                                                       float* __restrict__ binp,
                                                       uint32_t* __restrict__ zero_counters,
                                                       const uint16_t* __restrict__ k_new,
                                                       const uint16_t* __restrict__ v_new,
                                                       uint16_t* __restrict__ Kc, uint16_t* __restrict__ Vc,
                                                       const float* __restrict__ mu,
                                                       uint8_t* __restrict__ codes_w,
                                                       const float* __restrict__ alpha, uint2* __restrict__ kvq,
                                                       const int32_t* __restrict__ forced_idx, int n_forced,
                                                       int q_sum, int Hkv, int Hq, int R,
                                                       int Lmax, int nchunk, int chunk, int nhb) {
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
        if (zero_counters && c == 0 && tid < nrows * 8) zero_counters[row0 * (q_sum > 1 ? q_sum : 1) * 8 + tid] = 0u;
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
#pragma unroll
        for (int j = 0; j < kTokPerIter; ++j) {
            const int tok = base + j * BLK + tid;
            float acc[HB];
            if (tok == t_new) code[j] = *reinterpret_cast<const uint4*>(newcode);  // written before the barriers above
            score_token<HB>(code[j], lut, acc);
            if (tok < end) {
                bool forced = false;
                if constexpr (FORCED) forced = (fbits[(tok - start) >> 5] >> ((tok - start) & 31)) & 1u;
#pragma unroll
                for (int s = 0; s < HB; ++s) {
                    if (s < nh) {
                        // streamed once, read by the next kernel: keep it out of the way of the end-of-kernel write-back
                        __builtin_nontemporal_store(forced ? -INFINITY : acc[s], &scores[(row0 + s) * sstride + tok]);
                        if constexpr (HIST)
                            if (!forced) atomicAdd(&lhist[s * kBins + score_bin(acc[s], bp[s][0], bp[s][1])], 1u);
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

// Workgroup size.  Small launches (one sequence) are latency-bound: 512 threads = two wavefronts per SIMD share one
// table build and interleave their LDS reads and adds (measured on 1 x 8 KV heads: 5.6 against 6.5 us at 32K,
// 13.4 against 14.6 us at 128K).  Large launches are bound by LDS bandwidth either way and run a little faster
// as twice as many 256-thread workgroups (38 against 41 us on 32 x 8 heads x 16K).
static int score_block(const Dims& d, int nhb) {
    return static_cast<int64_t>(d.units()) * nhb * d.Lmax <= (2 << 20) ? 512 : 256;
}

// Tokens per workgroup: about 2 x 256 or 1 x 512 threads per compute unit, whole loop iterations of 1024
// tokens (so that the table build and the 2 KB histogram per head are amortised), at most kMaxChunks per head.
void score_plan(const Dims& d, int* nhb_out, int* nchunk, int* chunk) {
    const int nhb = (d.R + kHB - 1) / kHB;
    const int units = d.units() * nhb;
    // (scalar tables, R = 1: 62 registers, 8 wavefronts per SIMD fit, and a table costs 512 entries to build)
    const int target = score_block(d, nhb) == 512 ? 256 : (d.R == 1 ? 2048 : 512);
    int want = (target + units - 1) / units;
    if (want > kMaxChunks) want = kMaxChunks;
    int ch = (d.Lmax + want - 1) / want;
    ch = (ch + kIterTokens - 1) / kIterTokens * kIterTokens;
    while ((d.Lmax + ch - 1) / ch > kMaxChunks) ch += kIterTokens;
    *nhb_out = nhb;
    *chunk = ch;
    *nchunk = (d.Lmax + ch - 1) / ch;
}

bool score_plan_ok(const Dims& d) {
    int nhb, nchunk, chunk;
    score_plan(d, &nhb, &nchunk, &chunk);
    return chunk <= kMaxChunkTokens;
}

template <int DT>
static hipError_t launch_score_t(const Dims& d, const Workspace* w, bool zero, const Append& ap, const void* q,
                                 const float* codebook, const uint8_t* codes, const int32_t* seq_len,
                                 float* scores, const int32_t* forced_idx, int n_forced, int q_sum, hipStream_t s) {
    int nhb, nchunk, chunk;
    score_plan(d, &nhb, &nchunk, &chunk);
    const int grid = nchunk * nhb * d.units();
    auto qp = static_cast<const uint16_t*>(q);
#define SIK_SCORE1(HV, BLKV, FV, HBV)                                                                        \
    score_kernel<DT, HV, BLKV, FV, HBV><<<grid, BLKV, 0, s>>>(                                               \
        qp, codebook, codes, seq_len, scores, w ? w->sstride : d.Lmax, w ? w->parthist : nullptr,          \
        w ? w->binp : nullptr, zero ? w->counters : nullptr, ap.k_new, ap.v_new, ap.K, ap.V, ap.mu, ap.codes, \
        ap.alpha, static_cast<uint2*>(ap.kvq), forced_idx, n_forced, q_sum, d.Hkv, d.Hq, d.R, d.Lmax, nchunk, chunk, \
        nhb)
#define SIK_SCORE(HV, BLKV, FV)                                                                              \
    do {                                                                                                     \
        if (d.R == 1) SIK_SCORE1(HV, BLKV, FV, 1); else SIK_SCORE1(HV, BLKV, FV, kHB);                       \
    } while (0)
    const bool wide = score_block(d, nhb) == 512;
    if (!w) { if (wide) SIK_SCORE(false, 512, false); else SIK_SCORE(false, 256, false); }
    else if (n_forced > 0) { if (wide) SIK_SCORE(true, 512, true); else SIK_SCORE(true, 256, true); }
    else { if (wide) SIK_SCORE(true, 512, false); else SIK_SCORE(true, 256, false); }
#undef SIK_SCORE
#undef SIK_SCORE1
    return hipGetLastError();
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
