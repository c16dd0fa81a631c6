// Exact per-query-head top-k selection on gfx950 without sorting (the selection step after the
// retrieval equation in "Compressed-Domain Top-k Retrieval").
//
// Level 1: a 512-bin histogram of a monotone map of the score (built while scoring, or by the
// two stand-alone kernels below) locates the threshold bin b*: every token in a bin above b* is
// selected; tokens inside b* are candidates.
// Level 2: the candidates (typically L / 1000 of them) are gathered by all workgroups of the
// query head and ranked exactly by (score desc, index asc) by the last workgroup to finish, which
// fills the remaining k - c_gt slots.  If the threshold bin holds more than kCandCap tokens
// (degenerate score distributions, e.g. all scores equal) the same workgroup falls back to an
// 8-bit radix select over the bin's members, still exact.
#include "sik_device.h"
#include "sik_internal.h"
#include "sik_select.h"

namespace sik {

SIK_TL_DEFINE(sik_dbg_tl_topk)

constexpr int kSelChunkMax = 4096;  // scores scanned per select workgroup (bounds its LDS list)

// ---- stand-alone level 1, pass A: per-row min and max of the order-preserving keys ---------
__global__ __launch_bounds__(kBlock) void minmax_kernel(const float* __restrict__ scores,
                                                        const int32_t* __restrict__ seq_len,
                                                        uint32_t* __restrict__ counters, int Hq, int Lmax,
                                                        int nchunk, int chunk) {
    __shared__ uint32_t smin[kBlock / kWave], smax[kBlock / kWave];
    const int row = blockIdx.x / nchunk, c = blockIdx.x % nchunk, tid = threadIdx.x;
    int L = seq_len[row / Hq];
    L = L > Lmax ? Lmax : L;
    const int start = c * chunk, end = min(L, start + chunk);
    if (start >= end) return;
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    const float* s = scores + static_cast<size_t>(row) * Lmax;
#pragma unroll 8
    for (int i = start + tid; i < end; i += kBlock) {
        const uint32_t key = float_to_key(s[i]);
        kmin = min(kmin, key);
        kmax = max(kmax, key);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        kmin = min(kmin, static_cast<uint32_t>(__shfl_xor(static_cast<int>(kmin), o, 64)));
        kmax = max(kmax, static_cast<uint32_t>(__shfl_xor(static_cast<int>(kmax), o, 64)));
    }
    if ((tid & 63) == 0) {
        smin[tid >> 6] = kmin;
        smax[tid >> 6] = kmax;
    }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kBlock / kWave; ++w) {
            kmin = min(kmin, smin[w]);
            kmax = max(kmax, smax[w]);
        }
        atomic_max_u32(&counters[row * 8 + 4], ~kmin);  // the region starts at zero: keep ~min
        atomic_max_u32(&counters[row * 8 + 5], kmax);
    }
}

// ---- stand-alone level 1, pass B: per-chunk histograms over [min, max] -----------------------
__global__ __launch_bounds__(kBlock) void hist_kernel(const float* __restrict__ scores,
                                                      const int32_t* __restrict__ seq_len,
                                                      const uint32_t* __restrict__ counters,
                                                      uint32_t* __restrict__ parthist,
                                                      float* __restrict__ binp, int Hq, int Lmax, int nchunk,
                                                      int chunk) {
    __shared__ uint32_t lhist[kBins];
    const int row = blockIdx.x / nchunk, c = blockIdx.x % nchunk, tid = threadIdx.x;
    int L = seq_len[row / Hq];
    L = L < 0 ? 0 : (L > Lmax ? Lmax : L);
    const int start = c * chunk, end = min(L, start + chunk);
    if (start >= L && c != 0) return;
    const float lo = key_to_float(~counters[row * 8 + 4]);
    const float hi = key_to_float(counters[row * 8 + 5]);
    const float span = hi - lo;
    const float scale = (span > 1e-30f && span < 3.0e38f) ? static_cast<float>(kBins) / span : 0.0f;
    if (c == 0 && tid == 0) {
        binp[row * 2] = lo;
        binp[row * 2 + 1] = scale;
    }
    for (int e = tid; e < kBins; e += kBlock) lhist[e] = 0u;
    __syncthreads();
    const float* s = scores + static_cast<size_t>(row) * Lmax;
#pragma unroll 8
    for (int i = start + tid; i < end; i += kBlock) atomicAdd(&lhist[score_bin(s[i], lo, scale)], 1u);
    __syncthreads();
    publish_hist(lhist, parthist + (static_cast<size_t>(row) * nchunk + c) * kHistWords);
}

// ---- select: compaction against the threshold bin, exact resolution of the bin ---------------
__global__ __launch_bounds__(kBlock) void select_kernel(
    // (the first 14 dwords arrive in scalar registers with the wavefront: what the first loads need comes first;
    // chunks = hchunks | nchunk << 16)
    const float* __restrict__ scores, const int32_t* __restrict__ seq_len, const uint32_t* __restrict__ parthist,
    const float* __restrict__ binp, int sstride, int Hq, int Lmax, int chunk, int hchunk, uint32_t chunks,
    uint32_t* __restrict__ counters, uint32_t* __restrict__ cand, int32_t* __restrict__ idx, int k) {
    // 17 KB of LDS per workgroup, so that eight of them fit a compute unit: the selected tokens are kept as 16-bit
    // offsets into the chunk, and the candidate list shares its storage with the histogram staging of
    // find_threshold (dead after the barrier that follows it).
    static_assert(kSelChunkMax <= 65536, "16-bit chunk offsets");
    static_assert((kBlock / kWave) * kBins <= 2 * kCandCap + 16, "the staging area fits the candidate list");
    __shared__ uint32_t h256[kBlock];
    __shared__ uint16_t l_sel[kSelChunkMax];
    __shared__ __align__(8) uint32_t red[2 * kCandCap + 16];
    uint32_t* const l_cand = red;
    __shared__ int s_flag, sthr[3];
    __shared__ uint32_t s_nsel, s_ncand, s_base[2], sh[4];

    SIK_TL(8);
    const int hchunks = chunks & 0xffffu, nchunk = chunks >> 16;
    const int row = blockIdx.x / nchunk, c = blockIdx.x % nchunk, tid = threadIdx.x;
    int L = seq_len[row / Hq];
    L = L < 0 ? 0 : (L > Lmax ? Lmax : L);
    const int start = c * chunk, end = min(L, start + chunk);
    if (start >= L && c != 0) return;  // chunk 0 always runs: it may have to pad the row
    const int kk = min(k, L);
    const float* s = scores + static_cast<size_t>(row) * sstride;
    int32_t* out = idx + static_cast<size_t>(row) * k;

    // threshold bin of this query head from the chunk histograms of the producing kernel
    const float lo = binp[row * 2], scale = binp[row * 2 + 1];
    if (tid == 0) {
        s_nsel = 0u;
        s_ncand = 0u;
    }
    const int hact = L > 0 ? (L + hchunk - 1) / hchunk : 1;  // chunks the producer ran for this sequence
    // the first 4096 scores of the chunk (all of them: chunks are at most kSelChunkMax long) are requested
    // together with the histograms, one round trip for both
    const bool vec = (sstride & 3) == 0;  // rows are 16-byte aligned: vector loads
    const float4* s4 = reinterpret_cast<const float4*>(s);
    const int q0 = start >> 2, q1 = (end + 3) >> 2;  // start is a multiple of 256
    float4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int qi = q0 + j * kBlock + tid;
        v[j] = (vec && qi < q1) ? s4[qi] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const HistLoads hl = load_chunk_hists(parthist + static_cast<size_t>(row) * hchunks * kHistWords, hact);
    const Threshold th = find_threshold(hl, kk, L, red, sh, sthr);
    const int bstar = th.bstar, cgt = th.cgt, nb = th.nb;
    const bool ranked = nb <= kCandCap;
    __syncthreads();
    SIK_TL(9);

    auto classify = [&](float x, int i) {
        const int bin = bstar < 0 ? 0 : score_bin(x, lo, scale);
        if (bin > bstar) {
            l_sel[atomicAdd(&s_nsel, 1u)] = static_cast<uint16_t>(i - start);
        } else if (bin == bstar && ranked) {
            const uint32_t pos = atomicAdd(&s_ncand, 1u);
            if (pos < static_cast<uint32_t>(kCandCap)) {
                l_cand[2 * pos] = float_to_key(x);
                l_cand[2 * pos + 1] = static_cast<uint32_t>(i);
            }
        }
    };
    if (vec) {
        for (int base = q0; base < q1; base += 4 * kBlock) {
            if (base != q0) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int qi = base + j * kBlock + tid;
                    v[j] = qi < q1 ? s4[qi] : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int i = (base + j * kBlock + tid) * 4;
                if (i < end) classify(v[j].x, i);
                if (i + 1 < end) classify(v[j].y, i + 1);
                if (i + 2 < end) classify(v[j].z, i + 2);
                if (i + 3 < end) classify(v[j].w, i + 3);
            }
        }
    } else {
#pragma unroll 4
        for (int i = start + tid; i < end; i += kBlock) classify(s[i], i);
    }
    __syncthreads();
    SIK_TL(10);
    if (tid == 0) {
        s_base[0] = s_nsel ? atomic_add_u32(&counters[row * 8 + 0], s_nsel) : 0u;
        s_base[1] = s_ncand ? atomic_add_u32(&counters[row * 8 + 1], s_ncand) : 0u;
    }
    __syncthreads();
    for (uint32_t j = tid; j < s_nsel; j += kBlock) {
        const uint32_t pos = s_base[0] + j;
        if (pos < static_cast<uint32_t>(k)) out[pos] = start + static_cast<int32_t>(l_sel[j]);
    }
    const uint32_t ncand = min(s_ncand, static_cast<uint32_t>(kCandCap));
    uint32_t* crow = cand + static_cast<size_t>(row) * kCandCap * 2;
    for (uint32_t j = tid; j < ncand; j += kBlock) {
        const uint32_t pos = s_base[1] + j;
        if (pos < static_cast<uint32_t>(kCandCap)) {
            st_agent(&crow[2 * pos], l_cand[2 * j]);
            st_agent(&crow[2 * pos + 1], l_cand[2 * j + 1]);
        }
    }

    SIK_TL(11);
    const int nact = L > 0 ? (L + chunk - 1) / chunk : 1;
    if (!last_arriver(&counters[row * 8 + 2], static_cast<uint32_t>(nact), &s_flag)) return;

    SIK_TL_ANY(12);
    // ---- last workgroup of this query head: resolve the threshold bin, pad the row ----------
    const int need = kk - min(cgt, kk);
    if (need > 0) {
        if (ranked) {
            const int n = min(nb, kCandCap);
            const int npad = (n + 7) & ~7;  // padding entries outrank nothing
            for (int j = tid; j < 2 * npad; j += kBlock)
                l_cand[j] = j < 2 * n ? ld_agent(&crow[j]) : ((j & 1) ? 0xffffffffu : 0u);
            __syncthreads();
            const uint2* lc2 = reinterpret_cast<const uint2*>(l_cand);
            for (int a = tid; a < n; a += kBlock) {
                const uint2 me = lc2[a];
                int rank = 0;
                for (int x = 0; x < npad; x += 8) {  // eight LDS reads in flight
                    uint2 o8[8];
#pragma unroll
                    for (int y = 0; y < 8; ++y) o8[y] = lc2[x + y];
#pragma unroll
                    for (int y = 0; y < 8; ++y) rank += (o8[y].x > me.x || (o8[y].x == me.x && o8[y].y < me.y)) ? 1 : 0;
                }
                if (rank < need) out[cgt + rank] = static_cast<int32_t>(me.y);
            }
        } else {
            radix_select_in_bin(s, L, lo, scale, bstar, need, out + cgt, h256, sh);
        }
    }
    for (int j = kk + tid; j < k; j += kBlock) out[j] = -1;
    SIK_TL_ANY(13);
}

// ---------------------------------------------------------------------------------------
void select_plan(const Dims& d, int* nchunk, int* chunk) {
    const int rows = d.rows();
    int want = (512 + rows - 1) / rows;
    int ch = (d.Lmax + want - 1) / want;
    ch = (ch + kBlock - 1) / kBlock * kBlock;
    if (ch < 1024) ch = 1024;
    if (ch > kSelChunkMax) ch = kSelChunkMax;
    *chunk = ch;
    *nchunk = (d.Lmax + ch - 1) / ch;
}

// Chunks of the stand-alone histogram pass: at most kChunkCap tokens each (16-bit counts per bin and chunk) and
// at most kMaxChunks of them per row: max_len <= kMaxLen.
void hist_plan(const Dims& d, int* nchunk, int* chunk) {
    const int rows = d.rows();
    int want = (512 + rows - 1) / rows;
    if (want > kMaxChunks) want = kMaxChunks;
    int ch = (d.Lmax + want - 1) / want;
    ch = (ch + kBlock - 1) / kBlock * kBlock;
    if (ch < 2048) ch = 2048;
    if (ch > kChunkCap) ch = kChunkCap;
    *chunk = ch;
    *nchunk = (d.Lmax + ch - 1) / ch;
}

bool hist_plan_ok(const Dims& d) {
    int nchunk, chunk;
    hist_plan(d, &nchunk, &chunk);
    return chunk <= kChunkCap && nchunk <= kMaxChunks;
}

hipError_t launch_topk_hist(const Dims& d, const Workspace& w, const float* scores, const int32_t* seq_len,
                            hipStream_t s) {
    int nchunk, chunk;
    hist_plan(d, &nchunk, &chunk);
    const int grid = nchunk * d.rows();
    minmax_kernel<<<grid, kBlock, 0, s>>>(scores, seq_len, w.counters, d.Hq, d.Lmax, nchunk, chunk);
    hist_kernel<<<grid, kBlock, 0, s>>>(scores, seq_len, w.counters, w.parthist, w.binp, d.Hq, d.Lmax, nchunk,
                                        chunk);
    return hipGetLastError();
}

hipError_t launch_select(const Dims& d, const Workspace& w, bool hist_from_score, const float* scores,
                         const int32_t* seq_len, int k, int32_t* idx, hipStream_t s) {
    int nchunk, chunk, hchunks, hchunk, nhb;
    select_plan(d, &nchunk, &chunk);
    if (hist_from_score)
        score_plan(d, &nhb, &hchunks, &hchunk);
    else
        hist_plan(d, &hchunks, &hchunk);
    return launch_kernel(select_kernel, nchunk * d.rows(), kBlock, s, scores, seq_len, w.parthist, w.binp,
                         hist_from_score ? w.sstride : d.Lmax, d.Hq, d.Lmax, chunk, hchunk,
                         static_cast<uint32_t>(hchunks) | static_cast<uint32_t>(nchunk) << 16, w.counters, w.cand, idx,
                         k);
}

}  // namespace sik
