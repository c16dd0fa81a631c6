// Fused selection + sparse attention for the decode step on gfx950: one launch turns the scores and
// chunk histograms written by the scoring kernel into the attention output (the selection step of
// "Compressed-Domain Top-k Retrieval" followed by softmax(q K_S^T / sqrt(d)) V_S of "Background and
// Preliminaries").
//
// Workgroup (query head, token chunk):
//   1. loads, all at once: the head's chunk histograms, its own chunk of scores, the query row;
//   2. finds the threshold bin b* (every workgroup of the head finds the same one);
//   3. each wavefront compacts the tokens of its score registers that lie in bins above b* into a
//      private LDS list (ballot + popcount, deterministic order) and attends over them at once:
//      the selected tokens never travel through an index list in memory;
//   4. tokens inside b* ("candidates", about L/1000 of the head's tokens) are published with their
//      score keys; the partial softmax (m, l, o[D]) of the chunk is published;
//   5. the last workgroup of the head to arrive ranks the candidates exactly by (score desc, index
//      asc), attends over the k - c_gt best of them, merges all partials and writes the output row.
// A wavefront that finds more than kWaveCand candidates in its share puts the surplus into an overflow pool
// of the head (one atomic reservation per round), which the last workgroup reads in a second round trip.
// More than kCandCap tokens in b* (e.g. all scores equal) take an exact radix-select fallback in step 5.
#include "sik_attn_core.h"
#include "sik_device.h"
#include "sik_internal.h"
#include "sik_kvq.h"
#include "sik_select.h"

namespace sik {

SIK_TL_DEFINE(sik_dbg_tl_fused)

// Candidate exchange area of one query head: regions = 4 * nchunk (one per chunk and wavefront), kCandWaveWords
// words per region.  First the regions' counts, one word each (a count may exceed kWaveCand: the surplus is in
// the pool); then, 8-byte aligned, the (key, index) pairs as 64-bit words (key below), pair e of region r at
// pairs[e * regions + r]: the last workgroup, which reads one region per lane, issues 16 coalesced 64-bit loads.
// The pool of a head follows the regions of all heads: kCandCap (key, index) pairs, filled in the order of
// reservations on counter 4 of the head.
constexpr int kWaveCand = 16;                      // candidate slots per wavefront and chunk
constexpr int kCandWaveWords = 2 + 2 * kWaveCand;  // words per region (even: the pairs stay 8-byte aligned)

// NQ float4 of scores per lane: chunk = 1024 * NQ tokens.  KVQ: the selected tokens are gathered as 128-byte
// records of the 2-bit cache (kvq, alpha) and dequantised in registers, instead of as 16-bit K and V rows.
template <int DT, int ODT, int NQ, bool KVQ>
__global__ __launch_bounds__(kBlock, 4) void select_attend_kernel(
    // The first 14 dwords are preloaded into scalar registers with the wavefront: what the index arithmetic and
    // the first loads need comes first (small integers packed), so that they do not wait for a round trip to the
    // argument block.  dims0 = Hkv | Hq << 16, dims1 = R | nchunk << 16,
    // dims2 = hchunks | n_forced << 8 | shared << 16 | appended << 17 | stream << 18 (non-temporal row loads).
    const float* __restrict__ scores, const uint16_t* __restrict__ q, const uint32_t* __restrict__ parthist,
    const float* __restrict__ binp, const int32_t* __restrict__ lens, int sstride, uint32_t dims0, uint32_t dims1,
    uint32_t dims2, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V, const uint2* __restrict__ kvq,
    const float* __restrict__ alpha, uint32_t* __restrict__ counters, uint32_t* __restrict__ cand,
    float* __restrict__ partial, int32_t* __restrict__ idx_ws, int32_t* __restrict__ idx_out,
    void* __restrict__ out, float scale_log2e, int k, int Lmax, const int32_t* __restrict__ forced_idx,
    const uint16_t* __restrict__ fK, const uint16_t* __restrict__ fV, const float* __restrict__ mu,
    int k_per_mille, int32_t* __restrict__ seq_len) {
    constexpr int kChunk = 1024 * NQ;
    constexpr int kListCap = 512;  // selected-token slots per wavefront; flushed to the gather when half full
    const int Hkv = dims0 & 0xffffu, Hq = dims0 >> 16, R = dims1 & 0xffffu, nchunk = dims1 >> 16;
    const int hchunks = dims2 & 0xffu, n_forced = (dims2 >> 8) & 0xffu;
    const int shared = (dims2 >> 16) & 1u, appended = (dims2 >> 17) & 1u;
    // non-temporal row loads (large launches), except in the workgroup that also gathers the forced tokens: those
    // rows are read by every query head of the sequence and should stay cached
    const bool stream = ((dims2 >> 18) & 1u) && !(n_forced > 0 && blockIdx.x % nchunk == 0);
    __shared__ int32_t l_sel[kBlock / kWave][kListCap];
    __shared__ uint32_t red[(kBlock / kWave) * kBins];
    __shared__ __align__(8) uint32_t l_cand[2 * kCandCap + 64];
    __shared__ float sm[kBlock / kWave], sl[kBlock / kWave];
    __shared__ float sacc[kBlock / kWave][kD];
    __shared__ uint32_t lds4[4], sh[4];
    __shared__ int sthr[3], s_flag, s_over;
    __shared__ uint32_t s_ncand;
    __shared__ int32_t s_fidx[kMaxForced];  // forced tokens of the KV head, -1 where the slot names no token

    SIK_TL(24);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, p = lane & 15;
    const int row = blockIdx.x / nchunk, c = blockIdx.x % nchunk;
    const int b = row / Hq, hq = row % Hq;
    const size_t unit = static_cast<size_t>(b) * Hkv + hq / R;
    const int start = c * kChunk;
    // Group-shared selection (shared != 0): scores, histograms and bin bounds exist once per KV head (the scoring
    // launch ran on the summed query), so the R query heads of a group find the same threshold and select the
    // same tokens, each attending with its own query; the group's first head writes the one index list.
    const size_t srow = shared ? unit : static_cast<size_t>(row);

    // ---- 1. every load that does not depend on another goes out now ---------------------------
    const float4* s4 = reinterpret_cast<const float4*>(scores + srow * sstride + start);
    float4 sv[NQ];
#pragma unroll
    for (int j = 0; j < NQ; ++j) {
        const int i = start + (j * kBlock + tid) * 4;
        sv[j] = i < sstride ? s4[j * kBlock + tid] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const uint4 qraw = reinterpret_cast<const uint4*>(q + static_cast<size_t>(row) * kD)[p];
    float4 al0 = make_float4(0.f, 0.f, 0.f, 0.f), al1 = al0;
    if constexpr (KVQ) {
        al0 = reinterpret_cast<const float4*>(alpha + unit * kD)[2 * p];
        al1 = reinterpret_cast<const float4*>(alpha + unit * kD)[2 * p + 1];
    }
    const float lo = binp[srow * 2], scale = binp[srow * 2 + 1];
    const HistLoads hl = load_chunk_hists(parthist + srow * hchunks * kHistWords, hchunks);
    // the length as the scoring launch counted it (an appended token included): this launch only WRITES seq_len[b]
    int L = lens[b];
    // Everything above comes from the preloaded arguments; what follows needs the rest of the argument block,
    // which arrives a memory round trip after the wavefront started.
    int32_t* const orow = !idx_out ? nullptr
                          : !shared ? idx_out + static_cast<size_t>(row) * k
                                    : (hq % R == 0 ? idx_out + unit * k : nullptr);
    // StepOptions set (n_forced > 0): thread t < n_forced looks after entry t.  The scoring launch gave these tokens
    // -infinity, so they are never selected below; workgroup 0 of the head attends them on top of its own.
    int fi = -1;
    if (n_forced > 0 && tid < n_forced) fi = forced_idx[unit * n_forced + tid];
    float mu_dot = 0.0f;  // q . mu over this lane's channels: centres the full-precision forced keys
    if (KVQ && fK != nullptr && c == 0) {
        float qf[8];
        widen8<DT>(qraw, qf);
        const float4 m0 = reinterpret_cast<const float4*>(mu + unit * kD)[2 * p];
        const float4 m1 = reinterpret_cast<const float4*>(mu + unit * kD)[2 * p + 1];
        mu_dot = qf[0] * m0.x + qf[1] * m0.y + qf[2] * m0.z + qf[3] * m0.w + qf[4] * m1.x + qf[5] * m1.y +
                 qf[6] * m1.z + qf[7] * m1.w;
    }
    L = L < 0 ? 0 : (L > Lmax ? Lmax : L);
    const int nact = L > 0 ? (L + kChunk - 1) / kChunk : 1;
    if (c >= nact) return;  // no token of this chunk is valid; the ticket below counts nact workgroups
    const int end = min(L, start + kChunk);
    int nfv = 0;  // forced tokens that exist: the dynamic budget and the competing population shrink by them
    if (n_forced > 0) {
        const bool fv = fi >= 0 && fi < L;
        if (tid < kMaxForced) s_fidx[tid] = fv ? fi : -1;
        nfv = __syncthreads_count(fv ? 1 : 0);
        fi = fv ? fi : -1;
    }
    // Budget of this sequence: k, or with k_per_mille > 0 the smaller of k and ceil(L * k_per_mille / 1000) (a
    // fraction of the context, in integer arithmetic), but at least one token.
    const int kb = k_per_mille > 0 ? min(k, max(1, static_cast<int>((static_cast<int64_t>(L) * k_per_mille + 999) / 1000))) : k;
    const int Lc = L - nfv;                     // tokens that compete
    const int kk = max(0, min(kb - nfv, Lc));   // dynamic picks (the forced tokens may use up the budget)
    if (tid == 0) {
        s_over = 0;
        s_ncand = 0u;
    }

    // ---- 2. threshold bin ---------------------------------------------------------------------
    Threshold th;
    if (kk > 0) {
        th = find_threshold(hl, kk, Lc, red, lds4, sthr);
    } else {  // nothing to pick (empty sequence, or a budget the forced tokens fill): every test below fails
        th.bstar = kBins;
        th.cgt = 0;
        th.nb = 0;
    }
    const int bstar = th.bstar, cgt = th.cgt, nb = th.nb;
    const bool ranked = nb <= kCandCap;
    SIK_TL(25);

    // ---- 3. wave-private compaction of the selected tokens, candidates aside -------------------
    const uint4* Kp = KVQ ? nullptr : reinterpret_cast<const uint4*>(K + unit * Lmax * kD);
    const uint4* Vp = KVQ ? nullptr : reinterpret_cast<const uint4*>(V + unit * Lmax * kD);
    const uint2* Rp = KVQ ? kvq + unit * Lmax * kRecSlots : nullptr;
    Q2Query qq;
    if constexpr (KVQ) {
        const float a8[8] = {al0.x, al0.y, al0.z, al0.w, al1.x, al1.y, al1.z, al1.w};
        qq = q2_prepare<DT>(qraw, a8);
    }
    // Gather + online softmax over a list: wavefront-private lists go in steps of kStep entries, lists shared by
    // the workgroup's four wavefronts in interleaved steps.
    constexpr int kStep = KVQ ? 32 : 16;
    auto attend = [&](auto fetch, int n, int first, int step, SoftmaxState& s_) {
        if constexpr (KVQ)
            attend_list_q2(fetch, n, first, step, Rp, qq, scale_log2e, Lmax, s_);
        else if (stream)  // one branch per list, not per load: each variant keeps its loads back to back
            attend_list<DT, true>(fetch, n, first, step, Kp, Vp, qraw, scale_log2e, Lmax, s_);
        else
            attend_list<DT, false>(fetch, n, first, step, Kp, Vp, qraw, scale_log2e, Lmax, s_);
    };
    int n_sel = 0, n_cand = 0;  // wave-uniform
    const int regions = nchunk * (kBlock / kWave);
    uint32_t* crow = cand + static_cast<size_t>(row) * regions * kCandWaveWords;
    const int myreg = c * (kBlock / kWave) + wv;  // this wavefront's region
    uint64_t* cpairs = reinterpret_cast<uint64_t*>(crow + ((regions + 1) & ~1));
    uint32_t* pool = cand + static_cast<size_t>(gridDim.x / nchunk) * regions * kCandWaveWords +
                     static_cast<size_t>(row) * kCandCap * 2;
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    // bin(s) > b*  <=>  x >= b* + 1 and bin(s) == b*  <=>  b* <= x < b* + 1 with x = bin_coord(s),
    // the clamped end bins taking everything beyond them (score_bin is floor + clamp of the same x)
    // (open ends are -FLT_MAX, not -infinity: a forced token's score is -infinity and must fail every test)
    const float hi_f = bstar < 0 ? -3.4028235e38f : (bstar >= kBins - 1 ? INFINITY : static_cast<float>(bstar + 1));
    const float lo_f = bstar <= 0 ? -3.4028235e38f : (bstar >= kBins ? INFINITY : static_cast<float>(bstar));
    const bool has_cand = bstar >= 0 && bstar < kBins && ranked;
    SoftmaxState st;
    init_state(st);
    int32_t* mylist = l_sel[wv];
    // Stage A: one branch-free pass over this lane's 4 * NQ scores marks, in two bit masks, the ones
    // at or above the selection bound and the ones at or above the candidate bound (a few
    // instructions per score; about 3 % are selected, about 0.1 % are candidates).
    static_assert(4 * NQ <= 32, "one mask bit per score of the lane");
    uint32_t smask = 0u, gmask = 0u;
    if (start + kChunk <= end) {
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            const float v4[4] = {sv[j].x, sv[j].y, sv[j].z, sv[j].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float x = bin_coord(v4[e], lo, scale);
                smask |= (x >= hi_f ? 1u : 0u) << (4 * j + e);
                gmask |= (x >= lo_f ? 1u : 0u) << (4 * j + e);
            }
        }
    } else {  // last chunk of the sequence: slots at or beyond seq_len compare false (NaN)
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            const float v4[4] = {sv[j].x, sv[j].y, sv[j].z, sv[j].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = start + (j * kBlock + tid) * 4 + e;
                const float x = i < end ? bin_coord(v4[e], lo, scale) : __builtin_nanf("");
                smask |= (x >= hi_f ? 1u : 0u) << (4 * j + e);
                gmask |= (x >= lo_f ? 1u : 0u) << (4 * j + e);
            }
        }
    }
    uint32_t cmask = has_cand ? (gmask & ~smask) : 0u;
    // candidates: rounds of one mask bit per lane, as in stage B below; the score of the popped slot is
    // picked from the registers by a select chain (only wavefronts that hold candidates get here)
    while (true) {
        const bool has = cmask != 0u;
        const uint64_t bc = __ballot(has);
        if (bc == 0ull) break;
        const int bit = has ? __ffs(static_cast<int>(cmask)) - 1 : 0;
        cmask &= cmask - 1u;
        float v = 0.0f;
#pragma unroll
        for (int j = 0; j < NQ; ++j) {
            const float v4[4] = {sv[j].x, sv[j].y, sv[j].z, sv[j].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) v = bit == 4 * j + e ? v4[e] : v;
        }
        const int pos = n_cand + __popcll(bc & lt_mask);
        const uint32_t tok = static_cast<uint32_t>(start + (((bit >> 2) * kBlock + tid) * 4 + (bit & 3)));
        if (has && pos < kWaveCand) {
            st_agent(&cpairs[pos * regions + myreg], static_cast<uint64_t>(tok) << 32 | float_to_key(v));
        }
        n_cand += __popcll(bc);
        if (n_cand > kWaveCand) {  // rare: the surplus of this round goes to the head's pool
            const bool over = has && pos >= kWaveCand;
            const uint64_t bo = __ballot(over);
            const int leader = __ffsll(static_cast<unsigned long long>(bo)) - 1;
            uint32_t base = 0u;
            if (lane == leader) base = atomic_add_u32(&counters[row * 8 + 4], static_cast<uint32_t>(__popcll(bo)));
            base = static_cast<uint32_t>(__shfl(static_cast<int>(base), leader, 64));
            const uint32_t slot = base + static_cast<uint32_t>(__popcll(bo & lt_mask));
            if (over && slot < static_cast<uint32_t>(kCandCap)) {
                st_agent(&pool[2 * slot], float_to_key(v));
                st_agent(&pool[2 * slot + 1], tok);
            }
        }
    }
    // StepOptions tokens: workgroup 0 of the head takes them on.  Read like every other token (16-bit cache, or
    // 2-bit cache without side rows) they simply start the lists of the wavefronts that hold their entries;
    // given as 16-bit side rows they are attended here, each logit shifted by -q . mu because the records
    // they share the softmax with hold the centred key.
    if (n_forced > 0 && c == 0) {
        const bool fv = fi >= 0;
        const uint64_t bf = __ballot(fv);
        const bool side = KVQ && fK != nullptr;
        if (!side) {
            if (fv) mylist[__popcll(bf & lt_mask)] = fi;
            n_sel = __popcll(bf);
        } else {
            if (orow && bf != 0ull) {
                uint32_t base = 0u;
                if (lane == 0) base = atomic_add_u32(&counters[row * 8 + 0], static_cast<uint32_t>(__popcll(bf)));
                base = static_cast<uint32_t>(__shfl(static_cast<int>(base), 0, 64));
                if (fv) orow[base + __popcll(bf & lt_mask)] = fi;
            }
            const float zbias = -row16_sum(mu_dot) * scale_log2e;
            attend_list<DT>([&](int j) { return s_fidx[j] >= 0 ? j : -1; }, n_forced, wv * 16, (kBlock / kWave) * 16,
                            reinterpret_cast<const uint4*>(fK + unit * n_forced * kD),
                            reinterpret_cast<const uint4*>(fV + unit * n_forced * kD), qraw, scale_log2e, n_forced,
                            st, zbias);
        }
    }
    // Stage B: compaction of the marked scores into the wavefront's list, one mask bit per lane and
    // round (as many rounds as the busiest lane has selected scores); the list is gathered whenever
    // another round might not fit.
    while (true) {
        const bool has = smask != 0u;
        const uint64_t bal = __ballot(has);
        if (bal == 0ull) break;
        if (n_sel > kListCap - 64) {
            const int n16 = n_sel & ~(kStep - 1);  // complete gather steps now, the rest moves to the front
            if (orow) {
                uint32_t base = 0u;
                if (lane == 0) base = atomic_add_u32(&counters[row * 8 + 0], static_cast<uint32_t>(n16));
                base = static_cast<uint32_t>(__shfl(static_cast<int>(base), 0, 64));
                for (int t = lane; t < n16; t += 64)
                    if (base + t < static_cast<uint32_t>(k)) orow[base + t] = mylist[t];
            }
            attend([&](int t) { return mylist[t]; }, n16, 0, kStep, st);
            const int rem = n_sel - n16;
            const int keep = lane < rem ? mylist[n16 + lane] : 0;
            if (lane < rem) mylist[lane] = keep;
            n_sel = rem;
        }
        if (has) {
            const int bit = __ffs(static_cast<int>(smask)) - 1;
            smask &= smask - 1u;
            mylist[n_sel + __popcll(bal & lt_mask)] = start + (((bit >> 2) * kBlock + tid) * 4 + (bit & 3));
        }
        n_sel += __popcll(bal);
    }
    if (lane == 0) st_agent(&crow[myreg], static_cast<uint32_t>(n_cand));
    // optional index output: reserve this wave's slots now, write them after the gather
    uint32_t out_base = 0u;
    if (orow && n_sel > 0) {
        if (lane == 0) out_base = atomic_add_u32(&counters[row * 8 + 0], static_cast<uint32_t>(n_sel));
    }
    SIK_TL(26);

    // ---- 4. attend over this wavefront's own tokens, publish the chunk's partial ---------------
    attend([&](int j) { return mylist[j]; }, n_sel, 0, kStep, st);
    SIK_TL(27);
    if (orow && n_sel > 0) {
        out_base = static_cast<uint32_t>(__shfl(static_cast<int>(out_base), 0, 64));
        for (int j = lane; j < n_sel; j += 64)
            if (out_base + j < static_cast<uint32_t>(k)) orow[out_base + j] = mylist[j];
    }
    float M, Lsum, o;
    workgroup_merge(st, sm, sl, sacc, M, Lsum, o);
    float* prow = partial + (static_cast<size_t>(row) * kMaxChunks) * kPartStride;
    if (tid < kD) {
        float* pp = prow + static_cast<size_t>(c) * kPartStride;
        st_agent(&pp[2 + tid], o);
        if (tid == 0) {
            st_agent(&pp[0], M);
            st_agent(&pp[1], Lsum);
        }
    }
    SIK_TL(28);
    if (!last_arriver(&counters[row * 8 + 3], static_cast<uint32_t>(nact), &s_flag)) return;
    SIK_TL_ANY(29);

    // ---- 5. last workgroup of the head: candidates, merge, output ------------------------------
    // All exchange loads go out together: the (m, l) pair of every chunk (thread c), the first 8
    // chunks' o[d] (thread d), and one candidate region per thread.
    const int need = kk - min(cgt, kk);
    int32_t* olist = orow ? orow : idx_ws + static_cast<size_t>(row) * k;
    constexpr int kOPre = 8;
    float o_pre[kOPre];
    float pm = kNegBig, pl = 0.0f;
    if (tid < nact) {
        pm = ld_agent(&prow[static_cast<size_t>(tid) * kPartStride]);
        pl = ld_agent(&prow[static_cast<size_t>(tid) * kPartStride + 1]);
    }
#pragma unroll
    for (int s2 = 0; s2 < kOPre; ++s2)
        o_pre[s2] = (tid < kD && s2 < nact) ? ld_agent(&prow[static_cast<size_t>(s2) * kPartStride + 2 + tid]) : 0.0f;
    const bool want_cands = need > 0 && ranked;
    uint32_t cn = 0u, ent[2 * kWaveCand];
    if (want_cands && tid < nact * 4) {
        cn = ld_agent(&crow[tid]);
#pragma unroll
        for (int e = 0; e < kWaveCand; ++e) {
            const uint64_t pr = ld_agent(&cpairs[e * regions + tid]);
            ent[2 * e] = static_cast<uint32_t>(pr);
            ent[2 * e + 1] = static_cast<uint32_t>(pr >> 32);
        }
    }
    float* pml = reinterpret_cast<float*>(l_sel[0]);  // [2][kMaxChunks] in LDS (l_sel is free by now)
    if (tid < kMaxChunks) {
        pml[tid] = pm;
        pml[kMaxChunks + tid] = pl;
    }
    init_state(st);
    SIK_TL_ANY(32);
    if (need > 0) {
        bool use_radix = !ranked;
        if (ranked) {
            if (tid < nact * 4 && cn > 0u) {
                if (cn > static_cast<uint32_t>(kWaveCand)) {
                    s_over = 1;  // the rest of this wavefront's candidates is in the pool
                    cn = kWaveCand;
                }
                const uint32_t base = atomicAdd(&s_ncand, cn);
#pragma unroll
                for (int e = 0; e < kWaveCand; ++e) {
                    if (static_cast<uint32_t>(e) < cn && base + e < static_cast<uint32_t>(kCandCap)) {
                        // one 64-bit sort key per candidate: score key above, inverted index below, so
                        // that "larger" means better score, then smaller index
                        l_cand[2 * (base + e)] = ~ent[2 * e + 1];
                        l_cand[2 * (base + e) + 1] = ent[2 * e];
                    }
                }
            }
            __syncthreads();
            if (s_over != 0) {
                const uint32_t np = min(ld_agent(&counters[row * 8 + 4]), static_cast<uint32_t>(kCandCap));
                for (uint32_t j = tid; j < np; j += kBlock) {
                    const uint32_t key = ld_agent(&pool[2 * j]), tok = ld_agent(&pool[2 * j + 1]);
                    const uint32_t at = atomicAdd(&s_ncand, 1u);
                    if (at < static_cast<uint32_t>(kCandCap)) {
                        l_cand[2 * at] = ~tok;
                        l_cand[2 * at + 1] = key;
                    }
                }
                __syncthreads();
            }
            SIK_TL_ANY(33);
        }
        if (!use_radix) {
            const int n = min(static_cast<int>(s_ncand), kCandCap);
            uint32_t* rank_of = red;                                      // [kCandCap] partial-rank sums
            int32_t* chosen = reinterpret_cast<int32_t*>(red + kCandCap);  // rank r -> token index
            // Ranking by counting, spread over all 256 threads: P threads share one candidate and each
            // scans a slice of the list, padded to a multiple of 8 with entries that outrank nothing so
            // that eight LDS reads stay in flight.
            const int P = n <= 64 ? 4 : (n <= 128 ? 2 : 1);
            const int slice = ((n + P - 1) / P + 7) & ~7;
            for (int j = tid; j < P * slice - n; j += kBlock) {
                l_cand[2 * (n + j)] = 0u;  // padding: the smallest 64-bit key, outranks nothing
                l_cand[2 * (n + j) + 1] = 0u;
            }
            for (int j = tid; j < n; j += kBlock) rank_of[j] = 0u;
            __syncthreads();
            const unsigned long long* lc2 = reinterpret_cast<const unsigned long long*>(l_cand);
            const int per = kBlock / P;  // candidates handled per pass
            const int part = tid / per;
            for (int a = tid % per; a < n; a += per) {
                const unsigned long long me = lc2[a];
                uint32_t rank = 0;
                for (int x = part * slice; x < (part + 1) * slice; x += 8) {
                    unsigned long long o8[8];
#pragma unroll
                    for (int y = 0; y < 8; ++y) o8[y] = lc2[x + y];
#pragma unroll
                    for (int y = 0; y < 8; ++y) rank += o8[y] > me ? 1u : 0u;
                }
                if (P > 1) atomicAdd(&rank_of[a], rank); else rank_of[a] = rank;
            }
            __syncthreads();
            for (int a = tid; a < n; a += kBlock) {
                const int rank = static_cast<int>(rank_of[a]);
                if (rank < need) {
                    const int32_t ia = static_cast<int32_t>(~static_cast<uint32_t>(lc2[a]));
                    chosen[rank] = ia;
                    if (orow) olist[nfv + cgt + rank] = ia;
                }
            }
            __syncthreads();
            SIK_TL_ANY(34);
            attend([&](int j) { return chosen[j]; }, min(need, n), wv * kStep, (kBlock / kWave) * kStep, st);
        } else {
            // exact fallback: radix select over the members of b* in the whole row of scores
            radix_select_in_bin(scores + srow * sstride, L, lo, scale, bstar, need,
                                olist + nfv + cgt, red, sh);
            __threadfence_block();
            __syncthreads();
            const int32_t* gl = olist + nfv + cgt;
            attend([&](int j) { return gl[j]; }, need, wv * kStep, (kBlock / kWave) * kStep, st);
        }
    }
    SIK_TL_ANY(31);
    float M2, L2, o2;
    workgroup_merge(st, sm, sl, sacc, M2, L2, o2);  // has a barrier: pml is visible afterwards
    if (tid < kD) {
        float Mg = M2;
#pragma unroll 8
        for (int s2 = 0; s2 < nact; ++s2) Mg = fmaxf(Mg, pml[s2]);
        const float a2 = fast_exp2(M2 - Mg);
        float lt = L2 * a2, ot = o2 * a2;
#pragma unroll
        for (int s2 = 0; s2 < kOPre; ++s2) {  // fixed order: the result does not depend on arrival order
            if (s2 < nact) {
                const float a = fast_exp2(pml[s2] - Mg);
                lt += pml[kMaxChunks + s2] * a;
                ot += o_pre[s2] * a;
            }
        }
#pragma unroll 8
        for (int s2 = kOPre; s2 < nact; ++s2) {
            const float a = fast_exp2(pml[s2] - Mg);
            lt += pml[kMaxChunks + s2] * a;
            ot += ld_agent(&prow[static_cast<size_t>(s2) * kPartStride + 2 + tid]) * a;
        }
        store_out<ODT>(out, static_cast<size_t>(row) * kD + tid, lt > 0.0f ? ot / lt : 0.0f);
    }
    if (orow)
        for (int j = nfv + kk + tid; j < k; j += kBlock) olist[j] = -1;
    // the last query head of the sequence to finish publishes the new length (nothing in this launch reads
    // seq_len; at capacity nothing was appended and L is the old value)
    if (appended && tid == 0) {
        if (atomic_add_u32(&counters[static_cast<size_t>(b) * Hq * 8 + 7], 1u) == static_cast<uint32_t>(Hq) - 1u)
            seq_len[b] = L;
    }
    SIK_TL_ANY(30);
}

// Token chunk of the fused kernel: a power of two in [1024, 8192] (the instantiated sizes), aiming at
// about 400 workgroups; independent of the scoring kernel's chunks, whose histograms are only summed.
// Returns false when max_len needs more than kMaxChunks chunks of 8192 tokens.
bool fused_plan(const Dims& d, int* nchunk, int* chunk) {
    int want = (384 + d.rows() - 1) / d.rows();
    int ch = 1024;
    while (ch < 8192 && static_cast<int64_t>(ch) * want < d.Lmax) ch *= 2;
    while (ch < 8192 && (d.Lmax + ch - 1) / ch > kMaxChunks) ch *= 2;  // few rows, long context: fewer, larger chunks
    *chunk = ch;
    *nchunk = (d.Lmax + ch - 1) / ch;
    return *nchunk <= kMaxChunks;
}

size_t fused_cand_words(const Dims& d) {
    int nchunk, chunk;
    if (!fused_plan(d, &nchunk, &chunk)) return 0;
    return static_cast<size_t>(d.rows()) * nchunk * (kBlock / kWave) * kCandWaveWords +
           static_cast<size_t>(d.rows()) * kCandCap * 2;  // regions of every head, then the overflow pools
}

template <int DT, int ODT>
static hipError_t launch_fused_t(const Dims& d, const Workspace& w, const void* q, const void* K, const void* V,
                                 const void* kvq, const float* alpha, const StepOptions& fo, int32_t* seq_len,
                                 bool appended, int k, float scale, int32_t* idx_out, void* out, hipStream_t s) {
    int nhb, hchunks, hchunk, nchunk, chunk;
    Dims dscore = d;  // the launch that wrote the scores and histograms
    if (fo.group_shared) {
        dscore.Hq = d.Hkv;
        dscore.R = 1;
    }
    score_plan(dscore, &nhb, &hchunks, &hchunk);
    if (!fused_plan(d, &nchunk, &chunk)) return hipErrorInvalidValue;
    const float sl2 = (scale > 0.0f ? scale : 1.0f / sqrtf(static_cast<float>(d.D))) * 1.4426950408889634f;
    const int grid = nchunk * d.rows();
    auto qp = static_cast<const uint16_t*>(q);
    auto Kp = static_cast<const uint16_t*>(K);
    auto Vp = static_cast<const uint16_t*>(V);
    auto Rp = static_cast<const uint2*>(kvq);
    static_assert(kMaxChunks <= 0xff && kMaxForced <= 0xff, "8-bit argument fields");
    const uint32_t dims0 = static_cast<uint32_t>(d.Hkv) | static_cast<uint32_t>(d.Hq) << 16;
    const uint32_t dims1 = static_cast<uint32_t>(d.R) | static_cast<uint32_t>(nchunk) << 16;
    const uint32_t dims2 = static_cast<uint32_t>(hchunks) | static_cast<uint32_t>(fo.n) << 8 |
                           (fo.group_shared ? 1u << 16 : 0u) | (appended ? 1u << 17 : 0u) |
                           (gather_streams(d, k) ? 1u << 18 : 0u);
#define SIK_FUSED_Q(NQV, KVQV)                                                                              \
    launch_kernel(select_attend_kernel<DT, ODT, NQV, KVQV>, grid, kBlock, s, w.scores, qp, w.parthist, w.binp,   \
                  w.lens, w.sstride, dims0, dims1, dims2, Kp, Vp, Rp, alpha, w.counters, w.cand, w.partial, w.idx, \
                  idx_out, out, sl2, k, d.Lmax, fo.idx, fo.fK, fo.fV, fo.mu, fo.k_per_mille, seq_len)
#define SIK_FUSED(NQV) (kvq ? SIK_FUSED_Q(NQV, true) : SIK_FUSED_Q(NQV, false))
    switch (chunk) {
        case 1024: return SIK_FUSED(1);
        case 2048: return SIK_FUSED(2);
        case 4096: return SIK_FUSED(4);
        case 8192: return SIK_FUSED(8);
        default: return hipErrorInvalidValue;
    }
#undef SIK_FUSED
#undef SIK_FUSED_Q
}

hipError_t launch_fused(const Dims& d, const Workspace& w, const void* q, const void* K, const void* V,
                        const void* kvq, const float* alpha, const StepOptions& forced, int32_t* seq_len, bool appended,
                        int k, float scale, int32_t* idx_out, void* out, hipStream_t s) {
#define SIK_F(DTV, ODTV) \
    launch_fused_t<DTV, ODTV>(d, w, q, K, V, kvq, alpha, forced, seq_len, appended, k, scale, idx_out, out, s)
    if (d.kv_dtype == kBF16) return d.out_dtype == kF32 ? SIK_F(kBF16, kF32) : SIK_F(kBF16, kBF16);
    return d.out_dtype == kF32 ? SIK_F(kF16, kF32) : SIK_F(kF16, kF16);
#undef SIK_F
}

}  // namespace sik
