// Sparse softmax attention over the selected tokens for gfx950:
// out = softmax(q K_S^T / sqrt(d)) V_S on the stored 16-bit K and V rows (section "Background
// and Preliminaries"; token-wise random access as argued in "Token-Wise Quantization Format").
//
// A query head's index list is split over `nsplit` workgroups (split-K).  Inside a workgroup each
// wavefront gathers 16 rows per step: the 16 lanes of a DPP row load one 256 B key (and value)
// row with one 128-bit load per lane, so a wavefront load instruction covers 4 complete rows.
// Softmax is computed online in fp32 (base-2 exponent, scale * log2(e) folded into q); partial
// (m, l, o[D]) triples are merged by the last workgroup of the head to finish.
#include "sik_attn_core.h"
#include "sik_device.h"
#include "sik_internal.h"

namespace sik {

SIK_TL_DEFINE(sik_dbg_tl_attn)

template <int DT, int ODT>
__global__ __launch_bounds__(kBlock) void attn_kernel(
    // (the first 14 dwords arrive in scalar registers with the wavefront: what the first loads need comes first;
    // dims0 = Hkv | Hq << 16, dims1 = R | nsplit << 16)
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    const int32_t* __restrict__ idx, uint32_t dims0, uint32_t dims1, int k, int Lmax, int per, int idx_per_unit,
    float scale_log2e, uint32_t* __restrict__ counters, float* __restrict__ partial, void* __restrict__ out) {
    __shared__ float sm[kBlock / kWave], sl[kBlock / kWave];
    __shared__ float sacc[kBlock / kWave][kD];
    __shared__ int s_flag;

    SIK_TL(16);
    const int Hkv = dims0 & 0xffffu, Hq = dims0 >> 16, R = dims1 & 0xffffu, nsplit = dims1 >> 16;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int p = lane & 15;
    const int row = blockIdx.x / nsplit, sp = blockIdx.x % nsplit;
    const int b = row / Hq, hq = row % Hq;
    const size_t unit = static_cast<size_t>(b) * Hkv + hq / R;
    const uint4* Kp = reinterpret_cast<const uint4*>(K + unit * Lmax * kD);
    const uint4* Vp = reinterpret_cast<const uint4*>(V + unit * Lmax * kD);
    const int32_t* ip = idx + ((idx_per_unit & 1) ? unit : static_cast<size_t>(row)) * k;  // bit 1: stream

    const uint4 qraw = reinterpret_cast<const uint4*>(q + static_cast<size_t>(row) * kD)[p];

    SoftmaxState st;
    init_state(st);
    const int j0 = sp * per, j1 = min(k, j0 + per);
    auto fetch = [&](int j) { return ip[j0 + j]; };
    if (idx_per_unit & 2)
        attend_list<DT, true>(fetch, j1 - j0, wv * 16, (kBlock / kWave) * 16, Kp, Vp, qraw, scale_log2e, Lmax, st);
    else
        attend_list<DT, false>(fetch, j1 - j0, wv * 16, (kBlock / kWave) * 16, Kp, Vp, qraw, scale_log2e, Lmax, st);
    SIK_TL(17);
    float M, Lsum, o;
    workgroup_merge(st, sm, sl, sacc, M, Lsum, o);
    if (nsplit == 1) {
        if (tid < kD) store_out<ODT>(out, static_cast<size_t>(row) * kD + tid, Lsum > 0.0f ? o / Lsum : 0.0f);
        return;
    }
    float* prow = partial + (static_cast<size_t>(row) * kMaxSplit) * kPartStride;
    if (tid < kD) {
        float* pp = prow + static_cast<size_t>(sp) * kPartStride;
        st_agent(&pp[2 + tid], o);
        if (tid == 0) {
            st_agent(&pp[0], M);
            st_agent(&pp[1], Lsum);
        }
    }
    SIK_TL(18);
    if (!last_arriver(&counters[row * 8 + 3], static_cast<uint32_t>(nsplit), &s_flag)) return;
    SIK_TL_ANY(19);
    if (tid < kD) store_out<ODT>(out, static_cast<size_t>(row) * kD + tid, merge_partials(prow, nsplit, tid));
    SIK_TL_ANY(20);
}

// Group-shared selection: the query heads of a KV head attend over ONE index list (idx [B, Hkv, k]).  A workgroup
// takes a block of up to kSharedHeads query heads of one KV head and a slice of the list, gathers every row
// once and feeds it to all its heads: the gathered bytes are those of one head, not of R.

template <int DT, int ODT>
__global__ __launch_bounds__(kBlock) void attn_shared_kernel(
    // (argument order and packing as in attn_kernel)
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    const int32_t* __restrict__ idx, uint32_t dims0, uint32_t dims1, int k, int Lmax, int per, int nblk_flags,
    float scale_log2e, uint32_t* __restrict__ counters, float* __restrict__ partial, void* __restrict__ out) {
    constexpr int NH = kSharedHeads;
    const int nblk = nblk_flags & 0xffff;  // head blocks per KV head; bit 16: non-temporal row loads
    __shared__ float sm[kBlock / kWave], sl[kBlock / kWave];
    __shared__ float sacc[kBlock / kWave][kD];
    __shared__ int s_flag;

    const int Hkv = dims0 & 0xffffu, Hq = dims0 >> 16, R = dims1 & 0xffffu, nsplit = dims1 >> 16;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int p = lane & 15;
    const int sp = blockIdx.x % nsplit, ub = blockIdx.x / nsplit;
    const int blk = ub % nblk;
    const size_t unit = ub / nblk;
    const int b = static_cast<int>(unit / Hkv), h = static_cast<int>(unit % Hkv);
    const int hq0 = h * R + blk * NH;          // first query head of this workgroup
    const int nh = min(NH, R - blk * NH);      // real heads in the block
    const size_t row0 = static_cast<size_t>(b) * Hq + hq0;
    const uint4* Kp = reinterpret_cast<const uint4*>(K + unit * Lmax * kD);
    const uint4* Vp = reinterpret_cast<const uint4*>(V + unit * Lmax * kD);
    const int32_t* ip = idx + unit * k;

    uint4 qraw[NH];
    SoftmaxState st[NH];
#pragma unroll
    for (int x = 0; x < NH; ++x) {
        qraw[x] = x < nh ? reinterpret_cast<const uint4*>(q + (row0 + x) * kD)[p] : make_uint4(0u, 0u, 0u, 0u);
        init_state(st[x]);
    }
    const int j0 = sp * per, j1 = min(k, j0 + per);
    auto fetch = [&](int j) { return ip[j0 + j]; };
    if (nblk_flags >> 16)
        attend_list_multi<DT, NH, true>(fetch, j1 - j0, wv * 16, (kBlock / kWave) * 16, Kp, Vp, qraw, scale_log2e,
                                        Lmax, st);
    else
        attend_list_multi<DT, NH, false>(fetch, j1 - j0, wv * 16, (kBlock / kWave) * 16, Kp, Vp, qraw, scale_log2e,
                                         Lmax, st);
    float M[NH], Lsum[NH], o[NH];
#pragma unroll
    for (int x = 0; x < NH; ++x) {
        workgroup_merge(st[x], sm, sl, sacc, M[x], Lsum[x], o[x]);
        __syncthreads();  // the LDS staging is reused by the next head
    }
    if (nsplit == 1) {
#pragma unroll
        for (int x = 0; x < NH; ++x)
            if (x < nh && tid < kD)
                store_out<ODT>(out, (row0 + x) * kD + tid, Lsum[x] > 0.0f ? o[x] / Lsum[x] : 0.0f);
        return;
    }
#pragma unroll
    for (int x = 0; x < NH; ++x) {
        if (x < nh && tid < kD) {
            float* pp = partial + ((row0 + x) * kMaxSplit + sp) * kPartStride;
            st_agent(&pp[2 + tid], o[x]);
            if (tid == 0) {
                st_agent(&pp[0], M[x]);
                st_agent(&pp[1], Lsum[x]);
            }
        }
    }
    if (!last_arriver(&counters[row0 * 8 + 3], static_cast<uint32_t>(nsplit), &s_flag)) return;
    // two heads at a time: threads 0..127 and 128..255 each take a channel of one head
    for (int x = tid >> 7; x < nh; x += kBlock / kD)
        store_out<ODT>(out, (row0 + x) * kD + (tid & (kD - 1)),
                       merge_partials(partial + (row0 + x) * kMaxSplit * kPartStride, nsplit, tid & (kD - 1)));
}

static void attn_plan(const Dims& d, int k, int* nsplit, int* per) {
    const int rows = d.rows();
    int ns = (1024 + rows - 1) / rows;
    const int by_k = (k + 63) / 64;
    if (ns > by_k) ns = by_k;
    if (ns > kMaxSplit) ns = kMaxSplit;
    if (ns < 1) ns = 1;
    int pr = (k + ns - 1) / ns;
    pr = (pr + 63) / 64 * 64;
    *per = pr;
    *nsplit = (k + pr - 1) / pr;
}

hipError_t launch_attn(const Dims& d, const Workspace& w, const void* q, const void* K, const void* V,
                       const int32_t* idx, bool idx_per_unit, int k, float scale, void* out, hipStream_t s) {
    if (idx_per_unit && d.R > 1) {
        // one gather per block of up to 4 query heads; splits planned over those blocks
        const int nblk = (d.R + kSharedHeads - 1) / kSharedHeads;
        Dims db = d;
        db.Hq = d.Hkv * nblk;
        int nsplit, per;
        attn_plan(db, k, &nsplit, &per);
        const float sl2 = (scale > 0.0f ? scale : 1.0f / sqrtf(static_cast<float>(d.D))) * 1.4426950408889634f;
        const int grid = nsplit * d.units() * nblk;
        // every selected row is gathered once per head block here
        const bool stream = static_cast<int64_t>(d.units()) * nblk * k * 512 >= (64ll << 20);
        const uint32_t dims0 = static_cast<uint32_t>(d.Hkv) | static_cast<uint32_t>(d.Hq) << 16;
        const uint32_t dims1 = static_cast<uint32_t>(d.R) | static_cast<uint32_t>(nsplit) << 16;
        auto qp = static_cast<const uint16_t*>(q);
        auto Kp = static_cast<const uint16_t*>(K);
        auto Vp = static_cast<const uint16_t*>(V);
#define SIK_ATTNS(DTV, ODTV)                                                                                  \
    launch_kernel(attn_shared_kernel<DTV, ODTV>, grid, kBlock, s, qp, Kp, Vp, idx, dims0, dims1, k, d.Lmax, per, \
                  nblk | (stream ? 1 << 16 : 0), sl2, w.counters, w.partial, out)
        if (d.kv_dtype == kBF16) return d.out_dtype == kF32 ? SIK_ATTNS(kBF16, kF32) : SIK_ATTNS(kBF16, kBF16);
        return d.out_dtype == kF32 ? SIK_ATTNS(kF16, kF32) : SIK_ATTNS(kF16, kF16);
#undef SIK_ATTNS
    }
    int nsplit, per;
    attn_plan(d, k, &nsplit, &per);
    const float sl2 = (scale > 0.0f ? scale : 1.0f / sqrtf(static_cast<float>(d.D))) * 1.4426950408889634f;
    const int grid = nsplit * d.rows();
    const uint32_t dims0 = static_cast<uint32_t>(d.Hkv) | static_cast<uint32_t>(d.Hq) << 16;
    const uint32_t dims1 = static_cast<uint32_t>(d.R) | static_cast<uint32_t>(nsplit) << 16;
    auto qp = static_cast<const uint16_t*>(q);
    auto Kp = static_cast<const uint16_t*>(K);
    auto Vp = static_cast<const uint16_t*>(V);
#define SIK_ATTN(DTV, ODTV)                                                                                  \
    launch_kernel(attn_kernel<DTV, ODTV>, grid, kBlock, s, qp, Kp, Vp, idx, dims0, dims1, k, d.Lmax, per,      \
                  (idx_per_unit ? 1 : 0) | (gather_streams(d, k) ? 2 : 0), sl2, w.counters, w.partial, out)
    if (d.kv_dtype == kBF16) return d.out_dtype == kF32 ? SIK_ATTN(kBF16, kF32) : SIK_ATTN(kBF16, kBF16);
    return d.out_dtype == kF32 ? SIK_ATTN(kF16, kF32) : SIK_ATTN(kF16, kF16);
#undef SIK_ATTN
}

}  // namespace sik
