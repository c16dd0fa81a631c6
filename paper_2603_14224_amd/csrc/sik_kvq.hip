// 2-bit token-wise K/V cache for gfx950 (section "Token-Wise Quantization Format"): the per-channel alpha of
// the key magnitudes, the quantiser that writes one 128-byte record per token, and sparse attention that
// gathers records instead of 16-bit rows ("fused dequantisation": the rows are never materialised).
//
// Everything here is bound by HBM traffic: the quantiser reads 512 B and writes 128 B per token, attention
// reads 128 B per selected (query head, token) - a quarter of the 16-bit form.
#include "sik_kvq.h"

#include "sik_internal.h"

namespace sik {

// alpha starts at zero; non-negative floats order like their bit patterns, so the maximum is an integer max.
__global__ void alpha_clear_kernel(float* __restrict__ alpha, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) alpha[i] = 0.0f;
}

// alpha_d = max over tokens i < seq_len[b] of |K[i,d] - mu_d| (binary32 subtraction): per workgroup a slice
// of the tokens, 16 lanes per 256 B row, four rows in flight per lane; one atomic max per channel at the end.
template <int DT>
__global__ __launch_bounds__(kBlock) void alpha_kernel(const uint16_t* __restrict__ K,
                                                       const int32_t* __restrict__ seq_len,
                                                       const float* __restrict__ mu, float* __restrict__ alpha,
                                                       int Hkv, int Lmax, int nwg) {
    __shared__ float red[16][kD];
    const int tid = threadIdx.x, p = tid & 15, r = tid >> 4;
    const int unit = blockIdx.x / nwg, wg = blockIdx.x % nwg;
    int L = seq_len[unit / Hkv];
    L = L < 0 ? 0 : (L > Lmax ? Lmax : L);
    const int chunk = ((L + nwg - 1) / nwg + 15) & ~15;
    const int start = wg * chunk;
    const int end = min(L, start + chunk);
    const uint4* base = reinterpret_cast<const uint4*>(K + static_cast<size_t>(unit) * Lmax * kD);
    float m[8], acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int e = 0; e < 8; ++e) m[e] = mu[static_cast<size_t>(unit) * kD + 8 * p + e];
    int i = start + r;
    for (; i + 48 < end; i += 64) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = ld_stream(&base[static_cast<size_t>(i + 16 * u) * 16 + p]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float f[8];
            widen8<DT>(v[u], f);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaxf(acc[e], fabsf(f[e] - m[e]));
        }
    }
    for (; i < end; i += 16) {
        float f[8];
        widen8<DT>(base[static_cast<size_t>(i) * 16 + p], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaxf(acc[e], fabsf(f[e] - m[e]));
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[r][8 * p + e] = acc[e];
    __syncthreads();
    if (tid < kD) {
        float a = 0.0f;
#pragma unroll
        for (int rr = 0; rr < 16; ++rr) a = fmaxf(a, red[rr][tid]);
        if (a > 0.0f)
            atomic_max_u32(reinterpret_cast<uint32_t*>(alpha) + static_cast<size_t>(unit) * kD + tid,
                           __float_as_uint(a));
    }
}

// Records of tokens [t0, t0 + n) of every (b, h), or of [0, seq_len[b]) when seq_len is given: one 16-lane
// row per token (lane p = slot p), so a wavefront writes four complete 128 B records per store instruction.
template <int DT>
__global__ __launch_bounds__(kBlock) void quantize_kv_kernel(const uint16_t* __restrict__ K,
                                                             const uint16_t* __restrict__ V,
                                                             const int32_t* __restrict__ seq_len, int t0, int n,
                                                             const float* __restrict__ mu,
                                                             const float* __restrict__ alpha,
                                                             uint2* __restrict__ rec, int Hkv, int Lmax, int nwg) {
    const int tid = threadIdx.x, p = tid & 15, r = tid >> 4;
    const int unit = blockIdx.x / nwg, wg = blockIdx.x % nwg;
    int lo = t0, cnt = n;
    if (seq_len) {
        int L = seq_len[unit / Hkv];
        L = L < 0 ? 0 : (L > Lmax ? Lmax : L);
        lo = 0;
        cnt = L;
    }
    const int chunk = ((cnt + nwg - 1) / nwg + 15) & ~15;
    const int start = lo + wg * chunk;
    const int end = min(lo + cnt, start + chunk);
    const size_t row0 = static_cast<size_t>(unit) * Lmax;
    const uint4* Kb = reinterpret_cast<const uint4*>(K + row0 * kD);
    const uint4* Vb = reinterpret_cast<const uint4*>(V + row0 * kD);
    float m[8], a[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        m[e] = mu[static_cast<size_t>(unit) * kD + 8 * p + e];
        a[e] = alpha_reciprocal(alpha[static_cast<size_t>(unit) * kD + 8 * p + e]);
    }
    int i = start + r;
    for (; i + 16 < end; i += 32) {  // two rows (K and V of each) in flight per lane
        const uint4 k0 = ld_stream(&Kb[static_cast<size_t>(i) * 16 + p]), v0 = ld_stream(&Vb[static_cast<size_t>(i) * 16 + p]);
        const uint4 k1 = ld_stream(&Kb[static_cast<size_t>(i + 16) * 16 + p]),
                    v1 = ld_stream(&Vb[static_cast<size_t>(i + 16) * 16 + p]);
        st_stream(&rec[(row0 + i) * kRecSlots + p], kvq_make_slot<DT>(k0, v0, m, a, p));
        st_stream(&rec[(row0 + i + 16) * kRecSlots + p], kvq_make_slot<DT>(k1, v1, m, a, p));
    }
    for (; i < end; i += 16)
        rec[(row0 + i) * kRecSlots + p] =
            kvq_make_slot<DT>(Kb[static_cast<size_t>(i) * 16 + p], Vb[static_cast<size_t>(i) * 16 + p], m, a, p);
}

// Sparse attention over records: the split-K structure of attn_kernel with the record gather core.
template <int DT, int ODT>
__global__ __launch_bounds__(kBlock) void attn_q2_kernel(
    // (the first 14 dwords arrive in scalar registers with the wavefront: what the first loads need comes first;
    // dims0 = Hkv | Hq << 16, dims1 = R | nsplit << 16)
    const uint16_t* __restrict__ q, const uint2* __restrict__ rec, const float* __restrict__ alpha,
    const int32_t* __restrict__ idx, uint32_t dims0, uint32_t dims1, int k, int Lmax, int per, int idx_per_unit,
    float scale_log2e, uint32_t* __restrict__ counters, float* __restrict__ partial, void* __restrict__ out) {
    __shared__ float sm[kBlock / kWave], sl[kBlock / kWave];
    __shared__ float sacc[kBlock / kWave][kD];
    __shared__ int s_flag;

    const int Hkv = dims0 & 0xffffu, Hq = dims0 >> 16, R = dims1 & 0xffffu, nsplit = dims1 >> 16;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int p = lane & 15;
    const int row = blockIdx.x / nsplit, sp = blockIdx.x % nsplit;
    const int b = row / Hq, hq = row % Hq;
    const size_t unit = static_cast<size_t>(b) * Hkv + hq / R;
    const uint2* rp = rec + unit * Lmax * kRecSlots;
    const int32_t* ip = idx + (idx_per_unit ? unit : static_cast<size_t>(row)) * k;

    const uint4 qraw = reinterpret_cast<const uint4*>(q + static_cast<size_t>(row) * kD)[p];
    float a8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) a8[e] = alpha[unit * kD + 8 * p + e];
    const Q2Query qq = q2_prepare<DT>(qraw, a8);

    SoftmaxState st;
    init_state(st);
    const int j0 = sp * per, j1 = min(k, j0 + per);
    attend_list_q2([&](int j) { return ip[j0 + j]; }, j1 - j0, wv * 32, (kBlock / kWave) * 32, rp, qq, scale_log2e,
                   Lmax, st);
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
    if (!last_arriver(&counters[row * 8 + 3], static_cast<uint32_t>(nsplit), &s_flag)) return;
    if (tid < kD) store_out<ODT>(out, static_cast<size_t>(row) * kD + tid, merge_partials(prow, nsplit, tid));
}

// The same for a block of up to kSharedHeads query heads of one KV head that share an index list (group-shared
// selection): every record is gathered and dequantised once for the block.  Grid = units x head blocks x splits.
template <int DT, int ODT>
__global__ __launch_bounds__(kBlock) void attn_q2_shared_kernel(
    // (argument order and packing as in attn_q2_kernel)
    const uint16_t* __restrict__ q, const uint2* __restrict__ rec, const float* __restrict__ alpha,
    const int32_t* __restrict__ idx, uint32_t dims0, uint32_t dims1, int k, int Lmax, int per, int nblk,
    float scale_log2e, uint32_t* __restrict__ counters, float* __restrict__ partial, void* __restrict__ out) {
    constexpr int NH = kSharedHeads;
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
    const int hq0 = h * R + blk * NH;      // first query head of this workgroup
    const int nh = min(NH, R - blk * NH);  // real heads in the block
    const size_t row0 = static_cast<size_t>(b) * Hq + hq0;
    const uint2* rp = rec + unit * Lmax * kRecSlots;
    const int32_t* ip = idx + unit * k;

    float a8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) a8[e] = alpha[unit * kD + 8 * p + e];
    float qa[NH][8];  // q_e alpha_e of this lane's channels, per head
    SoftmaxState st[NH];
#pragma unroll
    for (int x = 0; x < NH; ++x) {
        const uint4 qraw =
            x < nh ? reinterpret_cast<const uint4*>(q + (row0 + x) * kD)[p] : make_uint4(0u, 0u, 0u, 0u);
        float qf[8];
        widen8<DT>(qraw, qf);
#pragma unroll
        for (int e = 0; e < 8; ++e) qa[x][e] = qf[e] * a8[e];
        init_state(st[x]);
    }
    const int j0 = sp * per, j1 = min(k, j0 + per);
    attend_list_q2_multi<NH>([&](int j) { return ip[j0 + j]; }, j1 - j0, wv * 16, (kBlock / kWave) * 16, rp, qa,
                             scale_log2e, Lmax, st);
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

static int kvq_workgroups(const Dims& d, int tokens) {
    int nwg = (tokens + 255) / 256;
    const int cap = 4096 / d.units() < 1 ? 1 : 4096 / d.units();
    if (nwg > cap) nwg = cap;
    return nwg < 1 ? 1 : nwg;
}

hipError_t launch_alpha(const Dims& d, const void* K, const int32_t* seq_len, const float* mu, float* alpha,
                        hipStream_t s) {
    const int n = d.units() * kD;
    const int nwg = kvq_workgroups(d, d.Lmax);
    auto Kp = static_cast<const uint16_t*>(K);
    alpha_clear_kernel<<<(n + kBlock - 1) / kBlock, kBlock, 0, s>>>(alpha, n);
    if (d.kv_dtype == kBF16)
        alpha_kernel<kBF16><<<d.units() * nwg, kBlock, 0, s>>>(Kp, seq_len, mu, alpha, d.Hkv, d.Lmax, nwg);
    else
        alpha_kernel<kF16><<<d.units() * nwg, kBlock, 0, s>>>(Kp, seq_len, mu, alpha, d.Hkv, d.Lmax, nwg);
    return hipGetLastError();
}

hipError_t launch_quantize_kv(const Dims& d, const void* K, const void* V, const int32_t* seq_len, int t0, int n,
                              const float* mu, const float* alpha, void* kvq, hipStream_t s) {
    const int tokens = seq_len ? d.Lmax : n;
    if (tokens == 0) return hipSuccess;
    const int nwg = kvq_workgroups(d, tokens);
    auto Kp = static_cast<const uint16_t*>(K);
    auto Vp = static_cast<const uint16_t*>(V);
    auto rp = static_cast<uint2*>(kvq);
    if (d.kv_dtype == kBF16)
        quantize_kv_kernel<kBF16><<<d.units() * nwg, kBlock, 0, s>>>(Kp, Vp, seq_len, t0, n, mu, alpha, rp, d.Hkv,
                                                                     d.Lmax, nwg);
    else
        quantize_kv_kernel<kF16><<<d.units() * nwg, kBlock, 0, s>>>(Kp, Vp, seq_len, t0, n, mu, alpha, rp, d.Hkv,
                                                                    d.Lmax, nwg);
    return hipGetLastError();
}

hipError_t launch_attn_q2(const Dims& d, const Workspace& w, const void* q, const void* kvq, const float* alpha,
                          const int32_t* idx, bool idx_per_unit, int k, float scale, void* out, hipStream_t s) {
    // one index list per KV head and a GQA group: one gather per block of up to kSharedHeads query heads
    const bool shared = idx_per_unit && d.R > 1;
    const int nblk = shared ? (d.R + kSharedHeads - 1) / kSharedHeads : 1;
    // splits of whole steps of the workgroup (4 wavefronts x 32 entries, x 16 in the shared kernel), about 1024
    // workgroups
    const int stepw = shared ? 64 : 128;
    const int rows = shared ? d.units() * nblk : d.rows();
    int ns = (1024 + rows - 1) / rows;
    const int by_k = (k + stepw - 1) / stepw;
    if (ns > by_k) ns = by_k;
    if (ns > kMaxSplit) ns = kMaxSplit;
    if (ns < 1) ns = 1;
    int per = (k + ns - 1) / ns;
    per = (per + stepw - 1) / stepw * stepw;
    const int nsplit = (k + per - 1) / per;
    const float sl2 = (scale > 0.0f ? scale : 1.0f / sqrtf(static_cast<float>(d.D))) * 1.4426950408889634f;
    const int grid = nsplit * rows;
    const uint32_t dims0 = static_cast<uint32_t>(d.Hkv) | static_cast<uint32_t>(d.Hq) << 16;
    const uint32_t dims1 = static_cast<uint32_t>(d.R) | static_cast<uint32_t>(nsplit) << 16;
    auto qp = static_cast<const uint16_t*>(q);
    auto rp = static_cast<const uint2*>(kvq);
#define SIK_ATTNQ(DTV, ODTV)                                                                                 \
    (shared ? launch_kernel(attn_q2_shared_kernel<DTV, ODTV>, grid, kBlock, s, qp, rp, alpha, idx, dims0, dims1, k, \
                            d.Lmax, per, nblk, sl2, w.counters, w.partial, out)                              \
            : launch_kernel(attn_q2_kernel<DTV, ODTV>, grid, kBlock, s, qp, rp, alpha, idx, dims0, dims1, k, d.Lmax, \
                            per, idx_per_unit ? 1 : 0, sl2, w.counters, w.partial, out))
    if (d.kv_dtype == kBF16) return d.out_dtype == kF32 ? SIK_ATTNQ(kBF16, kF32) : SIK_ATTNQ(kBF16, kBF16);
    return d.out_dtype == kF32 ? SIK_ATTNQ(kF16, kF32) : SIK_ATTNQ(kF16, kF16);
#undef SIK_ATTNQ
}

}  // namespace sik
