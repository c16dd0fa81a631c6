// Sparse softmax attention over the selected tokens for gfx950:
// out = softmax(q K_S^T / sqrt(d)) V_S on the stored 16-bit K and V rows (section "Background
// and Preliminaries"; token-wise random access as argued in "Token-Wise Quantization Format").
//
// A query head's index list is split over `nsplit` workgroups (split-K).  Inside a workgroup each
// wavefront gathers 16 rows per step: the 16 lanes of a DPP row load one 256 B key (and value)
// row with one 128-bit load per lane, so a wavefront load instruction covers 4 complete rows.
// Softmax is computed online in fp32 (base-2 exponent, scale * log2(e) folded into q); partial
// (m, l, o[D]) triples are merged by the last workgroup of the head to finish.
#include "sik_device.h"
#include "sik_internal.h"

namespace sik {

SIK_TL_DEFINE(sik_dbg_tl_attn)

constexpr int kPartStride = kD + 2;

struct SoftmaxState {
    float m, l;
    float acc[8];
};

__device__ __forceinline__ void merge_from_lane(SoftmaxState& st, int xor_mask) {
    const float mo = __shfl_xor(st.m, xor_mask, 64);
    const float lo = __shfl_xor(st.l, xor_mask, 64);
    const float M = fmaxf(st.m, mo);
    const float a = exp2f(st.m - M), b = exp2f(mo - M);
    st.l = st.l * a + lo * b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float ao = __shfl_xor(st.acc[e], xor_mask, 64);
        st.acc[e] = st.acc[e] * a + ao * b;
    }
    st.m = M;
}

template <int ODT>
__device__ __forceinline__ void store_out(void* out, size_t pos, float v) {
    if constexpr (ODT == kF32)
        static_cast<float*>(out)[pos] = v;
    else
        static_cast<uint16_t*>(out)[pos] = static_cast<uint16_t>(narrow16<ODT>(v));
}

template <int DT, int ODT>
__global__ __launch_bounds__(kBlock) void attn_kernel(const uint16_t* __restrict__ q,
                                                      const uint16_t* __restrict__ K,
                                                      const uint16_t* __restrict__ V,
                                                      const int32_t* __restrict__ idx, int k,
                                                      float scale_log2e, uint32_t* __restrict__ counters,
                                                      float* __restrict__ partial, void* __restrict__ out,
                                                      int Hkv, int Hq, int R, int Lmax, int nsplit, int per) {
    __shared__ float sm[kBlock / kWave], sl[kBlock / kWave];
    __shared__ float sacc[kBlock / kWave][kD];
    __shared__ int s_flag;

    SIK_TL(16);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int slot = lane >> 4, p = lane & 15;
    const int row = blockIdx.x / nsplit, sp = blockIdx.x % nsplit;
    const int b = row / Hq, hq = row % Hq;
    const size_t unit = static_cast<size_t>(b) * Hkv + hq / R;
    const uint4* Kp = reinterpret_cast<const uint4*>(K + unit * Lmax * kD);
    const uint4* Vp = reinterpret_cast<const uint4*>(V + unit * Lmax * kD);
    const int32_t* ip = idx + static_cast<size_t>(row) * k;

    float qf[8];
    widen8<DT>(reinterpret_cast<const uint4*>(q + static_cast<size_t>(row) * kD)[p], qf);
#pragma unroll
    for (int e = 0; e < 8; ++e) qf[e] *= scale_log2e;

    SoftmaxState st;
    st.m = kNegBig;
    st.l = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] = 0.0f;

    const int j0 = sp * per, j1 = min(k, j0 + per);
    for (int base = j0 + wv * 16; base < j1; base += (kBlock / kWave) * 16) {
        const int jj = base + p;
        const int mine = jj < j1 ? ip[jj] : -1;
        int id[4];
        uint4 kv[4], vv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            id[u] = __shfl(mine, (lane & 48) + 4 * u + slot, 64);
            const bool ok = id[u] >= 0 && id[u] < Lmax;
            const size_t r = ok ? static_cast<size_t>(id[u]) : 0;
            id[u] = ok ? id[u] : -1;
            kv[u] = Kp[r * 16 + p];
            vv[u] = Vp[r * 16 + p];
        }
        float z[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float kf[8];
            widen8<DT>(kv[u], kf);
            float dot = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) dot = fmaf(qf[e], kf[e], dot);
            dot = row16_sum(dot);
            z[u] = id[u] >= 0 ? dot : kNegBig;
        }
        const float mnew = fmaxf(fmaxf(st.m, fmaxf(z[0], z[1])), fmaxf(z[2], z[3]));
        const float corr = exp2f(st.m - mnew);
        st.l *= corr;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[e] *= corr;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float pu = id[u] >= 0 ? exp2f(z[u] - mnew) : 0.0f;
            float vf[8];
            widen8<DT>(vv[u], vf);
            st.l += pu;
#pragma unroll
            for (int e = 0; e < 8; ++e) st.acc[e] = fmaf(pu, vf[e], st.acc[e]);
        }
        st.m = mnew;
    }

    SIK_TL(17);
    // the four 16-lane rows of the wavefront hold four independent partial softmaxes
    merge_from_lane(st, 16);
    merge_from_lane(st, 32);
    if (slot == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) sacc[wv][8 * p + e] = st.acc[e];
        if (p == 0) {
            sm[wv] = st.m;
            sl[wv] = st.l;
        }
    }
    __syncthreads();

    float M = kNegBig, Lsum = 0.0f, o = 0.0f;
    if (tid < kD) {
#pragma unroll
        for (int w = 0; w < kBlock / kWave; ++w) M = fmaxf(M, sm[w]);
#pragma unroll
        for (int w = 0; w < kBlock / kWave; ++w) {
            const float a = exp2f(sm[w] - M);
            Lsum += sl[w] * a;
            o += sacc[w][tid] * a;
        }
    }
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
    if (tid < kD) {
        float Mg = kNegBig;
#pragma unroll 8
        for (int s2 = 0; s2 < nsplit; ++s2) Mg = fmaxf(Mg, ld_agent(&prow[static_cast<size_t>(s2) * kPartStride]));
        float lt = 0.0f, ot = 0.0f;
#pragma unroll 8
        for (int s2 = 0; s2 < nsplit; ++s2) {  // fixed order: the result does not depend on arrival order
            const float* pp = prow + static_cast<size_t>(s2) * kPartStride;
            const float a = exp2f(ld_agent(&pp[0]) - Mg);
            lt += ld_agent(&pp[1]) * a;
            ot += ld_agent(&pp[2 + tid]) * a;
        }
        store_out<ODT>(out, static_cast<size_t>(row) * kD + tid, lt > 0.0f ? ot / lt : 0.0f);
    }
    SIK_TL_ANY(20);
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
                       const int32_t* idx, int k, float scale, void* out, hipStream_t s) {
    int nsplit, per;
    attn_plan(d, k, &nsplit, &per);
    const float sl2 = (scale > 0.0f ? scale : 1.0f / sqrtf(static_cast<float>(d.D))) * 1.4426950408889634f;
    const int grid = nsplit * d.rows();
    auto qp = static_cast<const uint16_t*>(q);
    auto Kp = static_cast<const uint16_t*>(K);
    auto Vp = static_cast<const uint16_t*>(V);
#define SIK_ATTN(DTV, ODTV)                                                                                  \
    attn_kernel<DTV, ODTV><<<grid, kBlock, 0, s>>>(qp, Kp, Vp, idx, k, sl2, w.counters, w.partial, out, d.Hkv, \
                                                   d.Hq, d.R, d.Lmax, nsplit, per)
    if (d.kv_dtype == kBF16) {
        if (d.out_dtype == kF32) SIK_ATTN(kBF16, kF32); else SIK_ATTN(kBF16, kBF16);
    } else {
        if (d.out_dtype == kF32) SIK_ATTN(kF16, kF32); else SIK_ATTN(kF16, kF16);
    }
#undef SIK_ATTN
    return hipGetLastError();
}

}  // namespace sik
