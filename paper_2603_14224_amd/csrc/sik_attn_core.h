// Wavefront-level building blocks of the sparse attention kernels (gfx950): 16 lanes gather one
// 256 B key/value row with one 128-bit load each, online softmax in fp32 with a base-2 exponent.
#pragma once

#include "sik_device.h"

namespace sik {

constexpr int kPartStride = kD + 2;
constexpr int kSharedHeads = 4;  // query heads that share one gather in the group-shared attention kernels

struct SoftmaxState {
    float m, l;
    float acc[8];
};

__device__ __forceinline__ void merge_from_lane(SoftmaxState& st, int xor_mask) {
    const float mo = __shfl_xor(st.m, xor_mask, 64);
    const float lo = __shfl_xor(st.l, xor_mask, 64);
    const float M = fmaxf(st.m, mo);
    const float a = fast_exp2(st.m - M), b = fast_exp2(mo - M);
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

// One 16-byte slice of a gathered row.  stream: a non-temporal load - in large launches every row is read once
// by its query head and should not displace the code plane, the scores and the exchange data from the caches
// (32 x 8 KV heads x 16K: selection + attention 67.8 -> 64.2 us and the scoring launch that follows 30.4 -> 28 us);
// in small launches the plain load is faster (one sequence, 32K context: 13.2 against 14.6 us).
template <bool STREAM>
__device__ __forceinline__ uint4 load_row_slice(const uint4* p) {
    if constexpr (STREAM)
        return ld_stream(p);
    else
        return *p;
}

// Attend over token indices supplied by fetch(j): this wavefront takes entries first + it * step +
// (0..15), it = 0, 1, ... while below n (a workgroup sharing one list uses first = 16 * wave,
// step = 64; a wavefront with a private list first = 0, step = 16).  Negative or out-of-range
// entries are skipped.  qraw holds this lane's 8 query components in their 16-bit storage form; the
// logit is (q . k) * scale_log2e + zbias with scale_log2e = softmax_scale * log2(e); zbias (one constant per
// query) lets rows of an uncentred key share a softmax with logits taken against the centred key.
template <int DT, bool STREAM = false, class Fetch>
__device__ __forceinline__ void attend_list(Fetch fetch, int n, int first, int step,
                                            const uint4* __restrict__ Kp, const uint4* __restrict__ Vp,
                                            const uint4 qraw, float scale_log2e, int Lmax, SoftmaxState& st,
                                            float zbias = 0.0f) {
    const int lane = threadIdx.x & 63;
    const int slot = lane >> 4, p = lane & 15;
    for (int base = first; base < n; base += step) {
        const int jj = base + p;
        const int mine = jj < n ? fetch(jj) : -1;
        int id[4];
        uint4 kv[4], vv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            id[u] = __shfl(mine, (lane & 48) + 4 * u + slot, 64);
            const bool ok = id[u] >= 0 && id[u] < Lmax;
            const size_t r = ok ? static_cast<size_t>(id[u]) : 0;
            id[u] = ok ? id[u] : -1;
            kv[u] = load_row_slice<STREAM>(&Kp[r * 16 + p]);
            vv[u] = load_row_slice<STREAM>(&Vp[r * 16 + p]);
        }
        float z[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float dot = dot2_acc<DT>(qraw.x, kv[u].x, 0.0f);
            dot = dot2_acc<DT>(qraw.y, kv[u].y, dot);
            dot = dot2_acc<DT>(qraw.z, kv[u].z, dot);
            dot = dot2_acc<DT>(qraw.w, kv[u].w, dot);
            dot = fmaf(row16_sum(dot), scale_log2e, zbias);
            z[u] = id[u] >= 0 ? dot : kNegBig;
        }
        const float mnew = fmaxf(fmaxf(st.m, fmaxf(z[0], z[1])), fmaxf(z[2], z[3]));
        const float corr = fast_exp2(st.m - mnew);
        st.l *= corr;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[e] *= corr;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float pu = id[u] >= 0 ? fast_exp2(z[u] - mnew) : 0.0f;
            float vf[8];
            widen8<DT>(vv[u], vf);
            st.l += pu;
#pragma unroll
            for (int e = 0; e < 8; ++e) st.acc[e] = fmaf(pu, vf[e], st.acc[e]);
        }
        st.m = mnew;
    }
}

// attend_list for NH query heads that share one index list (group-shared selection): every row is gathered once
// and used NH times.  qraw[h] / st[h]: query slice and softmax state of head h.
template <int DT, int NH, bool STREAM = false, class Fetch>
__device__ __forceinline__ void attend_list_multi(Fetch fetch, int n, int first, int step,
                                                  const uint4* __restrict__ Kp, const uint4* __restrict__ Vp,
                                                  const uint4 (&qraw)[NH], float scale_log2e, int Lmax,
                                                  SoftmaxState (&st)[NH]) {
    const int lane = threadIdx.x & 63;
    const int slot = lane >> 4, p = lane & 15;
    for (int base = first; base < n; base += step) {
        const int jj = base + p;
        const int mine = jj < n ? fetch(jj) : -1;
        int id[4];
        uint4 kv[4], vv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            id[u] = __shfl(mine, (lane & 48) + 4 * u + slot, 64);
            const bool ok = id[u] >= 0 && id[u] < Lmax;
            const size_t r = ok ? static_cast<size_t>(id[u]) : 0;
            id[u] = ok ? id[u] : -1;
            kv[u] = load_row_slice<STREAM>(&Kp[r * 16 + p]);
            vv[u] = load_row_slice<STREAM>(&Vp[r * 16 + p]);
        }
        float z[NH][4];
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            float mnew = st[h].m;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float dot = dot2_acc<DT>(qraw[h].x, kv[u].x, 0.0f);
                dot = dot2_acc<DT>(qraw[h].y, kv[u].y, dot);
                dot = dot2_acc<DT>(qraw[h].z, kv[u].z, dot);
                dot = dot2_acc<DT>(qraw[h].w, kv[u].w, dot);
                dot = row16_sum(dot) * scale_log2e;
                z[h][u] = id[u] >= 0 ? dot : kNegBig;
                mnew = fmaxf(mnew, z[h][u]);
            }
            const float corr = fast_exp2(st[h].m - mnew);
            st[h].l *= corr;
#pragma unroll
            for (int e = 0; e < 8; ++e) st[h].acc[e] *= corr;
            st[h].m = mnew;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float vf[8];
            widen8<DT>(vv[u], vf);
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                const float pu = id[u] >= 0 ? fast_exp2(z[h][u] - st[h].m) : 0.0f;
                st[h].l += pu;
#pragma unroll
                for (int e = 0; e < 8; ++e) st[h].acc[e] = fmaf(pu, vf[e], st[h].acc[e]);
            }
        }
    }
}

// Combine the wavefronts' states into one (M, l, o[d]) triple of the workgroup: after the call
// thread d < kD holds o[d]; M and l are returned to every thread.  sm/sl: LDS [4], sacc: LDS [4][kD].
__device__ __forceinline__ void workgroup_merge(SoftmaxState& st, float* sm, float* sl, float (*sacc)[kD],
                                                float& M, float& Lsum, float& o) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int slot = lane >> 4, p = lane & 15;
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
    M = kNegBig;
    Lsum = 0.0f;
    o = 0.0f;
#pragma unroll
    for (int w = 0; w < kBlock / kWave; ++w) M = fmaxf(M, sm[w]);
#pragma unroll
    for (int w = 0; w < kBlock / kWave; ++w) {
        const float a = fast_exp2(sm[w] - M);
        Lsum += sl[w] * a;
        if (tid < kD) o += sacc[w][tid] * a;
    }
}

// Final value of channel d of one output row from the nsplit (m, l, o[D]) partials that its workgroups published
// (prow = the row's partial area): one pass in split order - the result does not depend on the arrival order -
// with 8 splits' loads in flight at a time.
__device__ __forceinline__ float merge_partials(const float* prow, int nsplit, int d) {
    float Mg = kNegBig, lt = 0.0f, ot = 0.0f;
    for (int s0 = 0; s0 < nsplit; s0 += 8) {
        float m[8], l[8], o[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float* pp = prow + static_cast<size_t>(s0 + j) * kPartStride;
            const bool on = s0 + j < nsplit;
            m[j] = on ? ld_agent(&pp[0]) : kNegBig;
            l[j] = on ? ld_agent(&pp[1]) : 0.0f;
            o[j] = on ? ld_agent(&pp[2 + d]) : 0.0f;
        }
        float Mb = Mg;
#pragma unroll
        for (int j = 0; j < 8; ++j) Mb = fmaxf(Mb, m[j]);
        const float keep = fast_exp2(Mg - Mb);
        lt *= keep;
        ot *= keep;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float a = fast_exp2(m[j] - Mb);
            lt += l[j] * a;
            ot += o[j] * a;
        }
        Mg = Mb;
    }
    return lt > 0.0f ? ot / lt : 0.0f;
}

__device__ __forceinline__ void init_state(SoftmaxState& st) {
    st.m = kNegBig;
    st.l = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] = 0.0f;
}

}  // namespace sik
