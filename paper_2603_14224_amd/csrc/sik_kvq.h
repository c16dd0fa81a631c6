// 2-bit token-wise K/V format (section "Token-Wise Quantization Format"): building one token's record
// and attending over gathered records, at wavefront level.
//
// Record = 128 B per (sequence, KV head, token) = 16 slots of 8 B; slot p covers channels 8p .. 8p+7, the
// channels one lane of a 16-lane row owns everywhere in this library:
//   byte 0    sign byte p of the token's 1-bit code (bit 7-e = [K >= mu] of channel 8p+e)
//   byte 1    0
//   bytes 2-3 K magnitude codes, little-endian: code of channel 8p+e in bits 2e+1:2e
//   bytes 4-5 V codes, same packing
//   bytes 6-7 one fp16 parameter of the 32-channel group p/4: K qs, K zp, V qs, V zp for p mod 4 = 0, 1, 2, 3
// so the four lanes of a quad hold the four parameters of their common group, one quad-permute away, and a
// selected token costs one 128 B line instead of 2 x 256 B of 16-bit rows.
//
// Quantisation of a group x[0..31] (B = 2): zp = fp16(min x), qs = fp16((max x - min x) / 3),
// Q = clamp(rint((x - zp) * (1 / qs)), 0, 3) with the stored qs, zp (qs = 0 gives Q = 0), D = qs Q + zp.
// V: x = the value.  K: x = |K - mu| * (1 / alpha) (alpha = per-channel max of |K - mu| over the fitted
// tokens; alpha = 0 gives x = 0), the sign travels as the code bit: K' ~ s alpha D.
// The codes are decided in binary32 in exactly this operation order: the two divisions of the paper's
// formulas are multiplications by a correctly rounded reciprocal (one per channel, one per group), which keeps
// the quantiser bound by memory instead of by per-element divisions.
#pragma once

#include "sik_attn_core.h"
#include "sik_device.h"

namespace sik {

constexpr int kRecBytes = 128;  // bytes per token record
constexpr int kRecSlots = 16;   // uint2 slots per record

// Value of lane (quad base + J) for every lane of the quad (DPP quad_perm broadcast).
template <int J>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t v) {
    return static_cast<uint32_t>(
        __builtin_amdgcn_update_dpp(0, static_cast<int>(v), J * 0x55, 0xf, 0xf, false));
}
__device__ __forceinline__ float quad_min(float v) {
    v = fminf(v, __uint_as_float(static_cast<uint32_t>(
                     __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xb1, 0xf, 0xf, false))));  // lanes 1,0,3,2
    return fminf(v, __uint_as_float(static_cast<uint32_t>(
                        __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4e, 0xf, 0xf, false))));  // lanes 2,3,0,1
}
__device__ __forceinline__ float quad_max(float v) {
    v = fmaxf(v, __uint_as_float(static_cast<uint32_t>(
                     __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xb1, 0xf, 0xf, false))));
    return fmaxf(v, __uint_as_float(static_cast<uint32_t>(
                        __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4e, 0xf, 0xf, false))));
}

__device__ __forceinline__ uint32_t fp16_bits(float f) {
    return __builtin_bit_cast(uint16_t, static_cast<_Float16>(f));  // round to nearest even
}
__device__ __forceinline__ float fp16_value(uint32_t h) {
    return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(h)));
}

// Minimum / maximum over the 8 lanes 8j .. 8j+7 (every lane gets it): the quad, then the other quad of the
// half row (row_half_mirror: lane i of each 8 reads lane 7 - i, which holds its own quad's result).
__device__ __forceinline__ float oct_min(float v) {
    v = quad_min(v);
    return fminf(v, __uint_as_float(static_cast<uint32_t>(
                        __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false))));
}
__device__ __forceinline__ float oct_max(float v) {
    v = quad_max(v);
    return fmaxf(v, __uint_as_float(static_cast<uint32_t>(
                        __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false))));
}

// x / 3 rounded to nearest, in three instructions: the product with the rounded 1/3 is at most one unit off, the
// fused residual x - 3 q is exact, and the correction lands on the correctly rounded quotient (checked against the
// division for every mantissa; a quotient in the subnormal range may differ in its last bit, and rounds to a
// zero fp16 step either way).
__device__ __forceinline__ float third(float x) {
    constexpr float c = 1.0f / 3.0f;
    const float q = x * c;
    return fmaf(fmaf(-3.0f, q, x), c, q);
}

// 1 / x for a normal positive x: the hardware estimate (one unit in the last place) and one Newton step, which
// leaves the correctly rounded reciprocal except next to a rounding tie.
__device__ __forceinline__ float reciprocal(float x) {
    const float r = __builtin_amdgcn_rcpf(x);
    return fmaf(fmaf(-x, r, 1.0f), r, r);
}

// Parameters and 2-bit codes of this lane's N values of one 32-value group that 32 / N neighbouring lanes hold
// together (all of them active); group_min / group_max reduce over those lanes.  Returns the 2 N code bits
// (value e in bits 2e+1:2e); qs_h, zp_h = the stored fp16 bits.  One function for every lane mapping, so that
// every kernel that builds records takes the same decisions.
template <int N, class GroupMin, class GroupMax>
__device__ __forceinline__ uint32_t quantize_lane(const float (&x)[N], GroupMin group_min, GroupMax group_max,
                                                  uint32_t& qs_h, uint32_t& zp_h) {
    float lo = x[0], hi = x[0];
#pragma unroll
    for (int e = 1; e < N; ++e) {
        lo = fminf(lo, x[e]);
        hi = fmaxf(hi, x[e]);
    }
    lo = group_min(lo) + 0.0f;  // a zero minimum is stored as +0 whatever the signs of the zeros
    hi = group_max(hi);
    qs_h = fp16_bits(third(hi - lo));
    zp_h = fp16_bits(lo);
    const float qs = fp16_value(qs_h), zp = fp16_value(zp_h);
    // The code word is assembled in floating point: sum_e c_e 4^e with c_e in {0, 1, 2, 3} stays below 2^16 and is
    // exact in binary32, so one fused multiply-add per value replaces a conversion, a shift and an OR.
    float word = 0.0f;
    if (qs > 0.0f) {
        const float rqs = reciprocal(qs);
#pragma unroll
        for (int e = 0; e < N; ++e) {
            const float c = __builtin_amdgcn_fmed3f(rintf((x[e] - zp) * rqs), 0.0f, 3.0f);  // clamp to [0, 3]
            word = fmaf(c, static_cast<float>(1u << (2 * e)), word);
        }
    }
    return static_cast<uint32_t>(word);
}

// 8 values per lane, the group in the 4 lanes of a quad (the 16-lanes-per-row mapping).
__device__ __forceinline__ uint32_t quantize_octet(const float (&x)[8], uint32_t& qs_h, uint32_t& zp_h) {
    return quantize_lane<8>(x, [](float v) { return quad_min(v); }, [](float v) { return quad_max(v); }, qs_h, zp_h);
}

// 1 / alpha, and 0 for a channel that never leaves its mean.
__device__ __forceinline__ float alpha_reciprocal(float alpha) { return alpha > 0.0f ? 1.0f / alpha : 0.0f; }

// One 8-byte slot of a token's record from this lane's 8 key and 8 value elements (16-bit storage form),
// the channel means and alpha reciprocals of the same 8 channels, and p = slot index (lane within the
// 16-lane row).
template <int DT>
__device__ __forceinline__ uint2 kvq_make_slot(const uint4 kraw, const uint4 vraw, const float (&mu)[8],
                                               const float (&ralpha)[8], int p) {
    float kf[8], vf[8], kh[8];
    widen8<DT>(kraw, kf);
    widen8<DT>(vraw, vf);
    uint32_t sign = 0u;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        sign |= (kf[e] >= mu[e] ? 1u : 0u) << (7 - e);
        const float kp = kf[e] - mu[e];
        kh[e] = fabsf(kp) * ralpha[e];
    }
    uint32_t kqs, kzp, vqs, vzp;
    const uint32_t kbits = quantize_octet(kh, kqs, kzp);
    const uint32_t vbits = quantize_octet(vf, vqs, vzp);
    const int which = p & 3;
    const uint32_t par = which == 0 ? kqs : (which == 1 ? kzp : (which == 2 ? vqs : vzp));
    return make_uint2(sign | (kbits << 16), vbits | (par << 16));
}

// What a lane keeps of the query for logits against records: |q_e alpha_e| and, packed like a sign byte
// (bit 7-e), the sign of q_e alpha_e, for its 8 channels.  q . K' = sum_e q_e s_e alpha_e D_e.
struct Q2Query {
    float absqa[8];
    uint32_t neg;  // bit 7-e set: q_e alpha_e < 0
};

template <int DT>
__device__ __forceinline__ Q2Query q2_prepare(const uint4 qraw, const float (&alpha)[8]) {
    Q2Query r;
    float qf[8];
    widen8<DT>(qraw, qf);
    r.neg = 0u;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float qa = qf[e] * alpha[e];
        r.absqa[e] = fabsf(qa);
        r.neg |= (qa < 0.0f ? 1u : 0u) << (7 - e);
    }
    return r;
}

// attend_list over records: same contract as attend_list (entries first + it * step + 0..31 per wavefront
// iteration, 8 rows per 16-lane group so that 8 x 8 B loads are in flight per lane).  rec = the (sequence,
// KV head)'s records as uint2 slots.
template <class Fetch>
__device__ __forceinline__ void attend_list_q2(Fetch fetch, int n, int first, int step,
                                               const uint2* __restrict__ rec, const Q2Query& qq,
                                               float scale_log2e, int Lmax, SoftmaxState& st) {
    constexpr int U = 8;
    const int lane = threadIdx.x & 63;
    const int slot = lane >> 4, p = lane & 15;
    float zsum = 0.0f;  // sum of weight * V zero point: the same for this lane's 8 channels
    for (int base = first; base < n; base += step) {
        const int jj = base + (lane & 31);
        const int mine = jj < n ? fetch(jj) : -1;
        int id[U];
        uint2 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            id[u] = __shfl(mine, 4 * u + slot, 64);
            const bool ok = id[u] >= 0 && id[u] < Lmax;
            const size_t t = ok ? static_cast<size_t>(id[u]) : 0;
            id[u] = ok ? id[u] : -1;
            r[u] = rec[t * kRecSlots + p];
        }
        float z[U], vqs[U], vzp[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t par = r[u].y >> 16;
            const float kqs = fp16_value(quad_bcast<0>(par)), kzp = fp16_value(quad_bcast<1>(par));
            vqs[u] = fp16_value(quad_bcast<2>(par));
            vzp[u] = fp16_value(quad_bcast<3>(par));
            // sign of the product q_e alpha_e K'_e: minus where exactly one of (code bit clear, q alpha < 0)
            const uint32_t flip = ((~r[u].x) ^ qq.neg) << 24;  // bit 31-e = flip channel e
            const uint32_t kb = r[u].x >> 16;
            float a = 0.0f, bsum = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float t = __uint_as_float(__float_as_uint(qq.absqa[e]) | ((flip << e) & 0x80000000u));
                const float c = static_cast<float>((kb >> (2 * e)) & 3u);
                a = fmaf(t, c, a);
                bsum += t;
            }
            const float dot = row16_sum(fmaf(kqs, a, kzp * bsum)) * scale_log2e;
            z[u] = id[u] >= 0 ? dot : kNegBig;
        }
        float mnew = st.m;
#pragma unroll
        for (int u = 0; u < U; ++u) mnew = fmaxf(mnew, z[u]);
        const float corr = fast_exp2(st.m - mnew);
        st.l *= corr;
        zsum *= corr;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[e] *= corr;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float pu = id[u] >= 0 ? fast_exp2(z[u] - mnew) : 0.0f;
            st.l += pu;
            const float ps = pu * vqs[u];
            zsum = fmaf(pu, vzp[u], zsum);
            const uint32_t vb = r[u].y;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                st.acc[e] = fmaf(ps, static_cast<float>((vb >> (2 * e)) & 3u), st.acc[e]);
        }
        st.m = mnew;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] += zsum;
}

// attend_list_q2 for NH query heads that share one index list (group-shared selection): every record is
// gathered and dequantised once - K'_e / alpha_e = s_e (qs Q_e + zp) per channel - and each head then costs one
// multiply-add per channel against its q_e alpha_e (qa[h][e]).  Entries first + it * step + (0..15) per wavefront
// iteration (4 rows per 16-lane group); step is a multiple of 16.
template <int NH, class Fetch>
__device__ __forceinline__ void attend_list_q2_multi(Fetch fetch, int n, int first, int step,
                                                     const uint2* __restrict__ rec, const float (&qa)[NH][8],
                                                     float scale_log2e, int Lmax, SoftmaxState (&st)[NH]) {
    constexpr int U = 4;
    const int lane = threadIdx.x & 63;
    const int slot = lane >> 4, p = lane & 15;
    float zsum[NH];  // sum of weight * V zero point per head: the same for this lane's 8 channels
#pragma unroll
    for (int h = 0; h < NH; ++h) zsum[h] = 0.0f;
    for (int base = first; base < n; base += step) {
        const int jj = base + p;
        const int mine = jj < n ? fetch(jj) : -1;
        int id[U];
        uint2 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            id[u] = __shfl(mine, (lane & 48) + 4 * u + slot, 64);
            const bool ok = id[u] >= 0 && id[u] < Lmax;
            const size_t t = ok ? static_cast<size_t>(id[u]) : 0;
            id[u] = ok ? id[u] : -1;
            r[u] = rec[t * kRecSlots + p];
        }
        float z[NH][U], vqs[U], vzp[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t par = r[u].y >> 16;
            const float kqs = fp16_value(quad_bcast<0>(par)), kzp = fp16_value(quad_bcast<1>(par));
            vqs[u] = fp16_value(quad_bcast<2>(par));
            vzp[u] = fp16_value(quad_bcast<3>(par));
            const uint32_t kb = r[u].x >> 16;
            const uint32_t minus = (~r[u].x) << 24;  // bit 31-e set: K' of channel e is negative (code bit clear)
            float w[8];                              // K'_e / alpha_e
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float mag = fmaf(kqs, static_cast<float>((kb >> (2 * e)) & 3u), kzp);  // >= 0
                w[e] = __uint_as_float(__float_as_uint(mag) | ((minus << e) & 0x80000000u));
            }
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                float dot = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) dot = fmaf(qa[h][e], w[e], dot);
                dot = row16_sum(dot) * scale_log2e;
                z[h][u] = id[u] >= 0 ? dot : kNegBig;
            }
        }
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            float mnew = st[h].m;
#pragma unroll
            for (int u = 0; u < U; ++u) mnew = fmaxf(mnew, z[h][u]);
            const float corr = fast_exp2(st[h].m - mnew);
            st[h].l *= corr;
            zsum[h] *= corr;
#pragma unroll
            for (int e = 0; e < 8; ++e) st[h].acc[e] *= corr;
            st[h].m = mnew;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t vb = r[u].y;
            float cv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) cv[e] = static_cast<float>((vb >> (2 * e)) & 3u);
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                const float pu = id[u] >= 0 ? fast_exp2(z[h][u] - st[h].m) : 0.0f;
                st[h].l += pu;
                const float ps = pu * vqs[u];
                zsum[h] = fmaf(pu, vzp[u], zsum[h]);
#pragma unroll
                for (int e = 0; e < 8; ++e) st[h].acc[e] = fmaf(ps, cv[e], st[h].acc[e]);
            }
        }
    }
#pragma unroll
    for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int e = 0; e < 8; ++e) st[h].acc[e] += zsum[h];
}

}  // namespace sik
