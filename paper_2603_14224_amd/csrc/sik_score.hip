// LUT-GEMV retrieval over the packed sign codes for gfx950 (section "Compressed-Domain
// Top-k Retrieval"): Table^(g)[j] = q^(g) . c_j^(g), score_i = sum_g Table^(g)[Code_g(k_i)].
//
// One workgroup serves one (batch, kv head) for a block of up to 4*NT query heads of its GQA
// group and a contiguous chunk of tokens.  The tables live in LDS as float4 entries holding the
// same (g, j) entry of four query heads: the 16 entries of a group span 256 B = all 64 LDS
// banks once, so the data-dependent ds_read_b128 of a wavefront (all lanes are at the same g)
// is bank-conflict free whatever the codes are.  Each lane owns one token: a single 128-bit
// load brings its 32 codes, i.e. a wavefront streams 1 KB of the code plane per load.
#include "sik_device.h"
#include "sik_internal.h"

namespace sik {

template <int DT, int NT, bool HIST>
__global__ __launch_bounds__(kBlock) void score_kernel(const uint16_t* __restrict__ q,
                                                       const float* __restrict__ codebook,
                                                       const uint8_t* __restrict__ codes,
                                                       const int32_t* __restrict__ seq_len,
                                                       float* __restrict__ scores,
                                                       uint32_t* __restrict__ hist,
                                                       float* __restrict__ binp, int Hkv, int Hq, int R,
                                                       int Lmax, int nchunk, int chunk, int nhb) {
    constexpr int HB = 4 * NT;
    __shared__ float4 lut[NT][kG * 16];
    __shared__ float qs[HB][kD];
    __shared__ float bp[HB][2];
    __shared__ uint32_t lhist[HIST ? HB * kBins : 1];

    const int tid = threadIdx.x;
    const int c = blockIdx.x % nchunk;
    const int u = blockIdx.x / nchunk;
    const int hb = u % nhb;
    const int unit = u / nhb;
    const int h = unit % Hkv, b = unit / Hkv;
    int L = seq_len[b];
    L = L > Lmax ? Lmax : L;
    const int start = c * chunk;
    if (start >= L && c != 0) return;
    const int end = min(L, start + chunk);
    const int hq0 = h * R + hb * HB;
    const int nh = min(HB, R - hb * HB);
    const size_t row0 = static_cast<size_t>(b) * Hq + hq0;

    // first code load goes out before the table build so that its latency is hidden
    const uint4* cp = reinterpret_cast<const uint4*>(codes + static_cast<size_t>(unit) * Lmax * kCodeBytes);
    int i = start + tid;
    uint4 cur = make_uint4(0u, 0u, 0u, 0u);
    if (i < end) cur = cp[i];

    for (int e = tid; e < HB * kD; e += kBlock) {
        const int s = e / kD, dd = e % kD;
        qs[s][dd] = s < nh ? widen16<DT>(q[(row0 + s) * kD + dd]) : 0.0f;
    }
    if constexpr (HIST)
        for (int e = tid; e < HB * kBins; e += kBlock) lhist[e] = 0u;
    __syncthreads();

    // Table^(g)[j] for the HB query heads, fp32
    for (int e = tid; e < kG * 16; e += kBlock) {
        const int g = e >> 4;
        const float4 cj = reinterpret_cast<const float4*>(codebook)[static_cast<size_t>(unit) * kG * 16 + e];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            float o[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float* qq = &qs[4 * t + s][4 * g];
                float a = qq[0] * cj.x;
                a = fmaf(qq[1], cj.y, a);
                a = fmaf(qq[2], cj.z, a);
                a = fmaf(qq[3], cj.w, a);
                o[s] = a;
            }
            lut[t][e] = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
    __syncthreads();

    if constexpr (HIST) {
        // Every score of head s lies in [sum_g min_j T, sum_g max_j T]; spread the bins over it.
        if (tid < HB * 32) {
            const int s = tid >> 5, g = tid & 31;
            float mx = -INFINITY, mn = INFINITY;
            for (int j = 0; j < 16; ++j) {
                const float4 v = lut[s >> 2][g * 16 + j];
                const float x = (s & 3) == 0 ? v.x : (s & 3) == 1 ? v.y : (s & 3) == 2 ? v.z : v.w;
                mx = fmaxf(mx, x);
                mn = fminf(mn, x);
            }
#pragma unroll
            for (int o = 16; o >= 1; o >>= 1) {
                mx += __shfl_xor(mx, o, 32);
                mn += __shfl_xor(mn, o, 32);
            }
            if (g == 0) {
                const float span = mx - mn;
                const float scale = span > 1e-30f ? static_cast<float>(kBins) / span : 0.0f;
                bp[s][0] = mn;
                bp[s][1] = scale;
                if (c == 0 && s < nh) {
                    binp[(row0 + s) * 2] = mn;
                    binp[(row0 + s) * 2 + 1] = scale;
                }
            }
        }
        __syncthreads();
    }

    for (int base = start; base < end; base += kBlock) {
        const bool valid = i < end;
        const uint4 code = cur;
        i += kBlock;
        if (i < end) cur = cp[i];  // prefetch the next token's codes
        float acc[HB];
#pragma unroll
        for (int s = 0; s < HB; ++s) acc[s] = 0.0f;
        const uint32_t w[4] = {code.x, code.y, code.z, code.w};
#pragma unroll
        for (int dw = 0; dw < 4; ++dw) {
#pragma unroll
            for (int by = 0; by < 4; ++by) {
                // byte (4 dw + by) of the token: high nibble = Code of group g, low nibble = group g+1
                const int g = 8 * dw + 2 * by;
                const uint32_t bits = w[dw] >> (8 * by);
                const uint32_t off_hi = bits & 0xf0u;        // Code * 16 B
                const uint32_t off_lo = (bits & 0x0fu) << 4;
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const float4 v = *reinterpret_cast<const float4*>(
                        reinterpret_cast<const char*>(&lut[t][g * 16]) + off_hi);
                    acc[4 * t + 0] += v.x;
                    acc[4 * t + 1] += v.y;
                    acc[4 * t + 2] += v.z;
                    acc[4 * t + 3] += v.w;
                }
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const float4 v = *reinterpret_cast<const float4*>(
                        reinterpret_cast<const char*>(&lut[t][(g + 1) * 16]) + off_lo);
                    acc[4 * t + 0] += v.x;
                    acc[4 * t + 1] += v.y;
                    acc[4 * t + 2] += v.z;
                    acc[4 * t + 3] += v.w;
                }
            }
        }
        if (valid) {
            const int tok = i - kBlock;
#pragma unroll
            for (int s = 0; s < HB; ++s) {
                if (s < nh) {
                    scores[(row0 + s) * Lmax + tok] = acc[s];
                    if constexpr (HIST) atomicAdd(&lhist[s * kBins + score_bin(acc[s], bp[s][0], bp[s][1])], 1u);
                }
            }
        }
    }

    if constexpr (HIST) {
        __syncthreads();
        for (int e = tid; e < nh * kBins; e += kBlock) {
            const uint32_t v = lhist[e];
            if (v) atomic_add_u32(&hist[row0 * kBins + e], v);
        }
    }
}

// Tokens per workgroup: aim at ~4 workgroups per compute unit, at least 256 tokens each.
static void score_plan(const Dims& d, int nhb, int* nchunk, int* chunk) {
    const int units = d.units() * nhb;
    int want = (1024 + units - 1) / units;  // chunks per unit
    int ch = (d.Lmax + want - 1) / want;
    ch = (ch + kBlock - 1) / kBlock * kBlock;
    if (ch < kBlock) ch = kBlock;
    if (ch > 16384) ch = 16384;
    *chunk = ch;
    *nchunk = (d.Lmax + ch - 1) / ch;
}

template <int DT>
static hipError_t launch_score_t(const Dims& d, const void* q, const float* codebook, const uint8_t* codes,
                                 const int32_t* seq_len, float* scores, uint32_t* hist, float* binp,
                                 hipStream_t s) {
    const int NT = d.R > 4 ? 2 : 1;
    const int HB = 4 * NT;
    const int nhb = (d.R + HB - 1) / HB;
    int nchunk, chunk;
    score_plan(d, nhb, &nchunk, &chunk);
    const int grid = nchunk * nhb * d.units();
    auto qp = static_cast<const uint16_t*>(q);
#define SIK_SCORE(NTV, HV)                                                                              \
    score_kernel<DT, NTV, HV><<<grid, kBlock, 0, s>>>(qp, codebook, codes, seq_len, scores, hist, binp, \
                                                      d.Hkv, d.Hq, d.R, d.Lmax, nchunk, chunk, nhb)
    if (hist) {
        if (NT == 1) SIK_SCORE(1, true); else SIK_SCORE(2, true);
    } else {
        if (NT == 1) SIK_SCORE(1, false); else SIK_SCORE(2, false);
    }
#undef SIK_SCORE
    return hipGetLastError();
}

hipError_t launch_score(const Dims& d, const void* q, const float* codebook, const uint8_t* codes,
                        const int32_t* seq_len, float* scores, uint32_t* hist, float* binp, hipStream_t s) {
    return d.kv_dtype == kBF16 ? launch_score_t<kBF16>(d, q, codebook, codes, seq_len, scores, hist, binp, s)
                               : launch_score_t<kF16>(d, q, codebook, codes, seq_len, scores, hist, binp, s);
}

}  // namespace sik
