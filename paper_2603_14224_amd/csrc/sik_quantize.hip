// Sign-based 1-bit quantiser of the key cache for gfx950:
//   channel means      (section "Entropy-Aware Normalization", K' = K - mu)
//   sign Code + pack   (section "Codebook Construction", Code equation)
//   16-centroid codebook per group, one pass (centroid equation)
// plus the decode-time append of one new key/value row per head.
//
// Work split: a (batch, kv-head) "unit" owns Lmax rows of 256 B.  A workgroup of 256 threads
// reads 16 rows per step: thread (r = tid / 16, p = tid % 16) loads the 16 B holding channels
// 8p .. 8p+7 of row r, so that every wavefront load covers 4 full rows (1 KB, coalesced).
#include "sik_device.h"
#include "sik_internal.h"

namespace sik {

// ---------------------------------------------------------------------------------------
// prep: zero the per-call counters/histograms and, optionally, append one row per (b, h).
// Blocks [0, nzb) zero; block nzb + b appends for sequence b and then increments seq_len[b].
template <int DT>
__global__ __launch_bounds__(kBlock) void prep_kernel(uint32_t* __restrict__ zero_begin, size_t zero_words,
                                                      int nzb, const uint16_t* __restrict__ k_new,
                                                      const uint16_t* __restrict__ v_new,
                                                      uint16_t* __restrict__ K, uint16_t* __restrict__ V,
                                                      int32_t* __restrict__ seq_len,
                                                      const float* __restrict__ mu,
                                                      uint8_t* __restrict__ codes, int Hkv, int Lmax) {
    const int tid = threadIdx.x;
    if (static_cast<int>(blockIdx.x) < nzb) {
        uint4* z = reinterpret_cast<uint4*>(zero_begin);
        const size_t n4 = zero_words / 4;  // region length is a multiple of 64 words
        for (size_t i = static_cast<size_t>(blockIdx.x) * kBlock + tid; i < n4;
             i += static_cast<size_t>(nzb) * kBlock)
            z[i] = make_uint4(0u, 0u, 0u, 0u);
        return;
    }
    const int b = static_cast<int>(blockIdx.x) - nzb;
    const int t = seq_len[b];
    if (t < 0 || t >= Lmax) return;  // no room: nothing is appended, the length stays
    const int p = tid & 15;
    for (int h = tid >> 4; h < Hkv; h += kBlock / 16) {
        const size_t unit = static_cast<size_t>(b) * Hkv + h;
        const uint4 kv = reinterpret_cast<const uint4*>(k_new + unit * kD)[p];
        const uint4 vv = reinterpret_cast<const uint4*>(v_new + unit * kD)[p];
        const size_t row = unit * Lmax + t;
        reinterpret_cast<uint4*>(K + row * kD)[p] = kv;
        reinterpret_cast<uint4*>(V + row * kD)[p] = vv;
        float f[8];
        widen8<DT>(kv, f);
        const float4 m0 = reinterpret_cast<const float4*>(mu + unit * kD)[2 * p];
        const float4 m1 = reinterpret_cast<const float4*>(mu + unit * kD)[2 * p + 1];
        const float m[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
        uint32_t byte = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) byte |= (f[e] >= m[e] ? 1u : 0u) << (7 - e);
        codes[row * kCodeBytes + p] = static_cast<uint8_t>(byte);
    }
    __syncthreads();
    if (tid == 0) seq_len[b] = t + 1;
}

// ---------------------------------------------------------------------------------------
// fit step 1: per-workgroup partial column sums in fp64 (the 16-bit inputs are exact in fp64,
// so the mean rounded to fp32 is reproducible and independent of the launch shape up to fp64
// rounding).  colsum[unit][wg][d].
template <int DT>
__global__ __launch_bounds__(kBlock) void colsum_kernel(const uint16_t* __restrict__ K,
                                                        const int32_t* __restrict__ seq_len,
                                                        double* __restrict__ colsum, int Hkv, int Lmax,
                                                        int nwg) {
    __shared__ double red[16][kD];
    const int tid = threadIdx.x, p = tid & 15, r = tid >> 4;
    const int unit = blockIdx.x / nwg, wg = blockIdx.x % nwg;
    const int b = unit / Hkv;
    int L = seq_len[b];
    L = L < 0 ? 0 : (L > Lmax ? Lmax : L);
    const int chunk = ((L + nwg - 1) / nwg + 15) & ~15;
    const int start = wg * chunk;
    const int end = min(L, start + chunk);
    const uint4* base = reinterpret_cast<const uint4*>(K + static_cast<size_t>(unit) * Lmax * kD);
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int i = start + r;
    for (; i + 48 < end; i += 64) {  // four independent loads in flight
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = ld_stream(&base[static_cast<size_t>(i + 16 * u) * 16 + p]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float f[8];
            widen8<DT>(v[u], f);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += static_cast<double>(f[e]);
        }
    }
    for (; i < end; i += 16) {
        float f[8];
        widen8<DT>(base[static_cast<size_t>(i) * 16 + p], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += static_cast<double>(f[e]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[r][8 * p + e] = acc[e];
    __syncthreads();
    if (tid < kD) {
        double s = 0.0;
#pragma unroll
        for (int rr = 0; rr < 16; ++rr) s += red[rr][tid];
        colsum[(static_cast<size_t>(unit) * kFitMaxWg + wg) * kD + tid] = s;
    }
}

// fit step 2: mu = (sum of partials, fixed order) / L.
__global__ __launch_bounds__(kBlock) void mean_kernel(const double* __restrict__ colsum,
                                                      const int32_t* __restrict__ seq_len,
                                                      float* __restrict__ mu, int Hkv, int Lmax, int nwg) {
    const int unit = blockIdx.x, tid = threadIdx.x;
    int L = seq_len[unit / Hkv];
    L = L < 0 ? 0 : (L > Lmax ? Lmax : L);
    if (tid < kD) {
        double s = 0.0;
#pragma unroll 8
        for (int w = 0; w < nwg; ++w) s += colsum[(static_cast<size_t>(unit) * kFitMaxWg + w) * kD + tid];
        mu[static_cast<size_t>(unit) * kD + tid] = L > 0 ? static_cast<float>(s / static_cast<double>(L)) : 0.0f;
    }
}

// fit step 3 / stand-alone encode: sign bits against mu, packed MSB-first; with CLUSTER also the
// per-(group, code) sums of K - mu and the member counts of this workgroup's token range.
//
// One lane owns one sign group of one token: lane = 32 * half + g reads the 8 bytes holding channels
// 4g .. 4g+3 (a wavefront load covers two complete 256 B rows) and derives the group's 4-bit Code.
// The cluster accumulators are private to the lane - LDS columns tabs[Code][lane] (the four sums as one
// float4: a 16-lane phase of the 128-bit access covers all 64 banks once, whatever the Codes) and
// tabc[Code][lane] (the count), always on the lane's own banks - so they are updated with plain
// read-add-write in token order: no atomics (LDS float atomics ran this kernel at 0.4 TB/s) and a
// sum order that does not depend on scheduling.  Workgroup partials go to part[unit][wg][g][80].
constexpr int kEncThreads = 128;                 // two wavefronts
constexpr int kEncEntries = 16 * 5;              // per group: 16 codes x (4 sums + count)
constexpr int kEncTokPerIter = kEncThreads / 32;  // tokens a workgroup takes per step
constexpr int kEncUnroll = 16;

template <int DT, bool CLUSTER>
__global__ __launch_bounds__(kEncThreads) void encode_kernel(const uint16_t* __restrict__ K,
                                                             const int32_t* __restrict__ seq_len, int t0, int n,
                                                             const float* __restrict__ mu,
                                                             uint8_t* __restrict__ codes,
                                                             float* __restrict__ part, int Hkv, int Lmax,
                                                             int nwg) {
    __shared__ float4 tabs[CLUSTER ? (kEncThreads / kWave) * 16 * kWave : 1];  // [wave][code][lane]: 4 sums
    __shared__ float tabc[CLUSTER ? (kEncThreads / kWave) * 16 * kWave : 1];    // [wave][code][lane]: count
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int g = lane & 31, sub = wv * 2 + (lane >> 5);  // sub: which of the 4 tokens of a step
    const int unit = blockIdx.x / nwg, wg = blockIdx.x % nwg;
    int lo, hi;
    if constexpr (CLUSTER) {
        int L = seq_len[unit / Hkv];
        lo = 0;
        hi = L < 0 ? 0 : (L > Lmax ? Lmax : L);
    } else {
        lo = t0;
        hi = t0 + n;
    }
    const int chunk = ((hi - lo + nwg - 1) / nwg + kEncTokPerIter - 1) / kEncTokPerIter * kEncTokPerIter;
    const int start = lo + wg * chunk;
    const int end = min(hi, start + chunk);
    const uint2* base = reinterpret_cast<const uint2*>(K + static_cast<size_t>(unit) * Lmax * kD);
    uint8_t* cbase = codes + static_cast<size_t>(unit) * Lmax * kCodeBytes;
    const float4 m = reinterpret_cast<const float4*>(mu + static_cast<size_t>(unit) * kD)[g];
    float4* cols = tabs + (CLUSTER ? wv * 16 * kWave + lane : 0);  // this lane's columns, stride 64 per code
    float* colc = tabc + (CLUSTER ? wv * 16 * kWave + lane : 0);
    if constexpr (CLUSTER) {
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            cols[c * kWave] = make_float4(0.f, 0.f, 0.f, 0.f);
            colc[c * kWave] = 0.0f;
        }
    }
    // The rows of the next iteration are requested before the current ones are processed (the accumulator
    // updates are a chain of dependent LDS accesses that would otherwise sit idle behind the HBM latency).
    // Every request is an unconditional load (rows past the end re-read the last row and are ignored), so that
    // the wait before processing counts the outstanding loads instead of draining them all.
    uint2 nx[kEncUnroll];
    const int last = end - 1;
    auto request = [&](int i0) {
#pragma unroll
        for (int u = 0; u < kEncUnroll; ++u) {
            const int i = min(i0 + u * kEncTokPerIter, last);
            nx[u] = ld_stream(&base[static_cast<size_t>(i) * 32 + g]);
        }
    };
    if (start < end) request(start + sub);
    for (int i0 = start + sub; i0 < end; i0 += kEncTokPerIter * kEncUnroll) {
        uint2 v[kEncUnroll];
#pragma unroll
        for (int u = 0; u < kEncUnroll; ++u) v[u] = nx[u];
        request(i0 + kEncTokPerIter * kEncUnroll);
#pragma unroll
        for (int u = 0; u < kEncUnroll; ++u) {
            const int i = i0 + u * kEncTokPerIter;
            if (i < end) {
                const float f[4] = {widen16<DT>(v[u].x & 0xffffu), widen16<DT>(v[u].x >> 16),
                                    widen16<DT>(v[u].y & 0xffffu), widen16<DT>(v[u].y >> 16)};
                const int code = (f[0] >= m.x ? 8 : 0) | (f[1] >= m.y ? 4 : 0) | (f[2] >= m.z ? 2 : 0) |
                                 (f[3] >= m.w ? 1 : 0);
                // the neighbouring lane holds the other nibble of this byte (groups 2j, 2j+1)
                const int other = __builtin_amdgcn_update_dpp(0, code, 0xB1 /* quad_perm:[1,0,3,2] */, 0xf, 0xf, false);
                if ((g & 1) == 0) cbase[static_cast<size_t>(i) * kCodeBytes + (g >> 1)] = static_cast<uint8_t>((code << 4) | other);
                if constexpr (CLUSTER) {
                    float4 a = cols[code * kWave];
                    a.x += f[0] - m.x;
                    a.y += f[1] - m.y;
                    a.z += f[2] - m.z;
                    a.w += f[3] - m.w;
                    cols[code * kWave] = a;
                    colc[code * kWave] += 1.0f;
                }
            }
        }
    }
    if constexpr (CLUSTER) {
        __syncthreads();
        float* pw = part + (static_cast<size_t>(unit) * kFitMaxWg + wg) * kG * kEncEntries;
        for (int e = tid; e < kG * kEncEntries; e += kEncThreads) {
            const int gg = e / kEncEntries, ent = e % kEncEntries, code = ent / 5, comp = ent % 5;
            float sum = 0.0f;
#pragma unroll
            for (int w = 0; w < kEncThreads / kWave; ++w) {
                const int at = (w * 16 + code) * kWave + gg;
                sum += comp < 4 ? reinterpret_cast<const float*>(&tabs[at])[comp] +
                                      reinterpret_cast<const float*>(&tabs[at + 32])[comp]
                                : tabc[at] + tabc[at + 32];
            }
            pw[e] = sum;
        }
    }
}

// fit step 4: centroid = (sum of the workgroup partials, fixed order, fp64) / member count; empty -> 0.
// Grid = units x 2; thread = one (group, code) entry.
__global__ __launch_bounds__(kBlock) void codebook_kernel(const float* __restrict__ part, int nwg,
                                                          int32_t* __restrict__ counts,
                                                          float* __restrict__ codebook) {
    const size_t unit = blockIdx.x >> 1;
    const int e = (blockIdx.x & 1) * kBlock + threadIdx.x;  // e = g * 16 + code
    double s[5] = {0, 0, 0, 0, 0};
    const float* p = part + (unit * kFitMaxWg * kG * 16 + e) * 5;
#pragma unroll 4
    for (int w = 0; w < nwg; ++w) {
#pragma unroll
        for (int c = 0; c < 5; ++c) s[c] += static_cast<double>(p[static_cast<size_t>(w) * kG * 16 * 5 + c]);
    }
    const int32_t cnt = static_cast<int32_t>(s[4] + 0.5);
    counts[unit * kG * 16 + e] = cnt;
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    if (cnt > 0)
        o = make_float4(static_cast<float>(s[0] / s[4]), static_cast<float>(s[1] / s[4]),
                        static_cast<float>(s[2] / s[4]), static_cast<float>(s[3] / s[4]));
    reinterpret_cast<float4*>(codebook)[unit * kG * 16 + e] = o;
}

// ---------------------------------------------------------------------------------------
static int fit_workgroups(const Dims& d) {
    int nwg = 2048 / d.units();
    if (nwg < 1) nwg = 1;
    if (nwg > kFitMaxWg) nwg = kFitMaxWg;
    const int by_len = (d.Lmax + 255) / 256;  // at least 256 rows per workgroup
    return nwg < by_len ? nwg : (by_len < 1 ? 1 : by_len);
}

hipError_t launch_prep(const Dims& d, const Workspace& w, const void* k_new, const void* v_new, void* K,
                       void* V, int32_t* seq_len, const float* mu, uint8_t* codes, hipStream_t s) {
    int nzb = static_cast<int>((w.zero_words / 4 + kBlock * 4 - 1) / (kBlock * 4));
    nzb = nzb < 1 ? 1 : (nzb > 512 ? 512 : nzb);
    const int nb = nzb + (k_new ? d.B : 0);
    auto kn = static_cast<const uint16_t*>(k_new);
    auto vn = static_cast<const uint16_t*>(v_new);
    auto Kp = static_cast<uint16_t*>(K);
    auto Vp = static_cast<uint16_t*>(V);
    return launch_kernel(d.kv_dtype == kBF16 ? prep_kernel<kBF16> : prep_kernel<kF16>, nb, kBlock, s, w.zero_begin,
                         w.zero_words, nzb, kn, vn, Kp, Vp, seq_len, mu, codes, d.Hkv, d.Lmax);
}

hipError_t launch_fit(const Dims& d, const Workspace& w, const void* K, const int32_t* seq_len, float* mu,
                      float* codebook, int32_t* counts, uint8_t* codes, hipStream_t s) {
    const int nwg = fit_workgroups(d);
    const int units = d.units();
    auto Kp = static_cast<const uint16_t*>(K);
    if (d.kv_dtype == kBF16)
        colsum_kernel<kBF16><<<units * nwg, kBlock, 0, s>>>(Kp, seq_len, w.colsum, d.Hkv, d.Lmax, nwg);
    else
        colsum_kernel<kF16><<<units * nwg, kBlock, 0, s>>>(Kp, seq_len, w.colsum, d.Hkv, d.Lmax, nwg);
    mean_kernel<<<units, kBlock, 0, s>>>(w.colsum, seq_len, mu, d.Hkv, d.Lmax, nwg);
    if (d.kv_dtype == kBF16)
        encode_kernel<kBF16, true><<<units * nwg, kEncThreads, 0, s>>>(Kp, seq_len, 0, 0, mu, codes, w.cpart, d.Hkv,
                                                                       d.Lmax, nwg);
    else
        encode_kernel<kF16, true><<<units * nwg, kEncThreads, 0, s>>>(Kp, seq_len, 0, 0, mu, codes, w.cpart, d.Hkv,
                                                                      d.Lmax, nwg);
    codebook_kernel<<<units * 2, kBlock, 0, s>>>(w.cpart, nwg, counts, codebook);
    return hipGetLastError();
}

hipError_t launch_encode(const Dims& d, const void* K, int t0, int n, const float* mu, uint8_t* codes,
                         hipStream_t s) {
    if (n == 0) return hipSuccess;
    int nwg = (n + 255) / 256;
    const int cap = 2048 / d.units() < 1 ? 1 : 2048 / d.units();
    if (nwg > cap) nwg = cap;
    auto Kp = static_cast<const uint16_t*>(K);
    if (d.kv_dtype == kBF16)
        encode_kernel<kBF16, false><<<d.units() * nwg, kEncThreads, 0, s>>>(Kp, nullptr, t0, n, mu, codes, nullptr,
                                                                            d.Hkv, d.Lmax, nwg);
    else
        encode_kernel<kF16, false><<<d.units() * nwg, kEncThreads, 0, s>>>(Kp, nullptr, t0, n, mu, codes, nullptr,
                                                                           d.Hkv, d.Lmax, nwg);
    return hipGetLastError();
}

}  // namespace sik
