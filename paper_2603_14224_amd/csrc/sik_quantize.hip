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
#include "sik_kvq.h"

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
// MINMAX: also the smallest and the largest key of each channel, colmm[unit][wg][0 | 1][d]: x -> |x - mu| peaks at
// an end of the range and the binary32 subtraction is monotone, so these two fix alpha = max_i |K_i - mu| bit
// for bit and the pass that used to compute alpha from K is not needed (the compares ride on a pass that waits
// for HBM anyway).
template <int DT, bool MINMAX>
__global__ __launch_bounds__(kBlock) void colsum_kernel(const uint16_t* __restrict__ K,
                                                        const int32_t* __restrict__ seq_len,
                                                        double* __restrict__ colsum, float* __restrict__ colmm,
                                                        int Hkv, int Lmax, int nwg) {
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
    float mn[8], mx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) mn[e] = INFINITY, mx[e] = -INFINITY;
    auto take = [&](const uint4 v) {
        float f[8];
        widen8<DT>(v, f);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            acc[e] += static_cast<double>(f[e]);
            if constexpr (MINMAX) {
                mn[e] = fminf(mn[e], f[e]);
                mx[e] = fmaxf(mx[e], f[e]);
            }
        }
    };
    int i = start + r;
    for (; i + 48 < end; i += 64) {  // four independent loads in flight
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = ld_stream(&base[static_cast<size_t>(i + 16 * u) * 16 + p]);
#pragma unroll
        for (int u = 0; u < 4; ++u) take(v[u]);
    }
    for (; i < end; i += 16) take(base[static_cast<size_t>(i) * 16 + p]);
#pragma unroll
    for (int e = 0; e < 8; ++e) red[r][8 * p + e] = acc[e];
    __syncthreads();
    if (tid < kD) {
        double s = 0.0;
#pragma unroll
        for (int rr = 0; rr < 16; ++rr) s += red[rr][tid];
        colsum[(static_cast<size_t>(unit) * kFitMaxWg + wg) * kD + tid] = s;
    }
    if constexpr (MINMAX) {
        __syncthreads();
        float* fr = reinterpret_cast<float*>(&red[0][0]);  // [2][16][kD] floats fit the fp64 staging area
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            fr[r * kD + 8 * p + e] = mn[e];
            fr[(16 + r) * kD + 8 * p + e] = mx[e];
        }
        __syncthreads();
        if (tid < kD) {
            float lo = INFINITY, hi = -INFINITY;  // a workgroup without tokens leaves the neutral elements
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) {
                lo = fminf(lo, fr[rr * kD + tid]);
                hi = fmaxf(hi, fr[(16 + rr) * kD + tid]);
            }
            float* out = colmm + (static_cast<size_t>(unit) * kFitMaxWg + wg) * 2 * kD;
            out[tid] = lo;
            out[kD + tid] = hi;
        }
    }
}

// fit step 2: mu = (sum of partials, fixed order) / L; with colmm also alpha_d = max(|max_i K_id - mu_d|,
// |min_i K_id - mu_d|) in binary32 (= max_i |K_id - mu_d|, see colsum_kernel), 0 for an empty sequence.
__global__ __launch_bounds__(kBlock) void mean_kernel(const double* __restrict__ colsum,
                                                      const float* __restrict__ colmm,
                                                      const int32_t* __restrict__ seq_len,
                                                      float* __restrict__ mu, float* __restrict__ alpha, int Hkv,
                                                      int Lmax, int nwg) {
    const int unit = blockIdx.x, tid = threadIdx.x;
    int L = seq_len[unit / Hkv];
    L = L < 0 ? 0 : (L > Lmax ? Lmax : L);
    if (tid < kD) {
        double s = 0.0;
#pragma unroll 8
        for (int w = 0; w < nwg; ++w) s += colsum[(static_cast<size_t>(unit) * kFitMaxWg + w) * kD + tid];
        const float m = L > 0 ? static_cast<float>(s / static_cast<double>(L)) : 0.0f;
        mu[static_cast<size_t>(unit) * kD + tid] = m;
        if (colmm != nullptr) {
            float lo = INFINITY, hi = -INFINITY;
            for (int w = 0; w < nwg; ++w) {
                const float* pm = colmm + (static_cast<size_t>(unit) * kFitMaxWg + w) * 2 * kD;
                lo = fminf(lo, pm[tid]);
                hi = fmaxf(hi, pm[kD + tid]);
            }
            alpha[static_cast<size_t>(unit) * kD + tid] = L > 0 ? fmaxf(fabsf(hi - m), fabsf(lo - m)) : 0.0f;
        }
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
constexpr int kEncTokPerIter = kEncThreads / 32;  // tokens the two encoding wavefronts take per step
constexpr int kEncUnroll = 16;

// The encoder's per-lane state and token step, shared by encode_kernel and compress_kernel.
template <int DT, bool CLUSTER>
struct SignEncoder {
    float4 m;        // channel means of this lane's sign group
    float4* cols;    // this lane's accumulator columns (stride kWave per code)
    float* colc;
    uint8_t* cbase;  // code plane of the (sequence, KV head)
    int g;

    __device__ __forceinline__ void clear() {
        if constexpr (CLUSTER) {
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                cols[c * kWave] = make_float4(0.f, 0.f, 0.f, 0.f);
                colc[c * kWave] = 0.0f;
            }
        }
    }
    // token i: code nibble of group g, the byte stored by the even lane of a pair, cluster sums updated
    __device__ __forceinline__ void token(int i, const uint2 v) {
        const float f[4] = {widen16<DT>(v.x & 0xffffu), widen16<DT>(v.x >> 16), widen16<DT>(v.y & 0xffffu),
                            widen16<DT>(v.y >> 16)};
        const int code = (f[0] >= m.x ? 8 : 0) | (f[1] >= m.y ? 4 : 0) | (f[2] >= m.z ? 2 : 0) | (f[3] >= m.w ? 1 : 0);
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
};

// Workgroup partial of the cluster sums: part[g][code][4 sums, count] from the accumulator columns of the
// encoding wavefronts (waves 0 and 1 of the workgroup); called by `nthreads` threads after a barrier.
__device__ __forceinline__ void publish_cluster_partial(const float4* tabs, const float* tabc, float* pw, int tid,
                                                        int nthreads) {
    for (int e = tid; e < kG * kEncEntries; e += nthreads) {
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
    SignEncoder<DT, CLUSTER> enc;
    enc.m = reinterpret_cast<const float4*>(mu + static_cast<size_t>(unit) * kD)[g];
    enc.cols = tabs + (CLUSTER ? wv * 16 * kWave + lane : 0);
    enc.colc = tabc + (CLUSTER ? wv * 16 * kWave + lane : 0);
    enc.cbase = codes + static_cast<size_t>(unit) * Lmax * kCodeBytes;
    enc.g = g;
    enc.clear();
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
            if (i < end) enc.token(i, v[u]);
        }
    }
    if constexpr (CLUSTER) {
        __syncthreads();
        publish_cluster_partial(tabs, tabc, part + (static_cast<size_t>(unit) * kFitMaxWg + wg) * kG * kEncEntries, tid,
                                kEncThreads);
    }
}

// Prefill-side compression with the 2-bit cache, second pass: sign codes, cluster sums AND records from one
// sweep over K and V (sections "One-Pass Sign-Based Clustering" and "Token-Wise Quantization Format").  The two
// jobs want different things from the machine - the cluster sums are chains of dependent LDS updates that need
// few instructions, the records are some 80 vector instructions per row and no LDS - so one workgroup runs both
// side by side: wavefronts 0 and 1 encode (one lane = one sign group of a token, as in encode_kernel), wavefronts
// 2 to 5 build records (16 lanes = one row, as in quantize_kv_kernel).  Both sides walk the workgroup's token range
// in blocks of kCmpBlock tokens and meet at a barrier after every block, so that the second reader of a key row
// finds it in the L2 cache: HBM sees K once here and V once.  (Measured on 4 x 8 x 64K keys: without the barrier
// 10 % slower; 64-token blocks need more registers than three workgroups per compute unit leave; the launch bound
// of five wavefronts per SIMD, 102 registers, beats six, which spills.)
constexpr int kCmpThreads = kEncThreads + 4 * kWave;
constexpr int kCmpBlock = 32;       // tokens per block: 8 steps of the encoders, 2 steps of the record builders
constexpr int kCmpEncSteps = kCmpBlock / kEncTokPerIter;
constexpr int kCmpRecSteps = kCmpBlock / 16;

template <int DT>
__global__ __launch_bounds__(kCmpThreads, 5) void compress_kernel(
    const uint16_t* __restrict__ K, const uint16_t* __restrict__ V, const int32_t* __restrict__ seq_len,
    const float* __restrict__ mu, const float* __restrict__ alpha, uint8_t* __restrict__ codes,
    float* __restrict__ part, uint2* __restrict__ rec, int Hkv, int Lmax, int nwg) {
    __shared__ float4 tabs[(kEncThreads / kWave) * 16 * kWave];
    __shared__ float tabc[(kEncThreads / kWave) * 16 * kWave];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int unit = blockIdx.x / nwg, wg = blockIdx.x % nwg;
    int L = seq_len[unit / Hkv];
    L = L < 0 ? 0 : (L > Lmax ? Lmax : L);
    // the token ranges of encode_kernel: every lane then adds the same values in the same order as there, so the
    // cluster sums (and the codebook) have the same bits whichever entry point fitted them
    const int chunk = ((L + nwg - 1) / nwg + kEncTokPerIter - 1) / kEncTokPerIter * kEncTokPerIter;
    const int start = wg * chunk;
    const int end = min(L, start + chunk);
    const int last = end - 1;
    const size_t row0 = static_cast<size_t>(unit) * Lmax;
    if (wv < kEncThreads / kWave) {
        // ---- encoders
        const int g = lane & 31, sub = wv * 2 + (lane >> 5);
        const uint2* base = reinterpret_cast<const uint2*>(K + row0 * kD);
        SignEncoder<DT, true> enc;
        enc.m = reinterpret_cast<const float4*>(mu + static_cast<size_t>(unit) * kD)[g];
        enc.cols = tabs + wv * 16 * kWave + lane;
        enc.colc = tabc + wv * 16 * kWave + lane;
        enc.cbase = codes + row0 * kCodeBytes;
        enc.g = g;
        enc.clear();
        uint2 nx[kCmpEncSteps];
        auto request = [&](int i0) {
#pragma unroll
            for (int u = 0; u < kCmpEncSteps; ++u)
                nx[u] = base[static_cast<size_t>(min(i0 + u * kEncTokPerIter, last)) * 32 + g];
        };
        if (start < end) request(start + sub);
        for (int blk = start; blk < end; blk += kCmpBlock) {  // the same trip count on both sides of the workgroup
            uint2 v[kCmpEncSteps];
#pragma unroll
            for (int u = 0; u < kCmpEncSteps; ++u) v[u] = nx[u];
            request(blk + kCmpBlock + sub);
#pragma unroll
            for (int u = 0; u < kCmpEncSteps; ++u) {
                const int i = blk + sub + u * kEncTokPerIter;
                if (i < end) enc.token(i, v[u]);
            }
            __syncthreads();
        }
    } else {
        // ---- record builders
        const int p = lane & 15, r = (lane >> 4) + 4 * (wv - kEncThreads / kWave);  // row of a 16-row step
        const uint4* Kb = reinterpret_cast<const uint4*>(K + row0 * kD);
        const uint4* Vb = reinterpret_cast<const uint4*>(V + row0 * kD);
        float m[8], a[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            m[e] = mu[static_cast<size_t>(unit) * kD + 8 * p + e];
            a[e] = alpha_reciprocal(alpha[static_cast<size_t>(unit) * kD + 8 * p + e]);
        }
        uint4 nk[kCmpRecSteps], nv[kCmpRecSteps];
        auto request = [&](int i0) {
#pragma unroll
            for (int u = 0; u < kCmpRecSteps; ++u) {
                const size_t i = static_cast<size_t>(min(i0 + 16 * u, last));
                nk[u] = Kb[i * 16 + p];
                nv[u] = ld_stream(&Vb[i * 16 + p]);
            }
        };
        if (start < end) request(start + r);
        for (int blk = start; blk < end; blk += kCmpBlock) {
            uint4 kk[kCmpRecSteps], vv[kCmpRecSteps];
#pragma unroll
            for (int u = 0; u < kCmpRecSteps; ++u) kk[u] = nk[u], vv[u] = nv[u];
            request(blk + kCmpBlock + r);
#pragma unroll
            for (int u = 0; u < kCmpRecSteps; ++u) {
                const int i = blk + r + 16 * u;
                if (i < end)  // uniform over the 16 lanes of a row
                    st_stream(&rec[(row0 + i) * kRecSlots + p], kvq_make_slot<DT>(kk[u], vv[u], m, a, p));
            }
            __syncthreads();
        }
    }
    __syncthreads();
    publish_cluster_partial(tabs, tabc, part + (static_cast<size_t>(unit) * kFitMaxWg + wg) * kG * kEncEntries, tid,
                            kCmpThreads);
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

// V == nullptr: means, codes, codebook.  Otherwise (prefill-compress with the 2-bit cache) also alpha and the
// records of the fitted tokens, K read twice and V once.
hipError_t launch_fit(const Dims& d, const Workspace& w, const void* K, const void* V, const int32_t* seq_len,
                      float* mu, float* codebook, int32_t* counts, uint8_t* codes, float* alpha, void* kvq,
                      hipStream_t s) {
    const int nwg = fit_workgroups(d);
    const int units = d.units();
    auto Kp = static_cast<const uint16_t*>(K);
    auto Vp = static_cast<const uint16_t*>(V);
    auto rp = static_cast<uint2*>(kvq);
    const bool bf = d.kv_dtype == kBF16;
    hipError_t e;
    if (V)
        e = launch_kernel(bf ? colsum_kernel<kBF16, true> : colsum_kernel<kF16, true>, units * nwg, kBlock, s, Kp,
                          seq_len, w.colsum, w.colmm, d.Hkv, d.Lmax, nwg);
    else
        e = launch_kernel(bf ? colsum_kernel<kBF16, false> : colsum_kernel<kF16, false>, units * nwg, kBlock, s, Kp,
                          seq_len, w.colsum, nullptr, d.Hkv, d.Lmax, nwg);
    if (e != hipSuccess) return e;
    e = launch_kernel(mean_kernel, units, kBlock, s, w.colsum, V ? w.colmm : nullptr, seq_len, mu, alpha, d.Hkv,
                      d.Lmax, nwg);
    if (e != hipSuccess) return e;
    if (V)
        e = launch_kernel(bf ? compress_kernel<kBF16> : compress_kernel<kF16>, units * nwg, kCmpThreads, s, Kp, Vp,
                          seq_len, mu, alpha, codes, w.cpart, rp, d.Hkv, d.Lmax, nwg);
    else
        e = launch_kernel(bf ? encode_kernel<kBF16, true> : encode_kernel<kF16, true>, units * nwg, kEncThreads, s,
                          Kp, seq_len, 0, 0, mu, codes, w.cpart, d.Hkv, d.Lmax, nwg);
    if (e != hipSuccess) return e;
    return launch_kernel(codebook_kernel, units * 2, kBlock, s, w.cpart, nwg, counts, codebook);
}

hipError_t launch_encode(const Dims& d, const void* K, int t0, int n, const float* mu, uint8_t* codes,
                         hipStream_t s) {
    if (n == 0) return hipSuccess;
    int nwg = (n + 255) / 256;
    const int cap = 2048 / d.units() < 1 ? 1 : 2048 / d.units();
    if (nwg > cap) nwg = cap;
    auto Kp = static_cast<const uint16_t*>(K);
    return launch_kernel(d.kv_dtype == kBF16 ? encode_kernel<kBF16, false> : encode_kernel<kF16, false>,
                         d.units() * nwg, kEncThreads, s, Kp, nullptr, t0, n, mu, codes, nullptr, d.Hkv, d.Lmax, nwg);
}

}  // namespace sik
