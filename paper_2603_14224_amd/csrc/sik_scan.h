// Table lookups of the LUT-GEMV scan over the packed sign codes (section "Compressed-Domain Top-k Retrieval":
// score_i = sum_g Table^(g)[Code_g(k_i)]), shared by the scoring kernel and the one-launch decode step.
#pragma once

#include "sik_device.h"

namespace sik {

constexpr int kHB = 4;  // query heads per workgroup = components of one float4 table entry

// (byte BY of w) & mask in one instruction (sub-dword operand select), for any BY; the compiler finds this form
// for the upper byte and the upper half only.
template <int BY>
__device__ __forceinline__ uint32_t byte_and(uint32_t w, uint32_t mask) {
    uint32_t r;
    if constexpr (BY == 0)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_0 src1_sel:DWORD"
            : "=v"(r) : "v"(w), "v"(mask));
    else if constexpr (BY == 1)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD"
            : "=v"(r) : "v"(w), "v"(mask));
    else if constexpr (BY == 2)
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2 src1_sel:DWORD"
            : "=v"(r) : "v"(w), "v"(mask));
    else
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3 src1_sel:DWORD"
            : "=v"(r) : "v"(w), "v"(mask));
    return r;
}

// Table lookups.  HB = 4: float4 entries (four query heads at once), 256 B per group; HB = 1: scalar entries,
// 64 B per group (one query head per KV head: multi-head attention, or the summed query of a group-shared
// selection) - a quarter of the LDS traffic, the 16 entries of a group on 16 different banks.
// A batch = the 8 lookups of one 32-bit word of a token's code (groups 8 dw .. 8 dw + 7).  A table offset costs
// one instruction: byte b of the code word, or of the word shifted by one nibble, under the mask that leaves
// Code x entry size (9 instructions per batch instead of 16).
template <int HB>
struct TableEntry {
    using type = float;
};
template <>
struct TableEntry<4> {
    using type = float4;
};

template <int HB>
__device__ __forceinline__ void lookup_batch(uint32_t word, int dw, const float* lut,
                                             typename TableEntry<HB>::type (&v)[8]) {
    using T = typename TableEntry<HB>::type;
    constexpr int kEnt = 4 * HB;            // bytes per table entry
    constexpr uint32_t kMask = 15u * kEnt;  // Code * kEnt
    constexpr int kUp = HB == 4 ? 0 : 2;    // high nibble (Code * 16) -> Code * kEnt: shift right by kUp
    constexpr int kDown = HB == 4 ? 4 : 2;  // low nibble -> Code * kEnt: shift left by kDown
    // byte `by` of the word: high nibble = Code of group 8 dw + 2 by, low nibble = Code of the next group
    const uint32_t whi = kUp ? word >> kUp : word;
    const uint32_t wlo = word << kDown;
    uint32_t off[8];
    off[0] = byte_and<0>(whi, kMask);
    off[1] = byte_and<0>(wlo, kMask);
    off[2] = byte_and<1>(whi, kMask);
    off[3] = byte_and<1>(wlo, kMask);
    off[4] = byte_and<2>(whi, kMask);
    off[5] = byte_and<2>(wlo, kMask);
    off[6] = byte_and<3>(whi, kMask);
    off[7] = byte_and<3>(wlo, kMask);
    const char* base = reinterpret_cast<const char*>(lut) + dw * 8 * 16 * kEnt;
#pragma unroll
    for (int n = 0; n < 8; ++n) v[n] = *reinterpret_cast<const T*>(base + n * 16 * kEnt + off[n]);
}

// The same batch from a table of 8-byte entries (four 16-bit values, one per query head) kept at the 16-byte stride
// of the float4 table, so that the offsets are the same ones: 16 entries x 8 B of a group lie on 32 different banks.
__device__ __forceinline__ void lookup_batch_x(uint32_t word, int dw, const void* lutx, uint2 (&v)[8]) {
    constexpr uint32_t kMask = 15u * 16u;
    const uint32_t wlo = word << 4;
    uint32_t off[8];
    off[0] = byte_and<0>(word, kMask);
    off[1] = byte_and<0>(wlo, kMask);
    off[2] = byte_and<1>(word, kMask);
    off[3] = byte_and<1>(wlo, kMask);
    off[4] = byte_and<2>(word, kMask);
    off[5] = byte_and<2>(wlo, kMask);
    off[6] = byte_and<3>(word, kMask);
    off[7] = byte_and<3>(wlo, kMask);
    const char* base = static_cast<const char*>(lutx) + dw * 8 * 16 * 16;
#pragma unroll
    for (int n = 0; n < 8; ++n) v[n] = *reinterpret_cast<const uint2*>(base + n * 16 * 16 + off[n]);
}

// The fp32 score of one token and one of the table's four heads, summed in ascending group order exactly as the
// batches above are added (the same bits), for the few tokens that are scored one at a time.
__device__ __forceinline__ float exact_score(const float* lut, const uint4 code, int s) {
    const uint32_t w[4] = {code.x, code.y, code.z, code.w};
    float acc = 0.0f;
#pragma unroll
    for (int dw = 0; dw < 4; ++dw) {
#pragma unroll
        for (int by = 0; by < 4; ++by) {
            const uint32_t b = (w[dw] >> (8 * by)) & 0xffu;
            const int g0 = dw * 8 + by * 2;
            const float t0 = lut[(g0 * 16 + static_cast<int>(b >> 4)) * kHB + s];
            const float t1 = lut[((g0 + 1) * 16 + static_cast<int>(b & 15u)) * kHB + s];
            acc = g0 == 0 ? t0 : acc + t0;
            acc += t1;
        }
    }
    return acc;
}

// Half a batch: the 4 lookups of bytes 2 HALF and 2 HALF + 1 of the code word (groups 8 dw + 4 HALF .. + 3), for
// kernels that cannot spare the registers of a whole batch in flight.
template <int HALF>
__device__ __forceinline__ void lookup_half(uint32_t word, int dw, const float* lut, float4 (&v)[4]) {
    constexpr uint32_t kMask = 15u * 16u;
    const uint32_t wlo = word << 4;
    uint32_t off[4];
    off[0] = byte_and<2 * HALF>(word, kMask);
    off[1] = byte_and<2 * HALF>(wlo, kMask);
    off[2] = byte_and<2 * HALF + 1>(word, kMask);
    off[3] = byte_and<2 * HALF + 1>(wlo, kMask);
    const char* base = reinterpret_cast<const char*>(lut) + (dw * 8 + HALF * 4) * 16 * 16;
#pragma unroll
    for (int n = 0; n < 4; ++n) v[n] = *reinterpret_cast<const float4*>(base + n * 16 * 16 + off[n]);
}
__device__ __forceinline__ void add_half(bool first, const float4 (&v)[4], float* acc) {
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        if (first && n == 0) {
            acc[0] = v[n].x, acc[1] = v[n].y, acc[2] = v[n].z, acc[3] = v[n].w;
        } else {
            acc[0] += v[n].x;
            acc[1] += v[n].y;
            acc[2] += v[n].z;
            acc[3] += v[n].w;
        }
    }
}

// acc (+)= the batch, groups in ascending order; the first batch of a token starts the sums.
template <int HB>
__device__ __forceinline__ void add_batch(bool first, const typename TableEntry<HB>::type (&v)[8], float* acc) {
#pragma unroll
    for (int n = 0; n < 8; ++n) {
        if constexpr (HB == 4) {
            if (first && n == 0) {
                acc[0] = v[n].x, acc[1] = v[n].y, acc[2] = v[n].z, acc[3] = v[n].w;
            } else {
                acc[0] += v[n].x;
                acc[1] += v[n].y;
                acc[2] += v[n].z;
                acc[3] += v[n].w;
            }
        } else {
            acc[0] = (first && n == 0) ? v[n] : acc[0] + v[n];
        }
    }
}

}  // namespace sik
