// Device-side helpers shared by the gfx950 kernels of the Self-Indexing KV cache path.
// Wavefront = 64 lanes; a key/value row of D = 128 16-bit values is 256 B = 16 lanes x 16 B.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sik {

constexpr int kD = 128;           // head_dim the kernels are specialised for
constexpr int kG = kD / 4;        // sign groups per key ("Codebook Construction": G = D / 4)
constexpr int kCodeBytes = kD / 8;  // 16 B of packed sign bits per key ("Overhead Analysis" (i))
constexpr int kWave = 64;
constexpr int kBlock = 256;       // threads per workgroup in every kernel
constexpr int kBins = 512;        // first-level selection histogram bins per query head
constexpr int kCandCap = 1024;    // candidates of the threshold bin resolved by ranking
constexpr int kMaxSplit = 64;     // upper bound of attention splits per query head
constexpr float kNegBig = -1.0e30f;

enum : int { kF16 = 0, kBF16 = 1, kF32 = 2 };

// ---- 16-bit storage <-> fp32 (both widenings are exact) -------------------------------
template <int DT>
__device__ __forceinline__ float widen16(uint32_t h16) {
    if constexpr (DT == kBF16) {
        return __uint_as_float(h16 << 16);
    } else {
        const _Float16 h = __builtin_bit_cast(_Float16, static_cast<uint16_t>(h16));
        return static_cast<float>(h);
    }
}

// Eight consecutive 16-bit values held in a 128-bit register quad -> fp32.
template <int DT>
__device__ __forceinline__ void widen8(const uint4 v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = widen16<DT>(w[i] & 0xffffu);
        f[2 * i + 1] = widen16<DT>(w[i] >> 16);
    }
}

// fp32 -> 16-bit storage, round to nearest even (finite inputs).
template <int DT>
__device__ __forceinline__ uint32_t narrow16(float f) {
    if constexpr (DT == kBF16) {
        const uint32_t u = __float_as_uint(f);
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    } else {
        const _Float16 h = static_cast<_Float16>(f);
        return __builtin_bit_cast(uint16_t, h);
    }
}

// Order-preserving map fp32 -> uint32 (larger float <=> larger key; -0 and +0 share a key,
// as they compare equal).
__device__ __forceinline__ uint32_t float_to_key(float f) {
    const uint32_t u = f == 0.0f ? 0u : __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
    const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

// Bin coordinate of a score, x = (s - lo) * scale evaluated as one fused multiply-add (-lo * scale is invariant
// wherever this is used in a loop): non-decreasing in s for scale >= 0.  Every kernel that bins or classifies
// scores goes through this one function, so that they agree on every score.
__device__ __forceinline__ float bin_shift(float lo, float scale) { return -lo * scale; }
__device__ __forceinline__ float bin_coord_shifted(float s, float scale, float shift) { return fmaf(s, scale, shift); }
__device__ __forceinline__ float bin_coord(float s, float lo, float scale) {
    return bin_coord_shifted(s, scale, bin_shift(lo, scale));
}
__device__ __forceinline__ int bin_of_coord(float x) {
    // clamp (median of x, 0, kBins - 1; 0 for a NaN), then truncate: equal to floor-then-clamp for every x
    return static_cast<int>(__builtin_amdgcn_fmed3f(x, 0.0f, static_cast<float>(kBins - 1)));
}

// Histogram bin of a score: a non-decreasing function of s for fixed (lo, scale >= 0), so that
// "bin above the threshold bin" implies "score above every score of the threshold bin".
__device__ __forceinline__ int score_bin(float s, float lo, float scale) {
    return bin_of_coord(bin_coord(s, lo, scale));
}

// Streaming (non-temporal) loads for data a kernel reads once: they do not displace what the launches around it
// keep in the caches.
__device__ __forceinline__ uint4 ld_stream(const uint4* p) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 x = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(x.x, x.y, x.z, x.w);
}
__device__ __forceinline__ uint2 ld_stream(const uint2* p) {
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 x = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
    return make_uint2(x.x, x.y);
}

__device__ __forceinline__ void st_stream(uint2* p, uint2 v) {
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    u32x2 x = {v.x, v.y};
    __builtin_nontemporal_store(x, reinterpret_cast<u32x2*>(p));
}

// Agent-scope relaxed atomics on global memory.
__device__ __forceinline__ uint32_t atomic_add_u32(uint32_t* p, uint32_t v) {
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t atomic_max_u32(uint32_t* p, uint32_t v) {
    return __hip_atomic_fetch_max(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- exchange between workgroups of one launch ---------------------------------------------
// MI355X has one L2 per XCD, so data handed from one workgroup to another inside a launch must
// not sit dirty in the writer's L2 or stale in the reader's.  A full agent-scope release fence
// (write back the whole L2) per workgroup costs more than the kernels themselves, so the exchange
// buffers are written and read with relaxed agent-scope atomic accesses instead (write-through
// stores, coherent loads), and ordering comes from waiting for the stores to complete before the
// workgroup takes its ticket.
__device__ __forceinline__ void st_agent(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(float* p, float v) {
    __hip_atomic_store(reinterpret_cast<uint32_t*>(p), __float_as_uint(v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(uint64_t* p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t ld_agent(const uint64_t* p) {
    return __hip_atomic_load(const_cast<uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p) {
    return __hip_atomic_load(const_cast<uint32_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
    return __uint_as_float(__hip_atomic_load(reinterpret_cast<uint32_t*>(const_cast<float*>(p)),
                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

// "Last workgroup to arrive" ticket.  Every workgroup first writes what it hands over with
// st_agent, then calls this from all its threads; the workgroup that draws total-1 may read what
// all the others wrote with ld_agent.  The ticket must start at zero.
__device__ __forceinline__ bool last_arriver(uint32_t* ticket, uint32_t total, int* lds_flag) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);  // every store of this lane has been acknowledged
    __syncthreads();
    if (threadIdx.x == 0) *lds_flag = (atomic_add_u32(ticket, 1u) == total - 1u) ? 1 : 0;
    __syncthreads();
    return *lds_flag != 0;
}

// ---- optional phase timeline (debug builds only, -DSIK_TIMELINE) ------------------------------
// SIK_TL(slot) stores the 100 MHz wall clock when thread 0 of the first, the middle or the last
// workgroup of the grid passes the mark (plain stores, three columns); SIK_TL_ANY(slot) is for code
// only one workgroup per row reaches: the one of row 0 writes (a variable `row` must be in scope).
#ifdef SIK_TIMELINE
#define SIK_TL_DEFINE(setter)                                                                     \
    static __device__ unsigned long long* sik_tl_buf = nullptr;                                   \
    extern "C" int setter(void* p) {                                                              \
        return hipMemcpyToSymbol(HIP_SYMBOL(sik_tl_buf), &p, sizeof(p)) == hipSuccess ? 0 : -1;   \
    }
#define SIK_TL(slot)                                                                              \
    do {                                                                                          \
        if (threadIdx.x == 0 && sik_tl_buf) {                                                     \
            const unsigned b_ = blockIdx.x, g_ = gridDim.x;                                       \
            const int col_ = b_ == 0 ? 0 : (b_ == g_ / 2 ? 1 : (b_ == g_ - 1 ? 2 : -1));          \
            if (col_ >= 0) sik_tl_buf[4 * (slot) + col_] = wall_clock64();                        \
        }                                                                                         \
    } while (0)
#define SIK_TL_ANY(slot)                                                                          \
    do {                                                                                          \
        if (threadIdx.x == 0 && sik_tl_buf && row == 0) sik_tl_buf[4 * (slot) + 3] = wall_clock64(); \
    } while (0)
#else
#define SIK_TL_DEFINE(setter)
#define SIK_TL(slot) \
    do {             \
    } while (0)
#define SIK_TL_ANY(slot) \
    do {                 \
    } while (0)
#endif

// c + a.lo * b.lo + a.hi * b.hi on two packed 16-bit values per register, fp32 accumulate: one
// instruction (v_dot2c_f32_bf16 / v_dot2c_f32_f16) instead of two widenings and two FMAs.
typedef __bf16 sik_bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 sik_f16x2 __attribute__((ext_vector_type(2)));
template <int DT>
__device__ __forceinline__ float dot2_acc(uint32_t a, uint32_t b, float c) {
    if constexpr (DT == kBF16)
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(sik_bf16x2, a), __builtin_bit_cast(sik_bf16x2, b), c,
                                               false);
    else
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(sik_f16x2, a), __builtin_bit_cast(sik_f16x2, b), c, false);
}

// 2^x as the bare hardware instruction (1 ulp; results below the normal range flush to zero, which
// is what a softmax weight that small should be; the library routine adds ~6 instructions of range
// handling per call).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Sum over the 16 lanes of a DPP row (lanes 16r .. 16r+15); every lane gets the total.  Four
// rotate-within-row DPP moves feeding adds: no LDS traffic, unlike ds_bpermute-based shuffles.
template <int N>
__device__ __forceinline__ float row_ror(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + N, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_sum(float v) {
    v += row_ror<8>(v);
    v += row_ror<4>(v);
    v += row_ror<2>(v);
    v += row_ror<1>(v);
    return v;
}

}  // namespace sik
