// Host side of the one-launch decode step: which kernel variant a layout takes (step_plan), the one-time zeroing of
// the synchronisation words, and the launch (the kernel itself: sik_step_kernel.h).
#include <atomic>

#include "sik_scan.h"
#include "sik_select.h"
#include "sik_step_args.h"

namespace sik {

// ---- host side ---------------------------------------------------------------------------------------------------
// instantiated (tokens per thread with scores in registers, further tokens with scores in LDS); chunk = 1024 x sum
constexpr int kStepT[][2] = {{1, 0}, {2, 0}, {3, 0}, {4, 0}, {6, 0}, {8, 0}, {12, 0}, {12, 4}, {14, 4}, {16, 4}};
// instantiated tokens per thread of the variant with the 16-bit first pass (two registers per token)
constexpr int kStepFx[] = {4, 8, 12, 16, 20};
// the pairs instantiated for the 2-bit cache as well
constexpr int kStepQ2[][2] = {{1, 0}, {4, 0}, {12, 0}, {12, 4}, {14, 4}, {16, 4}};

size_t step_sync_words(const Dims& d) {
    return kSyncHeader + static_cast<size_t>(d.rows()) * kSyncPerRow + static_cast<size_t>(d.B) * kSyncPerSeq;
}

// Upper bound of the chunks per head block any one-launch plan of this layout uses (sizes the histogram area).
int step_max_chunks(const Dims& d) {
    const int hbs = d.units() * ((d.R + kHB - 1) / kHB);
    const int byc = 320 / hbs;  // no part of this family has more compute units
    return byc < 1 ? 1 : (byc > kMaxChunks ? kMaxChunks : byc);
}

static size_t step_dyn_bytes(int chunk, int TL, int k, int* listcap) {
    const int cap = ((chunk < k ? chunk : k) + 7) & ~7;
    *listcap = cap;
    const size_t lists = ((static_cast<size_t>(kHB) * cap * 2 + 15) & ~size_t(15)) +
                         static_cast<size_t>(kHB) * kCandCap * 8 + static_cast<size_t>(TL) * kStepThreads * 16;
    const size_t tail = static_cast<size_t>(kHB) * (kCandCap + 8) * 8 + static_cast<size_t>(kHB) * 2 * kCandCap * 4;
    return lists > tail ? lists : tail;
}

// Tokens per thread of the one-launch step for this layout, or 0 when it does not apply: the smallest T whose
// grid fits the compute units (workgroups of a head block wait for each other, so they must all be resident);
// a single chunk per head block needs no wait and may exceed them.
int step_plan(const Dims& d, int k, bool appended, int cus, bool fx, bool kvq, int* nchunk_out, size_t* dyn_out,
              int* listcap_out) {
    if (d.R < 2 || d.R > 255 || cus < 1) return 0;
    const int hbs = d.units() * ((d.R + kHB - 1) / kHB);
    auto fits = [&](int tokens, int tl) {
        const int chunk = kStepThreads * tokens;
        const int nchunk = (d.Lmax + chunk - 1) / chunk;
        if (nchunk > kMaxChunks || nchunk > step_max_chunks(d)) return false;
        const bool resident = static_cast<int64_t>(hbs) * nchunk <= cus;
        if (!resident && nchunk != 1) return false;
        int listcap;
        const size_t dyn = step_dyn_bytes(chunk, tl, k, &listcap);
        if (dyn > kStepLdsBudget) return false;
        *nchunk_out = nchunk;
        *dyn_out = dyn;
        *listcap_out = listcap;
        return true;
    };
    if (fx) {
        if (kvq) return 0;
        for (const int t : kStepFx)
            if (fits(t, 0)) return kStepFxCode + t * 100;
        return 0;
    }
    if (kvq) {  // (the pairs instantiated for the 2-bit cache and for forced sets)
        for (const auto& tt : kStepQ2)
            if (fits(tt[0] + tt[1], tt[1])) return tt[0] * 100 + tt[1];
        return 0;
    }
    for (const auto& tt : kStepT)
        if (fits(tt[0] + tt[1], tt[1])) return tt[0] * 100 + tt[1];  // both numbers in one: T * 100 + TL
    return 0;
}

int device_compute_units() {
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

__global__ void fill_zero_kernel(uint32_t* p, size_t n) {
    for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n;
         i += static_cast<size_t>(gridDim.x) * blockDim.x)
        p[i] = 0u;
}

hipError_t launch_sync_init(const Dims& d, const Workspace& w, hipStream_t s) {
    const size_t n = step_sync_words(d);
    return launch_kernel(fill_zero_kernel, static_cast<int>((n + 255) / 256 > 64 ? 64 : (n + 255) / 256), 256, s,
                         w.sync, n);
}

hipError_t launch_step(const Dims& d, const Workspace& w, int T, int nchunk, size_t dyn, int listcap, const void* q,
                       const Append& ap, const float* codebook, const uint8_t* codes, int32_t* seq_len,
                       const void* K, const void* V, const void* kvq, const float* alpha, int k, const StepOptions& fo,
                       float scale, int32_t* idx_out, void* out, hipStream_t s) {
    StepArgs a{};
    a.k_per_mille = fo.k_per_mille;
    const int spin_limit = fo.spin_limit;
    a.k_new = ap.k_new, a.v_new = ap.v_new, a.Kw = ap.K, a.Vw = ap.V, a.mu = ap.mu, a.codes_w = ap.codes;
    a.kvq = static_cast<const uint2*>(kvq), a.kvq_w = static_cast<uint2*>(ap.kvq), a.alpha = alpha;
    a.forced_idx = fo.idx, a.n_forced = fo.n, a.fK = fo.fK, a.fV = fo.fV;
    if (fo.mu) a.mu = fo.mu;  // (the same vector the append uses)
    a.parthist = w.parthist, a.pool = w.cand, a.partial = w.partial, a.scores = w.scores, a.sync = w.sync;
    a.idx_out = idx_out, a.idx_ws = w.idx, a.out = out;
    a.sstride = w.sstride, a.k = k, a.spin_limit = spin_limit > 0 ? spin_limit : (1 << 20), a.listcap = listcap;
    a.scale_log2e = (scale > 0.0f ? scale : 1.0f / sqrtf(static_cast<float>(d.D))) * 1.4426950408889634f;
    const bool out_f32 = d.out_dtype == kF32;
    return d.kv_dtype == kBF16 ? launch_step_bf16(d, T, nchunk, dyn, q, codebook, codes, seq_len, K, V, a, out_f32, s)
                               : launch_step_f16(d, T, nchunk, dyn, q, codebook, codes, seq_len, K, V, a, out_f32, s);
}


}  // namespace sik
