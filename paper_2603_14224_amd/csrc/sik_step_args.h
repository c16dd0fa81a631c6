// Argument block and constants of the one-launch decode step, shared by its host side (sik_step.hip) and the two
// translation units that instantiate its kernel (sik_step_bf16.hip, sik_step_f16.hip: one per storage type, so that
// they compile side by side).
#pragma once

#include "sik_internal.h"

namespace sik {

constexpr int kStepThreads = 1024;
constexpr int kStepWaves = kStepThreads / kWave;
constexpr int kGroupThreads = 256;  // one group of four wavefronts per query head of the block

struct StepArgs {
    // appended row (all null: nothing is appended)
    const uint16_t* k_new;
    const uint16_t* v_new;
    uint16_t* Kw;
    uint16_t* Vw;
    const float* mu;
    uint8_t* codes_w;
    // 2-bit cache (KVQ): records read by the gather, written by the append; the frozen alpha
    const uint2* kvq;
    uint2* kvq_w;
    const float* alpha;
    // forced-inclusion set of every KV head ("Full Precision Sink Tokens"): forced_idx [B, Hkv, n_forced], entries
    // outside [0, L) name no token; with the 2-bit cache optionally 16-bit side rows fK, fV [B, Hkv, n_forced, D]
    const int32_t* forced_idx;
    const uint16_t* fK;
    const uint16_t* fV;
    int n_forced;
    // exchange areas
    uint32_t* parthist;  // [rows][nchunk][kHistWords]  chunk histograms, two 16-bit counts per word
    uint32_t* pool;      // [rows][kCandCap][2]  threshold-bin candidates of a head: (key, index)
    float* partial;      // [rows][kMaxChunks][kPartStride]
    float* scores;       // [rows][sstride]  only written when a threshold bin is too crowded to rank
    uint32_t* sync;      // status word, per-row and per-sequence counters (kSyncHeader / PerRow / PerSeq)
    int32_t* idx_out;
    int32_t* idx_ws;     // [rows][k]  index rows when the caller passes no idx_out (radix winners only)
    void* out;
    int sstride, k, spin_limit, listcap;
    int k_per_mille;     // > 0: the budget of a sequence is min(k, max(1, ceil(L * k_per_mille / 1000)))
    float scale_log2e;
};

constexpr int kSyncHeader = 8;  // word 0: status bits
constexpr int kSyncPerRow = 4;  // ticket, index-output reservation, candidate reservation, histogram arrivals
constexpr int kSyncPerSeq = 2;  // workgroups of the sequence that have left the kernel; one spare word

constexpr int kStepFxCode = 100000;   // added to T * 100 in the plan's return value: the 16-bit first pass
constexpr size_t kStepLdsBudget = 120 * 1024;  // dynamic LDS the kernel may ask for beside its static LDS

// The launch of the kernel variant that plan code T names (step_plan), for bf16 / fp16 K, V and q; out_f32: fp32
// output rows instead of the storage type.
hipError_t launch_step_bf16(const Dims& d, int T, int nchunk, size_t dyn, const void* q, const float* codebook,
                            const uint8_t* codes, int32_t* seq_len, const void* K, const void* V, const StepArgs& a,
                            bool out_f32, hipStream_t s);
hipError_t launch_step_f16(const Dims& d, int T, int nchunk, size_t dyn, const void* q, const float* codebook,
                           const uint8_t* codes, int32_t* seq_len, const void* K, const void* V, const StepArgs& a,
                           bool out_f32, hipStream_t s);

}  // namespace sik
