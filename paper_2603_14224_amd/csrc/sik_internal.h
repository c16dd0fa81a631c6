// Host-side plan (grid shapes, workspace carving) and kernel launchers behind the C ABI.
#pragma once

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/sik.h"

namespace sik {

struct Dims {
    int B, Hkv, Hq, R, D, Lmax;
    int kv_dtype, out_dtype;
    int rows() const { return B * Hq; }
    int units() const { return B * Hkv; }
};

// Carving of the caller's workspace.  All offsets are multiples of 256 bytes.
struct Workspace {
    // zeroed by the prep kernel at the start of every call that selects or attends
    uint32_t* zero_begin;   // start of the zero-initialised region
    size_t zero_words;      // its length in 32-bit words
    uint32_t* sync;         // one-launch decode step: status word and self-clearing counters (sik_workspace_init)
    uint32_t* counters;     // [rows][8]  0 index-output reservation, 1 candidate count (stand-alone selector),
                            //            2 select ticket, 3 attention / fused ticket, 4 ~min key (stand-alone
                            //            top-k) or candidate-pool reservation (fused kernel), 5 max key
                            //            (stand-alone top-k), 7 of a sequence's first head: heads finished
    // plain scratch
    uint32_t* parthist;     // [rows][nchunk][kBins/2]  per-chunk histograms, two 16-bit counts per word
    float* binp;            // [rows][2]          histogram origin, scale
    int32_t* lens;          // [B]  decode step: length of each sequence as the scoring launch counted it (the
                            //      appended token included), read by the selection + attention launch
    uint32_t* cand;         // (key, index) of threshold-bin members: per row [kCandCap][2] words for the
                            // stand-alone selector; for the fused kernel per row [33][4 * nchunk] words of
                            // wavefront regions, then per row an overflow pool of [kCandCap][2] words
    int32_t* idx;           // [rows][k]          selection when the caller passes no idx_out
    float* partial;         // [rows][kMaxSplit][D + 2]  split softmax partials (m, l, o[D])
    float* scores;          // [rows][sstride]    decode step only
    int sstride;            // Lmax rounded up to a multiple of 4 (16-byte aligned score rows)
    // quantiser fit
    double* colsum;         // [units][kFitMaxWg][D]
    float* colmm;           // [units][kFitMaxWg][2][D]  per-workgroup channel minima and maxima of K
    float* cpart;           // [units][kFitMaxWg][G][16][5]  per-workgroup cluster sums and counts
    size_t total_bytes;
};

constexpr int kFitMaxWg = 64;

// ---- kernel launches of the decode step ------------------------------------------------------------------
// The profiled entry points want each kernel's own execution time, as a profiler reports it (begin and end
// timestamps of the dispatch, not the interval between two events recorded around the launch, which contains
// the cost of the events themselves).  They set this pair before a launch; launch_kernel then hands it to the
// runtime with the dispatch and clears it.  Unset (the serving path): a plain launch.
struct LaunchEvents {
    hipEvent_t start = nullptr, stop = nullptr;
};
extern thread_local LaunchEvents g_launch_events;

template <class T>
struct SameType {
    using type = T;
};

// Launches kernel<<<grid, block, lds, s>>>(p...); the arguments convert to the kernel's parameter types here
// (lds = bytes of dynamic LDS, the optional last argument).
template <class... P>
inline hipError_t launch_kernel(void (*kernel)(P...), int grid, int block, hipStream_t s,
                                typename SameType<P>::type... p, size_t lds = 0) {
    if (g_launch_events.start) {
        const LaunchEvents ev = g_launch_events;
        g_launch_events = LaunchEvents{};
        void* args[] = {const_cast<void*>(static_cast<const void*>(&p))...};
        return hipExtLaunchKernel(reinterpret_cast<const void*>(kernel), dim3(grid), dim3(block), args, lds, s,
                                  ev.start, ev.stop, 0);
    }
    kernel<<<grid, block, lds, s>>>(p...);
    return hipGetLastError();
}

// Launches that gather at least 64 MB of 16-bit rows (512 B per query head and selected token) read them with
// non-temporal loads, smaller ones with plain loads (measured both ways on either side, see load_row_slice).
inline bool gather_streams(const Dims& d, int k) {
    return static_cast<int64_t>(d.rows()) * k * 512 >= (64ll << 20);
}

Workspace carve(const Dims& d, int k, void* base);

// launchers (return hipError_t of the launch)
hipError_t launch_prep(const Dims& d, const Workspace& w, const void* k_new, const void* v_new, void* K,
                       void* V, int32_t* seq_len, const float* mu, uint8_t* codes, hipStream_t s);
// Decode-time append folded into the scoring launch (all null: nothing is appended).
struct Append {
    const uint16_t* k_new;
    const uint16_t* v_new;
    uint16_t* K;
    uint16_t* V;
    const float* mu;
    uint8_t* codes;
    const float* alpha;  // with kvq: the row is stored as one record of the 2-bit cache instead of into K and V
    void* kvq;
};

// w == nullptr: scores only; otherwise also the per-chunk selection histograms, and with
// zero_counters the per-head counters are cleared (decode step without a preceding prep launch).
// With ap.k_new the new row of every (b, h) is encoded, stored and scored as token seq_len[b]; the
// length itself is left for launch_fused to increment.
// n_forced > 0 (with w): tokens of forced_idx [B, Hkv, n_forced] get score -infinity and no histogram count.
// q_sum > 1 (group-shared selection): d describes one query head per KV head (Hq = Hkv, R = 1) and the scores
// are those of the sum of the q_sum consecutive real query rows of each KV head; else q_sum = 1.
constexpr int kMaxForced = 128;
hipError_t launch_score(const Dims& d, const Workspace* w, bool zero_counters, const Append& ap, const void* q,
                        const float* codebook, const uint8_t* codes, const int32_t* seq_len, float* scores,
                        const int32_t* forced_idx, int n_forced, int q_sum, hipStream_t s);
hipError_t launch_topk_hist(const Dims& d, const Workspace& w, const float* scores, const int32_t* seq_len,
                            hipStream_t s);
void score_plan(const Dims& d, int* nhb, int* nchunk, int* chunk);
bool score_plan_ok(const Dims& d);
void hist_plan(const Dims& d, int* nchunk, int* chunk);
bool hist_plan_ok(const Dims& d);
void select_plan(const Dims& d, int* nchunk, int* chunk);
// hist_from_score: the chunk histograms come from the scoring kernel (else from launch_topk_hist)
hipError_t launch_select(const Dims& d, const Workspace& w, bool hist_from_score, const float* scores,
                         const int32_t* seq_len, int k, int32_t* idx, hipStream_t s);
// idx_per_unit: idx is [B, Hkv, k], one list shared by the query heads of a KV head; else [B, Hq, k]
hipError_t launch_attn(const Dims& d, const Workspace& w, const void* q, const void* K, const void* V,
                       const int32_t* idx, bool idx_per_unit, int k, float scale, void* out, hipStream_t s);
// select + attention in one launch; reads w.scores / w.parthist / w.binp written by launch_score
// `appended`: launch_score counted one more token than seq_len says; the last workgroup increments it
// kvq != nullptr: gather records of the 2-bit cache (K, V unused) with the per-channel alpha
// StepOptions set: n_forced entries per (b, KV head), always attended and outside the top-k (launch_score gave them
// -infinity); with fK, fV (2-bit cache only) they are attended from those 16-bit rows [B, Hkv, n_forced, D],
// centred by mu, instead of from their records.
struct StepOptions {  // what sik_decode_step_ex adds to the plain decode step
    const int32_t* idx;
    int n;
    const uint16_t* fK;
    const uint16_t* fV;
    const float* mu;
    int k_per_mille;    // > 0: per-sequence budget min(k, ceil(L * k_per_mille / 1000))
    bool group_shared;  // one index set per KV head from the summed scores of its query heads (unfused path)
    int launches;       // 0: the library chooses; 1 / 3: the one-launch step whenever its plan allows (3: with the
                        // 16-bit first pass); 2: never
    int spin_limit;     // polls a bounded wait of the one-launch step may take (0: the default)
};
hipError_t launch_fused(const Dims& d, const Workspace& w, const void* q, const void* K, const void* V,
                        const void* kvq, const float* alpha, const StepOptions& forced, int32_t* seq_len, bool appended,
                        int k, float scale, int32_t* idx_out, void* out, hipStream_t s);
bool fused_plan(const Dims& d, int* nchunk, int* chunk);
// one-launch decode step (sik_step.hip)
size_t step_sync_words(const Dims& d);
int step_max_chunks(const Dims& d);
int step_plan(const Dims& d, int k, bool appended, int cus, bool fx, bool kvq, int* nchunk, size_t* dyn_lds,
              int* listcap);
int device_compute_units();
hipError_t launch_sync_init(const Dims& d, const Workspace& w, hipStream_t s);
hipError_t launch_step(const Dims& d, const Workspace& w, int T, int nchunk, size_t dyn_lds, int listcap, const void* q,
                       const Append& ap, const float* codebook, const uint8_t* codes, int32_t* seq_len,
                       const void* K, const void* V, const void* kvq, const float* alpha, int k, const StepOptions& fo,
                       float scale, int32_t* idx_out, void* out, hipStream_t s);
size_t fused_cand_words(const Dims& d);
hipError_t launch_fit(const Dims& d, const Workspace& w, const void* K, const void* V, const int32_t* seq_len,
                      float* mu, float* codebook, int32_t* counts, uint8_t* codes, float* alpha, void* kvq,
                      hipStream_t s);
hipError_t launch_encode(const Dims& d, const void* K, int t0, int n, const float* mu, uint8_t* codes,
                         hipStream_t s);

// 2-bit token-wise K/V format
hipError_t launch_alpha(const Dims& d, const void* K, const int32_t* seq_len, const float* mu, float* alpha,
                        hipStream_t s);
// seq_len != nullptr: tokens [0, seq_len[b]); else tokens [t0, t0 + n)
hipError_t launch_quantize_kv(const Dims& d, const void* K, const void* V, const int32_t* seq_len, int t0, int n,
                              const float* mu, const float* alpha, void* kvq, hipStream_t s);
hipError_t launch_attn_q2(const Dims& d, const Workspace& w, const void* q, const void* kvq, const float* alpha,
                          const int32_t* idx, bool idx_per_unit, int k, float scale, void* out, hipStream_t s);

}  // namespace sik
