// C ABI of the Self-Indexing KV cache decode path: host-side validation, workspace carving and
// kernel sequencing.  Declarations and argument contracts live in include/sik.h.
#include "sik_device.h"
#include "sik_internal.h"
#include "sik_select.h"

#include <atomic>

namespace sik {

thread_local LaunchEvents g_launch_events;

// Scratch memory of sik_decode_step_static: one copy per GPU, part of the loaded code object.  On the host this
// name is only a handle for hipGetSymbolAddress; the device address it yields (per device) is what kernels get.
static __device__ __align__(256) unsigned char scratch[SIK_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (looked up once per device), or nullptr on an error.
static void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return nullptr;
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // every thread finds the same address
    }
    return p;
}

static size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

static int check_layout(const sik_layout* l, Dims* d) {
    if (!l) return SIK_ERR_NULL;
    if (l->batch < 1 || l->n_kv_heads < 1 || l->n_q_heads < 1 || l->max_len < 1) return SIK_ERR_SHAPE;
    if (l->head_dim != kD) return SIK_ERR_SHAPE;
    if (l->n_q_heads % l->n_kv_heads != 0) return SIK_ERR_SHAPE;
    if (l->n_q_heads > 0xffff) return SIK_ERR_SHAPE;  // kernels take the head counts as 16-bit argument fields
    if (static_cast<int64_t>(l->batch) * l->n_q_heads > (1 << 20)) return SIK_ERR_SHAPE;
    if (l->max_len > kMaxLen) return SIK_ERR_SHAPE;  // kMaxChunks chunks of at most kChunkCap tokens per head
    if (l->kv_dtype != SIK_F16 && l->kv_dtype != SIK_BF16) return SIK_ERR_DTYPE;
    if (l->out_dtype != l->kv_dtype && l->out_dtype != SIK_F32) return SIK_ERR_DTYPE;
    d->B = l->batch;
    d->Hkv = l->n_kv_heads;
    d->Hq = l->n_q_heads;
    d->R = l->n_q_heads / l->n_kv_heads;
    d->D = l->head_dim;
    d->Lmax = l->max_len;
    d->kv_dtype = l->kv_dtype;
    d->out_dtype = l->out_dtype;
    // every kernel that builds or sums chunk histograms relies on these bounds (16-bit counts per bin and chunk,
    // one bitmap bit per token of a chunk, kMaxChunks histograms per head)
    if (!score_plan_ok(*d) || !hist_plan_ok(*d)) return SIK_ERR_SHAPE;
    return SIK_OK;
}

Workspace carve(const Dims& d, int k, void* base) {
    Workspace w{};
    char* p = static_cast<char*>(base);
    size_t off = 0;
    const size_t rows = static_cast<size_t>(d.rows()), units = static_cast<size_t>(d.units());
    auto take = [&](size_t bytes) {
        char* r = p ? p + off : nullptr;
        off += align256(bytes);
        return r;
    };
    w.sync = reinterpret_cast<uint32_t*>(take(step_sync_words(d) * 4));  // first: sik_workspace_init finds it there
    const size_t sync_bytes = off;
    w.counters = reinterpret_cast<uint32_t*>(take(rows * 8 * 4));
    w.zero_begin = w.counters;
    w.zero_words = (off - sync_bytes) / 4;
    int nhb, nc_score, nc_hist, ch;
    score_plan(d, &nhb, &nc_score, &ch);
    hist_plan(d, &nc_hist, &ch);
    size_t nc = static_cast<size_t>(nc_score > nc_hist ? nc_score : nc_hist);
    if (static_cast<size_t>(step_max_chunks(d)) > nc) nc = static_cast<size_t>(step_max_chunks(d));
    w.parthist = reinterpret_cast<uint32_t*>(take(rows * nc * (kBins / 2) * 4));
    w.binp = reinterpret_cast<float*>(take(rows * 2 * 4));
    w.lens = reinterpret_cast<int32_t*>(take(static_cast<size_t>(d.B) * 4));
    size_t cand_words = rows * kCandCap * 2;
    if (fused_cand_words(d) > cand_words) cand_words = fused_cand_words(d);
    w.cand = reinterpret_cast<uint32_t*>(take(cand_words * 4));
    w.idx = reinterpret_cast<int32_t*>(take(rows * static_cast<size_t>(k > 0 ? k : 1) * 4));
    w.partial = reinterpret_cast<float*>(take(rows * kMaxSplit * (kD + 2) * 4));
    w.sstride = (d.Lmax + 3) & ~3;
    w.scores = reinterpret_cast<float*>(take(rows * static_cast<size_t>(w.sstride) * 4));
    w.colsum = reinterpret_cast<double*>(take(units * kFitMaxWg * kD * 8));
    w.colmm = reinterpret_cast<float*>(take(units * kFitMaxWg * 2 * kD * 4));
    w.cpart = reinterpret_cast<float*>(take(units * kFitMaxWg * kG * 80 * 4));
    w.total_bytes = off;
    return w;
}

static int check_ws(const Dims& d, int k, void* ws, size_t bytes, Workspace* w) {
    if (!ws) return SIK_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return SIK_ERR_WORKSPACE;
    *w = carve(d, k, ws);
    if (bytes < w->total_bytes) return SIK_ERR_WORKSPACE;
    return SIK_OK;
}

static int launched(hipError_t e) { return e == hipSuccess ? SIK_OK : SIK_ERR_LAUNCH; }

}  // namespace sik

using namespace sik;

extern "C" {

const char* sik_strerror(int status) {
    switch (status) {
        case SIK_OK: return "ok";
        case SIK_ERR_NULL: return "a required pointer is NULL";
        case SIK_ERR_SHAPE: return "unsupported layout (head_dim must be 128, n_q_heads a multiple of n_kv_heads, sizes positive)";
        case SIK_ERR_DTYPE: return "unsupported dtype (kv_dtype F16/BF16; out_dtype kv_dtype or F32)";
        case SIK_ERR_K_RANGE: return "k outside [1, max_len]";
        case SIK_ERR_CAPACITY: return "token range outside [0, max_len]";
        case SIK_ERR_WORKSPACE: return "workspace NULL, not 256-byte aligned, or smaller than sik_workspace_bytes";
        case SIK_ERR_LAUNCH: return "HIP runtime error while enqueueing";
        case SIK_ERR_FLAGS: return "unknown quantiser mode, or an option that does not apply (launches, spin_limit, side rows)";
        case SIK_ERR_STATIC_LIMIT:
            return "sik_decode_step_static: this layout / k needs more scratch memory than the library's built-in "
                   "buffer (SIK_STATIC_SCRATCH_BYTES); use sik_decode_step with a workspace";
        default: return "unknown status";
    }
}

int sik_version(void) { return 100; }

int sik_plan_info(const sik_layout* layout, int32_t* info) {
    Dims d;
    const int rc = check_layout(layout, &d);
    if (rc) return rc;
    if (!info) return SIK_ERR_NULL;
    int nhb, nchunk, chunk;
    score_plan(d, &nhb, &nchunk, &chunk);
    info[0] = nchunk, info[1] = chunk, info[2] = nhb;
    hist_plan(d, &nchunk, &chunk);
    info[3] = nchunk, info[4] = chunk;
    const bool fused = fused_plan(d, &nchunk, &chunk);
    info[5] = fused ? nchunk : 0, info[6] = chunk;
    // one-launch decode step: tokens per thread (chunk = 1024 x that) on the current device, 0 = not taken
    size_t dyn;
    int listcap, snc;
    const int tt = step_plan(d, 1, false, device_compute_units(), false, false, &snc, &dyn, &listcap);
    info[7] = tt / 100 + tt % 100;
    return SIK_OK;
}

int sik_workspace_init(const sik_layout* layout, int32_t k, void* workspace, size_t workspace_bytes, void* stream) {
    Dims d;
    int rc = check_layout(layout, &d);
    if (rc) return rc;
    if (k < 0 || k > d.Lmax) return SIK_ERR_K_RANGE;
    Workspace w;
    rc = check_ws(d, k, workspace, workspace_bytes, &w);
    if (rc) return rc;
    return launched(launch_sync_init(d, w, static_cast<hipStream_t>(stream)));
}

int sik_workspace_status(const void* workspace, void* stream, uint32_t* status) {
    if (!workspace || !status) return SIK_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(status, workspace, sizeof(uint32_t), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return SIK_ERR_LAUNCH;
    return SIK_OK;
}

size_t sik_workspace_bytes(const sik_layout* layout, int32_t k) {
    Dims d;
    if (check_layout(layout, &d) != SIK_OK || k < 0 || k > d.Lmax) return 0;
    return carve(d, k, nullptr).total_bytes;
}

int sik_quantize_keys(const sik_layout* layout, const void* K, const int32_t* seq_len, int32_t t0, int32_t n,
                      int mode, float* mu, float* codebook, int32_t* counts, uint8_t* codes, void* workspace,
                      size_t workspace_bytes, void* stream) {
    Dims d;
    int rc = check_layout(layout, &d);
    if (rc) return rc;
    if (mode != SIK_Q_FIT && mode != SIK_Q_ENCODE) return SIK_ERR_FLAGS;
    if (!K || !mu || !codes) return SIK_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (mode == SIK_Q_ENCODE) {
        if (t0 < 0 || n < 0 || static_cast<int64_t>(t0) + n > d.Lmax) return SIK_ERR_CAPACITY;
        return launched(launch_encode(d, K, t0, n, mu, codes, s));
    }
    if (!seq_len || !codebook || !counts) return SIK_ERR_NULL;
    Workspace w;
    rc = check_ws(d, 0, workspace, workspace_bytes, &w);
    if (rc) return rc;
    return launched(launch_fit(d, w, K, nullptr, seq_len, mu, codebook, counts, codes, nullptr, nullptr, s));
}

int sik_prefill_compress(const sik_layout* layout, const void* K, const void* V, const int32_t* seq_len, float* mu,
                         float* codebook, int32_t* counts, uint8_t* codes, float* alpha, void* kvq, void* workspace,
                         size_t workspace_bytes, void* stream) {
    Dims d;
    int rc = check_layout(layout, &d);
    if (rc) return rc;
    if (!K || !V || !seq_len || !mu || !codebook || !counts || !codes || !alpha || !kvq) return SIK_ERR_NULL;
    Workspace w;
    rc = check_ws(d, 0, workspace, workspace_bytes, &w);
    if (rc) return rc;
    return launched(launch_fit(d, w, K, V, seq_len, mu, codebook, counts, codes, alpha, kvq,
                               static_cast<hipStream_t>(stream)));
}

int sik_score(const sik_layout* layout, const void* q, const float* codebook, const uint8_t* codes,
              const int32_t* seq_len, float* scores, void* stream) {
    Dims d;
    int rc = check_layout(layout, &d);
    if (rc) return rc;
    if (!q || !codebook || !codes || !seq_len || !scores) return SIK_ERR_NULL;
    return launched(launch_score(d, nullptr, false, Append{}, q, codebook, codes, seq_len, scores, nullptr, 0, 1,
                                 static_cast<hipStream_t>(stream)));
}

int sik_topk(const sik_layout* layout, const float* scores, const int32_t* seq_len, int32_t k, int32_t* idx,
             void* workspace, size_t workspace_bytes, void* stream) {
    Dims d;
    int rc = check_layout(layout, &d);
    if (rc) return rc;
    if (!scores || !seq_len || !idx) return SIK_ERR_NULL;
    if (k < 1 || k > d.Lmax) return SIK_ERR_K_RANGE;
    Workspace w;
    rc = check_ws(d, k, workspace, workspace_bytes, &w);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = launch_prep(d, w, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, s);
    if (e == hipSuccess) e = launch_topk_hist(d, w, scores, seq_len, s);
    if (e == hipSuccess) e = launch_select(d, w, false, scores, seq_len, k, idx, s);
    return launched(e);
}

int sik_sparse_attn(const sik_layout* layout, const void* q, const void* K, const void* V, const int32_t* idx,
                    int32_t k, float softmax_scale, void* out, void* workspace, size_t workspace_bytes,
                    void* stream) {
    Dims d;
    int rc = check_layout(layout, &d);
    if (rc) return rc;
    if (!q || !K || !V || !idx || !out) return SIK_ERR_NULL;
    if (k < 1 || k > d.Lmax) return SIK_ERR_K_RANGE;
    Workspace w;
    rc = check_ws(d, k, workspace, workspace_bytes, &w);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = launch_prep(d, w, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, s);
    if (e == hipSuccess) e = launch_attn(d, w, q, K, V, idx, false, k, softmax_scale, out, s);
    return launched(e);
}

size_t sik_kvq_bytes(const sik_layout* layout) {
    Dims d;
    if (check_layout(layout, &d) != SIK_OK) return 0;
    return static_cast<size_t>(d.units()) * d.Lmax * SIK_KVQ_RECORD_BYTES;
}

int sik_quantize_kv(const sik_layout* layout, const void* K, const void* V, const int32_t* seq_len, int32_t t0,
                    int32_t n, int mode, const float* mu, float* alpha, void* kvq, void* stream) {
    Dims d;
    int rc = check_layout(layout, &d);
    if (rc) return rc;
    if (mode != SIK_Q_FIT && mode != SIK_Q_ENCODE) return SIK_ERR_FLAGS;
    if (!K || !V || !mu || !alpha || !kvq) return SIK_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (mode == SIK_Q_ENCODE) {
        if (t0 < 0 || n < 0 || static_cast<int64_t>(t0) + n > d.Lmax) return SIK_ERR_CAPACITY;
        return launched(launch_quantize_kv(d, K, V, nullptr, t0, n, mu, alpha, kvq, s));
    }
    if (!seq_len) return SIK_ERR_NULL;
    hipError_t e = launch_alpha(d, K, seq_len, mu, alpha, s);
    if (e == hipSuccess) e = launch_quantize_kv(d, K, V, seq_len, 0, 0, mu, alpha, kvq, s);
    return launched(e);
}

int sik_sparse_attn_q2(const sik_layout* layout, const void* q, const void* kvq, const float* alpha,
                       const int32_t* idx, int32_t k, float softmax_scale, void* out, void* workspace,
                       size_t workspace_bytes, void* stream) {
    Dims d;
    int rc = check_layout(layout, &d);
    if (rc) return rc;
    if (!q || !kvq || !alpha || !idx || !out) return SIK_ERR_NULL;
    if (k < 1 || k > d.Lmax) return SIK_ERR_K_RANGE;
    Workspace w;
    rc = check_ws(d, k, workspace, workspace_bytes, &w);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = launch_prep(d, w, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, s);
    if (e == hipSuccess) e = launch_attn_q2(d, w, q, kvq, alpha, idx, false, k, softmax_scale, out, s);
    return launched(e);
}

// Start / stop events of the (at most) SIK_N_KERNELS kernels of one profiled decode step.
struct StepTimers {
    hipEvent_t start[SIK_N_KERNELS], stop[SIK_N_KERNELS];
    bool used[SIK_N_KERNELS];
};

// kvq == nullptr: 16-bit cache (K, V); else the 2-bit cache (kvq, alpha), K and V unused.
static int decode_step_impl(const sik_layout* layout, const void* q, const void* k_new, const void* v_new,
                            void* K, void* V, void* kvq, const float* alpha, int32_t* seq_len, const float* mu,
                            const float* codebook, uint8_t* codes, int32_t k, float softmax_scale, void* out,
                            int32_t* idx_out, void* workspace, size_t workspace_bytes, void* stream,
                            StepTimers* tm, const StepOptions& opt = StepOptions{}) {
    Dims d;
    int rc = check_layout(layout, &d);
    if (rc) return rc;
    if (!q || !seq_len || !codebook || !codes || !out) return SIK_ERR_NULL;
    if (kvq ? !alpha : (!K || !V)) return SIK_ERR_NULL;
    if ((k_new == nullptr) != (v_new == nullptr)) return SIK_ERR_NULL;
    if (k_new && !mu) return SIK_ERR_NULL;
    if (k < 1 || k > d.Lmax) return SIK_ERR_K_RANGE;
    if (opt.k_per_mille < 0 || opt.k_per_mille > 1000) return SIK_ERR_K_RANGE;
    if (opt.n < 0 || opt.n > kMaxForced) return SIK_ERR_SHAPE;
    if (opt.n > 0 && !opt.idx) return SIK_ERR_NULL;
    if (opt.n > 0 && k <= opt.n) return SIK_ERR_K_RANGE;  // the budget k counts the forced tokens too
    if ((opt.fK == nullptr) != (opt.fV == nullptr)) return SIK_ERR_NULL;
    if (opt.fK && (!kvq || opt.n == 0)) return SIK_ERR_FLAGS;  // side rows go with the 2-bit cache only
    if (opt.fK && !mu) return SIK_ERR_NULL;
    Workspace w;
    rc = check_ws(d, k, workspace, workspace_bytes, &w);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int32_t* idx = idx_out ? idx_out : w.idx;
    // profiled call: kernel i of the step (0 prep / append, 1 scoring, 2 selection, 3 attention or selection +
    // attention) is dispatched with its own start / stop event pair
    auto timed = [&](int i) {
        if (tm) g_launch_events = LaunchEvents{tm->start[i], tm->stop[i]};
    };
    auto done = [&](int i, hipError_t e) {
        if (tm) {
            tm->used[i] = e == hipSuccess && g_launch_events.start == nullptr;
            g_launch_events = LaunchEvents{};
        }
        return e;
    };
    int fchunks, fchunk;
    const bool fused = fused_plan(d, &fchunks, &fchunk);
    if ((kvq || opt.n > 0 || opt.k_per_mille > 0) && !fused)
        return SIK_ERR_SHAPE;  // these run on the fused path only: max_len <= 524288
    // Group-shared selection: the scoring launch sees one query head per KV head (the summed query).
    Dims ds = d;
    if (opt.group_shared) {
        ds.Hq = d.Hkv;
        ds.R = 1;
        if (carve(ds, k, nullptr).total_bytes > w.total_bytes || !score_plan_ok(ds)) return SIK_ERR_WORKSPACE;
    }
    const int q_sum = opt.group_shared ? d.R : 1;
    // Large launches select once per KV head with the stand-alone selector and let the attention kernels read that
    // list (measured on 32 x 8 KV heads x 16K: 83 against 86 us; on 4 x 8 x 64K with 8:1 GQA: 57 against 71 us);
    // small ones, and everything that needs the fused kernel's extras, go through the fused kernel, where the R
    // query heads of a group each classify the shared scores (32K context, one sequence: 20 against 26 us).
    const bool plain = opt.n == 0 && opt.k_per_mille == 0 && !(kvq && k_new);
    const bool shared_unfused =
        opt.group_shared && (!fused || (plain && static_cast<int64_t>(d.units()) * d.Lmax > (2 << 20)));
    hipError_t e = hipSuccess;
    // One launch for the whole step whenever the plain step's grid fits the compute units (sik_step.hip): scores
    // stay in registers, chunks of a head exchange only histograms, partials and threshold-bin candidates.
    size_t step_dyn = 0;
    int step_nchunk = 0, step_listcap = 0;
    // (by default only for large launches: with one sequence the histogram exchange between the many chunks of a
    // head and the heavier barriers of 1024-thread workgroups cost more than the launch boundary they save)
    const bool large = static_cast<int64_t>(d.units()) * ((d.R + 3) / 4) * d.Lmax > (2 << 20);
    const bool one_launch = !opt.group_shared && opt.launches != 2 && (large || opt.launches != 0);
    const bool first_pass_16 = opt.launches == 3 && !kvq && opt.n == 0;
    int step_T = 0;
    if (one_launch && first_pass_16)
        step_T = step_plan(d, k, k_new != nullptr, device_compute_units(), true, false, &step_nchunk, &step_dyn,
                           &step_listcap);
    if (one_launch && step_T == 0)
        step_T = step_plan(d, k, k_new != nullptr, device_compute_units(), false, kvq != nullptr || opt.n > 0,
                           &step_nchunk, &step_dyn, &step_listcap);
    if (step_T > 0) {
        const Append ap{static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                        static_cast<uint16_t*>(K), static_cast<uint16_t*>(V), mu, codes, alpha, kvq};
        timed(3);
        e = done(3, launch_step(d, w, step_T, step_nchunk, step_dyn, step_listcap, q, k_new ? ap : Append{}, codebook,
                                codes, seq_len, K, V, kvq, alpha, k, opt, softmax_scale, idx_out, out, s));
    } else if (shared_unfused || !fused) {
        // prep (append + counters; skipped when nothing is appended: the scoring launch then clears the per-head
        // counters itself), scoring (on the summed query when the selection is shared), stand-alone selector (per
        // KV head when shared: idx_out is then [B, Hkv, k]), attention reading that index list.  Contexts beyond
        // 512K tokens take this route too.
        const Dims& dsel = shared_unfused ? ds : d;
        if (k_new) {
            timed(0);
            e = done(0, launch_prep(d, w, k_new, v_new, K, V, seq_len, mu, codes, s));
        }
        if (e == hipSuccess) {
            timed(1);
            e = done(1, launch_score(dsel, &w, k_new == nullptr, Append{}, q, codebook, codes, seq_len, w.scores,
                                     nullptr, 0, shared_unfused ? q_sum : 1, s));
        }
        if (e == hipSuccess) {
            timed(2);
            e = done(2, launch_select(dsel, w, true, w.scores, seq_len, k, idx, s));
        }
        if (e == hipSuccess) {
            timed(3);
            e = done(3, kvq ? launch_attn_q2(d, w, q, kvq, alpha, idx, shared_unfused, k, softmax_scale, out, s)
                            : launch_attn(d, w, q, K, V, idx, shared_unfused, k, softmax_scale, out, s));
        }
    } else {
        // Two launches: scoring (which also stores, encodes and scores an appended row and clears the
        // per-call counters), then selection + attention (which publishes the new length).
        const Append ap{static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                        static_cast<uint16_t*>(K), static_cast<uint16_t*>(V), mu, codes, alpha, kvq};
        timed(1);
        e = done(1, launch_score(ds, &w, true, k_new ? ap : Append{}, q, codebook, codes, seq_len, w.scores, opt.idx,
                                 opt.n, q_sum, s));
        if (e == hipSuccess) {
            timed(3);
            e = done(3, launch_fused(d, w, q, K, V, kvq, alpha,
                                     StepOptions{opt.idx, opt.n, opt.fK, opt.fV, mu, opt.k_per_mille, opt.group_shared, 0, 0},
                                     seq_len, k_new != nullptr, k, softmax_scale, idx_out, out, s));
        }
    }
    return launched(e);
}

// Runs one decode step with every kernel dispatched between its own start / stop events, waits for the stream
// and converts the events to execution times (see sik_decode_step_profiled).
extern "C++" template <class Run>
static int profiled(void* stream, float* kernel_us, Run run) {
    if (!kernel_us) return SIK_ERR_NULL;
    StepTimers tm{};
    int made = 0;
    for (; made < 2 * SIK_N_KERNELS; ++made)
        if (hipEventCreate(made & 1 ? &tm.stop[made / 2] : &tm.start[made / 2]) != hipSuccess) break;
    int rc = made == 2 * SIK_N_KERNELS ? SIK_OK : SIK_ERR_LAUNCH;
    if (rc == SIK_OK) rc = run(&tm);
    if (rc == SIK_OK && hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) rc = SIK_ERR_LAUNCH;
    int first = -1, last = -1;
    for (int i = 0; rc == SIK_OK && i < SIK_N_KERNELS; ++i) {
        float ms = 0.0f;
        if (tm.used[i]) {
            if (hipEventElapsedTime(&ms, tm.start[i], tm.stop[i]) != hipSuccess) rc = SIK_ERR_LAUNCH;
            if (first < 0) first = i;
            last = i;
        }
        kernel_us[i] = ms * 1000.0f;
    }
    if (rc == SIK_OK) {
        float ms = 0.0f;
        if (first >= 0 && hipEventElapsedTime(&ms, tm.start[first], tm.stop[last]) != hipSuccess) rc = SIK_ERR_LAUNCH;
        kernel_us[SIK_N_KERNELS] = ms * 1000.0f;
    }
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(i & 1 ? tm.stop[i / 2] : tm.start[i / 2]);
    return rc;
}

int sik_decode_step(const sik_layout* layout, const void* q, const void* k_new, const void* v_new, void* K,
                    void* V, int32_t* seq_len, const float* mu, const float* codebook, uint8_t* codes, int32_t k,
                    float softmax_scale, void* out, int32_t* idx_out, void* workspace, size_t workspace_bytes,
                    void* stream) {
    return decode_step_impl(layout, q, k_new, v_new, K, V, nullptr, nullptr, seq_len, mu, codebook, codes, k,
                            softmax_scale, out, idx_out, workspace, workspace_bytes, stream, nullptr);
}

int sik_decode_step_static(const sik_layout* layout, const void* q, const void* k_new, const void* v_new, void* K,
                           void* V, int32_t* seq_len, const float* mu, const float* codebook, uint8_t* codes,
                           int32_t k, float softmax_scale, void* out, int32_t* idx_out, void* stream) {
    Dims d;
    const int rc = check_layout(layout, &d);
    if (rc) return rc;
    if (k < 1 || k > d.Lmax) return SIK_ERR_K_RANGE;
    if (carve(d, k, nullptr).total_bytes > SIK_STATIC_SCRATCH_BYTES) return SIK_ERR_STATIC_LIMIT;
    void* ws = static_scratch();
    if (ws == nullptr) return SIK_ERR_LAUNCH;
    // always the two launches: nothing in them waits on another workgroup, so the shared buffer never needs the
    // one-time initialisation (and re-initialisation after a give-up) that the one-launch step asks of a workspace
    StepOptions opt{};
    opt.launches = 2;
    return decode_step_impl(layout, q, k_new, v_new, K, V, nullptr, nullptr, seq_len, mu, codebook, codes, k,
                            softmax_scale, out, idx_out, ws, SIK_STATIC_SCRATCH_BYTES, stream, nullptr, opt);
}

int sik_decode_step_profiled(const sik_layout* layout, const void* q, const void* k_new, const void* v_new,
                             void* K, void* V, int32_t* seq_len, const float* mu, const float* codebook,
                             uint8_t* codes, int32_t k, float softmax_scale, void* out, int32_t* idx_out,
                             void* workspace, size_t workspace_bytes, void* stream, float* kernel_us) {
    return profiled(stream, kernel_us, [&](StepTimers* ev) {
        return decode_step_impl(layout, q, k_new, v_new, K, V, nullptr, nullptr, seq_len, mu, codebook, codes, k,
                                softmax_scale, out, idx_out, workspace, workspace_bytes, stream, ev);
    });
}

int sik_decode_step_q2(const sik_layout* layout, const void* q, const void* k_new, const void* v_new, void* kvq,
                       int32_t* seq_len, const float* mu, const float* alpha, const float* codebook,
                       uint8_t* codes, int32_t k, float softmax_scale, void* out, int32_t* idx_out,
                       void* workspace, size_t workspace_bytes, void* stream, float* kernel_us) {
    if (!kvq) return SIK_ERR_NULL;
    if (!kernel_us)
        return decode_step_impl(layout, q, k_new, v_new, nullptr, nullptr, kvq, alpha, seq_len, mu, codebook, codes,
                                k, softmax_scale, out, idx_out, workspace, workspace_bytes, stream, nullptr);
    return profiled(stream, kernel_us, [&](StepTimers* ev) {
        return decode_step_impl(layout, q, k_new, v_new, nullptr, nullptr, kvq, alpha, seq_len, mu, codebook, codes,
                                k, softmax_scale, out, idx_out, workspace, workspace_bytes, stream, ev);
    });
}

int sik_decode_step_ex(const sik_layout* layout, const sik_decode_args* a) {
    if (!a) return SIK_ERR_NULL;
    const StepOptions opt{a->forced_idx, a->n_forced, static_cast<const uint16_t*>(a->forced_K),
                        static_cast<const uint16_t*>(a->forced_V), a->mu, a->k_per_mille, a->group_shared != 0,
                        a->launches, a->spin_limit};
    if (a->spin_limit < 0 || a->launches < 0 || a->launches > 3) return SIK_ERR_FLAGS;
    auto run = [&](StepTimers* ev) {
        return decode_step_impl(layout, a->q, a->k_new, a->v_new, a->K, a->V, a->kvq, a->alpha, a->seq_len, a->mu,
                                a->codebook, a->codes, a->k, a->softmax_scale, a->out, a->idx_out, a->workspace,
                                a->workspace_bytes, a->stream, ev, opt);
    };
    return a->kernel_us ? profiled(a->stream, a->kernel_us, run) : run(nullptr);
}

}  // extern "C"
