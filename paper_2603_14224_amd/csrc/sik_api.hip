// C ABI of the Self-Indexing KV cache decode path: host-side validation, workspace carving and
// kernel sequencing.  Declarations and argument contracts live in include/sik.h.
#include "sik_device.h"
#include "sik_internal.h"

namespace sik {

static size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

static int check_layout(const sik_layout* l, Dims* d) {
    if (!l) return SIK_ERR_NULL;
    if (l->batch < 1 || l->n_kv_heads < 1 || l->n_q_heads < 1 || l->max_len < 1) return SIK_ERR_SHAPE;
    if (l->head_dim != kD) return SIK_ERR_SHAPE;
    if (l->n_q_heads % l->n_kv_heads != 0) return SIK_ERR_SHAPE;
    if (l->n_q_heads > 0xffff) return SIK_ERR_SHAPE;  // kernels take the head counts as 16-bit argument fields
    if (static_cast<int64_t>(l->batch) * l->n_q_heads > (1 << 20)) return SIK_ERR_SHAPE;
    if (l->max_len > (1 << 22)) return SIK_ERR_SHAPE;  // 64 chunks of at most 65535 tokens per head
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
    w.counters = reinterpret_cast<uint32_t*>(take(rows * 8 * 4));
    w.zero_begin = w.counters;
    w.zero_words = off / 4;
    int nhb, nc_score, nc_hist, ch;
    score_plan(d, &nhb, &nc_score, &ch);
    hist_plan(d, &nc_hist, &ch);
    const size_t nc = static_cast<size_t>(nc_score > nc_hist ? nc_score : nc_hist);
    w.parthist = reinterpret_cast<uint32_t*>(take(rows * nc * (kBins / 2) * 4));
    w.binp = reinterpret_cast<float*>(take(rows * 2 * 4));
    size_t cand_words = rows * kCandCap * 2;
    if (fused_cand_words(d) > cand_words) cand_words = fused_cand_words(d);
    w.cand = reinterpret_cast<uint32_t*>(take(cand_words * 4));
    w.idx = reinterpret_cast<int32_t*>(take(rows * static_cast<size_t>(k > 0 ? k : 1) * 4));
    w.partial = reinterpret_cast<float*>(take(rows * kMaxSplit * (kD + 2) * 4));
    w.sstride = (d.Lmax + 3) & ~3;
    w.scores = reinterpret_cast<float*>(take(rows * static_cast<size_t>(w.sstride) * 4));
    w.colsum = reinterpret_cast<double*>(take(units * kFitMaxWg * kD * 8));
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
        case SIK_ERR_FLAGS: return "unknown quantiser mode";
        default: return "unknown status";
    }
}

int sik_version(void) { return 100; }

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
    return launched(launch_fit(d, w, K, seq_len, mu, codebook, counts, codes, s));
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

// kvq == nullptr: 16-bit cache (K, V); else the 2-bit cache (kvq, alpha), K and V unused.
static int decode_step_impl(const sik_layout* layout, const void* q, const void* k_new, const void* v_new,
                            void* K, void* V, void* kvq, const float* alpha, int32_t* seq_len, const float* mu,
                            const float* codebook, uint8_t* codes, int32_t k, float softmax_scale, void* out,
                            int32_t* idx_out, void* workspace, size_t workspace_bytes, void* stream,
                            hipEvent_t* ev, const StepOptions& opt = StepOptions{}) {
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
    auto mark = [&](int i) { return ev ? hipEventRecord(ev[i], s) : hipSuccess; };
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
    hipError_t e = mark(0);
    if (shared_unfused) {
        // prep, score (summed query), stand-alone selector per KV head, attention reading one index list per KV
        // head.  idx_out, if given, is [B, Hkv, k].
        // (nothing to append: no prep launch, the scoring launch clears the per-head counters itself)
        if (e == hipSuccess && k_new) e = launch_prep(d, w, k_new, v_new, K, V, seq_len, mu, codes, s);
        if (e == hipSuccess) e = mark(1);
        if (e == hipSuccess)
            e = launch_score(ds, &w, k_new == nullptr, Append{}, q, codebook, codes, seq_len, w.scores, nullptr, 0,
                             q_sum, s);
        if (e == hipSuccess) e = mark(2);
        if (e == hipSuccess) e = launch_select(ds, w, true, w.scores, seq_len, k, idx, s);
        if (e == hipSuccess) e = mark(3);
        if (e == hipSuccess)
            e = kvq ? launch_attn_q2(d, w, q, kvq, alpha, idx, true, k, softmax_scale, out, s)
                    : launch_attn(d, w, q, K, V, idx, true, k, softmax_scale, out, s);
    } else if (fused) {
        // Two launches: scoring (which also stores, encodes and scores an appended row and clears the
        // per-call counters), then selection + attention (which publishes the new length).  The first
        // and third event intervals are empty.
        const Append ap{static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                        static_cast<uint16_t*>(K), static_cast<uint16_t*>(V), mu, codes, alpha, kvq};
        if (e == hipSuccess) e = mark(1);
        if (e == hipSuccess)
            e = launch_score(ds, &w, true, k_new ? ap : Append{}, q, codebook, codes, seq_len, w.scores, opt.idx,
                             opt.n, q_sum, s);
        if (e == hipSuccess) e = mark(2);
        if (e == hipSuccess) e = mark(3);
        if (e == hipSuccess)
            e = launch_fused(d, w, q, K, V, kvq, alpha,
                             StepOptions{opt.idx, opt.n, opt.fK, opt.fV, mu, opt.k_per_mille, opt.group_shared},
                             seq_len,
                             k_new != nullptr, k, softmax_scale, idx_out, out, s);
    } else {
        // contexts beyond 512K tokens: prep (append + clear counters), score, select, attention
        if (e == hipSuccess && k_new) e = launch_prep(d, w, k_new, v_new, K, V, seq_len, mu, codes, s);
        if (e == hipSuccess) e = mark(1);
        if (e == hipSuccess)
            e = launch_score(d, &w, k_new == nullptr, Append{}, q, codebook, codes, seq_len, w.scores, nullptr, 0, 1,
                             s);
        if (e == hipSuccess) e = mark(2);
        if (e == hipSuccess) e = launch_select(d, w, true, w.scores, seq_len, k, idx, s);
        if (e == hipSuccess) e = mark(3);
        if (e == hipSuccess) e = launch_attn(d, w, q, K, V, idx, false, k, softmax_scale, out, s);
    }
    if (e == hipSuccess) e = mark(4);
    if (e == hipSuccess && ev) e = hipEventRecord(ev[5], s);  // empty interval: cost of an event pair
    return launched(e);
}

// Runs decode_step_impl between HIP events and converts them to intervals (see sik_decode_step_profiled).
extern "C++" template <class Run>
static int profiled(void* stream, float* kernel_us, Run run) {
    if (!kernel_us) return SIK_ERR_NULL;
    constexpr int kEvents = SIK_N_KERNELS + 2;
    hipEvent_t ev[kEvents];
    int made = 0;
    for (; made < kEvents; ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) break;
    int rc = made == kEvents ? SIK_OK : SIK_ERR_LAUNCH;
    if (rc == SIK_OK) rc = run(ev);
    if (rc == SIK_OK && hipEventSynchronize(ev[SIK_N_KERNELS + 1]) != hipSuccess) rc = SIK_ERR_LAUNCH;
    for (int i = 0; rc == SIK_OK && i <= SIK_N_KERNELS; ++i) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, ev[i], ev[i + 1]) != hipSuccess) rc = SIK_ERR_LAUNCH;
        kernel_us[i] = ms * 1000.0f;
    }
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    (void)stream;
    return rc;
}

int sik_decode_step(const sik_layout* layout, const void* q, const void* k_new, const void* v_new, void* K,
                    void* V, int32_t* seq_len, const float* mu, const float* codebook, uint8_t* codes, int32_t k,
                    float softmax_scale, void* out, int32_t* idx_out, void* workspace, size_t workspace_bytes,
                    void* stream) {
    return decode_step_impl(layout, q, k_new, v_new, K, V, nullptr, nullptr, seq_len, mu, codebook, codes, k,
                            softmax_scale, out, idx_out, workspace, workspace_bytes, stream, nullptr);
}

int sik_decode_step_profiled(const sik_layout* layout, const void* q, const void* k_new, const void* v_new,
                             void* K, void* V, int32_t* seq_len, const float* mu, const float* codebook,
                             uint8_t* codes, int32_t k, float softmax_scale, void* out, int32_t* idx_out,
                             void* workspace, size_t workspace_bytes, void* stream, float* kernel_us) {
    return profiled(stream, kernel_us, [&](hipEvent_t* ev) {
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
    return profiled(stream, kernel_us, [&](hipEvent_t* ev) {
        return decode_step_impl(layout, q, k_new, v_new, nullptr, nullptr, kvq, alpha, seq_len, mu, codebook, codes,
                                k, softmax_scale, out, idx_out, workspace, workspace_bytes, stream, ev);
    });
}

int sik_decode_step_ex(const sik_layout* layout, const sik_decode_args* a) {
    if (!a) return SIK_ERR_NULL;
    const StepOptions opt{a->forced_idx, a->n_forced, static_cast<const uint16_t*>(a->forced_K),
                        static_cast<const uint16_t*>(a->forced_V), a->mu, a->k_per_mille, a->group_shared != 0};
    auto run = [&](hipEvent_t* ev) {
        return decode_step_impl(layout, a->q, a->k_new, a->v_new, a->K, a->V, a->kvq, a->alpha, a->seq_len, a->mu,
                                a->codebook, a->codes, a->k, a->softmax_scale, a->out, a->idx_out, a->workspace,
                                a->workspace_bytes, a->stream, ev, opt);
    };
    return a->kernel_us ? profiled(a->stream, a->kernel_us, run) : run(nullptr);
}

}  // extern "C"
