/*
 * sik.h -- C ABI of the Self-Indexing KV cache decode path for AMD MI355X (gfx950).
 *
 * The library implements the decode-time path of "Self-Indexing KVCache: Predicting
 * Sparse Attention from Compressed Keys": sign-based 1-bit vector quantisation of the
 * key cache, scoring of a query against the packed sign codes through per-group
 * 16-entry lookup tables, per-query-head top-k selection, and softmax attention over
 * only the selected tokens.
 *
 * General rules
 *   - Every tensor pointer is a DEVICE pointer unless marked (host).  Buffers are
 *     caller-owned, contiguous, row-major, 16-byte aligned.  The library never
 *     allocates or frees device memory and keeps no state between calls.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream).  No call synchronises with the host.
 *   - Return value: SIK_OK (0) or a negative sik_status.  Arguments are validated on
 *     the host before anything is launched; a failed call launches nothing.
 *   - seq_len[b] (device, int32) is the number of valid tokens of sequence b; tokens
 *     at or beyond it are never read.  Values must lie in [0, max_len].
 *
 * Notation: B batch, Hkv KV heads, Hq query heads, R = Hq / Hkv (query head hq reads
 * KV head hq / R), D head_dim, G = D / 4 sign groups, Lmax = max_len token capacity.
 *
 * Layouts
 *   K, V      [B, Hkv, Lmax, D]      kv_dtype (one row = D 16-bit values)
 *   q         [B, Hq, D]             kv_dtype
 *   k_new, v_new [B, Hkv, D]         kv_dtype
 *   mu        [B, Hkv, D]            float   channel means of K
 *   codebook  [B, Hkv, G, 16, 4]     float   centroid j of group g, 4 components
 *   counts    [B, Hkv, G, 16]        int32   members per centroid
 *   codes     [B, Hkv, Lmax, D / 8]  uint8   packed sign bits, see sik_quantize_keys
 *   scores    [B, Hq, Lmax]          float
 *   idx       [B, Hq, k]             int32   selected token indices, -1 = empty slot
 *   out       [B, Hq, D]             out_dtype
 */
#ifndef SIK_H
#define SIK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SIK_F16 = 0, SIK_BF16 = 1, SIK_F32 = 2 } sik_dtype;

typedef enum {
    SIK_OK = 0,
    SIK_ERR_NULL = -1,      /* a required pointer is NULL                                   */
    SIK_ERR_SHAPE = -2,     /* bad batch / heads / head_dim / max_len combination           */
    SIK_ERR_DTYPE = -3,     /* kv_dtype not F16/BF16, or out_dtype not kv_dtype/F32         */
    SIK_ERR_K_RANGE = -4,   /* k < 1 or k > max_len                                          */
    SIK_ERR_CAPACITY = -5,  /* token range outside [0, max_len]                              */
    SIK_ERR_WORKSPACE = -6, /* workspace NULL, misaligned or smaller than sik_workspace_bytes */
    SIK_ERR_LAUNCH = -7,    /* the HIP runtime reported an error while enqueueing           */
    SIK_ERR_FLAGS = -8,     /* unknown quantiser mode, or an option value out of range      */
    SIK_ERR_STATIC_LIMIT = -9 /* sik_decode_step_static: the layout needs more scratch memory than the
                                 library's built-in buffer holds (SIK_STATIC_SCRATCH_BYTES)       */
} sik_status;

/* Shape of one attention layer's cache.  head_dim must be 128 (the head size of every
 * model the paper evaluates); n_q_heads must be a multiple of n_kv_heads.  Limits (SIK_ERR_SHAPE beyond them):
 * n_q_heads <= 65535, batch * n_q_heads <= 2^20, max_len <= SIK_MAX_LEN (64 token chunks per head of at most
 * 64512 tokens each: the per-chunk selection histograms count in 16 bits). */
#define SIK_MAX_LEN 4128768
typedef struct {
    int32_t batch;
    int32_t n_kv_heads;
    int32_t n_q_heads;
    int32_t head_dim;
    int32_t max_len;
    int32_t kv_dtype;  /* sik_dtype: SIK_F16 or SIK_BF16 -- type of K, V, q, k_new, v_new */
    int32_t out_dtype; /* sik_dtype: kv_dtype or SIK_F32  -- type of out                   */
} sik_layout;

/* Quantiser modes for sik_quantize_keys. */
enum {
    SIK_Q_FIT = 1,   /* prefill-compress: fit mu and codebook on tokens [0, seq_len[b]), encode them */
    SIK_Q_ENCODE = 2 /* encode tokens [t0, t0 + n) against the given mu; codebook untouched          */
};

/* Human-readable text for a status code (host pointer to a static string). */
const char *sik_strerror(int status);

/* Library version, major * 100 + minor. */
int sik_version(void);

/* Launch geometry the library derives for a layout (diagnostic: tests and tuning read it; no device is touched).
 * info (host pointer, SIK_PLAN_INFO_LEN int32): [0] token chunks per head of the scoring launch, [1] tokens per such
 * chunk, [2] blocks of up to 4 query heads per KV head, [3] chunks per row of the stand-alone histogram pass of
 * sik_topk, [4] tokens per such chunk, [5] chunks per query head of the fused selection + attention launch (0: max_len
 * is beyond that path), [6] tokens per such chunk, [7] tokens per thread of the one-launch decode step on the
 * current device (its chunks hold 1024 times that; 0: no one-launch plan fits this layout, the step always runs as
 * separate launches; sik_decode_step takes the one-launch step only for large launches, sik_decode_args.launches
 * chooses).  Every chunk holds at most 64512 tokens and there are at most 64 per head; a layout that cannot be cut
 * that way is SIK_ERR_SHAPE here and in every other call. */
#define SIK_PLAN_INFO_LEN 8
int sik_plan_info(const sik_layout *layout, int32_t *info);

/* Size in bytes of the scratch buffer the calls below need for this layout and k
 * (k may be 0 for sik_quantize_keys / sik_score only).  The same buffer may be
 * reused by every call on one stream; calls sharing it must not overlap in time.
 * Contents are not preserved.  Returns 0 on a bad layout.
 * The decode-step entry points additionally need the buffer's first words (a status word and the counters
 * through which the workgroups of a one-launch step meet) to be ZERO the first time they see the buffer:
 * call sik_workspace_init once after allocating it (or zero-fill it).  Every step leaves them at zero again. */
size_t sik_workspace_bytes(const sik_layout *layout, int32_t k);

/* Enqueues the zero-fill of the status word and step counters at the start of a workspace (a small fill kernel on
 * `stream`; may be captured into a graph).  Needed once per allocation, before the first decode step, and again
 * after a step that gave up (see sik_workspace_status). */
int sik_workspace_init(const sik_layout *layout, int32_t k, void *workspace, size_t workspace_bytes, void *stream);

/* Waits for `stream` and copies the workspace's status word to *status (host pointer).  0: every decode step on this
 * workspace since its initialisation completed.  Non-zero: a workgroup of a one-launch step waited for its peers
 * beyond the spin limit and left (bit 0: the exchange of the chunk histograms, the only wait there is); that step's
 * outputs are invalid, no kernel hangs, and the workspace must be initialised again.  This can only happen when the
 * step's workgroups were not all resident (another process occupying the compute units for seconds). */
int sik_workspace_status(const void *workspace, void *stream, uint32_t *status);

/* One-pass sign-based quantiser of the key cache (sections "One-Pass Sign-Based
 * Clustering" and "Entropy-Aware Normalization").
 *
 *   SIK_Q_FIT    mu[b,h,d] = mean over tokens i < seq_len[b] of K[b,h,i,d]  (normalisation
 *                equation, fp64 accumulation, stored as float); sign bit of (i, d) is 1 iff
 *                K[b,h,i,d] >= mu[b,h,d]; every group of 4 channels gives the 4-bit Code of
 *                the Code equation (first channel = most significant bit); codebook[b,h,g,j,:]
 *                = mean of K - mu over the tokens whose Code in group g is j (centroid
 *                equation; empty cluster -> 0) and counts[b,h,g,j] their number.  t0 and n are
 *                ignored.  mu, codebook, counts and codes[.., 0:seq_len[b], :] are written.
 *   SIK_Q_ENCODE encodes tokens t0 <= i < t0 + n of every (b, h) against the mu passed in
 *                (read only); codebook and counts may be NULL and are not touched.
 *
 * Packing: byte j of a token's 16 bytes holds Code(group 2j) in its high nibble and
 * Code(group 2j+1) in its low nibble, i.e. bit (7 - e) of byte j is the sign bit of
 * channel 8j + e.  Inputs must be finite. */
int sik_quantize_keys(const sik_layout *layout, const void *K, const int32_t *seq_len, int32_t t0,
                      int32_t n, int mode, float *mu, float *codebook, int32_t *counts,
                      uint8_t *codes, void *workspace, size_t workspace_bytes, void *stream);

/* Compressed-domain scores (section "Compressed-Domain Top-k Retrieval", retrieval
 * equation): Table[b,hq,g,j] = sum_e q[b,hq,4g+e] * codebook[b,hq/R,g,j,e] and
 * scores[b,hq,i] = sum_g Table[b,hq,g,Code_g(codes[b,hq/R,i])] for i < seq_len[b]
 * (fp32 table, fp32 sum in increasing g).  Entries i >= seq_len[b] are not written. */
int sik_score(const sik_layout *layout, const void *q, const float *codebook, const uint8_t *codes,
              const int32_t *seq_len, float *scores, void *stream);

/* Per query head, the indices of the k largest scores among i < seq_len[b] (the
 * selection step that follows the retrieval equation).  Exact selection; equal scores are
 * resolved toward the smaller index; the order inside idx[b,hq,:] is unspecified.  If
 * k >= seq_len[b] every valid token is returned and the rest of the row is -1.
 * Scores must not be NaN. */
int sik_topk(const sik_layout *layout, const float *scores, const int32_t *seq_len, int32_t k,
             int32_t *idx, void *workspace, size_t workspace_bytes, void *stream);

/* Sparse attention over the selected tokens (section "Background and Preliminaries",
 * softmax(q K^T / sqrt(d)) V restricted to the set idx[b,hq,:]): entries < 0 are skipped,
 * repeated entries count as repeats, entries must be < max_len.  softmax_scale <= 0 means
 * 1 / sqrt(head_dim).  fp32 accumulation; an empty selection gives a zero row. */
int sik_sparse_attn(const sik_layout *layout, const void *q, const void *K, const void *V,
                    const int32_t *idx, int32_t k, float softmax_scale, void *out,
                    void *workspace, size_t workspace_bytes, void *stream);

/* One decode step of one layer: [append] -> table -> scores -> top-k -> sparse attention.
 * If k_new and v_new are non-NULL (both or neither) the new key/value row of every (b, h)
 * is written to row seq_len[b] of K and V, its sign code is written to codes (encoded
 * against the frozen mu; codebook unchanged), and seq_len[b] is incremented on the device,
 * so that the new token competes in the selection (seq_len[b] < max_len is required).
 * idx_out ([B,Hq,k], may be NULL) receives the selected indices as in sik_topk. */
int sik_decode_step(const sik_layout *layout, const void *q, const void *k_new, const void *v_new,
                    void *K, void *V, int32_t *seq_len, const float *mu, const float *codebook,
                    uint8_t *codes, int32_t k, float softmax_scale, void *out, int32_t *idx_out,
                    void *workspace, size_t workspace_bytes, void *stream);

/* sik_decode_step for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture that must not call hipMalloc, tight serving loops, harnesses that forbid allocation.  Same arguments
 * and results as sik_decode_step without the workspace pair: the scratch memory is a buffer of
 * SIK_STATIC_SCRATCH_BYTES built into the library (one copy per GPU, held until the process ends).  A layout / k
 * whose sik_workspace_bytes exceeds that returns SIK_ERR_STATIC_LIMIT and launches nothing (the benchmark
 * workloads of one sequence, 32K and 128K tokens, fit; large batches do not).  The call allocates nothing and
 * frees nothing.  Every call on one GPU shares that GPU's buffer, whatever the stream or thread: calls that
 * overlap in time on one GPU race; calls on one stream are ordered and safe.  The buffer keeps the previous
 * call's contents; the step clears what it needs cleared itself, and always runs as separate scoring and selection
 * + attention launches (no workgroup waits for another, so the buffer needs no initialisation).  The first call on
 * a GPU looks the buffer's address up (hipGetSymbolAddress) and must therefore be made outside stream capture. */
#define SIK_STATIC_SCRATCH_BYTES (32u << 20)
int sik_decode_step_static(const sik_layout *layout, const void *q, const void *k_new, const void *v_new, void *K,
                           void *V, int32_t *seq_len, const float *mu, const float *codebook, uint8_t *codes,
                           int32_t k, float softmax_scale, void *out, int32_t *idx_out, void *stream);

/* Measurement aid for benchmarks (not for serving loops): runs exactly the kernels of sik_decode_step with the
 * same arguments, each dispatched with its own start / stop event pair (the begin and end timestamps of the
 * dispatch itself, as a profiler reports them, not an interval between events recorded around the launch), then
 * waits for the stream and returns, in microseconds, in kernel_us (host pointer, SIK_N_KERNELS + 1 floats): the
 * execution time of the prep / append, scoring, selection and attention (or fused selection + attention) kernels
 * in launch order, 0 for a kernel this step did not launch, then the span from the start of the first kernel to
 * the end of the last (the step as the GPU saw it, gaps between the kernels included). */
#define SIK_N_KERNELS 4
int sik_decode_step_profiled(const sik_layout *layout, const void *q, const void *k_new,
                             const void *v_new, void *K, void *V, int32_t *seq_len, const float *mu,
                             const float *codebook, uint8_t *codes, int32_t k, float softmax_scale,
                             void *out, int32_t *idx_out, void *workspace, size_t workspace_bytes,
                             void *stream, float *kernel_us);

/* ---- 2-bit token-wise K/V cache (section "Token-Wise Quantization Format") -------------------
 * The compressed form sparse attention can read instead of the 16-bit rows.  Per (b, h, token)
 * one record of SIK_KVQ_RECORD_BYTES = 128 bytes, kvq [B, Hkv, max_len, 128] uint8 (device,
 * caller-owned, 16-byte aligned), made of 16 slots of 8 bytes; slot p covers channels
 * 8p .. 8p+7:
 *   byte 0     sign byte p of the token's 1-bit code (bit 7-e = [K >= mu] of channel 8p+e)
 *   byte 1     0
 *   bytes 2-3  K magnitude codes, little-endian, code of channel 8p+e in bits 2e+1:2e
 *   bytes 4-5  V codes, same packing
 *   bytes 6-7  one fp16 parameter of the 32-channel group p/4: K qs, K zp, V qs, V zp for
 *              p mod 4 = 0, 1, 2, 3
 * i.e. the paper's 896 bits per token (128 sign bits, 2 x 256 code bits, 2 x 4 x 2 sixteen-bit
 * parameters) laid out so that a selected token is one aligned 128-byte line; 16 bytes are spare.
 * Quantisation function with B = 2, per token and per group x of 32 consecutive channels:
 *   zp = fp16(min x), qs = fp16((max x - min x) / 3), Q = clamp(round((x - zp) * (1 / qs)), 0, 3)
 *   with the stored qs and zp, round = nearest, ties to even, qs = 0 -> Q = 0; D = qs Q + zp.
 * V: x = the value.  K: x = |K - mu| * (1 / alpha) with alpha[b,h,d] = max over the fitted tokens
 * of |K - mu| (alpha = 0 -> x = 0); the reconstructed centred key is s * alpha * D, s = +1 where
 * the sign bit is set.  Codes are decided in binary32 in this operation order (each reciprocal is
 * one correctly rounded division).  Values must be finite and within the fp16 range. */
#define SIK_KVQ_RECORD_BYTES 128

/* Bytes of the record plane of a layout: B * Hkv * max_len * 128 (0 if the layout is invalid). */
size_t sik_kvq_bytes(const sik_layout *layout);

/* Writes records from 16-bit K and V ([B,Hkv,max_len,D] kv_dtype).
 *   SIK_Q_FIT    alpha (out, [B,Hkv,D] fp32) from tokens i < seq_len[b] against the given mu
 *                (as fitted by sik_quantize_keys), then the records of those tokens
 *   SIK_Q_ENCODE records of tokens t0 <= i < t0 + n of every (b, h) against the given mu and
 *                alpha (both inputs); seq_len is not read and may be NULL
 * Other records are left untouched.  Needs no workspace. */
int sik_quantize_kv(const sik_layout *layout, const void *K, const void *V, const int32_t *seq_len,
                    int32_t t0, int32_t n, int mode, const float *mu, float *alpha, void *kvq,
                    void *stream);

/* Prefill-side compression of one layer in one call: everything sik_quantize_keys(SIK_Q_FIT) followed by
 * sik_quantize_kv(SIK_Q_FIT) writes - mu, codes, codebook, counts, alpha and the records of tokens
 * i < seq_len[b] - with identical bits, in two passes over K and one over V instead of four and one (sections
 * "One-Pass Sign-Based Clustering", "Entropy-Aware Normalization" and "Token-Wise Quantization Format"; this is the
 * work the paper prices as the overhead on the time to the second token, "End to End Efficiency" (i), and as
 * "Clustering" in its module-timing table).  The first pass takes the column sums and, per channel, the smallest
 * and the largest key, which fix alpha = max_i |K_i - mu| (|x - mu| peaks at an end of the range); the second
 * writes codes, cluster sums and records.  All outputs are device pointers as in those two calls; K and V are
 * read only; the workspace is sik_workspace_bytes(layout, k) for any k >= 0. */
int sik_prefill_compress(const sik_layout *layout, const void *K, const void *V, const int32_t *seq_len, float *mu,
                         float *codebook, int32_t *counts, uint8_t *codes, float *alpha, void *kvq, void *workspace,
                         size_t workspace_bytes, void *stream);

/* Sparse attention as sik_sparse_attn, on records: the logit of token j is
 * softmax_scale * sum_d q_d * s_d alpha_d D(K)_jd (the centred key: the dropped q . mu is one
 * constant per query head and cancels in the softmax, normalisation section), the value row is
 * D(V)_j; both are rebuilt in registers from the gathered record, never written to memory. */
int sik_sparse_attn_q2(const sik_layout *layout, const void *q, const void *kvq, const float *alpha,
                       const int32_t *idx, int32_t k, float softmax_scale, void *out,
                       void *workspace, size_t workspace_bytes, void *stream);

/* One decode step on the 2-bit cache: as sik_decode_step, with the records in place of K and V.
 * With k_new / v_new ([B,Hkv,D] kv_dtype, both or neither) the new token of every (b, h) is
 * quantised against the frozen mu and alpha into record seq_len[b] of kvq, its sign code is
 * written to codes, and seq_len[b] is incremented on the device; the 16-bit row is not kept.
 * kernel_us: NULL, or a host pointer to SIK_N_KERNELS + 1 floats that receives the event
 * intervals exactly as sik_decode_step_profiled does (and makes the call wait for the stream).
 * max_len above 524288 is not supported on this path (SIK_ERR_SHAPE). */
int sik_decode_step_q2(const sik_layout *layout, const void *q, const void *k_new, const void *v_new,
                       void *kvq, int32_t *seq_len, const float *mu, const float *alpha,
                       const float *codebook, uint8_t *codes, int32_t k, float softmax_scale,
                       void *out, int32_t *idx_out, void *workspace, size_t workspace_bytes,
                       void *stream, float *kernel_us);

/* ---- forced-inclusion sets (section "Full Precision Sink Tokens"; decode-time tokens that are
 * "always included", "Experimental Setup") ---------------------------------------------------
 * The general decode step: everything sik_decode_step and sik_decode_step_q2 take, as one
 * argument block, plus a set of tokens per (sequence, KV head) that always takes part in the
 * attention of the R query heads of that KV head and never competes in the top-k:
 *   forced_idx [B,Hkv,n_forced] int32 (device), n_forced <= 128; entries outside
 *   [0, seq_len[b]) name no token (use -1 for unused slots; after an append the new token's
 *   index is valid); the valid entries of one (b, h) must be distinct.
 * The budget k counts the forced tokens: each query head attends its forced tokens and the
 * k - (number of valid forced tokens of its KV head) best of the remaining ones (k > n_forced
 * is required).  idx_out lists both kinds, order unspecified, -1 padded.
 * forced_K / forced_V (2-bit cache only, both or neither): [B,Hkv,n_forced,D] kv_dtype rows of
 * the forced tokens, slot by slot, kept in 16 bits by the caller; when given, the forced tokens
 * are attended from these rows, each key centred by mu (the records hold the centred key),
 * instead of from their records.
 * k_per_mille (0 = off, else 1..1000): a budget that follows the context length, as in the
 * paper's "retains only 7.5 % of the tokens" setting (75): sequence b attends
 * min(k, max(1, ceil(seq_len[b] * k_per_mille / 1000))) tokens (integer arithmetic; forced
 * tokens counted, they may use the budget up); k stays the row length of idx_out.
 * group_shared (0 / 1): one index set per KV head, shared by its R query heads (a selector
 * variant that cuts the gathered bytes by R): the k tokens with the largest SUM over the group's
 * query heads of the compressed-domain scores (the table is linear in the query, so this is the
 * score of the summed query); each query head attends over that set with its own query.
 * idx_out is then [B,Hkv,k].  Combines with forced_idx (forced tokens are per KV head anyway)
 * and k_per_mille.
 * Cache: K and V (16-bit rows) with kvq = NULL, or kvq and alpha (2-bit records) with K = V =
 * NULL.  kernel_us as in sik_decode_step_q2.  Zero-initialise the block and set what applies. */
typedef struct {
    const void *q, *k_new, *v_new;
    void *K, *V;
    void *kvq;
    const float *alpha;
    int32_t *seq_len;
    const float *mu, *codebook;
    uint8_t *codes;
    int32_t k;
    int32_t k_per_mille;
    int32_t group_shared;
    float softmax_scale;
    const int32_t *forced_idx;
    int32_t n_forced;
    const void *forced_K, *forced_V;
    void *out;
    int32_t *idx_out;
    void *workspace;
    size_t workspace_bytes;
    void *stream;
    float *kernel_us;
    int32_t launches;     /* 0: the library chooses; 1: the one-launch step whenever its plan allows (sik_plan_info);
                             2: always separate scoring and selection + attention launches; 3: as 1, with the
                             first scoring pass in 16-bit fixed point (exact scores for the band around the cut) */
    int32_t spin_limit;   /* polls a bounded wait of the one-launch step may take; 0 = default (about a second)  */
} sik_decode_args;

int sik_decode_step_ex(const sik_layout *layout, const sik_decode_args *args);

#ifdef __cplusplus
}
#endif
#endif /* SIK_H */
