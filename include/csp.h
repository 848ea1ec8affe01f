/*
 * csp.h — C ABI of the MI355X (gfx950) Cross-Self Pruning library.
 *
 * The library implements the KV-cache pruning pass of Cross-Self Pruning
 * (arXiv 2412.04652, Section "Method", Algorithm 1) and the n-softmax decode
 * attention over the pruned cache (Section "Smoothness recovery of attention
 * scores").  One call per step of the path:
 *
 *   csp_score        observation-window attention weights, summed per key and
 *                    split into intra- / inter-modality importance
 *   csp_select       budget rule, per-region top-K, union with the recent keys
 *   csp_compact      gather of the kept K/V rows into the pruned cache
 *   csp_decode_attn  one decode step of n-softmax attention over that cache
 *   csp_append_kv    append the new token's k, v to the pruned cache
 *   csp_decode_step  append + attend fused into one call
 *   csp_reprune      the same pruning pass applied in place to the grown cache
 *                    while decoding (with csp_gather_modality, csp_window_push)
 *
 * Conventions
 *  - "device" pointers are HIP device memory owned by the caller; "host"
 *    pointers are ordinary host memory.  The library never allocates, frees or
 *    retains memory and never synchronises the host: every call enqueues its
 *    kernels on `stream` (a hipStream_t passed as void*; NULL = the default
 *    stream) and returns.  Scratch memory is passed in by the caller, sized by
 *    the *_workspace_bytes functions (pure host functions).
 *  - Outputs must not alias inputs.
 *  - Return value: CSP_OK, or a negative error code.  Arguments are validated
 *    on the host before anything is launched, so a call that returns an error
 *    has launched nothing.  CSP_EHIP means a HIP launch failed; the HIP error
 *    stays readable through hipGetLastError().
 *  - Q/K/V element type: CSP_BF16 (2 bytes) or CSP_F32.  Rows of D elements are
 *    contiguous; D is 64 or 128; every row must start on a 16-byte boundary.
 *    All arithmetic accumulates in fp32.
 *  - Sequences are packed along the token axis: sequence b owns tokens
 *    cu_seqlens[b] .. cu_seqlens[b+1]-1 (ragged batches); key row (token t,
 *    KV head h) starts at element  t*k_stride_tok + h*k_stride_head.
 *  - Query head hq reads KV head hq / (H_q/H_kv).  A *selection group* is
 *    sel_group consecutive query heads whose scores are summed before the
 *    top-K (head-axis handling of Section "Cross-self pruning"): 1 = one index
 *    set per head (requires H_q == H_kv), H_q/H_kv = one per KV head, H_q =
 *    one per layer.  sel_group must be a multiple of H_q/H_kv and divide H_q.
 *    H_sel = H_q / sel_group.
 */
#ifndef CSP_H
#define CSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { CSP_BF16 = 0, CSP_F32 = 1 };

enum {
    CSP_OK = 0,
    CSP_EINVAL = -1,       /* null pointer, inconsistent sizes, bad stride or alignment */
    CSP_EUNSUPPORTED = -2, /* D or dtype the kernels are not built for */
    CSP_EWORKSPACE = -3,   /* workspace missing or too small */
    CSP_EHIP = -4          /* a HIP call failed */
};

/* Problem description shared by all calls (plain data; the library reads it
 * during the call only). */
typedef struct csp_desc {
    int32_t dtype;       /* CSP_BF16 | CSP_F32: type of Q, K, V and of the pruned cache */
    int32_t B;           /* sequences in the batch */
    int32_t H_q, H_kv;   /* query heads, KV heads (H_q % H_kv == 0) */
    int32_t D;           /* head dimension: 64 or 128 */
    int32_t sel_group;   /* query heads per selection group (see above) */
    int32_t window_O;    /* observation window: the last O queries (A[-O:, :-R]) */
    int32_t recent_R;    /* recent keys always kept and never ranked */
    int32_t causal;      /* 1: window query at position p sees keys j <= p; 0: sees all */
    int32_t max_seqlen;  /* >= every sequence length (sizes grids and workspaces) */
    double  n_score;     /* n of the n-softmax used for scoring; 0 = plain softmax */
    double  n_decode;    /* n of the n-softmax used by csp_decode_attn (paper: 1) */
    double  cross_ratio; /* share of the T-R selected keys given to the inter-modality
                            region (appendix table "Cross Ratio"); in [0,1] */
    const int32_t* cu_seqlens_host; /* host   int32[B+1], for validation and sizing */
    const int32_t* budget_T_host;   /* host   int32[B], maximum cache length T per sequence */
    const int32_t* cu_seqlens;      /* device int32[B+1], same values */
    const int32_t* budget_T;        /* device int32[B], same values */
    int64_t k_stride_tok, k_stride_head; /* elements */
    int64_t v_stride_tok, v_stride_head; /* elements */
    int32_t score_wait_us; /* csp_score / csp_reprune, single-read kernel: the longest time a workgroup waits for
                              the softmax statistics of the other chunks of its head before it recomputes them
                              itself, in microseconds; 0 = default (1000); negative = never wait (every task takes
                              the self-sufficient path: a test setting).  The result does not depend on it. */
} csp_desc;

/* Human-readable name of an error code (static string). */
const char* csp_strerror(int code);

/* Library version string (static). */
const char* csp_version(void);

/* Measurement aid, no part of the method: streams `bytes` (a multiple of 16) from src at the
 * rate the memory system allows.  With dst != NULL the data is copied there; with dst == NULL it
 * is only read (folded into a few words that are XORed into sink).  The benchmark reports the
 * two rates beside the kernels' figures as the ceilings of the box it ran on.
 *   src, dst  device, 16-byte aligned, `bytes` long
 *   sink      device, 4 KiB, caller-initialised
 * Returns CSP_EINVAL for a null or misaligned pointer or a size that is not a multiple of 16. */
int csp_probe_stream(const void* src, void* dst, size_t bytes, void* sink, void* stream);

/* ------------------------------------------------------------------------
 * csp_score — Eq. "A = softmax(QK^T/sqrt d)" (or Eq. "n-softmax" when
 * n_score > 0) for the last O queries against every cached key, then the
 * per-key sums over the query axis split by modality, Eq. "cross-self":
 *   score_self [s][t]  = sum over the group's heads and over window rows i
 *                        whose modality equals the key's, of A_ij
 *   score_cross[s][t]  = same over rows of the other modality
 * for prefix keys j < L-R (t = cu_seqlens[b] + j); entries of the last R keys
 * of each sequence are written as 0.  The softmax denominator runs over all
 * visible keys including the last R.
 *
 *   q_win     device [B][H_q][O][D]  queries of positions L_b-O .. L_b-1
 *   k         device keys, strides from the descriptor
 *   modality  device uint8[total_tokens], 0 = text, 1 = visual
 *   score_*   device float [H_sel][total_tokens]
 *   ws        device scratch of csp_score_workspace_bytes(desc) bytes, 16-byte aligned
 *             (counters, softmax statistics per chunk, reset by the call itself; for a
 *             selection group that is summed in several slices, also one partial score
 *             array per slice, added in slice order: the result does not depend on
 *             scheduling).  Two calls that overlap in time (different streams) need a
 *             workspace each.  The first 16 bytes are int32 counters the call writes:
 *             [0] = tasks of the single-read kernel whose wait ran out (see below; 0
 *             unless the GPU was shared or score_wait_us was set very low).
 * bf16 with O <= 128 and G * ceil(O/64) * ceil(max_seqlen/512) <= 256 (G = H_q/H_kv:
 * 131072 keys per sequence for G = 1, O <= 64) reads the keys ONCE: a resident set of
 * one workgroup per compute unit walks 512-key chunks, keeps a chunk's logits in
 * registers, and the workgroups of a head exchange the chunks' log-sum-exps inside the
 * launch, one pipeline step behind the logits.  A workgroup whose bounded wait for the
 * others runs out (score_wait_us) recomputes the statistics of the head's chunks by
 * itself with the same code, in the same order: the scores are bit-identical either
 * way.  Other shapes (fp32, longer sequences) read the keys twice; results are the same
 * up to rounding.
 * Requires O <= L_b and R <= L_b for every sequence (CSP_EINVAL otherwise);
 * O <= 128.
 * ---------------------------------------------------------------------- */
size_t csp_score_workspace_bytes(const csp_desc* desc);
int csp_score(const csp_desc* desc, const void* q_win, const void* k, const uint8_t* modality,
              float* score_self, float* score_cross, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * csp_score_lse — csp_score for callers that already hold the softmax
 * normaliser of every window row: the prefill attention of the same layer
 * computes, per query row, the log-sum-exp of its scaled logits, and the
 * statistics half of csp_score would only recompute it from a second pass
 * over the keys.
 *   row_lse   device float [B][H_q][O]: ln( sum over visible keys j of
 *             exp(q_i.k_j / sqrt(D)) ) for window row i (causal: j <= L-O+i;
 *             all keys when desc->causal == 0), WITHOUT the n of the n-softmax
 *             (n_score is added here)
 * Everything else as in csp_score (same workspace size; the keys are read
 * once instead of twice).  The result equals csp_score's up to the rounding
 * of row_lse.
 * ---------------------------------------------------------------------- */
int csp_score_lse(const csp_desc* desc, const void* q_win, const void* k, const uint8_t* modality,
                  const float* row_lse, float* score_self, float* score_cross,
                  void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * csp_select — Eq. "top-K" per region, the mask combination (read as the
 * union of the two independently selected sets), the recent keys of the
 * cache-construction equation, and Algorithm 1's early-out.
 *
 * Per sequence b and selection group s, with L = L_b, T = budget_T[b]:
 *  - L <= T: identity, kept = 0..L-1.
 *  - otherwise K_sel = T-R, K^c = floor(cross_ratio*K_sel), K^s = K_sel-K^c;
 *    candidates of the self region are prefix keys whose modality some window
 *    query shares, of the cross region prefix keys whose other modality some
 *    window query has; a region with fewer candidates than its share passes
 *    the excess to the other.  The K^s largest score_self among self
 *    candidates and the K^c largest score_cross among cross candidates are
 *    kept (ties: lower index first), plus positions L-R..L-1.
 *
 *   kept_idx  device int32 [B][H_sel][kept_cap]: kept positions within the
 *             sequence, ascending, unique; slots past the count hold -1
 *   kept_cap  >= min(T_b, L_b) for every b (CSP_EINVAL otherwise)
 *   kept_cnt  device int32 [B][H_sel][4]: {kept, K^s, K^c, keys in both masks}
 * With a single-modality window (the usual case) kept == min(T, L); a window
 * holding both modalities can select a key twice and keeps fewer.
 * T_b < R with L_b > T_b is CSP_EINVAL.  Scores must be >= 0 (they are sums
 * of probabilities); selection compares their fp32 bit patterns.
 * No workspace is needed: ws may be NULL.
 * ---------------------------------------------------------------------- */
size_t csp_select_workspace_bytes(const csp_desc* desc);
int csp_select(const csp_desc* desc, const float* score_self, const float* score_cross,
               const uint8_t* modality, int32_t* kept_idx, int32_t kept_cap, int32_t* kept_cnt,
               void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * csp_compact — cache construction, Eq. "K = (K.M) (+) K[-R:]": a bit copy
 *   k_out[b][h][t] = k[cu_seqlens[b] + kept_idx[b][s(h)][t]][h],  t < kept
 * (same for v), s(h) = selection group of KV head h.  Row (b, h, t) of the
 * output starts at element b*out_stride_b + h*out_stride_head + t*out_stride_tok;
 * the caller sizes it for kept_cap plus the tokens it will append.
 *   kv_len    device int32 [B][H_kv], receives the kept count (may be NULL)
 * ---------------------------------------------------------------------- */
int csp_compact(const csp_desc* desc, const void* k, const void* v, const int32_t* kept_idx,
                int32_t kept_cap, const int32_t* kept_cnt, void* k_out, void* v_out,
                int64_t out_stride_b, int64_t out_stride_head, int64_t out_stride_tok,
                int32_t* kv_len, void* stream);

/* ------------------------------------------------------------------------
 * csp_decode_attn — one decode step with Eq. "n-softmax":
 *   s_t = q.k_t / sqrt(D),  p_t = e^{s_t} / (n_decode + sum_u e^{s_u}),
 *   out = sum_t p_t v_t      over t < kv_len[b][h]; no causal mask.
 * n enters once per query head, scaled consistently with the running maximum
 * (it is a virtual key of logit ln n and zero value).
 *
 *   q         device [B][H_q][D] (dtype of the descriptor)
 *   k_cache, v_cache  device, row (b, h, t) at b*cache_stride_b +
 *             h*cache_stride_head + t*cache_stride_tok (elements)
 *   kv_len    device int32 [B][H_kv]
 *   max_kv_len  host upper bound on kv_len (sizes the split of the key axis)
 *   out       device float [B][H_q][D]
 *   ws        device scratch of csp_decode_workspace_bytes(desc, max_kv_len) bytes
 * kv_len == 0 gives out = 0.
 * ---------------------------------------------------------------------- */
size_t csp_decode_workspace_bytes(const csp_desc* desc, int32_t max_kv_len);
int csp_decode_attn(const csp_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                    int64_t cache_stride_b, int64_t cache_stride_head, int64_t cache_stride_tok,
                    const int32_t* kv_len, int32_t max_kv_len, float* out,
                    void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * csp_decode_attn_static — csp_decode_attn for callers that cannot allocate
 * device memory and so cannot bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments and the
 * same result (bit for bit: the same kernels run), without ws / ws_bytes: the
 * split-KV partials go to a device array that is part of the library's code
 * object (csp_static_scratch_bytes() = 2 MiB per GPU, held until the process
 * ends).  The call allocates and frees nothing; the first call on a device
 * looks up the array's address there.
 *  - csp_decode_workspace_bytes(desc, max_kv_len) > csp_static_scratch_bytes()
 *    is CSP_EWORKSPACE (nothing is launched): use csp_decode_attn.
 *  - Every call on a GPU shares that GPU's array: two calls that overlap in
 *    time on one GPU (different streams) race; calls on one stream are safe.
 *    Nothing has to start at zero (the first kernel writes every partial the
 *    second one reads).
 * ---------------------------------------------------------------------- */
size_t csp_static_scratch_bytes(void);
int csp_decode_attn_static(const csp_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                           int64_t cache_stride_b, int64_t cache_stride_head, int64_t cache_stride_tok,
                           const int32_t* kv_len, int32_t max_kv_len, float* out, void* stream);

/* ------------------------------------------------------------------------
 * csp_decode_step — csp_append_kv followed by csp_decode_attn in one call (one
 * kernel launch fewer per decode step): the new token's key and value (device
 * [B][H_kv][D]) are appended at row kv_len[b][h] of the pruned cache, attended
 * to together with the rows before them (Eq. "n-softmax"), and kv_len[b][h] is
 * incremented.  A slab that is already full (kv_len == cache_cap) is left
 * unchanged and the new token is not attended to.  ws is sized by
 * csp_decode_workspace_bytes(desc, cache_cap).  Other arguments as in
 * csp_decode_attn / csp_append_kv.
 * ---------------------------------------------------------------------- */
int csp_decode_step(const csp_desc* desc, const void* q, const void* k_new, const void* v_new,
                    void* k_cache, void* v_cache, int64_t cache_stride_b, int64_t cache_stride_head,
                    int64_t cache_stride_tok, int32_t cache_cap, int32_t* kv_len, float* out,
                    void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * csp_decode_step_phase — the two launches of csp_decode_step one at a time,
 * for callers that time or schedule them apart: phase 1 streams the cache
 * (split-KV partials into ws, new token stored), phase 2 merges the partials,
 * applies the n of Eq. "n-softmax" and increments kv_len.  Phase 1 followed by
 * phase 2 with the same arguments on the same stream is exactly
 * csp_decode_step.  Any other phase value is CSP_EINVAL.
 * ---------------------------------------------------------------------- */
int csp_decode_step_phase(const csp_desc* desc, int32_t phase, const void* q, const void* k_new,
                          const void* v_new, void* k_cache, void* v_cache, int64_t cache_stride_b,
                          int64_t cache_stride_head, int64_t cache_stride_tok, int32_t cache_cap,
                          int32_t* kv_len, float* out, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------
 * csp_append_kv — the KV-cache append of Section "Preliminary": writes the new
 * token's key and value (device [B][H_kv][D]) at row kv_len[b][h] of the
 * pruned cache and increments kv_len[b][h].  cache_cap is the number of rows
 * each (b, h) slab can hold; a full slab is left unchanged.
 * ---------------------------------------------------------------------- */
int csp_append_kv(const csp_desc* desc, const void* k_new, const void* v_new, void* k_cache,
                  void* v_cache, int64_t cache_stride_b, int64_t cache_stride_head,
                  int64_t cache_stride_tok, int32_t cache_cap, int32_t* kv_len, void* stream);

/* ------------------------------------------------------------------------
 * Re-pruning while decoding — the loop of Algorithm 1: at a generation step
 * the cache (pruned keys plus the tokens appended since) is checked against
 * the budget T and, when longer, pruned again with the same procedure: the
 * window is the last O queries, key t of the cache is visible to window row i
 * iff t <= L-O+i (L = current cache length; cache order is temporal order), the
 * last R rows are kept unranked, the regions follow the modality of the cached
 * keys.  The paper does not say how often this runs; the caller decides (every
 * step, or every few steps so that the cache oscillates between T and T+s).
 *
 * csp_gather_modality — companion of csp_compact: the modality of every kept
 * key next to the pruned cache, because each selection group keeps different
 * keys:  mod_cache[b][s][t] = modality[cu_seqlens[b] + kept_idx[b][s][t]] for
 * t < kept, 0 for kept <= t < cache_cap (tokens appended while decoding are
 * text).
 *   mod_cache device uint8 [B][H_sel][cache_cap]
 *
 * csp_window_push — stores the current step's queries (device [B][H_q][D]) in
 * slot `slot` (0 <= slot < O) of the ring q_ring (device [B][H_q][O][D]) that
 * holds the last O queries.
 *
 * csp_reprune — score -> select -> in-place compaction over the cache.
 *   q_ring, ring_start   the last O queries; ring_start is the slot of the
 *             oldest one (a window already in temporal order: ring_start = 0)
 *   k_cache, v_cache, strides, cache_cap, kv_len   as in csp_decode_step; kv_len
 *             is read (all KV heads of a selection group must agree) and
 *             receives the kept count
 *   mod_cache as above; kept flags are moved with their keys, the freed tail
 *             is cleared
 *   score_self, score_cross  device float [B][H_sel][cache_cap], written for
 *             the ranked keys of every sequence that is pruned
 *   kept_idx, kept_cap, kept_cnt   as in csp_select (cache positions); kept_cap
 *             >= every T_b
 *   ws        device scratch of csp_reprune_workspace_bytes(desc, cache_cap)
 * A sequence with kv_len <= T_b is left untouched (its scores are not
 * written, its kept_idx is the identity).  Requires T_b >= max(O, R) for every
 * b (CSP_EINVAL otherwise), so that a sequence that is pruned holds a full
 * window.  Descriptor fields read: dtype, B, H_q, H_kv, D, sel_group, window_O,
 * recent_R, causal, n_score, cross_ratio, budget_T_host, budget_T; cu_seqlens,
 * max_seqlen and the K/V strides are not used.
 * The compaction moves rows down inside one buffer: a workgroup owns one
 * (sequence, KV head) and orders its reads before its writes block by block;
 * K, V and mod_cache must not be accessed by other work until the call's
 * kernels have finished.
 * ---------------------------------------------------------------------- */
/* csp_decode_step_window — csp_decode_step that also does csp_window_push(q, q_ring, slot)
 * inside its first kernel (no extra launch per decode step). */
int csp_decode_step_window(const csp_desc* desc, const void* q, const void* k_new, const void* v_new,
                           void* k_cache, void* v_cache, int64_t cache_stride_b, int64_t cache_stride_head,
                           int64_t cache_stride_tok, int32_t cache_cap, int32_t* kv_len, float* out,
                           void* q_ring, int32_t slot, void* ws, size_t ws_bytes, void* stream);
int csp_gather_modality(const csp_desc* desc, const uint8_t* modality, const int32_t* kept_idx,
                        int32_t kept_cap, const int32_t* kept_cnt, uint8_t* mod_cache,
                        int32_t cache_cap, void* stream);
int csp_window_push(const csp_desc* desc, const void* q_new, void* q_ring, int32_t slot, void* stream);
size_t csp_reprune_workspace_bytes(const csp_desc* desc, int32_t cache_cap);
int csp_reprune(const csp_desc* desc, const void* q_ring, int32_t ring_start,
                void* k_cache, void* v_cache, int64_t cache_stride_b, int64_t cache_stride_head,
                int64_t cache_stride_tok, int32_t cache_cap, uint8_t* mod_cache, int32_t* kv_len,
                float* score_self, float* score_cross, int32_t* kept_idx, int32_t kept_cap,
                int32_t* kept_cnt, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CSP_H */
