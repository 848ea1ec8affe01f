// Internal declarations shared by the translation units of libcsp (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/csp.h"

namespace csp {

constexpr int kWave = 64;

// 16-byte vector used for every global <-> register <-> LDS move of K/V rows.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

struct bf16_tag {};  // element tags: storage type of Q/K/V
struct f32_tag {};

template <typename E> struct elem_bytes;
template <> struct elem_bytes<bf16_tag> { static constexpr int value = 2; };
template <> struct elem_bytes<f32_tag> { static constexpr int value = 4; };

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// v_exp_f32: 2^x (flushes denormal results, which is fine for softmax terms)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// ---- where a sequence's keys, modality flags and scores live ------------------
// Packed form (pruning after prefill): the rows of all sequences back to back on one token
// axis, lengths from cu_seqlens, modality [total], scores [H_sel][total].
// Cache form (re-pruning the grown cache): keys in the pruned cache [B][H_kv][cap][D], live
// lengths on the device, modality and scores per (sequence, selection group) [B][H_sel][cap].
struct SeqView {
    const int32_t* cu;        // packed: [B+1]
    const int32_t* kv_len;    // cache: [B][H_kv]; nullptr selects the packed form
    const int32_t* budget_T;  // cache: a sequence with kv_len <= budget is left alone
    int32_t H_kv, H_sel, cap;
    int64_t total_tokens;     // packed
    int64_t k_stride_batch;   // cache: elements between sequences
};

// live keys of sequence b as seen by KV head hk (all heads of a selection group agree)
__device__ __forceinline__ int view_len(const SeqView& v, int b, int hk) {
    if (!v.kv_len) return v.cu[b + 1] - v.cu[b];
    const int n = v.kv_len[b * v.H_kv + hk];
    return n < 0 ? 0 : (n > v.cap ? v.cap : n);  // a device-side count is never trusted beyond the capacity
}
// cache form only: the sequence already fits its budget, nothing is scored or moved
__device__ __forceinline__ bool view_fits(const SeqView& v, int b, int L) {
    return v.kv_len != nullptr && L <= v.budget_T[b];
}
// first key of sequence b in the modality array of selection group sg
__device__ __forceinline__ int64_t view_mod0(const SeqView& v, int b, int sg) {
    return v.kv_len ? ((int64_t)b * v.H_sel + sg) * v.cap : (int64_t)v.cu[b];
}
// ... in the score arrays of selection group sg
__device__ __forceinline__ int64_t view_score0(const SeqView& v, int b, int sg) {
    return v.kv_len ? ((int64_t)b * v.H_sel + sg) * v.cap : (int64_t)sg * v.total_tokens + v.cu[b];
}
// ... in the key tensor, in elements, without the head term
__device__ __forceinline__ int64_t view_key0(const SeqView& v, int b, int64_t k_stride_tok) {
    return v.kv_len ? (int64_t)b * v.k_stride_batch : (int64_t)v.cu[b] * k_stride_tok;
}

// ---- launch parameter blocks ------------------------------------------------
// a record of the single-read score kernel's task table (see score_single.hip)
struct alignas(16) PipeRec {
    int32_t rows_valid;    // window rows of the part (low 16 bits); bit 16 clear: nothing to compute (the addresses
                           // below still point at readable memory)
    int32_t L;             // keys of the sequence, at least 1
    int32_t c0;            // first key of the chunk
    int32_t pos0;          // absolute position of the part's window row 0
    uint32_t spare0, spare1;
    const char* kbase;     // key row 0 of the sequence, this KV head
    const char* qpart;     // query row 0 of the part
    const uint32_t* kbits; // modality of the chunk's keys, a word per 32 keys (bit j % 32 of word j / 32: key c0 + j is visual)
    float* stat;           // statistics of the head part: chunk 0, row 0
    float* out_self;       // self score of key 0 in the array this task writes (cross: + ScoreParams::cross_delta)
};
struct ScoreParams {
    const void* q_win;
    const void* k;
    const uint8_t* modality;
    float* score_self;
    float* score_cross;
    int32_t* counters;    // int32[4] at the start of the workspace: [0] = tasks of the single-read kernel whose wait
                          // for the other chunks ran out (statistics recomputed by the workgroup itself)
    float* part;          // two passes: [B][H_q][n_chunks][O][2] partial (max, sum) in log2 units;
                          // single read: [B][H_q][vsplit][n_chunks][64] log-sum-exp of a chunk in log2 units,
                          // NaN = not yet published
    int64_t spin_ticks;   // single read: longest wait for the other chunks, in 10 ns ticks; 0 = do not wait
    int32_t single;       // 1: one read of the keys (score_plan decides)
    int32_t single_chunks, vsplit;  // single read: 512-key chunks per sequence; parts of <= 64 window rows
    int32_t n_tasks, n_lin, n_iters;  // single read: tasks, padded task ids, pipeline steps (filled in by the launcher)
    PipeRec* table;            // single read: task table in the workspace, n_lin + 1 records (filled in by the launcher)
    uint32_t* modbits;         // single read: behind the table, the keys' modality as bits (see score_single.hip; written by
                               // the set-up kernel of the launch)
    int64_t cross_delta;              // single read: elements from the self score array (or slices) to the cross one
    int32_t D;                        // single read: head dimension
    float* slice_base;    // first of the per-slice score arrays in the workspace (slice_self/slice_cross are derived)
    const float* row_lse; // [B][H_q][O] natural-log normaliser of every window row, supplied by the caller
                          // (then the statistics pass is skipped and `part` is not used); nullptr otherwise
    float* slice_self;    // [gsplit][score_elems] per-slice sums of a split selection group (gsplit > 1)
    float* slice_cross;
    SeqView view;
    int64_t score_elems;  // floats in score_self (= in score_cross)
    int32_t B, H_q, G, sel_group, O, R, causal;
    int32_t n_chunks, chunk_keys;
    int32_t gsplit, gper;  // a selection group is summed in gsplit slices of gper consecutive heads
    int64_t k_stride_tok, k_stride_head;  // elements
    float scale_log2;     // log2(e) / sqrt(D)
    float n_score;
};

struct SelectParams {
    const float* score_self;
    const float* score_cross;
    const uint8_t* modality;
    SeqView view;
    const int32_t* budget_T;
    int32_t* kept_idx;
    int32_t* kept_cnt;
    int32_t B, H_sel, O, R, kept_cap;
    double cross_ratio;
};

struct CompactParams {
    const void* k;
    const void* v;
    const int32_t* kept_idx;
    const int32_t* kept_cnt;
    const int32_t* cu;
    void* k_out;
    void* v_out;
    int32_t* kv_len;
    int32_t B, H_kv, H_sel, kv_per_sel, kept_cap;
    int64_t k_stride_tok, k_stride_head, v_stride_tok, v_stride_head;  // bytes
    int64_t out_stride_b, out_stride_head, out_stride_tok;              // bytes
};

struct AppendParams {
    const void* k_new;
    const void* v_new;
    void* k_cache;
    void* v_cache;
    int32_t* kv_len;
    int32_t B, H_kv, cache_cap, row_bytes;
    int64_t stride_b, stride_head, stride_tok;  // bytes
};

struct DecodeParams {
    const void* q;
    const void* k_new;    // fused append (csp_decode_step); nullptr = attend only
    const void* v_new;
    void* k_cache;
    void* v_cache;
    int32_t* kv_len;
    int32_t cache_cap;
    void* q_ring;         // ring of the last ring_O queries [B][H_q][ring_O][D]; nullptr = not recorded
    int32_t ring_O, ring_slot;
    int32_t phases;       // bit 0: split kernel, bit 1: merge kernel
    float* out;
    float* part;          // [B][H_q][n_splits][D + 2]
    int32_t B, H_q, H_kv, G, n_splits, max_kv_len;
    int64_t stride_b, stride_head, stride_tok;  // bytes
    float scale_log2;
    float n_decode;
};

// in-place compaction of the grown cache, modality bookkeeping, window ring
struct RepruneParams {
    void* k_cache;
    void* v_cache;
    uint8_t* mod_cache;        // [B][H_sel][cache_cap]
    const int32_t* kept_idx;   // [B][H_sel][kept_cap]
    const int32_t* kept_cnt;   // [B][H_sel][4]
    const int32_t* budget_T;
    int32_t* kv_len;           // [B][H_kv]
    int32_t B, H_kv, H_sel, kv_per_sel, kept_cap, cache_cap;
    int64_t stride_b, stride_head, stride_tok;  // bytes
};

struct ModGatherParams {
    const uint8_t* modality;   // packed [total]
    const int32_t* cu;
    const int32_t* kept_idx;
    const int32_t* kept_cnt;
    uint8_t* mod_out;          // [B][H_sel][mod_cap]
    int32_t B, H_sel, kept_cap, mod_cap;
};

struct WindowParams {
    const void* src;
    void* dst;
    int32_t rows;              // B * H_q
    int32_t O, row_bytes;
    int32_t slot;              // push: ring slot written; unroll: ring slot of the oldest query
};

// ---- launchers (one per kernel family; each returns a hipError_t) -----------
hipError_t launch_score(const ScoreParams& p, int dtype, int D, int max_seqlen, hipStream_t s);
hipError_t launch_select(const SelectParams& p, int max_seqlen, hipStream_t s);
hipError_t launch_compact(const CompactParams& p, int row_bytes, hipStream_t s);
hipError_t launch_probe_stream(const void* src, void* dst, size_t bytes, uint32_t* sink, hipStream_t s);
hipError_t launch_append(const AppendParams& p, hipStream_t s);
hipError_t launch_decode(const DecodeParams& p, int dtype, int D, hipStream_t s);
hipError_t launch_mod_gather(const ModGatherParams& p, hipStream_t s);
hipError_t launch_reprune_move(const RepruneParams& p, int row_bytes, hipStream_t s);
hipError_t launch_window_push(const WindowParams& p, hipStream_t s);
hipError_t launch_window_unroll(const WindowParams& p, hipStream_t s);

// host-side sizing rules shared by the *_workspace_bytes functions and the launchers
struct ScorePlan {
    int chunk_keys, n_chunks, gper, gsplit;   // two passes over the keys
    bool single;           // statistics and column sums from one read of the keys
    int single_chunks, vsplit, single_gsplit; // ... its 512-key chunks, window parts and slice arrays
    int max_gsplit;        // slice arrays the workspace holds (covers both paths and csp_score_lse)
    size_t part_bytes;     // counters + statistics region at the start of the workspace (16-byte multiple)
};
constexpr int kScoreSingleChunk = 512;      // keys per task of the single-read kernel
constexpr int kScoreSingleRecBytes = 64;    // one task-table record
constexpr int kScoreSingleMaxIters = 2048;  // pipeline steps one workgroup may run
hipError_t launch_score_single(ScoreParams& p, int D, hipStream_t s);
ScorePlan score_plan(int B, int H_q, int H_kv, int sel_group, int max_seqlen, int dtype, int D, int O, bool have_row_lse);
int score_chunk_keys(int B, int H_q, int max_seqlen, int dtype, int D, int O);
// heads of a selection group that one workgroup of the column-sum pass sums itself
int score_heads_per_slice(int B, int H_q, int sel_group, int n_chunks);
int decode_num_splits(int B, int H_kv, int max_kv_len);

}  // namespace csp
