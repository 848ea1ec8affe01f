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

// ---- launch parameter blocks ------------------------------------------------
struct ScoreParams {
    const void* q_win;
    const void* k;
    const uint8_t* modality;
    float* score_self;
    float* score_cross;
    float* part;          // [B][H_q][n_chunks][O][2] partial (max, sum) in log2 units
    float* slice_self;    // [gsplit][H_sel][total] per-slice sums of a split selection group (gsplit > 1)
    float* slice_cross;
    const int32_t* cu;
    int32_t B, H_q, G, sel_group, O, R, causal;
    int32_t n_chunks, chunk_keys;
    int32_t gsplit, gper;  // a selection group is summed in gsplit slices of gper consecutive heads
    int64_t k_stride_tok, k_stride_head;  // elements
    int64_t total_tokens;
    float scale_log2;     // log2(e) / sqrt(D)
    float n_score;
};

struct SelectParams {
    const float* score_self;
    const float* score_cross;
    const uint8_t* modality;
    const int32_t* cu;
    const int32_t* budget_T;
    int32_t* kept_idx;
    int32_t* kept_cnt;
    int32_t B, H_sel, O, R, kept_cap;
    int64_t total_tokens;
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
    int32_t phases;       // bit 0: split kernel, bit 1: merge kernel
    float* out;
    float* part;          // [B][H_q][n_splits][D + 2]
    int32_t B, H_q, H_kv, G, n_splits, max_kv_len;
    int64_t stride_b, stride_head, stride_tok;  // bytes
    float scale_log2;
    float n_decode;
};

// ---- launchers (one per kernel family; each returns a hipError_t) -----------
hipError_t launch_score(const ScoreParams& p, int dtype, int D, int max_seqlen, hipStream_t s);
hipError_t launch_select(const SelectParams& p, int max_seqlen, hipStream_t s);
hipError_t launch_compact(const CompactParams& p, int row_bytes, hipStream_t s);
hipError_t launch_append(const AppendParams& p, hipStream_t s);
hipError_t launch_decode(const DecodeParams& p, int dtype, int D, hipStream_t s);

// host-side sizing rules shared by the *_workspace_bytes functions and the launchers
int score_chunk_keys(int B, int H_q, int max_seqlen);
// heads of a selection group that one workgroup of the column-sum pass sums itself
int score_heads_per_slice(int B, int H_q, int sel_group, int n_chunks);
int decode_num_splits(int B, int H_kv, int max_kv_len);

}  // namespace csp
