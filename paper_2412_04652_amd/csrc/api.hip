// C ABI of libcsp: host-side validation and marshalling (see include/csp.h for
// the contract of every entry point).  Nothing here touches the GPU until the
// arguments have been checked.
#include <cmath>
#include <cstring>
#include <mutex>

#include "csp_internal.h"

using namespace csp;

namespace {

struct Checked {
    int G, H_sel, kv_per_sel, EB, row_bytes;
    int64_t total_tokens;
    int max_len;
};

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Checks of the descriptor that every call shares.  need_lengths: the call
// reads cu_seqlens (everything but decode/append).
int check_desc(const csp_desc* d, bool need_lengths, Checked* c) {
    if (!d) return CSP_EINVAL;
    if (d->dtype != CSP_BF16 && d->dtype != CSP_F32) return CSP_EUNSUPPORTED;
    if (d->D != 64 && d->D != 128) return CSP_EUNSUPPORTED;
    if (d->B <= 0 || d->H_q <= 0 || d->H_kv <= 0 || d->H_q % d->H_kv != 0) return CSP_EINVAL;
    if (d->B > 32767) return CSP_EINVAL;
    c->G = d->H_q / d->H_kv;
    if (d->sel_group <= 0 || d->H_q % d->sel_group != 0 || d->sel_group % c->G != 0) return CSP_EINVAL;
    c->H_sel = d->H_q / d->sel_group;
    c->kv_per_sel = d->sel_group / c->G;
    c->EB = d->dtype == CSP_BF16 ? 2 : 4;
    c->row_bytes = d->D * c->EB;
    c->total_tokens = 0;
    c->max_len = 0;
    if (!(d->n_score >= 0.0) || !(d->n_decode >= 0.0) || !std::isfinite(d->n_score) || !std::isfinite(d->n_decode)) return CSP_EINVAL;
    if (!(d->cross_ratio >= 0.0 && d->cross_ratio <= 1.0)) return CSP_EINVAL;
    if (need_lengths) {
        if (!d->cu_seqlens_host || !d->cu_seqlens) return CSP_EINVAL;
        if (d->window_O <= 0 || d->recent_R < 0) return CSP_EINVAL;
        if (d->window_O > 128) return CSP_EUNSUPPORTED;
        if (d->cu_seqlens_host[0] != 0) return CSP_EINVAL;
        for (int b = 0; b < d->B; ++b) {
            const int64_t len = (int64_t)d->cu_seqlens_host[b + 1] - d->cu_seqlens_host[b];
            if (len <= 0 || len > d->max_seqlen) return CSP_EINVAL;
            if (d->window_O > len || d->recent_R > len) return CSP_EINVAL;
            if (len > c->max_len) c->max_len = (int)len;
        }
        c->total_tokens = d->cu_seqlens_host[d->B];
    }
    return CSP_OK;
}

int check_kv_strides(int64_t s_tok, int64_t s_head, int D, int EB) {
    if (s_tok < D || s_head < 0) return CSP_EINVAL;
    if ((s_tok * EB) % 16 != 0 || (s_head * EB) % 16 != 0) return CSP_EINVAL;
    return CSP_OK;
}

int check_budgets(const csp_desc* d, int kept_cap) {
    if (!d->budget_T_host || !d->budget_T) return CSP_EINVAL;
    for (int b = 0; b < d->B; ++b) {
        const int len = d->cu_seqlens_host[b + 1] - d->cu_seqlens_host[b];
        const int T = d->budget_T_host[b];
        if (T < 0) return CSP_EINVAL;
        if (len > T && T < d->recent_R) return CSP_EINVAL;
        if ((len < T ? len : T) > kept_cap) return CSP_EINVAL;
    }
    return CSP_OK;
}

const double kLog2e = 1.4426950408889634;

// plan -> launch parameters; slices: first byte of the per-slice score arrays
void set_score_plan(ScoreParams& p, const ScorePlan& pl, const csp_desc* d, char* slices) {
    p.single = pl.single ? 1 : 0;
    p.single_chunks = pl.single_chunks; p.vsplit = pl.vsplit;
    p.chunk_keys = pl.chunk_keys; p.n_chunks = pl.n_chunks; p.gper = pl.gper; p.gsplit = pl.gsplit;
    p.slice_base = pl.max_gsplit > 1 ? reinterpret_cast<float*>(slices) : nullptr;
    // longest wait of a single-read workgroup for the other chunks of its head, in 10 ns ticks
    p.spin_ticks = d->score_wait_us < 0 ? 0 : (d->score_wait_us == 0 ? 100000 : (int64_t)d->score_wait_us * 100);
}

}  // namespace

extern "C" {

const char* csp_strerror(int code) {
    switch (code) {
        case CSP_OK: return "ok";
        case CSP_EINVAL: return "invalid argument";
        case CSP_EUNSUPPORTED: return "unsupported head dimension, dtype or window size";
        case CSP_EWORKSPACE: return "workspace missing or too small";
        case CSP_EHIP: return "HIP call failed";
        default: return "unknown error";
    }
}

const char* csp_version(void) { return "csp-gfx950 0.1"; }


size_t csp_score_workspace_bytes(const csp_desc* d) {
    if (!d || d->B <= 0 || d->H_q <= 0 || d->max_seqlen <= 0 || d->window_O <= 0) return 0;
    if (d->sel_group <= 0 || d->H_q % d->sel_group != 0) return 0;
    const ScorePlan pl = score_plan(d->B, d->H_q, d->H_kv, d->sel_group, d->max_seqlen, d->dtype, d->D, d->window_O, false);
    size_t bytes = pl.part_bytes;
    // per-slice sums of a selection group that is split over several workgroups
    if (pl.max_gsplit > 1) {
        const size_t total = d->cu_seqlens_host ? (size_t)d->cu_seqlens_host[d->B] : (size_t)d->B * d->max_seqlen;
        bytes += (size_t)2 * pl.max_gsplit * (d->H_q / d->sel_group) * total * sizeof(float);
    }
    return bytes;
}

static int score_common(const csp_desc* d, const void* q_win, const void* k, const uint8_t* modality,
                        const float* row_lse, float* score_self, float* score_cross, void* ws, size_t ws_bytes,
                        void* stream) {
    Checked c;
    int rc = check_desc(d, true, &c);
    if (rc != CSP_OK) return rc;
    if (!q_win || !k || !modality || !score_self || !score_cross) return CSP_EINVAL;
    if (!aligned16(q_win) || !aligned16(k)) return CSP_EINVAL;
    if ((rc = check_kv_strides(d->k_stride_tok, d->k_stride_head, d->D, c.EB)) != CSP_OK) return rc;
    const size_t need = csp_score_workspace_bytes(d);
    if (!ws || ws_bytes < need || !aligned16(ws)) return CSP_EWORKSPACE;

    ScoreParams p;
    std::memset(&p, 0, sizeof(p));
    p.q_win = q_win; p.k = k; p.modality = modality;
    p.score_self = score_self; p.score_cross = score_cross;
    p.counters = static_cast<int32_t*>(ws);
    p.part = reinterpret_cast<float*>(static_cast<char*>(ws) + 16);
    p.row_lse = row_lse;
    p.view.cu = d->cu_seqlens; p.view.H_kv = d->H_kv; p.view.H_sel = c.H_sel; p.view.total_tokens = c.total_tokens;
    p.score_elems = (int64_t)c.H_sel * c.total_tokens;
    p.B = d->B; p.H_q = d->H_q; p.G = c.G; p.sel_group = d->sel_group;
    p.O = d->window_O; p.R = d->recent_R; p.causal = d->causal ? 1 : 0;
    const ScorePlan pl = score_plan(d->B, d->H_q, d->H_kv, d->sel_group, d->max_seqlen, d->dtype, d->D, d->window_O, row_lse != nullptr);
    set_score_plan(p, pl, d, static_cast<char*>(ws) + pl.part_bytes);
    p.k_stride_tok = d->k_stride_tok; p.k_stride_head = d->k_stride_head;
    p.scale_log2 = (float)(kLog2e / std::sqrt((double)d->D));
    p.n_score = (float)d->n_score;
    return launch_score(p, d->dtype, d->D, d->max_seqlen, static_cast<hipStream_t>(stream)) == hipSuccess ? CSP_OK : CSP_EHIP;
}

int csp_score(const csp_desc* d, const void* q_win, const void* k, const uint8_t* modality,
              float* score_self, float* score_cross, void* ws, size_t ws_bytes, void* stream) {
    return score_common(d, q_win, k, modality, nullptr, score_self, score_cross, ws, ws_bytes, stream);
}

int csp_score_lse(const csp_desc* d, const void* q_win, const void* k, const uint8_t* modality, const float* row_lse,
                  float* score_self, float* score_cross, void* ws, size_t ws_bytes, void* stream) {
    if (!row_lse) return CSP_EINVAL;
    return score_common(d, q_win, k, modality, row_lse, score_self, score_cross, ws, ws_bytes, stream);
}

size_t csp_select_workspace_bytes(const csp_desc*) { return 0; }

int csp_select(const csp_desc* d, const float* score_self, const float* score_cross,
               const uint8_t* modality, int32_t* kept_idx, int32_t kept_cap, int32_t* kept_cnt,
               void* /*ws*/, size_t /*ws_bytes*/, void* stream) {
    Checked c;
    int rc = check_desc(d, true, &c);
    if (rc != CSP_OK) return rc;
    if (!score_self || !score_cross || !modality || !kept_idx || !kept_cnt || kept_cap <= 0) return CSP_EINVAL;
    if ((rc = check_budgets(d, kept_cap)) != CSP_OK) return rc;
    SelectParams p;
    std::memset(&p, 0, sizeof(p));
    p.score_self = score_self; p.score_cross = score_cross; p.modality = modality;
    p.view.cu = d->cu_seqlens; p.view.H_kv = d->H_kv; p.view.H_sel = c.H_sel; p.view.total_tokens = c.total_tokens;
    p.budget_T = d->budget_T;
    p.kept_idx = kept_idx; p.kept_cnt = kept_cnt;
    p.B = d->B; p.H_sel = c.H_sel; p.O = d->window_O; p.R = d->recent_R; p.kept_cap = kept_cap;
    p.cross_ratio = d->cross_ratio;
    return launch_select(p, d->max_seqlen, static_cast<hipStream_t>(stream)) == hipSuccess ? CSP_OK : CSP_EHIP;
}

int csp_compact(const csp_desc* d, const void* k, const void* v, const int32_t* kept_idx,
                int32_t kept_cap, const int32_t* kept_cnt, void* k_out, void* v_out,
                int64_t out_stride_b, int64_t out_stride_head, int64_t out_stride_tok,
                int32_t* kv_len, void* stream) {
    Checked c;
    int rc = check_desc(d, true, &c);
    if (rc != CSP_OK) return rc;
    if (!k || !v || !kept_idx || !kept_cnt || !k_out || !v_out || kept_cap <= 0) return CSP_EINVAL;
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out)) return CSP_EINVAL;
    if ((rc = check_kv_strides(d->k_stride_tok, d->k_stride_head, d->D, c.EB)) != CSP_OK) return rc;
    if ((rc = check_kv_strides(d->v_stride_tok, d->v_stride_head, d->D, c.EB)) != CSP_OK) return rc;
    if ((rc = check_kv_strides(out_stride_tok, out_stride_head, d->D, c.EB)) != CSP_OK) return rc;
    if (out_stride_b < 0 || (out_stride_b * c.EB) % 16 != 0) return CSP_EINVAL;
    CompactParams p;
    std::memset(&p, 0, sizeof(p));
    p.k = k; p.v = v; p.kept_idx = kept_idx; p.kept_cnt = kept_cnt; p.cu = d->cu_seqlens;
    p.k_out = k_out; p.v_out = v_out; p.kv_len = kv_len;
    p.B = d->B; p.H_kv = d->H_kv; p.H_sel = c.H_sel; p.kv_per_sel = c.kv_per_sel; p.kept_cap = kept_cap;
    p.k_stride_tok = d->k_stride_tok * c.EB; p.k_stride_head = d->k_stride_head * c.EB;
    p.v_stride_tok = d->v_stride_tok * c.EB; p.v_stride_head = d->v_stride_head * c.EB;
    p.out_stride_b = out_stride_b * c.EB; p.out_stride_head = out_stride_head * c.EB; p.out_stride_tok = out_stride_tok * c.EB;
    return launch_compact(p, c.row_bytes, static_cast<hipStream_t>(stream)) == hipSuccess ? CSP_OK : CSP_EHIP;
}

// ---- csp_decode_attn_static: the split-KV partials live in a device array of the library ------
// Host code never passes the array's NAME to a kernel (in host code it is only a stand-in for the
// symbol): its device address is looked up once per device and kept.
#define CSP_STATIC_SCRATCH_BYTES (2u << 20)
static __device__ __align__(256) unsigned char scratch[CSP_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (each device holds its own copy).
int static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CSP_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return CSP_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return CSP_OK;
}
}  // namespace

size_t csp_decode_workspace_bytes(const csp_desc* d, int32_t max_kv_len) {
    if (!d || d->B <= 0 || d->H_q <= 0 || d->H_kv <= 0 || max_kv_len <= 0) return 0;
    const int ns = decode_num_splits(d->B, d->H_kv, max_kv_len);
    return (size_t)d->B * d->H_q * ns * (d->D + 2) * sizeof(float);
}

static int decode_common(const csp_desc* d, const void* q, const void* k_new, const void* v_new,
                         void* k_cache, void* v_cache, int64_t cache_stride_b, int64_t cache_stride_head,
                         int64_t cache_stride_tok, int32_t cache_cap, int32_t* kv_len, int32_t max_kv_len,
                         float* out, void* ws, size_t ws_bytes, void* stream, int phases = 3,
                         void* q_ring = nullptr, int32_t ring_slot = 0, bool static_ws = false) {
    Checked c;
    int rc = check_desc(d, false, &c);
    if (rc != CSP_OK) return rc;
    if (!q || !k_cache || !v_cache || !kv_len || !out || max_kv_len <= 0) return CSP_EINVAL;
    if (q_ring && (!aligned16(q_ring) || d->window_O <= 0 || ring_slot < 0 || ring_slot >= d->window_O)) return CSP_EINVAL;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache)) return CSP_EINVAL;
    if (k_new && (!v_new || !aligned16(k_new) || !aligned16(v_new) || cache_cap <= 0)) return CSP_EINVAL;
    if ((rc = check_kv_strides(cache_stride_tok, cache_stride_head, d->D, c.EB)) != CSP_OK) return rc;
    if (cache_stride_b < 0 || (cache_stride_b * c.EB) % 16 != 0) return CSP_EINVAL;
    const size_t need = csp_decode_workspace_bytes(d, max_kv_len);
    if (static_ws) {
        // the library's own scratch array; looked up only now, when every argument has been checked
        if (need > CSP_STATIC_SCRATCH_BYTES) return CSP_EWORKSPACE;
        if ((rc = static_scratch(&ws)) != CSP_OK) return rc;
        ws_bytes = CSP_STATIC_SCRATCH_BYTES;
    }
    if (!ws || ws_bytes < need || !aligned16(ws)) return CSP_EWORKSPACE;
    DecodeParams p;
    std::memset(&p, 0, sizeof(p));
    p.q = q; p.k_new = k_new; p.v_new = v_new; p.k_cache = k_cache; p.v_cache = v_cache; p.kv_len = kv_len; p.out = out;
    p.cache_cap = cache_cap;
    p.q_ring = q_ring; p.ring_O = d->window_O; p.ring_slot = ring_slot;
    p.phases = phases;
    p.part = static_cast<float*>(ws);
    p.B = d->B; p.H_q = d->H_q; p.H_kv = d->H_kv; p.G = c.G;
    p.n_splits = decode_num_splits(d->B, d->H_kv, max_kv_len);
    p.max_kv_len = max_kv_len;
    p.stride_b = cache_stride_b * c.EB; p.stride_head = cache_stride_head * c.EB; p.stride_tok = cache_stride_tok * c.EB;
    p.scale_log2 = (float)(kLog2e / std::sqrt((double)d->D));
    p.n_decode = (float)d->n_decode;
    return launch_decode(p, d->dtype, d->D, static_cast<hipStream_t>(stream)) == hipSuccess ? CSP_OK : CSP_EHIP;
}

int csp_decode_attn(const csp_desc* d, const void* q, const void* k_cache, const void* v_cache,
                    int64_t cache_stride_b, int64_t cache_stride_head, int64_t cache_stride_tok,
                    const int32_t* kv_len, int32_t max_kv_len, float* out,
                    void* ws, size_t ws_bytes, void* stream) {
    // attend only: nothing is written to the cache or to kv_len
    return decode_common(d, q, nullptr, nullptr, const_cast<void*>(k_cache), const_cast<void*>(v_cache), cache_stride_b,
                         cache_stride_head, cache_stride_tok, 0, const_cast<int32_t*>(kv_len), max_kv_len, out, ws,
                         ws_bytes, stream);
}

size_t csp_static_scratch_bytes(void) { return CSP_STATIC_SCRATCH_BYTES; }

int csp_decode_attn_static(const csp_desc* d, const void* q, const void* k_cache, const void* v_cache,
                           int64_t cache_stride_b, int64_t cache_stride_head, int64_t cache_stride_tok,
                           const int32_t* kv_len, int32_t max_kv_len, float* out, void* stream) {
    // sizes beyond the library's own scratch are refused first: use csp_decode_attn for those
    if (d && max_kv_len > 0 && csp_decode_workspace_bytes(d, max_kv_len) > CSP_STATIC_SCRATCH_BYTES) return CSP_EWORKSPACE;
    // the partials are written by the first kernel before the second reads them: nothing to clear
    return decode_common(d, q, nullptr, nullptr, const_cast<void*>(k_cache), const_cast<void*>(v_cache), cache_stride_b,
                         cache_stride_head, cache_stride_tok, 0, const_cast<int32_t*>(kv_len), max_kv_len, out, nullptr,
                         0, stream, 3, nullptr, 0, true);
}

int csp_decode_step(const csp_desc* d, const void* q, const void* k_new, const void* v_new, void* k_cache,
                    void* v_cache, int64_t cache_stride_b, int64_t cache_stride_head, int64_t cache_stride_tok,
                    int32_t cache_cap, int32_t* kv_len, float* out, void* ws, size_t ws_bytes, void* stream) {
    if (!k_new || !v_new) return CSP_EINVAL;
    return decode_common(d, q, k_new, v_new, k_cache, v_cache, cache_stride_b, cache_stride_head, cache_stride_tok,
                         cache_cap, kv_len, cache_cap, out, ws, ws_bytes, stream);
}

int csp_decode_step_window(const csp_desc* d, const void* q, const void* k_new, const void* v_new, void* k_cache,
                           void* v_cache, int64_t cache_stride_b, int64_t cache_stride_head, int64_t cache_stride_tok,
                           int32_t cache_cap, int32_t* kv_len, float* out, void* q_ring, int32_t slot, void* ws,
                           size_t ws_bytes, void* stream) {
    if (!k_new || !v_new || !q_ring) return CSP_EINVAL;
    return decode_common(d, q, k_new, v_new, k_cache, v_cache, cache_stride_b, cache_stride_head, cache_stride_tok,
                         cache_cap, kv_len, cache_cap, out, ws, ws_bytes, stream, 3, q_ring, slot);
}

int csp_decode_step_phase(const csp_desc* d, int32_t phase, const void* q, const void* k_new, const void* v_new,
                          void* k_cache, void* v_cache, int64_t cache_stride_b, int64_t cache_stride_head,
                          int64_t cache_stride_tok, int32_t cache_cap, int32_t* kv_len, float* out, void* ws,
                          size_t ws_bytes, void* stream) {
    if (!k_new || !v_new || (phase != 1 && phase != 2)) return CSP_EINVAL;
    return decode_common(d, q, k_new, v_new, k_cache, v_cache, cache_stride_b, cache_stride_head, cache_stride_tok,
                         cache_cap, kv_len, cache_cap, out, ws, ws_bytes, stream, phase);
}

int csp_append_kv(const csp_desc* d, const void* k_new, const void* v_new, void* k_cache,
                  void* v_cache, int64_t cache_stride_b, int64_t cache_stride_head,
                  int64_t cache_stride_tok, int32_t cache_cap, int32_t* kv_len, void* stream) {
    Checked c;
    int rc = check_desc(d, false, &c);
    if (rc != CSP_OK) return rc;
    if (!k_new || !v_new || !k_cache || !v_cache || !kv_len || cache_cap <= 0) return CSP_EINVAL;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache)) return CSP_EINVAL;
    if ((rc = check_kv_strides(cache_stride_tok, cache_stride_head, d->D, c.EB)) != CSP_OK) return rc;
    if (cache_stride_b < 0 || (cache_stride_b * c.EB) % 16 != 0) return CSP_EINVAL;
    AppendParams p;
    std::memset(&p, 0, sizeof(p));
    p.k_new = k_new; p.v_new = v_new; p.k_cache = k_cache; p.v_cache = v_cache; p.kv_len = kv_len;
    p.B = d->B; p.H_kv = d->H_kv; p.cache_cap = cache_cap; p.row_bytes = c.row_bytes;
    p.stride_b = cache_stride_b * c.EB; p.stride_head = cache_stride_head * c.EB; p.stride_tok = cache_stride_tok * c.EB;
    return launch_append(p, static_cast<hipStream_t>(stream)) == hipSuccess ? CSP_OK : CSP_EHIP;
}

int csp_gather_modality(const csp_desc* d, const uint8_t* modality, const int32_t* kept_idx, int32_t kept_cap,
                        const int32_t* kept_cnt, uint8_t* mod_cache, int32_t cache_cap, void* stream) {
    Checked c;
    int rc = check_desc(d, true, &c);
    if (rc != CSP_OK) return rc;
    if (!modality || !kept_idx || !kept_cnt || !mod_cache || kept_cap <= 0 || cache_cap <= 0) return CSP_EINVAL;
    ModGatherParams p;
    std::memset(&p, 0, sizeof(p));
    p.modality = modality; p.cu = d->cu_seqlens; p.kept_idx = kept_idx; p.kept_cnt = kept_cnt; p.mod_out = mod_cache;
    p.B = d->B; p.H_sel = c.H_sel; p.kept_cap = kept_cap; p.mod_cap = cache_cap;
    return launch_mod_gather(p, static_cast<hipStream_t>(stream)) == hipSuccess ? CSP_OK : CSP_EHIP;
}

int csp_window_push(const csp_desc* d, const void* q_new, void* q_ring, int32_t slot, void* stream) {
    Checked c;
    int rc = check_desc(d, false, &c);
    if (rc != CSP_OK) return rc;
    if (!q_new || !q_ring || !aligned16(q_new) || !aligned16(q_ring)) return CSP_EINVAL;
    if (d->window_O <= 0 || d->window_O > 128 || slot < 0 || slot >= d->window_O) return CSP_EINVAL;
    WindowParams p;
    std::memset(&p, 0, sizeof(p));
    p.src = q_new; p.dst = q_ring; p.rows = d->B * d->H_q; p.O = d->window_O; p.row_bytes = c.row_bytes; p.slot = slot;
    return launch_window_push(p, static_cast<hipStream_t>(stream)) == hipSuccess ? CSP_OK : CSP_EHIP;
}

namespace {
struct RepruneLayout {
    ScorePlan plan;
    size_t off_part, off_slices, total;
};
RepruneLayout reprune_layout(const csp_desc* d, int H_sel, int row_bytes, int cache_cap) {
    RepruneLayout l;
    l.plan = score_plan(d->B, d->H_q, d->H_kv, d->sel_group, cache_cap, d->dtype, d->D, d->window_O, false);
    auto up = [](size_t x) { return (x + 15) & ~(size_t)15; };
    l.off_part = up((size_t)d->B * d->H_q * d->window_O * row_bytes);                  // the window in temporal order
    l.off_slices = l.off_part + l.plan.part_bytes;
    l.total = l.off_slices + (l.plan.max_gsplit > 1 ? (size_t)2 * l.plan.max_gsplit * d->B * H_sel * cache_cap * sizeof(float) : 0);
    return l;
}
}  // namespace

size_t csp_reprune_workspace_bytes(const csp_desc* d, int32_t cache_cap) {
    if (!d || d->B <= 0 || d->H_q <= 0 || d->H_kv <= 0 || d->window_O <= 0 || cache_cap <= 0) return 0;
    if (d->sel_group <= 0 || d->H_q % d->sel_group != 0) return 0;
    const int EB = d->dtype == CSP_BF16 ? 2 : 4;
    return reprune_layout(d, d->H_q / d->sel_group, d->D * EB, cache_cap).total;
}

int csp_reprune(const csp_desc* d, const void* q_ring, int32_t ring_start, void* k_cache, void* v_cache,
                int64_t cache_stride_b, int64_t cache_stride_head, int64_t cache_stride_tok, int32_t cache_cap,
                uint8_t* mod_cache, int32_t* kv_len, float* score_self, float* score_cross, int32_t* kept_idx,
                int32_t kept_cap, int32_t* kept_cnt, void* ws, size_t ws_bytes, void* stream) {
    Checked c;
    int rc = check_desc(d, false, &c);
    if (rc != CSP_OK) return rc;
    if (!q_ring || !k_cache || !v_cache || !mod_cache || !kv_len || !score_self || !score_cross || !kept_idx || !kept_cnt)
        return CSP_EINVAL;
    if (!aligned16(q_ring) || !aligned16(k_cache) || !aligned16(v_cache)) return CSP_EINVAL;
    if (d->window_O <= 0 || d->recent_R < 0) return CSP_EINVAL;
    if (d->window_O > 128) return CSP_EUNSUPPORTED;
    if (ring_start < 0 || ring_start >= d->window_O || cache_cap <= 0 || kept_cap <= 0) return CSP_EINVAL;
    if ((rc = check_kv_strides(cache_stride_tok, cache_stride_head, d->D, c.EB)) != CSP_OK) return rc;
    if (cache_stride_b < 0 || (cache_stride_b * c.EB) % 16 != 0) return CSP_EINVAL;
    if (!d->budget_T_host || !d->budget_T) return CSP_EINVAL;
    for (int b = 0; b < d->B; ++b) {
        const int T = d->budget_T_host[b];
        if (T < d->window_O || T < d->recent_R || T > kept_cap) return CSP_EINVAL;
    }
    const RepruneLayout l = reprune_layout(d, c.H_sel, c.row_bytes, cache_cap);
    if (!ws || ws_bytes < l.total || !aligned16(ws)) return CSP_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* wsb = static_cast<char*>(ws);

    WindowParams w;
    std::memset(&w, 0, sizeof(w));
    w.src = q_ring; w.dst = wsb; w.rows = d->B * d->H_q; w.O = d->window_O; w.row_bytes = c.row_bytes; w.slot = ring_start;
    if (launch_window_unroll(w, st) != hipSuccess) return CSP_EHIP;

    SeqView view;
    std::memset(&view, 0, sizeof(view));
    view.kv_len = kv_len; view.budget_T = d->budget_T;
    view.H_kv = d->H_kv; view.H_sel = c.H_sel; view.cap = cache_cap;
    view.k_stride_batch = cache_stride_b;

    ScoreParams p;
    std::memset(&p, 0, sizeof(p));
    p.q_win = wsb; p.k = k_cache; p.modality = mod_cache;
    p.score_self = score_self; p.score_cross = score_cross;
    p.counters = reinterpret_cast<int32_t*>(wsb + l.off_part);
    p.part = reinterpret_cast<float*>(wsb + l.off_part + 16);
    p.view = view;
    p.score_elems = (int64_t)d->B * c.H_sel * cache_cap;
    p.B = d->B; p.H_q = d->H_q; p.G = c.G; p.sel_group = d->sel_group;
    p.O = d->window_O; p.R = d->recent_R; p.causal = d->causal ? 1 : 0;
    set_score_plan(p, l.plan, d, wsb + l.off_slices);
    p.k_stride_tok = cache_stride_tok; p.k_stride_head = cache_stride_head;
    p.scale_log2 = (float)(kLog2e / std::sqrt((double)d->D));
    p.n_score = (float)d->n_score;
    if (launch_score(p, d->dtype, d->D, cache_cap, st) != hipSuccess) return CSP_EHIP;

    SelectParams sp;
    std::memset(&sp, 0, sizeof(sp));
    sp.score_self = score_self; sp.score_cross = score_cross; sp.modality = mod_cache;
    sp.view = view; sp.budget_T = d->budget_T;
    sp.kept_idx = kept_idx; sp.kept_cnt = kept_cnt;
    sp.B = d->B; sp.H_sel = c.H_sel; sp.O = d->window_O; sp.R = d->recent_R; sp.kept_cap = kept_cap;
    sp.cross_ratio = d->cross_ratio;
    if (launch_select(sp, cache_cap, st) != hipSuccess) return CSP_EHIP;

    RepruneParams rp;
    std::memset(&rp, 0, sizeof(rp));
    rp.k_cache = k_cache; rp.v_cache = v_cache; rp.mod_cache = mod_cache;
    rp.kept_idx = kept_idx; rp.kept_cnt = kept_cnt; rp.budget_T = d->budget_T; rp.kv_len = kv_len;
    rp.B = d->B; rp.H_kv = d->H_kv; rp.H_sel = c.H_sel; rp.kv_per_sel = c.kv_per_sel;
    rp.kept_cap = kept_cap; rp.cache_cap = cache_cap;
    rp.stride_b = cache_stride_b * c.EB; rp.stride_head = cache_stride_head * c.EB; rp.stride_tok = cache_stride_tok * c.EB;
    return launch_reprune_move(rp, c.row_bytes, st) == hipSuccess ? CSP_OK : CSP_EHIP;
}

int csp_probe_stream(const void* src, void* dst, size_t bytes, void* sink, void* stream) {
    if (!src || !sink || bytes == 0 || bytes % 16 != 0 || !aligned16(src) || (dst && !aligned16(dst))) return CSP_EINVAL;
    return launch_probe_stream(src, dst, bytes, static_cast<uint32_t*>(sink), static_cast<hipStream_t>(stream)) == hipSuccess ? CSP_OK : CSP_EHIP;
}

}  // extern "C"
