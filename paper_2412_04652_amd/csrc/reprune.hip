// Kernels around re-pruning the grown cache during decoding (paper: the loop of
// Algorithm 1, which checks the cache length against the budget T at every
// generation step and prunes again with the current window).
//
// The scoring and selection kernels are the ones of the first pruning pass,
// reading the cache through the "cache form" of their sequence view.  Here:
//  - the modality flag of every kept key, gathered next to the pruned cache
//    (keys appended while decoding are text: flag 0), because each selection
//    group keeps different keys;
//  - the in-place compaction of K and V: kept positions ascend and are unique,
//    so row r moves down from idx[r] >= r.  One workgroup owns one (sequence,
//    KV head, K or V) and walks it in blocks of rows: all rows of a block are
//    read into registers, the workgroup meets at a barrier, then the block is
//    written.  Sources of later blocks lie above everything written so far, so
//    one barrier per block is enough;
//  - the ring of the last O queries: a slot write per decode step and the copy
//    that puts the ring in temporal order for the scoring pass.
#include "csp_internal.h"

namespace csp {
namespace {

constexpr int kMvThreads = 1024;
constexpr int kMvUnroll = 4;

// every lane's loads have landed in registers when this returns
__device__ __forceinline__ void wait_for(const u32x4& v) { asm volatile("" ::"v"(v)); }

template <int CPR>
__global__ __launch_bounds__(kMvThreads) void reprune_move_kernel(RepruneParams p) {
    constexpr int ROWS = kMvThreads / CPR;  // rows per step
    const int h = blockIdx.x, b = blockIdx.y;
    const bool is_v = blockIdx.z & 1;
    const int sg = h / p.kv_per_sel;
    int L = p.kv_len[b * p.H_kv + h];
    L = L < 0 ? 0 : (L > p.cache_cap ? p.cache_cap : L);
    if (L <= p.budget_T[b]) return;  // the cache fits its budget: nothing moves
    int n = p.kept_cnt[((size_t)b * p.H_sel + sg) * 4];
    n = n < 0 ? 0 : (n > p.kept_cap ? p.kept_cap : n);
    n = n > L ? L : n;
    const int32_t* idx = p.kept_idx + ((size_t)b * p.H_sel + sg) * p.kept_cap;
    char* base = reinterpret_cast<char*>(is_v ? p.v_cache : p.k_cache) + (int64_t)b * p.stride_b + (int64_t)h * p.stride_head;
    const int r = threadIdx.x / CPR, ch = threadIdx.x % CPR;
    for (int t0 = 0; t0 < n; t0 += ROWS * kMvUnroll) {  // uniform trip count: every wavefront reaches every barrier
        u32x4 val[kMvUnroll];
        bool mv[kMvUnroll];
        int j[kMvUnroll];
#pragma unroll
        for (int u = 0; u < kMvUnroll; ++u) {  // all index loads first, then all row loads
            const int tt = t0 + u * ROWS + r;
            j[u] = tt < n ? idx[tt] : -1;
        }
#pragma unroll
        for (int u = 0; u < kMvUnroll; ++u) {
            const int tt = t0 + u * ROWS + r;
            mv[u] = j[u] > tt && j[u] < L;  // j == tt: the row is already in place; anything else is not a valid source
            // unconditional load (row 0 when there is nothing to move) keeps the four loads in flight together
            val[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (int64_t)(mv[u] ? j[u] : 0) * p.stride_tok + ch * 16));
        }
#pragma unroll
        for (int u = 0; u < kMvUnroll; ++u) wait_for(val[u]);
        __syncthreads();
#pragma unroll
        for (int u = 0; u < kMvUnroll; ++u)
            if (mv[u]) __builtin_nontemporal_store(val[u], reinterpret_cast<u32x4*>(base + (int64_t)(t0 + u * ROWS + r) * p.stride_tok + ch * 16));
    }
}

// Modality flags of the kept keys moved down the same way, the freed tail cleared, and the
// live length of every KV head of the group set to the kept count.  Runs after the K/V move
// (which still reads the old length).
__global__ __launch_bounds__(kMvThreads) void reprune_finish_kernel(RepruneParams p) {
    const int sg = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int hk0 = sg * p.kv_per_sel;
    int L = p.kv_len[b * p.H_kv + hk0];
    L = L < 0 ? 0 : (L > p.cache_cap ? p.cache_cap : L);
    if (L <= p.budget_T[b]) return;
    int n = p.kept_cnt[((size_t)b * p.H_sel + sg) * 4];
    n = n < 0 ? 0 : (n > p.kept_cap ? p.kept_cap : n);
    n = n > L ? L : n;
    const int32_t* idx = p.kept_idx + ((size_t)b * p.H_sel + sg) * p.kept_cap;
    uint8_t* mod = p.mod_cache + ((size_t)b * p.H_sel + sg) * p.cache_cap;
    for (int t0 = 0; t0 < n; t0 += kMvThreads) {
        const int tt = t0 + tid;
        uint32_t m = 0u;
        bool mv = false;
        if (tt < n) {
            const int j = idx[tt];
            mv = j > tt && j < L;
            if (mv) m = mod[j];
        }
        asm volatile("" ::"v"(m));
        __syncthreads();
        if (mv) mod[tt] = (uint8_t)m;
    }
    __syncthreads();
    for (int tt = n + tid; tt < L; tt += kMvThreads) mod[tt] = 0;  // rows that later appends fill: text
    if (tid < p.kv_per_sel) p.kv_len[b * p.H_kv + hk0 + tid] = n;
}

// csp_compact's companion: modality of the kept keys of the packed sequence, zero beyond them
__global__ __launch_bounds__(256) void mod_gather_kernel(ModGatherParams p) {
    const int sg = blockIdx.y, b = blockIdx.z;
    const int tt = blockIdx.x * 256 + threadIdx.x;
    if (tt >= p.mod_cap) return;
    int n = p.kept_cnt[((size_t)b * p.H_sel + sg) * 4];
    n = n < 0 ? 0 : (n > p.kept_cap ? p.kept_cap : n);
    const int seq0 = p.cu[b], L = p.cu[b + 1] - seq0;
    uint8_t m = 0;
    if (tt < n) {
        const int j = p.kept_idx[((size_t)b * p.H_sel + sg) * p.kept_cap + tt];
        if (j >= 0 && j < L) m = p.modality[seq0 + j] ? 1 : 0;
    }
    p.mod_out[((size_t)b * p.H_sel + sg) * p.mod_cap + tt] = m;
}

// one 16-byte piece per thread; ring and window are [rows][O][row_bytes]
__global__ __launch_bounds__(256) void window_push_kernel(WindowParams p) {
    const int pieces = p.row_bytes / 16;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)p.rows * pieces) return;
    const int64_t row = i / pieces;
    const int c = (int)(i % pieces);
    const u32x4 w = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(p.src) + row * p.row_bytes + c * 16);
    *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(p.dst) + (row * p.O + p.slot) * p.row_bytes + c * 16) = w;
}

__global__ __launch_bounds__(256) void window_unroll_kernel(WindowParams p) {
    const int pieces = p.row_bytes / 16;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)p.rows * p.O * pieces) return;
    const int c = (int)(i % pieces);
    const int64_t ro = i / pieces;
    const int o = (int)(ro % p.O);
    const int64_t row = ro / p.O;
    int so = o + p.slot;
    so = so >= p.O ? so - p.O : so;
    const u32x4 w = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(p.src) + (row * p.O + so) * p.row_bytes + c * 16);
    *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(p.dst) + (row * p.O + o) * p.row_bytes + c * 16) = w;
}

template <int CPR>
hipError_t launch_move_cpr(const RepruneParams& p, hipStream_t s) {
    hipLaunchKernelGGL(reprune_move_kernel<CPR>, dim3(p.H_kv, p.B, 2), dim3(kMvThreads), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(reprune_finish_kernel, dim3(p.H_sel, p.B), dim3(kMvThreads), 0, s, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_reprune_move(const RepruneParams& p, int row_bytes, hipStream_t s) {
    switch (row_bytes / 16) {
        case 8: return launch_move_cpr<8>(p, s);
        case 16: return launch_move_cpr<16>(p, s);
        case 32: return launch_move_cpr<32>(p, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_mod_gather(const ModGatherParams& p, hipStream_t s) {
    hipLaunchKernelGGL(mod_gather_kernel, dim3((p.mod_cap + 255) / 256, p.H_sel, p.B), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_window_push(const WindowParams& p, hipStream_t s) {
    const int64_t n = (int64_t)p.rows * (p.row_bytes / 16);
    hipLaunchKernelGGL(window_push_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_window_unroll(const WindowParams& p, hipStream_t s) {
    const int64_t n = (int64_t)p.rows * p.O * (p.row_bytes / 16);
    hipLaunchKernelGGL(window_unroll_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace csp
