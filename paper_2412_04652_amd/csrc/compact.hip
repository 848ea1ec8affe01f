// csp_compact and csp_append_kv kernels for gfx950.
//
// What is computed (paper: cache construction "K = (K.M) (+) K[-R:]", and the
// KV-cache append of "Preliminary"): a bit copy of the kept rows of K and V
// into the pruned cache, in the ascending order csp_select produced.
//
// Design.  Pure data movement, bound by HBM.  A row is D elements (128..512
// bytes) moved as 16-byte pieces: CPR consecutive lanes own one row, so a
// wavefront instruction moves 64/CPR whole rows and every access is a full
// 16-byte-per-lane coalesced segment.  Each thread keeps UNROLL independent
// loads in flight before the first store.  K and V are copied by the same
// workgroup (blockIdx.z selects which) so the index list is read once per
// tensor from L2.
#include "csp_internal.h"

namespace csp {
namespace {

constexpr int kCpThreads = 256;
constexpr int kUnroll = 4;

template <int CPR>
__global__ __launch_bounds__(kCpThreads) void compact_kernel(CompactParams p) {
    constexpr int ROWS = kCpThreads / CPR;         // rows per workgroup per step
    constexpr int ROWS_PER_WG = ROWS * kUnroll;
    const int h = blockIdx.y;
    const int b = blockIdx.z >> 1;
    const bool is_v = blockIdx.z & 1;
    const int sg = h / p.kv_per_sel;
    int n = p.kept_cnt[((size_t)b * p.H_sel + sg) * 4];
    n = n < 0 ? 0 : (n > p.kept_cap ? p.kept_cap : n);  // never trust a count beyond the list's capacity
    const int t0 = blockIdx.x * ROWS_PER_WG;
    if (blockIdx.x == 0 && threadIdx.x == 0 && !is_v && p.kv_len) p.kv_len[b * p.H_kv + h] = n;
    if (t0 >= n) return;
    const int32_t* idx = p.kept_idx + ((size_t)b * p.H_sel + sg) * p.kept_cap;
    const int seq0 = p.cu[b];
    const int L = p.cu[b + 1] - seq0;
    const int64_t s_tok = is_v ? p.v_stride_tok : p.k_stride_tok;
    const int64_t s_head = is_v ? p.v_stride_head : p.k_stride_head;
    const char* src = reinterpret_cast<const char*>(is_v ? p.v : p.k) + (int64_t)seq0 * s_tok + (int64_t)h * s_head;
    char* dst = reinterpret_cast<char*>(is_v ? p.v_out : p.k_out) + (int64_t)b * p.out_stride_b + (int64_t)h * p.out_stride_head;
    const int r = threadIdx.x / CPR, ch = threadIdx.x % CPR;
    u32x4 val[kUnroll];
    int tt[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        tt[u] = t0 + u * ROWS + r;
        if (tt[u] < n) {
            const int j = idx[tt[u]];
            if (j < 0 || j >= L) { tt[u] = n; continue; }  // not a position of this sequence: skip the row
            val[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + (int64_t)j * s_tok + ch * 16));
        }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
        if (tt[u] < n)
            __builtin_nontemporal_store(val[u], reinterpret_cast<u32x4*>(dst + (int64_t)tt[u] * p.out_stride_tok + ch * 16));
}

__global__ __launch_bounds__(256) void append_kernel(AppendParams p) {
    const int h = blockIdx.x, b = blockIdx.y;
    const int len = p.kv_len[b * p.H_kv + h];
    if (len < 0 || len >= p.cache_cap) return;
    const int chunks = p.row_bytes / 16;
    const int64_t row = (int64_t)b * p.stride_b + (int64_t)h * p.stride_head + (int64_t)len * p.stride_tok;
    const size_t src = ((size_t)b * p.H_kv + h) * p.row_bytes;
    for (int c = threadIdx.x; c < 2 * chunks; c += blockDim.x) {
        const bool is_v = c >= chunks;
        const int cc = is_v ? c - chunks : c;
        const u32x4 w = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(is_v ? p.v_new : p.k_new) + src + cc * 16);
        *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(is_v ? p.v_cache : p.k_cache) + row + cc * 16) = w;
    }
    __syncthreads();
    if (threadIdx.x == 0) p.kv_len[b * p.H_kv + h] = len + 1;
}

template <int CPR>
hipError_t launch_cpr(const CompactParams& p, hipStream_t s) {
    constexpr int ROWS_PER_WG = (kCpThreads / CPR) * kUnroll;
    const dim3 grid((p.kept_cap + ROWS_PER_WG - 1) / ROWS_PER_WG, p.H_kv, p.B * 2);
    hipLaunchKernelGGL(compact_kernel<CPR>, grid, dim3(kCpThreads), 0, s, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_compact(const CompactParams& p, int row_bytes, hipStream_t s) {
    switch (row_bytes / 16) {
        case 8: return launch_cpr<8>(p, s);
        case 16: return launch_cpr<16>(p, s);
        case 32: return launch_cpr<32>(p, s);
        default: return hipErrorInvalidValue;
    }
}

// ---- measurement aid: the rate at which this device streams a buffer --------------------------
// Every lane reads 16 bytes at a time (non-temporal), 4 reads in flight, a few resident workgroups per
// compute unit take 16 KiB blocks of the buffer round-robin; the data is copied to dst, or, with
// dst == nullptr, folded into one word per workgroup (so that the reads are not optimised away) that
// is written to sink.
namespace {
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
// Launch shape as measured on MI355X (2 GiB): 4-wavefront workgroups, 4 loads of 16 bytes in flight
// per lane; 2 workgroups per compute unit read fastest (7.3 TB/s; 1 x 8 wavefronts 7.2, 4 x 4: 7.1,
// 8 x 4: 6.7, 2 loads in flight: 6.3), 4 per compute unit copy fastest (5.6 TB/s read + write;
// 2 x 4: 5.4, 1 x 8: 5.2).
constexpr int kProbeThreads = 256, kProbeUnroll = 4;
constexpr int kProbePerCuRead = 2, kProbePerCuCopy = 4;
// A workgroup takes blocks of kProbeThreads * kProbeUnroll * 16 bytes round-robin; within a block
// load u of lane l is piece u * kProbeThreads + l (every instruction of a wavefront reads 1 KiB of
// consecutive bytes).
__global__ __launch_bounds__(kProbeThreads) void probe_stream_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst, size_t n16, uint32_t* sink) {
    constexpr size_t kBlock = (size_t)kProbeThreads * kProbeUnroll;
    uint32_t acc = 0;
    const size_t n_full = n16 / kBlock;
    for (size_t blk = blockIdx.x; blk < n_full; blk += gridDim.x) {
        const size_t i = blk * kBlock + threadIdx.x;
        u32x4_t a[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) a[u] = __builtin_nontemporal_load(src + i + u * kProbeThreads);
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            if (dst) __builtin_nontemporal_store(a[u], dst + i + u * kProbeThreads);
            else acc ^= a[u].x ^ a[u].y ^ a[u].z ^ a[u].w;
        }
    }
    for (size_t i = n_full * kBlock + (size_t)blockIdx.x * kProbeThreads + threadIdx.x; i < n16; i += (size_t)gridDim.x * kProbeThreads) {
        const u32x4_t a = __builtin_nontemporal_load(src + i);
        if (dst) __builtin_nontemporal_store(a, dst + i);
        else acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (!dst) {
        for (int d = 32; d > 0; d >>= 1) acc ^= __shfl_xor(acc, d);
        if ((threadIdx.x & 63) == 0) atomicXor(sink + blockIdx.x % 1024, acc);
    }
}
}  // namespace

hipError_t launch_probe_stream(const void* src, void* dst, size_t bytes, uint32_t* sink, hipStream_t s) {
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    hipLaunchKernelGGL(probe_stream_kernel, dim3((unsigned)(cus * (dst ? kProbePerCuCopy : kProbePerCuRead))), dim3(kProbeThreads), 0, s,
                       reinterpret_cast<const u32x4_t*>(src), reinterpret_cast<u32x4_t*>(dst), bytes / 16, sink);
    return hipGetLastError();
}

hipError_t launch_append(const AppendParams& p, hipStream_t s) {
    hipLaunchKernelGGL(append_kernel, dim3(p.H_kv, p.B), dim3(64), 0, s, p);
    return hipGetLastError();
}

}  // namespace csp
