// Device helpers shared by the csp_score kernels (gfx950): tile geometry, the MFMA wrappers,
// query fragments, global -> register -> LDS moves of a 32-key tile, the workgroup -> task
// mapping and the wavefront reduce-scatter.
#pragma once

#include "csp_internal.h"

namespace csp {
namespace score_detail {

#ifndef CSP_SCORE_WAVES
#define CSP_SCORE_WAVES 4
#endif
constexpr int kWaves = CSP_SCORE_WAVES;
constexpr int kThreads = 64 * kWaves;
constexpr int kTile = 32;  // keys per wavefront tile (one MFMA block edge)

// Prefetch depth (tiles in flight per wavefront) of the two passes for 2-byte elements.
#ifndef CSP_SCORE_PF_A
#define CSP_SCORE_PF_A 1
#endif
#ifndef CSP_SCORE_PF_B
#define CSP_SCORE_PF_B 1
#endif
// Pass B query fragments: registers (0) or LDS in operand order (1, frees 32*NQB registers
// at the price of 16 KiB of LDS reads per tile).
#ifndef CSP_SCORE_QB_LDS
#define CSP_SCORE_QB_LDS 0
#endif
constexpr bool kQbLds = CSP_SCORE_QB_LDS != 0;
#ifndef CSP_SCORE_QA_LDS
#define CSP_SCORE_QA_LDS 0
#endif
constexpr bool kQaLds = CSP_SCORE_QA_LDS != 0;
// wavefronts per SIMD the two passes are compiled for (register budget = 512 / this)
#ifndef CSP_SCORE_WPE_A
#define CSP_SCORE_WPE_A 2
#endif
#ifndef CSP_SCORE_WPE_B
#define CSP_SCORE_WPE_B 2
#endif
template <typename E> struct Prefetch;
template <> struct Prefetch<bf16_tag> { static constexpr int A = CSP_SCORE_PF_A, B = CSP_SCORE_PF_B; };
template <> struct Prefetch<f32_tag> { static constexpr int A = 1, B = 1; };  // 4-byte rows: 64 registers per tile

template <typename E, int D>
struct Geom {
    static constexpr int EB = elem_bytes<E>::value;
    static constexpr int ROW_BYTES = D * EB;
    static constexpr int ROW_STRIDE = ROW_BYTES + 16;  // +16 B: conflict-free 16-byte LDS reads down a column
    static constexpr int CPR = ROW_BYTES / 16;         // 16-byte chunks per row
    static constexpr int RPI = kWave / CPR;            // rows covered by one wavefront load instruction
    static constexpr int NLD = kTile / RPI;            // load instructions per tile
    static constexpr int KSTEP = (EB == 2) ? 16 : 2;   // contraction depth of one MFMA
    static constexpr int NK = D / KSTEP;
    static constexpr int TILE_LDS = kTile * ROW_STRIDE;
    static constexpr int QSTRIDE = D + 4;              // floats; fp32 queries staged in LDS
};

__device__ __forceinline__ f32x16 mma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mma(float a, float b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Orders LDS writes of some lanes before LDS reads of other lanes of the same
// wavefront (the tile is wave-private, so no workgroup barrier is needed).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- query fragments --------------------------------------------------------
// MFMA operand layout (32 x KSTEP block): lane = (r = lane%32, half = lane/32)
// holds row r, contraction elements [s*KSTEP + half*KSTEP/2, +KSTEP/2).
// IN_LDS = false: fragments live in registers (bf16 only).  IN_LDS = true: staged once per
// head in LDS by the whole workgroup (caller barriers) and fetched per MFMA.
template <typename E, int D, int NQB, bool IN_LDS>
struct QFrags;

template <int D, int NQB>
struct QFrags<bf16_tag, D, NQB, false> {
    bf16x8 f[NQB][D / 16];
    // qhead: [O][D] bf16 of one head.  Rows >= O read as zero.
    __device__ __forceinline__ void load(const char* qhead, int O, int tid, float* /*q_lds*/) {
        const int lane = tid & 63, r = lane & 31, half = lane >> 5;
#pragma unroll
        for (int nb = 0; nb < NQB; ++nb)
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
                const int row = nb * 32 + r;
                u32x4 w = {0u, 0u, 0u, 0u};
                if (row < O) w = *reinterpret_cast<const u32x4*>(qhead + ((size_t)row * D + s * 16 + half * 8) * 2);
                f[nb][s] = __builtin_bit_cast(bf16x8, w);
            }
    }
    __device__ __forceinline__ bf16x8 get(int nb, int s, int /*lane*/, const float* /*q_lds*/) const { return f[nb][s]; }
    // The fragments have landed when this returns.  Called before the tile loop: loads still
    // pending at the loop's entry make the compiler wait for everything (the prefetched tiles
    // too) at the fragments' first use, on every iteration.
    __device__ __forceinline__ void settle() const {
#pragma unroll
        for (int nb = 0; nb < NQB; ++nb)
#pragma unroll
            for (int s = 0; s < D / 16; ++s) asm volatile("" ::"v"(f[nb][s]));
    }
    static constexpr int kLdsBytes = 0;
};

// bf16 queries in LDS, already in operand order: fragment (nb, s) of lane l is the 16 bytes at
// ((nb*NK + s)*64 + l)*16, so a wavefront fetch is one contiguous, conflict-free 1 KiB read.
template <int D, int NQB>
struct QFrags<bf16_tag, D, NQB, true> {
    static constexpr int NK = D / 16;
    static constexpr int N = NQB * NK * 64;                      // 16-byte pieces in all
    static constexpr int IT = (N + kThreads - 1) / kThreads;     // ... per thread
    // Staging in two steps, so that a caller can put other loads between them: issue() starts
    // the global loads into w, commit() writes them to LDS (the caller barriers afterwards).
    // Every lane loads (rows past the window re-read its last row and are zeroed in commit):
    // a load under a branch makes the compiler wait for every load in flight.
    __device__ __forceinline__ void issue(u32x4 (&w)[IT], const char* qhead, int O, int tid) const {
#pragma unroll
        for (int k = 0; k < IT; ++k) {
            const int e = min(tid + k * kThreads, N - 1);
            const int l = e & 63, s = (e >> 6) % NK, nb = e / (64 * NK);
            const int row = nb * 32 + (l & 31);
            w[k] = *reinterpret_cast<const u32x4*>(qhead + ((size_t)min(row, O - 1) * D + s * 16 + (l >> 5) * 8) * 2);
        }
    }
    __device__ __forceinline__ void commit(const u32x4 (&w)[IT], int O, int tid, float* q_lds) const {
#pragma unroll
        for (int k = 0; k < IT; ++k) {
            const int e = tid + k * kThreads;
            const int row = (e / (64 * NK)) * 32 + (e & 31);
            if (e < N) reinterpret_cast<u32x4*>(q_lds)[e] = row < O ? w[k] : u32x4{0u, 0u, 0u, 0u};
        }
    }
    __device__ __forceinline__ void load(const char* qhead, int O, int tid, float* q_lds) {
        u32x4 w[IT];
        issue(w, qhead, O, tid);
        commit(w, O, tid, q_lds);
    }
    __device__ __forceinline__ bf16x8 get(int nb, int s, int lane, const float* q_lds) const {
        return reinterpret_cast<const bf16x8*>(q_lds)[(nb * NK + s) * 64 + lane];
    }
    __device__ __forceinline__ void settle() const {}
    static constexpr int kLdsBytes = NQB * NK * 64 * 16;
};

template <int D, int NQB, bool IN_LDS>
struct QFrags<f32_tag, D, NQB, IN_LDS> {
    // fp32 queries are always staged in LDS (row-major, padded rows).
    __device__ __forceinline__ void load(const char* qhead, int O, int tid, float* q_lds) {
        constexpr int C4 = D / 4;
        for (int idx = tid; idx < NQB * 32 * C4; idx += kThreads) {
            const int row = idx / C4, c4 = idx % C4;
            float4 w = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < O) w = *reinterpret_cast<const float4*>(qhead + ((size_t)row * D + c4 * 4) * 4);
            *reinterpret_cast<float4*>(q_lds + row * Geom<f32_tag, D>::QSTRIDE + c4 * 4) = w;
        }
    }
    __device__ __forceinline__ float get(int nb, int s, int lane, const float* q_lds) const {
        return q_lds[(nb * 32 + (lane & 31)) * Geom<f32_tag, D>::QSTRIDE + s * 2 + (lane >> 5)];
    }
    __device__ __forceinline__ void settle() const {}
    static constexpr int kLdsBytes = NQB * 32 * Geom<f32_tag, D>::QSTRIDE * 4;
};

template <typename E, int D>
__device__ __forceinline__ auto k_frag(const char* tile, int s, int lane) {
    using G = Geom<E, D>;
    const int r = lane & 31, half = lane >> 5;
    if constexpr (G::EB == 2) {
        return *reinterpret_cast<const bf16x8*>(tile + r * G::ROW_STRIDE + s * 32 + half * 16);
    } else {
        return *reinterpret_cast<const float*>(tile + r * G::ROW_STRIDE + (s * 2 + half) * 4);
    }
}

// Global -> registers: tile rows j0 .. j0+31 of one (sequence, KV head); rows
// past the end of the sequence re-read row L-1 (masked by the caller).
template <typename E, int D, bool REUSED>
__device__ __forceinline__ void load_tile(u32x4 (&st)[(Geom<E, D>::NLD)], const char* kbase, int64_t tok_bytes,
                                          int j0, int L, int lane) {
    using G = Geom<E, D>;
    if constexpr (!REUSED) {
#pragma unroll
        for (int i = 0; i < G::NLD; ++i) {
            int j = j0 + i * G::RPI + lane / G::CPR;
            j = j < L ? j : L - 1;
            // streamed once per pass: non-temporal, measurably faster than plain loads here
            st[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kbase + (int64_t)j * tok_bytes + (lane % G::CPR) * 16));
        }
    } else {
        // other workgroups on this XCD stream the same keys at the same time: keep them in L2
#pragma unroll
        for (int i = 0; i < G::NLD; ++i) {
            int j = j0 + i * G::RPI + lane / G::CPR;
            j = j < L ? j : L - 1;
            st[i] = *reinterpret_cast<const u32x4*>(kbase + (int64_t)j * tok_bytes + (lane % G::CPR) * 16);
        }
    }
}

template <typename E, int D>
__device__ __forceinline__ void store_tile(const u32x4 (&st)[(Geom<E, D>::NLD)], char* tile, int lane) {
    using G = Geom<E, D>;
#pragma unroll
    for (int i = 0; i < G::NLD; ++i)
        *reinterpret_cast<u32x4*>(tile + (i * G::RPI + lane / G::CPR) * G::ROW_STRIDE + (lane % G::CPR) * 16) = st[i];
}

// key / query index of accumulator register v of a 32x32 MFMA result for the
// register-indexed axis (the other axis is lane%32)
__device__ __forceinline__ int acc_row(int v, int half) { return (v >> 2) * 8 + half * 4 + (v & 3); }

// Workgroup -> task, XCD-aware.  Workgroups go to the 8 XCDs round-robin by their linear id, and
// each XCD has its own L2.  Tasks are numbered so that the `share` tasks that stream the same
// keys (the query heads of a GQA group, the head slices of a selection group) are consecutive;
// this puts each such run on one XCD, back to back, so the keys come from HBM once and from that
// XCD's L2 afterwards.  With share == 1 the mapping is the identity.
__device__ __forceinline__ int xcd_task(int wg, int share) {
    const int xcd = wg & 7, j = wg >> 3;
    return ((j / share) * 8 + xcd) * share + j % share;
}

// x[r], r < N, holds this lane's value for register index r; on return lane l holds the
// reduction over the 32 lanes of its half for r = l % N (N == 16: lanes l and l^16 both).
template <int N, int W, bool MAX>
__device__ __forceinline__ void reduce_scatter_step(float (&x)[N], int lane) {
    // lanes l and l^W split values 0..2W-1 between them: the lane with bit W set keeps the upper W
    const bool up = (lane & W) != 0;
#pragma unroll
    for (int k = 0; k < W; ++k) {
        const float send = up ? x[k] : x[k + W];
        const float keep = up ? x[k + W] : x[k];
        const float recv = __shfl_xor(send, W);
        x[k] = MAX ? fmaxf(keep, recv) : keep + recv;
    }
    if constexpr (W > 1) reduce_scatter_step<N, W / 2, MAX>(x, lane);
}
template <int N, bool MAX>
__device__ __forceinline__ float reduce_scatter(float (&x)[N], int lane) {
    reduce_scatter_step<N, N / 2, MAX>(x, lane);
    float r = x[0];
    if constexpr (N == 16) {
        const float o = __shfl_xor(r, 16);
        r = MAX ? fmaxf(r, o) : r + o;
    }
    return r;
}

}  // namespace score_detail
}  // namespace csp
