// csp_score kernels for gfx950.
//
// What is computed (paper: Eq. "A = softmax(QK^T/sqrt d)" / Eq. "n-softmax",
// the window trim A[-O:, :-R], Eq. "cross-self"): for the last O queries of a
// sequence, attention weights over every cached key, then per-key sums over
// the query axis split by whether query and key share a modality.
//
// Design.  The per-key sums need the final softmax normaliser of every window
// row, which depends on all L keys, so the key stream is walked twice:
//   pass A (score_stats_kernel)  : S = K Q^T on MFMA with queries on the lane
//        axis, so the running (max, sum-exp) of a row lives in one lane and
//        needs no cross-lane traffic inside the loop;
//   pass B (score_colsum_kernel) : S = Q K^T with keys on the lane axis, so
//        the sum over queries of exp(S - lse) is an in-lane add chain.
// The two orientations use the same LDS tile and the same register fragments;
// only the operand order of the MFMA differs.
// A workgroup is 4 wavefronts that take the 32-key tiles of the workgroup's
// chunk round-robin; a tile is streamed with coalesced 16-byte
// global loads (4 full 256-byte rows per instruction for bf16/D=128) into a
// ring of register tiles PF tiles ahead (the loop is bound by HBM latency: the
// bytes in flight per compute unit, not the arithmetic, set the rate), a
// wave-private padded LDS tile as the transpose
// between the load layout and the MFMA operand layout, no workgroup barrier
// in the loop.  All exponentials are base 2 with log2(e)/sqrt(D) folded into
// one FMA per element.  Every memory operation in the two loops is issued on
// every path (no load or store under a branch): otherwise the compiler's wait
// counts degrade to "wait for everything" and the prefetch is lost.  Pass B
// keeps the chunk's scores in LDS and writes them in one burst at the end.
#include "csp_internal.h"

namespace csp {
namespace {

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

template <typename E, int D, int NQB, bool Q_IN_LDS>
struct Smem {
    using G = Geom<E, D>;
    static constexpr int kTiles = kWaves * G::TILE_LDS;
    static constexpr int kRed = kWaves * NQB * 32 * 8;    // float2 per (wave, query)
    static constexpr int kNlse = NQB * 32 * 4;
    static constexpr int kWq = NQB * 32;                   // uint8 modality of window rows
    static constexpr int kQ = QFrags<E, D, NQB, Q_IN_LDS>::kLdsBytes;
    static constexpr int off_red = kTiles;
    static constexpr int off_nlse = off_red + kRed;
    static constexpr int off_wq = off_nlse + kNlse;
    static constexpr int off_q = (off_wq + kWq + 15) & ~15;
    static constexpr int total = off_q + kQ;
};

// Online (max, sum-exp) update of this lane's rows with one key tile.  MASK: some keys of the
// tile are past the end of the sequence or not visible to some rows (causal tail).
template <int NQB, bool MASK>
__device__ __forceinline__ void stats_tile(f32x16 (&acc)[NQB], float c, int j0, int half, int L, int causal,
                                           const int (&pos_q)[NQB], float (&m_run)[NQB], float (&l_run)[NQB]) {
    const float NEG_INF = -__builtin_inff();
#pragma unroll
    for (int nb = 0; nb < NQB; ++nb) {
        if constexpr (MASK) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int j = j0 + acc_row(v, half);
                const bool ok = j < L && (!causal || j <= pos_q[nb]);
                acc[nb][v] = ok ? acc[nb][v] : NEG_INF;
            }
        }
        float mx0 = fmaxf(acc[nb][0], acc[nb][1]), mx1 = fmaxf(acc[nb][2], acc[nb][3]);
#pragma unroll
        for (int v = 4; v < 16; v += 4) {
            mx0 = fmaxf(mx0, fmaxf(acc[nb][v], acc[nb][v + 1]));      // v_max3
            mx1 = fmaxf(mx1, fmaxf(acc[nb][v + 2], acc[nb][v + 3]));
        }
        const float mnew = fmaxf(m_run[nb], fmaxf(mx0, mx1) * c);
        const float msafe = mnew == NEG_INF ? 0.f : mnew;
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;  // four add chains
#pragma unroll
        for (int v = 0; v < 16; v += 4) {
            s0 += fast_exp2(fmaf(acc[nb][v], c, -msafe));
            s1 += fast_exp2(fmaf(acc[nb][v + 1], c, -msafe));
            s2 += fast_exp2(fmaf(acc[nb][v + 2], c, -msafe));
            s3 += fast_exp2(fmaf(acc[nb][v + 3], c, -msafe));
        }
        l_run[nb] = l_run[nb] * fast_exp2(m_run[nb] - msafe) + ((s0 + s1) + (s2 + s3));
        m_run[nb] = mnew;
    }
}

// The 32-key tiles one wavefront of workgroup `chunk` visits: the workgroup owns keys
// [chunk*chunk_keys, (chunk+1)*chunk_keys) and its wavefronts take the tiles round-robin;
// first key of a wavefront's step: base + step*stride.
struct TileWalk {
    int ntiles, base, stride;
};
__device__ __forceinline__ TileWalk tile_walk(int L, int chunk, int chunk_keys, int wave) {
    TileWalk w;
    const int c0 = chunk * chunk_keys;
    const int ntc = c0 < L ? (min(c0 + chunk_keys, L) - c0 + kTile - 1) / kTile : 0;
    w.ntiles = ntc > wave ? (ntc - wave + kWaves - 1) / kWaves : 0;
    w.base = c0 + wave * kTile;
    w.stride = kWaves * kTile;
    return w;
}

// Workgroup -> task, XCD-aware.  Workgroups go to the 8 XCDs round-robin by their linear id, and
// each XCD has its own L2.  Tasks are numbered so that the `share` tasks that stream the same
// keys (the query heads of a GQA group, the head slices of a selection group) are consecutive;
// this puts each such run on one XCD, back to back, so the keys come from HBM once and from that
// XCD's L2 afterwards.  With share == 1 the mapping is the identity.
__device__ __forceinline__ int xcd_task(int wg, int share) {
    const int xcd = wg & 7, j = wg >> 3;
    return ((j / share) * 8 + xcd) * share + j % share;
}

// ---------------------------------------------------------------------------
// Pass A: per (sequence, query head, chunk) partial row statistics.
// ---------------------------------------------------------------------------
// REUSED: other workgroups stream the same keys (GQA): plain loads that stay in L2 instead of
// non-temporal ones.
template <typename E, int D, int NQB, bool REUSED>
__global__ __launch_bounds__(kThreads, NQB <= 2 ? CSP_SCORE_WPE_A : 1) void score_stats_kernel(ScoreParams p) {
    using G = Geom<E, D>;
    using QF = QFrags<E, D, NQB, kQaLds>;
    using SM = Smem<E, D, NQB, kQaLds>;
    extern __shared__ __align__(16) char smem[];
    // task = (query head within its GQA group, chunk, KV head, sequence), the first index fastest
    int task = xcd_task(blockIdx.x, p.G);
    if (task >= p.G * p.n_chunks * p.view.H_kv * p.B) return;
    const int g_in = task % p.G; task /= p.G;
    const int chunk = task % p.n_chunks; task /= p.n_chunks;
    const int hk = task % p.view.H_kv, b = task / p.view.H_kv;
    const int hq = hk * p.G + g_in;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    const int L = view_len(p.view, b, hk);
    if (chunk * p.chunk_keys >= L || view_fits(p.view, b, L)) return;
    const int O = p.O;
    const float c = p.scale_log2;
    const float NEG_INF = -__builtin_inff();

    char* tile = smem + wave * G::TILE_LDS;
    float2* red = reinterpret_cast<float2*>(smem + SM::off_red);
    float* q_lds = reinterpret_cast<float*>(smem + SM::off_q);

    const char* kbase = reinterpret_cast<const char*>(p.k) + (view_key0(p.view, b, p.k_stride_tok) + (int64_t)hk * p.k_stride_head) * G::EB;
    const int64_t tok_bytes = p.k_stride_tok * G::EB;

    // the four wavefronts take the chunk's 32-key tiles round-robin (wave w: tiles w, w+4, ...),
    // so a workgroup sweeps its chunk as one stream
    const TileWalk walk = tile_walk(L, chunk, p.chunk_keys, wave);
    const int ntiles = walk.ntiles;

    float m_run[NQB], l_run[NQB];
    int pos_q[NQB];  // absolute position of this lane's query in block nb
#pragma unroll
    for (int nb = 0; nb < NQB; ++nb) {
        m_run[nb] = NEG_INF;
        l_run[nb] = 0.f;
        pos_q[nb] = L - O + nb * 32 + (lane & 31);
    }
    const int mask_from = p.causal ? L - O : L;  // keys below this index are visible to every row

    // Ring of PF register tiles.  Every iteration issues exactly one tile of loads, valid or
    // not (rows past the end re-read row L-1, an L2 hit), so the number of loads in flight is
    // the same on every path and the wait before a tile is used covers that tile only.
    constexpr int PF = Prefetch<E>::A;
    u32x4 st[PF][G::NLD];
    // Tiles are visited in ascending order (the query heads of a GQA group start together on one
    // XCD and walk the same keys in the same order, so all but the first find a tile in that
    // XCD's L2).  A per-workgroup rotation of the order, once needed against channel camping with
    // many small chunks, measures no better with 512 large chunks.
    auto tile_key = [&](int t) {  // first key of the tile visited at step t (steps past the end: any valid row)
        return t < ntiles ? walk.base + t * walk.stride : L - 1;
    };
    // the key stream starts first; the queries (L2-resident, small) follow
    if (ntiles > 0) {
#pragma unroll
        for (int u = 0; u < PF; ++u) load_tile<E, D, REUSED>(st[u], kbase, tok_bytes, tile_key(u), L, lane);
    }
    QF qf;
    qf.load(reinterpret_cast<const char*>(p.q_win) + ((size_t)(b * p.H_q + hq) * O) * D * G::EB, O, tid, q_lds);
    if constexpr (QF::kLdsBytes > 0) __syncthreads();
    qf.settle();
    if (ntiles > 0) {
    for (int t0 = 0; t0 < ntiles; t0 += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int t = t0 + u;
            const int j0 = tile_key(t);
            const bool live = t < ntiles;  // uniform
            if (live) {
                wave_lds_sync();
                store_tile<E, D>(st[u], tile, lane);
                wave_lds_sync();
            }
            load_tile<E, D, REUSED>(st[u], kbase, tok_bytes, tile_key(t + PF), L, lane);
            if (!live) continue;

            f32x16 acc[NQB];
#pragma unroll
            for (int nb = 0; nb < NQB; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[nb][v] = 0.f;
#pragma unroll
            for (int s = 0; s < G::NK; ++s) {
                const auto kf = k_frag<E, D>(tile, s, lane);
#pragma unroll
                for (int nb = 0; nb < NQB; ++nb) acc[nb] = mma(kf, qf.get(nb, s, lane, q_lds), acc[nb]);
            }
            // acc[nb][v]: key j0 + acc_row(v, half), query nb*32 + lane%32
            if (j0 + kTile > mask_from) stats_tile<NQB, true>(acc, c, j0, half, L, p.causal, pos_q, m_run, l_run);
            else stats_tile<NQB, false>(acc, c, j0, half, L, p.causal, pos_q, m_run, l_run);
        }
    }
    }

    // combine the two lane halves, then the four wavefronts
#pragma unroll
    for (int nb = 0; nb < NQB; ++nb) {
        const float mo = __shfl_xor(m_run[nb], 32);
        const float lo = __shfl_xor(l_run[nb], 32);
        const float M = fmaxf(m_run[nb], mo);
        const float Ms = M == NEG_INF ? 0.f : M;
        const float Lc = l_run[nb] * fast_exp2(m_run[nb] - Ms) + lo * fast_exp2(mo - Ms);
        if (half == 0) red[wave * (NQB * 32) + nb * 32 + lane] = make_float2(M, Lc);
    }
    __syncthreads();
    if (tid < O) {
        float M = NEG_INF;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, red[w * (NQB * 32) + tid].x);
        const float Ms = M == NEG_INF ? 0.f : M;
        float Lc = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float2 r = red[w * (NQB * 32) + tid];
            Lc += r.y * fast_exp2(r.x - Ms);
        }
        float2* out = reinterpret_cast<float2*>(p.part) + ((size_t)(b * p.H_q + hq) * p.n_chunks + chunk) * O + tid;
        *out = make_float2(M, Lc);
    }
}

// Sum over the window rows held by this lane of 2^(c*acc) for one key tile.  MASK: rows may not
// see the key (causal tail) or the key is not ranked; MIXED: the window holds both modalities
// and text / visual rows are summed apart (ct / cv), otherwise everything goes to ct.
template <int NQB, bool MASK, bool MIXED>
__device__ __forceinline__ void colsum_tile(const f32x16 (&acc)[NQB], float c, const uint32_t (&text_bits)[(NQB + 1) / 2],
                                            int j, int half, int rank_end, int first_pos, int causal,
                                            float& ct, float& cv) {
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;  // four add chains
    float t0 = 0.f, t1 = 0.f;
#pragma unroll
    for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float pv = fast_exp2(acc[mb][v] * c);
            if constexpr (MASK) {
                const int i = mb * 32 + acc_row(v, half);
                const bool ok = j < rank_end && (!causal || j <= first_pos + i);
                pv = ok ? pv : 0.f;
            }
            if constexpr (MIXED) {
                const bool is_text = (text_bits[mb / 2] >> ((mb & 1) * 16 + v)) & 1u;
                if (v & 1) { t1 += is_text ? pv : 0.f; s1 += is_text ? 0.f : pv; }
                else { t0 += is_text ? pv : 0.f; s0 += is_text ? 0.f : pv; }
            } else {
                if ((v & 3) == 0) s0 += pv;
                else if ((v & 3) == 1) s1 += pv;
                else if ((v & 3) == 2) s2 += pv;
                else s3 += pv;
            }
        }
    if constexpr (MIXED) { ct = t0 + t1; cv = s0 + s1; }
    else { ct = (s0 + s1) + (s2 + s3); cv = 0.f; }
}

// ---------------------------------------------------------------------------
// Pass B: per (sequence, selection group, chunk) column sums.
// ---------------------------------------------------------------------------
template <typename E, int D, int NQB, bool REUSED>
__global__ __launch_bounds__(kThreads, NQB <= 2 ? CSP_SCORE_WPE_B : 1) void score_colsum_kernel(ScoreParams p) {
    using G = Geom<E, D>;
    using QF = QFrags<E, D, NQB, kQbLds>;
    using SM = Smem<E, D, NQB, kQbLds>;
    extern __shared__ __align__(16) char smem[];
    // a group summed by one workgroup (gsplit == 1) writes the result, otherwise each slice of
    // its heads writes its own partial array
    // task = (head slice, chunk, selection group, sequence), the first index fastest
    int task = xcd_task(blockIdx.x, p.gsplit);
    const int H_sel = p.H_q / p.sel_group;
    if (task >= p.gsplit * p.n_chunks * H_sel * p.B) return;
    const int slice = task % p.gsplit; task /= p.gsplit;
    const int chunk = task % p.n_chunks; task /= p.n_chunks;
    const int sg = task % H_sel, b = task / H_sel;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    const int L = view_len(p.view, b, (sg * p.sel_group) / p.G);
    if (chunk * p.chunk_keys >= L || view_fits(p.view, b, L)) return;
    const int O = p.O, R = p.R;
    const float c = p.scale_log2;
    const uint8_t* const mod = p.modality + view_mod0(p.view, b, sg);
    const int64_t key0 = view_key0(p.view, b, p.k_stride_tok);
    const size_t score0 = (size_t)view_score0(p.view, b, sg);
    const int g_begin = slice * p.gper, g_end = min(p.sel_group, g_begin + p.gper);
    const size_t slice_off = (size_t)slice * (size_t)p.score_elems;
    float* const out_self = p.gsplit > 1 ? p.slice_self + slice_off : p.score_self;
    float* const out_cross = p.gsplit > 1 ? p.slice_cross + slice_off : p.score_cross;
    const float NEG_INF = -__builtin_inff();
    const int n_chunks_b = (L + p.chunk_keys - 1) / p.chunk_keys;  // chunks that wrote statistics

    char* tile = smem + wave * G::TILE_LDS;
    float* nlse_s = reinterpret_cast<float*>(smem + SM::off_nlse);
    uint8_t* wq = reinterpret_cast<uint8_t*>(smem + SM::off_wq);
    float* q_lds = reinterpret_cast<float*>(smem + SM::off_q);
    float* sc_lds = reinterpret_cast<float*>(smem + SM::total);  // [2][chunk_keys]: self, cross scores of the chunk
    const int c0 = chunk * p.chunk_keys;

    // modality of the window rows; a window with one modality takes the fast path
    if (tid < NQB * 32) wq[tid] = tid < O ? (mod[L - O + tid] ? 1 : 0) : 2;
    __syncthreads();
    bool any_text = false, any_vis = false;
    for (int i = 0; i < O; ++i) {
        any_text |= wq[i] == 0;
        any_vis |= wq[i] == 1;
    }
    const bool mixed = any_text && any_vis;
    // bit (mb*16+v) set: the query of accumulator (mb, v) is a text query
    uint32_t text_bits[(NQB + 1) / 2];
#pragma unroll
    for (int w = 0; w < (NQB + 1) / 2; ++w) text_bits[w] = 0u;
#pragma unroll
    for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            if (wq[mb * 32 + acc_row(v, half)] == 0) text_bits[mb / 2] |= 1u << ((mb & 1) * 16 + v);

    // the four wavefronts take the chunk's 32-key tiles round-robin (wave w: tiles w, w+4, ...),
    // so a workgroup sweeps its chunk as one stream
    const TileWalk walk = tile_walk(L, chunk, p.chunk_keys, wave);
    const int ntiles = walk.ntiles;
    const int rank_end = L - R;                                   // keys >= rank_end are not ranked
    const int mask_from = min(rank_end, p.causal ? L - O : L);    // below: no masking needed
    const int64_t tok_bytes = p.k_stride_tok * G::EB;

    constexpr int PF = Prefetch<E>::B;
    auto tile_key = [&](int t) {  // first key of the tile visited at step t (steps past the end: any valid row)
        return t < ntiles ? walk.base + t * walk.stride : L - 1;
    };
    auto load_mod = [&](int j0) -> uint8_t {  // modality of key j0 + lane%32, fetched with its tile
        const int j = j0 + (lane & 31);
        return mod[j < L ? j : L - 1];
    };

    for (int g = g_begin; g < g_end; ++g) {
        const int hq = sg * p.sel_group + g;
        const int hk = hq / p.G;
        // the key stream starts first; the per-head set-up below overlaps with it
        const char* kbase = reinterpret_cast<const char*>(p.k) + (key0 + (int64_t)hk * p.k_stride_head) * G::EB;
        u32x4 st[PF][G::NLD];
        uint8_t kmod[PF];
        if (ntiles > 0) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                kmod[u] = load_mod(tile_key(u));  // before its tile: the oldest load is the cheapest to wait for
                load_tile<E, D, REUSED>(st[u], kbase, tok_bytes, tile_key(u), L, lane);
            }
        }
        __syncthreads();  // previous head's nlse_s / q_lds are no longer read
        if (tid < NQB * 32) {
            float nl = NEG_INF;
            if (tid < O && p.row_lse != nullptr) {
                // the caller's log-sum-exp of the scaled logits (natural log), e.g. from the prefill
                // attention kernel; the n of the n-softmax is added to the row sum here
                const float l2 = p.row_lse[(size_t)(b * p.H_q + hq) * O + tid] * 1.44269504088896340736f;
                nl = -(p.n_score > 0.f ? l2 + fast_log2(1.f + p.n_score * fast_exp2(-l2)) : l2) / c;
            } else if (tid < O) {
                const float2* part = reinterpret_cast<const float2*>(p.part) + ((size_t)(b * p.H_q + hq) * p.n_chunks) * O + tid;
                // merge of the chunk partials (max, sum): 8 independent loads at a time
                float M = NEG_INF, Ls = 0.f;
                for (int ch0 = 0; ch0 < n_chunks_b; ch0 += 8) {
                    float2 r[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        r[u] = ch0 + u < n_chunks_b ? part[(size_t)(ch0 + u) * O] : make_float2(NEG_INF, 0.f);
                    float Mn = M;
#pragma unroll
                    for (int u = 0; u < 8; ++u) Mn = fmaxf(Mn, r[u].x);
                    Ls *= fast_exp2(M - Mn);   // chunk 0 always holds a visible key, so Mn is finite
#pragma unroll
                    for (int u = 0; u < 8; ++u) Ls += r[u].y * fast_exp2(r[u].x - Mn);
                    M = Mn;
                }
                Ls += p.n_score * fast_exp2(-M);  // the n of the n-softmax, in the same scaled units
                nl = -(M + fast_log2(Ls)) / c;  // in units of the raw dot product: seeds the accumulator
            }
            nlse_s[tid] = nl;
        }
        QF qf;
        qf.load(reinterpret_cast<const char*>(p.q_win) + ((size_t)(b * p.H_q + hq) * O) * D * G::EB, O, tid, q_lds);
        __syncthreads();  // nlse_s (and staged queries) visible
        qf.settle();
        if (ntiles > 0) {
        for (int t0 = 0; t0 < ntiles; t0 += PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                const int t = t0 + u;
                const int j0 = tile_key(t);
                const bool live = t < ntiles;  // uniform
                if (live) {
                    wave_lds_sync();
                    store_tile<E, D>(st[u], tile, lane);
                    wave_lds_sync();
                }
                const bool key_text = kmod[u] == 0;
                // one tile of loads per iteration on every path (see the ring in pass A)
                kmod[u] = load_mod(tile_key(t + PF));
                load_tile<E, D, REUSED>(st[u], kbase, tok_bytes, tile_key(t + PF), L, lane);
                if (!live) continue;

                // the accumulator starts at -lse_i/c, so that 2^(c*acc) is the normalised weight
                f32x16 acc[NQB];
#pragma unroll
                for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
                    for (int v4 = 0; v4 < 4; ++v4) {
                        const float4 w = *reinterpret_cast<const float4*>(nlse_s + mb * 32 + v4 * 8 + half * 4);
                        acc[mb][v4 * 4 + 0] = w.x; acc[mb][v4 * 4 + 1] = w.y;
                        acc[mb][v4 * 4 + 2] = w.z; acc[mb][v4 * 4 + 3] = w.w;
                    }
#pragma unroll
                for (int s = 0; s < G::NK; ++s) {
                    const auto kf = k_frag<E, D>(tile, s, lane);
#pragma unroll
                    for (int mb = 0; mb < NQB; ++mb) acc[mb] = mma(qf.get(mb, s, lane, q_lds), kf, acc[mb]);
                }
                // acc[mb][v]: query mb*32 + acc_row(v, half), key j0 + lane%32
                const int j = j0 + (lane & 31);
                const bool need_mask = j0 + kTile > mask_from;
                float ct = 0.f, cv = 0.f;  // sums over text / visual window rows
                // four straight-line variants behind uniform branches (masking only touches the
                // last tiles of a sequence, a window with both modalities is rare)
                if (!need_mask) {
                    if (!mixed) colsum_tile<NQB, false, false>(acc, c, text_bits, j, half, rank_end, L - O, p.causal, ct, cv);
                    else colsum_tile<NQB, false, true>(acc, c, text_bits, j, half, rank_end, L - O, p.causal, ct, cv);
                } else {
                    if (!mixed) colsum_tile<NQB, true, false>(acc, c, text_bits, j, half, rank_end, L - O, p.causal, ct, cv);
                    else colsum_tile<NQB, true, true>(acc, c, text_bits, j, half, rank_end, L - O, p.causal, ct, cv);
                }
                ct += __shfl_xor(ct, 32);
                if (mixed) cv += __shfl_xor(cv, 32);
                else if (any_vis) { cv = ct; ct = 0.f; }  // an all-visual window: every row is a visual query
                // The chunk's scores are gathered in LDS and written in one burst when the workgroup
                // is done: small stores in the loop (128 bytes per tile and array) interleave writes
                // with the key stream and cost 15 % of the pass.  Lanes 0-31 hold the self score of
                // key j, lanes 32-63 its cross score; the same lane owns the same key for every head
                // of the group, so the running sum over heads is a private read-modify-write.
                {
                    const float s_self = key_text ? ct : cv;
                    const float s_cross = key_text ? cv : ct;
                    float* dst = sc_lds + (half ? p.chunk_keys : 0) + (j - c0);
                    float val = half ? s_cross : s_self;
                    if constexpr (REUSED) val += g > g_begin ? *dst : 0.f;
                    *dst = val;
                }
            }
        }
        }
    }
    // the chunk's scores: one coalesced burst per array
    __syncthreads();
    const int nk = min(p.chunk_keys, L - c0);
    for (int i = tid; i < nk; i += kThreads) {
        out_self[score0 + c0 + i] = sc_lds[i];
        out_cross[score0 + c0 + i] = sc_lds[p.chunk_keys + i];
    }
}

// ---------------------------------------------------------------------------
// One pass: statistics and column sums from a single read of the keys.
// ---------------------------------------------------------------------------
// A workgroup owns kFusedChunk keys and keeps their logits against the whole window in its
// accumulator registers (kFusedTiles tiles of 32 keys per wavefront).  It publishes the
// log-sum-exp of its chunk for every window row, reads the ones of the other chunks of the same
// head, and turns its registers into normalised weights: no second walk over the keys.
// The exchange uses agent-scope atomic stores and loads (write-through / read-through at the
// level the XCDs share) and no release fence, which on this part would write back a whole L2.
// Every statistic is set to NaN before the launch, so a value that reads as a number has been
// published: entries validate themselves and no ordering between different addresses is
// needed.  Workgroups start in the order of their linear id and the chunks of a head have
// consecutive ids, so the workgroups waited for are already running; the wait is bounded all the
// same, and a workgroup that gives up computes the row statistics of the whole head by itself
// (stats_whole_head), so the kernel ends whatever the scheduling.
#ifndef CSP_FUSED_TILES
#define CSP_FUSED_TILES 4
#endif
constexpr int kFusedTiles = CSP_FUSED_TILES;
constexpr int kFusedOccupancy = kFusedTiles <= 3 ? 3 : 2;  // workgroups per compute unit the registers allow
// query fragments of the one-pass kernel: LDS in operand order (1) or registers (0); with the
// chunk's logits held in 32 * kFusedTiles registers per 32 window rows, registers are the scarce side
#ifndef CSP_FUSED_Q_LDS
#define CSP_FUSED_Q_LDS 1
#endif
constexpr bool kFusedQLds = CSP_FUSED_Q_LDS != 0;
constexpr int kFusedChunk = kWaves * kTile * kFusedTiles;
#ifndef CSP_FUSED_POLL_SLEEP
#define CSP_FUSED_POLL_SLEEP 4
#endif

// LDS of the one-pass kernel.  The exchange buffers live inside the key tiles, which are dead once
// a wavefront has its logits: `red` row w in the first 512 bytes of wavefront w's own tile (a
// wavefront writes it right after its own last MFMA, while others may still read their tiles),
// the chunk's scores at the start of the tile area (written after several workgroup barriers).
template <typename E, int D, int NQB>
struct FusedSmem {
    using G = Geom<E, D>;
    static constexpr int NQ = NQB * 32;
    static constexpr int kTiles = kWaves * G::TILE_LDS;
    static constexpr int off_sc = 0;                               // float [2][kFusedChunk], aliases the tiles
    static constexpr int off_rowm = kTiles;                        // float [NQ] chunk maximum of every row
    static constexpr int off_f = off_rowm + NQ * 4;                // float [NQ] 2^(chunk maximum - lse)
    static constexpr int off_wq = off_f + NQ * 4;                  // uint8 [NQ]
    static constexpr int off_flag = off_wq + NQ;                   // int [2]: [1] = modalities present in the window
    static constexpr int off_q = (off_flag + 8 + 15) & ~15;        // queries in operand order
    static constexpr int total = off_q + QFrags<E, D, NQB, true>::kLdsBytes;
    static_assert(2 * kFusedChunk * 4 <= kTiles && 64 * 8 <= G::TILE_LDS, "exchange buffers must fit in the tiles");
    // float2 [64] of wavefront w
    __device__ static float2* red_row(char* smem, int w) { return reinterpret_cast<float2*>(smem + w * G::TILE_LDS); }
};

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

// (max, sum-exp) in log2 units of every window row over all L keys of one head, computed by
// this workgroup alone; thread i < NQ returns the statistics of row i.
template <typename E, int D, int NQB>
__device__ __forceinline__ float2 stats_whole_head(const ScoreParams& p, const char* kbase, int64_t tok_bytes, const char* qhead,
                                                int L, char* smem) {
    using G = Geom<E, D>;
    using SM = FusedSmem<E, D, NQB>;
    using QF = QFrags<E, D, NQB, true>;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    const float NEG_INF = -__builtin_inff();
    char* tile = smem + wave * G::TILE_LDS;
    float* q_lds = reinterpret_cast<float*>(smem + SM::off_q);
    QF qf;
    qf.load(qhead, p.O, tid, q_lds);
    __syncthreads();
    float m_run[NQB], l_run[NQB];
    int pos_q[NQB];
#pragma unroll
    for (int nb = 0; nb < NQB; ++nb) {
        m_run[nb] = NEG_INF;
        l_run[nb] = 0.f;
        pos_q[nb] = L - p.O + nb * 32 + (lane & 31);
    }
    for (int j0 = wave * kTile; j0 < L; j0 += kWaves * kTile) {
        u32x4 st[G::NLD];
        load_tile<E, D, false>(st, kbase, tok_bytes, j0, L, lane);
        wave_lds_sync();
        store_tile<E, D>(st, tile, lane);
        wave_lds_sync();
        f32x16 acc[NQB];
#pragma unroll
        for (int nb = 0; nb < NQB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][v] = 0.f;
#pragma unroll
        for (int s = 0; s < G::NK; ++s) {
            const auto kf = k_frag<E, D>(tile, s, lane);
#pragma unroll
            for (int nb = 0; nb < NQB; ++nb) acc[nb] = mma(kf, qf.get(nb, s, lane, q_lds), acc[nb]);
        }
        stats_tile<NQB, true>(acc, p.scale_log2, j0, half, L, p.causal, pos_q, m_run, l_run);
    }
#pragma unroll
    for (int nb = 0; nb < NQB; ++nb) {
        const float mo = __shfl_xor(m_run[nb], 32);
        const float lo = __shfl_xor(l_run[nb], 32);
        const float M = fmaxf(m_run[nb], mo);
        const float Ms = M == NEG_INF ? 0.f : M;
        const float Lc = l_run[nb] * fast_exp2(m_run[nb] - Ms) + lo * fast_exp2(mo - Ms);
        if (half == 0) SM::red_row(smem, wave)[nb * 32 + lane] = make_float2(M, Lc);
    }
    __syncthreads();
    float2 out = make_float2(NEG_INF, 0.f);
    if (tid < NQB * 32) {
        float M = NEG_INF;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) M = fmaxf(M, SM::red_row(smem, w)[tid].x);
        const float Ms = M == NEG_INF ? 0.f : M;
        float Lc = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float2 r = SM::red_row(smem, w)[tid];
            Lc += r.y * fast_exp2(r.x - Ms);
        }
        out = make_float2(M, Lc);
    }
    __syncthreads();  // the tiles are reused by the caller
    return out;
}

// Marks every (head, chunk, row) statistic as not yet published.
__global__ __launch_bounds__(256) void score_fused_clear_kernel(ScoreParams p) {
    const size_t n = (size_t)p.B * p.H_q * p.n_chunks * p.O;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p.part[i] = __builtin_nanf("");
}

template <typename E, int D, int NQB, bool REUSED>
__global__ __launch_bounds__(kThreads, kFusedOccupancy) void score_fused_kernel(ScoreParams p) {
    using G = Geom<E, D>;
    using QF = QFrags<E, D, NQB, kFusedQLds>;
    using SM = FusedSmem<E, D, NQB>;
    constexpr int NQ = NQB * 32, N = NQB * 16, NT = kFusedTiles;
    extern __shared__ __align__(16) char smem[];
    // task = (query head within its GQA group, chunk, KV head, sequence), the first index fastest:
    // the chunks of the G heads of a KV head occupy one run of G * n_chunks consecutive workgroup
    // ids (XCD-aware within it, so that the heads of a group meet in one L2)
    int task = xcd_task(blockIdx.x, p.G);
    if (task >= p.G * p.n_chunks * p.view.H_kv * p.B) return;
    const int g_in = task % p.G; task /= p.G;
    const int chunk = task % p.n_chunks; task /= p.n_chunks;
    const int hk = task % p.view.H_kv, b = task / p.view.H_kv;
    const int hq = hk * p.G + g_in;
    // selection group of the head; a group of several heads is summed from one array per head
    const int sg = hq / p.sel_group, slice = hq % p.sel_group;
    float* const out_self = p.gsplit > 1 ? p.slice_self + (size_t)slice * (size_t)p.score_elems : p.score_self;
    float* const out_cross = p.gsplit > 1 ? p.slice_cross + (size_t)slice * (size_t)p.score_elems : p.score_cross;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    const int L = view_len(p.view, b, hk);
    const int c0 = chunk * kFusedChunk;
    if (c0 >= L || view_fits(p.view, b, L)) return;
    const int O = p.O, R = p.R;
    const float c = p.scale_log2;
    const float NEG_INF = -__builtin_inff();
    const int n_chunks_b = (L + kFusedChunk - 1) / kFusedChunk;  // chunks of this sequence that publish statistics
    const int bh = b * p.H_q + hq;
    const uint8_t* const mod = p.modality + view_mod0(p.view, b, sg);
    const size_t score0 = (size_t)view_score0(p.view, b, sg);

    char* tile = smem + wave * G::TILE_LDS;
    float* rowm = reinterpret_cast<float*>(smem + SM::off_rowm);
    float* f_s = reinterpret_cast<float*>(smem + SM::off_f);
    float* sc_lds = reinterpret_cast<float*>(smem + SM::off_sc);
    uint8_t* wq = reinterpret_cast<uint8_t*>(smem + SM::off_wq);
    int* flag = reinterpret_cast<int*>(smem + SM::off_flag);

    const char* kbase = reinterpret_cast<const char*>(p.k) + (view_key0(p.view, b, p.k_stride_tok) + (int64_t)hk * p.k_stride_head) * G::EB;
    const int64_t tok_bytes = p.k_stride_tok * G::EB;
    const char* qhead = reinterpret_cast<const char*>(p.q_win) + ((size_t)bh * O) * D * G::EB;

    // wavefront w takes tiles w, w+4, w+8, w+12 of the chunk; tiles past the end of the sequence
    // re-read its last row and are masked out
    auto tile_j0 = [&](int t) { return c0 + (t * kWaves + wave) * kTile; };
#ifndef CSP_FUSED_PF
#define CSP_FUSED_PF 2
#endif
    constexpr int PF = CSP_FUSED_PF;
    u32x4 st[PF][G::NLD];
    float* q_lds = reinterpret_cast<float*>(smem + SM::off_q);
    QF qf;
    const uint8_t wq_mod = mod[L - O + (tid < O ? tid : 0)];  // modality of window row tid
    if constexpr (kFusedQLds) {
        // the queries (small, L2-resident) are requested first: loads return in order, so the
        // wait for them does not include the key tiles requested behind them
        u32x4 qw[QF::IT];
        qf.issue(qw, qhead, O, tid);
#pragma unroll
        for (int u = 0; u < PF; ++u) load_tile<E, D, REUSED>(st[u], kbase, tok_bytes, tile_j0(u), L, lane);
        qf.commit(qw, O, tid, q_lds);
        __syncthreads();
    } else {
#pragma unroll
        for (int u = 0; u < PF; ++u) load_tile<E, D, REUSED>(st[u], kbase, tok_bytes, tile_j0(u), L, lane);
        qf.load(qhead, O, tid, q_lds);
        qf.settle();
    }

    // ---- logits of the chunk: acc[t][mb][v] = q_i . k_j, i = mb*32 + acc_row(v, half), j = tile_j0(t) + lane%32
    f32x16 acc[NT][NQB];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        wave_lds_sync();
        store_tile<E, D>(st[t % PF], tile, lane);
        wave_lds_sync();
        if (t + PF < NT) load_tile<E, D, REUSED>(st[t % PF], kbase, tok_bytes, tile_j0(t + PF), L, lane);
#pragma unroll
        for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][mb][v] = 0.f;
#pragma unroll
        for (int s = 0; s < G::NK; ++s) {
            const auto kf = k_frag<E, D>(tile, s, lane);
#pragma unroll
            for (int mb = 0; mb < NQB; ++mb) acc[t][mb] = mma(qf.get(mb, s, lane, q_lds), kf, acc[t][mb]);
        }
    }
    if (tid < NQ) wq[tid] = tid < O ? (wq_mod ? 1 : 0) : 2;
    if (wave == 0) {  // does the window hold text rows, visual rows (bits 0, 1)
        const bool t = __ballot(tid < O && wq_mod == 0) != 0, v = __ballot(tid < O && wq_mod != 0) != 0;
        if (lane == 0) flag[1] = (t ? 1 : 0) | (v ? 2 : 0);
    }
    // keys past the end, and keys a row may not see (causal tail)
    if (c0 + kFusedChunk > (p.causal ? L - O : L)) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int j = tile_j0(t) + (lane & 31);
#pragma unroll
            for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int i = mb * 32 + acc_row(v, half);
                    const bool ok = j < L && (!p.causal || j <= L - O + i);
                    acc[t][mb][v] = ok ? acc[t][mb][v] : NEG_INF;
                }
        }
    }

    // ---- chunk statistics of every row: maximum, then sum of 2^(x - maximum)
    const int my_row = ((lane & (N - 1)) >> 4) * 32 + acc_row(lane & 15, half);  // row this lane ends up with after a reduce_scatter
    {
        float rm[N];
#pragma unroll
        for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float m = acc[0][mb][v];
#pragma unroll
                for (int t = 1; t < NT; ++t) m = fmaxf(m, acc[t][mb][v]);
                rm[mb * 16 + v] = m;
            }
        wave_lds_sync();  // this wavefront's last tile has been read
        SM::red_row(smem, wave)[my_row].x = reduce_scatter<N, true>(rm, lane) * c;
    }
    __syncthreads();
    if (tid < NQ) {
        float M = SM::red_row(smem, 0)[tid].x;
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, SM::red_row(smem, w)[tid].x);
        rowm[tid] = M == NEG_INF ? 0.f : M;   // a row that sees no key of the chunk: every weight is 0 anyway
    }
    __syncthreads();
    {
        float rs[N];
#pragma unroll
        for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const float4 w = *reinterpret_cast<const float4*>(rowm + mb * 32 + v4 * 8 + half * 4);
                const float ms[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int v = v4 * 4 + u;
                    float sum = 0.f;
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        acc[t][mb][v] = fast_exp2(fmaf(acc[t][mb][v], c, -ms[u]));
                        sum += acc[t][mb][v];
                    }
                    rs[mb * 16 + v] = sum;
                }
            }
        SM::red_row(smem, wave)[my_row].y = reduce_scatter<N, false>(rs, lane);
    }
    // modality of this lane's key in every tile: needed after the exchange, lands during the wait
    uint8_t kmod[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int j = tile_j0(t) + (lane & 31);
        kmod[t] = mod[j < L ? j : L - 1];
    }
    __syncthreads();
    if (tid < NQ) {
        float l = SM::red_row(smem, 0)[tid].y;
#pragma unroll
        for (int w = 1; w < kWaves; ++w) l += SM::red_row(smem, w)[tid].y;
        // log-sum-exp of the chunk (-inf when the row sees none of its keys)
        const float lse_c = l > 0.f ? rowm[tid] + fast_log2(l) : NEG_INF;
        if (tid < O) __hip_atomic_store(p.part + ((size_t)bh * p.n_chunks + chunk) * O + tid, lse_c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // ---- exchange: the log-sum-exps of all chunks of the head.  Every entry was set to NaN before
    // the launch, so an entry that reads as a number has been published; entries still NaN are read
    // again.  Thread (row = tid % 64, quarter = tid / 64) takes every fourth chunk, all its loads in
    // flight at once; then the four quarters are combined.
    float M = NEG_INF, Ls = 0.f;
    bool have_all = p.spin_ticks > 0;  // uniform
    if (have_all) {
        const uint64_t t_start = wall_clock64();
        const int row = tid & 63, quarter = tid >> 6;
        const float* part = p.part + ((size_t)bh * p.n_chunks) * O + (row < O ? row : 0);
        for (int cb = 0; cb < n_chunks_b && have_all; cb += 4 * 12) {
            float r[12];
            for (;;) {
                bool pending = false;
#pragma unroll
                for (int u = 0; u < 12; ++u) {
                    const int ch = cb + quarter + 4 * u;
                    r[u] = ch < n_chunks_b ? __hip_atomic_load(part + (size_t)ch * O, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : NEG_INF;
                    pending |= r[u] != r[u];
                }
                if (!__syncthreads_or(pending)) break;
                // bounded: a workgroup that has waited too long stops depending on the others
                if (__syncthreads_or(tid == 0 && wall_clock64() - t_start > (uint64_t)p.spin_ticks)) { have_all = false; break; }
                __builtin_amdgcn_s_sleep(CSP_FUSED_POLL_SLEEP);
            }
            if (!have_all) break;
            float Mn = M;
#pragma unroll
            for (int u = 0; u < 12; ++u) Mn = fmaxf(Mn, r[u]);
            const float Mns = Mn == NEG_INF ? 0.f : Mn;
            Ls *= fast_exp2(M - Mns);
#pragma unroll
            for (int u = 0; u < 12; ++u) Ls += fast_exp2(r[u] - Mns);
            M = Mn;
        }
    }
    if (have_all) {
        SM::red_row(smem, tid >> 6)[tid & 63] = make_float2(M, Ls);
        __syncthreads();
        M = NEG_INF; Ls = 0.f;
        if (tid < NQ) {
#pragma unroll
            for (int w = 0; w < kWaves; ++w) M = fmaxf(M, SM::red_row(smem, w)[tid].x);   // chunk 0 holds a visible key: finite
#pragma unroll
            for (int w = 0; w < kWaves; ++w) Ls += SM::red_row(smem, w)[tid].y * fast_exp2(SM::red_row(smem, w)[tid].x - M);
        }
    } else {
        const float2 whole = stats_whole_head<E, D, NQB>(p, kbase, tok_bytes, qhead, L, smem);
        M = whole.x; Ls = whole.y;
    }
    if (tid < NQ) {
        float f = 0.f;
        if (tid < O) {
            Ls += p.n_score * fast_exp2(-M);  // the n of the n-softmax, in the same scaled units
            f = fast_exp2(rowm[tid] - (M + fast_log2(Ls)));
        }
        f_s[tid] = f;
    }
    __syncthreads();

    // ---- column sums: weight = 2^(x - chunk maximum) * f_i
    const bool any_text = (flag[1] & 1) != 0, any_vis = (flag[1] & 2) != 0;
    const bool mixed = any_text && any_vis;
    float f[NQB][16];
#pragma unroll
    for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            const float4 w = *reinterpret_cast<const float4*>(f_s + mb * 32 + v4 * 8 + half * 4);
            f[mb][v4 * 4 + 0] = w.x; f[mb][v4 * 4 + 1] = w.y; f[mb][v4 * 4 + 2] = w.z; f[mb][v4 * 4 + 3] = w.w;
        }
    // bit (mb*16 + v) set: the query of accumulator (mb, v) is a text query (used by mixed windows)
    uint32_t text_bits = 0u;
    if (mixed) {
#pragma unroll
        for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (wq[mb * 32 + acc_row(v, half)] == 0) text_bits |= 1u << (mb * 16 + v);
    }
    const int rank_end = L - R;  // keys >= rank_end are not ranked
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        float ct = 0.f, cv = 0.f;  // sums over text / visual window rows
        if (!mixed) {
            float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
            for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; v += 4) {
                    s0 = fmaf(acc[t][mb][v], f[mb][v], s0);
                    s1 = fmaf(acc[t][mb][v + 1], f[mb][v + 1], s1);
                    s2 = fmaf(acc[t][mb][v + 2], f[mb][v + 2], s2);
                    s3 = fmaf(acc[t][mb][v + 3], f[mb][v + 3], s3);
                }
            ct = (s0 + s1) + (s2 + s3);
        } else {
            float t0 = 0.f, t1 = 0.f, v0 = 0.f, v1 = 0.f;
#pragma unroll
            for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const bool is_text = (text_bits >> (mb * 16 + v)) & 1u;
                    const float pv = acc[t][mb][v] * f[mb][v];
                    if (v & 1) { t1 += is_text ? pv : 0.f; v1 += is_text ? 0.f : pv; }
                    else { t0 += is_text ? pv : 0.f; v0 += is_text ? 0.f : pv; }
                }
            ct = t0 + t1; cv = v0 + v1;
        }
        ct += __shfl_xor(ct, 32);
        if (mixed) cv += __shfl_xor(cv, 32);
        else if (any_vis) { cv = ct; ct = 0.f; }  // an all-visual window: every row is a visual query
        const int j = tile_j0(t) + (lane & 31);
        const bool key_text = kmod[t] == 0;
        const float s_self = key_text ? ct : cv;
        const float s_cross = key_text ? cv : ct;
        // lanes 0-31 hold the self score of key j, lanes 32-63 its cross score
        sc_lds[(half ? kFusedChunk : 0) + (j - c0)] = j < rank_end ? (half ? s_cross : s_self) : 0.f;
    }
    __syncthreads();
    const int nk = min(kFusedChunk, L - c0);
    for (int i = tid; i < nk; i += kThreads) {
        out_self[score0 + c0 + i] = sc_lds[i];
        out_cross[score0 + c0 + i] = sc_lds[kFusedChunk + i];
    }
}

// Sum of the per-slice arrays of a split selection group, slices in ascending order
// (a fixed order: the result does not depend on scheduling).
__global__ __launch_bounds__(256) void score_slice_sum_kernel(ScoreParams p) {
    const size_t n = (size_t)p.score_elems;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const float* src = blockIdx.y == 0 ? p.slice_self : p.slice_cross;
    float acc = __builtin_nontemporal_load(src + i);
    for (int sl = 1; sl < p.gsplit; ++sl) acc += __builtin_nontemporal_load(src + (size_t)sl * n + i);
    (blockIdx.y == 0 ? p.score_self : p.score_cross)[i] = acc;
}

template <typename E, int D, int NQB>
hipError_t launch_fused(const ScoreParams& p, hipStream_t s) {
    if constexpr (NQB <= 2 && elem_bytes<E>::value == 2) {
        // the query heads of a GQA group stream the same keys at the same time: plain loads that stay in L2
        auto k = p.G > 1 ? score_fused_kernel<E, D, NQB, true> : score_fused_kernel<E, D, NQB, false>;
        const int64_t tasks = (int64_t)p.n_chunks * p.H_q * p.B;
        const unsigned grid = (unsigned)((tasks + 8 * p.G - 1) / (8 * p.G) * (8 * p.G));
        const size_t n_stats = (size_t)p.B * p.H_q * p.n_chunks * p.O;
        hipLaunchKernelGGL(score_fused_clear_kernel, dim3((unsigned)((n_stats + 255) / 256)), dim3(256), 0, s, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        const size_t smem = FusedSmem<E, D, NQB>::total;
        hipLaunchKernelGGL(k, dim3(grid), dim3(kThreads), smem, s, p);
        e = hipGetLastError();
        if (e != hipSuccess || p.gsplit == 1) return e;
        const size_t n = (size_t)p.score_elems;
        hipLaunchKernelGGL(score_slice_sum_kernel, dim3((unsigned)((n + 255) / 256), 2), dim3(256), 0, s, p);
        return hipGetLastError();
    } else {
        return hipErrorInvalidValue;  // excluded by score_plan
    }
}

template <typename E, int D, int NQB>
hipError_t launch_typed(const ScoreParams& p, hipStream_t s) {
    if (p.fused) return launch_fused<E, D, NQB>(p, s);
    const size_t smem_a = Smem<E, D, NQB, kQaLds>::total, smem_b = Smem<E, D, NQB, kQbLds>::total + (size_t)2 * p.chunk_keys * sizeof(float);
    // keys that several workgroups (GQA) or several head iterations of one workgroup stream stay in L2
    auto ka = p.G > 1 ? score_stats_kernel<E, D, NQB, true> : score_stats_kernel<E, D, NQB, false>;
    auto kb = (p.G > 1 || p.gper > 1) ? score_colsum_kernel<E, D, NQB, true> : score_colsum_kernel<E, D, NQB, false>;
    if (smem_a > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(ka), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_a);
        if (e != hipSuccess) return e;
    }
    if (smem_b > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kb), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_b);
        if (e != hipSuccess) return e;
    }
    if (smem_b > 160 * 1024) return hipErrorInvalidValue;  // excluded by score_chunk_keys
    const dim3 block(kThreads);
    auto padded = [](int64_t tasks, int share) { return (unsigned)((tasks + 8 * share - 1) / (8 * share) * (8 * share)); };
    const dim3 grid_a(padded((int64_t)p.n_chunks * p.H_q * p.B, p.G));
    const dim3 grid_b(padded((int64_t)p.n_chunks * (p.H_q / p.sel_group) * p.gsplit * p.B, p.gsplit));
    hipError_t e = hipSuccess;
    if (p.row_lse == nullptr) {  // the row normalisers are not given: first pass over the keys
        hipLaunchKernelGGL(ka, grid_a, block, smem_a, s, p);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kb, grid_b, block, smem_b, s, p);
    e = hipGetLastError();
    if (e != hipSuccess || p.gsplit == 1) return e;
    const size_t n = (size_t)p.score_elems;
    hipLaunchKernelGGL(score_slice_sum_kernel, dim3((unsigned)((n + 255) / 256), 2), dim3(256), 0, s, p);
    return hipGetLastError();
}

template <typename E, int D>
hipError_t launch_nqb(const ScoreParams& p, hipStream_t s) {
    if (p.O <= 32) return launch_typed<E, D, 1>(p, s);
    if (p.O <= 64) return launch_typed<E, D, 2>(p, s);
    return launch_typed<E, D, 4>(p, s);
}

}  // namespace

#ifndef CSP_SCORE_MIN_TASKS
#define CSP_SCORE_MIN_TASKS 512
#endif
int score_chunk_keys(int B, int H_q, int max_seqlen, int dtype, int D, int O) {
    // largest chunk that still gives every compute unit two workgroups (one resident set, no
    // second round with a ragged tail): long chunks amortise the per-head set-up of a workgroup
#ifndef CSP_SCORE_MAX_CHUNK
#define CSP_SCORE_MAX_CHUNK 4096
#endif
    int ck = CSP_SCORE_MAX_CHUNK;
    // the column-sum pass keeps the chunk's scores in LDS (8 bytes per key) next to its key tiles
    // and staged queries; fp32 with D = 128 and a window above 64 rows leaves room for 2048 keys
    if (dtype == CSP_F32 && D == 128 && O > 64 && ck > 2048) ck = 2048;
    while (ck > 128 && (int64_t)B * H_q * ((max_seqlen + ck - 1) / ck) < CSP_SCORE_MIN_TASKS) ck >>= 1;
    return ck;
}

int score_heads_per_slice(int B, int H_q, int sel_group, int n_chunks) {
    // one workgroup sums a whole group while that still leaves two workgroups per compute unit;
    // larger groups are cut into equal slices
    const int64_t groups = (int64_t)B * (H_q / sel_group) * n_chunks;
    int gper = sel_group;
    while (gper > 1 && groups * ((sel_group + gper - 1) / gper) < CSP_SCORE_MIN_TASKS) gper = (gper + 1) / 2;
    return gper;
}

#ifndef CSP_SCORE_FUSED
#define CSP_SCORE_FUSED 1
#endif
ScorePlan score_plan(int B, int H_q, int H_kv, int sel_group, int max_seqlen, int dtype, int D, int O, bool have_row_lse) {
    ScorePlan pl;
    auto up = [](size_t x) { return (x + 15) & ~(size_t)15; };
    // two passes over the keys
    const int ck = score_chunk_keys(B, H_q, max_seqlen, dtype, D, O);
    const int nc = (max_seqlen + ck - 1) / ck;
    const size_t two_pass = up((size_t)B * H_q * nc * O * 2 * sizeof(float));
    // one pass: a log-sum-exp per (head, chunk, row)
    const int nf = (max_seqlen + kFusedChunk - 1) / kFusedChunk;
    const size_t one_pass = up((size_t)B * H_q * nf * O * sizeof(float));
    // A workgroup of the one-pass kernel waits for the other chunks of its head.  Workgroups start in
    // id order and the chunks of the heads of one KV head occupy G * nf consecutive ids, so the ones
    // waited for are running as long as such a run fits the share of the resident set (512
    // workgroups on the whole chip) that the launch gets, also beside a second launch on another
    // stream: a quarter of it is allowed; longer sequences take the two-pass kernels.
    const int G = H_kv > 0 ? H_q / H_kv : 1;
    const bool can_fuse = CSP_SCORE_FUSED != 0 && dtype == CSP_BF16 && O <= 64 && (int64_t)G * nf <= 128;
    pl.part_bytes = can_fuse && one_pass > two_pass ? one_pass : two_pass;   // csp_score_lse shares the size
    pl.fused = can_fuse && !have_row_lse;
    pl.chunk_keys = pl.fused ? kFusedChunk : ck;
    pl.n_chunks = pl.fused ? nf : nc;
    // one pass: every head writes its own array and the heads of a group are added in order
    pl.gper = pl.fused ? 1 : score_heads_per_slice(B, H_q, sel_group, pl.n_chunks);
    pl.gsplit = (sel_group + pl.gper - 1) / pl.gper;
    // slice arrays sized for whichever path needs more of them
    pl.max_gsplit = pl.gsplit;
    if (can_fuse && sel_group > pl.max_gsplit) pl.max_gsplit = sel_group;
    return pl;
}

hipError_t launch_score(const ScoreParams& p, int dtype, int D, int /*max_seqlen*/, hipStream_t s) {
    if (dtype == CSP_BF16) return D == 128 ? launch_nqb<bf16_tag, 128>(p, s) : launch_nqb<bf16_tag, 64>(p, s);
    return D == 128 ? launch_nqb<f32_tag, 128>(p, s) : launch_nqb<f32_tag, 64>(p, s);
}

}  // namespace csp
