// csp_score kernels for gfx950.
//
// What is computed (paper: Eq. "A = softmax(QK^T/sqrt d)" / Eq. "n-softmax",
// the window trim A[-O:, :-R], Eq. "cross-self"): for the last O queries of a
// sequence, attention weights over every cached key, then per-key sums over
// the query axis split by whether query and key share a modality.
//
// This file: the two-pass kernels (fp32 inputs, parts of the window beyond what
// the single-read kernel takes, sequences too long for its resident set; the
// second pass alone when the caller supplies the rows' normalisers), the ordered
// sum of per-head score arrays of a selection group, the sizing rules
// (score_plan) and launch_score, which hands every bf16 case that fits to the
// single-read kernel of score_single.hip.
//
// Design of the two passes.  The per-key sums need the final softmax normaliser
// of every window row, which depends on all L keys, so the key stream is walked
// twice:
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
#include "score_tiles.h"

namespace csp {
using namespace score_detail;
namespace {

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
    if (blockIdx.x == 0 && threadIdx.x < 4) p.counters[threadIdx.x] = 0;   // no task of these kernels ever waits
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
    if (p.row_lse != nullptr && blockIdx.x == 0 && threadIdx.x < 4) p.counters[threadIdx.x] = 0;   // the only kernel of csp_score_lse
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

// Sum of the per-slice arrays of a split selection group, slices in ascending order
// (a fixed order: the result does not depend on scheduling).  Cache form: only what the scoring
// kernels wrote is read and written (positions below the live length of sequences that are pruned).
__global__ __launch_bounds__(256) void score_slice_sum_kernel(ScoreParams p) {
    const size_t n = (size_t)p.score_elems;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    if (p.view.kv_len != nullptr) {
        const int j = (int)(i % (size_t)p.view.cap);
        const int bs = (int)(i / (size_t)p.view.cap), b = bs / p.view.H_sel, sg = bs % p.view.H_sel;
        const int L = view_len(p.view, b, (sg * p.sel_group) / p.G);
        if (j >= L || view_fits(p.view, b, L)) return;
    }
    const float* src = blockIdx.y == 0 ? p.slice_self : p.slice_cross;
    float acc = __builtin_nontemporal_load(src + i);
    for (int sl = 1; sl < p.gsplit; ++sl) acc += __builtin_nontemporal_load(src + (size_t)sl * n + i);
    (blockIdx.y == 0 ? p.score_self : p.score_cross)[i] = acc;
}

template <typename E, int D, int NQB>
hipError_t launch_typed(const ScoreParams& p, hipStream_t s) {
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

#ifndef CSP_SCORE_SINGLE
#define CSP_SCORE_SINGLE 1
#endif
ScorePlan score_plan(int B, int H_q, int H_kv, int sel_group, int max_seqlen, int dtype, int D, int O, bool have_row_lse) {
    ScorePlan pl;
    auto up = [](size_t x) { return (x + 15) & ~(size_t)15; };
    // two passes over the keys
    pl.chunk_keys = score_chunk_keys(B, H_q, max_seqlen, dtype, D, O);
    pl.n_chunks = (max_seqlen + pl.chunk_keys - 1) / pl.chunk_keys;
    pl.gper = score_heads_per_slice(B, H_q, sel_group, pl.n_chunks);
    pl.gsplit = (sel_group + pl.gper - 1) / pl.gper;
    const size_t two_pass = up((size_t)B * H_q * pl.n_chunks * O * 2 * sizeof(float));
    // one read: a log-sum-exp per (head, part of the window rows, 512-key chunk, row).  The chunks
    // of the query heads of one KV head (times the parts of the window) must be at most one
    // pipeline step apart: one per compute unit (256) at most; longer sequences take the two passes
    // (the launch checks again against the device it runs on).
    const int G = H_kv > 0 ? H_q / H_kv : 1;
    pl.vsplit = O > 64 ? 2 : 1;
    pl.single_chunks = (max_seqlen + kScoreSingleChunk - 1) / kScoreSingleChunk;
    pl.single_gsplit = sel_group * pl.vsplit;
    const int64_t tasks = (int64_t)B * H_q * pl.vsplit * pl.single_chunks;
    const bool can = CSP_SCORE_SINGLE != 0 && dtype == CSP_BF16 && O <= 128 && (int64_t)G * pl.vsplit * pl.single_chunks <= 256 &&
                     tasks <= (int64_t)256 * kScoreSingleMaxIters;
    // ... and a 64-byte record per task (ids padded to a multiple of 8 * G * parts, plus one)
    const int64_t share8 = (int64_t)8 * G * pl.vsplit;
    // ... and the keys' modality as bits, a word per 32 keys, per (sequence, selection group)
    const size_t one_pass = up((size_t)B * H_q * pl.vsplit * pl.single_chunks * 64 * sizeof(float)) +
                            (size_t)((tasks + share8 - 1) / share8 * share8 + 1) * kScoreSingleRecBytes +
                            ((size_t)B * (H_q / sel_group) * pl.single_chunks * 16 + 2) * sizeof(uint32_t);
    pl.single = can && !have_row_lse;
    // csp_score_lse shares the size; 16 bytes of counters in front
    pl.part_bytes = 16 + (can && one_pass > two_pass ? one_pass : two_pass);
    // slice arrays sized for whichever path needs more of them
    pl.max_gsplit = pl.gsplit;
    if (can && pl.single_gsplit > pl.max_gsplit) pl.max_gsplit = pl.single_gsplit;
    return pl;
}

hipError_t launch_score(const ScoreParams& p_in, int dtype, int D, int /*max_seqlen*/, hipStream_t s) {
    ScoreParams p = p_in;
    if (p.single) {
        // one read of the keys; a shape that does not fit the device after all falls through to the two passes
        ScoreParams q = p;
        q.n_chunks = q.single_chunks;
        q.chunk_keys = kScoreSingleChunk;
        q.gper = 1;
        q.gsplit = q.sel_group * q.vsplit;
        q.slice_self = q.slice_base;
        q.slice_cross = q.slice_base + (size_t)q.gsplit * (size_t)q.score_elems;
        const hipError_t e = launch_score_single(q, D, s);
        if (e == hipSuccess && q.gsplit > 1) {
            const size_t n = (size_t)q.score_elems;
            hipLaunchKernelGGL(score_slice_sum_kernel, dim3((unsigned)((n + 255) / 256), 2), dim3(256), 0, s, q);
            return hipGetLastError();
        }
        if (e != hipErrorNotReady) return e;
    }
    p.single = 0;
    p.slice_self = p.slice_base;
    p.slice_cross = p.slice_base + (size_t)p.gsplit * (size_t)p.score_elems;
    if (dtype == CSP_BF16) return D == 128 ? launch_nqb<bf16_tag, 128>(p, s) : launch_nqb<bf16_tag, 64>(p, s);
    return D == 128 ? launch_nqb<f32_tag, 128>(p, s) : launch_nqb<f32_tag, 64>(p, s);
}

}  // namespace csp
