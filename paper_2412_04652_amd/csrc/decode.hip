// csp_decode_attn kernels for gfx950.
//
// What is computed (paper: Eq. "n-softmax"): for one new query per head,
//   p_t = e^{s_t} / (n + sum_u e^{s_u}),  s_t = q.k_t/sqrt(D),  out = sum_t p_t v_t
// over the pruned cache.
//
// Design.  One flop per byte: bound by HBM, so the kernel is a stream of the K
// and V slabs.  The key axis of each (sequence, KV head) is split over
// workgroups (split-KV); a workgroup's 8 wavefronts walk their slice with
// 16-byte loads, LPR consecutive lanes owning one row (a wavefront instruction
// reads 64/LPR whole rows), UNROLL rows in flight per lane group.  The dot
// product is an in-lane FMA chain over the lane's 16-byte slice of D plus a
// butterfly over the LPR lanes; the same lanes then own the same slice of V and
// of the output, so P.V needs no data exchange.  Online softmax in base 2 with
// log2(e)/sqrt(D) folded into q.  All query heads of a GQA group are served
// from one pass over the shared K/V rows.  Partials (max, sum, unnormalised
// out) go to a workspace; a small second kernel merges the splits and adds the
// n of the n-softmax exactly once, scaled by 2^-max like every other term.
#include "csp_internal.h"

namespace csp {
namespace {

#ifndef CSP_DECODE_WAVES
#define CSP_DECODE_WAVES 8
#endif
constexpr int kDecWaves = CSP_DECODE_WAVES;
constexpr int kDecThreads = kDecWaves * 64;
#ifndef CSP_DECODE_UNROLL
#define CSP_DECODE_UNROLL 4
#endif
constexpr int kDecUnroll = CSP_DECODE_UNROLL;

template <typename E> struct Unpack;
template <> struct Unpack<bf16_tag> {
    static constexpr int EPL = 8;
    __device__ static __forceinline__ void run(const u32x4& w, float (&f)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[2 * i] = bf16_lo(w[i]); f[2 * i + 1] = bf16_hi(w[i]); }
    }
};
template <> struct Unpack<f32_tag> {
    static constexpr int EPL = 4;
    __device__ static __forceinline__ void run(const u32x4& w, float (&f)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(w[i]);
    }
};

template <typename E, int D, int GT>
__global__ __launch_bounds__(kDecThreads) void decode_split_kernel(DecodeParams p) {
    constexpr int EB = elem_bytes<E>::value;
    constexpr int EPL = Unpack<E>::EPL;          // elements of D per lane
    constexpr int LPR = D / EPL;                 // lanes per row
    constexpr int RPW = kWave / LPR;             // rows per wavefront instruction
    constexpr int KPI = RPW * kDecUnroll;        // keys per wavefront iteration
    constexpr int PSTRIDE = D + 2;
    __shared__ float red[kDecWaves][GT][PSTRIDE];

    const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPR, sl = lane % LPR;  // row within the instruction, slice of D
    int kv_len = p.kv_len[b * p.H_kv + hk];
    kv_len = kv_len < 0 ? 0 : (kv_len > p.max_kv_len ? p.max_kv_len : kv_len);  // stay inside the slab
    // Fused append: the new token's k, v are row `new_row` of the stream; the lanes that meet
    // it read it from k_new / v_new and also store it into the cache (kv_len itself is bumped
    // by the merge kernel, after every workgroup of this launch has read it).
    const int new_row = (p.k_new != nullptr && kv_len < p.cache_cap && kv_len < p.max_kv_len) ? kv_len : -1;
    if (new_row >= 0) kv_len += 1;
    // The splits of one (sequence, KV head) interleave: workgroup `split` takes the key blocks
    // split, split + n_splits, ... of 4*KPI keys, so the workgroups of a head sweep its K and V
    // slabs together (fewer, wider streams for the memory system than one slice per workgroup).
    const int s0 = (split * kDecWaves + wave) * KPI;
    const int s1 = kv_len;
    const int t_step = p.n_splits * kDecWaves * KPI;
    const float NEG_INF = -__builtin_inff();

    char* kb = reinterpret_cast<char*>(p.k_cache) + (int64_t)b * p.stride_b + (int64_t)hk * p.stride_head + sl * 16;
    char* vb = reinterpret_cast<char*>(p.v_cache) + (int64_t)b * p.stride_b + (int64_t)hk * p.stride_head + sl * 16;
    const char* kn = reinterpret_cast<const char*>(p.k_new) + ((size_t)(b * p.H_kv + hk) * D) * EB + sl * 16;
    const char* vn = reinterpret_cast<const char*>(p.v_new) + ((size_t)(b * p.H_kv + hk) * D) * EB + sl * 16;

    for (int g0 = 0; g0 < p.G; g0 += GT) {
        float q[GT][EPL], o[GT][EPL], m[GT], l[GT];
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            m[g] = NEG_INF;
            l[g] = 0.f;
            const int hq = hk * p.G + g0 + g;
            u32x4 w = {0u, 0u, 0u, 0u};
            if (g0 + g < p.G) w = *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(p.q) + ((size_t)(b * p.H_q + hq) * D) * EB + sl * 16);
            // the step's query goes into the window ring on the way (one workgroup per head does it)
            if (p.q_ring != nullptr && split == 0 && wave == 0 && sub == 0 && g0 + g < p.G)
                *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(p.q_ring) +
                                          (((size_t)(b * p.H_q + hq) * p.ring_O + p.ring_slot) * D) * EB + sl * 16) = w;
            Unpack<E>::run(w, q[g]);
#pragma unroll
            for (int e = 0; e < EPL; ++e) { q[g][e] *= p.scale_log2; o[g][e] = 0.f; }
        }
        for (int t0 = s0; t0 < s1; t0 += t_step) {
            u32x4 kw[kDecUnroll], vw[kDecUnroll];
            bool ok[kDecUnroll];
#pragma unroll
            for (int u = 0; u < kDecUnroll; ++u) {
                const int t = t0 + u * RPW + sub;
                ok[u] = t < s1;
                const int tc = ok[u] ? t : s1 - 1;
                const bool is_new = tc == new_row;
                kw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(is_new ? kn : kb + (int64_t)tc * p.stride_tok));
                vw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(is_new ? vn : vb + (int64_t)tc * p.stride_tok));
                if (is_new && ok[u] && g0 == 0) {  // exactly one lane group of one workgroup meets the new row
                    *reinterpret_cast<u32x4*>(kb + (int64_t)tc * p.stride_tok) = kw[u];
                    *reinterpret_cast<u32x4*>(vb + (int64_t)tc * p.stride_tok) = vw[u];
                }
            }
            float s[GT][kDecUnroll];
#pragma unroll
            for (int u = 0; u < kDecUnroll; ++u) {
                float kf[EPL];
                Unpack<E>::run(kw[u], kf);
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    float d = 0.f;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) d = fmaf(q[g][e], kf[e], d);
#pragma unroll
                    for (int x = 1; x < LPR; x <<= 1) d += __shfl_xor(d, x);
                    s[g][u] = ok[u] ? d : NEG_INF;
                }
            }
            float vf[kDecUnroll][EPL];
#pragma unroll
            for (int u = 0; u < kDecUnroll; ++u) Unpack<E>::run(vw[u], vf[u]);
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                float mx = s[g][0];
#pragma unroll
                for (int u = 1; u < kDecUnroll; ++u) mx = fmaxf(mx, s[g][u]);
                const float mnew = fmaxf(m[g], mx);
                const float msafe = mnew == NEG_INF ? 0.f : mnew;
                const float alpha = fast_exp2(m[g] - msafe);
                float pu[kDecUnroll], ps = 0.f;
#pragma unroll
                for (int u = 0; u < kDecUnroll; ++u) { pu[u] = fast_exp2(s[g][u] - msafe); ps += pu[u]; }
                l[g] = l[g] * alpha + ps;
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    float acc = o[g][e] * alpha;
#pragma unroll
                    for (int u = 0; u < kDecUnroll; ++u) acc = fmaf(pu[u], vf[u][e], acc);
                    o[g][e] = acc;
                }
                m[g] = mnew;
            }
        }
        // merge the lane groups of the wavefront (each saw different rows, same slice of D)
#pragma unroll
        for (int g = 0; g < GT; ++g) {
#pragma unroll
            for (int x = LPR; x < kWave; x <<= 1) {
                const float mo = __shfl_xor(m[g], x);
                const float lo = __shfl_xor(l[g], x);
                const float M = fmaxf(m[g], mo);
                const float Ms = M == NEG_INF ? 0.f : M;
                const float a = fast_exp2(m[g] - Ms), bsc = fast_exp2(mo - Ms);
                l[g] = l[g] * a + lo * bsc;
#pragma unroll
                for (int e = 0; e < EPL; ++e) o[g][e] = o[g][e] * a + __shfl_xor(o[g][e], x) * bsc;
                m[g] = M;
            }
            if (sub == 0) {
#pragma unroll
                for (int e = 0; e < EPL; ++e) red[wave][g][sl * EPL + e] = o[g][e];
                if (sl == 0) { red[wave][g][D] = m[g]; red[wave][g][D + 1] = l[g]; }
            }
        }
        __syncthreads();
        // merge the wavefronts; thread d owns output dimension d
        for (int idx = tid; idx < GT * D; idx += kDecThreads) {
            const int g = idx / D, d = idx % D;
            if (g0 + g >= p.G) continue;
            float M = NEG_INF;
#pragma unroll
            for (int w = 0; w < kDecWaves; ++w) M = fmaxf(M, red[w][g][D]);
            const float Ms = M == NEG_INF ? 0.f : M;
            float od = 0.f, ls = 0.f;
#pragma unroll
            for (int w = 0; w < kDecWaves; ++w) {
                const float sc = fast_exp2(red[w][g][D] - Ms);
                od += red[w][g][d] * sc;
                ls += red[w][g][D + 1] * sc;
            }
            const int hq = hk * p.G + g0 + g;
            float* part = p.part + ((size_t)(b * p.H_q + hq) * p.n_splits + split) * PSTRIDE;
            part[d] = od;
            if (d == 0) { part[D] = M; part[D + 1] = ls; }
        }
        __syncthreads();
    }
}

// Merge of the splits and the n of the n-softmax: one workgroup per query head.
template <int D>
__global__ __launch_bounds__(D) void decode_merge_kernel(DecodeParams p) {
    constexpr int PSTRIDE = D + 2;
    const int hq = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    const float* part = p.part + ((size_t)(b * p.H_q + hq) * p.n_splits) * PSTRIDE;
    const float NEG_INF = -__builtin_inff();
    // everything this thread needs is requested up front (one memory round trip per four splits)
    const bool bump = p.k_new != nullptr && d == 0 && hq % p.G == 0;
    const int hk = hq / p.G;
    const int len = bump ? p.kv_len[b * p.H_kv + hk] : 0;
    float M = NEG_INF, od = 0.f, ls = 0.f;
    for (int s0 = 0; s0 < p.n_splits; s0 += 4) {
        float m[4], l[4], o[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool valid = s0 + u < p.n_splits;
            const float* ps = part + (size_t)(valid ? s0 + u : s0) * PSTRIDE;
            m[u] = ps[D];
            l[u] = ps[D + 1];
            o[u] = ps[d];
            if (!valid) m[u] = NEG_INF;
        }
        const float Mn = fmaxf(fmaxf(fmaxf(m[0], m[1]), fmaxf(m[2], m[3])), M);
        if (Mn == NEG_INF) continue;      // empty splits only so far
        const float keep = fast_exp2(M - Mn);  // 0 while M is still -inf
        od *= keep;
        ls *= keep;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float sc = fast_exp2(m[u] - Mn);  // 0 for an empty or missing split
            od = fmaf(o[u], sc, od);
            ls = fmaf(l[u], sc, ls);
        }
        M = Mn;
    }
    float outv = 0.f;
    if (M != NEG_INF) {
        // n + sum_u e^{s_u}, both scaled by e^{-max}: n enters once, here
        ls += p.n_decode * fast_exp2(-M);
        outv = od / ls;
    }
    p.out[(size_t)(b * p.H_q + hq) * D + d] = outv;
    // the fused append becomes visible to the next call
    if (bump && len >= 0 && len < p.cache_cap && len < p.max_kv_len) p.kv_len[b * p.H_kv + hk] = len + 1;
}

template <typename E, int D, int GT>
hipError_t launch_gt(const DecodeParams& p, hipStream_t s) {
    if (p.phases & 1) {
        hipLaunchKernelGGL((decode_split_kernel<E, D, GT>), dim3(p.n_splits, p.H_kv, p.B), dim3(kDecThreads), 0, s, p);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (p.phases & 2) hipLaunchKernelGGL((decode_merge_kernel<D>), dim3(p.H_q, p.B), dim3(D), 0, s, p);
    return hipGetLastError();
}

template <typename E, int D>
hipError_t launch_g(const DecodeParams& p, hipStream_t s) {
    if (p.G == 1) return launch_gt<E, D, 1>(p, s);
    if (p.G == 2) return launch_gt<E, D, 2>(p, s);
    if (p.G <= 4) return launch_gt<E, D, 4>(p, s);
    return launch_gt<E, D, 8>(p, s);
}

}  // namespace

// Splits per (sequence, KV head): enough for one 8-wavefront workgroup per compute unit, i.e.
// about two wavefronts per SIMD in all.  Measured on 4 x 32 heads x 8192 rows: 83 us per call at
// that count, 84 with twice as many 4-wavefront workgroups, 88-97 with four to eight times as
// many waves in flight (more concurrent streams than the memory system likes), 97-102 with one
// workgroup per head (half the compute units idle).
#ifndef CSP_DECODE_TARGET_WGS
#define CSP_DECODE_TARGET_WGS 256
#endif
int decode_num_splits(int B, int H_kv, int max_kv_len) {
    const int64_t heads = (int64_t)B * H_kv;
    int n = (int)((CSP_DECODE_TARGET_WGS + heads - 1) / heads);
    const int by_len = max_kv_len / 256;
    if (n > by_len) n = by_len;
    if (n > 64) n = 64;
    if (n < 1) n = 1;
    return n;
}

hipError_t launch_decode(const DecodeParams& p, int dtype, int D, hipStream_t s) {
    if (dtype == CSP_BF16) return D == 128 ? launch_g<bf16_tag, 128>(p, s) : launch_g<bf16_tag, 64>(p, s);
    return D == 128 ? launch_g<f32_tag, 128>(p, s) : launch_g<f32_tag, 64>(p, s);
}

}  // namespace csp
