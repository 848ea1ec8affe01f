// csp_select kernel for gfx950.
//
// What is computed (paper: the budget T of "Preliminary", Eq. "top-K" per
// region, the combination of the two masks read as a union, the recent keys of
// the cache-construction equation, Algorithm 1's early-out): per sequence and
// selection group, the sorted list of kept positions.
//
// Design.  One 1024-thread workgroup per (sequence, selection group).  Scores
// are non-negative floats, so their bit patterns order like unsigned integers:
// an MSB-first radix select (11 + 11 + 10 bits, LDS histograms for both
// regions at once) finds, per region, the bit pattern of the K-th largest score
// and how many keys equal to it still fit.  A final ordered sweep turns
// "greater than the threshold, or equal and among the first few equals" into
// keep flags and scatters the kept positions with a ballot/popcount prefix
// scan, which yields ascending indices and the lower-index-first tie rule
// without atomics on the output.
#include "csp_internal.h"

namespace csp {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kBins = 2048;

struct Thresh {
    uint32_t bits;   // bit pattern of the K-th largest score of the region
    uint32_t n_eq;   // how many keys equal to it are kept (lowest indices first)
};

// Exclusive prefix (over threads, in thread order) and grand total of a packed
// pair of 32-bit counters.  wsum: kSelWaves entries of scratch LDS.
__device__ __forceinline__ void block_scan_pair(uint64_t v, uint64_t* wsum, uint64_t& excl, uint64_t& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint64_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint64_t o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    uint64_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        const uint64_t s = wsum[w];
        if (w < wave) before += s;
        all += s;
    }
    excl = before + inc - v;
    total = all;
    __syncthreads();  // wsum may be reused
}

__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectParams p) {
    __shared__ uint32_t hist[2][kBins];
    __shared__ uint64_t wsum[kSelWaves];
    __shared__ uint32_t wcnt[3][kSelWaves];
    __shared__ uint32_t sh_has[2];
    __shared__ uint32_t sh_digit[2], sh_rem[2];

    const int sg = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seq0 = p.cu[b];
    const int L = p.cu[b + 1] - seq0;
    const int T = p.budget_T[b];
    const int R = p.R, O = p.O;
    int32_t* out = p.kept_idx + ((size_t)b * p.H_sel + sg) * p.kept_cap;
    int32_t* cnt = p.kept_cnt + ((size_t)b * p.H_sel + sg) * 4;

    if (L <= T) {  // the cache already fits the budget: keep everything
        for (int j = tid; j < p.kept_cap; j += kSelThreads) out[j] = j < L ? j : -1;
        if (tid == 0) { cnt[0] = L; cnt[1] = 0; cnt[2] = 0; cnt[3] = 0; }
        return;
    }

    const int P = L - R;  // rankable prefix
    const uint8_t* mod = p.modality + seq0;
    const float* sc_self = p.score_self + (size_t)sg * p.total_tokens + seq0;
    const float* sc_cross = p.score_cross + (size_t)sg * p.total_tokens + seq0;

    if (tid < 2) sh_has[tid] = 0;
    __syncthreads();
    for (int i = tid; i < O; i += kSelThreads) atomicOr(&sh_has[mod[L - O + i] ? 1 : 0], 1u);
    __syncthreads();
    const bool has0 = sh_has[0] != 0, has1 = sh_has[1] != 0;

    // ---- radix select, both regions at once ---------------------------------
    uint32_t prefix[2] = {0u, 0u};   // threshold bits found so far (high part)
    uint32_t k_rem[2] = {0u, 0u};    // keys still to take from the current bucket
    int K_s = 0, K_c = 0;
    bool none[2] = {false, false};
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
        const int nbits = pass == 2 ? 10 : 11;
        const int prev_shift = pass == 1 ? 21 : 10;  // bits above the current digit
        const uint32_t dmask = (1u << nbits) - 1u;
        for (int i = tid; i < 2 * kBins; i += kSelThreads) (&hist[0][0])[i] = 0u;
        __syncthreads();
        for (int j = tid; j < P; j += kSelThreads) {
            const int mj = mod[j] ? 1 : 0;
            const bool in_s = mj ? has1 : has0;   // some window query shares the key's modality
            const bool in_c = mj ? has0 : has1;   // some window query has the other modality
            if (in_s && !none[0]) {
                const uint32_t bits = __float_as_uint(sc_self[j]);
                if (pass == 0 || (bits >> prev_shift) == prefix[0]) atomicAdd(&hist[0][(bits >> shift) & dmask], 1u);
            }
            if (in_c && !none[1]) {
                const uint32_t bits = __float_as_uint(sc_cross[j]);
                if (pass == 0 || (bits >> prev_shift) == prefix[1]) atomicAdd(&hist[1][(bits >> shift) & dmask], 1u);
            }
        }
        __syncthreads();
        // thread t owns bins hi = nb-1-2t and lo = hi-1 (descending order over threads)
        const int nb = 1 << nbits;
        const int hi = nb - 1 - 2 * tid;
        uint32_t c_hi[2] = {0u, 0u}, c_lo[2] = {0u, 0u};
        if (hi >= 0) { c_hi[0] = hist[0][hi]; c_hi[1] = hist[1][hi]; }
        if (hi >= 1) { c_lo[0] = hist[0][hi - 1]; c_lo[1] = hist[1][hi - 1]; }
        uint64_t excl, total;
        block_scan_pair((uint64_t)(c_hi[0] + c_lo[0]) | ((uint64_t)(c_hi[1] + c_lo[1]) << 32), wsum, excl, total);
        if (pass == 0) {
            // budget rule: K_sel = T - R split by cross_ratio, excess of a short side spills over
            const int n_s = (int)(uint32_t)total, n_c = (int)(uint32_t)(total >> 32);
            const int K_sel = T - R;
            int kc = (int)floor(p.cross_ratio * (double)K_sel);
            kc = kc > K_sel ? K_sel : (kc < 0 ? 0 : kc);
            int ks = K_sel - kc;
            if (ks > n_s) { kc += ks - n_s; ks = n_s; }
            if (kc > n_c) { ks += kc - n_c; kc = n_c; }
            if (ks > n_s) ks = n_s;
            K_s = ks; K_c = kc;
            k_rem[0] = (uint32_t)ks; k_rem[1] = (uint32_t)kc;
            none[0] = ks == 0; none[1] = kc == 0;
        }
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            if (none[r]) continue;
            const uint32_t e = (uint32_t)(excl >> (32 * r));
            const uint32_t K = k_rem[r];
            if (hi >= 0 && e < K && K <= e + c_hi[r]) { sh_digit[r] = (uint32_t)hi; sh_rem[r] = K - e; }
            else if (hi >= 1 && e + c_hi[r] < K && K <= e + c_hi[r] + c_lo[r]) { sh_digit[r] = (uint32_t)(hi - 1); sh_rem[r] = K - e - c_hi[r]; }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            if (none[r]) continue;
            prefix[r] = (prefix[r] << nbits) | sh_digit[r];
            k_rem[r] = sh_rem[r];
        }
        __syncthreads();
    }
    Thresh th[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        th[r].bits = none[r] ? 0xffffffffu : prefix[r];  // no finite non-negative float has this pattern
        th[r].n_eq = none[r] ? 0u : k_rem[r];
    }

    // ---- ordered sweep: flags -> ranks -> scatter ----------------------------
    uint32_t base_eq[2] = {0u, 0u};  // equals of each region seen in earlier blocks
    uint32_t base_out = 0u, n_both = 0u;
    const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    for (int j0 = 0; j0 < L; j0 += kSelThreads) {
        const int j = j0 + tid;
        bool gt[2] = {false, false}, eq[2] = {false, false};
        const bool tail = j >= P && j < L;
        if (j < P) {
            const int mj = mod[j] ? 1 : 0;
            const bool in_s = mj ? has1 : has0;
            const bool in_c = mj ? has0 : has1;
            if (in_s) { const uint32_t bits = __float_as_uint(sc_self[j]); gt[0] = bits > th[0].bits; eq[0] = bits == th[0].bits; }
            if (in_c) { const uint32_t bits = __float_as_uint(sc_cross[j]); gt[1] = bits > th[1].bits; eq[1] = bits == th[1].bits; }
        }
        const uint64_t b0 = __ballot(eq[0]), b1 = __ballot(eq[1]);
        if (lane == 0) { wcnt[0][wave] = __popcll(b0); wcnt[1][wave] = __popcll(b1); }
        __syncthreads();
        uint32_t before0 = 0, before1 = 0, tot0 = 0, tot1 = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) {
            const uint32_t a = wcnt[0][w], c = wcnt[1][w];
            if (w < wave) { before0 += a; before1 += c; }
            tot0 += a; tot1 += c;
        }
        const uint32_t rank0 = base_eq[0] + before0 + __popcll(b0 & lt_mask);
        const uint32_t rank1 = base_eq[1] + before1 + __popcll(b1 & lt_mask);
        base_eq[0] += tot0; base_eq[1] += tot1;
        const bool keep_s = gt[0] || (eq[0] && rank0 < th[0].n_eq);
        const bool keep_c = gt[1] || (eq[1] && rank1 < th[1].n_eq);
        const bool keep = keep_s || keep_c || tail;
        const uint64_t bk = __ballot(keep);
        const uint64_t bb = __ballot(keep_s && keep_c);
        if (lane == 0) wcnt[2][wave] = __popcll(bk);
        n_both += __popcll(bb);  // per-wave partial, reduced at the end
        __syncthreads();
        uint32_t beforek = 0, totk = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) {
            const uint32_t a = wcnt[2][w];
            if (w < wave) beforek += a;
            totk += a;
        }
        if (keep) {
            const uint32_t pos = base_out + beforek + __popcll(bk & lt_mask);
            if (pos < (uint32_t)p.kept_cap) out[pos] = j;
        }
        base_out += totk;
    }
    for (int j = (int)base_out + tid; j < p.kept_cap; j += kSelThreads) out[j] = -1;
    // keys held by both masks: one partial per wavefront
    __syncthreads();
    if (lane == 0) wcnt[0][wave] = n_both;
    __syncthreads();
    if (tid == 0) {
        uint32_t both = 0;
        for (int w = 0; w < kSelWaves; ++w) both += wcnt[0][w];
        cnt[0] = (int32_t)base_out; cnt[1] = K_s; cnt[2] = K_c; cnt[3] = (int32_t)both;
    }
}

}  // namespace

hipError_t launch_select(const SelectParams& p, hipStream_t s) {
    const dim3 grid(p.H_sel, p.B);
    hipLaunchKernelGGL(select_kernel, grid, dim3(kSelThreads), 0, s, p);
    return hipGetLastError();
}

}  // namespace csp
