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
// and how many keys equal to it still fit.  Each wavefront owns a contiguous
// run of ITEMS*64 keys of a super-block of 1024*ITEMS keys and reads it with
// coalesced loads (lane l holds keys l, l+64, ...), so "greater than the
// threshold, or equal and among the first few equals" is a chain of wave
// ballots and popcounts in key order plus two block-wide exchanges of
// per-wavefront totals per super-block; the kept positions come out ascending,
// with the lower-index-first tie rule, and without atomics on the output.  With
// a single-modality window every key belongs to exactly one region: one bit
// pattern per key stays in registers for all passes when the sequence fits one
// super-block (up to 32 keys per thread: 32K keys; measured at 32K keys 39 us
// against 50 us with super-blocks of 8K keys re-read per pass).
#include "csp_internal.h"

namespace csp {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kBins = 2048;
constexpr uint32_t kNone = 0xffffffffu;  // "not a candidate": no finite non-negative float

// The first pass sees every key, and scores crowd into few digits (a handful of exponents): lanes of a
// wavefront that hit the same counter are served one after the other.  It spreads the lanes over
// kHistCopies copies of the histograms (lane % kHistCopies); the later passes see few keys and use copy 0.
constexpr int kHistCopies = 8;

struct SelShared {
    uint32_t hist[kHistCopies][2][kBins];
    uint64_t wsum[kSelWaves];
    uint32_t has[2];
    uint32_t digit[2], rem[2];
};

// Exclusive prefix (over threads, in thread order) and grand total of a packed
// pair of 32-bit counters.
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

struct SelCtx {
    const uint8_t* mod;
    const float* sc_self;
    const float* sc_cross;
    int32_t* out;
    int32_t* cnt;
    int L, P, T, R, kept_cap;
    bool has0, has1;
    double cross_ratio;
};

// ITEMS consecutive keys per thread and super-block.  DUAL: the window holds both
// modalities, every prefix key is a candidate of both regions (two bit patterns per
// key); otherwise one pattern plus a region bit.  CACHED: the sequence fits one
// super-block and the patterns are loaded once.
template <int ITEMS, bool DUAL, bool CACHED>
__device__ __forceinline__ void select_body(const SelCtx& c, SelShared& sh) {
    const int tid = threadIdx.x;
    constexpr int SUPER = kSelThreads * ITEMS;
    const int n_super = CACHED ? 1 : (c.L + SUPER - 1) / SUPER;

    static_assert(ITEMS <= 64, "a bit per item in a 64-bit mask");
    typedef uint64_t ItemMask;          // a bit per item of this thread
    uint32_t ka[ITEMS];                 // self-region pattern, or the key's only pattern
    uint32_t kb[DUAL ? ITEMS : 1];      // cross-region pattern (DUAL only)
    ItemMask in_cross = 0u;             // !DUAL: bit i set = key i ranks in the cross region

    const int lane = tid & 63, wave = tid >> 6;
    // key i of this lane in super-block sb
    auto key_index = [&](int sb, int i) { return sb * SUPER + wave * (ITEMS * kWave) + i * kWave + lane; };
    auto load_keys = [&](int sb) {
        in_cross = 0u;
        // (in groups of 16 items: what is in flight at once fits the registers also with 32 items per thread)
        constexpr int GROUP = ITEMS < 16 ? ITEMS : 16;
#pragma unroll
        for (int g0 = 0; g0 < ITEMS; g0 += GROUP) {
        uint8_t m[GROUP];
#pragma unroll
        for (int i = g0; i < g0 + GROUP; ++i) {
            const int j = key_index(sb, i);
            m[i - g0] = c.mod[j < c.P ? j : 0];   // every lane loads (a clamped index): no load under a branch
        }
#pragma unroll
        for (int i = g0; i < g0 + GROUP; ++i) {
            const int j = key_index(sb, i);
            if constexpr (DUAL) {
                ka[i] = j < c.P ? __float_as_uint(c.sc_self[j]) : kNone;
                kb[i] = j < c.P ? __float_as_uint(c.sc_cross[j]) : kNone;
            } else {
                // the window has one modality: keys sharing it rank in the self region, the rest in cross.
                // Both scores are requested at once, beside the modality, and one is picked: a load whose
                // address waits for the modality would add a memory round trip to a latency-bound kernel
                const int jc = j < c.P ? j : 0;
                const uint32_t ss = __float_as_uint(c.sc_self[jc]), sx = __float_as_uint(c.sc_cross[jc]);
                const bool self_key = m[i - g0] ? c.has1 : c.has0;
                ka[i] = j < c.P ? (self_key ? ss : sx) : kNone;
                if (!self_key) in_cross |= (ItemMask)1 << i;
            }
        }
        }
    };
    // region r pattern of key i (kNone if key i is not a candidate of region r)
    auto pat = [&](int i, int r) -> uint32_t {
        if constexpr (DUAL) {
            return r == 0 ? ka[i] : kb[i];
        } else {
            const bool cr = (in_cross >> i) & 1u;
            return (cr == (r == 1)) ? ka[i] : kNone;
        }
    };
    if (CACHED) load_keys(0);

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
        const int copies = pass == 0 ? kHistCopies : 1;
        for (int i = tid; i < copies * 2 * kBins; i += kSelThreads) (&sh.hist[0][0][0])[i] = 0u;
        uint32_t (*const my_hist)[kBins] = sh.hist[pass == 0 ? (tid & (kHistCopies - 1)) : 0];
        __syncthreads();
#pragma unroll 1
        for (int sb = 0; sb < n_super; ++sb) {
            if (!CACHED) load_keys(sb);
#pragma unroll
            for (int i = 0; i < ITEMS; ++i) {
                if constexpr (DUAL) {
#pragma unroll
                    for (int r = 0; r < 2; ++r) {
                        const uint32_t a = pat(i, r);
                        if (a != kNone && !none[r] && (pass == 0 || (a >> prev_shift) == prefix[r]))
                            atomicAdd(&my_hist[r][(a >> shift) & dmask], 1u);
                    }
                } else {
                    const int r = (in_cross >> i) & 1u;  // the key's only region
                    const uint32_t a = ka[i];
                    if (a != kNone && !(r ? none[1] : none[0]) && (pass == 0 || (a >> prev_shift) == (r ? prefix[1] : prefix[0])))
                        atomicAdd(&my_hist[r][(a >> shift) & dmask], 1u);
                }
            }
        }
        __syncthreads();
        // thread t owns bins hi = nb-1-2t and lo = hi-1 (descending order over threads)
        const int nb = 1 << nbits;
        const int hi = nb - 1 - 2 * tid;
        uint32_t c_hi[2] = {0u, 0u}, c_lo[2] = {0u, 0u};
        for (int cp = 0; cp < copies; ++cp) {
            if (hi >= 0) { c_hi[0] += sh.hist[cp][0][hi]; c_hi[1] += sh.hist[cp][1][hi]; }
            if (hi >= 1) { c_lo[0] += sh.hist[cp][0][hi - 1]; c_lo[1] += sh.hist[cp][1][hi - 1]; }
        }
        uint64_t excl, total;
        block_scan_pair((uint64_t)(c_hi[0] + c_lo[0]) | ((uint64_t)(c_hi[1] + c_lo[1]) << 32), sh.wsum, excl, total);
        if (pass == 0) {
            // budget rule: K_sel = T - R split by cross_ratio, excess of a short side spills over
            const int n_s = (int)(uint32_t)total, n_c = (int)(uint32_t)(total >> 32);
            const int K_sel = c.T - c.R;
            int kc = (int)floor(c.cross_ratio * (double)K_sel);
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
            if (hi >= 0 && e < K && K <= e + c_hi[r]) { sh.digit[r] = (uint32_t)hi; sh.rem[r] = K - e; }
            else if (hi >= 1 && e + c_hi[r] < K && K <= e + c_hi[r] + c_lo[r]) { sh.digit[r] = (uint32_t)(hi - 1); sh.rem[r] = K - e - c_hi[r]; }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            if (none[r]) continue;
            prefix[r] = (prefix[r] << nbits) | sh.digit[r];
            k_rem[r] = sh.rem[r];
        }
        __syncthreads();
    }
    uint32_t th_bits[2], th_eq[2];  // K-th largest pattern of the region; equals still to keep
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        th_bits[r] = none[r] ? 0xfffffffeu : prefix[r];  // above every finite non-negative float: nothing is kept
        th_eq[r] = none[r] ? 0u : k_rem[r];
    }

    // ---- ordered sweep: equal ranks, keep flags, positions --------------------
    uint32_t base_eq[2] = {0u, 0u};  // equals of each region in earlier super-blocks
    uint32_t base_out = 0u, n_both = 0u;
    const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    uint64_t* wtot = sh.wsum;
    // exclusive prefix over wavefronts and grand total of a packed pair of per-wavefront counters
    auto wave_exchange = [&](uint64_t mine, uint64_t& before, uint64_t& all) {
        if (lane == 0) wtot[wave] = mine;
        __syncthreads();
        before = 0; all = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) {
            const uint64_t v = wtot[w];
            if (w < wave) before += v;
            all += v;
        }
        __syncthreads();
    };
#pragma unroll 1
    for (int sb = 0; sb < n_super; ++sb) {
        if (!CACHED) load_keys(sb);
        // 1. equals of each region held by this wavefront
        uint32_t eqw[2] = {0u, 0u};
        ItemMask eq_any = 0u;  // bit i: some lane's key i equals a threshold (ties are rare: fast path below)
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const uint64_t b0 = __ballot(pat(i, 0) == th_bits[0]);
            const uint64_t b1 = __ballot(pat(i, 1) == th_bits[1]);
            eqw[0] += __popcll(b0);
            eqw[1] += __popcll(b1);
            eq_any |= (ItemMask)((b0 | b1) != 0ull ? 1u : 0u) << i;
        }
        uint64_t before, all;
        wave_exchange((uint64_t)eqw[0] | ((uint64_t)eqw[1] << 32), before, all);
        uint32_t run[2] = {base_eq[0] + (uint32_t)before, base_eq[1] + (uint32_t)(before >> 32)};
        base_eq[0] += (uint32_t)all;
        base_eq[1] += (uint32_t)(all >> 32);
        // 2. keep flags in key order (items ascend within the wavefront, lanes within an item)
        ItemMask keep_bits = 0u;
        uint32_t keep_w = 0u, both_w = 0u;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const int j = key_index(sb, i);
            const uint32_t a0 = pat(i, 0), a1 = pat(i, 1);
            bool kp0 = a0 != kNone && a0 > th_bits[0];
            bool kp1 = a1 != kNone && a1 > th_bits[1];
            if ((eq_any >> i) & 1u) {  // uniform: some key of this item ties with a threshold
                const bool e0 = a0 == th_bits[0], e1 = a1 == th_bits[1];
                const uint64_t b0 = __ballot(e0), b1 = __ballot(e1);
                kp0 = kp0 || (e0 && run[0] + __popcll(b0 & lt_mask) < th_eq[0]);
                kp1 = kp1 || (e1 && run[1] + __popcll(b1 & lt_mask) < th_eq[1]);
                run[0] += __popcll(b0);
                run[1] += __popcll(b1);
            }
            const bool keep = kp0 || kp1 || (j >= c.P && j < c.L);   // the last R keys are always kept
            keep_bits |= (ItemMask)(keep ? 1u : 0u) << i;
            keep_w += __popcll(__ballot(keep));
            if constexpr (DUAL) both_w += __popcll(__ballot(kp0 && kp1));
        }
        wave_exchange((uint64_t)keep_w | ((uint64_t)both_w << 32), before, all);
        // 3. positions
        uint32_t pos0 = base_out + (uint32_t)before;
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
            const bool keep = (keep_bits >> i) & 1u;
            const uint64_t bk = __ballot(keep);
            const uint32_t pos = pos0 + __popcll(bk & lt_mask);
            if (keep && pos < (uint32_t)c.kept_cap) c.out[pos] = key_index(sb, i);
            pos0 += __popcll(bk);
        }
        base_out += (uint32_t)all;
        n_both += (uint32_t)(all >> 32);
    }
    for (int j = (int)base_out + tid; j < c.kept_cap; j += kSelThreads) c.out[j] = -1;
    if (tid == 0) { c.cnt[0] = (int32_t)base_out; c.cnt[1] = K_s; c.cnt[2] = K_c; c.cnt[3] = (int32_t)n_both; }
}

template <int ITEMS>
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectParams p) {
    extern __shared__ __align__(16) char sel_smem[];
    SelShared& sh = *reinterpret_cast<SelShared*>(sel_smem);
    const int sg = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x;
    SelCtx c;
    c.L = view_len(p.view, b, sg * (p.view.H_kv / p.H_sel));
    c.T = p.budget_T[b];
    c.R = p.R;
    c.kept_cap = p.kept_cap;
    c.cross_ratio = p.cross_ratio;
    c.out = p.kept_idx + ((size_t)b * p.H_sel + sg) * p.kept_cap;
    c.cnt = p.kept_cnt + ((size_t)b * p.H_sel + sg) * 4;

    if (c.L <= c.T) {  // the cache already fits the budget: keep everything
        for (int j = tid; j < p.kept_cap; j += kSelThreads) c.out[j] = j < c.L ? j : -1;
        if (tid == 0) { c.cnt[0] = c.L; c.cnt[1] = 0; c.cnt[2] = 0; c.cnt[3] = 0; }
        return;
    }
    c.P = c.L - c.R;  // rankable prefix
    c.mod = p.modality + view_mod0(p.view, b, sg);
    c.sc_self = p.score_self + view_score0(p.view, b, sg);
    c.sc_cross = p.score_cross + view_score0(p.view, b, sg);

    if (tid < 2) sh.has[tid] = 0;
    __syncthreads();
    for (int i = tid; i < p.O; i += kSelThreads) atomicOr(&sh.has[c.mod[c.L - p.O + i] ? 1 : 0], 1u);
    __syncthreads();
    c.has0 = sh.has[0] != 0;
    c.has1 = sh.has[1] != 0;

    if (c.has0 && c.has1) {
        select_body<4, true, false>(c, sh);       // both regions cover every key: two patterns per key
    } else if (c.L <= kSelThreads * ITEMS) {
        select_body<ITEMS, false, true>(c, sh);   // one super-block, patterns stay in registers
    } else {
        select_body<8, false, false>(c, sh);      // longer than 32K keys: super-blocks re-read per pass
    }
}

}  // namespace

hipError_t launch_select(const SelectParams& p, int max_seqlen, hipStream_t s) {
    const dim3 grid(p.H_sel, p.B), block(kSelThreads);
    const int items = (max_seqlen + kSelThreads - 1) / kSelThreads;
    auto launch = [&](auto kernel) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(SelShared));
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kernel, grid, block, sizeof(SelShared), s, p);
        return hipGetLastError();
    };
    if (items <= 4) return launch(select_kernel<4>);
    if (items <= 8) return launch(select_kernel<8>);
    if (items <= 16) return launch(select_kernel<16>);
    return launch(select_kernel<32>);  // up to 32K keys stay in registers; beyond: several super-blocks (64 keys per thread
                                       // spill, and at 64K keys the re-reads are not what takes the time)  // up to 64K keys stay in registers (64 per thread); beyond: several super-blocks
}

}  // namespace csp
