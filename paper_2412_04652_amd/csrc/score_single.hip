// csp_score from ONE read of the keys: a persistent, software-pipelined kernel for gfx950.
//
// What is computed (paper: Eq. "A = softmax(QK^T/sqrt d)" / Eq. "n-softmax", the window trim
// A[-O:, :-R], Eq. "cross-self"; Algorithm 1 steps "A <- n-Softmax(O)" ... "A^s, A^c <- ..."):
// as in score.hip.
//
// Design.  The per-key sums need the final normaliser of every window row, which depends on all
// L keys.  A task is a chunk of 512 keys of one (sequence, query head, part of <= 64 window rows):
// the workgroup computes the chunk's logits against the part (S^T = K Q^T on
// v_mfma_f32_32x32x16_bf16, window rows on the lane axis, 8 wavefronts x 2 tiles of 32 keys),
// publishes the chunk's log-sum-exp per row, reads the ones of the other chunks of the head and
// turns its weights into normalised ones.  The exchange costs a memory round trip or two; a kernel
// that sits out that latency (and the latency of its first key tile) once per chunk runs at 45 % of
// the HBM rate.  Here it is hidden:
//  - one workgroup of 8 wavefronts per compute unit, resident for the whole launch (all 160 KiB of
//    LDS), two wavefronts per SIMD; tasks are dealt statically (workgroup w takes tasks w,
//    w + #workgroups, ...) from a table of 64-byte records that a set-up kernel writes per launch and
//    the pipeline reads through the scalar cache;
//  - three tasks are in flight per workgroup.  In step n: the logits of task n; the scores of task
//    n-2 (its weights have waited in registers as fp16 pairs, its rows' log-sum-exps in LDS since
//    the last step); maxima, weights and row sums of task n and, after a barrier, its published
//    log-sum-exp; THEN the merge of the statistics of task n-1, published most of a step ago by
//    everybody.  Two workgroup barriers per step;
//  - the vector ALU does one FMA, one exponential and two conversions per weight and little else.
//    With the window rows on the lane axis a row's maximum is an in-lane reduction (plus one
//    exchange with the lane 32 further on); the row sums are MFMAs of the fp16 weights with a
//    matrix of ones (v_mfma_f32_4x4x4_16b_f16: the contraction runs over a lane's registers, i.e.
//    over keys, and the small shape costs a quarter of the cycles and registers); an MFMA with a
//    permutation matrix hands every weight, unchanged, to the lane of its key, which is the layout
//    in which the column sums are again an MFMA (contraction over the window rows, the rows'
//    factors 2^(reference - lse) as the other operand, split by the rows' modality);
//  - every global load of the loop goes straight to LDS (global_load_lds, issued from inline
//    assembly): the key tiles of task n+1 are requested as soon as the MFMAs of task n have read a
//    tile buffer and from then on a few at a time between the exponentials (XOR-swizzled rows: the
//    LDS image is laid out by choosing each lane's global address), the queries of task n+1 once
//    every wavefront is past those MFMAs, the statistics of task n-1 behind the scores of task n-2.
//    No load holds a register.  The compiler knows nothing of these loads (had it known, it would
//    drain them all, s_waitcnt vmcnt(0), in front of every LDS access and barrier): the waits are
//    written by hand (s_waitcnt vmcnt with the number of younger loads; loads return in order), and
//    the workgroup barriers wait for LDS traffic only.
// What bounds it: the key tiles have one buffer (the LDS is full), so a tile can be requested only
// after the step's logits and must have landed before the next step's: all workgroups ask for
// their 128 KiB in the same two thirds of a step, and the step is about as long as the memory
// system needs for that plus the logits.  Shortening the arithmetic does not shorten the step
// (measured); requesting earlier does, up to the point where the requests queue at the memory
// pipeline and hold up the wavefront that issues them.
// The exchange uses agent-scope stores and loads (sc1; no release fence: on this multi-XCD part
// it would write back a whole L2).  Every statistic is set to NaN before the launch (set-up
// kernel), so a value that reads as a number has been published: entries validate themselves.
// No workgroup depends on one that has not started: the statistics of task n are published
// before anything of task n-1 is waited for, and the chunks of a head are at most one step
// apart (the host guarantees G * parts * chunks <= #workgroups), so every wait ends once all
// workgroups are resident, and they are when the launch has the chip to itself.  The wait is
// bounded all the same (the chip may be shared, compute units may be masked): a workgroup whose
// wait runs out notes the task, and when its own list is done recomputes the statistics of every
// chunk of that head by itself with the very same code (same order of operations: the result is
// bit-identical to the exchanged one) and finishes the task.  Such tasks are counted
// (ScoreParams::counters[0]).
#include "score_tiles.h"

// no implicit fusing of a*b+c: the two places that compute a chunk's statistics (the pipeline
// and the self-sufficient path) must round alike; fused operations are written as fmaf
#pragma clang fp contract(off)

namespace csp {
using namespace score_detail;
namespace {

constexpr int kSWaves = 8;                                  // wavefronts of a workgroup: two per SIMD
constexpr int kSThreads = kSWaves * kWave;
constexpr int kPipeTiles = 2;                               // 32-key tiles per wavefront and task
constexpr int kPipeChunk = kSWaves * kTile * kPipeTiles;    // 512 keys per task
constexpr int kStatRows = 64;                               // floats per (head part, chunk) in the statistics array
constexpr int kPoll = 4;                                    // statistics one lane requests ahead
constexpr int kFailWords = kScoreSingleMaxIters / 32;
static_assert(kPipeChunk == kScoreSingleChunk, "host and kernel agree on the chunk");

// Key tile in LDS as the direct loads lay it out: 32 rows of D bf16 back to back, the 16-byte
// pieces of a row XOR-swizzled so that the MFMA operand fetch (32 lanes reading the same piece
// of 32 different rows) is free of bank conflicts.
template <int D>
struct TileGeom {
    static constexpr int ROW_BYTES = D * 2;
    static constexpr int CPR = ROW_BYTES / 16;          // pieces per row
    static constexpr int RPI = kWave / CPR;             // rows one load instruction covers
    static constexpr int NLD = kTile / RPI;             // load instructions per tile
    static constexpr int NK = D / 16;                   // MFMA steps along the contraction
    static constexpr int TILE_LDS = kTile * ROW_BYTES;
    __device__ static __forceinline__ int key(int r) { return (r / (16 / CPR)) & (CPR - 1); }
    // LDS offset of piece cc of row r
    __device__ static __forceinline__ int at(int r, int cc) { return r * ROW_BYTES + ((cc ^ key(r)) * 16); }
};

// (a direct-to-LDS load writes a dword per lane whatever its size: byte loads arrive zero-extended)
template <int D, int NQB>
struct PipeSmem {
    using TG = TileGeom<D>;
    static constexpr int NQ = NQB * 32;
    static constexpr int kTiles = kSWaves * kPipeTiles * TG::TILE_LDS;
    static constexpr int kQ = NQB * TG::NK * 64 * 16;                      // queries in MFMA operand order
    static constexpr int off_q = kTiles;
    static constexpr int off_stat = off_q + kQ;                            // float [kSWaves][kPoll][64]: the head's statistics as loaded;
    static constexpr int kStat = kSWaves * kPoll * 64 * 4;                 //   later, in each wavefront's part, fp16 [4][NQ]: the factor rows of
    static_assert(4 * NQ * 2 <= kPoll * 64 * 4, "the factor rows fit");    //   its column-sum MFMAs
    static constexpr int off_wmax = off_stat + kStat;                      // float [kSWaves][NQ]: exponent references per wavefront
    static constexpr int off_wsum = off_wmax + kSWaves * NQ * 4;           // float [kSWaves][NQ]: row sums per wavefront
    static constexpr int off_nl = off_wsum + kSWaves * NQ * 4;             // float [NQ]: log-sum-exp of the head's rows
    static constexpr int off_zero = off_nl + NQ * 4;                       // 128 bytes of zeros: the factor rows 4..31
    static constexpr int off_flag = off_zero + 128;                        // int [kSWaves]: wavefront found its statistics
    static constexpr int off_fail = off_flag + kSWaves * 4;                // uint32 [kFailWords]
    static constexpr int total = off_fail + kFailWords * 4;
    static_assert(total <= 160 * 1024, "one workgroup per compute unit: 160 KiB of LDS");
};

// ---- the task table ---------------------------------------------------------------------------
// One task: 512 keys of one (sequence, query head, part of the window rows).  Everything a
// workgroup needs to know about a task is worked out once per launch by the set-up kernel and kept
// as a 64-byte record; the pipeline fetches a record with one scalar load where it needs it.  (The
// pipeline keeps many vector loads in flight and awaits them by their position in the queue: it
// issues no vector load of its own, and it has few scalar registers to spare for descriptors.)
static_assert(sizeof(PipeRec) == 64, "one record = one 16-dword scalar load");

// The keys' modality as bits: a row of bits_words words per sequence (packed form: every selection
// group of a sequence sees the same flags) or per (sequence, selection group) (cache form), bit
// j % 32 of word j / 32 = key j is a visual token; keys past the end: 0; two spare words at the end.
__device__ __host__ __forceinline__ int bits_words(const ScoreParams& p) { return p.n_chunks * (kScoreSingleChunk / 32); }
__device__ __forceinline__ int bits_row(const SeqView& v, int b, int sg) { return v.kv_len ? b * v.H_sel + sg : b; }
__device__ __host__ __forceinline__ size_t bits_rows(const ScoreParams& p) { return (size_t)p.B * (p.view.kv_len ? p.view.H_sel : 1); }

// record of task id `lin` (ids at or past n_lin: a record that is not valid)
__device__ PipeRec make_rec(const ScoreParams& p, int lin) {
    PipeRec t;
    const int share = p.G * p.vsplit;
    const bool in_range = lin < p.n_lin;
    int task = in_range ? xcd_task(lin, share) : 0;
    const bool real = in_range && task < p.n_tasks;
    if (!real) task = 0;
    const int v = task % p.vsplit; task /= p.vsplit;
    const int g_in = task % p.G; task /= p.G;
    const int chunk = task % p.n_chunks; task /= p.n_chunks;
    const int hk = task % p.view.H_kv, b = task / p.view.H_kv;
    const int hq = hk * p.G + g_in, sg = hq / p.sel_group;
    const int L = view_len(p.view, b, hk);
    t.L = L > 0 ? L : 1;
    t.c0 = chunk * kPipeChunk;
    const bool valid = real && L > 0 && t.c0 < L && !view_fits(p.view, b, L);
    if (!valid) t.c0 = 0;
    const int row0 = v * kStatRows;
    const int rows = min(kStatRows, p.O - row0);
    t.rows_valid = rows | (valid ? 1 << 16 : 0);
    t.pos0 = t.L - p.O + row0;
    const int bh = b * p.H_q + hq;
    t.kbase = reinterpret_cast<const char*>(p.k) + (view_key0(p.view, b, p.k_stride_tok) + (int64_t)hk * p.k_stride_head) * 2;
    t.qpart = reinterpret_cast<const char*>(p.q_win) + ((size_t)bh * p.O + row0) * p.D * 2;
    t.kbits = p.modbits + (size_t)bits_row(p.view, b, sg) * bits_words(p) + (t.c0 / kPipeChunk) * (kPipeChunk / 32);
    t.spare0 = t.spare1 = 0u;
    t.stat = p.part + ((size_t)(bh * p.vsplit + v) * p.n_chunks) * kStatRows;
    const int slice = (hq % p.sel_group) * p.vsplit + v;
    t.out_self = (p.gsplit > 1 ? p.slice_self + (size_t)slice * (size_t)p.score_elems : p.score_self) + (size_t)view_score0(p.view, b, sg);
    return t;
}

// Set-up of a launch: every statistic marked as not yet published, the counters cleared, the
// task table written (n_lin records and one that is not valid), the keys' modality flags packed
// into bits (a word per 32 keys of a (sequence, selection group); keys past the end: 0).
__global__ __launch_bounds__(256) void score_single_setup_kernel(ScoreParams p) {
    const size_t n = (size_t)p.B * p.H_q * p.vsplit * p.n_chunks * kStatRows;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) reinterpret_cast<uint32_t*>(p.part)[i] = 0x7fc00000u;   // a NaN, by its bit pattern
    if (i < 4) p.counters[i] = 0;
    if (i <= (size_t)p.n_lin) p.table[i] = make_rec(p, (int)i);
    const size_t keys_per_row = (size_t)bits_words(p) * 32;
    if (i < bits_rows(p) * keys_per_row) {   // (a multiple of 64: whole wavefronts)
        const int j = (int)(i % keys_per_row), row = (int)(i / keys_per_row);
        const int b = p.view.kv_len ? row / p.view.H_sel : row, sg = p.view.kv_len ? row % p.view.H_sel : 0;
        const int L = view_len(p.view, b, (sg * p.sel_group) / p.G);
        const bool vis = j < L && p.modality[view_mod0(p.view, b, sg) + j] != 0;
        const uint64_t bal = __ballot(vis);
        if ((threadIdx.x & 31) == 0) p.modbits[i / 32] = (uint32_t)(bal >> (threadIdx.x & 32));
    }
    if (i < 2) p.modbits[bits_rows(p) * bits_words(p) + i] = 0u;
}

// A task as the kernel uses it: the record at `rec`, through the scalar cache (written by the previous
// kernel, never by this one), its packed fields taken apart.
struct PipeTask {
    int32_t valid, L, c0, rows, pos0;
    const char* kbase;
    const char* qpart;
    const uint32_t* kbits;
    float* stat;
    float* out_self;
};
typedef int i32x16 __attribute__((ext_vector_type(16)));
__device__ __forceinline__ PipeTask load_rec(const PipeRec* rec) {
    i32x16 v;
    asm volatile("s_load_dwordx16 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(rec) : "memory");
    auto ptr = [&](int i) { return ((uint64_t)(uint32_t)v[i + 1] << 32) | (uint32_t)v[i]; };
    PipeTask t;
    t.valid = (v[0] >> 16) & 1; t.rows = v[0] & 0xffff; t.L = v[1]; t.c0 = v[2]; t.pos0 = v[3];
    t.kbase = reinterpret_cast<const char*>(ptr(6));
    t.qpart = reinterpret_cast<const char*>(ptr(8));
    t.kbits = reinterpret_cast<const uint32_t*>(ptr(10));
    t.stat = reinterpret_cast<float*>(ptr(12));
    t.out_self = reinterpret_cast<float*>(ptr(14));
    return t;
}
// one word of a task's key modality bits, through the scalar cache
__device__ __forceinline__ uint32_t load_bits(const uint32_t* at) {
    uint32_t v;
    asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(at) : "memory");
    return v;
}
// the modality bits of the 64 keys from position pos of the task's sequence on (bit i: key pos + i)
__device__ __forceinline__ uint64_t load_bits64(const PipeTask& t, int pos) {
    const uint32_t* const at = t.kbits - (t.c0 / kScoreSingleChunk) * (kScoreSingleChunk / 32) + pos / 32;
    uint32_t w0, w1, w2;
    asm volatile("s_load_dword %0, %3, 0x0\n\ts_load_dword %1, %3, 0x4\n\ts_load_dword %2, %3, 0x8\n\ts_waitcnt lgkmcnt(0)"
                 : "=&s"(w0), "=&s"(w1), "=&s"(w2) : "s"(at) : "memory");
    const int sh = pos % 32;
    const uint64_t lo = ((uint64_t)w1 << 32) | w0, hi = ((uint64_t)w2 << 32) | w1;
    return (uint64_t)(uint32_t)(lo >> sh) | ((uint64_t)(uint32_t)(hi >> sh) << 32);
}
__device__ __forceinline__ int rec_chunks(const PipeTask& t) { return (t.L + kPipeChunk - 1) / kPipeChunk; }

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr float kWeightShift = 15.f;   // weights are kept as 2^15 * 2^(x - maximum): the fp16 copies use the format's range
// The factor of a row, 2^(reference - lse) <= 2^-15, enters the column-sum MFMAs as fp16 scaled by 2^30.
constexpr float kFactorShift = 30.f;
constexpr float kFactorUnshift = 0x1p-30f;
struct PkQuad { f16x2 q[4]; };   // 8 weights of one lane: the B operand of one column-sum MFMA
__device__ __forceinline__ f32x16 mma_f16(f16x8 a, f16x8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }

// One wavefront instruction that loads 16, 4 or 1 bytes per lane from each lane's own global address
// (uniform base + the lane's unsigned 32-bit offset, or the lane's 64-bit address) straight into LDS at
// lds + lane * max(size, 4): byte loads arrive zero-extended to the lane's dword.  lds is the uniform
// LDS byte address.
// These loads are written in assembly so that the compiler does not know of them.  It cannot tell
// which LDS accesses touch their destinations, and it orders every LDS access and every workgroup
// barrier behind all of them (s_waitcnt vmcnt(0)): a pipeline that requests data a whole step before
// it is used would wait for it on the spot.  Here the waits are written by hand (wait_loads), with
// the number of younger loads; loads return in order.
// The wait states in front of the load: the address registers may have been written by a vector
// instruction just before (a scalar register brought back from a spill: 5 wait states before a
// memory instruction reads it), and m0 one instruction before (1 wait state).
#define CSP_DMA_ASM(OP, ADDR, MODS) "s_mov_b32 m0, %2\n\ts_nop 4\n\t" OP " " ADDR MODS
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}
// 16 bytes per lane, plain or non-temporal (keys that are streamed once)
template <bool NT_HINT>
__device__ __forceinline__ void load_to_lds_16(const void* base, uint32_t lane_off, uint32_t lds) {
    if constexpr (NT_HINT) asm volatile(CSP_DMA_ASM("global_load_lds_dwordx4", "%1, %0", " nt") ::"s"(base), "v"(lane_off), "s"(lds) : "memory", "m0");
    else asm volatile(CSP_DMA_ASM("global_load_lds_dwordx4", "%1, %0", "") ::"s"(base), "v"(lane_off), "s"(lds) : "memory", "m0");
}
template <bool NT_HINT>
__device__ __forceinline__ void load_to_lds_16(const void* lane_addr, uint32_t lds) {
    const uint64_t a = reinterpret_cast<uint64_t>(lane_addr);
    if constexpr (NT_HINT) asm volatile(CSP_DMA_ASM("global_load_lds_dwordx4", "%0, off", " nt") ::"v"(a), "s"(0), "s"(lds) : "memory", "m0");
    else asm volatile(CSP_DMA_ASM("global_load_lds_dwordx4", "%0, off", "") ::"v"(a), "s"(0), "s"(lds) : "memory", "m0");
}
// 4 bytes per lane at agent scope (sc1): sees what other workgroups published with agent-scope stores
__device__ __forceinline__ void load_to_lds_4_agent(const void* base, uint32_t lane_off, uint32_t lds) {
    asm volatile(CSP_DMA_ASM("global_load_lds_dword", "%1, %0", " sc1") ::"s"(base), "v"(lane_off), "s"(lds) : "memory", "m0");
}
// Waits until at most YOUNGER of this wavefront's vector memory loads are outstanding (they return
// in order: everything issued before the YOUNGER most recent ones has landed), and keeps the
// compiler from moving LDS accesses across.  Stores are never counted in YOUNGER: one that is still
// in flight only makes the wait stricter.
template <int YOUNGER>
__device__ __forceinline__ void wait_loads() {
    static_assert(YOUNGER >= 0 && YOUNGER < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(YOUNGER) : "memory");
}
// Workgroup barrier that orders LDS accesses only (this wavefront's are complete before it arrives).
// __syncthreads() would also wait for every outstanding global access: the score stores of the
// previous task, and with them the loads in flight.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Returns x, in a way the compiler cannot see through.  Per-lane address arithmetic that starts
// from such a value is redone where it is used instead of being hoisted out of the kernel's loop
// into registers that stay occupied for the whole launch (dozens, with every load address unrolled).
__device__ __forceinline__ int opaque(int x) {
    asm volatile("" : "+v"(x));
    return x;
}

// ---- lane-crossing reductions in the vector ALU (data-parallel primitives, no LDS) --------------
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
template <int CTRL>
__device__ __forceinline__ float lane_xchg(float x) {
    const int xi = __builtin_bit_cast(int, x);
    // (every lane has a source lane under these controls; written this way the move folds into the operation)
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, xi, CTRL, 0xf, 0xf, true));
}
template <bool MAX>
__device__ __forceinline__ float red_op(float a, float b) { return MAX ? fmaxf(a, b) : a + b; }
// All-reduce over aligned groups of GROUP = 8 or 16 lanes: every lane ends up with the same value
// (the two lanes of an exchange compute a op b and b op a).
template <int GROUP, bool MAX>
__device__ __forceinline__ float group_allreduce(float x) {
    static_assert(GROUP == 8 || GROUP == 16, "8 or 16 lanes");
    x = red_op<MAX>(x, lane_xchg<0xB1>(x));    // l ^ 1
    x = red_op<MAX>(x, lane_xchg<0x4E>(x));    // l ^ 2
    x = red_op<MAX>(x, lane_xchg<0x141>(x));   // l ^ 7: the other quad of the 8
    if constexpr (GROUP == 16) x = red_op<MAX>(x, lane_xchg<0x140>(x));   // row_mirror, 15 - l: the other 8 of the 16
    return x;
}

// All-reduce over the two lanes l and l ^ 32.
template <bool MAX>
__device__ __forceinline__ float halves_allreduce(float x) {
    const u32x2 s = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, x), false, false);
    const unsigned s0 = s[0], s1 = s[1];   // copies: a bit cast of a vector element reads element 0
    return red_op<MAX>(__builtin_bit_cast(float, s0), __builtin_bit_cast(float, s1));
}

template <bool V> struct Interleaved { static constexpr bool value = V; };

// Modality of this lane's window row (my_row) of a task, carried from its front stage to its back stage.
typedef uint32_t WindowBits;

// Development aid: -DCSP_SINGLE_TIMING=w makes wavefront w of workgroup 0 record the shader clock at the
// phase boundaries of every step behind the modality bits in the workspace (16 slots per step).
#ifdef CSP_SINGLE_TIMING
#define CSP_TS(slot) do { if (blockIdx.x == 0 && threadIdx.x == (CSP_SINGLE_TIMING) * 64 && ts_it >= 0 && ts_it < 64) ts_buf[ts_it * 16 + (slot)] = clock64(); } while (0)
#else
#define CSP_TS(slot) do { } while (0)
#endif
// ... -DCSP_SINGLE_TIMING_ALL: every workgroup records the constant-rate clock (10 ns ticks) at four
// points of every step (4 slots per step, 32 steps per workgroup), in the same place.
#ifdef CSP_SINGLE_TIMING_ALL
#define CSP_TSA(k) do { if (threadIdx.x == 0 && tsa_it >= 0 && tsa_it < 32) tsa_buf[((long long)blockIdx.x * 32 + tsa_it) * 4 + (k)] = wall_clock64(); } while (0)
#else
#define CSP_TSA(k) do { } while (0)
#endif

template <int D, int NQB, bool REUSED>
__global__ __launch_bounds__(kSThreads, 2) void score_single_kernel(ScoreParams p) {
#ifdef CSP_SINGLE_TIMING
    long long* const ts_buf = reinterpret_cast<long long*>(p.modbits + bits_rows(p) * bits_words(p) + 2);
    int ts_it = -1;
#endif
#ifdef CSP_SINGLE_TIMING_ALL
    long long* const tsa_buf = reinterpret_cast<long long*>(p.modbits + bits_rows(p) * bits_words(p) + 2);
    int tsa_it = -1;
#endif
    using TG = TileGeom<D>;
    using SM = PipeSmem<D, NQB>;
    constexpr int NQ = NQB * 32, N = NQB * 16, NT = kPipeTiles, EB = 2;
    constexpr int kQFrags = NQB * TG::NK;                               // 1 KiB query fragments
    constexpr int kQLoads = (kQFrags + kSWaves - 1) / kSWaves;          // ... each wavefront requests
    constexpr int kTileLoads = NT * TG::NLD;
        // requests for the next task's keys: a quarter when the MFMAs of the first tile are done (into that tile's
    // buffer), the rest between the exponentials
    // (keys that several tasks stream at the same time come from the L2: no head start, and the back stage first)
    constexpr int kEarlyLoads = REUSED ? 0 : kTileLoads / 4, kLateLoads = kTileLoads - kEarlyLoads;
    static_assert(kEarlyLoads <= TG::NLD, "the early requests go to the first tile");
    constexpr int kQueryLoads = kQLoads;                                // loads per wavefront of request_queries
    // statistics: wavefront w merges rows w*RPW .. of the window part, lane = (row, chunk group)
    constexpr int RPW = NQ / kSWaves;                                   // rows per wavefront: 8 or 4
    constexpr int CG = kWave / RPW;                                     // chunk groups: lane takes chunks cg, cg + CG, ...
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: lives in a scalar register
    const float c = p.scale_log2;
    const float NEG_INF = -__builtin_inff();
    const int64_t tok_bytes = p.k_stride_tok * EB;

    char* const q_lds = smem + SM::off_q;
    float* const stat_lds = reinterpret_cast<float*>(smem + SM::off_stat) + wave * (kPoll * 64);   // this wavefront's rows
    float* const wmax = reinterpret_cast<float*>(smem + SM::off_wmax);
    float* const wsum = reinterpret_cast<float*>(smem + SM::off_wsum);
    _Float16* const fac = reinterpret_cast<_Float16*>(stat_lds);         // second half of the back stage: this wavefront's factor rows
    float* const nl = reinterpret_cast<float*>(smem + SM::off_nl);
    int* const flag = reinterpret_cast<int*>(smem + SM::off_flag);
    uint32_t* const fail = reinterpret_cast<uint32_t*>(smem + SM::off_fail);
    auto tile_ptr = [&](int t4) { return smem + (wave * NT + t4) * TG::TILE_LDS; };
    const uint32_t lds0 = lds_addr(smem);
    auto tile_lds = [&](int t4) { return lds0 + (uint32_t)((wave * NT + t4) * TG::TILE_LDS); };
    // row of the window this lane looks after in the back stage: its reference, its modality, its factor
    // (a part of 32 rows: lanes l and l ^ 16 the same row)
    const int my_row = ((lane & (N - 1)) >> 4) * 32 + acc_row(lane & 15, half);
    // row and chunk group whose statistics this lane merges
    const int st_row = wave * RPW + lane / CG, st_cg = lane % CG;

    // where my_row sits in a factor row, which is laid out in MFMA operand order: contraction index i
    // of lane half h in step (mb, kb) is window row mb*32 + kb*16 + (i/4)*8 + h*4 + i%4
    const int fac_slot = ((lane >> 4) & (NQB - 1)) * 32 + ((lane >> 3) & 1) * 16 + half * 8 + (lane & 7);

    for (int i = tid; i < kFailWords; i += kSThreads) fail[i] = 0u;
    if (tid < 32) reinterpret_cast<uint32_t*>(smem + SM::off_zero)[tid] = 0u;

    auto tile_j0 = [&](const PipeTask& t, int t4) { return t.c0 + (t4 * kSWaves + wave) * kTile; };

    // ---- requests (direct to LDS; every wavefront issues the same number on every path) --------
    // the tiles this wavefront takes of the task's chunk: instruction i of a tile covers rows
    // i*RPI .. of the tile, lane l fills LDS piece (row i*RPI + l/CPR, slot l%CPR), which holds the
    // row's piece slot ^ key(row).  An instruction is addressed as a uniform base (its first row) + a
    // per-lane 32-bit offset (the host sends token strides of 64 MiB and more to the other kernels);
    // in a chunk that lies inside its sequence (all but the last) the offsets repeat every 16 rows and
    // are kept; rows past the end of the sequence re-read its last row.
    constexpr int NV = 16 / TG::RPI;
    uint32_t key_voff[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i)
        key_voff[i] = (uint32_t)(lane / TG::CPR) * (uint32_t)tok_bytes + (uint32_t)(((lane % TG::CPR) ^ TG::key(i * TG::RPI + lane / TG::CPR)) * 16);
    const int64_t row_step = (int64_t)TG::RPI * tok_bytes;   // uniform
    struct KeyCursor { const char* at; int j; };            // uniform: the next instruction's first row, address and index
    // (loads first .. first + count - 1 of the kTileLoads, in the order tile, instruction)
    // ... of a chunk that lies inside its sequence: no branches, so that the requests stay where they
    // are written, between the arithmetic
    auto request_keys_inside = [&](const PipeTask& t, KeyCursor& kc, int first, int count) {
#pragma unroll
        for (int idx = 0; idx < kTileLoads; ++idx) {
            if (idx < first || idx >= first + count) continue;
            const int t4 = idx / TG::NLD, i = idx % TG::NLD;
            if (i == 0) kc.at = t.kbase + (int64_t)tile_j0(t, t4) * tok_bytes;
            load_to_lds_16<!REUSED>(kc.at, key_voff[i % NV], tile_lds(t4) + i * 1024);
            kc.at += row_step;
        }
    };
    // ... of any chunk (the same loads, the same order), in one go
    auto request_keys_ragged = [&](const PipeTask& t, int first, int count) {
        const int ln = opaque(lane);
        const int row_in = ln / TG::CPR;
#pragma unroll
        for (int t4 = 0; t4 < NT; ++t4) {
            const int j0 = tile_j0(t, t4);
#pragma unroll
            for (int i = 0; i < TG::NLD; ++i) {
                if (t4 * TG::NLD + i < first || t4 * TG::NLD + i >= first + count) continue;
                const int first_row = j0 + i * TG::RPI, left = t.L - 1 - first_row;   // uniform: rows of the sequence after the first
                const uint32_t piece = (uint32_t)(((ln % TG::CPR) ^ TG::key(i * TG::RPI + row_in)) * 16);
                const char* const at = t.kbase + (int64_t)(left > 0 ? first_row : t.L - 1) * tok_bytes;
                load_to_lds_16<!REUSED>(at, (uint32_t)min(row_in, max(left, 0)) * (uint32_t)tok_bytes + piece, tile_lds(t4) + i * 1024);
            }
        }
    };
    auto chunk_inside = [&](const PipeTask& t) { return t.c0 + kPipeChunk <= t.L; };   // uniform
    // the queries in MFMA operand order (fragment (mb, s) of lane l at ((mb*NK + s)*64 + l)*16; window
    // rows past the part's last re-read it: finite logits that get weight 0)
    auto request_queries = [&](const PipeTask& t) {
        const int rows = t.rows;
        const char* qpart = t.qpart;
        const int ln = opaque(lane);
#pragma unroll
        for (int k = 0; k < kQLoads; ++k) {
            const int frag = min(k * kSWaves + wave, kQFrags - 1), s_ = frag % TG::NK, mb = frag / TG::NK;   // (a fragment may be requested twice)
            const int row = min(mb * 32 + (ln & 31), rows - 1);
            load_to_lds_16<false>(qpart + s_ * 32, (uint32_t)((row * D + (ln >> 5) * 8) * 2), lds0 + SM::off_q + frag * 1024);
        }
    };
    // the first kPoll chunks of this lane's chunk group of the head's statistics
    auto request_stats = [&](const PipeTask& t) {
        const int rows = t.rows, ncb = rec_chunks(t);
        const int ln = opaque(lane);
        const int row = wave * RPW + ln / CG, cg = ln % CG;
        const float* part = t.stat;
#pragma unroll
        for (int u = 0; u < kPoll; ++u) {
            const int ch = cg + CG * u;
            load_to_lds_4_agent(part, (uint32_t)((ch < ncb ? ch : ncb - 1) * kStatRows + (row < rows ? row : 0)) * 4u, lds0 + SM::off_stat + (wave * kPoll + u) * 256);
        }
    };

    // ---- front stage: logits, statistics and the published log-sum-exp of the chunk ----------
    // The chunk's keys and queries are in LDS.  When this wavefront has read a tile for the last time
    // it may request the next task's: first_tile_done() is called after the MFMAs of the first tile
    // (streamed keys) or of both, after_logits() when the logits are complete, and next_keys(first,
    // count) a few requests at a time between the exponentials (the memory pipeline takes a 1 KiB
    // request every 16 cycles or so: requested in one go they would stall the wavefront for thousands
    // of cycles), or next_keys_ragged(first, count) in one go in front of them where the next chunk is
    // the ragged end of a sequence.  (front_a: up to the per-wavefront maxima and sums in LDS; after a
    // workgroup barrier front_b publishes the chunk's log-sum-exp.)
    // On return pk holds the chunk's weights 2^15 * 2^(c*logit - wavefront maximum of the row) as fp16
    // pairs (pk[t4][mb][h]: accumulator registers 2h, 2h+1 of tile t4, query block mb), ref this
    // lane's row (my_row) of the references (maximum - 15) and win the modalities of the window rows.
    auto front_a = [&](f16x2 (&pk)[NT][NQB][8], float& ref, WindowBits& win, const PipeTask& t, bool next_inside, auto&& next_keys, auto&& next_keys_ragged, auto&& first_tile_done, auto&& after_logits) {
        const int pos0 = t.pos0, c0 = t.c0;
        const WindowBits win_new = (uint32_t)((load_bits64(t, t.pos0) >> my_row) & 1u);   // (the window rows are keys of the sequence)
        // acc[t4][mb][v] = k_j . q_i, j = tile_j0(t4) + acc_row(v, half), i = mb*32 + lane%32: window rows
        // on the lane axis, so that a row's maximum is found within a lane (and its other half) and
        // its sum by an MFMA whose contraction runs over the registers, i.e. over the keys
        f32x16 acc[NT][NQB];
        const f32x16 zero = {};   // (as the addend of an MFMA: a constant operand, no registers to clear)
        // the key operands of contraction step s+1 are requested before the MFMAs of step s are issued
        // (the fences keep the compiler from sinking the fetches back behind the MFMAs to save
        // registers); the other wavefront of the SIMD covers what latency is left
        // piece (s*2 + half) ^ key(r) of row r: the steps differ by an XOR of the byte offset with s*32
        const int ln = opaque(lane);
        const int kaddr0 = (ln & 31) * TG::ROW_BYTES + (((ln >> 5) ^ TG::key(ln & 31)) * 16);
        if constexpr (!REUSED) {
            // tile by tile: the first tile's buffer is free for the next task's keys while the second tile's
            // MFMAs run (the queries are read from LDS once per tile)
            bf16x8 kf[2];
    #pragma unroll
            for (int t4 = 0; t4 < NT; ++t4) {
                kf[0] = *reinterpret_cast<const bf16x8*>(tile_ptr(t4) + kaddr0);
    #pragma unroll
                for (int s_ = 0; s_ < TG::NK; ++s_) {
                    bf16x8 qa[NQB];
    #pragma unroll
                    for (int mb = 0; mb < NQB; ++mb) qa[mb] = *reinterpret_cast<const bf16x8*>(q_lds + ((mb * TG::NK + s_) * 64 + lane) * 16);
                    if (s_ + 1 < TG::NK) kf[(s_ + 1) & 1] = *reinterpret_cast<const bf16x8*>(tile_ptr(t4) + (kaddr0 ^ ((s_ + 1) * 32)));
                    __builtin_amdgcn_sched_barrier(0);
    #pragma unroll
                    for (int mb = 0; mb < NQB; ++mb) acc[t4][mb] = mma(kf[s_ & 1], qa[mb], s_ == 0 ? zero : acc[t4][mb]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (t4 == 0) first_tile_done();
            }
        } else {
            // keys that several tasks stream at the same time come from the L2: no hurry to ask for the next
            // ones, and the queries are read from LDS once per contraction step for both tiles
            bf16x8 kf[2][NT];
            auto fetch_keys = [&](int s_, int b2) {
#pragma unroll
                for (int t4 = 0; t4 < NT; ++t4) kf[b2][t4] = *reinterpret_cast<const bf16x8*>(tile_ptr(t4) + (kaddr0 ^ (s_ * 32)));
            };
            fetch_keys(0, 0);
#pragma unroll
            for (int s_ = 0; s_ < TG::NK; ++s_) {
                bf16x8 qa[NQB];
#pragma unroll
                for (int mb = 0; mb < NQB; ++mb) qa[mb] = *reinterpret_cast<const bf16x8*>(q_lds + ((mb * TG::NK + s_) * 64 + lane) * 16);
                if (s_ + 1 < TG::NK) fetch_keys(s_ + 1, (s_ + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t4 = 0; t4 < NT; ++t4)
#pragma unroll
                    for (int mb = 0; mb < NQB; ++mb) acc[t4][mb] = mma(kf[s_ & 1][t4], qa[mb], s_ == 0 ? zero : acc[t4][mb]);
                __builtin_amdgcn_sched_barrier(0);
            }
            first_tile_done();
        }
        CSP_TS(4);
        // Then the back stage of the task two steps back (whose registers pk, ref and win are about to be
        // reused).  (The requests for the next task's keys start as early as the single tile buffer allows,
        // with first_tile_done(): together the workgroups ask for more in a step than the memory delivers in
        // the part of it that is left after the logits.  More than a quarter of them in one go holds up the
        // wavefront at the memory pipeline for longer than the head start is worth.)
        after_logits();
        // keys past the end, and keys a row may not see (causal tail)
        if (c0 + kPipeChunk > (p.causal ? pos0 : t.L)) {
#pragma unroll
            for (int t4 = 0; t4 < NT; ++t4) {
                // (tile by tile: of the last chunk of a long sequence only the tiles of the window itself need it)
                if (tile_j0(t, t4) + kTile <= (p.causal ? pos0 : t.L)) continue;   // uniform
                const int lm = opaque(lane);   // (here: what follows stays behind the branch)
#pragma unroll
                for (int mb = 0; mb < NQB; ++mb) {
                    const int i = mb * 32 + (lm & 31);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int j = tile_j0(t, t4) + acc_row(v, lm >> 5);
                        const bool ok = j < t.L && (!p.causal || j <= pos0 + i);
                        acc[t4][mb][v] = ok ? acc[t4][mb][v] : NEG_INF;
                    }
                }
            }
        }
        // row maxima over this wavefront's keys: the reference of its exponentials.  A lane has 16
        // keys of each tile for its row, the lane 32 further on the other 16
        float* const wm = wmax + wave * NQ;
        float refs[NQB];
#pragma unroll
        for (int mb = 0; mb < NQB; ++mb) {
            float m = acc[0][mb][0];
#pragma unroll
            for (int t4 = 0; t4 < NT; ++t4)
#pragma unroll
                for (int v = (t4 == 0 ? 1 : 0); v < 16; ++v) m = fmaxf(m, acc[t4][mb][v]);
            m = halves_allreduce<true>(m) * c;
            refs[mb] = (m == NEG_INF ? 0.f : m) - kWeightShift;   // a row that sees none of these keys: every weight is 0 anyway
            wm[mb * 32 + (lane & 31)] = refs[mb];                 // (both halves write the same value)
        }
        CSP_TS(5);
        // weights in place of the logits, as fp16 (half the registers; 11 bits are within the tolerance,
        // and the scale keeps small weights normal).  Per block of 32 keys x 32 rows: the row sums are
        // MFMAs of the block with a matrix of ones (the contraction runs over a lane's registers: keys), and an
        // MFMA of the block with a permutation matrix hands every weight, unchanged, to the lane of its
        // key (the layout in which the back stage contracts over the window rows): what the vector ALU
        // does per weight is one FMA, one exponential and two conversions.
        auto weights = [&](auto interleave) {
            constexpr int kIters = NQB * NT * 4;
            const int lw = opaque(lane);
            const f16x4 ones = {(_Float16)1.f, (_Float16)1.f, (_Float16)1.f, (_Float16)1.f};
            f16x8 perm_lo, perm_hi;   // perm_lo/hi[e]: accumulator register e (8 + e) of this half is key lane%32 of the tile
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                perm_lo[e] = acc_row(e, lw >> 5) == (lw & 31) ? (_Float16)1.f : (_Float16)0.f;
                perm_hi[e] = acc_row(8 + e, lw >> 5) == (lw & 31) ? (_Float16)1.f : (_Float16)0.f;
            }
#pragma unroll
            for (int mb = 0; mb < NQB; ++mb) {
                f32x4 sums = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t4 = 0; t4 < NT; ++t4) {
                    f16x2 wt[8];
#pragma unroll
                    for (int v4 = 0; v4 < 4; ++v4) {
                        if constexpr (decltype(interleave)::value) {
                            const int idx = (mb * NT + t4) * 4 + v4;
                            const int first = kEarlyLoads + idx * kLateLoads / kIters, count = kEarlyLoads + (idx + 1) * kLateLoads / kIters - first;
                            __builtin_amdgcn_sched_barrier(0);   // (here, not all of them ahead of the arithmetic)
                            next_keys(first, count);
                            __builtin_amdgcn_sched_barrier(0);
                        }
#pragma unroll
                        for (int u = 0; u < 4; u += 2) {
                            const int v = v4 * 4 + u;
                            const f32x2 two = {fast_exp2(fmaf(acc[t4][mb][v], c, -refs[mb])), fast_exp2(fmaf(acc[t4][mb][v + 1], c, -refs[mb]))};
                            wt[v >> 1] = __builtin_convertvector(two, f16x2);
                        }
                    }
                    const f16x8 w_lo = __builtin_shufflevector(__builtin_shufflevector(wt[0], wt[1], 0, 1, 2, 3), __builtin_shufflevector(wt[2], wt[3], 0, 1, 2, 3), 0, 1, 2, 3, 4, 5, 6, 7);
                    const f16x8 w_hi = __builtin_shufflevector(__builtin_shufflevector(wt[4], wt[5], 0, 1, 2, 3), __builtin_shufflevector(wt[6], wt[7], 0, 1, 2, 3), 0, 1, 2, 3, 4, 5, 6, 7);
                    // (v_mfma_f32_4x4x4_16b_f16: sixteen 4x4 products per instruction; with a matrix of ones on the
                    // left every row of a lane's result is the sum of the lane's own four values)
#pragma unroll
                    for (int h = 0; h < 8; h += 2)
                        sums = __builtin_amdgcn_mfma_f32_4x4x4f16(ones, __builtin_shufflevector(wt[h], wt[h + 1], 0, 1, 2, 3), sums, 0, 0, 0);
                    f32x16 d = mma_f16(w_lo, perm_lo, zero);
                    d = mma_f16(w_hi, perm_hi, d);
#pragma unroll
                    for (int h = 0; h < 8; ++h) {
                        const f32x2 two = {d[2 * h], d[2 * h + 1]};
                        pk[t4][mb][h] = __builtin_convertvector(two, f16x2);
                    }
                }
                wsum[wave * NQ + mb * 32 + (lane & 31)] = halves_allreduce<false>(sums[0]);   // (the lane 32 further on has the row's other keys)
            }
        };
        if (next_inside) {
            weights(Interleaved<true>{});
        } else {
            next_keys_ragged(kEarlyLoads, kLateLoads);
            weights(Interleaved<false>{});
        }
        wave_lds_sync();
        ref = wm[my_row];
        win = win_new;
        CSP_TS(6);
    };
    auto front_b = [&](const PipeTask& t) {
        const int rows = t.rows;
        {
            // log-sum-exp of the chunk per row (-inf when the row sees none of its keys): wavefront w
            // takes rows w*RPW .., lane = (row, wavefront whose maximum and sum it brings in)
            const bool has = st_cg < kSWaves;
            const int at = (has ? st_cg : 0) * NQ + st_row;
            const float pm = has ? wmax[at] : NEG_INF, ps = has ? wsum[at] : 0.f;
            const float M = group_allreduce<CG, true>(pm);
            const float l = group_allreduce<CG, false>(ps * fast_exp2(pm - M));
            const float lse_c = l > 0.f ? M + fast_log2(l) : NEG_INF;
            if (st_cg == 0 && st_row < rows)
                __hip_atomic_store((__attribute__((address_space(1))) float*)(t.stat + (size_t)(t.c0 / kPipeChunk) * kStatRows + st_row), lse_c,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };

    // ---- back stage: the head's statistics, weights, column sums, scores ----------------------
    // The first round of statistics and the key modalities are in LDS.  back_a merges the statistics of
    // this wavefront's rows into the rows' log-sum-exp (LDS) and notes whether its wait ran out; after a
    // workgroup barrier back_b turns the waiting weights into scores and stores them, or returns false
    // (uniform) when some wavefront's wait ran out.
    auto back_a = [&](const PipeTask& t, int64_t spin) {
        const int rows = t.rows, n_chunks_b = rec_chunks(t);
        // (the few loads that the compiler sees, on the paths that are rarely taken: it waits for them
        // where their values are used, and with them for every load in flight)
        typedef const __attribute__((address_space(1))) float* GlobalStat;
        const GlobalStat part = (GlobalStat)(t.stat + (st_row < rows ? st_row : 0));
        auto load_stat = [&](int ch) {
            return __hip_atomic_load(part + (size_t)(ch < n_chunks_b ? ch : n_chunks_b - 1) * kStatRows, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        };
        // log-sum-exp of row st_row over the chunks st_cg, st_cg + CG, ... (then over the chunk groups)
        float M = NEG_INF, Ls = 0.f;
        bool ok = true, started = false;
        uint64_t t_start = 0;
        for (int cb = 0; cb < n_chunks_b; cb += CG * kPoll) {
            float rr[kPoll];
            if (cb == 0) {
#pragma unroll
                for (int u = 0; u < kPoll; ++u) rr[u] = stat_lds[u * 64 + lane];
            } else {
#pragma unroll
                for (int u = 0; u < kPoll; ++u) rr[u] = load_stat(cb + st_cg + CG * u);
                // used here: the wait for them stays on this path
#pragma unroll
                for (int u = 0; u < kPoll; ++u) asm volatile("" : "+v"(rr[u]));
            }
            auto pending = [&]() {   // per wavefront: is a statistic of its rows still missing
                bool miss = false;
#pragma unroll
                for (int u = 0; u < kPoll; ++u) {
                    if (cb + st_cg + CG * u >= n_chunks_b) rr[u] = NEG_INF;
                    miss |= (__builtin_bit_cast(uint32_t, rr[u]) & 0x7fffffffu) > 0x7f800000u;   // (a NaN; the file is compiled without them)
                }
                return __any(miss) != 0;
            };
            // the usual case: everything was published a step ago
            if (pending()) {
                if (!started) { t_start = wall_clock64(); started = true; }
                for (;;) {
                    // bounded: a wavefront that has waited too long stops depending on the others
                    if (spin <= 0 || wall_clock64() - t_start > (uint64_t)spin) { ok = false; break; }
                    __builtin_amdgcn_s_sleep(4);
#pragma unroll
                    for (int u = 0; u < kPoll; ++u) rr[u] = load_stat(cb + st_cg + CG * u);
                    if (!pending()) break;
                }
            }
            if (!ok) break;
            float Mn = M;
#pragma unroll
            for (int u = 0; u < kPoll; ++u) Mn = fmaxf(Mn, rr[u]);
            const float Mns = Mn == NEG_INF ? 0.f : Mn;
            if (cb > 0) Ls *= fast_exp2(M - Mns);   // (uniform; Ls is 0 in the first round)
#pragma unroll
            for (int u = 0; u < kPoll; ++u) Ls += fast_exp2(rr[u] - Mns);
            M = Mn;
        }
        // ... over the CG lanes of the row (a fixed tree: the result does not depend on who waited)
        {
            const float Mrow = group_allreduce<CG, true>(M);
            Ls = group_allreduce<CG, false>(Ls * fast_exp2(M - (Mrow == NEG_INF ? 0.f : Mrow)));
            M = Mrow;
        }
        if (lane == 0) flag[wave] = ok ? 1 : 0;
        if (st_cg == 0 && ok) {   // chunk 0 holds a visible key: M is finite
            const float Lh = fmaf(p.n_score, fast_exp2(-M), Ls);  // the n of the n-softmax, in the same scaled units
            nl[st_row] = st_row < rows ? M + fast_log2(Lh) : __builtin_inff();   // rows past the window: weight 0
        }
    };
    auto back_b = [&](const f16x2 (&pk)[NT][NQB][8], float ref, const WindowBits& win, const PipeTask& t) -> bool {
        bool all_ok = true;
#pragma unroll
        for (int w = 0; w < kSWaves; ++w) all_ok = all_ok && flag[w] != 0;
        if (!all_ok) return false;
        // Column sums on the matrix cores: (factor rows) x (weights).  The weights are the B operand as
        // they sit (keys on the lane axis; per lane and step 8 window rows).  The factor of this lane's
        // row, 2^(reference - lse), scaled into fp16's range and split into two fp16 (22 bits), goes to
        // rows 0 and 1 of the A operand when the row is a text query, to rows 2 and 3 when it is a visual
        // one; the other rows are zero.  Rows 0..3 of the product are the sums over the text rows (two
        // parts) and over the visual rows (two parts) for the 32 keys of the tile.
        {
            const float f = fast_exp2((ref + kFactorShift) - nl[my_row]);
            const _Float16 hi = (_Float16)f;
            const _Float16 lo = (_Float16)(f - (float)hi);
            const _Float16 z = (_Float16)0.f;
            const bool tx = win == 0;
            fac[0 * NQ + fac_slot] = tx ? hi : z;
            fac[1 * NQ + fac_slot] = tx ? lo : z;
            fac[2 * NQ + fac_slot] = tx ? z : hi;
            fac[3 * NQ + fac_slot] = tx ? z : lo;
        }
        wave_lds_sync();
        f32x16 cs[NT];
        const f32x16 zero = {};
        {
            const int ln = opaque(lane);
            const char* const fr = (ln & 31) < 4 ? reinterpret_cast<const char*>(fac) + (ln & 31) * (NQ * 2) + (ln >> 5) * 16 : smem + SM::off_zero;
#pragma unroll
            for (int mb = 0; mb < NQB; ++mb)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const f16x8 fa = *reinterpret_cast<const f16x8*>(fr + mb * 64 + kb * 32);
#pragma unroll
                    for (int t4 = 0; t4 < NT; ++t4) {
                        const PkQuad w = {{pk[t4][mb][4 * kb], pk[t4][mb][4 * kb + 1], pk[t4][mb][4 * kb + 2], pk[t4][mb][4 * kb + 3]}};
                        cs[t4] = mma_f16(fa, __builtin_bit_cast(f16x8, w), mb + kb == 0 ? zero : cs[t4]);
                    }
                }
        }
        // lanes 0-31 hold rows 0..3 of the product for key `lane` of each tile: they store its two scores
        // (32 consecutive floats per tile and array)
        if (half == 0) {
            typedef __attribute__((address_space(1))) float* GlobalScore;
            const int rank_end = t.L - p.R;  // keys >= rank_end are not ranked
#pragma unroll
            for (int t4 = 0; t4 < NT; ++t4) {
                const float ct = (cs[t4][0] + cs[t4][1]) * kFactorUnshift;   // over the text window rows
                const float cv = (cs[t4][2] + cs[t4][3]) * kFactorUnshift;   // over the visual window rows
                const bool key_text = ((load_bits(t.kbits + t4 * kSWaves + wave) >> lane) & 1u) == 0;   // (lane < 32 here)
                const int j = tile_j0(t, t4) + lane;
                const bool ranked = j < rank_end;
                if (j < t.L) {
                    const GlobalScore out_self = (GlobalScore)(t.out_self + j);
                    out_self[0] = ranked ? (key_text ? ct : cv) : 0.f;
                    out_self[p.cross_delta] = ranked ? (key_text ? cv : ct) : 0.f;
                }
            }
        }
        return true;
    };

    // ---- the pipeline -------------------------------------------------------------------------
    // Loads of a step, in issue order (per wavefront): the first kEarlyLoads of the next task's key
    // tiles, the statistics of the task one step back, the other kLateLoads of the key tiles, the
    // next task's queries (kQueryLoads).  Two workgroup barriers per step: at its start and between
    // the halves of the front stage.
    f16x2 pkA[NT][NQB][8], pkB[NT][NQB][8];
    float refA = 0.f, refB = 0.f;
    WindowBits winA = 0u, winB = 0u;
    const int nwg = gridDim.x;
    // record of this workgroup's task of step `it` (steps past the last: the record that is not valid)
    auto rec_of = [&](int it) { return p.table + (it >= 0 && it < p.n_iters ? min(it * nwg + (int)blockIdx.x, p.n_lin) : p.n_lin); };
    {
        const PipeTask t0 = load_rec(rec_of(0));
        request_queries(t0);
        request_keys_ragged(t0, 0, kTileLoads);
        wait_loads<0>();
    }
    // One step, for the tasks it, it - 1 and it - 2 of this workgroup: logits of task it; the scores of
    // task it - 2 from its waiting weights and the log-sum-exps merged in the previous step (reused
    // keys: the scores first); maxima, weights and sums of task it; barrier; its log-sum-exp
    // published; the published ones of task it - 1 merged.  What a workgroup publishes in a step is looked for by the others in their next step,
    // after they have published their own: they may be most of a step apart without anybody waiting.
    // The weights of a task are consumed right before the registers are filled with those of the task
    // two steps on.  Records are fetched where they are needed (a scalar load each) rather than
    // kept: scalar registers are scarce.
    auto step = [&](f16x2 (&pk)[NT][NQB][8], float& ref, WindowBits& win, int it) {
#ifdef CSP_SINGLE_TIMING
        ts_it = it;
#endif
#ifdef CSP_SINGLE_TIMING_ALL
        tsa_it = it;
#endif
        CSP_TS(0);
        lds_barrier();   // the front task's queries have landed for every wavefront; the rows' log-sum-exps of task it - 2 are in LDS
        CSP_TS(1);
        CSP_TSA(0);
        const PipeTask tn = load_rec(rec_of(it + 1));
        // (past the last task the record that is not valid is requested all the same: skipping those loads
        // makes the launch 2-5 us longer, measured)
        const bool next_inside = chunk_inside(tn);
        KeyCursor kcn;
        auto keys_next = [&](int first, int count) { request_keys_inside(tn, kcn, first, count); };
        auto keys_next_ragged = [&](int first, int count) { request_keys_ragged(tn, first, count); };
        auto first_tile_done = [&]() {
            if (next_inside) keys_next(0, kEarlyLoads);
            else keys_next_ragged(0, kEarlyLoads);
        };
        auto after_logits = [&]() {
            CSP_TS(2);
            const PipeTask tb = load_rec(rec_of(it - 2));
            if (tb.valid && !back_b(pk, ref, win, tb) && tid == 0) {
                fail[(it - 2) >> 5] |= 1u << ((it - 2) & 31);
                atomicAdd(p.counters, 1);
            }
            request_stats(load_rec(rec_of(it - 1)));
            CSP_TS(3);
        };
        auto nothing = [&]() {};
        if constexpr (REUSED) after_logits();
        const PipeTask tf = load_rec(rec_of(it));
        if (tf.valid) {
            if constexpr (REUSED) front_a(pk, ref, win, tf, next_inside, keys_next, keys_next_ragged, nothing, nothing);
            else front_a(pk, ref, win, tf, next_inside, keys_next, keys_next_ragged, first_tile_done, after_logits);
        } else {
            if constexpr (!REUSED) {
                first_tile_done();
                after_logits();
            }
            keys_next_ragged(kEarlyLoads, kLateLoads);
        }
        CSP_TS(7);
        lds_barrier();   // every wavefront is done with the queries; its maxima and sums are in LDS
        CSP_TS(8);
        request_queries(tn);
        if (tf.valid) front_b(tf);
        CSP_TS(9);
        CSP_TSA(3);
        wait_loads<kLateLoads + kQueryLoads>();   // the statistics of task it - 1 have landed (younger: the later keys, the queries)
        CSP_TS(10);
        CSP_TSA(1);
        {
            const PipeTask tm = load_rec(rec_of(it - 1));
            if (tm.valid) back_a(tm, p.spin_ticks);
        }
        CSP_TS(11);
        CSP_TSA(2);
        wait_loads<0>();   // the next task's keys and queries (this wavefront's) have landed
        CSP_TS(12);
        CSP_TS(13);
        CSP_TS(14);
    };
    for (int it = 0; it <= p.n_iters + 1; it += 2) {
        step(pkA, refA, winA, it);
        step(pkB, refB, winB, it + 1);
    }

    // ---- tasks whose wait ran out: every chunk's statistics recomputed here, own chunk last ----
    lds_barrier();
    for (int it = 0; it < p.n_iters; ++it) {
        if (!((fail[it >> 5] >> (it & 31)) & 1u)) continue;   // uniform
        const PipeTask t = load_rec(rec_of(it));
        const int ncb = rec_chunks(t), own = t.c0 / kPipeChunk;
        auto no_keys = [&](int, int) {};
        auto no_keys_ragged = [&](int, int) {};
        auto nothing = [&]() {};
        for (int k = 0; k < ncb; ++k) {
            PipeTask ty = t;   // the chunks of a head part differ in their first key only
            ty.c0 = (k < ncb - 1 ? (k < own ? k : k + 1) : own) * kPipeChunk;
            lds_barrier();
            request_queries(ty);
            request_keys_ragged(ty, 0, kTileLoads);
            wait_loads<0>();
            lds_barrier();
            front_a(pkA, refA, winA, ty, false, no_keys, no_keys_ragged, nothing, nothing);
            lds_barrier();
            front_b(ty);
        }
        wait_loads<0>();   // this wavefront's own stores of the statistics are complete (it reads back its own rows)
        lds_barrier();
        request_stats(t);
        wait_loads<0>();
        back_a(t, (int64_t)1 << 40);
        lds_barrier();
        back_b(pkA, refA, winA, t);
    }
}

template <int D, int NQB>
hipError_t launch_single_typed(const ScoreParams& p, int n_wg, hipStream_t s) {
    // several tasks stream the same keys at the same time (GQA heads, window parts): plain loads that stay in L2
    auto k = p.G * p.vsplit > 1 ? score_single_kernel<D, NQB, true> : score_single_kernel<D, NQB, false>;
    const size_t n_stats = (size_t)p.B * p.H_q * p.vsplit * p.n_chunks * kStatRows;
    const size_t n_bits = bits_rows(p) * bits_words(p) * 32;   // a thread per key
    size_t n_setup = n_stats > (size_t)p.n_lin + 1 ? n_stats : (size_t)p.n_lin + 1;
    if (n_bits > n_setup) n_setup = n_bits;
    hipLaunchKernelGGL(score_single_setup_kernel, dim3((unsigned)((n_setup + 255) / 256)), dim3(256), 0, s, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int smem = PipeSmem<D, NQB>::total;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k, dim3((unsigned)n_wg), dim3(kSThreads), (size_t)smem, s, p);
    return hipGetLastError();
}

}  // namespace

// Workgroups of the launch: one per compute unit of the current device.
static int compute_units() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 0;
        cached[dev] = n;
    }
    return cached[dev];
}

// Fills in the task list of `p` (n_tasks, n_lin, n_iters) and launches; returns hipErrorNotReady when the
// shape does not fit this device after all (the caller then takes the two-pass kernels).
hipError_t launch_score_single(ScoreParams& p, int D, hipStream_t s) {
    const int cus = compute_units();
    if (cus <= 0) return hipErrorInvalidDevice;
    const int share = p.G * p.vsplit;
    p.n_tasks = share * p.n_chunks * p.view.H_kv * p.B;
    p.n_lin = (p.n_tasks + 8 * share - 1) / (8 * share) * (8 * share);
    const int n_wg = p.n_lin < cus ? p.n_lin : cus;
    p.n_iters = (p.n_lin + n_wg - 1) / n_wg;
    // the chunks of the heads that share a KV head must be at most one step apart
    // (and the kernel addresses a key row as a 32-bit offset from the first row of its load instruction)
    if ((int64_t)share * p.n_chunks > n_wg || p.n_iters > kScoreSingleMaxIters || p.k_stride_tok >= ((int64_t)1 << 25)) return hipErrorNotReady;
    // the task table follows the statistics in the workspace
    const size_t n_stats = (size_t)p.B * p.H_q * p.vsplit * p.n_chunks * kStatRows;
    p.table = reinterpret_cast<PipeRec*>(reinterpret_cast<char*>(p.part) + ((n_stats * sizeof(float) + 15) & ~(size_t)15));
    p.modbits = reinterpret_cast<uint32_t*>(p.table + p.n_lin + 1);
    p.cross_delta = (p.gsplit > 1 ? p.slice_cross - p.slice_self : p.score_cross - p.score_self);
    p.D = D;
    const int rows = p.O < kStatRows ? p.O : kStatRows;
    if (D == 128) return rows <= 32 ? launch_single_typed<128, 1>(p, n_wg, s) : launch_single_typed<128, 2>(p, n_wg, s);
    return rows <= 32 ? launch_single_typed<64, 1>(p, n_wg, s) : launch_single_typed<64, 2>(p, n_wg, s);
}

}  // namespace csp
