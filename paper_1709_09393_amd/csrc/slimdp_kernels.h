// Kernels of libslimdp (gfx950).  Included only by slimdp.hip.
//
// Shared structure: the index range is cut into tiles of <= 4096 parameters (never across
// a segment).  Exact "top-need by (key desc, index asc)" selection, used both for the core
// (keys = score bits) and for the explorer (keys = bound - Philox word over the non-core
// parameters), is a three-level radix descent:
//   level 0 histogram over every key (fused into the kernel that produces the keys),
//   -> keys in the threshold bin become "candidates": a per-tile bitmap plus the candidate
//      keys of each 1024-parameter sub-tile compacted in index order at
//      cand_keys[tile_start + 1024*s ...] with their number in cnt_cand[4*tile + s]
//      (a sub-tile is what one wave handles on its own, without block barriers),
//   levels 1 and 2 histogram only candidates, giving the threshold key tau and the number
//   of keys == tau to take (quota, lowest index first),
//   count per tile -> scan over tiles -> ordered emission of the ascending index list.
#pragma once
#include "slimdp_device.h"

// Cache policy of the streaming accesses, per kernel (0 = default, 1 = non-temporal).  Measured on the VGG-16-sized
// workload: each switch alone moves its kernel by 0 to 5 %, all together take 0.07 ms off the 2.75 ms step.
#ifndef NT_BUILD
#define NT_BUILD 1
#endif
#ifndef NT_MERGE_LD
#define NT_MERGE_LD 1
#endif
#ifndef NT_MERGE_ST
#define NT_MERGE_ST 1
#endif
#ifndef NT_MERGE_VAL
#define NT_MERGE_VAL 1
#endif
#ifndef NT_PACKS
#define NT_PACKS 1
#endif
#ifndef NT_PACKC_LD
#define NT_PACKC_LD 1
#endif
#ifndef NT_PACKC_ST
#define NT_PACKC_ST 1
#endif
#ifndef NT_EXPLG
#define NT_EXPLG 1
#endif

namespace slimdp {

// ---------------------------------------------------------------------------------------
// small utilities
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_fill_u32(uint32_t* __restrict__ p, uint64_t count, uint32_t v)
{
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (uint64_t)gridDim.x * 256)
        p[i] = v;
}

// Tile tables of a flat model of n parameters, and the 64 flag words cleared (for a workspace that keeps the
// contents of an earlier, differently sized call).  grid ceil((T+1)/256).
__global__ __launch_bounds__(256) void k_flat_tables(uint32_t* __restrict__ tile_start, uint32_t* __restrict__ tile_seg,
                                                     uint32_t* __restrict__ seg_first_tile, uint32_t* __restrict__ flags,
                                                     uint32_t T, uint32_t n)
{
    const uint32_t t = blockIdx.x * 256 + threadIdx.x;
    if (t < T) { tile_start[t] = t * TILE; tile_seg[t] = 0; }
    if (t == T) { tile_start[T] = n; seg_first_tile[0] = 0; seg_first_tile[1] = T; }
    if (t < 64) flags[t] = 0;
}

// Writes the selection state of segments [seg0, seg0+count) for every batch.
// core != 0: fixed score-bit levels; else explorer levels derived from (bound_m1, shift0).
// Several fills in one launch (a launch costs more than a small fill).
struct FillJobs { uint32_t* p[4]; uint64_t count[4]; uint32_t v[4]; };
__global__ __launch_bounds__(256) void k_fill_multi(FillJobs jobs)
{
#pragma unroll
    for (int j = 0; j < 4; ++j)
        for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < jobs.count[j]; i += (uint64_t)gridDim.x * 256)
            jobs.p[j][i] = jobs.v[j];
}

__global__ __launch_bounds__(256) void k_init_state(SegState* __restrict__ st, SegInitChunk chunk, uint32_t seg0,
                                                    uint32_t count, uint32_t n_seg, uint32_t nbatch, int core)
{
    const uint32_t x = blockIdx.x * 256 + threadIdx.x;
    if (x >= count * nbatch) return;
    const uint32_t b = x / count, j = x % count;
    const SegInit in = chunk.s[j];
    SegState s;
    s.need0 = in.need; s.need = in.need; s.prefix = 0; s.none = (in.need == 0) ? 1u : 0u;
    s.tau = NONE; s.quota = 0; s.bound_m1 = in.bound_m1; s.tie_all = 0;
    s.sure_m1 = in.sure_m1; s.has_gt = core ? 1u : in.has_gt;
    if (core) {
        s.shift[0] = CORE_SHIFT0; s.nbins[0] = CORE_NB0;
        s.shift[1] = CORE_SHIFT1; s.nbins[1] = CORE_NB1;
        s.shift[2] = 0;           s.nbins[2] = CORE_NB2;
    } else {
        // explorer keys are bound_m1 - r for the words sure_m1 < r <= bound_m1 (all r <= bound_m1 without a sure zone)
        const uint32_t width_m1 = in.has_gt ? in.bound_m1 - in.sure_m1 - 1u : in.bound_m1;
        const uint32_t sh0 = in.shift0;
        const uint32_t bits1 = sh0 < 12u ? sh0 : 12u;
        const uint32_t sh1 = sh0 - bits1;
        s.shift[0] = sh0; s.nbins[0] = (width_m1 >> sh0) + 1u;
        s.shift[1] = sh1; s.nbins[1] = 1u << bits1;
        s.shift[2] = 0;   s.nbins[2] = 1u << sh1;
    }
    st[(size_t)b * n_seg + seg0 + j] = s;
}

// ---------------------------------------------------------------------------------------
// K4: the explorer draw of one (worker, sub-tile), by ONE wave with no block barrier: the
// Philox word r of each parameter, sorted into two zones chosen on the host so that the
// m-th smallest word of the segment falls into the second one:
//   sure zone       r <= sure_m1 (if has_sure): one bit in the "sure" bitmap; such a
//                   parameter is taken unless it turns out to be in the core;
//   candidate zone  sure_m1 < r <= bound_m1: one bit in the candidate bitmap plus the key
//                   bound_m1 - r (the smallest words are the largest keys), the keys of a
//                   sub-tile compacted in index order.
// The draw does not look at the core; a later pass applies it, so the same routine serves
// inside the scoring kernel (core not known yet) and stand-alone.
// PAIRS = 1 (every segment's candidate zone is narrow): no candidate bitmap; the sub-tile's
// slot holds (key, offset inside the sub-tile) pairs, at most PAIR_CAP of them: the count still
// reports any beyond, which the gathering pass turns into the exact rerun.
// wa, wb, wp: 32 words of LDS each, private to the calling wave (generic variant only).
// ---------------------------------------------------------------------------------------
struct PhiloxKey { uint32_t seed_lo, seed_hi, it_lo, it_hi; };
// PAIRS = 1: a sub-tile's (key, offset) pairs live in a slot of PAIR_SLOT words at
// cand_keys[(tile * SUBS + sub-tile) * PAIR_SLOT]: PAIR_CAP pairs, about a hundred times the expected number.
constexpr uint32_t PAIR_CAP = 16, PAIR_SLOT = 2 * PAIR_CAP;
struct DrawOut {                 // per batch (worker) base pointers
    uint32_t* sure_bits;         // [T * TILE_WORDS]
    uint32_t* cand_bits;         // [T * TILE_WORDS]
    uint32_t* cand_keys;         // [keys_stride]
    uint32_t* cnt_cand;          // [T * SUBS]
};

// LDS traffic between the lanes of one wave: the hardware keeps a wave's LDS operations in
// order, this keeps the compiler from moving them across the hand-over point.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_wave_barrier();
}

// Any tile start (tiles of a segmented model may begin inside a Philox block).
template <int PAIRS>
__device__ __forceinline__ void explore_subtile(uint32_t worker, uint32_t t, uint32_t sub, uint32_t start, uint32_t len,
                                                uint32_t bound_m1, uint32_t sure_m1, uint32_t has_sure, uint32_t skip,
                                                uint32_t* wa, uint32_t* wb, uint32_t* wp, DrawOut out, PhiloxKey pk)
{
    const uint32_t lane = lane_id();
    const uint32_t off = sub * SUB;
    const uint32_t sub_len = (len > off) ? ((len - off < SUB) ? len - off : SUB) : 0u;
    const size_t wbase = (size_t)t * TILE_WORDS + sub * SUB_WORDS;
    if (sub_len == 0 || skip) {                                   // uniform over the wave
        if (lane < SUB_WORDS) {
            if (!PAIRS) out.cand_bits[wbase + lane] = 0;
            out.sure_bits[wbase + lane] = 0;
        }
        if (lane == 0) out.cnt_cand[(size_t)t * SUBS + sub] = 0;
        return;
    }
    if (lane < SUB_WORDS) { wa[lane] = 0; wb[lane] = 0; }
    wave_sync();
    const uint32_t base = start + off;
    const uint32_t g0 = base >> 2, g1 = (base + sub_len - 1u) >> 2;     // Philox blocks touched: at most 257
    uint32_t key[5][4];
    uint32_t is_cand = 0;
#pragma unroll
    for (int it = 0; it < 5; ++it) {
        if (g1 - g0 < (uint32_t)it * 64u) break;                   // uniform: the 5th round only for unaligned starts
        const uint32_t gi = g0 + (uint32_t)it * 64u + lane;
        if (gi <= g1) {
            uint32_t r[4];
            philox4x32_10(gi, worker, pk.it_lo, pk.it_hi, pk.seed_lo, pk.seed_hi, r);
            const uint32_t i0 = gi << 2;
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const uint32_t e = i0 + cc - base;                  // wraps below the sub-tile start
                key[it][cc] = bound_m1 - r[cc];
                if (e < sub_len) {
                    if (has_sure && r[cc] <= sure_m1) atomicOr(&wa[e >> 5], 1u << (e & 31));
                    else if (r[cc] <= bound_m1) {
                        atomicOr(&wb[e >> 5], 1u << (e & 31));
                        is_cand |= 1u << (it * 4 + cc);
                    }
                }
            }
        }
    }
    wave_sync();
    const uint32_t cw = (lane < SUB_WORDS) ? wb[lane] : 0u;
    const uint32_t pc = __popc(cw);
    const uint32_t incl = wave_incl_scan(pc);
    if (lane < SUB_WORDS) {
        wp[lane] = incl - pc;
        if (!PAIRS) out.cand_bits[wbase + lane] = cw;
        out.sure_bits[wbase + lane] = wa[lane];
    }
    if (lane == SUB_WORDS - 1) out.cnt_cand[(size_t)t * SUBS + sub] = incl;
    wave_sync();
    if (is_cand) {
#pragma unroll
        for (int it = 0; it < 5; ++it) {
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                if (is_cand & (1u << (it * 4 + cc))) {
                    const uint32_t gi = g0 + (uint32_t)it * 64u + lane;
                    const uint32_t e = (gi << 2) + cc - base;
                    const uint32_t rank = wp[e >> 5] + __popc(wb[e >> 5] & mask_below(e & 31));
                    if (!PAIRS) out.cand_keys[(size_t)base + rank] = key[it][cc];
                    else if (rank < PAIR_CAP) {
                        out.cand_keys[((size_t)t * SUBS + sub) * PAIR_SLOT + 2u * rank] = key[it][cc];
                        out.cand_keys[((size_t)t * SUBS + sub) * PAIR_SLOT + 2u * rank + 1u] = e;
                    }
                }
            }
        }
    }
    wave_sync();
}

// Which of a lane's four parameters e0 .. e0+3 lie inside a ragged sub-tile of sub_len parameters.
__device__ __forceinline__ uint32_t inside_mask(uint32_t e0, uint32_t sub_len)
{
    const uint32_t left = (e0 < sub_len) ? sub_len - e0 : 0u;
    return (left >= 4u) ? 15u : ((1u << left) - 1u);
}

// The same for a sub-tile that starts on a Philox block (start + 1024*sub divisible by 4):
// no LDS at all.  Round `it` covers the 256 parameters [256*it, 256*it+256) of the sub-tile
// in index order (lane L owns parameters 4L..4L+3 of the round), so a candidate's place in
// the key list is the number of candidates in earlier rounds plus a wave ballot count, and
// the eight bitmap words of the round are OR-reductions over groups of eight lanes.
// KEYS: PhiloxKey, or PhiloxRoundKeys of a caller that draws under one key many times (pk then only names the iteration).
__device__ __forceinline__ void philox_words(uint32_t c0, uint32_t worker, const PhiloxKey& pk, const PhiloxKey&, uint32_t r[4])
{
    philox4x32_10(c0, worker, pk.it_lo, pk.it_hi, pk.seed_lo, pk.seed_hi, r);
}
__device__ __forceinline__ void philox_words(uint32_t c0, uint32_t worker, const PhiloxKey& pk, const PhiloxRoundKeys& rk, uint32_t r[4])
{
    philox4x32_10(c0, worker, pk.it_lo, pk.it_hi, rk, r);
}
template <int PAIRS, class KEYS = PhiloxKey>
__device__ __forceinline__ void explore_subtile_fast(uint32_t worker, uint32_t t, uint32_t sub, uint32_t start, uint32_t len,
                                                     uint32_t bound_m1, uint32_t sure_m1, uint32_t has_sure, uint32_t skip,
                                                     DrawOut out, PhiloxKey pk, const KEYS& keys)
{
    const uint32_t lane = lane_id();
    const uint32_t off = sub * SUB;
    const uint32_t sub_len = (len > off) ? ((len - off < SUB) ? len - off : SUB) : 0u;
    // the sub-tile's bitmap words and count through descriptors (t and sub are the same for the whole wave): scalar bases,
    // no per-lane 64-bit addresses that a caller's loop over workers would have to carry along
    const __amdgpu_buffer_rsrc_t rc = buffer_of(out.cand_bits + (size_t)t * TILE_WORDS + sub * SUB_WORDS, SUB_WORDS * 4u);
    const __amdgpu_buffer_rsrc_t rs = buffer_of(out.sure_bits + (size_t)t * TILE_WORDS + sub * SUB_WORDS, SUB_WORDS * 4u);
    const __amdgpu_buffer_rsrc_t rn = buffer_of(out.cnt_cand + (size_t)t * SUBS + sub, 4u);
    if (sub_len == 0 || skip) {                                   // uniform over the wave
        if (lane < SUB_WORDS) {
            if (!PAIRS) buffer_store1(rc, lane * 4u, 0u);
            buffer_store1(rs, lane * 4u, 0u);
        }
        if (lane == 0) buffer_store1(rn, 0u, 0u);
        return;
    }
    const uint32_t base = start + off;
    uint32_t* ckeys = PAIRS ? out.cand_keys + ((size_t)t * SUBS + sub) * PAIR_SLOT : out.cand_keys + (size_t)base;
    const uint32_t sure_excl = has_sure ? sure_m1 + 1u : 0u;         // sure_m1 < bound_m1: no overflow
    const uint32_t width_m1 = bound_m1 - sure_excl;                  // candidate words are sure_excl .. bound_m1
    uint32_t run = 0, sword = 0, cword = 0;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const uint32_t e0 = (uint32_t)it * 256u + lane * 4u;      // first of this lane's four parameters
        uint32_t r[4];
        philox_words((base + e0) >> 2, worker, pk, keys, r);
        // sure flags of the four parameters, without branches (word below sure_excl)
        uint32_t fs = (r[0] < sure_excl ? 1u : 0u) | (r[1] < sure_excl ? 2u : 0u) | (r[2] < sure_excl ? 4u : 0u) |
                      (r[3] < sure_excl ? 8u : 0u);
        if (sub_len != SUB) fs &= inside_mask(e0, sub_len);           // uniform: a ragged sub-tile
        // bitmap words: lanes 8j..8j+7 make word j of this round
        const uint32_t vs = or_reduce8(fs << (4u * (lane & 7u)));
        if ((lane & 7u) == (uint32_t)it) sword = vs;       // all eight lanes of a group hold the word: lane `it` of the group keeps it
        // candidate zone sure_excl <= word <= bound: one test for the four (the smallest distance above sure_excl;
        // words below it wrap to huge distances); the per-parameter work only when some lane of the wave has one,
        // which is rare with a narrow zone
        const uint32_t d0 = r[0] - sure_excl, d1 = r[1] - sure_excl, d2 = r[2] - sure_excl, d3 = r[3] - sure_excl;
        const uint32_t dmin = min(min(d0, d1), min(d2, d3));
        if (__ballot(dmin <= width_m1) != 0ull) {                     // uniform
            uint32_t fc = (d0 <= width_m1 ? 1u : 0u) | (d1 <= width_m1 ? 2u : 0u) | (d2 <= width_m1 ? 4u : 0u) |
                          (d3 <= width_m1 ? 8u : 0u);
            if (sub_len != SUB) fc &= inside_mask(e0, sub_len);
            if (!PAIRS) {
                const uint32_t vc = or_reduce8(fc << (4u * (lane & 7u)));
                if ((lane & 7u) == (uint32_t)it) cword = vc;
            }
            // place in the list: candidates of lower lanes in this round, all four components
            uint32_t below = 0, total = 0;
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const unsigned long long bal = __ballot((fc >> cc) & 1u);
                below += __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
                total += (uint32_t)__popcll(bal);
            }
            if (fc) {
                uint32_t pos = run + below;
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    if ((fc >> cc) & 1u) {
                        if (!PAIRS) ckeys[pos] = bound_m1 - r[cc];
                        else if (pos < PAIR_CAP) { ckeys[2u * pos] = bound_m1 - r[cc]; ckeys[2u * pos + 1u] = e0 + cc; }
                        ++pos;
                    }
                }
            }
            run += total;
        }
    }
    // the 32 bitmap words of the sub-tile in one store of one whole line by lanes 0..31 in address order (scattered
    // words make the memory side read the line first): word 8 * it + j sits in lane 8 * j + it
    {
        const int src = (int)(8u * (lane & 7u) + ((lane >> 3) & 3u));
        const uint32_t sw = __shfl(sword, src, 64);
        if (lane < SUB_WORDS) buffer_store1(rs, lane * 4u, sw);
        if (!PAIRS) {
            const uint32_t cw = __shfl(cword, src, 64);
            if (lane < SUB_WORDS) buffer_store1(rc, lane * 4u, cw);
        }
    }
    if (lane == 0) buffer_store1(rn, 0u, run);
}

// ---------------------------------------------------------------------------------------
// K1: significance of every parameter + level-0 histogram of its bits (per segment).
// Reads w and the W updates once, writes the score once: 4n(W+2) bytes.
// With DENSE = 1 (the iteration before a reselection, algorithm 1 / section 3.3 steps
// 3 and 6: every worker pushed its whole update) the model is first updated with all of them,
// w_new = fma(-lr, (+0 + g_0) + g_1 + ..., w), written to w_new (which may be w itself), and
// the significance is that of the new model: 4n(W+3) bytes.
// Persistent blocks over contiguous tile ranges keep the level-0 histogram in LDS.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void flush_hist(uint32_t* lds, uint32_t nb, uint32_t* __restrict__ g)
{
    for (uint32_t b = threadIdx.x; b < nb; b += BLOCK) {
        const uint32_t v = lds[b];
        if (v) { atomicAdd(&g[b], v); lds[b] = 0; }
    }
}

// PRE != 0 additionally draws the explorer zones of pre.nw workers for every tile
// (explore_subtile_fast<PRE - 1>): integer work that runs while other waves wait for memory.
struct PreArgs {
    uint32_t nw, worker0, n_seg;
    const SegState* states;
    uint32_t* sure_bits;
    uint32_t* cand_bits;
    uint32_t* cand_keys;
    uint32_t* cnt_cand;
    uint64_t keys_stride;
    PhiloxKey pk;
};

// SPEC = 1 (speculative packing, WT != 0 only) keeps, for every parameter of a full aligned
// tile whose significance reaches spec.lo[segment] - a little below the core threshold of
// the previous selection -, the W update values while they are in registers: one bit in
// spec.bits (beside each bitmap word: the entry number of its first parameter), and one
// entry of W consecutive values in spec.vals.  The entries of a sub-tile
// follow each other in index order from entry (tile start + 1024 * sub-tile); each round of
// 256 parameters starts on a 128-byte line and its last line is filled up, so that every
// line is written whole and at once (a line written in parts minutes apart leaves the cache
// in between and costs a read-modify-write in memory).
// If the coming selection's threshold is not below spec.lo, every core parameter is among
// them and the pack need not read the updates again.
struct SpecArgs {
    const uint32_t* lo;      // [n_seg] lowest captured significance (as bits)
    uint2* bits;             // [T * TILE_WORDS] x = the bits, y = number of the word's first entry inside its sub-tile
    float* vals;             // [entries][W]
};
// A sub-tile's entries live at spec.vals[(tile * SUBS + sub-tile) * SPEC_CAP * W]; entries beyond SPEC_CAP (a quarter
// of the sub-tile: two and a half times a 10 % core) are not kept (the descriptor's range drops their stores) and
// the pack reads those parameters from the update vectors.
constexpr uint32_t SPEC_CAP = SUB / 4;
__host__ __device__ constexpr uint32_t spec_align(uint32_t W) { return (W == 0u || W >= 32u) ? 1u : 32u / W; }   // entries per 128-byte line

#ifndef SCORE_MINB
#define SCORE_MINB 4
#endif
#ifndef SCORE_LD_AUX
#define SCORE_LD_AUX 2          // cache policy of the general scoring kernel's loads: non-temporal (the stress workload scores 4 % faster)
#endif
template <int WT, int PRE, int SPEC, int DENSE, int STRIDED>
__global__ __launch_bounds__(BLOCK, SCORE_MINB) void k_score(const float* __restrict__ w, PtrTab g, int Wrt, float c,
                                                 float* __restrict__ S, const uint32_t* __restrict__ tile_start,
                                                 const uint32_t* __restrict__ tile_seg, uint32_t T,
                                                 uint32_t* __restrict__ hist, int vec_ok, PreArgs pre, SpecArgs spec,
                                                 float* __restrict__ w_new, float lr)
{
    static_assert(!SPEC || WT != 0, "capture needs the update values in registers");
    static_assert(!(SPEC && DENSE), "a dense update is never followed by a pack of the same updates");
    // a significance is never negative: its sign bit is clear and the upper half of the level-0 bins stays empty
    constexpr uint32_t NB = CORE_NB0 / 2;
    __shared__ uint32_t h[NB];
    const int W = WT ? WT : Wrt;
    // the wave's number as a scalar: addresses below are then a scalar base plus a small per-lane offset
    const uint32_t lane = lane_id(), wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane16 = lane * 16u;      // byte offset of the lane's float4: a 32-bit offset beside a scalar base
    for (uint32_t b = threadIdx.x; b < NB; b += BLOCK) h[b] = 0;
    __syncthreads();
    // A block's tiles: a contiguous range (few segment changes, each of which flushes the histogram), or - flat model,
    // STRIDED - every gridDim.x-th tile, so that at any moment the whole chip streams through one window of each
    // array instead of a thousand separate places (fewer DRAM rows open at a time).  A compile-time choice: with the
    // step in a register the 16-worker variant spills more and loses 0.3 ms.
    const uint32_t t0 = STRIDED ? blockIdx.x : (uint32_t)((uint64_t)T * blockIdx.x / gridDim.x);
    const uint32_t t1 = STRIDED ? T : (uint32_t)((uint64_t)T * (blockIdx.x + 1) / gridDim.x);
    const uint32_t tstep = STRIDED ? gridDim.x : 1u;
    if (t0 >= t1) return;
    uint32_t cur_seg = tile_seg[t0];
    // Every wave owns sub-tile `wid` of each tile and runs through the block's tiles on its
    // own; the block only meets at a segment change and at the end (histogram flush).
    for (uint32_t t = t0; t < t1; t += tstep) {
        const uint32_t seg = tile_seg[t];
        if (seg != cur_seg) {
            __syncthreads();
            flush_hist(h, NB, hist + (size_t)cur_seg * H_STRIDE + H_L0);
            __syncthreads();
            cur_seg = seg;
        }
        const uint32_t start = tile_start[t], len = tile_start[t + 1] - start;
        // the candidate bound depends on the segment only (every worker draws the same number)
        uint32_t pre_bound = 0, pre_sure = 0, pre_has_sure = 0, pre_skip = 1;
        if (PRE) {
            const SegState* st = &pre.states[seg];
            pre_bound = st->bound_m1; pre_sure = st->sure_m1; pre_has_sure = st->has_gt; pre_skip = st->need0 == 0;
        }
        const bool vec = vec_ok && len == TILE && (start & 3u) == 0;
        uint32_t spec_lo = 0xFFFFFFFFu, spec_run = 0;
        if (SPEC) spec_lo = spec.lo[seg];
        if (!vec) {
            const uint32_t lo = wid * SUB, hi = (lo + SUB < len) ? lo + SUB : len;
            for (uint32_t l = lo + lane; l < hi; l += 64) {
                const size_t e = (size_t)start + l;
                float a = static_cast<const float*>(g.p[0])[e];
                for (int k = 1; k < W; ++k) a = a + static_cast<const float*>(g.p[k])[e];
                float we = w[e];
                if (DENSE) { we = __builtin_fmaf(-lr, a + 0.0f, we); w_new[e] = we; }      // dense update first
                const float sc = significance(we, a, c);
                S[e] = sc;
                atomicAdd(&h[(__float_as_uint(sc) >> CORE_SHIFT0) & (NB - 1u)], 1u);
            }
        }
        if (!vec && !PRE) continue;
        // the tile through buffer descriptors (scalar base per array, one 32-bit lane offset for all of them)
        const __amdgpu_buffer_rsrc_t rw = buffer_of(w + start, TILE * 4u);
        const __amdgpu_buffer_rsrc_t rS = buffer_of(S + start, TILE * 4u);
        const __amdgpu_buffer_rsrc_t rn = buffer_of(DENSE ? w_new + start : S + start, TILE * 4u);
        __amdgpu_buffer_rsrc_t rg[WT ? WT : 1];
        if (WT) {
#pragma unroll
            for (int k = 0; k < WT; ++k) rg[k] = buffer_of(static_cast<const float*>(g.p[k]) + start, TILE * 4u);
        }
#pragma unroll 1
        for (int r = 0; r < 4; ++r) {
            const size_t e0 = (size_t)start + (size_t)wid * SUB + (size_t)r * 256;      // uniform over the wave
            const uint32_t lane_bytes = (wid * SUB + (uint32_t)r * 256u) * 4u + lane16;  // of the lane's float4 inside the tile
            float4 wv = make_float4(0.f, 0.f, 0.f, 0.f);
            float4 x[WT ? WT : 1];
            if (vec) {          // request this round's lines first ...
                wv = buffer_load4_aux<SCORE_LD_AUX>(rw, lane_bytes);
                if (WT) {
#pragma unroll
                    for (int k = 0; k < WT; ++k) x[k] = buffer_load4_aux<SCORE_LD_AUX>(rg[k], lane_bytes);
                }
            }
            if (PRE) {          // ... do this round's share of the integer work while they fly ...
#pragma unroll 1
                for (uint32_t b = (uint32_t)r; b < pre.nw; b += 4) {
                    DrawOut out;
                    out.sure_bits = pre.sure_bits + (size_t)b * T * TILE_WORDS;
                    out.cand_bits = pre.cand_bits + (size_t)b * T * TILE_WORDS;
                    out.cand_keys = pre.cand_keys + (size_t)b * pre.keys_stride;
                    out.cnt_cand = pre.cnt_cand + (size_t)b * T * SUBS;
                    explore_subtile_fast<(PRE == 2) ? 1 : 0>(pre.worker0 + b, t, wid, start, len, pre_bound, pre_sure,
                                                             pre_has_sure, pre_skip, out, pre.pk, pre.pk);
                }
            }
            if (vec) {          // ... then score them
                float4 a;
                if (WT) {
                    a = x[0];
#pragma unroll
                    for (int k = 1; k < WT; ++k) { a.x = a.x + x[k].x; a.y = a.y + x[k].y; a.z = a.z + x[k].z; a.w = a.w + x[k].w; }
                } else {
                    a = *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(static_cast<const float*>(g.p[0]) + e0) + lane16);
                    for (int k = 1; k < W; ++k) {
                        const float4 y = *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(static_cast<const float*>(g.p[k]) + e0) + lane16);
                        a.x = a.x + y.x; a.y = a.y + y.y; a.z = a.z + y.z; a.w = a.w + y.w;
                    }
                }
                if (DENSE) {        // the server's dense update first (its sum starts from +0), then the new model's score
                    wv.x = __builtin_fmaf(-lr, a.x + 0.0f, wv.x); wv.y = __builtin_fmaf(-lr, a.y + 0.0f, wv.y);
                    wv.z = __builtin_fmaf(-lr, a.z + 0.0f, wv.z); wv.w = __builtin_fmaf(-lr, a.w + 0.0f, wv.w);
                    buffer_store4(rn, lane_bytes, 0u, wv);
                }
                float4 sc;
                sc.x = significance(wv.x, a.x, c); sc.y = significance(wv.y, a.y, c);
                sc.z = significance(wv.z, a.z, c); sc.w = significance(wv.w, a.w, c);
                buffer_store4(rS, lane_bytes, 0u, sc);
                atomicAdd(&h[(__float_as_uint(sc.x) >> CORE_SHIFT0) & (NB - 1u)], 1u);
                atomicAdd(&h[(__float_as_uint(sc.y) >> CORE_SHIFT0) & (NB - 1u)], 1u);
                atomicAdd(&h[(__float_as_uint(sc.z) >> CORE_SHIFT0) & (NB - 1u)], 1u);
                atomicAdd(&h[(__float_as_uint(sc.w) >> CORE_SHIFT0) & (NB - 1u)], 1u);
                if (SPEC) {
                    const uint32_t f = (__float_as_uint(sc.x) >= spec_lo ? 1u : 0u) | (__float_as_uint(sc.y) >= spec_lo ? 2u : 0u) |
                                       (__float_as_uint(sc.z) >= spec_lo ? 4u : 0u) | (__float_as_uint(sc.w) >= spec_lo ? 8u : 0u);
                    const uint32_t v = or_reduce8(f << (4u * (lane & 7u)));      // lanes 8j..8j+7 make bitmap word j of this round
                    uint32_t below = 0, total = 0;
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc) {
                        const unsigned long long bal = __ballot((f >> cc) & 1u);
                        below += __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
                        total += (uint32_t)__popcll(bal);
                    }
                    // lane 8j holds word j of the round and the number of captured parameters before it
                    if ((lane & 7u) == 0)
                        spec.bits[(size_t)t * TILE_WORDS + wid * SUB_WORDS + r * 8 + (lane >> 3)] = make_uint2(v, spec_run + below);
                    constexpr uint32_t A = spec_align(WT);
                    const uint32_t padded = (total + A - 1u) & ~(A - 1u);
                    // the sub-tile's entries through a descriptor: the entry number is the lane's part
                    const __amdgpu_buffer_rsrc_t rv = buffer_of(spec.vals + ((size_t)t * SUBS + wid) * SPEC_CAP * WT, SPEC_CAP * WT * 4u);
                    if (f) {
                        uint32_t pos = spec_run + below;
#pragma unroll
                        for (int cc = 0; cc < 4; ++cc) {
                            if ((f >> cc) & 1u) {
                                if (WT >= 4) {
#pragma unroll
                                    for (int k = 0; k < WT; k += 4) {
                                        float4 o;
                                        o.x = cc == 0 ? x[k].x : cc == 1 ? x[k].y : cc == 2 ? x[k].z : x[k].w;
                                        o.y = cc == 0 ? x[k + 1].x : cc == 1 ? x[k + 1].y : cc == 2 ? x[k + 1].z : x[k + 1].w;
                                        o.z = cc == 0 ? x[k + 2].x : cc == 1 ? x[k + 2].y : cc == 2 ? x[k + 2].z : x[k + 2].w;
                                        o.w = cc == 0 ? x[k + 3].x : cc == 1 ? x[k + 3].y : cc == 2 ? x[k + 3].z : x[k + 3].w;
                                        buffer_store4(rv, (pos * WT + k) * 4u, 0u, o);
                                    }
                                } else {
#pragma unroll
                                    for (int k = 0; k < WT; ++k)
                                        buffer_store1(rv, (pos * WT + k) * 4u,
                                                      __float_as_uint(cc == 0 ? x[k].x : cc == 1 ? x[k].y : cc == 2 ? x[k].z : x[k].w));
                                }
                                ++pos;
                            }
                        }
                    }
                    if (lane < padded - total) {          // fill the round's last line
#pragma unroll
                        for (int k = 0; k < WT; ++k) buffer_store1(rv, ((spec_run + total + lane) * WT + k) * 4u, 0u);
                    }
                    spec_run += padded;
                }
            }
        }
    }
    __syncthreads();
    flush_hist(h, NB, hist + (size_t)cur_seg * H_STRIDE + H_L0);
}

// ---------------------------------------------------------------------------------------
// K1 for a flat model whose arrays are 16-byte aligned: the same results as k_score, with
// the loads of the NEXT round of 256 parameters per wave (the next tile's first round after
// a tile's last) requested before the current round is worked on, so that a wave always has
// two rounds of nine 16-byte loads in flight, also while it draws explorer zones.  Whole
// arrays are addressed through one descriptor each (n < 2^30 parameters: byte offsets fit 32
// bits); block b takes the whole tiles b, b + gridDim.x, ...; the ragged last tile, if any,
// goes to one block after its loop, element by element.
// ---------------------------------------------------------------------------------------
#ifndef SCOREF_MINB
#define SCOREF_MINB 2
#endif
#ifndef SCOREF_LD_AUX
#define SCOREF_LD_AUX 2
#endif
#ifndef SCOREF_ST_AUX
#define SCOREF_ST_AUX 2
#endif
#ifndef SCOREF_CAP_AUX
#define SCOREF_CAP_AUX 2
#endif
// cls.pred[0] != NONE: every whole tile is also sorted against that predicted level-0 threshold bin, exactly as
// k_core_build would do it once the bin is known (certain bitmap, candidate bitmap, candidate keys compacted per
// sub-tile, counts): if the histogram then confirms the bin, the selection need not read the scores again.
struct ClsArgs {
    const uint32_t* pred;
    uint32_t* used;          // [0]: the bin this launch classified against (NONE: it did not)
    int mode;                // 1: pred[0]; test switches: 0 never classify, 2 take the bin above the prediction (always wrong)
    uint32_t *gt_bits, *cand_bits, *cand_keys, *cnt_gt, *cnt_cand;
};
template <int WT, int PRE, int SPEC, int DENSE>
__global__ __launch_bounds__(BLOCK, SCOREF_MINB) void k_score_flat(const float* __restrict__ w, PtrTab g, float c,
                                                                   float* __restrict__ S, uint64_t n, uint32_t* __restrict__ hist,
                                                                   PreArgs pre, SpecArgs spec, ClsArgs cls, float* __restrict__ w_new, float lr)
{
    static_assert(WT >= 1 && WT <= 8, "two rounds of W + 1 vectors must fit the registers");
    static_assert(!(SPEC && DENSE), "a dense update is never followed by a pack of the same updates");
    constexpr uint32_t NB = CORE_NB0 / 2;
    __shared__ uint32_t h[NB];
    __shared__ __align__(16) float stage[SPEC ? 4 * 256 * WT : 4];
    __shared__ uint32_t h1[CORE_NB1];                // level-1 digits of the candidates of the predicted bin
    const uint32_t lane = lane_id(), wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t T_full = (uint32_t)(n / TILE), T = (uint32_t)((n + TILE - 1) / TILE);
    for (uint32_t b = threadIdx.x; b < NB; b += BLOCK) h[b] = 0;
    for (uint32_t b = threadIdx.x; b < CORE_NB1; b += BLOCK) h1[b] = 0;
    __syncthreads();
    const uint32_t bytes = (uint32_t)(n * 4u);
    const __amdgpu_buffer_rsrc_t rw = buffer_of(w, bytes), rS = buffer_of(S, bytes), rn = buffer_of(DENSE ? w_new : S, bytes);
    __amdgpu_buffer_rsrc_t rg[WT];
#pragma unroll
    for (int k = 0; k < WT; ++k) rg[k] = buffer_of(g.p[k], bytes);
    uint32_t pre_bound = 0, pre_sure = 0, pre_has_sure = 0, pre_skip = 1;
    if (PRE) {
        const SegState* st = &pre.states[0];
        pre_bound = st->bound_m1; pre_sure = st->sure_m1; pre_has_sure = st->has_gt; pre_skip = st->need0 == 0;
    }
    uint32_t spec_lo = 0xFFFFFFFFu;
    if (SPEC) spec_lo = spec.lo[0];
    uint32_t b1 = cls.mode ? cls.pred[0] : NONE;     // predicted threshold bin, NONE: no prediction
    if (cls.mode == 2 && b1 != NONE) b1 += 1u;
    if (blockIdx.x == 0 && threadIdx.x == 0) cls.used[0] = b1;
    uint32_t crun = 0, ngt = 0, gw[4], cw[4];
    // byte offset of this lane's vector in round r of this wave's sub-tile of tile t
    auto voff = [&](uint32_t t, uint32_t r) { return (t * TILE + wid * SUB + r * 256u) * 4u + lane * 16u; };
    auto fetch = [&](float4 (&x)[WT + 1], uint32_t t, uint32_t r) {
        const uint32_t o = voff(t, r);
        x[WT] = buffer_load4_aux<SCOREF_LD_AUX>(rw, o);
#pragma unroll
        for (int k = 0; k < WT; ++k) x[k] = buffer_load4_aux<SCOREF_LD_AUX>(rg[k], o);
    };
    PhiloxRoundKeys rkeys;
    if (PRE) rkeys = philox_round_keys(pre.pk.seed_lo, pre.pk.seed_hi);
    auto draw = [&](uint32_t t, uint32_t len, uint32_t r) {      // this round's share of the announced draws
        if (PRE) {
#pragma unroll 1
            for (uint32_t b = r; b < pre.nw; b += 4) {
                DrawOut out;
                out.sure_bits = pre.sure_bits + (size_t)b * T * TILE_WORDS;
                out.cand_bits = pre.cand_bits + (size_t)b * T * TILE_WORDS;
                out.cand_keys = pre.cand_keys + (size_t)b * pre.keys_stride;
                out.cnt_cand = pre.cnt_cand + (size_t)b * T * SUBS;
                explore_subtile_fast<(PRE == 2) ? 1 : 0>(pre.worker0 + b, t, wid, t * TILE, len, pre_bound, pre_sure,
                                                         pre_has_sure, pre_skip, out, pre.pk, rkeys);
            }
        }
    };
    uint32_t spec_run = 0;
    uint2 bw[4];
    auto work = [&](float4 (&x)[WT + 1], uint32_t t, uint32_t r) {
        const uint32_t o = voff(t, r);
        float4 a = x[0];
#pragma unroll
        for (int k = 1; k < WT; ++k) { a.x = a.x + x[k].x; a.y = a.y + x[k].y; a.z = a.z + x[k].z; a.w = a.w + x[k].w; }
        float4 wv = x[WT];
        if (DENSE) {
            wv.x = __builtin_fmaf(-lr, a.x + 0.0f, wv.x); wv.y = __builtin_fmaf(-lr, a.y + 0.0f, wv.y);
            wv.z = __builtin_fmaf(-lr, a.z + 0.0f, wv.z); wv.w = __builtin_fmaf(-lr, a.w + 0.0f, wv.w);
            buffer_store4_aux<0>(rn, o, wv);
        }
        float4 sc;
        sc.x = significance(wv.x, a.x, c); sc.y = significance(wv.y, a.y, c);
        sc.z = significance(wv.z, a.z, c); sc.w = significance(wv.w, a.w, c);
        buffer_store4_aux<SCOREF_ST_AUX>(rS, o, sc);
        atomicAdd(&h[(__float_as_uint(sc.x) >> CORE_SHIFT0) & (NB - 1u)], 1u);
        atomicAdd(&h[(__float_as_uint(sc.y) >> CORE_SHIFT0) & (NB - 1u)], 1u);
        atomicAdd(&h[(__float_as_uint(sc.z) >> CORE_SHIFT0) & (NB - 1u)], 1u);
        atomicAdd(&h[(__float_as_uint(sc.w) >> CORE_SHIFT0) & (NB - 1u)], 1u);
        if (b1 != NONE) {                            // uniform
            if (r == 0) { crun = 0; ngt = 0; }
            const uint32_t d0 = __float_as_uint(sc.x) >> CORE_SHIFT0, d1 = __float_as_uint(sc.y) >> CORE_SHIFT0,
                           d2 = __float_as_uint(sc.z) >> CORE_SHIFT0, d3 = __float_as_uint(sc.w) >> CORE_SHIFT0;
            const uint32_t fg = (d0 > b1 ? 1u : 0u) | (d1 > b1 ? 2u : 0u) | (d2 > b1 ? 4u : 0u) | (d3 > b1 ? 8u : 0u);
            const uint32_t fc = (d0 == b1 ? 1u : 0u) | (d1 == b1 ? 2u : 0u) | (d2 == b1 ? 4u : 0u) | (d3 == b1 ? 8u : 0u);
            gw[r] = or_reduce8(fg << (4u * (lane & 7u)));
            cw[r] = or_reduce8(fc << (4u * (lane & 7u)));
            ngt += __popc(fg);
            if (__ballot(fc != 0u) != 0ull) {
                uint32_t below = 0, total = 0;
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    const unsigned long long bal = __ballot((fc >> cc) & 1u);
                    below += __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
                    total += (uint32_t)__popcll(bal);
                }
                if (fc) {
                    const __amdgpu_buffer_rsrc_t rk = buffer_of(cls.cand_keys + (size_t)t * TILE + wid * SUB, SUB * 4u);
                    uint32_t pos = crun + below;
                    if (fc & 1u) { buffer_store1(rk, 4u * pos++, __float_as_uint(sc.x)); atomicAdd(&h1[(__float_as_uint(sc.x) >> CORE_SHIFT1) & (CORE_NB1 - 1u)], 1u); }
                    if (fc & 2u) { buffer_store1(rk, 4u * pos++, __float_as_uint(sc.y)); atomicAdd(&h1[(__float_as_uint(sc.y) >> CORE_SHIFT1) & (CORE_NB1 - 1u)], 1u); }
                    if (fc & 4u) { buffer_store1(rk, 4u * pos++, __float_as_uint(sc.z)); atomicAdd(&h1[(__float_as_uint(sc.z) >> CORE_SHIFT1) & (CORE_NB1 - 1u)], 1u); }
                    if (fc & 8u) { buffer_store1(rk, 4u * pos, __float_as_uint(sc.w)); atomicAdd(&h1[(__float_as_uint(sc.w) >> CORE_SHIFT1) & (CORE_NB1 - 1u)], 1u); }
                }
                crun += total;
            }
            if (r == 3) {          // the sub-tile's 32 + 32 bitmap words as whole lines, its two counts
                const int src = (int)(8u * (lane & 7u));
                uint32_t og = 0, oc = 0;
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const uint32_t xg = __shfl(gw[rr], src, 64), xc = __shfl(cw[rr], src, 64);
                    if ((lane >> 3) == (uint32_t)rr) { og = xg; oc = xc; }
                }
                const size_t wbase = (size_t)t * TILE_WORDS + wid * SUB_WORDS;
                if (lane < SUB_WORDS) { cls.gt_bits[wbase + lane] = og; cls.cand_bits[wbase + lane] = oc; }
                const uint32_t ng = wave_sum(ngt);
                if (lane == 0) { cls.cnt_cand[(size_t)t * SUBS + wid] = crun; cls.cnt_gt[(size_t)t * SUBS + wid] = ng; }
            }
        }
        if (SPEC) {
            if (r == 0) spec_run = 0;
            const uint32_t f = (__float_as_uint(sc.x) >= spec_lo ? 1u : 0u) | (__float_as_uint(sc.y) >= spec_lo ? 2u : 0u) |
                               (__float_as_uint(sc.z) >= spec_lo ? 4u : 0u) | (__float_as_uint(sc.w) >= spec_lo ? 8u : 0u);
            const uint32_t v = or_reduce8(f << (4u * (lane & 7u)));
            uint32_t below = 0, total = 0;
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const unsigned long long bal = __ballot((f >> cc) & 1u);
                below += __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
                total += (uint32_t)__popcll(bal);
            }
            // bitmap words with their entry numbers: lane 8j holds word j of this round; after the sub-tile's last
            // round lanes 0..31 write all 32 of them at once (two whole lines)
            bw[r] = make_uint2(v, spec_run + below);
            if (r == 3) {
                const int src = (int)(8u * (lane & 7u));
                uint2 o = make_uint2(0u, 0u);
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const uint32_t ox = __shfl(bw[rr].x, src, 64), oy = __shfl(bw[rr].y, src, 64);
                    if ((lane >> 3) == (uint32_t)rr) o = make_uint2(ox, oy);
                }
                if (lane < SUB_WORDS) spec.bits[(size_t)t * TILE_WORDS + wid * SUB_WORDS + lane] = o;
            }
            constexpr uint32_t A = spec_align(WT);
            const uint32_t padded = (total + A - 1u) & ~(A - 1u);
            // the round's entries go through the wave's staging area in LDS, so that every 128-byte line of the capture is
            // written by one store instruction, whole (a line written piecewise by several instructions can leave the
            // cache half-written and costs a read-modify-write in memory)
            float* stf = stage + wid * (256 * WT);
            if (f) {
                uint32_t pos = below;
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) {
                    if ((f >> cc) & 1u) {
                        if (WT >= 4) {
#pragma unroll
                            for (int k = 0; k < WT; k += 4) {
                                float4 q;
                                q.x = cc == 0 ? x[k].x : cc == 1 ? x[k].y : cc == 2 ? x[k].z : x[k].w;
                                q.y = cc == 0 ? x[k + 1].x : cc == 1 ? x[k + 1].y : cc == 2 ? x[k + 1].z : x[k + 1].w;
                                q.z = cc == 0 ? x[k + 2].x : cc == 1 ? x[k + 2].y : cc == 2 ? x[k + 2].z : x[k + 2].w;
                                q.w = cc == 0 ? x[k + 3].x : cc == 1 ? x[k + 3].y : cc == 2 ? x[k + 3].z : x[k + 3].w;
                                *reinterpret_cast<float4*>(stf + pos * WT + k) = q;
                            }
                        } else {
#pragma unroll
                            for (int k = 0; k < WT; ++k)
                                stf[pos * WT + k] = cc == 0 ? x[k].x : cc == 1 ? x[k].y : cc == 2 ? x[k].z : x[k].w;
                        }
                        ++pos;
                    }
                }
            }
            if (lane < padded - total) {          // fill the round's last line
#pragma unroll
                for (int k = 0; k < WT; ++k) stf[(total + lane) * WT + k] = 0.0f;
            }
            wave_sync();
            {
                const __amdgpu_buffer_rsrc_t rv = buffer_of(spec.vals + ((size_t)t * SUBS + wid) * SPEC_CAP * WT, SPEC_CAP * WT * 4u);
                const uint32_t nchunk = padded * WT / 4u;          // 16-byte pieces: a multiple of 8 (whole lines)
                for (uint32_t cidx = lane; cidx < nchunk; cidx += 64)
                    buffer_store4_aux<SCOREF_CAP_AUX>(rv, spec_run * WT * 4u + cidx * 16u, *reinterpret_cast<const float4*>(stf + cidx * 4u));
            }
            wave_sync();
            spec_run += padded;
        }
    };
    float4 xa[WT + 1], xb[WT + 1];
    uint32_t t = blockIdx.x;
    if (t < T_full) fetch(xa, t, 0);
#pragma unroll 1
    for (; t < T_full; t += gridDim.x) {
        const uint32_t tn = t + gridDim.x;
        fetch(xb, t, 1); draw(t, TILE, 0); work(xa, t, 0);
        fetch(xa, t, 2); draw(t, TILE, 1); work(xb, t, 1);
        fetch(xb, t, 3); draw(t, TILE, 2); work(xa, t, 2);
        if (tn < T_full) fetch(xa, tn, 0);
        draw(t, TILE, 3); work(xb, t, 3);
    }
    // the ragged last tile
    if (T != T_full && blockIdx.x == T_full % gridDim.x) {
        const uint32_t start = T_full * TILE, len = (uint32_t)(n - start);
        const uint32_t lo = wid * SUB, hi = (lo + SUB < len) ? lo + SUB : len;
        for (uint32_t l = lo + lane; l < hi; l += 64) {
            const size_t e = (size_t)start + l;
            float a = static_cast<const float*>(g.p[0])[e];
#pragma unroll
            for (int k = 1; k < WT; ++k) a = a + static_cast<const float*>(g.p[k])[e];
            float we = w[e];
            if (DENSE) { we = __builtin_fmaf(-lr, a + 0.0f, we); w_new[e] = we; }
            const float sc = significance(we, a, c);
            S[e] = sc;
            atomicAdd(&h[(__float_as_uint(sc) >> CORE_SHIFT0) & (NB - 1u)], 1u);
        }
        for (uint32_t r = 0; r < 4; ++r) draw(T_full, len, r);
    }
    __syncthreads();
    flush_hist(h, NB, hist + H_L0);
    if (b1 != NONE) flush_hist(h1, CORE_NB1, hist + H_L1);
}

// ---------------------------------------------------------------------------------------
// Capture bound without an earlier selection (flat model): a sample of the significances about
// to be computed gives an estimate of the coming threshold.  k_sample_keys scores SAMPLE_PER
// consecutive parameters of every full tile, at a tile-dependent offset; k_sample_bound (one
// block) finds the sample's need-th largest key by a two-level radix descent (12 + 12 bits:
// 2^7 units in the last place) and writes it, less a margin, as the capture bound.  An
// estimate that turns out too high is caught by the selection's own verdict (the pack then
// gathers); one that is too low only makes the capture larger.
// ---------------------------------------------------------------------------------------
constexpr uint32_t SAMPLE_PER = 2;
constexpr uint32_t SAMPLE_MARGIN = 1u << 18;
__global__ __launch_bounds__(256) void k_sample_keys(const float* __restrict__ w, PtrTab g, int W, float c, uint32_t T_full,
                                                     uint32_t* __restrict__ keys)
{
    const uint32_t x = blockIdx.x * 256 + threadIdx.x;
    if (x >= T_full * SAMPLE_PER) return;
    const uint32_t t = x / SAMPLE_PER, j = x % SAMPLE_PER;
    const uint32_t off = ((t * 0x9E3779B1u) >> 21) * SAMPLE_PER;       // 0 .. 4094 in steps of 2: inside the tile
    const size_t i = (size_t)t * TILE + off + j;
    float a = static_cast<const float*>(g.p[0])[i];
    for (int k = 1; k < W; ++k) a = a + static_cast<const float*>(g.p[k])[i];
    keys[x] = __float_as_uint(significance(w[i], a, c));
}

// bias: test switch, added to the bound (in units of the last place, clamped).
__global__ __launch_bounds__(1024) void k_sample_bound(const uint32_t* __restrict__ keys, uint32_t N, uint32_t need,
                                                       long long bias, uint32_t* __restrict__ lo, uint32_t* __restrict__ pred)
{
    __shared__ uint32_t h[4096];
    __shared__ uint32_t wtot[16];
    __shared__ uint32_t sh[2];
    const uint32_t tid = threadIdx.x;
    if (need == 0 || need > N) { if (tid == 0) { lo[0] = NONE; pred[0] = NONE; } return; }   // nothing to estimate, nothing captured
    uint32_t prefix = 0, want = need;
#pragma unroll 1
    for (int level = 0; level < 2; ++level) {
        for (uint32_t b = tid; b < 4096; b += 1024) h[b] = 0;
        __syncthreads();
        for (uint32_t x = tid; x < N; x += 1024) {
            const uint32_t key = keys[x];
            if (level == 0) atomicAdd(&h[(key >> 19) & 4095u], 1u);
            else if ((key >> 19) == prefix) atomicAdd(&h[(key >> 7) & 4095u], 1u);
        }
        __syncthreads();
        // four bins per thread, from the largest digit down
        uint32_t cnt[4], sum = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) { cnt[e] = h[4095u - (tid * 4u + e)]; sum += cnt[e]; }
        uint32_t total;
        const uint32_t excl = block_excl_scan<16>(sum, wtot, total);
        if (excl < want && want <= excl + sum) {
            uint32_t run = excl;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (run < want && want <= run + cnt[e]) { sh[0] = 4095u - (tid * 4u + e); sh[1] = want - run; }
                run += cnt[e];
            }
        }
        __syncthreads();
        prefix = (level == 0) ? sh[0] : ((prefix << 12) | sh[0]);
        want = sh[1];
        __syncthreads();
    }
    if (tid == 0) {
        const long long tau = (long long)(prefix << 7);
        long long b = tau - (long long)SAMPLE_MARGIN + bias;
        if (b < 0) b = 0;
        if (b > 0x7FFFFFFFll) b = 0x7FFFFFFFll;
        lo[0] = (uint32_t)b;
        pred[0] = prefix >> 12;          // the level-0 bin of the estimated threshold
    }
}

// Level-0 histogram of a score array that did not come from k_score.
__global__ __launch_bounds__(BLOCK) void k_core_hist0(const float* __restrict__ S, const uint32_t* __restrict__ tile_start,
                                                      const uint32_t* __restrict__ tile_seg, uint32_t T,
                                                      uint32_t* __restrict__ hist)
{
    __shared__ uint32_t h[CORE_NB0];
    for (uint32_t b = threadIdx.x; b < CORE_NB0; b += BLOCK) h[b] = 0;
    __syncthreads();
    const uint32_t t0 = (uint32_t)((uint64_t)T * blockIdx.x / gridDim.x);
    const uint32_t t1 = (uint32_t)((uint64_t)T * (blockIdx.x + 1) / gridDim.x);
    if (t0 >= t1) return;
    uint32_t cur_seg = tile_seg[t0];
    for (uint32_t t = t0; t < t1; ++t) {
        const uint32_t seg = tile_seg[t];
        if (seg != cur_seg) {
            __syncthreads();
            flush_hist(h, CORE_NB0, hist + (size_t)cur_seg * H_STRIDE + H_L0);
            __syncthreads();
            cur_seg = seg;
        }
        const uint32_t start = tile_start[t], len = tile_start[t + 1] - start;
        for (uint32_t l = threadIdx.x; l < len; l += BLOCK)
            atomicAdd(&h[__float_as_uint(S[(size_t)start + l]) >> CORE_SHIFT0], 1u);
    }
    __syncthreads();
    flush_hist(h, CORE_NB0, hist + (size_t)cur_seg * H_STRIDE + H_L0);
}

// ---------------------------------------------------------------------------------------
// Threshold step of one radix level: walk the bins from the largest digit down until
// `need` keys are covered.  grid (n_seg, nbatch), 256 threads.
// mode 0: plain.  mode 1: explorer level 0 with zones: a miss on either side raises the
// rerun flag (flags[0]).  gate != 0: return at once if the flag is already up (the exact
// rerun k_explore_exact follows and overwrites everything); the kernels of the per-tile tail
// take the flag word as `gate` the same way (nullptr: always run).
// ---------------------------------------------------------------------------------------
// At the last level of a core selection with speculative packing on (st.next != nullptr):
// fail[seg] tells whether the threshold fell below what the scoring pass captured (cur), and
// next[seg] becomes the capture bound of the next scoring pass: the new threshold less
// 2^17 units in the last place (0.8 % to 1.6 %).
struct SpecTau { const uint32_t* cur; uint32_t* next; uint32_t* fail; };
// Core selection whose scoring pass already sorted every whole tile against a PREDICTED level-0 threshold bin
// (used[seg]: what the scoring pass took, normally pred[seg], the bin of the previous threshold): level 0 tells per
// segment whether the prediction held
// (skip[seg] = 1: the candidate pass has nothing left to do for whole tiles), the last level records the bin
// of the new threshold as the next prediction.  check = 0: the scoring pass did not classify.
struct CorePred { uint32_t* pred; uint32_t* skip; const uint32_t* used; int check; };
constexpr uint32_t SPEC_MARGIN = 1u << 17;

__global__ __launch_bounds__(256) void k_threshold(SegState* __restrict__ states, uint32_t* __restrict__ hist,
                                                   int level, uint32_t hist_off, uint32_t n_seg, int mode,
                                                   uint32_t* __restrict__ flags, const uint32_t* __restrict__ nsure, int gate,
                                                   SpecTau sp, CorePred cp)
{
    __shared__ uint32_t wtot[4];
    __shared__ uint32_t sh_bcast[2];
    if (gate) {          // other blocks of this launch may raise the flag: one read per block
        if (threadIdx.x == 0) sh_bcast[0] = flags[0];
        __syncthreads();
        if (sh_bcast[0] != 0) return;
    }
    const uint32_t seg = blockIdx.x, b = blockIdx.y;
    SegState* st = &states[(size_t)b * n_seg + seg];
    const uint32_t* hp = hist + ((size_t)b * n_seg + seg) * H_STRIDE + hist_off;
    if (mode == 1 && st->has_gt) {
        // the certainly taken ones (word below the sure bound, outside the core) come off the demand
        const uint32_t ns = nsure[(size_t)b * n_seg + seg];
        const uint32_t n0 = st->need0;
        __syncthreads();
        if (ns > n0) {                        // the sure zone alone is already too large: exact rerun
            if (threadIdx.x == 0) atomicOr(&flags[0], 1u);
            return;
        }
        if (threadIdx.x == 0) st->need = n0 - ns;
        __syncthreads();
    }
    const uint32_t need = st->need, none = st->none, nb = st->nbins[level];
    const uint32_t prefix = st->prefix;
    const uint32_t bits = (level == 0) ? 0u : (st->shift[level - 1] - st->shift[level]);
    __syncthreads();
    if (none || need == 0) {
        if (threadIdx.x == 0) {
            st->none = 1; st->need = 0; st->tau = NONE; st->quota = 0;
            if (level == 2 && sp.next) { sp.fail[seg] = 0; sp.next[seg] = NONE; }      // nothing selected, nothing to capture
            if (cp.skip && level == 0) cp.skip[seg] = 0;
            if (cp.pred && level == 2) cp.pred[seg] = NONE;
        }
        return;
    }
    const uint32_t C = (nb + 255u) / 256u;
    const uint32_t p0 = threadIdx.x * C;
    uint32_t sum = 0;
    for (uint32_t p = p0; p < p0 + C && p < nb; ++p) sum += hp[nb - 1u - p];
    uint32_t total;
    const uint32_t excl = block_excl_scan<4>(sum, wtot, total);
    if (total < need) {
        if (threadIdx.x == 0) {
            if (mode == 1) atomicOr(&flags[0], 1u);                    // too few candidates: exact rerun
            else { atomicOr(&flags[1], 2u); st->none = 1; st->need = 0; st->tau = NONE; st->quota = 0; }
            if (cp.skip && level == 0) cp.skip[seg] = 0;
        }
        return;
    }
    if (excl < need && need <= excl + sum) {
        uint32_t run = excl;
        for (uint32_t p = p0; p < p0 + C && p < nb; ++p) {
            const uint32_t bin = nb - 1u - p;
            const uint32_t cnt = hp[bin];
            if (run + cnt >= need) {
                const uint32_t np = (level == 0) ? bin : ((prefix << bits) | bin);
                st->prefix = np;
                st->need = need - run;
                if (cp.skip && level == 0) {
                    const uint32_t ok = (cp.check && cp.used[seg] == np) ? 1u : 0u;
                    cp.skip[seg] = ok;
                    sh_bcast[1] = ok;
                }
                if (cp.pred && level == 2) cp.pred[seg] = np >> CORE_SHIFT0;
                if (level == 2) {
                    st->tau = np; st->quota = need - run; st->tie_all = (need - run == cnt) ? 1u : 0u;
                    if (sp.next) {
                        sp.fail[seg] = (np < sp.cur[seg]) ? 1u : 0u;
                        sp.next[seg] = np > SPEC_MARGIN ? np - SPEC_MARGIN : 0u;
                    }
                }
                break;
            }
            run += cnt;
        }
    }
    if (cp.skip && level == 0 && cp.check) {
        // the scoring pass has already added the level-1 digits of ITS candidates: if they belong to another bin they go
        __syncthreads();
        if (sh_bcast[1] == 0) {
            uint32_t* h1 = hist + ((size_t)b * n_seg + seg) * H_STRIDE + H_L1;
            for (uint32_t x = threadIdx.x; x < CORE_NB1; x += 256) h1[x] = 0;
        }
    }
}

// ---------------------------------------------------------------------------------------
// K2: core candidates.  One pass over the score: parameters whose level-0 digit is above
// the threshold bin are certainly in the core (gt bitmap), those in the bin are candidates
// (bitmap + keys compacted per sub-tile) and feed the level-1 histogram.
// Every wave owns sub-tile `wid` of each of the block's tiles and needs no block barrier:
// round `it` covers parameters [256*it, 256*it+256) of the sub-tile in index order (lane L
// owns 4L..4L+3), the eight bitmap words of a round are OR-reductions over groups of
// eight lanes, a candidate's place in the key list comes from wave ballots.
// ---------------------------------------------------------------------------------------
// The 1024 scores of sub-tile `wid` of a tile as keys: lane L holds parameters 4L..4L+3 of each round of 256.
__device__ __forceinline__ void core_load_keys(const float* __restrict__ S, uint32_t start, uint32_t len, uint32_t wid,
                                               uint32_t lane, int vec_ok, uint32_t key[4][4])
{
    const uint32_t off = wid * SUB;
    const uint32_t sub_len = (len > off) ? ((len - off < SUB) ? len - off : SUB) : 0u;
    const float* src = S + (size_t)start + off;
    if (vec_ok && sub_len == SUB && (start & 3u) == 0) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const uint4 v = ld4u<NT_BUILD>(reinterpret_cast<const uint32_t*>(src + it * 256 + lane * 4));
            key[it][0] = v.x; key[it][1] = v.y; key[it][2] = v.z; key[it][3] = v.w;
        }
    } else {
#pragma unroll
        for (int it = 0; it < 4; ++it)
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const uint32_t e = (uint32_t)it * 256u + lane * 4u + cc;
                key[it][cc] = (e < sub_len) ? __float_as_uint(src[e]) : 0u;
            }
    }
}

// One sub-tile's keys against the level-0 threshold bin b1: bitmaps, candidate keys, counts, level-1 histogram (LDS).
__device__ __forceinline__ void core_classify(const uint32_t key[4][4], uint32_t t, uint32_t start, uint32_t len, uint32_t wid,
                                              uint32_t lane, uint32_t b1, uint32_t none, uint32_t* __restrict__ h,
                                              uint32_t* __restrict__ gt_bits, uint32_t* __restrict__ cand_bits,
                                              uint32_t* __restrict__ cand_keys, uint32_t* __restrict__ cnt_gt,
                                              uint32_t* __restrict__ cnt_cand)
{
    const uint32_t off = wid * SUB;
    const uint32_t sub_len = (len > off) ? ((len - off < SUB) ? len - off : SUB) : 0u;
    uint32_t* gwords = gt_bits + (size_t)t * TILE_WORDS + wid * SUB_WORDS;
    uint32_t* cwords = cand_bits + (size_t)t * TILE_WORDS + wid * SUB_WORDS;
    uint32_t* ckeys = cand_keys + (size_t)start + off;
    uint32_t run = 0, ngt = 0;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        uint32_t fg = 0, fc = 0;
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const uint32_t e = (uint32_t)it * 256u + lane * 4u + cc;
            if (e < sub_len && !none) {
                const uint32_t d = key[it][cc] >> CORE_SHIFT0;
                if (d > b1) fg |= 1u << cc;
                else if (d == b1) fc |= 1u << cc;
            }
        }
        const uint32_t vg = or_reduce8(fg << (4u * (lane & 7u))), vc = or_reduce8(fc << (4u * (lane & 7u)));
        if ((lane & 7u) == 0) { gwords[it * 8 + (lane >> 3)] = vg; cwords[it * 8 + (lane >> 3)] = vc; }
        ngt += __popc(fg);
        uint32_t below = 0, total = 0;
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const unsigned long long bal = __ballot((fc >> cc) & 1u);
            below += __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
            total += (uint32_t)__popcll(bal);
        }
        if (fc) {
            uint32_t pos = run + below;
#pragma unroll
            for (int cc = 0; cc < 4; ++cc)
                if ((fc >> cc) & 1u) {
                    ckeys[pos++] = key[it][cc];
                    atomicAdd(&h[(key[it][cc] >> CORE_SHIFT1) & (CORE_NB1 - 1u)], 1u);
                }
        }
        run += total;
    }
    ngt = wave_sum(ngt);
    if (lane == 0) { cnt_cand[(size_t)t * SUBS + wid] = run; cnt_gt[(size_t)t * SUBS + wid] = ngt; }
}

// skip [n_seg] (may be nullptr): 1 = the scoring pass has already classified every whole, 4-aligned tile of the
// segment against the right bin; only ragged or unaligned tiles are left.
__global__ __launch_bounds__(BLOCK) void k_core_build(const float* __restrict__ S, const uint32_t* __restrict__ tile_start,
                                                      const uint32_t* __restrict__ tile_seg, uint32_t T,
                                                      const SegState* __restrict__ states, const uint32_t* __restrict__ skip,
                                                      uint32_t* __restrict__ hist,
                                                      uint32_t* __restrict__ gt_bits, uint32_t* __restrict__ cand_bits,
                                                      uint32_t* __restrict__ cand_keys, uint32_t* __restrict__ cnt_gt,
                                                      uint32_t* __restrict__ cnt_cand, int vec_ok, int strided)
{
    __shared__ uint32_t h[CORE_NB1];
    const uint32_t lane = lane_id(), wid = threadIdx.x >> 6;
    // a contiguous range of tiles, or (flat model) every gridDim.x-th tile: see k_score
    uint32_t t0 = (uint32_t)((uint64_t)T * blockIdx.x / gridDim.x);
    uint32_t t1 = (uint32_t)((uint64_t)T * (blockIdx.x + 1) / gridDim.x);
    uint32_t tstep = 1;
    if (strided) { t0 = blockIdx.x; t1 = T; tstep = gridDim.x; }
    if (t0 >= t1) return;
    auto done = [&](uint32_t t) {       // already classified by the scoring pass?
        if (!skip || !skip[tile_seg[t]]) return false;
        const uint32_t start = tile_start[t];
        return tile_start[t + 1] - start == TILE && (start & 3u) == 0;
    };
    // flat model, prediction held: only a ragged last tile can be left; one block looks at it
    if (strided && skip && skip[0]) {
        if (blockIdx.x != 0) return;
        t0 = T - 1;
    }
    for (uint32_t b = threadIdx.x; b < CORE_NB1; b += BLOCK) h[b] = 0;
    __syncthreads();
    uint32_t cur_seg = tile_seg[t0];
    // two tiles a turn: the scores of both are requested before either is worked on
    for (uint32_t t = t0; t < t1; t += 2 * tstep) {
        const uint32_t tB = t + tstep;
        const bool one = !done(t), two = tB < t1 && !done(tB);
        if (!one && !two) continue;
        const uint32_t startA = tile_start[t], lenA = tile_start[t + 1] - startA;
        const uint32_t startB = two ? tile_start[tB] : 0u, lenB = two ? tile_start[tB + 1] - startB : 0u;
        uint32_t keyA[4][4], keyB[4][4];
        if (one) core_load_keys(S, startA, lenA, wid, lane, vec_ok, keyA);
        if (two) core_load_keys(S, startB, lenB, wid, lane, vec_ok, keyB);
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            if (half == 0 ? !one : !two) continue;
            const uint32_t tt = half ? tB : t;
            const uint32_t seg = tile_seg[tt];
            if (seg != cur_seg) {
                __syncthreads();
                flush_hist(h, CORE_NB1, hist + (size_t)cur_seg * H_STRIDE + H_L1);
                __syncthreads();
                cur_seg = seg;
            }
            const uint32_t b1 = states[seg].prefix, none = states[seg].none;
            if (half == 0) core_classify(keyA, tt, startA, lenA, wid, lane, b1, none, h, gt_bits, cand_bits, cand_keys, cnt_gt, cnt_cand);
            else core_classify(keyB, tt, startB, lenB, wid, lane, b1, none, h, gt_bits, cand_bits, cand_keys, cnt_gt, cnt_cand);
        }
    }
    __syncthreads();
    flush_hist(h, CORE_NB1, hist + (size_t)cur_seg * H_STRIDE + H_L1);
}

// Stand-alone draw over every (worker, tile); each wave owns one sub-tile of the block's
// tiles.  grid (blocks, n_workers).
template <int FAST, int PAIRS>
__global__ __launch_bounds__(BLOCK) void k_explore_keys(const uint32_t* __restrict__ tile_start,
                                                        const uint32_t* __restrict__ tile_seg, uint32_t T,
                                                        uint32_t n_seg, const SegState* __restrict__ states,
                                                        uint32_t* __restrict__ sure_bits, uint32_t* __restrict__ cand_bits,
                                                        uint32_t* __restrict__ cand_keys, uint32_t* __restrict__ cnt_cand,
                                                        uint64_t keys_stride, uint32_t worker0, PhiloxKey pk)
{
    __shared__ uint32_t wa[FAST ? 1 : 4][SUB_WORDS], wb[FAST ? 1 : 4][SUB_WORDS], wp[FAST ? 1 : 4][SUB_WORDS];
    const uint32_t b = blockIdx.y, worker = worker0 + b, wid = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t t0 = (uint32_t)((uint64_t)T * blockIdx.x / gridDim.x);
    const uint32_t t1 = (uint32_t)((uint64_t)T * (blockIdx.x + 1) / gridDim.x);
    DrawOut out;
    out.sure_bits = sure_bits + (size_t)b * T * TILE_WORDS;
    out.cand_bits = cand_bits + (size_t)b * T * TILE_WORDS;
    out.cand_keys = cand_keys + (size_t)b * keys_stride;
    out.cnt_cand = cnt_cand + (size_t)b * T * SUBS;
    for (uint32_t t = t0; t < t1; ++t) {
        const uint32_t seg = (n_seg == 1) ? 0u : tile_seg[t];
        const SegState* st = &states[(size_t)b * n_seg + seg];
        const uint32_t bound_m1 = st->bound_m1;
        const uint32_t sure_m1 = st->sure_m1, has_sure = st->has_gt;
        const uint32_t skip = st->need0 == 0;
        const uint32_t start = tile_start[t], len = tile_start[t + 1] - start;
        if (FAST)
            explore_subtile_fast<PAIRS>(worker, t, wid, start, len, bound_m1, sure_m1, has_sure, skip, out, pk, pk);
        else
            explore_subtile<PAIRS>(worker, t, wid, start, len, bound_m1, sure_m1, has_sure, skip, wa[FAST ? 0 : wid],
                            wb[FAST ? 0 : wid], wp[FAST ? 0 : wid], out, pk);
    }
}

// A wave walks one tile's candidates with every lane owning two bitmap words; the 16 lanes
// of a sub-tile find their place in that sub-tile's key list by a prefix inside the group.
__device__ __forceinline__ uint32_t sublist_pos(uint32_t lane, uint32_t my_count)
{
    const uint32_t excl = wave_incl_scan(my_count) - my_count;
    const uint32_t group0 = __shfl(excl, (int)(lane & ~15u), 64);
    return (lane >> 4) * SUB + (excl - group0);
}

// Where a tile is.  Flat model: no table look-ups, so that every load a tail kernel needs
// can be requested at once.
struct TileRef { uint32_t seg, start, len; };
__device__ __forceinline__ TileRef tile_ref(uint32_t t, uint32_t n_seg, uint64_t n, const uint32_t* __restrict__ tile_start,
                                            const uint32_t* __restrict__ tile_seg)
{
    TileRef r;
    if (n_seg == 1) {
        r.seg = 0; r.start = t * TILE;
        const uint64_t rest = n - (uint64_t)r.start;
        r.len = rest < TILE ? (uint32_t)rest : TILE;
    } else {
        r.seg = tile_seg[t]; r.start = tile_start[t]; r.len = tile_start[t + 1] - r.start;
    }
    return r;
}

// The first 16*KPL keys of each of a tile's four sub-lists, requested without waiting for
// the lists' lengths (the slots exist whatever the length; the unused ones are ignored):
// lane (s = lane/16, r = lane%16) holds entries r, r+16, ... of sub-list s.
template <int KPL>
__device__ __forceinline__ void load_sublists(const uint32_t* __restrict__ keys_tile, uint32_t lane, uint32_t kv[KPL])
{
    const uint32_t* p = keys_tile + (lane >> 4) * SUB + (lane & 15u);
#pragma unroll
    for (int i = 0; i < KPL; ++i) kv[i] = p[16 * i];
}

constexpr int EXPL_KPL = 2, CORE_KPL = 4;

// Bits [i0, i0 + 64) of a bitmap over all n parameters (i0 need not be word aligned).
__device__ __forceinline__ void bitmap_window(const uint32_t* __restrict__ bits, uint32_t n_words, uint32_t i0, uint32_t out[2])
{
    const uint32_t sh = i0 & 31u, wi = i0 >> 5;
    const uint32_t a0 = (wi < n_words) ? bits[wi] : 0u;
    const uint32_t a1 = (wi + 1 < n_words) ? bits[wi + 1] : 0u;
    const uint32_t a2 = (sh && wi + 2 < n_words) ? bits[wi + 2] : 0u;
    out[0] = sh ? ((a0 >> sh) | (a1 << (32u - sh))) : a0;
    out[1] = sh ? ((a1 >> sh) | (a2 << (32u - sh))) : a1;
}

// The draw does not know the core; this pass applies it.  Per (worker, tile), one wave:
//   sure zone: counts the sure parameters outside the core per sub-tile (cnt_gt; k_seg_sum
//     adds them up per segment); the bitmap itself stays as drawn, the emission masks it again;
//   candidate zone: candidates inside the core are dropped (bitmap bit cleared, the sub-tile's
//     key list closed up in place, its count lowered); the remaining keys feed the level-0
//     histogram.
// grid (blocks, n_workers), persistent so that the histogram stays in LDS.
__global__ __launch_bounds__(BLOCK) void k_explore_filter(const uint32_t* __restrict__ core_bits, uint64_t n,
                                                          const uint32_t* __restrict__ tile_start,
                                                          const uint32_t* __restrict__ tile_seg, uint32_t T,
                                                          uint32_t n_seg, const SegState* __restrict__ states,
                                                          uint32_t* __restrict__ hist, const uint32_t* __restrict__ sure_bits,
                                                          uint32_t* __restrict__ cnt_gt,
                                                          uint32_t* __restrict__ cand_bits, uint32_t* __restrict__ cand_keys,
                                                          uint32_t* __restrict__ cnt_cand, uint64_t keys_stride,
                                                          uint32_t n_words)
{
    __shared__ uint32_t h[4096];
    __shared__ uint32_t kl[4][SUB];
    const uint32_t b = blockIdx.y, lane = lane_id(), wid = threadIdx.x >> 6;
    for (uint32_t x = threadIdx.x; x < 4096; x += BLOCK) h[x] = 0;
    __syncthreads();
    const uint32_t t0 = (uint32_t)((uint64_t)T * blockIdx.x / gridDim.x);
    const uint32_t t1 = (uint32_t)((uint64_t)T * (blockIdx.x + 1) / gridDim.x);
    if (t0 >= t1) return;
    // one segment per block range: histogram in LDS; otherwise straight to global memory
    const uint32_t seg_first = (n_seg == 1) ? 0u : tile_seg[t0];
    const bool one_seg = (n_seg == 1) || seg_first == tile_seg[t1 - 1];
    const uint32_t hist_off = H_L0;
    uint32_t* klw = kl[wid];
    for (uint32_t t = t0 + wid; t < t1; t += 4) {
        const TileRef tr = tile_ref(t, n_seg, n, tile_start, tile_seg);
        const SegState* st = &states[(size_t)b * n_seg + tr.seg];
        const size_t bt = (size_t)b * T + t;
        // everything this tile needs is requested here, before any of it is used
        const uint2 s2 = *reinterpret_cast<const uint2*>(sure_bits + bt * TILE_WORDS + 2 * lane);
        const uint2 c2 = *reinterpret_cast<const uint2*>(cand_bits + bt * TILE_WORDS + 2 * lane);
        const uint32_t cnt = cnt_cand[bt * SUBS + (lane >> 4)];
        uint32_t kw[2];
        bitmap_window(core_bits, n_words, tr.start + lane * 64u, kw);
        const uint32_t need0 = st->need0, shift0 = st->shift[0], has_sure = st->has_gt;
        {
            uint32_t g = (has_sure && need0) ? __popc(s2.x & ~kw[0]) + __popc(s2.y & ~kw[1]) : 0u;
            g += __shfl_xor(g, 1, 64); g += __shfl_xor(g, 2, 64); g += __shfl_xor(g, 4, 64); g += __shfl_xor(g, 8, 64);
            if ((lane & 15u) == 0) cnt_gt[bt * SUBS + (lane >> 4)] = g;
        }
        if (need0 == 0) continue;
        const uint32_t cw[2] = {c2.x, c2.y};
        if (__ballot((cw[0] | cw[1]) != 0u) == 0ull) continue;
        const uint32_t nw[2] = {cw[0] & ~kw[0], cw[1] & ~kw[1]};
        const uint32_t oldc = __popc(cw[0]) + __popc(cw[1]), newc = __popc(nw[0]) + __popc(nw[1]);
        const uint32_t oi = wave_incl_scan(oldc), ni = wave_incl_scan(newc);
        const uint32_t og0 = __shfl(oi - oldc, (int)(lane & ~15u), 64), ng0 = __shfl(ni - newc, (int)(lane & ~15u), 64);
        uint32_t jo = oi - oldc - og0, jn = ni - newc - ng0;        // places in the sub-tile's old and new key list
        uint32_t* keys = cand_keys + (size_t)b * keys_stride + tr.start;
        uint32_t* hg = hist + ((size_t)b * n_seg + tr.seg) * H_STRIDE + hist_off;
#pragma unroll 1
        for (uint32_t s = 0; s < (uint32_t)SUBS; ++s) {
            const uint32_t c_s = __shfl(cnt, (int)(16u * s), 64);
            if (c_s == 0) continue;
            const bool mine = (lane >> 4) == s;
            const bool close_up = __ballot(mine && oldc != newc) != 0ull;
            uint32_t* ks = keys + s * SUB;
            for (uint32_t j = lane; j < c_s; j += 64) klw[j] = ks[j];   // the whole old list, before any of it is overwritten
            wave_sync();
            if (mine) {
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
                    uint32_t m = cw[hh];
                    while (m) {
                        const uint32_t p = __ffs(m) - 1;
                        m &= m - 1;
                        const uint32_t key = klw[jo++];
                        if ((kw[hh] >> p) & 1u) continue;
                        if (close_up) ks[jn] = key;
                        ++jn;
                        if (one_seg) atomicAdd(&h[key >> shift0], 1u);
                        else atomicAdd(&hg[key >> shift0], 1u);
                    }
                }
            }
            wave_sync();
            if (close_up && lane == 16u * s + 15u) cnt_cand[bt * SUBS + s] = ni - ng0;
        }
        if (__ballot(oldc != newc) != 0ull)
            *reinterpret_cast<uint2*>(cand_bits + bt * TILE_WORDS + 2 * lane) = make_uint2(nw[0], nw[1]);
    }
    __syncthreads();
    if (one_seg) flush_hist(h, 4096, hist + ((size_t)b * n_seg + seg_first) * H_STRIDE + hist_off);
}

// =======================================================================================
// Explorer, exact rerun.  When the zones of a draw missed (flags[0] raised; once in about
// 10^9 draws, or forced by a test switch) this kernel redoes the whole request from the
// definition, slowly and with no assumption: per worker one block walks every segment,
// finds the need-th smallest Philox word among the parameters outside the core by a
// three-pass radix descent over ALL of them (11 + 11 + 10 bits, words recomputed in every
// pass), then emits tile by tile in index order, ties at the threshold word going to the
// lowest indices.  grid (1, n_workers), 1024 threads; returns at once while the flag is down.
// =======================================================================================
__device__ __forceinline__ uint32_t explore_word(uint32_t i, uint32_t worker, PhiloxKey pk)
{
    uint32_t r[4];
    philox4x32_10(i >> 2, worker, pk.it_lo, pk.it_hi, pk.seed_lo, pk.seed_hi, r);
    const uint32_t c = i & 3u;
    return c == 0 ? r[0] : c == 1 ? r[1] : c == 2 ? r[2] : r[3];
}

__global__ __launch_bounds__(1024) void k_explore_exact(const uint32_t* __restrict__ core_bits, uint64_t n,
                                                        const uint32_t* __restrict__ tile_start,
                                                        const uint32_t* __restrict__ seg_first_tile, uint32_t T, uint32_t n_seg,
                                                        const SegState* __restrict__ states, uint32_t worker0, PhiloxKey pk,
                                                        MutPtrTab out_idx, MutPtrTab out_off, uint32_t expected,
                                                        uint32_t* __restrict__ flags)
{
    constexpr uint32_t NBIN = 2048;
    __shared__ uint32_t h[NBIN];
    __shared__ uint32_t wtot[16];
    __shared__ uint32_t sh[4];
    if (flags[0] == 0) return;                       // nobody raises the flag while this kernel runs
    const uint32_t b = blockIdx.y, worker = worker0 + b, tid = threadIdx.x;
    uint32_t* out = static_cast<uint32_t*>(out_idx.p[b]);
    uint32_t* off = static_cast<uint32_t*>(out_off.p[b]);
    uint32_t run = 0;                                // indices emitted so far (uniform)
    for (uint32_t seg = 0; seg < n_seg; ++seg) {
        const uint32_t f0 = seg_first_tile[seg], f1 = seg_first_tile[seg + 1];
        uint32_t need = states[(size_t)b * n_seg + seg].need0;
        // ---- the need-th smallest word: descent over bits 31..21, 20..10, 9..0
        uint32_t prefix = 0, short_of = 0;
        const uint32_t shifts[3] = {21u, 10u, 0u}, nbits[3] = {11u, 11u, 10u};
        for (int p = 0; p < 3 && need != 0 && !short_of; ++p) {
            for (uint32_t x = tid; x < NBIN; x += 1024) h[x] = 0;
            __syncthreads();
            const uint32_t hi_shift = shifts[p] + nbits[p];        // bits above this pass's digit
            for (uint32_t t = f0; t < f1; ++t) {
                const uint32_t start = tile_start[t], len = tile_start[t + 1] - start;
                for (uint32_t e = tid; e < len; e += 1024) {
                    const uint32_t i = start + e;
                    if ((core_bits[i >> 5] >> (i & 31u)) & 1u) continue;
                    const uint32_t r = explore_word(i, worker, pk);
                    if (hi_shift < 32u && (r >> hi_shift) != prefix) continue;
                    atomicAdd(&h[(r >> shifts[p]) & ((1u << nbits[p]) - 1u)], 1u);
                }
            }
            __syncthreads();
            // the bin that holds the need-th smallest: two bins per thread, ascending
            const uint32_t c0 = h[2 * tid], c1 = h[2 * tid + 1];
            uint32_t total;
            const uint32_t excl = block_excl_scan<16>(c0 + c1, wtot, total);
            if (tid == 0) sh[2] = (total < need) ? 1u : 0u;
            if (excl < need && need <= excl + c0) { sh[0] = 2 * tid; sh[1] = need - excl; }
            else if (excl + c0 < need && need <= excl + c0 + c1) { sh[0] = 2 * tid + 1; sh[1] = need - excl - c0; }
            __syncthreads();
            if (sh[2]) { short_of = 1; if (tid == 0) atomicOr(&flags[1], 2u); }     // fewer eligible parameters than requested
            else { prefix = (prefix << nbits[p]) | sh[0]; need = sh[1]; }
            __syncthreads();
        }
        // words below tau are taken, of the words equal to tau the first `need` in index order
        const uint32_t tau = short_of ? 0xFFFFFFFFu : prefix;
        const uint32_t take_all = short_of;
        const uint32_t want = states[(size_t)b * n_seg + seg].need0;
        uint32_t ties_seen = 0;                      // uniform
        // ---- ordered emission, tile by tile (four consecutive parameters per thread)
        for (uint32_t t = f0; t < f1; ++t) {
            const uint32_t start = tile_start[t], len = tile_start[t + 1] - start;
            uint32_t sel = 0, tie = 0;
            if (want != 0) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t e = 4u * tid + c;
                    if (e >= len) continue;
                    const uint32_t i = start + e;
                    if ((core_bits[i >> 5] >> (i & 31u)) & 1u) continue;
                    const uint32_t r = explore_word(i, worker, pk);
                    if (take_all || r < tau) sel |= 1u << c;
                    else if (r == tau) tie |= 1u << c;
                }
            }
            uint32_t tie_total;
            const uint32_t tie_excl = block_excl_scan<16>(__popc(tie), wtot, tie_total);
            uint32_t rank = ties_seen + tie_excl;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if ((tie >> c) & 1u) { if (rank < need) sel |= 1u << c; ++rank; }
            ties_seen += tie_total;
            uint32_t sel_total;
            uint32_t o = run + block_excl_scan<16>(__popc(sel), wtot, sel_total);
            if (tid == 0) off[t] = run;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if ((sel >> c) & 1u) { if (o < expected) out[o] = start + 4u * tid + c; ++o; }
            run += sel_total;
        }
    }
    if (tid == 0) {
        off[T] = run;
        if (run != expected) atomicOr(&flags[1], 1u);
    }
}

// =======================================================================================
// Explorer, short-list path (every segment's candidate zone is narrow, draw with PAIRS = 1).
// The few candidates outside the core are collected into one unordered list; the radix
// descent, the decision against tau and the tie ranks run over that list; the chosen
// candidates are then set in the sure bitmap, which alone drives the ordered emission.
// Every kernel of the path returns at once when flags[0] is raised (the exact rerun with
// the per-tile path follows), except where noted.
// =======================================================================================
// list entry: x = key, y = t * TILE + offset inside the tile, z = b * n_seg + seg, w = b
constexpr uint32_t FLAG_RERUN = 1u;

// Sure parameters outside the core, counted per tile (cnt_sel).  One wave per tile, serving
// BPW batches.  grid (ceil(T/4), ceil(nbatch / BPW)).  Runs whatever the flag.
template <int BPW>
__global__ __launch_bounds__(BLOCK) void k_sure_count(const uint32_t* __restrict__ core_bits, uint32_t n_words, uint64_t n,
                                                      const uint32_t* __restrict__ tile_start,
                                                      const uint32_t* __restrict__ tile_seg, uint32_t T, uint32_t n_seg,
                                                      uint32_t nbatch, const uint32_t* __restrict__ sure_bits,
                                                      uint32_t* __restrict__ cnt_sel)
{
    const uint32_t t = blockIdx.x * 4 + (threadIdx.x >> 6), b0 = blockIdx.y * BPW, lane = lane_id();
    if (t >= T) return;
    const TileRef tr = tile_ref(t, n_seg, n, tile_start, tile_seg);
    uint2 s2[BPW];
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        s2[bb] = make_uint2(0u, 0u);
        if (b0 + bb < nbatch)
            s2[bb] = *reinterpret_cast<const uint2*>(sure_bits + ((size_t)(b0 + bb) * T + t) * TILE_WORDS + 2 * lane);
    }
    uint32_t kw[2];
    bitmap_window(core_bits, n_words, tr.start + lane * 64u, kw);
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        if (b0 + bb >= nbatch) break;
        const uint32_t tot = wave_sum(__popc(s2[bb].x & ~kw[0]) + __popc(s2[bb].y & ~kw[1]));
        if (lane == 0) cnt_sel[(size_t)(b0 + bb) * T + t] = tot;
    }
}

// nsure[b][seg] = sum of `per` consecutive counts for every tile of the segment.  No atomics:
// thousands of them on one cache line take longer than this whole kernel.
// grid (n_seg, nbatch), 1024 threads.
__global__ __launch_bounds__(1024) void k_seg_sum(const uint32_t* __restrict__ counts, uint32_t per,
                                                  const uint32_t* __restrict__ seg_first_tile, uint32_t T, uint32_t n_seg,
                                                  uint32_t* __restrict__ nsure)
{
    __shared__ uint32_t wtot[16];
    const uint32_t seg = blockIdx.x, b = blockIdx.y;
    const size_t x0 = ((size_t)b * T + seg_first_tile[seg]) * per, x1 = ((size_t)b * T + seg_first_tile[seg + 1]) * per;
    uint32_t sum = 0;
    for (size_t x = x0 + threadIdx.x; x < x1; x += 1024) sum += counts[x];
    uint32_t total;
    (void)block_excl_scan<16>(sum, wtot, total);
    if (threadIdx.x == 0) nsure[(size_t)b * n_seg + seg] = total;
}

// Candidates outside the core -> list.  One thread per (batch, tile); a block reserves its
// share of the list with one atomic.  A sub-tile with more pairs than its slot holds, or a
// full list, raises the rerun flag.  keys_stride: words per batch of the pair slots.  grid ceil(nbatch * T / 1024), 1024 threads.
__global__ __launch_bounds__(1024) void k_cand_gather(const uint32_t* __restrict__ core_bits, uint64_t n,
                                                      const uint32_t* __restrict__ tile_start,
                                                      const uint32_t* __restrict__ tile_seg, uint32_t T, uint32_t n_seg,
                                                      uint32_t nbatch, const uint32_t* __restrict__ cand_keys,
                                                      uint64_t keys_stride, const uint32_t* __restrict__ cnt_cand,
                                                      uint4* __restrict__ list, uint32_t* __restrict__ list_count,
                                                      uint32_t list_cap, uint32_t* __restrict__ flags)
{
    __shared__ uint32_t wtot[16];
    __shared__ uint32_t sh_base;
    if (threadIdx.x == 0) sh_base = flags[0];      // other blocks may raise the flag: one read per block
    __syncthreads();
    if (sh_base != 0) return;
    const uint32_t x = blockIdx.x * 1024 + threadIdx.x;
    const bool live = x < nbatch * T;
    const uint32_t b = live ? x / T : 0u, t = live ? x % T : 0u;
    uint4 c4 = make_uint4(0u, 0u, 0u, 0u);
    if (live) c4 = *reinterpret_cast<const uint4*>(cnt_cand + (size_t)x * SUBS);
    uint32_t cs[SUBS] = {c4.x, c4.y, c4.z, c4.w};
    bool over = false;
#pragma unroll
    for (int sub = 0; sub < SUBS; ++sub)
        if (cs[sub] > PAIR_CAP) { over = true; cs[sub] = 0; }
    if (over) atomicOr(&flags[0], FLAG_RERUN);
    uint32_t mine = 0;
    TileRef tr{0u, 0u, 0u};
    const uint32_t* keys = cand_keys;
    if (cs[0] | cs[1] | cs[2] | cs[3]) {
        tr = tile_ref(t, n_seg, n, tile_start, tile_seg);
        keys = cand_keys + (size_t)b * keys_stride + (size_t)t * SUBS * PAIR_SLOT;
#pragma unroll 1
        for (int sub = 0; sub < SUBS; ++sub)
            for (uint32_t j = 0; j < cs[sub]; ++j) {
                const uint32_t i = tr.start + sub * SUB + keys[sub * PAIR_SLOT + 2 * j + 1];
                mine += ((core_bits[i >> 5] >> (i & 31u)) & 1u) ^ 1u;
            }
    }
    uint32_t total;
    const uint32_t excl = block_excl_scan<16>(mine, wtot, total);
    if (total == 0) return;
    if (threadIdx.x == 0) sh_base = atomicAdd(list_count, total);
    __syncthreads();
    const uint32_t base = sh_base;
    if (base + total > list_cap || base + total < base) {
        if (threadIdx.x == 0) atomicOr(&flags[0], FLAG_RERUN);
        return;
    }
    if (mine == 0) return;
    uint32_t o = base + excl;
#pragma unroll 1
    for (int sub = 0; sub < SUBS; ++sub)
        for (uint32_t j = 0; j < cs[sub]; ++j) {
            const uint32_t key = keys[sub * PAIR_SLOT + 2 * j], e = keys[sub * PAIR_SLOT + 2 * j + 1];
            const uint32_t i = tr.start + sub * SUB + e;
            if ((core_bits[i >> 5] >> (i & 31u)) & 1u) continue;
            list[o++] = make_uint4(key, t * TILE + sub * SUB + e, b * n_seg + tr.seg, b);
        }
}

// Histogram of one radix level over the list.  grid: any, grid-stride.
__global__ __launch_bounds__(256) void k_short_hist(const uint4* __restrict__ list, const uint32_t* __restrict__ list_count,
                                                    uint32_t list_cap, const SegState* __restrict__ states,
                                                    uint32_t* __restrict__ hist, uint32_t hist_off, int level,
                                                    const uint32_t* __restrict__ flags)
{
    if (flags[0] != 0) return;
    const uint32_t cnt = min(list_count[0], list_cap);
    for (uint32_t j = blockIdx.x * 256 + threadIdx.x; j < cnt; j += gridDim.x * 256) {
        const uint4 e = list[j];
        const SegState* st = &states[e.z];
        if (st->none) continue;
        uint32_t digit;
        if (level == 0) digit = e.x >> st->shift[0];
        else {
            if ((e.x >> st->shift[level - 1]) != st->prefix) continue;
            digit = (e.x >> st->shift[level]) & (st->nbins[level] - 1u);
        }
        atomicAdd(&hist[(size_t)e.z * H_STRIDE + hist_off + digit], 1u);
    }
}

// Decision of every list entry against its segment's tau.  A chosen candidate is added to
// the sure bitmap and to its tile's count.  Entries equal to tau: all taken if the quota
// covers them all, otherwise they go to the tie list for k_short_ties (a full tie list raises
// the rerun flag).
constexpr uint32_t TIE_CAP = 4096;
__device__ __forceinline__ void short_take(const uint4 e, uint32_t T, uint32_t* __restrict__ sure_bits,
                                           uint32_t* __restrict__ cnt_sel)
{
    const uint32_t t = e.y / TILE, o = e.y % TILE;
    atomicOr(&sure_bits[((size_t)e.w * T + t) * TILE_WORDS + (o >> 5)], 1u << (o & 31u));
    atomicAdd(&cnt_sel[(size_t)e.w * T + t], 1u);
}

__global__ __launch_bounds__(256) void k_short_mark(const uint4* __restrict__ list, const uint32_t* __restrict__ list_count,
                                                    uint32_t list_cap, const SegState* __restrict__ states, uint32_t T,
                                                    uint32_t* __restrict__ sure_bits, uint32_t* __restrict__ cnt_sel,
                                                    uint32_t* __restrict__ tie_list, uint32_t* __restrict__ tie_count,
                                                    uint32_t* __restrict__ flags)
{
    if (flags[0] != 0) return;
    const uint32_t cnt = min(list_count[0], list_cap);
    for (uint32_t j = blockIdx.x * 256 + threadIdx.x; j < cnt; j += gridDim.x * 256) {
        const uint4 e = list[j];
        const SegState* st = &states[e.z];
        if (st->none) continue;
        const uint32_t tau = st->tau;
        if (e.x > tau || (e.x == tau && st->tie_all)) short_take(e, T, sure_bits, cnt_sel);
        else if (e.x == tau && st->quota != 0) {
            const uint32_t slot = atomicAdd(tie_count, 1u);
            if (slot < TIE_CAP) tie_list[slot] = j;
            else atomicOr(&flags[0], FLAG_RERUN);
        }
    }
}

// Ties that the quota covers only in part: the quota goes to the lowest positions.  Every
// entry equal to its segment's tau is on the tie list, so the rank of a tied entry is the
// number of tie-list entries of its segment below it.  One block; nothing to do as a rule.
__global__ __launch_bounds__(1024) void k_short_ties(const uint4* __restrict__ list, const SegState* __restrict__ states,
                                                     uint32_t T, uint32_t* __restrict__ sure_bits,
                                                     uint32_t* __restrict__ cnt_sel, const uint32_t* __restrict__ tie_list,
                                                     const uint32_t* __restrict__ tie_count, const uint32_t* __restrict__ flags)
{
    if (flags[0] != 0) return;
    const uint32_t nt = min(tie_count[0], TIE_CAP);
    for (uint32_t q = threadIdx.x; q < nt; q += 1024) {
        const uint4 e = list[tie_list[q]];
        uint32_t rank = 0;
        for (uint32_t p = 0; p < nt; ++p) {
            const uint4 o = list[tie_list[p]];
            rank += (o.z == e.z && o.y < e.y) ? 1u : 0u;
        }
        if (rank < states[e.z].quota) short_take(e, T, sure_bits, cnt_sel);
    }
}

// Exclusive prefix of the tile counts inside chunks of SCAN_CHUNK tiles, and the chunk sums.
// grid (ceil(T / SCAN_CHUNK), nbatch), 1024 threads.
constexpr uint32_t SCAN_CHUNK = 8192, SCAN_PER = SCAN_CHUNK / 1024;
__device__ __forceinline__ uint32_t scan_phys(uint32_t x) { return x + (x >> 3); }     // one pad word per thread row

// vals: SCAN_CHUNK*9/8 words; wtot: 16 words.  Values of the chunk are already in vals
// (physical layout).  On return vals holds each value's exclusive prefix inside the chunk.
__device__ __forceinline__ uint32_t scan_chunk(uint32_t* vals, uint32_t* wtot)
{
    uint32_t s = 0;
    const uint32_t row = threadIdx.x * (SCAN_PER + 1);
#pragma unroll
    for (uint32_t e = 0; e < SCAN_PER; ++e) { const uint32_t v = vals[row + e]; vals[row + e] = s; s += v; }
    uint32_t total;
    const uint32_t base = block_excl_scan<16>(s, wtot, total);
#pragma unroll
    for (uint32_t e = 0; e < SCAN_PER; ++e) vals[row + e] += base;
    __syncthreads();
    return total;
}

__global__ __launch_bounds__(1024) void k_chunk_scan(uint32_t T, const uint32_t* __restrict__ cnt_sel, MutPtrTab out_off,
                                                     uint32_t* __restrict__ chunk_sum, const uint32_t* __restrict__ flags)
{
    __shared__ uint32_t vals[SCAN_CHUNK + SCAN_CHUNK / 8];
    __shared__ uint32_t wtot[16];
    if (flags[0] != 0) return;
    const uint32_t b = blockIdx.y, c0 = blockIdx.x * SCAN_CHUNK;
    const uint32_t* cs = cnt_sel + (size_t)b * T;
    uint32_t* off = static_cast<uint32_t*>(out_off.p[b]);
    for (uint32_t x = threadIdx.x; x < SCAN_CHUNK; x += 1024) vals[scan_phys(x)] = (c0 + x < T) ? cs[c0 + x] : 0u;
    __syncthreads();
    const uint32_t total = scan_chunk(vals, wtot);
    for (uint32_t x = threadIdx.x; x < SCAN_CHUNK && c0 + x < T; x += 1024) off[c0 + x] = vals[scan_phys(x)];
    if (threadIdx.x == 0) chunk_sum[(size_t)b * gridDim.x + blockIdx.x] = total;
}

// Ordered emission from the sure bitmap (chosen candidates included) minus the core.  One
// wave per tile and BPW batches; the wave also turns its tile's chunk-relative offset into
// the final one.  grid (ceil(T/4), ceil(nbatch/BPW)).
template <int BPW>
__global__ __launch_bounds__(BLOCK) void k_emit_bits(const uint32_t* __restrict__ core_bits, uint32_t n_words, uint64_t n,
                                                     const uint32_t* __restrict__ tile_start,
                                                     const uint32_t* __restrict__ tile_seg, uint32_t T, uint32_t n_seg,
                                                     uint32_t nbatch, const uint32_t* __restrict__ sure_bits,
                                                     const uint32_t* __restrict__ chunk_sum, uint32_t n_chunks,
                                                     MutPtrTab out_off, MutPtrTab out_idx, uint32_t expected,
                                                     uint32_t* __restrict__ flags)
{
    if (flags[0] != 0) return;
    const uint32_t t = blockIdx.x * 4 + (threadIdx.x >> 6), b0 = blockIdx.y * BPW, lane = lane_id();
    if (t >= T) return;
    const TileRef tr = tile_ref(t, n_seg, n, tile_start, tile_seg);
    const uint32_t chunk = t / SCAN_CHUNK;
    uint2 s2[BPW];
    uint32_t off_t[BPW];
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        s2[bb] = make_uint2(0u, 0u); off_t[bb] = 0;
        if (b0 + bb < nbatch) {
            s2[bb] = *reinterpret_cast<const uint2*>(sure_bits + ((size_t)(b0 + bb) * T + t) * TILE_WORDS + 2 * lane);
            off_t[bb] = static_cast<const uint32_t*>(out_off.p[b0 + bb])[t];
        }
    }
    uint32_t kw[2];
    bitmap_window(core_bits, n_words, tr.start + lane * 64u, kw);
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        const uint32_t b = b0 + bb;
        if (b >= nbatch) break;
        uint32_t first = off_t[bb];
        for (uint32_t c = 0; c < chunk; ++c) first += chunk_sum[(size_t)b * n_chunks + c];
        const uint32_t fm0 = s2[bb].x & ~kw[0], fm1 = s2[bb].y & ~kw[1];
        const uint32_t ocnt = __popc(fm0) + __popc(fm1);
        const uint32_t incl = wave_incl_scan(ocnt);
        uint32_t* out = static_cast<uint32_t*>(out_idx.p[b]);
        uint32_t* off = static_cast<uint32_t*>(out_off.p[b]);
        if (lane == 0) off[t] = first;
        if (t == T - 1 && lane == 63) {
            off[T] = first + incl;
            if (first + incl != expected) atomicOr(&flags[1], 1u);
        }
        uint32_t o = first + incl - ocnt;
        uint32_t m = fm0;
        while (m) {
            const uint32_t p = __ffs(m) - 1;
            m &= m - 1;
            if (o < expected) out[o] = tr.start + lane * 64u + p;     // never beyond the caller's list
            ++o;
        }
        m = fm1;
        while (m) {
            const uint32_t p = __ffs(m) - 1;
            m &= m - 1;
            if (o < expected) out[o] = tr.start + lane * 64u + 32u + p;
            ++o;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Levels 1 and 2: histogram of the candidates that still match the prefix.  One wave per
// tile, 16 lanes per sub-tile list; equal digits inside a wave are merged before the
// global atomic.  grid (ceil(T/4), nbatch).
// ---------------------------------------------------------------------------------------
template <int KPL, int BPW>
__global__ __launch_bounds__(BLOCK) void k_list_hist(uint64_t n, const uint32_t* __restrict__ tile_start,
                                                     const uint32_t* __restrict__ tile_seg, uint32_t T, uint32_t n_seg,
                                                     uint32_t nbatch, const SegState* __restrict__ states,
                                                     uint32_t* __restrict__ hist, uint32_t hist_off, int level,
                                                     const uint32_t* __restrict__ cand_keys,
                                                     const uint32_t* __restrict__ cnt_cand, uint64_t keys_stride,
                                                     const uint32_t* __restrict__ gate)
{
    const uint32_t t = blockIdx.x * 4 + (threadIdx.x >> 6), b0 = blockIdx.y * BPW, lane = lane_id();
    if (t >= T || (gate && gate[0] != 0)) return;
    const TileRef tr = tile_ref(t, n_seg, n, tile_start, tile_seg);
    // one wave serves the tile for BPW batches: all their loads are requested before any is used
    uint32_t kv[BPW][KPL], cnt[BPW];
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        const uint32_t b = b0 + bb;
        cnt[bb] = 0;
        if (b < nbatch) {
            load_sublists<KPL>(cand_keys + (size_t)b * keys_stride + tr.start, lane, kv[bb]);
            cnt[bb] = cnt_cand[((size_t)b * T + t) * SUBS + (lane >> 4)];
        }
    }
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        const uint32_t b = b0 + bb;
        if (b >= nbatch) break;
        const SegState* st = &states[(size_t)b * n_seg + tr.seg];
        if (st->none) continue;
        const uint32_t pshift = st->shift[level - 1], shift = st->shift[level], mask = st->nbins[level] - 1u;
        const uint32_t prefix = st->prefix;
        const uint32_t c = cnt[bb];
        const uint32_t maxcnt = max(max(__shfl(c, 0, 64), __shfl(c, 16, 64)), max(__shfl(c, 32, 64), __shfl(c, 48, 64)));
        const uint32_t* keys = cand_keys + (size_t)b * keys_stride + tr.start + (lane >> 4) * SUB;
        uint32_t* hp = hist + ((size_t)b * n_seg + tr.seg) * H_STRIDE + hist_off;
        for (uint32_t j0 = 0; j0 < maxcnt; j0 += 16) {
            const uint32_t j = j0 + (lane & 15u);
            uint32_t k = 0;
            if (j0 < 16u * KPL) {
#pragma unroll
                for (int i = 0; i < KPL; ++i) if (j0 == 16u * i) k = kv[bb][i];
            } else if (j < c) {
                k = keys[j];
            }
            bool part = (j < c) && (k >> pshift) == prefix;
            const uint32_t digit = (k >> shift) & mask;
            unsigned long long active = __ballot(part);
            while (active) {
                const int leader = __ffsll((long long)active) - 1;
                const uint32_t d = __shfl(digit, leader, 64);
                const unsigned long long same = __ballot(part && digit == d);
                if ((int)lane == leader) atomicAdd(&hp[d], (uint32_t)__popcll(same));
                if (digit == d) part = false;
                active &= ~same;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Per-tile counts once tau is known: selected-for-sure (gt + keys > tau) and ties (== tau).
// One wave per tile and BPW batches.  grid (ceil(T/4), ceil(nbatch/BPW)).
// ---------------------------------------------------------------------------------------
template <int KPL, int BPW>
__global__ __launch_bounds__(BLOCK) void k_count(uint64_t n, const uint32_t* __restrict__ tile_start,
                                                 const uint32_t* __restrict__ tile_seg, uint32_t T, uint32_t n_seg,
                                                 uint32_t nbatch, const SegState* __restrict__ states,
                                                 const uint32_t* __restrict__ cand_keys, const uint32_t* __restrict__ cnt_cand,
                                                 const uint32_t* __restrict__ cnt_gt, uint64_t keys_stride,
                                                 uint32_t* __restrict__ cnt_sel, uint32_t* __restrict__ cnt_tie,
                                                 const uint32_t* __restrict__ gate)
{
    const uint32_t t = blockIdx.x * 4 + (threadIdx.x >> 6), b0 = blockIdx.y * BPW, lane = lane_id();
    if (t >= T || (gate && gate[0] != 0)) return;
    const TileRef tr = tile_ref(t, n_seg, n, tile_start, tile_seg);
    uint32_t kv[BPW][KPL], cnt[BPW];
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        const uint32_t b = b0 + bb;
        cnt[bb] = 0;
        if (b < nbatch) {
            load_sublists<KPL>(cand_keys + (size_t)b * keys_stride + tr.start, lane, kv[bb]);
            cnt[bb] = cnt_cand[((size_t)b * T + t) * SUBS + (lane >> 4)];
        }
    }
    uint32_t gtc[BPW];
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        gtc[bb] = 0;
        if (cnt_gt && b0 + bb < nbatch) {
            const uint4 g4 = *reinterpret_cast<const uint4*>(cnt_gt + ((size_t)(b0 + bb) * T + t) * SUBS);
            gtc[bb] = g4.x + g4.y + g4.z + g4.w;
        }
    }
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        const uint32_t b = b0 + bb;
        if (b >= nbatch) break;
        const SegState* st = &states[(size_t)b * n_seg + tr.seg];
        uint32_t sel = 0, tie = 0;
        if (!st->none) {
            const uint32_t tau = st->tau, c = cnt[bb];
            const uint32_t* keys = cand_keys + (size_t)b * keys_stride + tr.start + (lane >> 4) * SUB;
#pragma unroll
            for (int i = 0; i < KPL; ++i) {
                const uint32_t k = kv[bb][i];
                if ((lane & 15u) + 16u * i < c) {
                    sel += (k > tau) ? 1u : 0u;
                    tie += (k == tau) ? 1u : 0u;
                }
            }
            for (uint32_t j = (lane & 15u) + 16u * KPL; j < c; j += 16) {
                const uint32_t k = keys[j];
                sel += (k > tau) ? 1u : 0u;
                tie += (k == tau) ? 1u : 0u;
            }
            sel = wave_sum(sel);
            tie = wave_sum(tie);
        }
        if (st->has_gt && st->need0) sel += gtc[bb];
        if (lane == 0) { cnt_sel[(size_t)b * T + t] = sel; cnt_tie[(size_t)b * T + t] = tie; }
    }
}

// ---------------------------------------------------------------------------------------
// Scan over tiles in chunks of SCAN_CHUNK tiles, one block per chunk and batch; a value
// of the whole array is its chunk-relative prefix plus the sums of the chunks before it
// (chunk_base).  Two passes: PASS 0 over the tie counts (tie_pre), PASS 1 over what each
// tile emits (certain ones plus the ties it takes under its segment's quota) -> out_off.
// The emission turns the chunk-relative offsets into final ones.
// grid (ceil(T / SCAN_CHUNK), nbatch), 1024 threads.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t chunk_base(const uint32_t* __restrict__ sums, uint32_t chunk)
{
    uint32_t base = 0;
    for (uint32_t c = 0; c < chunk; ++c) base += sums[c];
    return base;
}

template <int PASS>
__global__ __launch_bounds__(1024) void k_tile_scan(const uint32_t* __restrict__ tile_seg,
                                                    const uint32_t* __restrict__ seg_first_tile, uint32_t T, uint32_t n_seg,
                                                    const SegState* __restrict__ states, const uint32_t* __restrict__ cnt_sel,
                                                    const uint32_t* __restrict__ cnt_tie, uint32_t* __restrict__ tie_pre,
                                                    uint32_t* __restrict__ tie_sum, MutPtrTab out_off,
                                                    uint32_t* __restrict__ off_sum, const uint32_t* __restrict__ gate)
{
    __shared__ uint32_t vals[SCAN_CHUNK + SCAN_CHUNK / 8];
    __shared__ uint32_t wtot[16];
    if (gate && gate[0] != 0) return;
    const uint32_t b = blockIdx.y, c0 = blockIdx.x * SCAN_CHUNK, n_chunks = gridDim.x;
    const uint32_t* cs = cnt_sel + (size_t)b * T;
    const uint32_t* ct = cnt_tie + (size_t)b * T;
    uint32_t* tp = tie_pre + (size_t)b * (T + 1);
    const uint32_t* ts = tie_sum + (size_t)b * n_chunks;
    for (uint32_t x = threadIdx.x; x < SCAN_CHUNK; x += 1024) {
        const uint32_t t = c0 + x;
        uint32_t v = 0;
        if (t < T) {
            const uint32_t c = ct[t];
            if (PASS == 0) v = c;
            else {
                // ties before this tile inside its segment, against the segment's quota
                const SegState* st = states + (size_t)b * n_seg;
                const uint32_t seg = (n_seg == 1) ? 0u : tile_seg[t];
                uint32_t before = tp[t] + chunk_base(ts, blockIdx.x);
                if (n_seg != 1) {
                    const uint32_t f = seg_first_tile[seg];
                    before -= tp[f] + chunk_base(ts, f / SCAN_CHUNK);
                }
                const uint32_t q = st[seg].quota;
                const uint32_t room = (q > before) ? q - before : 0u;
                v = cs[t] + (room < c ? room : c);
            }
        }
        vals[scan_phys(x)] = v;
    }
    __syncthreads();
    const uint32_t total = scan_chunk(vals, wtot);
    uint32_t* dst = (PASS == 0) ? tp : static_cast<uint32_t*>(out_off.p[b]);
    for (uint32_t x = threadIdx.x; x < SCAN_CHUNK && c0 + x < T; x += 1024) dst[c0 + x] = vals[scan_phys(x)];
    if (threadIdx.x == 0) ((PASS == 0) ? tie_sum : off_sum)[(size_t)b * n_chunks + blockIdx.x] = total;
}

// ---------------------------------------------------------------------------------------
// K3: ordered emission.  One wave per (tile, batch), each lane owning two consecutive
// bitmap words: decide every candidate against tau, hand out the tie quota in index
// order, and write the tile's chosen indices at its offset.  grid (ceil(T/4), nbatch).
// ---------------------------------------------------------------------------------------
template <int KPL, int BPW>
__global__ __launch_bounds__(BLOCK) void k_emit(uint64_t n, const uint32_t* __restrict__ tile_start,
                                                const uint32_t* __restrict__ tile_seg,
                                                const uint32_t* __restrict__ seg_first_tile, uint32_t T, uint32_t n_seg,
                                                uint32_t nbatch, const SegState* __restrict__ states,
                                                const uint32_t* __restrict__ gt_bits, const uint32_t* __restrict__ cand_bits,
                                                const uint32_t* __restrict__ cand_keys, uint64_t keys_stride,
                                                const uint32_t* __restrict__ tie_pre, MutPtrTab out_off, MutPtrTab out_idx,
                                                uint32_t expected, uint32_t* __restrict__ pub_bits,
                                                const uint32_t* __restrict__ excl_bits, uint32_t n_words,
                                                const uint32_t* __restrict__ gate, const uint32_t* __restrict__ tie_sum,
                                                const uint32_t* __restrict__ off_sum, uint32_t n_chunks,
                                                uint32_t* __restrict__ flags)
{
    __shared__ uint32_t kb[4][SUBS * 16 * KPL];
    const uint32_t wid = threadIdx.x >> 6;
    const uint32_t t = blockIdx.x * 4 + wid, b0 = blockIdx.y * BPW, lane = lane_id();
    if (t >= T || (gate && gate[0] != 0)) return;
    const TileRef tr = tile_ref(t, n_seg, n, tile_start, tile_seg);
    const uint32_t start = tr.start, len = tr.len, seg = tr.seg;
    // one wave serves the tile for BPW batches: all their loads are requested before any is used
    uint2 c2[BPW];
    uint32_t kv[BPW][KPL], off_t[BPW], tp_t[BPW];
    uint2 g2[BPW];
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        const uint32_t b = b0 + bb;
        c2[bb] = make_uint2(0u, 0u); g2[bb] = make_uint2(0u, 0u); off_t[bb] = 0; tp_t[bb] = 0;
        if (b < nbatch) {
            if (gt_bits) g2[bb] = *reinterpret_cast<const uint2*>(gt_bits + ((size_t)b * T + t) * TILE_WORDS + 2 * lane);
            c2[bb] = *reinterpret_cast<const uint2*>(cand_bits + ((size_t)b * T + t) * TILE_WORDS + 2 * lane);
            load_sublists<KPL>(cand_keys + (size_t)b * keys_stride + start, lane, kv[bb]);
            off_t[bb] = static_cast<const uint32_t*>(out_off.p[b])[t];
            tp_t[bb] = tie_pre[(size_t)b * (T + 1) + t];
        }
    }
    uint32_t xw[2] = {0u, 0u};      // parameters that the certainly-selected bitmap must not contribute (explorer: the core)
    if (excl_bits) bitmap_window(excl_bits, n_words, start + lane * 64u, xw);
    uint32_t* kbw = kb[wid];
#pragma unroll
    for (int bb = 0; bb < BPW; ++bb) {
        const uint32_t b = b0 + bb;
        if (b >= nbatch) break;
        const SegState* st = &states[(size_t)b * n_seg + seg];
        const uint32_t* keys = cand_keys + (size_t)b * keys_stride + start;
        const uint32_t* tp = tie_pre + (size_t)b * (T + 1);
        const uint32_t none = st->none, tau = st->tau, quota = st->quota;
        uint32_t cw[2] = {0u, 0u}, gw[2] = {0u, 0u};
        if (!none) { cw[0] = c2[bb].x; cw[1] = c2[bb].y; }
        if (st->has_gt && st->need0) { gw[0] = g2[bb].x & ~xw[0]; gw[1] = g2[bb].y & ~xw[1]; }
        wave_sync();
#pragma unroll
        for (int i = 0; i < KPL; ++i) kbw[(lane >> 4) * (16 * KPL) + (lane & 15u) + 16 * i] = kv[bb][i];
        wave_sync();
        const uint32_t pos = sublist_pos(lane, __popc(cw[0]) + __popc(cw[1]));
        const uint32_t sub = pos >> 10;
        uint32_t j = pos & (SUB - 1u);
        uint32_t selmask[2] = {0u, 0u}, tiemask[2] = {0u, 0u};
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t m = cw[h];
            while (m) {
                const uint32_t p = __ffs(m) - 1;
                m &= m - 1;
                const uint32_t k = (j < 16u * KPL) ? kbw[sub * (16 * KPL) + j] : keys[sub * SUB + j];
                ++j;
                if (k > tau) selmask[h] |= 1u << p;
                else if (k == tau) tiemask[h] |= 1u << p;
            }
        }
        const uint32_t tcnt = __popc(tiemask[0]) + __popc(tiemask[1]);
        uint32_t taken[2] = {0u, 0u};
        if (__ballot(tcnt != 0)) {
            const uint32_t* ts = tie_sum + (size_t)b * n_chunks;
            uint32_t tp_seg = 0;
            if (n_seg != 1) {
                const uint32_t f = seg_first_tile[seg];
                tp_seg = tp[f] + chunk_base(ts, f / SCAN_CHUNK);
            }
            const uint32_t tbase = tp_t[bb] + chunk_base(ts, t / SCAN_CHUNK) - tp_seg + wave_incl_scan(tcnt) - tcnt;
            uint32_t take = (quota > tbase) ? quota - tbase : 0u;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                uint32_t m = tiemask[h];
                while (m && take) { const uint32_t low = m & (0u - m); taken[h] |= low; m ^= low; --take; }
            }
        }
        const uint32_t fm0 = gw[0] | selmask[0] | taken[0], fm1 = gw[1] | selmask[1] | taken[1];
        const uint32_t ocnt = __popc(fm0) + __popc(fm1);
        uint32_t* out = static_cast<uint32_t*>(out_idx.p[b]);
        // the tile's offset so far counts from its chunk: make it final, for this emission and for the caller
        const uint32_t first = off_t[bb] + chunk_base(off_sum + (size_t)b * n_chunks, t / SCAN_CHUNK);
        const uint32_t oincl = wave_incl_scan(ocnt);
        uint32_t* off = static_cast<uint32_t*>(out_off.p[b]);
        if (lane == 0) off[t] = first;
        if (t == T - 1 && lane == 63) {
            off[T] = first + oincl;
            if (first + oincl != expected) atomicOr(&flags[1], 1u);
        }
        uint32_t o = first + oincl - ocnt;
        {
            uint32_t m = fm0;
            while (m) {
                const uint32_t p = __ffs(m) - 1;
                m &= m - 1;
                if (o < expected) out[o] = start + lane * 64u + p;     // never beyond the caller's list
                ++o;
            }
            m = fm1;
            while (m) {
                const uint32_t p = __ffs(m) - 1;
                m &= m - 1;
                if (o < expected) out[o] = start + lane * 64u + 32u + p;
                ++o;
            }
        }
        if (pub_bits) {
            uint32_t* pb = pub_bits + (start >> 5) + 2 * lane;
            if (lane * 64u < len) pb[0] = fm0;
            if (lane * 64u + 32u < len) pb[1] = fm1;
        }
    }
}

// Segmented models: the public bitmap is built from the index list (tiles may start inside a word).
__global__ __launch_bounds__(256) void k_bits_from_idx(const uint32_t* __restrict__ idx, uint64_t count, uint64_t n,
                                                       uint32_t* __restrict__ bits)
{
    for (uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x; j < count; j += (uint64_t)gridDim.x * 256) {
        const uint32_t i = idx[j];
        if (i < n) atomicOr(&bits[i >> 5], 1u << (i & 31u));
    }
}

// ---------------------------------------------------------------------------------------
// Tile offsets of an ascending index list by binary search.  One thread per tile boundary.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_tile_offsets(const uint32_t* __restrict__ idx, uint64_t count,
                                                      const uint32_t* __restrict__ tile_start, uint32_t T, uint64_t n,
                                                      uint32_t* __restrict__ off)
{
    const uint32_t t = blockIdx.x * 256 + threadIdx.x;
    if (t > T) return;
    const uint64_t target = (t == T) ? n : tile_start[t];
    uint64_t lo = 0, hi = count;                 // first position with idx >= target
    while (lo < hi) {
        const uint64_t mid = (lo + hi) >> 1;
        if ((uint64_t)idx[mid] < target) lo = mid + 1; else hi = mid;
    }
    off[t] = (uint32_t)lo;
}

// ---------------------------------------------------------------------------------------
// K5: pack (src_is_w == 0: the workers' updates) and the read half of pull (one shared
// source).  One block per tile; the tile's slice of every list is a short contiguous run,
// and the gathered lines of the source are shared by the core and explorer reads.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_gather(PtrTab src, int shared_src, uint32_t nw, uint64_t n,
                                                  const uint32_t* __restrict__ core_idx, const uint32_t* __restrict__ core_off,
                                                  PtrTab expl_idx, PtrTab expl_off, MutPtrTab core_val, MutPtrTab expl_val,
                                                  MutPtrTab scatter_dst)
{
    __shared__ uint32_t elo[MAXW], ecn[MAXW];
    const uint32_t t = blockIdx.x;
    // the tile's slices of all explorer lists are requested first, in one go (one list after the other would wait
    // for memory three times per worker)
    if (threadIdx.x < nw) {
        const uint32_t* eo = static_cast<const uint32_t*>(expl_off.p[threadIdx.x]);
        const uint32_t lo = eo[t];
        elo[threadIdx.x] = lo;
        ecn[threadIdx.x] = eo[t + 1] - lo;
    }
    const uint32_t c0 = core_off[t], c1 = core_off[t + 1];
    for (uint32_t j = c0 + threadIdx.x; j < c1; j += BLOCK) {
        const uint32_t i = core_idx[j];
        if (i >= n) continue;
        if (shared_src) {
            const float v = static_cast<const float*>(src.p[0])[i];
            for (uint32_t q = 0; q < nw; ++q) {
                static_cast<float*>(core_val.p[q])[j] = v;
                if (scatter_dst.p[q]) static_cast<float*>(scatter_dst.p[q])[i] = v;
            }
        } else {
            for (uint32_t q0 = 0; q0 < nw; q0 += 8) {          // eight workers' loads together
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = (q0 + u < nw) ? static_cast<const float*>(src.p[q0 + u])[i] : 0.0f;
#pragma unroll
                for (int u = 0; u < 8; ++u) if (q0 + u < nw) static_cast<float*>(core_val.p[q0 + u])[j] = v[u];
            }
        }
    }
    __syncthreads();
    uint32_t E = 0;
    for (uint32_t q = 0; q < nw; ++q) E += ecn[q];
    for (uint32_t x0 = 0; x0 < E; x0 += 2 * BLOCK) {            // two entries per thread in flight
        uint32_t qq[2], jj[2], ii[2];
        float vv[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t x = x0 + u * BLOCK + threadIdx.x;
            qq[u] = 0; jj[u] = 0; ii[u] = 0xFFFFFFFFu;
            if (x < E) {
                uint32_t q = 0, run = 0;
                while (q + 1 < nw && run + ecn[q] <= x) { run += ecn[q]; ++q; }
                qq[u] = q; jj[u] = elo[q] + (x - run);
                ii[u] = static_cast<const uint32_t*>(expl_idx.p[q])[jj[u]];
            }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u)
            vv[u] = (ii[u] < n) ? static_cast<const float*>(src.p[shared_src ? 0 : qq[u]])[ii[u]] : 0.0f;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (ii[u] >= n) continue;
            static_cast<float*>(expl_val.p[qq[u]])[jj[u]] = vv[u];
            float* sd = static_cast<float*>(scatter_dst.p[qq[u]]);
            if (sd) sd[ii[u]] = vv[u];
        }
    }
}

// ---------------------------------------------------------------------------------------
// Pack after a scoring pass that captured the update values of every parameter at or above
// spec_lo (k_score<.., SPEC = 1>): the core values of a captured tile come from the compact
// capture (rank of the parameter among the captured ones of its sub-tile), not from the
// update vectors.  Tiles that were not captured (ragged, unaligned, or a segment whose
// threshold fell below the capture bound) gather from the update vectors.
// One wave per tile, all workers (the rank is the same for all).  grid ceil(T/4).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void k_pack_core_spec(PtrTab g, uint32_t nw, uint64_t n,
                                                          const uint32_t* __restrict__ tile_start,
                                                          const uint32_t* __restrict__ tile_seg, uint32_t T,
                                                          const uint32_t* __restrict__ core_idx,
                                                          const uint32_t* __restrict__ core_off,
                                                          const uint2* __restrict__ spec_bits,
                                                          const float* __restrict__ spec_vals,
                                                          const uint32_t* __restrict__ spec_fail, int vec_ok, MutPtrTab core_val)
{
    __shared__ uint32_t wd[4][TILE_WORDS], pre[4][TILE_WORDS];
    const uint32_t wid = threadIdx.x >> 6, t = blockIdx.x * 4 + wid, lane = lane_id();
    if (t >= T) return;
    const uint32_t start = tile_start[t], len = tile_start[t + 1] - start;
    const uint32_t j0 = core_off[t], j1 = core_off[t + 1];
    if (j0 >= j1) return;
    const bool captured = vec_ok && len == TILE && (start & 3u) == 0 && spec_fail[tile_seg[t]] == 0;
    if (captured) {
        // entry number of every captured parameter inside its sub-tile: lanes 4r..4r+3 hold the eight bitmap
        // words of round r (16 rounds a tile, 4 a sub-tile); a round's entries start on a multiple of A
        const uint32_t A = spec_align(nw);
        const uint4 w4 = *reinterpret_cast<const uint4*>(spec_bits + (size_t)t * TILE_WORDS + 2 * lane);
        const uint2 w2 = make_uint2(w4.x, w4.z);
        const uint32_t pc = __popc(w2.x) + __popc(w2.y);
        const uint32_t incl = wave_incl_scan(pc);
        const uint32_t round0 = __shfl(incl - pc, (int)(lane & ~3u), 64);                     // captured before this round
        const uint32_t round_total = __shfl(incl, (int)(lane | 3u), 64) - round0;
        const uint32_t round_padded = (round_total + A - 1u) & ~(A - 1u);
        const uint32_t pin = wave_incl_scan((lane & 3u) == 0 ? round_padded : 0u);            // padded rounds up to this one
        const uint32_t sub0 = __shfl(pin - ((lane & 3u) == 0 ? round_padded : 0u), (int)(lane & ~15u), 64);
        const uint32_t first = (__shfl(pin, (int)(lane & ~3u), 64) - round_padded) - sub0 + (incl - pc - round0);
        wd[wid][2 * lane] = w2.x; wd[wid][2 * lane + 1] = w2.y;
        pre[wid][2 * lane] = first; pre[wid][2 * lane + 1] = first + __popc(w2.x);
        wave_sync();
        // four list entries per lane and pass: all their index loads are requested first, then all their values
        constexpr int U = 4;
        for (uint32_t jb = j0; jb < j1; jb += 64 * U) {
            uint32_t e[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t j = jb + u * 64 + lane;
                e[u] = (j < j1) ? core_idx[j] - start : 0xFFFFFFFFu;       // beyond the tile: the caller's lists are inconsistent
            }
            if ((nw & 3u) == 0) {
                for (uint32_t q = 0; q < nw; q += 4) {
                    float4 v[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (e[u] < TILE) {
                            const uint32_t entry = pre[wid][e[u] >> 5] + __popc(wd[wid][e[u] >> 5] & mask_below(e[u] & 31u));
                            if (entry < SPEC_CAP)
                                v[u] = *reinterpret_cast<const float4*>(spec_vals + (((size_t)t * SUBS + (e[u] >> 10)) * SPEC_CAP + entry) * nw + q);
                            else {
                                const size_t i = (size_t)start + e[u];
                                v[u].x = static_cast<const float*>(g.p[q])[i]; v[u].y = static_cast<const float*>(g.p[q + 1])[i];
                                v[u].z = static_cast<const float*>(g.p[q + 2])[i]; v[u].w = static_cast<const float*>(g.p[q + 3])[i];
                            }
                        }
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const uint32_t j = jb + u * 64 + lane;
                        if (e[u] < TILE) {
                            static_cast<float*>(core_val.p[q])[j] = v[u].x; static_cast<float*>(core_val.p[q + 1])[j] = v[u].y;
                            static_cast<float*>(core_val.p[q + 2])[j] = v[u].z; static_cast<float*>(core_val.p[q + 3])[j] = v[u].w;
                        }
                    }
                }
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t j = jb + u * 64 + lane;
                    if (e[u] >= TILE) continue;
                    const uint32_t entry = pre[wid][e[u] >> 5] + __popc(wd[wid][e[u] >> 5] & mask_below(e[u] & 31u));
                    const float* src = spec_vals + (((size_t)t * SUBS + (e[u] >> 10)) * SPEC_CAP + entry) * nw;
                    for (uint32_t q = 0; q < nw; ++q)
                        static_cast<float*>(core_val.p[q])[j] = (entry < SPEC_CAP) ? src[q] : static_cast<const float*>(g.p[q])[(size_t)start + e[u]];
                }
            }
        }
    } else {
        for (uint32_t j = j0 + lane; j < j1; j += 64) {
            const uint32_t i = core_idx[j];
            if (i >= n) continue;
            for (uint32_t q = 0; q < nw; ++q) static_cast<float*>(core_val.p[q])[j] = static_cast<const float*>(g.p[q])[i];
        }
    }
}

// The same for a flat model, one thread per list entry: the tile and the bitmap word follow
// from the index itself, the word's first entry number is stored beside the word.  Every wave
// writes 64 consecutive list positions per worker (whole, aligned lines: a store that covers
// a line only in part makes the memory side read it first).  grid: any, grid-stride.
__global__ __launch_bounds__(256) void k_pack_core_flat(PtrTab g, uint32_t nw, uint64_t n, uint32_t T_full,
                                                        const uint32_t* __restrict__ core_idx, uint32_t k,
                                                        const uint2* __restrict__ spec_bits,
                                                        const float* __restrict__ spec_vals,
                                                        const uint32_t* __restrict__ spec_fail, int vec_ok, MutPtrTab core_val)
{
    constexpr int U = 4;
    const bool ok = vec_ok && spec_fail[0] == 0;
    const uint32_t stride = gridDim.x * 256u;
    for (uint32_t jb = blockIdx.x * 256u + threadIdx.x; jb < k; jb += U * stride) {
        uint32_t i[U];
#pragma unroll
        for (int u = 0; u < U; ++u) i[u] = (jb + u * stride < k) ? core_idx[jb + u * stride] : 0xFFFFFFFFu;
        uint2 bp[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            bp[u] = make_uint2(0u, 0u);
            if (i[u] < n && ok && (i[u] >> 12) < T_full) bp[u] = spec_bits[i[u] >> 5];      // tile * 128 + word in tile
        }
        if ((nw & 3u) == 0) {
            // eight workers (two 16-byte pieces of an entry) per turn, all loads of a turn requested before any store
            for (uint32_t q = 0; q < nw; q += 8) {
                float4 v[U][2];
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        v[u][h] = make_float4(0.f, 0.f, 0.f, 0.f);
                        const uint32_t qq = q + 4u * h;
                        if (i[u] >= n || qq >= nw) continue;
                        const uint32_t entry = bp[u].y + __popc(bp[u].x & mask_below(i[u] & 31u));
                        if (ok && (i[u] >> 12) < T_full && entry < SPEC_CAP) {
                            v[u][h] = ld4<NT_PACKC_LD>(spec_vals + ((size_t)(i[u] >> 10) * SPEC_CAP + entry) * nw + qq);
                        } else {
                            v[u][h].x = static_cast<const float*>(g.p[qq])[i[u]]; v[u][h].y = static_cast<const float*>(g.p[qq + 1])[i[u]];
                            v[u][h].z = static_cast<const float*>(g.p[qq + 2])[i[u]]; v[u][h].w = static_cast<const float*>(g.p[qq + 3])[i[u]];
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t j = jb + u * stride;
                    if (i[u] >= n) continue;
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const uint32_t qq = q + 4u * h;
                        if (qq >= nw) continue;
                        st1<NT_PACKC_ST>(static_cast<float*>(core_val.p[qq]) + j, v[u][h].x);
                        st1<NT_PACKC_ST>(static_cast<float*>(core_val.p[qq + 1]) + j, v[u][h].y);
                        st1<NT_PACKC_ST>(static_cast<float*>(core_val.p[qq + 2]) + j, v[u][h].z);
                        st1<NT_PACKC_ST>(static_cast<float*>(core_val.p[qq + 3]) + j, v[u][h].w);
                    }
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t j = jb + u * stride;
                if (i[u] >= n) continue;
                const uint32_t entry = bp[u].y + __popc(bp[u].x & mask_below(i[u] & 31u));
                if (ok && (i[u] >> 12) < T_full && entry < SPEC_CAP) {
                    const float* src = spec_vals + ((size_t)(i[u] >> 10) * SPEC_CAP + entry) * nw;
                    for (uint32_t q = 0; q < nw; ++q) static_cast<float*>(core_val.p[q])[j] = src[q];
                } else {
                    for (uint32_t q = 0; q < nw; ++q) static_cast<float*>(core_val.p[q])[j] = static_cast<const float*>(g.p[q])[i[u]];
                }
            }
        }
    }
}

// Explorer values by gathering from the update vectors.  grid (blocks, n_workers).
struct CountTab { uint32_t c[MAXW]; };
__global__ __launch_bounds__(256) void k_pack_expl_gather(PtrTab g, uint64_t n, PtrTab expl_idx, CountTab m_w,
                                                          MutPtrTab expl_val)
{
    const uint32_t q = blockIdx.y, cnt = m_w.c[q];
    const float* src = static_cast<const float*>(g.p[q]);
    const uint32_t* idx = static_cast<const uint32_t*>(expl_idx.p[q]);
    float* out = static_cast<float*>(expl_val.p[q]);
    const uint32_t stride = gridDim.x * 256u;
    for (uint32_t j = blockIdx.x * 256u + threadIdx.x; j < cnt; j += 4u * stride) {
        uint32_t i[4];
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) i[u] = (j + u * stride < cnt) ? idx[j + u * stride] : 0u;
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = (j + u * stride < cnt && i[u] < n) ? ld1<NT_EXPLG>(src + i[u]) : 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u) if (j + u * stride < cnt) out[j + u * stride] = v[u];
    }
}

template <int NBUF>
__global__ __launch_bounds__(BLOCK) void k_pack_stream(PtrTab g, uint32_t nw, const uint32_t* __restrict__ tile_start,
                                                       const uint32_t* __restrict__ core_idx,
                                                       const uint32_t* __restrict__ core_off, PtrTab expl_idx,
                                                       PtrTab expl_off, MutPtrTab core_val, MutPtrTab expl_val, int vec_ok)
{
    __shared__ float buf[NBUF][TILE];
    __shared__ uint16_t cpos[TILE];          // the tile's core positions: the same for every worker
    __shared__ uint32_t elo[MAXW], ehi[MAXW];
    const uint32_t t = blockIdx.x;
    const uint32_t start = tile_start[t], len = tile_start[t + 1] - start;
    const bool vec = vec_ok && len == TILE && (start & 3u) == 0;
    const uint32_t c0 = core_off[t], c1 = core_off[t + 1];
    const uint32_t ccnt = (c1 - c0 < TILE) ? c1 - c0 : TILE;
    if (threadIdx.x < nw) {
        const uint32_t* eo = static_cast<const uint32_t*>(expl_off.p[threadIdx.x]);
        elo[threadIdx.x] = eo[t];
        ehi[threadIdx.x] = eo[t + 1];
    }
    for (uint32_t x = threadIdx.x; x < ccnt; x += BLOCK) {
        const uint32_t pos = core_idx[c0 + x] - start;
        cpos[x] = (pos < len) ? (uint16_t)pos : (uint16_t)0xFFFF;
    }
    __syncthreads();
    // Loads are requested one worker ahead and nothing inside the loop waits for a load that
    // was requested in the same iteration: the tile of updates and this thread's explorer
    // index of the next worker travel while the current worker's values are picked from LDS.
    float r[EPT];
    uint32_t epos = 0xFFFFFFFFu;             // explorer entry elo[q] + threadIdx.x of the coming worker, if any
    auto fetch = [&](uint32_t q) {
        const float* src = static_cast<const float*>(g.p[q]) + start;
        if (vec) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float4 v = ld4<NT_PACKS>(src + k * 1024 + threadIdx.x * 4);
                r[4 * k + 0] = v.x; r[4 * k + 1] = v.y; r[4 * k + 2] = v.z; r[4 * k + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < EPT; ++j) {
                const uint32_t e = elem_scl(j);
                r[j] = (e < len) ? src[e] : 0.0f;
            }
        }
        // the index itself: anything computed from it here would make the wave wait for this load, and with it for the
        // tile requested just before, on the spot
        const uint32_t j = elo[q] + threadIdx.x;
        epos = 0xFFFFFFFFu;
        if (j < ehi[q]) epos = static_cast<const uint32_t*>(expl_idx.p[q])[j];
    };
    fetch(0);
    for (uint32_t q = 0; q < nw; ++q) {
        float* b = buf[NBUF == 2 ? (q & 1u) : 0];
        if (NBUF == 1 && q) __syncthreads();     // the previous worker's readers are done with the buffer
        if (vec) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                *reinterpret_cast<float4*>(b + k * 1024 + threadIdx.x * 4) = make_float4(r[4 * k], r[4 * k + 1], r[4 * k + 2], r[4 * k + 3]);
        } else {
#pragma unroll
            for (int j = 0; j < EPT; ++j) b[elem_scl(j)] = r[j];
        }
        const uint32_t my_epos = epos - start;      // no entry: wraps to a position beyond any tile (start + len < 2^32)
        __syncthreads();     // with two buffers this also orders a buffer's readers (two workers ago) before its writers
        if (q + 1 < nw) fetch(q + 1);
        float* cv = static_cast<float*>(core_val.p[q]);
        for (uint32_t x = threadIdx.x; x < ccnt; x += BLOCK) {
            const uint32_t pos = cpos[x];
            if (pos != 0xFFFFu) cv[c0 + x] = b[pos];
        }
        float* ev = static_cast<float*>(expl_val.p[q]);
        const uint32_t e0 = elo[q], e1 = ehi[q];
        if (my_epos < len) ev[e0 + threadIdx.x] = b[my_epos];
        if (e1 - e0 > BLOCK) {               // dense explorers: the rest of the slice, loaded here
            const uint32_t* ei = static_cast<const uint32_t*>(expl_idx.p[q]);
            for (uint32_t j = e0 + BLOCK + threadIdx.x; j < e1; j += BLOCK) {
                const uint32_t pos = ei[j] - start;
                if (pos < len) ev[j] = b[pos];
            }
        }
    }
}

// The same pack with the two halves of the work in different waves (512 threads: waves 0..3 load, waves 4..7 store).
// A wave's vector-memory operations retire in issue order, so a wave that stores a worker's slices and then needs the
// next worker's tile waits for its own stores to be acknowledged by the cache, every step; here the loading waves never
// store and the storing waves never load from memory: the tile of updates, the core positions and the explorer
// positions all reach them through LDS.  Consecutive tiles go to the same die (blocks are dealt to the eight dies in
// turn), so that the partial lines at the two ends of a tile's output slices meet their other halves in one L2.
// grid: 8 * ceil(T / 8) blocks.
__global__ __launch_bounds__(2 * BLOCK) void k_pack_stream_ws(PtrTab g, uint32_t nw, uint32_t T,
                                                               const uint32_t* __restrict__ tile_start,
                                                               const uint32_t* __restrict__ core_idx,
                                                               const uint32_t* __restrict__ core_off, PtrTab expl_idx,
                                                               PtrTab expl_off, MutPtrTab core_val, MutPtrTab expl_val, int vec_ok)
{
    __shared__ float buf[2][TILE];
    __shared__ uint16_t cpos[TILE];          // the tile's core positions: the same for every worker
    __shared__ uint32_t epos[2][BLOCK];      // the first BLOCK explorer positions of the worker whose tile is in buf[.]
    __shared__ uint32_t elo[MAXW], ehi[MAXW];
    const uint32_t chunk = gridDim.x >> 3;
    const uint32_t t = (blockIdx.x & 7u) * chunk + (blockIdx.x >> 3);
    if (t >= T) return;                      // uniform over the block
    const uint32_t start = tile_start[t], len = tile_start[t + 1] - start;
    const bool vec = vec_ok && len == TILE && (start & 3u) == 0;
    const uint32_t c0 = core_off[t], c1 = core_off[t + 1];
    const uint32_t ccnt = (c1 - c0 < TILE) ? c1 - c0 : TILE;
    const bool loader = threadIdx.x < BLOCK;
    const uint32_t tid = threadIdx.x & (BLOCK - 1u);
    if (threadIdx.x < nw) {
        const uint32_t* eo = static_cast<const uint32_t*>(expl_off.p[threadIdx.x]);
        elo[threadIdx.x] = eo[t];
        ehi[threadIdx.x] = eo[t + 1];
    }
    for (uint32_t x = threadIdx.x; x < ccnt; x += 2 * BLOCK) {
        const uint32_t pos = core_idx[c0 + x] - start;
        cpos[x] = (pos < len) ? (uint16_t)pos : (uint16_t)0xFFFF;
    }
    __syncthreads();
    float r[EPT];
    uint32_t ep = 0xFFFFFFFFu;
    auto fetch = [&](uint32_t q) {
        const float* src = static_cast<const float*>(g.p[q]) + start;
        if (vec) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float4 v = ld4<NT_PACKS>(src + k * 1024 + tid * 4);
                r[4 * k + 0] = v.x; r[4 * k + 1] = v.y; r[4 * k + 2] = v.z; r[4 * k + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < EPT; ++j) {
                const uint32_t e = (uint32_t)j * BLOCK + tid;
                r[j] = (e < len) ? src[e] : 0.0f;
            }
        }
        // the index itself: anything computed from it here would make the wave wait for this load, and with it for the
        // tile requested just before, on the spot
        const uint32_t j = elo[q] + tid;
        ep = 0xFFFFFFFFu;
        if (j < ehi[q]) ep = static_cast<const uint32_t*>(expl_idx.p[q])[j];
    };
    if (loader) fetch(0);
    for (uint32_t q = 0; q < nw; ++q) {
        float* b = buf[q & 1u];
        if (loader) {
            if (vec) {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    *reinterpret_cast<float4*>(b + k * 1024 + tid * 4) = make_float4(r[4 * k], r[4 * k + 1], r[4 * k + 2], r[4 * k + 3]);
            } else {
#pragma unroll
                for (int j = 0; j < EPT; ++j) b[(uint32_t)j * BLOCK + tid] = r[j];
            }
            epos[q & 1u][tid] = ep - start;       // no entry: wraps to a position beyond any tile (start + len < 2^32)
            if (q + 1 < nw) fetch(q + 1);
        }
        // the tile of worker q is in LDS; the storing waves are done with the buffer it replaced (worker q - 2): they
        // passed the previous barrier only after issuing its last LDS reads, and LDS operations of a wave finish in order
        __syncthreads();
        if (!loader) {
            float* cv = static_cast<float*>(core_val.p[q]);
            for (uint32_t x = tid; x < ccnt; x += BLOCK) {
                const uint32_t pos = cpos[x];
                if (pos != 0xFFFFu) cv[c0 + x] = b[pos];
            }
            float* ev = static_cast<float*>(expl_val.p[q]);
            const uint32_t e0 = elo[q], e1 = ehi[q];
            const uint32_t my = epos[q & 1u][tid];
            if (my < len) ev[e0 + tid] = b[my];
            if (e1 - e0 > BLOCK) {               // dense explorers: the rest of the slice, positions loaded here
                const uint32_t* ei = static_cast<const uint32_t*>(expl_idx.p[q]);
                for (uint32_t j = e0 + BLOCK + tid; j < e1; j += BLOCK) {
                    const uint32_t pos = ei[j] - start;
                    if (pos < len) ev[j] = b[pos];
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// K6: merge.  One block per tile of the global model; no atomics on global memory and a
// result that does not depend on scheduling.
//
// Core: every worker sends a value for each core index, so the thread that owns entry j of
// the tile's slice of the core list sums the W values in worker order in registers.
//
// Explorers: each entry of the tile takes a ticket at its position (LDS byte counter).  A
// position with one or two entries is summed in ticket order -- with at most two addends
// the binary32 sum does not depend on their order.  Positions with three or more entries
// (rare), or with two on top of a core sum (only if a list overlaps the core), go to a short
// list that one thread replays in worker order.  Tiles with more
// explorer entries than the fast path holds in registers, or with too many such positions,
// take the generic path: entries staged through LDS and applied one worker at a time.
//
// All loads of a tile (its w, its core slice, its explorer entries) are requested in one
// go right after the tile's offsets are known.
// ---------------------------------------------------------------------------------------
// Sum of the W workers' values of core entry j, from +0 in worker order.  The loads of eight workers are requested
// together (a loop with one load and one add per turn waits for memory W times in a row).
__device__ __forceinline__ float core_sum(const PtrTab& core_val, uint32_t nw, uint32_t j)
{
    float a = 0.0f;
    for (uint32_t q0 = 0; q0 < nw; q0 += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = (q0 + u < nw) ? ld1<NT_MERGE_VAL>(static_cast<const float*>(core_val.p[q0 + u]) + j) : 0.0f;
#pragma unroll
        for (int u = 0; u < 8; ++u) if (q0 + u < nw) a = a + v[u];
    }
    return a;
}

constexpr int MERGE_R = 4;                 // explorer entries per thread kept in registers
constexpr uint32_t MERGE_HOT_CAP = 128;
constexpr uint32_t MERGE_STAGE = 256;

__global__ __launch_bounds__(BLOCK) void k_merge(float* __restrict__ w, float lr, uint32_t nw,
                                                 const uint32_t* __restrict__ tile_start,
                                                 const uint32_t* __restrict__ core_idx, const uint32_t* __restrict__ core_off,
                                                 PtrTab core_val, PtrTab expl_idx, PtrTab expl_off, PtrTab expl_val,
                                                 int vec_ok, uint64_t n, uint32_t n_seg)
{
    __shared__ float acc[TILE];
    __shared__ uint32_t cnt[TILE / 4];     // one byte per position: bit 7 = core, low bits = explorer entries
    __shared__ uint32_t elo[MAXW], ecn[MAXW];
    __shared__ uint16_t hpos[MERGE_HOT_CAP];
    __shared__ uint8_t hq[MERGE_HOT_CAP];
    __shared__ float hval[MERGE_HOT_CAP];
    __shared__ uint32_t hcount;
    __shared__ uint16_t spos[MERGE_STAGE];
    __shared__ float sval[MERGE_STAGE];
    const uint32_t t = blockIdx.x;
    // flat model: no table look-up before the tile's loads can be requested
    uint32_t start, len;
    if (n_seg == 1) {
        start = t * TILE;
        const uint64_t rest = n - (uint64_t)start;
        len = rest < TILE ? (uint32_t)rest : TILE;
    } else {
        start = tile_start[t]; len = tile_start[t + 1] - start;
    }
    const bool vec = vec_ok && len == TILE && (start & 3u) == 0;
    const uint32_t c0 = core_off[t], c1 = core_off[t + 1];
    float wv[EPT];
    if (vec) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float4 v = ld4<NT_MERGE_LD>(w + (size_t)start + r * 1024 + threadIdx.x * 4);
            wv[4 * r + 0] = v.x; wv[4 * r + 1] = v.y; wv[4 * r + 2] = v.z; wv[4 * r + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const uint32_t e = elem_scl(j);
            wv[j] = (e < len) ? w[(size_t)start + e] : 0.0f;
        }
    }
    for (uint32_t x = threadIdx.x; x < TILE / 4; x += BLOCK) cnt[x] = 0;
    if (threadIdx.x == 0) hcount = 0;
    if (threadIdx.x < nw) {
        const uint32_t* eo = static_cast<const uint32_t*>(expl_off.p[threadIdx.x]);
        const uint32_t lo = eo[t];
        elo[threadIdx.x] = lo;
        ecn[threadIdx.x] = eo[t + 1] - lo;
    }
    __syncthreads();
    uint32_t E = 0;
    for (uint32_t q = 0; q < nw; ++q) E += ecn[q];
    const bool fast = E <= (uint32_t)(BLOCK * MERGE_R);
    // explorer entries of the fast path: requested now, held in registers
    uint32_t epos[MERGE_R], eq[MERGE_R], etk[MERGE_R];
    float eval[MERGE_R];
    if (fast) {
#pragma unroll
        for (int i = 0; i < MERGE_R; ++i) {
            const uint32_t x = threadIdx.x + (uint32_t)i * BLOCK;
            epos[i] = 0xFFFFFFFFu; eq[i] = 0; etk[i] = 0; eval[i] = 0.0f;
            if (x < E) {
                uint32_t q = 0, run = 0;
                while (q + 1 < nw && run + ecn[q] <= x) { run += ecn[q]; ++q; }
                const uint32_t j = elo[q] + (x - run);
                const uint32_t pos = static_cast<const uint32_t*>(expl_idx.p[q])[j] - start;
                eval[i] = static_cast<const float*>(expl_val.p[q])[j];
                eq[i] = q;
                if (pos < len) epos[i] = pos;
            }
        }
    }
    // core: every worker contributes, in worker order
    for (uint32_t j = c0 + threadIdx.x; j < c1; j += BLOCK) {
        const uint32_t pos = core_idx[j] - start;
        const float a = core_sum(core_val, nw, j);
        if (pos < len) { acc[pos] = a; atomicOr(&cnt[pos >> 2], 0x80u << (8u * (pos & 3u))); }
    }
    if (fast) {
#pragma unroll
        for (int i = 0; i < MERGE_R; ++i) {
            if (epos[i] != 0xFFFFFFFFu) {
                const uint32_t sh = 8u * (epos[i] & 3u);
                etk[i] = (atomicAdd(&cnt[epos[i] >> 2], 1u << sh) >> sh) & 0x7Fu;
            }
        }
    }
    __syncthreads();
    uint32_t nhot = 0;
    if (fast) {
        // first and second entry of a position, in ticket order; the rest is replayed in worker order
        uint32_t tot[MERGE_R];
#pragma unroll
        for (int i = 0; i < MERGE_R; ++i) {
            tot[i] = 0;
            if (epos[i] != 0xFFFFFFFFu) {
                const uint32_t byte = (cnt[epos[i] >> 2] >> (8u * (epos[i] & 3u))) & 0xFFu;
                tot[i] = byte & 0x7Fu;
                // two explorer entries on top of a core sum (lists that overlap the core: invalid input) would make
                // the result depend on the ticket order: such a position is replayed in worker order as well
                if (tot[i] == 2u && (byte & 0x80u)) tot[i] = 3u;
                if (tot[i] <= 2u) {
                    if (etk[i] == 0) acc[epos[i]] = ((byte & 0x80u) ? acc[epos[i]] : 0.0f) + eval[i];
                } else {
                    const uint32_t slot = atomicAdd(&hcount, 1u);
                    if (slot < MERGE_HOT_CAP) { hpos[slot] = (uint16_t)epos[i]; hq[slot] = (uint8_t)eq[i]; hval[slot] = eval[i]; }
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < MERGE_R; ++i)
            if (epos[i] != 0xFFFFFFFFu && tot[i] == 2u && etk[i] == 1u) acc[epos[i]] = acc[epos[i]] + eval[i];
        nhot = hcount;
        if (nhot && nhot <= MERGE_HOT_CAP && threadIdx.x == 0) {
            for (uint32_t i = 0; i < nhot; ++i) {
                const uint32_t pos = hpos[i];
                if (!((cnt[pos >> 2] >> (8u * (pos & 3u))) & 0x80u)) acc[pos] = 0.0f;
            }
            for (uint32_t q = 0; q < nw; ++q)
                for (uint32_t i = 0; i < nhot; ++i)
                    if (hq[i] == q) acc[hpos[i]] = acc[hpos[i]] + hval[i];
        }
    }
    __syncthreads();
    if (!fast || nhot > MERGE_HOT_CAP) {
        // generic path: every explorer entry staged through LDS, applied one worker at a time.
        // The counters keep their core bits; a set low bit now means "an explorer sum is in acc".
        for (uint32_t x = threadIdx.x; x < TILE / 4; x += BLOCK) cnt[x] &= 0x80808080u;
        if (nhot > MERGE_HOT_CAP) {       // the fast path wrote partial sums over core sums: redo the core
            __syncthreads();
            for (uint32_t j = c0 + threadIdx.x; j < c1; j += BLOCK) {
                const uint32_t pos = core_idx[j] - start;
                const float a = core_sum(core_val, nw, j);
                if (pos < len) acc[pos] = a;
            }
        }
        __syncthreads();
        uint8_t* hit = reinterpret_cast<uint8_t*>(cnt);
        for (uint32_t cb = 0; cb < E; cb += MERGE_STAGE) {
            const uint32_t cn = (E - cb < MERGE_STAGE) ? E - cb : MERGE_STAGE;
            for (uint32_t x = threadIdx.x; x < cn; x += BLOCK) {
                const uint32_t v = cb + x;
                uint32_t q = 0, run = 0;
                while (q + 1 < nw && run + ecn[q] <= v) { run += ecn[q]; ++q; }
                const uint32_t j = elo[q] + (v - run);
                const uint32_t pos = static_cast<const uint32_t*>(expl_idx.p[q])[j] - start;
                spos[x] = (pos < len) ? (uint16_t)pos : (uint16_t)0xFFFF;
                sval[x] = static_cast<const float*>(expl_val.p[q])[j];
            }
            __syncthreads();
            uint32_t run = 0;
            for (uint32_t q = 0; q < nw; ++q) {
                const uint32_t qlo = run, qhi = run + ecn[q];
                run = qhi;
                if (qhi <= cb || qlo >= cb + cn) continue;
                const uint32_t lo = (qlo > cb) ? qlo - cb : 0u;
                const uint32_t hi = (qhi - cb < cn) ? qhi - cb : cn;
                for (uint32_t x = lo + threadIdx.x; x < hi; x += BLOCK) {
                    const uint32_t pos = spos[x];
                    if (pos != 0xFFFFu) {
                        acc[pos] = (hit[pos] ? acc[pos] : 0.0f) + sval[x];
                        hit[pos] |= 1;
                    }
                }
                __syncthreads();
            }
            __syncthreads();
        }
    }
    // apply and stream the tile back
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const uint32_t e = vec ? elem_vec(j) : elem_scl(j);
        if (e < len && ((cnt[e >> 2] >> (8u * (e & 3u))) & 0xFFu)) {
            wv[j] = __builtin_fmaf(-lr, acc[e], wv[j]);
            if (!vec) w[(size_t)start + e] = wv[j];
        }
    }
    if (vec) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            st4<NT_MERGE_ST>(w + (size_t)start + r * 1024 + threadIdx.x * 4,
                             make_float4(wv[4 * r], wv[4 * r + 1], wv[4 * r + 2], wv[4 * r + 3]));
    }
}

// ---------------------------------------------------------------------------------------
// Worker side, LocalTrain (section 3.3 step 1): one mini-batch step on every worker's LOCAL
// model, w_q <- fma(-eta, grad_q, w_q), and the accumulation of the update that the next
// push sends, delta_q = grad_1 + grad_2 + ... in binary32 in mini-batch order (first: a new
// accumulation starts with this gradient; delta is then not read).  20 bytes per parameter
// and worker (16 when first).  grid (blocks, n_workers).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_local_step(MutPtrTab w_local, PtrTab grad, MutPtrTab delta, uint64_t n, float eta,
                                                    int first, int vec_ok)
{
    const uint32_t q = blockIdx.y;
    float* w = static_cast<float*>(w_local.p[q]);
    const float* g = static_cast<const float*>(grad.p[q]);
    float* d = static_cast<float*>(delta.p[q]);
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    const uint64_t n4 = vec_ok ? n / 4 : 0;
    for (uint64_t x = (uint64_t)blockIdx.x * 256 + threadIdx.x; x < n4; x += 2 * stride) {       // two vectors per turn in flight
        const uint64_t x2 = x + stride;
        const bool two = x2 < n4;
        const float4 ga = ld4<1>(g + 4 * x), wa = ld4<1>(w + 4 * x);
        const float4 gb = two ? ld4<1>(g + 4 * x2) : make_float4(0.f, 0.f, 0.f, 0.f);
        const float4 wb = two ? ld4<1>(w + 4 * x2) : make_float4(0.f, 0.f, 0.f, 0.f);
        float4 da = ga, db = gb;
        if (!first) {
            const float4 oa = ld4<1>(d + 4 * x);
            da = make_float4(oa.x + ga.x, oa.y + ga.y, oa.z + ga.z, oa.w + ga.w);
            if (two) {
                const float4 ob = ld4<1>(d + 4 * x2);
                db = make_float4(ob.x + gb.x, ob.y + gb.y, ob.z + gb.z, ob.w + gb.w);
            }
        }
        st4<1>(w + 4 * x, make_float4(__builtin_fmaf(-eta, ga.x, wa.x), __builtin_fmaf(-eta, ga.y, wa.y),
                                      __builtin_fmaf(-eta, ga.z, wa.z), __builtin_fmaf(-eta, ga.w, wa.w)));
        st4<1>(d + 4 * x, da);
        if (two) {
            st4<1>(w + 4 * x2, make_float4(__builtin_fmaf(-eta, gb.x, wb.x), __builtin_fmaf(-eta, gb.y, wb.y),
                                           __builtin_fmaf(-eta, gb.z, wb.z), __builtin_fmaf(-eta, gb.w, wb.w)));
            st4<1>(d + 4 * x2, db);
        }
    }
    for (uint64_t i = 4 * n4 + (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {      // tail, or unaligned arrays
        const float gi = g[i];
        w[i] = __builtin_fmaf(-eta, gi, w[i]);
        d[i] = first ? gi : d[i] + gi;
    }
}

// ---------------------------------------------------------------------------------------
// LocalTrain and Push in one pass (section 3.3 steps 1 and 3): the last mini-batch step before a
// communication already streams the accumulated update of every worker; picking the values at
// the communication set while a tile of the new update sits in LDS saves the extraction its own
// scan of the update vectors (the full scan that section 3.5 counts per extraction).  Same
// results as k_local_step followed by k_pack_stream on delta.  One block per tile, workers in
// turn, the next worker's three tiles in flight while the current one is picked from.
// ---------------------------------------------------------------------------------------
template <int NBUF>
__global__ __launch_bounds__(BLOCK) void k_local_step_pack(MutPtrTab w_local, PtrTab grad, MutPtrTab delta, float eta, int first,
                                                           uint32_t nw, const uint32_t* __restrict__ tile_start,
                                                           const uint32_t* __restrict__ core_idx,
                                                           const uint32_t* __restrict__ core_off, PtrTab expl_idx, PtrTab expl_off,
                                                           MutPtrTab core_val, MutPtrTab expl_val, int vec_ok)
{
    __shared__ float buf[NBUF][TILE];
    __shared__ uint16_t cpos[TILE];          // the tile's core positions: the same for every worker
    __shared__ uint32_t elo[MAXW], ehi[MAXW];
    const uint32_t t = blockIdx.x;
    const uint32_t start = tile_start[t], len = tile_start[t + 1] - start;
    const bool vec = vec_ok && len == TILE && (start & 3u) == 0;
    const uint32_t c0 = core_off[t], c1 = core_off[t + 1];
    const uint32_t ccnt = (c1 - c0 < TILE) ? c1 - c0 : TILE;
    if (threadIdx.x < nw) {
        const uint32_t* eo = static_cast<const uint32_t*>(expl_off.p[threadIdx.x]);
        elo[threadIdx.x] = eo[t];
        ehi[threadIdx.x] = eo[t + 1];
    }
    for (uint32_t x = threadIdx.x; x < ccnt; x += BLOCK) {
        const uint32_t pos = core_idx[c0 + x] - start;
        cpos[x] = (pos < len) ? (uint16_t)pos : (uint16_t)0xFFFF;
    }
    __syncthreads();
    float rg[EPT], rw[EPT], rd[EPT];
    uint32_t epos = 0xFFFFFFFFu;
    auto fetch = [&](uint32_t q) {
        const float* g = static_cast<const float*>(grad.p[q]) + start;
        const float* w = static_cast<const float*>(w_local.p[q]) + start;
        const float* d = static_cast<const float*>(delta.p[q]) + start;
        if (vec) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t o = k * 1024 + threadIdx.x * 4;
                const float4 a = ld4<1>(g + o), b = ld4<1>(w + o);
                rg[4 * k + 0] = a.x; rg[4 * k + 1] = a.y; rg[4 * k + 2] = a.z; rg[4 * k + 3] = a.w;
                rw[4 * k + 0] = b.x; rw[4 * k + 1] = b.y; rw[4 * k + 2] = b.z; rw[4 * k + 3] = b.w;
                if (!first) {
                    const float4 c = ld4<1>(d + o);
                    rd[4 * k + 0] = c.x; rd[4 * k + 1] = c.y; rd[4 * k + 2] = c.z; rd[4 * k + 3] = c.w;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < EPT; ++j) {
                const uint32_t e = elem_scl(j);
                rg[j] = (e < len) ? g[e] : 0.0f;
                rw[j] = (e < len) ? w[e] : 0.0f;
                rd[j] = (e < len && !first) ? d[e] : 0.0f;
            }
        }
        // the index itself: anything computed from it here would make the wave wait for this load, and with it for the
        // tile requested just before, on the spot
        const uint32_t j = elo[q] + threadIdx.x;
        epos = 0xFFFFFFFFu;
        if (j < ehi[q]) epos = static_cast<const uint32_t*>(expl_idx.p[q])[j];
    };
    fetch(0);
    for (uint32_t q = 0; q < nw; ++q) {
        float* b = buf[NBUF == 2 ? (q & 1u) : 0];
        float* w = static_cast<float*>(w_local.p[q]) + start;
        float* d = static_cast<float*>(delta.p[q]) + start;
        if (NBUF == 1 && q) __syncthreads();     // the previous worker's readers are done with the buffer
        // the step and the accumulation; the new update goes to memory and to LDS
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            rw[j] = __builtin_fmaf(-eta, rg[j], rw[j]);
            rd[j] = first ? rg[j] : rd[j] + rg[j];
        }
        if (vec) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t o = k * 1024 + threadIdx.x * 4;
                st4<1>(w + o, make_float4(rw[4 * k], rw[4 * k + 1], rw[4 * k + 2], rw[4 * k + 3]));
                st4<1>(d + o, make_float4(rd[4 * k], rd[4 * k + 1], rd[4 * k + 2], rd[4 * k + 3]));
                *reinterpret_cast<float4*>(b + o) = make_float4(rd[4 * k], rd[4 * k + 1], rd[4 * k + 2], rd[4 * k + 3]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < EPT; ++j) {
                const uint32_t e = elem_scl(j);
                if (e < len) { w[e] = rw[j]; d[e] = rd[j]; }
                b[e] = rd[j];
            }
        }
        const uint32_t my_epos = epos - start;      // no entry: wraps to a position beyond any tile (start + len < 2^32)
        __syncthreads();     // with two buffers this also orders a buffer's readers (two workers ago) before its writers
        if (q + 1 < nw) fetch(q + 1);
        float* cv = static_cast<float*>(core_val.p[q]);
        for (uint32_t x = threadIdx.x; x < ccnt; x += BLOCK) {
            const uint32_t pos = cpos[x];
            if (pos != 0xFFFFu) cv[c0 + x] = b[pos];
        }
        float* ev = static_cast<float*>(expl_val.p[q]);
        const uint32_t e0 = elo[q], e1 = ehi[q];
        if (my_epos < len) ev[e0 + threadIdx.x] = b[my_epos];
        if (e1 - e0 > BLOCK) {               // dense explorers: the rest of the slice, loaded here
            const uint32_t* ei = static_cast<const uint32_t*>(expl_idx.p[q]);
            for (uint32_t j = e0 + BLOCK + threadIdx.x; j < e1; j += BLOCK) {
                const uint32_t pos = ei[j] - start;
                if (pos < len) ev[j] = b[pos];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Pull, local Merge and LocalTrain in one pass (section 3.3 steps 4, 5 and 1 of the next round): the local model
// is overwritten with the global one at the worker's communication set, then stepped.  The first local step after a
// communication streams every local model anyway; applying the pulled values there saves the pull its own pass,
// whose scattered 4-byte writes touch nearly every line of every local model.  Same results as k_gather with a
// scatter destination followed by k_local_step.  STEP = 0: the overwrite alone (the write half of a pull with local
// models: workers without one are skipped).  One block per tile: the tile of the global model stays in
// registers for all workers, the communication set of a worker is a bitmap in LDS (core positions once per tile,
// explorer positions per worker, marked one worker ahead), the next worker's three tiles travel meanwhile.
// ---------------------------------------------------------------------------------------
template <int STEP>
__global__ __launch_bounds__(BLOCK) void k_pull_local_step(const float* __restrict__ w, MutPtrTab w_local, PtrTab grad, MutPtrTab delta,
                                                           float eta, int first, uint32_t nw,
                                                           const uint32_t* __restrict__ tile_start,
                                                           const uint32_t* __restrict__ core_idx,
                                                           const uint32_t* __restrict__ core_off, PtrTab expl_idx, PtrTab expl_off,
                                                           int vec_ok)
{
    __shared__ uint32_t cm[TILE_WORDS];          // core positions of the tile
    __shared__ uint32_t em[2][TILE_WORDS];       // explorer positions of a worker
    __shared__ uint32_t elo[MAXW], ehi[MAXW];
    const uint32_t t = blockIdx.x;
    const uint32_t start = tile_start[t], len = tile_start[t + 1] - start;
    const bool vec = vec_ok && len == TILE && (start & 3u) == 0;
    const uint32_t c0 = core_off[t], c1 = core_off[t + 1];
    if (threadIdx.x < nw) {
        const uint32_t* eo = static_cast<const uint32_t*>(expl_off.p[threadIdx.x]);
        elo[threadIdx.x] = eo[t];
        ehi[threadIdx.x] = eo[t + 1];
    }
    if (threadIdx.x < TILE_WORDS) { cm[threadIdx.x] = 0; em[0][threadIdx.x] = 0; }
    // this thread's elements of the global model: the same positions as its elements of every local model
    float wv[EPT];
    if (vec) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float4 v = ld4<1>(w + (size_t)start + k * 1024 + threadIdx.x * 4);
            wv[4 * k + 0] = v.x; wv[4 * k + 1] = v.y; wv[4 * k + 2] = v.z; wv[4 * k + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const uint32_t e = elem_scl(j);
            wv[j] = (e < len) ? w[(size_t)start + e] : 0.0f;
        }
    }
    __syncthreads();
    for (uint32_t j = c0 + threadIdx.x; j < c1; j += BLOCK) {
        const uint32_t pos = core_idx[j] - start;
        if (pos < len) atomicOr(&cm[pos >> 5], 1u << (pos & 31u));
    }
    // explorer positions of worker q into em[q & 1] (zeroed before): the first BLOCK entries from the index each
    // thread already holds (requested a turn ago with the tiles), the rest, if any, read here
    uint32_t epre = 0xFFFFFFFFu;
    auto mark = [&](uint32_t q, uint32_t held, uint32_t from) {
        const uint32_t p0 = held - start;        // no entry: wraps beyond any tile
        if (p0 < len) atomicOr(&em[q & 1u][p0 >> 5], 1u << (p0 & 31u));
        const uint32_t* ei = static_cast<const uint32_t*>(expl_idx.p[q]);
        for (uint32_t j = elo[q] + from + threadIdx.x; j < ehi[q]; j += BLOCK) {
            const uint32_t pos = ei[j] - start;
            if (pos < len) atomicOr(&em[q & 1u][pos >> 5], 1u << (pos & 31u));
        }
    };
    float rg[EPT], rl[EPT], rd[EPT];
    auto fetch = [&](uint32_t q) {
        const float* g = STEP ? static_cast<const float*>(grad.p[q]) + start : nullptr;
        const float* l = static_cast<const float*>(w_local.p[q]) + start;
        const float* d = STEP ? static_cast<const float*>(delta.p[q]) + start : nullptr;
        if (!STEP && !w_local.p[q]) {
            // a worker without a local model to patch (uniform over the block)
        } else if (vec) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t o = k * 1024 + threadIdx.x * 4;
                const float4 b = ld4<1>(l + o);
                rl[4 * k + 0] = b.x; rl[4 * k + 1] = b.y; rl[4 * k + 2] = b.z; rl[4 * k + 3] = b.w;
                if (STEP) {
                    const float4 a = ld4<1>(g + o);
                    rg[4 * k + 0] = a.x; rg[4 * k + 1] = a.y; rg[4 * k + 2] = a.z; rg[4 * k + 3] = a.w;
                }
                if (STEP && !first) {
                    const float4 c = ld4<1>(d + o);
                    rd[4 * k + 0] = c.x; rd[4 * k + 1] = c.y; rd[4 * k + 2] = c.z; rd[4 * k + 3] = c.w;
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < EPT; ++j) {
                const uint32_t e = elem_scl(j);
                rg[j] = (STEP && e < len) ? g[e] : 0.0f;
                rl[j] = (e < len) ? l[e] : 0.0f;
                rd[j] = (STEP && e < len && !first) ? d[e] : 0.0f;
            }
        }
        // this thread's explorer index of the worker after: held, not used, until that worker's marks are made
        epre = 0xFFFFFFFFu;
        if (q + 1 < nw) {
            const uint32_t j = elo[q + 1] + threadIdx.x;
            if (j < ehi[q + 1]) epre = static_cast<const uint32_t*>(expl_idx.p[q + 1])[j];
        }
    };
    mark(0, 0xFFFFFFFFu, 0u);
    fetch(0);
    for (uint32_t q = 0; q < nw; ++q) {
        // the marks of worker q (made a turn ago) are complete; the other bitmap is free (its reader finished a turn ago)
        __syncthreads();
        if (threadIdx.x < TILE_WORDS) em[(q + 1u) & 1u][threadIdx.x] = 0;
        float nl[EPT], nd[EPT];
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const uint32_t e = vec ? elem_vec(j) : elem_scl(j);
            const uint32_t bit = ((cm[e >> 5] | em[q & 1u][e >> 5]) >> (e & 31u)) & 1u;
            const float base = bit ? wv[j] : rl[j];                  // steps 4, 5: the pulled value replaces the local one
            nl[j] = STEP ? __builtin_fmaf(-eta, rg[j], base) : base; // step 1 of the next round
            nd[j] = first ? rg[j] : rd[j] + rg[j];
        }
        const bool patch = STEP || w_local.p[q] != nullptr;          // uniform over the block
        float* l = static_cast<float*>(w_local.p[q]) + start;
        float* d = STEP ? static_cast<float*>(delta.p[q]) + start : nullptr;
        __syncthreads();                         // the other bitmap is zero everywhere before the next worker's marks go in
        // the next worker's marks and tiles, requested before this worker's stores: the wait for them need not cover the
        // stores' acknowledgements
        if (q + 1 < nw) { mark(q + 1, epre, BLOCK); fetch(q + 1); }
        if (!patch) {
        } else if (vec) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t o = k * 1024 + threadIdx.x * 4;
                st4<1>(l + o, make_float4(nl[4 * k], nl[4 * k + 1], nl[4 * k + 2], nl[4 * k + 3]));
                if (STEP) st4<1>(d + o, make_float4(nd[4 * k], nd[4 * k + 1], nd[4 * k + 2], nd[4 * k + 3]));
            }
        } else {
#pragma unroll
            for (int j = 0; j < EPT; ++j) {
                const uint32_t e = elem_scl(j);
                if (e < len) { l[e] = nl[j]; if (STEP) d[e] = nd[j]; }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Quantised wire values (section 2.2, last sentences; section 4.2: random quantisation, 8 bits,
// buckets of 512).  Per bucket of QB consecutive list entries: scale = largest magnitude;
// per value: code = sign bit | level, level = floor(y) + (u < y - floor(y)), y = (|v| / scale) * 127
// in binary32, u = (random word >> 8) * 2^-24; the word of entry j: word (j mod 4) of
// Philox4x32-10 with counter (j div 4, worker, iteration low, high) and key
// (seed low ^ 0x51534744, seed high ^ kind).  One wave per bucket: lane L holds entries
// 4L..4L+3 and 256+4L..256+4L+3 (two Philox calls), the maximum is a wave reduction (exact,
// whatever the order), the 512 codes leave as two stores of whole lines.
// grid (ceil(buckets / 4), n_workers).
// ---------------------------------------------------------------------------------------
constexpr uint32_t QB = 512;
struct Count64Tab { uint64_t c[MAXW]; };
__device__ __forceinline__ uint32_t quant_code(float v, float s, uint32_t word)
{
    uint32_t level = 0;
    if (s > 0.0f) {
        const float y = (__builtin_fabsf(v) / s) * 127.0f;
        const float l = __builtin_floorf(y);
        const float u = (float)(word >> 8) * 0x1p-24f;
        level = (uint32_t)l + ((u < y - l) ? 1u : 0u);
    }
    return ((__float_as_uint(v) >> 24) & 0x80u) | level;
}

__global__ __launch_bounds__(BLOCK) void k_quantize(PtrTab val, Count64Tab count, uint32_t kind, uint32_t worker0,
                                                    PhiloxKey pk, MutPtrTab code, MutPtrTab scale, int vec_ok)
{
    const uint32_t q = blockIdx.y, lane = lane_id();
    const uint64_t cnt = count.c[q];
    const uint64_t b = (uint64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const uint64_t j0 = b * QB;
    if (j0 >= cnt) return;
    const float* v = static_cast<const float*>(val.p[q]);
    uint8_t* out = static_cast<uint8_t*>(code.p[q]);
    const uint32_t len = (cnt - j0 < QB) ? (uint32_t)(cnt - j0) : QB;
    float x[2][4];
    if (vec_ok && len == QB) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float4 t = ld4<1>(v + j0 + h * 256 + lane * 4);
            x[h][0] = t.x; x[h][1] = t.y; x[h][2] = t.z; x[h][3] = t.w;
        }
    } else {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t e = h * 256 + lane * 4 + c;
                x[h][c] = (e < len) ? v[j0 + e] : 0.0f;
            }
    }
    float s = 0.0f;
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int c = 0; c < 4; ++c) s = __builtin_fmaxf(s, __builtin_fabsf(x[h][c]));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s = __builtin_fmaxf(s, __shfl_xor(s, d, 64));
    if (lane == 0) static_cast<float*>(scale.p[q])[b] = s;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        uint32_t r[4];
        philox4x32_10((uint32_t)((j0 + h * 256 + lane * 4) >> 2), worker0 + q, pk.it_lo, pk.it_hi, pk.seed_lo ^ 0x51534744u,
                      pk.seed_hi ^ kind, r);
        uint32_t packed = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) packed |= quant_code(x[h][c], s, r[c]) << (8 * c);
        const uint32_t e = h * 256 + lane * 4;
        if (vec_ok && len == QB) *reinterpret_cast<uint32_t*>(out + j0 + e) = packed;
        else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (e + c < len) out[j0 + e + c] = (uint8_t)(packed >> (8 * c));
        }
    }
}

// value = sign * ((scale * level) / 127): two binary32 roundings.  Four codes per thread.  grid (blocks, n_workers).
__global__ __launch_bounds__(256) void k_dequantize(PtrTab code, PtrTab scale, Count64Tab count, MutPtrTab val, int vec_ok)
{
    const uint32_t q = blockIdx.y;
    const uint64_t cnt = count.c[q];
    const uint8_t* in = static_cast<const uint8_t*>(code.p[q]);
    const float* sc = static_cast<const float*>(scale.p[q]);
    float* out = static_cast<float*>(val.p[q]);
    const uint64_t stride = (uint64_t)gridDim.x * 256;
    const uint64_t n4 = vec_ok ? cnt / 4 : 0;
    auto one = [](uint32_t c, float s) {
        const float mag = (s * (float)(c & 0x7Fu)) / 127.0f;
        return (c & 0x80u) ? -mag : mag;
    };
    for (uint64_t x = (uint64_t)blockIdx.x * 256 + threadIdx.x; x < n4; x += stride) {
        const uint32_t p = *reinterpret_cast<const uint32_t*>(in + 4 * x);
        const float s = sc[(4 * x) / QB];
        st4<1>(out + 4 * x, make_float4(one(p & 0xFFu, s), one((p >> 8) & 0xFFu, s), one((p >> 16) & 0xFFu, s), one(p >> 24, s)));
    }
    for (uint64_t j = 4 * n4 + (uint64_t)blockIdx.x * 256 + threadIdx.x; j < cnt; j += stride) out[j] = one(in[j], sc[j / QB]);
}

// Signature of the cached keys: sum over list positions j of mix(idx[j] + 2^32 j) modulo 2^64, mix = the output
// function of SplitMix64.  A wrapping integer sum: any order of the partial sums gives the same bits.
// *sig must be zero at launch.  grid: any, 256 threads.
__device__ __forceinline__ uint64_t splitmix64_mix(uint64_t x)
{
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void k_signature(const uint32_t* __restrict__ idx, uint64_t k, unsigned long long* __restrict__ sig)
{
    __shared__ unsigned long long part[4];
    unsigned long long s = 0;
    for (uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x; j < k; j += (uint64_t)gridDim.x * 256)
        s += splitmix64_mix((uint64_t)idx[j] + (j << 32));
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);
    if ((threadIdx.x & 63u) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long t = part[0] + part[1] + part[2] + part[3];
        if (t) atomicAdd(sig, t);
    }
}

// Raw random words of the explorer for indices i0 .. i0+count-1.
__global__ __launch_bounds__(256) void k_debug_philox(uint32_t seed_lo, uint32_t seed_hi, uint32_t it_lo, uint32_t it_hi,
                                                      uint32_t worker, uint32_t i0, uint64_t count, uint32_t* __restrict__ out)
{
    for (uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x; j < count; j += (uint64_t)gridDim.x * 256) {
        const uint32_t i = i0 + (uint32_t)j;
        uint32_t r[4];
        philox4x32_10(i >> 2, worker, it_lo, it_hi, seed_lo, seed_hi, r);
        out[j] = r[i & 3u];
    }
}

}  // namespace slimdp
