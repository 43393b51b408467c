// Device-side building blocks of libslimdp (gfx950, wave64).  Included only by slimdp.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "slimdp.h"

namespace slimdp {

constexpr uint32_t TILE = SLIMDP_TILE;            // parameters per tile
constexpr uint32_t TILE_WORDS = TILE / 32;        // bitmap words per tile
constexpr uint32_t SUB = 1024, SUB_WORDS = SUB / 32, SUBS = TILE / SUB;   // sub-tile: one wave's share of a tile
constexpr uint32_t NONE = 0xFFFFFFFFu;
constexpr int MAXW = SLIMDP_MAX_WORKERS;
constexpr int BLOCK = 256;                        // threads per block in the tile kernels
constexpr int EPT = TILE / BLOCK;                 // elements per thread per tile (16)

// Histogram storage per (batch, segment): level 0, level 1, level 2.
constexpr uint32_t H_L0 = 0, H_L1 = 8192, H_L2 = 12288, H_STRIDE = 16384;

// Core ranking key = raw bits of the score: 13 + 12 + 7 bits.
constexpr uint32_t CORE_SHIFT0 = 19, CORE_NB0 = 8192, CORE_SHIFT1 = 7, CORE_NB1 = 4096, CORE_NB2 = 128;

struct PtrTab { const void* p[MAXW]; };           // host pointer tables travel as kernel arguments
struct MutPtrTab { void* p[MAXW]; };

// Selection state of one (batch, segment): the radix descent towards the threshold key.
struct SegState {
    uint32_t need0;     // number of elements to select
    uint32_t need;      // of those, how many still come from the keys matching `prefix`
    uint32_t prefix;    // keys still in play satisfy (key >> shift[level-1]) == prefix
    uint32_t none;      // 1: nothing is selected here
    uint32_t tau;       // threshold key once all levels are done
    uint32_t quota;     // how many keys == tau are taken, lowest index first
    uint32_t bound_m1;  // explorer only: candidates are words r <= bound_m1, key = bound_m1 - r
    uint32_t tie_all;   // 1: the quota covers every key equal to tau
    uint32_t shift[3];  // digit of level l = (key >> shift[l]) & (nbins[l] - 1); level 0 unmasked
    uint32_t nbins[3];
    uint32_t sure_m1;   // explorer: words r <= sure_m1 are taken without looking at their rank (if has_gt)
    uint32_t has_gt;    // a bitmap of certainly selected parameters exists (core: always; explorer: narrow zone)
};
static_assert(sizeof(SegState) == 64, "SegState layout");

struct SegInit { uint32_t need; uint32_t bound_m1; uint32_t shift0; uint32_t sure_m1; uint32_t has_gt; };
constexpr int INIT_CHUNK = 128;
struct SegInitChunk { SegInit s[INIT_CHUNK]; };

// ---------------------------------------------------------------------------------------
// wave / block primitives
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    const uint32_t lane = lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t t = __shfl_up(v, d, 64);
        if (lane >= (uint32_t)d) v += t;
    }
    return v;
}

// Buffer addressing: a 128-bit descriptor in scalar registers (base, byte range, no stride)
// plus one 32-bit per-lane byte offset and a scalar offset.  Compared with flat 64-bit
// per-lane addresses this keeps the address arithmetic out of the vector registers, and
// accesses outside [0, bytes) are dropped by the hardware.  Callers pass 0 as the scalar
// offset and fold the wave's part into the lane offset: with a scalar-register offset the
// 16-byte forms were seen to store, now and then, a stale first dword on this target
// (caught by the several-tiles-per-block scoring test).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_of(const void* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float4 buffer_load4(__amdgpu_buffer_rsrc_t r, uint32_t lane_bytes, uint32_t wave_bytes)
{
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_bytes, (int)wave_bytes, 0);
    return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
// The same with a cache policy (the intrinsic's auxiliary operand must be a constant: 0 = default, 2 = non-temporal,
// for data that is touched once).
template <int AUX>
__device__ __forceinline__ float4 buffer_load4_aux(__amdgpu_buffer_rsrc_t r, uint32_t lane_bytes)
{
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)lane_bytes, 0, AUX);
    return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
template <int AUX>
__device__ __forceinline__ void buffer_store4_aux(__amdgpu_buffer_rsrc_t r, uint32_t lane_bytes, float4 f)
{
    u32x4 v;
    v.x = __float_as_uint(f.x); v.y = __float_as_uint(f.y); v.z = __float_as_uint(f.z); v.w = __float_as_uint(f.w);
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)lane_bytes, 0, AUX);
}
__device__ __forceinline__ void buffer_store4(__amdgpu_buffer_rsrc_t r, uint32_t lane_bytes, uint32_t wave_bytes, float4 f)
{
    u32x4 v;
    v.x = __float_as_uint(f.x); v.y = __float_as_uint(f.y); v.z = __float_as_uint(f.z); v.w = __float_as_uint(f.w);
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)lane_bytes, (int)wave_bytes, 0);
}

__device__ __forceinline__ void buffer_store1(__amdgpu_buffer_rsrc_t r, uint32_t lane_bytes, uint32_t v)
{
    __builtin_amdgcn_raw_buffer_store_b32(v, r, (int)lane_bytes, 0, 0);
}

// OR over aligned groups of eight lanes, every lane of a group getting the result.  Three
// data-parallel-primitive moves inside a row of 16 lanes (swap neighbours, swap pairs, mirror
// each half row) instead of three trips through the LDS crossbar.
__device__ __forceinline__ uint32_t or_reduce8(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);      // quad_perm [1,0,3,2]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);      // quad_perm [2,3,0,1]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true);     // row_half_mirror
    return v;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// Exclusive prefix sum over the block (NWAVES*64 threads, all must call).  wtot: NWAVES words
// of shared memory, free for reuse on return.
template <int NWAVES>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* wtot, uint32_t& total)
{
    const uint32_t lane = lane_id(), wid = threadIdx.x >> 6;
    const uint32_t incl = wave_incl_scan(v);
    if (lane == 63) wtot[wid] = incl;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) {
        const uint32_t t = wtot[w];
        if ((uint32_t)w < wid) base += t;
        tot += t;
    }
    __syncthreads();
    total = tot;
    return base + incl - v;
}

// Local element handled by (thread, slot j) of a tile.  Vector layout: four consecutive
// elements per thread and round (16-byte loads); scalar layout: one element per thread and round.
__device__ __forceinline__ uint32_t elem_vec(int j) { return (uint32_t)(j >> 2) * 1024u + threadIdx.x * 4u + (uint32_t)(j & 3); }
__device__ __forceinline__ uint32_t elem_scl(int j) { return (uint32_t)j * BLOCK + threadIdx.x; }

__device__ __forceinline__ uint32_t mask_below(uint32_t bit) { return (1u << bit) - 1u; }   // bit in 0..31

// Accesses to data that is touched once (streamed): NT != 0 marks them non-temporal, so that they do not
// push lines that will be used again out of the caches.  A non-temporal store must cover whole 128-byte lines
// per instruction (a partial one goes to memory as a read-modify-write).
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
template <int NT> __device__ __forceinline__ float4 ld4(const float* p)
{
    if (NT) {
        const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
        return make_float4(v.x, v.y, v.z, v.w);
    }
    return *reinterpret_cast<const float4*>(p);
}
template <int NT> __device__ __forceinline__ uint4 ld4u(const uint32_t* p)
{
    if (NT) {
        const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
        return make_uint4(v.x, v.y, v.z, v.w);
    }
    return *reinterpret_cast<const uint4*>(p);
}
template <int NT> __device__ __forceinline__ void st4(float* p, float4 v)
{
    if (NT) {
        f32x4_t o; o.x = v.x; o.y = v.y; o.z = v.z; o.w = v.w;
        __builtin_nontemporal_store(o, reinterpret_cast<f32x4_t*>(p));
    } else *reinterpret_cast<float4*>(p) = v;
}
template <int NT, class Tp> __device__ __forceinline__ Tp ld1(const Tp* p)
{
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}
template <int NT, class Tp> __device__ __forceinline__ void st1(Tp* p, Tp v)
{
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// ---------------------------------------------------------------------------------------
// Philox4x32 with 10 rounds (Salmon et al., SC'11): the explorer's random words.
// Counter (c0, c1, c2, c3), key (k0, k1).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t out[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        // three-input exclusive or in one instruction (truth table 0x96)
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The same with the ten round keys handed over (key + round * Weyl constant): a kernel that draws many words under
// one key computes them once and, made opaque to the compiler, keeps them in vector registers; left to itself the
// compiler holds them in scalar registers, runs out of those and reloads each with a lane read before every use.
struct PhiloxRoundKeys { uint32_t k0[10], k1[10]; };
__device__ __forceinline__ PhiloxRoundKeys philox_round_keys(uint32_t k0, uint32_t k1)
{
    PhiloxRoundKeys rk;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        rk.k0[r] = k0 + (uint32_t)r * 0x9E3779B9u;
        rk.k1[r] = k1 + (uint32_t)r * 0xBB67AE85u;
        asm volatile("" : "+v"(rk.k0[r]), "+v"(rk.k1[r]));
    }
    return rk;
}
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, const PhiloxRoundKeys& rk,
                                              uint32_t out[4])
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, rk.k0[r], 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, rk.k1[r], 0x96);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Equation (1) with the rounding the interface promises: one fused multiply-add, canonical NaN.
__device__ __forceinline__ float significance(float w, float gsum, float c)
{
    float s = __builtin_fmaf(c, __builtin_fabsf(gsum), __builtin_fabsf(w));
    if (s != s) s = __uint_as_float(0x7FC00000u);
    return s;
}

}  // namespace slimdp
