// Device-side building blocks of the AsyncMesh stage update for gfx950 (wave64).
//
// Geometry (group, tile, superblock, line, block): am_geometry.h.
// A tile's first entry in a packed list (of selected coordinates, or of the whole lines a tile
// owns in a ring slot) is  sb_base[tile >> 9] + local_off[tile]  (ring slots: the low 24 bits of
// the tile's word; the high 8 bits hold the number of lines the tile owns).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "am_geometry.h"

namespace am {

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two 32x32->64 multiplies.
// ---------------------------------------------------------------------------------------------
struct U4 { uint32_t x0, x1, x2, x3; };

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return U4{c0, c1, c2, c3};
}

struct SubsetKey {
    uint32_t seed_lo, seed_hi;   // Philox key
    uint32_t step_lo, step_hi;   // counter words 2, 3
    uint64_t threshold;          // floor(p 2^32); 2^32 selects everything
    uint32_t mode;               // kDrawCoordinate, kDrawLine or kDrawStratified
    uint32_t block;              // kDrawStratified: B, the block length
};
constexpr uint32_t kDrawCoordinate = 0;   // every coordinate drawn on its own
constexpr uint32_t kDrawLine = 1;         // aligned blocks of 32 coordinates drawn as a whole
constexpr uint32_t kDrawStratified = 2;   // exactly one coordinate of every aligned block of B

// 4-bit membership mask of the coordinates 4*group .. 4*group+3 (bit j = coordinate 4*group+j),
// restricted to the first nvalid of them.
__device__ __forceinline__ uint32_t member_mask(const SubsetKey &k, uint64_t group, int nvalid)
{
    if (k.mode == kDrawStratified) {
        // coordinate mu is selected iff mu - b B == floor(X_b B / 2^32), b = mu / B, X_b the word
        // coordinate number b would get.  The four coordinates of a group lie in at most four
        // consecutive blocks, hence in at most two generator counters.
        const uint32_t B = k.block, mu0 = (uint32_t)(group << 2);
        uint32_t b = mu0 / B, r = mu0 - b * B;
        uint32_t b_last = b, r_last = r;                      // block of the group's last coordinate
#pragma unroll
        for (int j = 0; j < 3; ++j)
            if (++r_last == B) { r_last = 0; ++b_last; }
        const uint32_t c_first = b >> 2, c_last = b_last >> 2;
        const U4 xa = philox4x32_10(c_first, 0u, k.step_lo, k.step_hi, k.seed_lo, k.seed_hi);
        U4 xb = xa;
        if (c_last != c_first) xb = philox4x32_10(c_last, 0u, k.step_lo, k.step_hi, k.seed_lo, k.seed_hi);
        uint32_t m = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool first = (b >> 2) == c_first;
            const uint32_t w0 = first ? xa.x0 : xb.x0, w1 = first ? xa.x1 : xb.x1;
            const uint32_t w2 = first ? xa.x2 : xb.x2, w3 = first ? xa.x3 : xb.x3;
            const uint32_t q = b & 3u;
            const uint32_t word = q == 0u ? w0 : q == 1u ? w1 : q == 2u ? w2 : w3;
            const uint32_t pick = (uint32_t)(((uint64_t)word * B) >> 32);
            m |= (r == pick) ? (1u << j) : 0u;
            if (++r == B) { r = 0; ++b; }
        }
        return m & ((1u << nvalid) - 1u);
    }
    if (k.mode == kDrawLine) {
        // block b = 32 coordinates = 8 groups takes the place of coordinate b in the generator
        const uint64_t b = group >> 3, bg = b >> 2;
        const U4 x = philox4x32_10((uint32_t)bg, (uint32_t)(bg >> 32), k.step_lo, k.step_hi, k.seed_lo, k.seed_hi);
        const uint32_t word = (b & 3u) == 0u ? x.x0 : (b & 3u) == 1u ? x.x1 : (b & 3u) == 2u ? x.x2 : x.x3;
        return ((uint64_t)word < k.threshold) ? ((1u << nvalid) - 1u) : 0u;
    }
    const U4 x = philox4x32_10((uint32_t)group, (uint32_t)(group >> 32), k.step_lo, k.step_hi,
                               k.seed_lo, k.seed_hi);
    uint32_t m = 0;
    m |= ((uint64_t)x.x0 < k.threshold) ? 1u : 0u;
    m |= ((uint64_t)x.x1 < k.threshold) ? 2u : 0u;
    m |= ((uint64_t)x.x2 < k.threshold) ? 4u : 0u;
    m |= ((uint64_t)x.x3 < k.threshold) ? 8u : 0u;
    return m & ((1u << nvalid) - 1u);
}

// ---------------------------------------------------------------------------------------------
// wave64 helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lanes_below(uint64_t ballot)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(ballot >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ballot, 0u));
}

// Exclusive prefix, over the lanes of the wave in lane order, of popcount(mask4); total = sum over
// the whole wave.  Must be called by all 64 lanes together.
__device__ __forceinline__ uint32_t wave_prefix_mask4(uint32_t mask4, uint32_t &total)
{
    uint32_t pre = 0, tot = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint64_t b = __ballot((mask4 >> j) & 1u);
        pre += lanes_below(b);
        tot += (uint32_t)__popcll(b);
    }
    total = tot;
    return pre;
}

// A 32-bit word at an address that is the same for every lane of the wave and that no kernel in
// flight writes (subset offsets written by an earlier kernel): read through the constant address
// space, so that the compiler may use a scalar load that does not queue behind the vector loads.
__device__ __forceinline__ uint32_t uniform_load(const uint32_t *p, uint32_t idx)
{
    typedef const uint32_t __attribute__((address_space(4))) *const_u32_ptr;
    return ((const_u32_ptr)(uintptr_t)p)[idx];
}

// Direct global -> LDS load of 16 bytes per active lane: lane l of the wave writes
// lds_wave_base[4 l .. 4 l + 3] (lds_wave_base must be the same for all lanes); no registers are
// held while the load is in flight.  The data is in LDS once the wave's vector-memory counter has
// drained (lds_dma_wait) -- other waves must additionally pass a workgroup barrier.
__device__ __forceinline__ void lds_dma_16(const float *src, float *lds_wave_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}
__device__ __forceinline__ void lds_dma_wait() { __builtin_amdgcn_s_waitcnt(0x0F70); }     // vmcnt(0)

// ---------------------------------------------------------------------------------------------
// 128-bit accesses with a scalar tail (only the last group of an array can be partial)
// ---------------------------------------------------------------------------------------------
struct F4 { float v[4]; };
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef uint32_t v2u __attribute__((ext_vector_type(2)));

// The arrays of this update are streamed: every element is read once and written once per step,
// so the dense accesses carry the non-temporal hint.
__device__ __forceinline__ F4 load_f32x4(const float *__restrict__ p, uint64_t mu, int nvalid)
{
    F4 r;
    if (nvalid == 4) {
        const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p + mu));
        r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) r.v[j] = (j < nvalid) ? p[mu + j] : 0.0f;
    }
    return r;
}

__device__ __forceinline__ void store_f32x4(float *__restrict__ p, uint64_t mu, int nvalid, const F4 &x)
{
    if (nvalid == 4) {
        const v4f t = {x.v[0], x.v[1], x.v[2], x.v[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<v4f *>(p + mu));
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < nvalid) p[mu + j] = x.v[j];
    }
}

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// round-to-nearest-even fp32 -> bfloat16 (the compiler selects the gfx950 conversion instruction)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    const __bf16 b = (__bf16)f;
    return __builtin_bit_cast(uint16_t, b);
}

// What a value becomes on the wire: 0 = fp32, 1 = bfloat16, 2 = E4M3 (1-4-3, bias 7, no infinity,
// largest finite 448; round to nearest even, saturating).  x / quantum is exact in fp32 (quantum is
// a power of two), so rintf gives the correctly rounded result.
__device__ __forceinline__ float quantize_message(float x, uint32_t msg_dtype)
{
    if (msg_dtype == 1u) return bf16_bits_to_f32(f32_to_bf16_bits(x));
    if (msg_dtype == 2u) {
        const float ax = fabsf(x);
        if (!(ax > 0.0f)) return x;                                   // zero (and NaN) unchanged
        int e = (int)((__float_as_uint(ax) >> 23) & 0xFFu) - 127;      // floor(log2 ax) for normal ax
        e = e < -6 ? -6 : e;                                           // subnormal range: quantum 2^-9
        const float quantum = __uint_as_float((uint32_t)(e - 3 + 127) << 23);
        float r = rintf(ax / quantum) * quantum;
        r = r > 448.0f ? 448.0f : r;
        return copysignf(r, x);
    }
    return x;
}

__device__ __forceinline__ F4 load_bf16x4(const uint16_t *__restrict__ p, uint64_t mu, int nvalid)
{
    F4 r;
    if (nvalid == 4) {
        const v2u t = __builtin_nontemporal_load(reinterpret_cast<const v2u *>(p + mu));
        r.v[0] = __uint_as_float(t.x << 16);
        r.v[1] = __uint_as_float(t.x & 0xFFFF0000u);
        r.v[2] = __uint_as_float(t.y << 16);
        r.v[3] = __uint_as_float(t.y & 0xFFFF0000u);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) r.v[j] = (j < nvalid) ? bf16_bits_to_f32(p[mu + j]) : 0.0f;
    }
    return r;
}

// fp64 -> bfloat16 with ONE rounding to nearest even: the value is first rounded to odd in fp32
// (truncated magnitude, last bit forced to 1 when inexact), which keeps enough information
// (16 spare bits) for the final rounding to land where a direct rounding of the fp64 value would.
__device__ __forceinline__ uint16_t f64_to_bf16_bits(double x)
{
    float f = (float)x;
    const double back = (double)f;
    if (back != x) {
        uint32_t u = __float_as_uint(f);
        if (fabs(back) > fabs(x)) u -= 1u;             // the nearest fp32 was the one further from zero
        f = __uint_as_float(u | 1u);
    }
    return f32_to_bf16_bits(f);
}

__device__ __forceinline__ void store_bf16x4_from_f64(uint16_t *__restrict__ p, uint64_t mu, int nvalid, const double (&x)[4])
{
    if (nvalid == 4) {
        v2u t;
        t.x = (uint32_t)f64_to_bf16_bits(x[0]) | ((uint32_t)f64_to_bf16_bits(x[1]) << 16);
        t.y = (uint32_t)f64_to_bf16_bits(x[2]) | ((uint32_t)f64_to_bf16_bits(x[3]) << 16);
        __builtin_nontemporal_store(t, reinterpret_cast<v2u *>(p + mu));
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < nvalid) p[mu + j] = f64_to_bf16_bits(x[j]);
    }
}

}  // namespace am
