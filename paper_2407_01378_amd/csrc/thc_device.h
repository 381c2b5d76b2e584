// Device-side helpers shared by the gfx950 kernels: Philox4x32-10, the two random
// streams (sign diagonal, rounding bytes) and small bit utilities.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#pragma clang fp contract(off)

namespace thc {

constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;
constexpr uint32_t kTagSign = 0x5349474Eu;   // fourth counter word of the sign stream
constexpr uint32_t kTagRound = 0x524F554Eu;  // fourth counter word of the rounding stream
constexpr int kRoundingBits = 8;             // random bits per coordinate
constexpr int kCoordsPerRoundBlock = 128 / kRoundingBits;  // 16
// fp32 evaluation order of the quantizer, by the grid's largest index L.  Up to here the
// position plus noise is t = fma(y, inv, L/2 + u); above (8-bit payloads) the offset is
// rounded first, t = fma(y + s, inv, u): inv = L / (2 s) carries a relative rounding error
// of 2^-24, which the first form turns into an absolute error of up to (L/2) 2^-24 in t -
// 7.6e-6 for L = 255, more than the 1e-6 max(1, |t|) an index is allowed to depend on.
constexpr uint32_t kSingleFmaMaxLevels = 31;

// Narrowest range of a chunk (2 s on the symmetric grids, hi - lo on the min/max grid) that is
// quantized by the rounding rule.  The rule needs the reciprocal grid step L / range, which
// fp32 cannot hold for much smaller ranges (255 / 2^-121 overflows); a narrower range is
// treated like an empty one: every index 0 (the centre on the signed grid), and the chunk
// decodes at most 2^-119 off per rotated coordinate.  `range >= kMinRange` is also false for a
// NaN, which then takes the same path.
constexpr float kMinRange = 0x1p-119f;

struct u32x4 {
    uint32_t w[4];
};

// a ^ b ^ c as one three-input bitwise operation (truth table 0x96); the compiler does
// not form it from two xors by itself.
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// a ^ (b & c) as one operation (truth table 0x78).
__device__ __forceinline__ uint32_t xor_masked(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x78);
}

// Largest of the 64 lanes' values in unsigned order, returned to every lane.  Lane
// exchanges are data-parallel-primitive moves inside the vector ALU (no LDS traffic):
// within quads, within half rows, within rows of 16, then row 0 -> 1 and 2 -> 3, then
// rows 0..1 -> 2..3, which leaves the result in lane 63.  All 64 lanes must be active.
__device__ __forceinline__ uint32_t wave_umax(uint32_t x) {
    auto step = [&](auto ctrl, auto rows) {
        const uint32_t y = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, decltype(ctrl)::value,
                                                                 decltype(rows)::value, 0xF, false);
        x = y > x ? y : x;
    };
    using std::integral_constant;
    step(integral_constant<int, 0xB1>{}, integral_constant<int, 0xF>{});   // quad_perm [1,0,3,2]
    step(integral_constant<int, 0x4E>{}, integral_constant<int, 0xF>{});   // quad_perm [2,3,0,1]
    step(integral_constant<int, 0x141>{}, integral_constant<int, 0xF>{});  // row_half_mirror
    step(integral_constant<int, 0x140>{}, integral_constant<int, 0xF>{});  // row_mirror
    step(integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{});  // row_bcast:15 into rows 1, 3
    step(integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{});  // row_bcast:31 into rows 2, 3
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies and
// a word permutation, key bumped by the Weyl constants between rounds.
__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    u32x4 o;
    o.w[0] = c0;
    o.w[1] = c1;
    o.w[2] = c2;
    o.w[3] = c3;
    return o;
}

// 128 sign bits of coordinates [128*block, 128*block + 128): bit (g mod 32) of
// word ((g div 32) mod 4); identical for every worker.
__device__ __forceinline__ u32x4 sign_block(uint64_t block, uint32_t k0, uint32_t k1) {
    return philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), 0u, kTagSign, k0, k1);
}

// 16 rounding bytes of coordinates [16*block, 16*block + 16) of one worker.
__device__ __forceinline__ u32x4 round_block(uint64_t block, uint32_t worker, uint32_t k0,
                                             uint32_t k1) {
    return philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), worker, kTagRound, k0, k1);
}

// 16-byte accesses that tell the memory system the data will not be used again soon
// (a payload read for the last time, an output nobody in this library reads back): they
// leave the caches to the data that is reused.
typedef uint32_t u32x4_vec __attribute__((ext_vector_type(4)));
typedef float f32x4_vec __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_last_use(const uint4* p) {
    const u32x4_vec q = __builtin_nontemporal_load(reinterpret_cast<const u32x4_vec*>(p));
    return make_uint4(q.x, q.y, q.z, q.w);
}
__device__ __forceinline__ uint2 load_last_use(const uint2* p) {
    typedef uint32_t u32x2_vec __attribute__((ext_vector_type(2)));
    const u32x2_vec q = __builtin_nontemporal_load(reinterpret_cast<const u32x2_vec*>(p));
    return make_uint2(q.x, q.y);
}
__device__ __forceinline__ void store_streaming(float* p, float a, float b, float c, float d) {
    const f32x4_vec q = {a, b, c, d};
    __builtin_nontemporal_store(q, reinterpret_cast<f32x4_vec*>(p));
}

__device__ __forceinline__ float flip_sign(float v, uint32_t bit) {
    return __uint_as_float(__float_as_uint(v) ^ (bit << 31));
}

__device__ __forceinline__ float bf16_bits_to_float(uint32_t h) {
    return __uint_as_float(h << 16);
}

}  // namespace thc
