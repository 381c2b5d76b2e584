// Device building blocks of the chunk-2^14 kernels: one workgroup of 256 threads (4
// waves) rotates one chunk held 64 coordinates per thread.  Butterfly stages run in
// stride order 1, 2, 4, ..., 8192, every stage one fp32 add and one fp32 subtract per
// pair, so results are bit-identical to the stage-by-stage definition; between the
// three register-resident groups of stages the chunk is re-shuffled through LDS with
// the conflict-free maps of thc_layout14.h.
#pragma once

#include "thc_device.h"
#include "thc_layout14.h"

#pragma clang fp contract(off)

namespace thc {
namespace k14 {

constexpr int kThreads = 256;
constexpr int kChunkLog2 = 14;
constexpr int kChunk = 1 << kChunkLog2;
constexpr int kRegs = 64;                 // coordinates per thread
constexpr float kInvSqrtC = 0.0078125f;   // 2^-7, exact

struct alignas(16) Shared {
    float xb[kChunk];            // exchange buffer, 64 KB
    uint32_t sgn[kChunk / 32];   // sign diagonal of the chunk, one bit per coordinate
    float red[8];
    uint32_t misc[4];
};

// Butterflies on register-index bits [LO, HI): v[i], v[i+h] <- v[i] + v[i+h], v[i] - v[i+h].
template <int LO, int HI>
__device__ __forceinline__ void butterflies(float (&v)[kRegs]) {
#pragma unroll
    for (int b = LO; b < HI; ++b) {
        const int h = 1 << b;
#pragma unroll
        for (int i = 0; i < kRegs; ++i) {
            if ((i & h) == 0) {
                const float lo = v[i], hi = v[i + h];
                v[i] = lo + hi;
                v[i + h] = lo - hi;
            }
        }
    }
}

// 128 threads compute the 16384 sign bits of the chunk that starts at coordinate g0
// (a multiple of 16384) into sh.sgn.  Needs a barrier before use.
__device__ __forceinline__ void fill_sign_table(Shared& sh, uint64_t g0, uint32_t key0,
                                                uint32_t key1, uint32_t t) {
    if (t < kChunk / 128) {
        const u32x4 s = sign_block((g0 >> 7) + t, key0, key1);
        *reinterpret_cast<uint4*>(&sh.sgn[4 * t]) = make_uint4(s.w[0], s.w[1], s.w[2], s.w[3]);
    }
}

// ---------------------------------------------------------------- input -> layout L1
// Raw 16-byte units in load order (thread t, round j holds unit 256 j + t).
template <int UNITS>  // 8 for bf16, 16 for fp32
struct Raw {
    uint4 u[UNITS];
};

// Coalesced loads of one chunk.  `valid` = number of coordinates of this chunk that
// exist (1..16384); the rest read as zero.  ELEM = bytes per coordinate.
template <int UNITS, int ELEM>
__device__ __forceinline__ void load_raw(Raw<UNITS>& raw, const void* chunk_ptr, uint32_t valid,
                                         uint32_t t) {
    constexpr uint32_t kPerUnit = 16 / ELEM;
    const uint4* src = static_cast<const uint4*>(chunk_ptr);
    if (valid == (uint32_t)kChunk) {
#pragma unroll
        for (int j = 0; j < UNITS; ++j) raw.u[j] = src[j * 256 + t];
    } else {
#pragma unroll
        for (int j = 0; j < UNITS; ++j) {
            const uint32_t unit = j * 256 + t;
            const uint32_t first = unit * kPerUnit;
            uint4 q = make_uint4(0u, 0u, 0u, 0u);
            if (first + kPerUnit <= valid) {
                q = src[unit];
            } else if (first < valid) {
                uint32_t w[4] = {0u, 0u, 0u, 0u};
                if (ELEM == 2) {
                    const uint16_t* p = static_cast<const uint16_t*>(chunk_ptr) + first;
                    for (uint32_t e = 0; first + e < valid; ++e) w[e >> 1] |= (uint32_t)p[e] << (16 * (e & 1));
                } else {
                    const uint32_t* p = static_cast<const uint32_t*>(chunk_ptr) + first;
                    for (uint32_t e = 0; first + e < valid; ++e) w[e] = p[e];
                }
                q = make_uint4(w[0], w[1], w[2], w[3]);
            }
            raw.u[j] = q;
        }
    }
}

template <int UNITS>
__device__ __forceinline__ void raw_to_lds(Shared& sh, const Raw<UNITS>& raw, uint32_t t) {
    constexpr uint32_t kShift = UNITS == 8 ? 3 : 4;
    uint4* dst = reinterpret_cast<uint4*>(sh.xb) + lay14::e0_store_unit(t, 0, kShift);
#pragma unroll
    for (int j = 0; j < UNITS; ++j) dst[j * 256] = raw.u[j];
}

// Reads this thread's 64 consecutive coordinates back (layout L1), widens bf16,
// and applies the sign diagonal when SIGNED.
template <int UNITS, bool SIGNED>
__device__ __forceinline__ void lds_to_l1(const Shared& sh, float (&v)[kRegs], uint32_t t) {
    const uint4* src = reinterpret_cast<const uint4*>(sh.xb);
    uint32_t sw[2] = {0u, 0u};
    if (SIGNED) {
        sw[0] = sh.sgn[2 * t];
        sw[1] = sh.sgn[2 * t + 1];
    }
#pragma unroll
    for (int k = 0; k < UNITS; ++k) {
        const uint4 q = src[lay14::e0_load_unit(t, k, UNITS)];
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
        if (UNITS == 8) {  // bf16: 8 coordinates per unit, two per dword
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int r = 8 * k + 2 * d;  // even coordinate of the pair
                const int rr = r & 31;
                uint32_t x = w[d];
                if (SIGNED) {
                    const uint32_t s = sw[r >> 5];
                    const uint32_t m_lo = (rr <= 15 ? (s << (15 - rr)) : (s >> (rr - 15))) & 0x8000u;
                    const uint32_t m_hi = (s << (30 - rr)) & 0x80000000u;
                    x ^= m_lo | m_hi;
                }
                v[r] = __uint_as_float(x << 16);
                v[r + 1] = __uint_as_float(x & 0xFFFF0000u);
            }
        } else {  // fp32: 4 coordinates per unit
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int r = 4 * k + d;
                uint32_t x = w[d];
                if (SIGNED) x ^= (sw[r >> 5] << (31 - (r & 31))) & 0x80000000u;
                v[r] = __uint_as_float(x);
            }
        }
    }
}

// ------------------------------------------------------------------ LDS exchanges
// L1 -> L2 (inside each wave's quarter of the buffer).
__device__ __forceinline__ void exchange_x1_store(Shared& sh, const float (&v)[kRegs], uint32_t lane,
                                                  uint32_t wave) {
    float* reg = sh.xb + wave * 4096;
#pragma unroll
    for (int q = 0; q < 16; ++q)
        *reinterpret_cast<float4*>(reg + lay14::x1_store(lane, q)) =
            make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
}
__device__ __forceinline__ void exchange_x1_load(const Shared& sh, float (&v)[kRegs], uint32_t lane,
                                                 uint32_t wave) {
    const float* reg = sh.xb + wave * 4096;
#pragma unroll
    for (int r = 0; r < kRegs; ++r) v[r] = reg[lay14::x1_load(lane, r)];
}
// L2 -> L3 (whole buffer).
__device__ __forceinline__ void exchange_x2_store(Shared& sh, const float (&v)[kRegs], uint32_t lane,
                                                  uint32_t wave) {
#pragma unroll
    for (int q = 0; q < 16; ++q)
        *reinterpret_cast<float4*>(sh.xb + lay14::x2_store(wave, lane, q)) =
            make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
}
__device__ __forceinline__ void exchange_x2_load(const Shared& sh, float (&v)[kRegs], uint32_t lane,
                                                 uint32_t wave) {
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e + 16 * s] = sh.xb[lay14::x2_load(wave, lane, e, s)];
}

// Stages 0..13 on a chunk that sits in layout L1 in v; result (unnormalised H_c x) in
// layout L3: v[e + 16 s] is coordinate 4096 s + 16 t + e of the chunk.  Uses the whole
// exchange buffer; it is free again after the trailing barrier of this function.
__device__ __forceinline__ void rotate_l1_to_l3(Shared& sh, float (&v)[kRegs], uint32_t lane,
                                                uint32_t wave) {
    butterflies<0, 6>(v);          // strides 1..32
    __syncthreads();               // every thread is past its reads of the buffer
    exchange_x1_store(sh, v, lane, wave);
    __syncthreads();
    exchange_x1_load(sh, v, lane, wave);
    butterflies<0, 6>(v);          // strides 64..2048
    __syncthreads();
    exchange_x2_store(sh, v, lane, wave);
    __syncthreads();
    exchange_x2_load(sh, v, lane, wave);
    butterflies<4, 6>(v);          // strides 4096, 8192
    __syncthreads();
}

// max |v| over the whole chunk (all threads return it).  One barrier pair.
__device__ __forceinline__ float chunk_absmax(Shared& sh, const float (&v)[kRegs], uint32_t lane,
                                              uint32_t wave) {
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < kRegs; i += 2) m = fmaxf(m, fmaxf(fabsf(v[i]), fabsf(v[i + 1])));
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    if (lane == 0) sh.red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(sh.red[0], sh.red[1]), fmaxf(sh.red[2], sh.red[3]));
    __syncthreads();
    return m;
}

// --------------------------------------------------------------------- quantizer
// Stochastic rounding of the L3-resident chunk onto the 2^BITS-point grid of [-s, s],
// packed and stored.  v holds the UNNORMALISED rotation; y = v * 2^-7.
//   g0       global index of the chunk's first coordinate
//   payload  start of this worker's payload
template <int BITS>
__device__ __forceinline__ void quantize_store(const float (&v)[kRegs], float s, uint64_t g0,
                                               uint32_t worker, uint32_t key0, uint32_t key1,
                                               uint8_t* payload, uint32_t t) {
    constexpr uint32_t L = (1u << BITS) - 1u;
    const float two = s + s;
    const float inv = two != 0.0f ? (float)L / two : 0.0f;
#pragma unroll
    for (int run = 0; run < 4; ++run) {
        const uint64_t g = g0 + (uint64_t)run * 4096u + (uint64_t)t * 16u;
        const u32x4 rb = round_block(g >> 4, worker, key0, key1);
        uint32_t pk[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float y = v[e + 16 * run] * kInvSqrtC;
            const float pos = (y + s) * inv;
            const uint32_t r = (rb.w[e >> 2] >> (8 * (e & 3))) & 0xFFu;
            const float u = __builtin_fmaf((float)r, 0x1p-8f, 0x1p-9f);   // (r + 0.5) / 256, exact
            const float tt = pos + u;
            uint32_t q = (uint32_t)tt;                                     // tt >= 0: truncation = floor
            q = q < L ? q : L;
            const int bit = e * BITS;
            pk[bit >> 5] |= q << (bit & 31);
        }
        uint8_t* dst = payload + (g * BITS) / 8u;
        if (BITS == 8) {
            *reinterpret_cast<uint4*>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        } else if (BITS == 4) {
            *reinterpret_cast<uint2*>(dst) = make_uint2(pk[0], pk[1]);
        } else {
            *reinterpret_cast<uint32_t*>(dst) = pk[0];
        }
    }
}

// Output side of the inverse rotation: x = D (v * 2^-7), L3 layout, first `valid`
// coordinates of the chunk are stored.
__device__ __forceinline__ void store_signed_l3(const Shared& sh, const float (&v)[kRegs], float* out,
                                                uint32_t valid, uint32_t t) {
#pragma unroll
    for (int run = 0; run < 4; ++run) {
        const uint32_t i0 = run * 4096u + t * 16u;
        const uint32_t sb = (sh.sgn[i0 >> 5] >> (i0 & 31u)) & 0xFFFFu;
        float x[16];
#pragma unroll
        for (int e = 0; e < 16; ++e)
            x[e] = __uint_as_float(__float_as_uint(v[e + 16 * run] * kInvSqrtC) ^
                                   ((sb << (31 - e)) & 0x80000000u));
        if (i0 + 16u <= valid) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                *reinterpret_cast<float4*>(out + i0 + 4 * k) =
                    make_float4(x[4 * k], x[4 * k + 1], x[4 * k + 2], x[4 * k + 3]);
        } else {
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if (i0 + e < valid) out[i0 + e] = x[e];
        }
    }
}

}  // namespace k14
}  // namespace thc
