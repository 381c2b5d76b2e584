// Device building blocks of the chunk-2^14 kernels: one workgroup of 512 threads (8
// waves) rotates one chunk held 32 coordinates per thread.  Butterfly stages run in
// stride order 1, 2, 4, ..., 8192, every stage one fp32 add and one fp32 subtract per
// pair, so results are bit-identical to the stage-by-stage definition; between the
// three register-resident groups of stages (5 + 5 + 4) the chunk is re-shuffled through
// LDS with the conflict-free maps of thc_layout14.h, and once more into the layout the
// consumer wants (32 consecutive coordinates per thread for the quantizer, 4 per lane
// for coalesced fp32 stores).
#pragma once

#include "thc_device.h"
#include "thc_layout14.h"

#pragma clang fp contract(off)

namespace thc {
namespace k14 {

constexpr int kThreads = 512;
constexpr int kChunkLog2 = 14;
constexpr int kChunk = 1 << kChunkLog2;
constexpr int kRegs = 32;                 // coordinates per thread
constexpr float kInvSqrtC = 0.0078125f;   // 2^-7, exact

// Wave priorities (s_setprio) by phase.  Two workgroups share a CU; a wave inside the
// rotation alternates short bursts of arithmetic with LDS exchanges and barriers, while
// the phase after the rotation (quantize and pack, or scale and store) is one long run of
// independent arithmetic.  Letting the rotation go first keeps its LDS and barrier
// latencies off the critical path and leaves the long run to fill the gaps; measured on
// the encode kernel this is worth 9 %.
constexpr int kPrioRotateEarly = 1;   // stages before the second exchange
constexpr int kPrioRotateLate = 2;    // stages after it
constexpr int kPrioExchange = 3;      // issuing LDS stores / loads of an exchange
constexpr int kPrioTail = 0;          // everything after the last exchange
// The memory-bound decode kernels run every phase at the default priority (PRIO = false):
// there the same scheme delays the next item's loads and costs 15 %.
template <bool PRIO, int LEVEL>
__device__ __forceinline__ void set_prio() {
    if constexpr (PRIO) __builtin_amdgcn_s_setprio(LEVEL);
}

struct alignas(16) SignTable {
    uint32_t sgn[kChunk / 32];   // sign diagonal of a chunk, bit (i mod 32) of word i / 32
    uint32_t sgx[kChunk / 32];   // the same words with even bits gathered in the low half,
                                 // odd bits in the high half (for bf16 pairs)
};
struct alignas(16) Shared {
    float xb[kChunk];            // exchange buffer, 64 KB
    SignTable sign[2];           // persistent kernels fill the next chunk's table ahead of time
    float red[8];                // one slot per wave for workgroup-wide reductions
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

// Even bits of x to the low half, odd bits to the high half (bit 2p -> p, 2p+1 -> 16+p).
__device__ __forceinline__ uint32_t unshuffle_bits(uint32_t x) {
    uint32_t t;
    t = (x ^ (x >> 1)) & 0x22222222u; x ^= t ^ (t << 1);
    t = (x ^ (x >> 2)) & 0x0C0C0C0Cu; x ^= t ^ (t << 2);
    t = (x ^ (x >> 4)) & 0x00F000F0u; x ^= t ^ (t << 4);
    t = (x ^ (x >> 8)) & 0x0000FF00u; x ^= t ^ (t << 8);
    return x;
}

// 128 threads (two waves; which two is chosen by `turn`, so that persistent kernels can
// spread this work over the SIMDs from item to item) compute the 16384 sign bits of the
// chunk that starts at coordinate g0 (a multiple of 16384).  SGN / SGX select the forms
// the caller will read.  Needs a barrier before use.
template <bool SGN, bool SGX>
__device__ __forceinline__ void fill_sign_table(SignTable& tab, uint64_t g0, uint32_t key0,
                                                uint32_t key1, uint32_t t, uint32_t turn = 0u) {
    if ((t >> 7) == (turn & 3u)) {
        const uint32_t b = t & 127u;
        const u32x4 s = sign_block((g0 >> 7) + b, key0, key1);
        if (SGN) *reinterpret_cast<uint4*>(&tab.sgn[4 * b]) = make_uint4(s.w[0], s.w[1], s.w[2], s.w[3]);
        if (SGX)
            *reinterpret_cast<uint4*>(&tab.sgx[4 * b]) =
                make_uint4(unshuffle_bits(s.w[0]), unshuffle_bits(s.w[1]), unshuffle_bits(s.w[2]),
                           unshuffle_bits(s.w[3]));
    }
}

// ---------------------------------------------------------------- input -> layout L1
// Raw 16-byte units of a chunk in load order.  Coalesced order: thread t, round j holds
// unit 512 j + t, and the chunk passes through LDS to reach layout L1.  Direct order:
// thread t holds units UNITS t + j, its own 32 consecutive coordinates (layout L1 at
// once; every load instruction of a wave then touches UNITS times as many cache lines,
// each of which the wave's other loads hit again in the vector cache).
template <int UNITS>  // 4 for bf16, 8 for fp32
struct Raw {
    uint4 u[UNITS];
};

// Coalesced loads of one chunk.  `valid` = number of coordinates of this chunk that
// exist (1..16384); the rest read as zero.  ELEM = bytes per coordinate.
template <int UNITS, int ELEM, bool DIRECT = false>
__device__ __forceinline__ void load_raw(Raw<UNITS>& raw, const void* chunk_ptr, uint32_t valid,
                                         uint32_t t) {
    constexpr uint32_t kPerUnit = 16 / ELEM;
    const uint4* src = static_cast<const uint4*>(chunk_ptr);
    if (valid == (uint32_t)kChunk) {
#pragma unroll
        for (int j = 0; j < UNITS; ++j) raw.u[j] = src[DIRECT ? UNITS * t + j : j * kThreads + t];
    } else {
#pragma unroll
        for (int j = 0; j < UNITS; ++j) {
            const uint32_t unit = DIRECT ? UNITS * t + j : j * kThreads + t;
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
    uint4* dst = reinterpret_cast<uint4*>(sh.xb) + lay14::e0_store_unit(t, 0, UNITS);
#pragma unroll
    for (int j = 0; j < UNITS; ++j) dst[j * kThreads] = raw.u[j];
}

// The thread's 32 consecutive coordinates as UNITS 16-byte units -> fp32 registers
// (layout L1): widens bf16 and applies the sign diagonal when SIGNED.
template <int UNITS, bool SIGNED>
__device__ __forceinline__ void units_to_l1(const SignTable& tab, const uint4 (&unit)[UNITS],
                                            float (&v)[kRegs], uint32_t t) {
    if (UNITS == 4) {  // bf16: 8 coordinates per unit, two per dword
        const uint32_t sx = SIGNED ? tab.sgx[t] : 0u;
#pragma unroll
        for (int k = 0; k < UNITS; ++k) {
            const uint32_t w[4] = {unit[k].x, unit[k].y, unit[k].z, unit[k].w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int pair = 4 * k + d;  // coordinates 2 pair, 2 pair + 1
                uint32_t x = w[d];
                // sign bits of the pair sit at bits `pair` and 16 + `pair` of sx
                if (SIGNED) x = xor_masked(x, pair == 15 ? sx : (sx << (15 - pair)), 0x80008000u);
                v[2 * pair] = __uint_as_float(x << 16);
                v[2 * pair + 1] = __uint_as_float(x & 0xFFFF0000u);
            }
        }
    } else {  // fp32: 4 coordinates per unit
        const uint32_t sw = SIGNED ? tab.sgn[t] : 0u;
#pragma unroll
        for (int k = 0; k < UNITS; ++k) {
            const uint32_t w[4] = {unit[k].x, unit[k].y, unit[k].z, unit[k].w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int r = 4 * k + d;
                uint32_t x = w[d];
                if (SIGNED) x = xor_masked(x, r == 31 ? sw : (sw << (31 - r)), 0x80000000u);
                v[r] = __uint_as_float(x);
            }
        }
    }
}

// Reads this thread's 32 consecutive coordinates back from the buffer (after raw_to_lds
// and a barrier) into layout L1.
template <int UNITS, bool SIGNED>
__device__ __forceinline__ void lds_to_l1(const Shared& sh, const SignTable& tab, float (&v)[kRegs],
                                          uint32_t t) {
    const uint4* src = reinterpret_cast<const uint4*>(sh.xb);
    uint4 unit[UNITS];
#pragma unroll
    for (int k = 0; k < UNITS; ++k) unit[k] = src[lay14::e0_load_unit(t, k, UNITS)];
    units_to_l1<UNITS, SIGNED>(tab, unit, v, t);
}

// ------------------------------------------------------------------ LDS exchanges
__device__ __forceinline__ void x1_store(Shared& sh, const float (&v)[kRegs], uint32_t lane, uint32_t wave) {
    float* reg = sh.xb + wave * 2048;
#pragma unroll
    for (int q = 0; q < 8; ++q)
        *reinterpret_cast<float4*>(reg + lay14::x1_store(lane, q)) =
            make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
}
__device__ __forceinline__ void x1_load(const Shared& sh, float (&v)[kRegs], uint32_t lane, uint32_t wave) {
    const float* reg = sh.xb + wave * 2048;
#pragma unroll
    for (int r = 0; r < kRegs; ++r) v[r] = reg[lay14::x1_load(lane, r)];
}
__device__ __forceinline__ void x2_store(Shared& sh, const float (&v)[kRegs], uint32_t lane, uint32_t wave) {
#pragma unroll
    for (int q = 0; q < 8; ++q)
        *reinterpret_cast<float4*>(sh.xb + lay14::x2_store(wave, lane, q)) =
            make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
}
__device__ __forceinline__ void x2_load(const Shared& sh, float (&v)[kRegs], uint32_t lane, uint32_t wave) {
#pragma unroll
    for (int r = 0; r < kRegs; ++r) v[r] = sh.xb[lay14::x2_load(wave, lane, r)];
}
__device__ __forceinline__ void x3e_store(Shared& sh, const float (&v)[kRegs], uint32_t lane, uint32_t wave) {
#pragma unroll
    for (int r = 0; r < kRegs; ++r) sh.xb[lay14::x3e_store(wave, lane, r)] = v[r];
}
__device__ __forceinline__ void x3e_load(const Shared& sh, float (&v)[kRegs], uint32_t lane, uint32_t wave) {
    const float4* units = reinterpret_cast<const float4*>(sh.xb);   // unit-indexed: provably 16-byte aligned
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const float4 f = units[lay14::x3e_load_unit(wave, lane, q)];
        v[4 * q] = f.x;
        v[4 * q + 1] = f.y;
        v[4 * q + 2] = f.z;
        v[4 * q + 3] = f.w;
    }
}
__device__ __forceinline__ void x3d_store(Shared& sh, const float (&v)[kRegs], uint32_t lane, uint32_t wave) {
#pragma unroll
    for (int r = 0; r < kRegs; ++r) sh.xb[lay14::x3d_store(wave, lane, r)] = v[r];
}
__device__ __forceinline__ void x3d_load(const Shared& sh, float (&v)[kRegs], uint32_t lane, uint32_t wave) {
    const float4* units = reinterpret_cast<const float4*>(sh.xb);   // unit-indexed: provably 16-byte aligned
#pragma unroll
    for (int h = 0; h < 8; ++h) {
        const float4 f = units[lay14::x3d_load_unit(wave, lane, h)];
        v[4 * h] = f.x;
        v[4 * h + 1] = f.y;
        v[4 * h + 2] = f.z;
        v[4 * h + 3] = f.w;
    }
}

// Stages 0..13 on a chunk that sits in layout L1 in v; result (unnormalised H_c x) in
// layout L3.  Starts with a barrier (every thread is past its earlier reads of the
// buffer); the buffer is still being read when it returns.  hook.at<K>() is called at
// three points that are separated by an LDS exchange each (K = 0 before the first group
// of stages, 1 before the second, 2 before the third): a persistent kernel hangs the
// next item's global loads there.
struct NoHook {
    template <int K>
    __device__ __forceinline__ void at() {}
};
template <bool PRIO, class Hook>
__device__ __forceinline__ void rotate_l1_to_l3(Shared& sh, float (&v)[kRegs], uint32_t lane,
                                                uint32_t wave, Hook& hook) {
    set_prio<PRIO, kPrioRotateEarly>();
    hook.template at<0>();
    butterflies<0, 5>(v);          // strides 1..16
    __syncthreads();
    // the first exchange stays inside each wave's own 8 KB of the buffer, and a wave's
    // LDS accesses execute in order: no barrier between its stores and loads
    set_prio<PRIO, kPrioExchange>();
    x1_store(sh, v, lane, wave);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    x1_load(sh, v, lane, wave);
    set_prio<PRIO, kPrioRotateEarly>();
    hook.template at<1>();
    butterflies<0, 5>(v);          // strides 32..512
    __syncthreads();
    set_prio<PRIO, kPrioExchange>();
    x2_store(sh, v, lane, wave);
    __syncthreads();
    x2_load(sh, v, lane, wave);
    set_prio<PRIO, kPrioRotateLate>();
    hook.template at<2>();
    butterflies<1, 5>(v);          // strides 1024..8192 (register bit 0 is i9, already done)
}
template <bool PRIO>
__device__ __forceinline__ void rotate_l1_to_l3(Shared& sh, float (&v)[kRegs], uint32_t lane,
                                                uint32_t wave) {
    NoHook none;
    rotate_l1_to_l3<PRIO>(sh, v, lane, wave, none);
}

// max |v| over this thread's registers, then over the wave.
__device__ __forceinline__ float wave_absmax(const float (&v)[kRegs]) {
    float m = 0.0f;
#pragma unroll
    for (int i = 0; i < kRegs; i += 2)
        asm("v_max3_f32 %0, %1, |%2|, |%3|" : "=v"(m) : "v"(m), "v"(v[i]), "v"(v[i + 1]));
    // m >= 0: floats of one sign order like their bit patterns
    return __uint_as_float(wave_umax(__float_as_uint(m)));
}

// max |v| over the whole chunk (every thread returns it).  Two barriers.
__device__ __forceinline__ float chunk_absmax(Shared& sh, const float (&v)[kRegs], uint32_t lane,
                                              uint32_t wave) {
    float m = wave_absmax(v);
    if (lane == 0) sh.red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(fmaxf(sh.red[0], sh.red[1]), fmaxf(sh.red[2], sh.red[3])),
              fmaxf(fmaxf(sh.red[4], sh.red[5]), fmaxf(sh.red[6], sh.red[7])));
    __syncthreads();
    return m;
}

// (min, max) of v over the whole chunk (every thread returns both).  Two barriers.
struct MinMax {
    float lo, hi;
};
__device__ __forceinline__ MinMax chunk_minmax(Shared& sh, const float (&v)[kRegs], uint32_t lane,
                                               uint32_t wave) {
    float lo = v[0], hi = v[0];
#pragma unroll
    for (int i = 1; i < kRegs; ++i) {
        lo = fminf(lo, v[i]);
        hi = fmaxf(hi, v[i]);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, o, 64));
        hi = fmaxf(hi, __shfl_xor(hi, o, 64));
    }
    float* red_lo = reinterpret_cast<float*>(sh.sign[1].sgn);   // second table: free in one-chunk kernels
    if (lane == 0) {
        sh.red[wave] = hi;
        red_lo[wave] = lo;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        hi = fmaxf(hi, sh.red[k]);
        lo = fminf(lo, red_lo[k]);
    }
    __syncthreads();
    return MinMax{lo, hi};
}

// (min, max) over this thread's registers.
__device__ __forceinline__ MinMax thread_minmax(const float (&v)[kRegs]) {
    float lo = v[0], hi = v[0];
#pragma unroll
    for (int i = 1; i < kRegs; ++i) {
        lo = fminf(lo, v[i]);
        hi = fmaxf(hi, v[i]);
    }
    return MinMax{lo, hi};
}

// Order-preserving map of floats onto unsigned words that are never zero for anything
// but a NaN (in the words workgroups exchange, zero means "not published yet"):
// x <= y  <=>  order_key(x) <= order_key(y).
__device__ __forceinline__ uint32_t order_key(float x) {
    const uint32_t b = __float_as_uint(x);
    const uint32_t k = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    return k != 0u ? k : 1u;
}
__device__ __forceinline__ float order_value(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

// L3 -> L4e through the buffer (two barriers); v then holds coordinates 32 t .. 32 t + 31.
template <bool PRIO>
__device__ __forceinline__ void l3_to_l4e(Shared& sh, float (&v)[kRegs], uint32_t lane, uint32_t wave) {
    __syncthreads();
    set_prio<PRIO, kPrioExchange>();
    x3e_store(sh, v, lane, wave);
    __syncthreads();
    x3e_load(sh, v, lane, wave);
    set_prio<PRIO, kPrioTail>();
}
// L3 -> L4d: v[4 h + e] is coordinate 2048 h + 4 t + e.
template <bool PRIO>
__device__ __forceinline__ void l3_to_l4d(Shared& sh, float (&v)[kRegs], uint32_t lane, uint32_t wave) {
    __syncthreads();
    set_prio<PRIO, kPrioExchange>();
    x3d_store(sh, v, lane, wave);
    __syncthreads();
    x3d_load(sh, v, lane, wave);
    set_prio<PRIO, kPrioTail>();
}

// --------------------------------------------------------------------- quantizer
// Stochastic rounding of the L4e-resident chunk onto a grid of L + 1 points, packed.
// v holds the UNNORMALISED rotation; y = v * 2^-7.  For one coordinate
//     c   = fma(float(r), 2^-8, base)          exact; r the coordinate's random byte
//     t   = fma(y - sub, mul, c)               ONE rounding (y - sub is rounded first when RANGED)
//     idx = floor(t)   (clamped to L when CLAMP)
// Symmetric grid on [-s, s]:  sub unused, mul = L / (2 s), base = L/2 + 2^-9, so that
//     t = y * inv + L/2 + (r + 0.5) / 256.
// Min/max grid on [lo, hi] (RANGED):  sub = lo, mul = L / (hi - lo), base = 2^-9.
//   g        global index of the thread's first coordinate
//   CLAMP    false only when the range is the chunk's own: the symmetric grid with s the
//            largest |y| of the chunk (then 0 < t < L + 1 for every coordinate: |y * inv| <=
//            L/2 (1 + 2^-24) and 2^-9 <= c - L/2 <= 255.5 / 256), or the min/max grid with
//            lo and hi the chunk's extremes (fl(y - lo) <= fl(hi - lo) = width, and width *
//            fl(L / width) <= L (1 + 2^-24), so t < L + 255.5/256 + L 2^-24 < L + 1); the
//            minimum with L never binds.  Both bounds need mul finite: the callers set mul = 0
//            for a range below kMinRange, which then gives t = c.  A range handed in by a
//            caller keeps the clamp.
//   FOLD     y = v * 2^-7 is not formed; mul already carries the factor 2^-7 and sub is given
//            in v's units (v - 2^7 lo = 2^7 (y - lo), rounded alike).  Exact as long
//            as the power of two moves nothing into the subnormal range or past the largest
//            float: the callers fold only for 2^-100 <= s <= 2^100.
// Packing: float -> integer conversion writes its result straight into one byte of a
// 32-bit register (sub-dword destination select), so 32 conversions leave 8 registers of 4
// index bytes each and no shift-or per coordinate; register m holds, in byte i, the index
// of coordinate (32 / BITS) * (m / kSub) ... chosen so that the payload word is
//     8 bits:  register d itself                         (bytes = coordinates 4d .. 4d+3)
//     4 bits:  A_d | B_d << 4                            (A: even, B: odd coordinates of 8d .. 8d+7)
//     2 bits:  R_d0 | R_d1 << 2 | R_d2 << 4 | R_d3 << 6  (R_dm byte i = coordinate 16d + 4i + m)
template <int BYTE, bool FIRST>
__device__ __forceinline__ void cvt_into_byte(uint32_t& acc, float tt) {
    static_assert(BYTE >= 0 && BYTE < 4, "byte index");
    if constexpr (FIRST) {   // writes the byte, zeroes the rest of the register
        if constexpr (BYTE == 0) asm("v_cvt_u32_f32_sdwa %0, %1 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:DWORD" : "=v"(acc) : "v"(tt));
        if constexpr (BYTE == 1) asm("v_cvt_u32_f32_sdwa %0, %1 dst_sel:BYTE_1 dst_unused:UNUSED_PAD src0_sel:DWORD" : "=v"(acc) : "v"(tt));
        if constexpr (BYTE == 2) asm("v_cvt_u32_f32_sdwa %0, %1 dst_sel:BYTE_2 dst_unused:UNUSED_PAD src0_sel:DWORD" : "=v"(acc) : "v"(tt));
        if constexpr (BYTE == 3) asm("v_cvt_u32_f32_sdwa %0, %1 dst_sel:BYTE_3 dst_unused:UNUSED_PAD src0_sel:DWORD" : "=v"(acc) : "v"(tt));
    } else {                 // writes the byte, keeps the rest
        if constexpr (BYTE == 0) asm("v_cvt_u32_f32_sdwa %0, %1 dst_sel:BYTE_0 dst_unused:UNUSED_PRESERVE src0_sel:DWORD" : "+v"(acc) : "v"(tt));
        if constexpr (BYTE == 1) asm("v_cvt_u32_f32_sdwa %0, %1 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD" : "+v"(acc) : "v"(tt));
        if constexpr (BYTE == 2) asm("v_cvt_u32_f32_sdwa %0, %1 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD" : "+v"(acc) : "v"(tt));
        if constexpr (BYTE == 3) asm("v_cvt_u32_f32_sdwa %0, %1 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD" : "+v"(acc) : "v"(tt));
    }
}

template <int BITS, bool CLAMP, bool FOLD, bool RANGED>
__device__ __forceinline__ void quantize_pack(const float (&v)[kRegs], float sub, float mul, float base,
                                              uint32_t L, uint64_t g, uint32_t worker, uint32_t key0,
                                              uint32_t key1, uint32_t (&pk)[BITS]) {
    constexpr int kSub = 8 / BITS;        // coordinates per payload byte: 1, 2, 4
    uint32_t by[8];                       // index bytes; by[m] serves payload word m / kSub
    const float Lf = (float)L;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const u32x4 rb = round_block((g >> 4) + half, worker, key0, key1);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int r = 16 * half + e;
            float y = FOLD ? v[r] : v[r] * kInvSqrtC;
            if (RANGED) y = y - sub;
            const uint32_t rnd = (rb.w[e >> 2] >> (8 * (e & 3))) & 0xFFu;
            const float c = __builtin_fmaf((float)rnd, 0x1p-8f, base);
            float tt = __builtin_fmaf(y, mul, c);            // tt >= 0: truncation = floor
            if (CLAMP) tt = fminf(tt, Lf);                   // floor(min(t, L)) = min(floor(t), L)
            // coordinate r sits in payload word d = r / (32 / BITS), at slot j = r % (32 / BITS);
            // its index goes to byte j / kSub of register kSub * d + j % kSub
            constexpr int kPerWord = 32 / BITS;
            const int d = r / kPerWord, j = r % kPerWord;
            const int m = kSub * d + j % kSub, byte = j / kSub;
            switch (byte) {
                case 0: cvt_into_byte<0, true>(by[m], tt); break;
                case 1: cvt_into_byte<1, false>(by[m], tt); break;
                case 2: cvt_into_byte<2, false>(by[m], tt); break;
                default: cvt_into_byte<3, false>(by[m], tt); break;
            }
        }
    }
#pragma unroll
    for (int d = 0; d < BITS; ++d) {
        if constexpr (BITS == 8) pk[d] = by[d];
        if constexpr (BITS == 4) pk[d] = by[2 * d] | (by[2 * d + 1] << 4);
        if constexpr (BITS == 2)
            pk[d] = by[4 * d] | (by[4 * d + 1] << 2) | (by[4 * d + 2] << 4) | (by[4 * d + 3] << 6);
    }
}

template <int BITS>
__device__ __forceinline__ void store_packed(const uint32_t (&pk)[BITS], uint8_t* dst) {
    if constexpr (BITS == 8) {
        reinterpret_cast<uint4*>(dst)[0] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        reinterpret_cast<uint4*>(dst)[1] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
    } else if constexpr (BITS == 4) {
        *reinterpret_cast<uint4*>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
    } else {
        *reinterpret_cast<uint2*>(dst) = make_uint2(pk[0], pk[1]);
    }
}

// Symmetric grid.  An all-zero chunk (s = 0; also one with 2 s < kMinRange) gets index 0 everywhere on the 2^BITS-point
// grid (L odd) and the centre index L/2 on the signed grid (L even).  Evaluation order by
// grid size (kSingleFmaMaxLevels): 2- and 4-bit grids t = fma(y, inv, L/2 + u); 8-bit
// grids t = fma(y + s, inv, u), which is the ranged form with sub = -s.  The clamp stays
// dead there too when s is the chunk's largest magnitude: 0 <= y + s <= 2 s, and
// 2 s * inv <= L (1 + 2^-24), so t < L + 255.5/256 + L 2^-24 < L + 1.
template <int BITS, bool CLAMP>
__device__ __forceinline__ void quantize_store(const float (&v)[kRegs], float s, uint32_t L, uint64_t g0,
                                               uint32_t worker, uint32_t key0, uint32_t key1,
                                               uint8_t* payload, uint32_t t) {
    constexpr bool kOffset = ((1u << BITS) - 2u) > kSingleFmaMaxLevels;   // both grids of this width
    const float two = s + s;
    const bool ranged = two >= kMinRange;   // false: an all-zero chunk, or one too small for L / two
    const float inv = ranged ? (float)L / two : 0.0f;
    const float centre = (ranged ? !kOffset : (L & 1u) == 0u) ? 0.5f * (float)L : 0.0f;
    const float base = centre + 0x1p-9f;   // exact
    const uint64_t g = g0 + (uint64_t)t * 32u;
    uint32_t pk[BITS];   // 32 coordinates * BITS bits = BITS dwords
    if (s >= 0x1p-100f && s <= 0x1p100f)   // the same for every thread of the workgroup
        quantize_pack<BITS, CLAMP, true, kOffset>(v, -128.0f * s, inv * kInvSqrtC, base, L, g, worker, key0, key1, pk);
    else
        quantize_pack<BITS, CLAMP, false, kOffset>(v, -s, inv, base, L, g, worker, key0, key1, pk);
    store_packed<BITS>(pk, payload + (g * BITS) / 8u);
}

// Min/max grid: idx = floor((y - lo) * inv + u), inv = L / (hi - lo) (0 for a constant chunk
// and for one narrower than kMinRange).
// ROTATED false: v holds y itself (the unrotated, zero-padded gradient), not 2^7 y.
template <int BITS, bool ROTATED = true, bool CLAMP = true>
__device__ __forceinline__ void quantize_store_range(const float (&v)[kRegs], float lo, float hi, uint32_t L,
                                                     uint64_t g0, uint32_t worker, uint32_t key0,
                                                     uint32_t key1, uint8_t* payload, uint32_t t) {
    const float width = hi - lo;
    const float inv = width >= kMinRange ? (float)L / width : 0.0f;
    const uint64_t g = g0 + (uint64_t)t * 32u;
    uint32_t pk[BITS];
    quantize_pack<BITS, CLAMP, !ROTATED, true>(v, lo, inv, 0x1p-9f, L, g, worker, key0, key1, pk);
    store_packed<BITS>(pk, payload + (g * BITS) / 8u);
}

// Output side of the inverse rotation: x = D (v * norm), norm = 2^-7, from layout L4d; the
// first `valid` coordinates of the chunk are stored.  (The first pass of a longer rotation
// passes norm = 1: its normalisation is one multiplication at the very end.)
template <bool SIGNED = true>
__device__ __forceinline__ void store_signed_l4d(const SignTable& tab, const float (&v)[kRegs], float* out,
                                                 uint32_t valid, uint32_t t, float norm = kInvSqrtC) {
#pragma unroll
    for (int h = 0; h < 8; ++h) {
        const uint32_t i0 = h * 2048u + t * 4u;
        const uint32_t sb = SIGNED ? tab.sgn[i0 >> 5] >> (i0 & 31u) : 0u;   // bits 0..3: signs of the 4 coordinates
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            x[e] = __uint_as_float(__float_as_uint(v[4 * h + e] * norm) ^ ((sb << (31 - e)) & 0x80000000u));
        if (i0 + 4u <= valid) {
            store_streaming(out + i0, x[0], x[1], x[2], x[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (i0 + e < valid) out[i0 + e] = x[e];
        }
    }
}

}  // namespace k14
}  // namespace thc
