// LDS address maps of the chunk-2^14 kernels (256 threads = 4 waves of 64 lanes, 64
// coordinates per thread).  i = 14-bit position inside the chunk, bits i0..i13.
//
// The rotation runs its 14 butterfly stages in stride order 1, 2, 4, ... as three
// register-resident groups; between groups the (lane, register) assignment of the
// chunk is re-shuffled through LDS:
//
//   layout L1  register = i0..i5,              lane = i6..i11, wave = i12..i13   (stages 0-5)
//   layout L2  register = i6..i11,             lane = i0..i5,  wave = i12..i13   (stages 6-11)
//   layout L3  register = i0..i3 + 16*(i12,i13), lane = i4..i9, wave = i10..i11  (stages 12-13)
//
// In L3 a thread owns four runs of 16 consecutive coordinates, which is what the
// quantizer (one Philox block per 16 coordinates), the bit-packer and the stores want.
//
// Every map below is a bijection of the index bits onto dword addresses, chosen so
// that the 128-bit side of an exchange has 8 consecutive lanes on 8 distinct 16-byte
// bank groups and the 32-bit side has 32 consecutive lanes on 32 distinct banks.  The
// XOR terms only involve low register bits, so a thread needs at most 8 base addresses
// per exchange and every access is base + immediate offset.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define THC_HD __host__ __device__ __forceinline__
#else
#define THC_HD inline
#endif

namespace thc {
namespace lay14 {

// ---- E0: raw input units (16 bytes each) from load order to L1 order -------------------
// Unit u = i / (coordinates per unit).  Load order: thread t, round j holds unit 256 j + t.
// L1 order: thread T needs units per*T .. per*T + per-1 (per = 8 for bf16, 16 for fp32).
// Unit u is kept at unit address u ^ ((u >> shift) & 7), shift = log2(per).
THC_HD uint32_t e0_store_unit(uint32_t t, uint32_t j, uint32_t shift) {
    return j * 256u + (t ^ ((t >> shift) & 7u));
}
THC_HD uint32_t e0_load_unit(uint32_t T, uint32_t k, uint32_t per) {
    return per * T + (k ^ (T & 7u));
}

// ---- X1: L1 -> L2, inside one wave's 4096-dword region ---------------------------------
// dword address of (i0..i11): (i6..i11) << 6 | (i0..i5) ^ ((i6..i8) << 2)
// writer (L1): lane = i6..i11 stores registers 4q..4q+3 as one 128-bit word
THC_HD uint32_t x1_store(uint32_t lane, uint32_t q) {  // q = 0..15
    return (lane << 6) | (((q & 7u) ^ (lane & 7u)) << 2) | ((q >> 3) << 5);
}
// reader (L2): lane = i0..i5 loads register r = i6..i11
THC_HD uint32_t x1_load(uint32_t lane, uint32_t r) {  // r = 0..63
    return (lane ^ ((r & 7u) << 2)) + (r << 6);
}

// ---- X2: L2 -> L3, whole 16384-dword buffer ----------------------------------------------
// address bits: a0 a1 = i6 i7 | a2 a3 a4 = i0^i4, i1^i5, i2^i8 | a5 = i3 | a6 a7 = i4 i5 |
//               a8 a9 a10 a11 = i8 i9 i10 i11 | a12 a13 = i12 i13
// writer (L2): wave = i12..i13, lane = i0..i5, stores registers 4q..4q+3 (r = i6..i11)
THC_HD uint32_t x2_store(uint32_t wave, uint32_t lane, uint32_t q) {  // q = 0..15 = i8..i11
    const uint32_t e8 = q & 1u;
    const uint32_t base = (((lane & 7u) ^ (((lane >> 4) & 3u) | (e8 << 2))) << 2) |
                          (((lane >> 3) & 7u) << 5) | (e8 << 8) | (wave << 12);
    return base + ((q >> 1) << 9);
}
// reader (L3): wave = i10..i11, lane = i4..i9, loads register e + 16 s (e = i0..i3, s = i12..i13)
THC_HD uint32_t x2_load(uint32_t wave, uint32_t lane, uint32_t e, uint32_t s) {
    const uint32_t k = e & 7u;
    const uint32_t base = ((lane >> 2) & 3u) |
                          ((k ^ ((lane & 3u) | (((lane >> 4) & 1u) << 2))) << 2) |
                          ((lane & 3u) << 6) | (((lane >> 4) & 3u) << 8) | (wave << 10);
    return base + ((e >> 3) << 5) + (s << 12);
}

}  // namespace lay14
}  // namespace thc
