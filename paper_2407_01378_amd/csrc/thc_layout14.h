// LDS address maps of the chunk-2^14 kernels: 512 threads = 8 waves of 64 lanes, 32
// coordinates per thread.  i = 14-bit position inside the chunk, bits i0..i13.
//
// The rotation runs its 14 butterfly stages in stride order 1, 2, 4, ... as three
// register-resident groups (5 + 5 + 4 stages); between groups, and once more at the
// end, the (wave, lane, register) assignment of the chunk is re-shuffled through LDS:
//
//   L1   register = i0..i4        lane = i5..i10               wave = i11..i13   stages 0-4
//   L2   register = i5..i9        lane = i0..i4, i10           wave = i11..i13   stages 5-9
//   L3   register = i9, i10..i13  lane = i5, i6, i0, i1, i2, i3  wave = i4, i7, i8   stages 10-13
//   L4e  = L1: 32 consecutive coordinates per thread (quantize, pack, 16-byte payload store)
//   L4d  register = i0, i1, i11..i13   lane = i2..i7   wave = i8..i10   (coalesced fp32 store)
//
// Eight waves per chunk keep four waves resident per SIMD with two chunks per CU in
// flight (LDS holds one 64 KB chunk per workgroup), so that one chunk's LDS exchanges and
// barriers overlap the other's vector arithmetic.
//
// Every map is a bijection of the index bits onto dword addresses such that, as measured on
// gfx950 (timings and the bank-conflict counter of ds_read / ds_write with GF(2)-linear
// functions of the lane index as addresses): 32-bit accesses put the 32 lanes of each half
// wave on 32 distinct banks (dword address mod 32); 128-bit stores put 8 consecutive lanes on
// the 8 distinct 16-byte columns of a 128-byte row; 128-bit loads run at twice the bandwidth
// of 32-bit ones, 16 lanes a clock: the lanes of a half wave whose bits 2, 3 and 4 have the
// same parity are served together and must sit on the 16 distinct columns of a 256-byte row.
// XOR terms involve at most three register bits, so a thread needs at most 8 base addresses
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
// Load order: thread t (0..511), round j holds unit 512 j + t.  L1 order: thread T needs
// units per*T .. per*T + per-1 (per = 4 for bf16: 8 coordinates a unit; 8 for fp32: 4 a unit).
// Unit u is kept at unit address u ^ swz(u): bf16 swz = (u >> 4) & 3, fp32 swz = (u >> 4) & 7
// (a half wave of readers then covers all 16 columns of a 256-byte row: columns
// 4 (T & 3) + (k ^ (T >> 2 & 3)) for bf16, 8 (T & 1) + (k ^ (T >> 1 & 7)) for fp32).
THC_HD uint32_t e0_store_unit(uint32_t t, uint32_t j, uint32_t per) {
    const uint32_t swz = per == 4 ? ((t >> 4) & 3u) : ((t >> 4) & 7u);
    return j * 512u + (t ^ swz);
}
THC_HD uint32_t e0_load_unit(uint32_t T, uint32_t k, uint32_t per) {
    const uint32_t swz = per == 4 ? ((T >> 2) & 3u) : ((T >> 1) & 7u);
    return per * T + (k ^ swz);
}

// ---- X1: L1 -> L2, inside one wave's 2048-dword region ----------------------------------
// dword address of (i0..i10): a0 a1 = i0 i1 | a2 a3 a4 = i2^i5, i3^i6, i4^i7 | a5..a10 = i5..i10
// writer (L1): lane = i5..i10 stores registers 4q..4q+3 (q = i2..i4) as one 128-bit word
THC_HD uint32_t x1_store(uint32_t lane, uint32_t q) {  // q = 0..7
    return (lane << 5) | ((q ^ (lane & 7u)) << 2);
}
// reader (L2): lane = (i0..i4, i10) loads register r = i5..i9
THC_HD uint32_t x1_load(uint32_t lane, uint32_t r) {  // r = 0..31
    const uint32_t low = lane & 31u;                 // i0..i4
    return (low ^ ((r & 7u) << 2)) | (r << 5) | ((lane >> 5) << 10);
}

// ---- X2: L2 -> L3, whole 16384-dword buffer, no XOR needed -------------------------------
// a0 a1 = i5 i6 | a2..a6 = i0..i4 | a7 a8 = i7 i8 | a9..a13 = i9..i13
// writer (L2): wave = i11..i13, lane = (i0..i4, i10), stores registers 4q..4q+3, q = (i7,i8,i9)
THC_HD uint32_t x2_store(uint32_t wave, uint32_t lane, uint32_t q) {  // q = 0..7
    return ((lane & 31u) << 2) | ((lane >> 5) << 10) | (wave << 11) | ((q & 3u) << 7) | ((q >> 2) << 9);
}
// reader (L3): wave = (i4,i7,i8), lane = (i5,i6,i0,i1,i2,i3), loads register rho = (i9..i13)
THC_HD uint32_t x2_load(uint32_t wave, uint32_t lane, uint32_t rho) {  // rho = 0..31
    return ((lane & 3u) | (((lane >> 2) & 15u) << 2) | ((wave & 1u) << 6) | ((wave >> 1) << 7)) + (rho << 9);
}

// ---- X3e: L3 -> L4e (= L1), whole buffer ---------------------------------------------------
// a0 a1 = i0 i1 | a2 a3 = i5 i6 | a4 = i2^i7 | a5 = i8 | a6 = i4 | a7 = i7 | a8 = i3 | a9..a13 = i9..i13
// The readers' 16 lanes that are served together differ in i5, i6 and in (i7, i8, i9) of one
// parity: their columns (a2..a5) = (i5, i6, i2^i7, i8) are all different.
// writer (L3): 32-bit stores of register rho
THC_HD uint32_t x3e_store(uint32_t wave, uint32_t lane, uint32_t rho) {
    const uint32_t i5i6 = lane & 3u, i0i1 = (lane >> 2) & 3u, i2 = (lane >> 4) & 1u, i3 = (lane >> 5) & 1u;
    const uint32_t i4 = wave & 1u, i7 = (wave >> 1) & 1u, i8 = (wave >> 2) & 1u;
    return (i0i1 | (i5i6 << 2) | ((i2 ^ i7) << 4) | (i8 << 5) | (i4 << 6) | (i7 << 7) | (i3 << 8)) + (rho << 9);
}
// reader (L4e): wave = i11..i13, lane = i5..i10, loads registers 4q..4q+3 (q = i2..i4) as 128 bits;
// returns the index of the 16-byte unit
THC_HD uint32_t x3e_load_unit(uint32_t wave, uint32_t lane, uint32_t q) {  // q = 0..7
    const uint32_t i5i6 = lane & 3u, i7 = (lane >> 2) & 1u, i8 = (lane >> 3) & 1u, i9i10 = lane >> 4;
    const uint32_t i2 = q & 1u, i3 = (q >> 1) & 1u, i4 = q >> 2;
    return i5i6 | ((i2 ^ i7) << 2) | (i8 << 3) | (i4 << 4) | (i7 << 5) | (i3 << 6) | (i9i10 << 7) | (wave << 9);
}
THC_HD uint32_t x3e_load(uint32_t wave, uint32_t lane, uint32_t q) { return x3e_load_unit(wave, lane, q) << 2; }

// ---- X3d: L3 -> L4d, whole buffer ----------------------------------------------------------
// a0 a1 = i0 i1 | a2 = i2 | a3 = i3^i5 | a4 = i4^i6 | a5 = i4 | a6 = i5 | a7 a8 = i7 i8 | a9..a13 = i9..i13
// The readers' 16 lanes that are served together differ in i2, i3 and in (i4, i5, i6) of one
// parity; their columns (a2..a5) = (i2, i3^i5, i5^parity, i4) are all different.
THC_HD uint32_t x3d_store(uint32_t wave, uint32_t lane, uint32_t rho) {
    const uint32_t i5 = lane & 1u, i6 = (lane >> 1) & 1u, i0i1 = (lane >> 2) & 3u, i2 = (lane >> 4) & 1u,
                   i3 = (lane >> 5) & 1u;
    const uint32_t i4 = wave & 1u, i7i8 = wave >> 1;
    return (i0i1 | (i2 << 2) | ((i3 ^ i5) << 3) | ((i4 ^ i6) << 4) | (i4 << 5) | (i5 << 6) | (i7i8 << 7)) + (rho << 9);
}
// reader (L4d): wave = i8..i10, lane = i2..i7, loads registers (i0,i1) of group h = (i11..i13) as 128 bits;
// returns the index of the 16-byte unit
THC_HD uint32_t x3d_load_unit(uint32_t wave, uint32_t lane, uint32_t h) {  // h = 0..7
    const uint32_t i2 = lane & 1u, i3 = (lane >> 1) & 1u, i4 = (lane >> 2) & 1u, i5 = (lane >> 3) & 1u,
                   i6 = (lane >> 4) & 1u, i7 = (lane >> 5) & 1u;
    const uint32_t i8 = wave & 1u, i9i10 = wave >> 1;
    return i2 | ((i3 ^ i5) << 1) | ((i4 ^ i6) << 2) | (i4 << 3) | (i5 << 4) | (i7 << 5) | (i8 << 6) |
           (i9i10 << 7) | (h << 9);
}
THC_HD uint32_t x3d_load(uint32_t wave, uint32_t lane, uint32_t h) { return x3d_load_unit(wave, lane, h) << 2; }

}  // namespace lay14
}  // namespace thc
