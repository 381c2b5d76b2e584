// Tuned kernels for chunk_log2 = 14 (the chunk size of every large workload): one
// workgroup of 512 threads per chunk, the chunk lives in registers (32 coordinates per
// thread) and is re-shuffled through LDS between groups of butterfly stages, see
// thc_core14.h.  Used when every pointer is 16-byte aligned; the generic kernels cover
// everything else with identical results.
#include "thc_core14.h"
#include "thc_internal.h"

#pragma clang fp contract(off)

namespace thc {
namespace k14 {
namespace {

// One chunk per workgroup, gradient of ONE worker: rotation / range / encode.
//   BF16   input type;  MODE  Forward | Absmax | Encode;  BITS payload width (Encode)
template <bool BF16, Mode MODE, int BITS>
__global__ __launch_bounds__(kThreads) void per_worker_kernel(const ChunkArgs a) {
    __shared__ Shared sh;
    constexpr int kUnits = BF16 ? 4 : 8;
    constexpr int kElem = BF16 ? 2 : 4;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint64_t p = blockIdx.x;
    const uint64_t g0 = p << kChunkLog2;
    const uint64_t left = a.n - g0;
    const uint32_t valid = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;

    Raw<kUnits> raw;
    load_raw<kUnits, kElem>(raw, static_cast<const uint8_t*>(a.in) + g0 * kElem, valid, t);
    fill_sign_table<!BF16, BF16>(sh.sign[0], g0, a.key0, a.key1, t);
    raw_to_lds<kUnits>(sh, raw, t);
    __syncthreads();
    float v[kRegs];
    lds_to_l1<kUnits, true>(sh, sh.sign[0], v, t);
    rotate_l1_to_l3<false>(sh, v, lane, wave);

    if constexpr (MODE == Mode::Forward) {
        l3_to_l4d<false>(sh, v, lane, wave);
        float* y = static_cast<float*>(a.out) + g0;
#pragma unroll
        for (int h = 0; h < 8; ++h)
            *reinterpret_cast<float4*>(y + h * 2048 + t * 4) =
                make_float4(v[4 * h] * a.inv_sqrt_c, v[4 * h + 1] * a.inv_sqrt_c, v[4 * h + 2] * a.inv_sqrt_c,
                            v[4 * h + 3] * a.inv_sqrt_c);   // 2^-7, or 1 as the first pass of a longer rotation
    } else if constexpr (MODE == Mode::Absmax) {
        const float m = chunk_absmax(sh, v, lane, wave) * kInvSqrtC;
        if (t == 0) static_cast<float*>(a.out)[p] = m;
    } else if constexpr (MODE == Mode::MinMax) {
        const MinMax r = chunk_minmax(sh, v, lane, wave);
        if (t == 0) {
            static_cast<float*>(a.out)[2 * p] = r.lo * kInvSqrtC;
            static_cast<float*>(a.out)[2 * p + 1] = r.hi * kInvSqrtC;
        }
    } else if (a.range_in) {   // Encode on the min/max grid
        const float lo = a.range_in[2 * p], hi = a.range_in[2 * p + 1];
        l3_to_l4e<false>(sh, v, lane, wave);
        quantize_store_range<BITS>(v, lo, hi, a.levels, g0, a.worker, a.key0, a.key1,
                                   static_cast<uint8_t*>(a.out), t);
    } else {
        float s;
        if (a.scale_in) {
            s = a.scale_in[p];
        } else {
            s = chunk_absmax(sh, v, lane, wave) * kInvSqrtC;
        }
        if (a.scale_out && t == 0) a.scale_out[p] = s;
        l3_to_l4e<false>(sh, v, lane, wave);
        quantize_store<BITS, true>(v, s, a.levels, g0, a.worker, a.key0, a.key1, static_cast<uint8_t*>(a.out), t);
    }
}

// The "no rotation" arm of the min/max variant: y is the zero-padded gradient itself, so a
// chunk needs no exchange at all.  Thread t loads its 32 consecutive coordinates, and
// either the workgroup reduces them to (min, max) or the thread quantizes them onto the
// given range and stores its 4 * BITS payload bytes.
template <bool BF16, Mode MODE, int BITS>
__global__ __launch_bounds__(kThreads) void unrotated_kernel(const ChunkArgs a) {
    __shared__ Shared sh;
    constexpr int kUnits = BF16 ? 4 : 8;
    constexpr int kElem = BF16 ? 2 : 4;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint64_t p = blockIdx.x;
    const uint64_t g0 = p << kChunkLog2;
    const uint64_t left = a.n - g0;
    const uint32_t valid = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
    Raw<kUnits> raw;
    load_raw<kUnits, kElem, true>(raw, static_cast<const uint8_t*>(a.in) + g0 * kElem, valid, t);
    float v[kRegs];
    units_to_l1<kUnits, false>(sh.sign[0], raw.u, v, t);
    if constexpr (MODE == Mode::MinMax) {
        const MinMax r = chunk_minmax(sh, v, lane, wave);
        if (t == 0) {
            static_cast<float*>(a.out)[2 * p] = r.lo;
            static_cast<float*>(a.out)[2 * p + 1] = r.hi;
        }
    } else {
        const float lo = a.range_in[2 * p], hi = a.range_in[2 * p + 1];
        quantize_store_range<BITS, false>(v, lo, hi, a.levels, g0, a.worker, a.key0, a.key1,
                                          static_cast<uint8_t*>(a.out), t);
    }
}

// Inverse direction, one chunk per workgroup.
//   SRC 0: rotated fp32 values (rht_inverse);  1: u8 sums;  2: u16 sums (thc_decode);
//       3: packed saturated aggregate, offset binary (thc_sat_decode)
//   SIGNED false: no sign diagonal on output (a pass of the full rotation)
template <int SRC, bool SIGNED = true>
__global__ __launch_bounds__(kThreads) void inverse_kernel(const ChunkArgs a) {
    __shared__ Shared sh;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint64_t p = blockIdx.x;
    const uint64_t g0 = p << kChunkLog2;
    const uint64_t left = a.n - g0;
    const uint32_t valid = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
    float v[kRegs];
    if (SIGNED) fill_sign_table<true, false>(sh.sign[0], g0, a.key0, a.key1, t);
    if constexpr (SRC == 0) {
        Raw<8> raw;   // y is complete (padded), so every unit exists
        load_raw<8, 4>(raw, static_cast<const float*>(a.in) + g0, (uint32_t)kChunk, t);
        raw_to_lds<8>(sh, raw, t);
        __syncthreads();
        lds_to_l1<8, false>(sh, sh.sign[0], v, t);
    } else {
        // symmetric grid: yhat = S q - s;  min/max grid: yhat = S q + lo
        const bool ranged = a.range_in != nullptr;
        const float lo = ranged ? a.range_in[2 * p] : 0.0f;
        const float s = ranged ? -lo : a.scale_in[a.scale_shared ? 0 : p];
        const float step = (ranged ? a.range_in[2 * p + 1] - lo : s + s) / (float)a.levels;
        const float q = step / (float)a.W;
        if constexpr (SRC == 3) {
            // 32 coordinates = 4 * bits bytes per thread
            const uint32_t bits = a.bits;
            const uint32_t* src = reinterpret_cast<const uint32_t*>(
                static_cast<const uint8_t*>(a.in) + (g0 * bits) / 8u + (uint64_t)t * (4u * bits));
            const int centre = (int)(a.levels >> 1);
            uint32_t word[8];
#pragma unroll
            for (int d = 0; d < 8; ++d) word[d] = (uint32_t)d < bits ? src[d] : 0u;
#pragma unroll
            for (int r = 0; r < kRegs; ++r) {
                uint32_t A;
                if (bits == 2) A = (word[r >> 4] >> (2 * (r & 15))) & 3u;
                else if (bits == 4) A = (word[r >> 3] >> (4 * (r & 7))) & 15u;
                else A = (word[r >> 2] >> (8 * (r & 3))) & 255u;
                v[r] = (float)((int)A - centre) * q;
            }
        } else if constexpr (SRC == 1) {
            const uint4* src = reinterpret_cast<const uint4*>(static_cast<const uint8_t*>(a.in) + g0) + 2 * t;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const uint4 w = src[k];
                const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int d = 0; d < 4; ++d)
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        v[16 * k + 4 * d + b] = (float)((ww[d] >> (8 * b)) & 0xFFu) * q - s;
            }
        } else {
            const uint4* src = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(a.in) + g0) + 4 * t;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint4 w = src[k];
                const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int d = 0; d < 4; ++d)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        v[8 * k + 2 * d + b] = (float)((ww[d] >> (16 * b)) & 0xFFFFu) * q - s;
            }
        }
    }
    rotate_l1_to_l3<false>(sh, v, lane, wave);
    l3_to_l4d<false>(sh, v, lane, wave);
    store_signed_l4d<SIGNED>(sh.sign[0], v, static_cast<float*>(a.out) + g0, valid, t, a.inv_sqrt_c);
}

template <bool BF16, Mode MODE>
hipError_t launch_bits(const ChunkArgs& a, dim3 grid, hipStream_t stream) {
    if constexpr (MODE == Mode::Encode) {
        if (a.bits == 2)
            hipLaunchKernelGGL((per_worker_kernel<BF16, MODE, 2>), grid, dim3(kThreads), 0, stream, a);
        else if (a.bits == 4)
            hipLaunchKernelGGL((per_worker_kernel<BF16, MODE, 4>), grid, dim3(kThreads), 0, stream, a);
        else
            hipLaunchKernelGGL((per_worker_kernel<BF16, MODE, 8>), grid, dim3(kThreads), 0, stream, a);
    } else {
        hipLaunchKernelGGL((per_worker_kernel<BF16, MODE, 4>), grid, dim3(kThreads), 0, stream, a);
    }
    return hipGetLastError();
}

template <bool BF16>
hipError_t launch_unrotated(Mode mode, const ChunkArgs& a, dim3 grid, hipStream_t stream) {
    if (mode == Mode::MinMax)
        hipLaunchKernelGGL((unrotated_kernel<BF16, Mode::MinMax, 4>), grid, dim3(kThreads), 0, stream, a);
    else if (a.bits == 2)
        hipLaunchKernelGGL((unrotated_kernel<BF16, Mode::Encode, 2>), grid, dim3(kThreads), 0, stream, a);
    else if (a.bits == 4)
        hipLaunchKernelGGL((unrotated_kernel<BF16, Mode::Encode, 4>), grid, dim3(kThreads), 0, stream, a);
    else
        hipLaunchKernelGGL((unrotated_kernel<BF16, Mode::Encode, 8>), grid, dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace
}  // namespace k14

bool fast14_applicable(Mode mode, const ChunkArgs& a) {
    if (a.chunk_log2 != 14) return false;
    if ((a.padded >> 14) > 0x7FFFFFFFull) return false;
    if (a.out_bf16 || mode == Mode::Plain || mode == Mode::PlainDecode) return false;
    // without the rotation: the range and the encoder on a given range have a tuned form
    if (a.no_rotate && !(mode == Mode::MinMax || (mode == Mode::Encode && a.range_in))) return false;
    return k14::aligned16(a.in) && k14::aligned16(a.out);
}

hipError_t launch_fast14(Mode mode, const ChunkArgs& a, hipStream_t stream) {
    using namespace k14;
    const dim3 grid((uint32_t)(a.padded >> 14));
    if (grid.x == 0) return hipSuccess;
    if (a.no_rotate)
        return a.in_bf16 ? launch_unrotated<true>(mode, a, grid, stream) : launch_unrotated<false>(mode, a, grid, stream);
    switch (mode) {
        case Mode::Forward:
            return a.in_bf16 ? launch_bits<true, Mode::Forward>(a, grid, stream)
                             : launch_bits<false, Mode::Forward>(a, grid, stream);
        case Mode::Absmax:
            return a.in_bf16 ? launch_bits<true, Mode::Absmax>(a, grid, stream)
                             : launch_bits<false, Mode::Absmax>(a, grid, stream);
        case Mode::MinMax:
            return a.in_bf16 ? launch_bits<true, Mode::MinMax>(a, grid, stream)
                             : launch_bits<false, Mode::MinMax>(a, grid, stream);
        case Mode::Encode:
            return a.in_bf16 ? launch_bits<true, Mode::Encode>(a, grid, stream)
                             : launch_bits<false, Mode::Encode>(a, grid, stream);
        case Mode::Inverse:
            hipLaunchKernelGGL(inverse_kernel<0>, grid, dim3(kThreads), 0, stream, a);
            return hipGetLastError();
        case Mode::Plain:
            hipLaunchKernelGGL((inverse_kernel<0, false>), grid, dim3(kThreads), 0, stream, a);
            return hipGetLastError();
        case Mode::PlainDecode:
            if (a.sum_bytes == 1)
                hipLaunchKernelGGL((inverse_kernel<1, false>), grid, dim3(kThreads), 0, stream, a);
            else
                hipLaunchKernelGGL((inverse_kernel<2, false>), grid, dim3(kThreads), 0, stream, a);
            return hipGetLastError();
        case Mode::Decode:
            if (a.sat)
                hipLaunchKernelGGL(inverse_kernel<3>, grid, dim3(kThreads), 0, stream, a);
            else if (a.sum_bytes == 1)
                hipLaunchKernelGGL(inverse_kernel<1>, grid, dim3(kThreads), 0, stream, a);
            else
                hipLaunchKernelGGL(inverse_kernel<2>, grid, dim3(kThreads), 0, stream, a);
            return hipGetLastError();
    }
    return hipErrorInvalidValue;
}

}  // namespace thc
