// Full rotation (l' = l): the Hadamard transform of a whole gradient padded to 2^l
// coordinates, l > 14, as the paper's baseline for the partial rotation.  Stages run in
// the same order as everywhere else (stride 1, 2, 4, ..., 2^(l-1), every stage one
// separately rounded fp32 add and subtract), so results are bit-identical to the
// stage-by-stage definition:
//   stages 0..13    the chunk-2^14 kernels (thc_fast14.hip), data in registers and LDS
//   stages 14..l-1  "high passes" over the fp32 array in global memory, up to 9 stages per
//                   pass (this file), in place
// plus the elementwise steps of the quantizer on rotated data (range, encode, decode),
// which the partial-rotation path fuses into its rotation kernels.
#include "thc_device.h"
#include "thc_internal.h"

#pragma clang fp contract(off)

namespace thc {
namespace {

constexpr int kThreads = 512;
constexpr int kTileLog2 = 14;   // coordinates per workgroup

// One pass over stages [s0, s0 + m), 1 <= m <= 9, s0 >= 14.  A tile is 512 "rows" of 32
// consecutive floats; row bit b (b = 0..8) is stage s0 + b - skip for b >= skip = 9 - m
// and an extension of the column index below that (no butterfly), so that short passes
// still move whole 128-byte lines.  A thread holds 8 rows x 4 consecutive floats; the
// three row-bit triples take turns in the registers, with one wave-local and one
// cross-wave exchange through LDS in 16-byte units (8 consecutive lanes = 128 bytes).
struct HighPassArgs {
    float* data;        // 2^l floats, transformed in place (unless `out`)
    float* out;         // last pass of the inverse: x (n floats); else null
    uint64_t n;         // coordinates to write to `out`
    uint32_t s0, m;
    uint32_t last;      // 1: multiply by `factor`
    float factor;
    uint32_t key0, key1;
    uint64_t valid;     // floats of `data` that hold values; what lies beyond reads as zero and
                        // is neither read nor, in a pass that is not the last, written (the zero
                        // padding behind the gradient is implied, pass after pass, until the
                        // last pass mixes it with everything)
    uint32_t* absmax;   // last forward pass: receives max |value written| by an unsigned atomic
                        // maximum (zeroed beforehand); may be null
};

__device__ __forceinline__ void row_butterflies(float (&v)[32], int bit, bool enabled) {
    if (!enabled) return;   // uniform over the grid
    const int h = 1 << bit;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        if ((r & h) == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = v[4 * r + e], hi = v[4 * (r + h) + e];
                v[4 * r + e] = lo + hi;
                v[4 * (r + h) + e] = lo - hi;
            }
        }
    }
}

template <bool TO_X>
__global__ __launch_bounds__(kThreads) void high_pass_kernel(const HighPassArgs a) {
    __shared__ float4 xb[4096];
    const uint32_t t = threadIdx.x, lane = t & 63u, w = t >> 6;
    const uint32_t jq = lane & 7u, la = lane >> 3;
    const uint32_t skip = 9u - a.m;
    const uint32_t jb_bits = a.s0 - 5u - skip;                  // column blocks per 2^s0 run
    const uint64_t tile = blockIdx.x;
    const uint64_t jb = tile & ((1ull << jb_bits) - 1ull);
    const uint64_t hi = tile >> jb_bits;
    // a tile mixes values of one block of 2^(s0 + m) floats: if that block lies in the implied
    // zero padding its results are zero too, and the next pass is told so instead of reading them
    if ((hi << (a.s0 + a.m)) >= a.valid) return;
    const uint64_t base = (hi << (a.s0 + a.m)) + (jb << (5u + skip));
    auto offset = [&](uint32_t row) -> uint64_t {               // first float of (row, jq)
        const uint64_t k = row >> skip;
        const uint32_t jext = row & ((1u << skip) - 1u);
        return base + (k << a.s0) + (uint64_t)(jext * 32u + 4u * jq);
    };

    float v[32];
    // rows r + 8 la + 64 w
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        // (the load is unconditional, from the array's start where the row lies in the implied
        // padding, so that the eight loads stay back to back; the select comes afterwards)
        const uint64_t g = offset(r + 8u * la + 64u * w);   // a multiple of 4, as `valid` is
        const bool in = g < a.valid;
        const float4 q = *reinterpret_cast<const float4*>(a.data + (in ? g : 0u));
        v[4 * r] = in ? q.x : 0.0f;
        v[4 * r + 1] = in ? q.y : 0.0f;
        v[4 * r + 2] = in ? q.z : 0.0f;
        v[4 * r + 3] = in ? q.w : 0.0f;
    }
#pragma unroll
    for (int b = 0; b < 3; ++b) row_butterflies(v, b, (uint32_t)b >= skip);

    // exchange 1, inside the wave's own 512 units: registers <-> lane bits 3..5
    float4* mine = xb + 512u * w;
#pragma unroll
    for (int r = 0; r < 8; ++r)
        mine[(r + 8u * la) * 8u + jq] = make_float4(v[4 * r], v[4 * r + 1], v[4 * r + 2], v[4 * r + 3]);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
    for (int r = 0; r < 8; ++r) {   // now: row = la + 8 r + 64 w
        const float4 q = mine[(la + 8u * r) * 8u + jq];
        v[4 * r] = q.x;
        v[4 * r + 1] = q.y;
        v[4 * r + 2] = q.z;
        v[4 * r + 3] = q.w;
    }
#pragma unroll
    for (int b = 0; b < 3; ++b) row_butterflies(v, b, (uint32_t)(3 + b) >= skip);

    // exchange 2, across waves: registers <-> wave index
#pragma unroll
    for (int r = 0; r < 8; ++r)
        mine[(la + 8u * r) * 8u + jq] = make_float4(v[4 * r], v[4 * r + 1], v[4 * r + 2], v[4 * r + 3]);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 8; ++r) {   // now: row = la + 8 w + 64 r
        const float4 q = xb[512u * r + (la + 8u * w) * 8u + jq];
        v[4 * r] = q.x;
        v[4 * r + 1] = q.y;
        v[4 * r + 2] = q.z;
        v[4 * r + 3] = q.w;
    }
#pragma unroll
    for (int b = 0; b < 3; ++b) row_butterflies(v, b, (uint32_t)(6 + b) >= skip);

    float largest = 0.0f;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const uint64_t g = offset(la + 8u * w + 64u * (uint32_t)r);
        float o[4] = {v[4 * r], v[4 * r + 1], v[4 * r + 2], v[4 * r + 3]};
        if (a.last) {
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = o[e] * a.factor;
        }
        if (!TO_X) largest = fmaxf(fmaxf(largest, fmaxf(fabsf(o[0]), fabsf(o[1]))), fmaxf(fabsf(o[2]), fabsf(o[3])));
        if constexpr (TO_X) {
            if (g < a.n) {
                const u32x4 sb = sign_block(g >> 7, a.key0, a.key1);
                const uint32_t bits4 = sb.w[(g >> 5) & 3u] >> (g & 31u);   // g is a multiple of 4
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = flip_sign(o[e], (bits4 >> e) & 1u);
                if (g + 4u <= a.n) {
                    *reinterpret_cast<float4*>(a.out + g) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (g + e < a.n) a.out[g + e] = o[e];
                }
            }
        } else {
            *reinterpret_cast<float4*>(a.data + g) = make_float4(o[0], o[1], o[2], o[3]);
        }
    }
    if (!TO_X && a.absmax) {   // (uniform over the grid) non-negative floats order like their bit patterns
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) largest = fmaxf(largest, __shfl_xor(largest, o, 64));
        // (a stale read only costs an atomic more; most workgroups stay below the running maximum)
        if (lane == 0 && __float_as_uint(largest) > __hip_atomic_load(a.absmax, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
            atomicMax(a.absmax, __float_as_uint(largest));
    }
}

// ---- elementwise steps on rotated data ---------------------------------------------------
// Largest |y| of the whole array into *absmax (zeroed beforehand): non-negative floats
// order like their bit patterns, so an unsigned atomic max does it.
__global__ __launch_bounds__(256) void full_absmax_kernel(const float* y, uint64_t count, uint32_t* absmax) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x * 4u;
    float m = 0.0f;
    for (uint64_t i = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4u; i < count; i += stride) {
        const float4 q = *reinterpret_cast<const float4*>(y + i);
        m = fmaxf(fmaxf(m, fmaxf(fabsf(q.x), fabsf(q.y))), fmaxf(fabsf(q.z), fabsf(q.w)));
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
    if ((threadIdx.x & 63u) == 0) atomicMax(absmax, __float_as_uint(m));
}

// Stochastic rounding of rotated values (already normalised) onto the grid of [-s, s]:
// same arithmetic and random stream as the fused encoders.  One thread: 16 coordinates,
// one Philox block, 2 * BITS payload bytes.
template <int BITS>
__global__ __launch_bounds__(256) void full_encode_kernel(const float* y, uint64_t count, const float* scale,
                                                          uint32_t levels, uint32_t worker, uint32_t key0,
                                                          uint32_t key1, uint8_t* payload) {
    const uint64_t blk = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t g0 = blk * 16u;
    if (g0 >= count) return;
    const float s = scale[0];
    const float two = s + s;
    const float Lf = (float)levels;
    const bool ranged = two >= kMinRange;
    const float inv = ranged ? Lf / two : 0.0f;
    const bool single = levels <= kSingleFmaMaxLevels;   // evaluation order by grid size
    const float half = (single && ranged) ? 0.5f * Lf : 0.0f;   // an all-zero (or vanishingly small) vector gets index 0
    const float off = single ? 0.0f : s;
    const u32x4 rb = round_block(blk, worker, key0, key1);
    uint32_t pk[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float4 q = *reinterpret_cast<const float4*>(y + g0 + 4 * k);
        const float yv[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = 4 * k + e;
            const uint32_t r = (rb.w[k] >> (8 * e)) & 0xFFu;
            const float u = ((float)r + 0.5f) * (1.0f / 256.0f);
            // small grids: fma(y, inv, L/2 + u); large grids: fma(y + s, inv, u)
            const float tt = __builtin_fmaf(yv[e] + off, inv, half + u);
            const uint32_t idx = (uint32_t)fminf(floorf(tt), Lf);
            const int bit = j * BITS;
            pk[bit >> 5] |= idx << (bit & 31);
        }
    }
    uint8_t* dst = payload + blk * (2u * BITS);
    if constexpr (BITS == 8) {
        *reinterpret_cast<uint4*>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
    } else if constexpr (BITS == 4) {
        *reinterpret_cast<uint2*>(dst) = make_uint2(pk[0], pk[1]);
    } else {
        *reinterpret_cast<uint32_t*>(dst) = pk[0];
    }
}

// sums -> rotated-domain estimate of the mean: yhat = S * (step / W) - s.
template <typename SumT>
__global__ __launch_bounds__(256) void full_decode_kernel(const SumT* sums, uint64_t count, const float* scale,
                                                          uint32_t levels, uint32_t W, float* yhat) {
    const uint64_t g0 = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4u;
    if (g0 >= count) return;
    const float s = scale[0];
    const float step = (s + s) / (float)levels;
    const float q = step / (float)W;
    float o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (float)(uint32_t)sums[g0 + e] * q - s;
    *reinterpret_cast<float4*>(yhat + g0) = make_float4(o[0], o[1], o[2], o[3]);
}

}  // namespace

// Stages 14 .. l-1 on data (2^l floats, stages 0..13 already done), in place; the last pass
// multiplies by `factor`, and for the inverse direction (`x` non-null) applies the sign
// diagonal and writes the first n coordinates to x instead.  Forward direction: only the
// first `valid` floats of data have been written (the rest is the zero padding, which the
// first pass supplies by itself), and `absmax`, if not null, receives the largest
// magnitude of the result (the word is zeroed here first).
hipError_t launch_high_passes(float* data, uint32_t log2_size, float factor, float* x, uint64_t n,
                              uint32_t key0, uint32_t key1, hipStream_t stream, uint64_t valid,
                              float* absmax) {
    if (absmax) {
        const hipError_t e = launch_zero_words(reinterpret_cast<uint32_t*>(absmax), 1, stream);
        if (e != hipSuccess) return e;
    }
    const uint32_t high = log2_size - kTileLog2;
    const uint32_t passes = (high + 8u) / 9u;
    const dim3 grid((uint32_t)(1ull << (log2_size - kTileLog2))), block(kThreads);
    uint32_t s0 = kTileLog2;
    for (uint32_t p = 0; p < passes; ++p) {
        const uint32_t left = log2_size - s0;
        // spread the stages evenly so that no pass is needlessly short
        const uint32_t m = (left + (passes - p) - 1u) / (passes - p);
        HighPassArgs a{};
        a.data = data;
        a.s0 = s0;
        a.m = m;
        a.last = p + 1u == passes;
        a.factor = factor;
        a.key0 = key0;
        a.key1 = key1;
        a.n = n;
        a.valid = valid;
        a.absmax = (a.last && !x) ? reinterpret_cast<uint32_t*>(absmax) : nullptr;
        if (a.last && x) {
            a.out = x;
            hipLaunchKernelGGL(high_pass_kernel<true>, grid, block, 0, stream, a);
        } else {
            hipLaunchKernelGGL(high_pass_kernel<false>, grid, block, 0, stream, a);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        // what is not zero afterwards: the blocks of 2^(s0 + m) floats that held a value
        const uint64_t block = 1ull << (s0 + m);
        valid = (valid + block - 1) / block * block;
        s0 += m;
    }
    return hipSuccess;
}

hipError_t launch_full_absmax(const float* y, uint32_t log2_size, float* absmax, hipStream_t stream) {
    const hipError_t e = launch_zero_words(reinterpret_cast<uint32_t*>(absmax), 1, stream);
    if (e != hipSuccess) return e;
    const uint64_t count = 1ull << log2_size;
    uint64_t blocks = count / (256u * 4u * 8u);   // 8 vectors per thread
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(full_absmax_kernel, dim3((uint32_t)blocks), dim3(256), 0, stream, y, count,
                       reinterpret_cast<uint32_t*>(absmax));
    return hipGetLastError();
}

hipError_t launch_full_encode(const float* y, uint32_t log2_size, const float* scale, uint32_t levels,
                              uint32_t bits, uint32_t worker, uint32_t key0, uint32_t key1,
                              uint8_t* payload, hipStream_t stream) {
    const uint64_t count = 1ull << log2_size;
    const uint64_t blocks = (count / 16u + 255u) / 256u;
    const dim3 grid((uint32_t)blocks), block(256);
    if (bits == 2)
        hipLaunchKernelGGL(full_encode_kernel<2>, grid, block, 0, stream, y, count, scale, levels, worker, key0, key1, payload);
    else if (bits == 4)
        hipLaunchKernelGGL(full_encode_kernel<4>, grid, block, 0, stream, y, count, scale, levels, worker, key0, key1, payload);
    else
        hipLaunchKernelGGL(full_encode_kernel<8>, grid, block, 0, stream, y, count, scale, levels, worker, key0, key1, payload);
    return hipGetLastError();
}

hipError_t launch_full_decode(const void* sums, uint32_t sum_bytes, uint32_t log2_size, const float* scale,
                              uint32_t levels, uint32_t W, float* yhat, hipStream_t stream) {
    const uint64_t count = 1ull << log2_size;
    const uint64_t blocks = (count / 4u + 255u) / 256u;
    const dim3 grid((uint32_t)blocks), block(256);
    if (sum_bytes == 1)
        hipLaunchKernelGGL(full_decode_kernel<uint8_t>, grid, block, 0, stream, static_cast<const uint8_t*>(sums), count, scale, levels, W, yhat);
    else
        hipLaunchKernelGGL(full_decode_kernel<uint16_t>, grid, block, 0, stream, static_cast<const uint16_t*>(sums), count, scale, levels, W, yhat);
    return hipGetLastError();
}

}  // namespace thc
