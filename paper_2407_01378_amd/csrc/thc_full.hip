// Full rotation (l' = l): the Hadamard transform of a whole gradient padded to 2^l
// coordinates, l > 14, as the paper's baseline for the partial rotation.  Stages run in
// the same order as everywhere else (stride 1, 2, 4, ..., 2^(l-1), every stage one
// separately rounded fp32 add and subtract), so results are bit-identical to the
// stage-by-stage definition:
//   stages 0..13    the chunk-2^14 kernels (thc_fast14.hip), data in registers and LDS
//   stages 14..l-1  "high passes" over the fp32 array in global memory, up to 9 stages per
//                   pass (this file), in place
// plus the steps of the quantizer on rotated data, which the partial-rotation path fuses into
// its rotation kernels: as elementwise kernels on stored values (range, encode, decode), and
// as variants of the last forward pass that keep only the range of its results, or quantize
// them once the shared scale is known, so that the rotated values are never stored.
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
    uint32_t last;      // host side: the pass that multiplies by `factor` (a template argument of the kernels)
    float factor;
    uint32_t key0, key1;
    uint64_t valid;     // floats of `data` that hold values; what lies beyond reads as zero and
                        // is neither read nor, in a pass that is not the last, written (the zero
                        // padding behind the gradient is implied, pass after pass, until the
                        // last pass mixes it with everything)
    uint32_t* absmax;   // last forward pass: receives max |value written| by an unsigned atomic
                        // maximum (zeroed beforehand); may be null
    // last forward pass evaluated for the quantizer instead of being stored (encode_pass_kernel):
    const float* scale; // one float, shared by all workers
    uint32_t levels;    // largest grid index L
    uint32_t worker;
    uint8_t* payload;   // 2^l * bits / 8 bytes
};

// What a pass does with its results.
constexpr int kInPlace = 0;    // written back to `data`
constexpr int kToX = 1;        // inverse direction, last pass: sign diagonal, first n values to `out`
constexpr int kRangeOnly = 2;  // forward direction, last pass: only their largest magnitude is kept

// Stochastic rounding of rotated values (already normalised) onto the grid of [-s, s]:
// same arithmetic and random stream as the fused encoders.
struct FullQuant {
    float s, inv, half, off, Lf;
};
__device__ __forceinline__ FullQuant full_quant(float s, uint32_t levels) {
    FullQuant q;
    q.s = s;
    const float two = s + s;
    q.Lf = (float)levels;
    const bool ranged = two >= kMinRange;
    q.inv = ranged ? q.Lf / two : 0.0f;
    const bool single = levels <= kSingleFmaMaxLevels;   // evaluation order by grid size
    q.half = (single && ranged) ? 0.5f * q.Lf : 0.0f;   // an all-zero (or vanishingly small) vector gets index 0
    q.off = single ? 0.0f : s;
    return q;
}
// 16 consecutive coordinates (the ones of Philox block `blk` of the rounding stream) -> 2 * BITS payload bytes.
template <int BITS>
__device__ __forceinline__ void quantize_run(const float (&yv)[16], uint64_t blk, const FullQuant& q, uint32_t worker,
                                             uint32_t key0, uint32_t key1, uint8_t* payload) {
    const u32x4 rb = round_block(blk, worker, key0, key1);
    uint32_t pk[4] = {0u, 0u, 0u, 0u};
    // u = (r + 0.5) / 256 and L/2 + u are exact in fp32, so one multiply-add gives the same c = L/2 + u
    // (or u alone on the large grids); t >= 0, so the conversion's truncation is the floor.
    const float c0 = q.half + 0x1p-9f;
    const uint32_t L = (uint32_t)q.Lf;
    auto place = [&](int j, float y) {
        const uint32_t r = (rb.w[j >> 2] >> (8 * (j & 3))) & 0xFFu;
        const float c = __builtin_fmaf((float)r, 0x1p-8f, c0);
        const float tt = __builtin_fmaf(y, q.inv, c);
        const uint32_t idx = min((uint32_t)tt, L);
        const int bit = j * BITS;
        pk[bit >> 5] |= idx << (bit & 31);
    };
    if (q.off != 0.0f) {   // (uniform) large grids: fma(y + s, inv, u)
#pragma unroll
        for (int j = 0; j < 16; ++j) place(j, yv[j] + q.off);
    } else {               // small grids: fma(y, inv, L/2 + u)
#pragma unroll
        for (int j = 0; j < 16; ++j) place(j, yv[j]);
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

// Where a thread's share of a tile lies.
struct Tile {
    uint64_t base;
    uint32_t skip, s0;
    uint32_t jq, la, w;   // lane & 7, lane >> 3, wave
    __device__ __forceinline__ uint64_t row_start(uint32_t row) const {   // first float of a row
        const uint64_t k = row >> skip;
        const uint32_t jext = row & ((1u << skip) - 1u);
        return base + (k << s0) + (uint64_t)(jext * 32u);
    }
    __device__ __forceinline__ uint64_t offset(uint32_t row) const { return row_start(row) + 4u * jq; }
};
// `block` receives the first float of the 2^(s0 + m) block the tile belongs to.
template <int SKIP>
__device__ __forceinline__ Tile make_tile(const HighPassArgs& a, uint64_t tile, uint32_t t, uint64_t& block) {
    Tile T;
    T.skip = (uint32_t)SKIP;   // = 9 - a.m, a constant of the kernel so that the stage loops are straight-line code
    T.s0 = a.s0;
    const uint32_t lane = t & 63u;
    T.jq = lane & 7u;
    T.la = lane >> 3;
    T.w = t >> 6;
    const uint32_t jb_bits = a.s0 - 5u - T.skip;                  // column blocks per 2^s0 run
    const uint64_t jb = tile & ((1ull << jb_bits) - 1ull);
    const uint64_t hi = tile >> jb_bits;
    block = hi << (a.s0 + a.m);
    T.base = block + (jb << (5u + T.skip));
    return T;
}

// Sixteen bytes of zeros: where rows in the implied padding are read from.
__device__ const float4 kZeroRow = {0.0f, 0.0f, 0.0f, 0.0f};

// Rows r + 8 la + 64 w, r = 0..7, of the tile: 8 loads back to back.  (A row in the implied
// padding is loaded from kZeroRow instead: a select of the address, none of the values.)
__device__ __forceinline__ void load_rows(const HighPassArgs& a, const Tile& T, float4 (&raw)[8]) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const uint64_t g = T.offset(r + 8u * T.la + 64u * T.w);   // a multiple of 4, as `valid` is
        const float4* src = g < a.valid ? reinterpret_cast<const float4*>(a.data + g) : &kZeroRow;
        raw[r] = *src;
    }
}
__device__ __forceinline__ void take_rows(const float4 (&raw)[8], float (&v)[32]) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        v[4 * r] = raw[r].x;
        v[4 * r + 1] = raw[r].y;
        v[4 * r + 2] = raw[r].z;
        v[4 * r + 3] = raw[r].w;
    }
}

// The stages of the pass on one tile.  In: rows r + 8 la + 64 w; out: rows la + 8 w + 64 r.
__device__ __forceinline__ void rotate_tile(const Tile& T, float (&v)[32], float4* xb) {
    const uint32_t skip = T.skip, la = T.la, jq = T.jq, w = T.w;
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
}

// A workgroup takes two neighbouring tiles (they lie in the same 2^(s0 + m) block); the second
// one's loads are in flight while the first one is transformed and stored.
template <int KIND, int SKIP, bool LAST>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void high_pass_kernel(const HighPassArgs a) {
    constexpr bool TO_X = KIND == kToX;
    __shared__ float4 xb[4096];
    const uint32_t t = threadIdx.x, lane = t & 63u;
    uint64_t block;
    Tile T = make_tile<SKIP>(a, 2ull * blockIdx.x, t, block);
    // a tile mixes values of one block of 2^(s0 + m) floats: if that block lies in the implied
    // zero padding its results are zero too, and the next pass is told so instead of reading them
    // (the last pass writes everything: an empty gradient gives zeros)
    if (!LAST && block >= a.valid) return;

    float4 raw[8];
    load_rows(a, T, raw);
    float largest = 0.0f;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        float v[32];
        take_rows(raw, v);
        const Tile now = T;
        if (k == 0) {
            T = make_tile<SKIP>(a, 2ull * blockIdx.x + 1ull, t, block);
            load_rows(a, T, raw);
        }
        rotate_tile(now, v, xb);
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const uint64_t g = now.offset(now.la + 8u * now.w + 64u * (uint32_t)r);
            float o[4] = {v[4 * r], v[4 * r + 1], v[4 * r + 2], v[4 * r + 3]};
            if (LAST) {
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = o[e] * a.factor;
            }
            if (!TO_X) {   // (two three-input maxima)
                largest = fmaxf(fmaxf(largest, fabsf(o[0])), fabsf(o[1]));
                largest = fmaxf(fmaxf(largest, fabsf(o[2])), fabsf(o[3]));
            }
            if constexpr (KIND == kRangeOnly) {
                (void)g;
            } else if constexpr (TO_X) {
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
        if (k == 0) {
            // the second tile's values are first needed here, not where the scheduler would like them;
            // its first exchange must not overwrite units another wave is still reading
#pragma unroll
            for (int r = 0; r < 8; ++r)
                asm volatile("" : "+v"(raw[r].x), "+v"(raw[r].y), "+v"(raw[r].z), "+v"(raw[r].w));
            __syncthreads();
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

// The last forward pass evaluated for the quantizer: the results of a tile are quantized and
// packed instead of being stored (`data` is only read).  A workgroup takes two neighbouring
// tiles; the second one's loads are in flight while the first one is quantized.
template <int BITS, int SKIP>
__global__ __launch_bounds__(kThreads) void encode_pass_kernel(const HighPassArgs a) {
    __shared__ float4 xb[4096];
    const uint32_t t = threadIdx.x, lane = t & 63u;
    uint64_t block;
    Tile T = make_tile<SKIP>(a, 2ull * blockIdx.x, t, block);
    float4 raw[8];
    load_rows(a, T, raw);
    const FullQuant fq = full_quant(a.scale[0], a.levels);
    float4* mine = xb + 512u * T.w;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        float v[32];
        take_rows(raw, v);
        rotate_tile(T, v, xb);
        // exchange 3, inside the wave: 4 lanes x 4 floats of a row -> 16 consecutive floats in one
        // lane, the coordinates of one block of the rounding stream and 2 * BITS payload bytes.
        __syncthreads();   // every wave has taken its share of exchange 2 out of this wave's units
#pragma unroll
        for (int r = 0; r < 8; ++r)   // unit (row of the wave, jq), row of the wave = la + 8 r
            mine[((uint32_t)r * 8u + T.la) * 8u + T.jq] =
                make_float4(v[4 * r] * a.factor, v[4 * r + 1] * a.factor, v[4 * r + 2] * a.factor, v[4 * r + 3] * a.factor);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        const Tile now = T;
        if (k == 0) {
            T = make_tile<SKIP>(a, 2ull * blockIdx.x + 1ull, t, block);
            load_rows(a, T, raw);
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t run = lane + 64u * (uint32_t)h;   // (row of the wave, half of the row), 0 .. 127
            const uint32_t rho = run >> 1, half = run & 1u;
            const uint64_t g = now.row_start((rho & 7u) + 8u * now.w + 64u * (rho >> 3)) + 16u * half;
            float yv[16];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 q = mine[rho * 8u + 4u * half + (uint32_t)i];
                yv[4 * i] = q.x;
                yv[4 * i + 1] = q.y;
                yv[4 * i + 2] = q.z;
                yv[4 * i + 3] = q.w;
            }
            quantize_run<BITS>(yv, g >> 4, fq, a.worker, a.key0, a.key1, a.payload);
        }
        if (k == 0) {
            // the second tile's values are first needed here, not where the scheduler would like them
#pragma unroll
            for (int r = 0; r < 8; ++r)
                asm volatile("" : "+v"(raw[r].x), "+v"(raw[r].y), "+v"(raw[r].z), "+v"(raw[r].w));
        }
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

// The quantizer on stored rotated values.  One thread: 16 coordinates, one Philox block,
// 2 * BITS payload bytes.
template <int BITS>
__global__ __launch_bounds__(256) void full_encode_kernel(const float* y, uint64_t count, const float* scale,
                                                          uint32_t levels, uint32_t worker, uint32_t key0,
                                                          uint32_t key1, uint8_t* payload) {
    const uint64_t blk = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t g0 = blk * 16u;
    if (g0 >= count) return;
    const FullQuant fq = full_quant(scale[0], levels);
    float yv[16];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float4 q = *reinterpret_cast<const float4*>(y + g0 + 4 * k);
        yv[4 * k] = q.x;
        yv[4 * k + 1] = q.y;
        yv[4 * k + 2] = q.z;
        yv[4 * k + 3] = q.w;
    }
    quantize_run<BITS>(yv, blk, fq, worker, key0, key1, payload);
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

// One instantiation per number of stages of the pass (skip = 9 - m = 0 .. 8).
template <int KIND, bool LAST>
void launch_pass(uint32_t skip, dim3 grid, dim3 block, hipStream_t stream, const HighPassArgs& a) {
    switch (skip) {
        case 0: hipLaunchKernelGGL((high_pass_kernel<KIND, 0, LAST>), grid, block, 0, stream, a); break;
        case 1: hipLaunchKernelGGL((high_pass_kernel<KIND, 1, LAST>), grid, block, 0, stream, a); break;
        case 2: hipLaunchKernelGGL((high_pass_kernel<KIND, 2, LAST>), grid, block, 0, stream, a); break;
        case 3: hipLaunchKernelGGL((high_pass_kernel<KIND, 3, LAST>), grid, block, 0, stream, a); break;
        case 4: hipLaunchKernelGGL((high_pass_kernel<KIND, 4, LAST>), grid, block, 0, stream, a); break;
        case 5: hipLaunchKernelGGL((high_pass_kernel<KIND, 5, LAST>), grid, block, 0, stream, a); break;
        case 6: hipLaunchKernelGGL((high_pass_kernel<KIND, 6, LAST>), grid, block, 0, stream, a); break;
        case 7: hipLaunchKernelGGL((high_pass_kernel<KIND, 7, LAST>), grid, block, 0, stream, a); break;
        default: hipLaunchKernelGGL((high_pass_kernel<KIND, 8, LAST>), grid, block, 0, stream, a); break;
    }
}
template <int BITS>
void launch_encode_pass(uint32_t skip, dim3 grid, dim3 block, hipStream_t stream, const HighPassArgs& a) {
    switch (skip) {
        case 0: hipLaunchKernelGGL((encode_pass_kernel<BITS, 0>), grid, block, 0, stream, a); break;
        case 1: hipLaunchKernelGGL((encode_pass_kernel<BITS, 1>), grid, block, 0, stream, a); break;
        case 2: hipLaunchKernelGGL((encode_pass_kernel<BITS, 2>), grid, block, 0, stream, a); break;
        case 3: hipLaunchKernelGGL((encode_pass_kernel<BITS, 3>), grid, block, 0, stream, a); break;
        case 4: hipLaunchKernelGGL((encode_pass_kernel<BITS, 4>), grid, block, 0, stream, a); break;
        case 5: hipLaunchKernelGGL((encode_pass_kernel<BITS, 5>), grid, block, 0, stream, a); break;
        case 6: hipLaunchKernelGGL((encode_pass_kernel<BITS, 6>), grid, block, 0, stream, a); break;
        case 7: hipLaunchKernelGGL((encode_pass_kernel<BITS, 7>), grid, block, 0, stream, a); break;
        default: hipLaunchKernelGGL((encode_pass_kernel<BITS, 8>), grid, block, 0, stream, a); break;
    }
}

}  // namespace

// Stages 14 .. l-1 on data (2^l floats, stages 0..13 already done), in place; the last pass
// multiplies by `factor`, and for the inverse direction (`x` non-null) applies the sign
// diagonal and writes the first n coordinates to x instead.  Forward direction: only the
// first `valid` floats of data have been written (the rest is the zero padding, which the
// first pass supplies by itself), and `absmax`, if not null, receives the largest
// magnitude of the result (the word is zeroed here first).  `deferred`, forward direction:
// RangeOnly = the last pass only reports the range and leaves data as the pass before it wrote
// it; EncodeOnly = only the last pass runs, on such data, and its results go through the
// quantizer into deferred->payload.
hipError_t launch_high_passes(float* data, uint32_t log2_size, float factor, float* x, uint64_t n,
                              uint32_t key0, uint32_t key1, hipStream_t stream, uint64_t valid,
                              float* absmax, const FullDeferred* deferred) {
    const bool range_only = deferred && deferred->kind == FullLast::RangeOnly;
    const bool encode_only = deferred && deferred->kind == FullLast::EncodeOnly;
    if ((deferred && (x || range_only == encode_only)) || (range_only && !absmax)) return hipErrorInvalidValue;
    if (absmax) {
        const hipError_t e = launch_zero_words(reinterpret_cast<uint32_t*>(absmax), 1, stream);
        if (e != hipSuccess) return e;
    }
    const uint32_t high = log2_size - kTileLog2;
    const uint32_t passes = (high + 8u) / 9u;
    const dim3 grid((uint32_t)(1ull << (log2_size - kTileLog2 - 1u))), block(kThreads);   // tile pairs (log2_size >= 15)
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
        const uint32_t skip = 9u - m;
        if (a.last && x) {
            a.out = x;
            launch_pass<kToX, true>(skip, grid, block, stream, a);
        } else if (a.last && range_only) {
            launch_pass<kRangeOnly, true>(skip, grid, block, stream, a);
        } else if (a.last && encode_only) {
            a.scale = deferred->scale;
            a.levels = deferred->levels;
            a.worker = deferred->worker;
            a.payload = deferred->payload;
            if (deferred->bits == 2) launch_encode_pass<2>(skip, grid, block, stream, a);
            else if (deferred->bits == 4) launch_encode_pass<4>(skip, grid, block, stream, a);
            else launch_encode_pass<8>(skip, grid, block, stream, a);
        } else if (!encode_only) {
            if (a.last) launch_pass<kInPlace, true>(skip, grid, block, stream, a);
            else launch_pass<kInPlace, false>(skip, grid, block, stream, a);
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
