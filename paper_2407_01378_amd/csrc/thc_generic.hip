// Generic per-chunk kernels: every chunk_log2 in [1, 14], both input types, all
// payload widths.  One workgroup of 1024 threads owns a tile of 2^14 consecutive
// coordinates (one chunk of 2^14, or 2^(14-l') smaller chunks); each thread owns 16
// consecutive coordinates.  Butterfly stages run in the order stride 1, 2, 4, ...
// - strides below 16 in registers, the rest through LDS - so every value sees the
// same sequence of separately rounded fp32 additions as the reference definition.
// The tuned kernels for chunk_log2 = 14 live in their own file; this path is the
// fallback for every other shape and for unaligned gradients.
#include "thc_device.h"
#include "thc_internal.h"

#pragma clang fp contract(off)

namespace thc {
namespace {

constexpr int kTileLog2 = 14;
constexpr int kTile = 1 << kTileLog2;
constexpr int kThreads = 1024;
constexpr int kEpt = 16;  // coordinates per thread

template <Mode MODE>
__global__ __launch_bounds__(kThreads) void generic_kernel(const ChunkArgs a) {
    __shared__ float buf[kTile];
    __shared__ float red[kThreads];
    __shared__ float red_lo[kThreads];
    __shared__ uint32_t sgn[kTile / 32];

    const uint32_t t = threadIdx.x;
    const uint64_t base = (uint64_t)blockIdx.x << kTileLog2;
    const uint64_t g0 = base + (uint64_t)t * kEpt;
    const uint32_t l = a.chunk_log2;
    const uint32_t c = 1u << l;
    const uint64_t chunks = a.padded >> l;
    constexpr bool kFromGradient =
        MODE == Mode::Forward || MODE == Mode::Absmax || MODE == Mode::Encode || MODE == Mode::MinMax;
    const bool rotate = a.no_rotate == 0u;

    // Sign diagonal of the tile: 128 Philox blocks of 128 bits each.
    if (t < kTile / 128) {
        const u32x4 s = sign_block((base >> 7) + t, a.key0, a.key1);
#pragma unroll
        for (int i = 0; i < 4; ++i) sgn[4 * t + i] = s.w[i];
    }

    float v[kEpt];
    if constexpr (kFromGradient) {
        if (a.in_bf16) {
            const uint16_t* x = static_cast<const uint16_t*>(a.in);
#pragma unroll
            for (int j = 0; j < kEpt; ++j) {
                const uint64_t g = g0 + j;
                v[j] = g < a.n ? bf16_bits_to_float(x[g]) : 0.0f;
            }
        } else {
            const float* x = static_cast<const float*>(a.in);
#pragma unroll
            for (int j = 0; j < kEpt; ++j) {
                const uint64_t g = g0 + j;
                v[j] = g < a.n ? x[g] : 0.0f;
            }
        }
    } else if constexpr (MODE == Mode::Inverse) {
        const float* y = static_cast<const float*>(a.in);
#pragma unroll
        for (int j = 0; j < kEpt; ++j) {
            const uint64_t g = g0 + j;
            v[j] = g < a.padded ? y[g] : 0.0f;
        }
    } else {  // Decode: sums (or the saturated aggregate) -> rotated-domain estimate of the mean
        const float Lf = (float)a.levels;
        const float Wf = (float)a.W;
        const int centre = (int)(a.levels >> 1);   // M of the signed grid
#pragma unroll
        for (int j = 0; j < kEpt; ++j) {
            const uint64_t g = g0 + j;
            float val = 0.0f;
            if (g < a.padded) {
                if (a.range_in) {   // min/max grid: yhat = S * (step / W) + lo
                    const float lo = a.range_in[2 * (g >> l)], hi = a.range_in[2 * (g >> l) + 1];
                    const float step = (hi - lo) / Lf;
                    const float q = step / Wf;
                    const uint32_t S = a.sum_bytes == 1
                                           ? (uint32_t) static_cast<const uint8_t*>(a.in)[g]
                                           : (uint32_t) static_cast<const uint16_t*>(a.in)[g];
                    v[j] = (float)S * q + lo;
                    continue;
                }
                const float s = a.scale_in[g >> l];
                const float step = (s + s) / Lf;
                const float q = step / Wf;
                if (a.sat) {
                    const uint64_t bit = g * a.bits;
                    const uint32_t A = ((uint32_t) static_cast<const uint8_t*>(a.in)[bit >> 3] >> (bit & 7u)) &
                                       ((1u << a.bits) - 1u);
                    val = (float)((int)A - centre) * q;
                } else {
                    const uint32_t S = a.sum_bytes == 1
                                           ? (uint32_t) static_cast<const uint8_t*>(a.in)[g]
                                           : (uint32_t) static_cast<const uint16_t*>(a.in)[g];
                    val = (float)S * q - s;
                }
            }
            v[j] = val;
        }
    }
    __syncthreads();  // sgn[] is complete
    const uint32_t sbits = (sgn[(t * kEpt) >> 5] >> ((t * kEpt) & 31u)) & 0xFFFFu;
    if constexpr (kFromGradient) {
        if (rotate) {
#pragma unroll
            for (int j = 0; j < kEpt; ++j) v[j] = flip_sign(v[j], (sbits >> j) & 1u);
        }
    }

    // Stages with stride 1, 2, 4, 8: both partners live in this thread.
#pragma unroll
    for (int h = 1; h < kEpt; h <<= 1) {
        if ((uint32_t)h < c && rotate) {
#pragma unroll
            for (int i = 0; i < kEpt; ++i) {
                if ((i & h) == 0) {
                    const float lo = v[i], hi = v[i + h];
                    v[i] = lo + hi;
                    v[i + h] = lo - hi;
                }
            }
        }
    }
    // Stages with stride >= 16 through LDS, one barrier per stage.
    if (c > (uint32_t)kEpt && rotate) {
#pragma unroll
        for (int j = 0; j < kEpt; ++j) buf[t * kEpt + j] = v[j];
        for (uint32_t h = kEpt; h < c; h <<= 1) {
            __syncthreads();
#pragma unroll
            for (int i = 0; i < kTile / 2 / kThreads; ++i) {
                const uint32_t k = t + i * kThreads;
                const uint32_t lo_i = ((k & ~(h - 1u)) << 1) | (k & (h - 1u));
                const float lo = buf[lo_i], hi = buf[lo_i + h];
                buf[lo_i] = lo + hi;
                buf[lo_i + h] = lo - hi;
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kEpt; ++j) v[j] = buf[t * kEpt + j];
    }
    if (rotate) {
#pragma unroll
        for (int j = 0; j < kEpt; ++j) v[j] = v[j] * a.inv_sqrt_c;
    }

    if constexpr (MODE == Mode::Forward) {
        float* y = static_cast<float*>(a.out);
#pragma unroll
        for (int j = 0; j < kEpt; ++j)
            if (g0 + j < a.padded) y[g0 + j] = v[j];
    } else if constexpr (MODE == Mode::Inverse || MODE == Mode::Decode) {
#pragma unroll
        for (int j = 0; j < kEpt; ++j) {
            if (g0 + j < a.n) {
                const float val = rotate ? flip_sign(v[j], (sbits >> j) & 1u) : v[j];
                if (a.out_bf16) {   // round to nearest, ties to even
                    const uint32_t u = __float_as_uint(val);
                    static_cast<uint16_t*>(a.out)[g0 + j] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
                } else {
                    static_cast<float*>(a.out)[g0 + j] = val;
                }
            }
        }
    } else if constexpr (MODE == Mode::MinMax) {
        // (min, max) of each chunk
        float own_lo[kEpt], own_hi[kEpt];
        if (c >= (uint32_t)kEpt) {
            float mn = v[0], mx = v[0];
#pragma unroll
            for (int j = 1; j < kEpt; ++j) {
                mn = fminf(mn, v[j]);
                mx = fmaxf(mx, v[j]);
            }
            const uint32_t tpc = c / kEpt;  // threads per chunk
            red[t] = mx;
            red_lo[t] = mn;
            for (uint32_t s = tpc >> 1; s >= 1; s >>= 1) {
                __syncthreads();
                if ((t & (tpc - 1u)) < s) {
                    red[t] = fmaxf(red[t], red[t + s]);
                    red_lo[t] = fminf(red_lo[t], red_lo[t + s]);
                }
            }
            __syncthreads();
            mx = red[t & ~(tpc - 1u)];
            mn = red_lo[t & ~(tpc - 1u)];
#pragma unroll
            for (int j = 0; j < kEpt; ++j) {
                own_lo[j] = mn;
                own_hi[j] = mx;
            }
        } else {
#pragma unroll
            for (int j = 0; j < kEpt; ++j) {
                float mn = v[j], mx = v[j];
#pragma unroll
                for (int i = 0; i < kEpt; ++i)
                    if ((uint32_t)(i >> l) == (uint32_t)(j >> l)) {
                        mn = fminf(mn, v[i]);
                        mx = fmaxf(mx, v[i]);
                    }
                own_lo[j] = mn;
                own_hi[j] = mx;
            }
        }
        float* dst = static_cast<float*>(a.out);
#pragma unroll
        for (int j = 0; j < kEpt; ++j) {
            const uint64_t g = g0 + j;
            if ((g & (uint64_t)(c - 1u)) == 0 && (g >> l) < chunks) {
                dst[2 * (g >> l)] = own_lo[j];
                dst[2 * (g >> l) + 1] = own_hi[j];
            }
        }
    } else {
        // Range of each chunk: largest |rotated value|.
        float own[kEpt];  // own[j]: absmax of the chunk that holds coordinate j
        if (c >= (uint32_t)kEpt) {
            float m = 0.0f;
#pragma unroll
            for (int j = 0; j < kEpt; ++j) m = fmaxf(m, fabsf(v[j]));
            const uint32_t tpc = c / kEpt;  // threads per chunk
            red[t] = m;
            for (uint32_t s = tpc >> 1; s >= 1; s >>= 1) {
                __syncthreads();
                if ((t & (tpc - 1u)) < s) red[t] = fmaxf(red[t], red[t + s]);
            }
            __syncthreads();
            m = red[t & ~(tpc - 1u)];
#pragma unroll
            for (int j = 0; j < kEpt; ++j) own[j] = m;
        } else {
#pragma unroll
            for (int j = 0; j < kEpt; ++j) {
                float m = 0.0f;
#pragma unroll
                for (int i = 0; i < kEpt; ++i)
                    if ((uint32_t)(i >> l) == (uint32_t)(j >> l)) m = fmaxf(m, fabsf(v[i]));
                own[j] = m;
            }
        }
        // First coordinate of a chunk reports that chunk's value.
        auto report = [&](float* dst, const float* val) {
#pragma unroll
            for (int j = 0; j < kEpt; ++j) {
                const uint64_t g = g0 + j;
                if ((g & (uint64_t)(c - 1u)) == 0 && (g >> l) < chunks) dst[g >> l] = val[j];
            }
        };
        if constexpr (MODE == Mode::Absmax) {
            report(static_cast<float*>(a.out), own);
        } else {  // Encode
            float s_el[kEpt];
#pragma unroll
            for (int j = 0; j < kEpt; ++j) {
                const uint64_t p = (g0 + j) >> l;
                s_el[j] = a.scale_in ? (p < chunks ? a.scale_in[p] : 0.0f) : own[j];
            }
            if (a.scale_out) report(a.scale_out, s_el);

            const float Lf = (float)a.levels;
            const u32x4 rb = round_block(g0 >> 4, a.worker, a.key0, a.key1);
            uint32_t pk[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < kEpt; ++j) {
                const uint32_t r = (rb.w[j >> 2] >> (8 * (j & 3))) & 0xFFu;
                const float u = ((float)r + 0.5f) * (1.0f / 256.0f);
                float tt;   // position in grid units + noise, one fused operation
                if (a.range_in) {   // min/max grid: (y - lo) * inv + u
                    const uint64_t p = (g0 + j) >> l;
                    const float lo = p < chunks ? a.range_in[2 * p] : 0.0f;
                    const float hi = p < chunks ? a.range_in[2 * p + 1] : 0.0f;
                    const float width = hi - lo;
                    const float inv = width >= kMinRange ? Lf / width : 0.0f;
                    tt = __builtin_fmaf(v[j] - lo, inv, u);
                } else {            // symmetric grid: y * inv + L/2 + u
                    const float s = s_el[j];
                    const float two = s + s;
                    const bool ranged = two >= kMinRange;
                    const float inv = ranged ? Lf / two : 0.0f;
                    // all-zero chunk (or one too small for L / two): index 0 on the 2^bits-point
                    // grid, the centre on the signed one
                    const float zero_idx = (!ranged && (a.levels & 1u) == 0u) ? 0.5f * Lf : 0.0f;
                    if (a.levels <= kSingleFmaMaxLevels)   // small grids: one rounding from y itself
                        tt = __builtin_fmaf(v[j], inv, (ranged ? 0.5f * Lf : zero_idx) + u);
                    else                                   // large grids: the offset y + s is rounded first
                        tt = __builtin_fmaf(v[j] + s, inv, zero_idx + u);
                }
                uint32_t q = (uint32_t)fminf(floorf(tt), Lf);
                if (g0 + j >= a.padded) q = 0u;
                const uint32_t bit = (uint32_t)j * a.bits;
                pk[bit >> 5] |= q << (bit & 31u);
            }
            const uint64_t nbytes = 2u * a.bits;  // 16 coordinates
            const uint64_t byte0 = (g0 >> 4) * nbytes;
            uint8_t* dst = static_cast<uint8_t*>(a.out) + byte0;
            if (byte0 + nbytes <= a.payload_bytes) {
                if (a.bits == 8) {
                    *reinterpret_cast<uint4*>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                } else if (a.bits == 4) {
                    *reinterpret_cast<uint2*>(dst) = make_uint2(pk[0], pk[1]);
                } else {
                    *reinterpret_cast<uint32_t*>(dst) = pk[0];
                }
            } else {
                for (uint32_t i = 0; i < nbytes && byte0 + i < a.payload_bytes; ++i)
                    dst[i] = (uint8_t)(pk[i >> 2] >> (8 * (i & 3)));
            }
        }
    }
}

// ---------------------------------------------------------------- aggregation
// Each thread sums one 16-byte slice of the payloads (128 / BITS coordinates) over a
// batch of at most 16 workers in packed sub-word lanes, then widens to the sum type.
template <int BITS, typename SumT>
__global__ __launch_bounds__(256) void aggregate_kernel(const PayloadBatch batch, uint32_t count,
                                                        bool accumulate, uint64_t payload_bytes,
                                                        uint64_t padded, SumT* sums) {
    constexpr int kCoords = 128 / BITS;
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t byte0 = i * 16u;
    if (byte0 >= payload_bytes) return;
    const bool whole = byte0 + 16u <= payload_bytes;

    uint32_t acc[kCoords];
#pragma unroll
    for (int e = 0; e < kCoords; ++e) acc[e] = 0u;

    for (uint32_t w = 0; w < count; ++w) {
        uint32_t x[4] = {0u, 0u, 0u, 0u};
        const uint8_t* src = batch.p[w] + byte0;
        if (whole) {
            const uint4 q = *reinterpret_cast<const uint4*>(src);
            x[0] = q.x;
            x[1] = q.y;
            x[2] = q.z;
            x[3] = q.w;
        } else {
            for (uint32_t b = 0; byte0 + b < payload_bytes; ++b)
                x[b >> 2] |= (uint32_t)src[b] << (8 * (b & 3));
        }
#pragma unroll
        for (int e = 0; e < kCoords; ++e) {
            const int bit = e * BITS;
            acc[e] += (x[bit >> 5] >> (bit & 31)) & ((1u << BITS) - 1u);
        }
    }
    const uint64_t g0 = i * kCoords;
#pragma unroll
    for (int e = 0; e < kCoords; ++e) {
        const uint64_t g = g0 + e;
        if (g < padded) {
            uint32_t s = acc[e];
            if (accumulate) s += (uint32_t)sums[g];
            sums[g] = (SumT)s;
        }
    }
}

// Saturating aggregation in worker order: a_0 = z_0, a_w = Sat(a_(w-1), z_w), z = idx - M.
// Each thread owns one 16-byte slice of the payloads (128 / BITS coordinates) and writes
// the same slice of the aggregate (offset binary, a + M).  COUNT: also count the
// coordinates (below `padded`) for which at least one step clipped.
template <int BITS, bool COUNT>
__global__ __launch_bounds__(256) void sat_aggregate_kernel(const FusedPayloadPtrs ptrs, uint32_t W,
                                                            uint64_t payload_bytes, uint64_t padded,
                                                            uint8_t* aggregate,
                                                            unsigned long long* overflow) {
    constexpr int kCoords = 128 / BITS;
    constexpr int M = (1 << (BITS - 1)) - 1;
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t byte0 = i * 16u;
    uint32_t clipped_here = 0u;
    if (byte0 < payload_bytes) {
        const bool whole = byte0 + 16u <= payload_bytes;
        int acc[kCoords];
        uint32_t clipped[kCoords];
        for (uint32_t w = 0; w < W; ++w) {
            uint32_t x[4] = {0u, 0u, 0u, 0u};
            const uint8_t* src = ptrs.p[w] + byte0;
            if (whole) {
                const uint4 q = *reinterpret_cast<const uint4*>(src);
                x[0] = q.x;
                x[1] = q.y;
                x[2] = q.z;
                x[3] = q.w;
            } else {
                for (uint32_t b = 0; byte0 + b < payload_bytes; ++b)
                    x[b >> 2] |= (uint32_t)src[b] << (8 * (b & 3));
            }
#pragma unroll
            for (int e = 0; e < kCoords; ++e) {
                const int bit = e * BITS;
                const int z = (int)((x[bit >> 5] >> (bit & 31)) & ((1u << BITS) - 1u)) - M;
                if (w == 0) {
                    acc[e] = z;
                    clipped[e] = 0u;
                } else {
                    const int raw = acc[e] + z;
                    const int a = raw < -M ? -M : (raw > M ? M : raw);
                    if (COUNT) clipped[e] |= (uint32_t)(raw != a);
                    acc[e] = a;
                }
            }
        }
        uint32_t o[4] = {0u, 0u, 0u, 0u};
        const uint64_t g0 = i * kCoords;
#pragma unroll
        for (int e = 0; e < kCoords; ++e) {
            const int bit = e * BITS;
            const bool real = g0 + e < padded;
            o[bit >> 5] |= (real ? (uint32_t)(acc[e] + M) : 0u) << (bit & 31);
            if (COUNT && real) clipped_here += clipped[e];
        }
        uint8_t* dst = aggregate + byte0;
        if (whole) {
            *reinterpret_cast<uint4*>(dst) = make_uint4(o[0], o[1], o[2], o[3]);
        } else {
            for (uint32_t b = 0; byte0 + b < payload_bytes; ++b) dst[b] = (uint8_t)(o[b >> 2] >> (8 * (b & 3)));
        }
    }
    if (COUNT) {   // one atomic per wave
        uint32_t tot = clipped_here;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) tot += __shfl_xor(tot, off, 64);
        if ((threadIdx.x & 63u) == 0 && tot != 0u) atomicAdd(overflow, (unsigned long long)tot);
    }
}

__global__ __launch_bounds__(256) void scale_reduce_kernel(const float* absmax_all, uint32_t W,
                                                           uint64_t chunks, float* scale) {
    const uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= chunks) return;
    float m = absmax_all[p];
    for (uint32_t w = 1; w < W; ++w) m = fmaxf(m, absmax_all[(uint64_t)w * chunks + p]);
    scale[p] = m;
}

__global__ __launch_bounds__(256) void range_reduce_kernel(const float* range_all, uint32_t W,
                                                           uint64_t chunks, float* range) {
    const uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= chunks) return;
    float lo = range_all[2 * p], hi = range_all[2 * p + 1];
    for (uint32_t w = 1; w < W; ++w) {
        lo = fminf(lo, range_all[2 * ((uint64_t)w * chunks + p)]);
        hi = fmaxf(hi, range_all[2 * ((uint64_t)w * chunks + p) + 1]);
    }
    range[2 * p] = lo;
    range[2 * p + 1] = hi;
}

}  // namespace

hipError_t launch_generic(Mode mode, const ChunkArgs& a, hipStream_t stream) {
    const uint64_t tiles = (a.padded + kTile - 1) / kTile;
    if (tiles == 0) return hipSuccess;
    if (tiles > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)tiles), block(kThreads);
    switch (mode) {
        case Mode::Forward:
            hipLaunchKernelGGL(generic_kernel<Mode::Forward>, grid, block, 0, stream, a);
            break;
        case Mode::Absmax:
            hipLaunchKernelGGL(generic_kernel<Mode::Absmax>, grid, block, 0, stream, a);
            break;
        case Mode::Encode:
            hipLaunchKernelGGL(generic_kernel<Mode::Encode>, grid, block, 0, stream, a);
            break;
        case Mode::Inverse:
            hipLaunchKernelGGL(generic_kernel<Mode::Inverse>, grid, block, 0, stream, a);
            break;
        case Mode::Decode:
            hipLaunchKernelGGL(generic_kernel<Mode::Decode>, grid, block, 0, stream, a);
            break;
        case Mode::MinMax:
            hipLaunchKernelGGL(generic_kernel<Mode::MinMax>, grid, block, 0, stream, a);
            break;
        case Mode::Plain:
        case Mode::PlainDecode:
            return hipErrorInvalidValue;   // only the tuned chunk-2^14 kernels implement it
    }
    return hipGetLastError();
}

hipError_t launch_aggregate(const PayloadBatch& batch, uint32_t count, bool accumulate,
                            uint32_t bits, uint32_t sum_bytes, uint64_t payload_bytes,
                            uint64_t padded, void* sums, hipStream_t stream) {
    const uint64_t threads = (payload_bytes + 15u) / 16u;
    if (threads == 0) return hipSuccess;
    const uint64_t blocks = (threads + 255u) / 256u;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)blocks), block(256);
#define THC_AGG(B, T)                                                                         \
    hipLaunchKernelGGL((aggregate_kernel<B, T>), grid, block, 0, stream, batch, count,        \
                       accumulate, payload_bytes, padded, static_cast<T*>(sums))
    if (sum_bytes == 1) {
        if (bits == 2) THC_AGG(2, uint8_t);
        else if (bits == 4) THC_AGG(4, uint8_t);
        else THC_AGG(8, uint8_t);
    } else {
        if (bits == 2) THC_AGG(2, uint16_t);
        else if (bits == 4) THC_AGG(4, uint16_t);
        else THC_AGG(8, uint16_t);
    }
#undef THC_AGG
    return hipGetLastError();
}

hipError_t launch_sat_aggregate(const FusedPayloadPtrs& ptrs, uint32_t W, uint32_t bits,
                                uint64_t payload_bytes, uint64_t padded, uint8_t* aggregate,
                                unsigned long long* overflow, hipStream_t stream) {
    const uint64_t threads = (payload_bytes + 15u) / 16u;
    if (threads == 0) return hipSuccess;
    const uint64_t blocks = (threads + 255u) / 256u;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    const dim3 grid((uint32_t)blocks), block(256);
#define THC_SAT(B)                                                                              \
    do {                                                                                        \
        if (overflow)                                                                           \
            hipLaunchKernelGGL((sat_aggregate_kernel<B, true>), grid, block, 0, stream, ptrs, W,  \
                               payload_bytes, padded, aggregate, overflow);                     \
        else                                                                                    \
            hipLaunchKernelGGL((sat_aggregate_kernel<B, false>), grid, block, 0, stream, ptrs, W, \
                               payload_bytes, padded, aggregate, overflow);                     \
    } while (0)
    if (bits == 2) THC_SAT(2);
    else if (bits == 4) THC_SAT(4);
    else THC_SAT(8);
#undef THC_SAT
    return hipGetLastError();
}

hipError_t launch_range_reduce(const float* range_all, uint32_t W, uint64_t chunks, float* range,
                               hipStream_t stream) {
    if (chunks == 0) return hipSuccess;
    const uint64_t blocks = (chunks + 255u) / 256u;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(range_reduce_kernel, dim3((uint32_t)blocks), dim3(256), 0, stream, range_all, W,
                       chunks, range);
    return hipGetLastError();
}

hipError_t launch_scale_reduce(const float* absmax_all, uint32_t W, uint64_t chunks, float* scale,
                               hipStream_t stream) {
    if (chunks == 0) return hipSuccess;
    const uint64_t blocks = (chunks + 255u) / 256u;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(scale_reduce_kernel, dim3((uint32_t)blocks), dim3(256), 0, stream,
                       absmax_all, W, chunks, scale);
    return hipGetLastError();
}

}  // namespace thc
