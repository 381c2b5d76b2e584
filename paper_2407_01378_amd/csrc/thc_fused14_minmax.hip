// One-pass kernels of the min/max-range variant for chunk_log2 = 14 (with or without the
// rotation): the counterpart of thc_fused14.hip's encode_all / aggregate_decode for the grid
// that runs from the chunk's smallest to its largest value.
//
// encode_all_minmax: a work item is (chunk p, worker w).  The workgroup that owns it brings
// the chunk into registers (rotated or as it is), publishes its (min, max) to per-chunk
// words in global memory, waits until all W workers of the chunk have published, and
// quantizes onto the shared range - every gradient is read from HBM once (the
// one-call-per-step form reads it twice).  Grid, item order, bounded waits and the
// self-clearing workspace follow thc_fused14.hip's encode_all_kernel, with two words per wave.
//
// unrotated_aggregate_decode: without the rotation the decoder is elementwise, so it is
// written for coalescing instead of for the rotation's register layout.
#include "thc_core14.h"
#include "thc_internal.h"

#pragma clang fp contract(off)

namespace thc {
namespace k14 {
namespace {

constexpr uint32_t kWaves = kThreads / 64;
constexpr int kWavesPerSimd = 4;   // two workgroups of 8 waves per CU
constexpr int kFirstPollSleep = 32;
constexpr int kPollSleep = 8;

// Order-preserving map of floats onto unsigned words that are never zero for anything
// but a NaN (zero means "not published yet"): x <= y  <=>  key(x) <= key(y).
__device__ __forceinline__ uint32_t order_key(float x) {
    const uint32_t b = __float_as_uint(x);
    const uint32_t k = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    return k != 0u ? k : 1u;
}
__device__ __forceinline__ float order_value(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
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

template <bool BF16, int BITS, bool ROTATE>
__global__ __launch_bounds__(kThreads, kWavesPerSimd) void encode_all_minmax_kernel(const EncodeAllArgs a,
                                                                                    const FusedWorkerPtrs ptrs) {
    __shared__ Shared sh;
    constexpr int kUnits = BF16 ? 4 : 8;
    constexpr int kElem = BF16 ? 2 : 4;
    constexpr uint32_t kNone = 0xFFFFFFFFu;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t p0 = blockIdx.x / a.W;
    const uint32_t w = blockIdx.x - p0 * a.W;      // the grid is a multiple of W
    const uint32_t dp = gridDim.x / a.W;
    const uint32_t half = kWaves * a.W;            // words of one kind per chunk: maxima, then minima
    const uint32_t nwords = 2u * half;
    const uint32_t mine = kWaves * w + wave;
    if (p0 >= a.chunks) return;
    uint32_t prev = kNone;
    // bf16 input (16 registers per thread) is loaded one item ahead; fp32 input (32 registers)
    // when its item starts
    constexpr bool kAhead = BF16;
    Raw<kUnits> raw;
    auto load = [&](uint64_t p) {
        const uint64_t g0 = p << kChunkLog2;
        const uint64_t left = a.n - g0;
        const uint32_t valid = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
        const uint8_t* src = static_cast<const uint8_t*>(ptrs.grad[w]) + g0 * kElem;
        // rotated: coalesced order, dealt out through the buffer.  Unrotated bf16: thread t
        // loads its own 64 consecutive bytes (coordinates 32 t .. 32 t + 31).  Unrotated fp32
        // would be 128 bytes per thread, and the 16 waves of a CU would keep 128 KB of
        // half-used lines in a 32 KB vector cache: coalesced order as well.
        load_raw<kUnits, kElem, !ROTATE && BF16>(raw, src, valid, t);
    };
    if (kAhead) load(p0);
    for (uint64_t p = p0; p < a.chunks; p += dp) {
        const uint64_t g0 = p << kChunkLog2;
        const bool more = p + dp < a.chunks;
        float v[kRegs];
        if (!kAhead) load(p);
        if constexpr (ROTATE || !BF16) {
            __syncthreads();   // the previous item's last reads of the buffer and the table are done
            if (ROTATE) fill_sign_table<!BF16, BF16>(sh.sign[0], g0, a.key0, a.key1, t);
            raw_to_lds<kUnits>(sh, raw, t);
            __syncthreads();
            if (kAhead && more) load(p + dp);
            lds_to_l1<kUnits, ROTATE>(sh, sh.sign[0], v, t);
            if (ROTATE) rotate_l1_to_l3<true>(sh, v, lane, wave);
        } else {
            // y is the zero-padded gradient itself, already in the layout the quantizer wants
            units_to_l1<kUnits, false>(sh.sign[0], raw.u, v, t);
#pragma unroll
            for (int i = 0; i < kRegs; ++i) asm volatile("" : "+v"(v[i]));   // converted before `raw` is reloaded
            asm volatile("" ::: "memory");
            if (more) load(p + dp);
        }
        // this wave's share of the chunk's range, one word each for max and -min (so that
        // both are combined by a maximum), value in the rotation's normalised units
        MinMax r = thread_minmax(v);
        if (ROTATE) {
            r.lo *= kInvSqrtC;   // exact, and monotone: the order of min and scaling does not matter
            r.hi *= kInvSqrtC;
        }
        const uint32_t khi = wave_umax(order_key(r.hi));
        const uint32_t klo = wave_umax(order_key(-r.lo));
        if (lane == 0) {
            __hip_atomic_store(&a.slots[p * nwords + mine], khi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&a.slots[p * nwords + half + mine], klo, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
        if (ROTATE) l3_to_l4e<true>(sh, v, lane, wave);

        // wait for every wave of every worker of the chunk; bounded, as in encode_all_kernel
        const uint32_t* slot = a.slots + p * nwords;
        uint32_t mxh = 0u, mxl = 0u;
        bool done = false;
        __builtin_amdgcn_s_sleep(kFirstPollSleep);
        for (uint32_t spins = 0;; ++spins) {
            uint32_t all_valid = 1u;
            mxh = mxl = 0u;
            for (uint32_t base = 0; base < half; base += 64u) {
                const uint32_t i = base + lane;
                const bool in = i < half;
                const uint32_t vh = in ? __hip_atomic_load(&slot[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 1u;
                const uint32_t vl =
                    in ? __hip_atomic_load(&slot[half + i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 1u;
                all_valid &= (uint32_t)(vh != 0u && vl != 0u);
                if (in) {
                    mxh = vh > mxh ? vh : mxh;
                    mxl = vl > mxl ? vl : mxl;
                }
            }
            done = __all(all_valid != 0u);
            if (done || spins >= a.max_spins) break;
            __builtin_amdgcn_s_sleep(kPollSleep);
        }
        if (!done && lane == 0)
            __hip_atomic_store(a.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // The workspace leaves the kernel all zero: with every word of this chunk seen, no
        // peer will read the words of the workgroup's previous chunk again (a peer publishes
        // for this chunk only after all its waves have finished reading the previous one's
        // words, which the barriers of the rotation - or, without a rotation, the barrier
        // below - guarantee), and this wave clears its own two.
        if (done && prev != kNone && lane == 0) {
            __hip_atomic_store(&a.slots[(uint64_t)prev * nwords + mine], 0u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&a.slots[(uint64_t)prev * nwords + half + mine], 0u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        }
        prev = (uint32_t)p;
        // a timed-out wait may have seen no word at all: fall back to this wave's own range
        const uint32_t kh = wave_umax(mxh), kl = wave_umax(mxl);
        const float hi = order_value(kh > khi ? kh : khi);
        const float lo = -order_value(kl > klo ? kl : klo);
        if (w == 0 && t == 0) {
            a.scale[2 * p] = lo;
            a.scale[2 * p + 1] = hi;
        }
        quantize_store_range<BITS, ROTATE>(v, lo, hi, a.levels, g0, w, a.key0, a.key1, ptrs.payload[w], t);
        if (!ROTATE) __syncthreads();   // every wave has read this chunk's words before any publishes the next
    }
    // The workgroup's last chunk has no later chunk to vouch for it: the W workgroups of the
    // chunk count themselves off and the last one clears the chunk's words and the counter.
    __syncthreads();
    if (wave != 0) return;
    uint32_t arrived = 0u;
    if (lane == 0)
        arrived = __hip_atomic_fetch_add(&a.done[prev], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    arrived = (uint32_t)__builtin_amdgcn_readfirstlane((int)arrived);
    if (arrived == a.W - 1u) {
        uint32_t* words = a.slots + (uint64_t)prev * nwords;
        for (uint32_t i = lane; i < nwords; i += 64u)
            __hip_atomic_store(&words[i], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (lane == 0) __hip_atomic_store(&a.done[prev], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// out[g] = float(sum of the W indices of coordinate g) * (step / W) + lo, no rotation.
// A thread takes 8 consecutive coordinates: BITS bytes of every payload (a wave reads 64 BITS
// contiguous bytes per worker) and two 16-byte stores (a wave writes 2 KB contiguous).
template <int BITS>
__global__ __launch_bounds__(256) void unrotated_aggregate_decode_kernel(const FusedPayloadPtrs ptrs, uint32_t W,
                                                                         const float* range, uint32_t levels,
                                                                         uint64_t n, uint64_t groups, float* out) {
    const float Lf = (float)levels, Wf = (float)W;
    for (uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; k < groups;
         k += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t g = k * 8u;
        const uint64_t p = g >> kChunkLog2;
        const float lo = range[2 * p], hi = range[2 * p + 1];
        const float step = (hi - lo) / Lf;
        const float q = step / Wf;
        uint32_t S[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        for (uint32_t w = 0; w < W; ++w) {
            const uint8_t* src = ptrs.p[w] + k * BITS;
            if constexpr (BITS == 8) {
                const uint2 x = load_last_use(reinterpret_cast<const uint2*>(src));
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    S[e] += (x.x >> (8 * e)) & 0xFFu;
                    S[4 + e] += (x.y >> (8 * e)) & 0xFFu;
                }
            } else if constexpr (BITS == 4) {
                const uint32_t x = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(src));
#pragma unroll
                for (int e = 0; e < 8; ++e) S[e] += (x >> (4 * e)) & 0xFu;
            } else {
                const uint32_t x = __builtin_nontemporal_load(reinterpret_cast<const uint16_t*>(src));
#pragma unroll
                for (int e = 0; e < 8; ++e) S[e] += (x >> (2 * e)) & 0x3u;
            }
        }
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = (float)S[e] * q + lo;
        if (g + 8u <= n) {
            store_streaming(out + g, x[0], x[1], x[2], x[3]);
            store_streaming(out + g + 4, x[4], x[5], x[6], x[7]);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (g + e < n) out[g + e] = x[e];
        }
    }
}

template <auto kernel>
uint32_t resident_grid_minmax() {
    static uint32_t cached = 0;   // one per kernel
    if (cached == 0) {
        int occ = 0, dev = 0;
        hipDeviceProp_t prop;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, kThreads, 0) != hipSuccess || occ < 1) return 0;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
        cached = (uint32_t)(occ * prop.multiProcessorCount);
    }
    return cached;
}

template <bool BF16, int BITS, bool ROTATE>
hipError_t launch_minmax_t(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, hipStream_t stream) {
    uint32_t G = resident_grid_minmax<encode_all_minmax_kernel<BF16, BITS, ROTATE>>();
    if (G == 0) return hipErrorInvalidValue;
    const uint64_t total = a.chunks * a.W;
    if (G > total) G = (uint32_t)total;
    // the W workgroups of a chunk wait for one another: all of them must be resident
    if (G < a.W) return hipErrorInvalidConfiguration;
    G -= G % a.W;
    hipLaunchKernelGGL((encode_all_minmax_kernel<BF16, BITS, ROTATE>), dim3(G), dim3(kThreads), 0, stream, a, ptrs);
    return hipGetLastError();
}

template <bool BF16, bool ROTATE>
hipError_t launch_minmax_bits(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, uint32_t bits, hipStream_t stream) {
    if (bits == 2) return launch_minmax_t<BF16, 2, ROTATE>(a, ptrs, stream);
    if (bits == 4) return launch_minmax_t<BF16, 4, ROTATE>(a, ptrs, stream);
    return launch_minmax_t<BF16, 8, ROTATE>(a, ptrs, stream);
}

}  // namespace
}  // namespace k14

uint32_t encode_all_minmax_slot_words(uint32_t W) { return 2u * k14::kWaves * W; }

hipError_t launch_encode_all_minmax(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, bool bf16, bool rotate,
                                    uint32_t bits, hipStream_t stream) {
    if (a.chunks == 0) return hipSuccess;
    if (bf16) return rotate ? k14::launch_minmax_bits<true, true>(a, ptrs, bits, stream)
                            : k14::launch_minmax_bits<true, false>(a, ptrs, bits, stream);
    return rotate ? k14::launch_minmax_bits<false, true>(a, ptrs, bits, stream)
                  : k14::launch_minmax_bits<false, false>(a, ptrs, bits, stream);
}

hipError_t launch_unrotated_aggregate_decode(const FusedPayloadPtrs& ptrs, uint32_t W, const float* range,
                                             uint32_t bits, uint64_t n, float* out, hipStream_t stream) {
    const uint64_t groups = (n + 7u) / 8u;
    if (groups == 0) return hipSuccess;
    uint64_t blocks = (groups + 255u) / 256u;
    if (blocks > 256u * 16u) blocks = 256u * 16u;
    const dim3 grid((uint32_t)blocks), block(256);
    const uint32_t levels = grid_levels(bits, false);
    if (bits == 2)
        hipLaunchKernelGGL(k14::unrotated_aggregate_decode_kernel<2>, grid, block, 0, stream, ptrs, W, range, levels,
                           n, groups, out);
    else if (bits == 4)
        hipLaunchKernelGGL(k14::unrotated_aggregate_decode_kernel<4>, grid, block, 0, stream, ptrs, W, range, levels,
                           n, groups, out);
    else
        hipLaunchKernelGGL(k14::unrotated_aggregate_decode_kernel<8>, grid, block, 0, stream, ptrs, W, range, levels,
                           n, groups, out);
    return hipGetLastError();
}

}  // namespace thc
