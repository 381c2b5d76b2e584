// One-pass kernels of the min/max-range variant for chunk_log2 = 14 that have no counterpart
// in thc_fused14.hip (with the rotation the variant runs in that file's encode_all_kernel and
// aggregate_decode_kernel, compiled for the min/max grid).
//
// encode_all_unrotated: a work item is (chunk p, worker w).  The workgroup that owns it brings
// the chunk into registers as it is, publishes its (min, max) to per-chunk words in global
// memory, waits until all W workers of the chunk have published, and quantizes onto the
// shared range - every gradient is read from HBM once (the one-call-per-step form reads it
// twice).  Grid, item order, bounded waits and the self-clearing workspace follow
// encode_all_kernel, with two words per wave.  Two kernels: one item at a time with one
// polling wave per workgroup (fp32 input, odd bf16 counts), and for bf16 input a pipeline
// that publishes an item's range one item before it waits for it.
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
// lo and hi are the chunk's own extremes over all workers: fl(y - lo) <= fl(hi - lo) and
// (hi - lo) * fl(L / (hi - lo)) <= L (1 + 2^-24), so t < L + 255.5/256 + L 2^-24 < L + 1 and
// the minimum with L never binds
constexpr bool kClampRanged = false;

// ---- the range words of a chunk: one 8-byte pair per wave of every worker's workgroup,
// (key of the maximum) << 32 | key of the negated minimum (so that both are combined by a
// maximum).  An aligned 8-byte store is one transaction: a reader sees both keys or neither.
struct Words {
    const EncodeAllArgs& a;
    uint32_t half;     // pairs per chunk
    uint32_t nwords;   // 2 * half 32-bit words
    uint32_t mine;     // this wave's pair
    uint32_t lane;

    __device__ __forceinline__ uint64_t* pairs(uint64_t p) const {
        return reinterpret_cast<uint64_t*>(a.slots + p * nwords);
    }
    __device__ __forceinline__ void publish(uint64_t p, uint32_t khi, uint32_t klo) const {
        if (lane == 0)
            __hip_atomic_store(pairs(p) + mine, ((uint64_t)khi << 32) | klo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // Waits until every wave of every worker of chunk p has published; bounded by
    // a.max_spins polls, after which the error word is set and the wave carries on with
    // what it has seen and its own range (khi, klo).  Returns the keys of (hi, -lo).
    template <bool SLEEP_FIRST = true>
    __device__ __forceinline__ bool wait(uint64_t p, uint32_t& khi, uint32_t& klo) const {
        const uint64_t* pair = pairs(p);
        uint32_t mxh = 0u, mxl = 0u;
        bool done = false;
        if (SLEEP_FIRST) __builtin_amdgcn_s_sleep(kFirstPollSleep);
        for (uint32_t spins = 0;; ++spins) {
            uint32_t all_valid = 1u;
            mxh = mxl = 0u;
            for (uint32_t base = 0; base < half; base += 64u) {
                const uint32_t i = base + lane;
                if (i < half) {
                    const uint64_t v = __hip_atomic_load(&pair[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const uint32_t vh = (uint32_t)(v >> 32), vl = (uint32_t)v;
                    all_valid &= (uint32_t)(v != 0ull);   // (neither key is ever zero)
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
        const uint32_t kh = wave_umax(mxh), kl = wave_umax(mxl);
        khi = kh > khi ? kh : khi;
        klo = kl > klo ? kl : klo;
        return done;
    }
    // This wave's pair of an earlier chunk back to zero.
    __device__ __forceinline__ void clear_mine(uint32_t chunk) const {
        if (lane == 0) __hip_atomic_store(pairs(chunk) + mine, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // A workgroup's last chunks have no later chunk to vouch for them: the W workgroups of the
    // chunk count themselves off and the last one clears all its words and the counter.  Called
    // by one wave, after a barrier behind the workgroup's last read of the words.
    __device__ __forceinline__ void count_off(uint32_t chunk) const {
        uint32_t arrived = 0u;
        if (lane == 0)
            arrived = __hip_atomic_fetch_add(&a.done[chunk], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        arrived = (uint32_t)__builtin_amdgcn_readfirstlane((int)arrived);
        if (arrived == a.W - 1u) {
            uint32_t* words = a.slots + (uint64_t)chunk * nwords;
            for (uint32_t i = lane; i < nwords; i += 64u)
                __hip_atomic_store(&words[i], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (lane == 0) __hip_atomic_store(&a.done[chunk], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
};

// "no chunk"
constexpr uint32_t kNone = 0xFFFFFFFFu;

// Without the rotation: y is the zero-padded gradient itself, already in the layout the
// quantizer wants.  An item has nothing to do between publishing its range and reading its
// peers', so the time the words take to travel is exposed; what hides it is more workgroups
// per CU: the bf16 form needs no LDS at all and is compiled for three workgroups per CU
// (85 registers) instead of two.  This kernel serves fp32 input and bf16 input with an odd
// number of coordinates; bf16 input otherwise takes the pipelined kernel below.
template <bool BF16, int BITS>
__global__ __launch_bounds__(kThreads, BF16 ? 6 : kWavesPerSimd) void encode_all_unrotated_kernel(
    const EncodeAllArgs a, const FusedWorkerPtrs ptrs) {
    __shared__ Shared sh;   // fp32 only (the bf16 form never touches it, so it is not allocated)
    __shared__ uint32_t bcast[3];
    constexpr int kUnits = BF16 ? 4 : 8;
    constexpr int kElem = BF16 ? 2 : 4;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t p0 = blockIdx.x / a.W;
    const uint32_t w = blockIdx.x - p0 * a.W;
    const uint32_t dp = gridDim.x / a.W;
    const Words words{a, kWaves * a.W, 2u * kWaves * a.W, kWaves * w + wave, lane};
    if (p0 >= a.chunks) return;
    // bf16: thread t loads its own 64 consecutive bytes (coordinates 32 t .. 32 t + 31), an
    // item ahead.  fp32 would be 128 bytes per thread, and the 16 waves of a CU would keep
    // 128 KB of half-used lines in a 32 KB vector cache: coalesced order, dealt out through
    // the buffer, loaded when the item starts.
    Raw<kUnits> raw;
    auto load = [&](uint64_t p) {
        const uint64_t g0 = p << kChunkLog2;
        const uint64_t left = a.n - g0;
        const uint32_t valid = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
        load_raw<kUnits, kElem, BF16>(raw, static_cast<const uint8_t*>(ptrs.grad[w]) + g0 * kElem, valid, t);
    };
    if (BF16) load(p0);
    uint32_t prev = kNone;
    for (uint64_t p = p0; p < a.chunks; p += dp) {
        float v[kRegs];
        if constexpr (BF16) {
            units_to_l1<kUnits, false>(sh.sign[0], raw.u, v, t);
            // the conversion is complete before the registers of `raw` are loaded again
#pragma unroll
            for (int i = 0; i < kRegs; ++i) asm volatile("" : "+v"(v[i]));
            asm volatile("" ::: "memory");
            if (p + dp < a.chunks) load(p + dp);
        } else {
            load(p);
            raw_to_lds<kUnits>(sh, raw, t);
            __syncthreads();
            lds_to_l1<kUnits, false>(sh, sh.sign[0], v, t);
        }
        const MinMax m = thread_minmax(v);
        uint32_t khi = wave_umax(order_key(m.hi));
        uint32_t klo = wave_umax(order_key(-m.lo));
        words.publish(p, khi, klo);
        // One wave polls for the workgroup.  Without a rotation the waves would spend most of
        // an item polling, eight of them per workgroup, and that traffic (uncached reads served
        // at the memory side) delays the very words it is waiting for.
        if (wave == 0) {
            const bool ok = words.wait(p, khi, klo);
            if (lane == 0) {
                bcast[0] = khi;
                bcast[1] = klo;
                bcast[2] = ok ? 1u : 0u;
            }
        }
        __syncthreads();
        khi = bcast[0];
        klo = bcast[1];
        const bool done = bcast[2] != 0u;
        // as in the rotated kernel; the barrier that lets a peer conclude that this workgroup
        // has finished with the previous chunk's words is the one at the end of the item
        if (done && prev != kNone) words.clear_mine(prev);
        prev = (uint32_t)p;
        const float hi = order_value(khi), lo = -order_value(klo);
        if (w == 0 && t == 0) {
            a.scale[2 * p] = lo;
            a.scale[2 * p + 1] = hi;
        }
        quantize_store_range<BITS, false, kClampRanged>(v, lo, hi, a.levels, p << kChunkLog2, w, a.key0, a.key1, ptrs.payload[w], t);
        __syncthreads();   // every wave has read this chunk's words (and the buffer) before the next item
    }
    if (wave == 0) words.count_off(prev);   // behind the barrier that ended the last item
}

// A thread's 32 consecutive bf16 coordinates (four 16-byte units) as fp32 values.
__device__ __forceinline__ void widen_bf16(const uint4 (&unit)[4], float (&v)[kRegs]) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint32_t x[4] = {unit[k].x, unit[k].y, unit[k].z, unit[k].w};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            v[8 * k + 2 * d] = __uint_as_float(x[d] << 16);
            v[8 * k + 2 * d + 1] = __uint_as_float(x[d] & 0xFFFF0000u);
        }
    }
}

// The bf16 form of the same, as a pipeline three items deep.  A thread's 32 coordinates are
// 16 registers while they stay packed, so a wave can hold the item it quantizes, the next
// one (whose range it has already published) and the loads of the one after that: by the
// time an item is quantized its peers' words were published a whole item ago and the wait
// is one read.  No LDS and no barrier: every wave publishes, polls and clears for itself.
// A wave that has seen all words of item k knows that every wave of every peer has
// published k, which a wave does after its wait for item k - 2: nobody reads the words of
// k - 2 again, and the wave clears its own.  The last two items of a workgroup are counted
// off by the workgroups of their chunks as in the other kernels.
template <int BITS>
__global__ __launch_bounds__(kThreads, kWavesPerSimd) void encode_all_unrotated_bf16_kernel(
    const EncodeAllArgs a, const FusedWorkerPtrs ptrs) {
    constexpr int kUnits = 4;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t p0 = blockIdx.x / a.W;
    const uint32_t w = blockIdx.x - p0 * a.W;
    const uint32_t dp = gridDim.x / a.W;
    const Words words{a, kWaves * a.W, 2u * kWaves * a.W, kWaves * w + wave, lane};
    if (p0 >= a.chunks) return;
    // Through a buffer descriptor whose range is the part of the chunk that exists (n is even:
    // the range check works on dwords): reads beyond it return zero, and a chunk past the end
    // has range 0, so the loads are unconditional.
    auto load = [&](Raw<kUnits>& raw, uint64_t p) {
        const uint64_t g0 = p << kChunkLog2;
        uint64_t left = p < a.chunks ? a.n - g0 : 0u;
        if (left > (uint64_t)kChunk) left = kChunk;
        uint64_t addr = reinterpret_cast<uint64_t>(ptrs.grad[w]) + (p < a.chunks ? g0 * 2u : 0u);
        addr = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(addr >> 32)) << 32) |
               (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)addr);
        __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(addr), 0, (uint32_t)left * 2u, 0x00020000);
        typedef uint32_t u4v __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int j = 0; j < kUnits; ++j) {
            const u4v q = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (kUnits * t + j) * 16u, 0, 0);
            raw.u[j] = make_uint4(q.x, q.y, q.z, q.w);
        }
    };
    // this wave's share of the item's range, published
    auto announce = [&](const Raw<kUnits>& raw, uint64_t p, uint32_t& khi, uint32_t& klo) {
        float v[kRegs];
        widen_bf16(raw.u, v);
        const MinMax m = thread_minmax(v);
        khi = wave_umax(order_key(m.hi));
        klo = wave_umax(order_key(-m.lo));
        words.publish(p, khi, klo);
    };
    Raw<kUnits> r0, r1, r2;
    load(r0, p0);
    load(r1, (uint64_t)p0 + dp);
    uint32_t khi, klo, nhi = 0u, nlo = 0u;
    announce(r0, p0, khi, klo);
    uint32_t prev1 = kNone, prev2 = kNone;
    // One item: `cur` holds item p, `next` item p + dp (in flight since the item before),
    // `far` is free and receives item p + 2 dp.
    auto item = [&](Raw<kUnits>& cur, Raw<kUnits>& next, Raw<kUnits>& far, uint64_t p) {
        if (p + dp < a.chunks) announce(next, p + dp, nhi, nlo);
        const bool done = words.wait<false>(p, khi, klo);
        // (after the wait: vector-memory operations complete in order, so a load issued before
        // the read of the words would have to arrive before that read is seen)
        load(far, p + 2u * dp);
        if (done && prev2 != kNone) words.clear_mine(prev2);
        prev2 = prev1;
        prev1 = (uint32_t)p;
        const float hi = order_value(khi), lo = -order_value(klo);
        if (w == 0 && t == 0) {
            a.scale[2 * p] = lo;
            a.scale[2 * p + 1] = hi;
        }
        float v[kRegs];
        widen_bf16(cur.u, v);
        quantize_store_range<BITS, false, kClampRanged>(v, lo, hi, a.levels, p << kChunkLog2, w, a.key0, a.key1, ptrs.payload[w], t);
        khi = nhi;
        klo = nlo;
    };
    // (three items per trip so that the register sets take turns without copies: a copy of a
    // set whose loads are in flight would wait for them)
    for (uint64_t p = p0; p < a.chunks;) {
        item(r0, r1, r2, p);
        p += dp;
        if (p >= a.chunks) break;
        item(r1, r2, r0, p);
        p += dp;
        if (p >= a.chunks) break;
        item(r2, r0, r1, p);
        p += dp;
    }
    __syncthreads();   // every wave has read the words of the last two items
    if (wave == 0) {
        if (prev2 != kNone) words.count_off(prev2);
        words.count_off(prev1);
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
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    // the payload bytes of 8 coordinates of one worker, as one register pair
    auto fetch = [&](uint32_t w, uint64_t k) -> uint2 {
        const uint8_t* src = ptrs.p[w] + k * BITS;
        if constexpr (BITS == 8) return load_last_use(reinterpret_cast<const uint2*>(src));
        else if constexpr (BITS == 4) return make_uint2(__builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(src)), 0u);
        else return make_uint2(__builtin_nontemporal_load(reinterpret_cast<const uint16_t*>(src)), 0u);
    };
    auto add = [&](uint32_t (&S)[8], const uint2 x) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if constexpr (BITS == 8) S[e] += ((e < 4 ? x.x : x.y) >> (8 * (e & 3))) & 0xFFu;
            else if constexpr (BITS == 4) S[e] += (x.x >> (4 * e)) & 0xFu;
            else S[e] += (x.x >> (2 * e)) & 0x3u;
        }
    };
    auto finish = [&](const uint32_t (&S)[8], uint64_t k) {
        const uint64_t g = k * 8u;
        const uint64_t p = g >> kChunkLog2;
        const float lo = range[2 * p], hi = range[2 * p + 1];
        const float step = (hi - lo) / Lf;
        const float q = step / Wf;
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
    };
    // two groups a grid apart per trip: twice the loads in flight, every access still coalesced
    uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; k + stride < groups; k += 2u * stride) {
        uint32_t S0[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u}, S1[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        for (uint32_t w = 0; w < W; ++w) {
            const uint2 a0 = fetch(w, k), a1 = fetch(w, k + stride);
            add(S0, a0);
            add(S1, a1);
        }
        finish(S0, k);
        finish(S1, k + stride);
    }
    if (k < groups) {
        uint32_t S0[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        for (uint32_t w = 0; w < W; ++w) add(S0, fetch(w, k));
        finish(S0, k);
    }
}

// The same estimate from stored sums (thc_decode_minmax without rotation), any chunk size:
// out[g] = float(S_g) * (step / W) + lo.  8 coordinates per thread: one 8- or 16-byte load,
// 32 (fp32) or 16 (bf16) bytes stored.  bf16: round to nearest, ties to even.
template <typename SUM, bool OUT_BF16>
__global__ __launch_bounds__(256) void unrotated_decode_kernel(const SUM* sums, const float* range, uint32_t W,
                                                               uint32_t levels, uint32_t chunk_log2, uint64_t n,
                                                               uint64_t groups, void* out) {
    const float Lf = (float)levels, Wf = (float)W;
    for (uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; k < groups;
         k += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t g = k * 8u;
        uint32_t S[8];
        if constexpr (sizeof(SUM) == 1) {
            const uint2 x = load_last_use(reinterpret_cast<const uint2*>(sums + g));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                S[e] = (x.x >> (8 * e)) & 0xFFu;
                S[4 + e] = (x.y >> (8 * e)) & 0xFFu;
            }
        } else {
            const uint4 x = load_last_use(reinterpret_cast<const uint4*>(sums + g));
            const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) S[e] = (w[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
        }
        float x[8];
        if (chunk_log2 >= 3u) {   // the 8 coordinates share a chunk
            const uint64_t p = g >> chunk_log2;
            const float lo = range[2 * p], hi = range[2 * p + 1];
            const float q = ((hi - lo) / Lf) / Wf;
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = (float)S[e] * q + lo;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint64_t p = (g + e) >> chunk_log2;
                const float lo = range[2 * p], hi = range[2 * p + 1];
                x[e] = (float)S[e] * (((hi - lo) / Lf) / Wf) + lo;
            }
        }
        if constexpr (OUT_BF16) {
            uint16_t* dst = static_cast<uint16_t*>(out) + g;
            uint32_t h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t u = __float_as_uint(x[e]);
                h[e] = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
            }
            if (g + 8u <= n) {
                *reinterpret_cast<uint4*>(dst) =
                    make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (g + e < n) dst[e] = (uint16_t)h[e];
            }
        } else {
            float* dst = static_cast<float*>(out) + g;
            if (g + 8u <= n) {
                store_streaming(dst, x[0], x[1], x[2], x[3]);
                store_streaming(dst + 4, x[4], x[5], x[6], x[7]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (g + e < n) dst[e] = x[e];
            }
        }
    }
}

// Largest grid of the decoder for stored sums, in blocks of 256 threads (131 MB moved per
// bucket: 4096 blocks 32.4 us, 16384 blocks 29.2 us, 65536 blocks 28.8 us).
constexpr uint64_t kElementwiseBlocks = 16384;

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

template <bool BF16, int BITS>
hipError_t launch_unrotated_t(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, hipStream_t stream) {
    if (BF16 && (a.n & 1u) == 0u) {
        uint32_t G = resident_grid_minmax<encode_all_unrotated_bf16_kernel<BITS>>();
        if (G == 0) return hipErrorInvalidValue;
        const uint64_t total = a.chunks * a.W;
        if (G > total) G = (uint32_t)total;
        if (G < a.W) return hipErrorInvalidConfiguration;
        G -= G % a.W;
        hipLaunchKernelGGL((encode_all_unrotated_bf16_kernel<BITS>), dim3(G), dim3(kThreads), 0, stream, a, ptrs);
        return hipGetLastError();
    }
    uint32_t G = resident_grid_minmax<encode_all_unrotated_kernel<BF16, BITS>>();
    if (G == 0) return hipErrorInvalidValue;
    const uint64_t total = a.chunks * a.W;
    if (G > total) G = (uint32_t)total;
    // the W workgroups of a chunk wait for one another: all of them must be resident
    if (G < a.W) return hipErrorInvalidConfiguration;
    G -= G % a.W;
    hipLaunchKernelGGL((encode_all_unrotated_kernel<BF16, BITS>), dim3(G), dim3(kThreads), 0, stream, a, ptrs);
    return hipGetLastError();
}

template <bool BF16>
hipError_t launch_unrotated_bits(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, uint32_t bits,
                                 hipStream_t stream) {
    if (bits == 2) return launch_unrotated_t<BF16, 2>(a, ptrs, stream);
    if (bits == 4) return launch_unrotated_t<BF16, 4>(a, ptrs, stream);
    return launch_unrotated_t<BF16, 8>(a, ptrs, stream);
}

}  // namespace
}  // namespace k14

uint32_t encode_all_minmax_slot_words(uint32_t W) { return 2u * k14::kWaves * W; }

hipError_t launch_encode_all_minmax(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, bool bf16, bool rotate,
                                    uint32_t bits, hipStream_t stream) {
    if (a.chunks == 0) return hipSuccess;
    // with the rotation: the kernel of thc_encode_all, compiled for the min/max grid
    if (rotate) return launch_encode_all_ranged(a, ptrs, bf16, bits, stream);
    return bf16 ? k14::launch_unrotated_bits<true>(a, ptrs, bits, stream)
                : k14::launch_unrotated_bits<false>(a, ptrs, bits, stream);
}

hipError_t launch_unrotated_aggregate_decode(const FusedPayloadPtrs& ptrs, uint32_t W, const float* range,
                                             uint32_t bits, uint64_t n, float* out, hipStream_t stream) {
    const uint64_t groups = (n + 7u) / 8u;
    if (groups == 0) return hipSuccess;
    uint64_t blocks = (groups + 255u) / 256u;
    if (blocks > 4096u) blocks = 4096u;   // (two groups per trip; 16384 blocks: 53.7 against 48 us)
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

// Tuned form of the unrotated thc_decode_minmax: sums, range and out as for that call; `out`
// 16-byte aligned.  The sums buffer holds whole chunks, so groups of 8 never run past it
// (chunks of fewer than 8 coordinates: the padded size is still a multiple of 8 only if
// chunks * c is; the caller checks).
hipError_t launch_unrotated_decode(const void* sums, uint32_t sum_bytes, const float* range, uint32_t W,
                                   uint32_t bits, uint32_t chunk_log2, uint64_t n, bool out_bf16, void* out,
                                   hipStream_t stream) {
    const uint64_t groups = (n + 7u) / 8u;
    if (groups == 0) return hipSuccess;
    uint64_t blocks = (groups + 255u) / 256u;
    if (blocks > k14::kElementwiseBlocks) blocks = k14::kElementwiseBlocks;
    const dim3 grid((uint32_t)blocks), block(256);
    const uint32_t levels = grid_levels(bits, false);
#define THC_UNROT(T, B)                                                                                      \
    hipLaunchKernelGGL((k14::unrotated_decode_kernel<T, B>), grid, block, 0, stream, static_cast<const T*>(sums), \
                       range, W, levels, chunk_log2, n, groups, out)
    if (sum_bytes == 1) {
        if (out_bf16) THC_UNROT(uint8_t, true);
        else THC_UNROT(uint8_t, false);
    } else {
        if (out_bf16) THC_UNROT(uint16_t, true);
        else THC_UNROT(uint16_t, false);
    }
#undef THC_UNROT
    return hipGetLastError();
}

}  // namespace thc
