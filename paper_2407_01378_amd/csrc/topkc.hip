// TopK Chunked (TopKC): per-chunk squared norms in half precision, their sum over workers,
// selection of the J chunks with the largest sums, and the fp16 sum of the selected chunks
// ("Our proposed improvement: Chunks" of the paper's TopK case study).  Everything here is
// a streaming scan; the only part that is not elementwise is the selection, a two-pass
// radix select over the 16-bit keys followed by an ordered compaction.
#include <hip/hip_fp16.h>

#include "thc_device.h"
#include "thc_internal.h"

#pragma clang fp contract(off)

namespace thc {
namespace {

// fp32 -> fp16 bits, round to nearest even (subnormals kept, overflow to inf).
__device__ __forceinline__ uint32_t f32_to_f16_bits(float x) {
    return (uint32_t)__half_as_ushort(__float2half_rn(x));
}
__device__ __forceinline__ float f16_bits_to_f32(uint32_t h) {
    return __half2float(__ushort_as_half((unsigned short)h));
}
// fp16 + fp16 -> fp16: the fp32 sum of two fp16 numbers is exact, so one rounding.
__device__ __forceinline__ uint32_t add_f16_bits(uint32_t a, uint32_t b) {
    return f32_to_f16_bits(f16_bits_to_f32(a) + f16_bits_to_f32(b));
}

// 8 consecutive coordinates starting at g (a multiple of 8), widened to fp32; zeros past n.
template <bool BF16>
__device__ __forceinline__ void load8(const void* grad, uint64_t g, uint64_t n, float (&x)[8]) {
    if (g + 8u <= n) {
        if (BF16) {
            const uint4 q = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(grad) + g);
            const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                x[2 * d] = __uint_as_float(w[d] << 16);
                x[2 * d + 1] = __uint_as_float(w[d] & 0xFFFF0000u);
            }
        } else {
            const float4 a = *reinterpret_cast<const float4*>(static_cast<const float*>(grad) + g);
            const float4 b = *reinterpret_cast<const float4*>(static_cast<const float*>(grad) + g + 4);
            x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
            x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = 0.0f;
            if (g + e < n)
                v = BF16 ? bf16_bits_to_float(static_cast<const uint16_t*>(grad)[g + e])
                         : static_cast<const float*>(grad)[g + e];
            x[e] = v;
        }
    }
}

// Squared norm of every chunk of C = 8 * lanes_per_chunk coordinates: squares in fp32,
// summed as a balanced tree over adjacent pairs (inside the thread, then across lanes
// 1, 2, 4, ... apart), rounded to fp16.  Group k (8 coordinates) belongs to thread k mod T of
// a grid of T threads; a thread takes four groups T apart per trip, loaded before any is
// used (streaming loads, the gradient is read once), so a wave keeps 4 KB in flight.  T is a
// multiple of 64 and the loop bounds are too: the lanes of a wave stay together, which the
// lane exchanges need.
template <bool BF16>
__device__ __forceinline__ void raw8(const void* grad, uint64_t g, uint64_t n, uint4 (&q)[2]) {
    // whole groups only; BF16: one 16-byte unit, fp32: two
    if (BF16) {
        q[0] = load_last_use(reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(grad) + g));
    } else {
        q[0] = load_last_use(reinterpret_cast<const uint4*>(static_cast<const float*>(grad) + g));
        q[1] = load_last_use(reinterpret_cast<const uint4*>(static_cast<const float*>(grad) + g + 4));
    }
}
template <bool BF16>
__device__ __forceinline__ void widen8(const uint4 (&q)[2], float (&x)[8]) {
    if (BF16) {
        const uint32_t w[4] = {q[0].x, q[0].y, q[0].z, q[0].w};
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            x[2 * d] = __uint_as_float(w[d] << 16);
            x[2 * d + 1] = __uint_as_float(w[d] & 0xFFFF0000u);
        }
    } else {
        const uint32_t w[8] = {q[0].x, q[0].y, q[0].z, q[0].w, q[1].x, q[1].y, q[1].z, q[1].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = __uint_as_float(w[e]);
    }
}
__device__ __forceinline__ void norm_of_group(const float (&x)[8], uint64_t k, uint64_t groups,
                                              uint32_t lanes_per_chunk, uint16_t* norms) {
    float s[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) s[e] = x[e] * x[e];
    float t = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
    for (uint32_t o = 1; o < lanes_per_chunk; o <<= 1) t = t + __shfl_xor(t, (int)o, 64);
    if (k < groups && (k & (uint64_t)(lanes_per_chunk - 1u)) == 0)
        norms[k / lanes_per_chunk] = (uint16_t)f32_to_f16_bits(t);
}
template <bool BF16>
__global__ __launch_bounds__(256) void norms_kernel(const void* grad, uint64_t n, uint32_t lanes_per_chunk,
                                                    uint64_t groups, uint16_t* norms) {
    const uint64_t T = (uint64_t)gridDim.x * blockDim.x;
    const uint64_t whole = (n / 8u) & ~63ull;   // groups below this are complete, in complete waves
    uint64_t k = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; k - (k & 63u) + 3u * T + 64u <= whole; k += 4u * T) {
        uint4 q[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u) raw8<BF16>(grad, (k + u * T) * 8u, n, q[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float x[8];
            widen8<BF16>(q[u], x);
            norm_of_group(x, k + u * T, groups, lanes_per_chunk, norms);
        }
    }
    // the rest, a group per trip, with the element-wise loader where the gradient ends
    const uint64_t bound = (groups + 63u) & ~63ull;
    for (; k < bound; k += T) {
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = 0.0f;
        if (k < groups) load8<BF16>(grad, k * 8u, n, x);
        norm_of_group(x, k, groups, lanes_per_chunk, norms);
    }
}

// s_p = fp16 sum over workers, in worker order, of norms_all[w * P + p].
__global__ __launch_bounds__(256) void sum_norms_kernel(const uint16_t* norms_all, uint32_t W, uint64_t P,
                                                        uint16_t* s) {
    const uint64_t p = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    uint32_t acc = norms_all[p];
    for (uint32_t w = 1; w < W; ++w) acc = add_f16_bits(acc, norms_all[(uint64_t)w * P + p]);
    s[p] = (uint16_t)acc;
}
// The same, four chunks per thread through 8-byte loads (P a multiple of 4, both arrays
// 8-byte aligned: then every worker's row is too).
__global__ __launch_bounds__(256) void sum_norms4_kernel(const uint16_t* norms_all, uint32_t W, uint64_t P,
                                                         uint16_t* s) {
    const uint64_t q = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;   // chunks 4 q .. 4 q + 3
    if (q * 4u >= P) return;
    uint32_t acc[4];
    for (uint32_t w = 0; w < W; ++w) {
        const uint2 x = load_last_use(reinterpret_cast<const uint2*>(norms_all + (uint64_t)w * P) + q);
        const uint32_t h[4] = {x.x & 0xFFFFu, x.x >> 16, x.y & 0xFFFFu, x.y >> 16};
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = w == 0 ? h[e] : add_f16_bits(acc[e], h[e]);
    }
    reinterpret_cast<uint2*>(s)[q] = make_uint2(acc[0] | (acc[1] << 16), acc[2] | (acc[3] << 16));
}

// ---- selection -----------------------------------------------------------------------------
// Workspace words: [0,256) histogram of the keys' high bytes, [256,512) histogram of the
// low bytes inside the threshold bucket, [512] threshold bucket, [513] still to take
// inside it, [514] threshold key T, [515] how many keys equal to T are taken, then per
// segment of kSegment keys the pair (keys above T, keys equal to T), scanned in place.
constexpr uint32_t kSegment = 2048;
constexpr uint32_t kHdr = 516;

// PASS 0: histogram of key >> 8.  PASS 1: of key & 255 among keys with key >> 8 == ws[512].
// VEC (s 16-byte aligned): a thread takes 8 consecutive keys per load and adds runs of equal
// bins with one LDS atomic each (norms that underflow to zero, or lie in one bucket, come in
// runs); the keys past the last whole group of 8 are left to the first block.
template <int PASS, bool VEC>
__global__ __launch_bounds__(256) void hist_kernel(const uint16_t* s, uint64_t P, uint32_t* ws) {
    __shared__ uint32_t h[256];
    h[threadIdx.x] = 0u;
    __syncthreads();
    const uint32_t bucket = PASS == 1 ? ws[512] : 0u;
    auto bin_of = [&](uint32_t key) -> int {
        if (PASS == 0) return (int)(key >> 8);
        return (key >> 8) == bucket ? (int)(key & 255u) : -1;
    };
    const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    if (VEC) {
        const uint64_t groups = P / 8u;
        for (uint64_t g = tid; g < groups; g += stride) {
            const uint4 q = load_last_use(reinterpret_cast<const uint4*>(s) + g);
            const uint32_t w[4] = {q.x, q.y, q.z, q.w};
            int cur = -1;
            uint32_t cnt = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int b = bin_of((w[e >> 1] >> (16 * (e & 1))) & 0xFFFFu);
                if (b != cur) {
                    if (cur >= 0) atomicAdd(&h[cur], cnt);
                    cur = b;
                    cnt = 1u;
                } else {
                    ++cnt;
                }
            }
            if (cur >= 0) atomicAdd(&h[cur], cnt);
        }
        if (blockIdx.x == 0 && groups * 8u + threadIdx.x < P) {   // fewer than 8 keys
            const int b = bin_of(s[groups * 8u + threadIdx.x]);
            if (b >= 0) atomicAdd(&h[b], 1u);
        }
    } else {
        for (uint64_t p = tid; p < P; p += stride) {
            const int b = bin_of(s[p]);
            if (b >= 0) atomicAdd(&h[b], 1u);
        }
    }
    __syncthreads();
    const uint32_t c = h[threadIdx.x];
    if (c) atomicAdd(&ws[256 * PASS + threadIdx.x], c);
}

// One wave walks the 256-bin histogram from the top: the largest bin b whose count together
// with the counts above it reaches `want` (bin 0 if none does), and the count above it.
// PASS 0: finds the bucket in which the J-th largest key lies.  PASS 1: finds the key itself
// and how many of its equals to take.  Lane i holds bins 4 i .. 4 i + 3.
template <int PASS>
__global__ __launch_bounds__(64) void find_kernel(uint32_t* ws, uint32_t J) {
    if (blockIdx.x != 0) return;
    const uint32_t lane = threadIdx.x;
    const uint32_t want = PASS == 0 ? J : ws[513];
    const uint32_t* bins = ws + 256 * PASS + 4u * lane;   // (the workspace is only 4-byte aligned)
    const uint4 c = make_uint4(bins[0], bins[1], bins[2], bins[3]);
    const uint32_t tot = c.x + c.y + c.z + c.w;
    uint32_t suf = tot;   // -> this lane's bins and all above them
    for (uint32_t o = 1; o < 64u; o <<= 1) {
        const uint32_t y = __shfl_down(suf, o, 64);
        if (lane + o < 64u) suf += y;
    }
    const uint32_t s4 = suf - tot;   // everything above bin 4 lane + 3
    const uint32_t s3 = s4 + c.w, s2 = s3 + c.z, s1 = s2 + c.y, s0 = s1 + c.x;
    int best = -1;
    uint32_t above = 0;
    if (s3 >= want) { best = 3; above = s4; }
    else if (s2 >= want) { best = 2; above = s3; }
    else if (s1 >= want) { best = 1; above = s2; }
    else if (s0 >= want) { best = 0; above = s1; }
    const unsigned long long found = __ballot(best >= 0);
    uint32_t b = 0, ab = __shfl(s1, 0, 64);   // nothing reaches `want`: bin 0, as the walk from the top would end
    if (found != 0ull) {
        const int winner = 63 - __builtin_clzll(found);
        b = 4u * (uint32_t)winner + (uint32_t)__shfl(best, winner, 64);
        ab = __shfl(above, winner, 64);
    }
    if (lane == 0) {
        if (PASS == 0) {
            ws[512] = b;
            ws[513] = want - ab;          // still to take inside bucket b (>= 1)
        } else {
            ws[514] = (ws[512] << 8) | b;
            ws[515] = want - ab;          // keys equal to T that are taken (>= 1)
        }
    }
}

__global__ __launch_bounds__(256) void seg_count_kernel(const uint16_t* s, uint64_t P, uint32_t* ws) {
    __shared__ uint32_t cnt[2];
    if (threadIdx.x < 2) cnt[threadIdx.x] = 0u;
    __syncthreads();
    const uint32_t T = ws[514];
    const uint64_t base = (uint64_t)blockIdx.x * kSegment;
    uint32_t above = 0, equal = 0;
    for (uint32_t i = threadIdx.x; i < kSegment; i += 256u) {
        const uint64_t p = base + i;
        if (p < P) {
            const uint32_t key = s[p];
            above += key > T;
            equal += key == T;
        }
    }
    if (above) atomicAdd(&cnt[0], above);
    if (equal) atomicAdd(&cnt[1], equal);
    __syncthreads();
    if (threadIdx.x < 2) ws[kHdr + 2u * blockIdx.x + threadIdx.x] = cnt[threadIdx.x];
}

// Exclusive scan of the per-segment pairs, one workgroup (segments are few: P / 2048).
__global__ __launch_bounds__(1024) void seg_scan_kernel(uint32_t* ws, uint32_t segments) {
    __shared__ uint32_t wave_tot[2][16];
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t per = (segments + 1023u) / 1024u;
    const uint32_t lo = t * per, hi = min(lo + per, segments);
    uint32_t a = 0, e = 0;
    for (uint32_t i = lo; i < hi; ++i) {
        a += ws[kHdr + 2u * i];
        e += ws[kHdr + 2u * i + 1u];
    }
    // exclusive scan of the 1024 thread totals: inclusive inside each wave by lane shifts,
    // then the totals of the waves before this one
    uint32_t ia = a, ie = e;
    for (uint32_t o = 1; o < 64u; o <<= 1) {
        const uint32_t ya = __shfl_up(ia, o, 64), ye = __shfl_up(ie, o, 64);
        if (lane >= o) {
            ia += ya;
            ie += ye;
        }
    }
    if (lane == 63u) {
        wave_tot[0][wave] = ia;
        wave_tot[1][wave] = ie;
    }
    __syncthreads();
    uint32_t oa = 0, oe = 0;
    for (uint32_t w = 0; w < wave; ++w) {
        oa += wave_tot[0][w];
        oe += wave_tot[1][w];
    }
    a = oa + ia - a;
    e = oe + ie - e;
    for (uint32_t i = lo; i < hi; ++i) {
        const uint32_t xa = ws[kHdr + 2u * i], xe = ws[kHdr + 2u * i + 1u];
        ws[kHdr + 2u * i] = a;
        ws[kHdr + 2u * i + 1u] = e;
        a += xa;
        e += xe;
    }
}

// Ordered compaction: chunk p is selected if its key is above T, or equal to T with fewer
// than `need` equal keys before it; its place is (#above before) + min(#equal before, need).
__global__ __launch_bounds__(256) void write_indices_kernel(const uint16_t* s, uint64_t P, const uint32_t* ws,
                                                            uint32_t* indices) {
    __shared__ uint32_t wave_tot[2][4];
    const uint32_t T = ws[514], need = ws[515];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint64_t base = (uint64_t)blockIdx.x * kSegment;
    uint32_t above_before = ws[kHdr + 2u * blockIdx.x], equal_before = ws[kHdr + 2u * blockIdx.x + 1u];
    // a thread owns 8 consecutive keys, so index order = (thread, k) order
    uint32_t key[8];
    uint32_t a = 0, e = 0;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const uint64_t p = base + 8u * threadIdx.x + k;
        key[k] = p < P ? (uint32_t)s[p] : 0xFFFFFFFFu;   // sentinel: neither above (masked) nor equal
        if (p < P) {
            a += key[k] > T;
            e += key[k] == T;
        }
    }
    // exclusive scan of (a, e) over the 256 threads
    uint32_t ia = a, ie = e;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t ua = __shfl_up(ia, o, 64), ue = __shfl_up(ie, o, 64);
        if (lane >= (uint32_t)o) {
            ia += ua;
            ie += ue;
        }
    }
    if (lane == 63) {
        wave_tot[0][wave] = ia;
        wave_tot[1][wave] = ie;
    }
    __syncthreads();
    for (uint32_t w = 0; w < wave; ++w) {
        above_before += wave_tot[0][w];
        equal_before += wave_tot[1][w];
    }
    above_before += ia - a;
    equal_before += ie - e;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const uint64_t p = base + 8u * threadIdx.x + k;
        if (p < P) {
            const bool is_above = key[k] > T, is_equal = key[k] == T;
            if (is_above || (is_equal && equal_before < need))
                indices[above_before + min(equal_before, need)] = (uint32_t)p;
            above_before += is_above;
            equal_before += is_equal;
        }
    }
}

// ---- selected chunks --------------------------------------------------------------------------
// values[j * C + e] = fp16 sum over workers, in worker order, of fp16(x_w[indices[j] * C + e]).
template <bool BF16>
__global__ __launch_bounds__(256) void gather_sum_kernel(const FusedWorkerPtrs ptrs, uint32_t W, uint64_t n,
                                                         uint32_t C, const uint32_t* indices, uint64_t threads,
                                                         uint16_t* values) {
    const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= threads) return;
    const uint64_t flat = tid * 8u;                 // position in the J x C value array
    const uint64_t j = flat / C;
    const uint32_t e0 = (uint32_t)(flat - j * C);
    const uint64_t g = (uint64_t)indices[j] * C + e0;
    uint32_t acc[8];
    for (uint32_t w = 0; w < W; ++w) {
        float x[8];
        load8<BF16>(ptrs.grad[w], g, n, x);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t h = f32_to_f16_bits(x[e]);
            acc[e] = w == 0 ? h : add_f16_bits(acc[e], h);
        }
    }
    *reinterpret_cast<uint4*>(values + flat) =
        make_uint4(acc[0] | (acc[1] << 16), acc[2] | (acc[3] << 16), acc[4] | (acc[5] << 16), acc[6] | (acc[7] << 16));
}

// out[indices[j] * C + e] = float(values[j * C + e]) / W  (out zeroed beforehand).
__global__ __launch_bounds__(256) void scatter_kernel(const uint16_t* values, const uint32_t* indices, uint32_t C,
                                                      uint32_t W, uint64_t n, uint64_t threads, float* out) {
    const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tid >= threads) return;
    const uint64_t flat = tid * 8u;
    const uint64_t j = flat / C;
    const uint32_t e0 = (uint32_t)(flat - j * C);
    const uint64_t g = (uint64_t)indices[j] * C + e0;
    const uint4 q = *reinterpret_cast<const uint4*>(values + flat);
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    const float Wf = (float)W;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float v = f16_bits_to_f32((w[e >> 1] >> (16 * (e & 1))) & 0xFFFFu) / Wf;
        if (g + e < n) out[g + e] = v;
    }
}

// The dense estimate in ONE pass over the output: every coordinate is written exactly once,
// float(value) / W inside the selected chunks and 0 elsewhere.  `indices` is ascending, so a
// workgroup that owns a contiguous range of chunks finds its first selected chunk by one
// binary search and then walks the list: per tile of kTileChunks chunks, thread t looks at
// indices[j + t] and, if that chunk lies in the tile, records its rank j + t for the
// chunk; no more than kTileChunks selected chunks can lie in a tile, so one look per thread
// sees them all.  `out` must be 16-byte aligned.
constexpr int kScatterThreads = 256;
constexpr int kTileChunks = kScatterThreads;
__global__ __launch_bounds__(kScatterThreads) void scatter_dense_kernel(
    const uint16_t* values, const uint32_t* indices, uint32_t J, uint32_t C, uint32_t W, uint64_t n, uint64_t P,
    uint64_t chunks_per_group, float* out) {
    __shared__ int32_t rank[kTileChunks];
    __shared__ uint32_t first;
    const uint32_t t = threadIdx.x;
    const uint64_t begin = (uint64_t)blockIdx.x * chunks_per_group;
    if (begin >= P) return;
    const uint64_t end = begin + chunks_per_group < P ? begin + chunks_per_group : P;
    if (t == 0) {   // first j with indices[j] >= begin
        uint32_t lo = 0, hi = J;
        while (lo < hi) {
            const uint32_t mid = lo + (hi - lo) / 2u;
            if ((uint64_t)indices[mid] < begin) lo = mid + 1u;
            else hi = mid;
        }
        first = lo;
    }
    __syncthreads();
    uint32_t j = first;
    const float Wf = (float)W;
    const uint32_t units_per_chunk = C / 4u;            // 16-byte units of fp32 output per chunk
    const uint32_t shift = 31u - (uint32_t)__builtin_clz(units_per_chunk);
    for (uint64_t c0 = begin; c0 < end; c0 += kTileChunks) {
        const uint64_t c1 = c0 + kTileChunks < end ? c0 + kTileChunks : end;
        rank[t] = -1;
        __syncthreads();
        const uint64_t cand = (uint64_t)j + t < (uint64_t)J ? (uint64_t)indices[j + t] : ~0ull;
        const bool inside = cand >= c0 && cand < c1;    // cand >= c0 whenever the list is ascending
        if (inside) rank[cand - c0] = (int32_t)(j + t);
        j += (uint32_t)__syncthreads_count(inside);     // also orders the writes of rank before its reads
        const uint64_t unit0 = c0 * units_per_chunk;
        const uint64_t units = (c1 - c0) * units_per_chunk;
        for (uint64_t u = t; u < units; u += kScatterThreads) {
            const uint32_t lc = (uint32_t)(u >> shift);
            const uint32_t e0 = ((uint32_t)u & (units_per_chunk - 1u)) * 4u;
            const int32_t r = rank[lc];
            float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (r >= 0) {
                const uint2 q = *reinterpret_cast<const uint2*>(values + (uint64_t)(uint32_t)r * C + e0);
                x[0] = f16_bits_to_f32(q.x & 0xFFFFu) / Wf;
                x[1] = f16_bits_to_f32(q.x >> 16) / Wf;
                x[2] = f16_bits_to_f32(q.y & 0xFFFFu) / Wf;
                x[3] = f16_bits_to_f32(q.y >> 16) / Wf;
            }
            const uint64_t g = (unit0 + u) * 4u;
            if (g + 4u <= n) {
                store_streaming(out + g, x[0], x[1], x[2], x[3]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (g + e < n) out[g + e] = x[e];
            }
        }
        __syncthreads();                                // rank is rewritten by the next tile
    }
}

// Largest grid of the norm kernel, in blocks of 256 threads (measured on a 2.6 GB gradient:
// 2048 .. 16384 blocks read at 4.8 .. 5.4 TB/s, 32768 and 65536 at 5.7, 262144 at 5.5).
constexpr uint64_t kNormBlocks = 32768;

uint32_t blocks_for(uint64_t threads, uint32_t per_block) {
    return (uint32_t)((threads + per_block - 1) / per_block);
}

}  // namespace

hipError_t launch_topkc_norms(const void* grad, bool bf16, uint64_t n, uint32_t C, uint16_t* norms,
                              hipStream_t stream) {
    const uint64_t P = (n + C - 1) / C;
    const uint64_t threads = P * (C / 8u);
    if (threads == 0) return hipSuccess;
    // (a thread per group while that is at most kNormBlocks blocks, grid-stride beyond)
    uint64_t blocks = blocks_for(threads, 256);
    if (blocks > kNormBlocks) blocks = kNormBlocks;
    const dim3 grid((uint32_t)blocks), block(256);
    if (bf16)
        hipLaunchKernelGGL(norms_kernel<true>, grid, block, 0, stream, grad, n, C / 8u, threads, norms);
    else
        hipLaunchKernelGGL(norms_kernel<false>, grid, block, 0, stream, grad, n, C / 8u, threads, norms);
    return hipGetLastError();
}

hipError_t launch_topkc_sum_norms(const uint16_t* norms_all, uint32_t W, uint64_t P, uint16_t* s,
                                  hipStream_t stream) {
    if (P == 0) return hipSuccess;
    if (P % 4u == 0 && reinterpret_cast<uint64_t>(norms_all) % 8u == 0 && reinterpret_cast<uint64_t>(s) % 8u == 0)
        hipLaunchKernelGGL(sum_norms4_kernel, dim3(blocks_for(P / 4u, 256)), dim3(256), 0, stream, norms_all, W, P, s);
    else
        hipLaunchKernelGGL(sum_norms_kernel, dim3(blocks_for(P, 256)), dim3(256), 0, stream, norms_all, W, P, s);
    return hipGetLastError();
}

uint64_t topkc_select_workspace_words(uint64_t P) {
    return kHdr + 2u * ((P + kSegment - 1) / kSegment);
}

hipError_t launch_topkc_select(const uint16_t* s, uint64_t P, uint32_t J, uint32_t* indices, uint32_t* ws,
                               hipStream_t stream) {
    const uint32_t segments = (uint32_t)((P + kSegment - 1) / kSegment);
    hipError_t e = launch_zero_words(ws, kHdr, stream);
    if (e != hipSuccess) return e;
    uint32_t hb = blocks_for(P, 256 * 16);
    if (hb > 2048) hb = 2048;
    const bool vec = (reinterpret_cast<uintptr_t>(s) & 15u) == 0;
    if (vec) hipLaunchKernelGGL((hist_kernel<0, true>), dim3(hb), dim3(256), 0, stream, s, P, ws);
    else hipLaunchKernelGGL((hist_kernel<0, false>), dim3(hb), dim3(256), 0, stream, s, P, ws);
    hipLaunchKernelGGL(find_kernel<0>, dim3(1), dim3(64), 0, stream, ws, J);
    if (vec) hipLaunchKernelGGL((hist_kernel<1, true>), dim3(hb), dim3(256), 0, stream, s, P, ws);
    else hipLaunchKernelGGL((hist_kernel<1, false>), dim3(hb), dim3(256), 0, stream, s, P, ws);
    hipLaunchKernelGGL(find_kernel<1>, dim3(1), dim3(64), 0, stream, ws, J);
    hipLaunchKernelGGL(seg_count_kernel, dim3(segments), dim3(256), 0, stream, s, P, ws);
    hipLaunchKernelGGL(seg_scan_kernel, dim3(1), dim3(1024), 0, stream, ws, segments);
    hipLaunchKernelGGL(write_indices_kernel, dim3(segments), dim3(256), 0, stream, s, P, ws, indices);
    return hipGetLastError();
}

hipError_t launch_topkc_gather_sum(const FusedWorkerPtrs& ptrs, bool bf16, uint32_t W, uint64_t n, uint32_t C,
                                   const uint32_t* indices, uint32_t J, uint16_t* values, hipStream_t stream) {
    const uint64_t threads = (uint64_t)J * (C / 8u);
    if (threads == 0) return hipSuccess;
    const dim3 grid(blocks_for(threads, 256)), block(256);
    if (bf16)
        hipLaunchKernelGGL(gather_sum_kernel<true>, grid, block, 0, stream, ptrs, W, n, C, indices, threads, values);
    else
        hipLaunchKernelGGL(gather_sum_kernel<false>, grid, block, 0, stream, ptrs, W, n, C, indices, threads, values);
    return hipGetLastError();
}

hipError_t launch_topkc_scatter(const uint16_t* values, const uint32_t* indices, uint32_t J, uint32_t C,
                                uint32_t W, uint64_t n, float* out, hipStream_t stream) {
    const uint64_t P = (n + C - 1) / C;
    if (P == 0) return hipSuccess;
    if ((reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
        // one pass: contiguous ranges of whole tiles
        const uint64_t tiles = (P + kTileChunks - 1) / kTileChunks;
        uint64_t groups = 16384u;   // (5.2 GB written: 2048 groups 1.37 ms, 4096 1.20, 16384 1.12, 32768 1.11)
        if (groups > tiles) groups = tiles;
        const uint64_t chunks_per_group = (tiles + groups - 1) / groups * kTileChunks;
        groups = (P + chunks_per_group - 1) / chunks_per_group;
        hipLaunchKernelGGL(scatter_dense_kernel, dim3((uint32_t)groups), dim3(kScatterThreads), 0, stream, values,
                           indices, J, C, W, n, P, chunks_per_group, out);
        return hipGetLastError();
    }
    // an output that is only 4-byte aligned: fill, then scatter
    hipError_t e = launch_zero_words(reinterpret_cast<uint32_t*>(out), n, stream);
    if (e != hipSuccess) return e;
    const uint64_t threads = (uint64_t)J * (C / 8u);
    if (threads == 0) return hipSuccess;
    hipLaunchKernelGGL(scatter_kernel, dim3(blocks_for(threads, 256)), dim3(256), 0, stream, values, indices, C,
                       W, n, threads, out);
    return hipGetLastError();
}

}  // namespace thc
