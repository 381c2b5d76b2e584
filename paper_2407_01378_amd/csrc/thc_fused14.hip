// Fused kernels for chunk_log2 = 14.
//
// encode_all: ONE pass over every worker's gradient.  A work item is (chunk p, worker
// w); the workgroup that owns it rotates the chunk, publishes the chunk's largest
// magnitude to per-chunk slots in global memory, waits until all W workers of chunk p
// have published, and only then quantizes - the rotated chunk never leaves registers,
// so each gradient is read from HBM once.  The grid is persistent and no larger than
// what is resident at once (occupancy x CUs), items are dealt round-robin
// (item = workgroup + k * grid), so the W owners of a chunk run side by side and every
// wait is for a workgroup that is already running.  Waits are bounded: on time-out an
// error word is set and the wave carries on, so every wave always exits.
//
// aggregate_decode: sums the W payloads of a chunk in packed sub-word lanes straight
// into the inverse rotation; the integer sums never touch HBM unless asked for.
#include "thc_core14.h"
#include "thc_internal.h"

#pragma clang fp contract(off)

namespace thc {
namespace k14 {
namespace {

constexpr uint32_t kWaves = kThreads / 64;
// Second argument of __launch_bounds__ (waves per SIMD the compiler must allow): two
// workgroups of 8 waves per CU = 4 waves on each of the 4 SIMDs = at most 128 VGPRs.
constexpr int kWavesPerSimd = 4;
// Pauses of the wait for the peers' range words, in units of 64 clocks (s_sleep).
constexpr int kFirstPollSleep = 32;
constexpr int kPollSleep = 8;
// Above this many workers the one-pass encoder publishes one range word per workgroup.
#ifndef THC_WGWORD_ABOVE
#define THC_WGWORD_ABOVE 16
#endif
constexpr uint32_t kPerWaveWordsMaxWorkers = THC_WGWORD_ABOVE;
// ------------------------------------------------------------------ encode_all
// The records of a batched launch were written by earlier kernels and are never written by
// this one: reading them through the constant address space lets the compiler use scalar
// loads (one request per wave, served by the scalar cache) where a global pointer, which
// might alias the kernel's stores, would get a vector load and its full memory latency.
#define THC_CONSTANT __attribute__((address_space(4)))
typedef const BatchRecord THC_CONSTANT* ConstRecordPtr;
typedef const uint64_t THC_CONSTANT* ConstU64Ptr;
// A pointer that was read from a record as an integer, as a pointer into global memory: the
// compiler then uses global loads and stores for it, as it does for pointers that arrive as
// kernel arguments, instead of the slower generic (flat) ones, which also count as LDS
// operations in the wait counters.
template <typename T>
__device__ __forceinline__ T* global_ptr(uint64_t address) {
    typedef T __attribute__((address_space(1))) * Global;
    return (T*)(Global)address;
}
__device__ __forceinline__ ConstRecordPtr batch_record(const BatchArgs& batch, uint32_t k) {
    return (ConstRecordPtr)(batch.records + (uint64_t)k * batch.record_bytes);
}

// What an item needs to know about the bucket its chunk belongs to; the same for every
// lane, so it lives in scalar registers.  A single-bucket call has one view for good; a
// batched call looks the view up in the records as its chunks move from bucket to bucket.
struct BucketView {
    uint64_t n;          // coordinates of the bucket
    uint64_t chunk0;     // number of its first chunk in the launch's chunk numbering
    uint32_t key0, key1;
    const void* grad;    // of this workgroup's worker
    uint8_t* payload;
    float* scale;
};

// ODD: bf16 input with an odd number of coordinates.  Its last coordinate shares a dword
// with nothing, which the range check of a buffer load (done per dword) would cut off, so
// that shape keeps the element-wise loader; every other shape loads through a descriptor.
// BATCH: the launch covers several buckets (a.chunks is their total, chunks are numbered
// through all of them); everything per bucket comes from the records in device memory.
// MINMAX: the grid runs from the chunk's smallest to its largest value instead of
// symmetrically around zero: every wave publishes two words (the maximum, then the negated
// minimum, both through order_key() so that both are combined by a maximum), `scale` receives
// (lo, hi) pairs, and the quantizer subtracts lo.
// WGWORD: one range word per WORKGROUP instead of one per wave (the waves' maxima are combined
// through LDS at the barrier that opens the last exchange, and wave 0 publishes and clears).
// For many workers: with W = 64 a chunk would otherwise have 512 words, every polling wave
// would read 2 KB per poll, and that traffic delays the words it waits for.  At W = 8 the
// later publication costs more than the lighter polls save, so the per-wave form stays.
template <bool BF16, bool ODD, bool BATCH, bool MINMAX = false, bool WGWORD = false>
struct EncodeAllCtx {
    static_assert(!(MINMAX && WGWORD), "the per-workgroup word exists for the symmetric grid only");
    static constexpr uint32_t kWordsPerWorker = WGWORD ? 1u : kWaves;
    static constexpr int kUnits = BF16 ? 4 : 8;
    static constexpr int kElem = BF16 ? 2 : 4;
    // bf16: every thread loads its own 64 consecutive bytes one item ahead, so the input
    // never crosses LDS.  fp32 (128 bytes per thread, 32 registers in flight) loads in
    // coalesced order when the item starts and goes through the buffer.
    static constexpr bool kDirect = BF16;
    const EncodeAllArgs& a;
    const FusedWorkerPtrs& ptrs;
    const BatchArgs& batch;
    Shared& sh;
    Raw<kUnits> raw;        // input of the next item to enter the pipeline, in flight
    uint32_t t, lane, wave, nwords;
    uint32_t w;             // worker of every item of this workgroup (the grid is a multiple of W)
    uint32_t dp;            // chunk stride between consecutive items of this workgroup
    uint32_t parity;        // which sign table the next front() reads
    uint32_t prev;          // chunk of the workgroup's previous item, kNone before the first
    uint32_t bidx;          // BATCH: bucket of the most recent look-up (chunks only move forward)
    uint64_t boundary;      // BATCH: first chunk of the bucket after that one
    BucketView cur, nxt;    // of the item being processed / of the item whose input is in flight
    static constexpr uint32_t kNone = 0xFFFFFFFFu;

    // MINMAX: the chunk's words as 8-byte pairs (the slots start 16-byte aligned and a chunk
    // has an even number of 32-bit words)
    __device__ __forceinline__ uint64_t* pairs(uint64_t p) const {
        return reinterpret_cast<uint64_t*>(a.slots + p * nwords);
    }

    __device__ __forceinline__ BucketView view_of(uint64_t p) {
        if constexpr (BATCH) {
            while (bidx + 1u < batch.count && p >= batch_record(batch, bidx + 1u)->chunk0) ++bidx;
            ConstRecordPtr r = batch_record(batch, bidx);
            boundary = bidx + 1u < batch.count ? batch_record(batch, bidx + 1u)->chunk0 : ~0ull;
            ConstU64Ptr ptr = (ConstU64Ptr)(r + 1);   // W gradients, then W payloads
            BucketView bv{r->n, r->chunk0, r->key0, r->key1, reinterpret_cast<const void*>(ptr[w]),
                          reinterpret_cast<uint8_t*>(ptr[a.W + w]), r->scale};
            // The record has arrived before the look-up returns.  Scalar loads complete out of
            // order, so one that is still in flight when the item's LDS exchanges start would
            // make every wait on an LDS load a wait for ALL of them (no overlap of the
            // exchange with the arithmetic that follows it), on every item, although a
            // look-up happens once per bucket.
            asm volatile("" : "+s"(bv.n), "+s"(bv.chunk0), "+s"(bv.key0), "+s"(bv.key1), "+s"(bv.grad),
                         "+s"(bv.payload), "+s"(bv.scale), "+s"(boundary), "+s"(bidx));
            return bv;
        } else {
            return BucketView{a.n, 0u, a.key0, a.key1, ptrs.grad[w], ptrs.payload[w], a.scale};
        }
    }

    // The chunk's raw 16-byte units.  Through a buffer descriptor whose range is the part of
    // the chunk that exists, reads beyond it return zero: there is no ragged path, and the
    // load may be issued for a chunk past the end (range 0), which keeps the prefetch of the
    // next item unconditional.
    __device__ __forceinline__ void load(uint64_t p, const BucketView& bv) {
        const uint64_t g0 = (p - bv.chunk0) << kChunkLog2;
        uint64_t left = p < a.chunks ? bv.n - g0 : 0u;
        if (left > (uint64_t)kChunk) left = kChunk;
        uint64_t addr = reinterpret_cast<uint64_t>(bv.grad) + (p < a.chunks ? g0 * kElem : 0u);
        if constexpr (ODD) {
            if (left != 0u) load_raw<kUnits, kElem, kDirect>(raw, reinterpret_cast<const void*>(addr), (uint32_t)left, t);
        } else {
            // the descriptor is the same for every lane: it belongs in scalar registers
            addr = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(addr >> 32)) << 32) |
                   (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)addr);
            const uint32_t bytes = (uint32_t)left * kElem;   // a multiple of 4: the count is even
            __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                reinterpret_cast<void*>(addr), 0, bytes, 0x00020000);
            typedef uint32_t u4v __attribute__((ext_vector_type(4)));
#pragma unroll
            for (int j = 0; j < kUnits; ++j) {
                const uint32_t unit = kDirect ? kUnits * t + j : j * kThreads + t;
                const u4v q = __builtin_amdgcn_raw_buffer_load_b128(rsrc, unit * 16u, 0, 0);
                raw.u[j] = make_uint4(q.x, q.y, q.z, q.w);
            }
        }
    }
    __device__ __forceinline__ void fill_signs(uint64_t p, const BucketView& bv, uint32_t which) {
        fill_sign_table<!BF16, BF16>(sh.sign[which], (p - bv.chunk0) << kChunkLog2, bv.key0, bv.key1, t);
    }

    // Front half of an item: bring the input into registers (layout L1), rotate, publish
    // this wave's share of the chunk's range, and bring the chunk into the quantizer's
    // layout.  The direct form also fills the sign table of the workgroup's next item,
    // which is read only after the barriers of this item's exchanges.
    __device__ __forceinline__ void front(float (&v)[kRegs], uint64_t p) {
        const bool more = p + dp < a.chunks;
        if (kDirect) {
            units_to_l1<kUnits, true>(sh.sign[parity], raw.u, v, t);
            // the conversion is complete before the registers of `raw` are loaded again: without
            // this the compiler moves it below the loads and copies `raw` out of their way
#pragma unroll
            for (int i = 0; i < kRegs; ++i) asm volatile("" : "+v"(v[i]));
            asm volatile("" ::: "memory");
            if (BATCH && more && p + dp >= boundary) nxt = view_of(p + dp);   // rarely: a new bucket
            load(p + dp, nxt);
            if (more) fill_signs(p + dp, nxt, parity ^ 1u);
            parity ^= 1u;
        } else {
            load(p, cur);
            __syncthreads();   // the previous item's last reads of the buffer and table are done
            fill_signs(p, cur, 0u);
            raw_to_lds<kUnits>(sh, raw, t);
            __syncthreads();
            lds_to_l1<kUnits, true>(sh, sh.sign[0], v, t);
            if (BATCH && more && p + dp >= boundary) nxt = view_of(p + dp);
        }
        rotate_l1_to_l3<true>(sh, v, lane, wave);
        // One word per wave, value | valid bit (non-negative floats order like their bit
        // patterns and leave bit 31 free).  The words travel between workgroups only
        // through device-scope stores and loads, which are served at the memory side, so
        // no cache write-back or invalidate is needed.  The slots start zeroed.
        if constexpr (MINMAX) {
            // (the scaling by 2^-7 is exact and monotone: it commutes with min and max)
            const MinMax r = thread_minmax(v);
            const uint32_t khi = wave_umax(order_key(r.hi * kInvSqrtC));
            const uint32_t klo = wave_umax(order_key(-(r.lo * kInvSqrtC)));
            // one 8-byte word per wave, (key of the maximum) << 32 | key of the negated minimum:
            // an aligned 8-byte store is one transaction, so a reader sees both or neither
            if (lane == 0)
                __hip_atomic_store(pairs(p) + kWaves * w + wave, ((uint64_t)khi << 32) | klo, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        } else if constexpr (WGWORD) {
            const float m = wave_absmax(v) * kInvSqrtC;
            if (lane == 0) sh.red[wave] = m;
            // l3_to_l4e with the publication behind its first barrier
            __syncthreads();
            set_prio<true, kPrioExchange>();
            if (wave == 0 && lane == 0) {
                float mw = fmaxf(fmaxf(fmaxf(sh.red[0], sh.red[1]), fmaxf(sh.red[2], sh.red[3])),
                                 fmaxf(fmaxf(sh.red[4], sh.red[5]), fmaxf(sh.red[6], sh.red[7])));
                __hip_atomic_store(&a.slots[p * nwords + w], __float_as_uint(mw) | 0x80000000u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
            x3e_store(sh, v, lane, wave);
            __syncthreads();
            x3e_load(sh, v, lane, wave);
            set_prio<true, kPrioTail>();
            return;
        } else {
            const float m = wave_absmax(v) * kInvSqrtC;
            if (lane == 0)
                __hip_atomic_store(&a.slots[p * nwords + kWaves * w + wave],
                                   __float_as_uint(m) | 0x80000000u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
        l3_to_l4e<true>(sh, v, lane, wave);
    }

    // Back half: wait until every wave of every worker of the chunk has published, take
    // the largest value as the shared scale, quantize and store.  The wait is bounded:
    // on time-out the error word is set and the wave carries on.
    template <int BITS>
    __device__ __forceinline__ void back(const float (&v)[kRegs], uint64_t p) {
        const uint32_t* slot = a.slots + p * nwords;
        uint32_t mx = 0u, mx2 = 0u;   // mx2: MINMAX only, the negated minima
        bool done = false;
        // The peers of a chunk publish up to about 2 us apart and a word takes about as long
        // to travel, so the first read waits a little: reads that come back incomplete are not
        // free (they load the path the words travel on), and measured on the headline bucket a
        // first read after 32 x 64 clocks and further reads 8 x 64 clocks apart make the launch
        // 3 % faster than reading at once and every 64 clocks.
        __builtin_amdgcn_s_sleep(kFirstPollSleep);
        for (uint32_t spins = 0;; ++spins) {
            if constexpr (MINMAX) {
                const uint32_t half = kWaves * a.W;
                const uint64_t* pair = pairs(p);
                bool all_valid = true;
                mx = mx2 = 0u;
                for (uint32_t base = 0; base < half; base += 64u) {
                    const uint32_t i = base + lane;
                    if (i < half) {
                        const uint64_t v = __hip_atomic_load(&pair[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        const uint32_t vh = (uint32_t)(v >> 32), vl = (uint32_t)v;
                        all_valid = all_valid && v != 0ull;   // (neither key is ever zero)
                        mx = vh > mx ? vh : mx;
                        mx2 = vl > mx2 ? vl : mx2;
                    }
                }
                done = __all(all_valid);
            } else {
                uint32_t all_valid = 0x80000000u;
                mx = 0u;
                for (uint32_t base = 0; base < nwords; base += 64u) {
                    const uint32_t i = base + lane;
                    const uint32_t val =
                        i < nwords ? __hip_atomic_load(&slot[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                   : 0x80000000u;
                    all_valid &= val;
                    const uint32_t mag = val & 0x7FFFFFFFu;
                    mx = mag > mx ? mag : mx;
                }
                done = __all(all_valid != 0u);
            }
            if (done || spins >= a.max_spins) break;
            __builtin_amdgcn_s_sleep(kPollSleep);
        }
        // Every earlier vector-memory operation of the wave has completed (the read of the range
        // words just did), among them the loads of the next item's input.  Passing those
        // registers through an empty asm tells the compiler so: the next item then starts
        // without a wait on them, which would also wait for the stores issued below.
        if (kDirect) {
#pragma unroll
            for (int j = 0; j < kUnits; ++j)
                asm volatile("" : "+v"(raw.u[j].x), "+v"(raw.u[j].y), "+v"(raw.u[j].z), "+v"(raw.u[j].w));
        }
        if (!done && lane == 0)
            __hip_atomic_store(a.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // The workspace leaves the kernel as it entered it, all zero.  A peer's wave
        // publishes for this chunk only after the barriers of this item's rotation,
        // which every wave of its workgroup reaches only after reading the words of
        // the workgroup's previous chunk; with all of this chunk's words seen, nobody
        // will read the previous chunk's words again, and this wave clears its own.
        if (done && prev != kNone && lane == 0 && (!WGWORD || wave == 0)) {
            if constexpr (MINMAX)
                __hip_atomic_store(pairs(prev) + kWaves * w + wave, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else
                __hip_atomic_store(&a.slots[(uint64_t)prev * nwords + kWordsPerWorker * w + (WGWORD ? 0u : wave)],
                                   0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        const uint32_t sbits = wave_umax(mx);
        prev = (uint32_t)p;
        const uint64_t pl = p - cur.chunk0;   // the chunk's number inside its bucket
        if constexpr (MINMAX) {
            // (after an expired wait a word may be missing; zero then stands for "nothing seen")
            const uint32_t lbits = wave_umax(mx2);
            const float hi = sbits != 0u ? order_value(sbits) : 0.0f;
            const float lo = lbits != 0u ? -order_value(lbits) : 0.0f;
            float* range = global_ptr<float>(reinterpret_cast<uint64_t>(cur.scale));
            if (w == 0 && t == 0) {
                range[2 * pl] = lo;
                range[2 * pl + 1] = hi;
            }
            // (no clamp: lo and hi are the chunk's own extremes, see quantize_pack)
            quantize_store_range<BITS, true, false>(v, lo, hi, a.levels, pl << kChunkLog2, w, cur.key0, cur.key1,
                                             global_ptr<uint8_t>(reinterpret_cast<uint64_t>(cur.payload)), t);
            return;
        }
        const float s = __uint_as_float(sbits);
        // (the view's pointers are re-tagged as global here: in a batched launch they come out of
        // the look-up's register barrier as plain addresses)
        if (w == 0 && t == 0) global_ptr<float>(reinterpret_cast<uint64_t>(cur.scale))[pl] = s;
        quantize_store<BITS, false>(v, s, a.levels, pl << kChunkLog2, w, cur.key0, cur.key1,
                                    global_ptr<uint8_t>(reinterpret_cast<uint64_t>(cur.payload)), t);
    }

    // After the workgroup's last item: its words have no later chunk to vouch for them, so
    // the workgroups of the chunk count themselves off and the last one clears the words
    // of all of them, and the counter.
    __device__ __forceinline__ void finish() {
        if (prev == kNone) return;
        __syncthreads();   // every wave of this workgroup has read the chunk's words
        if (wave != 0) return;
        uint32_t arrived = 0u;
        if (lane == 0)
            arrived = __hip_atomic_fetch_add(&a.done[prev], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        arrived = (uint32_t)__builtin_amdgcn_readfirstlane((int)arrived);
        if (arrived == a.W - 1u) {
            uint32_t* words = a.slots + (uint64_t)prev * nwords;
            for (uint32_t i = lane; i < nwords; i += 64u)
                __hip_atomic_store(&words[i], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (lane == 0)
                __hip_atomic_store(&a.done[prev], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
};

constexpr int kStaggerSleeps = 6;   // late start of half the grid, in units of s_sleep 16 (1024 clocks)

// Items are (chunk, worker) pairs; workgroup g of a grid of G (a multiple of W) takes worker
// g mod W of chunks g / W, g / W + G / W, ...  The peers of an item are therefore items of
// the same round of other workgroups, and with every workgroup resident no wait is circular.
template <bool BF16, int BITS, bool ODD, bool BATCH, bool MINMAX = false, bool WGWORD = false>
__global__ __launch_bounds__(kThreads, kWavesPerSimd) void encode_all_kernel(const EncodeAllArgs a,
                                                                 const FusedWorkerPtrs ptrs,
                                                                 const BatchArgs batch) {
    __shared__ Shared sh;
    using Ctx = EncodeAllCtx<BF16, ODD, BATCH, MINMAX, WGWORD>;
    const uint32_t t = threadIdx.x;
    const uint32_t p0 = blockIdx.x / a.W;
    Ctx c{a, ptrs, batch, sh, {}, t, t & 63u, t >> 6, (MINMAX ? 2u : 1u) * Ctx::kWordsPerWorker * a.W, blockIdx.x - p0 * a.W,
          gridDim.x / a.W, 0u, Ctx::kNone, 0u, 0u, {}, {}};
    if (p0 >= a.chunks) return;
    // With more than one round of items, the second half of the grid starts about 2.6 us late
    // (6 x 1024 clocks; the halves are cut between chunks, so all workgroups of a chunk lie in
    // the same half and nobody waits longer for a peer).  Measured, 50 buckets of 1600 chunks with a decode launch in between: 4 to 7
    // such units shorten the step by 1.3 to 3 %, 9 and more lengthen it, quarters or eighths
    // of the grid in steps do no better.
    if (a.chunks > c.dp && p0 >= (c.dp >> 1))
        for (int i = 0; i < kStaggerSleeps; ++i) __builtin_amdgcn_s_sleep(16);
    c.cur = c.nxt = c.view_of(p0);
    if (Ctx::kDirect) {
        c.load(p0, c.cur);
        c.fill_signs(p0, c.cur, 0u);
        __syncthreads();
        // the first chunk's input has arrived before the loop is entered, as every later
        // chunk's has by the time its item starts (see the end of the wait in back())
#pragma unroll
        for (int j = 0; j < Ctx::kUnits; ++j)
            asm volatile("" : "+v"(c.raw.u[j].x), "+v"(c.raw.u[j].y), "+v"(c.raw.u[j].z), "+v"(c.raw.u[j].w));
    }
    for (uint64_t p = p0; p < a.chunks; p += c.dp) {
        float v[kRegs];
        c.front(v, p);
        c.template back<BITS>(v, p);
        if (BATCH) c.cur = c.nxt;
    }
    c.finish();
}

// Copies `count` 32-bit words that arrive as kernel arguments to device memory: how the
// batched calls put their per-bucket records where the kernels can read them, without a
// host-to-device copy (which would need a staging allocation or pinned memory).
struct WordBlob {
    uint32_t w[kBlobWords];
};
__global__ __launch_bounds__(256) void write_words_kernel(uint32_t* dst, const WordBlob blob, uint32_t count) {
    for (uint32_t i = threadIdx.x; i < count; i += 256u) dst[i] = blob.w[i];
}

// Fill with zeros (a kernel, not a memset node, so that callers can capture it in a
// graph).  Words before the first and after the last 16-byte boundary are written one
// by one by the first block; the aligned middle goes out as 16-byte stores.
__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t* dst, uint64_t words) {
    const uint64_t addr = reinterpret_cast<uint64_t>(dst);
    uint64_t head = ((16u - (addr & 15u)) & 15u) / 4u;   // dst is 4-byte aligned
    if (head > words) head = words;
    const uint64_t vecs = (words - head) / 4u;
    const uint64_t tail0 = head + 4u * vecs;
    if (blockIdx.x == 0) {
        if (threadIdx.x < head) dst[threadIdx.x] = 0u;
        if (tail0 + threadIdx.x < words) dst[tail0 + threadIdx.x] = 0u;
    }
    uint4* mid = reinterpret_cast<uint4*>(dst + head);
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < vecs;
         i += (uint64_t)gridDim.x * blockDim.x)
        mid[i] = make_uint4(0u, 0u, 0u, 0u);
}

__global__ void copy_word_kernel(const uint32_t* src, uint32_t* dst) { *dst = *src; }

// ------------------------------------------------------------- aggregate_decode
// One chunk per work item, persistent grid.  Thread t owns coordinates 32 t .. 32 t + 31
// (layout L1): 4 * BITS payload bytes (BITS dwords) per worker.
template <int BITS>
struct PayloadWords {
    uint32_t w[BITS];
};
template <int BITS>
__device__ __forceinline__ PayloadWords<BITS> load_payload_words(const uint8_t* p) {
    PayloadWords<BITS> r;
    if (BITS == 2) {
        const uint2 q = load_last_use(reinterpret_cast<const uint2*>(p));
        r.w[0] = q.x;
        r.w[1] = q.y;
    } else {
#pragma unroll
        for (int k = 0; k < BITS / 4; ++k) {
            const uint4 q = load_last_use(reinterpret_cast<const uint4*>(p) + k);
            r.w[4 * k] = q.x;
            r.w[4 * k + 1] = q.y;
            r.w[4 * k + 2] = q.z;
            r.w[4 * k + 3] = q.w;
        }
    }
    return r;
}

// Sum of the workers' payload words of one thread (its 32 coordinates) in sub-word lanes,
// built up group by group: a group is the payload of kGroup workers in flight at once.
// WIDE: 16-bit accumulators for 4-bit payloads too (W * L > 255: more than 17 workers); lane q
// then holds coordinates q (low half) and q + 16 / BITS (high half) of the dword's 32 / BITS.
template <int BITS, bool BATCH = false, bool WIDE = false>
struct PayloadSum {
    static_assert(!(WIDE && BITS == 8), "8-bit payloads always sum in 16-bit lanes");
    static constexpr int kWords = BITS;                        // payload dwords per worker per thread
    static constexpr int kLanes = BITS == 8 ? 2 : (WIDE ? 16 : 8) / BITS;   // sub-word accumulators per dword
    static constexpr uint32_t kMask = BITS == 8 ? 0x00FF00FFu
                                      : WIDE    ? (BITS == 4 ? 0x000F000Fu : 0x00030003u)
                                                : (BITS == 4 ? 0x0F0F0F0Fu : 0x03030303u);
    static constexpr int kGroup = BITS == 8 ? 2 : 4;           // at most 16 registers in flight
    const FusedPayloadPtrs& ptrs;   // single bucket: the payload pointers, in the kernel arguments
    ConstU64Ptr pp;                 // batched: those of the bucket being summed, in its record
    uint32_t W;
    uint32_t acc[kWords][kLanes];
    PayloadWords<BITS> x[kGroup];

    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int d = 0; d < kWords; ++d)
#pragma unroll
            for (int k = 0; k < kLanes; ++k) acc[d][k] = 0u;
    }
    __device__ __forceinline__ void issue(uint64_t byte0, uint32_t group) {
#pragma unroll
        for (int j = 0; j < kGroup; ++j)
            if (group * kGroup + j < W) {
                const uint8_t* src = BATCH ? global_ptr<const uint8_t>(pp[group * kGroup + j])
                                           : ptrs.p[group * kGroup + j];
                x[j] = load_payload_words<BITS>(src + byte0);
            }
    }
    __device__ __forceinline__ void add(uint32_t group) {
#pragma unroll
        for (int j = 0; j < kGroup; ++j)
            if (group * kGroup + j < W) {
#pragma unroll
                for (int d = 0; d < kWords; ++d)
#pragma unroll
                    for (int q = 0; q < kLanes; ++q) acc[d][q] += (x[j].w[d] >> (BITS * q)) & kMask;
            }
    }
    __device__ __forceinline__ uint32_t groups() const { return (W + kGroup - 1) / kGroup; }
};

// Called from inside the rotation of the current chunk: loads and sums the first three
// worker groups of the workgroup's NEXT chunk, one exchange of latency apart.
template <int BITS, bool BATCH, bool WIDE>
struct NextChunkLoads {
    PayloadSum<BITS, BATCH, WIDE>& sum;
    uint64_t byte0;
    bool active;
    template <int K>
    __device__ __forceinline__ void at() {
        if (!active) return;
        if (K > 0) sum.add(K - 1);
        sum.issue(byte0, K);
    }
};

// The bucket a decode item belongs to (uniform).  A single-bucket call has one for good; a
// batched call looks it up in the records as its chunks move from bucket to bucket.
struct DecodeView {
    uint64_t n, chunk0;
    uint32_t key0, key1;
    const float* scale;
    float* out;
    ConstU64Ptr pp;      // the bucket's W payload pointers
};

// RANGED: `scale` holds (lo, hi) pairs of the min/max grid instead of the symmetric scale.
template <int BITS, bool BATCH, bool RANGED = false, bool WIDE = false>
__global__ __launch_bounds__(kThreads, kWavesPerSimd) void aggregate_decode_kernel(const AggDecodeArgs a,
                                                                       const FusedPayloadPtrs ptrs,
                                                                       const BatchArgs batch) {
    __shared__ Shared sh;
    using Sum = PayloadSum<BITS, BATCH, WIDE>;
    constexpr int kWords = Sum::kWords, kLanes = Sum::kLanes;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const float Lf = (float)((1u << BITS) - 1u);
    const float Wf = (float)a.W;
    const uint64_t thread_byte = (uint64_t)t * (4u * BITS);

    uint32_t bidx = 0u;
    uint64_t boundary = 0u;   // first chunk of the bucket after bidx
    auto view_of = [&](uint64_t p) -> DecodeView {
        if constexpr (BATCH) {
            while (bidx + 1u < batch.count && p >= batch_record(batch, bidx + 1u)->chunk0) ++bidx;
            ConstRecordPtr r = batch_record(batch, bidx);
            boundary = bidx + 1u < batch.count ? batch_record(batch, bidx + 1u)->chunk0 : ~0ull;
            ConstU64Ptr pp = (ConstU64Ptr)(r + 1) + a.W;   // the payload pointers follow the gradient pointers
            DecodeView dv{r->n, r->chunk0, r->key0, r->key1, r->scale, r->out, pp};
            // the record has arrived before the look-up returns (see EncodeAllCtx::view_of)
            asm volatile("" : "+s"(dv.n), "+s"(dv.chunk0), "+s"(dv.key0), "+s"(dv.key1), "+s"(dv.scale),
                         "+s"(dv.out), "+s"(boundary), "+s"(bidx));
            return dv;
        } else {
            return DecodeView{a.n, 0u, a.key0, a.key1, a.scale, a.out, nullptr};
        }
    };

    if (blockIdx.x >= a.chunks) return;
    DecodeView cur = view_of(blockIdx.x);
    Sum sum{ptrs, cur.pp, a.W};
    sum.clear();
    {   // the first chunk's payload, without overlap
        const uint64_t byte0 = (((blockIdx.x - cur.chunk0) << kChunkLog2) * BITS) / 8u + thread_byte;
        for (uint32_t g = 0; g < sum.groups(); ++g) {
            sum.issue(byte0, g);
            sum.add(g);
        }
    }
    for (uint64_t p = blockIdx.x; p < a.chunks; p += gridDim.x) {
        const uint64_t pl = p - cur.chunk0;      // the chunk's number inside its bucket
        const uint64_t g0 = pl << kChunkLog2;
        const uint64_t left = cur.n - g0;
        const uint32_t valid = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
        __syncthreads();   // the previous item's last reads of the buffer and sign table are done
        fill_sign_table<true, false>(sh.sign[0], g0, cur.key0, cur.key1, t);

        // sums -> rotated-domain estimate of the mean, layout L1
        // symmetric grid: yhat = S q - s;  min/max grid: yhat = S q + lo = S q - (-lo)
        const float* scale = global_ptr<const float>(reinterpret_cast<uint64_t>(cur.scale));
        const float s = RANGED ? -scale[2 * pl] : scale[pl];
        const float step = (RANGED ? scale[2 * pl + 1] + s : s + s) / Lf;
        const float qf = step / Wf;
        float v[kRegs];
        uint32_t S[kRegs];
#pragma unroll
        for (int d = 0; d < kWords; ++d) {
            if (BITS == 8) {         // dword d: coordinates 4d..4d+3; lane 0 = even, lane 1 = odd
                S[4 * d + 0] = sum.acc[d][0] & 0xFFFFu;
                S[4 * d + 1] = sum.acc[d][1] & 0xFFFFu;
                S[4 * d + 2] = sum.acc[d][0] >> 16;
                S[4 * d + 3] = sum.acc[d][1] >> 16;
            } else if (WIDE) {       // dword d: 32/BITS coordinates; lane q = coordinates q and q + 16/BITS
                constexpr int per = 32 / BITS;
#pragma unroll
                for (int q = 0; q < kLanes; ++q) {
                    S[per * d + q] = sum.acc[d][q] & 0xFFFFu;
                    S[per * d + kLanes + q] = sum.acc[d][q] >> 16;
                }
            } else {                 // dword d: 32/BITS coordinates; lane q byte b = coordinate (8/BITS) b + q
                constexpr int per = 32 / BITS;
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                    for (int q = 0; q < kLanes; ++q)
                        S[per * d + kLanes * b + q] = (sum.acc[d][q] >> (8 * b)) & 0xFFu;
            }
        }
#pragma unroll
        for (int r = 0; r < kRegs; ++r) v[r] = (float)S[r] * qf - s;

        if (!BATCH && a.sums) {   // the caller also wants the integer aggregate
            if (BITS == 8 || WIDE) {
                uint16_t* dst = static_cast<uint16_t*>(a.sums) + g0 + 32u * t;
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    *reinterpret_cast<uint4*>(dst + 8 * k) =
                        make_uint4(S[8 * k] | (S[8 * k + 1] << 16), S[8 * k + 2] | (S[8 * k + 3] << 16),
                                   S[8 * k + 4] | (S[8 * k + 5] << 16), S[8 * k + 6] | (S[8 * k + 7] << 16));
            } else {
                uint8_t* dst = static_cast<uint8_t*>(a.sums) + g0 + 32u * t;
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    uint32_t o[4];
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const int r = 16 * k + 4 * d;
                        o[d] = S[r] | (S[r + 1] << 8) | (S[r + 2] << 16) | (S[r + 3] << 24);
                    }
                    *reinterpret_cast<uint4*>(dst + 16 * k) = make_uint4(o[0], o[1], o[2], o[3]);
                }
            }
        }

        // the next chunk's payload arrives while this one rotates
        const uint64_t pn = p + gridDim.x;
        const bool more = pn < a.chunks;
        DecodeView nxt = cur;
        if (BATCH && more && pn >= boundary) nxt = view_of(pn);   // rarely: a new bucket
        sum.pp = nxt.pp;
        NextChunkLoads<BITS, BATCH, WIDE> next{sum, (((pn - nxt.chunk0) << kChunkLog2) * BITS) / 8u + thread_byte, more};
        sum.clear();
        rotate_l1_to_l3<false>(sh, v, lane, wave, next);
        if (next.active) {
            sum.add(2);
            for (uint32_t g = 3; g < sum.groups(); ++g) {
                sum.issue(next.byte0, g);
                sum.add(g);
            }
        }
        l3_to_l4d<false>(sh, v, lane, wave);
        store_signed_l4d(sh.sign[0], v, global_ptr<float>(reinterpret_cast<uint64_t>(cur.out)) + g0, valid, t);
        cur = nxt;
    }
}

// ------------------------------------------------- saturating aggregate + decode
// Same shape as aggregate_decode_kernel, but the W payloads are combined coordinate by
// coordinate with Sat in worker order (a <- clamp(a + z_w, -M, M), z = idx - M, starting
// from a = 0, which leaves a = z_0 after the first worker), so the running value never
// needs more than BITS bits.  Optionally stores the packed aggregate (a + M) and counts
// the coordinates with at least one clipped step.
// Called from inside the rotation of the current chunk: loads the first worker group of
// the workgroup's next chunk.
template <int BITS, int GROUP>
struct NextSatLoads {
    PayloadWords<BITS> (&x)[GROUP];
    const FusedPayloadPtrs& ptrs;
    uint32_t W;
    uint64_t byte0;
    bool active;
    template <int K>
    __device__ __forceinline__ void at() {
        if (K != 0 || !active) return;
#pragma unroll
        for (int j = 0; j < GROUP; ++j)
            if ((uint32_t)j < W) x[j] = load_payload_words<BITS>(ptrs.p[j] + byte0);
    }
};

template <int BITS, bool COUNT>
__global__ __launch_bounds__(kThreads, kWavesPerSimd) void sat_aggregate_decode_kernel(
    const SatAggDecodeArgs a, const FusedPayloadPtrs ptrs) {
    __shared__ Shared sh;
    constexpr int M = (1 << (BITS - 1)) - 1;
    constexpr int kGroup = (BITS == 8 || COUNT) ? 2 : 4;   // the counting form needs the registers
    constexpr uint32_t kField = (1u << BITS) - 1u;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const float Lf = (float)(2 * M);
    const float Wf = (float)a.W;
    uint32_t clipped_total = 0u;
    const uint64_t thread_byte = (uint64_t)t * (4u * BITS);

    PayloadWords<BITS> first[kGroup];   // the first worker group of the chunk about to start
    {
        NextSatLoads<BITS, kGroup> now{first, ptrs, a.W, (((uint64_t)blockIdx.x << kChunkLog2) * BITS) / 8u + thread_byte,
                                       blockIdx.x < a.chunks};
        now.template at<0>();
    }
    for (uint64_t p = blockIdx.x; p < a.chunks; p += gridDim.x) {
        const uint64_t g0 = p << kChunkLog2;
        const uint64_t left = a.n - g0;
        const uint32_t valid = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
        __syncthreads();   // the previous item's last reads of the buffer and sign table are done
        fill_sign_table<true, false>(sh.sign[0], g0, a.key0, a.key1, t);

        int acc[kRegs];
        uint32_t clip[kRegs];
#pragma unroll
        for (int r = 0; r < kRegs; ++r) {
            acc[r] = 0;
            clip[r] = 0u;
        }
        const uint64_t byte0 = (g0 * BITS) / 8u + thread_byte;
        for (uint32_t w0 = 0; w0 < a.W; w0 += kGroup) {
            PayloadWords<BITS> x[kGroup];
#pragma unroll
            for (int j = 0; j < kGroup; ++j)
                if (w0 + j < a.W) x[j] = w0 == 0 ? first[j] : load_payload_words<BITS>(ptrs.p[w0 + j] + byte0);
#pragma unroll
            for (int j = 0; j < kGroup; ++j)
                if (w0 + j < a.W) {
#pragma unroll
                    for (int r = 0; r < kRegs; ++r) {
                        const int bit = r * BITS;
                        const int raw = acc[r] + (int)((x[j].w[bit >> 5] >> (bit & 31)) & kField) - M;
                        const int c = raw < -M ? -M : (raw > M ? M : raw);
                        if (COUNT) clip[r] |= (uint32_t)(raw ^ c);
                        acc[r] = c;
                    }
                }
        }
        if (COUNT) {
#pragma unroll
            for (int r = 0; r < kRegs; ++r) clipped_total += clip[r] != 0u ? 1u : 0u;
        }
        if (a.aggregate) {
            uint32_t pk[BITS];
#pragma unroll
            for (int d = 0; d < BITS; ++d) pk[d] = 0u;
#pragma unroll
            for (int r = 0; r < kRegs; ++r) {
                const int bit = r * BITS;
                pk[bit >> 5] |= (uint32_t)(acc[r] + M) << (bit & 31);
            }
            uint8_t* dst = a.aggregate + byte0;
            if constexpr (BITS == 8) {
                reinterpret_cast<uint4*>(dst)[0] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                reinterpret_cast<uint4*>(dst)[1] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
            } else if constexpr (BITS == 4) {
                *reinterpret_cast<uint4*>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
            } else {
                *reinterpret_cast<uint2*>(dst) = make_uint2(pk[0], pk[1]);
            }
        }

        // aggregate -> rotated-domain estimate of the mean, layout L1
        const float s = a.scale[p];
        const float step = (s + s) / Lf;
        const float qf = step / Wf;
        float v[kRegs];
#pragma unroll
        for (int r = 0; r < kRegs; ++r) v[r] = (float)acc[r] * qf;
        // the next chunk's first payloads arrive while this one rotates
        const uint64_t pn = p + gridDim.x;
        NextSatLoads<BITS, kGroup> next{first, ptrs, a.W, ((pn << kChunkLog2) * BITS) / 8u + thread_byte,
                                        pn < a.chunks};
        rotate_l1_to_l3<false>(sh, v, lane, wave, next);
        l3_to_l4d<false>(sh, v, lane, wave);
        store_signed_l4d(sh.sign[0], v, a.out + g0, valid, t);
    }
    if (COUNT) {   // one atomic per wave
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) clipped_total += __shfl_xor(clipped_total, off, 64);
        if (lane == 0 && clipped_total != 0u) atomicAdd(a.overflow, (unsigned long long)clipped_total);
    }
}

// ------------------------------------------------------------------ aggregate only
// Streaming sum of W payloads: each thread owns 16 payload bytes per worker.
template <int BITS, typename SumT>
__global__ __launch_bounds__(256) void aggregate_fast_kernel(const FusedPayloadPtrs ptrs, uint32_t W,
                                                             uint64_t vecs, SumT* sums) {
    constexpr bool kWide = BITS != 8 && sizeof(SumT) == 2;   // 16-bit lanes for 2- and 4-bit payloads
    constexpr int kLanes = BITS == 8 ? 2 : (kWide ? 16 : 8) / BITS;
    constexpr uint32_t kMask = BITS == 8 ? 0x00FF00FFu
                               : kWide   ? (BITS == 4 ? 0x000F000Fu : 0x00030003u)
                                         : (BITS == 4 ? 0x0F0F0F0Fu : 0x03030303u);
    constexpr int kCoords = 128 / BITS;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < vecs;
         i += (uint64_t)gridDim.x * blockDim.x) {
        uint32_t acc[4][kLanes];
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int q = 0; q < kLanes; ++q) acc[d][q] = 0u;
        for (uint32_t w0 = 0; w0 < W; w0 += 8) {
            uint4 x[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (w0 + j < W) x[j] = reinterpret_cast<const uint4*>(ptrs.p[w0 + j])[i];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (w0 + j < W) {
                    const uint32_t ww[4] = {x[j].x, x[j].y, x[j].z, x[j].w};
#pragma unroll
                    for (int d = 0; d < 4; ++d)
#pragma unroll
                        for (int q = 0; q < kLanes; ++q) acc[d][q] += (ww[d] >> (BITS * q)) & kMask;
                }
        }
        SumT* dst = sums + i * kCoords;
        if constexpr (kWide) {   // lane q = coordinates q (low half) and q + kLanes (high half) of the dword
            constexpr int per = 32 / BITS;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                uint32_t o[per / 2];   // pairs of consecutive coordinates
#pragma unroll
                for (int c = 0; c < per; c += 2) {
                    const uint32_t lo = c < kLanes ? (acc[d][c] & 0xFFFFu) : (acc[d][c - kLanes] >> 16);
                    const uint32_t hi = c + 1 < kLanes ? (acc[d][c + 1] & 0xFFFFu) : (acc[d][c + 1 - kLanes] >> 16);
                    o[c / 2] = lo | (hi << 16);
                }
#pragma unroll
                for (int k = 0; k < per / 8; ++k)
                    reinterpret_cast<uint4*>(dst + per * d)[k] = make_uint4(o[4 * k], o[4 * k + 1], o[4 * k + 2], o[4 * k + 3]);
            }
        } else if (BITS == 8) {   // u16 sums: (even, odd) pairs
            uint32_t o[8];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                o[2 * d] = __builtin_amdgcn_perm(acc[d][1], acc[d][0], 0x05040100u);
                o[2 * d + 1] = __builtin_amdgcn_perm(acc[d][1], acc[d][0], 0x07060302u);
            }
            reinterpret_cast<uint4*>(dst)[0] = make_uint4(o[0], o[1], o[2], o[3]);
            reinterpret_cast<uint4*>(dst)[1] = make_uint4(o[4], o[5], o[6], o[7]);
        } else if (BITS == 4) {   // u8 sums: lane 0 = even coordinates, lane 1 = odd
            uint32_t o[8];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                o[2 * d] = __builtin_amdgcn_perm(acc[d][1], acc[d][0], 0x05010400u);
                o[2 * d + 1] = __builtin_amdgcn_perm(acc[d][1], acc[d][0], 0x07030602u);
            }
            reinterpret_cast<uint4*>(dst)[0] = make_uint4(o[0], o[1], o[2], o[3]);
            reinterpret_cast<uint4*>(dst)[1] = make_uint4(o[4], o[5], o[6], o[7]);
        } else {                  // 2 bits: lane q byte b = coordinate 4 b + q of the dword's 16
            uint32_t o[16];
#pragma unroll
            for (int d = 0; d < 4; ++d)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    uint32_t v = 0u;
#pragma unroll
                    for (int q = 0; q < 4; ++q) v |= ((acc[d][q] >> (8 * b)) & 0xFFu) << (8 * q);
                    o[4 * d + b] = v;
                }
#pragma unroll
            for (int k = 0; k < 4; ++k)
                reinterpret_cast<uint4*>(dst)[k] = make_uint4(o[4 * k], o[4 * k + 1], o[4 * k + 2], o[4 * k + 3]);
        }
    }
}

int g_cus = 0;
int device_cus() {
    if (g_cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            g_cus = prop.multiProcessorCount;
    }
    return g_cus;
}

// Workgroups of `kernel` that are resident at once on the whole device.  The occupancy
// query is slow (tens of microseconds), so the answer is kept per kernel.
template <auto kernel>
uint32_t resident_grid() {
    static uint32_t cached = 0;   // one per kernel
    if (cached == 0) {
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, kThreads, 0) != hipSuccess || occ < 1)
            return 0;
        const int cus = device_cus();
        if (cus <= 0) return 0;
        cached = (uint32_t)(occ * cus);
    }
    return cached;
}

template <bool BF16, int BITS, bool ODD, bool BATCH>
hipError_t launch_encode_all_t(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, const BatchArgs& batch,
                               hipStream_t stream) {
    uint32_t G = resident_grid<encode_all_kernel<BF16, BITS, ODD, BATCH>>();
    if (G == 0) return hipErrorInvalidValue;
    const uint64_t total = a.chunks * a.W;
    if (G > total) G = (uint32_t)total;
    // every workgroup keeps one worker, so the grid is a whole number of chunks per round;
    // fewer resident workgroups than workers would leave peers that never run
    if (G < a.W) return hipErrorInvalidConfiguration;
    G -= G % a.W;
    if constexpr (!BATCH) {
        if (a.W > kPerWaveWordsMaxWorkers) {   // many workers: one range word per workgroup
            hipLaunchKernelGGL((encode_all_kernel<BF16, BITS, ODD, false, false, true>), dim3(G), dim3(kThreads), 0,
                               stream, a, ptrs, batch);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((encode_all_kernel<BF16, BITS, ODD, BATCH>), dim3(G), dim3(kThreads), 0, stream, a, ptrs,
                       batch);
    return hipGetLastError();
}

template <bool BATCH>
hipError_t launch_encode_all_pick(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, const BatchArgs& batch,
                                  bool bf16, bool odd, uint32_t bits, hipStream_t stream) {
    if (bf16 && odd) {   // an odd count of bf16 somewhere: element-wise loader for the last coordinate
        if (bits == 2) return launch_encode_all_t<true, 2, true, BATCH>(a, ptrs, batch, stream);
        if (bits == 4) return launch_encode_all_t<true, 4, true, BATCH>(a, ptrs, batch, stream);
        return launch_encode_all_t<true, 8, true, BATCH>(a, ptrs, batch, stream);
    }
    if (bf16) {
        if (bits == 2) return launch_encode_all_t<true, 2, false, BATCH>(a, ptrs, batch, stream);
        if (bits == 4) return launch_encode_all_t<true, 4, false, BATCH>(a, ptrs, batch, stream);
        return launch_encode_all_t<true, 8, false, BATCH>(a, ptrs, batch, stream);
    }
    if (bits == 2) return launch_encode_all_t<false, 2, false, BATCH>(a, ptrs, batch, stream);
    if (bits == 4) return launch_encode_all_t<false, 4, false, BATCH>(a, ptrs, batch, stream);
    return launch_encode_all_t<false, 8, false, BATCH>(a, ptrs, batch, stream);
}

// 4-bit payloads of so many workers that the sums need 16 bits.
template <int BITS, bool BATCH, bool RANGED>
hipError_t launch_aggregate_decode_wide(const AggDecodeArgs& a, const FusedPayloadPtrs& ptrs, const BatchArgs& batch,
                                        hipStream_t stream) {
    uint32_t G = resident_grid<aggregate_decode_kernel<BITS, BATCH, RANGED, true>>();
    if (G == 0) return hipErrorInvalidValue;
    if (G > a.chunks) G = (uint32_t)a.chunks;
    hipLaunchKernelGGL((aggregate_decode_kernel<BITS, BATCH, RANGED, true>), dim3(G), dim3(kThreads), 0, stream, a,
                       ptrs, batch);
    return hipGetLastError();
}
// (2-bit payloads would need more than 85 workers, beyond what the one-launch forms take)
__host__ inline bool wide_sums(uint32_t W, uint32_t bits) { return bits == 4u && W * 15u > 255u; }

template <bool BATCH>
hipError_t launch_aggregate_decode_pick(const AggDecodeArgs& a, const FusedPayloadPtrs& ptrs, const BatchArgs& batch,
                                        uint32_t bits, hipStream_t stream) {
    if (a.chunks == 0) return hipSuccess;
    if (wide_sums(a.W, bits)) return launch_aggregate_decode_wide<4, BATCH, false>(a, ptrs, batch, stream);
    uint32_t G = 0;
    if (bits == 2) G = resident_grid<aggregate_decode_kernel<2, BATCH>>();
    else if (bits == 4) G = resident_grid<aggregate_decode_kernel<4, BATCH>>();
    else G = resident_grid<aggregate_decode_kernel<8, BATCH>>();
    if (G == 0) return hipErrorInvalidValue;
    if (G > a.chunks) G = (uint32_t)a.chunks;
    if (bits == 2)
        hipLaunchKernelGGL((aggregate_decode_kernel<2, BATCH>), dim3(G), dim3(kThreads), 0, stream, a, ptrs, batch);
    else if (bits == 4)
        hipLaunchKernelGGL((aggregate_decode_kernel<4, BATCH>), dim3(G), dim3(kThreads), 0, stream, a, ptrs, batch);
    else
        hipLaunchKernelGGL((aggregate_decode_kernel<8, BATCH>), dim3(G), dim3(kThreads), 0, stream, a, ptrs, batch);
    return hipGetLastError();
}

}  // namespace
}  // namespace k14

uint32_t encode_all_slot_words(uint32_t W) { return k14::kWaves * W; }

// Workgroups of the one-pass encoder that the device keeps resident at once.
static uint32_t encode_all_resident(bool bf16, uint32_t bits) {
    using namespace k14;
    if (bf16) return bits == 2 ? resident_grid<encode_all_kernel<true, 2, false, false>>()
                   : bits == 4 ? resident_grid<encode_all_kernel<true, 4, false, false>>()
                               : resident_grid<encode_all_kernel<true, 8, false, false>>();
    return bits == 2 ? resident_grid<encode_all_kernel<false, 2, false, false>>()
         : bits == 4 ? resident_grid<encode_all_kernel<false, 4, false, false>>()
                     : resident_grid<encode_all_kernel<false, 8, false, false>>();
}

bool encode_all_fused_applicable(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, uint32_t chunk_log2,
                                 bool bf16, uint32_t bits) {
    if (chunk_log2 != 14 || a.W > (uint32_t)kMaxFusedWorkers) return false;
    if (a.chunks * a.W >= 0x7FFFFFFFull) return false;
    // the W workgroups of a chunk wait for one another: all of them must be resident
    if (encode_all_resident(bf16, bits) < a.W) return false;
    for (uint32_t w = 0; w < a.W; ++w)
        if ((reinterpret_cast<uintptr_t>(ptrs.grad[w]) & 15u) || (reinterpret_cast<uintptr_t>(ptrs.payload[w]) & 15u))
            return false;
    return true;
}

hipError_t launch_zero_words(uint32_t* dst, uint64_t words, hipStream_t stream) {
    if (words == 0) return hipSuccess;
    const uint64_t blocks = (words / 4u + 255u) / 256u;
    hipLaunchKernelGGL(k14::zero_words_kernel, dim3((uint32_t)(blocks < 1u ? 1u : (blocks > 8192u ? 8192u : blocks))),
                       dim3(256), 0, stream, dst, words);
    return hipGetLastError();
}

hipError_t launch_copy_word(const uint32_t* src, uint32_t* dst, hipStream_t stream) {
    hipLaunchKernelGGL(k14::copy_word_kernel, dim3(1), dim3(1), 0, stream, src, dst);
    return hipGetLastError();
}

hipError_t launch_encode_all_fused(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, bool bf16,
                                   uint32_t bits, hipStream_t stream) {
    return k14::launch_encode_all_pick<false>(a, ptrs, BatchArgs{}, bf16, (a.n & 1u) != 0u, bits, stream);
}

// The min/max grid through the same kernel: a.scale receives (lo, hi) pairs and a.slots has
// twice the words per chunk.
hipError_t launch_encode_all_ranged(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, bool bf16,
                                    uint32_t bits, hipStream_t stream) {
    using namespace k14;
    const BatchArgs none{};
    const bool odd = (a.n & 1u) != 0u;
#define THC_RANGED(BF, B, O)                                                                       \
    do {                                                                                           \
        uint32_t G = resident_grid<encode_all_kernel<BF, B, O, false, true>>();                    \
        if (G == 0) return hipErrorInvalidValue;                                                   \
        const uint64_t total = a.chunks * a.W;                                                     \
        if (G > total) G = (uint32_t)total;                                                        \
        if (G < a.W) return hipErrorInvalidConfiguration;                                          \
        G -= G % a.W;                                                                              \
        hipLaunchKernelGGL((encode_all_kernel<BF, B, O, false, true>), dim3(G), dim3(kThreads), 0, \
                           stream, a, ptrs, none);                                                 \
        return hipGetLastError();                                                                  \
    } while (0)
    if (a.chunks == 0) return hipSuccess;
    if (bf16 && odd) {
        if (bits == 2) THC_RANGED(true, 2, true);
        if (bits == 4) THC_RANGED(true, 4, true);
        THC_RANGED(true, 8, true);
    }
    if (bf16) {
        if (bits == 2) THC_RANGED(true, 2, false);
        if (bits == 4) THC_RANGED(true, 4, false);
        THC_RANGED(true, 8, false);
    }
    if (bits == 2) THC_RANGED(false, 2, false);
    if (bits == 4) THC_RANGED(false, 4, false);
    THC_RANGED(false, 8, false);
#undef THC_RANGED
}

hipError_t launch_encode_all_batch(const EncodeAllArgs& a, const BatchArgs& batch, bool bf16, bool any_odd,
                                   uint32_t bits, hipStream_t stream) {
    return k14::launch_encode_all_pick<true>(a, FusedWorkerPtrs{}, batch, bf16, any_odd, bits, stream);
}

hipError_t launch_write_words(uint32_t* dst, const uint32_t* host_words, uint32_t count, hipStream_t stream) {
    // the words travel as kernel arguments, kBlobWords at a time
    for (uint32_t done = 0; done < count; done += (uint32_t)kBlobWords) {
        k14::WordBlob blob;
        const uint32_t now = count - done < (uint32_t)kBlobWords ? count - done : (uint32_t)kBlobWords;
        for (uint32_t i = 0; i < now; ++i) blob.w[i] = host_words[done + i];
        hipLaunchKernelGGL(k14::write_words_kernel, dim3(1), dim3(256), 0, stream, dst + done, blob, now);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

bool aggregate_decode_fused_applicable(uint32_t W, uint32_t chunk_log2, uint32_t bits) {
    if (chunk_log2 != 14 || W > (uint32_t)kMaxFusedPayloads) return false;
    // packed accumulators: 8-bit lanes for 2- and 4-bit payloads, 16-bit lanes for 8-bit.
    // The kernel stores the sums at the width of its lanes, so the shape qualifies only
    // when that is also the width the caller's buffer has (one worker of 8-bit payloads
    // has one-byte sums and takes the unfused path).
    static_assert(kMaxFusedPayloads * 3 <= 255, "2-bit payloads have narrow lanes only");
    const uint32_t top = W * ((1u << bits) - 1u);
    return bits == 8 ? (top > 255u && top <= 65535u) : top <= 65535u;
}

hipError_t launch_aggregate_decode_fused(const AggDecodeArgs& a, const FusedPayloadPtrs& ptrs,
                                         uint32_t bits, hipStream_t stream) {
    return k14::launch_aggregate_decode_pick<false>(a, ptrs, BatchArgs{}, bits, stream);
}

// a.scale holds (lo, hi) pairs.
hipError_t launch_aggregate_decode_ranged(const AggDecodeArgs& a, const FusedPayloadPtrs& ptrs,
                                          uint32_t bits, hipStream_t stream) {
    using namespace k14;
    if (a.chunks == 0) return hipSuccess;
    if (wide_sums(a.W, bits)) return launch_aggregate_decode_wide<4, false, true>(a, ptrs, BatchArgs{}, stream);
    uint32_t G = bits == 2   ? resident_grid<aggregate_decode_kernel<2, false, true>>()
                 : bits == 4 ? resident_grid<aggregate_decode_kernel<4, false, true>>()
                             : resident_grid<aggregate_decode_kernel<8, false, true>>();
    if (G == 0) return hipErrorInvalidValue;
    if (G > a.chunks) G = (uint32_t)a.chunks;
    const BatchArgs none{};
    if (bits == 2)
        hipLaunchKernelGGL((aggregate_decode_kernel<2, false, true>), dim3(G), dim3(kThreads), 0, stream, a, ptrs, none);
    else if (bits == 4)
        hipLaunchKernelGGL((aggregate_decode_kernel<4, false, true>), dim3(G), dim3(kThreads), 0, stream, a, ptrs, none);
    else
        hipLaunchKernelGGL((aggregate_decode_kernel<8, false, true>), dim3(G), dim3(kThreads), 0, stream, a, ptrs, none);
    return hipGetLastError();
}

hipError_t launch_aggregate_decode_batch(const AggDecodeArgs& a, const BatchArgs& batch, uint32_t bits,
                                         hipStream_t stream) {
    return k14::launch_aggregate_decode_pick<true>(a, FusedPayloadPtrs{}, batch, bits, stream);
}

bool sat_aggregate_decode_fused_applicable(uint32_t W, uint32_t chunk_log2) {
    return chunk_log2 == 14 && W <= (uint32_t)kMaxFusedPayloads;
}

hipError_t launch_sat_aggregate_decode_fused(const SatAggDecodeArgs& a, const FusedPayloadPtrs& ptrs,
                                             uint32_t bits, hipStream_t stream) {
    using namespace k14;
    if (a.chunks == 0) return hipSuccess;
    uint32_t G = 0;
#define THC_SATDEC(B, C)                                                                          \
    do {                                                                                          \
        G = resident_grid<sat_aggregate_decode_kernel<B, C>>();                                   \
        if (G == 0) return hipErrorInvalidValue;                                                  \
        if ((uint64_t)G > a.chunks) G = (uint32_t)a.chunks;                                       \
        hipLaunchKernelGGL((sat_aggregate_decode_kernel<B, C>), dim3(G), dim3(kThreads), 0, stream, \
                           a, ptrs);                                                              \
    } while (0)
    if (a.overflow) {
        if (bits == 2) THC_SATDEC(2, true);
        else if (bits == 4) THC_SATDEC(4, true);
        else THC_SATDEC(8, true);
    } else {
        if (bits == 2) THC_SATDEC(2, false);
        else if (bits == 4) THC_SATDEC(4, false);
        else THC_SATDEC(8, false);
    }
#undef THC_SATDEC
    return hipGetLastError();
}

bool aggregate_fast_applicable(uint32_t W, uint32_t bits, uint32_t sum_bytes, uint64_t payload_bytes) {
    if (W > (uint32_t)kMaxFusedPayloads || (payload_bytes & 15u)) return false;
    return (bits != 2 && sum_bytes == 2) || (bits != 8 && sum_bytes == 1);
}

hipError_t launch_aggregate_fast(const FusedPayloadPtrs& ptrs, uint32_t W, uint32_t bits,
                                 uint64_t payload_bytes, void* sums, hipStream_t stream) {
    using namespace k14;
    const uint64_t vecs = payload_bytes / 16u;
    if (vecs == 0) return hipSuccess;
    const int cus = device_cus();
    uint64_t blocks = (vecs + 255u) / 256u;
    const uint64_t cap = (uint64_t)(cus > 0 ? cus : 256) * 16u;
    if (blocks > cap) blocks = cap;
    const dim3 grid((uint32_t)blocks), block(256);
    if (wide_sums(W, bits))   // 4-bit payloads of more than 17 workers: the sums take 16 bits
        hipLaunchKernelGGL((aggregate_fast_kernel<4, uint16_t>), grid, block, 0, stream, ptrs, W, vecs,
                           static_cast<uint16_t*>(sums));
    else if (bits == 2)
        hipLaunchKernelGGL((aggregate_fast_kernel<2, uint8_t>), grid, block, 0, stream, ptrs, W, vecs,
                           static_cast<uint8_t*>(sums));
    else if (bits == 4)
        hipLaunchKernelGGL((aggregate_fast_kernel<4, uint8_t>), grid, block, 0, stream, ptrs, W, vecs,
                           static_cast<uint8_t*>(sums));
    else
        hipLaunchKernelGGL((aggregate_fast_kernel<8, uint16_t>), grid, block, 0, stream, ptrs, W, vecs,
                           static_cast<uint16_t*>(sums));
    return hipGetLastError();
}

}  // namespace thc
