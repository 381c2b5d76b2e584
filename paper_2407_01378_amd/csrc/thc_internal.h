// Host-side declarations shared by the C ABI layer and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "thc.h"

namespace thc {

// Plain: unsigned, fp32 to fp32 chunk transform (first pass of the full inverse rotation).
// MinMax: per-chunk (min, max) of the rotated values (the min/max-range variant).
// PlainDecode: Plain with the dequantization of stored sums in front (one scale for all chunks).
enum class Mode : int { Forward = 0, Absmax = 1, Encode = 2, Inverse = 3, Decode = 4, Plain = 5, MinMax = 6, PlainDecode = 7 };

// Largest grid index of the two quantization grids: 2^bits points for exact sums,
// 2^bits - 1 points (signed symmetric, centre M = 2^(bits-1) - 1) for saturating sums.
inline uint32_t grid_levels(uint32_t bits, bool sat) { return (1u << bits) - (sat ? 2u : 1u); }

// One description for every per-chunk kernel (rotation, range, encode, decode).
struct ChunkArgs {
    const void* in;         // gradient (fp32/bf16), y (fp32) or sums (u8/u16)
    void* out;              // y, absmax, payload or x
    const float* scale_in;  // shared scale (encode, may be null) / scale (decode)
    float* scale_out;       // scale actually used by encode (may be null)
    uint64_t n;             // coordinates of one worker
    uint64_t padded;        // chunks * c
    uint64_t payload_bytes; // ceil(padded * bits / 8)
    uint32_t chunk_log2;
    uint32_t key0, key1;    // seed, low and high word
    uint32_t worker;
    uint32_t bits;
    uint32_t W;
    uint32_t in_bf16;       // 1: gradient is bf16
    uint32_t sum_bytes;     // decode: 1 or 2
    uint32_t levels;        // encode / decode: largest grid index L
    uint32_t sat;           // decode: 1 = `in` is the packed saturated aggregate (offset binary)
    const float* range_in;  // encode / decode: (lo, hi) per chunk -> min/max grid; null -> symmetric
    uint32_t no_rotate;     // 1: no sign diagonal, no butterflies, no normalisation
    uint32_t out_bf16;      // inverse / decode: 1 = output is bf16 (round to nearest even)
    float inv_sqrt_c;       // fp32 nearest of c^(-1/2)
    uint32_t scale_shared;  // decode: 1 = scale_in is ONE float for all chunks (full rotation)
};

// Generic path: any chunk_log2 in [1, 14], any alignment the ABI allows.
hipError_t launch_generic(Mode mode, const ChunkArgs& a, hipStream_t stream);

// Tuned path for chunk_log2 == 14 and 16-byte aligned buffers; same results.
bool fast14_applicable(Mode mode, const ChunkArgs& a);
hipError_t launch_fast14(Mode mode, const ChunkArgs& a, hipStream_t stream);

// Picks the tuned kernels when they apply, the generic ones otherwise.
inline hipError_t launch_chunks(Mode mode, const ChunkArgs& a, hipStream_t stream) {
    return fast14_applicable(mode, a) ? launch_fast14(mode, a, stream)
                                      : launch_generic(mode, a, stream);
}

// ---- fused paths (chunk_log2 == 14) ------------------------------------------------
constexpr int kMaxFusedWorkers = 64;
struct FusedWorkerPtrs {
    const void* grad[kMaxFusedWorkers];
    uint8_t* payload[kMaxFusedWorkers];
};
struct EncodeAllArgs {
    uint64_t n;
    uint64_t chunks;
    uint32_t W;
    uint32_t key0, key1;
    uint32_t max_spins;  // bound on the polls of one wait
    uint32_t levels;     // largest grid index L
    float* scale;        // out: chunks shared scales
    uint32_t* slots;     // zero on entry and on exit: chunks x encode_all_slot_words(W) words
    uint32_t* done;      // zero on entry and on exit: one arrival counter per chunk
    uint32_t* error;     // zeroed: set to 1 if a wait timed out
};
// ---- batched forms: several buckets in one launch ---------------------------------------
// One record per bucket in device memory, followed by the bucket's W gradient pointers and
// its W payload pointers; the records are sorted by chunk0.
struct BatchRecord {
    uint64_t n;         // coordinates of the bucket (> 0)
    uint64_t chunk0;    // chunks of all earlier buckets of the launch
    uint32_t key0, key1;
    float* scale;
    float* out;         // decode only
};
inline uint32_t batch_record_bytes(uint32_t W) { return (uint32_t)sizeof(BatchRecord) + 16u * W; }
struct BatchArgs {
    const uint8_t* records;
    uint32_t record_bytes;
    uint32_t count;
};
constexpr int kBlobWords = 832;   // 32-bit words one launch of the record writer carries as arguments
// dst[0 .. count) = host_words[0 .. count), by small kernels that take the words as arguments.
hipError_t launch_write_words(uint32_t* dst, const uint32_t* host_words, uint32_t count, hipStream_t stream);
// a.n is unused, a.chunks the total over the buckets, a.scale unused.
hipError_t launch_encode_all_batch(const struct EncodeAllArgs& a, const BatchArgs& batch, bool bf16, bool any_odd,
                                   uint32_t bits, hipStream_t stream);
hipError_t launch_aggregate_decode_batch(const struct AggDecodeArgs& a, const BatchArgs& batch, uint32_t bits,
                                         hipStream_t stream);

// Words per chunk in `slots`: one for every wave of every worker's workgroup.
uint32_t encode_all_slot_words(uint32_t W);
bool encode_all_fused_applicable(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs,
                                 uint32_t chunk_log2, bool bf16, uint32_t bits);
hipError_t launch_encode_all_fused(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, bool bf16,
                                   uint32_t bits, hipStream_t stream);
hipError_t launch_zero_words(uint32_t* dst, uint64_t words, hipStream_t stream);
// *dst = *src, one 32-bit word, on the stream (a kernel, so that it can be captured).
hipError_t launch_copy_word(const uint32_t* src, uint32_t* dst, hipStream_t stream);

constexpr int kMaxFusedPayloads = 64;
struct FusedPayloadPtrs {
    const uint8_t* p[kMaxFusedPayloads];
};
struct AggDecodeArgs {
    uint64_t n;
    uint64_t chunks;
    uint32_t W;
    uint32_t key0, key1;
    const float* scale;
    void* sums;  // may be null
    float* out;
};
bool aggregate_decode_fused_applicable(uint32_t W, uint32_t chunk_log2, uint32_t bits);
hipError_t launch_aggregate_decode_fused(const AggDecodeArgs& a, const FusedPayloadPtrs& ptrs,
                                         uint32_t bits, hipStream_t stream);
// min/max grid: a.scale holds (lo, hi) pairs
hipError_t launch_aggregate_decode_ranged(const AggDecodeArgs& a, const FusedPayloadPtrs& ptrs,
                                          uint32_t bits, hipStream_t stream);
// The rotated one-pass encoder on the min/max grid (thc_fused14.hip, the kernel of thc_encode_all).
hipError_t launch_encode_all_ranged(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, bool bf16,
                                    uint32_t bits, hipStream_t stream);
// One-pass encoder of the min/max variant (thc_fused14_minmax.hip): a.scale receives (lo, hi)
// pairs, a.slots has encode_all_minmax_slot_words(W) words per chunk.
uint32_t encode_all_minmax_slot_words(uint32_t W);
hipError_t launch_encode_all_minmax(const EncodeAllArgs& a, const FusedWorkerPtrs& ptrs, bool bf16, bool rotate,
                                    uint32_t bits, hipStream_t stream);
hipError_t launch_unrotated_aggregate_decode(const FusedPayloadPtrs& ptrs, uint32_t W, const float* range,
                                             uint32_t bits, uint64_t n, float* out, hipStream_t stream);
hipError_t launch_unrotated_decode(const void* sums, uint32_t sum_bytes, const float* range, uint32_t W,
                                   uint32_t bits, uint32_t chunk_log2, uint64_t n, bool out_bf16, void* out,
                                   hipStream_t stream);
bool aggregate_fast_applicable(uint32_t W, uint32_t bits, uint32_t sum_bytes, uint64_t payload_bytes);
hipError_t launch_aggregate_fast(const FusedPayloadPtrs& ptrs, uint32_t W, uint32_t bits,
                                 uint64_t payload_bytes, void* sums, hipStream_t stream);

// ---- saturating aggregation ----------------------------------------------------------
struct SatAggDecodeArgs {
    uint64_t n;
    uint64_t chunks;
    uint32_t W;
    uint32_t key0, key1;
    const float* scale;
    uint8_t* aggregate;             // may be null: packed b-bit aggregate, offset binary
    unsigned long long* overflow;   // may be null: += coordinates with a clipped Sat step
    float* out;
};
bool sat_aggregate_decode_fused_applicable(uint32_t W, uint32_t chunk_log2);
hipError_t launch_sat_aggregate_decode_fused(const SatAggDecodeArgs& a, const FusedPayloadPtrs& ptrs,
                                             uint32_t bits, hipStream_t stream);
// Any chunk size: W <= kMaxFusedPayloads payloads -> packed aggregate (+ overflow count).
hipError_t launch_sat_aggregate(const FusedPayloadPtrs& ptrs, uint32_t W, uint32_t bits,
                                uint64_t payload_bytes, uint64_t padded, uint8_t* aggregate,
                                unsigned long long* overflow, hipStream_t stream);

// ---- full rotation (thc_full.hip) -----------------------------------------------------
// The last forward pass put off until the shared scale is known: evaluated for the range only
// (every earlier pass runs as usual), or run on its own with its results quantized instead of
// stored.  (No FullDeferred at all: every pass runs and stores.)
enum class FullLast : int { RangeOnly = 1, EncodeOnly = 2 };
struct FullDeferred {
    FullLast kind;
    const float* scale;
    uint32_t levels, bits, worker;
    uint8_t* payload;
};
hipError_t launch_high_passes(float* data, uint32_t log2_size, float factor, float* x, uint64_t n,
                              uint32_t key0, uint32_t key1, hipStream_t stream, uint64_t valid,
                              float* absmax, const FullDeferred* deferred = nullptr);
hipError_t launch_full_absmax(const float* y, uint32_t log2_size, float* absmax, hipStream_t stream);
hipError_t launch_full_encode(const float* y, uint32_t log2_size, const float* scale, uint32_t levels,
                              uint32_t bits, uint32_t worker, uint32_t key0, uint32_t key1,
                              uint8_t* payload, hipStream_t stream);
hipError_t launch_full_decode(const void* sums, uint32_t sum_bytes, uint32_t log2_size, const float* scale,
                              uint32_t levels, uint32_t W, float* yhat, hipStream_t stream);

// ---- TopKC (topkc.hip) ----------------------------------------------------------------
hipError_t launch_topkc_norms(const void* grad, bool bf16, uint64_t n, uint32_t C, uint16_t* norms,
                              hipStream_t stream);
hipError_t launch_topkc_sum_norms(const uint16_t* norms_all, uint32_t W, uint64_t P, uint16_t* s,
                                  hipStream_t stream);
uint64_t topkc_select_workspace_words(uint64_t P);
hipError_t launch_topkc_select(const uint16_t* s, uint64_t P, uint32_t J, uint32_t* indices, uint32_t* ws,
                               hipStream_t stream);
hipError_t launch_topkc_gather_sum(const FusedWorkerPtrs& ptrs, bool bf16, uint32_t W, uint64_t n, uint32_t C,
                                   const uint32_t* indices, uint32_t J, uint16_t* values, hipStream_t stream);
hipError_t launch_topkc_scatter(const uint16_t* values, const uint32_t* indices, uint32_t J, uint32_t C,
                                uint32_t W, uint64_t n, float* out, hipStream_t stream);

constexpr int kMaxAggBatch = 16;
struct PayloadBatch {
    const uint8_t* p[kMaxAggBatch];
};

hipError_t launch_aggregate(const PayloadBatch& batch, uint32_t count, bool accumulate,
                            uint32_t bits, uint32_t sum_bytes, uint64_t payload_bytes,
                            uint64_t padded, void* sums, hipStream_t stream);

hipError_t launch_scale_reduce(const float* absmax_all, uint32_t W, uint64_t chunks, float* scale,
                               hipStream_t stream);
// (lo, hi) pairs: min of the workers' minima, max of their maxima.
hipError_t launch_range_reduce(const float* range_all, uint32_t W, uint64_t chunks, float* range,
                               hipStream_t stream);

}  // namespace thc
