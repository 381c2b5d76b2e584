// C ABI of the library: argument checking on the host (before any HIP call), then
// dispatch to the kernel launchers.  See include/thc.h for the contract.
#include <math.h>
#include <string.h>

#include <mutex>

#include "thc_internal.h"

namespace {

using thc::ChunkArgs;
using thc::Mode;

constexpr uint64_t kMaxCoords = 1ull << 44;  // keeps every byte count far below 2^63

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_common(uint64_t n, uint32_t chunk_log2) {
    if (chunk_log2 < 1 || chunk_log2 > 14) return THC_ERR_CHUNK;
    if (n > kMaxCoords) return THC_ERR_SIZE;
    return THC_OK;
}

int check_bits(uint32_t bits) { return (bits == 2 || bits == 4 || bits == 8) ? THC_OK : THC_ERR_BITS; }

int check_dtype(int dt) { return (dt == THC_F32 || dt == THC_BF16) ? THC_OK : THC_ERR_DTYPE; }

uint64_t padded_coords(uint64_t n, uint32_t chunk_log2) {
    const uint64_t c = 1ull << chunk_log2;
    return (n + c - 1) / c * c;
}

ChunkArgs base_args(uint64_t n, uint32_t chunk_log2, uint64_t seed) {
    ChunkArgs a{};
    a.n = n;
    a.padded = padded_coords(n, chunk_log2);
    a.chunk_log2 = chunk_log2;
    a.key0 = (uint32_t)seed;
    a.key1 = (uint32_t)(seed >> 32);
    a.inv_sqrt_c = (float)(1.0 / sqrt((double)(1ull << chunk_log2)));
    return a;
}

int finish(hipError_t e) { return e == hipSuccess ? THC_OK : THC_ERR_HIP; }

}  // namespace

extern "C" {

const char* thc_status_string(int status) {
    switch (status) {
        case THC_OK: return "ok";
        case THC_ERR_NULL: return "a required pointer is NULL";
        case THC_ERR_BITS: return "bits must be 2, 4 or 8";
        case THC_ERR_CHUNK: return "chunk_log2 must be in [1, 14]";
        case THC_ERR_WORKERS: return "W must be >= 1 and W * (2^bits - 1) <= 65535";
        case THC_ERR_DTYPE: return "dtype must be THC_F32 or THC_BF16";
        case THC_ERR_SIZE: return "size out of range";
        case THC_ERR_HIP: return "HIP call failed";
        case THC_ERR_ALIGN: return "pointer not aligned as required";
        default: return "unknown status";
    }
}

int thc_version(void) { return 200; }

uint32_t thc_rounding_bits(void) { return 8; }

uint64_t thc_num_chunks(uint64_t n, uint32_t chunk_log2) {
    if (check_common(n, chunk_log2) != THC_OK) return 0;
    return padded_coords(n, chunk_log2) >> chunk_log2;
}

uint64_t thc_payload_bytes(uint64_t n, uint32_t chunk_log2, uint32_t bits) {
    if (check_common(n, chunk_log2) != THC_OK || check_bits(bits) != THC_OK) return 0;
    return (padded_coords(n, chunk_log2) * bits + 7) / 8;
}

uint32_t thc_sum_bytes(uint32_t W, uint32_t bits) {
    if (W == 0 || check_bits(bits) != THC_OK) return 0;
    const uint64_t top = (uint64_t)W * ((1u << bits) - 1u);
    if (top <= 255) return 1;
    if (top <= 65535) return 2;
    return 0;
}

int rht_forward(const void* x, thc_dtype dt, uint64_t n, uint32_t chunk_log2, uint64_t seed,
                float* y, void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_dtype(dt);
    if (rc != THC_OK) return rc;
    if (n == 0) return THC_OK;
    if (!x || !y) return THC_ERR_NULL;
    if (!aligned(x, dt == THC_F32 ? 4 : 2) || !aligned(y, 4)) return THC_ERR_ALIGN;
    ChunkArgs a = base_args(n, chunk_log2, seed);
    a.in = x;
    a.out = y;
    a.in_bf16 = dt == THC_BF16;
    return finish(thc::launch_chunks(Mode::Forward, a, static_cast<hipStream_t>(stream)));
}

int rht_inverse(const float* y, uint64_t n, uint32_t chunk_log2, uint64_t seed, float* x,
                void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc != THC_OK) return rc;
    if (n == 0) return THC_OK;
    if (!x || !y) return THC_ERR_NULL;
    if (!aligned(x, 4) || !aligned(y, 4)) return THC_ERR_ALIGN;
    ChunkArgs a = base_args(n, chunk_log2, seed);
    a.in = y;
    a.out = x;
    return finish(thc::launch_chunks(Mode::Inverse, a, static_cast<hipStream_t>(stream)));
}

int thc_chunk_absmax(const void* grad, thc_dtype dt, uint64_t n, uint32_t chunk_log2,
                     uint64_t seed, float* absmax, void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_dtype(dt);
    if (rc != THC_OK) return rc;
    if (n == 0) return THC_OK;
    if (!grad || !absmax) return THC_ERR_NULL;
    if (!aligned(grad, dt == THC_F32 ? 4 : 2) || !aligned(absmax, 4)) return THC_ERR_ALIGN;
    ChunkArgs a = base_args(n, chunk_log2, seed);
    a.in = grad;
    a.out = absmax;
    a.in_bf16 = dt == THC_BF16;
    return finish(thc::launch_chunks(Mode::Absmax, a, static_cast<hipStream_t>(stream)));
}

int thc_scale_reduce(const float* absmax_all, uint32_t W, uint64_t chunks, float* scale,
                     void* stream) {
    if (W == 0) return THC_ERR_WORKERS;
    if (chunks > kMaxCoords || (uint64_t)W * chunks > kMaxCoords) return THC_ERR_SIZE;
    if (chunks == 0) return THC_OK;
    if (!absmax_all || !scale) return THC_ERR_NULL;
    if (!aligned(absmax_all, 4) || !aligned(scale, 4)) return THC_ERR_ALIGN;
    return finish(
        thc::launch_scale_reduce(absmax_all, W, chunks, scale, static_cast<hipStream_t>(stream)));
}

static int encode_impl(const void* grad, thc_dtype dt, uint64_t n, uint32_t chunk_log2, uint64_t seed,
                       uint32_t worker, uint32_t bits, const float* shared_scale, uint8_t* payload,
                       float* scale_out, void* stream, bool sat) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_dtype(dt);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (n == 0) return THC_OK;
    if (!grad || !payload) return THC_ERR_NULL;
    if (!aligned(grad, dt == THC_F32 ? 4 : 2) || !aligned(payload, 16) ||
        !aligned(shared_scale, 4) || !aligned(scale_out, 4))
        return THC_ERR_ALIGN;
    ChunkArgs a = base_args(n, chunk_log2, seed);
    a.in = grad;
    a.out = payload;
    a.scale_in = shared_scale;
    a.scale_out = scale_out;
    a.in_bf16 = dt == THC_BF16;
    a.worker = worker;
    a.bits = bits;
    a.levels = thc::grid_levels(bits, sat);
    a.payload_bytes = (a.padded * bits + 7) / 8;
    return finish(thc::launch_chunks(Mode::Encode, a, static_cast<hipStream_t>(stream)));
}

int thc_encode(const void* grad, thc_dtype dt, uint64_t n, uint32_t chunk_log2, uint64_t seed,
               uint32_t worker, uint32_t bits, const float* shared_scale, uint8_t* payload,
               float* scale_out, void* stream) {
    return encode_impl(grad, dt, n, chunk_log2, seed, worker, bits, shared_scale, payload, scale_out,
                       stream, false);
}

int thc_aggregate(const uint8_t* const* payloads, uint32_t W, uint64_t n, uint32_t chunk_log2,
                  uint32_t bits, void* sums, void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    const uint32_t sum_bytes = thc_sum_bytes(W, bits);
    if (sum_bytes == 0) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    if (!payloads || !sums) return THC_ERR_NULL;
    for (uint32_t w = 0; w < W; ++w) {
        if (!payloads[w]) return THC_ERR_NULL;
        if (!aligned(payloads[w], 16)) return THC_ERR_ALIGN;
    }
    if (!aligned(sums, 16)) return THC_ERR_ALIGN;
    const uint64_t padded = padded_coords(n, chunk_log2);
    const uint64_t payload_bytes = (padded * bits + 7) / 8;
    if (thc::aggregate_fast_applicable(W, bits, sum_bytes, payload_bytes)) {
        thc::FusedPayloadPtrs ptrs{};
        for (uint32_t w = 0; w < W; ++w) ptrs.p[w] = payloads[w];
        return finish(thc::launch_aggregate_fast(ptrs, W, bits, payload_bytes, sums,
                                                 static_cast<hipStream_t>(stream)));
    }
    for (uint32_t w0 = 0; w0 < W; w0 += thc::kMaxAggBatch) {
        thc::PayloadBatch batch{};
        const uint32_t count = (W - w0 < (uint32_t)thc::kMaxAggBatch) ? W - w0 : thc::kMaxAggBatch;
        for (uint32_t i = 0; i < count; ++i) batch.p[i] = payloads[w0 + i];
        const hipError_t e =
            thc::launch_aggregate(batch, count, w0 != 0, bits, sum_bytes, payload_bytes, padded,
                                  sums, static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return THC_ERR_HIP;
    }
    return THC_OK;
}

int thc_decode(const void* sums, const float* scale, uint32_t W, uint64_t n, uint32_t chunk_log2,
               uint64_t seed, uint32_t bits, float* out, void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    const uint32_t sum_bytes = thc_sum_bytes(W, bits);
    if (sum_bytes == 0) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    if (!sums || !scale || !out) return THC_ERR_NULL;
    if (!aligned(sums, 16) || !aligned(scale, 4) || !aligned(out, 4)) return THC_ERR_ALIGN;
    ChunkArgs a = base_args(n, chunk_log2, seed);
    a.in = sums;
    a.out = out;
    a.scale_in = scale;
    a.bits = bits;
    a.levels = thc::grid_levels(bits, false);
    a.W = W;
    a.sum_bytes = sum_bytes;
    return finish(thc::launch_chunks(Mode::Decode, a, static_cast<hipStream_t>(stream)));
}

// ------------------------------------------------------------- batched / fused forms
static uint32_t g_spin_limit = 1u << 22;

void thc_set_spin_limit(uint32_t polls) { g_spin_limit = polls; }

uint64_t thc_encode_all_workspace_bytes(uint32_t W, uint64_t n, uint32_t chunk_log2) {
    if (W == 0 || check_common(n, chunk_log2) != THC_OK) return 0;
    const uint64_t chunks = padded_coords(n, chunk_log2) >> chunk_log2;
    // error word (padded to 16 bytes) + one word per chunk for every wave of every
    // worker's workgroup (the unfused fallback keeps its per-worker ranges there too) +
    // one arrival counter per chunk
    return 16 + 4 * ((uint64_t)thc::encode_all_slot_words(W) + 1u) * chunks;
}

int thc_workspace_clear(void* workspace, uint64_t workspace_bytes, void* stream) {
    if (workspace_bytes == 0) return THC_OK;
    if (!workspace) return THC_ERR_NULL;
    if (!aligned(workspace, 16) || (workspace_bytes & 3u) != 0) return THC_ERR_ALIGN;
    return finish(thc::launch_zero_words(static_cast<uint32_t*>(workspace), workspace_bytes / 4,
                                         static_cast<hipStream_t>(stream)));
}

static int encode_all_impl(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n,
                           uint32_t chunk_log2, uint64_t seed, uint32_t bits, uint8_t* const* payloads,
                           float* scale, void* workspace, uint64_t workspace_bytes, void* stream,
                           bool sat, bool cleared) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_dtype(dt);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (thc_sum_bytes(W, bits) == 0) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    if (!grads || !payloads || !scale || !workspace) return THC_ERR_NULL;
    for (uint32_t w = 0; w < W; ++w) {
        if (!grads[w] || !payloads[w]) return THC_ERR_NULL;
        if (!aligned(grads[w], dt == THC_F32 ? 4 : 2) || !aligned(payloads[w], 16)) return THC_ERR_ALIGN;
    }
    if (!aligned(scale, 4) || !aligned(workspace, 16)) return THC_ERR_ALIGN;
    if (workspace_bytes < thc_encode_all_workspace_bytes(W, n, chunk_log2)) return THC_ERR_SIZE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint64_t chunks = padded_coords(n, chunk_log2) >> chunk_log2;
    uint32_t* words = static_cast<uint32_t*>(workspace);

    thc::EncodeAllArgs a{};
    a.n = n;
    a.chunks = chunks;
    a.W = W;
    a.key0 = (uint32_t)seed;
    a.key1 = (uint32_t)(seed >> 32);
    a.max_spins = g_spin_limit;
    a.levels = thc::grid_levels(bits, sat);
    a.scale = scale;
    const uint64_t slot_words = (uint64_t)thc::encode_all_slot_words(W) * chunks;
    a.error = words;
    a.slots = words + 4;
    a.done = words + 4 + slot_words;
    if (W <= (uint32_t)thc::kMaxFusedWorkers) {
        thc::FusedWorkerPtrs ptrs{};
        for (uint32_t w = 0; w < W; ++w) {
            ptrs.grad[w] = grads[w];
            ptrs.payload[w] = payloads[w];
        }
        if (thc::encode_all_fused_applicable(a, ptrs, chunk_log2, dt == THC_BF16, bits)) {
            // The kernel needs the words zero and leaves them zero (the last wave to have
            // read a chunk's words clears them), so a workspace known to be clear skips this.
            if (!cleared && thc::launch_zero_words(words, 4 + slot_words + chunks, st) != hipSuccess)
                return THC_ERR_HIP;
            return finish(thc::launch_encode_all_fused(a, ptrs, dt == THC_BF16, bits, st));
        }
    }
    // Fallback: the unfused sequence, per-worker ranges kept in the workspace.
    if (!cleared && thc::launch_zero_words(words, 4, st) != hipSuccess) return THC_ERR_HIP;
    float* absmax_all = reinterpret_cast<float*>(words + 4);
    for (uint32_t w = 0; w < W; ++w) {
        rc = thc_chunk_absmax(grads[w], dt, n, chunk_log2, seed, absmax_all + (uint64_t)w * chunks, stream);
        if (rc != THC_OK) return rc;
    }
    rc = thc_scale_reduce(absmax_all, W, chunks, scale, stream);
    for (uint32_t w = 0; rc == THC_OK && w < W; ++w)
        rc = encode_impl(grads[w], dt, n, chunk_log2, seed, w, bits, scale, payloads[w], nullptr, stream, sat);
    // a workspace that came in clear goes out clear
    if (cleared && thc::launch_zero_words(words + 4, (uint64_t)W * chunks, st) != hipSuccess) return THC_ERR_HIP;
    return rc;
}

int thc_encode_all(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n,
                   uint32_t chunk_log2, uint64_t seed, uint32_t bits, uint8_t* const* payloads,
                   float* scale, void* workspace, uint64_t workspace_bytes, void* stream) {
    return encode_all_impl(grads, dt, W, n, chunk_log2, seed, bits, payloads, scale, workspace,
                           workspace_bytes, stream, false, false);
}

int thc_encode_all_cleared(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n,
                           uint32_t chunk_log2, uint64_t seed, uint32_t bits, uint8_t* const* payloads,
                           float* scale, void* workspace, uint64_t workspace_bytes, void* stream) {
    return encode_all_impl(grads, dt, W, n, chunk_log2, seed, bits, payloads, scale, workspace,
                           workspace_bytes, stream, false, true);
}

// ---- several buckets in one launch -------------------------------------------------------
namespace {

constexpr uint32_t kMaxBatch = 4096;

struct BatchPlan {
    uint64_t total_chunks = 0;
    uint64_t record_words = 0;    // 32-bit words of all records, padded to 16 bytes
    bool any_odd = false;
};

// Checks that do not depend on the direction, and the sizes that follow from the buckets.
int plan_batch(const thc_bucket* buckets, uint32_t count, uint32_t W, uint32_t chunk_log2, uint32_t bits,
               BatchPlan* plan) {
    if (chunk_log2 != 14) return THC_ERR_CHUNK;
    int rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (thc_sum_bytes(W, bits) == 0 || W > (uint32_t)thc::kMaxFusedWorkers) return THC_ERR_WORKERS;
    if (count > kMaxBatch) return THC_ERR_SIZE;
    if (count != 0 && !buckets) return THC_ERR_NULL;
    for (uint32_t b = 0; b < count; ++b) {
        if (buckets[b].n > kMaxCoords) return THC_ERR_SIZE;
        plan->total_chunks += padded_coords(buckets[b].n, chunk_log2) >> chunk_log2;
        plan->any_odd = plan->any_odd || (buckets[b].n & 1u);
    }
    if (plan->total_chunks * W >= 0x7FFFFFFFull) return THC_ERR_SIZE;
    plan->record_words = ((uint64_t)count * thc::batch_record_bytes(W) + 15u) / 16u * 4u;
    return THC_OK;
}

// Writes the records of the non-empty buckets to `dst` (device) on the stream; returns their number.
int write_records(const thc_bucket* buckets, uint32_t count, uint32_t W, uint32_t chunk_log2, bool decode,
                  uint32_t* dst, hipStream_t st, uint32_t* written) {
    // staged on the stack, one batch of kernel arguments at a time: no host allocation either
    uint32_t stage[thc::kBlobWords];
    const uint32_t rec_words = thc::batch_record_bytes(W) / 4u;
    uint32_t used = 0, live = 0;
    uint64_t chunk0 = 0;
    uint32_t* out = dst;
    for (uint32_t b = 0; b < count; ++b) {
        const thc_bucket& k = buckets[b];
        if (k.n == 0) continue;
        if (used + rec_words > (uint32_t)thc::kBlobWords) {
            if (thc::launch_write_words(out, stage, used, st) != hipSuccess) return THC_ERR_HIP;
            out += used;
            used = 0;
        }
        thc::BatchRecord r{};
        r.n = k.n;
        r.chunk0 = chunk0;
        r.key0 = (uint32_t)k.seed;
        r.key1 = (uint32_t)(k.seed >> 32);
        r.scale = k.scale;
        r.out = decode ? k.out : nullptr;
        memcpy(stage + used, &r, sizeof r);
        uint64_t* ptr = reinterpret_cast<uint64_t*>(stage + used + sizeof(r) / 4u);
        for (uint32_t w = 0; w < W; ++w) {
            ptr[w] = decode ? 0u : reinterpret_cast<uint64_t>(k.grads[w]);
            ptr[W + w] = reinterpret_cast<uint64_t>(k.payloads[w]);
        }
        used += rec_words;
        chunk0 += padded_coords(k.n, chunk_log2) >> chunk_log2;
        ++live;
    }
    if (used != 0 && thc::launch_write_words(out, stage, used, st) != hipSuccess) return THC_ERR_HIP;
    *written = live;
    return THC_OK;
}

}  // namespace

uint64_t thc_batch_workspace_bytes(const thc_bucket* buckets, uint32_t count, uint32_t W, uint32_t chunk_log2) {
    BatchPlan plan;
    if (plan_batch(buckets, count, W, chunk_log2, 4, &plan) != THC_OK) return 0;
    // error word (16 bytes) + records + range words and arrival counters as in thc_encode_all
    return 16 + 4 * plan.record_words + 4 * ((uint64_t)thc::encode_all_slot_words(W) + 1u) * plan.total_chunks;
}

int thc_encode_all_batch(const thc_bucket* buckets, uint32_t count, thc_dtype dt, uint32_t W,
                         uint32_t chunk_log2, uint32_t bits, void* workspace, uint64_t workspace_bytes,
                         void* stream) {
    int rc = check_dtype(dt);
    BatchPlan plan;
    if (rc == THC_OK) rc = plan_batch(buckets, count, W, chunk_log2, bits, &plan);
    if (rc != THC_OK) return rc;
    if (plan.total_chunks == 0) return THC_OK;
    if (!workspace) return THC_ERR_NULL;
    if (!aligned(workspace, 16)) return THC_ERR_ALIGN;
    for (uint32_t b = 0; b < count; ++b) {
        const thc_bucket& k = buckets[b];
        if (k.n == 0) continue;
        if (!k.grads || !k.payloads || !k.scale) return THC_ERR_NULL;
        if (!aligned(k.scale, 4)) return THC_ERR_ALIGN;
        for (uint32_t w = 0; w < W; ++w) {
            if (!k.grads[w] || !k.payloads[w]) return THC_ERR_NULL;
            if (!aligned(k.grads[w], 16) || !aligned(k.payloads[w], 16)) return THC_ERR_ALIGN;
        }
    }
    if (workspace_bytes < thc_batch_workspace_bytes(buckets, count, W, chunk_log2)) return THC_ERR_SIZE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t* words = static_cast<uint32_t*>(workspace);
    uint32_t* records = words + 4;
    uint32_t* slots = records + plan.record_words;
    const uint64_t slot_words = (uint64_t)thc::encode_all_slot_words(W) * plan.total_chunks;

    thc::EncodeAllArgs a{};
    a.chunks = plan.total_chunks;
    a.W = W;
    a.max_spins = g_spin_limit;
    a.levels = thc::grid_levels(bits, false);
    a.error = words;
    a.slots = slots;
    a.done = slots + slot_words;
    thc::BatchArgs batch{};
    batch.records = reinterpret_cast<const uint8_t*>(records);
    batch.record_bytes = thc::batch_record_bytes(W);
    rc = write_records(buckets, count, W, chunk_log2, false, records, st, &batch.count);
    if (rc != THC_OK) return rc;
    if (thc::launch_zero_words(words, 4, st) != hipSuccess) return THC_ERR_HIP;
    if (thc::launch_zero_words(slots, slot_words + plan.total_chunks, st) != hipSuccess) return THC_ERR_HIP;
    const hipError_t e = thc::launch_encode_all_batch(a, batch, dt == THC_BF16, plan.any_odd, bits, st);
    if (e == hipErrorInvalidConfiguration) return THC_ERR_WORKERS;   // fewer resident workgroups than workers
    return finish(e);
}

int thc_aggregate_decode_batch(const thc_bucket* buckets, uint32_t count, uint32_t W, uint32_t chunk_log2,
                               uint32_t bits, void* workspace, uint64_t workspace_bytes, void* stream) {
    BatchPlan plan;
    int rc = plan_batch(buckets, count, W, chunk_log2, bits, &plan);
    if (rc != THC_OK) return rc;
    if (!thc::aggregate_decode_fused_applicable(W, chunk_log2, bits)) return THC_ERR_WORKERS;
    if (plan.total_chunks == 0) return THC_OK;
    if (!workspace) return THC_ERR_NULL;
    if (!aligned(workspace, 16)) return THC_ERR_ALIGN;
    for (uint32_t b = 0; b < count; ++b) {
        const thc_bucket& k = buckets[b];
        if (k.n == 0) continue;
        if (!k.payloads || !k.scale || !k.out) return THC_ERR_NULL;
        if (!aligned(k.scale, 4) || !aligned(k.out, 16)) return THC_ERR_ALIGN;
        for (uint32_t w = 0; w < W; ++w) {
            if (!k.payloads[w]) return THC_ERR_NULL;
            if (!aligned(k.payloads[w], 16)) return THC_ERR_ALIGN;
        }
    }
    if (workspace_bytes < 16 + 4 * plan.record_words) return THC_ERR_SIZE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t* records = static_cast<uint32_t*>(workspace) + 4;
    thc::AggDecodeArgs a{};
    a.chunks = plan.total_chunks;
    a.W = W;
    thc::BatchArgs batch{};
    batch.records = reinterpret_cast<const uint8_t*>(records);
    batch.record_bytes = thc::batch_record_bytes(W);
    rc = write_records(buckets, count, W, chunk_log2, true, records, st, &batch.count);
    if (rc != THC_OK) return rc;
    return finish(thc::launch_aggregate_decode_batch(a, batch, bits, st));
}

// ---- thc_encode_all for callers that cannot allocate ---------------------------------
// The workspace is a file-scope device array: every GPU the library runs on holds its own
// copy at its own address until the process ends.  In host code the array's name is only
// a stand-in for that address; the address is asked for once per device, with that device
// current, and only the pointer obtained that way is handed to kernels.
static __device__ __align__(256) uint32_t scratch[THC_STATIC_SCRATCH_BYTES / 4];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
uint32_t* g_scratch_ptr[kMaxDevices];   // per device, filled on the first call there

int static_scratch(uint32_t** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return THC_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return THC_ERR_HIP;
        g_scratch_ptr[dev] = static_cast<uint32_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return THC_OK;
}
}  // namespace

int thc_encode_all_static(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n,
                          uint32_t chunk_log2, uint64_t seed, uint32_t bits, uint8_t* const* payloads,
                          float* scale, uint32_t* timed_out, void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_dtype(dt);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (thc_sum_bytes(W, bits) == 0) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    if (!aligned(timed_out, 4)) return THC_ERR_ALIGN;
    if (thc_encode_all_workspace_bytes(W, n, chunk_log2) > (uint64_t)THC_STATIC_SCRATCH_BYTES) return THC_ERR_SIZE;
    uint32_t* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != THC_OK) return rc;
    // the array keeps the previous call's contents: this form clears the words it uses first
    rc = encode_all_impl(grads, dt, W, n, chunk_log2, seed, bits, payloads, scale, ws,
                         (uint64_t)THC_STATIC_SCRATCH_BYTES, stream, false, false);
    if (rc != THC_OK || timed_out == nullptr) return rc;
    return finish(thc::launch_copy_word(ws, timed_out, static_cast<hipStream_t>(stream)));
}

int thc_aggregate_decode_is_fused(uint32_t W, uint32_t chunk_log2, uint32_t bits) {
    if (check_bits(bits) != THC_OK || thc_sum_bytes(W, bits) == 0) return 0;
    return thc::aggregate_decode_fused_applicable(W, chunk_log2, bits) ? 1 : 0;
}

int thc_aggregate_decode(const uint8_t* const* payloads, uint32_t W, const float* scale,
                         uint64_t n, uint32_t chunk_log2, uint64_t seed, uint32_t bits,
                         void* sums, float* out, void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (thc_sum_bytes(W, bits) == 0) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    if (!payloads || !scale || !out) return THC_ERR_NULL;
    for (uint32_t w = 0; w < W; ++w) {
        if (!payloads[w]) return THC_ERR_NULL;
        if (!aligned(payloads[w], 16)) return THC_ERR_ALIGN;
    }
    if (!aligned(scale, 4) || !aligned(out, 4) || !aligned(sums, 16)) return THC_ERR_ALIGN;
    if (thc::aggregate_decode_fused_applicable(W, chunk_log2, bits) && aligned(out, 16)) {
        thc::FusedPayloadPtrs ptrs{};
        for (uint32_t w = 0; w < W; ++w) ptrs.p[w] = payloads[w];
        thc::AggDecodeArgs a{};
        a.n = n;
        a.chunks = padded_coords(n, chunk_log2) >> chunk_log2;
        a.W = W;
        a.key0 = (uint32_t)seed;
        a.key1 = (uint32_t)(seed >> 32);
        a.scale = scale;
        a.sums = sums;
        a.out = out;
        return finish(thc::launch_aggregate_decode_fused(a, ptrs, bits, static_cast<hipStream_t>(stream)));
    }
    if (!sums) return THC_ERR_NULL;
    rc = thc_aggregate(payloads, W, n, chunk_log2, bits, sums, stream);
    if (rc != THC_OK) return rc;
    return thc_decode(sums, scale, W, n, chunk_log2, seed, bits, out, stream);
}

// ------------------------------------------------- saturation-based aggregation
uint32_t thc_sat_max(uint32_t bits) {
    return check_bits(bits) == THC_OK ? (1u << (bits - 1)) - 1u : 0u;
}

int thc_sat_encode(const void* grad, thc_dtype dt, uint64_t n, uint32_t chunk_log2, uint64_t seed,
                   uint32_t worker, uint32_t bits, const float* shared_scale, uint8_t* payload,
                   float* scale_out, void* stream) {
    return encode_impl(grad, dt, n, chunk_log2, seed, worker, bits, shared_scale, payload, scale_out,
                       stream, true);
}

int thc_sat_encode_all(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n,
                       uint32_t chunk_log2, uint64_t seed, uint32_t bits, uint8_t* const* payloads,
                       float* scale, void* workspace, uint64_t workspace_bytes, void* stream) {
    return encode_all_impl(grads, dt, W, n, chunk_log2, seed, bits, payloads, scale, workspace,
                           workspace_bytes, stream, true, false);
}

int thc_sat_encode_all_cleared(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n,
                               uint32_t chunk_log2, uint64_t seed, uint32_t bits,
                               uint8_t* const* payloads, float* scale, void* workspace,
                               uint64_t workspace_bytes, void* stream) {
    return encode_all_impl(grads, dt, W, n, chunk_log2, seed, bits, payloads, scale, workspace,
                           workspace_bytes, stream, true, true);
}

static int check_sat_payloads(const uint8_t* const* payloads, uint32_t W) {
    if (W == 0 || W > (uint32_t)thc::kMaxFusedPayloads) return THC_ERR_WORKERS;
    if (!payloads) return THC_ERR_NULL;
    for (uint32_t w = 0; w < W; ++w) {
        if (!payloads[w]) return THC_ERR_NULL;
        if (!aligned(payloads[w], 16)) return THC_ERR_ALIGN;
    }
    return THC_OK;
}

int thc_sat_aggregate(const uint8_t* const* payloads, uint32_t W, uint64_t n, uint32_t chunk_log2,
                      uint32_t bits, uint8_t* aggregate, unsigned long long* overflow_count,
                      void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (W == 0 || W > (uint32_t)thc::kMaxFusedPayloads) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    rc = check_sat_payloads(payloads, W);
    if (rc != THC_OK) return rc;
    if (!aggregate) return THC_ERR_NULL;
    if (!aligned(aggregate, 16) || !aligned(overflow_count, 8)) return THC_ERR_ALIGN;
    const uint64_t padded = padded_coords(n, chunk_log2);
    thc::FusedPayloadPtrs ptrs{};
    for (uint32_t w = 0; w < W; ++w) ptrs.p[w] = payloads[w];
    return finish(thc::launch_sat_aggregate(ptrs, W, bits, (padded * bits + 7) / 8, padded, aggregate,
                                            overflow_count, static_cast<hipStream_t>(stream)));
}

int thc_sat_decode(const uint8_t* aggregate, const float* scale, uint32_t W, uint64_t n,
                   uint32_t chunk_log2, uint64_t seed, uint32_t bits, float* out, void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (W == 0) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    if (!aggregate || !scale || !out) return THC_ERR_NULL;
    if (!aligned(aggregate, 16) || !aligned(scale, 4) || !aligned(out, 4)) return THC_ERR_ALIGN;
    ChunkArgs a = base_args(n, chunk_log2, seed);
    a.in = aggregate;
    a.out = out;
    a.scale_in = scale;
    a.bits = bits;
    a.levels = thc::grid_levels(bits, true);
    a.W = W;
    a.sat = 1;
    return finish(thc::launch_chunks(Mode::Decode, a, static_cast<hipStream_t>(stream)));
}

int thc_sat_aggregate_decode_is_fused(uint32_t W, uint32_t chunk_log2, uint32_t bits) {
    if (check_bits(bits) != THC_OK || W == 0) return 0;
    return thc::sat_aggregate_decode_fused_applicable(W, chunk_log2) ? 1 : 0;
}

int thc_sat_aggregate_decode(const uint8_t* const* payloads, uint32_t W, const float* scale,
                             uint64_t n, uint32_t chunk_log2, uint64_t seed, uint32_t bits,
                             uint8_t* aggregate, unsigned long long* overflow_count, float* out,
                             void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (W == 0 || W > (uint32_t)thc::kMaxFusedPayloads) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    rc = check_sat_payloads(payloads, W);
    if (rc != THC_OK) return rc;
    if (!scale || !out) return THC_ERR_NULL;
    if (!aligned(scale, 4) || !aligned(out, 4) || !aligned(aggregate, 16) || !aligned(overflow_count, 8))
        return THC_ERR_ALIGN;
    if (thc::sat_aggregate_decode_fused_applicable(W, chunk_log2) && aligned(out, 16)) {
        thc::FusedPayloadPtrs ptrs{};
        for (uint32_t w = 0; w < W; ++w) ptrs.p[w] = payloads[w];
        thc::SatAggDecodeArgs a{};
        a.n = n;
        a.chunks = padded_coords(n, chunk_log2) >> chunk_log2;
        a.W = W;
        a.key0 = (uint32_t)seed;
        a.key1 = (uint32_t)(seed >> 32);
        a.scale = scale;
        a.aggregate = aggregate;
        a.overflow = overflow_count;
        a.out = out;
        return finish(thc::launch_sat_aggregate_decode_fused(a, ptrs, bits, static_cast<hipStream_t>(stream)));
    }
    if (!aggregate) return THC_ERR_NULL;
    rc = thc_sat_aggregate(payloads, W, n, chunk_log2, bits, aggregate, overflow_count, stream);
    if (rc != THC_OK) return rc;
    return thc_sat_decode(aggregate, scale, W, n, chunk_log2, seed, bits, out, stream);
}

// ------------------------------------------------------------------ min/max range
int thc_chunk_minmax(const void* grad, thc_dtype dt, uint64_t n, uint32_t chunk_log2, uint64_t seed,
                     int rotate, float* range, void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_dtype(dt);
    if (rc != THC_OK) return rc;
    if (n == 0) return THC_OK;
    if (!grad || !range) return THC_ERR_NULL;
    if (!aligned(grad, dt == THC_F32 ? 4 : 2) || !aligned(range, 8)) return THC_ERR_ALIGN;
    ChunkArgs a = base_args(n, chunk_log2, seed);
    a.in = grad;
    a.out = range;
    a.in_bf16 = dt == THC_BF16;
    a.no_rotate = rotate ? 0u : 1u;
    return finish(thc::launch_chunks(Mode::MinMax, a, static_cast<hipStream_t>(stream)));
}

int thc_range_reduce(const float* range_all, uint32_t W, uint64_t chunks, float* range, void* stream) {
    if (W == 0) return THC_ERR_WORKERS;
    if (chunks > kMaxCoords || (uint64_t)W * chunks > kMaxCoords) return THC_ERR_SIZE;
    if (chunks == 0) return THC_OK;
    if (!range_all || !range) return THC_ERR_NULL;
    if (!aligned(range_all, 8) || !aligned(range, 8)) return THC_ERR_ALIGN;
    return finish(thc::launch_range_reduce(range_all, W, chunks, range, static_cast<hipStream_t>(stream)));
}

int thc_encode_minmax(const void* grad, thc_dtype dt, uint64_t n, uint32_t chunk_log2, uint64_t seed,
                      uint32_t worker, uint32_t bits, int rotate, const float* range, uint8_t* payload,
                      void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_dtype(dt);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (n == 0) return THC_OK;
    if (!grad || !payload || !range) return THC_ERR_NULL;
    if (!aligned(grad, dt == THC_F32 ? 4 : 2) || !aligned(payload, 16) || !aligned(range, 8))
        return THC_ERR_ALIGN;
    ChunkArgs a = base_args(n, chunk_log2, seed);
    a.in = grad;
    a.out = payload;
    a.range_in = range;
    a.in_bf16 = dt == THC_BF16;
    a.worker = worker;
    a.bits = bits;
    a.levels = thc::grid_levels(bits, false);
    a.payload_bytes = (a.padded * bits + 7) / 8;
    a.no_rotate = rotate ? 0u : 1u;
    return finish(thc::launch_chunks(Mode::Encode, a, static_cast<hipStream_t>(stream)));
}

int thc_decode_minmax(const void* sums, const float* range, uint32_t W, uint64_t n, uint32_t chunk_log2,
                      uint64_t seed, uint32_t bits, int rotate, thc_dtype out_dt, void* out, void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc == THC_OK) rc = check_dtype(out_dt);
    if (rc != THC_OK) return rc;
    const uint32_t sum_bytes = thc_sum_bytes(W, bits);
    if (sum_bytes == 0) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    if (!sums || !range || !out) return THC_ERR_NULL;
    if (!aligned(sums, 16) || !aligned(range, 8) || !aligned(out, out_dt == THC_F32 ? 4 : 2))
        return THC_ERR_ALIGN;
    // without the rotation the decoder is elementwise: a kernel written for coalescing, whenever
    // groups of 8 coordinates stay inside the sums buffer and the output allows 16-byte stores
    if (!rotate && aligned(out, 16) && (padded_coords(n, chunk_log2) & 7u) == 0u)
        return finish(thc::launch_unrotated_decode(sums, sum_bytes, range, W, bits, chunk_log2, n,
                                                   out_dt == THC_BF16, out, static_cast<hipStream_t>(stream)));
    ChunkArgs a = base_args(n, chunk_log2, seed);
    a.in = sums;
    a.out = out;
    a.range_in = range;
    a.bits = bits;
    a.levels = thc::grid_levels(bits, false);
    a.W = W;
    a.sum_bytes = sum_bytes;
    a.no_rotate = rotate ? 0u : 1u;
    a.out_bf16 = out_dt == THC_BF16;
    return finish(thc::launch_chunks(Mode::Decode, a, static_cast<hipStream_t>(stream)));
}

// --------------------------------------------------------------------- full rotation
static int check_full(uint64_t n, uint32_t log2_size) {
    if (log2_size < 15 || log2_size > 33) return THC_ERR_CHUNK;
    if (n > (1ull << log2_size)) return THC_ERR_SIZE;
    return THC_OK;
}

static float full_factor(uint32_t log2_size) {
    // the whole normalisation fl(2^(-l/2)) is ONE multiplication after the last stage (the
    // chunk kernels of the first pass are told to multiply by 1): a 2^-7 taken early would
    // round where an intermediate value is subnormal
    return (float)(1.0 / sqrt((double)(1ull << log2_size)));
}

uint32_t thc_full_log2(uint64_t n) {
    uint32_t l = 15;
    while (l < 33 && (1ull << l) < n) ++l;
    return (1ull << l) >= n ? l : 0;
}

static int forward_full(const void* x, thc_dtype dt, uint64_t n, uint32_t log2_size, uint64_t seed,
                        float* y, float* absmax, void* stream, bool defer_last = false) {
    int rc = check_full(n, log2_size);
    if (rc == THC_OK) rc = check_dtype(dt);
    if (rc != THC_OK) return rc;
    if (!y || (n != 0 && !x)) return THC_ERR_NULL;
    if (!aligned(x, 16) || !aligned(y, 16)) return THC_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    ChunkArgs a = base_args(n, 14, seed);
    a.in = x;
    a.out = y;
    a.in_bf16 = dt == THC_BF16;
    a.inv_sqrt_c = 1.0f;
    if (n != 0 && thc::launch_fast14(Mode::Forward, a, st) != hipSuccess) return THC_ERR_HIP;
    // (the zero padding behind the last chunk is not written: the first pass reads it as zero)
    thc::FullDeferred d{};
    d.kind = thc::FullLast::RangeOnly;
    return finish(thc::launch_high_passes(y, log2_size, full_factor(log2_size), nullptr, 0, a.key0, a.key1, st,
                                          a.padded, absmax, defer_last ? &d : nullptr));
}

int rht_forward_full(const void* x, thc_dtype dt, uint64_t n, uint32_t log2_size, uint64_t seed,
                     float* y, void* stream) {
    return forward_full(x, dt, n, log2_size, seed, y, nullptr, stream);
}

int rht_forward_full_absmax(const void* x, thc_dtype dt, uint64_t n, uint32_t log2_size, uint64_t seed,
                            float* y, float* absmax, void* stream) {
    if (!absmax) return THC_ERR_NULL;
    if (!aligned(absmax, 4)) return THC_ERR_ALIGN;
    return forward_full(x, dt, n, log2_size, seed, y, absmax, stream);
}

int rht_forward_full_deferred(const void* x, thc_dtype dt, uint64_t n, uint32_t log2_size, uint64_t seed,
                              float* y, float* absmax, void* stream) {
    if (!absmax) return THC_ERR_NULL;
    if (!aligned(absmax, 4)) return THC_ERR_ALIGN;
    return forward_full(x, dt, n, log2_size, seed, y, absmax, stream, true);
}

int thc_full_encode_deferred(const float* y, uint64_t n, uint32_t log2_size, uint64_t seed, uint32_t worker,
                             uint32_t bits, const float* scale, uint8_t* payload, void* stream) {
    int rc = check_full(n, log2_size);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (!y || !scale || !payload) return THC_ERR_NULL;
    if (!aligned(y, 16) || !aligned(scale, 4) || !aligned(payload, 16)) return THC_ERR_ALIGN;
    thc::FullDeferred d{};
    d.kind = thc::FullLast::EncodeOnly;
    d.scale = scale;
    d.levels = thc::grid_levels(bits, false);
    d.bits = bits;
    d.worker = worker;
    d.payload = payload;
    // (the kernel only reads y; `valid` is what rht_forward_full_deferred left behind for this n)
    return finish(thc::launch_high_passes(const_cast<float*>(y), log2_size, full_factor(log2_size), nullptr, 0,
                                          (uint32_t)seed, (uint32_t)(seed >> 32), static_cast<hipStream_t>(stream),
                                          padded_coords(n, 14), nullptr, &d));
}

int rht_inverse_full(float* y, uint64_t n, uint32_t log2_size, uint64_t seed, float* x, void* stream) {
    int rc = check_full(n, log2_size);
    if (rc != THC_OK) return rc;
    if (n == 0) return THC_OK;
    if (!y || !x) return THC_ERR_NULL;
    if (!aligned(x, 16) || !aligned(y, 16)) return THC_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint64_t total = 1ull << log2_size;
    ChunkArgs a = base_args(total, 14, seed);
    a.in = y;
    a.out = y;
    a.inv_sqrt_c = 1.0f;
    if (thc::launch_fast14(Mode::Plain, a, st) != hipSuccess) return THC_ERR_HIP;
    return finish(thc::launch_high_passes(y, log2_size, full_factor(log2_size), x, n, a.key0, a.key1, st,
                                          total, nullptr));
}

int thc_full_absmax(const float* y, uint32_t log2_size, float* absmax, void* stream) {
    int rc = check_full(0, log2_size);
    if (rc != THC_OK) return rc;
    if (!y || !absmax) return THC_ERR_NULL;
    if (!aligned(y, 16) || !aligned(absmax, 4)) return THC_ERR_ALIGN;
    return finish(thc::launch_full_absmax(y, log2_size, absmax, static_cast<hipStream_t>(stream)));
}

int thc_full_encode(const float* y, uint32_t log2_size, uint64_t seed, uint32_t worker, uint32_t bits,
                    const float* scale, uint8_t* payload, void* stream) {
    int rc = check_full(0, log2_size);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (!y || !scale || !payload) return THC_ERR_NULL;
    if (!aligned(y, 16) || !aligned(scale, 4) || !aligned(payload, 16)) return THC_ERR_ALIGN;
    return finish(thc::launch_full_encode(y, log2_size, scale, thc::grid_levels(bits, false), bits, worker,
                                          (uint32_t)seed, (uint32_t)(seed >> 32), payload,
                                          static_cast<hipStream_t>(stream)));
}

int thc_full_decode(const void* sums, const float* scale, uint32_t W, uint32_t log2_size, uint32_t bits,
                    float* yhat, void* stream) {
    int rc = check_full(0, log2_size);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    const uint32_t sum_bytes = thc_sum_bytes(W, bits);
    if (sum_bytes == 0) return THC_ERR_WORKERS;
    if (!sums || !scale || !yhat) return THC_ERR_NULL;
    if (!aligned(sums, 16) || !aligned(scale, 4) || !aligned(yhat, 16)) return THC_ERR_ALIGN;
    return finish(thc::launch_full_decode(sums, sum_bytes, log2_size, scale, thc::grid_levels(bits, false), W,
                                          yhat, static_cast<hipStream_t>(stream)));
}

int thc_full_decode_inverse(const void* sums, const float* scale, uint32_t W, uint64_t n, uint32_t log2_size,
                            uint64_t seed, uint32_t bits, float* work, float* x, void* stream) {
    int rc = check_full(n, log2_size);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    const uint32_t sum_bytes = thc_sum_bytes(W, bits);
    if (sum_bytes == 0) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    if (!sums || !scale || !work || !x) return THC_ERR_NULL;
    if (!aligned(sums, 16) || !aligned(scale, 4) || !aligned(work, 16) || !aligned(x, 16)) return THC_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint64_t total = 1ull << log2_size;
    ChunkArgs a = base_args(total, 14, seed);
    a.in = sums;
    a.out = work;
    a.scale_in = scale;
    a.scale_shared = 1;
    a.levels = thc::grid_levels(bits, false);
    a.W = W;
    a.bits = bits;
    a.sum_bytes = sum_bytes;
    a.inv_sqrt_c = 1.0f;
    if (thc::launch_fast14(Mode::PlainDecode, a, st) != hipSuccess) return THC_ERR_HIP;
    return finish(thc::launch_high_passes(work, log2_size, full_factor(log2_size), x, n, a.key0, a.key1, st,
                                          total, nullptr));
}

// ----------------------------------------------------------------------------- TopKC
static int check_topkc(uint64_t n, uint32_t C) {
    if (C < 8 || C > 512 || (C & (C - 1)) != 0) return THC_ERR_CHUNK;
    if (n > kMaxCoords || (n + C - 1) / C > 0xFFFFFFFFull) return THC_ERR_SIZE;
    return THC_OK;
}

uint64_t topkc_num_chunks(uint64_t n, uint32_t C) {
    return check_topkc(n, C) == THC_OK ? (n + C - 1) / C : 0;
}

int topkc_chunk_norms(const void* grad, thc_dtype dt, uint64_t n, uint32_t C, uint16_t* norms, void* stream) {
    int rc = check_topkc(n, C);
    if (rc == THC_OK) rc = check_dtype(dt);
    if (rc != THC_OK) return rc;
    if (n == 0) return THC_OK;
    if (!grad || !norms) return THC_ERR_NULL;
    if (!aligned(grad, 16) || !aligned(norms, 2)) return THC_ERR_ALIGN;
    return finish(thc::launch_topkc_norms(grad, dt == THC_BF16, n, C, norms, static_cast<hipStream_t>(stream)));
}

int topkc_sum_norms(const uint16_t* norms_all, uint32_t W, uint64_t P, uint16_t* s, void* stream) {
    if (W == 0) return THC_ERR_WORKERS;
    if (P > 0xFFFFFFFFull) return THC_ERR_SIZE;
    if (P == 0) return THC_OK;
    if (!norms_all || !s) return THC_ERR_NULL;
    if (!aligned(norms_all, 2) || !aligned(s, 2)) return THC_ERR_ALIGN;
    return finish(thc::launch_topkc_sum_norms(norms_all, W, P, s, static_cast<hipStream_t>(stream)));
}

uint64_t topkc_select_workspace_bytes(uint64_t P) {
    return P > 0xFFFFFFFFull ? 0 : 4 * thc::topkc_select_workspace_words(P);
}

int topkc_select(const uint16_t* s, uint64_t P, uint32_t J, uint32_t* indices, void* workspace,
                 uint64_t workspace_bytes, void* stream) {
    if (P > 0xFFFFFFFFull || J == 0 || (uint64_t)J > P) return THC_ERR_SIZE;
    if (!s || !indices || !workspace) return THC_ERR_NULL;
    if (!aligned(s, 2) || !aligned(indices, 4) || !aligned(workspace, 4)) return THC_ERR_ALIGN;
    if (workspace_bytes < topkc_select_workspace_bytes(P)) return THC_ERR_SIZE;
    return finish(thc::launch_topkc_select(s, P, J, indices, static_cast<uint32_t*>(workspace),
                                           static_cast<hipStream_t>(stream)));
}

int topkc_gather_sum(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n, uint32_t C,
                     const uint32_t* indices, uint32_t J, uint16_t* values, void* stream) {
    int rc = check_topkc(n, C);
    if (rc == THC_OK) rc = check_dtype(dt);
    if (rc != THC_OK) return rc;
    if (W == 0 || W > (uint32_t)thc::kMaxFusedWorkers) return THC_ERR_WORKERS;
    if ((uint64_t)J > (n + C - 1) / C) return THC_ERR_SIZE;
    if (J == 0) return THC_OK;
    if (!grads || !indices || !values) return THC_ERR_NULL;
    thc::FusedWorkerPtrs ptrs{};
    for (uint32_t w = 0; w < W; ++w) {
        if (!grads[w]) return THC_ERR_NULL;
        if (!aligned(grads[w], 16)) return THC_ERR_ALIGN;
        ptrs.grad[w] = grads[w];
    }
    if (!aligned(indices, 4) || !aligned(values, 16)) return THC_ERR_ALIGN;
    return finish(thc::launch_topkc_gather_sum(ptrs, dt == THC_BF16, W, n, C, indices, J, values,
                                               static_cast<hipStream_t>(stream)));
}

int topkc_scatter_mean(const uint16_t* values, const uint32_t* indices, uint32_t J, uint32_t C, uint32_t W,
                       uint64_t n, float* out, void* stream) {
    int rc = check_topkc(n, C);
    if (rc != THC_OK) return rc;
    if (W == 0) return THC_ERR_WORKERS;
    if ((uint64_t)J > (n + C - 1) / C || n > 0x7FFFFFFFFFull) return THC_ERR_SIZE;
    if (n == 0) return THC_OK;
    if (!out || (J != 0 && (!values || !indices))) return THC_ERR_NULL;
    if (!aligned(values, 16) || !aligned(indices, 4) || !aligned(out, 4)) return THC_ERR_ALIGN;
    return finish(thc::launch_topkc_scatter(values, indices, J, C, W, n, out, static_cast<hipStream_t>(stream)));
}

/* ---- one-pass forms of the min/max variant (chunk_log2 == 14) ---------------------------- */
uint64_t thc_encode_all_minmax_workspace_bytes(uint32_t W, uint64_t n, uint32_t chunk_log2) {
    if (chunk_log2 != 14 || n > kMaxCoords || W == 0 || W > (uint32_t)thc::kMaxFusedWorkers) return 0;
    const uint64_t chunks = padded_coords(n, chunk_log2) >> chunk_log2;
    return 16 + 4 * ((uint64_t)thc::encode_all_minmax_slot_words(W) + 1u) * chunks;
}

int thc_encode_all_minmax(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n, uint32_t chunk_log2,
                          uint64_t seed, uint32_t bits, int rotate, uint8_t* const* payloads, float* range,
                          void* workspace, uint64_t workspace_bytes, void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK && chunk_log2 != 14) rc = THC_ERR_CHUNK;
    if (rc == THC_OK) rc = check_dtype(dt);
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (thc_sum_bytes(W, bits) == 0 || W > (uint32_t)thc::kMaxFusedWorkers) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    if (!grads || !payloads || !range || !workspace) return THC_ERR_NULL;
    for (uint32_t w = 0; w < W; ++w) {
        if (!grads[w] || !payloads[w]) return THC_ERR_NULL;
        if (!aligned(grads[w], 16) || !aligned(payloads[w], 16)) return THC_ERR_ALIGN;
    }
    if (!aligned(range, 8) || !aligned(workspace, 16)) return THC_ERR_ALIGN;
    if (workspace_bytes < thc_encode_all_minmax_workspace_bytes(W, n, chunk_log2)) return THC_ERR_SIZE;
    const uint64_t chunks = padded_coords(n, chunk_log2) >> chunk_log2;
    if (chunks * W >= 0x7FFFFFFFull) return THC_ERR_SIZE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t* words = static_cast<uint32_t*>(workspace);
    thc::EncodeAllArgs a{};
    a.n = n;
    a.chunks = chunks;
    a.W = W;
    a.key0 = (uint32_t)seed;
    a.key1 = (uint32_t)(seed >> 32);
    a.max_spins = g_spin_limit;
    a.levels = thc::grid_levels(bits, false);
    a.scale = range;
    const uint64_t slot_words = (uint64_t)thc::encode_all_minmax_slot_words(W) * chunks;
    a.error = words;
    a.slots = words + 4;
    a.done = words + 4 + slot_words;
    thc::FusedWorkerPtrs ptrs{};
    for (uint32_t w = 0; w < W; ++w) {
        ptrs.grad[w] = grads[w];
        ptrs.payload[w] = payloads[w];
    }
    if (thc::launch_zero_words(words, 4 + slot_words + chunks, st) != hipSuccess) return THC_ERR_HIP;
    const hipError_t e = thc::launch_encode_all_minmax(a, ptrs, dt == THC_BF16, rotate != 0, bits, st);
    if (e == hipErrorInvalidConfiguration) return THC_ERR_WORKERS;   // fewer resident workgroups than workers
    return finish(e);
}

int thc_aggregate_decode_minmax(const uint8_t* const* payloads, uint32_t W, const float* range, uint64_t n,
                                uint32_t chunk_log2, uint64_t seed, uint32_t bits, int rotate, float* out,
                                void* stream) {
    int rc = check_common(n, chunk_log2);
    if (rc == THC_OK && chunk_log2 != 14) rc = THC_ERR_CHUNK;
    if (rc == THC_OK) rc = check_bits(bits);
    if (rc != THC_OK) return rc;
    if (thc_sum_bytes(W, bits) == 0 || W > (uint32_t)thc::kMaxFusedPayloads) return THC_ERR_WORKERS;
    if (rotate && !thc::aggregate_decode_fused_applicable(W, chunk_log2, bits)) return THC_ERR_WORKERS;
    if (n == 0) return THC_OK;
    if (!payloads || !range || !out) return THC_ERR_NULL;
    thc::FusedPayloadPtrs ptrs{};
    for (uint32_t w = 0; w < W; ++w) {
        if (!payloads[w]) return THC_ERR_NULL;
        if (!aligned(payloads[w], 16)) return THC_ERR_ALIGN;
        ptrs.p[w] = payloads[w];
    }
    if (!aligned(range, 8) || !aligned(out, 16)) return THC_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (!rotate) return finish(thc::launch_unrotated_aggregate_decode(ptrs, W, range, bits, n, out, st));
    thc::AggDecodeArgs a{};
    a.n = n;
    a.chunks = padded_coords(n, chunk_log2) >> chunk_log2;
    a.W = W;
    a.key0 = (uint32_t)seed;
    a.key1 = (uint32_t)(seed >> 32);
    a.scale = range;
    a.sums = nullptr;
    a.out = out;
    return finish(thc::launch_aggregate_decode_ranged(a, ptrs, bits, st));
}

}  // extern "C"
