/*
 * thc.h - C ABI of the MI355X (gfx950) library for the all-reduce-compatible
 * gradient quantization path of the paper's THC case study:
 *
 *   partial rotation (randomized Hadamard transform of every 2^l' chunk)
 *     -> per-chunk range shared by all workers
 *     -> stochastic rounding onto a 2^bits-point grid
 *     -> exact integer summation of the workers' payloads
 *     -> dequantize + inverse rotation.
 *
 * Conventions for every entry point
 *   - All pointers are DEVICE pointers unless the comment says HOST.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it and never synchronise.
 *   - The caller owns every buffer.  Unless an entry point says otherwise the
 *     library allocates nothing.  Process-wide state, all of it: the poll limit set by
 *     thc_set_spin_limit (one unsynchronised word read by every one-pass encode
 *     launch), the device's compute-unit count and per-kernel occupancy (queried once,
 *     then cached), and for thc_encode_all_static the per-device address of its fixed
 *     device array.  Nothing else survives a call.
 *   - Inputs and outputs of one call must not overlap.
 *   - n is the number of gradient coordinates of ONE worker, c = 2^chunk_log2 the
 *     chunk length (1 <= chunk_log2 <= 14), chunks = ceil(n / c).  Coordinates
 *     with index >= n inside the last chunk are zeros on input and are not
 *     written on output of length n.
 *   - n == 0 is a successful no-op.
 *   - Arguments are checked on the host before any HIP call; a bad argument
 *     returns a negative thc_status and enqueues nothing.  A failed launch
 *     returns THC_ERR_HIP.
 *   - Gradient, y and output pointers must be aligned to their element size;
 *     payload and sums pointers to 16 bytes (THC_ERR_ALIGN otherwise).
 *   - Non-finite gradient values are not detected: the scale and payload of the
 *     chunk that holds them are unspecified, other chunks are unaffected.
 *
 * Random streams (the paper names no generator; both are Philox4x32-10, key =
 * (low, high) 32 bits of `seed`, g the coordinate's index within the call):
 *   sign of coordinate g : bit (g mod 32) of word ((g div 32) mod 4) of the
 *       block with counter (lo32(g div 128), hi32(g div 128), 0, 0x5349474E);
 *       the same for every worker.
 *   rounding byte r_g    : byte (g mod 16) (little-endian through words 0..3) of
 *       the block with counter (lo32(g div 16), hi32(g div 16), worker,
 *       0x524F554E); u_g = (r_g + 0.5) / 256.
 */
#ifndef THC_H_
#define THC_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of a gradient buffer.  A plain int at the boundary, so that a caller's
 * out-of-range value is an error code (THC_ERR_DTYPE), not undefined behaviour. */
typedef int thc_dtype;
enum { THC_F32 = 0, THC_BF16 = 1 };

typedef enum {
    THC_OK = 0,
    THC_ERR_NULL = -1,    /* a required pointer is NULL */
    THC_ERR_BITS = -2,    /* bits not in {2, 4, 8} */
    THC_ERR_CHUNK = -3,   /* chunk_log2 outside [1, 14] */
    THC_ERR_WORKERS = -4, /* W == 0 or W * (2^bits - 1) > 65535 */
    THC_ERR_DTYPE = -5,   /* dtype not THC_F32 / THC_BF16 */
    THC_ERR_SIZE = -6,    /* a size overflows or exceeds a stated maximum */
    THC_ERR_HIP = -7,     /* a HIP call failed; see hipGetLastError */
    THC_ERR_ALIGN = -8    /* a pointer is not aligned as required */
} thc_status;

/* Text for a status code.  Static storage, never NULL. */
const char* thc_status_string(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int thc_version(void);

/* Random bits consumed per coordinate by the stochastic rounding (8). */
uint32_t thc_rounding_bits(void);

/* ceil(n / 2^chunk_log2): the number of independently rotated chunks ("Partial
 * rotation").  0 if chunk_log2 is out of range. */
uint64_t thc_num_chunks(uint64_t n, uint32_t chunk_log2);

/* Bytes of one worker's packed payload: chunks * 2^chunk_log2 * bits / 8 (the
 * padded tail of the last chunk is part of the payload).  0 on bad arguments. */
uint64_t thc_payload_bytes(uint64_t n, uint32_t chunk_log2, uint32_t bits);

/* Bytes per aggregated coordinate: 1 if W * (2^bits - 1) <= 255, 2 if <= 65535,
 * else 0.  This is the widened aggregate of the paper's "simple adaptation"
 * (b >= q bits so that sums of q-bit values cannot overflow). */
uint32_t thc_sum_bytes(uint32_t W, uint32_t bits);

/* Partial rotation, forward: y = (1/sqrt(c)) H_c D x for every chunk, H_c the
 * Sylvester-ordered Hadamard matrix, D the seeded +-1 diagonal above.
 *   x   n values of dtype dt (fp32, or bf16 widened exactly)
 *   y   chunks * c fp32 values (the zero-padded tail is rotated too) */
int rht_forward(const void* x, thc_dtype dt, uint64_t n, uint32_t chunk_log2, uint64_t seed,
                float* y, void* stream);

/* Partial rotation, inverse: x = D (1/sqrt(c)) H_c y; undoes rht_forward.  The paper
 * describes the sender only; the receiver's rotation back is implied by it (THC
 * background paragraph: the aggregate is decoded into the gradient estimate).
 *   y   chunks * c fp32 values;   x   n fp32 values */
int rht_inverse(const float* y, uint64_t n, uint32_t chunk_log2, uint64_t seed,
                float* x, void* stream);

/* Per-chunk range of one worker after the partial rotation (the "Partial rotation"
 * paragraph takes the value range chunk by chunk), in the symmetric form used here:
 * absmax[p] = max_j |y_j| over chunk p of rht_forward(grad).
 *   absmax   chunks fp32 values */
int thc_chunk_absmax(const void* grad, thc_dtype dt, uint64_t n, uint32_t chunk_log2,
                     uint64_t seed, float* absmax, void* stream);

/* Shared grid: scale[p] = max over workers of absmax_all[w][p].  The paper is silent on
 * how workers agree on a chunk's range ("Partial rotation" paragraph); this is the
 * reading taken: one range per chunk, the largest over the workers.  Stands in for
 * the small max-all-reduce that lets every worker quantize onto the same grid,
 * so that integer payloads can be summed.
 *   absmax_all   W * chunks fp32, worker-major;   scale   chunks fp32 */
int thc_scale_reduce(const float* absmax_all, uint32_t W, uint64_t chunks, float* scale,
                     void* stream);

/* Encode one worker (THC background paragraph of the quantization subsection: q-bit
 * stochastic quantization after the rotation): rotate, then stochastically round every rotated value onto
 * the 2^bits-point grid of [-s_p, +s_p] (index 0 at -s_p, index L = 2^bits - 1 at
 * +s_p), and bit-pack:
 *     inv = L / (s_p + s_p),  u = (r + 0.5) / 256,
 *     idx = min(floor(t), L),  t = y * inv + L/2 + u;   s_p + s_p < 2^-119: idx = 0
 * (the position in grid units plus the noise u; inv is one correctly rounded division;
 * t is evaluated as fma(y, inv, L/2 + u) for bits = 2 and 4, where L/2 + u is exact in
 * fp32, and as fma(y + s_p, inv, u) for bits = 8, which keeps t within 1e-6 max(1, |t|) of
 * its exact value on the 256-point grid).  A chunk whose range s_p + s_p is below 2^-119 -
 * an all-zero chunk, or one so small that fp32 cannot hold L / (s_p + s_p) - is sent as
 * zeros; it keeps its scale and decodes at most 2^-119 off per rotated coordinate.
 *   shared_scale  chunks fp32 (the output of thc_scale_reduce), or NULL to use
 *                 this worker's own absmax
 *   payload       thc_payload_bytes bytes; coordinate g occupies bits
 *                 [(g*bits) mod 8, +bits) of byte (g*bits) div 8
 *   scale_out     chunks fp32 receiving the scale that was used; may be NULL */
int thc_encode(const void* grad, thc_dtype dt, uint64_t n, uint32_t chunk_log2, uint64_t seed,
               uint32_t worker, uint32_t bits, const float* shared_scale, uint8_t* payload,
               float* scale_out, void* stream);

/* Aggregate: sums[g] = sum over w < W of the index worker w stored for
 * coordinate g; exact (the reduction an all-reduce of the payloads performs,
 * with b >= q bits per coordinate so it cannot overflow).
 *   payloads   HOST array of W device pointers, each thc_payload_bytes bytes
 *   sums       chunks * c elements of thc_sum_bytes(W, bits) bytes each */
int thc_aggregate(const uint8_t* const* payloads, uint32_t W, uint64_t n, uint32_t chunk_log2,
                  uint32_t bits, void* sums, void* stream);

/* Decode the aggregate into the estimate of the workers' MEAN gradient (the receiver side
 * the THC background paragraph implies; the paper evaluates the estimate of the average):
 *     step = (s_p + s_p) / L,  yhat = float(sum) * (step / W) - s_p,
 *     out  = D (1/sqrt(c)) H_c yhat   (first n coordinates)
 *   sums    as written by thc_aggregate;   scale   chunks fp32;   out   n fp32 */
int thc_decode(const void* sums, const float* scale, uint32_t W, uint64_t n, uint32_t chunk_log2,
               uint64_t seed, uint32_t bits, float* out, void* stream);

/* ---- batched / fused entry points -------------------------------------------------
 * Same mathematics as the calls above and byte-identical payloads, scales, sums and
 * outputs; these forms read each gradient once and never store the integer sums. */

/* Bytes of scratch thc_encode_all needs for W workers of n coordinates (it may be in
 * any state: the call clears what it uses).  0 on bad arguments. */
uint64_t thc_encode_all_workspace_bytes(uint32_t W, uint64_t n, uint32_t chunk_log2);

/* Encode all W workers in one pass: per chunk, rotate every worker's gradient, agree
 * on the shared scale (max over workers of the per-chunk range: the steps
 * thc_chunk_absmax + thc_scale_reduce), quantize onto it and pack (thc_encode).
 *   grads      HOST array of W device pointers, n values of dtype dt each
 *   payloads   HOST array of W device pointers, thc_payload_bytes each
 *   scale      chunks fp32, receives the shared scale
 *   workspace  device scratch of at least thc_encode_all_workspace_bytes bytes, 16-byte
 *              aligned.  Its first 32-bit word is 0 after a good run and 1 if a bounded
 *              wait between workgroups expired (the payloads are then invalid); check it
 *              after synchronising the stream.
 * Calls that share a workspace must not overlap in time.  The workgroups of a chunk wait
 * for one another, so the launch is sized to be resident on the device all at once; other
 * kernels running at the same time only delay it (their workgroups finish and free their
 * place), but two thc_encode_all / thc_sat_encode_all calls must not run concurrently on
 * one device (issue them on one stream), and a device kept busy by other work for longer
 * than the spin limit makes the call report a time-out. */
int thc_encode_all(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n,
                   uint32_t chunk_log2, uint64_t seed, uint32_t bits, uint8_t* const* payloads,
                   float* scale, void* workspace, uint64_t workspace_bytes, void* stream);

/* thc_encode_all without its clearing launch, for a caller that keeps a workspace of its
 * own across calls (one workspace per bucket of a training step, say).
 * thc_workspace_clear zeroes a workspace (workspace_bytes a multiple of 4, pointer 16-byte
 * aligned); thc_encode_all_cleared expects every byte of the workspace to be zero on
 * entry and leaves it so: inside the kernel a chunk's range words are cleared as soon as
 * every workgroup of the chunk has read them.  Same arguments, results and rules as
 * thc_encode_all otherwise.  Exception: after a time-out the first word is 1 (it is how
 * the time-out is reported) and other words may be left set; clear the workspace again
 * before the next call.  A workspace that is not
 * all zero gives wrong payloads without any error: when in doubt use thc_encode_all,
 * which clears what it uses itself and accepts a workspace in any state. */
int thc_workspace_clear(void* workspace, uint64_t workspace_bytes, void* stream);
int thc_encode_all_cleared(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n,
                           uint32_t chunk_log2, uint64_t seed, uint32_t bits, uint8_t* const* payloads,
                           float* scale, void* workspace, uint64_t workspace_bytes, void* stream);

/* ---- several buckets per launch ---------------------------------------------------------
 * A gradient that is processed bucket by bucket (the headline configuration cuts 1.3e9
 * coordinates into 25 * 2^20-coordinate buckets, as data-parallel training frameworks do)
 * can hand any number of ready buckets to ONE call: the kernels run over all their chunks
 * in one persistent launch, so the start-up and the partly filled last round of a launch
 * are paid once instead of once per bucket.  Results are byte for byte those of
 * thc_encode_all / thc_aggregate_decode called bucket by bucket.
 * Restrictions (negative status otherwise): chunk_log2 == 14 (THC_ERR_CHUNK); W <= 64 and,
 * for the decode side, the shapes for which thc_aggregate_decode_is_fused is 1
 * (THC_ERR_WORKERS); gradients, payloads and outputs 16-byte aligned (THC_ERR_ALIGN); at
 * most 4096 buckets (THC_ERR_SIZE).  A bucket with n == 0 is skipped. */
typedef struct {
    const void* const* grads;  /* HOST array of W device pointers, n values each; encode only */
    uint8_t* const* payloads;  /* HOST array of W device pointers, thc_payload_bytes(n, 14, bits) each */
    float* scale;              /* device, chunks fp32: written by the encode call, read by the decode call */
    float* out;                /* device, n fp32: decode only */
    uint64_t n;                /* coordinates of one worker in this bucket */
    uint64_t seed;             /* the bucket's seed, as passed to the per-bucket calls */
} thc_bucket;

/* Bytes of device scratch the two batched calls need for these buckets (the decode call
 * uses only the first 16 + count * (40 + 16 W) bytes, rounded up to 16).  0 on bad arguments.
 *   buckets   HOST array; only n is read */
uint64_t thc_batch_workspace_bytes(const thc_bucket* buckets, uint32_t count, uint32_t W,
                                   uint32_t chunk_log2);

/* thc_encode_all over every bucket.  The workspace may be in any state (the call clears
 * what it uses); its first 32-bit word reports an expired wait as for thc_encode_all.  The
 * per-bucket records travel to the device as arguments of small kernels: no host-to-device
 * copy, no allocation.  Same rules about concurrent calls as thc_encode_all. */
int thc_encode_all_batch(const thc_bucket* buckets, uint32_t count, thc_dtype dt, uint32_t W,
                         uint32_t chunk_log2, uint32_t bits, void* workspace, uint64_t workspace_bytes,
                         void* stream);

/* thc_aggregate_decode (sums == NULL) over every bucket; writes out[0 .. n) of each. */
int thc_aggregate_decode_batch(const thc_bucket* buckets, uint32_t count, uint32_t W, uint32_t chunk_log2,
                               uint32_t bits, void* workspace, uint64_t workspace_bytes, void* stream);

/* thc_encode_all for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Not a
 * step of the paper: the same computation as thc_encode_all, with the workspace taken from
 * a fixed array of THC_STATIC_SCRATCH_BYTES bytes that the library holds in device memory
 * on every GPU it runs on, for as long as the process lives.  The call allocates and frees
 * nothing (no hipMalloc / hipFree, no allocating library routine) and never synchronises.
 *   grads, payloads, scale   as for thc_encode_all
 *   timed_out   NULL, or one 4-byte aligned device word that receives 0 after a good run
 *               and 1 if a bounded wait between workgroups expired (payloads then invalid)
 * THC_ERR_SIZE if thc_encode_all_workspace_bytes(W, n, chunk_log2) exceeds
 * THC_STATIC_SCRATCH_BYTES (at W = 8 that is 8065 chunks of 2^14 coordinates).  All calls on
 * one GPU share that GPU's array, which keeps the previous call's contents; the call
 * clears the words it uses with a fill kernel first.  Calls that overlap in time on one
 * GPU (two streams, two host threads) race on the array: issue them on one stream. */
#define THC_STATIC_SCRATCH_BYTES (2u << 20)
int thc_encode_all_static(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n,
                          uint32_t chunk_log2, uint64_t seed, uint32_t bits, uint8_t* const* payloads,
                          float* scale, uint32_t* timed_out, void* stream);

/* Upper bound on the polls of one inter-workgroup wait inside thc_encode_all (default
 * 2^22, about seconds).  A tuning and test knob: with a tiny limit the waits expire, the
 * error word is set and every wave still exits.  PROCESS-GLOBAL and not thread-safe: the
 * value is read when a call is enqueued, by every thread's calls; changing it while another
 * thread encodes makes that thread's waits expire early, which only the error word of its
 * workspace reports. */
void thc_set_spin_limit(uint32_t polls);

/* 1 if thc_aggregate_decode can run fused for this shape, in which case `sums` may be
 * NULL; 0 if it will fall back to thc_aggregate + thc_decode and needs `sums`. */
int thc_aggregate_decode_is_fused(uint32_t W, uint32_t chunk_log2, uint32_t bits);

/* thc_aggregate followed by thc_decode.
 *   sums   as for thc_aggregate; when the fused form applies it may be NULL and the
 *          integer sums are then never stored */
int thc_aggregate_decode(const uint8_t* const* payloads, uint32_t W, const float* scale,
                         uint64_t n, uint32_t chunk_log2, uint64_t seed, uint32_t bits,
                         void* sums, float* out, void* stream);

/* ---- saturation-based aggregation ("Saturation-based aggregation" paragraph of the
 * paper's proposed improvements to THC) ----------------------------------------------
 * Partial aggregates are combined with Sat(x, y) = min(M, max(-M, x + y)),
 * M = 2^(bits-1) - 1, so the aggregate never needs more than the `bits` bits a worker
 * sends (b = q).  Readings taken where the paper is silent:
 *   - a worker's coordinate is rounded onto the 2M + 1 evenly spaced points of
 *     [-s_p, +s_p] (same rule and random stream as thc_encode with L = 2M, except that
 *     an all-zero chunk - and one with s_p + s_p < 2^-119, as in thc_encode - gets the centre
 *     index M so that z = 0); the payload
 *     holds idx in [0, 2M] in `bits` bits, packed as for thc_encode; z = idx - M;
 *   - Sat is not associative: a_0 = z_0, a_w = Sat(a_(w-1), z_w) in worker order
 *     w = 1 .. W-1 (the order payloads[] is given in);
 *   - the aggregate is stored offset binary (a + M) in `bits` bits, packed like a
 *     payload (thc_payload_bytes bytes);
 *   - decode: step = (s_p + s_p) / (2M), yhat = float(a) * (step / W), then the inverse
 *     rotation as in thc_decode.
 * W <= 64 (THC_ERR_WORKERS otherwise).  Rotation, range and scale sharing are the same
 * as in the exact-sum path: use thc_chunk_absmax / thc_scale_reduce. */

/* M = 2^(bits-1) - 1; 0 on bad bits. */
uint32_t thc_sat_max(uint32_t bits);

/* thc_encode / thc_encode_all on the 2M + 1-point grid; same arguments. */
int thc_sat_encode(const void* grad, thc_dtype dt, uint64_t n, uint32_t chunk_log2, uint64_t seed,
                   uint32_t worker, uint32_t bits, const float* shared_scale, uint8_t* payload,
                   float* scale_out, void* stream);
int thc_sat_encode_all(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n,
                       uint32_t chunk_log2, uint64_t seed, uint32_t bits, uint8_t* const* payloads,
                       float* scale, void* workspace, uint64_t workspace_bytes, void* stream);
/* thc_encode_all_cleared on the 2M + 1-point grid. */
int thc_sat_encode_all_cleared(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n,
                               uint32_t chunk_log2, uint64_t seed, uint32_t bits,
                               uint8_t* const* payloads, float* scale, void* workspace,
                               uint64_t workspace_bytes, void* stream);

/* Saturating aggregate of W payloads.
 *   payloads        HOST array of W device pointers
 *   aggregate       thc_payload_bytes(n, chunk_log2, bits) bytes, 16-byte aligned
 *   overflow_count  NULL, or one 8-byte aligned device counter to which the number of
 *                   coordinates (padding included) with at least one clipped Sat step is
 *                   ADDED; the caller zeroes it */
int thc_sat_aggregate(const uint8_t* const* payloads, uint32_t W, uint64_t n, uint32_t chunk_log2,
                      uint32_t bits, uint8_t* aggregate, unsigned long long* overflow_count,
                      void* stream);

/* Saturated aggregate -> estimate of the workers' mean gradient (n fp32). */
int thc_sat_decode(const uint8_t* aggregate, const float* scale, uint32_t W, uint64_t n,
                   uint32_t chunk_log2, uint64_t seed, uint32_t bits, float* out, void* stream);

/* 1 if thc_sat_aggregate_decode runs as one kernel for this shape (then `aggregate` may
 * be NULL), 0 if it falls back to thc_sat_aggregate + thc_sat_decode. */
int thc_sat_aggregate_decode_is_fused(uint32_t W, uint32_t chunk_log2, uint32_t bits);

/* thc_sat_aggregate followed by thc_sat_decode; identical results. */
int thc_sat_aggregate_decode(const uint8_t* const* payloads, uint32_t W, const float* scale,
                             uint64_t n, uint32_t chunk_log2, uint64_t seed, uint32_t bits,
                             uint8_t* aggregate, unsigned long long* overflow_count, float* out,
                             void* stream);

/* ---- min/max range (the range as the THC background paragraph and the "Partial rotation"
 * paragraph word it: from the chunk's smallest to its largest value, split evenly), with
 * the rotation optional (the "No Rotation" column of the THC throughput table) and an
 * optional bf16 output ------------------------------------------------------------------
 * range arrays hold (lo, hi) pairs, 2 floats per chunk, 8-byte aligned.  The grid of a chunk
 * has 2^bits points, index 0 at lo and index L at hi, shared by all workers:
 *     inv = L / (hi - lo)  (0 when hi - lo < 2^-119: a constant chunk, or a range too narrow
 *     for fp32 to hold its reciprocal step),  idx = min(floor(fma(y - lo, inv, u)), L)
 *     (the subtraction is rounded on its own; the product and the sum are one fused op)
 *     step = (hi - lo) / L,  yhat = float(sum) * (step / W) + lo
 * rotate != 0: y is the chunk's rotated gradient as in thc_encode; rotate == 0: y is the
 * zero-padded gradient itself (no sign diagonal, no butterflies, no normalisation).
 * Payloads and sums have the formats of thc_encode / thc_aggregate (use thc_aggregate). */

/* range[2p], range[2p+1] = min, max over chunk p of one worker's y. */
int thc_chunk_minmax(const void* grad, thc_dtype dt, uint64_t n, uint32_t chunk_log2, uint64_t seed,
                     int rotate, float* range, void* stream);

/* Shared ranges: range_all holds W arrays of `chunks` pairs back to back; range receives
 * (min over workers of lo, max over workers of hi) per chunk. */
int thc_range_reduce(const float* range_all, uint32_t W, uint64_t chunks, float* range, void* stream);

int thc_encode_minmax(const void* grad, thc_dtype dt, uint64_t n, uint32_t chunk_log2, uint64_t seed,
                      uint32_t worker, uint32_t bits, int rotate, const float* range, uint8_t* payload,
                      void* stream);

/*   out_dt  THC_F32 or THC_BF16 (fp32 result rounded to nearest, ties to even);  out  n values */
int thc_decode_minmax(const void* sums, const float* range, uint32_t W, uint64_t n, uint32_t chunk_log2,
                      uint64_t seed, uint32_t bits, int rotate, thc_dtype out_dt, void* out, void* stream);

/* One-pass forms of the variant for chunk_log2 == 14 (THC_ERR_CHUNK otherwise), the
 * counterparts of thc_encode_all / thc_aggregate_decode: every gradient is read once.
 * The same results, bit for bit, as thc_chunk_minmax + thc_range_reduce + thc_encode_minmax
 * per worker, and as thc_aggregate + thc_decode_minmax with out_dt = THC_F32.
 *   grads, payloads   HOST arrays of W (<= 64, THC_ERR_WORKERS) device pointers, 16-byte aligned
 *   range             2 floats per chunk, written by the encoder ((lo, hi) shared by all workers),
 *                     read by the decoder; 8-byte aligned
 *   workspace         thc_encode_all_minmax_workspace_bytes(W, n, 14) bytes, 16-byte aligned, any
 *                     state (the call clears what it uses; its first 32-bit word is set to 1 if
 *                     a bounded wait between workgroups expired, as for thc_encode_all)
 *   out               n fp32 values, 16-byte aligned
 * The decoder with rotate != 0 accepts the shapes for which thc_aggregate_decode_is_fused is
 * 1 (THC_ERR_WORKERS otherwise); with rotate == 0 every W up to 64. */
uint64_t thc_encode_all_minmax_workspace_bytes(uint32_t W, uint64_t n, uint32_t chunk_log2);
int thc_encode_all_minmax(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n, uint32_t chunk_log2,
                          uint64_t seed, uint32_t bits, int rotate, uint8_t* const* payloads, float* range,
                          void* workspace, uint64_t workspace_bytes, void* stream);
int thc_aggregate_decode_minmax(const uint8_t* const* payloads, uint32_t W, const float* range, uint64_t n,
                                uint32_t chunk_log2, uint64_t seed, uint32_t bits, int rotate, float* out,
                                void* stream);

/* ---- full rotation (l' = l): the baseline the paper's "Partial rotation" paragraph and
 * its THC throughput table compare against ---------------------------------------------
 * The whole gradient, zero-padded to 2^log2_size coordinates (the notation table pads
 * gradients to a power of two), is ONE chunk: y = 2^(-l/2) H_(2^l) D x with the same stage
 * order, sign diagonal and rounding as the chunked path (identical to it with
 * chunk_log2 = log2_size, which the chunked entry points do not accept above 14).
 * Stages above 2^14 run as passes over y in global memory, in place, so rotated data is
 * materialised and the quantizer's steps are separate elementwise calls:
 *     rht_forward_full -> thc_full_absmax (or rht_forward_full_absmax for both)
 *     -> (thc_scale_reduce with chunks = 1)
 *     -> thc_full_encode -> thc_aggregate(n = 2^log2_size, chunk_log2 = 14)
 *        (or rht_forward_full_deferred -> thc_scale_reduce -> thc_full_encode_deferred)
 *     -> thc_full_decode -> rht_inverse_full (or thc_full_decode_inverse for both)
 * 15 <= log2_size <= 33 (THC_ERR_CHUNK otherwise), n <= 2^log2_size (THC_ERR_SIZE);
 * x, y, payload, sums and yhat must be 16-byte aligned. */

/* Smallest valid log2_size for n coordinates (0 if n > 2^33). */
uint32_t thc_full_log2(uint64_t n);

/*   x   n values of dtype dt;   y   2^log2_size fp32, receives the rotated vector */
int rht_forward_full(const void* x, thc_dtype dt, uint64_t n, uint32_t log2_size, uint64_t seed,
                     float* y, void* stream);

/* The same, and *absmax = max |y_g| in the same launches (what thc_full_absmax computes in a
 * pass of its own over y); absmax: device, one float, 4-byte aligned. */
int rht_forward_full_absmax(const void* x, thc_dtype dt, uint64_t n, uint32_t log2_size, uint64_t seed,
                            float* y, float* absmax, void* stream);

/* The rotation put off until the scale is known, for a caller that only needs the payload:
 * rht_forward_full_deferred runs every pass but the last in place in y and evaluates the
 * last one for *absmax only (y then holds the data as the pass before the last wrote it, NOT
 * the rotated values); after thc_scale_reduce over the workers' absmax,
 * thc_full_encode_deferred runs the last pass again on that y (read only) and quantizes
 * its results directly.  Same scale and payload bytes as rht_forward_full_absmax +
 * thc_full_encode, with the rotated values never stored.  n and log2_size of the two calls
 * must be the same. */
int rht_forward_full_deferred(const void* x, thc_dtype dt, uint64_t n, uint32_t log2_size, uint64_t seed,
                              float* y, float* absmax, void* stream);
int thc_full_encode_deferred(const float* y, uint64_t n, uint32_t log2_size, uint64_t seed, uint32_t worker,
                             uint32_t bits, const float* scale, uint8_t* payload, void* stream);

/*   y   2^log2_size fp32 rotated values, USED AS SCRATCH (garbage afterwards);
 *   x   n fp32, receives D 2^(-l/2) H y */
int rht_inverse_full(float* y, uint64_t n, uint32_t log2_size, uint64_t seed, float* x, void* stream);

/* *absmax = max |y_g| over the 2^log2_size values (the call zeroes it first). */
int thc_full_absmax(const float* y, uint32_t log2_size, float* absmax, void* stream);

/* Stochastic rounding of rotated values onto the 2^bits-point grid of [-s, s], s = *scale
 * (device, one float, shared by all workers); payload 2^log2_size * bits / 8 bytes. */
int thc_full_encode(const float* y, uint32_t log2_size, uint64_t seed, uint32_t worker, uint32_t bits,
                    const float* scale, uint8_t* payload, void* stream);

/* yhat_g = float(sum_g) * (step / W) - s for the 2^log2_size sums written by
 * thc_aggregate; feed yhat to rht_inverse_full. */
int thc_full_decode(const void* sums, const float* scale, uint32_t W, uint32_t log2_size, uint32_t bits,
                    float* yhat, void* stream);

/* thc_full_decode and rht_inverse_full in one call: the dequantization runs in front of
 * stages 0..13, so yhat is never stored (same results, bit for bit).
 *   work   2^log2_size fp32 of scratch (garbage afterwards), 16-byte aligned
 *   x      n fp32, 16-byte aligned: the estimate of the mean gradient */
int thc_full_decode_inverse(const void* sums, const float* scale, uint32_t W, uint64_t n, uint32_t log2_size,
                            uint64_t seed, uint32_t bits, float* work, float* x, void* stream);

/* ---- TopK Chunked (TopKC), "Our proposed improvement: Chunks" of the paper's TopK case
 * study: the all-reduce-compatible sparsifier ------------------------------------------
 * The gradient of n coordinates is cut into P = ceil(n / C) chunks of C coordinates (C a
 * power of two, 8 <= C <= 512, zero padding at the end).  Steps and the readings taken
 * where the paper is silent:
 *   1. topkc_chunk_norms  each worker: squared L2 norm of every chunk, in half precision
 *        (squares and their sum in fp32, summed as a balanced tree over adjacent pairs,
 *        then rounded to fp16, nearest even);
 *   2. topkc_sum_norms    s_p = sum over workers, as an fp16 all-reduce would compute it:
 *        fp16 accumulation in worker order, one rounding per addition;
 *   3. topkc_select       the J chunks with the largest s_p, equal values lowest index
 *        first; indices are returned in ascending order;
 *   4. topkc_gather_sum   the selected chunks of every worker rounded to fp16 and summed
 *        in fp16 in worker order (the FP16 all-reduce of the sparsified gradients);
 *   5. topkc_scatter_mean dense fp32 estimate of the mean gradient: float(sum) / W on the
 *        selected chunks, 0 elsewhere.
 * Cost on the wire: 16 (J C / n + 1 / C) bits per coordinate.
 * fp16 arrays are passed as uint16_t bit patterns.  Gradients and `values` must be
 * 16-byte aligned.  Errors: THC_ERR_CHUNK for a bad C, THC_ERR_SIZE for P >= 2^32,
 * J == 0 (select) or J > P. */

uint64_t topkc_num_chunks(uint64_t n, uint32_t C);

/*   norms   P fp16 values of ONE worker */
int topkc_chunk_norms(const void* grad, thc_dtype dt, uint64_t n, uint32_t C, uint16_t* norms, void* stream);

/*   norms_all   W arrays of P fp16 values back to back;   s   P fp16 sums */
int topkc_sum_norms(const uint16_t* norms_all, uint32_t W, uint64_t P, uint16_t* s, void* stream);

/* Scratch bytes topkc_select needs for P chunks (the call clears what it uses). */
uint64_t topkc_select_workspace_bytes(uint64_t P);

/*   s   P non-negative fp16 values;   indices   receives J chunk indices, ascending */
int topkc_select(const uint16_t* s, uint64_t P, uint32_t J, uint32_t* indices, void* workspace,
                 uint64_t workspace_bytes, void* stream);

/*   grads   HOST array of W (<= 64) device pointers;   values   J * C fp16 values,
 *   chunk indices[j] at values[j * C .. j * C + C) */
int topkc_gather_sum(const void* const* grads, thc_dtype dt, uint32_t W, uint64_t n, uint32_t C,
                     const uint32_t* indices, uint32_t J, uint16_t* values, void* stream);

/*   out   n fp32 values, fully written (zeros outside the selected chunks) */
int topkc_scatter_mean(const uint16_t* values, const uint32_t* indices, uint32_t J, uint32_t C, uint32_t W,
                       uint64_t n, float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* THC_H_ */
