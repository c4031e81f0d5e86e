/*
 * eden.h -- C ABI of the MI355X (gfx950) EDEN library.
 *
 * EDEN (arXiv 2108.08842) is a distributed-mean-estimation method: each of n senders
 * holds a d-dimensional fp32 vector x_c, sends one short message, and a receiver
 * returns an estimate of (1/n) sum_c x_c  (Sec. 2.1, the DME problem statement).
 *
 * The three hot calls follow that statement:
 *   eden_encode            -- the senders' side  (Sec. 2.2.1 rotation, quantization, Sec. 2.3 scale)
 *   eden_decode_accumulate -- the receiver's per-sender reconstruction, summed (Sec. 2.2.2, Sec. 4.2)
 *   eden_finalize_mean     -- the division by n   (Sec. 2.2.2)
 * (eden_decode_mean is the last two in one call, for a round that one call decodes.)
 *
 * Conventions common to every call
 *   - Return value: 0 (EDEN_OK) or a negative eden_status.  Nothing throws or aborts.
 *   - "_dev" pointers are HIP device pointers on the context's device; pointer ARRAYS
 *     (x_dev[], msgs_dev[], recv_bitmaps_dev[]) and the id / budget arrays are HOST arrays,
 *     read before the call returns and not retained.
 *   - The caller owns every buffer it passes.  The library reads inputs, writes outputs,
 *     and keeps no caller pointer after the call returns.  Its only own device memory is the
 *     context workspace allocated by eden_create.
 *   - eden_encode, eden_decode_accumulate, eden_decode_mean and eden_finalize_mean only launch kernels on `stream`: no
 *     allocation (every buffer any budget needs is allocated by eden_create), no memset, no host synchronisation,
 *     so they may be captured in a HIP graph.
 *   - A context serialises its work through that workspace: calls on one context must be issued from
 *     one thread at a time and on one stream (or on streams the caller orders); two calls that run
 *     concurrently on the same context race.  Use one context per concurrent stream.
 *   - `stream` is a hipStream_t cast to void* (NULL = the default stream).  Encode, decode and
 *     finalize only enqueue work on that stream; they never synchronise the host.
 *     Conditions that can only be seen on the device (zero or non-finite vector, nothing
 *     received, header mismatch) are recorded in the message header's status word and in a
 *     device status word that eden_last_device_status() reads (it synchronises).
 *
 * Dimensions and layout
 *   - d is padded with zeros to D = 2^ceil(log2 d); the rotation, the quantization and the
 *     payload cover all D coordinates; the decoder drops the tail.  1 <= d <= 2^27.
 *   - Rotation: R x = D^-1/2 H (s o x), H = Sylvester-ordered Hadamard matrix, s = +-1 diagonal
 *     drawn from the shared seed and the sender's id (Sec. 2.1 shared randomness, Sec. 5
 *     randomized Hadamard transform).  Bit (i & 63) of hash word (i >> 6) of the SIGN stream is 1
 *     where s_i = -1.
 *   - Hash: word(key, j) = mix(key + PHI*(j+1)), mix = the splitmix64 output function,
 *     key = mix(mix(seed + PHI) + PHI*((stream << 32) | client) + PHI), PHI = 0x9E3779B97F4A7C15;
 *     streams: 0 = signs, 1 = sub-sampling, 2 = packet loss, 3 = mix (which coordinates get the extra bit),
 *     4 = sparse (sort keys of the m-of-64 sparsification).
 *   - Bit budget b is passed as b_q8 = 256*b.  Supported: 256, 512, ..., 2048 (b = 1..8, the
 *     2^b-level Lloyd-Max quantizer of N(0,1), Sec. 3; for b = 5, 6, 7 at multi-pass sizes the indices are
 *     packed by a kernel of their own from a byte buffer of D_max bytes per workspace slot); 128 (b = 1/2: the b = 1 quantizer,
 *     then of every two consecutive rotated coordinates (2g, 2g+1) only the one at offset
 *     bit (g & 63) of word (g >> 6) of the SUB-SAMPLING stream is sent; Sec. 4.1, applied after
 *     the rotation, so the receiver treats the rest like lost coordinates, Sec. 4.2); and
 *     384, 640, 896 (b = k + 1/2, k = 1, 2, 3; Sec. 4.1, non-integer b > 1: of every pair
 *     (2g, 2g+1) the coordinate at offset bit (g & 63) of word (g >> 6) of the MIX stream is quantized
 *     with I_{k+1}, the other one with I_k.  The paper flips an independent coin per coordinate,
 *     which makes the message length random; choosing exactly one coordinate of every pair is as
 *     content independent and gives exactly (k + 1/2) D bits at positions known without a scan).
 *     EDEN_B_COIN(q) (0x40000 | q, 256 < q < 1024, q not a multiple of 256): b = q/256, the non-integer budgets of
 *     Sec. 4.1 in the paper's own form: coordinate i is quantized with I_{floor(b)+1} iff its coin says so, the coin
 *     being "byte (i & 7) of word (i >> 3) of the MIX stream is below q & 255" (probability b - floor(b), independent
 *     from coordinate to coordinate), else with I_{floor(b)}.  The message length then depends on the coins (never on
 *     the data): eden_message_bytes returns the room that fits any outcome; the header records how many coordinates
 *     got the extra bit, and the message ends 8 ceil(that / 64) bytes after the first part of the payload.
 *     EDEN_B_HALF_PRE (0x10080): b = 1/2 with the sparsification before the rotation (Sec. 4.1, the
 *     paper's default for b < 1): x'[g] = 2 x[2g + o_g], g < ceil(d/2), o_g = bit (g & 63) of word (g >> 6)
 *     of the SUB-SAMPLING stream (x read as 0 beyond d), is encoded with b = 1 in dimension ceil(d/2): the
 *     transform and the message are half as large; the decoder puts value g back at 2g + o_g and leaves the
 *     other coordinate of the pair 0.  In one call either every sender uses this budget or none (the
 *     transform dimension differs).  The header keeps d and this b_q8; log2(D) is that of ceil(d/2).
 *     EDEN_B_SPARSE(m) (0x20000 | m, 1 <= m <= 63): b = m/64, sub-bit compression with p = m/64 and the
 *     sparsification before the rotation (Sec. 4.1).  Of every 64 consecutive coordinates of x (the last block
 *     padded with virtual zeros) exactly the m with the smallest 16-bit keys are kept, ties broken by position;
 *     key of coordinate i = bits 16 (i & 3) .. +15 of word (i >> 2) of the SPARSE stream (stream 4).  The
 *     m ceil(d/64) kept values, in order, are encoded with b = 1 (unscaled: the method is scale equivariant), and
 *     the decoder multiplies by 64/m and puts them back.  Senders that share m are processed in batches, others
 *     one at a time; a call uses such budgets for all senders or for none; packets of a received-packet bitmap refer
 *     to the kept vector.  When d is not a multiple of 64 some of the last block's kept positions fall on its virtual
 *     zeros; for d < 64 it can happen that no real coordinate is kept at all (d = 4, m = 6, seed 0, client 0 is such a
 *     case).  The message is then that of a zero vector: status EDEN_DEV_ZERO_VECTOR, S = 0, and the sender contributes
 *     nothing to the mean in that round (the estimate stays unbiased over the seeds: every real coordinate is still kept
 *     with probability m/64).  A caller that must tell this from x = 0 compares |x|^2 in the header with its own.
 *     EDEN_B_GRID(q) (0x30000 | q, 1 <= q <= 65535): the uniform-grid quantizer of Sec. 4.3 with
 *     Delta = q / 32768: index n = sign(z) ceil(|z| / Delta - 1/2) (the nearest grid point; a value half way between
 *     two goes to the one closer to zero, as the footnote of Sec. 2.2.1 asks), clipped to +-127 and sent as one signed byte
 *     per coordinate (the payload is D bytes; an entropy coder would bring it to about H(Delta) bits per
 *     coordinate, 3 bits at Delta = 0.5224); the value of index n is the centre of mass of N(0,1) on
 *     [Delta (n - 1/2), Delta (n + 1/2)] (the outermost intervals run to infinity).  A vector whose coordinates
 *     all round to n = 0 is reported like a zero vector.
 *   - Index of a coordinate = rank of its interval in ascending order (0 = most negative).  At an
 *     interval endpoint the interval closer to zero is taken; z = 0 belongs to the non-negative
 *     side (Sec. 2.2.1 and its footnote).
 *   - Message = 64-byte little-endian header + payload of uint32 words:
 *       off  0 u32 magic 0x4E454445   off  4 u32 log2(D)      off  8 u64 d
 *       off 16 u32 b_q8               off 20 u32 client id    off 24 u32 status bits
 *       off 28 u32 extra bits (EDEN_B_COIN: coordinates with a coin; else 0)
 *                                     off 32 f64 S            off 40 f64 |x|^2
 *       off 48 f64 <R(x), Q>          off 56 u64 seed
 *     Payload: the j-th transmitted index occupies bits [(j*b) mod 32, +b) of word floor(j*b/32),
 *     least significant bit first; the payload is padded with zero bits to a multiple of 64 bits.
 *     For b = k + 1/2 the payload has two such parts: first the low k bits of every coordinate's index
 *     (packed as for budget k), then, 64-bit aligned, one bit per pair: the top bit of the (k+1)-bit
 *     index of the pair's chosen coordinate.
 *     For EDEN_B_COIN the payload has two parts as well: the low floor(b) bits of every coordinate's index, then, 64-bit
 *     aligned, one bit for every coordinate with a coin, in coordinate order: the top bit of its index.
 *     S = |x|^2 / <R(x), Q(eta R(x))> is the sender's scale (Sec. 2.3), always computed over all
 *     D coordinates (the sender does not change under loss or sub-sampling, Sec. 4.2).
 *   - A packet is 1024 consecutive rotated coordinates (one packet if D < 1024).  A received-packet
 *     bitmap has bit (j & 31) of uint32 word (j >> 5) set when packet j arrived.
 */
#ifndef EDEN_H
#define EDEN_H

#define EDEN_B_HALF_PRE 0x10080u
#define EDEN_B_SPARSE(m) (0x20000u | (unsigned)(m))
#define EDEN_B_GRID(q) (0x30000u | (unsigned)(q))
#define EDEN_B_COIN(q) (0x40000u | (unsigned)(q))

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct eden_ctx eden_ctx;

typedef enum eden_status {
    EDEN_OK = 0,
    EDEN_ERR_INVALID_ARG = -1,      /* NULL pointer, d = 0, d > 2^27, n = 0, unsupported budget, n or d above the context's limits */
    EDEN_ERR_CAPACITY = -2,         /* a message buffer is smaller than eden_message_bytes() */
    EDEN_ERR_HIP = -3,              /* a HIP runtime call failed */
    EDEN_ERR_NO_DEVICE = -4,        /* no usable gfx950 device / device index out of range */
    EDEN_ERR_STATIC_LIMIT = -5      /* eden_encode_static: n or d above EDEN_STATIC_MAX_N / EDEN_STATIC_MAX_D */
} eden_status;

/* bits of the status word in a message header and of the device status word */
#define EDEN_DEV_ZERO_VECTOR     1u   /* |x|^2 == 0: S = 0, payload zero, decodes to nothing (Sec. 2.1 footnote) */
#define EDEN_DEV_NONFINITE       2u   /* |x|^2 is inf or nan: message marked, decodes to nothing */
#define EDEN_DEV_HEADER_MISMATCH 4u   /* decode: header disagrees with the call (magic, D, d, budget, client, seed) */
#define EDEN_DEV_NOTHING_ARRIVED 8u   /* decode: every packet of a message was lost; it contributes nothing */

#define EDEN_HEADER_BYTES 64
#define EDEN_PACKET_COORDS 1024
#define EDEN_MAX_LOG2_D 27

/* Creates a context on HIP device `hip_device` able to handle vectors up to d_max coordinates and
 * batches up to n_max senders per call.  Allocates everything any later call needs: per workspace slot (there are
 * min(n_max, 32)) 4 * D_max bytes for the transform's intermediate passes, D_max bytes for the one-byte indices of
 * b = 5, 6, 7 and 3/16 * D_max bytes for the coins of the EDEN_B_COIN budgets (none of the three if D_max <= 4096);
 * 4 * (d_max + 64) bytes for the kept coordinates of an EDEN_B_SPARSE sender; 32 MiB for sender-group sums of the last
 * decode pass when D_max >= 2^19 and n_max > 1; plus a few KiB of partial sums per sender;
 * solves the Lloyd-Max tables of Sec. 3 in double precision on the host and uploads them.
 * On failure *out is NULL. */
int eden_create(eden_ctx **out, uint64_t d_max, uint32_t n_max, int hip_device);

/* Frees the workspace.  The caller must have synchronised the streams it used. */
int eden_destroy(eden_ctx *ctx);

/* Header + payload size in bytes of one message for dimension d and budget b_q8; 0 if unsupported. */
size_t eden_message_bytes(uint64_t d, uint32_t b_q8);

/* Sender side for n senders at once (each sender is independent; batching only amortises launches).
 *   x_dev[c]        device fp32[d], sender c's vector, read-only               (Sec. 2.1)
 *   client_ids[c]   the id that selects sender c's independent rotation         (Sec. 2.1, 2.2.1)
 *   b_q8[c]         sender c's bit budget                                        (Sec. 4.1)
 *   seed            the round's shared seed                                      (Sec. 2.1)
 *   msgs_dev[c]     device buffer of at least eden_message_bytes(d, b_q8[c]) bytes, 16-byte aligned,
 *                   written: header then payload
 *   msg_capacity[c] size of that buffer in bytes
 * Per sender: u = H (s o x) by a fast Walsh-Hadamard transform, |x|^2, indices of u/|x| against the
 * Lloyd-Max thresholds, <R(x),Q>, S, packed payload. */
int eden_encode(eden_ctx *ctx, const float *const *x_dev, const uint32_t *client_ids,
                const uint32_t *b_q8, uint32_t n, uint64_t d, uint64_t seed,
                void *const *msgs_dev, const size_t *msg_capacity, void *stream);

/* eden_encode for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and bit-identical messages as eden_encode, but no context: the
 * workspace is a fixed device array inside the library (about 47 MiB on every GPU the library is loaded on, held until
 * the process ends), so the call is limited to n <= EDEN_STATIC_MAX_N senders of d <= EDEN_STATIC_MAX_D coordinates;
 * beyond that it returns EDEN_ERR_STATIC_LIMIT and does nothing.  It runs on the current HIP device and calls no
 * hipMalloc, hipFree or other allocating routine; the first call on a device also looks up the array's address, uploads
 * the Lloyd-Max tables through kernel arguments and synchronises `stream` once.  Device-side conditions are recorded in
 * the message headers only.  All calls on one GPU share the array, which keeps the last call's contents (every call
 * overwrites what it reads): calls that overlap on one GPU, on any streams, race. */
#define EDEN_STATIC_MAX_D 1048576u
#define EDEN_STATIC_MAX_N 8u
int eden_encode_static(const float *const *x_dev, const uint32_t *client_ids, const uint32_t *b_q8, uint32_t n,
                       uint64_t d, uint64_t seed, void *const *msgs_dev, const size_t *msg_capacity, void *stream);

/* Receiver side for a batch of n messages: for each, unpack, centroid lookup, zero the coordinates
 * that were not sampled or whose packet did not arrive, multiply by S/p with p = (coordinates that
 * arrived)/D counted from the bitmap (Sec. 4.2), inverse rotation (Sec. 2.2.2); the n reconstructions
 * are summed in registers and added once to acc_dev:  acc[i] += sum_c x^_c[i],  i < d.
 *   msgs_dev[c]          device message as written by eden_encode, read-only
 *   client_ids[c], b_q8[c], seed, d   what the receiver agreed with sender c; checked against the header
 *   recv_bitmaps_dev     NULL (nothing lost) or host array of n device pointers, each NULL or a
 *                        bitmap of ceil(max(1, D/1024) / 32) uint32 words
 *   acc_dev              device fp32[d], 16-byte aligned, read and written; the caller zeroes it once per round */
int eden_decode_accumulate(eden_ctx *ctx, const void *const *msgs_dev, const uint32_t *client_ids,
                           const uint32_t *b_q8, uint32_t n, uint64_t d, uint64_t seed,
                           const uint32_t *const *recv_bitmaps_dev, float *acc_dev, void *stream);

/* The receiver's whole round in one call (Sec. 2.2.2: reconstruct every sender's vector, average):
 *   mean[i] = (1/n) sum_c x^_c[i],  i < d,
 * the same numbers, bit for bit, as zeroing an accumulator, eden_decode_accumulate over the n messages and
 * eden_finalize_mean with this n.  Arguments as in eden_decode_accumulate; mean_dev (device fp32[d], 16-byte
 * aligned) is written only, whatever it held.  For rounds whose n messages are decoded by one call.  When one launch of
 * the last pass sums all senders (no EDEN_B_SPARSE budget, padded dimension of the transform 2^19 .. 2^24 -- up to 2^27
 * without EDEN_B_HALF_PRE --, n at most 32) that pass stores the mean directly and the accumulator's three extra passes
 * over memory (zero, read, divide) do not happen; in every other case the call runs those three steps itself on
 * mean_dev. */
int eden_decode_mean(eden_ctx *ctx, const void *const *msgs_dev, const uint32_t *client_ids,
                     const uint32_t *b_q8, uint32_t n, uint64_t d, uint64_t seed,
                     const uint32_t *const *recv_bitmaps_dev, float *mean_dev, void *stream);

/* mean[i] = acc[i] / n for i < d (Sec. 2.2.2: the plain average, also with mixed budgets).
 * mean_dev may alias acc_dev. */
int eden_finalize_mean(eden_ctx *ctx, const float *acc_dev, uint64_t d, uint32_t n, float *mean_dev,
                       void *stream);

/* Synchronises `stream`, returns the OR of the device status bits raised since the last call of this
 * function, and clears them. */
int eden_last_device_status(eden_ctx *ctx, void *stream, uint32_t *status_out);

/* Synchronises `stream` and copies to flags_out[0 .. n-1] (host) the status bits of the first n messages of the most recent
 * eden_decode_accumulate call on this context, in the order of that call: EDEN_DEV_HEADER_MISMATCH, EDEN_DEV_NOTHING_ARRIVED,
 * or the sender's own EDEN_DEV_ZERO_VECTOR / EDEN_DEV_NONFINITE; 0 for a message that was decoded and added.  Tells which
 * message of a batch the OR in eden_last_device_status came from.  n must not exceed that call's n. */
int eden_last_decode_flags(eden_ctx *ctx, void *stream, uint32_t *flags_out, uint32_t n);

/* Bytes of a message that have to travel, from a HOST copy of its 64-byte header: eden_message_bytes(d, b_q8) for every
 * budget but EDEN_B_COIN, whose second part is as long as the coins made it; 0 if the header is not one of this library. */
size_t eden_message_length(const void *header_host);

/* Test helpers: the kernels' own hash streams, written out so that masks can be compared bit for bit.
 *   eden_make_loss_bitmap   packet j of `client` is dropped iff the top 32 bits of word(LOSS key, j)
 *                           are below drop_q32 (drop probability drop_q32 / 2^32); writes
 *                           ceil(max(1, D/1024)/32) words
 *   eden_make_sign_bits     writes D/64 (at least 1) uint64 words of the SIGN stream
 *   eden_make_subsample_bits writes max(1, D/128) uint64 words of the SUB-SAMPLING stream */
int eden_make_loss_bitmap(eden_ctx *ctx, uint64_t seed, uint32_t client_id, uint64_t D,
                          uint32_t drop_q32, uint32_t *bitmap_dev, void *stream);
int eden_make_sign_bits(eden_ctx *ctx, uint64_t seed, uint32_t client_id, uint64_t D,
                        uint64_t *bits_dev, void *stream);
int eden_make_subsample_bits(eden_ctx *ctx, uint64_t seed, uint32_t client_id, uint64_t D,
                             uint64_t *bits_dev, void *stream);

/* Experiment helper (not on the hot path): out_dev[0] = sum_i (a_i - b_i)^2, out_dev[1] = sum_i a_i^2 over
 * i < d, accumulated in double, deterministic.  With a = x and b = the decoded estimate, out[0] / out[1] is
 * the squared error normalised by |x|^2 whose expectation is the vNMSE (Sec. 2.3, Thm 2.3); with a = the true
 * mean of n vectors, out[0] * n / sum_c |x_c|^2 is the NMSE of Sec. 2.1.
 * a_dev, b_dev: device, fp32[d], read only.  out_dev: device, 2 doubles, written.  Asynchronous on `stream`;
 * uses the context's encoder scratch, so it must not overlap an eden_encode on another stream. */
int eden_sq_error(eden_ctx *ctx, const float *a_dev, const float *b_dev, uint64_t d, double *out_dev, void *stream);

/* Experiment helper (Sec. 4.3): out_dev[0] = the empirical entropy -sum f log2 f, in bits per coordinate, of the D
 * one-byte indices of a message encoded with an EDEN_B_GRID budget: what an ideal entropy coder would spend.
 * msg_dev: device, the message; out_dev: device, 1 double, written.  Asynchronous on `stream`; uses 1 KiB of the
 * context, so calls on one context must not overlap. */
int eden_index_entropy(eden_ctx *ctx, const void *msg_dev, uint64_t d, uint32_t b_q8, double *out_dev, void *stream);

/* Copies the library's own Lloyd-Max tables for an integer budget `bits` (1..8) to host arrays:
 * thresholds[2^bits - 1] and centroids[2^bits], ascending, double precision (Sec. 3). */
int eden_get_tables(uint32_t bits, double *thresholds, double *centroids);

/* Kernel timing for the benchmark: while enabled, every launch of a kernel whose kind is in
 * `kind_mask` (bit k = kind k) is bracketed by two HIP events on the caller's stream.
 * eden_profile_enable allocates the event pool (max_records pairs) on first use; passing kind_mask = 0
 * switches timing off.  eden_profile_collect synchronises the recorded events, writes up to `cap`
 * records (kind, senders in that launch, elapsed milliseconds) in launch order, stores the number
 * written in *count, and empties the pool.  Launches beyond max_records are not recorded. */
typedef enum eden_kernel_kind {
    EDEN_K_ENC_FIRST = 0,      /* encode: contiguous pass (reads x, signs, |x|^2) */
    EDEN_K_MID = 1,            /* middle strided pass of the three-pass sizes, in place on the workspace */
    EDEN_K_ENC_LAST = 2,       /* encode: last strided pass + quantize + pack */
    EDEN_K_DEC_PREPARE = 3,    /* decode: per-message scalars */
    EDEN_K_DEC_FIRST = 4,      /* decode: unpack + dequantize + first strided pass */
    EDEN_K_DEC_LAST = 5,       /* decode: contiguous pass + signs + sum over senders */
    EDEN_K_FINALIZE = 6,       /* division by n */
    EDEN_K_ENC_SMALL = 7,      /* encode, D <= 4096, one workgroup per sender */
    EDEN_K_DEC_SMALL = 8,      /* decode, D <= 4096 */
    EDEN_K_ENC_NORM = 9,       /* encode: |x|^2 from per-workgroup partials, scaled thresholds */
    EDEN_K_ENC_FINISH = 10,    /* encode: <R(x),Q>, S, header */
    EDEN_K_COUNT = 11
} eden_kernel_kind;
int eden_profile_enable(eden_ctx *ctx, uint32_t kind_mask, uint32_t max_records);
int eden_profile_collect(eden_ctx *ctx, uint32_t *kinds, uint32_t *senders, float *ms, uint32_t cap,
                         uint32_t *count);
const char *eden_kernel_name(uint32_t kind);

const char *eden_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* EDEN_H */
