// Host-callable launchers of the EDEN kernels (all asynchronous on the given stream).
#ifndef EDEN_KERNELS_H
#define EDEN_KERNELS_H

#include "eden.h"
#include "eden_device.h"

namespace eden {

// Encode runs the contiguous pass first (it reads x) and the strided passes after it, the last one quantizing and
// packing; decode runs the strided passes first (the first one unpacks) and the contiguous pass last (it sums the
// senders into acc).  Launchers of kernels that leave per-workgroup partial sums return how many partials each
// sender got.

// wave-tile passes and the small kernels (eden_kernels.hip)
// `d` with a `pre` flag next to it is the caller's dimension; pre != 0 (b = 1/2 with the sparsification before the
// rotation) means the transformed vector has dimension ceil(d/2).  Every other `d` is the transformed dimension.
uint32_t launch_enc_lo_first(const EncBatch &B, uint32_t n, uint64_t d, int pre, int log2D, uint64_t seed, float *T,
                             double *partials, uint32_t partial_stride, hipStream_t st);
uint32_t launch_enc_hi_last(int M, const EncBatch &B, uint32_t n, uint64_t valid_elems, int log2D, int p, uint64_t seed,
                            const float *T, double *partials, uint32_t partial_stride, const EncScratch *scratch,
                            const CoinTables &ct, hipStream_t st);
// coin budgets (multi-pass sizes): the coins of the senders that have such a budget, with their prefix sums; `part_b`
// (encode) points at the second part of every such sender's payload, which is cleared; null on the receiver's side
void launch_coin_pack(const uint32_t *b_q8, const uint32_t *const *pieces, void *const *part_b, uint32_t n, int log2D,
                      const CoinTables &ct, hipStream_t st);
void launch_coin_tables(const uint32_t *clients, const uint32_t *b_q8, void *const *part_b, uint32_t n, uint64_t seed, int log2D,
                        const CoinTables &ct, hipStream_t st);
// wide strided tiles (8 rows x 512 columns per wave) for the top three index bits of D >= 2^25; b = 1, 2, 4, 5..8 and
// the uniform grid
uint32_t launch_enc_wide_last(const EncBatch &B, uint32_t n, uint64_t valid_elems, int log2D, const float *T, double *partials,
                              uint32_t partial_stride, const EncScratch *scratch, hipStream_t st);
void launch_dec_wide_first(const DecBatch &B, uint32_t n, uint64_t keep_elems, int log2D, const DecScratch *scratch, float *T,
                           hipStream_t st);
void launch_enc_norm(const EncBatch &B, uint32_t n, const double *partials, uint32_t partial_stride, uint32_t nparts,
                     EncScratch *scratch, const DevTables *tab, hipStream_t st);
void launch_enc_finish(const EncBatch &B, uint32_t n, uint64_t hdr_d, int log2D, uint64_t seed,
                       const double *partials_n2, uint32_t nparts_n2, const double *partials_ip, uint32_t nparts_ip,
                       uint32_t partial_stride, uint32_t *dev_status, const uint32_t *coin_total, hipStream_t st);
void launch_dec_prepare(const DecBatch &B, uint32_t n, uint64_t hdr_d, int log2D, uint64_t seed, const DevTables *tab,
                        DecScratch *scratch, uint32_t *dev_status, const uint32_t *coin_total, uint32_t *msg_flags,
                        hipStream_t st);
void launch_dec_hi_first(int M, const DecBatch &B, uint32_t n, uint64_t keep_elems, int log2D, int p, uint64_t seed,
                         const DecScratch *scratch, int narrow, float *T, const CoinTables &ct, hipStream_t st);
// pre: 0 = sum the senders into acc; 1 = the same with the pairs scatter of EDEN_B_HALF_PRE; 2 = no sum, every sender's
// decoded vector goes back into its own workspace slot (fp32, `narrow` must be 0)
void launch_dec_lo_last(const DecBatch &B, uint32_t n, uint64_t d, int pre, int log2D, uint64_t seed, float *T,
                        const DecScratch *scratch, int narrow, float *acc, hipStream_t st);
void launch_finalize_mean(const float *acc, uint64_t d, uint32_t n, float *mean, hipStream_t st);
void launch_enc_small(const EncBatch &B, uint32_t n, uint64_t d, int pre, uint64_t hdr_d, int log2D, uint64_t seed,
                      const DevTables *tab, uint32_t *dev_status, hipStream_t st);
// `msg_flags` (may be null): one status word per message of the launch, written by the kernel that checks the headers
void launch_dec_small(const DecBatch &B, uint32_t n, uint64_t d, int pre, uint64_t hdr_d, int log2D, uint64_t seed,
                      const DevTables *tab, float *acc, uint32_t *dev_status, uint32_t *msg_flags, hipStream_t st);
// b = m/64: the kept coordinates of x packed into `stage` (m per block of 64), and added back from it into acc
void launch_sparse_gather(const float *x, uint64_t d, uint32_t m, uint64_t seed, uint32_t client, float *stage, hipStream_t st);
void launch_sparse_scatter(const float *stage, uint64_t d, uint32_t m, uint64_t seed, uint32_t client, float *acc, hipStream_t st);
void launch_sparse_gather_batch(const EncBatch &B, uint32_t n, uint64_t d, uint32_t m, uint64_t seed, float *T, int log2Dk,
                                hipStream_t st);
void launch_sparse_scatter_batch(const DecBatch &B, uint32_t n, uint64_t d, uint32_t m, uint64_t seed, const float *T, int log2Dk,
                                 float *acc, hipStream_t st);
// b = 5, 6, 7: one-byte indices (B.codes[c], null for other senders) <-> the packed payload
void launch_pack_bits(const EncBatch &B, uint32_t n, int log2D, hipStream_t st);
void launch_unpack_bits(const DecBatch &B, uint32_t n, int log2D, uint8_t *codes_all, hipStream_t st);
void launch_fill_zero(float *p, uint64_t count, hipStream_t st);
// dst[i] = src_host[i], i < count <= kArgDoubles: the values travel as kernel arguments (no copy is staged)
constexpr int kArgDoubles = 256;
void launch_store_doubles(const double *src_host, uint32_t count, double *dst, hipStream_t st);
void launch_byte_entropy(const uint8_t *bytes, uint64_t count, uint32_t *hist, double *out, hipStream_t st);
void launch_sq_error(const float *a, const float *b, uint64_t d, double *partials, uint32_t max_parts, double *out,
                     hipStream_t st);
void launch_hash_bits(uint64_t key, uint64_t nwords, uint64_t *out, hipStream_t st);
void launch_loss_bitmap(uint64_t key, uint32_t npk, uint32_t drop_q32, uint32_t *bitmap, hipStream_t st);

// workgroup-tile strided passes for D >= 2^21 (eden_kernels_wg.hip)
uint32_t launch_enc_hix_last(int M, int blocked, const EncBatch &B, uint32_t n, uint64_t d, int log2D, uint64_t seed, const float *T,
                             double *partials, uint32_t partial_stride, const EncScratch *scratch, const CoinTables &ct,
                             hipStream_t st);
void launch_hix_mid(int M, uint32_t n, float *T, int log2D, uint64_t load_elems, uint64_t store_elems, hipStream_t st);
// What dec_prepare_wave needs besides the batch; a first decode pass that is given it (`prep` not null) may do the work of
// launch_dec_prepare itself, in one of its workgroups per sender, and then returns true: the caller leaves that launch out.
struct DecPrepareArgs {
    uint64_t hdr_d, seed;
    const DevTables *tab;
    DecScratch *scratch;
    uint32_t *dev_status;
    uint32_t *msg_flags;                 // null or one word per sender of the batch
};
bool launch_dec_hix_first(int M, const DecBatch &B, uint32_t n, uint64_t d, int log2D, uint64_t seed,
                          const DecScratch *scratch, int narrow, float *T, const CoinTables &ct, const DecPrepareArgs *prep,
                          hipStream_t st);
// whether launch_dec_hix_first would do so for this batch
bool dec_hix_first_prepares(int M, const DecBatch &B, uint32_t n, int narrow);

// 14-bit contiguous passes for D >= 2^19 (eden_kernels_lo14.hip)
// `blocked`: write the workspace in the blocked layout (eden_device.h: blocked_offset) that launch_enc_hix_last reads
// when told so; not for a first pass that works in place on the workspace
uint32_t launch_enc_lo14_first(const EncBatch &B, uint32_t n, uint64_t d, int pre, int blocked, int log2D, uint64_t seed, float *T,
                               double *partials, uint32_t partial_stride, hipStream_t st);
// `resident`: workgroups of the kernel the device holds at once (2 per CU); `partial`: room for `partial_tiles`
// tiles of 2^14 floats, used when tiles are split over several workgroups by sender.
// `mean_n` > 0 (pre == 0 only): acc is not read; acc[i] = (0 + the sum over the senders) / mean_n
void launch_dec_lo14_last(const DecBatch &B, uint32_t n, uint64_t d, int pre, int log2D, uint64_t seed, float *T,
                          const DecScratch *scratch, int narrow, float *acc, uint32_t resident, float *partial,
                          uint32_t partial_tiles, float mean_n, hipStream_t st);

}  // namespace eden
#endif
