// Device-side building blocks shared by the EDEN kernels (gfx950, wave64).
#ifndef EDEN_DEVICE_H
#define EDEN_DEVICE_H

#include <hip/hip_runtime.h>

#include <utility>
#include <stddef.h>
#include <stdint.h>

#include "eden.h"                    // status bits, packet size

namespace eden {

constexpr int kMaxBatch = 32;            // senders handled by one launch; larger batches are chunked
constexpr int kLoBits = 12;              // index bits transformed by the contiguous (wave-tile) pass
constexpr int kLoTile = 1 << kLoBits;    // 4096 coordinates = 64 lanes x 64 registers
constexpr int kLdsRow = 68;              // padded row length (floats) of the 64x64 LDS transpose

// ---- shared randomness (Sec. 2.1): counter hash = splitmix64 stream started at a per-(seed,stream,client) key
constexpr uint64_t kPhi = 0x9E3779B97F4A7C15ull;
enum : uint32_t { kStreamSign = 0, kStreamSubsample = 1, kStreamLoss = 2, kStreamMix = 3, kStreamSparse = 4 };

__host__ __device__ inline uint64_t mix64(uint64_t z) {
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}
__host__ __device__ inline uint64_t stream_key(uint64_t seed, uint32_t stream, uint32_t client) {
    const uint64_t tag = ((uint64_t)stream << 32) | (uint64_t)client;
    return mix64(mix64(seed + kPhi) + kPhi * tag + kPhi);
}
__host__ __device__ inline uint64_t hash_word(uint64_t key, uint64_t j) { return mix64(key + kPhi * (j + 1)); }

// ---- bit budgets (Sec. 4.1): b_q8 = 256 b -> bits per transmitted index, keep one coordinate in k.
// b = 1.5, 2.5, 3.5 ("mixed"): every coordinate has floor(b) bits in the first part of the payload and one
// coordinate of every pair, chosen by the MIX stream, one more bit in a second part (it is quantized with the
// next finer table).
// b = 1/2 with the sparsification before the rotation (Sec. 4.1, the paper's default for b < 1): the vector
// x'[g] = 2 x[2g + offset_g] of dimension ceil(d/2) is encoded with b = 1; the kernels then see b_q8 = 256 and
// only the gather (first encode pass), the scatter (last decode pass) and the header know about it.
constexpr uint32_t kPreHalf = 0x10000u | 128u;
// b = m/64, 1 <= m <= 63 (Sec. 4.1 sub-bit compression with p = m/64, sparsification before the rotation): of every
// 64 consecutive coordinates the m with the smallest 16-bit keys of the SPARSE stream are kept (ties by position)
// and the vector of kept coordinates is encoded with b = 1; the receiver multiplies by 64/m.  Only a gather kernel
// before the encoder, a scatter kernel after the decoder and the header know about it.
constexpr uint32_t kSparseFlag = 0x20000u;
__host__ __device__ inline uint32_t sparse_m(uint32_t b_q8) {
    const uint32_t m = b_q8 & 0xFFFFu;
    return ((b_q8 & ~0xFFFFu) == kSparseFlag && m >= 1 && m <= 63) ? m : 0;
}
// Uniform-grid quantizer of Sec. 4.3: the intervals [Delta (n - 1/2), Delta (n + 1/2)], Delta = (b_q8 & 0xFFFF) / 32768;
// the index n of the interval that holds z (endpoints: closer to zero), clipped to +-127, travels as one signed byte (what an entropy coder would shrink to
// about H(Delta) bits); the value of an interval is its centre of mass under N(0,1).
constexpr uint32_t kGridFlag = 0x30000u;
constexpr int kGridMax = 127;
__host__ __device__ inline uint32_t grid_q15(uint32_t b_q8) {
    return ((b_q8 & ~0xFFFFu) == kGridFlag && (b_q8 & 0xFFFFu) >= 1u) ? (b_q8 & 0xFFFFu) : 0u;
}
// b = 5..8: the Lloyd-Max quantizers with 32..256 levels.  Like the uniform grid they are handled one byte per
// coordinate inside the kernels (index = rank of the interval); for b = 5, 6, 7 a separate kernel packs the bytes to
// b bits (and unpacks them before decoding), for b = 8 the bytes are the payload.
__host__ __device__ inline uint32_t wide_bits(uint32_t b_q8) {
    return (b_q8 == 1280u || b_q8 == 1536u || b_q8 == 1792u || b_q8 == 2048u) ? (b_q8 >> 8) : 0u;
}
__host__ __device__ inline bool byte_budget(uint32_t b_q8) { return grid_q15(b_q8) != 0u || wide_bits(b_q8) != 0u; }
__host__ __device__ inline bool budget_mixed(uint32_t b_q8) { return b_q8 == 384 || b_q8 == 640 || b_q8 == 896; }
// General non-integer b > 1 in the paper's own form (Sec. 4.1): every coordinate is quantized with I_{floor(b)+1} with
// probability b - floor(b), by an independent coin from the shared randomness: coordinate i gets the extra bit iff byte
// (i & 7) of word (i >> 3) of the MIX stream is below 256 (b - floor(b)).  b = (b_q8 & 0xFFFF) / 256, 1 < b < 4, not an
// integer.  The message length then depends on the coins (never on the data); positions in the second part of the payload
// come from a prefix sum over the coins that a small kernel computes for sender and receiver alike.
constexpr uint32_t kCoinFlag = 0x40000u;
__host__ __device__ inline uint32_t coin_q8(uint32_t b_q8) {
    const uint32_t low = b_q8 & 0xFFFFu;
    return ((b_q8 & ~0xFFFFu) == kCoinFlag && low > 256u && low < 1024u && (low & 255u) != 0u) ? low : 0u;
}
// some coordinates carry one bit more than the others: the stratified k + 1/2 budgets and the coin budgets
__host__ __device__ inline bool budget_two_tables(uint32_t b_q8) { return budget_mixed(b_q8) || coin_q8(b_q8) != 0u; }
__host__ __device__ inline bool budget_of(uint32_t b_q8, int &bits, int &k) {
    if (coin_q8(b_q8)) { bits = (int)(coin_q8(b_q8) >> 8); k = 1; return true; }
    if (b_q8 == 128) { bits = 1; k = 2; return true; }
    if (b_q8 == 256 || b_q8 == 512 || b_q8 == 768 || b_q8 == 1024 || budget_mixed(b_q8)) {
        bits = (int)(b_q8 >> 8); k = 1; return true;
    }
    if (grid_q15(b_q8)) { bits = 8; k = 1; return true; }
    if (wide_bits(b_q8)) { bits = (int)wide_bits(b_q8); k = 1; return true; }
    return false;
}
// bytes of the first part of the payload (the floor(b)-bit indices), a multiple of 8
__host__ __device__ inline uint64_t payload_a_bytes(uint64_t D, int bits, int k) {
    return ((((D / (uint64_t)k) * (uint64_t)bits) + 63) / 64) * 8;
}
// bytes of the second part (one bit per pair of coordinates) of a mixed budget; for a coin budget the room that fits
// any outcome of the coins (one bit per coordinate)
__host__ __device__ inline uint64_t payload_b_bytes(uint64_t D, uint32_t b_q8) {
    if (coin_q8(b_q8)) return ((D + 63) / 64) * 8;
    return budget_mixed(b_q8) ? ((D / 2 + 63) / 64) * 8 : 0;
}
// bytes of the second part of a coin budget whose coins gave `extra_bits` coordinates the extra bit
__host__ __device__ inline uint64_t coin_b_bytes(uint64_t extra_bits) { return ((extra_bits + 63) / 64) * 8; }

// Coins of one sender, written by k_coin_masks / k_coin_scan: a lane mask per 64 consecutive coordinates, the number of
// coins before each such block inside its group of 256 blocks, the number of coins before each group, and the total.
constexpr int kCoinGroup = 256;          // blocks of 64 coordinates per group (one workgroup of k_coin_masks)
struct CoinTables {
    uint64_t *mask;                      // slot c: mask + (c << (log2D - 6)); bit j of word w: coordinate 64 w + j has a coin
    uint32_t *local;                     // slot c: local + (c << (log2D - 6)); coins before block w inside its group
    uint32_t *group;                     // slot c: group + c * group_stride; coins before group g
    uint32_t *total;                     // total[c]: all coins of sender c = bits of the second part of its payload
    uint32_t group_stride;
};
__device__ inline bool coin_of(uint64_t mixkey, uint64_t i, uint32_t frac) {
    return ((uint32_t)(hash_word(mixkey, i >> 3) >> (8u * (uint32_t)(i & 7u))) & 0xFFu) < frac;
}

// ---- message header (64 bytes, little endian)
struct MsgHeader {
    uint32_t magic, log2D;
    uint64_t d;
    uint32_t b_q8, client, status, extra_bits;   // extra_bits: coin budgets only (bits of the second part), else 0
    double S, N2, IP;
    uint64_t seed;
};
static_assert(sizeof(MsgHeader) == 64, "header layout");
constexpr uint32_t kMagic = 0x4E454445u;

// the positive centroid of I_1, sqrt(2/pi) (Sec. 3: Q_{I_1} = {+-sqrt(2/pi)}); b = 1 and b = 1/2 need no other table
constexpr float kQ1 = 0.7978845608028654f;

// ---- device copies of the Lloyd-Max tables (positive halves, Sec. 3), index [bits][k]
struct DevTables {
    double t[5][8];
    double q[5][8];
    double t_big[4][128];   // b = 5..8 at index b - 5
    double q_big[4][128];
};

// per-sender scalars that travel between the passes of one encode
struct EncScratch {
    double n2;              // |x|^2 (Sec. 2.2.1: equals |R(x)|^2)
    float thr[8];           // positive thresholds of I_b times |x|: compared against |H(s o x)|
    float qpos[8];          // positive centroids
    float thr2[8];          // mixed budgets: the same for I_{floor(b)+1}
    float qpos2[8];
    float grid_inv;         // uniform grid: 1 / (Delta |x|), so that round(u * grid_inv) is the index
    unsigned pad;
    float grid_c[kGridMax + 1];     // uniform grid: centre of mass of the interval of index n >= 0; b = 5..8: positive centroids
    float wide_thr[128];            // b = 5..8: positive thresholds times |x|
};

static_assert(offsetof(EncScratch, wide_thr) == offsetof(EncScratch, grid_c) + 128 * sizeof(float),
              "the kernels copy centroids and thresholds as one run of 256 floats");

// per-message scalars of one decode
struct DecScratch {
    float deq[16];          // (S / (p sqrt(D))) * q_l for every index l (all zero if the message contributes nothing)
    float deq2[16];         // mixed budgets: the same for the indices of I_{floor(b)+1}
    uint32_t flags;
    uint32_t pad[3];
    float grid_deq[kGridMax + 1];   // uniform grid and b = 5..8: (S / (p sqrt(D))) * positive centroid
};

struct EncBatch {
    const float *x[kMaxBatch];
    void *msg[kMaxBatch];
    uint32_t client[kMaxBatch];
    uint32_t b_q8[kMaxBatch];       // what the kernels quantize with
    uint32_t hdr_b_q8[kMaxBatch];   // what the header says (differs for the budgets that sparsify before the rotation)
    uint8_t *codes[kMaxBatch];      // b = 5, 6, 7: where the one-byte indices go before they are packed (else null)
};
struct DecBatch {
    const void *msg[kMaxBatch];
    const uint32_t *bitmap[kMaxBatch];
    uint32_t client[kMaxBatch];
    uint32_t b_q8[kMaxBatch];
    uint32_t hdr_b_q8[kMaxBatch];
    const uint8_t *codes[kMaxBatch];    // b = 5, 6, 7: the unpacked one-byte indices (else null)
};

// ---- wave-level helpers
__device__ inline uint32_t lane_id() { return threadIdx.x & 63u; }
__device__ inline uint32_t wave_in_block() { return __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); }

// LDS traffic of one wave is processed in issue order; this only stops the compiler from moving
// the reads of a transpose above the writes of other lanes.
__device__ inline void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// v or -v per lane, chosen by bit `lane` of a wave-uniform 64-bit mask (one VALU op: the mask is
// used directly as the lane-select operand).  Written with the builtin, not inline assembly: an SGPR
// written by a vector instruction (v_readlane, v_cmp) needs wait states before a vector instruction
// reads it, and the compiler only inserts them for instructions it can see.
__device__ inline float negate_where(float v, uint64_t mask) {
    return __builtin_amdgcn_inverse_ballot_w64(mask) ? -v : v;
}

// v or 0 per lane, chosen by bit `lane` of a wave-uniform mask
__device__ inline float keep_where(float v, uint64_t mask) {
    return __builtin_amdgcn_inverse_ballot_w64(mask) ? v : 0.0f;
}

// The 64-bit value held by lane `src` (compile-time constant), as a wave-uniform scalar.
__device__ inline uint64_t wave_read64(uint64_t v, int src) {
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)v, src);
    const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(v >> 32), src);
    return ((uint64_t)hi << 32) | lo;
}

// ---- buffer addressing: one resource descriptor per sender buffer, a per-lane byte offset in a VGPR and
// a wave-uniform byte offset in an SGPR per access.  Strided passes issue 64 loads back to back; with flat
// 64-bit addresses each of them would pin two VGPRs.  Reads beyond `bytes` return 0 and writes beyond it
// are dropped, which is exactly the zero padding of d up to D.
using rsrc_t = __amdgpu_buffer_rsrc_t;
__device__ inline rsrc_t make_rsrc(const void *base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
constexpr int kStream = 2;   // cache-policy bit "nt": the data is touched once per pass (measured +5..9% on copies)
__device__ inline float buf_load(rsrc_t r, uint32_t lane_off, uint32_t wave_off) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)lane_off, (int)wave_off, kStream));
}
__device__ inline void buf_store(rsrc_t r, uint32_t lane_off, uint32_t wave_off, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, (int)lane_off, (int)wave_off, kStream);
}
// read-modify-write data that another kernel reads soon (the accumulator): default cache policy
__device__ inline float buf_load_keep(rsrc_t r, uint32_t lane_off, uint32_t wave_off) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)lane_off, (int)wave_off, 0));
}
__device__ inline void buf_store_keep(rsrc_t r, uint32_t lane_off, uint32_t wave_off, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, (int)lane_off, (int)wave_off, 0);
}

// Sub-word accesses of neighbouring lanes go through whole dwords (a byte or half-word load per lane is not merged
// with its neighbours': measured 3x slower on the first decode pass of the one-byte budgets).
// The byte at `byte_off` (lane part) + `wave_off` of the buffer; descriptor base and wave_off are multiples of 4.
__device__ inline uint32_t buf_load_byte(rsrc_t r, uint32_t byte_off, uint32_t wave_off) {
    const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(r, (int)(byte_off & ~3u), (int)wave_off, 0);
    return (w >> (8u * (byte_off & 3u))) & 0xFFu;
}
__device__ inline uint32_t buf_load_half(rsrc_t r, uint32_t byte_off, uint32_t wave_off) {     // byte_off even
    const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(r, (int)(byte_off & ~3u), (int)wave_off, 0);
    return (w >> (8u * (byte_off & 2u))) & 0xFFFFu;
}
// The bytes of lanes 4k .. 4k+3 as one dword (byte of lane 4k + i in bits 8i..), in all four lanes.
__device__ inline uint32_t quad_bytes(uint32_t byte, uint32_t lane) {
    uint32_t x = (byte & 0xFFu) << (8u * (lane & 3u));
    x |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, true);     // quad_perm [1,0,3,2]: lane ^ 1
    x |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, true);     // quad_perm [2,3,0,1]: lane ^ 2
    return x;
}

// In-register Walsh-Hadamard butterflies over the register index: (a,b) -> (a+b, a-b) at spans 1..N/2.
template <int N>
__device__ inline void fwht_regs(float (&v)[N]) {
#pragma unroll
    for (int h = 1; h < N; h <<= 1) {
#pragma unroll
        for (int i = 0; i < N; i += 2 * h) {
#pragma unroll
            for (int j = i; j < i + h; ++j) {
                const float a = v[j], b = v[j + h];
                v[j] = a + b;
                v[j + h] = a - b;
            }
        }
    }
}

__device__ inline double wave_sum(double v) {          // fixed order: deterministic
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ inline uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// block-level deterministic sum of one double per thread; result valid in thread 0
template <int THREADS>
__device__ inline double block_sum(double v, double *red /* shared, THREADS/64 */) {
    v = wave_sum(v);
    const uint32_t w = threadIdx.x >> 6;
    if (lane_id() == 0) red[w] = v;
    __syncthreads();
    double total = 0.0;
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < THREADS / 64; ++i) total += red[i];
    }
    __syncthreads();
    return total;
}

// Interval rank of one coordinate of the unnormalised transform against the scaled thresholds of I_b
// (Sec. 2.2.1, Sec. 3), and its contribution |u| q to sum_i u_i Q_i (Sec. 2.3).  H = 2^(b-1) levels per sign.
// A value exactly on a threshold stays in the interval closer to zero (strict compare); u = +0 is
// non-negative.  thr[0] is unused (it is the threshold 0, decided by the sign).
// The thresholds are wave-uniform scalars (sc->thr); the centroid is looked up in `qtab`, a copy of sc->qpos
// (entries 0..7) and sc->qpos2 (8..15) in LDS: counting the thresholds below |u| and one LDS read cost 2 H + 3
// instructions where a select chain that carries the centroid along costs 3 H (measured 20% on a b = 4 pass).
__device__ inline void fill_qtab(float *qtab, const EncScratch *sc, uint32_t lane) {
    if (lane < 8) qtab[lane] = sc->qpos[lane];
    else if (lane < 16) qtab[lane] = sc->qpos2[lane - 8];
}
template <int H>
__device__ inline uint32_t magnitude_rank(float a, const float (&thr)[8]) {
    uint32_t mag = 0;
#pragma unroll
    for (int t = 1; t < H; ++t) mag += (a > thr[t]) ? 1u : 0u;
    return mag;
}
template <int H>
__device__ inline uint32_t quantize_one(float u, const EncScratch *sc, const float *qtab, float &ip) {
    const float a = fabsf(u);
    const uint32_t mag = magnitude_rank<H>(a, sc->thr);
    ip = fmaf(a, qtab[mag], ip);
    const uint32_t neg = __float_as_uint(u) >> 31;
    return neg ? (uint32_t)(H - 1) - mag : (uint32_t)H + mag;
}

// The same search through a table, for kernels that spend their time on it (H = 8: fourteen instructions above).  |u| is
// cut into kRankCells cells of equal width, the last threshold falling into the last but one; a cell holds at most one
// threshold (the Lloyd-Max thresholds of up to 16 levels lie at least six cells apart), so the rank is the number of
// thresholds in lower cells plus one compare.  The result is the one of magnitude_rank for every input: the cell number is a
// monotone function of |u| (a rounded product, clamped and truncated), hence a value in a higher cell than a threshold is above
// it and one in a lower cell is below it, and inside the threshold's own cell the compare decides as it does there.  |x| = 0:
// `inv` is 0, every value is 0 and lands in cell 0, whose threshold is 0: rank 0.  A vector so small that 62 / threshold
// overflows (|x| / sqrt(D) below 1e-37) would put several thresholds into one cell: fill_rank_table reports that (a cell's
// `below` of kRankCollision) and the caller counts thresholds for that sender instead.
constexpr int kRankCells = 64;
constexpr uint32_t kRankCollision = 0x80000000u;
struct RankCell {
    float thr;              // the threshold inside the cell, +inf if there is none
    float q_below, q_above; // centroids of the rank without and with that threshold passed
    uint32_t below;         // thresholds in lower cells
};
__device__ inline uint32_t rank_cell_of(float a, float inv) { return (uint32_t)fminf(a * inv, (float)(kRankCells - 1)); }
__device__ inline float rank_cell_scale(const EncScratch *sc, int H) {
    const float last = sc->thr[H - 1];
    return last > 0.0f ? (float)(kRankCells - 2) / last : 0.0f;
}
template <int H>
__device__ inline void fill_rank_table(RankCell *cells, const EncScratch *sc, uint32_t thread, float inv) {
    if (thread >= (uint32_t)kRankCells) return;
    RankCell e{__builtin_inff(), 0.0f, 0.0f, 0u};
    uint32_t here = 0;
#pragma unroll
    for (int t = 1; t < H; ++t) {
        const uint32_t cell = rank_cell_of(sc->thr[t], inv);
        e.below += cell < thread ? 1u : 0u;
        if (cell == thread) { e.thr = sc->thr[t]; ++here; }
    }
    const bool collision = __ballot(here > 1u && sc->thr[H - 1] > 0.0f) != 0ull;      // (threads 0..63 are one wave)
    e.q_below = sc->qpos[e.below];
    e.q_above = sc->qpos[e.below + 1u < (uint32_t)H ? e.below + 1u : (uint32_t)H - 1u];
    if (collision) e.below = kRankCollision;
    cells[thread] = e;
}
template <int H>
__device__ inline uint32_t quantize_one_table(float u, const RankCell *cells, float inv, float &ip) {
    const float a = fabsf(u);
    const RankCell e = cells[rank_cell_of(a, inv)];
    const bool above = a > e.thr;
    const uint32_t mag = e.below + (above ? 1u : 0u);
    ip = fmaf(a, above ? e.q_above : e.q_below, ip);
    const uint32_t neg = (uint32_t)((int)__float_as_uint(u) >> 31);      // all ones for a negative value
    return (mag ^ neg) + (uint32_t)H;                                    // H + mag, or H - 1 - mag
}

// ---- collecting ballots in lanes, and bit interleaving for the packed payload
__device__ inline uint32_t lo32(uint64_t x) { return (uint32_t)x; }
__device__ inline uint32_t hi32(uint64_t x) { return (uint32_t)(x >> 32); }
// v_writelane_b32 through its compiler intrinsic (this compiler has no builtin of that name): the compiler then
// also places the wait states an SGPR written by v_cmp needs before a vector instruction may read it.
extern "C" __device__ int eden_writelane_i32(int value, int lane, int old) __asm("llvm.amdgcn.writelane.i32");
template <int LANE>
__device__ inline uint32_t put_lane(uint32_t value, uint32_t old) {      // old with lane LANE replaced by a wave-uniform value
    return (uint32_t)eden_writelane_i32((int)value, LANE, (int)old);
}
template <class F, int... I>
__device__ inline void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ inline void static_for(F &&f) {                       // f(integral_constant<int, 0>) ... f(<N-1>)
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}
// The value of lane (l ^ X) of the same row of 16 lanes: data-parallel primitives where one exists for the pattern, the
// cross-lane swizzle of the LDS unit (no memory access) for X = 4.
template <int X>
__device__ inline uint32_t lane_xor_u32(uint32_t v) {
    static_assert(X == 1 || X == 2 || X == 4 || X == 8, "one lane bit");
    if constexpr (X == 1) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false);        // quad_perm [1,0,3,2]
    else if constexpr (X == 2) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
    else if constexpr (X == 8) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x128, 0xF, 0xF, false);  // row_ror:8
    else return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x001F | (4 << 10));
}
// A word holds N = 32 / BITS items of BITS bits; the N lanes that differ only in their low log2 N lane bits transpose
// them: item i of lane j becomes item j of lane i.  One step per lane bit b: the two lanes of a pair swap the items
// whose index differs from their own side in bit b (a rotation by the width of 2^b items brings them into place; what it
// wraps around falls outside the mask).
template <int BITS, int B = 0>
__device__ inline uint32_t transpose_items(uint32_t x, uint32_t lane) {
    constexpr int N = 32 / BITS;
    if constexpr ((1 << B) >= N) {
        return x;
    } else {
        constexpr uint32_t width = (uint32_t)BITS << B;
        constexpr uint32_t unit = (1u << width) - 1u;
        uint32_t keep_low = 0;                               // items whose index has bit B clear
#pragma unroll
        for (uint32_t pos = 0; pos < 32u; pos += 2u * width) keep_low |= unit << pos;
        const uint32_t t = lane_xor_u32<(1 << B)>(x);
        const bool up = (lane >> B) & 1u;
        const uint32_t other = __builtin_amdgcn_alignbit(t, t, up ? width : 32u - width);
        const uint32_t mask = up ? ~keep_low : keep_low;
        return transpose_items<BITS, B + 1>((mask & x) | (~mask & other), lane);
    }
}
__device__ inline uint32_t even_bits(uint32_t x) {               // bits 0,2,4,..,30 -> bits 0..15
    x &= 0x55555555u;
    x = (x | (x >> 1)) & 0x33333333u;
    x = (x | (x >> 2)) & 0x0F0F0F0Fu;
    x = (x | (x >> 4)) & 0x00FF00FFu;
    return (x | (x >> 8)) & 0x0000FFFFu;
}
__device__ inline uint32_t spread2(uint32_t x) {                 // bit j of the low 16 -> bit 2j
    x &= 0xFFFFu;
    x = (x | (x << 8)) & 0x00FF00FFu;
    x = (x | (x << 4)) & 0x0F0F0F0Fu;
    x = (x | (x << 2)) & 0x33333333u;
    return (x | (x << 1)) & 0x55555555u;
}
__device__ inline uint32_t spread4(uint32_t x) {                 // bit j of the low 8 -> bit 4j
    x &= 0xFFu;
    x = (x | (x << 12)) & 0x000F000Fu;
    x = (x | (x << 6)) & 0x03030303u;
    return (x | (x << 3)) & 0x11111111u;
}

__device__ inline uint32_t spread3(uint32_t x) {                 // bit j of the low 11 -> bit 3j
    const uint32_t top = ((x >> 10) & 1u) << 30;
    x &= 0x3FFu;
    x = (x | (x << 16)) & 0x030000FFu;
    x = (x | (x << 8)) & 0x0300F00Fu;
    x = (x | (x << 4)) & 0x030C30C3u;
    x = (x | (x << 2)) & 0x09249249u;
    return x | top;
}
// 3-bit codes of 32 consecutive coordinates, given as three bit planes (bit i of plane k = bit k of code i),
// as the 96-bit little-endian string in which code i occupies bits 3i .. 3i+2
__device__ inline void pack3_planes(uint32_t p0, uint32_t p1, uint32_t p2, uint32_t (&out)[3]) {
    const uint32_t plane[3] = {p0, p1, p2};
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int k = 0; k < 3; ++k) {
#pragma unroll
        for (int c = 0; c < 3; ++c) {                            // coordinates 11c .. 11c+10 start at bit 33c + k
            const uint64_t v = (uint64_t)spread3((plane[k] >> (11 * c)) & 0x7FFu) << ((33 * c + k) & 31);
            w[(33 * c + k) >> 5] |= (uint32_t)v;
            w[((33 * c + k) >> 5) + 1] |= (uint32_t)(v >> 32);
        }
    }
    out[0] = w[0]; out[1] = w[1]; out[2] = w[2];
}
// the `bits`-wide code that starts `shift` bits into the 64-bit little-endian window w1:w0
__device__ inline uint32_t code_at(uint32_t w0, uint32_t w1, uint32_t shift, int bits) {
    return __builtin_amdgcn_alignbit(w1, w0, shift) & ((1u << bits) - 1u);
}

// Centre of mass of N(0,1) on [delta (n - 1/2), delta (n + 1/2)], n >= 1; the interval of n = 127 runs to infinity
// (Sec. 3: the optimal value of an interval; Sec. 4.3: the uniform grid).
__device__ inline double grid_centroid(double delta, int n) {
    const double a = delta * (n - 0.5), b = delta * (n + 0.5);
    const bool open = n >= kGridMax;
    const double mass = 0.5 * (erfc(a * 0.7071067811865476) - (open ? 0.0 : erfc(b * 0.7071067811865476)));
    const double num = 0.3989422804014327 * (exp(-0.5 * a * a) - (open ? 0.0 : exp(-0.5 * b * b)));
    return mass > 0.0 ? num / mass : a;
}
// index of one coordinate on the uniform grid (as a signed byte in the low 8 bits) and its contribution |u| c to
// sum_i u_i Q_i; `ctab`: the centres of mass in LDS
// (a value on an interval endpoint goes to the interval closer to zero, Sec. 2.2.1 footnote: |n| = ceil(|z| / Delta - 1/2);
// the subtraction is exact for every quotient that matters, so the rounding of the quotient is the only error)
__device__ inline uint32_t quantize_grid(float u, float grid_inv, const float *ctab, float &ip) {
    const float m = fminf(ceilf(fabsf(u * grid_inv) - 0.5f), (float)kGridMax);
    const int mag = (int)m;                                      // -0.0 below half a step: 0
    ip = fmaf(fabsf(u), ctab[mag], ip);
    return (uint32_t)((__float_as_uint(u) >> 31) ? -mag : mag) & 0xFFu;
}
// value of a received byte: sign(n) * table[|n|]
__device__ inline float dequantize_grid(uint32_t byte, const float *dtab) {
    const int n = (int)(int8_t)byte;
    const int a = n < 0 ? -n : n;
    const float m = dtab[a > kGridMax ? kGridMax : a];           // (a sender never writes -128)
    return n < 0 ? -m : m;
}

// One-byte budgets.  `tab` in LDS: [0..127] the positive centroids (centres of mass), [128..255] the positive
// thresholds times |x| (b = 5..8 only; entries from H on are +inf).  b = 5..8: rank of |u| among the H - 1 positive
// thresholds by bisection over all 128 entries (seven reads, no branch: the padding never moves the rank), index =
// H + rank or H - 1 - rank (Sec. 2.2.1, Sec. 3).  GRID is a compile-time choice so that loops over many values
// stay free of branches (with a branch per value the compiler waits for every load before it issues the next).
template <bool GRID>
__device__ inline uint32_t quantize_byte(float u, uint32_t H, float grid_inv, const float *tab, float &ip) {
    if constexpr (GRID) {
        return quantize_grid(u, grid_inv, tab, ip);
    } else {
        const float a = fabsf(u);
        uint32_t mag = 0;
#pragma unroll
        for (uint32_t step = 64; step; step >>= 1) mag += (a > tab[128u + mag + step]) ? step : 0u;    // strict: ties stay closer to zero
        ip = fmaf(a, tab[mag], ip);
        return (__float_as_uint(u) >> 31) ? H - 1u - mag : H + mag;
    }
}
template <bool GRID>
__device__ inline float dequantize_byte(uint32_t byte, uint32_t H, const float *dtab) {
    if constexpr (GRID) {
        return dequantize_grid(byte, dtab);
    } else {
        const uint32_t code = byte & (2u * H - 1u);
        const float m = dtab[code >= H ? code - H : H - 1u - code];
        return code >= H ? m : -m;
    }
}
__device__ inline uint32_t wide_half_levels(uint32_t b_q8) { return wide_bits(b_q8) ? 1u << (wide_bits(b_q8) - 1u) : 0u; }

// b = K + 1/2 (Sec. 4.1): the index of one coordinate, K+1 bits wide where `up` (quantized with I_{K+1}), else K
// bits (I_K), and its contribution |u| q to sum_i u_i Q_i.
template <int K>
__device__ inline uint32_t quantize_mixed(float u, bool up, const EncScratch *sc, const float *qtab, float &ip) {
    constexpr int HL = 1 << (K - 1), HH = 1 << K;
    const float a = fabsf(u);
    const uint32_t mag_lo = magnitude_rank<HL>(a, sc->thr), mag_hi = magnitude_rank<HH>(a, sc->thr2);
    ip = fmaf(a, qtab[up ? 8u + mag_hi : mag_lo], ip);
    const bool neg = (__float_as_uint(u) >> 31) != 0u;
    const uint32_t code_lo = neg ? (uint32_t)(HL - 1) - mag_lo : (uint32_t)HL + mag_lo;
    const uint32_t code_hi = neg ? (uint32_t)(HH - 1) - mag_hi : (uint32_t)HH + mag_hi;
    return up ? code_hi : code_lo;
}

// ---- operands of the matrix instructions (v_mfma_f32_32x32x16_f16 / _fp8_fp8).  Lane l = 32 h + m holds, of A (32 x 16), row m
// and k = 8 h .. 8 h + 7; of B (16 x 32), column m and the same k; of the 32 x 32 result, column m and rows
// 8 (r / 4) + 4 h + r % 4 in registers r = 0 .. 15 (checked on the device with random integer matrices).
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
// entry (a, b) of the Sylvester Hadamard matrix
__device__ inline _Float16 hadamard_entry(uint32_t a, uint32_t b) {
    return (__builtin_popcount(a & b) & 1) ? (_Float16)-1.0f : (_Float16)1.0f;
}
// the second operand of the second of two chained transforms: the 16 result registers of the first product (rows of D1 in
// the order above) are, packed to fp16 in pairs, the B operands of two instructions (registers 0..7 and 8..15); entry e of
// instruction q on lane (h, m) of the Hadamard A operand must then stand for row 16 q + 8 (e / 4) + 4 h + e % 4
__device__ inline half8_t hadamard_rows_of_result(uint32_t q, uint32_t h, uint32_t m) {
    half8_t r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = hadamard_entry(16u * q + 8u * ((uint32_t)e >> 2) + 4u * h + ((uint32_t)e & 3u), m);
    return r;
}

// ---- narrow decode workspace.  After the strided pass of a two-pass size the values of a b <= 1 sender are integers of
// magnitude at most 2^10 (+-1 or 0 through at most ten butterfly stages): the workspace holds them as fp16, which is exact
// (11 significant bits) and is the operand type of the matrix-core pass that reads them back.
__device__ inline short narrow_bits(float v) { return __builtin_bit_cast(short, (_Float16)v); }
__device__ inline float narrow_value(short bits) { return (float)__builtin_bit_cast(_Float16, bits); }
// two int16 in one register -> two fp16, in place (written out: the compiler converts into two registers and packs them)
__device__ inline uint32_t narrow_pair_from_int16(uint32_t w) {
    asm("v_cvt_f16_i16_sdwa %0, %0 dst_sel:WORD_0 dst_unused:UNUSED_PRESERVE src0_sel:WORD_0\n\t"
        "v_cvt_f16_i16_sdwa %0, %0 dst_sel:WORD_1 dst_unused:UNUSED_PRESERVE src0_sel:WORD_1"
        : "+v"(w));
    return w;
}

// ---- blocked layout of the encoder's workspace between the 14-bit contiguous pass and a workgroup-tile strided pass that
// covers all the bits above it.  Element (row r, column block cb of 32 coordinates, column) of a sender's slot sits, in
// floats, at ((r / R) * 512 + cb) * (R * 32) + (r % R) * 32 + column with R = kBlockRows: the 128-byte segments of R
// consecutive rows are interleaved.  Row-major would be r * 2^14 + cb * 32 + column.  (At 16 senders of 2^24: R = 4 took the
// strided pass from 170 to 156 us and left the contiguous pass where it was; R = 8 slowed both passes by 10 us.)
constexpr uint32_t kBlockRows = 4;
constexpr uint32_t kBlockRowBits = 2;
__host__ __device__ inline size_t blocked_offset(uint32_t row, uint32_t cb) {
    return ((size_t)(row >> kBlockRowBits) << (14 + kBlockRowBits)) + ((size_t)cb << (5 + kBlockRowBits)) +
           ((size_t)(row & (kBlockRows - 1u)) << 5);
}

// ---- coin budgets: positions in the second part of the payload
// coins before the block of 64 coordinates number w of sender slot c
__device__ inline uint32_t coins_before(const CoinTables &ct, uint32_t c, int log2D, uint32_t w) {
    return ct.group[(size_t)c * ct.group_stride + w / (uint32_t)kCoinGroup] + ct.local[((size_t)c << (log2D - 6)) + w];
}
__device__ inline uint64_t coin_mask_of(const CoinTables &ct, uint32_t c, int log2D, uint32_t w) {
    return ct.mask[((size_t)c << (log2D - 6)) + w];
}
// set bits of `mask` below this lane's position
__device__ inline uint32_t lanes_below(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi(hi32(mask), __builtin_amdgcn_mbcnt_lo(lo32(mask), 0u));
}
// the bits of `value` at the set positions of `mask`, moved together towards bit 0 in the same order
__device__ inline uint64_t compress_bits(uint64_t value, uint64_t mask) {
    uint64_t out = 0, place = 1;
    while (mask) {
        const uint64_t lowest = mask & (0 - mask);
        if (value & lowest) out |= place;
        place <<= 1;
        mask ^= lowest;
    }
    return out;
}
// ORs the low `count` bits of `value` (the others are zero) into a zeroed little-endian bit string at bit `off`.  The string
// starts on an 8-byte boundary (the second part of a payload does) and is a whole number of 8-byte words long: 64-bit atomics,
// one per piece unless the piece straddles a word (about a third fewer than with 32-bit ones; they are what this costs).
__device__ inline void or_bits(uint32_t *words, uint32_t off, uint64_t value, uint32_t count) {
    if (!count) return;
    unsigned long long *q = reinterpret_cast<unsigned long long *>(words) + (off >> 6);
    const uint32_t sh = off & 63u;
    const unsigned long long lo = value << sh, hi = sh ? value >> (64u - sh) : 0ull;
    if (lo) atomicOr(q, lo);
    if (hi) atomicOr(q + 1, hi);
}

// Butterflies over the low LOGB bits of the register index only (FIRST = 2: all but the stage over bit 0).
template <int N, int LOGB, int FIRST = 1>
__device__ inline void fwht_regs_low(float (&v)[N]) {
#pragma unroll
    for (int h = FIRST; h < (1 << LOGB); h <<= 1) {
#pragma unroll
        for (int i = 0; i < N; i += 2 * h) {
#pragma unroll
            for (int j = i; j < i + h; ++j) {
                const float a = v[j], b = v[j + h];
                v[j] = a + b;
                v[j + h] = a - b;
            }
        }
    }
}

// ---- decode: what the receiver derives from a message's header and its packet bitmap
//
// One wave per message: check the header against what the receiver agreed on, count the coordinates
// that arrived (Sec. 4.2: the receiver finds p by counting), and build the dequantization table
// (S / (p sqrt(D))) * q_l  -- S/p from Sec. 4.2, D^-1/2 from the inverse rotation.
// `hdr_d`, `hdr_b_q8`: what the header must say; `b_q8`: the budget the kernels dequantize with.
// `extra_bits`: coin budgets only, the number of coins the receiver counted itself; the header must agree.
__device__ inline void dec_prepare_wave(const void *msg, const uint32_t *bitmap, uint32_t client, uint32_t b_q8,
                                        uint32_t hdr_b_q8, uint64_t hdr_d, int log2D, uint64_t seed, const DevTables *tab,
                                        DecScratch *out, uint32_t *dev_status, uint32_t extra_bits = 0,
                                        uint32_t *msg_flag = nullptr) {
    const uint32_t lane = lane_id();
    const MsgHeader h = *static_cast<const MsgHeader *>(msg);
    uint32_t flags = 0;
    if (h.magic != kMagic || h.log2D != (uint32_t)log2D || h.d != hdr_d || h.b_q8 != hdr_b_q8 ||
        h.client != client || h.seed != seed || (coin_q8(b_q8) && h.extra_bits != extra_bits))
        flags |= EDEN_DEV_HEADER_MISMATCH;
    else
        flags |= h.status & (EDEN_DEV_ZERO_VECTOR | EDEN_DEV_NONFINITE);
    const uint64_t D = 1ull << log2D;
    const uint32_t npk = D >= EDEN_PACKET_COORDS ? (uint32_t)(D / EDEN_PACKET_COORDS) : 1u;
    uint32_t got = 0;
    if (bitmap) {
        const uint32_t nw = (npk + 31u) / 32u;
        for (uint32_t w = lane; w < nw; w += 64) {
            uint32_t bits = bitmap[w];
            if (w == nw - 1 && (npk & 31u)) bits &= (1u << (npk & 31u)) - 1u;
            got += __popc(bits);
        }
        got = wave_sum_u32(got);
    } else {
        got = npk;
    }
    int bits, k;
    budget_of(b_q8, bits, k);
    const uint64_t per_packet = D >= EDEN_PACKET_COORDS ? EDEN_PACKET_COORDS : D;
    const uint64_t arrived = (uint64_t)got * per_packet / (uint64_t)k;
    if (flags == 0 && arrived == 0) flags |= EDEN_DEV_NOTHING_ARRIVED;
    double coef = 0.0;
    if (flags == 0) coef = h.S * exp2(0.5 * (double)log2D) / (double)arrived;     // S / (p sqrt(D)), p = arrived / D
    if (sparse_m(hdr_b_q8)) coef *= 64.0 / (double)sparse_m(hdr_b_q8);             // the 1/p of the sparsification (Sec. 4.1)
    if (lane < 32) {                                             // lanes 16..31: the finer table of a mixed budget
        const int tb = (lane < 16 || !budget_two_tables(b_q8)) ? bits : bits + 1;
        const int H = 1 << (tb - 1), l = (int)(lane & 15u);
        double q = 0.0;
        if (l < 2 * H) q = (l >= H) ? tab->q[tb][l - H] : -tab->q[tb][H - 1 - l];
        if (lane < 16) out->deq[l] = (float)(coef * q);
        else out->deq2[l] = (float)(coef * q);
    }
    if (grid_q15(b_q8)) {                                        // uniform grid: the centres of mass, two per lane
        const double delta = (double)grid_q15(b_q8) / 32768.0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int n = (int)lane + 64 * h;
            out->grid_deq[n] = n ? (float)(coef * grid_centroid(delta, n)) : 0.0f;
        }
    } else if (const uint32_t wb = wide_bits(b_q8)) {            // b = 5..8: the positive centroids, two per lane
#pragma unroll
        for (int h = 0; h < 2; ++h) out->grid_deq[lane + 64 * h] = (float)(coef * tab->q_big[wb - 5u][lane + 64 * h]);
    }
    if (lane == 0) {
        out->flags = flags;
        if (msg_flag) *msg_flag = flags;                         // per message, for eden_last_decode_flags
        if (flags & (EDEN_DEV_HEADER_MISMATCH | EDEN_DEV_NOTHING_ARRIVED)) atomicOr(dev_status, flags);
    }
}


}  // namespace eden
#endif
