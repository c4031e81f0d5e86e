// HIP kernels of the EDEN hot path for gfx950 (MI355X), wave-tile passes and the small sizes.  Wave64 throughout.
//
// The rotation R x = D^-1/2 H (s o x) (Sec. 2.2.1; Sec. 5: randomized Hadamard transform) is computed
// unnormalised, u = H (s o x), with the D^-1/2 folded into scalars.  The index bits of the padded
// dimension D = 2^L are split into groups; one kernel ("pass") transforms one group:
//
//   lo pass   bits 0..11   one wave owns 4096 consecutive coordinates: 64 registers per lane, six
//                          butterfly stages in registers, a 64x64 transpose through LDS, six more.
//   hi pass   bits p..p+M-1 (M <= 6): one wave owns 2^M rows of 64 consecutive coordinates at stride 2^p;
//                          every lane keeps one column in registers; no LDS at all.
//
// Encode runs the lo pass first (it reads x, applies the signs and sums |x|^2, and only touches the tiles
// that hold part of x) and the hi passes after it, the last one fused with quantization, <R(x),Q> and bit
// packing (Sec. 2.2.1, 2.3).  Decode runs the hi passes first, the first one fused with unpacking and centroid
// lookup (Sec. 2.2.2, 4.2), and the lo pass last: it applies the signs and sums the senders in registers before
// touching the accumulator once.  D <= 4096 is handled by one workgroup per sender with the vector in LDS.
#include "eden_device.h"
#include "eden_kernels.h"

namespace eden {

// After |x|^2 is known: the thresholds of I_b scaled to the unnormalised transform.
// z = eta R(x) = u / |x| (Sec. 2.2.1 with d -> D), so z > t  <=>  u > t |x|.
__device__ inline void fill_enc_scratch(EncScratch *s, double n2, uint32_t b_q8, const DevTables *tab) {
    int bits, k;
    budget_of(b_q8, bits, k);
    s->n2 = n2;
    const double norm = sqrt(n2);
    if (grid_q15(b_q8)) {                                        // uniform grid: no table of thresholds, only the step
        s->grid_inv = (float)(32768.0 / ((double)grid_q15(b_q8) * norm));
        return;
    }
    if (wide_bits(b_q8)) return;                                 // b = 5..8: the long tables are filled by fill_byte_tables
    const int finer = budget_two_tables(b_q8) ? bits + 1 : bits;
    for (int i = 0; i < 8; ++i) {
        s->thr[i] = (float)(tab->t[bits][i] * norm);
        s->qpos[i] = (float)tab->q[bits][i];
        s->thr2[i] = (float)(tab->t[finer][i] * norm);
        s->qpos2[i] = (float)tab->q[finer][i];
    }
}
// The tables of the one-byte budgets, one entry per thread (tid < 128): the centres of mass of the uniform grid's
// intervals, or the positive centroids and scaled thresholds of the 32..256-level quantizers.
__device__ inline void fill_byte_tables(EncScratch *s, uint32_t b_q8, double n2, const DevTables *tab, uint32_t tid) {
    if (tid > (uint32_t)kGridMax) return;
    if (const uint32_t q15 = grid_q15(b_q8)) {
        s->grid_c[tid] = tid ? (float)grid_centroid((double)q15 / 32768.0, (int)tid) : 0.0f;
    } else if (const uint32_t wb = wide_bits(b_q8)) {
        const uint32_t H = 1u << (wb - 1u);
        s->grid_c[tid] = tid < H ? (float)tab->q_big[wb - 5u][tid] : 0.0f;
        s->wide_thr[tid] = tid < H ? (float)(tab->t_big[wb - 5u][tid] * sqrt(n2)) : INFINITY;   // padding for the bisection
    }
}

// ------------------------------------------------------------------------------------------------
// hi passes
template <int M>
__device__ inline void hi_tile_origin(uint32_t tile, int p, uint64_t &base) {
    const uint32_t cb_bits = (uint32_t)p - 6u;                  // 2^(p-6) blocks of 64 columns
    const uint32_t colblock = tile & ((1u << cb_bits) - 1u);
    const uint32_t upper = tile >> cb_bits;
    base = ((uint64_t)upper << (p + M)) | ((uint64_t)colblock << 6);
}

// The K-bit indices of one row segment of 64 consecutive coordinates, given as bit planes (plane[b][0/1]: bit b of
// the indices of coordinates 0..31 / 32..63), written as the 2K payload words that start at coordinate `first`
// (a multiple of 64): index i occupies bits K i .. K i + K - 1 of the little-endian bit string.
template <int K>
__device__ inline void store_row_planes(const uint32_t (&plane)[4][2], uint32_t *payload, uint64_t first) {
    if constexpr (K == 1) {
        *reinterpret_cast<uint2 *>(payload + (first >> 5)) = make_uint2(plane[0][0], plane[0][1]);
    } else if constexpr (K == 2) {
        uint32_t o[4];                                           // word k: coordinates 16 k .. 16 k + 15
#pragma unroll
        for (int k = 0; k < 4; ++k)
            o[k] = spread2(plane[0][k >> 1] >> (16 * (k & 1))) | (spread2(plane[1][k >> 1] >> (16 * (k & 1))) << 1);
        *reinterpret_cast<uint4 *>(payload + (first >> 4)) = make_uint4(o[0], o[1], o[2], o[3]);
    } else if constexpr (K == 3) {
        uint32_t lo[3], hi[3];                                   // 64 coordinates x 3 bits = 6 words
        pack3_planes(plane[0][0], plane[1][0], plane[2][0], lo);
        pack3_planes(plane[0][1], plane[1][1], plane[2][1], hi);
        uint2 *dst = reinterpret_cast<uint2 *>(payload + (first >> 6) * 6u);
        dst[0] = make_uint2(lo[0], lo[1]);
        dst[1] = make_uint2(lo[2], hi[0]);
        dst[2] = make_uint2(hi[1], hi[2]);
    } else {
        uint32_t o[8];                                           // word k: coordinates 8 k .. 8 k + 7
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            o[k] = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) o[k] |= spread4(plane[b][k >> 2] >> (8 * (k & 3))) << b;
        }
        uint4 *dst = reinterpret_cast<uint4 *>(payload + (first >> 3));
        dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
        dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
    }
}

// Quantizes the R rows of a wave tile (register r = row r, one column per lane) and packs them.  K: bits of every
// index in the first part of the payload.  MIX = 1 (b = K + 1/2, Sec. 4.1): the coordinate of every pair that the MIX
// stream selects is quantized with I_{K+1}; the top bit of its index goes to the second part, one bit per pair.
// MIX = 2 (coin budgets, Sec. 4.1): the coordinates with a coin (`my_mask`: the coins of this lane's row) are quantized
// with I_{K+1}; their top bits go to the second part in coordinate order, the row's first one at bit `my_off`.
// `my_row`: first coordinate of the row that this lane (< R) finishes.
template <int R, int K, int MIX>
__device__ inline void hi_quantize_pack(const float (&v)[R], const EncScratch *sc, const float *qtab, uint64_t mixkey,
                                        uint64_t my_row, uint32_t *part_a, uint32_t *part_b, float &ip,
                                        uint64_t my_mask = 0, uint32_t my_off = 0) {
    constexpr int H = 1 << (K - 1);
    const uint32_t lane = lane_id();
    uint32_t plane[4][2], top[2] = {0u, 0u};
#pragma unroll
    for (int b = 0; b < 4; ++b) plane[b][0] = plane[b][1] = 0;
    // 64 pairs per hash word = 128 coordinates; a row segment uses 32 of them
    const uint32_t offs_mine = MIX == 1 ? (uint32_t)(hash_word(mixkey, my_row >> 7) >> (32u * (uint32_t)((my_row >> 6) & 1u))) : 0u;
    static_for<R>([&](auto RR) {
        constexpr int r = decltype(RR)::value;
        uint32_t code;
        if constexpr (MIX != 0) {
            bool up;
            if constexpr (MIX == 1) {
                const uint32_t offs = __builtin_amdgcn_readlane(offs_mine, r);
                up = ((offs >> (lane >> 1)) & 1u) == (lane & 1u);
            } else {
                up = __builtin_amdgcn_inverse_ballot_w64(wave_read64(my_mask, r));
            }
            code = quantize_mixed<K>(v[r], up, sc, qtab, ip);
            const uint64_t m = __ballot((code >> K) & 1u);
            top[0] = put_lane<r>(lo32(m), top[0]);
            top[1] = put_lane<r>(hi32(m), top[1]);
        } else {
            code = quantize_one<H>(v[r], sc, qtab, ip);
        }
#pragma unroll
        for (int b = 0; b < K; ++b) {
            const uint64_t m = __ballot((code >> b) & 1u);
            plane[b][0] = put_lane<r>(lo32(m), plane[b][0]);
            plane[b][1] = put_lane<r>(hi32(m), plane[b][1]);
        }
    });
    if (lane < R) {
        store_row_planes<K>(plane, part_a, my_row);
        if constexpr (MIX == 1)                                  // only the chosen coordinate of a pair can have the bit
            part_b[my_row >> 6] = even_bits(top[0] | (top[0] >> 1)) | (even_bits(top[1] | (top[1] >> 1)) << 16);
        if constexpr (MIX == 2) {                                // only a coordinate with a coin can have the bit
            const uint64_t top64 = (uint64_t)top[0] | ((uint64_t)top[1] << 32);
            or_bits(part_b, my_off, compress_bits(top64, my_mask), (uint32_t)__popcll(my_mask));
        }
    }
}

// Encode, last pass in wave tiles: T -> payload.  Index bits p .. p+M-1 of H, then quantization to the
// Lloyd-Max intervals (Sec. 2.2.1, Sec. 3), sum_i u_i q_i for the scale (Sec. 2.3), sub-sampling for b = 1/2
// (Sec. 4.1), packing.  Register r is row r of the tile = 64 consecutive coordinates across the lanes, so a
// ballot of one index bit is 64 payload bits of that row; lane r collects the ballots of row r and packs them.
// Workspace elements at or above `valid_elems` were not written by the earlier passes because they are
// zero (transformed zero padding): the buffer bounds return 0 for them.
// ONLY != 0: every sender of the launch has this budget (1, 2 or 4 bits); the instance then holds that one branch.
template <int M, uint32_t ONLY = 0>
__global__ __launch_bounds__(256) void k_enc_hi_last(EncBatch B, uint64_t valid_elems, int log2D, int p, uint64_t seed,
                                                     const float *T, double *partials, uint32_t partial_stride,
                                                     const EncScratch *scratch, CoinTables ct) {
    constexpr int R = 1 << M;
    __shared__ double red[4];
    __shared__ float qtabs[4][16];
    __shared__ float gtabs[4][256];                              // one-byte budgets: centroids and thresholds
    const uint32_t c = blockIdx.y;
    const uint32_t lane = lane_id();
    const uint32_t tile = blockIdx.x * 4u + wave_in_block();
    const uint32_t ntiles = 1u << (log2D - 6 - M);
    float ip = 0.0f;
    if (tile < ntiles) {
        uint64_t base;
        hi_tile_origin<M>(tile, p, base);
        const rsrc_t rt = make_rsrc(T + ((size_t)c << log2D), (uint32_t)(valid_elems * 4));
        const uint32_t lane_off = lane * 4u, base_off = (uint32_t)base * 4u;
        float v[R];
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] = buf_load(rt, lane_off, base_off + ((uint32_t)r << (p + 2)));
        fwht_regs<R>(v);
        uint32_t *payload = reinterpret_cast<uint32_t *>(static_cast<char *>(B.msg[c]) + EDEN_HEADER_BYTES);
        const uint32_t b_q8 = ONLY ? ONLY : B.b_q8[c];
        const uint64_t my_row = base + ((uint64_t)(lane & (R - 1)) << p);       // lane r < R finishes row r
        if (b_q8 <= 256u) {
            // I_1 = {(-inf,0],[0,inf)}: the index is the sign; <R(x),Q> = q_1 sum |u| / sqrt(D)
            float sa = 0.0f;
#pragma unroll
            for (int r = 0; r < R; ++r) sa += fabsf(v[r]);
            ip = sa * kQ1;
            uint32_t wlo = 0, whi = 0;
            static_for<R>([&](auto RR) {
                constexpr int r = decltype(RR)::value;
                const uint64_t m = __ballot((__float_as_uint(v[r]) >> 31) == 0u);    // index 1 = non-negative
                wlo = put_lane<r>(lo32(m), wlo);
                whi = put_lane<r>(hi32(m), whi);
            });
            if (lane < R) {
                if (b_q8 == 256u) {
                    *reinterpret_cast<uint2 *>(payload + (my_row >> 5)) = make_uint2(wlo, whi);
                } else {
                    // b = 1/2: of each pair (2g, 2g+1) send the coordinate chosen by the sub-sampling stream;
                    // 64 pairs per hash word = 128 coordinates, a row segment uses 32 of them
                    const uint64_t key = stream_key(seed, kStreamSubsample, B.client[c]);
                    const uint32_t off = (uint32_t)(hash_word(key, my_row >> 7) >> (32u * (uint32_t)((my_row >> 6) & 1u)));
                    const uint32_t ev = even_bits(wlo) | (even_bits(whi) << 16);
                    const uint32_t od = even_bits(wlo >> 1) | (even_bits(whi >> 1) << 16);
                    payload[my_row >> 6] = (ev & ~off) | (od & off);
                }
            }
        } else {
            const EncScratch *sc = &scratch[c];
            float *qtab = qtabs[wave_in_block()];
            fill_qtab(qtab, sc, lane);
            wave_lds_sync();
            const uint64_t mixkey = stream_key(seed, kStreamMix, B.client[c]);
            uint32_t *part_b = payload + payload_a_bytes(1ull << log2D, (int)(b_q8 >> 8), 1) / 4;
            if (byte_budget(b_q8)) {
                // uniform grid (Sec. 4.3) or b = 5..8: one byte per coordinate; a row of the tile is 64 consecutive bytes
                float *ctab = gtabs[wave_in_block()];
                const float *byte_tab = sc->grid_c;              // grid_c[128] and wide_thr[128] are one run of 256 floats
#pragma unroll
                for (int q = 0; q < 4; ++q) ctab[64 * q + lane] = byte_tab[64 * q + lane];       // centroids, then thresholds
                wave_lds_sync();
                const float inv = sc->grid_inv;
                uint8_t *bytes = B.codes[c] ? B.codes[c] : reinterpret_cast<uint8_t *>(payload);
                const uint32_t H = wide_half_levels(b_q8);
                if (grid_q15(b_q8)) {                            // the indices replace the values in their registers
#pragma unroll
                    for (int r = 0; r < R; ++r) v[r] = __uint_as_float(quantize_byte<true>(v[r], H, inv, ctab, ip));
                } else {
#pragma unroll
                    for (int r = 0; r < R; ++r) v[r] = __uint_as_float(quantize_byte<false>(v[r], H, inv, ctab, ip));
                }
#pragma unroll
                for (int r = 0; r < R; ++r) {                    // four lanes' bytes = one dword store
                    const uint32_t quad = quad_bytes(__float_as_uint(v[r]), lane);
                    if (!(lane & 3u)) *reinterpret_cast<uint32_t *>(bytes + base + ((uint64_t)r << p) + lane) = quad;
                }
            } else if (const uint32_t cq = coin_q8(b_q8)) {
                // the coins of this lane's row, and where the row's first extra bit goes in the second part
                const uint32_t w = (uint32_t)(my_row >> 6);
                const uint64_t my_mask = coin_mask_of(ct, c, log2D, w);
                const uint32_t my_off = coins_before(ct, c, log2D, w);
                uint32_t *part_c = payload + payload_a_bytes(1ull << log2D, (int)(cq >> 8), 1) / 4;
                if ((cq >> 8) == 1u) hi_quantize_pack<R, 1, 2>(v, sc, qtab, mixkey, my_row, payload, part_c, ip, my_mask, my_off);
                else if ((cq >> 8) == 2u) hi_quantize_pack<R, 2, 2>(v, sc, qtab, mixkey, my_row, payload, part_c, ip, my_mask, my_off);
                else hi_quantize_pack<R, 3, 2>(v, sc, qtab, mixkey, my_row, payload, part_c, ip, my_mask, my_off);
            } else
            switch (b_q8) {
                case 384u: hi_quantize_pack<R, 1, 1>(v, sc, qtab, mixkey, my_row, payload, part_b, ip); break;
                case 512u: hi_quantize_pack<R, 2, 0>(v, sc, qtab, mixkey, my_row, payload, part_b, ip); break;
                case 640u: hi_quantize_pack<R, 2, 1>(v, sc, qtab, mixkey, my_row, payload, part_b, ip); break;
                case 768u: hi_quantize_pack<R, 3, 0>(v, sc, qtab, mixkey, my_row, payload, part_b, ip); break;
                case 896u: hi_quantize_pack<R, 3, 1>(v, sc, qtab, mixkey, my_row, payload, part_b, ip); break;
                default: hi_quantize_pack<R, 4, 0>(v, sc, qtab, mixkey, my_row, payload, part_b, ip); break;
            }
        }
    }
    const double block_total = block_sum<256>((double)ip, red);
    if (threadIdx.x == 0) partials[(size_t)c * partial_stride + blockIdx.x] = block_total;
}

// One workgroup per sender: sums the per-workgroup partials of |x|^2 in index order (deterministic)
// and scales the thresholds.  Runs between the first pass and the quantizing pass because eta
// depends on the whole vector (Sec. 2.2.1).
__global__ __launch_bounds__(256) void k_enc_norm(EncBatch B, const double *partials, uint32_t partial_stride,
                                                  uint32_t nparts, EncScratch *scratch, const DevTables *tab) {
    __shared__ double red[4];
    const uint32_t c = blockIdx.x;
    const double *pc = partials + (size_t)c * partial_stride;
    double s = 0.0;
    for (uint32_t i = threadIdx.x; i < nparts; i += 256) s += pc[i];
    const double total = block_sum<256>(s, red);
    __shared__ double n2_all;
    if (threadIdx.x == 0) {
        fill_enc_scratch(&scratch[c], total, B.b_q8[c], tab);
        n2_all = total;
    }
    __syncthreads();
    fill_byte_tables(&scratch[c], B.b_q8[c], n2_all, tab, threadIdx.x);
}

// Decode, first pass in wave tiles (Sec. 2.2.2, 4.2): unpack, centroid lookup times S/(p sqrt D) (or the unit
// pattern +-1 when the workspace of a b <= 1 sender is fp16), zero for coordinates that were not sampled or
// whose packet was lost, then index bits p .. p+M-1 of H.  Every (tile, sender) pair is independent.
// Elements at or above `keep_elems` are never read by the later passes (they end in the padding): the buffer
// bounds drop their stores.
// (Five waves per SIMD are requested: the budgets with two loads per value would otherwise set the register count
// for all of them; measured 0.057 against 0.073 ms on 32 senders at D = 2^20.)
// ONLY != 0: every sender of the launch has this budget (1, 2 or 4 bits, indices in the payload); the instance then holds
// that one branch (the shared one spills 304 bytes at its 96 registers).
template <int M, uint32_t ONLY = 0>
__global__ __launch_bounds__(256, 5) void k_dec_hi_first(DecBatch B, uint64_t keep_elems, int log2D, int p, uint64_t seed,
                                                      const DecScratch *scratch, int narrow, float *T, CoinTables ct) {
    constexpr int R = 1 << M;
    __shared__ float table[4][32];
    __shared__ float gtabs[4][kGridMax + 1];                     // uniform grid: dequantized centres of mass
    const uint32_t c = blockIdx.y;
    const uint32_t lane = lane_id(), wv = wave_in_block();
    const uint32_t tile = blockIdx.x * 4u + wv;
    const uint32_t ntiles = 1u << (log2D - 6 - M);
    if (tile >= ntiles) return;
    uint64_t base;
    hi_tile_origin<M>(tile, p, base);
    const uint32_t b_q8 = ONLY ? ONLY : B.b_q8[c];
    const bool i16 = narrow && b_q8 <= 256u;
    if (lane < 16) table[wv][lane] = (i16 && lane == 1) ? 1.0f : scratch[c].deq[lane];
    else if (lane < 32) table[wv][lane] = scratch[c].deq2[lane - 16];
    if (byte_budget(b_q8)) { gtabs[wv][lane] = scratch[c].grid_deq[lane]; gtabs[wv][64 + lane] = scratch[c].grid_deq[64 + lane]; }
    wave_lds_sync();
    const float *tb = table[wv], *tb2 = table[wv] + 16;
    const uint32_t *payload = reinterpret_cast<const uint32_t *>(static_cast<const char *>(B.msg[c]) + EDEN_HEADER_BYTES);
    int bits, k;
    budget_of(b_q8, bits, k);
    const uint32_t payload_bytes = (uint32_t)(((((1ull << log2D) >> (k == 2)) * (uint32_t)bits + 63) >> 6) << 3);
    const uint64_t my_row = base + ((uint64_t)(lane & (R - 1)) << p);       // lane r looks after row r
    uint64_t recv = ~0ull;                                       // bit r: the packet of row r arrived
    if (const uint32_t *bm = B.bitmap[c]) {
        const uint32_t pk = (uint32_t)(my_row >> 10);
        recv = __ballot((bm[pk >> 5] >> (pk & 31u)) & 1u);
    }
    float v[R];
    if (b_q8 == 128) {
        // b = 1/2: pair j = i >> 1 carries one bit; coordinate i was sent iff (i & 1) equals the pair's offset bit
        const uint64_t key = stream_key(seed, kStreamSubsample, B.client[c]);
        const uint32_t offs_mine = (uint32_t)(hash_word(key, my_row >> 7) >> (32u * (uint32_t)((base >> 6) & 1u)));
        const rsrc_t rp = make_rsrc(payload + (base >> 6), payload_bytes - (uint32_t)(base >> 6) * 4u);
        const uint32_t mag = __float_as_uint(tb[1]);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(rp, 0, (int)(((uint32_t)r << (p - 6)) * 4u), 0);
            const uint32_t offs = __builtin_amdgcn_readlane(offs_mine, r);
            const bool kept = ((offs >> (lane >> 1)) & 1u) == (lane & 1u);
            const uint32_t neg = (~(w >> (lane >> 1)) & 1u) << 31;          // index 0 = negative
            v[r] = kept ? __uint_as_float(mag | neg) : 0.0f;
        }
    } else if (byte_budget(b_q8)) {
        // one byte per coordinate: the index on the uniform grid (Sec. 4.3) or of a 32..256-level quantizer
        const uint8_t *bytes = B.codes[c] ? B.codes[c] : reinterpret_cast<const uint8_t *>(payload);
        const rsrc_t rp = make_rsrc(bytes + base, (1u << log2D) - (uint32_t)base);
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] = __uint_as_float(buf_load_byte(rp, lane, (uint32_t)r << p));
        const uint32_t H = wide_half_levels(b_q8);
        if (grid_q15(b_q8)) {                                    // the values replace the bytes in their registers
#pragma unroll
            for (int r = 0; r < R; ++r) v[r] = dequantize_byte<true>(__float_as_uint(v[r]), H, gtabs[wv]);
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r) v[r] = dequantize_byte<false>(__float_as_uint(v[r]), H, gtabs[wv]);
        }
    } else if (budget_mixed(b_q8)) {
        // b = bits + 1/2 (Sec. 4.1): every coordinate has `bits` bits in the first part; the coordinate of each pair
        // that the MIX stream selects was quantized with the finer table and has its top bit in the second part
        const uint64_t key = stream_key(seed, kStreamMix, B.client[c]);
        const uint32_t offs_mine = (uint32_t)(hash_word(key, my_row >> 7) >> (32u * (uint32_t)((base >> 6) & 1u)));
        const uint32_t lbits = lane * (uint32_t)bits, words_row = 2u * (uint32_t)bits;      // words of one row segment
        const rsrc_t rp = make_rsrc(payload + (base >> 6) * words_row, payload_bytes - (uint32_t)(base >> 6) * words_row * 4u);
        const uint32_t *part_b = payload + payload_bytes / 4u;
        const rsrc_t rb = make_rsrc(part_b + (base >> 6), (uint32_t)payload_b_bytes(1ull << log2D, b_q8) - (uint32_t)(base >> 6) * 4u);
        const uint32_t voff = (lbits >> 5) * 4u, shift = lbits & 31u;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int soff = (int)((((uint32_t)r * words_row) << (p - 6)) * 4u);
            const uint32_t w0 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, soff, 0);
            const uint32_t w1 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff + 4, soff, 0);    // always: no branch per value
            const uint32_t low = code_at(w0, w1, shift, bits);
            const uint32_t wb = __builtin_amdgcn_raw_buffer_load_b32(rb, 0, (int)(((uint32_t)r << (p - 6)) * 4u), 0);
            const uint32_t offs = __builtin_amdgcn_readlane(offs_mine, r);
            const bool up = ((offs >> (lane >> 1)) & 1u) == (lane & 1u);
            const uint32_t top = (wb >> (lane >> 1)) & 1u;
            v[r] = up ? tb2[(top << bits) | low] : tb[low];
        }
    } else if (coin_q8(b_q8)) {
        // coin budgets (Sec. 4.1): every coordinate has `bits` bits in the first part; a coordinate with a coin was
        // quantized with the finer table and has its top bit in the second part, at the position of its rank among the coins
        const uint32_t w = (uint32_t)(my_row >> 6);
        const uint64_t mask_mine = coin_mask_of(ct, c, log2D, w);
        const uint32_t off_mine = coins_before(ct, c, log2D, w);
        const uint32_t lbits = lane * (uint32_t)bits, words_row = 2u * (uint32_t)bits;
        const rsrc_t rp = make_rsrc(payload + (base >> 6) * words_row, payload_bytes - (uint32_t)(base >> 6) * words_row * 4u);
        const rsrc_t rb = make_rsrc(payload + payload_bytes / 4u, (uint32_t)coin_b_bytes(ct.total[c]));
        const uint32_t voff = (lbits >> 5) * 4u, shift = lbits & 31u;
        // the top bits of a row's coins are at most 64 consecutive bits of the second part, from bit off_mine on: the lane
        // that looks after the row fetches them once (beyond the part: 0), and every lane finds its bit in that window
        uint64_t window_mine;
        {
            const int at = (int)((off_mine >> 5) * 4u);
            const uint32_t b0 = __builtin_amdgcn_raw_buffer_load_b32(rb, at, 0, 0), b1 = __builtin_amdgcn_raw_buffer_load_b32(rb, at + 4, 0, 0);
            const uint32_t b2 = __builtin_amdgcn_raw_buffer_load_b32(rb, at + 8, 0, 0);
            window_mine = ((uint64_t)__builtin_amdgcn_alignbit(b2, b1, off_mine & 31u) << 32) | __builtin_amdgcn_alignbit(b1, b0, off_mine & 31u);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int soff = (int)((((uint32_t)r * words_row) << (p - 6)) * 4u);
            const uint32_t w0 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, soff, 0);
            const uint32_t w1 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff + 4, soff, 0);    // always: no branch per value
            const uint32_t low = code_at(w0, w1, shift, bits);
            const uint64_t m = wave_read64(mask_mine, r);
            const uint32_t top = (uint32_t)(wave_read64(window_mine, r) >> lanes_below(m)) & 1u;
            v[r] = __builtin_amdgcn_inverse_ballot_w64(m) ? tb2[(top << bits) | low] : tb[low];
        }
    } else if (bits == 3) {
        // 64 columns x 3 bits = 6 words per row; an index may straddle two words
        const uint32_t lbits = lane * 3u;
        const rsrc_t rp = make_rsrc(payload + (base >> 6) * 6u, payload_bytes - (uint32_t)(base >> 6) * 24u);
        const uint32_t voff = (lbits >> 5) * 4u, shift = lbits & 31u;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int soff = (int)((((uint32_t)r * 6u) << (p - 6)) * 4u);
            const uint32_t w0 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, soff, 0);
            const uint32_t w1 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff + 4, soff, 0);
            v[r] = tb[code_at(w0, w1, shift, 3)];
        }
    } else {
        const uint32_t lbits = lane * (uint32_t)bits;
        const rsrc_t rp = make_rsrc(payload + ((base * (uint32_t)bits) >> 5), payload_bytes - (uint32_t)((base * (uint32_t)bits) >> 5) * 4u);
        const uint32_t voff = (lbits >> 5) * 4u, shift = lbits & 31u;
        const uint32_t mag = __float_as_uint(tb[1]);
#pragma unroll
        for (int r = 0; r < R; ++r)                              // all loads first, no choice per value in between
            v[r] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, (int)((((uint32_t)r * (uint32_t)bits) << (p - 5)) * 4u), 0));
        if (bits == 1) {
#pragma unroll
            for (int r = 0; r < R; ++r) v[r] = __uint_as_float(mag | ((~(__float_as_uint(v[r]) >> shift) & 1u) << 31));
        } else {
#pragma unroll
            for (int r = 0; r < R; ++r) v[r] = tb[(__float_as_uint(v[r]) >> shift) & ((1u << bits) - 1u)];
        }
    }
    if (B.bitmap[c]) {
#pragma unroll
        for (int r = 0; r < R; ++r) v[r] = ((recv >> r) & 1ull) ? v[r] : 0.0f;     // wave-uniform per row
    }
    fwht_regs<R>(v);
    if (i16) {                                                   // exact integers of magnitude <= 2^M, as fp16
        const rsrc_t rt = make_rsrc(T + ((size_t)c << log2D), (uint32_t)(keep_elems * 2));
#pragma unroll
        for (int r = 0; r < R; ++r)
            __builtin_amdgcn_raw_buffer_store_b16(narrow_bits(v[r]), rt, (int)(lane * 2u),
                                                  (int)(((uint32_t)base + ((uint32_t)r << p)) * 2u), kStream);
    } else {
        const rsrc_t rt = make_rsrc(T + ((size_t)c << log2D), (uint32_t)(keep_elems * 4));
#pragma unroll
        for (int r = 0; r < R; ++r) buf_store(rt, lane * 4u, ((uint32_t)base + ((uint32_t)r << p)) * 4u, v[r]);
    }
}

// ------------------------------------------------------------------------------------------------
// Wide strided tiles for the top three index bits of the three-pass sizes (D >= 2^25), budgets b = 1, 2, 4 and the
// one-byte budgets (b = 5..8, uniform grid):
// a wave owns 8 rows of 512 consecutive coordinates at stride 2^p (p = log2 D - 3).  A lane holds, of every row,
// the columns 4 l .. 4 l + 3 and 256 + 4 l .. 256 + 4 l + 3: each workspace access of a wave is then one dense
// kilobyte (16 bytes per lane, no gaps; with 8 adjacent columns per lane the two halves of every 128-byte line
// were written by different instructions and 1.7x the bytes reached memory), and a lane's four indices of a
// half row are 4 b bits of payload: a half-word / byte / nibble per lane, 32..128 dense bytes per wave
// (the one-column-per-lane wave tile moves a b = 4 payload in 32-byte pieces).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kWideRows = 8, kWideCols = 512;

__device__ inline void wide_fwht(float (&v)[kWideRows][8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        float col[kWideRows];
#pragma unroll
        for (int r = 0; r < kWideRows; ++r) col[r] = v[r][e];
        fwht_regs<kWideRows>(col);
#pragma unroll
        for (int r = 0; r < kWideRows; ++r) v[r][e] = col[r];
    }
}
__device__ inline uint32_t wide_lane_xor1(uint32_t x) {         // value held by lane ^ 1
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, true);
}

// Encode, last pass (see k_enc_hi_last): index bits p .. p+2, quantization, sum_i u_i q_i, packing.
__global__ __launch_bounds__(256) void k_enc_wide_last(EncBatch B, uint64_t valid_elems, int log2D, const float *T,
                                                       double *partials, uint32_t partial_stride,
                                                       const EncScratch *scratch) {
    __shared__ double red[4];
    const uint32_t c = blockIdx.y;
    const uint32_t lane = lane_id();
    const int p = log2D - 3;
    const uint32_t tile = blockIdx.x * 4u + wave_in_block();     // 2^(p-9) column blocks, all 8 rows
    const uint32_t base = tile * (uint32_t)kWideCols;
    const rsrc_t rt = make_rsrc(T + ((size_t)c << log2D), (uint32_t)(valid_elems * 4));
    float v[kWideRows][8];
#pragma unroll
    for (int r = 0; r < kWideRows; ++r) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const u32x4_t q = __builtin_amdgcn_raw_buffer_load_b128(rt, (int)(lane * 16u),
                                                                     (int)((base + 256u * h + ((uint32_t)r << p)) * 4u), kStream);
            v[r][4 * h] = __uint_as_float(q.x); v[r][4 * h + 1] = __uint_as_float(q.y);
            v[r][4 * h + 2] = __uint_as_float(q.z); v[r][4 * h + 3] = __uint_as_float(q.w);
        }
    }
    wide_fwht(v);
    char *payload = static_cast<char *>(B.msg[c]) + EDEN_HEADER_BYTES;
    const uint32_t b_q8 = B.b_q8[c];
    const EncScratch *sc = &scratch[c];
    __shared__ float qtabs[4][16];
    __shared__ float gtabs[4][256];                              // one-byte budgets: centroids and thresholds
    float *qtab = qtabs[wave_in_block()], *gtab = gtabs[wave_in_block()];
    fill_qtab(qtab, sc, lane);
    const float *byte_tab = sc->grid_c;                          // grid_c[128] and wide_thr[128] are one run of 256 floats
    if (byte_budget(b_q8)) {
#pragma unroll
        for (int q = 0; q < 4; ++q) gtab[64 * q + lane] = byte_tab[64 * q + lane];
    }
    wave_lds_sync();
    float ip = 0.0f;
    // the choice of the budget sits outside the loops over the 16 groups (group = this lane's 4 coordinates of a row half)
    auto for_groups = [&](auto &&pack) {
#pragma unroll
        for (int r = 0; r < kWideRows; ++r)
#pragma unroll
            for (int h = 0; h < 2; ++h) pack((base + 256u * h + ((uint32_t)r << p)) / 4u + lane, r, h);
    };
    if (b_q8 == 256u) {                                          // I_1: the index is the sign, |Q| = q_1
        for_groups([&](uint32_t group, int r, int h) {
            float sa = 0.0f;
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                sa += fabsf(v[r][4 * h + e]);
                word |= ((~__float_as_uint(v[r][4 * h + e])) >> 31) << e;            // index 1 = non-negative
            }
            ip = fmaf(sa, kQ1, ip);
            word |= wide_lane_xor1(word) << 4;                   // two lanes = one byte
            if (!(lane & 1u)) reinterpret_cast<uint8_t *>(payload)[group >> 1] = (uint8_t)word;
        });
    } else if (b_q8 == 512u) {
        for_groups([&](uint32_t group, int r, int h) {
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) word |= quantize_one<2>(v[r][4 * h + e], sc, qtab, ip) << (2 * e);
            reinterpret_cast<uint8_t *>(payload)[group] = (uint8_t)word;
        });
    } else if (grid_q15(b_q8)) {                                  // uniform grid: one byte per coordinate
        const float inv = sc->grid_inv;
        for_groups([&](uint32_t group, int r, int h) {
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) word |= quantize_byte<true>(v[r][4 * h + e], 0u, inv, gtab, ip) << (8 * e);
            reinterpret_cast<uint32_t *>(payload)[group] = word;
        });
    } else if (wide_bits(b_q8)) {                                 // b = 5..8: one byte per coordinate
        const uint32_t H = wide_half_levels(b_q8);
        uint32_t *dst = reinterpret_cast<uint32_t *>(B.codes[c] ? reinterpret_cast<char *>(B.codes[c]) : payload);
        for_groups([&](uint32_t group, int r, int h) {
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) word |= quantize_byte<false>(v[r][4 * h + e], H, 0.0f, gtab, ip) << (8 * e);
            dst[group] = word;
        });
    } else {
        for_groups([&](uint32_t group, int r, int h) {
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) word |= quantize_one<8>(v[r][4 * h + e], sc, qtab, ip) << (4 * e);
            reinterpret_cast<uint16_t *>(payload)[group] = (uint16_t)word;
        });
    }
    const double block_total = block_sum<256>((double)ip, red);
    if (threadIdx.x == 0) partials[(size_t)c * partial_stride + blockIdx.x] = block_total;
}

// Decode, first pass (see k_dec_hi_first): unpack, dequantize, zero the rows whose packet was lost, index bits
// p .. p+2.  A row segment of 512 coordinates lies inside one packet of 1024.
__global__ __launch_bounds__(256) void k_dec_wide_first(DecBatch B, uint64_t keep_elems, int log2D, const DecScratch *scratch,
                                                        float *T) {
    __shared__ float table[4][16];
    const uint32_t c = blockIdx.y;
    const uint32_t lane = lane_id(), wv = wave_in_block();
    const int p = log2D - 3;
    const uint32_t tile = blockIdx.x * 4u + wv;
    const uint32_t base = tile * (uint32_t)kWideCols;
    __shared__ float gtabs[4][kGridMax + 1];
    const uint32_t b_q8 = B.b_q8[c];
    if (lane < 16) table[wv][lane] = scratch[c].deq[lane];
    if (byte_budget(b_q8)) { gtabs[wv][lane] = scratch[c].grid_deq[lane]; gtabs[wv][64 + lane] = scratch[c].grid_deq[64 + lane]; }
    wave_lds_sync();
    const float *tb = table[wv];
    const char *payload = static_cast<const char *>(B.msg[c]) + EDEN_HEADER_BYTES;
    const char *bytes = B.codes[c] ? reinterpret_cast<const char *>(B.codes[c]) : payload;
    const uint32_t *bm = B.bitmap[c];
    // which of the 8 rows arrived (wave-uniform), then all payload loads, then the table look-ups: the choice of the
    // budget sits outside the loops so that the loads are issued back to back
    uint32_t here = 0xFFu;
    if (bm) {
        here = 0;
#pragma unroll
        for (int r = 0; r < kWideRows; ++r) {
            const uint32_t pk = (base + ((uint32_t)r << p)) >> 10;
            here |= ((bm[pk >> 5] >> (pk & 31u)) & 1u) << r;
        }
    }
    float v[kWideRows][8];
    uint32_t word[kWideRows][2];
    auto for_groups = [&](auto &&fetch) {                        // group = this lane's 4 coordinates of (row, half)
#pragma unroll
        for (int r = 0; r < kWideRows; ++r)
#pragma unroll
            for (int h = 0; h < 2; ++h) word[r][h] = fetch((base + ((uint32_t)r << p) + 256u * h) / 4u + lane);
    };
    auto for_values = [&](auto &&value) {
#pragma unroll
        for (int r = 0; r < kWideRows; ++r)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int e = 0; e < 4; ++e) v[r][4 * h + e] = ((here >> r) & 1u) ? value(word[r][h], e) : 0.0f;
    };
    const float *gt = gtabs[wv];
    if (b_q8 == 256u) {
        for_groups([&](uint32_t g) { return (uint32_t)reinterpret_cast<const uint8_t *>(payload)[g >> 1] >> (4u * (lane & 1u)); });
        for_values([&](uint32_t w, int e) { return tb[(w >> e) & 1u]; });
    } else if (b_q8 == 512u) {
        for_groups([&](uint32_t g) { return (uint32_t)reinterpret_cast<const uint8_t *>(payload)[g]; });
        for_values([&](uint32_t w, int e) { return tb[(w >> (2 * e)) & 3u]; });
    } else if (grid_q15(b_q8)) {
        for_groups([&](uint32_t g) { return reinterpret_cast<const uint32_t *>(bytes)[g]; });
        for_values([&](uint32_t w, int e) { return dequantize_byte<true>((w >> (8 * e)) & 0xFFu, 0u, gt); });
    } else if (wide_bits(b_q8)) {
        const uint32_t H = wide_half_levels(b_q8);
        for_groups([&](uint32_t g) { return reinterpret_cast<const uint32_t *>(bytes)[g]; });
        for_values([&](uint32_t w, int e) { return dequantize_byte<false>((w >> (8 * e)) & 0xFFu, H, gt); });
    } else {
        for_groups([&](uint32_t g) { return (uint32_t)reinterpret_cast<const uint16_t *>(payload)[g]; });
        for_values([&](uint32_t w, int e) { return tb[(w >> (4 * e)) & 15u]; });
    }
    wide_fwht(v);
    const rsrc_t rt = make_rsrc(T + ((size_t)c << log2D), (uint32_t)(keep_elems * 4));
#pragma unroll
    for (int r = 0; r < kWideRows; ++r) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            u32x4_t q = {__float_as_uint(v[r][4 * h]), __float_as_uint(v[r][4 * h + 1]), __float_as_uint(v[r][4 * h + 2]),
                         __float_as_uint(v[r][4 * h + 3])};
            // (no scalar offset on a store of more than 64 bits: see the note in k_dec_hix_first_mfma)
            __builtin_amdgcn_raw_buffer_store_b128(q, rt, (int)(lane * 16u + (base + 256u * h + ((uint32_t)r << p)) * 4u), 0, kStream);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Encode, first pass in wave tiles: x -> T.  Zero padding (Sec. 5: the transform needs a power of two), the
// sign diagonal of the rotation from the shared seed (Sec. 2.1), |x|^2 for eta and S (Sec. 2.2.1, 2.3), index
// bits 0..11 of H.  Only the ceil(d / 4096) tiles that hold part of x are transformed and written; the strided
// pass that follows reads the others as zero through its buffer bounds.  Loads and stores are both in the
// layout "register j = coordinates 64 j + lane" (256 contiguous bytes per wave access), so the tile goes
// through the wave-private 64x64 LDS transpose twice.
// `pre` (b = 1/2 with the sparsification first, Sec. 4.1): the vector that is transformed is
// x'[g] = 2 x[2g + o_g], g < ceil(d_src/2), o_g from the SUB-SAMPLING stream; x is read as 0 beyond d_src.
__global__ __launch_bounds__(128) void k_enc_lo_first(EncBatch B, uint64_t d_src, int pre, int log2D, uint64_t seed, float *T,
                                                      double *partials, uint32_t partial_stride) {
    __shared__ float lds[2][64 * kLdsRow];
    __shared__ double red[2];
    const uint32_t c = blockIdx.y;
    const uint32_t lane = lane_id();
    const uint32_t wv = wave_in_block();
    const uint32_t tile = blockIdx.x * 2u + wv;
    const uint64_t tile_base = (uint64_t)tile << kLoBits;
    const uint64_t d = pre ? (d_src + 1) / 2 : d_src;            // dimension of the vector that is transformed
    double n2 = 0.0;
    if (tile_base < d) {                                         // wave-uniform; no block-wide barrier inside
        const rsrc_t rx = make_rsrc(B.x[c], (uint32_t)(d_src * 4));      // reads past d_src give the zero padding
        float v[64];
        if (pre) {
            // register j = 64 consecutive pairs = one word of offsets: lane l hashes the word of register l
            const uint64_t offs = hash_word(stream_key(seed, kStreamSubsample, B.client[c]), (tile_base >> 6) + lane);
#pragma unroll
            for (int j = 0; j < 64; ++j) {
                const uint32_t odd = __builtin_amdgcn_inverse_ballot_w64(wave_read64(offs, j)) ? 4u : 0u;
                v[j] = 2.0f * buf_load(rx, lane * 8u + odd, (uint32_t)tile_base * 8u + 512u * j);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 64; ++j) v[j] = buf_load(rx, lane * 4u, (uint32_t)tile_base * 4u + 256u * j);
        }
#pragma unroll
        for (int j = 0; j < 64; ++j) n2 += (double)v[j] * (double)v[j];
        // register j = 64 consecutive coordinates = one sign word: lane l hashes the word of register l,
        // register j reads it back as a lane mask
        const uint64_t mine = hash_word(stream_key(seed, kStreamSign, B.client[c]), (tile_base >> 6) + lane);
#pragma unroll
        for (int j = 0; j < 64; ++j) v[j] = negate_where(v[j], wave_read64(mine, j)) + 0.0f;   // + 0: no negative zeros
        fwht_regs<64>(v);                                        // index bits 6..11
        float *L = lds[wv];
#pragma unroll
        for (int j = 0; j < 64; ++j) L[j * kLdsRow + lane] = v[j];
        wave_lds_sync();
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const float4 t = *reinterpret_cast<const float4 *>(&L[lane * kLdsRow + 4 * q]);
            v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
        }
        fwht_regs<64>(v);                                        // index bits 0..5; lane holds 64 consecutive values
        wave_lds_sync();
#pragma unroll
        for (int q = 0; q < 16; ++q)
            *reinterpret_cast<float4 *>(&L[lane * kLdsRow + 4 * q]) = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
        wave_lds_sync();
        float *Tc = T + ((size_t)c << log2D) + tile_base + lane;
#pragma unroll
        for (int j = 0; j < 64; ++j) __builtin_nontemporal_store(L[j * kLdsRow + lane], Tc + 64 * j);
    }
    const double block_total = block_sum<128>(n2, red);
    if (threadIdx.x == 0) partials[(size_t)c * partial_stride + blockIdx.x] = block_total;
}

// One workgroup per sender: sums the partials of sum_i u_i q_i in index order, forms
// <R(x),Q> = D^-1/2 sum and the scale S = |x|^2 / <R(x),Q> (Sec. 2.3), writes the header.
// A zero or non-finite vector gets S = 0, a status bit and an all-zero payload.
__global__ __launch_bounds__(256) void k_enc_finish(EncBatch B, uint64_t hdr_d, int log2D, uint64_t seed,
                                                    const double *partials_n2, uint32_t nparts_n2,
                                                    const double *partials_ip, uint32_t nparts_ip,
                                                    uint32_t partial_stride, uint32_t payload_words_b1,
                                                    uint32_t *dev_status, const uint32_t *coin_total) {
    __shared__ double red[4];
    __shared__ double n2_shared;
    const uint32_t c = blockIdx.x;
    const double *pn = partials_n2 + (size_t)c * partial_stride;
    const double *pi = partials_ip + (size_t)c * partial_stride;
    double s = 0.0;
    for (uint32_t i = threadIdx.x; i < nparts_n2; i += 256) s += pn[i];
    const double n2_t0 = block_sum<256>(s, red);                  // |x|^2, same summation order as k_enc_norm
    s = 0.0;
    for (uint32_t i = threadIdx.x; i < nparts_ip; i += 256) s += pi[i];
    const double total = block_sum<256>(s, red);
    if (threadIdx.x == 0) n2_shared = n2_t0;
    __syncthreads();
    const double n2 = n2_shared;
    __shared__ double ip_shared;
    if (threadIdx.x == 0) ip_shared = total;
    __syncthreads();
    // <R(x),Q> = 0 can only happen on a uniform grid so coarse that every coordinate falls into the interval around 0
    const bool valid = (n2 > 0.0) && (n2 < INFINITY) && (ip_shared > 0.0);
    const uint32_t b_q8 = B.b_q8[c];
    if (!valid) {
        uint32_t *payload = reinterpret_cast<uint32_t *>(static_cast<char *>(B.msg[c]) + EDEN_HEADER_BYTES);
        int bits, k;
        budget_of(b_q8, bits, k);
        const uint64_t D = 32ull * payload_words_b1;
        const uint64_t nw = (payload_a_bytes(D, bits, k) + (coin_q8(b_q8) ? coin_b_bytes(coin_total[c]) : payload_b_bytes(D, b_q8))) / 4;
        for (uint64_t i = threadIdx.x; i < nw; i += 256) payload[i] = 0u;
    }
    if (threadIdx.x == 0) {
        MsgHeader h;
        h.magic = kMagic; h.log2D = (uint32_t)log2D; h.d = hdr_d; h.b_q8 = B.hdr_b_q8[c]; h.client = B.client[c];
        h.extra_bits = coin_q8(b_q8) ? coin_total[c] : 0u; h.seed = seed; h.N2 = n2;
        if (valid) {
            h.IP = total * exp2(-0.5 * (double)log2D);       // <R(x),Q> = D^-1/2 sum u_i q_i
            h.S = n2 / h.IP;                                  // Sec. 2.3
            h.status = 0;
        } else {
            h.IP = 0.0; h.S = 0.0;
            h.status = (n2 >= 0.0 && n2 < INFINITY) ? EDEN_DEV_ZERO_VECTOR : EDEN_DEV_NONFINITE;
            atomicOr(dev_status, h.status);
        }
        *static_cast<MsgHeader *>(B.msg[c]) = h;
    }
}

// ------------------------------------------------------------------------------------------------
// decode side
//
__global__ __launch_bounds__(64) void k_dec_prepare(DecBatch B, uint64_t hdr_d, int log2D, uint64_t seed,
                                                    const DevTables *tab, DecScratch *scratch, uint32_t *dev_status,
                                                    const uint32_t *coin_total, uint32_t *msg_flags) {
    const uint32_t c = blockIdx.x;
    dec_prepare_wave(B.msg[c], B.bitmap[c], B.client[c], B.b_q8[c], B.hdr_b_q8[c], hdr_d, log2D, seed, tab, &scratch[c], dev_status,
                     coin_q8(B.b_q8[c]) ? coin_total[c] : 0u, msg_flags ? msg_flags + c : nullptr);
}

// ---- coin budgets (Sec. 4.1): the coins of every sender of a launch that has such a budget, as lane masks per block of 64
// coordinates, with the prefix sums that give every block its place in the second part of the payload.  Both sides run
// this from the shared seed alone.  One thread per block of 64 coordinates (8 hash words of 8 coins each).
struct CoinBatch {
    uint32_t client[kMaxBatch];
    uint32_t b_q8[kMaxBatch];
    void *part_b[kMaxBatch];             // encode: the second part of the sender's payload, cleared here; decode: null
};
__device__ inline uint32_t block_exclusive_scan_256(uint32_t mine, uint32_t *wave_totals /* shared, 4 */, uint32_t &block_total) {
    const uint32_t lane = lane_id(), wv = threadIdx.x >> 6;
    uint32_t incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t v = (uint32_t)__shfl_up((int)incl, o, 64);
        if (lane >= (uint32_t)o) incl += v;
    }
    if (lane == 63) wave_totals[wv] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (uint32_t i = 0; i < 4; ++i) { before += i < wv ? wave_totals[i] : 0u; all += wave_totals[i]; }
    __syncthreads();
    block_total = all;
    return before + incl - mine;
}
__global__ __launch_bounds__(256) void k_coin_masks(CoinBatch B, uint64_t seed, int log2D, CoinTables ct) {
    __shared__ uint32_t wave_totals[4];
    const uint32_t c = blockIdx.y;
    const uint32_t frac = coin_q8(B.b_q8[c]) & 255u;
    if (!frac) return;                                           // not a coin budget: the whole workgroup leaves
    const uint32_t words = 1u << (log2D - 6);
    const uint32_t w = blockIdx.x * (uint32_t)kCoinGroup + threadIdx.x;
    uint64_t m = 0;
    if (w < words) {
        const uint64_t key = stream_key(seed, kStreamMix, B.client[c]);
#pragma unroll
        for (uint32_t j = 0; j < 8; ++j) {
            const uint64_t h = hash_word(key, 8ull * w + j);
#pragma unroll
            for (uint32_t b = 0; b < 8; ++b)
                if (((uint32_t)(h >> (8u * b)) & 0xFFu) < frac) m |= 1ull << (8u * j + b);
        }
    }
    uint32_t group_total;
    const uint32_t before = block_exclusive_scan_256((uint32_t)__popcll(m), wave_totals, group_total);
    if (w < words) {
        ct.mask[((size_t)c << (log2D - 6)) + w] = m;
        ct.local[((size_t)c << (log2D - 6)) + w] = before;
        if (B.part_b[c]) static_cast<uint64_t *>(B.part_b[c])[w] = 0ull;
    }
    if (threadIdx.x == 0) ct.group[(size_t)c * ct.group_stride + blockIdx.x] = group_total;
}
// One workgroup per sender: the group totals become the number of coins before each group, and the grand total.
__global__ __launch_bounds__(256) void k_coin_scan(CoinBatch B, int log2D, CoinTables ct) {
    __shared__ uint32_t wave_totals[4];
    const uint32_t c = blockIdx.x;
    if (!coin_q8(B.b_q8[c])) return;
    const uint32_t words = 1u << (log2D - 6);
    const uint32_t groups = (words + (uint32_t)kCoinGroup - 1) / (uint32_t)kCoinGroup;
    const uint32_t per = (groups + 255u) / 256u;
    uint32_t *g = ct.group + (size_t)c * ct.group_stride;
    const uint32_t first = threadIdx.x * per;
    uint32_t mine = 0;
    for (uint32_t i = first; i < first + per && i < groups; ++i) mine += g[i];
    uint32_t all;
    uint32_t run = block_exclusive_scan_256(mine, wave_totals, all);
    for (uint32_t i = first; i < first + per && i < groups; ++i) {
        const uint32_t v = g[i];
        g[i] = run;
        run += v;
    }
    if (threadIdx.x == 0) ct.total[c] = all;
}

// Coin budgets, encoder in workgroup tiles: the last pass leaves, for every segment of 32 consecutive coordinates, the top
// bits of its coins moved together towards bit 0, one word per segment, in `pieces` (bits above the segment's number of
// coins are 0).  This kernel strings them together into the second part of the payload (Sec. 4.1: one more bit for every
// coordinate with a coin, in coordinate order).  A thread looks after one block of 64 coordinates; if one of the part's 64-bit
// words begins inside the block's run of bits, the thread assembles that word from its own pieces and those of the blocks
// after it.  Every word is written by exactly one thread: no atomics (they cost the last encode pass a third of its time).
struct CoinPackBatch {
    uint32_t b_q8[kMaxBatch];
    const uint32_t *pieces[kMaxBatch];   // null: the sender's bits were placed by the last pass itself
    uint64_t *part_b[kMaxBatch];
};
__global__ __launch_bounds__(256) void k_coin_pack(CoinPackBatch B, int log2D, CoinTables ct) {
    const uint32_t c = blockIdx.y;
    const uint32_t *pieces = B.pieces[c];
    if (!coin_q8(B.b_q8[c]) || !pieces) return;
    const uint32_t blocks = 1u << (log2D - 6);
    const uint32_t k = blockIdx.x * 256u + threadIdx.x;
    if (k >= blocks) return;
    const uint64_t mine = coin_mask_of(ct, c, log2D, k);
    const uint32_t count = (uint32_t)__popcll(mine);
    const uint32_t start = coins_before(ct, c, log2D, k);       // this block's bits are [start, start + count) of the part
    const uint32_t word = (start + 63u) >> 6;                    // the first word that begins at or after `start`
    if ((uint64_t)word * 64u >= (uint64_t)start + count) return; // none begins inside this block's run
    uint32_t skip = word * 64u - start;                          // bits of this block that belong to the word before
    uint64_t bits = 0;
    uint32_t have = 0;
    for (uint32_t kk = k; have < 64u && kk < blocks; ++kk) {
        const uint64_t m = kk == k ? mine : coin_mask_of(ct, c, log2D, kk);
        const uint32_t lo = (uint32_t)__popc(lo32(m));
        uint32_t n = lo + (uint32_t)__popc(hi32(m));
        if (n == 0u) continue;
        uint64_t run = (uint64_t)pieces[2u * kk] | ((uint64_t)pieces[2u * kk + 1u] << lo);
        run >>= skip;                                            // (only the first block has bits to skip, fewer than it holds)
        n -= skip;
        skip = 0;
        bits |= run << have;
        have += n;
    }
    B.part_b[c][word] = bits;
}

// Decode, last pass in wave tiles: index bits 0..11 of H for every sender, that sender's sign diagonal
// (R^-1 = s o D^-1/2 H, Sec. 2.2.2; D^-1/2 is inside the dequantization scale), sum over senders in registers,
// one contiguous read-modify-write of acc.  A lane ends with 64 consecutive coordinates = one sign word.
// `pre` (b = 1/2 with the sparsification first, Sec. 4.1): the decoded vector has dimension ceil(d_src/2) and value g
// of sender c belongs at coordinate 2g + o_g of acc (o_g from c's SUB-SAMPLING stream); since the places differ from
// sender to sender, every sender's values are added to acc directly.
// pre == 2: nothing is summed; every sender's decoded vector is written back into its own workspace slot (fp32, in
// place: a wave has read its tile before it writes it), for a caller that puts the values elsewhere afterwards.
__global__ __launch_bounds__(128) void k_dec_lo_last(DecBatch B, uint32_t n, uint64_t d_src, int pre, int log2D, uint64_t seed,
                                                     float *T, const DecScratch *scratch, int narrow, float *acc) {
    __shared__ float lds[2][64 * kLdsRow];
    const uint32_t lane = lane_id(), wv = wave_in_block();
    const uint32_t tile = blockIdx.x * 2u + wv;
    const uint64_t tile_base = (uint64_t)tile << kLoBits;
    const uint64_t d = pre == 1 ? (d_src + 1) / 2 : d_src;       // dimension of the decoded vector
    if (tile_base >= d) return;                                  // whole tile in the padding (no block-wide barrier below)
    const uint64_t first = tile_base + 64u * lane;               // this lane's 64 coordinates after the transpose
    float *L = lds[wv];
    float sum[64];
#pragma unroll
    for (int k = 0; k < 64; ++k) sum[k] = 0.0f;
    for (uint32_t c = 0; c < n; ++c) {
        const bool i16 = narrow && B.b_q8[c] <= 256u;
        float v[64];
        if (i16) {
            const short *t16 = reinterpret_cast<const short *>(T + ((size_t)c << log2D)) + tile_base + lane;
#pragma unroll
            for (int j = 0; j < 64; ++j) v[j] = narrow_value(__builtin_nontemporal_load(t16 + 64 * j));
        } else {
            const float *t32 = T + ((size_t)c << log2D) + tile_base + lane;
#pragma unroll
            for (int j = 0; j < 64; ++j) v[j] = __builtin_nontemporal_load(t32 + 64 * j);
        }
        fwht_regs<64>(v);                                        // index bits 6..11
#pragma unroll
        for (int j = 0; j < 64; ++j) L[j * kLdsRow + lane] = v[j];
        wave_lds_sync();
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const float4 t = *reinterpret_cast<const float4 *>(&L[lane * kLdsRow + 4 * q]);
            v[4 * q] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
        }
        wave_lds_sync();                                         // the next sender overwrites the rows
        fwht_regs<64>(v);                                        // index bits 0..5
        const uint32_t scale = __float_as_uint(i16 ? scratch[c].deq[1] : 1.0f) & 0x7FFFFFFFu;   // > 0; x*1+s is exact
        const uint64_t word = hash_word(stream_key(seed, kStreamSign, B.client[c]), first >> 6);
        const uint32_t wlo = (uint32_t)word, whi = (uint32_t)(word >> 32);
        if (pre == 2) {
            float *dst = T + ((size_t)c << log2D) + first;
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                float o4[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = 4 * q + e;
                    const uint32_t sbit = ((k < 32 ? wlo : whi) << (31 - (k & 31))) & 0x80000000u;
                    o4[e] = v[k] * __uint_as_float(scale | sbit);
                }
                *reinterpret_cast<float4 *>(dst + 4 * q) = make_float4(o4[0], o4[1], o4[2], o4[3]);
            }
            continue;
        }
        if (pre) {
            const uint64_t offs = hash_word(stream_key(seed, kStreamSubsample, B.client[c]), first >> 6);
#pragma unroll
            for (int k = 0; k < 64; ++k) {
                const uint32_t sbit = ((k < 32 ? wlo : whi) << (31 - (k & 31))) & 0x80000000u;
                const uint64_t pos = 2 * (first + k) + ((offs >> k) & 1ull);
                if (first + k < d && pos < d_src) acc[pos] = fmaf(v[k], __uint_as_float(scale | sbit), acc[pos]);
            }
            continue;
        }
#pragma unroll
        for (int k = 0; k < 32; ++k)
            sum[k] = fmaf(v[k], __uint_as_float(scale | ((wlo << (31 - k)) & 0x80000000u)), sum[k]);   // bit 1 -> s_i = -1
#pragma unroll
        for (int k = 0; k < 32; ++k)
            sum[32 + k] = fmaf(v[32 + k], __uint_as_float(scale | ((whi << (31 - k)) & 0x80000000u)), sum[32 + k]);
    }
    if (pre) return;
    if (first + 64 <= d) {
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            float4 a = *reinterpret_cast<const float4 *>(acc + first + 4 * q);
            a.x += sum[4 * q]; a.y += sum[4 * q + 1]; a.z += sum[4 * q + 2]; a.w += sum[4 * q + 3];
            *reinterpret_cast<float4 *>(acc + first + 4 * q) = a;
        }
    } else {
#pragma unroll
        for (int k = 0; k < 64; ++k)
            if (first + k < d) acc[first + k] += sum[k];
    }
}

typedef float f32x4 __attribute__((ext_vector_type(4)));
// Sec. 2.2.2: the plain average.  Four coordinates per thread when both pointers are 16-byte aligned.
__global__ void k_finalize_mean(const float *acc, uint64_t d, float n, float *mean, int vec) {
    const uint64_t i = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) * (vec ? 4u : 1u);
    if (vec && i + 3 < d) {
        f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(acc + i));
        a.x /= n; a.y /= n; a.z /= n; a.w /= n;
        *reinterpret_cast<f32x4 *>(mean + i) = a;
    } else {
        for (uint64_t e = i; e < d && e < i + (vec ? 4u : 1u); ++e) mean[e] = acc[e] / n;
    }
}

// ---- b = m/64: sparsification before the rotation with p = m/64 (Sec. 4.1).  Of every block of 64 consecutive
// coordinates the m with the smallest (key, position) pairs are kept, the 16-bit key of coordinate i being bits
// 16 (i & 3) .. +15 of word i >> 2 of the SPARSE stream; a kept coordinate's slot is block * m + its rank among the
// kept ones in position order.
// A wave takes four blocks: lane 16 r + l holds the four pairs of coordinates 64 block_r + 4 l .. + 3 (one word of the
// stream).  The 64 pairs of a block are sorted by a bitonic network over (lane, register): register pairs inside the
// lane, lanes through the cross-lane swizzle; the pair of rank m is the threshold.  The pairs travel as floats in
// [1, 2) (22 bits in the mantissa: the same order), so that one median instruction is "the smaller" (third operand 0),
// "the larger" (4) or "whichever this lane's side of the exchange keeps".
template <int X>
__device__ inline float lane_xor(float v) {          // the value of lane (l ^ X), X < 32
    return __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), 0x001F | (X << 10)));
}
__device__ inline void order2(float &a, float &b) {
    const float lo = __builtin_amdgcn_fmed3f(a, b, 0.0f), hi = __builtin_amdgcn_fmed3f(a, b, 4.0f);
    a = lo; b = hi;
}
// exchange with lane l ^ X (register 3 - e instead of e when FLIP); `side` is 0 in the lane that keeps the smaller
template <int X, bool FLIP>
__device__ inline void exchange(float (&v)[4], float side) {
    float p[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) p[e] = lane_xor<X>(v[FLIP ? 3 - e : e]);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = __builtin_amdgcn_fmed3f(v[e], p[e], side);
}
__device__ inline void order_in_lane(float (&v)[4]) {     // distances 2 and 1 of a merge
    order2(v[0], v[2]); order2(v[1], v[3]); order2(v[0], v[1]); order2(v[2], v[3]);
}
template <int N> __device__ inline uint32_t row_shr(uint32_t v) {     // lane l - N of the row of 16, 0 below the row
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x110 | N, 0xF, 0xF, true);
}
// Bit e of the result: coordinate 64 block + 4 (lane & 15) + e is kept; slot0: the slot in the block of this lane's
// first kept coordinate (the others follow).  Every lane of the wave must call it (cross-lane exchanges).  Block
// numbers and coordinates fit 32 bits (d <= 2^EDEN_MAX_LOG2_D).
__device__ inline uint32_t sparse_kept4(uint64_t key, uint32_t block, uint32_t m, uint32_t lane, uint32_t &slot0) {
    const uint32_t l = lane & 15u;
    const uint64_t word = hash_word(key, (uint64_t)(block * 16u + l));
    const uint32_t half[2] = {(uint32_t)word, (uint32_t)(word >> 32)};
    float v[4], mine[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const uint32_t k16 = (e & 1) ? (half[e >> 1] >> 16) : (half[e >> 1] & 0xFFFFu);
        v[e] = mine[e] = __uint_as_float((0x3F800000u + (uint32_t)e + 4u * l) | (k16 << 6));     // all 64 different
    }
    float side[4];                                       // lane bit b set: the upper partner at lane distance 2^b
#pragma unroll
    for (int b = 0; b < 4; ++b) side[b] = ((l >> b) & 1u) ? 4.0f : 0.0f;
    // merges of 2, 4, ..., 64: the first step of a merge pairs position g with g ^ (size - 1), the others g ^ distance
    order2(v[0], v[1]); order2(v[2], v[3]);
    order2(v[0], v[3]); order2(v[1], v[2]); order2(v[0], v[1]); order2(v[2], v[3]);
    exchange<1, true>(v, side[0]); order_in_lane(v);
    exchange<3, true>(v, side[1]); exchange<1, false>(v, side[0]); order_in_lane(v);
    exchange<7, true>(v, side[2]); exchange<2, false>(v, side[1]); exchange<1, false>(v, side[0]); order_in_lane(v);
    exchange<15, true>(v, side[3]); exchange<4, false>(v, side[2]); exchange<2, false>(v, side[1]);
    exchange<1, false>(v, side[0]); order_in_lane(v);
    // the pair of rank m (0-based) sits in register m & 3 of lane m >> 2 of the row; the m pairs below it are kept
    const float at = (m & 2u) ? ((m & 1u) ? v[3] : v[2]) : ((m & 1u) ? v[1] : v[0]);
    const float t = __shfl(at, (int)((lane & 48u) | (m >> 2)));
    uint32_t kept = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) kept |= (mine[e] < t ? 1u : 0u) << e;
    const uint32_t cnt = (uint32_t)__popc(kept);
    uint32_t incl = cnt;
    incl += row_shr<1>(incl); incl += row_shr<2>(incl); incl += row_shr<4>(incl); incl += row_shr<8>(incl);
    slot0 = incl - cnt;
    return kept;
}
__device__ inline uint32_t sparse_block_of_lane(uint32_t lane) {
    return ((blockIdx.x * 4u + wave_in_block()) << 2) + (lane >> 4);
}
// the four coordinates of a lane: one 16-byte load when `vec` (pointer aligned) and all four are below d, else 0-padded
__device__ inline void load4_padded(const float *x, uint32_t i, uint32_t d, bool vec, float (&v)[4]) {
    if (vec && i + 3 < d) {
        const float4 q = *reinterpret_cast<const float4 *>(x + i);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (i + e < d) ? x[i + e] : 0.0f;
    }
}
// stage[block m + slot] = x[i] for the kept coordinates (0 for a kept position beyond d)
__global__ __launch_bounds__(256) void k_sparse_gather(const float *x, uint32_t d, uint32_t m, uint64_t key, float *stage) {
    const uint32_t lane = lane_id();
    const uint32_t block = sparse_block_of_lane(lane);
    uint32_t slot;
    const uint32_t kept = sparse_kept4(key, block, m, lane, slot);
    if (block * 64u >= d) return;
    float v[4];
    load4_padded(x, block * 64u + 4u * (lane & 15u), d, (reinterpret_cast<uintptr_t>(x) & 15u) == 0, v);
    slot += block * m;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if ((kept >> e) & 1u) stage[slot++] = v[e];
}
// acc[i] += stage[block m + slot] for the kept coordinates below d (the factor 64/m is already in the values)
__global__ __launch_bounds__(256) void k_sparse_scatter(const float *stage, uint32_t d, uint32_t m, uint64_t key, float *acc) {
    const uint32_t lane = lane_id();
    const uint32_t block = sparse_block_of_lane(lane);
    uint32_t slot;
    const uint32_t kept = sparse_kept4(key, block, m, lane, slot);
    if (block * 64u >= d) return;
    const uint32_t i = block * 64u + 4u * (lane & 15u);
    slot += block * m;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if ((kept >> e) & 1u) {
            const float s = stage[slot++];
            if (i + e < d) acc[i + e] += s;
        }
}
// The same for a batch of senders that share m: sender blockIdx.y gathers into its workspace slot, and the scatter
// adds, coordinate by coordinate, the values of all senders whose selection holds the coordinate.
__global__ __launch_bounds__(256) void k_sparse_gather_batch(EncBatch B, uint32_t d, uint32_t m, uint64_t seed, float *T,
                                                             int log2Dk) {
    const uint32_t lane = lane_id(), c = blockIdx.y;
    const uint32_t block = sparse_block_of_lane(lane);
    uint32_t slot;
    const uint32_t kept = sparse_kept4(stream_key(seed, kStreamSparse, B.client[c]), block, m, lane, slot);
    if (block * 64u >= d) return;
    const float *x = B.x[c];
    float v[4];
    load4_padded(x, block * 64u + 4u * (lane & 15u), d, (reinterpret_cast<uintptr_t>(x) & 15u) == 0, v);
    float *out = T + ((size_t)c << log2Dk);
    slot += block * m;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if ((kept >> e) & 1u) out[slot++] = v[e];
}
__global__ __launch_bounds__(256) void k_sparse_scatter_batch(DecBatch B, uint32_t n, uint32_t d, uint32_t m, uint64_t seed,
                                                              const float *T, int log2Dk, float *acc) {
    const uint32_t lane = lane_id();
    const uint32_t block = sparse_block_of_lane(lane);
    if ((block & ~3u) * 64u >= d) return;                // the whole wave is beyond d
    float sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const bool inside = block * 64u < d;
    for (uint32_t c = 0; c < n; ++c) {
        uint32_t slot;
        const uint32_t kept = sparse_kept4(stream_key(seed, kStreamSparse, B.client[c]), block, m, lane, slot);
        const float *in = T + ((size_t)c << log2Dk);
        slot += block * m;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (inside && ((kept >> e) & 1u)) sum[e] += in[slot++];
    }
    if (!inside) return;
    const uint32_t i = block * 64u + 4u * (lane & 15u);
    if ((reinterpret_cast<uintptr_t>(acc) & 15u) == 0 && i + 3 < d) {
        float4 a = *reinterpret_cast<float4 *>(acc + i);
        a.x += sum[0]; a.y += sum[1]; a.z += sum[2]; a.w += sum[3];
        *reinterpret_cast<float4 *>(acc + i) = a;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (i + e < d) acc[i + e] += sum[e];
    }
}
// b = 5, 6, 7: the one-byte indices of a sender, in coordinate order, to the payload's bit string (index j in bits
// j b .. j b + b - 1, Sec. 2.2.1 message) and back.  A thread handles 32 indices = 32 bytes = b payload words.
template <int BITS>
__device__ inline void pack32(const uint8_t *codes, uint32_t *words) {
    uint32_t in[8];
    const uint4 lo = reinterpret_cast<const uint4 *>(codes)[0], hi = reinterpret_cast<const uint4 *>(codes)[1];
    in[0] = lo.x; in[1] = lo.y; in[2] = lo.z; in[3] = lo.w; in[4] = hi.x; in[5] = hi.y; in[6] = hi.z; in[7] = hi.w;
    uint32_t out[BITS];
#pragma unroll
    for (int w = 0; w < BITS; ++w) out[w] = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const uint32_t code = (in[j >> 2] >> (8 * (j & 3))) & ((1u << BITS) - 1u);
        const int pos = j * BITS;
        out[pos >> 5] |= code << (pos & 31);
        if ((pos & 31) + BITS > 32) out[(pos >> 5) + 1] |= code >> (32 - (pos & 31));
    }
#pragma unroll
    for (int w = 0; w < BITS; ++w) words[w] = out[w];
}
template <int BITS>
__device__ inline void unpack32(const uint32_t *words, uint8_t *codes) {
    uint32_t in[BITS + 1];
#pragma unroll
    for (int w = 0; w < BITS; ++w) in[w] = words[w];
    in[BITS] = 0;
    uint32_t out[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) out[q] = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const int pos = j * BITS;
        const uint32_t code = code_at(in[pos >> 5], in[(pos >> 5) + 1], (uint32_t)(pos & 31), BITS);
        out[j >> 2] |= code << (8 * (j & 3));
    }
    reinterpret_cast<uint4 *>(codes)[0] = make_uint4(out[0], out[1], out[2], out[3]);
    reinterpret_cast<uint4 *>(codes)[1] = make_uint4(out[4], out[5], out[6], out[7]);
}
__global__ __launch_bounds__(256) void k_pack_bits(EncBatch B, int log2D) {
    const uint32_t c = blockIdx.y;
    const uint8_t *codes = B.codes[c];
    const uint32_t bits = wide_bits(B.b_q8[c]);
    if (!codes || bits < 5u || bits > 7u) return;                // (a coin sender's buffer holds the pieces of its second part)
    const uint64_t g = (uint64_t)blockIdx.x * 256u + threadIdx.x;        // group of 32 indices
    if (g >= (1ull << log2D) / 32) return;
    uint32_t *payload = reinterpret_cast<uint32_t *>(static_cast<char *>(B.msg[c]) + EDEN_HEADER_BYTES) + g * bits;
    if (bits == 5) pack32<5>(codes + 32 * g, payload);
    else if (bits == 6) pack32<6>(codes + 32 * g, payload);
    else pack32<7>(codes + 32 * g, payload);
}
__global__ __launch_bounds__(256) void k_unpack_bits(DecBatch B, int log2D, uint8_t *codes_all) {
    const uint32_t c = blockIdx.y;
    if (!B.codes[c]) return;
    const uint64_t g = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (g >= (1ull << log2D) / 32) return;
    const uint32_t bits = wide_bits(B.b_q8[c]);
    const uint32_t *payload = reinterpret_cast<const uint32_t *>(static_cast<const char *>(B.msg[c]) + EDEN_HEADER_BYTES) + g * bits;
    uint8_t *codes = codes_all + ((size_t)c << log2D) + 32 * g;
    if (bits == 5) unpack32<5>(payload, codes);
    else if (bits == 6) unpack32<6>(payload, codes);
    else unpack32<7>(payload, codes);
}
__global__ __launch_bounds__(256) void k_fill_zero(float *p, uint64_t count) {
    const uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (i < count) p[i] = 0.0f;
}

// Experiment helper (Sec. 4.3): histogram of the one-byte indices of a uniform-grid message and its entropy
// -sum f log2 f in bits per coordinate, what an ideal entropy coder would spend.
__global__ __launch_bounds__(256) void k_byte_histogram(const uint8_t *bytes, uint64_t count, uint32_t *hist) {
    __shared__ uint32_t local[256];
    local[threadIdx.x] = 0;
    __syncthreads();
    for (uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x; i < count; i += (uint64_t)gridDim.x * 256u)
        atomicAdd(&local[bytes[i]], 1u);
    __syncthreads();
    if (local[threadIdx.x]) atomicAdd(&hist[threadIdx.x], local[threadIdx.x]);
}
__global__ __launch_bounds__(256) void k_histogram_entropy(const uint32_t *hist, uint64_t count, double *out) {
    __shared__ double red[4];
    const double f = (double)hist[threadIdx.x] / (double)count;
    const double h = block_sum<256>(f > 0.0 ? -f * log2(f) : 0.0, red);
    if (threadIdx.x == 0) out[0] = h;
}

// Experiment helper: sum_i (a_i - b_i)^2 and sum_i a_i^2 in double, the two terms of the (v)NMSE definitions
// (Sec. 2.1: NMSE; Sec. 2.3: vNMSE).  Per-workgroup partials, then one workgroup adds them in index order.
__global__ __launch_bounds__(256) void k_sq_error(const float *a, const float *b, uint64_t d, double *partials) {
    __shared__ double red[4];
    double e2 = 0.0, a2 = 0.0;
    for (uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x; i < d; i += (uint64_t)gridDim.x * 256u) {
        const double x = a[i], y = b[i];
        e2 += (x - y) * (x - y);
        a2 += x * x;
    }
    const double te = block_sum<256>(e2, red);
    const double ta = block_sum<256>(a2, red);
    if (threadIdx.x == 0) { partials[2 * blockIdx.x] = te; partials[2 * blockIdx.x + 1] = ta; }
}
__global__ __launch_bounds__(256) void k_sq_error_finish(const double *partials, uint32_t nparts, double *out) {
    __shared__ double red[4];
    double e2 = 0.0, a2 = 0.0;
    for (uint32_t i = threadIdx.x; i < nparts; i += 256) { e2 += partials[2 * i]; a2 += partials[2 * i + 1]; }
    const double te = block_sum<256>(e2, red);
    const double ta = block_sum<256>(a2, red);
    if (threadIdx.x == 0) { out[0] = te; out[1] = ta; }
}

// ------------------------------------------------------------------------------------------------
// D <= 4096: one workgroup per sender, the padded vector lives in LDS.
__device__ inline void fwht_lds(float *buf, uint32_t D) {
    for (uint32_t h = 1; h < D; h <<= 1) {
        __syncthreads();
        for (uint32_t pidx = threadIdx.x; pidx < D / 2; pidx += blockDim.x) {
            const uint32_t i = ((pidx & ~(h - 1)) << 1) | (pidx & (h - 1));
            const float a = buf[i], b = buf[i + h];
            buf[i] = a + b;
            buf[i + h] = a - b;
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(256) void k_enc_small(EncBatch B, uint64_t d, int pre, uint64_t hdr_d, int log2D, uint64_t seed,
                                                   const DevTables *tab, uint32_t *dev_status) {
    __shared__ float buf[kLoTile];
    __shared__ uint8_t code[kLoTile];
    __shared__ double red[4];
    __shared__ EncScratch s;
    __shared__ __attribute__((aligned(8))) uint32_t coin_words[kLoTile / 32];   // coin budgets: the second part of the payload
    __shared__ uint32_t wave_totals[4];
    const uint32_t c = blockIdx.x;
    const uint32_t D = 1u << log2D;
    const float *x = B.x[c];
    const uint64_t key = stream_key(seed, kStreamSign, B.client[c]);
    const uint64_t prekey = stream_key(seed, kStreamSubsample, B.client[c]);
    double n2p = 0.0;
    for (uint32_t i = threadIdx.x; i < D; i += 256) {
        float xi;
        if (pre) {                                             // Sec. 4.1: x'[i] = 2 x[2i + o_i], sparsification before the rotation
            const uint64_t src = 2ull * i + ((hash_word(prekey, i >> 6) >> (i & 63u)) & 1ull);
            xi = (src < d) ? 2.0f * x[src] : 0.0f;
        } else {
            xi = (i < d) ? x[i] : 0.0f;
        }
        n2p += (double)xi * (double)xi;
        const bool neg = (hash_word(key, i >> 6) >> (i & 63u)) & 1ull;
        buf[i] = (neg ? -xi : xi) + 0.0f;
    }
    const double n2t = block_sum<256>(n2p, red);
    const uint32_t b_q8 = B.b_q8[c];
    if (threadIdx.x == 0) fill_enc_scratch(&s, n2t, b_q8, tab);
    __syncthreads();
    fill_byte_tables(&s, b_q8, s.n2, tab, threadIdx.x);
    fwht_lds(buf, D);                                          // includes the barriers that publish `s`
    int bits, k;
    budget_of(b_q8, bits, k);
    const int H = 1 << (bits - 1);
    const double n2 = s.n2;
    float ip = 0.0f;
    const bool mix = budget_mixed(b_q8);                       // b = k + 1/2: one coordinate of every pair uses I_{k+1}
    const uint32_t coin_frac = coin_q8(b_q8) & 255u;           // coin budgets: a coordinate with a coin uses I_{k+1}
    const uint64_t mixkey = stream_key(seed, kStreamMix, B.client[c]);
    const bool bytes = byte_budget(b_q8);                      // uniform grid (Sec. 4.3) or b = 5..8: one-byte indices
    for (uint32_t i = threadIdx.x; i < D; i += 256) {
        const float u = buf[i];
        if (bytes) {                                           // grid_c and wide_thr are adjacent
            code[i] = (uint8_t)(grid_q15(b_q8) ? quantize_byte<true>(u, 0u, s.grid_inv, s.grid_c, ip)
                                               : quantize_byte<false>(u, wide_half_levels(b_q8), 0.0f, s.grid_c, ip));
            continue;
        }
        const float a = fabsf(u);
        const uint32_t g = i >> 1;
        const bool up = coin_frac ? coin_of(mixkey, i, coin_frac)
                                  : (mix && ((uint32_t)((hash_word(mixkey, g >> 6) >> (g & 63u)) & 1ull) == (i & 1u)));
        const float *thr = up ? s.thr2 : s.thr, *qp = up ? s.qpos2 : s.qpos;
        const int Hu = up ? 2 * H : H;
        uint32_t mag = 0;
        for (int t = 1; t < Hu; ++t) mag = (a > thr[t]) ? (uint32_t)t : mag;
        ip = fmaf(a, qp[mag], ip);
        const uint32_t neg = __float_as_uint(u) >> 31;
        code[i] = (uint8_t)(neg ? (uint32_t)(Hu - 1) - mag : (uint32_t)Hu + mag);
    }
    const double ipt_t0 = block_sum<256>((double)ip, red);     // barriers inside also publish `code`
    __shared__ double ip_shared;
    if (threadIdx.x == 0) ip_shared = ipt_t0;
    __syncthreads();
    const double ipt = ip_shared;
    // (a uniform grid so coarse that every coordinate falls into the interval around 0 leaves <R(x),Q> = 0)
    const bool valid = (n2 > 0.0) && (n2 < INFINITY) && (ipt > 0.0);
    uint32_t *payload = reinterpret_cast<uint32_t *>(static_cast<char *>(B.msg[c]) + EDEN_HEADER_BYTES);
    const uint32_t nsent = D / (uint32_t)k;                    // transmitted indices
    const uint32_t nwords = 2u * ((nsent * (uint32_t)bits + 63u) / 64u);
    const uint64_t subkey = stream_key(seed, kStreamSubsample, B.client[c]);
    for (uint32_t w = threadIdx.x; w < nwords; w += 256) {       // payload bit 32 w + e = bit (pos % bits) of index pos / bits
        uint32_t word = 0;
        for (uint32_t e = 0; e < 32u; ++e) {
            const uint32_t pos = 32u * w + e, j = pos / (uint32_t)bits, r = pos % (uint32_t)bits;
            if (j >= nsent) break;
            uint32_t i = j;
            if (k == 2) i = 2u * j + (uint32_t)((hash_word(subkey, j >> 6) >> (j & 63u)) & 1ull);
            word |= (((uint32_t)code[i] >> r) & 1u) << e;
        }
        payload[w] = valid ? word : 0u;
    }
    if (mix) {                                                 // second part: the top bit of every pair's finer index
        const uint32_t npairs = D / 2u, nwords_b = 2u * ((npairs + 63u) / 64u);
        for (uint32_t w = threadIdx.x; w < nwords_b; w += 256) {
            uint32_t word = 0;
            for (uint32_t e = 0; e < 32u; ++e) {
                const uint32_t g = 32u * w + e;
                if (g >= npairs) break;
                const uint32_t i = 2u * g + (uint32_t)((hash_word(mixkey, g >> 6) >> (g & 63u)) & 1ull);
                word |= (((uint32_t)code[i] >> bits) & 1u) << e;
            }
            payload[nwords + w] = valid ? word : 0u;
        }
    }
    uint32_t extra_bits = 0;
    if (coin_frac) {
        // second part: the top bits of the coordinates with a coin, in coordinate order.  A thread looks after 16
        // consecutive coordinates; a scan over the threads gives the place of its bits.
        for (uint32_t w = threadIdx.x; w < (uint32_t)kLoTile / 32u; w += 256) coin_words[w] = 0u;
        uint32_t m16 = 0, t16 = 0;
        for (uint32_t e = 0; e < 16u; ++e) {
            const uint32_t i = 16u * threadIdx.x + e;
            if (i < D && coin_of(mixkey, i, coin_frac)) {
                m16 |= 1u << e;
                t16 |= (((uint32_t)code[i] >> bits) & 1u) << e;
            }
        }
        const uint32_t before = block_exclusive_scan_256((uint32_t)__popc(m16), wave_totals, extra_bits);   // barriers inside
        or_bits(coin_words, before, compress_bits(t16, m16), (uint32_t)__popc(m16));
        __syncthreads();
        const uint32_t nwords_b = 2u * ((extra_bits + 63u) / 64u);
        for (uint32_t w = threadIdx.x; w < nwords_b; w += 256) payload[nwords + w] = valid ? coin_words[w] : 0u;
    }
    if (threadIdx.x == 0) {
        MsgHeader h;
        h.magic = kMagic; h.log2D = (uint32_t)log2D; h.d = hdr_d; h.b_q8 = B.hdr_b_q8[c]; h.client = B.client[c];
        h.extra_bits = extra_bits; h.seed = seed; h.N2 = n2;
        if (valid) {
            h.IP = ipt * exp2(-0.5 * (double)log2D);
            h.S = n2 / h.IP;
            h.status = 0;
        } else {
            h.IP = 0.0; h.S = 0.0;
            h.status = (n2 >= 0.0 && n2 < INFINITY) ? EDEN_DEV_ZERO_VECTOR : EDEN_DEV_NONFINITE;
            atomicOr(dev_status, h.status);
        }
        *static_cast<MsgHeader *>(B.msg[c]) = h;
    }
}

// One workgroup decodes the whole batch: per sender fill LDS with the dequantized rotated vector,
// transform, apply the signs and add into per-thread sums; acc is touched once at the end.
__global__ __launch_bounds__(256) void k_dec_small(DecBatch B, uint32_t n, uint64_t d, int pre, uint64_t hdr_d, int log2D,
                                                   uint64_t seed, const DevTables *tab, float *acc, uint32_t *dev_status,
                                                   uint32_t *msg_flags) {
    __shared__ float buf[kLoTile];
    __shared__ DecScratch s;
    __shared__ uint32_t coin_m16[256], coin_pre[256], wave_totals[4];   // coin budgets: coins of 16 coordinates, coins before them
    const uint32_t D = 1u << log2D;
    float sum[kLoTile / 256];
#pragma unroll
    for (int r = 0; r < kLoTile / 256; ++r) sum[r] = 0.0f;
    for (uint32_t c = 0; c < n; ++c) {
        __syncthreads();
        const uint32_t coin_frac = coin_q8(B.b_q8[c]) & 255u;
        uint32_t extra_bits = 0;
        if (coin_frac) {                                         // the receiver draws the same coins and counts them
            const uint64_t ckey = stream_key(seed, kStreamMix, B.client[c]);
            uint32_t m16 = 0;
            for (uint32_t e = 0; e < 16u; ++e) {
                const uint32_t i = 16u * threadIdx.x + e;
                if (i < D && coin_of(ckey, i, coin_frac)) m16 |= 1u << e;
            }
            coin_m16[threadIdx.x] = m16;
            coin_pre[threadIdx.x] = block_exclusive_scan_256((uint32_t)__popc(m16), wave_totals, extra_bits);
        }
        if (threadIdx.x < 64)
            dec_prepare_wave(B.msg[c], B.bitmap[c], B.client[c], B.b_q8[c], B.hdr_b_q8[c], hdr_d, log2D, seed, tab, &s, dev_status,
                             extra_bits, msg_flags ? msg_flags + c : nullptr);
        __syncthreads();
        const uint32_t b_q8 = B.b_q8[c];
        int bits, k;
        budget_of(b_q8, bits, k);
        const uint32_t *payload = reinterpret_cast<const uint32_t *>(static_cast<const char *>(B.msg[c]) + EDEN_HEADER_BYTES);
        const uint32_t *bm = B.bitmap[c];
        const uint64_t subkey = stream_key(seed, kStreamSubsample, B.client[c]);
        const uint32_t nwords = 2u * (((D / (uint32_t)k) * (uint32_t)bits + 63u) / 64u);
        const bool mix = budget_mixed(b_q8);
        const uint64_t mixkey = stream_key(seed, kStreamMix, B.client[c]);
        for (uint32_t i = threadIdx.x; i < D; i += 256) {
            const uint32_t pk = i >> 10;
            bool here = bm ? ((bm[pk >> 5] >> (pk & 31u)) & 1u) : true;
            uint32_t j = i;
            if (k == 2) {
                j = i >> 1;
                const uint32_t off = (uint32_t)((hash_word(subkey, j >> 6) >> (j & 63u)) & 1ull);
                here = here && ((i & 1u) == off);
            }
            const uint32_t bitpos = j * (uint32_t)bits, w0 = bitpos >> 5;
            const uint32_t next = (w0 + 1u < nwords) ? payload[w0 + 1u] : 0u;       // a 3-bit index may straddle two words
            const uint32_t idx = code_at(payload[w0], next, bitpos & 31u, bits);
            float val = grid_q15(b_q8) ? dequantize_byte<true>(idx, 0u, s.grid_deq)
                      : wide_bits(b_q8) ? dequantize_byte<false>(idx, wide_half_levels(b_q8), s.grid_deq) : s.deq[idx & 15u];
            if (mix) {
                const uint32_t g = i >> 1;
                if ((uint32_t)((hash_word(mixkey, g >> 6) >> (g & 63u)) & 1ull) == (i & 1u))
                    val = s.deq2[(((payload[nwords + (g >> 5)] >> (g & 31u)) & 1u) << bits) | idx];
            }
            if (coin_frac && ((coin_m16[i >> 4] >> (i & 15u)) & 1u)) {
                const uint32_t rank = coin_pre[i >> 4] + (uint32_t)__popc(coin_m16[i >> 4] & ((1u << (i & 15u)) - 1u));
                val = s.deq2[(((payload[nwords + (rank >> 5)] >> (rank & 31u)) & 1u) << bits) | idx];
            }
            buf[i] = here ? val : 0.0f;
        }
        fwht_lds(buf, D);
        const uint64_t key = stream_key(seed, kStreamSign, B.client[c]);
#pragma unroll
        for (int r = 0; r < kLoTile / 256; ++r) {
            const uint32_t i = threadIdx.x + 256u * r;
            if (i < D) {
                const bool neg = (hash_word(key, i >> 6) >> (i & 63u)) & 1ull;
                const float val = neg ? -buf[i] : buf[i];
                if (pre) {                                     // value i of this sender belongs at 2i + o_i (Sec. 4.1)
                    const uint64_t pos = 2ull * i + ((hash_word(subkey, i >> 6) >> (i & 63u)) & 1ull);
                    if (pos < d) acc[pos] += val;
                } else {
                    sum[r] += val;
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kLoTile / 256; ++r) {
        const uint32_t i = threadIdx.x + 256u * r;
        if (!pre && i < d && i < D) acc[i] += sum[r];
    }
}

// Writes up to kArgDoubles doubles that travel as kernel arguments (for a caller that may neither allocate nor stage a copy).
struct ArgDoubles { double v[kArgDoubles]; };
__global__ __launch_bounds__(kArgDoubles) void k_store_doubles(ArgDoubles a, uint32_t count, double *dst) {
    if (threadIdx.x < count) dst[threadIdx.x] = a.v[threadIdx.x];
}

// ------------------------------------------------------------------------------------------------
// test helpers: the hash streams written out
__global__ void k_hash_bits(uint64_t key, uint64_t nwords, uint64_t *out) {
    const uint64_t j = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < nwords) out[j] = hash_word(key, j);
}
__global__ void k_loss_bitmap(uint64_t key, uint32_t npk, uint32_t drop_q32, uint32_t *bitmap) {
    const uint32_t w = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t nw = (npk + 31u) / 32u;
    if (w >= nw) return;
    uint32_t bits = 0;
    for (uint32_t e = 0; e < 32; ++e) {
        const uint32_t j = w * 32u + e;
        if (j >= npk) break;
        const uint32_t top = (uint32_t)(hash_word(key, j) >> 32);
        if (top >= drop_q32) bits |= 1u << e;                  // received
    }
    bitmap[w] = bits;
}

// ------------------------------------------------------------------------------------------------
// host-side launchers
#define EDEN_HI_SWITCH(M, CALL)            \
    switch (M) {                           \
        case 1: { constexpr int MM = 1; CALL; } break; \
        case 2: { constexpr int MM = 2; CALL; } break; \
        case 3: { constexpr int MM = 3; CALL; } break; \
        case 4: { constexpr int MM = 4; CALL; } break; \
        case 5: { constexpr int MM = 5; CALL; } break; \
        default: { constexpr int MM = 6; CALL; } break; \
    }

uint32_t launch_enc_hi_last(int M, const EncBatch &B, uint32_t n, uint64_t valid_elems, int log2D, int p, uint64_t seed,
                            const float *T, double *partials, uint32_t partial_stride, const EncScratch *scratch,
                            const CoinTables &ct, hipStream_t st) {
    const uint32_t ntiles = 1u << (log2D - 6 - M);
    dim3 grid((ntiles + 3) / 4, n);
    bool all1 = M >= 5, all2 = M >= 5, all4 = M >= 5;            // one budget for all (two-pass sizes): its own instance
    for (uint32_t c = 0; c < n; ++c) {
        all1 = all1 && B.b_q8[c] == 256u;
        all2 = all2 && B.b_q8[c] == 512u;
        all4 = all4 && B.b_q8[c] == 1024u;
    }
#define EDEN_ENC_HI_LAST(MM, ONLY)                                                                                            \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(k_enc_hi_last<MM, ONLY>), grid, dim3(256), 0, st, B, valid_elems, log2D, p, seed, T, partials, \
                       partial_stride, scratch, ct)
    if (all1) { if (M == 5) EDEN_ENC_HI_LAST(5, 256u); else EDEN_ENC_HI_LAST(6, 256u); }
    else if (all2) { if (M == 5) EDEN_ENC_HI_LAST(5, 512u); else EDEN_ENC_HI_LAST(6, 512u); }
    else if (all4) { if (M == 5) EDEN_ENC_HI_LAST(5, 1024u); else EDEN_ENC_HI_LAST(6, 1024u); }
    else EDEN_HI_SWITCH(M, EDEN_ENC_HI_LAST(MM, 0u));
#undef EDEN_ENC_HI_LAST
    return grid.x;
}
uint32_t launch_enc_wide_last(const EncBatch &B, uint32_t n, uint64_t valid_elems, int log2D, const float *T, double *partials,
                              uint32_t partial_stride, const EncScratch *scratch, hipStream_t st) {
    dim3 grid(1u << (log2D - 3 - 9 - 2), n);                     // D / 8 rows / 512 columns / 4 waves
    hipLaunchKernelGGL(k_enc_wide_last, grid, dim3(256), 0, st, B, valid_elems, log2D, T, partials, partial_stride, scratch);
    return grid.x;
}
void launch_dec_wide_first(const DecBatch &B, uint32_t n, uint64_t keep_elems, int log2D, const DecScratch *scratch, float *T,
                           hipStream_t st) {
    dim3 grid(1u << (log2D - 3 - 9 - 2), n);
    hipLaunchKernelGGL(k_dec_wide_first, grid, dim3(256), 0, st, B, keep_elems, log2D, scratch, T);
}
void launch_enc_norm(const EncBatch &B, uint32_t n, const double *partials, uint32_t partial_stride, uint32_t nparts,
                     EncScratch *scratch, const DevTables *tab, hipStream_t st) {
    hipLaunchKernelGGL(k_enc_norm, dim3(n), dim3(256), 0, st, B, partials, partial_stride, nparts, scratch, tab);
}
void launch_enc_finish(const EncBatch &B, uint32_t n, uint64_t hdr_d, int log2D, uint64_t seed,
                       const double *partials_n2, uint32_t nparts_n2, const double *partials_ip, uint32_t nparts_ip,
                       uint32_t partial_stride, uint32_t *dev_status, const uint32_t *coin_total, hipStream_t st) {
    const uint32_t words_b1 = 1u << (log2D - 5);
    hipLaunchKernelGGL(k_enc_finish, dim3(n), dim3(256), 0, st, B, hdr_d, log2D, seed, partials_n2, nparts_n2, partials_ip,
                       nparts_ip, partial_stride, words_b1, dev_status, coin_total);
}
void launch_coin_tables(const uint32_t *clients, const uint32_t *b_q8, void *const *part_b, uint32_t n, uint64_t seed, int log2D,
                        const CoinTables &ct, hipStream_t st) {
    CoinBatch B;
    for (uint32_t i = 0; i < (uint32_t)kMaxBatch; ++i) {
        B.client[i] = i < n ? clients[i] : 0u;
        B.b_q8[i] = i < n ? b_q8[i] : 0u;
        B.part_b[i] = (i < n && part_b) ? part_b[i] : nullptr;
    }
    const uint32_t words = 1u << (log2D - 6);
    hipLaunchKernelGGL(k_coin_masks, dim3((words + kCoinGroup - 1) / kCoinGroup, n), dim3(256), 0, st, B, seed, log2D, ct);
    hipLaunchKernelGGL(k_coin_scan, dim3(n), dim3(256), 0, st, B, log2D, ct);
}
void launch_coin_pack(const uint32_t *b_q8, const uint32_t *const *pieces, void *const *part_b, uint32_t n, int log2D,
                      const CoinTables &ct, hipStream_t st) {
    CoinPackBatch B;
    for (uint32_t i = 0; i < (uint32_t)kMaxBatch; ++i) {
        B.b_q8[i] = i < n ? b_q8[i] : 0u;
        B.pieces[i] = i < n ? pieces[i] : nullptr;
        B.part_b[i] = i < n ? static_cast<uint64_t *>(part_b[i]) : nullptr;
    }
    const uint32_t blocks = 1u << (log2D - 6);
    hipLaunchKernelGGL(k_coin_pack, dim3((blocks + 255u) / 256u, n), dim3(256), 0, st, B, log2D, ct);
}
void launch_dec_hi_first(int M, const DecBatch &B, uint32_t n, uint64_t keep_elems, int log2D, int p, uint64_t seed,
                         const DecScratch *scratch, int narrow, float *T, const CoinTables &ct, hipStream_t st) {
    const uint32_t ntiles = 1u << (log2D - 6 - M);
    dim3 grid((ntiles + 3) / 4, n);
    bool all1 = M >= 5, all2 = M >= 5, all4 = M >= 5;            // one budget for all (two-pass sizes): its own instance
    for (uint32_t c = 0; c < n; ++c) {
        all1 = all1 && B.b_q8[c] == 256u;
        all2 = all2 && B.b_q8[c] == 512u && !B.codes[c];
        all4 = all4 && B.b_q8[c] == 1024u && !B.codes[c];
    }
#define EDEN_DEC_HI_FIRST(MM, ONLY)                                                                                           \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(k_dec_hi_first<MM, ONLY>), grid, dim3(256), 0, st, B, keep_elems, log2D, p, seed, scratch, \
                       narrow, T, ct)
    if (all1) { if (M == 5) EDEN_DEC_HI_FIRST(5, 256u); else EDEN_DEC_HI_FIRST(6, 256u); }
    else if (all2) { if (M == 5) EDEN_DEC_HI_FIRST(5, 512u); else EDEN_DEC_HI_FIRST(6, 512u); }
    else if (all4) { if (M == 5) EDEN_DEC_HI_FIRST(5, 1024u); else EDEN_DEC_HI_FIRST(6, 1024u); }
    else EDEN_HI_SWITCH(M, EDEN_DEC_HI_FIRST(MM, 0u));
#undef EDEN_DEC_HI_FIRST
}
uint32_t launch_enc_lo_first(const EncBatch &B, uint32_t n, uint64_t d_src, int pre, int log2D, uint64_t seed, float *T,
                             double *partials, uint32_t partial_stride, hipStream_t st) {
    const uint64_t d = pre ? (d_src + 1) / 2 : d_src;
    const uint32_t tiles = (uint32_t)((d + (1u << kLoBits) - 1) >> kLoBits);
    dim3 grid((tiles + 1) / 2, n);
    hipLaunchKernelGGL(k_enc_lo_first, grid, dim3(128), 0, st, B, d_src, pre, log2D, seed, T, partials, partial_stride);
    return grid.x;
}
void launch_dec_prepare(const DecBatch &B, uint32_t n, uint64_t hdr_d, int log2D, uint64_t seed, const DevTables *tab,
                        DecScratch *scratch, uint32_t *dev_status, const uint32_t *coin_total, uint32_t *msg_flags,
                        hipStream_t st) {
    hipLaunchKernelGGL(k_dec_prepare, dim3(n), dim3(64), 0, st, B, hdr_d, log2D, seed, tab, scratch, dev_status, coin_total,
                       msg_flags);
}
void launch_dec_lo_last(const DecBatch &B, uint32_t n, uint64_t d, int pre, int log2D, uint64_t seed, float *T,
                        const DecScratch *scratch, int narrow, float *acc, hipStream_t st) {
    dim3 grid(1u << (log2D - kLoBits - 1));
    hipLaunchKernelGGL(k_dec_lo_last, grid, dim3(128), 0, st, B, n, d, pre, log2D, seed, T, scratch, narrow, acc);
}
void launch_finalize_mean(const float *acc, uint64_t d, uint32_t n, float *mean, hipStream_t st) {
    const int vec = ((reinterpret_cast<uintptr_t>(acc) | reinterpret_cast<uintptr_t>(mean)) & 15u) == 0;
    const uint64_t per_block = 256u * (vec ? 4u : 1u);
    const uint32_t blocks = (uint32_t)((d + per_block - 1) / per_block);
    hipLaunchKernelGGL(k_finalize_mean, dim3(blocks), dim3(256), 0, st, acc, d, (float)n, mean, vec);
}
void launch_sparse_gather(const float *x, uint64_t d, uint32_t m, uint64_t seed, uint32_t client, float *stage, hipStream_t st) {
    const uint32_t blocks = (uint32_t)((d + 63) / 64);
    hipLaunchKernelGGL(k_sparse_gather, dim3((blocks + 15) / 16), dim3(256), 0, st, x, (uint32_t)d, m, stream_key(seed, kStreamSparse, client),
                       stage);
}
void launch_sparse_scatter(const float *stage, uint64_t d, uint32_t m, uint64_t seed, uint32_t client, float *acc, hipStream_t st) {
    const uint32_t blocks = (uint32_t)((d + 63) / 64);
    hipLaunchKernelGGL(k_sparse_scatter, dim3((blocks + 15) / 16), dim3(256), 0, st, stage, (uint32_t)d, m,
                       stream_key(seed, kStreamSparse, client), acc);
}
void launch_sparse_gather_batch(const EncBatch &B, uint32_t n, uint64_t d, uint32_t m, uint64_t seed, float *T, int log2Dk,
                                hipStream_t st) {
    const uint32_t blocks = (uint32_t)((d + 63) / 64);
    hipLaunchKernelGGL(k_sparse_gather_batch, dim3((blocks + 15) / 16, n), dim3(256), 0, st, B, (uint32_t)d, m, seed, T, log2Dk);
}
void launch_sparse_scatter_batch(const DecBatch &B, uint32_t n, uint64_t d, uint32_t m, uint64_t seed, const float *T, int log2Dk,
                                 float *acc, hipStream_t st) {
    const uint32_t blocks = (uint32_t)((d + 63) / 64);
    hipLaunchKernelGGL(k_sparse_scatter_batch, dim3((blocks + 15) / 16), dim3(256), 0, st, B, n, (uint32_t)d, m, seed, T, log2Dk, acc);
}
void launch_pack_bits(const EncBatch &B, uint32_t n, int log2D, hipStream_t st) {          // multi-pass sizes: D >= 2^13
    const uint64_t groups = (1ull << log2D) / 32;
    hipLaunchKernelGGL(k_pack_bits, dim3((uint32_t)((groups + 255) / 256), n), dim3(256), 0, st, B, log2D);
}
void launch_unpack_bits(const DecBatch &B, uint32_t n, int log2D, uint8_t *codes_all, hipStream_t st) {
    const uint64_t groups = (1ull << log2D) / 32;
    hipLaunchKernelGGL(k_unpack_bits, dim3((uint32_t)((groups + 255) / 256), n), dim3(256), 0, st, B, log2D, codes_all);
}
void launch_fill_zero(float *p, uint64_t count, hipStream_t st) {
    hipLaunchKernelGGL(k_fill_zero, dim3((uint32_t)((count + 255) / 256)), dim3(256), 0, st, p, count);
}
void launch_byte_entropy(const uint8_t *bytes, uint64_t count, uint32_t *hist, double *out, hipStream_t st) {
    launch_fill_zero(reinterpret_cast<float *>(hist), 256, st);          // 256 words of zero bits
    uint32_t blocks = (uint32_t)((count + 4095) / 4096);
    if (blocks > 2048u) blocks = 2048u;
    if (blocks < 1u) blocks = 1u;
    hipLaunchKernelGGL(k_byte_histogram, dim3(blocks), dim3(256), 0, st, bytes, count, hist);
    hipLaunchKernelGGL(k_histogram_entropy, dim3(1), dim3(256), 0, st, hist, count, out);
}
void launch_sq_error(const float *a, const float *b, uint64_t d, double *partials, uint32_t max_parts, double *out,
                     hipStream_t st) {
    uint32_t blocks = (uint32_t)((d + 1023) / 1024);
    if (blocks > 1024u) blocks = 1024u;
    if (blocks > max_parts) blocks = max_parts;
    if (blocks < 1u) blocks = 1u;
    hipLaunchKernelGGL(k_sq_error, dim3(blocks), dim3(256), 0, st, a, b, d, partials);
    hipLaunchKernelGGL(k_sq_error_finish, dim3(1), dim3(256), 0, st, partials, blocks, out);
}
void launch_enc_small(const EncBatch &B, uint32_t n, uint64_t d, int pre, uint64_t hdr_d, int log2D, uint64_t seed,
                      const DevTables *tab, uint32_t *dev_status, hipStream_t st) {
    hipLaunchKernelGGL(k_enc_small, dim3(n), dim3(256), 0, st, B, d, pre, hdr_d, log2D, seed, tab, dev_status);
}
void launch_dec_small(const DecBatch &B, uint32_t n, uint64_t d, int pre, uint64_t hdr_d, int log2D, uint64_t seed,
                      const DevTables *tab, float *acc, uint32_t *dev_status, uint32_t *msg_flags, hipStream_t st) {
    hipLaunchKernelGGL(k_dec_small, dim3(1), dim3(256), 0, st, B, n, d, pre, hdr_d, log2D, seed, tab, acc, dev_status, msg_flags);
}
void launch_store_doubles(const double *src_host, uint32_t count, double *dst, hipStream_t st) {
    ArgDoubles a;
    for (uint32_t i = 0; i < (uint32_t)kArgDoubles; ++i) a.v[i] = i < count ? src_host[i] : 0.0;
    hipLaunchKernelGGL(k_store_doubles, dim3(1), dim3(kArgDoubles), 0, st, a, count, dst);
}
void launch_hash_bits(uint64_t key, uint64_t nwords, uint64_t *out, hipStream_t st) {
    hipLaunchKernelGGL(k_hash_bits, dim3((uint32_t)((nwords + 255) / 256)), dim3(256), 0, st, key, nwords, out);
}
void launch_loss_bitmap(uint64_t key, uint32_t npk, uint32_t drop_q32, uint32_t *bitmap, hipStream_t st) {
    const uint32_t nw = (npk + 31u) / 32u;
    hipLaunchKernelGGL(k_loss_bitmap, dim3((nw + 255) / 256), dim3(256), 0, st, key, npk, drop_q32, bitmap);
}

}  // namespace eden
