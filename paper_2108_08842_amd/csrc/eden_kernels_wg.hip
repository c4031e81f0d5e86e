// Workgroup-tile strided passes of the Walsh-Hadamard transform for large D (2^21 .. 2^27), gfx950.
//
// Two passes through memory are enough for D <= 2^24 when a workgroup keeps 2^14 .. 2^15 coordinates on chip
// (registers + one or two exchanges through LDS):
//
//   lo14 pass (contiguous, index bits 0 .. 13): in eden_kernels_lo14.hip.
//   hiX pass  (strided, index bits 14 .. 14+M-1, M = 7..10): a workgroup owns 2^M rows of 32 consecutive
//             coordinates (128-byte segments) at stride 2^14.  Every thread keeps 64 rows of one column in
//             registers (six butterfly stages), the remaining M-6 row bits are reached by one exchange through
//             LDS (for M = 10 in two halves of 64 KiB so that two workgroups fit on a CU).
//
// The strided pass is the one next to the payload: encode runs it last and fuses quantization against the
// Lloyd-Max thresholds, <R(x),Q> and packing (Sec. 2.2.1, 2.3, 3, 4.1); decode runs it first and fuses
// unpacking and dequantization with S/(p sqrt D) (Sec. 2.2.2, 4.2).  The contiguous pass is the one next to x
// and to the accumulator, where the zero padding of d up to D costs nothing.
#include "eden_device.h"
#include "eden_kernels.h"

namespace eden {

// ------------------------------------------------------------------------------------------------
constexpr int kHixP = 14;     // lowest index bit of every workgroup-tile strided pass (it sits on top of lo14)

template <int M>
struct HiX {
    static constexpr int RL = 1 << (M - 6);       // row groups: the low M-6 row bits live across thread groups
    static constexpr int THREADS = 32 * RL;
    static constexpr int PH = (M == 10) ? 2 : 1;  // halves of the exchange
    static constexpr int RP = 64 / PH;            // registers exchanged per half
    static constexpr int RHL = RP / RL;           // high-row values a thread holds after the exchange
    static constexpr int LDS_FLOATS = RP * RL * 32;
};

// Workgroups are dealt to the 8 XCDs round robin and each XCD has its own L2.  Neighbouring tiles touch
// neighbouring 64..128-byte pieces of the same rows (and, in decode, the same 64-byte sectors of the payload),
// so runs of 16 consecutive tiles are kept on one XCD.
template <int RUN = 16>
__device__ inline uint32_t xcd_local_tile() {
    uint32_t tile = blockIdx.x;
    if (gridDim.x % (8u * RUN) == 0) {
        const uint32_t xcd = tile & 7u, q = tile >> 3;
        tile = ((q / RUN) * 8u + xcd) * RUN + (q % RUN);
    }
    return tile;
}

// The payload starts 64 bytes into a message, so its 128-byte memory lines do not start where the runs of neighbouring
// tiles start: every line would be shared by two runs (two XCDs) and fetched twice (measured: 64 MiB for a 32 MiB payload).
// Rotates the column-block index of a tile so that the runs start on line boundaries.  `row_bytes`: payload bytes of one
// tile row, a power of two below 128; `cb_bits`: log2 of the column blocks per row.
__device__ inline uint32_t align_runs_to_lines(uint32_t tile, uint32_t cb_bits, const void *payload, uint32_t row_bytes) {
    const uint32_t per_line = 128u / row_bytes;
    const uint32_t shift = (uint32_t)(reinterpret_cast<uintptr_t>(payload) / row_bytes) & (per_line - 1u);
    const uint32_t mask = (1u << cb_bits) - 1u;
    return (tile & ~mask) | ((tile - shift) & mask);
}

template <int M>
__device__ inline uint64_t hix_base(uint32_t tile, int p) {
    const uint32_t cb_bits = (uint32_t)p - 5u;                   // 2^(p-5) blocks of 32 columns
    const uint32_t cb = tile & ((1u << cb_bits) - 1u);
    const uint32_t upper = tile >> cb_bits;
    return ((uint64_t)upper << (p + M)) | ((uint64_t)cb << 5);
}

// row held in stage-1 register r by a thread of group g
template <int M>
__device__ inline uint32_t hix_row1(uint32_t g, uint32_t r) { return g + (uint32_t)HiX<M>::RL * r; }
// row held after the exchange of half ph in register s by a thread of group g
template <int M>
__device__ inline uint32_t hix_row2(uint32_t g, int ph, int s) {
    using X = HiX<M>;
    const uint32_t e = (uint32_t)s / X::RL, rl = (uint32_t)s % X::RL;
    const uint32_t rh = (uint32_t)ph * X::RP + g * X::RHL + e;
    return rl + (uint32_t)X::RL * rh;
}

// Exchange of half `PHASE`: stage-1 registers -> LDS -> registers that hold all low row bits of
// RHL high-row values; then the butterflies over those low row bits.  Split in two so that a caller can
// start loading the next tile into the registers the write has just freed.
template <int M, int PHASE>
__device__ inline void hix_exchange_write(const float (&v)[64], float *lds) {
    using X = HiX<M>;
    const uint32_t col = threadIdx.x & 31u, g = threadIdx.x >> 5;
#pragma unroll
    for (int i = 0; i < X::RP; ++i) lds[(i * X::RL + g) * 32 + col] = v[PHASE * X::RP + i];
}
// ALL_STAGES = false leaves out the stage over bit 0 of the register index (see hix_sign_words_pairs).
template <int M, bool ALL_STAGES = true>
__device__ inline void hix_exchange_read(float *lds, float (&out)[HiX<M>::RP]) {
    using X = HiX<M>;
    const uint32_t col = threadIdx.x & 31u, g = threadIdx.x >> 5;
    __syncthreads();
#pragma unroll
    for (int s = 0; s < X::RP; ++s) {
        const int e = s / X::RL, rl = s % X::RL;
        out[s] = lds[((g * X::RHL + e) * X::RL + rl) * 32 + col];
    }
    __syncthreads();
    fwht_regs_low<X::RP, M - 6, ALL_STAGES ? 1 : 2>(out);
}
template <int M, int PHASE>
__device__ inline void hix_exchange(const float (&v)[64], float *lds, float (&out)[HiX<M>::RP]) {
    hix_exchange_write<M, PHASE>(v, lds);
    hix_exchange_read<M>(lds, out);
}

// ---- packing in the strided layout.  After a tile's last butterfly a register holds, across the two halves of
// a wave, two row segments of 32 consecutive coordinates: exactly one payload word each at b = 1.  A ballot
// of one bit of the index gives both words at once; lane j of each half collects the words of register j
// (v_writelane), and after the last register every lane finishes and stores the words of "its" row.
// row of the tile whose words lane j holds for register block w after half ph of the exchange
template <int M>
__device__ inline uint32_t hix_word_row(int ph, int w) {
    using X = HiX<M>;
    const uint32_t s = 32u * (uint32_t)w + (lane_id() & 31u), g = threadIdx.x >> 5;
    return s % X::RL + (uint32_t)X::RL * ((uint32_t)ph * X::RP + g * X::RHL + s / X::RL);
}

// Quantizes and packs the RP values a thread holds after one half of the exchange (rows hix_row2(g, PH, s)).
// `word0`: payload word index of this tile's 32 columns in row 0; `base`: first coordinate of the tile.
// BITS: bits of every index in the first part of the payload.  MIX = 1 (b = BITS + 1/2, Sec. 4.1): the coordinate of
// every pair that the MIX stream selects is quantized with I_{BITS+1}; the top bit of its index goes to the
// second part of the payload, one bit per pair = 16 bits per row segment of a tile.  MIX = 2 (coin budgets, Sec. 4.1):
// the coordinates with a coin use I_{BITS+1}; their top bits go to the second part (`part_c`) in coordinate order, at the
// place the prefix sums over the coins give the row segment.
// TRANSPOSE (BITS = 4, MIX = 0): instead of the ballots, a lane collects the indices of eight registers (rows) of its
// column in one word, and the lanes of eight neighbouring columns transpose their words: each then holds one payload word of
// one row.  2 instructions per register instead of 12, but more code: only the kernel instance whose senders all have b = 4
// uses it (in the instance shared by all budgets it raised the register spills and cost b = 2 a quarter of its speed).
template <int M, int BITS, int MIX, bool TRANSPOSE = false>
__device__ inline void hix_quantize_pack(const float (&out)[HiX<M>::RP], int ph, const EncScratch *sc, const float *qtab,
                                         uint32_t *payload, uint16_t *part_b, uint64_t mixkey, uint64_t base, float &ip,
                                         const CoinTables &ct, uint32_t c, int log2D, uint32_t *part_c,
                                         const RankCell *cells = nullptr, float cell_scale = 0.0f, uint32_t *pieces = nullptr) {
    using X = HiX<M>;
    constexpr int p = kHixP;
    constexpr int H = 1 << (BITS - 1);
    constexpr int NW = X::RP / 32;                               // registers come in blocks of 32 = one word lane each
    const uint32_t lane = lane_id(), col = lane & 31u;
    const uint32_t word0 = (uint32_t)(base >> 5);
    if constexpr (TRANSPOSE) {
        static_assert(MIX == 0 && BITS == 4, "one nibble per coordinate");
        constexpr int PER = 32 / BITS;
        const uint32_t g = threadIdx.x >> 5, j = col & (uint32_t)(PER - 1), q = col / (uint32_t)PER;
        const bool by_table = cells[0].below != kRankCollision;  // (see fill_rank_table; the same for the whole workgroup)
        static_for<X::RP / PER>([&](auto K) {
            constexpr int k = decltype(K)::value;
            uint32_t items = 0;
            if (by_table) {
#pragma unroll
                for (int i = 0; i < PER; ++i) items |= quantize_one_table<H>(out[PER * k + i], cells, cell_scale, ip) << (BITS * i);
            } else {
#pragma unroll
                for (int i = 0; i < PER; ++i) items |= quantize_one<H>(out[PER * k + i], sc, qtab, ip) << (BITS * i);
            }
            items = transpose_items<BITS>(items, lane);
            const uint32_t row = hix_row2<M>(g, ph, (int)(PER * k + j));
            payload[(uint32_t)BITS * (word0 + (row << (p - 5))) + q] = items;
        });
        return;
    }
    uint32_t plane[BITS][NW], top[NW], offs16[NW], coin_off[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        top[w] = 0;
#pragma unroll
        for (int b = 0; b < BITS; ++b) plane[b][w] = 0;
        // this lane's row for register block w, and the 16 pair offsets of that row segment (64 pairs per hash word)
        const uint64_t first = base + ((uint64_t)hix_word_row<M>(ph, w) << p);
        offs16[w] = MIX == 1 ? (uint32_t)(hash_word(mixkey, first >> 7) >> (16u * (uint32_t)((first >> 5) & 3u))) & 0xFFFFu : 0u;
        coin_off[w] = 0;
        if constexpr (MIX == 2) {                                // the 32 coins of that row segment: half of a block of 64
            const uint32_t blk = (uint32_t)(first >> 6), upper = (uint32_t)(first >> 5) & 1u;
            const uint64_t m64 = coin_mask_of(ct, c, log2D, blk);
            offs16[w] = upper ? hi32(m64) : lo32(m64);
            coin_off[w] = coins_before(ct, c, log2D, blk) + (upper ? (uint32_t)__popc(lo32(m64)) : 0u);
        }
    }
    static_for<X::RP>([&](auto S) {
        constexpr int s = decltype(S)::value;
        uint32_t code;
        if constexpr (MIX != 0) {
            const uint32_t oa = __builtin_amdgcn_readlane(offs16[s / 32], s % 32);
            const uint32_t ob = __builtin_amdgcn_readlane(offs16[s / 32], 32 + s % 32);
            const uint32_t offs = (lane < 32u) ? oa : ob;
            const bool up = MIX == 1 ? ((offs >> (col >> 1)) & 1u) == (col & 1u) : ((offs >> col) & 1u) != 0u;
            code = quantize_mixed<BITS>(out[s], up, sc, qtab, ip);
            const uint64_t m = __ballot((code >> BITS) & 1u);
            top[s / 32] = put_lane<s % 32>(lo32(m), top[s / 32]);
            top[s / 32] = put_lane<32 + s % 32>(hi32(m), top[s / 32]);
        } else {
            code = quantize_one<H>(out[s], sc, qtab, ip);
        }
#pragma unroll
        for (int b = 0; b < BITS; ++b) {
            const uint64_t m = __ballot((code >> b) & 1u);
            plane[b][s / 32] = put_lane<s % 32>(lo32(m), plane[b][s / 32]);
            plane[b][s / 32] = put_lane<32 + s % 32>(hi32(m), plane[b][s / 32]);
        }
    });
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const uint32_t word = word0 + (hix_word_row<M>(ph, w) << (p - 5));
        if constexpr (BITS == 1) {
            payload[word] = plane[0][w];
        } else if constexpr (BITS == 2) {
            const uint32_t a = plane[0][w], b = plane[1][w];
            *reinterpret_cast<uint2 *>(payload + 2u * word) =
                make_uint2(spread2(a) | (spread2(b) << 1), spread2(a >> 16) | (spread2(b >> 16) << 1));
        } else if constexpr (BITS == 3) {
            uint32_t o[3];                                       // 32 coordinates x 3 bits = 3 words
            pack3_planes(plane[0][w], plane[1][w], plane[2][w], o);
            payload[3u * word] = o[0];
            payload[3u * word + 1u] = o[1];
            payload[3u * word + 2u] = o[2];
        } else {
            uint32_t o[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                o[k] = spread4(plane[0][w] >> (8 * k)) | (spread4(plane[1][w] >> (8 * k)) << 1) |
                       (spread4(plane[2][w] >> (8 * k)) << 2) | (spread4(plane[3][w] >> (8 * k)) << 3);
            *reinterpret_cast<uint4 *>(payload + 4u * word) = make_uint4(o[0], o[1], o[2], o[3]);
        }
        if constexpr (MIX == 1) part_b[word] = (uint16_t)even_bits(top[w] | (top[w] >> 1));    // only the chosen one can be set
        if constexpr (MIX == 2) {                                // only a coordinate with a coin can have the bit
            const uint32_t piece = (uint32_t)compress_bits(top[w], offs16[w]);
            // either the piece goes to the staging array (word = number of the segment of 32 coordinates; k_coin_pack strings
            // the pieces together) or straight to its bits of the second part, which neighbouring tiles share: atomics
            if (pieces) pieces[word] = piece;
            else or_bits(part_c, coin_off[w], piece, (uint32_t)__popc(offs16[w]));
        }
    }
}

// b = 1 and b = 1/2: the index is the sign (I_1, Sec. 3), <R(x),Q> = q_1 sum |u| / sqrt(D).  Leaves in words[w],
// lane j of each half, the 32 index bits of the row segment held in register 32 w + j.
template <int M>
__device__ inline void hix_sign_words(const float (&out)[HiX<M>::RP], float &ip, uint32_t (&words)[HiX<M>::RP / 32]) {
    using X = HiX<M>;
    float sa = 0.0f;
#pragma unroll
    for (int s = 0; s < X::RP; ++s) sa += fabsf(out[s]);
    ip = fmaf(sa, kQ1, ip);
#pragma unroll
    for (int w = 0; w < X::RP / 32; ++w) words[w] = 0;
    static_for<X::RP>([&](auto S) {
        constexpr int s = decltype(S)::value;
        const uint64_t m = __ballot((__float_as_uint(out[s]) >> 31) == 0u);      // index 1 = non-negative
        words[s / 32] = put_lane<s % 32>(lo32(m), words[s / 32]);
        words[s / 32] = put_lane<32 + s % 32>(hi32(m), words[s / 32]);
    });
}

// The same from the values BEFORE the last butterfly stage (registers 2 i and 2 i + 1 hold a and b; the transformed values
// would be a + b and a - b).  The sign quantizer needs of them only their signs and the sum of their magnitudes:
// a + b >= 0 is "not a < -b", a - b >= 0 is "not a < b" (the same decisions: rounding never changes the sign of a sum, and
// the passes before leave no negative zeros), and |a + b| + |a - b| = 2 max(|a|, |b|), which, unlike the two sums, is exact.
// Four instructions per pair (max, add, two compares) instead of six.
template <int M>
__device__ inline void hix_sign_words_pairs(const float (&out)[HiX<M>::RP], float &ip, uint32_t (&words)[HiX<M>::RP / 32]) {
    using X = HiX<M>;
    float sa = 0.0f;
#pragma unroll
    for (int s = 0; s < X::RP; s += 2) sa += fmaxf(fabsf(out[s]), fabsf(out[s + 1]));
    ip = fmaf(2.0f * sa, kQ1, ip);
#pragma unroll
    for (int w = 0; w < X::RP / 32; ++w) words[w] = 0;
    static_for<X::RP>([&](auto S) {
        constexpr int s = decltype(S)::value;
        const float a = out[s & ~1], b = out[s | 1];
        const uint64_t m = (s & 1) ? __ballot(!(a < b)) : __ballot(!(a < -b));     // index 1 = non-negative
        words[s / 32] = put_lane<s % 32>(lo32(m), words[s / 32]);
        words[s / 32] = put_lane<32 + s % 32>(hi32(m), words[s / 32]);
    });
}

template <int N> struct WordVec;
template <> struct WordVec<1> { using type = uint32_t; };
template <> struct WordVec<2> { using type = uint2; };
template <> struct WordVec<4> { using type = uint4; };

// Encode, last pass: T -> payload.  Index bits 14 .. 14+M-1 of H, then quantization to the Lloyd-Max intervals
// (Sec. 2.2.1, Sec. 3), sum_i u_i q_i for the scale (Sec. 2.3), sub-sampling for b = 1/2 (Sec. 4.1), packing.
// Rows of the workspace at or above ceil(d / 2^14) were not written by the first pass (they are zero padding
// transformed over bits 0..13, i.e. zero): the buffer bounds return 0 for them without touching memory.
// A workgroup handles TPW neighbouring column blocks; the loads of the next one are issued into the registers
// that each half of the exchange has just written to LDS.  MODE 0: every sender of the launch has b <= 1; the
// words of the TPW tiles are then kept and stored together (one row of a tile is only 4 bytes of payload).
// MODE 1: any integer budget or b = 1/2.  MODE 2: also the budgets k + 1/2 (they need more registers).
// MODE 3: every sender of the launch has b = 4 (the instance holds nothing else: no spills, and the transposing pack).
// BLK: the first pass wrote the workspace in the blocked layout (blocked_offset in eden_device.h).
// ONLY != 0: every sender of the launch has this budget; the instance holds that one branch of the quantizers.
template <int M, int TPW, int MODE, bool BLK, uint32_t ONLY = 0>
__global__ __launch_bounds__(HiX<M>::THREADS, TPW == 1 ? 4 : 1) void k_enc_hix_last(EncBatch B, uint64_t d, int log2D, uint64_t seed,
                                                                   const float *T, double *partials,
                                                                   uint32_t partial_stride, const EncScratch *scratch,
                                                                   CoinTables ct) {
    using X = HiX<M>;
    __shared__ float lds[X::LDS_FLOATS];
    __shared__ double red[X::THREADS / 64];
    __shared__ float qtab[16];                                   // centroids; published by the first barrier of the exchange
    __shared__ float gtab[256];                                  // one-byte budgets: centroids and thresholds
    __shared__ RankCell cells[MODE == 3 ? kRankCells : 1];       // b = 4 alone: the interval search by table
    constexpr int p = kHixP;
    constexpr int NW = X::RP / 32;
    constexpr bool UNIT = MODE == 0;
    const uint32_t c = blockIdx.y;
    const uint32_t tile0 = xcd_local_tile<16 / TPW>() * TPW;
    const uint32_t col = threadIdx.x & 31u, g = threadIdx.x >> 5;
    uint32_t rows_written = (uint32_t)((d + (1u << p) - 1) >> p);
    if (BLK) rows_written = (rows_written + kBlockRows - 1u) / kBlockRows * kBlockRows;      // whole blocks of rows are written
    const rsrc_t rt = make_rsrc(T + ((size_t)c << log2D), rows_written << (p + 2));
    uint32_t *payload = reinterpret_cast<uint32_t *>(static_cast<char *>(B.msg[c]) + EDEN_HEADER_BYTES);
    const uint32_t b_q8 = ONLY ? ONLY : B.b_q8[c];
    const EncScratch *sc = &scratch[c];
    // stage-1 rows: g + RL r.  Byte offset of (row, column) inside the slot = a per-thread part + a part that is the same for
    // the whole workgroup (row_off(r)) + the tile's column block
    constexpr uint32_t RLB = X::RL >= kBlockRows ? X::RL / kBlockRows : 1u;
    const uint32_t off1 = !BLK ? ((g << p) + col) * 4u
                               : X::RL >= kBlockRows ? (((g >> kBlockRowBits) << (p + kBlockRowBits)) + ((g & (kBlockRows - 1u)) << 5) + col) * 4u
                                                     : ((g << 5) + col) * 4u;
    auto row_off = [](int r) -> uint32_t {                       // r is a compile-time constant after unrolling
        if (!BLK) return ((uint32_t)X::RL * (uint32_t)r) << (p + 2);
        if (X::RL >= kBlockRows) return (RLB * (uint32_t)r) << (p + kBlockRowBits + 2);
        const uint32_t row = (uint32_t)X::RL * (uint32_t)r;      // RL = 2: rows g + 2 r, g = 0, 1
        return ((row >> kBlockRowBits) << (p + kBlockRowBits + 2)) + ((row & (kBlockRows - 1u)) << 7);
    };
    auto tile_off = [](uint32_t tile) -> uint32_t {              // (two-pass plans: the tile index is the column block)
        return BLK ? tile << (7 + kBlockRowBits) : (uint32_t)hix_base<M>(tile, p) * 4u;
    };
    const uint64_t mixkey = stream_key(seed, kStreamMix, B.client[c]);
    float cell_scale = 0.0f;
    if constexpr (MODE == 3) {
        cell_scale = rank_cell_scale(sc, 8);
        fill_rank_table<8>(cells, sc, threadIdx.x, cell_scale);  // published, like qtab, by the first barrier of the exchange
    }
    if (!UNIT) {
        fill_qtab(qtab, sc, threadIdx.x);
        if (byte_budget(b_q8)) {                                 // centroids, then thresholds: one run of 256 floats
            const float *byte_tab = sc->grid_c;
            for (uint32_t i = threadIdx.x; i < 256u; i += X::THREADS) gtab[i] = byte_tab[i];
        }
    }
    float ip = 0.0f;
    uint32_t held[TPW][X::PH][NW];
    float v[64];
    {
        const uint32_t b0 = tile_off(tile0);
#pragma unroll
        for (int r = 0; r < 64; ++r) v[r] = buf_load(rt, off1, b0 + row_off(r));
    }
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
        const uint64_t base = hix_base<M>(tile0 + k, p);
        const uint32_t next_off = tile_off(tile0 + k + 1);
        fwht_regs<64>(v);
        float out[X::RP];
#pragma unroll
        for (int ph = 0; ph < X::PH; ++ph) {
            if (ph == 0) hix_exchange_write<M, 0>(v, lds);
            else hix_exchange_write<M, X::PH - 1>(v, lds);
            if (k + 1 < TPW) {
#pragma unroll
                for (int r = ph * X::RP; r < (ph + 1) * X::RP; ++r)
                    v[r] = buf_load(rt, off1, next_off + row_off(r));
            }
            hix_exchange_read<M, !UNIT>(lds, out);               // every sender b <= 1: the last stage is fused into the signs
            if (UNIT) hix_sign_words_pairs<M>(out, ip, held[k][ph]);
            else if (MODE == 3) {
                hix_quantize_pack<M, 4, 0, true>(out, ph, sc, qtab, payload, reinterpret_cast<uint16_t *>(payload), mixkey, base, ip, ct,
                                                 c, log2D, payload, cells, cell_scale);
            } else if (b_q8 <= 256u) hix_sign_words<M>(out, ip, held[k][ph]);
            else if (byte_budget(b_q8)) {
                // uniform grid (Sec. 4.3) or b = 5..8: one byte per coordinate; a row segment of the tile is 32 bytes
                uint8_t *bytes = (B.codes[c] ? B.codes[c] : reinterpret_cast<uint8_t *>(payload)) + base + col;
                const float inv = sc->grid_inv;
                const uint32_t H = wide_half_levels(b_q8);
                if (grid_q15(b_q8)) {                            // the indices replace the values in their registers
#pragma unroll
                    for (int s2 = 0; s2 < X::RP; ++s2) out[s2] = __uint_as_float(quantize_byte<true>(out[s2], H, inv, gtab, ip));
                } else {
#pragma unroll
                    for (int s2 = 0; s2 < X::RP; ++s2) out[s2] = __uint_as_float(quantize_byte<false>(out[s2], H, inv, gtab, ip));
                }
#pragma unroll
                for (int s2 = 0; s2 < X::RP; ++s2) {             // four lanes' bytes = one dword store
                    const uint32_t quad = quad_bytes(__float_as_uint(out[s2]), col);
                    if (!(col & 3u)) *reinterpret_cast<uint32_t *>(bytes + ((uint64_t)hix_row2<M>(g, ph, s2) << p)) = quad;
                }
            } else {
                int ibits, ik;
                budget_of(b_q8, ibits, ik);
                uint32_t *part_c = payload + payload_a_bytes(1ull << log2D, ibits, 1) / 4;       // second part, if any
                uint16_t *part_b = reinterpret_cast<uint16_t *>(part_c);
                const uint32_t cq = MODE == 2 ? coin_q8(b_q8) : 0u;
                // coin budgets: a staging array for the pieces of the second part, if the host gave this sender one
                uint32_t *pieces = cq ? reinterpret_cast<uint32_t *>(B.codes[c]) : nullptr;
#define EDEN_HIX_PACK(BITS, MIX) \
    hix_quantize_pack<M, BITS, MIX>(out, ph, sc, qtab, payload, part_b, mixkey, base, ip, ct, c, log2D, part_c, nullptr, 0.0f, pieces)
                if (cq && ibits == 1) EDEN_HIX_PACK(1, 2);
                else if (cq && ibits == 2) EDEN_HIX_PACK(2, 2);
                else if (cq) EDEN_HIX_PACK(3, 2);
                else if (MODE == 2 && b_q8 == 384u) EDEN_HIX_PACK(1, 1);
                else if (MODE == 2 && b_q8 == 640u) EDEN_HIX_PACK(2, 1);
                else if (MODE == 2 && b_q8 == 896u) EDEN_HIX_PACK(3, 1);
                else if (b_q8 == 512u) EDEN_HIX_PACK(2, 0);
                else if (b_q8 == 768u) EDEN_HIX_PACK(3, 0);
                else EDEN_HIX_PACK(4, 0);
#undef EDEN_HIX_PACK
            }
        }
    }
    if (UNIT || (MODE != 3 && b_q8 <= 256u)) {
        // tile0 is a multiple of TPW: the TPW words of a row are neighbours, aligned to their common size
        const uint64_t base0 = hix_base<M>(tile0, p);
        const uint32_t word0 = (uint32_t)(base0 >> 5);
        const uint64_t subkey = stream_key(seed, kStreamSubsample, B.client[c]);
#pragma unroll
        for (int ph = 0; ph < X::PH; ++ph) {
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const uint32_t row = hix_word_row<M>(ph, w);
                const uint32_t word = word0 + (row << (p - 5));
                uint32_t o[TPW];
                if (b_q8 == 256u) {
#pragma unroll
                    for (int k = 0; k < TPW; ++k) o[k] = held[k][ph][w];
                    typename WordVec<TPW>::type pack;
                    __builtin_memcpy(&pack, o, sizeof(pack));
                    *reinterpret_cast<typename WordVec<TPW>::type *>(payload + word) = pack;
                } else {
                    // b = 1/2 (Sec. 4.1): of each pair (2k, 2k+1) send the coordinate chosen by the sub-sampling
                    // stream; 64 pairs per hash word = 128 coordinates = four neighbouring row segments
                    const uint64_t first = base0 + ((uint64_t)row << p);
                    const uint64_t hw = hash_word(subkey, first >> 7) >> (16u * (uint32_t)((first >> 5) & 3u));
                    uint16_t *half = reinterpret_cast<uint16_t *>(payload) + word;
#pragma unroll
                    for (int k = 0; k < TPW; ++k) {
                        const uint32_t off = (uint32_t)(hw >> (16 * k)) & 0xFFFFu;
                        const uint32_t ev = even_bits(held[k][ph][w]), od = even_bits(held[k][ph][w] >> 1);
                        o[k] = (ev & ~off) | (od & off);
                    }
                    if constexpr (TPW == 1) half[0] = (uint16_t)o[0];
                    else if constexpr (TPW == 2) *reinterpret_cast<uint32_t *>(half) = o[0] | (o[1] << 16);
                    else *reinterpret_cast<uint2 *>(half) = make_uint2(o[0] | (o[1] << 16), o[2] | (o[3] << 16));
                }
            }
        }
    }
    const double block_total = block_sum<X::THREADS>((double)ip, red);
    if (threadIdx.x == 0) partials[(size_t)c * partial_stride + blockIdx.x] = block_total;
}

// Middle pass of the three-pass sizes, in place on the workspace (tiles are disjoint).  Elements at or above
// `load_elems` were not written by the pass before (encode: zero padding) and read as zero; elements at or above
// `store_elems` are not read by the pass after (decode: they end in the padding) and are not written.  A tile
// that lies wholly beyond either bound has nothing to do.
// TPW neighbouring column blocks per workgroup: the loads of the next one are issued into the registers that each
// half of the exchange has just written to LDS (see k_enc_hix_last).
template <int M, int TPW>
__global__ __launch_bounds__(HiX<M>::THREADS) void k_hix_mid(float *T, int log2D, uint64_t load_elems, uint64_t store_elems) {
    using X = HiX<M>;
    __shared__ float lds[X::LDS_FLOATS];
    constexpr int p = kHixP;
    const uint32_t tile0 = blockIdx.x * TPW;                     // the TPW tiles lie in the same 2^(p+M) block
    const uint64_t base0 = hix_base<M>(tile0, p);
    const uint64_t block_start = base0 >> (p + M) << (p + M);
    if (block_start >= load_elems || block_start >= store_elems) return;     // same decision in the whole workgroup
    const uint32_t col = threadIdx.x & 31u, g = threadIdx.x >> 5;
    const rsrc_t rl = make_rsrc(T + ((size_t)blockIdx.y << log2D), (uint32_t)(load_elems * 4));
    const rsrc_t rs = make_rsrc(T + ((size_t)blockIdx.y << log2D), (uint32_t)(store_elems * 4));
    const uint32_t off1 = ((g << p) + col) * 4u;
    const uint32_t off2 = (((g * X::RHL * X::RL) << p) + col) * 4u;
    float v[64];
#pragma unroll
    for (int r = 0; r < 64; ++r) v[r] = buf_load(rl, off1, (uint32_t)base0 * 4u + (((uint32_t)X::RL * r) << (p + 2)));
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
        const uint32_t base_off = (uint32_t)hix_base<M>(tile0 + k, p) * 4u;
        const uint32_t next_off = (uint32_t)hix_base<M>(tile0 + k + 1, p) * 4u;
        fwht_regs<64>(v);
        float out[X::RP];
#pragma unroll
        for (int ph = 0; ph < X::PH; ++ph) {
            if (ph == 0) hix_exchange_write<M, 0>(v, lds);
            else hix_exchange_write<M, X::PH - 1>(v, lds);
            if (k + 1 < TPW) {
#pragma unroll
                for (int r = ph * X::RP; r < (ph + 1) * X::RP; ++r)
                    v[r] = buf_load(rl, off1, next_off + (((uint32_t)X::RL * r) << (p + 2)));
            }
            hix_exchange_read<M>(lds, out);
#pragma unroll
            for (int s = 0; s < X::RP; ++s) buf_store(rs, off2, base_off + (hix_row2<M>(0, ph, s) << (p + 2)), out[s]);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Decode runs the strided passes first and the contiguous pass last.  The first pass has no dependency
// between senders, so every (tile, sender) pair is its own workgroup; the last pass sums the senders in
// registers and touches acc once, with fully contiguous accesses.

// First decode pass (Sec. 2.2.2, 4.2): unpack, centroid lookup times S/(p sqrt D) (or the unit pattern when the
// workspace is fp16), zero for coordinates that were not sampled or whose packet was lost, then index bits
// 14 .. 14+M-1 of H.
// ONLY != 0: every sender of the launch has this budget (2, 3 or 4 bits, or k + 1/2; indices in the payload): the instance then
// holds that one branch, which takes it from 128 registers and spills to 97 (16 senders at D = 2^24: 0.180 -> 0.160 ms).
template <int M, uint32_t ONLY = 0>
__global__ __launch_bounds__(HiX<M>::THREADS, 4) void k_dec_hix_first(DecBatch B, uint64_t d, int log2D, uint64_t seed,
                                                                    const DecScratch *scratch, int narrow, float *T,
                                                                    CoinTables ct) {
    using X = HiX<M>;
    constexpr int p = kHixP;
    __shared__ float lds[X::LDS_FLOATS];
    __shared__ float table[32];
    __shared__ float gtab[kGridMax + 1];                         // uniform grid: dequantized centres of mass
    const uint32_t c = blockIdx.y;
    const uint32_t b_q8 = ONLY ? ONLY : B.b_q8[c];
    uint32_t tile = xcd_local_tile();
    {   // payload bytes of one tile row: 4 per index bit; the budgets with a power of two (2, 4, 8 bits) get aligned runs
        int tb, tk;
        budget_of(b_q8, tb, tk);
        if (tk == 1 && (tb == 2 || tb == 4 || tb == 8) && !B.codes[c])
            tile = align_runs_to_lines(tile, p - 5, static_cast<const char *>(B.msg[c]) + EDEN_HEADER_BYTES, 4u * (uint32_t)tb);
    }
    const uint64_t base = hix_base<M>(tile, p);
    const uint32_t col = threadIdx.x & 31u, g = threadIdx.x >> 5, lane = lane_id();
    const uint32_t g0 = 2u * wave_in_block();
    const bool i16 = narrow && b_q8 <= 256u;
    const DecScratch *sc = &scratch[c];
    if (threadIdx.x < 16) table[threadIdx.x] = (i16 && threadIdx.x == 1) ? 1.0f : sc->deq[threadIdx.x];
    else if (threadIdx.x < 32) table[threadIdx.x] = sc->deq2[threadIdx.x - 16];
    if (byte_budget(b_q8))
        for (uint32_t i = threadIdx.x; i <= (uint32_t)kGridMax; i += X::THREADS) gtab[i] = sc->grid_deq[i];
    __syncthreads();
    const uint32_t *payload = reinterpret_cast<const uint32_t *>(static_cast<const char *>(B.msg[c]) + EDEN_HEADER_BYTES);
    int bits, k;
    budget_of(b_q8, bits, k);
    const uint32_t payload_bytes = (uint32_t)(((((1ull << log2D) >> (k == 2)) * (uint32_t)bits + 63) >> 6) << 3);

    // rows of this wave whose packet arrived, as lane masks over the register index (bit r <-> register r)
    const uint64_t row_a = (uint64_t)hix_row1<M>(g0, lane) << p, row_b = (uint64_t)hix_row1<M>(g0 + 1, lane) << p;
    uint64_t recv_a = ~0ull, recv_b = ~0ull;
    const uint32_t *bm = B.bitmap[c];
    if (bm) {
        const uint32_t pa = (uint32_t)((base + row_a) >> 10), pb = (uint32_t)((base + row_b) >> 10);
        recv_a = __ballot((bm[pa >> 5] >> (pa & 31u)) & 1u);
        recv_b = __ballot((bm[pb >> 5] >> (pb & 31u)) & 1u);
    }
    float v[64];
    if (b_q8 == 128) {
        // b = 1/2: pair j = i >> 1 carries one bit; coordinate i was sent iff (i & 1) equals the pair's offset bit
        const uint64_t key = stream_key(seed, kStreamSubsample, B.client[c]);
        const uint32_t sh = 16u * (uint32_t)((base >> 5) & 3u);                  // this tile's 16 pairs inside a hash word
        const uint32_t fa = (uint32_t)(hash_word(key, (base + row_a) >> 7) >> sh) & 0xFFFFu;
        const uint32_t fb = (uint32_t)(hash_word(key, (base + row_b) >> 7) >> sh) & 0xFFFFu;
        const uint32_t both = fa | (fb << 16);
        const rsrc_t rp = make_rsrc(payload + (base >> 6), payload_bytes - (uint32_t)(base >> 6) * 4u);
        const uint32_t voff = (g << (p - 6)) * 4u;
        const uint32_t bitpos = 16u * (uint32_t)((base >> 5) & 1u) + (col >> 1);
        const uint32_t mag = __float_as_uint(table[1]);
#pragma unroll
        for (int r = 0; r < 64; ++r) {
            const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, (int)((((uint32_t)X::RL * r) << (p - 6)) * 4u), 0);
            const uint32_t offs = __builtin_amdgcn_readlane(both, r) >> (16u * (lane >> 5));
            const bool kept = ((offs >> (col >> 1)) & 1u) == (col & 1u);
            const uint32_t neg = (~(w >> bitpos) & 1u) << 31;                    // index 0 = negative
            v[r] = kept ? __uint_as_float(mag | neg) : 0.0f;
        }
    } else if (byte_budget(b_q8)) {
        // one byte per coordinate: the index on the uniform grid (Sec. 4.3) or of a 32..256-level quantizer
        const uint8_t *bytes = B.codes[c] ? B.codes[c] : reinterpret_cast<const uint8_t *>(payload);
        const rsrc_t rp = make_rsrc(bytes + base, (1u << log2D) - (uint32_t)base);
        const uint32_t voff = (g << p) + col;
#pragma unroll
        for (int r = 0; r < 64; ++r) v[r] = __uint_as_float(buf_load_byte(rp, voff, ((uint32_t)X::RL * r) << p));
        const uint32_t H = wide_half_levels(b_q8);
        if (grid_q15(b_q8)) {                                    // the values replace the bytes in their registers
#pragma unroll
            for (int r = 0; r < 64; ++r) v[r] = dequantize_byte<true>(__float_as_uint(v[r]), H, gtab);
        } else {
#pragma unroll
            for (int r = 0; r < 64; ++r) v[r] = dequantize_byte<false>(__float_as_uint(v[r]), H, gtab);
        }
    } else if (coin_q8(b_q8)) {
        // coin budgets (Sec. 4.1): every coordinate has `bits` bits in the first part; a coordinate with a coin was
        // quantized with the finer table and has its top bit in the second part, at the position of its rank among the
        // coins.  Lane l fetches the coins of the two row segments the wave reads into register l.
        const uint32_t upper = (uint32_t)(base >> 5) & 1u;       // which half of a block of 64 coordinates this tile's columns are
        const uint32_t blk_a = (uint32_t)((base + row_a) >> 6), blk_b = (uint32_t)((base + row_b) >> 6);
        const uint64_t m64_a = coin_mask_of(ct, c, log2D, blk_a), m64_b = coin_mask_of(ct, c, log2D, blk_b);
        const uint32_t ma = upper ? hi32(m64_a) : lo32(m64_a), mb = upper ? hi32(m64_b) : lo32(m64_b);
        const uint32_t oa = coins_before(ct, c, log2D, blk_a) + (upper ? (uint32_t)__popc(lo32(m64_a)) : 0u);
        const uint32_t ob = coins_before(ct, c, log2D, blk_b) + (upper ? (uint32_t)__popc(lo32(m64_b)) : 0u);
        const uint32_t cbits = col * (uint32_t)bits;
        const rsrc_t rp = make_rsrc(payload + ((base * (uint32_t)bits) >> 5), payload_bytes - (uint32_t)((base * (uint32_t)bits) >> 5) * 4u);
        const uint32_t voff = (((g * (uint32_t)bits) << (p - 5)) + (cbits >> 5)) * 4u;
        const uint32_t shift = cbits & 31u;
        const rsrc_t rb = make_rsrc(payload + payload_bytes / 4u, (uint32_t)coin_b_bytes(ct.total[c]));
        const uint32_t below = (1u << col) - 1u;
        // the top bits of a row segment's coins are at most 32 consecutive bits of the second part, from bit oa (ob) on: this
        // lane fetches them for "its" two rows once (beyond the part: 0), and every lane finds its bit in the window
        auto window = [&](uint32_t first_bit) {
            const uint32_t lo = __builtin_amdgcn_raw_buffer_load_b32(rb, (int)((first_bit >> 5) * 4u), 0, 0);
            const uint32_t hi = __builtin_amdgcn_raw_buffer_load_b32(rb, (int)((first_bit >> 5) * 4u + 4u), 0, 0);
            return __builtin_amdgcn_alignbit(hi, lo, first_bit & 31u);
        };
        const uint32_t wa = window(oa), wb = window(ob);
#pragma unroll
        for (int r = 0; r < 64; ++r) {
            const int soff = (int)((((uint32_t)X::RL * r * (uint32_t)bits) << (p - 5)) * 4u);
            const uint32_t w0 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, soff, 0);
            const uint32_t w1 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff + 4, soff, 0);    // always: no branch per value
            const uint32_t low = code_at(w0, w1, shift, bits);
            const uint32_t m = (lane < 32u) ? __builtin_amdgcn_readlane(ma, r) : __builtin_amdgcn_readlane(mb, r);
            const uint32_t wnd = (lane < 32u) ? __builtin_amdgcn_readlane(wa, r) : __builtin_amdgcn_readlane(wb, r);
            const uint32_t top = (wnd >> (uint32_t)__popc(m & below)) & 1u;
            v[r] = ((m >> col) & 1u) ? table[16u + ((top << bits) | low)] : table[low];
        }
    } else if (budget_mixed(b_q8)) {
        // b = bits + 1/2 (Sec. 4.1): every coordinate has `bits` bits in the first part; the coordinate of each pair
        // that the MIX stream selects was quantized with the finer table and has its top bit in the second part
        const uint64_t key = stream_key(seed, kStreamMix, B.client[c]);
        const uint32_t sh = 16u * (uint32_t)((base >> 5) & 3u);                  // this tile's 16 pairs inside a hash word
        const uint32_t fa = (uint32_t)(hash_word(key, (base + row_a) >> 7) >> sh) & 0xFFFFu;
        const uint32_t fb = (uint32_t)(hash_word(key, (base + row_b) >> 7) >> sh) & 0xFFFFu;
        const uint32_t both = fa | (fb << 16);
        const uint32_t cbits = col * (uint32_t)bits;
        const rsrc_t rp = make_rsrc(payload + ((base * (uint32_t)bits) >> 5), payload_bytes - (uint32_t)((base * (uint32_t)bits) >> 5) * 4u);
        const uint32_t voff = (((g * (uint32_t)bits) << (p - 5)) + (cbits >> 5)) * 4u;
        const uint32_t shift = cbits & 31u;
        // second part: 16 bits per row segment; the descriptor starts at the part (8-byte aligned) so that the
        // half-words can be fetched as whole dwords
        const rsrc_t rb = make_rsrc(payload + payload_bytes / 4u, (uint32_t)payload_b_bytes(1ull << log2D, b_q8));
        const uint32_t voffb = ((uint32_t)(base >> 5) + (g << (p - 5))) * 2u;
#pragma unroll
        for (int r = 0; r < 64; ++r) {
            const int soff = (int)((((uint32_t)X::RL * r * (uint32_t)bits) << (p - 5)) * 4u);
            const uint32_t w0 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, soff, 0);
            const uint32_t w1 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff + 4, soff, 0);    // always: no branch per value
            const uint32_t low = code_at(w0, w1, shift, bits);
            const uint32_t hb = buf_load_half(rb, voffb, (((uint32_t)X::RL * r) << (p - 5)) * 2u);
            const uint32_t offs = __builtin_amdgcn_readlane(both, r) >> (16u * (lane >> 5));
            const bool up = ((offs >> (col >> 1)) & 1u) == (col & 1u);
            const uint32_t top = (hb >> (col >> 1)) & 1u;
            v[r] = up ? table[16u + ((top << bits) | low)] : table[low];
        }
    } else {
        const uint32_t cbits = col * (uint32_t)bits;
        const rsrc_t rp = make_rsrc(payload + ((base * (uint32_t)bits) >> 5), payload_bytes - (uint32_t)((base * (uint32_t)bits) >> 5) * 4u);
        const uint32_t voff = (((g * (uint32_t)bits) << (p - 5)) + (cbits >> 5)) * 4u;
        const uint32_t shift = cbits & 31u;
        if (b_q8 == 256) {
            const uint32_t mag = __float_as_uint(table[1]);
#pragma unroll
            for (int r = 0; r < 64; ++r) {
                const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, (int)((((uint32_t)X::RL * r) << (p - 5)) * 4u), 0);
                v[r] = __uint_as_float(mag | ((~(w >> shift) & 1u) << 31));
            }
        } else if (b_q8 == 512) {
#pragma unroll
            for (int r = 0; r < 64; ++r) {
                const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, (int)((((uint32_t)X::RL * r * 2u) << (p - 5)) * 4u), 0);
                v[r] = table[(w >> shift) & 3u];
            }
        } else if (b_q8 == 768) {                                // an index may straddle two words
#pragma unroll
            for (int r = 0; r < 64; ++r) {
                const int soff = (int)((((uint32_t)X::RL * r * 3u) << (p - 5)) * 4u);
                const uint32_t w0 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, soff, 0);
                const uint32_t w1 = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff + 4, soff, 0);
                v[r] = table[code_at(w0, w1, shift, 3)];
            }
        } else {
#pragma unroll
            for (int r = 0; r < 64; ++r) {
                const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, (int)((((uint32_t)X::RL * r * 4u) << (p - 5)) * 4u), 0);
                v[r] = table[(w >> shift) & 15u];
            }
        }
    }
    if (bm) {
#pragma unroll
        for (int r = 0; r < 64; ++r) {
            const uint64_t m = (((recv_a >> r) & 1ull) ? 0x00000000FFFFFFFFull : 0ull) |
                               (((recv_b >> r) & 1ull) ? 0xFFFFFFFF00000000ull : 0ull);
            v[r] = keep_where(v[r], m);
        }
    }
    fwht_regs<64>(v);
    const uint32_t base_off = (uint32_t)base * 4u;
    const uint32_t off2 = (((g * X::RHL * X::RL) << p) + col) * 4u;
    const char *slot = reinterpret_cast<const char *>(T + ((size_t)c << log2D));
    // rows at or above ceil(d / 2^14) are never read by the last pass: the bounds drop their stores
    const uint32_t rows_used = (uint32_t)((d + (1u << p) - 1) >> p);
    float out[X::RP];
    if (i16) {
        // exact integers of magnitude <= 2^M: fp16 at the same element index
        const rsrc_t rt = make_rsrc(slot + (base_off >> 1), (rows_used << (p + 1)) - (base_off >> 1));
        hix_exchange<M, 0>(v, lds, out);
#pragma unroll
        for (int s = 0; s < X::RP; ++s)
            __builtin_amdgcn_raw_buffer_store_b16(narrow_bits(out[s]), rt, (int)(off2 >> 1), (int)((hix_row2<M>(0, 0, s) << (p + 2)) >> 1), kStream);
        if constexpr (X::PH == 2) {
            hix_exchange<M, 1>(v, lds, out);
#pragma unroll
            for (int s = 0; s < X::RP; ++s)
                __builtin_amdgcn_raw_buffer_store_b16(narrow_bits(out[s]), rt, (int)(off2 >> 1), (int)((hix_row2<M>(0, 1, s) << (p + 2)) >> 1), kStream);
        }
    } else {
        const rsrc_t rt = make_rsrc(slot + base_off, (rows_used << (p + 2)) - base_off);
        hix_exchange<M, 0>(v, lds, out);
#pragma unroll
        for (int s = 0; s < X::RP; ++s) buf_store(rt, off2, hix_row2<M>(0, 0, s) << (p + 2), out[s]);
        if constexpr (X::PH == 2) {
            hix_exchange<M, 1>(v, lds, out);
#pragma unroll
            for (int s = 0; s < X::RP; ++s) buf_store(rt, off2, hix_row2<M>(0, 1, s) << (p + 2), out[s]);
        }
    }
}

// First decode pass for senders with b <= 1, two columns per thread.  The unit pattern is +-1 or 0 and M <= 10
// stages keep every value within +-1024, so the whole pass runs on pairs of int16 packed in one register
// (v_pk_add_i16 / v_pk_sub_i16: two butterflies per instruction) and a tile is 64 columns wide: the workspace
// is written in 128-byte segments, each pair converted to fp16 (the narrow workspace's type) just before its store.
typedef short s16x2 __attribute__((ext_vector_type(2)));

template <int N, int LOGB>
__device__ inline void fwht_pk(s16x2 (&v)[N]) {
#pragma unroll
    for (int h = 1; h < (1 << LOGB); h <<= 1) {
#pragma unroll
        for (int i = 0; i < N; i += 2 * h) {
#pragma unroll
            for (int j = i; j < i + h; ++j) {
                const s16x2 a = v[j], b = v[j + h];
                v[j] = a + b;
                v[j + h] = a - b;
            }
        }
    }
}

// (Four waves per SIMD are requested so that two of the 512-thread workgroups of M = 10 share a CU: measured
// 0.103 ms against 0.133 ms per launch on 16 senders at D = 2^24, at the price of five spilled registers.)
template <int M>
__global__ __launch_bounds__(HiX<M>::THREADS, 4) void k_dec_hix_first_pk(DecBatch B, uint64_t d, int log2D, uint64_t seed, float *T) {
    using X = HiX<M>;
    constexpr int p = kHixP;
    __shared__ uint32_t lds[X::LDS_FLOATS];
    const uint32_t c = blockIdx.y;
    const uint32_t b_q8 = B.b_q8[c];
    const uint32_t *payload = reinterpret_cast<const uint32_t *>(static_cast<const char *>(B.msg[c]) + EDEN_HEADER_BYTES);
    // 64-column blocks: 2^(p-6) of them per row, 8 (b = 1) or 4 (b = 1/2) payload bytes per row each
    const uint32_t tile = align_runs_to_lines(xcd_local_tile(), p - 6, payload, b_q8 == 256u ? 8u : 4u);
    const uint32_t cb = tile & ((1u << (p - 6)) - 1u), upper = tile >> (p - 6);
    const uint64_t base = ((uint64_t)upper << (p + M)) | ((uint64_t)cb << 6);
    const uint32_t cp = threadIdx.x & 31u, g = threadIdx.x >> 5, lane = lane_id();
    const uint32_t g0 = 2u * wave_in_block();
    const uint32_t payload_bytes = (uint32_t)(((((1ull << log2D) >> (b_q8 == 128u)) + 63) >> 6) << 3);
    const uint64_t row_a = (uint64_t)hix_row1<M>(g0, lane) << p, row_b = (uint64_t)hix_row1<M>(g0 + 1, lane) << p;
    uint64_t recv_a = ~0ull, recv_b = ~0ull;                     // bit r: did the packet of register r's row arrive
    const uint32_t *bm = B.bitmap[c];
    if (bm) {
        const uint32_t pa = (uint32_t)((base + row_a) >> 10), pb = (uint32_t)((base + row_b) >> 10);
        recv_a = __ballot((bm[pa >> 5] >> (pa & 31u)) & 1u);
        recv_b = __ballot((bm[pb >> 5] >> (pb & 31u)) & 1u);
    }
    uint32_t v32[64];
    if (b_q8 == 256) {
        // the two index bits of columns 2cp, 2cp+1 -> (+-1, +-1); index 1 = non-negative
        const rsrc_t rp = make_rsrc(payload + (base >> 5), payload_bytes - (uint32_t)(base >> 5) * 4u);
        const uint32_t voff = ((g << (p - 5)) + (cp >> 4)) * 4u;
        const uint32_t sh = 2u * (cp & 15u);
#pragma unroll
        for (int r = 0; r < 64; ++r) {
            const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, (int)((((uint32_t)X::RL * r) << (p - 5)) * 4u), 0);
            const uint32_t x = w >> sh;
            v32[r] = 0xFFFFFFFFu ^ (((x & 1u) * 0xFFFEu) | ((x & 2u) * 0x7FFF0000u));
        }
    } else {
        // b = 1/2: the pair (2cp, 2cp+1) carries one bit; the offset bit of the sub-sampling stream says which one
        const uint64_t key = stream_key(seed, kStreamSubsample, B.client[c]);
        const uint32_t hs = 32u * (uint32_t)((base >> 6) & 1u);
        const uint32_t fa = (uint32_t)(hash_word(key, (base + row_a) >> 7) >> hs);
        const uint32_t fb = (uint32_t)(hash_word(key, (base + row_b) >> 7) >> hs);
        const rsrc_t rp = make_rsrc(payload + (base >> 6), payload_bytes - (uint32_t)(base >> 6) * 4u);
        const uint32_t voff = (g << (p - 6)) * 4u;
#pragma unroll
        for (int r = 0; r < 64; ++r) {
            const uint32_t w = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)voff, (int)((((uint32_t)X::RL * r) << (p - 6)) * 4u), 0);
            const uint32_t offs = (lane < 32u) ? __builtin_amdgcn_readlane(fa, r) : __builtin_amdgcn_readlane(fb, r);
            const uint32_t val = ((w >> cp) & 1u) ? 0x0001u : 0xFFFFu;           // +1 or -1 as int16
            v32[r] = ((offs >> cp) & 1u) ? (val << 16) : val;
        }
    }
    if (bm) {
#pragma unroll
        for (int r = 0; r < 64; ++r) {
            const uint64_t m = (((recv_a >> r) & 1ull) ? 0x00000000FFFFFFFFull : 0ull) |
                               (((recv_b >> r) & 1ull) ? 0xFFFFFFFF00000000ull : 0ull);
            v32[r] = __float_as_uint(keep_where(__uint_as_float(v32[r]), m));
        }
    }
    s16x2 v[64];
#pragma unroll
    for (int r = 0; r < 64; ++r) v[r] = __builtin_bit_cast(s16x2, v32[r]);
    fwht_pk<64, 6>(v);
    // element i of the sender's slot (fp16) sits at byte 2 i: the pair of this thread is one 32-bit store, converted last
    char *slot = reinterpret_cast<char *>(T + ((size_t)c << log2D)) + base * 2u;
    // rows at or above ceil(d / 2^14) are never read by the last pass: the bounds drop their stores
    const uint32_t rows_used = (uint32_t)((d + (1u << p) - 1) >> p);
    const rsrc_t rt = make_rsrc(slot, (rows_used << (p + 1)) - (uint32_t)base * 2u);
    const uint32_t off2 = (((g * X::RHL * X::RL) << p) * 2u) + cp * 4u;
    const uint32_t col = cp;                                     // exchange slot of this thread
#pragma unroll
    for (int ph = 0; ph < X::PH; ++ph) {
#pragma unroll
        for (int i = 0; i < X::RP; ++i) lds[(i * X::RL + g) * 32 + col] = __builtin_bit_cast(uint32_t, v[ph * X::RP + i]);
        __syncthreads();
        s16x2 out[X::RP];
#pragma unroll
        for (int s2 = 0; s2 < X::RP; ++s2) {
            const int e = s2 / X::RL, rl = s2 % X::RL;
            out[s2] = __builtin_bit_cast(s16x2, lds[((g * X::RHL + e) * X::RL + rl) * 32 + col]);
        }
        __syncthreads();
        fwht_pk<X::RP, M - 6>(out);
#pragma unroll
        for (int s2 = 0; s2 < X::RP; ++s2)
            __builtin_amdgcn_raw_buffer_store_b32(narrow_pair_from_int16(__builtin_bit_cast(uint32_t, out[s2])), rt, (int)off2,
                                                  (int)((hix_row2<M>(0, ph, s2) << p) * 2u), kStream);
    }
}

// First decode pass of a b = 1 round at D = 2^24 (ten strided bits) on the matrix cores: index bits 14..23 of the H in
// R^-1 = s o D^-1/2 H (Sec. 2.2.2) applied to the unit pattern of the payload (+-1 per coordinate, I_1 of Sec. 3; 0 where the
// packet was lost, Sec. 4.2).  The factor S / (p sqrt(D)) q_1 waits for the last pass.
//
// A tile is 64 columns x 1024 rows; the input is one payload bit per element (+1 for a set bit, 0 where the packet was
// lost).  Row rho = 32 i + k.  For ONE column the 1024 values are a 32 x 32 matrix X[i][k] and the transform is H X H:
//   step 1  D1[i][k'] = sum_k X[i][k] H[k][k']   v_mfma_f32_32x32x16_fp8_fp8 twice: X as the A operand, fp8 bytes 0x38 / 0xB8 / 0
//                                                (+1 / -1 / 0 in e4m3), built from the payload bits with shifts and masks;
//   step 2  D2[i'][k'] = sum_i H[i'][i] D1[i][k']  the result registers of step 1, packed to fp16 (|D1| <= 32: exact), are the
//                                                B operands of two v_mfma_f32_32x32x16_f16 (see hadamard_rows_of_result).
// Every sum is an integer of magnitude at most 1024: exact.  A wave handles eight neighbouring columns = one byte of each
// row's payload word: the bytes of four rows are gathered into one register (three byte permutes per four rows, once per
// tile), and column t of the eight is one shift and one and-or away from an operand register.
// The 2-byte results of a column lie 32 KiB apart in the workspace, so the tile goes through LDS (16-byte chunks swizzled by
// the row: conflict free both ways) and leaves in 128-byte row segments, 16 bytes per lane.  64 columns x 1024 rows of fp16
// are 128 KiB, twice what two workgroups per CU can have: the tile is computed twice (the matrix cores and the operand
// building are cheap) and each time only the rows of one half (i' < 16, i' >= 16) are kept and written.
// Vector instructions per element: about 2.5 (operands 1, packing D1 1, packing the results 0.5) against 10 in the packed
// int16 version; the pass is then bound by its stores.
constexpr uint32_t kFp8One = 0x38383838u, kFp8Sign = 0x80808080u;
constexpr int kPayRow = 33;                                      // LDS stride of the staged payload words: 32 + 1

// The two Hadamard operands of the pass, per lane l = 32 h + m, built by the compiler: words 0..3 the fp8 B operand of step 1
// (two instructions q of 8 bytes: entry e is H[k][k'] with k = 16 q + 8 h + e, k' = m), words 4..11 the fp16 A operand of
// step 2 (two instructions of 8 halves, rows in the order hadamard_rows_of_result documents).  Loading twelve words costs a
// lane nothing next to computing 32 parities.
struct FirstPassOperands { uint32_t w[64][12]; };
constexpr uint32_t parity_of(uint32_t x) { x ^= x >> 16; x ^= x >> 8; x ^= x >> 4; x ^= x >> 2; x ^= x >> 1; return x & 1u; }
constexpr FirstPassOperands make_first_pass_operands() {
    FirstPassOperands t{};
    for (uint32_t l = 0; l < 64; ++l) {
        const uint32_t h = l >> 5, m = l & 31u;
        for (uint32_t q = 0; q < 2; ++q)
            for (uint32_t e = 0; e < 8; ++e) {
                const uint32_t k = 16u * q + 8u * h + e;
                t.w[l][2 * q + (e >> 2)] |= (0x38u | (parity_of(k & m) << 7)) << (8 * (e & 3));
                const uint32_t row = 16u * q + 8u * (e >> 2) + 4u * h + (e & 3u);
                t.w[l][4 + 4 * q + (e >> 1)] |= (0x3C00u | (parity_of(row & m) << 15)) << (16 * (e & 1));       // fp16 +-1
            }
    }
    return t;
}
__device__ const FirstPassOperands kFirstPassOperands = make_first_pass_operands();

// TPW neighbouring tiles per workgroup, one after the other: the Hadamard operands are built once, and the payload of the
// next tile is fetched while this one is computed.
// PREP: the first workgroup of every sender also does what k_dec_prepare does for that sender (nothing in this pass
// depends on it; the last pass, a later launch, reads it).
// HALF: every sender of the launch has b = 1/2 with the sub-sampling after the rotation (Sec. 4.1): a row's 64 columns are
// 32 pairs with one payload bit each, and the SUBSAMPLE stream says which member of a pair the bit belongs to; the other
// member is 0.  The operand bytes are then sign | magnitude with the magnitude 0x40 (2.0: one bit, so that a shift and a
// mask make it from the presence bit) or 0, and the Hadamard operand of step 2 holds +-1/2 instead of +-1.
// M < 10 (D = 2^22, 2^23: 256 or 512 rows): the same products with the missing rows as zeros.  Row 32 i + k belongs to A row
// i = lane m of step 1, so lanes m >= 2^(M-5) supply zero operands (their sign mask and magnitude are 0), the results with
// i' < 2^(M-5) are the transform over M bits, and the rest (copies of them) is not stored.  The matrix cores and the operand
// building then work 2^(10-M) times per stored byte, which the pass has room for.
template <bool LOSS, int TPW, bool PREP, bool HALF, int M>
__global__ __launch_bounds__(512, 4) void k_dec_hix_first_mfma(DecBatch B, uint64_t d, int log2D, uint64_t seed, float *T,
                                                               DecPrepareArgs prep) {
    static_assert(M >= 8 && M <= 10, "rows of the tile");
    constexpr uint32_t kRows = 1u << M;
    constexpr int p = kHixP;
    __shared__ __attribute__((aligned(16))) uint32_t out_lds[512 * 32];          // one half of the tile: 512 rows x 128 bytes
    __shared__ uint32_t pay_lds[(LOSS ? 3 : 2) * 32 * kPayRow];                  // payload word 0, word 1 (, arrived) of every row
    const uint32_t c = blockIdx.y, t = threadIdx.x, lane = t & 63u, wv = wave_in_block(), h = lane >> 5, m = lane & 31u;
    const uint32_t *payload = reinterpret_cast<const uint32_t *>(static_cast<const char *>(B.msg[c]) + EDEN_HEADER_BYTES);
    const uint32_t tile0 = xcd_local_tile<16 / TPW>() * TPW;
    const rsrc_t rp = make_rsrc(payload, 1u << (log2D - (HALF ? 4 : 3)));
    const uint32_t *bm = LOSS ? B.bitmap[c] : nullptr;
    const uint64_t subkey = HALF ? stream_key(seed, kStreamSubsample, B.client[c]) : 0ull;
    if constexpr (PREP) {
        if (blockIdx.x == 0 && wv == 0)
            dec_prepare_wave(B.msg[c], B.bitmap[c], B.client[c], B.b_q8[c], B.hdr_b_q8[c], prep.hdr_d, log2D, prep.seed, prep.tab,
                             &prep.scratch[c], prep.dev_status, 0u, prep.msg_flags ? prep.msg_flags + c : nullptr);
    }
    auto column_block = [&](uint32_t k) {
        return align_runs_to_lines(tile0 + k, p - 6, payload, HALF ? 4u : 8u) & ((1u << (p - 6)) - 1u);
    };
    // the tile's 8 payload bytes of rows t and t + 512 (and whether their packets arrived); HALF: 4 payload bytes, and the
    // tile's half of the row's word of the SUBSAMPLE stream (64 pairs per word)
    auto fetch = [&](uint32_t cb, uint32_t (&w)[2][2], uint32_t (&arrived)[2]) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t row = t + 512u * (uint32_t)j;
            if constexpr (HALF) {
                w[j][0] = __builtin_amdgcn_raw_buffer_load_b32(rp, (int)(row << (p - 4)), (int)(cb * 4u), 0);
                w[j][1] = (uint32_t)(hash_word(subkey, (((uint64_t)row << p) + cb * 64u) >> 7) >> (32u * (cb & 1u)));
            } else {
                const auto w2 = __builtin_amdgcn_raw_buffer_load_b64(rp, (int)(row << (p - 3)), (int)(cb * 8u), 0);
                w[j][0] = w2[0]; w[j][1] = w2[1];
            }
            arrived[j] = 0xFFFFFFFFu;
            if constexpr (LOSS) {
                const uint32_t pa = (row << (p - 10)) + (cb >> 4);                  // packet of 1024 coordinates that holds this row's 64
                arrived[j] = (row < kRows && (!bm || ((bm[pa >> 5] >> (pa & 31u)) & 1u))) ? 0xFFFFFFFFu : 0u;
            }
        }
    };

    // the two Hadamard operands (kFirstPassOperands)
    long Hk[2];
    half8_t Hn[2];
    {
        const u32x4_t *mine = reinterpret_cast<const u32x4_t *>(kFirstPassOperands.w[lane]);
        const u32x4_t k01 = mine[0], n0 = mine[1], n1 = mine[2];
        Hk[0] = (long)(((uint64_t)k01[1] << 32) | k01[0]);
        Hk[1] = (long)(((uint64_t)k01[3] << 32) | k01[2]);
        Hn[0] = __builtin_bit_cast(half8_t, HALF ? n0 - 0x04000400u : n0);       // fp16 +-1 -> +-1/2: one off the exponent
        Hn[1] = __builtin_bit_cast(half8_t, HALF ? n1 - 0x04000400u : n1);
    }
    // rows at or above ceil(d / 2^14) are never read by the last pass: the buffer bounds drop their stores (leaving them out
    // of the exchange as well would take branches that cost more registers than the kernel has)
    const uint32_t rows_used = (uint32_t)((d + (1u << p) - 1) >> p);
    const rsrc_t rt = make_rsrc(T + ((size_t)c << log2D), rows_used << (p + 1));
    const bool row_exists = m < (kRows >> 5);                    // A row i = m of step 1 holds rows 32 m + k of the tile
    uint32_t one = row_exists ? kFp8One : 0u;                    // in a vector register: shift, and-or are then two instructions
    asm volatile("" : "+v"(one));
    const uint32_t sign_mask = row_exists ? kFp8Sign : 0u, two_mask = row_exists ? 0x40404040u : 0u;
    const uint32_t dc = wv >> 2, cbyte = wv & 3u;                // this wave's eight columns: byte cbyte of payload word dc

    uint32_t next_w[2][2], next_arrived[2];
    fetch(column_block(0), next_w, next_arrived);
#pragma unroll 1
    for (uint32_t k = 0; k < (uint32_t)TPW; ++k) {
        const uint32_t cb = column_block(k);
        // ---- staged so that lane m of a wave finds row 32 m + k at k * 33 + m (the last reads of the previous tile's
        // words lie three barriers back)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t row = t + 512u * (uint32_t)j;
            const uint32_t at = (row & 31u) * kPayRow + (row >> 5);
            pay_lds[at] = next_w[j][0];
            pay_lds[32 * kPayRow + at] = next_w[j][1];
            if constexpr (LOSS) pay_lds[2 * 32 * kPayRow + at] = next_arrived[j];
        }
        __syncthreads();                                         // also: every wave has read the previous tile's second half
        if (k + 1 < (uint32_t)TPW) fetch(column_block(k + 1), next_w, next_arrived);

        // ---- this wave's byte of this lane's 16 rows, four rows per register
        uint32_t Gn[2][2], Z[2][2];                              // [instruction q][rows 4 eps .. 4 eps + 3 of its eight]
        uint32_t Pn[2][2];                                       // HALF: bit t of a byte = column t of that row holds a value
        if constexpr (HALF) {
            // this wave's eight columns are four pairs: nibble 4 dc + cbyte of the row's payload word and of its offsets
            const uint32_t nib = 4u * dc + cbyte, bsel = nib >> 1, nsh = 4u * (nib & 1u);
            const uint32_t sel = 0x0C0C0000u | ((4u + bsel) << 8) | bsel;
            auto pairs_to_columns = [](uint32_t x) {             // bit g of every byte's low nibble -> bit 2 g of the byte
                x = (x | (x << 2)) & 0x33333333u;
                return (x | (x << 1)) & 0x55555555u;
            };
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int eps = 0; eps < 2; ++eps) {
                    uint32_t w[4], f[4], z[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t at = (16u * q + 8u * h + 4u * eps + e) * kPayRow + m;
                        w[e] = pay_lds[at];
                        f[e] = pay_lds[32 * kPayRow + at];
                        z[e] = LOSS ? pay_lds[2 * 32 * kPayRow + at] : 0u;
                    }
                    const uint32_t gw = __builtin_amdgcn_perm(__builtin_amdgcn_perm(w[3], w[2], sel), __builtin_amdgcn_perm(w[1], w[0], sel), 0x05040100u);
                    const uint32_t gf = __builtin_amdgcn_perm(__builtin_amdgcn_perm(f[3], f[2], sel), __builtin_amdgcn_perm(f[1], f[0], sel), 0x05040100u);
                    const uint32_t bits = pairs_to_columns((gw >> nsh) & 0x0F0F0F0Fu), second = pairs_to_columns((gf >> nsh) & 0x0F0F0F0Fu);
                    Gn[q][eps] = ~(bits | (bits << 1));          // both members carry the pair's bit; a set bit is +1: sign clear
                    Pn[q][eps] = (second << 1) | (second ^ 0x55555555u);          // the second member where the offset bit is set
                    Z[q][eps] = 0xFFFFFFFFu;
                    if constexpr (LOSS)
                        Pn[q][eps] &= __builtin_amdgcn_perm(__builtin_amdgcn_perm(z[3], z[2], 0x0C0C0400u),
                                                            __builtin_amdgcn_perm(z[1], z[0], 0x0C0C0400u), 0x05040100u);
                }
        } else {
            const uint32_t sel = 0x0C0C0000u | ((4u + cbyte) << 8) | cbyte;      // byte c of the second, then of the first operand
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int eps = 0; eps < 2; ++eps) {
                    uint32_t w[4], z[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t at = (16u * q + 8u * h + 4u * eps + e) * kPayRow + m;
                        w[e] = pay_lds[dc * 32 * kPayRow + at];
                        z[e] = LOSS ? pay_lds[2 * 32 * kPayRow + at] : 0u;
                    }
                    const uint32_t g01 = __builtin_amdgcn_perm(w[1], w[0], sel), g23 = __builtin_amdgcn_perm(w[3], w[2], sel);
                    Gn[q][eps] = ~__builtin_amdgcn_perm(g23, g01, 0x05040100u);   // a set payload bit is +1: sign bit clear
                    Z[q][eps] = 0xFFFFFFFFu;
                    if constexpr (LOSS)
                        Z[q][eps] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(z[3], z[2], 0x0C0C0400u),
                                                          __builtin_amdgcn_perm(z[1], z[0], 0x0C0C0400u), 0x05040100u);
                }
        }
        // ---- all eight columns once.  Of every result the half i' < 16 (rows 0 .. 511) goes to LDS at once, one dword (two
        // columns of one row) per store; the half i' >= 16 waits in registers until the first half has left the LDS.
        // The dword of column pair tp of row r sits at position tp ^ ((r >> 3) & 3) of its 16-byte chunk, the chunk at
        // position chunk ^ (r & 7) of the row: the 32 lanes of a store (32 consecutive rows) then hit 32 different banks.
        uint32_t out1[4][8];                                     // [column pair][result register 8 + rr]: two fp16
        const uint32_t chunk_mine = 4u * dc + cbyte;
        static_for<4>([&](auto TP) {
            constexpr int tp = decltype(TP)::value;
            float keep[16];                                      // the even column of the pair
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int col = 2 * tp + u;                      // bit of the gathered bytes
                long a[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    uint32_t lo, hi;
                    if constexpr (HALF) {                        // fp8 2.0 where the column holds a value (and its packet arrived)
                        const uint32_t mlo = col < 7 ? (Pn[q][0] << (6 - (col < 7 ? col : 0))) & two_mask : (Pn[q][0] >> 1) & two_mask;
                        const uint32_t mhi = col < 7 ? (Pn[q][1] << (6 - (col < 7 ? col : 0))) & two_mask : (Pn[q][1] >> 1) & two_mask;
                        lo = ((Gn[q][0] << (7 - col)) & sign_mask) | mlo;
                        hi = ((Gn[q][1] << (7 - col)) & sign_mask) | mhi;
                    } else {
                        lo = ((Gn[q][0] << (7 - col)) & sign_mask) | one;
                        hi = ((Gn[q][1] << (7 - col)) & sign_mask) | one;
                        if constexpr (LOSS) { lo &= Z[q][0]; hi &= Z[q][1]; }
                    }
                    a[q] = (long)(((uint64_t)hi << 32) | lo);
                }
                float16_t d1 = {0};
                d1 = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a[0], Hk[0], d1, 0, 0, 0);
                d1 = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a[1], Hk[1], d1, 0, 0, 0);
                u32x4_t b2[2];
#pragma unroll
                for (int r = 0; r < 16; r += 2)
                    b2[r >> 3][(r & 7) >> 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(d1[r], d1[r + 1]));
                float16_t d2 = {0};
                d2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Hn[0], __builtin_bit_cast(half8_t, b2[0]), d2, 0, 0, 0);
                d2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Hn[1], __builtin_bit_cast(half8_t, b2[1]), d2, 0, 0, 0);
                if (u == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) keep[r] = d2[r];
                } else {
#pragma unroll
                    for (int rr = 0; rr < (M == 8 ? 4 : 8); ++rr) {          // (M = 8: rows below 256 are i' < 8)
                        // result register rr holds i' = 8 (rr / 4) + 4 h + rr % 4: row 32 i' + m of the first half
                        const uint32_t row = 32u * (8u * ((uint32_t)rr >> 2) + 4u * h + ((uint32_t)rr & 3u)) + m;
                        const uint32_t at = row * 32u + ((chunk_mine ^ (m & 7u)) << 2) + ((uint32_t)tp ^ ((m >> 3) & 3u));
                        out_lds[at] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(keep[rr], d2[rr]));
                        if constexpr (M == 10)
                            out1[tp][rr] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(keep[8 + rr], d2[8 + rr]));
                    }
                }
                // one column after the other: interleaving them keeps several 16-register results alive and spills; the
                // other waves of the SIMD fill the gaps
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        __syncthreads();
        // (stores: the whole offset in the vector register and none in the scalar one.  For a store of more than 64 bits WITH
        // a scalar offset the compiler assumes that the data registers may be overwritten by the very next instruction; on
        // this chip that replaced the first of the four dwords, in some lanes, when the memory pipeline was busy.)
        // first half: a thread's row in turn `it` is 256 (it / 4) + 32 wave + 8 (it % 4) + lane / 8, so that (row >> 3) & 3,
        // the position swizzle of the dwords, is it % 4: known when the code is compiled
#pragma unroll
        for (int it = 0; it < (M == 8 ? 4 : 8); ++it) {
            const uint32_t row = ((uint32_t)(it >> 2) << 8) + (wv << 5) + ((uint32_t)(it & 3) << 3) + (lane >> 3), chunk = lane & 7u;
            const u32x4_t v = *reinterpret_cast<const u32x4_t *>(&out_lds[(row * 8u + (chunk ^ (row & 7u))) * 4u]);
            const u32x4_t o = {v[0 ^ (it & 3)], v[1 ^ (it & 3)], v[2 ^ (it & 3)], v[3 ^ (it & 3)]};
            __builtin_amdgcn_raw_buffer_store_b128(o, rt, (int)((row << (p + 1)) + cb * 128u + chunk * 16u), 0, kStream);
        }
        if constexpr (M == 10) {
            __syncthreads();                                     // the first half has left the LDS
#pragma unroll
            for (int rr = 0; rr < 8; ++rr) {
                const uint32_t row = 32u * (8u * ((uint32_t)rr >> 2) + 4u * h + ((uint32_t)rr & 3u)) + m;
                const u32x4_t v = {out1[0][rr], out1[1][rr], out1[2][rr], out1[3][rr]};
                *reinterpret_cast<u32x4_t *>(&out_lds[(row * 8u + (chunk_mine ^ (row & 7u))) * 4u]) = v;
            }
            __syncthreads();
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const uint32_t row = 64u * (uint32_t)it + (t >> 3), chunk = t & 7u;
                const u32x4_t v = *reinterpret_cast<const u32x4_t *>(&out_lds[(row * 8u + (chunk ^ (row & 7u))) * 4u]);
                __builtin_amdgcn_raw_buffer_store_b128(v, rt, (int)(((512u + row) << (p + 1)) + cb * 128u + chunk * 16u), 0, kStream);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
#define EDEN_HIX_SWITCH(M, CALL)                         \
    switch (M) {                                         \
        case 7: { constexpr int MM = 7; CALL; } break;   \
        case 8: { constexpr int MM = 8; CALL; } break;   \
        case 9: { constexpr int MM = 9; CALL; } break;   \
        default: { constexpr int MM = 10; CALL; } break; \
    }

static uint32_t hix_tiles(int M, int log2D) { return 1u << (log2D - M - 5); }

uint32_t launch_enc_hix_last(int M, int blocked, const EncBatch &B, uint32_t n, uint64_t d, int log2D, uint64_t seed, const float *T,
                             double *partials, uint32_t partial_stride, const EncScratch *scratch, const CoinTables &ct,
                             hipStream_t st) {
    const uint32_t tiles = hix_tiles(M, log2D);                  // 512 whenever this pass sits directly on lo14
    bool unit = true, mixed = false, four = true;                // every sender b <= 1; some sender b = k + 1/2; every sender b = 4
    for (uint32_t c = 0; c < n; ++c) {
        unit = unit && B.b_q8[c] <= 256u;
        mixed = mixed || budget_two_tables(B.b_q8[c]);
        four = four && B.b_q8[c] == 1024u;
    }
#define EDEN_ENC_HIX_LAST(TPW, MODE)                                                                                          \
    if (blocked) {                                                                                                            \
        EDEN_HIX_SWITCH(M, hipLaunchKernelGGL(HIP_KERNEL_NAME(k_enc_hix_last<MM, TPW, MODE, true>), grid, dim3(HiX<MM>::THREADS), \
                                              0, st, B, d, log2D, seed, T, partials, partial_stride, scratch, ct))            \
    } else {                                                                                                                  \
        EDEN_HIX_SWITCH(M, hipLaunchKernelGGL(HIP_KERNEL_NAME(k_enc_hix_last<MM, TPW, MODE, false>), grid, dim3(HiX<MM>::THREADS), \
                                              0, st, B, d, log2D, seed, T, partials, partial_stride, scratch, ct))            \
    }
    if (unit && tiles % 256u == 0) {                             // two neighbouring tiles per workgroup (with the blocked
        dim3 grid(tiles / 2, n);                                 // workspace: 148 us against 158 with four and 160 with one)
        EDEN_ENC_HIX_LAST(2, 0);
        return grid.x;
    }
    // every other launch: one tile per workgroup (with the blocked workspace two tiles per workgroup are slower at every size:
    // 16 senders at D = 2^23, 0.151 -> 0.142 ms at b = 2, 0.34 -> 0.18 ms at b = 1.5, 0.255 -> 0.144 ms for the b = 4 instance)
    dim3 grid(tiles, n);
    // One budget for all senders: b = 3 and the budgets k + 1/2 have instances that hold only their branch (the shared ones
    // spill 76 and 188 bytes at M = 10; 16 senders at D = 2^24: 0.40 -> 0.24 ms at b = 1.5, 0.277 -> 0.253 ms at b = 3; at
    // b = 2 such an instance gained nothing).
    uint32_t same = B.b_q8[0];
    for (uint32_t c = 1; c < n; ++c) if (B.b_q8[c] != same) same = 0;
#define EDEN_ENC_HIX_ONLY(MODE, ONLY)                                                                                         \
    if (blocked) {                                                                                                            \
        EDEN_HIX_SWITCH(M, hipLaunchKernelGGL(HIP_KERNEL_NAME(k_enc_hix_last<MM, 1, MODE, true, ONLY>), grid, dim3(HiX<MM>::THREADS), \
                                              0, st, B, d, log2D, seed, T, partials, partial_stride, scratch, ct))            \
    } else {                                                                                                                  \
        EDEN_HIX_SWITCH(M, hipLaunchKernelGGL(HIP_KERNEL_NAME(k_enc_hix_last<MM, 1, MODE, false, ONLY>), grid, dim3(HiX<MM>::THREADS), \
                                              0, st, B, d, log2D, seed, T, partials, partial_stride, scratch, ct))            \
    }
    if (four) { EDEN_ENC_HIX_LAST(1, 3); }
    else if (same == 768u) { EDEN_ENC_HIX_ONLY(1, 768u); }
    else if (same == 384u) { EDEN_ENC_HIX_ONLY(2, 384u); }
    else if (same == 640u) { EDEN_ENC_HIX_ONLY(2, 640u); }
    else if (same == 896u) { EDEN_ENC_HIX_ONLY(2, 896u); }
    else if (mixed) { EDEN_ENC_HIX_LAST(1, 2); } else { EDEN_ENC_HIX_LAST(1, 1); }
#undef EDEN_ENC_HIX_ONLY
#undef EDEN_ENC_HIX_LAST
    return grid.x;
}
void launch_hix_mid(int M, uint32_t n, float *T, int log2D, uint64_t load_elems, uint64_t store_elems, hipStream_t st) {
    dim3 grid(hix_tiles(M, log2D) / 2, n);                       // 2^(p-5) = 512 tiles per block of 2^(p+M): pairs never straddle
    EDEN_HIX_SWITCH(M, hipLaunchKernelGGL(HIP_KERNEL_NAME(k_hix_mid<MM, 2>), grid, dim3(HiX<MM>::THREADS), 0, st, T, log2D,
                                          load_elems, store_elems));
}
bool dec_hix_first_prepares(int M, const DecBatch &B, uint32_t n, int narrow) {        // all b = 1 or all b = 1/2 at D = 2^22 .. 2^24
    bool all_same = narrow != 0 && M >= 8 && (B.b_q8[0] == 256u || B.b_q8[0] == 128u);
    for (uint32_t c = 1; c < n; ++c) all_same = all_same && B.b_q8[c] == B.b_q8[0];
    return all_same;
}
bool launch_dec_hix_first(int M, const DecBatch &B, uint32_t n, uint64_t d, int log2D, uint64_t seed,
                          const DecScratch *scratch, int narrow, float *T, const CoinTables &ct, const DecPrepareArgs *prep,
                          hipStream_t st) {
    bool all_unit = narrow != 0;                                 // every sender b <= 1: packed int16 kernel
    for (uint32_t c = 0; c < n; ++c) all_unit = all_unit && B.b_q8[c] <= 256u;
    bool loss = false;
    for (uint32_t c = 0; c < n; ++c) loss = loss || B.bitmap[c] != nullptr;
    if (dec_hix_first_prepares(M, B, n, narrow)) {               // every sender b = 1 (or 1/2) at D = 2^24: the matrix-core pass
        constexpr int TPW = 1;                                   // (two: 86 us against 77, the loop needs more registers than there are)
        dim3 grid(hix_tiles(M, log2D) / 2 / TPW, n);             // 64-column tiles, TPW per workgroup
        const DecPrepareArgs none{};
        const bool half = B.b_q8[0] == 128u;
#define EDEN_DEC_MFMA_M(LOSS, PREP, HALF, MM)                                                                                      \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(k_dec_hix_first_mfma<LOSS, TPW, PREP, HALF, MM>), grid, dim3(512), 0, st, B, d, log2D, seed, T, \
                       prep ? *prep : none)
#define EDEN_DEC_MFMA(LOSS, PREP, HALF)                                    \
    do {                                                                   \
        if (M == 10) EDEN_DEC_MFMA_M(LOSS, PREP, HALF, 10);                \
        else if (M == 9) EDEN_DEC_MFMA_M(LOSS, PREP, HALF, 9);             \
        else EDEN_DEC_MFMA_M(LOSS, PREP, HALF, 8);                         \
    } while (0)
#define EDEN_DEC_MFMA2(LOSS, PREP) do { if (half) EDEN_DEC_MFMA(LOSS, PREP, true); else EDEN_DEC_MFMA(LOSS, PREP, false); } while (0)
        if (loss) { if (prep) EDEN_DEC_MFMA2(true, true); else EDEN_DEC_MFMA2(true, false); }
        else { if (prep) EDEN_DEC_MFMA2(false, true); else EDEN_DEC_MFMA2(false, false); }
#undef EDEN_DEC_MFMA2
#undef EDEN_DEC_MFMA
#undef EDEN_DEC_MFMA_M
        return prep != nullptr;
    }
    if (all_unit) {
        dim3 grid(hix_tiles(M, log2D) / 2, n);                   // 64-column tiles
        EDEN_HIX_SWITCH(M, hipLaunchKernelGGL(k_dec_hix_first_pk<MM>, grid, dim3(HiX<MM>::THREADS), 0, st, B, d, log2D, seed, T));
        return false;
    }
    dim3 grid(hix_tiles(M, log2D), n);
    bool all2 = true, all4 = true;                               // one budget for all: the instance that holds nothing else
    for (uint32_t c = 0; c < n; ++c) {
        all2 = all2 && B.b_q8[c] == 512u && !B.codes[c];
        all4 = all4 && B.b_q8[c] == 1024u && !B.codes[c];
    }
#define EDEN_DEC_HIX_FIRST(ONLY)                                                                                              \
    EDEN_HIX_SWITCH(M, hipLaunchKernelGGL(HIP_KERNEL_NAME(k_dec_hix_first<MM, ONLY>), grid, dim3(HiX<MM>::THREADS), 0, st, B, d, \
                                          log2D, seed, scratch, narrow, T, ct))
    uint32_t same = B.b_q8[0];
    for (uint32_t c = 1; c < n; ++c) if (B.b_q8[c] != same) same = 0;
    if (all2) { EDEN_DEC_HIX_FIRST(512u); } else if (all4) { EDEN_DEC_HIX_FIRST(1024u); }
    else if (same == 768u) { EDEN_DEC_HIX_FIRST(768u); } else if (same == 384u) { EDEN_DEC_HIX_FIRST(384u); }
    else if (same == 640u) { EDEN_DEC_HIX_FIRST(640u); } else if (same == 896u) { EDEN_DEC_HIX_FIRST(896u); }
    else { EDEN_DEC_HIX_FIRST(0u); }
#undef EDEN_DEC_HIX_FIRST
    return false;
}
}  // namespace eden
