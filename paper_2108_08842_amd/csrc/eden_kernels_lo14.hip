// The 14-bit contiguous pass with 32 registers per thread (gfx950).
//
// A workgroup of 8 waves owns 2^14 consecutive coordinates.  Every thread keeps 32 values, so the 14 index
// bits are covered by three groups of in-register butterfly stages:
//
//   group 1   bits 9..13   v[a] = coordinate 512 a + 64 wave + lane  (coalesced loads, 256 B per wave load)
//   exchange  through LDS between all waves (registers <-> bits 4..8)
//   group 2   bits 4..8
//   exchange  through LDS inside groups of 16 lanes (registers <-> bits 0..3, bit 4 stays a register bit)
//   group 3   bits 0..3
//
// Afterwards thread t holds the 32 consecutive coordinates 32 t + e, e = 0..31: one half of a 64-bit sign word
// of the rotation, and one 128-byte line of the workspace or the accumulator.
//
// 32 registers (instead of 64) halve the LDS a wave needs for its exchanges, which doubles the number of
// resident waves per CU (16).  The encode pass built on this is bound by memory, the decode pass (which repeats
// the transform for every sender of a tile) by vector-ALU issue.
#include "eden_device.h"
#include "eden_kernels.h"

namespace eden {

constexpr int kLo14Bits = 14;
constexpr int kXaSlab = 8 * 64 + 16;            // words per value of a: 8 waves x 64 lanes, +16 so that the two
                                                // slabs read by a half-wave fall into different banks
constexpr int kXbRow = 36;                      // 32 values + 4: rows of consecutive lanes start 4 banks apart
constexpr int kXbWave = 64 * kXbRow + 48;       // one wave's region of the second exchange
constexpr int kLo14LdsWords = 8 * kXbWave;      // 75264 bytes; the first exchange needs 32 * kXaSlab words
static_assert(kLo14LdsWords >= 32 * kXaSlab, "LDS sizing");

// in:  v[a] = coordinate 512 a + 64 wave + lane of the tile
// out: v[e] = coordinate 512 (t >> 4) + 32 (t & 15) + e, fully transformed over the 14 bits
__device__ inline void lo14_forward32(float (&v)[32], float *lds) {
    const uint32_t t = threadIdx.x, lane = t & 63u, wv = t >> 6;
    fwht_regs<32>(v);                                            // bits 9..13
#pragma unroll
    for (int a = 0; a < 32; ++a) lds[a * kXaSlab + wv * 64 + lane] = v[a];
    __syncthreads();
    const uint32_t c0123 = t & 15u, a2 = t >> 4;
#pragma unroll
    for (int r = 0; r < 32; ++r) v[r] = lds[a2 * kXaSlab + (r >> 2) * 64 + (r & 3) * 16 + c0123];
    fwht_regs<32>(v);                                            // bits 4..8 (register bit 0 = index bit 4)
    __syncthreads();                                             // all reads done before the regions are reused
    float *L = lds + wv * kXbWave;
    const uint32_t g = lane >> 4;
#pragma unroll
    for (int r = 0; r < 32; ++r) L[(g * 16 + (r >> 1)) * kXbRow + g * 16 + (r & 1) * 16 + c0123] = v[r];
    wave_lds_sync();
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const float4 x = *reinterpret_cast<const float4 *>(&L[lane * kXbRow + g * 16 + 4 * q]);
        v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
    }
    fwht_regs_low<32, 4>(v);                                     // bits 0..3 (bit 4 rides along)
}

// Stores the 32 consecutive values every thread holds after lo14_forward32 as whole 128-byte lines: thread t's
// run starts at coordinate 32 t of the tile, so a wave owns 2048 consecutive coordinates; a wave-private
// transpose through LDS (quads swizzled by the low three bits of the row: eight neighbouring lanes then hit 32
// different banks in both directions; measured with SQ_LDS_BANK_CONFLICT) lets 8 neighbouring lanes store one line.
// `L`: this wave's 2048 floats of LDS; `Tc`: the sender's workspace slot; `tile`: the tile = row of the strided pass.
// BLOCKED: the 128-byte segments of kBlockRows consecutive rows are interleaved (see blocked_offset): the strided pass
// then finds kBlockRows of its 128-byte pieces next to each other.  Stores cost the same either way (6.9 TB/s in a pure
// store loop); a pure read of the strided pattern went from 4.8 to 5.9 TB/s.
template <bool BLOCKED>
__device__ inline void lo14_store_runs(const float (&v)[32], float *L, float *Tc, uint32_t tile, uint32_t wv) {
    const uint32_t lane = threadIdx.x & 63u;
    wave_lds_sync();
    const uint32_t swz = lane & 7u;
#pragma unroll
    for (int q = 0; q < 8; ++q)
        *reinterpret_cast<float4 *>(&L[lane * 32u + 4u * ((uint32_t)q ^ swz)]) = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    wave_lds_sync();
    const uint32_t pos = lane & 7u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t row = 8u * (uint32_t)j + (lane >> 3);     // segment of 32 coordinates inside the wave's 2048
        const float4 x = *reinterpret_cast<const float4 *>(&L[row * 32u + 4u * pos]);
        const uint32_t quad = pos ^ (row & 7u);
        // (write-back stores: with the streaming hint this pass ran 13% slower; the pass that reads the tiles back does
        // better with the hint on its loads)
        const size_t at = BLOCKED ? blocked_offset(tile, 64u * wv + row) + 4u * quad
                                  : ((size_t)tile << kLo14Bits) + 2048u * wv + row * 32u + 4u * quad;
        *reinterpret_cast<float4 *>(Tc + at) = x;
    }
}

// Encode, first pass: x -> T.  Zero padding (Sec. 5: the transform needs a power of two), the sign diagonal of
// the rotation from the shared seed (Sec. 2.1), |x|^2 for eta and S (Sec. 2.2.1, 2.3), index bits 0..13 of H.
// Only the ceil(d / 2^14) tiles that hold part of x (rounded up to whole blocks of rows in the blocked layout) are
// transformed and written: a tile of padding stays zero under these 14 bits, and the strided pass that follows reads it
// as zero through its buffer bounds.
// PRE (b = 1/2 with the sparsification first, Sec. 4.1): the vector that is transformed is x'[g] = 2 x[2g + o_g],
// g < ceil(d_src/2), o_g from the SUB-SAMPLING stream; x is read as 0 beyond d_src.
template <bool PRE, bool BLOCKED>
__global__ __launch_bounds__(512, 4) void k_enc_lo14_first(EncBatch B, uint64_t d_src, int log2D, uint64_t seed, float *T,
                                                        double *partials, uint32_t partial_stride) {
    __shared__ __attribute__((aligned(16))) float lds[kLo14LdsWords];
    __shared__ double red[8];
    const uint32_t c = blockIdx.y, t = threadIdx.x, lane = t & 63u;
    const uint32_t wv = wave_in_block();
    const rsrc_t rx = make_rsrc(B.x[c], (uint32_t)(d_src * 4));           // reads past d_src give the zero padding
    float *Tc = T + ((size_t)c << log2D);
    const uint64_t key = stream_key(seed, kStreamSign, B.client[c]);
    const uint32_t lane_off = (wv * 64u + lane) * 4u;
    const uint32_t tile = blockIdx.x;                            // one tile per workgroup: two workgroups share a CU, and
                                                                 // their phases interleave better than two tiles in one
                                                                 // workgroup with the second one's loads issued early
    // element 512 a + 64 wave + lane of the tile; with PRE it comes from x[2 i + o_i], and register a of this wave is
    // 64 consecutive pairs = one word of offsets (lane l < 32 hashes the word of register l)
    float u[32];
    if constexpr (PRE) {
        const uint64_t prekey = stream_key(seed, kStreamSubsample, B.client[c]);
        const uint64_t offs = hash_word(prekey, ((uint64_t)tile << (kLo14Bits - 6)) + 8u * (lane & 31u) + wv);
#pragma unroll
        for (int a = 0; a < 32; ++a) {
            const uint32_t odd = __builtin_amdgcn_inverse_ballot_w64(wave_read64(offs, a)) ? 4u : 0u;
            u[a] = 2.0f * buf_load(rx, 2u * lane_off + odd, (tile << (kLo14Bits + 3)) + 4096u * a);
        }
    } else {
#pragma unroll
        for (int a = 0; a < 32; ++a) u[a] = buf_load(rx, lane_off, (tile << (kLo14Bits + 2)) + 2048u * a);
    }
    double n2 = 0.0;
#pragma unroll
    for (int a = 0; a < 32; ++a) {
        n2 += (double)u[a] * (double)u[a];
        if ((a & 7) == 7) __builtin_amdgcn_sched_barrier(0);     // keeps the widened values of one group live at a time
    }
    // register a of this wave = 64 consecutive coordinates = one sign word: lane l < 32 hashes the word of
    // register l, register a reads it back as a lane mask
    const uint64_t mine = hash_word(key, ((uint64_t)tile << (kLo14Bits - 6)) + 8u * (lane & 31u) + wv);
#pragma unroll
    for (int a = 0; a < 32; ++a) u[a] = negate_where(u[a], wave_read64(mine, a)) + 0.0f;   // + 0: no negative zeros
    lo14_forward32(u, lds);
    lo14_store_runs<BLOCKED>(u, lds + wv * kXbWave, Tc, tile, wv);
    const double block_total = block_sum<512>(n2, red);
    if (t == 0) partials[(size_t)c * partial_stride + blockIdx.x] = block_total;
}

// Decode, last pass: index bits 0..13 of H for every sender, that sender's sign diagonal (R^-1 = s o D^-1/2 H,
// Sec. 2.2.2), sum over senders in registers, one contiguous read-modify-write of acc.
// `narrow`: senders with b <= 1 have an fp16 workspace holding exact integers; their magnitude S/(p sqrt D) q_1
// is applied together with the sign.
//
// Work split.  A workgroup's time is proportional to the senders it sums and the chip holds `2 x CUs` of these
// workgroups at once, so a tile count far below that would leave most of the chip idle.  The first `full_tiles`
// tiles get one workgroup each that sums all n senders into acc.  Each of the remaining tiles gets K workgroups: group 0 sums its share of the senders into acc,
// group k > 0 stores its sum in partial[k-1][tile - full_tiles][2^14]; k_dec_lo14_combine then adds those to
// acc in the order k = 1, 2, ... (fixed, so the result does not depend on scheduling).
//
// PRE (b = 1/2 with the sparsification first, Sec. 4.1): the decoded vectors have dimension ceil(d_src/2) and value g
// of sender c belongs at coordinate 2g + o_g of acc (o_g from c's SUB-SAMPLING stream).  A thread then keeps the 64
// accumulator coordinates of its 32 pairs in registers and adds every value to the member of the pair it belongs
// to; the launcher does not split tiles in this mode.
// `separate`: K = n, one sender per workgroup, nothing is summed: every sender's decoded tile is written back into its own
// workspace slot (`partial` is then the workspace; fp32, in place: the workgroup has read the tile before it writes
// it), for a caller that puts the values elsewhere afterwards.
// WIDE_ONLY: no sender of the launch has an fp16 slot (every b > 1): the instance without that branch in the sender loop
// (116 registers instead of 125; 16 senders at D = 2^24: 0.170 -> 0.160 ms).
template <bool PRE, bool WIDE_ONLY = false>
__global__ __launch_bounds__(512) void k_dec_lo14_last(DecBatch B, uint32_t n, uint64_t d_src, int log2D, uint64_t seed,
                                                       const float *T, const DecScratch *scratch, int narrow_arg, float *acc,
                                                       uint32_t full_tiles, uint32_t K, uint32_t split_tiles,
                                                       float *partial, int separate, float mean_n) {
    __shared__ __attribute__((aligned(16))) float lds[kLo14LdsWords];
    const int narrow = WIDE_ONLY ? 0 : narrow_arg;
    constexpr int NS = PRE ? 64 : 32;                            // accumulator coordinates per thread
    const uint64_t d = d_src;                                    // bound of acc
    const uint32_t t = threadIdx.x, lane = t & 63u, wv = t >> 6;
    uint32_t tile = blockIdx.x, c_begin = 0, c_end = n;
    float *part_run = nullptr;                                   // this thread's 32 values in the partial buffer
    if (blockIdx.x >= full_tiles) {
        const uint32_t idx = blockIdx.x - full_tiles, k = idx % K;
        tile = full_tiles + idx / K;
        c_begin = (uint32_t)(((uint64_t)n * k) / K);
        c_end = (uint32_t)(((uint64_t)n * (k + 1)) / K);
        if (separate) part_run = partial + ((size_t)k << log2D) + ((size_t)tile << kLo14Bits) + 32u * t;
        else if (k > 0) part_run = partial + (((size_t)(k - 1) * split_tiles + (tile - full_tiles)) << kLo14Bits) + 32u * t;
    }
    const uint64_t tile_base = (uint64_t)tile << kLo14Bits;
    const uint64_t first = tile_base + 32u * t;
    const size_t in_off = tile_base + wv * 64u + lane;
    float sum[NS];
#pragma unroll
    for (int e = 0; e < NS; ++e) sum[e] = 0.0f;

    auto load = [&](uint32_t c, float (&dst_regs)[32]) {
        if (narrow && B.b_q8[c] <= 256u) {
            const short *t16 = reinterpret_cast<const short *>(T + ((size_t)c << log2D)) + in_off;
#pragma unroll
            for (int a = 0; a < 32; ++a) dst_regs[a] = __int_as_float((int)__builtin_nontemporal_load(t16 + 512 * a));
        } else {
            const float *t32 = T + ((size_t)c << log2D) + in_off;
#pragma unroll
            for (int a = 0; a < 32; ++a) dst_regs[a] = __builtin_nontemporal_load(t32 + 512 * a);
        }
    };
    // One sender: `cur` holds its 32 loaded values (PRE: they are loaded here, with 64 accumulators there is no room to
    // load ahead); the loads of sender c + 1 go into the same registers once the values have been converted.  (Two
    // alternating register sets would save the compiler's copy of the loaded set, but need more than 128 registers.)
    auto one_sender = [&](uint32_t c, float (&cur)[32]) {
        const bool i16 = narrow && B.b_q8[c] <= 256u;
        float u[32];
        if constexpr (PRE) load(c, cur);
#pragma unroll
        for (int a = 0; a < 32; ++a) {
            u[a] = i16 ? narrow_value((short)__float_as_int(cur[a])) : cur[a];
        }
        __builtin_amdgcn_sched_barrier(0);                       // the conversions stay above the next sender's loads
        if (!PRE && c + 1 < c_end) load(c + 1, cur);
        lo14_forward32(u, lds);
        const uint32_t scale = __float_as_uint(i16 ? scratch[c].deq[1] : 1.0f) & 0x7FFFFFFFu;   // > 0; x*1+s is exact
        // the wave's 2048 coordinates use 32 sign words: lane l < 32 hashes word l, every thread fetches its own
        const uint64_t key = stream_key(seed, kStreamSign, B.client[c]);
        const uint64_t mine = hash_word(key, ((tile_base + 512u * (wv * 4u)) >> 6) + (lane & 31u));
        const uint32_t src = ((lane >> 4) * 8u) + ((lane & 15u) >> 1);      // word of this thread's run, wave-relative
        const uint32_t wlo = (uint32_t)__shfl((int)(uint32_t)mine, (int)src, 64);
        const uint32_t whi = (uint32_t)__shfl((int)(uint32_t)(mine >> 32), (int)src, 64);
        const uint32_t bits = (t & 1u) ? whi : wlo;              // 32 sign bits of this thread's run
        if constexpr (PRE) {
            const uint64_t okey = stream_key(seed, kStreamSubsample, B.client[c]);
            const uint64_t omine = hash_word(okey, ((tile_base + 512u * (wv * 4u)) >> 6) + (lane & 31u));
            const uint32_t olo = (uint32_t)__shfl((int)(uint32_t)omine, (int)src, 64);
            const uint32_t ohi = (uint32_t)__shfl((int)(uint32_t)(omine >> 32), (int)src, 64);
            const uint32_t offs = (t & 1u) ? ohi : olo;          // which member of each of this thread's 32 pairs
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                const uint32_t sgn = (bits << (31 - e)) & 0x80000000u;
                const float val = u[e] * __uint_as_float(scale | sgn);
                const bool odd = (offs >> e) & 1u;
                sum[2 * e] += odd ? 0.0f : val;
                sum[2 * e + 1] += odd ? val : 0.0f;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 32; ++e) {
                // hash bit 1 -> s_i = -1: the factor is the scale with bit e of the sign word moved to the sign position
                // (one shift, one bit-field insert)
                const uint32_t shifted = bits << (31 - e);
                const uint32_t factor = (scale & 0x7FFFFFFFu) | (shifted & 0x80000000u);
                sum[e] = fmaf(u[e], __uint_as_float(factor), sum[e]);
            }
        }
        __syncthreads();                                         // LDS is reused by the next sender
    };
    float loaded[32];
    if (!PRE && c_begin < c_end) load(c_begin, loaded);
    for (uint32_t c = c_begin; c < c_end; ++c) one_sender(c, loaded);
    if constexpr (PRE) {                                         // this thread's 32 pairs = 64 consecutive coordinates of acc
        const uint64_t out = 2 * first;
        if (out + 64 <= d) {
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                float4 a = *reinterpret_cast<const float4 *>(acc + out + 4 * q);
                a.x += sum[4 * q]; a.y += sum[4 * q + 1]; a.z += sum[4 * q + 2]; a.w += sum[4 * q + 3];
                *reinterpret_cast<float4 *>(acc + out + 4 * q) = a;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 64; ++e)
                if (out + e < d) acc[out + e] += sum[e];
        }
        return;
    }
    if (part_run) {
#pragma unroll
        for (int q = 0; q < 8; ++q)
            *reinterpret_cast<float4 *>(part_run + 4 * q) = make_float4(sum[4 * q], sum[4 * q + 1], sum[4 * q + 2], sum[4 * q + 3]);
        return;
    }
    // mean_n > 0: acc is written, not added to; the division happens here when no other workgroup adds to this tile
    const bool overwrite = mean_n > 0.0f;
    const float div = (overwrite && blockIdx.x < full_tiles) ? mean_n : 1.0f;
    if (tile_base + (1u << kLo14Bits) <= d) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (!overwrite) a = *reinterpret_cast<const float4 *>(acc + first + 4 * q);
            a.x = (a.x + sum[4 * q]) / div; a.y = (a.y + sum[4 * q + 1]) / div;
            a.z = (a.z + sum[4 * q + 2]) / div; a.w = (a.w + sum[4 * q + 3]) / div;
            *reinterpret_cast<float4 *>(acc + first + 4 * q) = a;
        }
    } else {                                                     // the one tile that straddles d
#pragma unroll
        for (int e = 0; e < 32; ++e)
            if (first + e < d) acc[first + e] = ((overwrite ? 0.0f : acc[first + e]) + sum[e]) / div;
    }
}

// ---- the same pass (index bits 0..13 of H, the sign diagonal and the sum over the senders, Sec. 2.2.2) for launches whose
// senders all have an fp16 workspace of small exact integers (b <= 1, D <= 2^24:
// |value| <= 2^10 after at most ten strided bits), with ten of the fourteen bits on the matrix cores.
//
// The tile is a 16 x 32 x 32 array (u, n, k) = index bits 10..13, 5..9, 0..4.  A wave owns two values of u.  For one u:
//   step 1  bits 0..4   D1[n][k'] = sum_k X[n][k] H[k][k']: v_mfma_f32_32x32x16_f16 twice, X as the A operand straight from
//           memory (a lane holds 16 consecutive fp16 of its row n: exact integers, |x| <= 2^10 < 2^11).
//   step 2  bits 5..9   D2[n'][k'] = sum_n H[n'][n] D1[n][k']: the registers that hold D1 ARE a B operand (lane = column k',
//           registers = 8 values of n per lane half), the Hadamard A operand is built with its columns in that order, so
//           nothing moves between the steps.  |D1| <= 2^15 does not fit fp16's 11 bits: every value is split into its fp16
//           truncation and the remainder (<= 5 bits, exact), and both go through the matrix cores into the same fp32
//           accumulators (four instructions).  All sums are integers below 2^24: exact in fp32 in any order.
//   exchange through LDS: lds[u][r][lane] = register r of the wave that owns u; wave w reads r = 2w, 2w + 1 of all 16 u
//           (same lane: the exchange swaps the register index with the wave index, conflict free in both directions).
//   step 3  bits 10..13 four butterfly stages over the 16 values of u in registers (fp32, exact).
// Register (u, j) of thread (wave w, lane l = 32 h + m) then holds coordinate 1024 u + 32 n' + m of the tile with
// n' = 8 (w / 2) + 4 h + 2 (w % 2) + j: 32 lanes cover one 128-byte line of acc, and the 32 sign bits of those lanes are one
// half (j) of one 64-bit word of the sender's SIGN stream.
// Per coordinate and sender this leaves about 9 vector instructions (split 2, butterflies 4, sign and accumulate 3)
// where the all-vector version spends 19, and one exchange instead of two.
// x - (float)h for the fp16 in the low (HIGH = 0) or high half of `packed`: one mixed-precision fused multiply-add
// (-1 * h + x, exact: h is x truncated to 11 bits)
template <int HIGH>
__device__ inline float minus_half(float x, uint32_t packed) {
    float r;
    if (HIGH) asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(-1.0f), "v"(x));
    else asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(-1.0f), "v"(x));
    return r;
}

__global__ __launch_bounds__(512, 4) void k_dec_lo14_last_mfma(DecBatch B, uint32_t n, uint64_t d, int log2D, uint64_t seed,
                                                               const float *T, const DecScratch *scratch, float *acc,
                                                               uint32_t full_tiles, uint32_t K, uint32_t split_tiles,
                                                               float *partial, float mean_n) {
    __shared__ __attribute__((aligned(16))) float lds[1 << kLo14Bits];
    const uint32_t t = threadIdx.x, lane = t & 63u, wv = wave_in_block(), h = lane >> 5, m = lane & 31u;
    uint32_t tile = blockIdx.x, c_begin = 0, c_end = n;
    float *part = nullptr;                                       // this tile in the partial buffer
    if (blockIdx.x >= full_tiles) {
        const uint32_t idx = blockIdx.x - full_tiles, k = idx % K;
        tile = full_tiles + idx / K;
        c_begin = (uint32_t)(((uint64_t)n * k) / K);
        c_end = (uint32_t)(((uint64_t)n * (k + 1)) / K);
        if (k > 0) part = partial + (((size_t)(k - 1) * split_tiles + (tile - full_tiles)) << kLo14Bits);
    }
    const uint64_t tile_base = (uint64_t)tile << kLo14Bits;

    // the two Hadamard operands: entry e of instruction q on lane (h, m)
    //   step 1, B[k][k']: k' = m, k = 16 h + 8 q + e    (the 16 consecutive fp16 a lane loads are k = 16 h .. 16 h + 15)
    //   step 2, A[n'][n]: n' = m, n = row of D1 that register 8 q + e of lane half h holds = 16 q + 8 (e / 4) + 4 h + e % 4
    half8_t Hk[2], Hn[2];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            Hk[q][e] = hadamard_entry(16u * h + 8u * q + e, m);
        }
    Hn[0] = hadamard_rows_of_result(0, h, m);
    Hn[1] = hadamard_rows_of_result(1, h, m);

    float sum[32];                                               // sum[16 j + u]
#pragma unroll
    for (int e = 0; e < 32; ++e) sum[e] = 0.0f;

    // raw[2 s + q]: fp16 k = 16 h + 8 q .. + 7 of row n = m of unit u = wv + 8 s
    const uint32_t lane_off = (m * 32u + 16u * h) * 2u;
    auto load = [&](uint32_t c, uint32_t (&raw)[4][4]) {
        const rsrc_t r16 = make_rsrc(T + ((size_t)c << log2D), 2u << log2D);       // the tile lies inside the slot
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                // (default cache policy: the two instructions q take the two 16-byte halves of every 32 bytes, and with the
                // streaming hint the second one fetched some lines again: 106 against 103 us)
                const auto x = __builtin_amdgcn_raw_buffer_load_b128(
                    r16, (int)lane_off, (int)(((uint32_t)tile_base + (wv + 8u * s) * 1024u + 8u * q) * 2u), 0);
                raw[2 * s + q][0] = x[0]; raw[2 * s + q][1] = x[1]; raw[2 * s + q][2] = x[2]; raw[2 * s + q][3] = x[3];
            }
    };
    // sign words of this wave's coordinates: word (u, hh) = 16 u + 4 (wv / 2) + (wv % 2) + 2 hh of the tile; lane 16 hh + u
    // of either half of the wave hashes it
    const uint32_t my_word = 16u * (lane & 15u) + 4u * (wv >> 1) + (wv & 1u) + 2u * ((lane >> 4) & 1u);

    uint32_t raw[4][4];
    if (c_begin < c_end) load(c_begin, raw);
    for (uint32_t c = c_begin; c < c_end; ++c) {
        half8_t x[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const u32x4_t v = {raw[i][0], raw[i][1], raw[i][2], raw[i][3]};
            x[i] = __builtin_bit_cast(half8_t, v);
        }
        if (c + 1 < c_end) load(c + 1, raw);
        if (c > c_begin) __syncthreads();                        // every wave has read the previous sender's values
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            float16_t d1 = {0};
            d1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(x[2 * s], Hk[0], d1, 0, 0, 0);
            d1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(x[2 * s + 1], Hk[1], d1, 0, 0, 0);
            u32x4_t hi[2], lo[2];                                  // fp16 pairs: registers 2 i, 2 i + 1 of d1
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const uint32_t top = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(d1[r], d1[r + 1]));   // truncated to 11 bits
                hi[r >> 3][(r & 7) >> 1] = top;
                lo[r >> 3][(r & 7) >> 1] = __builtin_bit_cast(                                  // what is left: at most 5 bits
                    uint32_t, __builtin_amdgcn_cvt_pkrtz(minus_half<0>(d1[r], top), minus_half<1>(d1[r + 1], top)));
            }
            float16_t d2 = {0};
            d2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Hn[0], __builtin_bit_cast(half8_t, hi[0]), d2, 0, 0, 0);
            d2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Hn[1], __builtin_bit_cast(half8_t, hi[1]), d2, 0, 0, 0);
            d2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Hn[0], __builtin_bit_cast(half8_t, lo[0]), d2, 0, 0, 0);
            d2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Hn[1], __builtin_bit_cast(half8_t, lo[1]), d2, 0, 0, 0);
            float *L = lds + (wv + 8u * s) * 1024u + lane;
#pragma unroll
            for (int r = 0; r < 16; ++r) L[64 * r] = d2[r];
        }
        __syncthreads();
        float v0[16], v1[16];                                    // j = 0, 1
        const float *R = lds + 128u * wv + lane;
#pragma unroll
        for (int u = 0; u < 16; ++u) { v0[u] = R[1024 * u]; v1[u] = R[1024 * u + 64]; }
        fwht_regs<16>(v0);
        fwht_regs<16>(v1);
        const uint32_t scale = __float_as_uint(scratch[c].deq[1]) & 0x7FFFFFFFu;     // > 0
        const uint64_t key = stream_key(seed, kStreamSign, B.client[c]);
        const uint64_t mine = hash_word(key, (tile_base >> 6) + my_word);
        const uint32_t mine_lo = (uint32_t)mine, mine_hi = (uint32_t)(mine >> 32);
        const float pos = __uint_as_float(scale);
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            // hash bit 1 -> s_i = -1.  Lanes u and 16 + u hold the words of the two halves of the wave: their low (j = 0) or high
            // (j = 1) halves, side by side in a scalar register pair, are the 64 sign bits of the wave's lanes, and a select
            // driven by that pair needs no lane to fetch or shift anything
            const uint64_t neg0 = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)mine_lo, 16 + u) << 32) |
                                  (uint32_t)__builtin_amdgcn_readlane((int)mine_lo, u);
            const uint64_t neg1 = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)mine_hi, 16 + u) << 32) |
                                  (uint32_t)__builtin_amdgcn_readlane((int)mine_hi, u);
            sum[u] = fmaf(v0[u], __builtin_amdgcn_inverse_ballot_w64(neg0) ? -pos : pos, sum[u]);
            sum[16 + u] = fmaf(v1[u], __builtin_amdgcn_inverse_ballot_w64(neg1) ? -pos : pos, sum[16 + u]);
        }
    }
    // register (u, j): coordinate 1024 u + 32 n' + m of the tile
    const uint32_t nrow = 8u * (wv >> 1) + 4u * h + 2u * (wv & 1u);
    const uint32_t mine_off = 32u * nrow + m;
    if (part) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            part[1024 * u + mine_off] = sum[u];
            part[1024 * u + mine_off + 32] = sum[16 + u];
        }
        return;
    }
    // mean_n > 0: acc is written, not added to; the division happens here when no other workgroup adds to this tile
    const bool overwrite = mean_n > 0.0f;
    const float div = (overwrite && blockIdx.x < full_tiles) ? mean_n : 1.0f;
    if (tile_base + (1u << kLo14Bits) <= d) {
        float *A = acc + tile_base + mine_off;
        float old[32];
#pragma unroll
        for (int e = 0; e < 32; ++e) old[e] = 0.0f;
        if (!overwrite) {
#pragma unroll
            for (int u = 0; u < 16; ++u) { old[u] = A[1024 * u]; old[16 + u] = A[1024 * u + 32]; }
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) { A[1024 * u] = (old[u] + sum[u]) / div; A[1024 * u + 32] = (old[16 + u] + sum[16 + u]) / div; }
    } else {                                                     // the one tile that straddles d
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const uint64_t i = tile_base + 1024u * u + mine_off;
            if (i < d) acc[i] = ((overwrite ? 0.0f : acc[i]) + sum[u]) / div;
            if (i + 32 < d) acc[i + 32] = ((overwrite ? 0.0f : acc[i + 32]) + sum[16 + u]) / div;
        }
    }
}

// ---- the same matrix-core pass for senders that sparsified by pairs before the rotation (EDEN_B_HALF_PRE, Sec. 4.1): the
// decoded vector has ceil(d / 2) coordinates, and coordinate g of sender c belongs to position 2 g + o_c(g) of the output
// (o from the sender's SUBSAMPLE stream), the other position of the pair getting nothing from this sender.  Every
// coordinate therefore needs two sums, and a thread of the kernel above has no registers for 64: here a workgroup has 16
// waves, wave w owns the one unit u = w in steps 1 and 2, and reads register w of all 16 units back from the exchange,
// so that a thread holds 16 coordinates (two sums each).  Register u of thread (wave w, lane 32 h + m) is coordinate
// 1024 u + 32 n' + m of the tile with n' = 8 (w / 4) + 4 h + w % 4: its bit of the SIGN and SUBSAMPLE streams is bit
// 32 (w % 2) + m of word 16 u + 4 (w / 4) + 2 h + (w / 2) % 2 of the tile, and the 32 lanes m write 64 consecutive floats.
// mean_n > 0: the output is written ((0 + sum) / mean_n) instead of added to.
__global__ __launch_bounds__(1024) void k_dec_lo14_last_pairs(DecBatch B, uint32_t n, uint64_t d_src, int log2D, uint64_t seed,
                                                              const float *T, const DecScratch *scratch, float *acc, float mean_n) {
    __shared__ __attribute__((aligned(16))) float lds[1 << kLo14Bits];
    const uint32_t t = threadIdx.x, lane = t & 63u, wv = wave_in_block(), h = lane >> 5, m = lane & 31u;
    const uint64_t tile_base = (uint64_t)blockIdx.x << kLo14Bits;

    half8_t Hk[2], Hn[2];                                        // as in k_dec_lo14_last_mfma
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) Hk[q][e] = hadamard_entry(16u * h + 8u * q + e, m);
    Hn[0] = hadamard_rows_of_result(0, h, m);
    Hn[1] = hadamard_rows_of_result(1, h, m);

    float even[16], odd[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) even[u] = odd[u] = 0.0f;

    // raw[q]: fp16 k = 16 h + 8 q .. + 7 of row n = m of unit u = wv
    const uint32_t lane_off = (m * 32u + 16u * h) * 2u;
    auto load = [&](uint32_t c, uint32_t (&raw)[2][4]) {
        const rsrc_t r16 = make_rsrc(T + ((size_t)c << log2D), 2u << log2D);       // the tile lies inside the slot
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const auto x = __builtin_amdgcn_raw_buffer_load_b128(r16, (int)lane_off,
                                                                 (int)(((uint32_t)tile_base + wv * 1024u + 8u * q) * 2u), 0);
            raw[q][0] = x[0]; raw[q][1] = x[1]; raw[q][2] = x[2]; raw[q][3] = x[3];
        }
    };
    // lane 16 hh + uu of either half of the wave hashes word (uu, hh)
    const uint32_t my_word = 16u * (lane & 15u) + 4u * (wv >> 2) + 2u * ((lane >> 4) & 1u) + ((wv >> 1) & 1u);

    uint32_t raw[2][4];
    load(0, raw);
    for (uint32_t c = 0; c < n; ++c) {
        half8_t x[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const u32x4_t v = {raw[q][0], raw[q][1], raw[q][2], raw[q][3]};
            x[q] = __builtin_bit_cast(half8_t, v);
        }
        if (c + 1 < n) load(c + 1, raw);
        if (c > 0) __syncthreads();                              // every wave has read the previous sender's values
        {
            float16_t d1 = {0};
            d1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(x[0], Hk[0], d1, 0, 0, 0);
            d1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(x[1], Hk[1], d1, 0, 0, 0);
            u32x4_t hi[2], lo[2];                                // fp16 pairs: the truncation to 11 bits and what is left
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const uint32_t top = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(d1[r], d1[r + 1]));
                hi[r >> 3][(r & 7) >> 1] = top;
                lo[r >> 3][(r & 7) >> 1] = __builtin_bit_cast(
                    uint32_t, __builtin_amdgcn_cvt_pkrtz(minus_half<0>(d1[r], top), minus_half<1>(d1[r + 1], top)));
            }
            float16_t d2 = {0};
            d2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Hn[0], __builtin_bit_cast(half8_t, hi[0]), d2, 0, 0, 0);
            d2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Hn[1], __builtin_bit_cast(half8_t, hi[1]), d2, 0, 0, 0);
            d2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Hn[0], __builtin_bit_cast(half8_t, lo[0]), d2, 0, 0, 0);
            d2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(Hn[1], __builtin_bit_cast(half8_t, lo[1]), d2, 0, 0, 0);
            float *L = lds + wv * 1024u + lane;
#pragma unroll
            for (int r = 0; r < 16; ++r) L[64 * r] = d2[r];
        }
        __syncthreads();
        float v[16];
        const float *R = lds + 64u * wv + lane;
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = R[1024 * u];
        fwht_regs<16>(v);
        const uint32_t scale = __float_as_uint(scratch[c].deq[1]) & 0x7FFFFFFFu;     // > 0
        // one hash per lane serves both streams: lanes 0..31 take the words of the SIGN stream, lanes 32..63 the same words of
        // the SUBSAMPLE stream
        const uint64_t sign_key = stream_key(seed, kStreamSign, B.client[c]), pick_key = stream_key(seed, kStreamSubsample, B.client[c]);
        const uint64_t word = hash_word(h ? pick_key : sign_key, (tile_base >> 6) + my_word);
        const uint32_t half = (wv & 1u) ? (uint32_t)(word >> 32) : (uint32_t)word;
        const float pos = __uint_as_float(scale);
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            // Lanes u and 16 + u hold the SIGN words of the two halves of the wave, lanes 32 + u and 48 + u the SUBSAMPLE words:
            // side by side in a scalar register pair they are the 64 bits of the wave's lanes, and selects driven by such a
            // pair need no lane to fetch or shift anything.  Hash bit 1 -> s_i = -1; offset bit 1 -> the pair's second position.
            const uint64_t neg = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)half, 16 + u) << 32) |
                                 (uint32_t)__builtin_amdgcn_readlane((int)half, u);
            const uint64_t second = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)half, 48 + u) << 32) |
                                    (uint32_t)__builtin_amdgcn_readlane((int)half, 32 + u);
            const float factor = __builtin_amdgcn_inverse_ballot_w64(neg) ? -pos : pos;
            const bool to_second = __builtin_amdgcn_inverse_ballot_w64(second);
            even[u] = fmaf(v[u], to_second ? 0.0f : factor, even[u]);
            odd[u] = fmaf(v[u], to_second ? factor : 0.0f, odd[u]);
        }
    }
    const bool overwrite = mean_n > 0.0f;
    const float div = overwrite ? mean_n : 1.0f;
    const uint32_t nrow = 8u * (wv >> 2) + 4u * h + (wv & 3u);
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const uint64_t out = 2u * (tile_base + 1024u * (uint32_t)u + 32u * nrow + m);
        if (out + 1 < d_src) {
            float2 a = make_float2(0.0f, 0.0f);
            if (!overwrite) a = *reinterpret_cast<const float2 *>(acc + out);
            a.x = (a.x + even[u]) / div; a.y = (a.y + odd[u]) / div;
            *reinterpret_cast<float2 *>(acc + out) = a;
        } else if (out < d_src) {
            acc[out] = ((overwrite ? 0.0f : acc[out]) + even[u]) / div;
        }
    }
}

// acc[i] += partial[0][i'] + partial[1][i'] + ... for the tiles that k_dec_lo14_last split over K workgroups
// (added one after the other, in this order); with mean_n > 0 the total is divided by it.  One thread per four coordinates.
__global__ __launch_bounds__(256) void k_dec_lo14_combine(float *acc, uint64_t d, uint32_t full_tiles, uint32_t K,
                                                          uint32_t split_tiles, const float *partial, float mean_n) {
    const uint64_t local = ((uint64_t)blockIdx.x * 256u + threadIdx.x) * 4u;         // inside the split tiles
    const uint64_t i = ((uint64_t)full_tiles << kLo14Bits) + local;
    if (local >= ((uint64_t)split_tiles << kLo14Bits) || i >= d) return;
    float s[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) s[e] = (i + e < d) ? acc[i + e] : 0.0f;
    for (uint32_t k = 1; k < K; ++k) {
        const float4 p = *reinterpret_cast<const float4 *>(partial + (((size_t)(k - 1) * split_tiles) << kLo14Bits) + local);
        s[0] += p.x; s[1] += p.y; s[2] += p.z; s[3] += p.w;
    }
    const float div = mean_n > 0.0f ? mean_n : 1.0f;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (i + e < d) acc[i + e] = s[e] / div;
}

uint32_t launch_enc_lo14_first(const EncBatch &B, uint32_t n, uint64_t d_src, int pre, int blocked, int log2D, uint64_t seed, float *T,
                               double *partials, uint32_t partial_stride, hipStream_t st) {
    const uint64_t d = pre ? (d_src + 1) / 2 : d_src;
    uint32_t tiles = (uint32_t)((d + (1u << kLo14Bits) - 1) >> kLo14Bits);
    // blocked layout: whole blocks of rows are written (a tile beyond d reads zeros and stores zeros), so that the strided
    // pass finds no unwritten row inside a block
    if (blocked) tiles = (tiles + kBlockRows - 1) / kBlockRows * kBlockRows;
    dim3 grid(tiles, n);
#define EDEN_ENC_LO14(PRE, BLK) \
    hipLaunchKernelGGL(HIP_KERNEL_NAME(k_enc_lo14_first<PRE, BLK>), grid, dim3(512), 0, st, B, d_src, log2D, seed, T, partials, partial_stride)
    if (pre) { if (blocked) EDEN_ENC_LO14(true, true); else EDEN_ENC_LO14(true, false); }
    else { if (blocked) EDEN_ENC_LO14(false, true); else EDEN_ENC_LO14(false, false); }
#undef EDEN_ENC_LO14
    return grid.x;
}
void launch_dec_lo14_last(const DecBatch &B, uint32_t n, uint64_t d_src, int pre, int log2D, uint64_t seed, float *T,
                          const DecScratch *scratch, int narrow, float *acc, uint32_t resident, float *partial,
                          uint32_t partial_tiles, float mean_n, hipStream_t st) {
    const uint64_t d = pre == 1 ? (d_src + 1) / 2 : d_src;       // dimension of the decoded vectors
    const uint32_t tiles = (uint32_t)((d + (1u << kLo14Bits) - 1) >> kLo14Bits);     // tiles that reach below d
    if (pre == 1) {
        if (narrow)                                              // fp16 workspace of small integers: on the matrix cores
            hipLaunchKernelGGL(k_dec_lo14_last_pairs, dim3(tiles), dim3(1024), 0, st, B, n, d_src, log2D, seed, T, scratch, acc,
                               mean_n);
        else
            hipLaunchKernelGGL(HIP_KERNEL_NAME(k_dec_lo14_last<true>), dim3(tiles), dim3(512), 0, st, B, n, d_src, log2D, seed, T,
                               scratch, narrow, acc, tiles, 1u, 0u, partial, 0, 0.0f);
        return;
    }
    if (pre == 2) {                                              // every sender on its own, back into its workspace slot
        hipLaunchKernelGGL(HIP_KERNEL_NAME(k_dec_lo14_last<false>), dim3(tiles * n), dim3(512), 0, st, B, n, d_src, log2D, seed,
                           T, scratch, 0, acc, 0u, n, tiles, T, 1, 0.0f);
        return;
    }
    bool all16 = narrow != 0;                                    // every sender's workspace slot holds fp16
    for (uint32_t c = 0; c < n; ++c) all16 = all16 && B.b_q8[c] <= 256u;
    // Fewer tiles than half the resident workgroups: split every tile K ways by sender so that the chip is filled
    // (measured 2.2x on 64 tiles x 32 senders).  With more tiles than resident workgroups, splitting only the
    // last, partly filled wave of workgroups was measured 3..10% slower than leaving it: a CU with one workgroup runs it faster.
    uint32_t full = 0, rest = tiles, K = 1;
    if (2 * tiles <= resident) {
        K = resident / tiles;
        if (K > n) K = n;
        while (K > 1 && (uint64_t)(K - 1) * rest > partial_tiles) --K;    // what the partial buffer holds
    }
    if (K == 1) { full = tiles; rest = 0; }
    dim3 grid(full + rest * K);
    if (all16)                                                   // |values| <= 2^10: ten of the bits on the matrix cores
        hipLaunchKernelGGL(k_dec_lo14_last_mfma, grid, dim3(512), 0, st, B, n, d_src, log2D, seed, T, scratch, acc, full, K, rest,
                           partial, mean_n);
    else {
        bool none16 = true;                                      // no sender with an fp16 slot
        for (uint32_t c = 0; c < n; ++c) none16 = none16 && !(narrow && B.b_q8[c] <= 256u);
        if (none16)
            hipLaunchKernelGGL(HIP_KERNEL_NAME(k_dec_lo14_last<false, true>), grid, dim3(512), 0, st, B, n, d_src, log2D, seed, T,
                               scratch, narrow, acc, full, K, rest, partial, 0, mean_n);
        else
            hipLaunchKernelGGL(HIP_KERNEL_NAME(k_dec_lo14_last<false>), grid, dim3(512), 0, st, B, n, d_src, log2D, seed, T, scratch,
                               narrow, acc, full, K, rest, partial, 0, mean_n);
    }
    if (K > 1) {
        dim3 cgrid((uint32_t)((((uint64_t)rest << kLo14Bits) / 4 + 255) / 256));
        hipLaunchKernelGGL(k_dec_lo14_combine, cgrid, dim3(256), 0, st, acc, d, full, K, rest, partial, mean_n);
    }
}

}  // namespace eden
