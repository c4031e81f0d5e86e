// The 14-bit contiguous pass with 32 registers per thread (gfx950).
//
// A workgroup of 8 waves owns 2^14 consecutive coordinates.  Every thread keeps 32 values, so the 14 index
// bits are covered by three rounds of in-register butterflies:
//
//   round 1   bits 9..13   v[a] = coordinate 512 a + 64 wave + lane  (coalesced loads, 256 B per wave load)
//   exchange  through LDS between all waves (registers <-> bits 4..8)
//   round 2   bits 4..8
//   exchange  through LDS inside groups of 16 lanes (registers <-> bits 0..3, bit 4 stays a register bit)
//   round 3   bits 0..3
//
// Afterwards thread t holds the 32 consecutive coordinates 512 (t >> 4) + 32 (t & 15) + e, e = 0..31: one
// packed word for b = 1, and one half of a 64-bit sign word of the rotation.
//
// 32 registers (instead of 64) halve the LDS a wave needs for its exchanges, which doubles the number of
// resident waves per CU (16); these passes are bound by vector-ALU issue, not by memory.
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

__device__ inline uint32_t lane_xor1(uint32_t x) {              // value held by lane ^ 1
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, true);
}

template <int BITS>
__device__ inline void quantize_store32(const float (&u)[32], const EncScratch *s, uint32_t *payload, uint64_t first,
                                        float &ip) {
    constexpr int H = 1 << (BITS - 1);
    float thr[H], qp[H];
#pragma unroll
    for (int i = 0; i < H; ++i) { thr[i] = s->thr[i]; qp[i] = s->qpos[i]; }
    uint32_t w[BITS];
#pragma unroll
    for (int i = 0; i < BITS; ++i) w[i] = 0;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        const uint32_t code = quantize_one<H>(u[e], thr, qp, ip);
        w[(e * BITS) / 32] |= code << ((e * BITS) % 32);
    }
    if constexpr (BITS == 2) *reinterpret_cast<uint2 *>(payload + (first >> 4)) = make_uint2(w[0], w[1]);
    else *reinterpret_cast<uint4 *>(payload + (first >> 3)) = make_uint4(w[0], w[1], w[2], w[3]);
}

// Encode, last pass: T -> payload.  Quantization to the Lloyd-Max intervals (Sec. 2.2.1, Sec. 3), sum_i u_i q_i
// for the scale (Sec. 2.3), sub-sampling for b = 1/2 (Sec. 4.1), packing.  TPW tiles per workgroup: the next
// tile's loads are in flight while the current tile is transformed.
template <int TPW>
__global__ __launch_bounds__(512) void k_enc_lo14(EncBatch B, int log2D, uint64_t seed, const float *T, double *partials,
                                                  uint32_t partial_stride, const EncScratch *scratch) {
    __shared__ __attribute__((aligned(16))) float lds[kLo14LdsWords];
    __shared__ double red[8];
    const uint32_t c = blockIdx.y, t = threadIdx.x;
    const EncScratch *s = &scratch[c];
    const uint32_t b_q8 = B.b_q8[c];
    uint32_t *payload = reinterpret_cast<uint32_t *>(static_cast<char *>(B.msg[c]) + EDEN_HEADER_BYTES);
    const float *Tw = T + ((size_t)c << log2D) + (t >> 6) * 64u + (t & 63u);
    const uint32_t run = 512u * (t >> 4) + 32u * (t & 15u);      // this thread's 32 coordinates inside a tile
    float ip = 0.0f;
    float next[32];
#pragma unroll
    for (int a = 0; a < 32; ++a) next[a] = __builtin_nontemporal_load(Tw + (((uint64_t)blockIdx.x * TPW) << kLo14Bits) + 512 * a);
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
        const uint64_t tile_base = ((uint64_t)blockIdx.x * TPW + k) << kLo14Bits;
        float u[32];
#pragma unroll
        for (int a = 0; a < 32; ++a) u[a] = next[a];
        if (k + 1 < TPW) {
#pragma unroll
            for (int a = 0; a < 32; ++a) next[a] = __builtin_nontemporal_load(Tw + tile_base + (1u << kLo14Bits) + 512 * a);
        }
        lo14_forward32(u, lds);
        const uint64_t first = tile_base + run;
        if (b_q8 == 256 || b_q8 == 128) {
            // I_1 = {(-inf,0],[0,inf)}: the index is the sign; <R(x),Q> = q_1 sum |u| / sqrt(D)
            float sa = 0.0f;
#pragma unroll
            for (int e = 0; e < 32; ++e) sa += fabsf(u[e]);
            ip += sa * kQ1;
            if (b_q8 == 256) {
                uint32_t neg = 0;                                // shift the sign bits in, last coordinate first
#pragma unroll
                for (int e = 31; e >= 0; --e) neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(u[e]), 31);
                payload[first >> 5] = ~neg;                      // index 1 = non-negative
            } else {
                // b = 1/2: of each pair (2g, 2g+1) send the coordinate chosen by the sub-sampling stream
                uint32_t ev = 0, od = 0;
#pragma unroll
                for (int g = 15; g >= 0; --g) {
                    ev = __builtin_amdgcn_alignbit(ev, __float_as_uint(u[2 * g]), 31);
                    od = __builtin_amdgcn_alignbit(od, __float_as_uint(u[2 * g + 1]), 31);
                }
                const uint64_t key = stream_key(seed, kStreamSubsample, B.client[c]);
                const uint64_t hw = hash_word(key, first >> 7);  // 64 pairs per hash word = 128 coordinates
                const uint32_t off = (uint32_t)(hw >> (16u * (uint32_t)((first >> 5) & 3u))) & 0xFFFFu;
                const uint32_t mine = ((~ev & ~off) | (~od & off)) & 0xFFFFu;
                const uint32_t other = lane_xor1(mine);
                if (!(t & 1u)) payload[first >> 6] = mine | (other << 16);
            }
        } else if (b_q8 == 512) {
            quantize_store32<2>(u, s, payload, first, ip);
        } else {
            quantize_store32<4>(u, s, payload, first, ip);
        }
        if (k + 1 < TPW) __syncthreads();                        // LDS is reused by the next tile
    }
    const double block_total = block_sum<512>((double)ip, red);
    if (t == 0) partials[(size_t)c * partial_stride + blockIdx.x] = block_total;
}

// Decode, last pass: index bits 0..13 of H for every sender, that sender's sign diagonal (R^-1 = s o D^-1/2 H,
// Sec. 2.2.2), sum over senders in registers, one contiguous read-modify-write of acc.
// `narrow`: senders with b <= 1 have an int16 workspace holding exact integers; their magnitude S/(p sqrt D) q_1
// is applied together with the sign.
__global__ __launch_bounds__(512) void k_dec_lo14_last(DecBatch B, uint32_t n, uint64_t d, int log2D, uint64_t seed,
                                                       const float *T, const DecScratch *scratch, int narrow, float *acc) {
    __shared__ __attribute__((aligned(16))) float lds[kLo14LdsWords];
    const uint64_t tile_base = (uint64_t)blockIdx.x << kLo14Bits;
    if (tile_base >= d) return;                                  // whole tile in the padding
    const uint32_t t = threadIdx.x, lane = t & 63u, wv = t >> 6;
    const uint64_t first = tile_base + 512u * (t >> 4) + 32u * (t & 15u);
    const size_t in_off = tile_base + wv * 64u + lane;
    float sum[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) sum[e] = 0.0f;

    auto load = [&](uint32_t c, float (&dst)[32]) {
        if (narrow && B.b_q8[c] <= 256u) {
            const short *t16 = reinterpret_cast<const short *>(T + ((size_t)c << log2D)) + in_off;
#pragma unroll
            for (int a = 0; a < 32; ++a) dst[a] = __int_as_float((int)__builtin_nontemporal_load(t16 + 512 * a));
        } else {
            const float *t32 = T + ((size_t)c << log2D) + in_off;
#pragma unroll
            for (int a = 0; a < 32; ++a) dst[a] = __builtin_nontemporal_load(t32 + 512 * a);
        }
    };
    float next[32];
    load(0, next);
    for (uint32_t c = 0; c < n; ++c) {
        const bool i16 = narrow && B.b_q8[c] <= 256u;
        float u[32];
#pragma unroll
        for (int a = 0; a < 32; ++a) u[a] = i16 ? (float)__float_as_int(next[a]) : next[a];
        if (c + 1 < n) load(c + 1, next);
        lo14_forward32(u, lds);
        const uint32_t scale = __float_as_uint(i16 ? scratch[c].deq[1] : 1.0f) & 0x7FFFFFFFu;   // > 0; x*1+s is exact
        // the wave's 2048 coordinates use 32 sign words: lane l < 32 hashes word l, every thread fetches its own
        const uint64_t key = stream_key(seed, kStreamSign, B.client[c]);
        const uint64_t mine = hash_word(key, ((tile_base + 512u * (wv * 4u)) >> 6) + (lane & 31u));
        const uint32_t src = ((lane >> 4) * 8u) + ((lane & 15u) >> 1);      // word of this thread's run, wave-relative
        const uint32_t wlo = (uint32_t)__shfl((int)(uint32_t)mine, (int)src, 64);
        const uint32_t whi = (uint32_t)__shfl((int)(uint32_t)(mine >> 32), (int)src, 64);
        const uint32_t bits = (t & 1u) ? whi : wlo;              // 32 sign bits of this thread's run
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            const uint32_t sgn = (bits << (31 - e)) & 0x80000000u;          // hash bit 1 -> s_i = -1
            sum[e] = fmaf(u[e], __uint_as_float(scale | sgn), sum[e]);
        }
        __syncthreads();                                         // LDS is reused by the next sender
    }
    if (tile_base + (1u << kLo14Bits) <= d) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float4 a = *reinterpret_cast<const float4 *>(acc + first + 4 * q);
            a.x += sum[4 * q]; a.y += sum[4 * q + 1]; a.z += sum[4 * q + 2]; a.w += sum[4 * q + 3];
            *reinterpret_cast<float4 *>(acc + first + 4 * q) = a;
        }
    } else {                                                     // the one tile that straddles d
#pragma unroll
        for (int e = 0; e < 32; ++e)
            if (first + e < d) acc[first + e] += sum[e];
    }
}

uint32_t launch_enc_lo14(const EncBatch &B, uint32_t n, int log2D, uint64_t seed, const float *T, double *partials,
                         uint32_t partial_stride, const EncScratch *scratch, hipStream_t st) {
    const uint32_t tiles = 1u << (log2D - kLo14Bits);
    if (tiles >= 1024) {                                         // still >= 4 workgroups per resident slot
        dim3 grid(tiles / 8, n);
        hipLaunchKernelGGL(k_enc_lo14<8>, grid, dim3(512), 0, st, B, log2D, seed, T, partials, partial_stride, scratch);
        return grid.x;
    }
    if (tiles >= 256) {
        dim3 grid(tiles / 4, n);
        hipLaunchKernelGGL(k_enc_lo14<4>, grid, dim3(512), 0, st, B, log2D, seed, T, partials, partial_stride, scratch);
        return grid.x;
    }
    dim3 grid(tiles, n);
    hipLaunchKernelGGL(k_enc_lo14<1>, grid, dim3(512), 0, st, B, log2D, seed, T, partials, partial_stride, scratch);
    return grid.x;
}
void launch_dec_lo14_last(const DecBatch &B, uint32_t n, uint64_t d, int log2D, uint64_t seed, const float *T,
                          const DecScratch *scratch, int narrow, float *acc, hipStream_t st) {
    dim3 grid(1u << (log2D - kLo14Bits));
    hipLaunchKernelGGL(k_dec_lo14_last, grid, dim3(512), 0, st, B, n, d, log2D, seed, T, scratch, narrow, acc);
}

}  // namespace eden
