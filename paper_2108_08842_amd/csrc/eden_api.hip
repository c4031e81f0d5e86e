// C ABI of the EDEN library (see include/eden.h for the contract of every call).
// Host code only: argument checks, the pass plan, workspace, launches.  Every step of the path runs
// in the kernels of eden_kernels.hip, eden_kernels_lo14.hip and eden_kernels_wg.hip.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "eden.h"
#include "eden_device.h"
#include "eden_kernels.h"
#include "eden_tables.h"

using namespace eden;

struct eden_ctx {
    int device;
    uint64_t d_max;
    int log2D_max;
    uint32_t n_max;          // senders per call the workspace was sized for (chunks of kMaxBatch are used)
    uint32_t slots;          // workspace slots = min(n_max, kMaxBatch)
    float *T;                // slots * D_max floats (nullptr if D_max <= 4096)
    double *partials;        // 2 * slots * partial_stride doubles: |x|^2 partials, then sum u q partials
    uint32_t partial_stride;
    uint32_t compute_units;      // of the context's device
    float *dec_partial;          // sums of sender groups when the last decode pass splits tiles (D_max >= 2^19)
    uint32_t dec_partial_tiles;  // its size in tiles of 2^14 floats
    uint32_t *hist;              // 256 counters for eden_index_entropy
    uint8_t *codes;              // slots * D_max bytes: one-byte indices of b = 5, 6, 7 senders before packing / after
                                 // unpacking (multi-pass sizes only)
    float *stage;                // d_max + 64 floats: the kept coordinates of one sender with a budget b = m/64
    CoinTables coin;             // coin budgets at multi-pass sizes: masks and prefix sums of the coins, per slot
    EncScratch *enc_scratch; // slots
    DecScratch *dec_scratch; // slots
    DevTables *tables;
    uint32_t *dev_status;
    uint32_t *msg_flags;         // n_max words: the status bits of every message of the last eden_decode_accumulate call
    uint32_t last_decode_n = 0;  // how many of them that call wrote
    // optional kernel timing (eden_profile_*)
    uint32_t prof_mask = 0;
    uint32_t prof_used = 0;
    std::vector<hipEvent_t> prof_start, prof_stop;
    std::vector<uint32_t> prof_kind, prof_senders;
};

namespace {

int ceil_log2(uint64_t d) {
    int l = 0;
    while ((1ull << l) < d) ++l;
    return l;
}

// groups of kCoinGroup blocks of 64 coordinates at the largest dimension
uint32_t coin_group_stride(int log2D_max) {
    const uint64_t words = log2D_max > 6 ? (1ull << (log2D_max - 6)) : 1;
    return (uint32_t)((words + kCoinGroup - 1) / kCoinGroup);
}

// d rounded up to a multiple of 2^bits
uint64_t round_up(uint64_t d, int bits) { return ((d + (1ull << bits) - 1) >> bits) << bits; }

// Pass plan.  The contiguous pass covers the low 12 bits (wave tiles) or 14 bits (workgroup tiles); the
// bits above it are covered by one or two strided passes: wave tiles handle up to 6 bits each,
// workgroup tiles 7..10 bits.  D <= 2^24 needs two passes in all, D up to 2^27 three.  Encode runs the
// passes in ascending bit order (contiguous first), decode in descending order (contiguous last).
struct HiPass {
    bool wg;    // workgroup-tile kernel (32-column tiles) or wave-tile kernel (64-column tiles)
    int M, p;   // bits transformed, lowest bit
    bool wide;  // wave-tile kernel with 8 columns per lane (top pass of the three-pass sizes; b = 1, 2, 4, 5..8, grid)
};
struct Plan {
    int lo_bits;        // 0: single-workgroup path (D <= 4096)
    int nhi;
    HiPass hi[2];       // ascending p
};
// `wide_ok`: every sender of the launch has b = 1, 2, 4 or a one-byte budget (what the wide top tile packs).
Plan make_plan(int log2D, bool wide_ok) {
    Plan pl{};
    if (log2D <= kLoBits) return pl;
    if (log2D <= 18) {
        pl.lo_bits = 12; pl.nhi = 1; pl.hi[0] = {false, log2D - 12, 12, false};
    } else if (log2D <= 24) {
        const int M = log2D - 14;
        pl.lo_bits = 14; pl.nhi = 1; pl.hi[0] = {M > 6, M, 14, false};
    } else if (wide_ok) {
        pl.lo_bits = 14; pl.nhi = 2; pl.hi[0] = {true, log2D - 17, 14, false}; pl.hi[1] = {false, 3, log2D - 3, true};
    } else {
        // the pass next to the payload gets as many rows per wave as the remaining bits allow (16..64)
        pl.lo_bits = 14; pl.nhi = 2; pl.hi[0] = {true, 7, 14, false}; pl.hi[1] = {false, log2D - 21, 21, false};
    }
    return pl;
}

struct DeviceGuard {
    int prev = -1;
    bool ok = true;
    explicit DeviceGuard(int dev) {
        if (hipGetDevice(&prev) != hipSuccess) { ok = false; return; }
        if (prev != dev && hipSetDevice(dev) != hipSuccess) ok = false;
        if (prev == dev) prev = -1;
    }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};

bool launch_ok() { return hipGetLastError() == hipSuccess; }

// The Lloyd-Max tables of Sec. 3 (positive halves) in the layout the kernels read.
void fill_host_tables(DevTables &host) {
    std::memset(&host, 0, sizeof(host));
    for (int bits = 1; bits <= EDEN_MAX_TABLE_BITS; ++bits) {
        const EdenHalfTable *ht = eden_half_table(bits);
        for (int i = 0; i < ht->half_levels; ++i) {
            if (bits <= 4) { host.t[bits][i] = ht->t[i]; host.q[bits][i] = ht->q[i]; }
            else { host.t_big[bits - 5][i] = ht->t[i]; host.q_big[bits - 5][i] = ht->q[i]; }
        }
    }
}

// Brackets one kernel launch with two events when timing of that kernel kind is switched on.
struct Timed {
    eden_ctx *ctx;
    hipStream_t st;
    int slot = -1;
    Timed(eden_ctx *c, uint32_t kind, uint32_t senders, hipStream_t s) : ctx(c), st(s) {
        if (!((c->prof_mask >> kind) & 1u) || c->prof_used >= c->prof_start.size()) return;
        slot = (int)c->prof_used++;
        c->prof_kind[slot] = kind;
        c->prof_senders[slot] = senders;
        (void)hipEventRecord(c->prof_start[slot], st);
    }
    ~Timed() { if (slot >= 0) (void)hipEventRecord(ctx->prof_stop[slot], st); }
};

}  // namespace

extern "C" {

size_t eden_message_bytes(uint64_t d, uint32_t b_q8) {
    if (b_q8 == kPreHalf) return d >= 2 ? eden_message_bytes((d + 1) / 2, 256) : 0;
    if (sparse_m(b_q8)) return (d >= 1 && d <= (1ull << EDEN_MAX_LOG2_D)) ? eden_message_bytes(sparse_m(b_q8) * ((d + 63) / 64), 256) : 0;
    int bits, k;
    if (d == 0 || d > (1ull << EDEN_MAX_LOG2_D) || !budget_of(b_q8, bits, k)) return 0;
    const uint64_t D = 1ull << ceil_log2(d);
    if (D < (uint64_t)k || (budget_mixed(b_q8) && D < 2)) return 0;
    return EDEN_HEADER_BYTES + (size_t)(payload_a_bytes(D, bits, k) + payload_b_bytes(D, b_q8));
}

int eden_create(eden_ctx **out, uint64_t d_max, uint32_t n_max, int hip_device) {
    if (!out) return EDEN_ERR_INVALID_ARG;
    *out = nullptr;
    if (d_max == 0 || d_max > (1ull << EDEN_MAX_LOG2_D) || n_max == 0) return EDEN_ERR_INVALID_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || hip_device < 0 || hip_device >= ndev) return EDEN_ERR_NO_DEVICE;
    DeviceGuard guard(hip_device);
    if (!guard.ok) return EDEN_ERR_HIP;

    eden_ctx *ctx = new (std::nothrow) eden_ctx();
    if (!ctx) return EDEN_ERR_HIP;
    ctx->device = hip_device;
    ctx->d_max = d_max;
    ctx->log2D_max = ceil_log2(d_max);
    ctx->n_max = n_max;
    ctx->slots = n_max < (uint32_t)kMaxBatch ? n_max : (uint32_t)kMaxBatch;
    const uint64_t D_max = 1ull << ctx->log2D_max;
    ctx->partial_stride = (uint32_t)(D_max / 256 + 16);
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, hip_device) != hipSuccess || cus <= 0) cus = 256;
    ctx->compute_units = (uint32_t)cus;

    bool ok = true;
    if (ctx->log2D_max > kLoBits) {
        ok = ok && hipMalloc(&ctx->T, (size_t)ctx->slots * D_max * sizeof(float)) == hipSuccess;
        ok = ok && hipMalloc(&ctx->codes, (size_t)ctx->slots * D_max) == hipSuccess;
    }
    ok = ok && hipMalloc(&ctx->stage, (size_t)(d_max + 64) * sizeof(float)) == hipSuccess;
    ctx->coin = CoinTables{};
    ctx->coin.group_stride = coin_group_stride(ctx->log2D_max);
    if (ctx->log2D_max > kLoBits) {
        ok = ok && hipMalloc(&ctx->coin.mask, (size_t)ctx->slots * (D_max / 64) * sizeof(uint64_t)) == hipSuccess;
        ok = ok && hipMalloc(&ctx->coin.local, (size_t)ctx->slots * (D_max / 64) * sizeof(uint32_t)) == hipSuccess;
        ok = ok && hipMalloc(&ctx->coin.group, (size_t)ctx->slots * ctx->coin.group_stride * sizeof(uint32_t)) == hipSuccess;
    }
    ok = ok && hipMalloc(&ctx->coin.total, ctx->slots * sizeof(uint32_t)) == hipSuccess;
    if (ctx->log2D_max >= 19 && ctx->slots > 1) {                // at most as many split tiles as workgroups fit on the chip
        ctx->dec_partial_tiles = 2 * ctx->compute_units;
        ok = ok && hipMalloc(&ctx->dec_partial, ((size_t)ctx->dec_partial_tiles << 14) * sizeof(float)) == hipSuccess;
    }
    ok = ok && hipMalloc(&ctx->partials, 2 * (size_t)ctx->slots * ctx->partial_stride * sizeof(double)) == hipSuccess;
    ok = ok && hipMalloc(&ctx->enc_scratch, ctx->slots * sizeof(EncScratch)) == hipSuccess;
    ok = ok && hipMalloc(&ctx->dec_scratch, ctx->slots * sizeof(DecScratch)) == hipSuccess;
    ok = ok && hipMalloc(&ctx->tables, sizeof(DevTables)) == hipSuccess;
    ok = ok && hipMalloc(&ctx->dev_status, sizeof(uint32_t)) == hipSuccess;
    ok = ok && hipMalloc(&ctx->msg_flags, (size_t)n_max * sizeof(uint32_t)) == hipSuccess;
    ok = ok && hipMalloc(&ctx->hist, 256 * sizeof(uint32_t)) == hipSuccess;
    if (ok) {
        std::vector<DevTables> host_tables(1);                   // 9 KiB: not on the stack
        DevTables &host = host_tables[0];
        fill_host_tables(host);
        ok = ok && hipMemcpy(ctx->tables, &host, sizeof(host), hipMemcpyHostToDevice) == hipSuccess;
        ok = ok && hipMemset(ctx->enc_scratch, 0, ctx->slots * sizeof(EncScratch)) == hipSuccess;
        ok = ok && hipMemset(ctx->dec_scratch, 0, ctx->slots * sizeof(DecScratch)) == hipSuccess;
        ok = ok && hipMemset(ctx->dev_status, 0, sizeof(uint32_t)) == hipSuccess;
        ok = ok && hipMemset(ctx->msg_flags, 0, (size_t)n_max * sizeof(uint32_t)) == hipSuccess;
        ok = ok && hipDeviceSynchronize() == hipSuccess;
    }
    if (!ok) {
        eden_destroy(ctx);
        return EDEN_ERR_HIP;
    }
    *out = ctx;
    return EDEN_OK;
}

int eden_destroy(eden_ctx *ctx) {
    if (!ctx) return EDEN_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    bool ok = guard.ok;
    for (hipEvent_t e : ctx->prof_start) ok = (hipEventDestroy(e) == hipSuccess) && ok;
    for (hipEvent_t e : ctx->prof_stop) ok = (hipEventDestroy(e) == hipSuccess) && ok;
    void *ptrs[] = {ctx->T, ctx->dec_partial, ctx->stage, ctx->codes, ctx->hist, ctx->partials, ctx->enc_scratch, ctx->dec_scratch, ctx->tables, ctx->dev_status,
                    ctx->coin.mask, ctx->coin.local, ctx->coin.group, ctx->coin.total, ctx->msg_flags};
    for (void *p : ptrs)
        if (p) ok = (hipFree(p) == hipSuccess) && ok;
    delete ctx;
    return ok ? EDEN_OK : EDEN_ERR_HIP;
}

static bool packs_bytes(uint32_t b_q8) { return wide_bits(b_q8) >= 5u && wide_bits(b_q8) <= 7u; }

// Encodes n senders whose transformed vectors all have the same dimension.  `b_kernel`: the budgets the kernels
// quantize with; `b_hdr`, `hdr_d`: what the headers record; `d_src`, `pre`: the length of the vectors x points to and
// whether they are sparsified in pairs on the way in.
static int encode_range(eden_ctx *ctx, const float *const *x_dev, const uint32_t *client_ids, const uint32_t *b_kernel,
                        const uint32_t *b_hdr, uint32_t n, uint64_t d_src, int pre, uint64_t hdr_d, uint64_t seed,
                        void *const *msgs_dev, hipStream_t st) {
    const uint64_t d = pre ? (d_src + 1) / 2 : d_src;            // dimension of the vector that is transformed
    const int log2D = ceil_log2(d);
    bool wide_ok = true;
    for (uint32_t c = 0; c < n; ++c)
        wide_ok = wide_ok && (b_kernel[c] == 256u || b_kernel[c] == 512u || b_kernel[c] == 1024u || byte_budget(b_kernel[c]));
    const Plan pl = make_plan(log2D, wide_ok);

    for (uint32_t first = 0; first < n; first += kMaxBatch) {
        const uint32_t nb = (n - first < (uint32_t)kMaxBatch) ? n - first : (uint32_t)kMaxBatch;
        EncBatch B;
        std::memset(&B, 0, sizeof(B));
        for (uint32_t i = 0; i < nb; ++i) {
            B.x[i] = x_dev[first + i];
            B.msg[i] = msgs_dev[first + i];
            B.client[i] = client_ids[first + i];
            B.b_q8[i] = b_kernel[first + i];
            B.hdr_b_q8[i] = b_hdr[first + i];
        }
        bool pack = false;                                       // b = 5, 6, 7: bytes first, packed by a kernel of its own
        if (pl.lo_bits != 0) {
            for (uint32_t i = 0; i < nb; ++i) pack = pack || packs_bytes(B.b_q8[i]);
            for (uint32_t i = 0; i < nb; ++i)
                if (packs_bytes(B.b_q8[i])) B.codes[i] = ctx->codes + ((size_t)i << log2D);
        }
        if (pl.lo_bits == 0) {
            Timed t(ctx, EDEN_K_ENC_SMALL, nb, st);
            launch_enc_small(B, nb, d_src, pre, hdr_d, log2D, seed, ctx->tables, ctx->dev_status, st);
        } else {
            // contiguous pass first (it reads x, and only the tiles that hold part of x), strided passes after it in
            // place on the workspace, the last one quantizing and packing
            uint32_t nparts_n2 = 0, nparts_ip = 0;
            double *part_n2 = ctx->partials, *part_ip = ctx->partials + (size_t)ctx->slots * ctx->partial_stride;
            bool need_thresholds = false;                        // b = 1 and 1/2 quantize by sign alone
            for (uint32_t i = 0; i < nb; ++i) need_thresholds = need_thresholds || B.b_q8[i] > 256u;
            bool coins = false;                                  // coin budgets: masks and prefix sums of the coins first
            void *part_b[kMaxBatch] = {};
            for (uint32_t i = 0; i < nb; ++i) {
                if (!coin_q8(B.b_q8[i])) continue;
                coins = true;
                part_b[i] = static_cast<char *>(B.msg[i]) + EDEN_HEADER_BYTES + payload_a_bytes(1ull << log2D, (int)(coin_q8(B.b_q8[i]) >> 8), 1);
            }
            if (coins) launch_coin_tables(B.client, B.b_q8, part_b, nb, seed, log2D, ctx->coin, st);
            // Coin senders whose last pass runs in workgroup tiles leave the pieces of the second part in the byte-index buffer
            // (a word per 32 coordinates) and a small kernel strings them together: no atomics in the last pass.
            const uint32_t *pieces[kMaxBatch] = {};
            bool staged = false;
            if (coins && ctx->codes && pl.hi[pl.nhi - 1].wg) {
                for (uint32_t i = 0; i < nb; ++i) {
                    if (!coin_q8(B.b_q8[i])) continue;
                    B.codes[i] = ctx->codes + ((size_t)i << log2D);
                    pieces[i] = reinterpret_cast<const uint32_t *>(B.codes[i]);
                    staged = true;
                }
            }
            // The workspace goes through the blocked layout when a workgroup-tile pass reads it back right away (two-pass
            // plans of D >= 2^21), unless the first pass works in place on the workspace (its input is a slot): its
            // workgroups would then overwrite rows that others have not read yet.
            bool blocked = pl.lo_bits == 14 && pl.nhi == 1 && pl.hi[0].wg;
            for (uint32_t i = 0; i < nb; ++i)
                blocked = blocked && !(ctx->T && B.x[i] >= ctx->T && B.x[i] < ctx->T + ((size_t)ctx->slots << ctx->log2D_max));
            {
                Timed t(ctx, EDEN_K_ENC_FIRST, nb, st);
                nparts_n2 = pl.lo_bits == 14
                                ? launch_enc_lo14_first(B, nb, d_src, pre, blocked, log2D, seed, ctx->T, part_n2, ctx->partial_stride, st)
                                : launch_enc_lo_first(B, nb, d_src, pre, log2D, seed, ctx->T, part_n2, ctx->partial_stride, st);
            }
            if (need_thresholds) {
                Timed t(ctx, EDEN_K_ENC_NORM, nb, st);
                launch_enc_norm(B, nb, part_n2, ctx->partial_stride, nparts_n2, ctx->enc_scratch, ctx->tables, st);
            }
            uint64_t valid = round_up(d, pl.lo_bits);            // workspace elements written so far; the rest is zero
            for (int i = 0; i < pl.nhi; ++i) {
                const HiPass &h = pl.hi[i];
                if (i < pl.nhi - 1) {
                    Timed t(ctx, EDEN_K_MID, nb, st);
                    launch_hix_mid(h.M, nb, ctx->T, log2D, valid, 1ull << log2D, st);
                    valid = round_up(d, h.p + h.M);
                } else {
                    Timed t(ctx, EDEN_K_ENC_LAST, nb, st);
                    nparts_ip = h.wg     ? launch_enc_hix_last(h.M, blocked, B, nb, d, log2D, seed, ctx->T, part_ip, ctx->partial_stride,
                                                               ctx->enc_scratch, ctx->coin, st)
                                : h.wide ? launch_enc_wide_last(B, nb, valid, log2D, ctx->T, part_ip, ctx->partial_stride,
                                                                ctx->enc_scratch, st)
                                         : launch_enc_hi_last(h.M, B, nb, valid, log2D, h.p, seed, ctx->T, part_ip,
                                                              ctx->partial_stride, ctx->enc_scratch, ctx->coin, st);
                }
            }
            if (pack) launch_pack_bits(B, nb, log2D, st);
            if (staged) launch_coin_pack(B.b_q8, pieces, part_b, nb, log2D, ctx->coin, st);
            Timed t(ctx, EDEN_K_ENC_FINISH, nb, st);
            launch_enc_finish(B, nb, hdr_d, log2D, seed, part_n2, nparts_n2, part_ip, nparts_ip, ctx->partial_stride,
                              ctx->dev_status, ctx->coin.total, st);
        }
        if (!launch_ok()) return EDEN_ERR_HIP;
    }
    return EDEN_OK;
}

// Budgets that change the dimension of the transform (sparsification before the rotation) cannot share a call with
// the others: 0 = none of the senders, 1 = all in pairs (EDEN_B_HALF_PRE), 2 = all m-of-64, -1 = a mix.
static int sparsify_mode(const uint32_t *b_q8, uint32_t n) {
    uint32_t pre = 0, sp = 0;
    for (uint32_t c = 0; c < n; ++c) { pre += (b_q8[c] == kPreHalf); sp += (sparse_m(b_q8[c]) != 0); }
    if (pre == 0 && sp == 0) return 0;
    if (pre == n) return 1;
    if (sp == n) return 2;
    return -1;
}

// Argument checks of eden_encode that do not depend on a context.
static int check_encode_args(const float *const *x_dev, const uint32_t *client_ids, const uint32_t *b_q8, uint32_t n, uint64_t d,
                             void *const *msgs_dev, const size_t *msg_capacity) {
    if (!x_dev || !client_ids || !b_q8 || !msgs_dev || !msg_capacity || n == 0 || d == 0) return EDEN_ERR_INVALID_ARG;
    for (uint32_t c = 0; c < n; ++c) {
        if (!x_dev[c] || !msgs_dev[c] || (reinterpret_cast<uintptr_t>(msgs_dev[c]) & 15u)) return EDEN_ERR_INVALID_ARG;
        const size_t need = eden_message_bytes(d, b_q8[c]);
        if (need == 0) return EDEN_ERR_INVALID_ARG;
        if (msg_capacity[c] < need) return EDEN_ERR_CAPACITY;
    }
    return sparsify_mode(b_q8, n) < 0 ? EDEN_ERR_INVALID_ARG : EDEN_OK;
}

// The sender side on a context whose device is current and whose limits the arguments respect.
static int encode_on(eden_ctx *ctx, const float *const *x_dev, const uint32_t *client_ids, const uint32_t *b_q8, uint32_t n,
                     uint64_t d, uint64_t seed, void *const *msgs_dev, hipStream_t st) {
    const int mode = sparsify_mode(b_q8, n);
    uint32_t ones_small[64];                                     // the sparsifying budgets quantize with b = 1
    std::vector<uint32_t> ones_big;
    const uint32_t *ones = ones_small;
    if (n <= 64) { for (uint32_t c = 0; c < n; ++c) ones_small[c] = 256u; }
    else { ones_big.assign(n, 256u); ones = ones_big.data(); }
    if (mode == 0) return encode_range(ctx, x_dev, client_ids, b_q8, b_q8, n, d, 0, d, seed, msgs_dev, st);
    if (mode == 1) return encode_range(ctx, x_dev, client_ids, ones, b_q8, n, d, 1, d, seed, msgs_dev, st);
    // b = m/64.  Senders that share m and a multi-pass size: a launch gathers the kept coordinates of a batch into the
    // workspace slots, and the 1-bit method then runs on the slots in place (a first-pass workgroup has read a tile
    // before it writes it).
    const uint32_t m0 = sparse_m(b_q8[0]);
    const uint64_t dk0 = (uint64_t)m0 * ((d + 63) / 64);
    bool same_m = ctx->T != nullptr && ceil_log2(dk0) > kLoBits;
    for (uint32_t c = 0; c < n; ++c) same_m = same_m && sparse_m(b_q8[c]) == m0;
    if (same_m) {
        const int log2Dk = ceil_log2(dk0);
        for (uint32_t first = 0; first < n; first += ctx->slots) {
            const uint32_t nb = (n - first < ctx->slots) ? n - first : ctx->slots;
            EncBatch B;
            std::memset(&B, 0, sizeof(B));
            const float *slots_x[kMaxBatch];
            for (uint32_t i = 0; i < nb; ++i) {
                B.x[i] = x_dev[first + i];
                B.client[i] = client_ids[first + i];
                slots_x[i] = ctx->T + ((size_t)i << log2Dk);
            }
            launch_sparse_gather_batch(B, nb, d, m0, seed, ctx->T, log2Dk, st);
            if (!launch_ok()) return EDEN_ERR_HIP;
            const int rc = encode_range(ctx, slots_x, &client_ids[first], ones, &b_q8[first], nb, dk0, 0, d, seed,
                                        &msgs_dev[first], st);
            if (rc != EDEN_OK) return rc;
        }
        return EDEN_OK;
    }
    // otherwise sender by sender: the kept coordinates packed into the staging vector, then the 1-bit method on it
    for (uint32_t c = 0; c < n; ++c) {
        const uint32_t m = sparse_m(b_q8[c]);
        launch_sparse_gather(x_dev[c], d, m, seed, client_ids[c], ctx->stage, st);
        if (!launch_ok()) return EDEN_ERR_HIP;
        const float *xs = ctx->stage;
        const int rc = encode_range(ctx, &xs, &client_ids[c], ones, &b_q8[c], 1, (uint64_t)m * ((d + 63) / 64), 0, d, seed,
                                    &msgs_dev[c], st);
        if (rc != EDEN_OK) return rc;
    }
    return EDEN_OK;
}

int eden_encode(eden_ctx *ctx, const float *const *x_dev, const uint32_t *client_ids, const uint32_t *b_q8, uint32_t n,
                uint64_t d, uint64_t seed, void *const *msgs_dev, const size_t *msg_capacity, void *stream) {
    if (!ctx || n > ctx->n_max || d > ctx->d_max) return EDEN_ERR_INVALID_ARG;
    const int rc = check_encode_args(x_dev, client_ids, b_q8, n, d, msgs_dev, msg_capacity);
    if (rc != EDEN_OK) return rc;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    return encode_on(ctx, x_dev, client_ids, b_q8, n, d, seed, msgs_dev, static_cast<hipStream_t>(stream));
}

// ---- eden_encode_static: the sender side for callers that cannot allocate.  Everything eden_encode keeps in a context
// (workspace slots, byte indices, staging vector, partial sums, per-sender scalars, tables) lives in one file-scope
// device array instead; every GPU the library is loaded on holds its own copy until the process ends.
namespace {
constexpr size_t static_align(size_t x) { return (x + 255) & ~(size_t)255; }
constexpr int kStaticLog2D = 20;
static_assert((1ull << kStaticLog2D) == EDEN_STATIC_MAX_D && EDEN_STATIC_MAX_N <= kMaxBatch, "limits of the static entry point");
constexpr size_t kStaticDmax = (size_t)1 << kStaticLog2D;
constexpr uint32_t kStaticPartialStride = (uint32_t)(kStaticDmax / 256 + 16);
constexpr size_t kOffT = 0;
constexpr size_t kOffCodes = kOffT + static_align(EDEN_STATIC_MAX_N * kStaticDmax * sizeof(float));
constexpr size_t kOffStage = kOffCodes + static_align(EDEN_STATIC_MAX_N * kStaticDmax);
constexpr size_t kOffPartials = kOffStage + static_align((kStaticDmax + 64) * sizeof(float));
constexpr size_t kOffEncScratch = kOffPartials + static_align(2 * (size_t)EDEN_STATIC_MAX_N * kStaticPartialStride * sizeof(double));
constexpr size_t kOffTables = kOffEncScratch + static_align(EDEN_STATIC_MAX_N * sizeof(EncScratch));
constexpr size_t kOffStatus = kOffTables + static_align(sizeof(DevTables));
constexpr size_t kStaticCoinWords = kStaticDmax / 64;           // blocks of 64 coordinates per slot
constexpr size_t kStaticCoinGroups = (kStaticCoinWords + kCoinGroup - 1) / kCoinGroup;
constexpr size_t kOffCoinMask = kOffStatus + 256;
constexpr size_t kOffCoinLocal = kOffCoinMask + static_align(EDEN_STATIC_MAX_N * kStaticCoinWords * sizeof(uint64_t));
constexpr size_t kOffCoinGroup = kOffCoinLocal + static_align(EDEN_STATIC_MAX_N * kStaticCoinWords * sizeof(uint32_t));
constexpr size_t kOffCoinTotal = kOffCoinGroup + static_align(EDEN_STATIC_MAX_N * kStaticCoinGroups * sizeof(uint32_t));
constexpr size_t kStaticBytes = kOffCoinTotal + 256;            // about 47 MiB
constexpr int kStaticMaxDevices = 64;
}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {
struct StaticDevice {
    bool ready = false;
    eden_ctx ctx;
};
StaticDevice g_static[kStaticMaxDevices];
std::mutex g_static_mutex;

// Once per device, with that device current: the address of this device's copy of `scratch` (the array's name is only a
// host-side handle, never a device address), the context that points into it, zeroed scalars and the tables.  The
// tables travel as kernel arguments, so nothing here allocates or stages a copy.
int static_context(int dev, hipStream_t st, eden_ctx **out) {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticDevice &S = g_static[dev];
    if (!S.ready) {
        unsigned char *ptr = nullptr;
        if (hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return EDEN_ERR_HIP;
        eden_ctx &c = S.ctx;
        c.device = dev;
        c.d_max = EDEN_STATIC_MAX_D;
        c.log2D_max = kStaticLog2D;
        c.n_max = EDEN_STATIC_MAX_N;
        c.slots = EDEN_STATIC_MAX_N;
        c.T = reinterpret_cast<float *>(ptr + kOffT);
        c.codes = ptr + kOffCodes;
        c.stage = reinterpret_cast<float *>(ptr + kOffStage);
        c.partials = reinterpret_cast<double *>(ptr + kOffPartials);
        c.partial_stride = kStaticPartialStride;
        c.enc_scratch = reinterpret_cast<EncScratch *>(ptr + kOffEncScratch);
        c.tables = reinterpret_cast<DevTables *>(ptr + kOffTables);
        c.dev_status = reinterpret_cast<uint32_t *>(ptr + kOffStatus);
        c.coin.mask = reinterpret_cast<uint64_t *>(ptr + kOffCoinMask);
        c.coin.local = reinterpret_cast<uint32_t *>(ptr + kOffCoinLocal);
        c.coin.group = reinterpret_cast<uint32_t *>(ptr + kOffCoinGroup);
        c.coin.total = reinterpret_cast<uint32_t *>(ptr + kOffCoinTotal);
        c.coin.group_stride = (uint32_t)kStaticCoinGroups;
        c.dec_partial = nullptr; c.dec_partial_tiles = 0; c.hist = nullptr; c.dec_scratch = nullptr;
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        c.compute_units = (uint32_t)cus;
        launch_fill_zero(reinterpret_cast<float *>(ptr + kOffEncScratch), (kOffStatus + 256 - kOffEncScratch) / sizeof(float), st);
        std::vector<DevTables> host_tables(1);
        fill_host_tables(host_tables[0]);
        const double *src = reinterpret_cast<const double *>(&host_tables[0]);
        const uint32_t total = (uint32_t)(sizeof(DevTables) / sizeof(double));
        for (uint32_t first = 0; first < total; first += kArgDoubles) {
            const uint32_t count = total - first < (uint32_t)kArgDoubles ? total - first : (uint32_t)kArgDoubles;
            launch_store_doubles(src + first, count, reinterpret_cast<double *>(c.tables) + first, st);
        }
        if (!launch_ok()) return EDEN_ERR_HIP;
        // a later call may come on another stream: the set-up must have finished before it starts
        if (hipStreamSynchronize(st) != hipSuccess) return EDEN_ERR_HIP;
        S.ready = true;
    }
    *out = &S.ctx;
    return EDEN_OK;
}
}  // namespace

int eden_encode_static(const float *const *x_dev, const uint32_t *client_ids, const uint32_t *b_q8, uint32_t n, uint64_t d,
                       uint64_t seed, void *const *msgs_dev, const size_t *msg_capacity, void *stream) {
    if (n > EDEN_STATIC_MAX_N || (d > EDEN_STATIC_MAX_D && d <= (1ull << EDEN_MAX_LOG2_D))) return EDEN_ERR_STATIC_LIMIT;
    const int rc = check_encode_args(x_dev, client_ids, b_q8, n, d, msgs_dev, msg_capacity);
    if (rc != EDEN_OK) return rc;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return EDEN_ERR_HIP;
    if (dev < 0 || dev >= kStaticMaxDevices) return EDEN_ERR_NO_DEVICE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    eden_ctx *ctx = nullptr;
    const int rs = static_context(dev, st, &ctx);
    if (rs != EDEN_OK) return rs;
    return encode_on(ctx, x_dev, client_ids, b_q8, n, d, seed, msgs_dev, st);
}

// Decodes n messages whose transformed vectors all have the same dimension and adds them to acc (see encode_range
// for the arguments; `d_src` is the length of acc, `bitmaps` may be null).  pre == 2 (multi-pass sizes only, n at
// most one launch): nothing is added to acc; every sender's decoded vector is left in its workspace slot.
// `flags_out`: where the status word of message 0 of this range goes (device, one word per message).
// `mean_n` > 0 (only where fused_mean_applies says so): acc is written with the sum divided by mean_n instead of added to.
static int decode_range(eden_ctx *ctx, const void *const *msgs_dev, const uint32_t *client_ids, const uint32_t *b_kernel,
                        const uint32_t *b_hdr, uint32_t n, uint64_t d_src, int pre, uint64_t hdr_d, uint64_t seed,
                        const uint32_t *const *bitmaps, float *acc_dev, uint32_t *flags_out, hipStream_t st,
                        float mean_n = 0.0f) {
    const uint64_t d = pre == 1 ? (d_src + 1) / 2 : d_src;       // dimension of the decoded vectors
    const int log2D = ceil_log2(d);
    bool wide_ok = true;
    for (uint32_t c = 0; c < n; ++c)
        wide_ok = wide_ok && (b_kernel[c] == 256u || b_kernel[c] == 512u || b_kernel[c] == 1024u || byte_budget(b_kernel[c]));
    const Plan pl = make_plan(log2D, wide_ok);

    for (uint32_t first = 0; first < n; first += kMaxBatch) {
        const uint32_t nb = (n - first < (uint32_t)kMaxBatch) ? n - first : (uint32_t)kMaxBatch;
        DecBatch B;
        std::memset(&B, 0, sizeof(B));
        for (uint32_t i = 0; i < nb; ++i) {
            B.msg[i] = msgs_dev[first + i];
            B.bitmap[i] = bitmaps ? bitmaps[first + i] : nullptr;
            B.client[i] = client_ids[first + i];
            B.b_q8[i] = b_kernel[first + i];
            B.hdr_b_q8[i] = b_hdr[first + i];
        }
        if (pl.lo_bits != 0) {                                   // b = 5, 6, 7: the payload is unpacked to bytes first
            bool unpack = false;
            for (uint32_t i = 0; i < nb; ++i) unpack = unpack || packs_bytes(B.b_q8[i]);
            if (unpack) {
                for (uint32_t i = 0; i < nb; ++i)
                    if (packs_bytes(B.b_q8[i])) B.codes[i] = ctx->codes + ((size_t)i << log2D);
                launch_unpack_bits(B, nb, log2D, ctx->codes, st);
            }
        }
        if (pl.lo_bits == 0) {
            Timed t(ctx, EDEN_K_DEC_SMALL, nb, st);
            launch_dec_small(B, nb, d_src, pre, hdr_d, log2D, seed, ctx->tables, acc_dev, ctx->dev_status, flags_out + first, st);
        } else {
            // Strided passes first (every sender on its own), contiguous pass last (sums the senders in registers
            // and touches acc once).  With a single strided pass the workspace of a b <= 1 sender holds fp16 (narrow_bits in eden_device.h).
            const int narrow = (pl.nhi == 1 && pre != 2) ? 1 : 0;
            bool coins = false;                                  // the receiver draws and counts the same coins
            for (uint32_t i = 0; i < nb; ++i) coins = coins || coin_q8(B.b_q8[i]);
            if (coins) launch_coin_tables(B.client, B.b_q8, nullptr, nb, seed, log2D, ctx->coin, st);
            // header checks, arrival counts and dequantization tables: a launch of its own, unless the first pass does them
            const DecPrepareArgs prep{hdr_d, seed, ctx->tables, ctx->dec_scratch, ctx->dev_status, flags_out + first};
            const HiPass &top = pl.hi[pl.nhi - 1];
            const bool first_prepares = top.wg && !coins && dec_hix_first_prepares(top.M, B, nb, narrow);
            if (!first_prepares) {
                Timed t(ctx, EDEN_K_DEC_PREPARE, nb, st);
                launch_dec_prepare(B, nb, hdr_d, log2D, seed, ctx->tables, ctx->dec_scratch, ctx->dev_status, ctx->coin.total,
                                   flags_out + first, st);
            }
            for (int i = pl.nhi - 1; i >= 0; --i) {
                const HiPass &h = pl.hi[i];
                // what the passes after this one read: whole tiles of theirs that hold part of the first d coordinates
                const uint64_t keep = round_up(d, h.p);
                if (i == pl.nhi - 1) {
                    Timed t(ctx, EDEN_K_DEC_FIRST, nb, st);
                    if (h.wg) launch_dec_hix_first(h.M, B, nb, d, log2D, seed, ctx->dec_scratch, narrow, ctx->T, ctx->coin,
                                                   first_prepares ? &prep : nullptr, st);
                    else if (h.wide) launch_dec_wide_first(B, nb, keep, log2D, ctx->dec_scratch, ctx->T, st);
                    else launch_dec_hi_first(h.M, B, nb, keep, log2D, h.p, seed, ctx->dec_scratch, narrow, ctx->T, ctx->coin, st);
                } else {
                    Timed t(ctx, EDEN_K_MID, nb, st);
                    launch_hix_mid(h.M, nb, ctx->T, log2D, round_up(d, h.p + h.M), keep, st);
                }
            }
            Timed t(ctx, EDEN_K_DEC_LAST, nb, st);
            if (pl.lo_bits == 14)
                launch_dec_lo14_last(B, nb, d_src, pre, log2D, seed, ctx->T, ctx->dec_scratch, narrow, acc_dev, 2 * ctx->compute_units,
                                     ctx->dec_partial, ctx->dec_partial_tiles, mean_n, st);
            else launch_dec_lo_last(B, nb, d_src, pre, log2D, seed, ctx->T, ctx->dec_scratch, narrow, acc_dev, st);
        }
        if (!launch_ok()) return EDEN_ERR_HIP;
    }
    return EDEN_OK;
}

// Argument checks shared by the two decode entry points; returns the sparsification mode (>= 0) or an error.
static int check_decode_args(eden_ctx *ctx, const void *const *msgs_dev, const uint32_t *client_ids, const uint32_t *b_q8,
                             uint32_t n, uint64_t d, const float *out_dev) {
    if (!ctx || !msgs_dev || !client_ids || !b_q8 || !out_dev) return EDEN_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(out_dev) & 15u) return EDEN_ERR_INVALID_ARG;
    if (n == 0 || n > ctx->n_max || d == 0 || d > ctx->d_max) return EDEN_ERR_INVALID_ARG;
    for (uint32_t c = 0; c < n; ++c) {
        if (!msgs_dev[c] || (reinterpret_cast<uintptr_t>(msgs_dev[c]) & 15u)) return EDEN_ERR_INVALID_ARG;
        if (eden_message_bytes(d, b_q8[c]) == 0) return EDEN_ERR_INVALID_ARG;
    }
    const int mode = sparsify_mode(b_q8, n);
    return mode < 0 ? EDEN_ERR_INVALID_ARG : mode;
}

static int decode_accumulate_on(eden_ctx *ctx, int mode, const void *const *msgs_dev, const uint32_t *client_ids,
                                const uint32_t *b_q8, uint32_t n, uint64_t d, uint64_t seed,
                                const uint32_t *const *recv_bitmaps_dev, float *acc_dev, hipStream_t st);

int eden_decode_accumulate(eden_ctx *ctx, const void *const *msgs_dev, const uint32_t *client_ids,
                           const uint32_t *b_q8, uint32_t n, uint64_t d, uint64_t seed,
                           const uint32_t *const *recv_bitmaps_dev, float *acc_dev, void *stream) {
    const int mode = check_decode_args(ctx, msgs_dev, client_ids, b_q8, n, d, acc_dev);
    if (mode < 0) return mode;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    return decode_accumulate_on(ctx, mode, msgs_dev, client_ids, b_q8, n, d, seed, recv_bitmaps_dev, acc_dev,
                                static_cast<hipStream_t>(stream));
}

// The whole round of a receiver in one call.  When one launch of the 14-bit contiguous pass sums all the senders (no
// sparsification before the rotation or the one by pairs, D >= 2^19, at most kMaxBatch senders) that pass writes the mean
// itself: the accumulator is neither zeroed, nor read, nor passed over once more for the division.  Otherwise the three
// steps run one after the other on mean_dev.
int eden_decode_mean(eden_ctx *ctx, const void *const *msgs_dev, const uint32_t *client_ids, const uint32_t *b_q8,
                     uint32_t n, uint64_t d, uint64_t seed, const uint32_t *const *recv_bitmaps_dev, float *mean_dev,
                     void *stream) {
    const int mode = check_decode_args(ctx, msgs_dev, client_ids, b_q8, n, d, mean_dev);
    if (mode < 0) return mode;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (mode == 0 && n <= (uint32_t)kMaxBatch && make_plan(ceil_log2(d), false).lo_bits == 14) {
        ctx->last_decode_n = n;
        return decode_range(ctx, msgs_dev, client_ids, b_q8, b_q8, n, d, 0, d, seed, recv_bitmaps_dev, mean_dev, ctx->msg_flags, st,
                            (float)n);
    }
    if (mode == 1 && n <= (uint32_t)kMaxBatch) {                 // pairs before the rotation: the same with one strided pass
        const Plan pl = make_plan(ceil_log2((d + 1) / 2), true);
        if (pl.lo_bits == 14 && pl.nhi == 1) {
            std::vector<uint32_t> ones(n, 256u);
            ctx->last_decode_n = n;
            return decode_range(ctx, msgs_dev, client_ids, ones.data(), b_q8, n, d, 1, d, seed, recv_bitmaps_dev, mean_dev,
                                ctx->msg_flags, st, (float)n);
        }
    }
    launch_fill_zero(mean_dev, d, st);
    if (!launch_ok()) return EDEN_ERR_HIP;
    const int rc = decode_accumulate_on(ctx, mode, msgs_dev, client_ids, b_q8, n, d, seed, recv_bitmaps_dev, mean_dev, st);
    if (rc != EDEN_OK) return rc;
    {
        Timed t(ctx, EDEN_K_FINALIZE, n, st);
        launch_finalize_mean(mean_dev, d, n, mean_dev, st);
    }
    return launch_ok() ? EDEN_OK : EDEN_ERR_HIP;
}

static int decode_accumulate_on(eden_ctx *ctx, int mode, const void *const *msgs_dev, const uint32_t *client_ids,
                                const uint32_t *b_q8, uint32_t n, uint64_t d, uint64_t seed,
                                const uint32_t *const *recv_bitmaps_dev, float *acc_dev, hipStream_t st) {
    std::vector<uint32_t> ones(n, 256u);
    ctx->last_decode_n = n;
    if (mode == 0) return decode_range(ctx, msgs_dev, client_ids, b_q8, b_q8, n, d, 0, d, seed, recv_bitmaps_dev, acc_dev, ctx->msg_flags, st);
    if (mode == 1) return decode_range(ctx, msgs_dev, client_ids, ones.data(), b_q8, n, d, 1, d, seed, recv_bitmaps_dev, acc_dev, ctx->msg_flags, st);
    // b = m/64 (the factor 64/m is folded into the dequantization).  Senders that share m and a multi-pass size: a batch
    // is decoded without summing, every sender into its own workspace slot, and one launch adds the values to the
    // coordinates of acc they were taken from.
    const uint32_t m0 = sparse_m(b_q8[0]);
    const uint64_t dk0 = (uint64_t)m0 * ((d + 63) / 64);
    bool same_m = ctx->T != nullptr && ceil_log2(dk0) > kLoBits;
    for (uint32_t c = 0; c < n; ++c) same_m = same_m && sparse_m(b_q8[c]) == m0;
    if (same_m) {
        const int log2Dk = ceil_log2(dk0);
        for (uint32_t first = 0; first < n; first += ctx->slots) {
            const uint32_t nb = (n - first < ctx->slots) ? n - first : ctx->slots;
            const int rc = decode_range(ctx, &msgs_dev[first], &client_ids[first], ones.data(), &b_q8[first], nb, dk0, 2, d, seed,
                                        recv_bitmaps_dev ? &recv_bitmaps_dev[first] : nullptr, acc_dev, ctx->msg_flags + first, st);
            if (rc != EDEN_OK) return rc;
            DecBatch B;
            std::memset(&B, 0, sizeof(B));
            for (uint32_t i = 0; i < nb; ++i) B.client[i] = client_ids[first + i];
            launch_sparse_scatter_batch(B, nb, d, m0, seed, ctx->T, log2Dk, acc_dev, st);
            if (!launch_ok()) return EDEN_ERR_HIP;
        }
        return EDEN_OK;
    }
    // otherwise sender by sender (the kept coordinates differ): the 1-bit decode into the staging vector, then the values
    // go back to their coordinates of acc
    for (uint32_t c = 0; c < n; ++c) {
        const uint32_t m = sparse_m(b_q8[c]);
        const uint64_t dk = (uint64_t)m * ((d + 63) / 64);
        launch_fill_zero(ctx->stage, dk, st);
        if (!launch_ok()) return EDEN_ERR_HIP;
        const uint32_t *bm = recv_bitmaps_dev ? recv_bitmaps_dev[c] : nullptr;
        const int rc = decode_range(ctx, &msgs_dev[c], &client_ids[c], ones.data(), &b_q8[c], 1, dk, 0, d, seed,
                                    recv_bitmaps_dev ? &bm : nullptr, ctx->stage, ctx->msg_flags + c, st);
        if (rc != EDEN_OK) return rc;
        launch_sparse_scatter(ctx->stage, d, m, seed, client_ids[c], acc_dev, st);
        if (!launch_ok()) return EDEN_ERR_HIP;
    }
    return EDEN_OK;
}

int eden_finalize_mean(eden_ctx *ctx, const float *acc_dev, uint64_t d, uint32_t n, float *mean_dev, void *stream) {
    if (!ctx || !acc_dev || !mean_dev || d == 0 || d > ctx->d_max || n == 0) return EDEN_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    {
        Timed t(ctx, EDEN_K_FINALIZE, n, static_cast<hipStream_t>(stream));
        launch_finalize_mean(acc_dev, d, n, mean_dev, static_cast<hipStream_t>(stream));
    }
    return launch_ok() ? EDEN_OK : EDEN_ERR_HIP;
}

int eden_last_device_status(eden_ctx *ctx, void *stream, uint32_t *status_out) {
    if (!ctx || !status_out) return EDEN_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t v = 0;
    if (hipMemcpyAsync(&v, ctx->dev_status, sizeof(v), hipMemcpyDeviceToHost, st) != hipSuccess) return EDEN_ERR_HIP;
    if (hipMemsetAsync(ctx->dev_status, 0, sizeof(uint32_t), st) != hipSuccess) return EDEN_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return EDEN_ERR_HIP;
    *status_out = v;
    return EDEN_OK;
}

int eden_last_decode_flags(eden_ctx *ctx, void *stream, uint32_t *flags_out, uint32_t n) {
    if (!ctx || !flags_out || n == 0 || n > ctx->last_decode_n) return EDEN_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(flags_out, ctx->msg_flags, (size_t)n * sizeof(uint32_t), hipMemcpyDeviceToHost, st) != hipSuccess) return EDEN_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return EDEN_ERR_HIP;
    return EDEN_OK;
}

size_t eden_message_length(const void *header_host) {
    if (!header_host) return 0;
    MsgHeader h;
    std::memcpy(&h, header_host, sizeof(h));
    if (h.magic != kMagic || h.log2D > (uint32_t)EDEN_MAX_LOG2_D) return 0;
    const size_t room = eden_message_bytes(h.d, h.b_q8);
    if (room == 0 || !coin_q8(h.b_q8)) return room;
    const uint64_t D = 1ull << h.log2D;
    if (h.extra_bits > D) return 0;
    return EDEN_HEADER_BYTES + (size_t)(payload_a_bytes(D, (int)(coin_q8(h.b_q8) >> 8), 1) + coin_b_bytes(h.extra_bits));
}

static bool pow2_dim(uint64_t D) { return D >= 1 && D <= (1ull << EDEN_MAX_LOG2_D) && (D & (D - 1)) == 0; }

int eden_make_loss_bitmap(eden_ctx *ctx, uint64_t seed, uint32_t client_id, uint64_t D, uint32_t drop_q32,
                          uint32_t *bitmap_dev, void *stream) {
    if (!ctx || !bitmap_dev || !pow2_dim(D)) return EDEN_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    const uint32_t npk = D >= EDEN_PACKET_COORDS ? (uint32_t)(D / EDEN_PACKET_COORDS) : 1u;
    launch_loss_bitmap(stream_key(seed, kStreamLoss, client_id), npk, drop_q32, bitmap_dev,
                       static_cast<hipStream_t>(stream));
    return launch_ok() ? EDEN_OK : EDEN_ERR_HIP;
}

int eden_make_sign_bits(eden_ctx *ctx, uint64_t seed, uint32_t client_id, uint64_t D, uint64_t *bits_dev, void *stream) {
    if (!ctx || !bits_dev || !pow2_dim(D)) return EDEN_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    const uint64_t nwords = D >= 64 ? D / 64 : 1;
    launch_hash_bits(stream_key(seed, kStreamSign, client_id), nwords, bits_dev, static_cast<hipStream_t>(stream));
    return launch_ok() ? EDEN_OK : EDEN_ERR_HIP;
}

int eden_make_subsample_bits(eden_ctx *ctx, uint64_t seed, uint32_t client_id, uint64_t D, uint64_t *bits_dev,
                             void *stream) {
    if (!ctx || !bits_dev || !pow2_dim(D)) return EDEN_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    const uint64_t nwords = D >= 128 ? D / 128 : 1;
    launch_hash_bits(stream_key(seed, kStreamSubsample, client_id), nwords, bits_dev, static_cast<hipStream_t>(stream));
    return launch_ok() ? EDEN_OK : EDEN_ERR_HIP;
}

int eden_index_entropy(eden_ctx *ctx, const void *msg_dev, uint64_t d, uint32_t b_q8, double *out_dev, void *stream) {
    if (!ctx || !msg_dev || !out_dev || d == 0 || d > ctx->d_max || !grid_q15(b_q8)) return EDEN_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    const uint64_t D = 1ull << ceil_log2(d);
    launch_byte_entropy(static_cast<const uint8_t *>(msg_dev) + EDEN_HEADER_BYTES, D, ctx->hist, out_dev,
                        static_cast<hipStream_t>(stream));
    return launch_ok() ? EDEN_OK : EDEN_ERR_HIP;
}

int eden_sq_error(eden_ctx *ctx, const float *a_dev, const float *b_dev, uint64_t d, double *out_dev, void *stream) {
    if (!ctx || !a_dev || !b_dev || !out_dev || d == 0) return EDEN_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    // the partial-sum area of the encoder doubles as scratch: 2 doubles per workgroup
    const uint32_t max_parts = ctx->slots * ctx->partial_stride;
    launch_sq_error(a_dev, b_dev, d, ctx->partials, max_parts, out_dev, static_cast<hipStream_t>(stream));
    return launch_ok() ? EDEN_OK : EDEN_ERR_HIP;
}

int eden_get_tables(uint32_t bits, double *thresholds, double *centroids) {
    const EdenHalfTable *ht = eden_half_table((int)bits);
    if (!ht || !thresholds || !centroids) return EDEN_ERR_INVALID_ARG;
    const int h = ht->half_levels;
    for (int i = 0; i < h; ++i) {
        centroids[h + i] = ht->q[i];
        centroids[h - 1 - i] = -ht->q[i];
    }
    thresholds[h - 1] = 0.0;
    for (int i = 1; i < h; ++i) {
        thresholds[h - 1 + i] = ht->t[i];
        thresholds[h - 1 - i] = -ht->t[i];
    }
    return EDEN_OK;
}

int eden_profile_enable(eden_ctx *ctx, uint32_t kind_mask, uint32_t max_records) {
    if (!ctx || max_records > (1u << 20)) return EDEN_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    while (ctx->prof_start.size() < max_records) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return EDEN_ERR_HIP;
        if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return EDEN_ERR_HIP; }
        ctx->prof_start.push_back(a);
        ctx->prof_stop.push_back(b);
    }
    ctx->prof_kind.resize(ctx->prof_start.size());
    ctx->prof_senders.resize(ctx->prof_start.size());
    ctx->prof_mask = kind_mask;
    return EDEN_OK;
}

int eden_profile_collect(eden_ctx *ctx, uint32_t *kinds, uint32_t *senders, float *ms, uint32_t cap, uint32_t *count) {
    if (!ctx || !kinds || !senders || !ms || !count) return EDEN_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (!guard.ok) return EDEN_ERR_HIP;
    uint32_t n = 0;
    for (uint32_t i = 0; i < ctx->prof_used && n < cap; ++i, ++n) {
        if (hipEventSynchronize(ctx->prof_stop[i]) != hipSuccess) return EDEN_ERR_HIP;
        float t = 0.0f;
        if (hipEventElapsedTime(&t, ctx->prof_start[i], ctx->prof_stop[i]) != hipSuccess) return EDEN_ERR_HIP;
        kinds[n] = ctx->prof_kind[i];
        senders[n] = ctx->prof_senders[i];
        ms[n] = t;
    }
    ctx->prof_used = 0;
    *count = n;
    return EDEN_OK;
}

const char *eden_kernel_name(uint32_t kind) {
    static const char *names[EDEN_K_COUNT] = {"enc_first", "mid", "enc_last", "dec_prepare", "dec_first", "dec_last",
                                              "finalize_mean", "enc_small", "dec_small", "enc_norm", "enc_finish"};
    return kind < EDEN_K_COUNT ? names[kind] : "?";
}

const char *eden_strerror(int status) {
    switch (status) {
        case EDEN_OK: return "ok";
        case EDEN_ERR_INVALID_ARG: return "invalid argument";
        case EDEN_ERR_CAPACITY: return "message buffer too small";
        case EDEN_ERR_HIP: return "HIP runtime error";
        case EDEN_ERR_NO_DEVICE: return "no usable device";
        case EDEN_ERR_STATIC_LIMIT: return "beyond the size limits of the allocation-free entry point";
        default: return "unknown status";
    }
}

}  // extern "C"
