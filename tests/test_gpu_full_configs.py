"""GPU parity at the full sizes of the large synthetic configurations, in the launch configuration the
benchmark times (all senders in one call).  The oracle checks whole senders where it can afford to
(one sender of config 4 costs a few seconds) and properties that hold at any size elsewhere."""
import math

import numpy as np
import pytest

from oracle import eden_oracle as o
from paper_2108_08842_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _check_senders_threaded(xs, seed, ids, budgets, omsgs, senders, threads=8):
    """check_encode for several whole senders, a few at a time (numpy releases the interpreter lock in its loops)."""
    from concurrent.futures import ThreadPoolExecutor

    def one(c):
        st = parity.EncodeParity()
        parity.check_encode(xs[c], seed, ids[c], budgets[c], omsgs[c], st)
        return st

    stats = parity.EncodeParity()
    with ThreadPoolExecutor(threads) as pool:
        for c, st in zip(senders, pool.map(one, senders)):
            print(f"  sender {c}: coords={st.coords} mismatches={st.mismatches}", flush=True)
            stats.merge(st)
    return stats


@pytest.mark.timeout(900)
def test_config4_full_size():
    from paper_2108_08842_amd import eden
    w = synth.config(4)
    n, d = w.n, w.d
    D = o.padded_dim(d)
    assert D == 1 << 24
    print(f"config 4: n={n} d={d} D=2^24 b=1 seed={w.seed}", flush=True)
    xs = [synth.client_vector(w, c) for c in range(n)]
    x_dev = [torch.from_numpy(x).cuda() for x in xs]
    ctx = eden.Context(d_max=d, n_max=n, device=0)
    msgs = ctx.encode(x_dev, w.client_ids, w.b_q8, w.seed)
    torch.cuda.synchronize()
    assert ctx.last_device_status() == 0
    # encode parity on every sender, coordinate by coordinate
    omsgs = [parity.to_oracle_message(m) for m in msgs]
    stats = _check_senders_threaded(xs, w.seed, w.client_ids, w.b_q8, omsgs, list(range(n)))
    parity.finish_encode(stats)
    print("encode:", stats, flush=True)
    assert stats.coords == n * D
    # decode parity, the whole batch as the benchmark runs it: the oracle decodes the GPU's 16 messages
    acc16 = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, w.client_ids, w.b_q8, d, w.seed, acc16)
    mean16 = ctx.finalize_mean(acc16.clone(), n).cpu().numpy()
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(8) as pool:
        want = sum(pool.map(lambda m: o.decode(m, d), omsgs)) / n
    err = parity.rel_l2(mean16, want)
    print(f"decode of {n} senders: rel L2 {err:.2e}", flush=True)
    assert err <= parity.MEAN_REL_L2
    # the call the benchmark times for the receiver's round: the same bits, into a buffer that held something else
    one_call = torch.full((d,), float("nan"), device="cuda")
    ctx.decode_mean(msgs, w.client_ids, w.b_q8, d, w.seed, one_call)
    assert torch.equal(one_call.cpu().view(torch.int32), torch.from_numpy(mean16).view(torch.int32))
    # the same batch in two halves gives the same sums (linearity of the receiver), and the NMSE is near the
    # single-sender vNMSE over n (Lemma 2.2; Sec. 3 Example 1)
    half = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs[:8], w.client_ids[:8], w.b_q8[:8], d, w.seed, half)
    ctx.decode_accumulate(msgs[8:], w.client_ids[8:], w.b_q8[8:], d, w.seed, half)
    assert ((acc16 - half).norm() / acc16.norm()).item() < 1e-6
    true_mean = sum(x.astype(np.float64) for x in xs) / n
    nm = float(np.sum((mean16.astype(np.float64) - true_mean) ** 2) /
               (sum(float(np.dot(x.astype(np.float64), x.astype(np.float64))) for x in xs) / n))
    theory = (math.pi / 2 - 1) / n * d / D        # the error is spread over all D outputs, d of them are kept
    print(f"NMSE of 16 senders {nm:.4f}, (pi/2-1)/n * d/D = {theory:.4f}", flush=True)
    assert 0.8 < nm / theory < 1.25
    assert ctx.last_device_status() == 0
    ctx.close()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("d,drop,b_q8", [(9_000_001, 0.1, 256), ((1 << 24) - 5, 0.0, 256), (8_400_000, 0.5, 256),
                                         (9_500_003, 0.1, 128), ((1 << 24) - 5, 0.0, 128)])
def test_one_bit_round_at_two_to_the_24(d, drop, b_q8):
    # every sender at b = 1 (or every sender at b = 1/2, sub-sampled after the rotation) and D = 2^24: both decode passes run
    # on the matrix cores; with and without lost packets, d just above 2^23 (few rows of the second half of the workspace
    # are kept), near 2^24 (all of them) and in between
    from paper_2108_08842_amd import eden
    n = 3
    w = synth.Workload("t", n, d, [b_q8] * n, 515 + d % 100, "lognormal_signed")
    D = o.padded_dim(d)
    assert D == 1 << 24
    print(f"b = {b_q8 / 256} round: n={n} d={d} D=2^24 drop={drop} seed={w.seed}", flush=True)
    xs = [synth.client_vector(w, c) for c in range(n)]
    ids = [7, 70, 700]
    ctx = eden.Context(d_max=d, n_max=n, device=0)
    msgs = ctx.encode([torch.from_numpy(x).cuda() for x in xs], ids, w.b_q8, w.seed)
    omsgs = [parity.to_oracle_message(m) for m in msgs]
    bitmaps_dev = bitmaps_np = None
    if drop:
        bitmaps_dev = [ctx.make_loss_bitmap(w.seed, c, D, int(drop * 2 ** 32)) for c in ids]
        bitmaps_dev[1] = None                                   # a sender whose packets all arrived, among others
        bitmaps_np = [None if b is None else b.cpu().numpy().view(np.uint32) for b in bitmaps_dev]
    mean = torch.full((d,), float("nan"), device="cuda")
    ctx.decode_mean(msgs, ids, w.b_q8, d, w.seed, mean, bitmaps_dev)
    torch.cuda.synchronize()
    assert ctx.last_device_status() == 0
    want = o.decode_mean(omsgs, d, bitmaps_np)
    err = parity.rel_l2(mean.cpu().numpy(), want)
    print(f"decode: rel L2 {err:.2e}", flush=True)
    assert err <= parity.MEAN_REL_L2
    assert ctx.last_decode_flags(n) == [0] * n
    # the first pass also checks the headers and counts the arrivals here: a sender that the receiver expects under
    # another id contributes nothing and is reported; the other two are decoded as before
    wrong = [ids[0], ids[1] + 1, ids[2]]
    ctx.decode_mean(msgs, wrong, w.b_q8, d, w.seed, mean, bitmaps_dev)
    assert ctx.last_device_status() == eden.DEV_HEADER_MISMATCH
    assert ctx.last_decode_flags(n) == [0, eden.DEV_HEADER_MISMATCH, 0]
    want2 = (o.decode(omsgs[0], d, None if bitmaps_np is None else bitmaps_np[0]) +
             o.decode(omsgs[2], d, None if bitmaps_np is None else bitmaps_np[2])) / n
    assert parity.rel_l2(mean.cpu().numpy(), want2) <= parity.MEAN_REL_L2
    ctx.close()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("b_q8", [1024, 384, 768])
def test_round_of_one_budget_at_two_to_the_24(b_q8):
    # every sender at b = 4 (or 1.5, or 3) and D = 2^24: the strided passes next to the payload are the instances that hold
    # only this budget (b = 4: indices packed by a transpose across lanes), one tile per workgroup
    from paper_2108_08842_amd import eden
    n, d = 2, 9_000_000
    w = synth.Workload("t", n, d, [b_q8] * n, 4024, "lognormal_signed")
    print(f"b = {b_q8 / 256} round: n={n} d={d} D=2^24 seed={w.seed}", flush=True)
    xs = [synth.client_vector(w, c) for c in range(n)]
    ids = [31, 32]
    ctx = eden.Context(d_max=d, n_max=n, device=0)
    msgs = ctx.encode([torch.from_numpy(x).cuda() for x in xs], ids, w.b_q8, w.seed)
    omsgs = [parity.to_oracle_message(m) for m in msgs]
    stats = _check_senders_threaded(xs, w.seed, ids, w.b_q8, omsgs, [0, 1], threads=2)
    parity.finish_encode(stats)
    mean = torch.full((d,), float("nan"), device="cuda")
    ctx.decode_mean(msgs, ids, w.b_q8, d, w.seed, mean)
    torch.cuda.synchronize()
    assert ctx.last_device_status() == 0
    err = parity.rel_l2(mean.cpu().numpy(), o.decode_mean(omsgs, d))
    print(f"decode: rel L2 {err:.2e}", flush=True)
    assert err <= parity.MEAN_REL_L2
    ctx.close()


@pytest.mark.timeout(600)
def test_half_bit_before_the_rotation_at_two_to_the_24():
    # b = 1/2 with the sparsification first (Sec. 4.1) at d = 2 x 10^7: the transformed vector has 10^7 + 1 coordinates, so
    # the 1-bit path runs at D = 2^24 and the receiver's first pass is the matrix-core one; the last pass scatters the pairs
    from paper_2108_08842_amd import eden
    n, d = 2, 20_000_001
    w = synth.Workload("t", n, d, [eden.B_HALF_PRE] * n, 61, "lognormal_signed")
    print(f"b = 1/2 before the rotation: n={n} d={d} seed={w.seed}", flush=True)
    xs = [synth.client_vector(w, c) for c in range(n)]
    ids = [4, 44]
    ctx = eden.Context(d_max=d, n_max=n, device=0)
    msgs = ctx.encode([torch.from_numpy(x).cuda() for x in xs], ids, w.b_q8, w.seed)
    omsgs = [parity.to_oracle_message(m) for m in msgs]
    stats = _check_senders_threaded(xs, w.seed, ids, w.b_q8, omsgs, [0], threads=1)
    parity.finish_encode(stats)
    mean = torch.full((d,), float("nan"), device="cuda")
    ctx.decode_mean(msgs, ids, w.b_q8, d, w.seed, mean)
    torch.cuda.synchronize()
    assert ctx.last_device_status() == 0
    err = parity.rel_l2(mean.cpu().numpy(), o.decode_mean(omsgs, d))
    print(f"decode: rel L2 {err:.2e}", flush=True)
    assert err <= parity.MEAN_REL_L2
    ctx.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("ms", [[56, 56], [50, 60]], ids=["same_m", "different_m"])
def test_m_of_64_budgets_at_two_to_the_24(ms):
    # b = m/64 at d = 1.2 x 10^7: the kept coordinates (m ceil(d/64) = 9.4 .. 11.3 million) are a 1-bit problem at D = 2^24.
    # Senders that share m go through the workspace in one batch (the first encode pass works in place there: no blocked
    # layout; the decode leaves every sender's vector in its slot); different m go sender by sender through the staging
    # vector, and each of those decodes is a one-sender b = 1 round on the matrix-core passes
    from paper_2108_08842_amd import eden
    n, d = 2, 12_000_000
    budgets = [eden.B_SPARSE(m) for m in ms]
    w = synth.Workload("t", n, d, budgets, 88, "lognormal_signed")
    print(f"m of 64: d={d} m={ms} seed={w.seed}", flush=True)
    xs = [synth.client_vector(w, c) for c in range(n)]
    ids = [12, 21]
    ctx = eden.Context(d_max=d, n_max=n, device=0)
    msgs = ctx.encode([torch.from_numpy(x).cuda() for x in xs], ids, w.b_q8, w.seed)
    assert ctx.last_device_status() == 0
    omsgs = [parity.to_oracle_message(m) for m in msgs]
    stats = _check_senders_threaded(xs, w.seed, ids, w.b_q8, omsgs, [1], threads=1)
    parity.finish_encode(stats)
    mean = torch.full((d,), float("nan"), device="cuda")
    ctx.decode_mean(msgs, ids, w.b_q8, d, w.seed, mean)
    torch.cuda.synchronize()
    assert ctx.last_device_status() == 0
    err = parity.rel_l2(mean.cpu().numpy(), o.decode_mean(omsgs, d))
    print(f"decode: rel L2 {err:.2e}", flush=True)
    assert err <= parity.MEAN_REL_L2
    ctx.close()


@pytest.mark.timeout(600)
def test_more_senders_than_one_launch_at_two_to_the_24():
    # 33 senders at b = 1, D = 2^24: encode and decode go through in launches of 32 and 1; the sum equals the two parts
    # decoded by separate calls, bit for bit, and the part of one sender is the oracle's
    from paper_2108_08842_amd import eden
    n, d = 33, 8_500_000
    w = synth.Workload("t", n, d, [256] * n, 97, "normal")
    print(f"33 senders: d={d} seed={w.seed}", flush=True)
    ctx = eden.Context(d_max=d, n_max=n, device=0)
    xs = [torch.from_numpy(synth.client_vector(w, c)).cuda() for c in range(n)]
    ids = list(range(100, 100 + n))
    msgs = ctx.encode(xs, ids, w.b_q8, w.seed)
    assert ctx.last_device_status() == 0
    whole = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, ids, w.b_q8, d, w.seed, whole)
    parts = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs[:32], ids[:32], w.b_q8[:32], d, w.seed, parts)
    last = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs[32:], ids[32:], w.b_q8[32:], d, w.seed, last)
    parts += last
    assert torch.equal(whole, parts)
    one_call = torch.empty(d, device="cuda")
    ctx.decode_mean(msgs, ids, w.b_q8, d, w.seed, one_call)
    assert torch.equal(one_call, ctx.finalize_mean(whole.clone(), n))
    om = parity.to_oracle_message(msgs[32])
    st = parity.EncodeParity()
    parity.check_encode(xs[32].cpu().numpy(), w.seed, ids[32], 256, om, st)
    parity.finish_encode(st)
    assert parity.rel_l2(last.cpu().numpy(), o.decode(om, d)) <= parity.MEAN_REL_L2
    assert ctx.last_device_status() == 0
    ctx.close()


@pytest.mark.timeout(600)
def test_every_budget_at_the_headline_size():
    """d = 11,173,962 (D = 2^24: the 10-bit workgroup tile with its two exchange halves), one sender per budget kind,
    every sender checked coordinate by coordinate against the oracle, then decoded with 10% of the packets lost."""
    from paper_2108_08842_amd import eden
    d = synth.config(4).d
    groups = [[128, 384, 512, 640, 768, 896, 1024, eden.B_GRID(0.5224), 1280, 1536, 1792, 2048, eden.B_COIN(2.7)],   # one call: same transform dimension
              [eden.B_HALF_PRE, eden.B_HALF_PRE],
              [eden.B_SPARSE(6), eden.B_SPARSE(45)]]
    ctx = eden.Context(d_max=d, n_max=13, device=0)
    for gi, budgets in enumerate(groups):
        n = len(budgets)
        w = synth.Workload("all_budgets", n, d, budgets, 60 + gi, "layers")
        xs = [synth.client_vector(w, c) for c in range(n)]
        ids = list(range(20, 20 + n))
        print(f"headline size, budgets {budgets}", flush=True)
        msgs = ctx.encode([torch.from_numpy(x).cuda() for x in xs], ids, budgets, w.seed)
        assert ctx.last_device_status() == 0
        stats = parity.EncodeParity()
        om = [parity.to_oracle_message(m) for m in msgs]
        for c in range(n):
            parity.check_encode(xs[c], w.seed, ids[c], budgets[c], om[c], stats)
        parity.finish_encode(stats)
        print("encode:", stats, flush=True)
        # packets refer to the transformed vector; the m-of-64 senders have their own dimensions
        if o.sparse_m(budgets[0]):
            Ds = [o.padded_dim(o.sparse_m(b) * ((d + 63) // 64)) for b in budgets]
        else:
            Ds = [o.padded_dim((d + 1) // 2 if o.pre_rotation(budgets[0]) else d)] * n
        bm = [ctx.make_loss_bitmap(w.seed, ids[c], Ds[c], int(0.1 * 2 ** 32)) for c in range(n)]
        acc = torch.zeros(d, device="cuda")
        ctx.decode_accumulate(msgs, ids, budgets, d, w.seed, acc, bm)
        got = ctx.finalize_mean(acc, n).cpu().numpy()
        want = o.decode_mean(om, d, [b.cpu().numpy().view(np.uint32) for b in bm])
        err = parity.rel_l2(got, want)
        print(f"decode with 10% loss: rel L2 {err:.2e}", flush=True)
        assert err <= parity.MEAN_REL_L2
        assert ctx.last_device_status() == 0
    ctx.close()


def _sampled_rows_check(x64, seed, client, idx_gpu_at, samples, thresholds):
    """Indices of single coordinates computed one by one: z_i = sqrt(D)/|x| * D^-1/2 * sum_j H[i][j] s_j x_j."""
    D = o.padded_dim(x64.size)
    s = o.rademacher(seed, client, D)
    xp = np.zeros(D)
    xp[:x64.size] = x64
    sx = s * xp
    n2 = float(np.dot(x64, x64))
    j = np.arange(D, dtype=np.int64)
    near = 0
    for i in samples:
        par = np.bitwise_and(j, int(i))
        # parity of popcount(i & j) by folding
        for sh in (32, 16, 8, 4, 2, 1):
            par ^= par >> sh
        row = 1.0 - 2.0 * (par & 1)
        z = float(np.dot(row, sx)) / np.sqrt(n2)
        want = int(o.quantize_indices(np.array([z]), thresholds)[0])
        got = int(idx_gpu_at(int(i)))
        if got != want:
            assert abs(got - want) == 1 and abs(z - thresholds[min(got, want)]) <= parity.INDEX_BOUNDARY_TOL, (i, z, got, want)
            near += 1
    return near


def test_three_pass_size():
    """D = 2^25: lo14, workgroup-tile strided pass on bits 14..20, wave-tile strided pass on bits 21..24."""
    from paper_2108_08842_amd import eden
    d = (1 << 24) + 12345
    coin = eden.B_COIN(1.5)
    w = synth.Workload("three_pass", 3, d, [256, 768, coin], 25, "normal_outliers")
    print(f"three passes: n=3 d={d} D=2^25 budgets={w.b_q8} seed={w.seed}", flush=True)
    xs = [synth.client_vector(w, c) for c in range(3)]
    ctx = eden.Context(d_max=d, n_max=3, device=0)
    msgs = ctx.encode([torch.from_numpy(x).cuda() for x in xs], [5, 9, 12], w.b_q8, w.seed)
    assert ctx.last_device_status() == 0
    stats = parity.EncodeParity()
    om = [parity.to_oracle_message(m) for m in msgs]
    parity.check_encode(xs[1], w.seed, 9, 768, om[1], stats)         # two whole senders through the oracle (b = 3, 1.5)
    parity.check_encode(xs[2], w.seed, 12, coin, om[2], stats)
    parity.finish_encode(stats)
    print("encode:", stats, flush=True)
    bm = [ctx.make_loss_bitmap(w.seed, cid, 1 << 25, int(0.1 * 2 ** 32)) for cid in (5, 9, 12)]
    acc = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs[1:], [9, 12], [768, coin], d, w.seed, acc, bm[1:])
    got = ctx.finalize_mean(acc, 2).cpu().numpy()
    want = o.decode_mean(om[1:], d, [b.cpu().numpy().view(np.uint32) for b in bm[1:]])
    err = parity.rel_l2(got, want)
    print(f"decode with 10% loss: rel L2 {err:.2e}", flush=True)
    assert err <= parity.MEAN_REL_L2
    # b = 1 sender: sampled coordinates against rows of H computed one by one
    bits1 = o.unpack_indices(om[0].payload, 1, 1 << 25)
    rng = np.random.default_rng(3)
    samples = rng.integers(0, 1 << 25, 6)
    t1, _ = o.tables(1)
    _sampled_rows_check(xs[0].astype(np.float64), w.seed, 5, lambda i: bits1[i], samples, t1)
    assert ctx.last_device_status() == 0
    ctx.close()


def test_three_pass_size_wide_tiles():
    """D = 2^25 with b = 1, 2, 4 only: lo14, workgroup-tile strided pass on bits 14..21, and the wide wave tile
    (8 rows x 512 columns, 8 columns per lane) on bits 22..24 next to the payload."""
    from paper_2108_08842_amd import eden
    d = (1 << 24) + 54321
    w = synth.Workload("three_pass_wide", 5, d, [256, 512, 1024, eden.B_GRID(0.5224), 1536], 26, "lognormal_signed")
    print(f"three passes, wide tiles: n=5 d={d} D=2^25 budgets={w.b_q8} seed={w.seed}", flush=True)
    xs = [synth.client_vector(w, c) for c in range(5)]
    ctx = eden.Context(d_max=d, n_max=5, device=0)
    ids = [2, 7, 11, 13, 17]
    msgs = ctx.encode([torch.from_numpy(x).cuda() for x in xs], ids, w.b_q8, w.seed)
    assert ctx.last_device_status() == 0
    stats = parity.EncodeParity()
    om = [parity.to_oracle_message(m) for m in msgs]
    for c in range(5):
        parity.check_encode(xs[c], w.seed, ids[c], w.b_q8[c], om[c], stats)
    parity.finish_encode(stats)
    print("encode:", stats, flush=True)
    bm = [ctx.make_loss_bitmap(w.seed, cid, 1 << 25, int(0.1 * 2 ** 32)) for cid in ids]
    acc = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, ids, w.b_q8, d, w.seed, acc, bm)
    got = ctx.finalize_mean(acc, 5).cpu().numpy()
    want = o.decode_mean(om, d, [b.cpu().numpy().view(np.uint32) for b in bm])
    err = parity.rel_l2(got, want)
    print(f"decode of 5 senders with 10% loss: rel L2 {err:.2e}", flush=True)
    assert err <= parity.MEAN_REL_L2
    assert ctx.last_device_status() == 0
    ctx.close()


def _sampled_decode_check(om, acc_at, d, samples):
    """Coordinates of one sender's reconstruction computed one by one from the message the GPU wrote:
    x^_i = s_i D^-1/2 sum_j H[i][j] y^_j with y^ = S q[index] (Sec. 2.2.2), against the GPU's accumulator."""
    D = 1 << om.log2D
    yhat = o.decode_rotated(om)
    s = o.rademacher(om.seed, om.client, D)
    j = np.arange(D, dtype=np.int64)
    scale = float(np.sqrt(np.mean(yhat ** 2)))
    for i in samples:
        par = np.bitwise_and(j, int(i))
        for sh in (32, 16, 8, 4, 2, 1):
            par ^= par >> sh
        want = s[int(i)] * float(np.dot(1.0 - 2.0 * (par & 1), yhat)) / math.sqrt(D)
        got = float(acc_at(int(i)))
        assert abs(got - want) <= 1e-5 * scale * 4.0, (i, got, want)      # a coordinate's error against the vector's rms


@pytest.mark.timeout(1200)
def test_config5_full_size():
    """n=8, d=2^27, b=4: three passes through memory (lo14, the 10-bit workgroup tile, the wide wave tile).  One whole
    sender goes through the oracle coordinate by coordinate in both directions; two more are checked on sampled
    coordinates computed from single rows of H; the batch through properties that hold at any size."""
    from paper_2108_08842_amd import eden
    w = synth.config(5)
    n, d = w.n, w.d
    print(f"config 5: n={n} d=2^27 b=4 seed={w.seed}", flush=True)
    ctx = eden.Context(d_max=d, n_max=n, device=0)
    x_dev = []
    keep = {}
    for c in range(n):
        x = synth.client_vector(w, c)
        if c in (0, 5):
            keep[c] = x
        x_dev.append(torch.from_numpy(x).cuda())
        del x
    msgs = ctx.encode(x_dev, w.client_ids, w.b_q8, w.seed)
    torch.cuda.synchronize()
    assert ctx.last_device_status() == 0
    # sender 0, whole: every index against the oracle
    m0 = parity.to_oracle_message(msgs[0])
    stats = parity.EncodeParity()
    print("oracle encode of sender 0 ...", flush=True)
    parity.check_encode(keep[0], w.seed, w.client_ids[0], w.b_q8[0], m0, stats)
    print(f"encode: coords={stats.coords} mismatches={stats.mismatches} worst distance {stats.worst_boundary_distance:.2e}", flush=True)
    assert stats.coords == 1 << 27
    parity.finish_encode(stats)
    # sender 0, whole: the oracle decodes the GPU's message
    acc = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs[:1], w.client_ids[:1], w.b_q8[:1], d, w.seed, acc)
    got = acc.cpu().numpy()
    print("oracle decode of sender 0 ...", flush=True)
    want = o.decode(m0, d)
    err = parity.rel_l2(got, want)
    print(f"decode of sender 0: rel L2 {err:.2e}", flush=True)
    assert err <= parity.MEAN_REL_L2
    n2 = float(np.dot(keep[0].astype(np.float64), keep[0].astype(np.float64)))
    dot = float(np.dot(got.astype(np.float64), keep[0].astype(np.float64)))
    assert abs(dot / n2 - 1.0) < 1e-5, dot / n2                  # tangent property <x^, x> = |x|^2 (Sec. 2.3)
    del got, want
    # sender 5: sampled indices and sampled reconstructed coordinates, one row of H each
    t4, q4 = o.tables(4)
    m5 = parity.to_oracle_message(msgs[5])
    words = m5.payload
    rng = np.random.default_rng(11)
    near = _sampled_rows_check(keep[5].astype(np.float64), w.seed, w.client_ids[5],
                               lambda i: (int(words[i >> 3]) >> (4 * (i & 7))) & 15, rng.integers(0, 1 << 27, 6), t4)
    print(f"sender 5: sampled indices ok ({near} near a threshold)", flush=True)
    acc5 = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs[5:6], w.client_ids[5:6], w.b_q8[5:6], d, w.seed, acc5)
    _sampled_decode_check(m5, lambda i: acc5[i].item(), d, rng.integers(0, 1 << 27, 6))
    print("sender 5: sampled reconstructed coordinates ok", flush=True)
    # the batch of 8 as the benchmark runs it: linear in the messages
    acc8 = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, w.client_ids, w.b_q8, d, w.seed, acc8)
    half = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs[:3], w.client_ids[:3], w.b_q8[:3], d, w.seed, half)
    ctx.decode_accumulate(msgs[3:], w.client_ids[3:], w.b_q8[3:], d, w.seed, half)
    assert ((acc8 - half).norm() / acc8.norm()).item() < 1e-6
    assert ctx.last_device_status() == 0
    ctx.close()


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("budgets", [[512], [768, 384]], ids=["wide_plan_b2", "wave_plan_b3_b1p5"])
def test_two_to_the_26(budgets):
    """D = 2^26, whole senders through the oracle in both pass plans: lo14 + the 9-bit workgroup tile + the wide wave
    tile (every sender b in {1, 2, 4}), and lo14 + the 7-bit workgroup tile + a 5-bit wave tile on bits 21..25."""
    from paper_2108_08842_amd import eden
    d = (1 << 26) - 70_001                                       # a ragged last tile in every pass
    n = len(budgets)
    w = synth.Workload("two_to_the_26", n, d, budgets, 26 + n, "normal_outliers")
    ids = [3 + 4 * c for c in range(n)]
    print(f"D=2^26: n={n} d={d} budgets={budgets} seed={w.seed}", flush=True)
    xs = [synth.client_vector(w, c) for c in range(n)]
    ctx = eden.Context(d_max=d, n_max=n, device=0)
    msgs = ctx.encode([torch.from_numpy(x).cuda() for x in xs], ids, budgets, w.seed)
    assert ctx.last_device_status() == 0
    om = [parity.to_oracle_message(m) for m in msgs]
    stats = parity.EncodeParity()
    for c in range(n):
        print(f"oracle encode of sender {c} (b_q8={budgets[c]}) ...", flush=True)
        parity.check_encode(xs[c], w.seed, ids[c], budgets[c], om[c], stats)
    print(f"encode: coords={stats.coords} mismatches={stats.mismatches} worst distance {stats.worst_boundary_distance:.2e}", flush=True)
    assert stats.coords == n << 26
    parity.finish_encode(stats)
    bm = [ctx.make_loss_bitmap(w.seed, cid, 1 << 26, int(0.1 * 2 ** 32)) for cid in ids]
    acc = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, ids, budgets, d, w.seed, acc, bm)
    got = ctx.finalize_mean(acc, n).cpu().numpy()
    print("oracle decode ...", flush=True)
    want = o.decode_mean(om, d, [b.cpu().numpy().view(np.uint32) for b in bm])
    err = parity.rel_l2(got, want)
    print(f"decode with 10% loss: rel L2 {err:.2e}", flush=True)
    assert err <= parity.MEAN_REL_L2
    assert ctx.last_device_status() == 0
    ctx.close()
