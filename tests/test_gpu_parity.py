"""GPU parity: the HIP library (through its C ABI) against the float64 oracle, element by element."""
import numpy as np
import pytest

from oracle import eden_oracle as o
from paper_2108_08842_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def ctx():
    from paper_2108_08842_amd import eden
    assert torch.cuda.is_available(), "these tests need the MI355X"
    c = eden.Context(d_max=1 << 23, n_max=40, device=0)
    yield c
    torch.cuda.synchronize()
    c.close()


def _run_case(ctx, xs, client_ids, budgets, seed, drop_q32=0, also_oracle_msgs=True):
    """Encode on the GPU, compare with the oracle; decode the same messages on both sides."""
    from paper_2108_08842_amd import eden
    n, d = len(xs), xs[0].size
    if o.sparse_m(budgets[0]):                                  # dimension of the transform (packet bitmaps refer to it)
        assert drop_q32 == 0 or len({o.sparse_m(b) for b in budgets}) == 1
        D = o.padded_dim(o.sparse_m(budgets[0]) * ((d + 63) // 64))
    else:
        D = o.padded_dim((d + 1) // 2 if o.pre_rotation(budgets[0]) else d)
    print(f"case n={n} d={d} D=2^{D.bit_length() - 1} budgets={sorted(set(budgets))} seed={seed} drop={drop_q32}", flush=True)
    x_dev = [torch.from_numpy(x).cuda() for x in xs]
    msgs = ctx.encode(x_dev, client_ids, budgets, seed)
    torch.cuda.synchronize()
    assert ctx.last_device_status() == 0
    stats = parity.EncodeParity()
    omsgs = []
    for c in range(n):
        gm = parity.to_oracle_message(msgs[c])
        parity.check_encode(xs[c], seed, client_ids[c], budgets[c], gm, stats)
        omsgs.append(gm)
    parity.finish_encode(stats)
    print("encode:", stats, flush=True)

    bitmaps_np, bitmaps_dev = None, None
    if drop_q32:
        bitmaps_dev = [ctx.make_loss_bitmap(seed, client_ids[c], D, drop_q32) for c in range(n)]
        bitmaps_np = [b.cpu().numpy().view(np.uint32) for b in bitmaps_dev]
        for c in range(n):            # the helper's mask is the oracle's mask, bit for bit
            np.testing.assert_array_equal(bitmaps_np[c], o.loss_bitmap(seed, client_ids[c], D, drop_q32))

    # receiver: both sides decode the GPU's messages
    acc = torch.zeros(d, dtype=torch.float32, device="cuda")
    ctx.decode_accumulate(msgs, client_ids, budgets, d, seed, acc, bitmaps_dev)
    mean = ctx.finalize_mean(acc, n).cpu().numpy()
    assert ctx.last_device_status() == 0
    want = o.decode_mean(omsgs, d, bitmaps_np)
    err = parity.rel_l2(mean, want)
    assert err <= parity.MEAN_REL_L2, f"decoded mean off by {err:.3e}"

    if also_oracle_msgs:
        # and the GPU decodes messages the oracle wrote
        ref_msgs = [o.encode(xs[c].astype(np.float64), seed, client_ids[c], budgets[c]) for c in range(n)]
        dev_msgs = [torch.from_numpy(np.frombuffer(m.to_bytes(), dtype=np.uint8).copy()).cuda() for m in ref_msgs]
        acc2 = torch.zeros(d, dtype=torch.float32, device="cuda")
        ctx.decode_accumulate(dev_msgs, client_ids, budgets, d, seed, acc2, bitmaps_dev)
        mean2 = ctx.finalize_mean(acc2, n).cpu().numpy()
        want2 = o.decode_mean(ref_msgs, d, bitmaps_np)
        err2 = parity.rel_l2(mean2, want2)
        assert err2 <= parity.MEAN_REL_L2, f"decode of oracle messages off by {err2:.3e}"
    return stats


def test_hash_streams_bit_exact(ctx):
    for seed, client, D in [(0, 0, 64), (1, 5, 1024), (2 ** 63 + 11, 4_000_000_000, 1 << 16), (7, 3, 1 << 20)]:
        s = ctx.make_sign_bits(seed, client, D).cpu().numpy().view(np.uint64)
        want = o.hash_words(o.stream_key(seed, o.STREAM_SIGN, client), 0, max(1, D // 64))
        np.testing.assert_array_equal(s, want)
        m = ctx.make_subsample_bits(seed, client, D).cpu().numpy().view(np.uint64)
        want = o.hash_words(o.stream_key(seed, o.STREAM_SUBSAMPLE, client), 0, max(1, D // 128))
        np.testing.assert_array_equal(m, want)
        for drop in (0, int(0.1 * 2 ** 32), 2 ** 32 - 1):
            bm = ctx.make_loss_bitmap(seed, client, D, drop).cpu().numpy().view(np.uint32)
            np.testing.assert_array_equal(bm, o.loss_bitmap(seed, client, D, drop))


@pytest.mark.parametrize("d", [1, 2, 3, 5, 63, 64, 65, 1000, 1024, 4095, 4096])
def test_single_workgroup_sizes(ctx, d):
    w = synth.Workload("t", 3, d, [256, 512, 1024], 100 + d, "normal")
    xs = [synth.client_vector(w, c) for c in range(3)]
    _run_case(ctx, xs, [0, 1, 2], w.b_q8, w.seed)
    if d >= 2:
        _run_case(ctx, xs, [7, 8, 9], [128, 768, 256], w.seed + 1)
        _run_case(ctx, xs, [4, 5, 6], [384, 640, 896], w.seed + 2)


@pytest.mark.parametrize("d", [4097, 8192, 20_000, (1 << 16) + 17, 300_000, 1 << 18])
def test_multi_pass_sizes(ctx, d):
    w = synth.Workload("t", 8, d, [128, 256, 512, 1024, 768, 384, 640, 896], 200 + d % 1000, "lognormal_signed")
    xs = [synth.client_vector(w, c) for c in range(8)]
    _run_case(ctx, xs, [3, 1, 4, 1_000_000, 5, 9, 2, 6], w.b_q8, w.seed)
    if d > 60_000:                                            # and with lost packets
        _run_case(ctx, xs[5:], [9, 2, 6], w.b_q8[5:], w.seed, drop_q32=int(0.2 * 2 ** 32), also_oracle_msgs=False)


@pytest.mark.parametrize("d,budgets", [(1 << 21, [256, 1024]), ((1 << 21) + 5, [128, 512, 768]), (5_000_000, [256, 512]),
                                       (3_000_000, [768, 768]), (2_500_000, [384, 640, 896]), (1 << 23, [384, 256])])
def test_workgroup_tile_sizes(ctx, d, budgets):
    # D = 2^21, 2^22, 2^23: strided pass of 7, 8, 9 bits in workgroup tiles + 14-bit contiguous pass
    n = len(budgets)
    w = synth.Workload("t", n, d, budgets, 400 + d % 1000, "normal_outliers")
    xs = [synth.client_vector(w, c) for c in range(n)]
    _run_case(ctx, xs, list(range(11, 11 + n)), w.b_q8, w.seed, drop_q32=int(0.05 * 2 ** 32),
              also_oracle_msgs=(d == 1 << 21))


@pytest.mark.parametrize("d,n", [((1 << 19) + 3, 5), (1_500_000, 3), (2_500_001, 4), (5_000_000, 2), (1 << 23, 2)])
def test_rounds_of_at_most_one_bit(ctx, d, n):
    # every sender at b <= 1 and D = 2^20 .. 2^23: the receiver's contiguous pass runs ten of its fourteen bits on the
    # matrix cores (exact integer arithmetic in fp16 pieces); few tiles (the small d) are also split over the senders
    budgets = [256, 128, 256, 256, 128][:n]
    w = synth.Workload("t", n, d, budgets, 900 + d % 1000, "lognormal_signed")
    xs = [synth.client_vector(w, c) for c in range(n)]
    _run_case(ctx, xs, list(range(21, 21 + n)), w.b_q8, w.seed, drop_q32=int(0.1 * 2 ** 32), also_oracle_msgs=False)
    _run_case(ctx, xs[:2], [5, 6], [256, 256], w.seed, also_oracle_msgs=(d < 2_000_000))


@pytest.mark.parametrize("d,b_q8,drop", [(3_000_001, 256, 0.1), (2_200_000, 128, 0.0), (6_000_000, 256, 0.0),
                                         (4_300_007, 128, 0.2), (1 << 23, 128, 0.0)])
def test_uniform_rounds_on_the_matrix_cores_below_two_to_the_24(ctx, d, b_q8, drop):
    # every sender at b = 1, or every sender at b = 1/2, at D = 2^22 and 2^23: the first decode pass is the matrix-core one with
    # 256 or 512 of its 1024 rows present (a mix of the two budgets, as in the test above, takes the packed-integer pass)
    n = 3
    w = synth.Workload("t", n, d, [b_q8] * n, 321 + d % 1000, "lognormal_signed")
    xs = [synth.client_vector(w, c) for c in range(n)]
    _run_case(ctx, xs, [11, 12, 13], w.b_q8, w.seed, drop_q32=int(drop * 2 ** 32) if drop else None)


@pytest.mark.parametrize("d", [(1 << 21) - 3, 3_000_001, 5_000_001])
def test_rounds_of_four_bits_on_workgroup_tiles(ctx, d):
    # every sender at b = 4 and D = 2^21 .. 2^23 (2^24: test_gpu_full_configs.py): the strided encode pass is the instance that holds only this budget (its
    # indices are packed by a transpose across lanes instead of ballots)
    n = 2
    w = synth.Workload("t", n, d, [1024] * n, 4000 + d % 1000, "lognormal_signed")
    xs = [synth.client_vector(w, c) for c in range(n)]
    _run_case(ctx, xs, [31, 32], w.b_q8, w.seed, drop_q32=int(0.1 * 2 ** 32) if d < 4_000_000 else 0, also_oracle_msgs=False)


@pytest.mark.parametrize("d,b_q8", [(400_000, 512), (400_001, 1024), (1 << 20, 512), (900_000, 1024), (3_000_000, 512),
                                    (2_200_000, 768), (2_500_000, 384), (3_000_001, 640), (5_000_000, 896), (6_000_000, 768)])
def test_rounds_of_one_integer_budget(ctx, d, b_q8):
    # every sender at the same budget (2, 3, 4 bits or k + 1/2) at the two-pass sizes: the strided passes next to the payload
    # run the instances that hold only that budget (wave tiles at D = 2^19, 2^20; workgroup tiles above)
    n = 3
    w = synth.Workload("t", n, d, [b_q8] * n, 7000 + d % 1000, "lognormal_signed")
    xs = [synth.client_vector(w, c) for c in range(n)]
    _run_case(ctx, xs, [41, 42, 43], w.b_q8, w.seed, drop_q32=int(0.15 * 2 ** 32), also_oracle_msgs=(d < 1_000_000))


@pytest.mark.parametrize("scale", [1.0, 2e-38])
def test_four_bit_instance_writes_what_the_shared_kernel_writes(ctx, scale):
    # a launch whose senders all have b = 4 (interval search by table, transposing pack) and a launch that mixes budgets (threshold
    # counting, ballots) write the same message for the same sender, bit for bit; also for a vector so small that the table's
    # cell width underflows and the instance has to count thresholds itself
    d = (1 << 21) - 3
    w = synth.Workload("t", 2, d, [1024, 1024], 99, "lognormal_signed")
    xs = [synth.client_vector(w, c) for c in range(2)]
    xs[0] = (xs[0] / np.abs(xs[0]).max() * np.float32(scale)).astype(np.float32)
    assert np.count_nonzero(xs[0]) > d // 2
    x_dev = [torch.from_numpy(x).cuda() for x in xs]
    alone = ctx.encode(x_dev, [5, 6], [1024, 1024], w.seed)
    mixed = ctx.encode(x_dev, [5, 6], [1024, 512], w.seed)
    torch.cuda.synchronize()
    assert ctx.last_device_status() == 0
    assert torch.equal(alone[0], mixed[0])


@pytest.mark.parametrize("d", [5000, 70_000, 300_000])
def test_packet_loss_and_mixed_budgets(ctx, d):
    w = synth.Workload("t", 6, d, [128, 256, 512, 1024, 768, 128], 300 + d % 1000, "lognormal")
    xs = [synth.client_vector(w, c) for c in range(6)]
    _run_case(ctx, xs, list(range(6)), w.b_q8, w.seed, drop_q32=int(0.1 * 2 ** 32))
    _run_case(ctx, xs, list(range(6)), w.b_q8, w.seed, drop_q32=int(0.6 * 2 ** 32), also_oracle_msgs=False)


def test_config1_exact(ctx):
    w = synth.config(1)
    xs = [synth.client_vector(w, c) for c in range(w.n)]
    _run_case(ctx, xs, w.client_ids, w.b_q8, w.seed)


def test_config2_full_size(ctx):
    w = synth.config(2)
    xs = [synth.client_vector(w, c) for c in range(w.n)]
    st = _run_case(ctx, xs, w.client_ids, w.b_q8, w.seed, also_oracle_msgs=False)
    print("config 2:", st)


def test_config3_full_size(ctx):
    w = synth.config(3)
    assert set(w.b_q8) == {128, 256, 512, 1024}
    xs = [synth.client_vector(w, c) for c in range(w.n)]
    st = _run_case(ctx, xs, w.client_ids, w.b_q8, w.seed, drop_q32=w.drop_q32, also_oracle_msgs=False)
    print("config 3:", st)


def test_batches_larger_than_one_launch(ctx):
    # 40 senders: the library splits them into launches of at most 32
    d = 5000
    w = synth.Workload("t", 40, d, [256] * 40, 77, "normal")
    xs = [synth.client_vector(w, c) for c in range(40)]
    _run_case(ctx, xs, list(range(40)), w.b_q8, w.seed, also_oracle_msgs=False)


def test_decode_is_additive_and_repeatable(ctx):
    d = 100_000
    w = synth.Workload("t", 5, d, [256, 512, 1024, 128, 256], 55, "layers")
    xs = [torch.from_numpy(synth.client_vector(w, c)).cuda() for c in range(5)]
    ids = list(range(5))
    msgs = ctx.encode(xs, ids, w.b_q8, w.seed)
    msgs_again = ctx.encode(xs, ids, w.b_q8, w.seed)
    for a, b in zip(msgs, msgs_again):                       # encode is deterministic, bit for bit
        assert torch.equal(a, b)
    acc_all = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, ids, w.b_q8, d, w.seed, acc_all)
    acc_split = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs[:2], ids[:2], w.b_q8[:2], d, w.seed, acc_split)
    ctx.decode_accumulate(msgs[2:], ids[2:], w.b_q8[2:], d, w.seed, acc_split)
    err = (acc_all - acc_split).norm() / acc_all.norm()
    assert err < 1e-6
    acc_all2 = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, ids, w.b_q8, d, w.seed, acc_all2)
    assert torch.equal(acc_all, acc_all2)


def test_degenerate_vectors_and_status(ctx):
    from paper_2108_08842_amd import eden
    for d in (100, 10_000):
        x0 = np.zeros(d, dtype=np.float32)
        x1 = synth.client_vector(synth.Workload("t", 1, d, [256], 1, "normal"), 0)
        xn = x1.copy(); xn[d // 2] = np.inf
        xs = [x0, x1, xn]
        x_dev = [torch.from_numpy(x).cuda() for x in xs]
        msgs = ctx.encode(x_dev, [0, 1, 2], [256, 512, 256], 9)
        status = ctx.last_device_status()
        assert status == eden.DEV_ZERO_VECTOR | eden.DEV_NONFINITE
        stats = parity.EncodeParity()
        for c in range(3):
            parity.check_encode(xs[c], 9, c, [256, 512, 256][c], parity.to_oracle_message(msgs[c]), stats)
        acc = torch.zeros(d, device="cuda")
        ctx.decode_accumulate(msgs, [0, 1, 2], [256, 512, 256], d, 9, acc)
        only = torch.zeros(d, device="cuda")
        ctx.decode_accumulate(msgs[1:2], [1], [512], d, 9, only)
        assert torch.equal(acc, only)                        # zero / non-finite senders add nothing
        assert ctx.last_device_status() == 0
        # every packet lost -> contributes nothing, flagged
        D = o.padded_dim(d)
        empty = torch.zeros(max(1, (max(1, D // 1024) + 31) // 32), dtype=torch.int32, device="cuda")
        acc2 = torch.zeros(d, device="cuda")
        ctx.decode_accumulate(msgs[1:2], [1], [512], d, 9, acc2, [empty])
        assert not acc2.any().item()
        assert ctx.last_device_status() == eden.DEV_NOTHING_ARRIVED
        # receiver expecting another client id / seed / budget: flagged, nothing added
        acc3 = torch.zeros(d, device="cuda")
        ctx.decode_accumulate(msgs[1:2], [5], [512], d, 9, acc3)
        ctx.decode_accumulate(msgs[1:2], [1], [512], d, 10, acc3)
        ctx.decode_accumulate(msgs[1:2], [1], [256], d, 9, acc3)
        assert not acc3.any().item()
        assert ctx.last_device_status() == eden.DEV_HEADER_MISMATCH
        # which message of a batch it was: one status word per message of the last call
        acc4 = torch.zeros(d, device="cuda")
        ctx.decode_accumulate([msgs[1], msgs[1], msgs[1], msgs[0]], [1, 5, 1, 0], [512, 512, 512, 256], d, 9, acc4,
                              [None, None, empty, None])
        assert ctx.last_decode_flags(4) == [0, eden.DEV_HEADER_MISMATCH, eden.DEV_NOTHING_ARRIVED, eden.DEV_ZERO_VECTOR]
        assert ctx.last_decode_flags(2) == [0, eden.DEV_HEADER_MISMATCH]
        with pytest.raises(eden.EdenError):
            ctx.last_decode_flags(5)
        ctx.last_device_status()


def test_argument_errors(ctx):
    from paper_2108_08842_amd import eden
    d = 1000
    x = torch.zeros(d, device="cuda")
    msg = torch.zeros(eden.message_bytes(d, 256), dtype=torch.uint8, device="cuda")
    acc = torch.zeros(d, device="cuda")
    ok = dict(x_ptrs=[x.data_ptr()], client_ids=[0], b_q8=[256], d=d, seed=1, msg_ptrs=[msg.data_ptr()],
              msg_caps=[msg.numel()])
    assert ctx.encode_raw(**ok) == eden.OK
    assert ctx.encode_raw(**{**ok, "b_q8": [300]}) == eden.ERR_INVALID_ARG
    assert ctx.encode_raw(**{**ok, "b_q8": [2304]}) == eden.ERR_INVALID_ARG
    assert ctx.encode_raw(**{**ok, "d": 0}) == eden.ERR_INVALID_ARG
    assert ctx.encode_raw(**{**ok, "d": (1 << 23) + 1}) == eden.ERR_INVALID_ARG
    assert ctx.encode_raw(**{**ok, "x_ptrs": [None]}) == eden.ERR_INVALID_ARG
    assert ctx.encode_raw(**{**ok, "msg_caps": [msg.numel() - 1]}) == eden.ERR_CAPACITY
    assert ctx.encode_raw(**{**ok, "msg_ptrs": [msg.data_ptr() + 4]}) == eden.ERR_INVALID_ARG
    assert ctx.encode_raw([], [], [], d, 1, [], []) == eden.ERR_INVALID_ARG
    assert ctx.decode_accumulate_raw([msg.data_ptr()], [0], [256], d, 1, None, acc.data_ptr()) == eden.OK
    assert ctx.decode_accumulate_raw([msg.data_ptr()], [0], [256], d, 1, None, None) == eden.ERR_INVALID_ARG
    assert ctx.decode_accumulate_raw([None], [0], [256], d, 1, None, acc.data_ptr()) == eden.ERR_INVALID_ARG
    assert ctx.finalize_mean_raw(acc.data_ptr(), d, 0, acc.data_ptr()) == eden.ERR_INVALID_ARG
    assert eden.message_bytes(1, 128) == 0                   # one coordinate cannot be sub-sampled in pairs
    assert eden.message_bytes((1 << 27) + 1, 256) == 0
    torch.cuda.synchronize()
    ctx.last_device_status()


@pytest.mark.parametrize("d", [2, 3, 100, 4097, 8191, 8193, 20_001, 300_000, (1 << 20) + 3, 2_500_001])
def test_sparsification_before_the_rotation(ctx, d):
    # b = 1/2, the paper's default variant (Sec. 4.1): gather, 1-bit method in dimension ceil(d/2), scatter
    from paper_2108_08842_amd import eden
    w = synth.Workload("t", 3, d, [eden.B_HALF_PRE] * 3, 900 + d % 1000, "lognormal_signed")
    xs = [synth.client_vector(w, c) for c in range(3)]
    _run_case(ctx, xs, [3, 4, 5], w.b_q8, w.seed)
    if d > 5000:
        _run_case(ctx, xs, [3, 4, 5], w.b_q8, w.seed + 1, drop_q32=int(0.25 * 2 ** 32), also_oracle_msgs=False)
    # a call mixes this budget with others: refused
    x_dev = [torch.from_numpy(x).cuda() for x in xs[:2]]
    msgs = ctx.alloc_messages(d, [eden.B_HALF_PRE, eden.B_HALF_PRE])
    rc = ctx.encode_raw([t.data_ptr() for t in x_dev], [0, 1], [eden.B_HALF_PRE, 256], d, 1, [m.data_ptr() for m in msgs],
                        [m.numel() + 1 << 20 for m in msgs])
    assert rc == eden.ERR_INVALID_ARG


@pytest.mark.parametrize("d,m", [(40, 50), (64, 63), (65, 6), (1000, 3), (5000, 45), (70_000, 6), (300_001, 13), (3_000_000, 6),
                                 (11_173_962 // 4, 32)])
def test_sparse_budgets_m_of_64(ctx, d, m):
    # b = m/64 (Sec. 4.1, sub-bit compression with p = m/64): gather, 1-bit method on the kept coordinates, scatter
    from paper_2108_08842_amd import eden
    B = eden.B_SPARSE(m)
    w = synth.Workload("t", 3, d, [B] * 3, 1300 + d % 1000, "lognormal_signed")
    xs = [synth.client_vector(w, c) for c in range(3)]
    _run_case(ctx, xs, [8, 9, 10], w.b_q8, w.seed)
    if m * ((d + 63) // 64) >= 8192:
        _run_case(ctx, xs, [8, 9, 10], w.b_q8, w.seed + 1, drop_q32=int(0.25 * 2 ** 32), also_oracle_msgs=False)
    assert eden.message_bytes(d, B) == o.message_bytes(d, B)


def test_sparse_budget_that_keeps_only_padding(ctx):
    # d < 64 where every kept position of the block is a virtual zero: the documented outcome is a zero-vector message
    # (status bit, S = 0, all-zero payload) that contributes nothing, exactly as the oracle has it
    from paper_2108_08842_amd import eden
    d, m, seed = 4, 6, 0
    assert (o.sparse_selection(seed, 0, d, m) >= d).all()
    x = np.array([1.0, -2.0, 3.0, 0.5], dtype=np.float32)
    msgs = ctx.encode([torch.from_numpy(x).cuda()], [0], [eden.B_SPARSE(m)], seed)
    assert ctx.last_device_status() == eden.DEV_ZERO_VECTOR
    gm = parity.to_oracle_message(msgs[0])
    parity.check_encode(x, seed, 0, eden.B_SPARSE(m), gm, parity.EncodeParity())
    assert gm.status == o.STATUS_ZERO_VECTOR and gm.S == 0.0
    acc = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, [0], [eden.B_SPARSE(m)], d, seed, acc)
    assert not acc.any().item()
    assert ctx.last_device_status() == 0          # a zero vector is not a receiver-side fault


def test_sparse_budgets_with_different_m_in_one_call(ctx):
    # senders with different m have kept vectors of different sizes: they go through one at a time; senders that
    # share m go through in batches; both ways give the same messages and the same sum
    from paper_2108_08842_amd import eden
    d = 200_000
    budgets = [eden.B_SPARSE(6), eden.B_SPARSE(32), eden.B_SPARSE(6), eden.B_SPARSE(63)]
    w = synth.Workload("t", 4, d, budgets, 1444, "lognormal")
    xs = [torch.from_numpy(synth.client_vector(w, c)).cuda() for c in range(4)]
    ids = [5, 6, 7, 8]
    msgs = ctx.encode(xs, ids, budgets, w.seed)
    acc = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, ids, budgets, d, w.seed, acc)
    same = ctx.encode([xs[0], xs[2]], [5, 7], [budgets[0], budgets[2]], w.seed)      # batched path (same m)
    assert torch.equal(same[0], msgs[0]) and torch.equal(same[1], msgs[2])
    one_by_one = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(same, [5, 7], [budgets[0], budgets[2]], d, w.seed, one_by_one)
    for c in (1, 3):
        ctx.decode_accumulate([msgs[c]], [ids[c]], [budgets[c]], d, w.seed, one_by_one)
    assert ctx.last_device_status() == 0
    assert float((acc - one_by_one).norm() / one_by_one.norm()) < 1e-6
    want = o.decode_mean([parity.to_oracle_message(m) for m in msgs], d)
    assert parity.rel_l2((acc / 4).cpu().numpy(), want) <= parity.MEAN_REL_L2


@pytest.mark.parametrize("d", [1, 70, 4096, 5000, 70_000, 300_000, (1 << 20) + 1, 2_500_000])
def test_uniform_grid_budgets(ctx, d):
    # Sec. 4.3: index = round(z / Delta) in one byte; Delta_3 = 0.5224 (3 bits of entropy), a fine and a coarse grid
    from paper_2108_08842_amd import eden
    budgets = [eden.B_GRID(0.5224), eden.B_GRID(0.1), eden.B_GRID(1.5), 512]
    w = synth.Workload("t", 4, d, budgets, 1700 + d % 1000, "normal_outliers")
    xs = [synth.client_vector(w, c) for c in range(4)]
    _run_case(ctx, xs, [1, 2, 3, 4], w.b_q8, w.seed)
    if d >= (1 << 14):
        _run_case(ctx, xs, [1, 2, 3, 4], w.b_q8, w.seed + 1, drop_q32=int(0.2 * 2 ** 32), also_oracle_msgs=False)
    assert eden.message_bytes(d, budgets[0]) == o.message_bytes(d, budgets[0])


@pytest.mark.parametrize("d", [1, 3, 70, 4096, 5000, 70_000, 300_000, (1 << 20) + 1, 2_500_000, 6_000_000])
def test_budgets_of_five_to_eight_bits(ctx, d):
    # b = 5..8: 32..256-level Lloyd-Max quantizers; one-byte indices inside the kernels, packed to b bits for b = 5, 6, 7
    from paper_2108_08842_amd import eden
    budgets = [1280, 1536, 1792, 2048, 512]
    w = synth.Workload("t", 5, d, budgets, 2100 + d % 1000, "lognormal_signed")
    xs = [synth.client_vector(w, c) for c in range(5)]
    _run_case(ctx, xs, [1, 2, 3, 4, 5], w.b_q8, w.seed, also_oracle_msgs=(d <= 300_000))
    if d >= (1 << 14):
        _run_case(ctx, xs, [1, 2, 3, 4, 5], w.b_q8, w.seed + 1, drop_q32=int(0.2 * 2 ** 32), also_oracle_msgs=False)
    for b in budgets:
        assert eden.message_bytes(d, b) == o.message_bytes(d, b)


@pytest.mark.parametrize("d", [1, 2, 3, 70, 4096, 5000, 70_000, 300_000, (1 << 20) + 1, 2_500_000, 6_000_000])
def test_coin_budgets(ctx, d):
    # general non-integer b > 1 (Sec. 4.1): an independent coin per coordinate decides which quantizer it uses; the
    # message length follows from the coins and must agree with the oracle's to the word
    from paper_2108_08842_amd import eden
    budgets = [eden.B_COIN(1.3), eden.B_COIN(2.5), eden.B_COIN(3.9), eden.B_COIN(1 + 1 / 256), 384 if d >= 2 else 512]
    w = synth.Workload("t", 5, d, budgets, 2600 + d % 1000, "lognormal_signed")
    xs = [synth.client_vector(w, c) for c in range(5)]
    _run_case(ctx, xs, [6, 7, 8, 9, 10], w.b_q8, w.seed, also_oracle_msgs=(d <= 300_000))
    if d >= (1 << 14):
        _run_case(ctx, xs, [6, 7, 8, 9, 10], w.b_q8, w.seed + 1, drop_q32=int(0.2 * 2 ** 32), also_oracle_msgs=False)
    for b in budgets:
        assert eden.message_bytes(d, b) == o.message_bytes(d, b)


def test_coin_and_packed_byte_budgets_in_one_call(ctx):
    # at the workgroup-tile sizes a coin sender's pieces of the second part and a b = 5..7 sender's one-byte indices both pass
    # through the context's byte buffer, each in its sender's slot: one call with both kinds, and the very sparse and very dense coins
    from paper_2108_08842_amd import eden
    d = 2_300_007
    budgets = [eden.B_COIN(2.3), 1536, eden.B_COIN(1 + 1 / 256), 1280, eden.B_COIN(3 + 255 / 256), 256]
    w = synth.Workload("t", len(budgets), d, budgets, 2626, "lognormal_signed")
    xs = [synth.client_vector(w, c) for c in range(len(budgets))]
    _run_case(ctx, xs, list(range(60, 60 + len(budgets))), w.b_q8, w.seed, also_oracle_msgs=False)


def test_random_shapes_and_budgets(ctx):
    # 60 seeded random cases: dimension (log-uniform up to 2^18 + tail), number of senders, any supported budget
    # per sender, sometimes lost packets, sometimes the sparsification before the rotation
    from paper_2108_08842_amd import eden
    rng = np.random.default_rng(20240)
    budgets_all = [128, 256, 384, 512, 640, 768, 896, 1024, 1280, 1536, 1792, 2048, eden.B_COIN(1.7), eden.B_COIN(2.1),
                   eden.B_COIN(3.5)]
    dists = ["normal", "lognormal", "lognormal_signed", "normal_outliers", "layers"]
    for case in range(60):
        d = int(2 ** rng.uniform(1.0, 18.2))
        n = int(rng.integers(1, 6))
        pre = rng.random() < 0.15
        budgets = [eden.B_HALF_PRE] * n if pre else [int(b) for b in rng.choice(budgets_all, n)]
        w = synth.Workload("t", n, d, budgets, 5000 + case, dists[case % len(dists)])
        xs = [synth.client_vector(w, c) for c in range(n)]
        ids = [int(v) for v in rng.choice(1 << 20, n, replace=False)]
        drop = int(rng.choice([0, 0, int(0.3 * 2 ** 32)])) if d >= (1 << 14) else 0    # at least 8 packets
        _run_case(ctx, xs, ids, w.b_q8, int(rng.integers(0, 2 ** 62)), drop_q32=drop, also_oracle_msgs=(case % 4 == 0))


@pytest.mark.parametrize("kind", ["every_kind", "m_of_64_same", "m_of_64_different"])
def test_step_can_be_captured_in_a_graph(ctx, kind):
    # encode + decode + mean make no allocation and no host synchronisation, so a caller may capture them; every
    # replay, with other work in between, must reproduce the eager result bit for bit.  Covers the budgets whose
    # buffers the context holds from its creation (byte indices of b = 6, staging of the m-of-64 budgets, coin tables).
    from paper_2108_08842_amd import eden
    d = 300_000
    budgets = {"every_kind": [128, 256, 384, 512, 768, 1024, 1536, eden.B_COIN(2.3)],
               "m_of_64_same": [eden.B_SPARSE(6)] * 3,
               "m_of_64_different": [eden.B_SPARSE(6), eden.B_SPARSE(40)]}[kind]
    n = len(budgets)
    w = synth.Workload("t", n, d, budgets, 4242, "lognormal")
    D = o.padded_dim(d)
    xs = [torch.from_numpy(synth.client_vector(w, c)).cuda() for c in range(n)]
    ids = list(range(n))
    msgs = ctx.alloc_messages(d, w.b_q8)
    bitmaps = [ctx.make_loss_bitmap(w.seed, c, D, int(0.1 * 2 ** 32)) for c in ids] if kind == "every_kind" else None
    acc = torch.zeros(d, device="cuda")
    mean = torch.empty_like(acc)
    mean_one_call = torch.empty_like(acc)

    def step():
        acc.zero_()
        ctx.encode(xs, ids, w.b_q8, w.seed, msgs=msgs)
        ctx.decode_accumulate(msgs, ids, w.b_q8, d, w.seed, acc, bitmaps)
        ctx.finalize_mean(acc, n, out=mean)
        ctx.decode_mean(msgs, ids, w.b_q8, d, w.seed, mean_one_call, bitmaps)

    step()
    torch.cuda.synchronize()
    eager = mean.clone()
    assert torch.equal(mean_one_call, eager)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                               # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(3):
        mean.fill_(7.0)
        mean_one_call.fill_(9.0)
        for m in msgs:
            m.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(mean, eager)
        assert torch.equal(mean_one_call, eager)
        assert float((acc * 2).sum()) == float((acc * 2).sum())      # eager work between the replays
    assert ctx.last_device_status() == 0


@pytest.mark.parametrize("d,budgets,drop", [
    (3000, [256, 512, 1024], 0),                               # one workgroup per sender: the three steps inside the call
    (200_000, [128, 256, 768], 0.2),                           # 12-bit contiguous pass: the same
    ((1 << 19) + 77, [256, 256, 128, 256, 256], 0.1),          # few tiles, split over the senders, matrix-core pass
    (700_000, [512, 256, 1024, 384], 0),                       # few tiles, vector pass
    (5_000_000, [256, 256, 256], 0.05),                        # many tiles, matrix-core pass, last tile ragged
    (1 << 23, [1024, 256], 0),                                 # many tiles, vector pass
    (2_500_001, [0x10080, 0x10080], 0),                        # pairs before the rotation: the pair-scattering pass stores the mean
    (1_100_000, [0x10080] * 5, 0.15),                          # the same below the workgroup-tile sizes, with loss
    (200_001, [0x10080, 0x10080], 0),                          # 12-bit contiguous pass: the three steps
    (400_000, ["sparse6", "sparse6"], 0),
    (600_000, [256, 128, 512, 1024] * 10, 0.1),                # more senders than one launch takes: the three steps
])
def test_decode_mean_equals_the_three_steps(ctx, d, budgets, drop):
    # eden_decode_mean writes what zero + eden_decode_accumulate + eden_finalize_mean leave, bit for bit, whatever the
    # output buffer held, in the cases where the last pass stores the mean itself and in those where it does not
    from paper_2108_08842_amd import eden
    budgets = [eden.B_SPARSE(6) if b == "sparse6" else b for b in budgets]
    n = len(budgets)
    w = synth.Workload("t", n, d, budgets, 77 + d % 1000, "lognormal_signed")
    xs = [torch.from_numpy(synth.client_vector(w, c)).cuda() for c in range(n)]
    ids = list(range(50, 50 + n))
    msgs = ctx.encode(xs, ids, w.b_q8, w.seed)
    bitmaps = None
    if drop:
        D = o.padded_dim(d)
        bitmaps = [ctx.make_loss_bitmap(w.seed, c, D, int(drop * 2 ** 32)) for c in ids]
    acc = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, ids, w.b_q8, d, w.seed, acc, bitmaps)
    want = ctx.finalize_mean(acc, n, out=torch.empty_like(acc))
    got = torch.full((d,), float("nan"), device="cuda")
    ctx.decode_mean(msgs, ids, w.b_q8, d, w.seed, got, bitmaps)
    torch.cuda.synchronize()
    assert ctx.last_device_status() == 0
    assert torch.equal(got.view(torch.int32), want.view(torch.int32))
    assert ctx.last_decode_flags(n) == [0] * n
    assert ctx.decode_mean_raw([m.data_ptr() for m in msgs], ids, w.b_q8, d, w.seed, None, got.data_ptr() + 4) == eden.ERR_INVALID_ARG


def test_decode_mean_on_random_shapes(ctx):
    # 40 seeded random rounds (dimension log-uniform up to 6e6, 1..6 senders, any budget per sender, sometimes lost
    # packets, sometimes a sparsifying budget): the one-call receiver and the three calls leave the same bits
    from paper_2108_08842_amd import eden
    rng = np.random.default_rng(777)
    budgets_all = [128, 256, 384, 512, 768, 1024, 1536, 2048, eden.B_COIN(2.3), eden.B_GRID(0.4)]
    for case in range(40):
        d = int(2 ** rng.uniform(1.0, 22.5))
        n = int(rng.integers(1, 7))
        kind = rng.random()
        if kind < 0.1:
            budgets = [eden.B_HALF_PRE] * n
        elif kind < 0.2:
            budgets = [eden.B_SPARSE(int(rng.integers(1, 64)))] * n
        elif kind < 0.5:
            budgets = [int(b) for b in rng.choice([128, 256], n)]      # a round of at most one bit
        else:
            budgets = [int(b) for b in rng.choice(budgets_all, n)]
        budgets = [b if eden.message_bytes(d, b) else 512 for b in budgets]
        w = synth.Workload("t", n, d, budgets, 9000 + case, "lognormal_signed")
        xs = [torch.from_numpy(synth.client_vector(w, c)).cuda() for c in range(n)]
        ids = [int(v) for v in rng.choice(1 << 20, n, replace=False)]
        seed = int(rng.integers(0, 2 ** 62))
        print(f"case {case}: d={d} n={n} budgets={budgets} seed={seed}", flush=True)
        msgs = ctx.encode(xs, ids, w.b_q8, seed)
        bitmaps = None
        if d >= (1 << 14) and budgets[0] < 0x10000 and rng.random() < 0.4:
            bitmaps = [ctx.make_loss_bitmap(seed, c, o.padded_dim(d), int(0.25 * 2 ** 32)) for c in ids]
        acc = torch.zeros(d, device="cuda")
        ctx.decode_accumulate(msgs, ids, w.b_q8, d, seed, acc, bitmaps)
        want = ctx.finalize_mean(acc, n, out=torch.empty_like(acc))
        flags = ctx.last_decode_flags(n)
        got = torch.full((d,), float("nan"), device="cuda")
        ctx.decode_mean(msgs, ids, w.b_q8, d, seed, got, bitmaps)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int32), want.view(torch.int32))
        assert ctx.last_decode_flags(n) == flags
        ctx.last_device_status()                                 # a zero vector or nothing arrived is a legitimate outcome here


def test_two_contexts_on_two_streams_and_kernel_timing(ctx):
    # one context per concurrent stream: two rounds in flight at once give the results of the same rounds run alone;
    # the optional kernel timing reports every launch of the kinds it was asked for
    from paper_2108_08842_amd import eden
    d, n = 1_500_000, 4
    w = synth.Workload("t", n, d, [256, 512, 128, 1024], 777, "layers")
    xs = [torch.from_numpy(synth.client_vector(w, c)).cuda() for c in range(n)]
    ids = list(range(n))
    other = eden.Context(d_max=d, n_max=n, device=0)

    def round_on(context, seed, stream):
        with torch.cuda.stream(stream):
            msgs = context.encode(xs, ids, w.b_q8, seed)
            acc = torch.zeros(d, device="cuda")
            context.decode_accumulate(msgs, ids, w.b_q8, d, seed, acc)
            return msgs, context.finalize_mean(acc, n)

    cur = torch.cuda.current_stream()
    alone = [round_on(ctx, 1, cur), round_on(other, 2, cur)]
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    s1.wait_stream(cur); s2.wait_stream(cur)
    together = [round_on(ctx, 1, s1), round_on(other, 2, s2)]
    torch.cuda.synchronize()
    for (m_a, mean_a), (m_t, mean_t) in zip(alone, together):
        assert all(torch.equal(a, b) for a, b in zip(m_a, m_t)) and torch.equal(mean_a, mean_t)
    assert ctx.last_device_status() == 0 and other.last_device_status() == 0

    other.profile_enable(["enc_first", "enc_last", "dec_first", "dec_last"], 64)
    round_on(other, 3, cur)
    torch.cuda.synchronize()
    recs = other.profile_collect()
    assert [k for k, _, _ in recs] == ["enc_first", "enc_last", "dec_first", "dec_last"]
    assert all(s == n and 0.0 < ms < 50.0 for _, s, ms in recs)
    other.profile_enable([], 0)
    other.close()


def test_mismatch_fraction_over_all_cases():
    # runs last in this file: every encode comparison made so far in this process is in the pool
    pool = parity.check_pool()
    print("all cases:", pool, flush=True)
