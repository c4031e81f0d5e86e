"""eden_encode_static, the sender side for callers that cannot allocate, against eden_encode: the two run the same
kernels, so their messages must agree bit for bit (header, scale and payload).  Two calls in a row on the shared
static workspace, the second with a smaller input, then the size limits."""
import numpy as np
import pytest

from paper_2108_08842_amd import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _both_ways(eden, ctx, n, d, budgets, seed, dist):
    w = synth.Workload("static", n, d, budgets, seed, dist)
    ids = [11 + 3 * c for c in range(n)]
    xs = [torch.from_numpy(synth.client_vector(w, c)).cuda() for c in range(n)]
    want = ctx.encode(xs, ids, budgets, seed)
    # the caller's buffers, filled with a pattern first: the call must write every byte it owns
    got = [torch.full((eden.message_bytes(d, b),), 0xA5, dtype=torch.uint8, device="cuda") for b in budgets]
    eden.encode_static(xs, ids, budgets, seed, got)
    torch.cuda.synchronize()
    for c in range(n):
        a, b = want[c].cpu().numpy(), got[c].cpu().numpy()
        assert a.size == b.size
        assert np.array_equal(a[:64], b[:64]), f"header of sender {c} differs"
        assert np.array_equal(a, b), f"payload of sender {c} (b_q8={budgets[c]}) differs at byte {int(np.flatnonzero(a != b)[0])}"
    return got


def test_static_encode_matches_encode_on_two_calls_in_a_row():
    from paper_2108_08842_amd import eden
    assert torch.cuda.is_available()
    ctx = eden.Context(d_max=eden.STATIC_MAX_D, n_max=eden.STATIC_MAX_N, device=0)
    print("static encode: n=8 d=300001, every kind of budget", flush=True)
    _both_ways(eden, ctx, 8, 300_001, [256, 512, 128, 768, 1536, 384, eden.B_COIN(2.4), eden.B_GRID(0.5224)], 71, "lognormal_signed")
    print("static encode: n=2 d=5000 (smaller, same workspace)", flush=True)
    _both_ways(eden, ctx, 2, 5000, [256, 1024], 72, "normal")
    print("static encode: n=3 d=2^20 (the limit), then d=700 (one workgroup per sender)", flush=True)
    _both_ways(eden, ctx, 3, 1 << 20, [1792, 256, 640], 73, "layers")
    _both_ways(eden, ctx, 4, 700, [256, 128, 512, 2048], 74, "normal")
    print("static encode: sparsification before the rotation", flush=True)
    _both_ways(eden, ctx, 2, 200_000, [eden.B_HALF_PRE, eden.B_HALF_PRE], 75, "normal")
    _both_ways(eden, ctx, 3, 200_000, [eden.B_SPARSE(6), eden.B_SPARSE(6), eden.B_SPARSE(6)], 76, "normal")
    _both_ways(eden, ctx, 2, 200_000, [eden.B_SPARSE(6), eden.B_SPARSE(40)], 77, "normal")
    assert ctx.last_device_status() == 0
    # the messages decode like any others
    n, d, budgets = 4, 70_000, [256, 512, 1024, 384]
    w = synth.Workload("static", n, d, budgets, 78, "normal")
    ids = list(range(n))
    xs = [torch.from_numpy(synth.client_vector(w, c)).cuda() for c in range(n)]
    msgs = eden.encode_static(xs, ids, budgets, 78, ctx.alloc_messages(d, budgets))
    acc = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, ids, budgets, d, 78, acc)
    ref = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(ctx.encode(xs, ids, budgets, 78), ids, budgets, d, 78, ref)
    assert torch.equal(acc, ref)
    assert ctx.last_device_status() == 0
    ctx.close()


def test_static_encode_limits_and_argument_errors():
    from paper_2108_08842_amd import eden
    x = torch.ones(16, device="cuda")
    msg = torch.empty(eden.message_bytes(16, 256), dtype=torch.uint8, device="cuda")
    ok = eden.encode_static_raw([x.data_ptr()], [0], [256], 16, 1, [msg.data_ptr()], [msg.numel()])
    assert ok == eden.OK
    # beyond the limits: a clear status, nothing launched (the sizes are only declared, no memory of that size is touched)
    rc = eden.encode_static_raw([x.data_ptr()], [0], [256], eden.STATIC_MAX_D + 1, 1, [msg.data_ptr()], [1 << 30])
    assert rc == eden.ERR_STATIC_LIMIT and "allocation-free" in eden.strerror(rc)
    nine = eden.STATIC_MAX_N + 1
    rc = eden.encode_static_raw([x.data_ptr()] * nine, list(range(nine)), [256] * nine, 16, 1, [msg.data_ptr()] * nine,
                                [msg.numel()] * nine)
    assert rc == eden.ERR_STATIC_LIMIT
    assert eden.encode_static_raw([x.data_ptr()], [0], [256], 16, 1, [msg.data_ptr()], [msg.numel() - 1]) == eden.ERR_CAPACITY
    assert eden.encode_static_raw([x.data_ptr()], [0], [300], 16, 1, [msg.data_ptr()], [msg.numel()]) == eden.ERR_INVALID_ARG
    assert eden.encode_static_raw([0], [0], [256], 16, 1, [msg.data_ptr()], [msg.numel()]) == eden.ERR_INVALID_ARG
    torch.cuda.synchronize()
