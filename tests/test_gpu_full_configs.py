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
    # encode parity on three whole senders
    stats = parity.EncodeParity()
    checked = [0, 7, 15]
    omsgs = {c: parity.to_oracle_message(msgs[c]) for c in checked}
    for c in checked:
        parity.check_encode(xs[c], w.seed, w.client_ids[c], w.b_q8[c], omsgs[c], stats)
    parity.finish_encode(stats)
    print("encode:", stats, flush=True)
    # every header is sane and obeys |x|^2 exactly
    for c in range(n):
        m = parity.to_oracle_message(msgs[c])
        n2 = float(np.dot(xs[c].astype(np.float64), xs[c].astype(np.float64)))
        assert m.status == 0 and abs(m.N2 - n2) <= 1e-12 * n2 and m.S > 0
    # decode parity: the oracle decodes the GPU's messages of the three senders
    acc = torch.zeros(d, device="cuda")
    sub = [msgs[c] for c in checked]
    ctx.decode_accumulate(sub, [w.client_ids[c] for c in checked], [w.b_q8[c] for c in checked], d, w.seed, acc)
    got = ctx.finalize_mean(acc, len(checked)).cpu().numpy()
    want = o.decode_mean([omsgs[c] for c in checked], d)
    err = parity.rel_l2(got, want)
    print(f"decode of 3 senders: rel L2 {err:.2e}", flush=True)
    assert err <= parity.MEAN_REL_L2
    # the full batch of 16, as the benchmark runs it: equals the sum of two half batches (linearity of
    # the receiver) and its NMSE is near the single-sender vNMSE over n (Lemma 2.2; Sec. 3 Example 1)
    acc16 = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs, w.client_ids, w.b_q8, d, w.seed, acc16)
    half = torch.zeros(d, device="cuda")
    ctx.decode_accumulate(msgs[:8], w.client_ids[:8], w.b_q8[:8], d, w.seed, half)
    ctx.decode_accumulate(msgs[8:], w.client_ids[8:], w.b_q8[8:], d, w.seed, half)
    assert ((acc16 - half).norm() / acc16.norm()).item() < 1e-6
    mean16 = ctx.finalize_mean(acc16, n).cpu().numpy().astype(np.float64)
    true_mean = sum(x.astype(np.float64) for x in xs) / n
    nm = float(np.sum((mean16 - true_mean) ** 2) / (sum(float(np.dot(x.astype(np.float64), x.astype(np.float64))) for x in xs) / n))
    theory = (math.pi / 2 - 1) / n * d / D        # the error is spread over all D outputs, d of them are kept
    print(f"NMSE of 16 senders {nm:.4f}, (pi/2-1)/n * d/D = {theory:.4f}", flush=True)
    assert 0.8 < nm / theory < 1.25
    assert ctx.last_device_status() == 0
    ctx.close()
