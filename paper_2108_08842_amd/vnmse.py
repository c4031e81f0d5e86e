"""Empirical vNMSE / NMSE of EDEN on the GPU next to the paper's asymptotic values.

    python -m paper_2108_08842_amd.vnmse --dist lognormal --log2d 20 --budgets 0.5 1 2 4 --trials 100 --senders 8
    python -m paper_2108_08842_amd.vnmse --dist lognormal --log2d 19 --budgets 1 --tail-drop 0.1 0.3 0.5 0.7

For every budget b the vector x is encoded by `trials` independent senders (same x, different client ids, so
independent rotations; 100 trials per point as in Sec. 5.2), each message is decoded on its own and
|x - x_hat|^2 / |x|^2 is averaged: that is the vNMSE of Sec. 2.3.  Non-integer budgets above 1 use the coin budgets
(Sec. 4.1, an independent coin per coordinate); budgets below 1 other than 1/2 use m of every 64 coordinates.
`--tail-drop f` loses the last fraction f of the packets at the receiver (the "tail drops" of App. "Loss vs. Sub-bit")
and prints, next to it, the sub-bit budget that sends the same fraction of coordinates and the bound of Lemma 4.3.  Theory (d -> infinity): 1 / E[Q^2] - 1 for b >= 1 (Cor. 2.4 with the Lloyd-Max levels of
Sec. 3: pi/2 - 1 at b = 1), and 1 / (p E[Q^2]) - 1 when only a fraction p of the rotated coordinates is sent or
arrives (Lemma 4.3; b = 1/2 sends p = 1/2 of them with the 1-bit quantizer: pi - 1), and the half-and-half mixture
of E[Q^2] for b = k + 1/2 (Sec. 4.1: 0.317 at b = 1.5).  For `senders` different
vectors the NMSE of the estimated mean is compared with Thm 2.2's (1/n^2) sum_c vNMSE_c |x_c|^2 / ((1/n) sum_c |x_c|^2).

The inputs are synthetic draws of the distributions the paper's appendix uses for this experiment
(LogNormal(0,1), Normal(0,1), Exponential(1), chi^2(1), Half-Normal, Beta(2,5)); torch generates them on the device.
Everything that is measured runs in the library's kernels; torch only holds the memory.
"""
from __future__ import annotations

import argparse
import math


def expected_q2(bits: int) -> float:
    """E[Q(z)^2] for z ~ N(0,1) and the library's Lloyd-Max table of 2^bits levels (Sec. 3)."""
    from . import eden
    t, q = eden.get_tables(bits)
    edges = [-math.inf] + list(t) + [math.inf]
    cdf = lambda v: 0.5 * (1.0 + math.erf(v / math.sqrt(2.0)))
    return sum((cdf(edges[k + 1]) - cdf(edges[k])) * q[k] ** 2 for k in range(len(q)))


def theory_sparse(m: int, d: int) -> float:
    """b = m/64 with the sparsification before the rotation (Sec. 4.1): error of the sparsification, 1/p - 1, plus
    1/p times the 1-bit error of the kept vector; that vector has m ceil(d/64) entries and is padded to a power of
    two, which spreads the 1-bit error over the padding as well."""
    p = m / 64.0
    kept = m * ((d + 63) // 64)
    padded = 1 << max(0, (kept - 1).bit_length())
    return (1.0 + (1.0 / expected_q2(1) - 1.0) * kept / padded) / p - 1.0


def theory_grid(delta: float):
    """Uniform grid of Sec. 4.3 with step delta: (asymptotic vNMSE 1/E[Q^2] - 1, entropy of the indices in bits), from
    the interval probabilities and centres of mass under N(0,1)."""
    cdf = lambda v: 0.5 * math.erfc(-v / math.sqrt(2.0))
    pdf = lambda v: math.exp(-0.5 * v * v) / math.sqrt(2.0 * math.pi)
    eq2, ent = 0.0, 0.0
    n = 0
    while delta * (n - 0.5) < 8.5:
        a, b = delta * (n - 0.5), delta * (n + 0.5)
        p = cdf(b) - cdf(a) if n == 0 else 0.5 * (math.erfc(a / math.sqrt(2.0)) - math.erfc(b / math.sqrt(2.0)))
        if p > 0.0:
            c = (pdf(a) - pdf(b)) / p
            w = 1.0 if n == 0 else 2.0                  # the interval of -n mirrors the one of n
            eq2 += w * p * c * c
            ent -= w * p * math.log2(p)
        n += 1
    return 1.0 / eq2 - 1.0, ent


def theory_vnmse(b: float, keep: float = 1.0) -> float:
    """Asymptotic vNMSE for budget b when a fraction `keep` of the packets arrives.  b < 1 sends a fraction b of the
    coordinates with the 1-bit quantizer; a non-integer b > 1 mixes the two neighbouring quantizers with weights
    1 - f and f, f = b - floor(b) (Sec. 4.1: 0.317 at b = 1.5)."""
    bits = max(1, int(b))
    p = keep * min(1.0, b)
    e = expected_q2(bits)
    if b > 1 and b != int(b):
        f = b - int(b)
        e = (1.0 - f) * e + f * expected_q2(bits + 1)
    return 1.0 / (p * e) - 1.0


def budget_code(b: float, pairs: bool = False, pre_rotation: bool = False):
    """-> (the budget actually used, its b_q8 code).  b = 1/2: one of every two rotated coordinates (or, with
    `pre_rotation`, of every two coordinates of x); other b < 1: m = round(64 b) of every 64 coordinates of x;
    integers 1..8; other b in (1, 4): the coin budgets (with `pairs`, k + 1/2 uses the one-of-every-pair variant)."""
    from . import eden
    if b == 0.5:
        return b, (eden.B_HALF_PRE if pre_rotation else 128)
    if b < 1:
        m = max(1, min(63, int(round(b * 64))))
        return m / 64.0, eden.B_SPARSE(m)
    if b == int(b):
        return b, int(b) * 256
    if pairs and 2 * b == int(2 * b):
        return b, int(b * 256)
    q = int(round(256 * b))
    return q / 256.0, eden.B_COIN(q / 256.0)


def tail_drop_bitmap(D: int, fraction: float, device):
    """Received-packet bitmap (bit j & 31 of word j >> 5 set = packet j arrived) that loses the last
    round(fraction * packets) packets of 1024 rotated coordinates.  Built on the host: it is an input of the receiver."""
    import numpy as np
    import torch
    npk = max(1, D // 1024)
    lost = int(round(fraction * npk))
    flags = np.zeros(32 * ((npk + 31) // 32), dtype=np.uint8)
    flags[: npk - lost] = 1
    words = np.packbits(flags.reshape(-1, 32), axis=1, bitorder="little").view("<u4").reshape(-1)
    return torch.from_numpy(words.astype(np.int32)).to(device), (npk - lost) / npk


def eden_b_half_pre() -> int:
    from . import eden
    return eden.B_HALF_PRE


def draw(dist: str, d: int, gen, device):
    import torch
    n = lambda: torch.randn(d, generator=gen, device=device, dtype=torch.float32)
    if dist == "normal":
        return n()
    if dist == "lognormal":
        return torch.exp(n())
    if dist == "exponential":
        return -torch.log1p(-torch.rand(d, generator=gen, device=device, dtype=torch.float32))
    if dist == "chi2":
        return n() ** 2
    if dist == "halfnormal":
        return n().abs()
    if dist == "beta":            # Beta(2,5) as a ratio of sums of exponentials (Gamma(2) / (Gamma(2) + Gamma(5)))
        e = lambda k: sum(-torch.log1p(-torch.rand(d, generator=gen, device=device, dtype=torch.float32)) for _ in range(k))
        a, c = e(2), e(5)
        return a / (a + c)
    raise ValueError(dist)


DISTS = ["lognormal", "normal", "exponential", "chi2", "halfnormal", "beta"]


def measure_vnmse(ctx, x, b_q8: int, trials: int, seed: int, drop_q32: int = 0, bitmap=None):
    """Mean and standard error of |x - x_hat|^2 / |x|^2 over `trials` independent senders of the same x (client ids
    0 .. trials-1, encoded in batches of the context's size).  `drop_q32`: every sender loses its own seeded Bernoulli
    sample of packets; `bitmap`: every sender loses the packets this bitmap marks (e.g. tail_drop_bitmap)."""
    import torch
    d = x.numel()
    dt = d                                              # dimension of the transform (the packets of a loss bitmap refer to it)
    if b_q8 == eden_b_half_pre():
        dt = (d + 1) // 2
    elif (b_q8 >> 16) == 2:
        dt = (b_q8 & 0xFFFF) * ((d + 63) // 64)
    D = 1 << max(0, (dt - 1).bit_length())
    acc = torch.empty(d, dtype=torch.float32, device=x.device)
    outs = torch.empty(trials, 2, dtype=torch.float64, device=x.device)
    for first in range(0, trials, ctx.n_max):
        ids = list(range(first, min(trials, first + ctx.n_max)))
        msgs = ctx.encode([x] * len(ids), ids, [b_q8] * len(ids), seed)
        for k, c in enumerate(ids):
            acc.zero_()
            bm = [bitmap] if bitmap is not None else ([ctx.make_loss_bitmap(seed, c, D, drop_q32)] if drop_q32 else None)
            ctx.decode_accumulate([msgs[k]], [c], [b_q8], d, seed, acc, bm)
            ctx.sq_error(x, acc, out=outs[c])
    torch.cuda.synchronize()
    r = (outs[:, 0] / outs[:, 1]).cpu()
    return float(r.mean()), float(r.std(unbiased=True) / math.sqrt(trials)) if trials > 1 else 0.0


def measure_nmse(ctx, xs, b_q8, seed: int):
    """|mean - estimate|^2 / ((1/n) sum |x_c|^2) for one round with the vectors xs (Sec. 2.1)."""
    import torch
    n, d = len(xs), xs[0].numel()
    msgs = ctx.encode(xs, list(range(n)), b_q8, seed)
    acc = torch.zeros(d, dtype=torch.float32, device=xs[0].device)
    ctx.decode_accumulate(msgs, list(range(n)), b_q8, d, seed, acc)
    est = ctx.finalize_mean(acc, n)
    true_acc = torch.zeros(d, dtype=torch.float32, device=xs[0].device)
    zero = torch.zeros(d, dtype=torch.float32, device=xs[0].device)
    norms = 0.0
    for x in xs:
        true_acc += x                                   # memory-side bookkeeping of the experiment, not the method
        norms += float(ctx.sq_error(x, zero)[1])
    true_mean = true_acc / n
    e2 = float(ctx.sq_error(true_mean, est)[0])
    return e2 / (norms / n)


def main(argv=None):
    import torch
    from . import eden
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--dist", default="lognormal", choices=DISTS + ["all"])
    ap.add_argument("--log2d", type=int, nargs="+", default=[20])
    ap.add_argument("--budgets", type=float, nargs="+", default=[0.5, 1, 2, 4])
    ap.add_argument("--trials", type=int, default=100, help="independent senders per point (Sec. 5.2: 100)")
    ap.add_argument("--tail-drop", type=float, nargs="*", default=[],
                    help="fractions of the packets lost at the tail (b = 1), each next to the sub-bit budget of the same rate")
    ap.add_argument("--pairs", action="store_true", help="b = k + 1/2 with one coordinate of every pair instead of coins")
    ap.add_argument("--senders", type=int, default=8, help="senders of the NMSE round (0: skip it)")
    ap.add_argument("--loss", type=float, default=0.0, help="fraction of packets dropped at the receiver")
    ap.add_argument("--pre-rotation", action="store_true",
                    help="b = 0.5 sparsifies before the rotation (Sec. 4.1, the paper's default) instead of after it")
    ap.add_argument("--grid", type=float, nargs="*", default=[],
                    help="steps Delta of the uniform-grid quantizer (Sec. 4.3) to measure as well, e.g. 0.5224")
    ap.add_argument("--seed", type=int, default=1)
    args = ap.parse_args(argv)
    assert torch.cuda.is_available(), "this experiment runs on the GPU"
    eden.lib()
    dev = torch.device("cuda:0")
    drop_q32 = int(args.loss * 2 ** 32)
    print(f"{'dist':11s} {'d':>9s} {'b':>4s} {'vNMSE':>9s} {'+-':>8s} {'theory':>8s} {'NMSE(n)':>9s} {'theory':>8s}")
    for dist in (DISTS if args.dist == "all" else [args.dist]):
        for l2 in args.log2d:
            d = 1 << l2
            gen = torch.Generator(device=dev)
            gen.manual_seed(args.seed * 1000 + l2)
            trials = args.trials
            ctx = eden.Context(d_max=d, n_max=max(min(trials, 32), args.senders, 1), device=0)
            x = draw(dist, d, gen, dev)
            for b in args.budgets:
                b, b_q8 = budget_code(b, args.pairs, args.pre_rotation)
                if (b_q8 >> 16) == 2:
                    th = theory_sparse(b_q8 & 0xFFFF, d) if not drop_q32 else float("nan")
                else:
                    th = theory_vnmse(b, 1.0 - args.loss)
                v, se = measure_vnmse(ctx, x, b_q8, trials, args.seed, drop_q32)
                line = f"{dist:11s} {d:9d} {b:4.3g} {v:9.5f} {se:8.5f} {th:8.5f}"
                if args.senders > 0 and not drop_q32:
                    xs = [draw(dist, d, gen, dev) for _ in range(args.senders)]
                    nm = measure_nmse(ctx, xs, [b_q8] * args.senders, args.seed + 1)
                    line += f" {nm:9.5f} {th / args.senders:8.5f}"
                print(line, flush=True)
            for f in args.tail_drop:
                bm, kept = tail_drop_bitmap(d, f, dev)
                v, se = measure_vnmse(ctx, x, 256, trials, args.seed, bitmap=bm)
                m = max(1, min(63, int(round(kept * 64))))
                vs, ses = measure_vnmse(ctx, x, eden.B_SPARSE(m), trials, args.seed)
                print(f"{dist:11s} {d:9d} b=1, last {1 - kept:.3f} of the packets lost: vNMSE {v:.5f} +- {se:.5f}; "
                      f"sub-bit b={m}/64: {vs:.5f} +- {ses:.5f}; 1/(p E[Q^2]) - 1 = {theory_vnmse(1, kept):.5f} / "
                      f"{theory_sparse(m, d):.5f}", flush=True)
            for delta in args.grid:
                b_q8 = eden.B_GRID(delta)
                v, se = measure_vnmse(ctx, x, b_q8, trials, args.seed, drop_q32)
                th, ent = theory_grid(delta)
                msg = ctx.encode([x], [0], [b_q8], args.seed)[0]
                h = float(ctx.index_entropy(msg, d, b_q8)[0])
                print(f"{dist:11s} {d:9d} grid Delta={delta:g}: vNMSE {v:.6f} +- {se:.6f} (theory {th:.6f}), "
                      f"entropy {h:.4f} bits (theory {ent:.4f})", flush=True)


if __name__ == "__main__":
    main()
