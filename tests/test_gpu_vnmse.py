"""The experiment helper and harness: eden_sq_error against numpy, and the empirical vNMSE / NMSE of the GPU path
against the asymptotic values the paper prints (Sec. 3: 0.571 at b = 1, 0.134 at b = 2; Sec. 4.1: pi - 1 at
b = 1/2 with p = 1/2; Sec. 4.2: 1/(p E[Q^2]) - 1 under loss; Thm 2.2: NMSE = vNMSE / n for equal budgets)."""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2108_08842_amd import eden
    assert torch.cuda.is_available()
    return eden.Context(d_max=1 << 18, n_max=32, device=0)


def test_sq_error_matches_float64(ctx):
    rng = np.random.default_rng(5)
    for d in (1, 7, 1000, 100_003, 1 << 18):
        a = rng.standard_normal(d).astype(np.float32)
        b = (a + 0.1 * rng.standard_normal(d)).astype(np.float32)
        out = ctx.sq_error(torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()).cpu().numpy()
        e2 = float(np.sum((a.astype(np.float64) - b.astype(np.float64)) ** 2))
        a2 = float(np.sum(a.astype(np.float64) ** 2))
        assert abs(out[0] - e2) <= 1e-12 * e2 + 1e-300
        assert abs(out[1] - a2) <= 1e-12 * a2


def test_theory_values_are_the_printed_ones():
    from paper_2108_08842_amd import vnmse
    assert abs(vnmse.theory_vnmse(1) - (math.pi / 2 - 1)) < 1e-12          # Sec. 3, Example 1: 0.571
    assert abs(vnmse.theory_vnmse(2) - 0.1331) < 1e-3                       # Example 2 prints 0.134 (from 0.88228)
    assert abs(vnmse.theory_vnmse(0.5) - (math.pi - 1)) < 1e-12             # Sec. 4.1 / Lemma 4.3 with p = 1/2
    assert abs(vnmse.theory_vnmse(1, keep=0.9) - (math.pi / 2 / 0.9 - 1)) < 1e-12
    assert abs(vnmse.theory_vnmse(1.5) - 0.317) < 1e-3                      # Sec. 4.1
    assert abs(vnmse.theory_vnmse(3) - 0.03572) < 1e-4                      # Sec. 4.3 (the I_3 value)


@pytest.mark.parametrize("dist", ["normal", "lognormal"])
def test_vnmse_close_to_theory(ctx, dist):
    from paper_2108_08842_amd import vnmse
    d = 1 << 16
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)
    x = vnmse.draw(dist, d, gen, torch.device("cuda:0"))
    for b in (0.5, 1, 1.5, 2, 2.5, 3, 3.5, 4, 5, 6, 7, 8):
        v, se = vnmse.measure_vnmse(ctx, x, int(b * 256), 16, seed=3)
        th = vnmse.theory_vnmse(b)
        print(f"{dist} b={b}: vNMSE {v:.5f} +- {se:.5f}, theory {th:.5f}", flush=True)
        assert abs(v - th) <= 5 * se + 0.03 * th


def test_vnmse_with_sparsification_before_the_rotation(ctx):
    # Sec. 4.1: "the resulting vNMSE is similar in both cases"; (1/p)(1 + vNMSE_1) - 1 = pi - 1 at p = 1/2
    from paper_2108_08842_amd import eden, vnmse
    d = 1 << 16
    gen = torch.Generator(device="cuda")
    gen.manual_seed(14)
    x = vnmse.draw("normal", d, gen, torch.device("cuda:0"))
    v, se = vnmse.measure_vnmse(ctx, x, eden.B_HALF_PRE, 16, seed=6)
    print(f"pre-rotation b=0.5: vNMSE {v:.5f} +- {se:.5f}, theory {math.pi - 1:.5f}", flush=True)
    assert abs(v - (math.pi - 1)) <= 5 * se + 0.03 * (math.pi - 1)


def test_vnmse_of_sparse_budgets(ctx):
    # Sec. 4.1: (1 + vNMSE_1)/p - 1 = (pi/2)/p - 1, the form the paper evaluates at p = 0.1; p = m/64 here
    from paper_2108_08842_amd import eden, vnmse
    d = 1 << 16
    gen = torch.Generator(device="cuda")
    gen.manual_seed(15)
    x = vnmse.draw("lognormal", d, gen, torch.device("cuda:0"))
    for m in (4, 6, 45):                                        # 4: the kept vector is a power of two long (no padding)
        v, se = vnmse.measure_vnmse(ctx, x, eden.B_SPARSE(m), 24, seed=7)
        th = vnmse.theory_sparse(m, d)
        print(f"b={m}/64: vNMSE {v:.4f} +- {se:.4f}, theory {th:.4f}", flush=True)
        assert abs(v - th) <= 5 * se + 0.03 * th
    assert abs(vnmse.theory_sparse(4, d) - (math.pi / 2 * 16 - 1)) < 1e-12


def test_uniform_grid_vnmse_and_entropy(ctx):
    # Sec. 4.3: Delta_3 = 0.5224 gives 3 bits of entropy and vNMSE 0.022741
    from paper_2108_08842_amd import eden, vnmse
    th, ent = vnmse.theory_grid(0.5224)
    assert abs(th - 0.022741) < 2e-6 and abs(ent - 3.0) < 2e-3
    d = 1 << 17
    gen = torch.Generator(device="cuda")
    gen.manual_seed(16)
    x = vnmse.draw("lognormal", d, gen, torch.device("cuda:0"))
    B = eden.B_GRID(0.5224)
    v, se = vnmse.measure_vnmse(ctx, x, B, 16, seed=8)
    msg = ctx.encode([x], [0], [B], 8)[0]
    h = float(ctx.index_entropy(msg, d, B)[0])
    print(f"grid 0.5224: vNMSE {v:.6f} +- {se:.6f} (0.022741), entropy {h:.4f} bits (3.0)", flush=True)
    assert abs(v - 0.022741) <= 5 * se + 0.02 * 0.022741
    assert abs(h - 3.0) < 0.02
    # the entropy kernel against numpy on the same bytes
    raw = msg.cpu().numpy()[64:64 + d]
    counts = np.bincount(raw, minlength=256).astype(np.float64)
    f = counts[counts > 0] / d
    assert abs(h - float(-(f * np.log2(f)).sum())) < 1e-12


def test_vnmse_with_packet_loss(ctx):
    from paper_2108_08842_amd import vnmse
    d = 1 << 18                                                  # 256 packets: the arrived fraction is close to 0.9
    gen = torch.Generator(device="cuda")
    gen.manual_seed(12)
    x = vnmse.draw("normal", d, gen, torch.device("cuda:0"))
    v, se = vnmse.measure_vnmse(ctx, x, 256, 16, seed=4, drop_q32=int(0.1 * 2 ** 32))
    th = vnmse.theory_vnmse(1, keep=0.9)
    print(f"loss 10%: vNMSE {v:.5f} +- {se:.5f}, theory {th:.5f}", flush=True)
    assert abs(v - th) <= 5 * se + 0.05 * th


def test_nmse_is_vnmse_over_n(ctx):
    from paper_2108_08842_amd import vnmse
    d, n = 1 << 16, 8
    gen = torch.Generator(device="cuda")
    gen.manual_seed(13)
    xs = [vnmse.draw("normal", d, gen, torch.device("cuda:0")) for _ in range(n)]
    got = np.mean([vnmse.measure_nmse(ctx, xs, [256] * n, seed=s) for s in range(6)])
    th = vnmse.theory_vnmse(1) / n
    print(f"NMSE n={n}: {got:.5f}, theory {th:.5f}", flush=True)
    assert abs(got - th) <= 0.1 * th
