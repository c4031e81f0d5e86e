"""Parity checker: compares the HIP library's output with the float64 oracle on the same inputs.

Bars (from the project's stated tolerances):
  * header integers, signs, masks, bitmaps: bit exact
  * packed indices: bit exact, except coordinates whose scaled rotated value lies within 1e-5 of the
    threshold between the two indices; those are counted and their fraction must be <= 1e-6.  A fraction
    of 1e-6 cannot be resolved on fewer than 10^6 coordinates (fp32 butterflies put roughly 2e-7 of the
    b = 4 coordinates on the other side of a threshold), so a single case is allowed the bar's expected count
    plus four standard deviations of a Poisson count plus one, and the bar itself is asserted on the pool of
    all cases of a test session (POOL).
    The uniform grid of Sec. 4.3 has a boundary every Delta, so the same fp32 error (E|dz| about 1.2e-7) puts
    2 E|dz| / Delta of its coordinates on the other side of one: its bar is max(1e-6, 5e-7 / Delta)
    (1e-6 down to Delta = 0.5, 5e-6 at Delta = 0.1); for the same reason the quantizers with 32..256 levels
    (b = 5..8), whose thresholds lie twice as dense with every bit, get 1e-6 * 2^(b - 4)
  * |x|^2: relative 1e-12;  S and <R(x),Q>: relative 1e-6 against the float64 value for the indices
    that the message actually carries (they differ from the oracle's only at the counted coordinates)
  * decoded means: relative L2 error <= 1e-5 (fp32 arithmetic on the GPU, float64 in the oracle),
    both sides decoding the same messages
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

from oracle import eden_oracle as o

INDEX_BOUNDARY_TOL = 1e-5
INDEX_MISMATCH_FRACTION = 1e-6
SCALE_RTOL = 1e-6
MEAN_REL_L2 = 1e-5


@dataclass
class EncodeParity:
    coords: int = 0
    mismatches: int = 0
    worst_boundary_distance: float = 0.0
    allowed: float = 0.0          # sum over the compared senders of coordinates x the fraction their budget allows


def allowed_fraction(b_q8: int) -> float:
    delta = o.grid_delta(b_q8)
    if delta:
        return max(INDEX_MISMATCH_FRACTION, 5e-7 / delta)
    if b_q8 in (1280, 1536, 1792, 2048):            # b = 5..8: twice as many thresholds per unit of z with every bit
        return INDEX_MISMATCH_FRACTION * 2.0 ** (b_q8 // 256 - 4)
    return INDEX_MISMATCH_FRACTION


def to_oracle_message(msg_tensor) -> o.Message:
    return o.Message.from_bytes(msg_tensor.cpu().numpy().tobytes())


def check_encode(x: np.ndarray, seed: int, client: int, b_q8: int, gpu_msg: o.Message, stats: EncodeParity):
    """x: the fp32 input as given to the GPU.  Raises AssertionError on any violation."""
    ref, tr = o.encode(x.astype(np.float64), seed, client, b_q8, want_trace=True)
    assert (gpu_msg.log2D, gpu_msg.d, gpu_msg.b_q8, gpu_msg.client, gpu_msg.seed) == \
           (ref.log2D, ref.d, ref.b_q8, ref.client, ref.seed & (2 ** 64 - 1))
    assert gpu_msg.status == ref.status
    assert gpu_msg.payload.size == ref.payload.size
    if ref.status != 0:
        assert gpu_msg.S == 0.0 and not gpu_msg.payload.any()
        return
    assert abs(gpu_msg.N2 - ref.N2) <= 1e-12 * ref.N2
    if o.pre_rotation(b_q8) or o.sparse_m(b_q8):
        b_q8 = 256          # the trace is that of the 1-bit message of the sparsified vector (Sec. 4.1)
    if o.grid_delta(b_q8):
        return _check_encode_grid(ref, tr, b_q8, gpu_msg, stats)
    bits, _ = o.budget(b_q8)
    thresholds, centroids = o.tables(bits)
    D = tr.z.size
    allbits = ((gpu_msg.payload[:, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(-1)
    if o.mixed(b_q8):
        # b = bits + 1/2: per-coordinate width; both parts of the payload are zero after their last bit
        wa, wb = o.plane_words(D, b_q8)
        assert not allbits[D * bits: wa * 32].any() and not allbits[wa * 32 + D // 2:].any()
        got = o.unpack_mixed(gpu_msg.payload, D, b_q8, tr.up)
        want = tr.idx
        t_hi, c_hi = o.tables(bits + 1)
        z_sent, up_sent = tr.z, tr.up
    else:
        nsent = tr.kept.size
        got = o.unpack_indices(gpu_msg.payload, bits, nsent)
        want = tr.idx[tr.kept]
        assert not allbits[nsent * bits:].any()                  # padding bits after the last index are zero
        z_sent, up_sent = tr.z[tr.kept], None
    bad = np.flatnonzero(got != want)
    stats.coords += want.size
    stats.mismatches += bad.size
    stats.allowed += want.size * allowed_fraction(b_q8)
    if bad.size:
        lo = np.minimum(got[bad], want[bad])
        assert np.all(np.abs(got[bad] - want[bad]) == 1), "index differs by more than one interval"
        if up_sent is None:
            thr = thresholds[lo]
        else:
            thr = np.where(up_sent[bad], t_hi[np.minimum(lo, t_hi.size - 1)], thresholds[np.minimum(lo, thresholds.size - 1)])
        dist = np.abs(z_sent[bad] - thr)
        stats.worst_boundary_distance = max(stats.worst_boundary_distance, float(dist.max()))
        assert dist.max() <= INDEX_BOUNDARY_TOL, f"index mismatch {dist.max():.3e} away from its threshold"
    # The scale belongs to the message's own indices (Sec. 2.3: S = |x|^2 / <R(x), Q>): one allowed flip at an
    # outer threshold moves <R(x),Q> by ~1e-7..1e-6 of its value at D = 2^20, so the reference is the float64
    # inner product taken with the indices the GPU actually sent.
    idx_gpu = tr.idx.copy()
    if up_sent is None:
        idx_gpu[tr.kept] = got
        Q = centroids[idx_gpu]
    else:
        idx_gpu = got
        Q = np.where(tr.up, c_hi[np.minimum(idx_gpu, c_hi.size - 1)], centroids[np.minimum(idx_gpu, centroids.size - 1)])
    y = tr.z * (math.sqrt(ref.N2) / math.sqrt(tr.z.size))          # R(x) = z / eta
    ip_ref = float(np.dot(y, Q))
    assert abs(gpu_msg.IP - ip_ref) <= SCALE_RTOL * ip_ref, (gpu_msg.IP, ip_ref, ref.IP)
    s_ref = ref.N2 / ip_ref
    assert abs(gpu_msg.S - s_ref) <= SCALE_RTOL * s_ref


def _check_encode_grid(ref, tr, b_q8, gpu_msg, stats):
    """Uniform grid (Sec. 4.3): byte i = round(z_i / Delta); the boundaries are Delta (n + 1/2)."""
    delta = o.grid_delta(b_q8)
    D = tr.z.size
    raw = np.frombuffer(gpu_msg.payload.tobytes(), dtype=np.int8)
    assert not raw[D:].any()
    got = raw[:D].astype(np.int64)
    want = tr.idx
    bad = np.flatnonzero(got != want)
    stats.coords += D
    stats.mismatches += bad.size
    stats.allowed += D * allowed_fraction(b_q8)
    if bad.size:
        assert np.all(np.abs(got[bad] - want[bad]) == 1), "index differs by more than one interval"
        dist = np.abs(tr.z[bad] - delta * (np.minimum(got[bad], want[bad]) + 0.5))
        stats.worst_boundary_distance = max(stats.worst_boundary_distance, float(dist.max()))
        assert dist.max() <= INDEX_BOUNDARY_TOL, f"index mismatch {dist.max():.3e} away from its boundary"
    Q = np.sign(got) * o.grid_centroids(delta)[np.abs(got)]
    y = tr.z * (math.sqrt(ref.N2) / math.sqrt(D))
    ip_ref = float(np.dot(y, Q))
    assert abs(gpu_msg.IP - ip_ref) <= SCALE_RTOL * ip_ref, (gpu_msg.IP, ip_ref, ref.IP)
    assert abs(gpu_msg.S - ref.N2 / ip_ref) <= SCALE_RTOL * ref.N2 / ip_ref


POOL = EncodeParity()        # every case of the session


def finish_encode(stats: EncodeParity):
    POOL.coords += stats.coords
    POOL.mismatches += stats.mismatches
    POOL.allowed += stats.allowed
    POOL.worst_boundary_distance = max(POOL.worst_boundary_distance, stats.worst_boundary_distance)
    # one case is a sample: its count may exceed the expected bar by Poisson noise (4 sigma); the pool may not
    allowed = int(stats.allowed + 4.0 * math.sqrt(stats.allowed) + 1.0)
    assert stats.mismatches <= allowed, f"{stats.mismatches} near-boundary mismatches in {stats.coords} coordinates"


def check_pool():
    """The fraction over everything the session has compared so far."""
    assert POOL.coords == 0 or POOL.mismatches <= max(1, int(POOL.allowed)), \
        f"{POOL.mismatches} near-boundary mismatches in {POOL.coords} coordinates"
    return POOL


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    den = float(np.linalg.norm(b))
    return float(np.linalg.norm(a.astype(np.float64) - b)) / (den if den > 0 else 1.0)
