"""Parity checker: compares the HIP library's output with the float64 oracle on the same inputs.

Bars (from the project's stated tolerances):
  * header integers, signs, masks, bitmaps: bit exact
  * packed indices: bit exact, except coordinates whose scaled rotated value lies within 1e-5 of the
    threshold between the two indices; those are counted and their fraction must be <= 1e-6.
    Two classes of budgets are counted apart and never subsidise each other:
      strict   b = 1/2 (either kind), m/64, 1, 2, 3, 4 and k + 1/2 / the general non-integer budgets: the bar is 1e-6.
               A case of at least 10^7 coordinates must meet the plain fraction; a smaller case is a sample (a
               fraction of 1e-6 cannot be resolved on fewer than 10^6 coordinates) and may show the bar's expected
               count plus four standard deviations of a Poisson count plus one; the pool of all cases of a test
               session (STRICT_POOL) must meet the plain fraction again.
      relaxed  the uniform grid of Sec. 4.3 has a boundary every Delta, so the fp32 error of the transform
               (E|dz| about 1.2e-7) puts 2 E|dz| / Delta of its coordinates on the other side of one: its bar is
               max(1e-6, 5e-7 / Delta); the quantizers with 32..256 levels (b = 5..8), whose thresholds lie twice
               as dense with every bit, get 1e-6 * 2^(b - 4) for the same reason.  Same rule for single cases
               and for their own pool (RELAXED_POOL).
  * |x|^2: relative 1e-12;  S and <R(x),Q>: relative 1e-6 against the float64 value for the indices
    that the message actually carries (they differ from the oracle's only at the counted coordinates)
  * decoded means: relative L2 error <= 1e-5 (fp32 arithmetic on the GPU, float64 in the oracle),
    both sides decoding the same messages
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

from oracle import eden_oracle as o

INDEX_BOUNDARY_TOL = 1e-5
INDEX_MISMATCH_FRACTION = 1e-6
LARGE_CASE_COORDS = 10 ** 7
SCALE_RTOL = 1e-6
MEAN_REL_L2 = 1e-5
UNPACK_CHUNK = 1 << 22          # coordinates unpacked at a time (bounds the memory of the bit arrays)


@dataclass
class Counter:
    coords: int = 0
    mismatches: int = 0
    allowed: float = 0.0          # sum over the compared senders of coordinates x the fraction their budget allows

    def add(self, other: "Counter"):
        self.coords += other.coords
        self.mismatches += other.mismatches
        self.allowed += other.allowed


@dataclass
class EncodeParity:
    strict: Counter = field(default_factory=Counter)
    relaxed: Counter = field(default_factory=Counter)
    worst_boundary_distance: float = 0.0

    @property
    def coords(self) -> int:
        return self.strict.coords + self.relaxed.coords

    @property
    def mismatches(self) -> int:
        return self.strict.mismatches + self.relaxed.mismatches

    def merge(self, other: "EncodeParity"):
        self.strict.add(other.strict)
        self.relaxed.add(other.relaxed)
        self.worst_boundary_distance = max(self.worst_boundary_distance, other.worst_boundary_distance)


def allowed_fraction(b_q8: int) -> float:
    delta = o.grid_delta(b_q8)
    if delta:
        return max(INDEX_MISMATCH_FRACTION, 5e-7 / delta)
    if b_q8 in (1280, 1536, 1792, 2048):            # b = 5..8: twice as many thresholds per unit of z with every bit
        return INDEX_MISMATCH_FRACTION * 2.0 ** (b_q8 // 256 - 4)
    return INDEX_MISMATCH_FRACTION


def is_relaxed(b_q8: int) -> bool:
    return bool(o.grid_delta(b_q8)) or b_q8 in (1280, 1536, 1792, 2048)


def _count(stats: EncodeParity, b_q8: int, coords: int, mismatches: int):
    c = stats.relaxed if is_relaxed(b_q8) else stats.strict
    c.coords += coords
    c.mismatches += mismatches
    c.allowed += coords * allowed_fraction(b_q8)


def to_oracle_message(msg_tensor) -> o.Message:
    return o.Message.from_bytes(msg_tensor.cpu().numpy().tobytes())


def unpack_chunked(words: np.ndarray, bits: int, count: int) -> np.ndarray:
    """o.unpack_indices over slices of whole words (32 indices = `bits` words), so that the bit arrays stay small."""
    if count <= UNPACK_CHUNK:
        return o.unpack_indices(words, bits, count)
    out = np.empty(count, dtype=np.int64)
    for a in range(0, count, UNPACK_CHUNK):
        b = min(count, a + UNPACK_CHUNK)
        w0, w1 = a * bits // 32, (b * bits + 31) // 32
        out[a:b] = o.unpack_indices(words[w0:w1], bits, b - a)
    return out


def _tail_bits_zero(words: np.ndarray, used_bits: int) -> bool:
    """True when every payload bit from `used_bits` on is zero."""
    w = used_bits // 32
    if w >= words.size:
        return True
    first = int(words[w]) >> (used_bits % 32)
    return first == 0 and not words[w + 1:].any()


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
    if o.fractional(b_q8):
        return _check_encode_fractional(ref, tr, b_q8, gpu_msg, stats)
    bits, _ = o.budget(b_q8)
    thresholds, centroids = o.tables(bits)
    D = tr.z.size
    if o.mixed(b_q8):
        # b = bits + 1/2: per-coordinate width; both parts of the payload are zero after their last bit
        wa, wb = o.plane_words(D, b_q8)
        assert _tail_bits_zero(gpu_msg.payload[:wa], D * bits) and _tail_bits_zero(gpu_msg.payload[wa:], D // 2)
        got = o.unpack_mixed(gpu_msg.payload, D, b_q8, tr.up)
        want = tr.idx
        t_hi, c_hi = o.tables(bits + 1)
        z_sent, up_sent = tr.z, tr.up
    else:
        nsent = tr.kept.size
        got = unpack_chunked(gpu_msg.payload, bits, nsent)
        want = tr.idx[tr.kept]
        assert _tail_bits_zero(gpu_msg.payload, nsent * bits)    # padding bits after the last index are zero
        z_sent, up_sent = tr.z[tr.kept], None
    bad = np.flatnonzero(got != want)
    _count(stats, b_q8, want.size, bad.size)
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
    _check_scale(ref, tr, Q, gpu_msg)


def _check_scale(ref, tr, Q, gpu_msg):
    y = tr.z * (math.sqrt(ref.N2) / math.sqrt(tr.z.size))          # R(x) = z / eta
    ip_ref = float(np.dot(y, Q))
    assert abs(gpu_msg.IP - ip_ref) <= SCALE_RTOL * ip_ref, (gpu_msg.IP, ip_ref, ref.IP)
    s_ref = ref.N2 / ip_ref
    assert abs(gpu_msg.S - s_ref) <= SCALE_RTOL * s_ref


def _check_encode_fractional(ref, tr, b_q8, gpu_msg, stats):
    """General non-integer b > 1 (Sec. 4.1): per-coordinate width from the shared coins; the message length follows
    from the coins alone, so it must agree exactly."""
    k, _ = o.budget(b_q8)
    D = tr.z.size
    assert o.payload_words_fractional(D, b_q8, gpu_msg.seed, gpu_msg.client) == gpu_msg.payload.size
    got = o.unpack_fractional(gpu_msg.payload, D, b_q8, tr.up)
    wa, wb = o.plane_words_fractional(D, b_q8, int(tr.up.sum()))
    assert _tail_bits_zero(gpu_msg.payload[:wa], D * k) and _tail_bits_zero(gpu_msg.payload[wa:], int(tr.up.sum()))
    want = tr.idx
    t_lo, c_lo = o.tables(k)
    t_hi, c_hi = o.tables(k + 1)
    bad = np.flatnonzero(got != want)
    _count(stats, b_q8, D, bad.size)
    if bad.size:
        lo = np.minimum(got[bad], want[bad])
        assert np.all(np.abs(got[bad] - want[bad]) == 1), "index differs by more than one interval"
        thr = np.where(tr.up[bad], t_hi[np.minimum(lo, t_hi.size - 1)], t_lo[np.minimum(lo, t_lo.size - 1)])
        dist = np.abs(tr.z[bad] - thr)
        stats.worst_boundary_distance = max(stats.worst_boundary_distance, float(dist.max()))
        assert dist.max() <= INDEX_BOUNDARY_TOL, f"index mismatch {dist.max():.3e} away from its threshold"
    Q = np.where(tr.up, c_hi[np.minimum(got, c_hi.size - 1)], c_lo[np.minimum(got, c_lo.size - 1)])
    _check_scale(ref, tr, Q, gpu_msg)


def _check_encode_grid(ref, tr, b_q8, gpu_msg, stats):
    """Uniform grid (Sec. 4.3): byte i = round(z_i / Delta); the boundaries are Delta (n + 1/2)."""
    delta = o.grid_delta(b_q8)
    D = tr.z.size
    raw = np.frombuffer(gpu_msg.payload.tobytes(), dtype=np.int8)
    assert not raw[D:].any()
    got = raw[:D].astype(np.int64)
    want = tr.idx
    bad = np.flatnonzero(got != want)
    _count(stats, b_q8, D, bad.size)
    if bad.size:
        assert np.all(np.abs(got[bad] - want[bad]) == 1), "index differs by more than one interval"
        dist = np.abs(np.abs(tr.z[bad]) - delta * (np.minimum(np.abs(got[bad]), np.abs(want[bad])) + 0.5))
        stats.worst_boundary_distance = max(stats.worst_boundary_distance, float(dist.max()))
        assert dist.max() <= INDEX_BOUNDARY_TOL, f"index mismatch {dist.max():.3e} away from its boundary"
    Q = np.sign(got) * o.grid_centroids(delta)[np.abs(got)]
    _check_scale(ref, tr, Q, gpu_msg)


STRICT_POOL = Counter()       # every case of the session, budgets held to 1e-6
RELAXED_POOL = Counter()      # every case of the session, uniform grid and b = 5..8
POOL_WORST = [0.0]


def _case_limit(c: Counter) -> int:
    if c.coords >= LARGE_CASE_COORDS:
        return int(c.allowed)                                    # the plain fraction
    return int(c.allowed + 4.0 * math.sqrt(c.allowed) + 1.0)     # a sample: Poisson noise of the count


def finish_encode(stats: EncodeParity):
    STRICT_POOL.add(stats.strict)
    RELAXED_POOL.add(stats.relaxed)
    POOL_WORST[0] = max(POOL_WORST[0], stats.worst_boundary_distance)
    for name, c in (("strict", stats.strict), ("relaxed", stats.relaxed)):
        assert c.mismatches <= _case_limit(c), \
            f"{c.mismatches} near-boundary mismatches in {c.coords} coordinates ({name} budgets, limit {_case_limit(c)})"


def check_pool():
    """The fractions over everything the session has compared so far, each class on its own."""
    for name, c in (("strict", STRICT_POOL), ("relaxed", RELAXED_POOL)):
        assert c.coords == 0 or c.mismatches <= max(1, int(c.allowed)), \
            f"{c.mismatches} near-boundary mismatches in {c.coords} coordinates ({name} budgets)"
    return {"strict": STRICT_POOL, "relaxed": RELAXED_POOL, "worst_boundary_distance": POOL_WORST[0]}


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    den = float(np.linalg.norm(b))
    return float(np.linalg.norm(a.astype(np.float64) - b)) / (den if den > 0 else 1.0)
