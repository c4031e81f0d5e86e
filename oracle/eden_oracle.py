"""EDEN reference oracle: float64, CPU, numpy.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain statement of what the EDEN encode / decode / mean
path computes (EDEN = the distributed-mean-estimation method of arXiv 2108.08842).
It exists to check the HIP library; it shares no code with it and neither
imports the other.  Only tests, the smoke check and the CPU-baseline leg of the
benchmark may call it.  The product path never routes through this file.

Every function cites the passage of the paper it follows (section / equation /
theorem / lemma numbers).  Where the paper is silent the reading taken is the
one written in the repository's design document; those places are marked
"reading:" below.

Pins (tests/test_oracle_*.py) tie each part to something other than itself:
  * FWHT / rotation  -> dense Sylvester-matrix product, hand-typed H_2/H_4/H_8,
                        norm preservation, R^-1 R = I
  * Lloyd-Max tables -> closed form for b=1, printed values for b=2, printed
                        vNMSE for b=3, printed entropies, quadrature of the
                        fixed-point conditions, E[Q^2] = 1 - MSE
  * quantizer        -> brute-force nearest-centroid argmin, symmetry, tie rule
  * scale            -> tangent identity <x^,x> = |x|^2, the exact SSE identity,
                        the b=1 sign/L1 closed form
  * whole path       -> a d=4 case worked by hand, unbiasedness over 10^4 seeds
                        (Haar matrices from scipy for the theorem itself, the
                        structured rotation on a light-tailed vector for the path),
                        empirical vNMSE against the printed asymptotic values
  * b = k + 1/2      -> a d=4 case worked by hand with the printed I_1 / I_2 values, the printed
                        0.317 at b = 1.5, exact size and mask structure, tangent identity
  * uniform grid     -> the printed Delta_3 = 0.5224 with entropy 3 bits and vNMSE 0.022741 (Sec. 4.3),
                        quadrature of the centres of mass, nearest-grid-point property
  * hash             -> the published splitmix64 test vector (seed 0)
parity unpinned: the b=4 table has no printed value in the paper (it is pinned
only by the Lloyd fixed-point conditions, symmetry and the rate-distortion
bound); the choice of hash is this build's own (the paper only asks for a
shared PRNG seed), so the sign / mask / drop streams are pinned only by the
splitmix64 vector, by statistics, and by the two independent implementations
agreeing.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

# ----------------------------------------------------------------------------
# Shared randomness (Sec. 2.1: every sender shares a PRNG seed with the
# receiver, and the senders' streams are independent of each other).
# reading: a stateless counter hash.  word(key, j) is the j-th output of the
# splitmix64 generator (Steele, Lea, Flood 2014) started from state `key`;
# key mixes (round seed, stream id, client id).
# ----------------------------------------------------------------------------
_MASK64 = (1 << 64) - 1
_PHI = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB

STREAM_SIGN = 0        # Rademacher diagonal of the rotation
STREAM_SUBSAMPLE = 1   # which coordinate of each group is kept when b < 1
STREAM_LOSS = 2        # Bernoulli packet drops (test helper)
STREAM_MIX = 3         # which coordinates get the extra bit when b > 1 is not an integer
STREAM_SPARSE = 4      # sort keys of the m-of-64 sparsification before the rotation (b = m/64)

PACKET_COORDS = 1024   # reading: a packet is 1024 consecutive rotated coordinates


def mix64(z: int) -> int:
    """splitmix64 output function on a Python int (mod 2^64)."""
    z &= _MASK64
    z ^= z >> 30
    z = (z * _M1) & _MASK64
    z ^= z >> 27
    z = (z * _M2) & _MASK64
    z ^= z >> 31
    return z


def stream_key(seed: int, stream: int, client: int) -> int:
    """64-bit key of one (round seed, stream, client) triple."""
    tag = ((stream & 0xFFFFFFFF) << 32) | (client & 0xFFFFFFFF)
    return mix64(mix64(seed + _PHI) + _PHI * tag + _PHI)


def hash_words(key: int, first: int, count: int) -> np.ndarray:
    """word(key, j) = mix64(key + PHI*(j+1)) for j = first .. first+count-1, as uint64."""
    with np.errstate(over="ignore"):
        j = np.arange(first + 1, first + 1 + count, dtype=np.uint64)
        z = np.uint64(key) + np.uint64(_PHI) * j
        z ^= z >> np.uint64(30)
        z *= np.uint64(_M1)
        z ^= z >> np.uint64(27)
        z *= np.uint64(_M2)
        z ^= z >> np.uint64(31)
    return z


def _bits_of_words(words: np.ndarray, nbits: int) -> np.ndarray:
    """bit (i & 63) of words[i >> 6] for i < nbits, as uint8 0/1."""
    shifts = np.arange(64, dtype=np.uint64)
    bits = ((words[:, None] >> shifts[None, :]) & np.uint64(1)).astype(np.uint8)
    return bits.reshape(-1)[:nbits]


def sign_bits(seed: int, client: int, D: int) -> np.ndarray:
    """Bit i is 1 where the rotation's diagonal entry s_i is -1 (Sec. 5: randomized
    Hadamard transform = Hadamard matrix times a random +-1 diagonal)."""
    key = stream_key(seed, STREAM_SIGN, client)
    return _bits_of_words(hash_words(key, 0, (D + 63) // 64), D)


def rademacher(seed: int, client: int, D: int) -> np.ndarray:
    return 1.0 - 2.0 * sign_bits(seed, client, D).astype(np.float64)


def subsample_offsets(seed: int, client: int, n_groups: int) -> np.ndarray:
    """For b = 1/2: offset (0 or 1) of the kept coordinate in each pair of consecutive
    rotated coordinates (Sec. 4.1 random sparsification; reading: stratified mask of
    exact size D/2, applied after the rotation, treated by the receiver like a loss)."""
    key = stream_key(seed, STREAM_SUBSAMPLE, client)
    return _bits_of_words(hash_words(key, 0, (n_groups + 63) // 64), n_groups)


def mix_offsets(seed: int, client: int, n_pairs: int) -> np.ndarray:
    """For b = k + 1/2 (Sec. 4.1, super-bit compression with a non-integer budget): offset (0 or 1)
    of the coordinate of each pair (2g, 2g+1) that is quantized with k+1 bits; the other one uses k.
    reading: the paper draws an independent coin per coordinate from the shared randomness, which
    makes the message length random; here exactly one coordinate of every pair is chosen (the
    choice is still content independent, which is all the proofs of Thm 2.1 / 2.2 use), so the
    message has exactly (k + 1/2) D bits and every position in it is known without a scan."""
    key = stream_key(seed, STREAM_MIX, client)
    return _bits_of_words(hash_words(key, 0, (n_pairs + 63) // 64), n_pairs)


def coin_bits(seed: int, client: int, D: int, frac_q8: int) -> np.ndarray:
    """For a general non-integer budget b > 1 (Sec. 4.1, super-bit compression): True at the coordinates that are
    quantized with I_{floor(b)+1}.  The paper simulates an independent coin of probability b - floor(b) per
    coordinate from the shared randomness.  reading: the coin of coordinate i is the byte (i & 7) of word (i >> 3)
    of the MIX stream, and the coordinate gets the extra bit iff that byte is below frac_q8 = 256 (b - floor(b)),
    so budgets are resolved in steps of 1/256 bit."""
    key = stream_key(seed, STREAM_MIX, client)
    words = hash_words(key, 0, (D + 7) // 8)
    shifts = np.uint64(8) * np.arange(8, dtype=np.uint64)
    coins = ((words[:, None] >> shifts[None, :]) & np.uint64(0xFF)).reshape(-1)[:D]
    return coins < np.uint64(frac_q8)


def n_packets(D: int) -> int:
    return max(1, D // PACKET_COORDS)


def loss_bitmap(seed: int, client: int, D: int, drop_q32: int) -> np.ndarray:
    """Received-packet bitmap (uint32 words, bit j&31 of word j>>5 set = packet j arrived).
    Packet j is dropped iff the top 32 bits of word(key_loss, j) are < drop_q32
    (Sec. 4.2 models loss as an oblivious mask on the rotated vector; the Bernoulli
    law and its hash are a test helper of this build)."""
    npk = n_packets(D)
    key = stream_key(seed, STREAM_LOSS, client)
    w = hash_words(key, 0, npk)
    received = ((w >> np.uint64(32)) >= np.uint64(drop_q32)).astype(np.uint64)
    out = np.zeros((npk + 31) // 32, dtype=np.uint32)
    for j in range(npk):            # small: at most D/1024 packets
        if received[j]:
            out[j >> 5] |= np.uint32(1 << (j & 31))
    return out


def bitmap_to_packet_flags(bitmap: np.ndarray | None, D: int) -> np.ndarray:
    npk = n_packets(D)
    if bitmap is None:
        return np.ones(npk, dtype=bool)
    j = np.arange(npk)
    return ((bitmap[j >> 5] >> (j & 31).astype(np.uint32)) & 1).astype(bool)


# ----------------------------------------------------------------------------
# Rotation (Sec. 2.2.1: R^T R = I;  Sec. 5 / App. "Structured Rotation": the
# randomized Hadamard transform, one transform).
# reading: R x = D^-1/2 H (s o x) with H the Sylvester-ordered Hadamard matrix,
# H[i][j] = (-1)^popcount(i & j); d is zero-padded to D = 2^ceil(log2 d).
# ----------------------------------------------------------------------------
def padded_dim(d: int) -> int:
    if d < 1:
        raise ValueError("d must be >= 1")
    return 1 << (d - 1).bit_length()


def fwht(a: np.ndarray) -> np.ndarray:
    """Unnormalised Walsh-Hadamard transform H a by the plain butterfly recursion
    (a_lo, a_hi) -> (a_lo + a_hi, a_lo - a_hi) at spans 1, 2, 4, ..., D/2."""
    a = np.array(a, dtype=np.float64, copy=True)
    D = a.size
    if D & (D - 1):
        raise ValueError("length must be a power of two")
    h = 1
    while h < D:
        v = a.reshape(-1, 2, h)
        lo = v[:, 0, :].copy()
        hi = v[:, 1, :].copy()
        v[:, 0, :] = lo + hi
        v[:, 1, :] = lo - hi
        h *= 2
    return a


def rotate(x: np.ndarray, seed: int, client: int) -> np.ndarray:
    """R_c(x): pad to D, flip signs, transform, scale by D^-1/2."""
    d = x.size
    D = padded_dim(d)
    xp = np.zeros(D, dtype=np.float64)
    xp[:d] = x
    return fwht(rademacher(seed, client, D) * xp) / math.sqrt(D)


def rotate_inverse(y: np.ndarray, seed: int, client: int) -> np.ndarray:
    """R_c^-1(y) = R_c^T y = s o (D^-1/2 H y)   (H is symmetric, H H = D I)."""
    D = y.size
    return rademacher(seed, client, D) * (fwht(y) / math.sqrt(D))


# ----------------------------------------------------------------------------
# Lloyd-Max tables for N(0,1) (Sec. 3: the optimal 2^b-value scalar quantizer of
# the standard normal, precomputed offline; centre of mass q_I = E[z | z in I],
# Sec. 2.2.1).
# ----------------------------------------------------------------------------
def _pdf(t: float) -> float:
    return 0.0 if math.isinf(t) else math.exp(-0.5 * t * t) / math.sqrt(2.0 * math.pi)


def _mass(a: float, b: float) -> float:
    """P(a <= z <= b), computed on whichever tail keeps the digits."""
    if a >= 0.0:
        return 0.5 * (math.erfc(a / math.sqrt(2.0)) - math.erfc(b / math.sqrt(2.0)))
    if b <= 0.0:
        return 0.5 * (math.erfc(-b / math.sqrt(2.0)) - math.erfc(-a / math.sqrt(2.0)))
    return 0.5 * (math.erf(b / math.sqrt(2.0)) - math.erf(a / math.sqrt(2.0)))


def centre_of_mass(a: float, b: float) -> float:
    """q_I for I=[a,b]:  (pdf(a) - pdf(b)) / P(a<=z<=b)   (Sec. 2.2.1)."""
    return (_pdf(a) - _pdf(b)) / _mass(a, b)


def lloyd_max(levels: int, tol: float = 1e-14, max_iter: int = 2_000_000):
    """Fixed point of Lloyd's iteration on the N(0,1) density:
    thresholds are midpoints of neighbouring centroids, centroids are the centres
    of mass of their intervals.  Returns (thresholds[levels-1], centroids[levels]),
    ascending, float64."""
    if levels < 2:
        raise ValueError("need at least two levels")
    # start from equal-probability-ish spread; symmetric
    q = np.array([-3.0 + 6.0 * (k + 0.5) / levels for k in range(levels)], dtype=np.float64)
    t = np.empty(levels - 1)
    for _ in range(max_iter):
        t = 0.5 * (q[:-1] + q[1:])
        edges = [-math.inf, *t.tolist(), math.inf]
        q_new = np.array([centre_of_mass(edges[k], edges[k + 1]) for k in range(levels)])
        # keep the exact symmetry the interval family must have (Sec. 2.2.1, property 1)
        q_new = 0.5 * (q_new - q_new[::-1])
        delta = float(np.max(np.abs(q_new - q)))
        q = q_new
        if delta < tol:
            break
    t = 0.5 * (q[:-1] + q[1:])
    if levels % 2 == 0:
        t[levels // 2 - 1] = 0.0
    return t, q


def max_shooting(levels: int):
    """The same fixed point (Sec. 3: centroids are centres of mass, thresholds are midpoints) for an even number of
    levels, found the way Max (1960) did: guess the smallest positive centroid q_0; the centroid condition on
    [0, t_1] gives t_1, the midpoint condition gives q_1 = 2 t_1 - q_0, the centroid condition on [t_1, t_2] gives t_2,
    and so on; the guess is right when the last centroid equals the centre of mass of the last, unbounded interval.
    Bisection on q_0.  Lloyd's iteration needs minutes for 256 levels; this takes a fraction of a second."""
    from scipy.optimize import brentq
    if levels < 4 or levels % 2:
        raise ValueError("even number of levels >= 4")
    H = levels // 2

    def chain(q0):
        t, q = [0.0], [q0]
        for _ in range(H - 1):
            a, target = t[-1], q[-1]
            if not a < target < centre_of_mass(a, math.inf):
                return None, (1.0 if target >= centre_of_mass(a, math.inf) else -1.0)
            hi = target + 1.0
            while centre_of_mass(a, hi) < target:
                hi += 1.0
            b = brentq(lambda v: centre_of_mass(a, v) - target, target, hi, xtol=1e-15, rtol=1e-15)
            t.append(b)
            q.append(2.0 * b - target)
        return (t, q), q[-1] - centre_of_mass(t[-1], math.inf)

    lo, hi = 1e-9, math.sqrt(2.0 / math.pi)
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        _, r = chain(mid)
        if r > 0.0:
            hi = mid
        else:
            lo = mid
        if hi - lo < 1e-17:
            break
    (t, q), _ = chain(lo)
    tp, qp = np.array(t[1:]), np.array(q)
    return np.concatenate([-tp[::-1], [0.0], tp]), np.concatenate([-qp[::-1], qp])


_TABLE_CACHE: dict[int, tuple[np.ndarray, np.ndarray]] = {}


def tables(bits: int):
    """(thresholds, centroids) of I_b / Q_{I_b} for an integer bit budget b (Sec. 3).  Up to 32 levels by Lloyd's
    iteration, above that by the shooting method (both solve the same two conditions)."""
    if bits not in _TABLE_CACHE:
        _TABLE_CACHE[bits] = lloyd_max(1 << bits) if bits <= 5 else max_shooting(1 << bits)
    return _TABLE_CACHE[bits]


def expected_q2(thresholds: np.ndarray, centroids: np.ndarray) -> float:
    """E[Q(z)^2] = sum_I q_I^2 P(z in I)   (Example 1 / Example 2 of Sec. 3)."""
    edges = [-math.inf, *thresholds.tolist(), math.inf]
    return float(sum(centroids[k] ** 2 * _mass(edges[k], edges[k + 1]) for k in range(len(centroids))))


def interval_entropy_bits(thresholds: np.ndarray) -> float:
    """H_I = -sum p_I log2 p_I   (Sec. 4.3)."""
    edges = [-math.inf, *thresholds.tolist(), math.inf]
    p = [_mass(edges[k], edges[k + 1]) for k in range(len(edges) - 1)]
    return float(-sum(pi * math.log2(pi) for pi in p if pi > 0))


# ----------------------------------------------------------------------------
# Quantization (Sec. 2.2.1: z is mapped to the centre of mass of the interval that
# contains it; at an endpoint the interval closer to zero is taken).
# reading of the tie rule: positive threshold -> equality stays below it;
# negative threshold -> equality goes above it; threshold 0 -> z >= 0 is the upper side.
# Index = rank of the interval in ascending order (0 = most negative).
# ----------------------------------------------------------------------------
def quantize_indices(z: np.ndarray, thresholds: np.ndarray) -> np.ndarray:
    idx = np.zeros(z.shape, dtype=np.int64)
    for t in thresholds:
        if t > 0.0:
            idx += (z > t)
        else:
            idx += (z >= t)
    return idx


# ----------------------------------------------------------------------------
# Bit budgets (Sec. 4.1).  b is carried as b_q8 = round(256*b).
# Supported here: integer b >= 1 (Q_{I_b});  b = 1/2 (Q_{I_1} + keep one of every
# two rotated coordinates).
# ----------------------------------------------------------------------------
PRE_ROTATION = 0x10000   # flag in b_q8: sub-sample before the rotation (with b_q8 & 0xFFFF = 128)


def pre_rotation(b_q8: int) -> bool:
    """Sec. 4.1, the paper's default for b < 1: sparsify first, then run the 1-bit method in the smaller
    dimension.  reading: b = 1/2 only, the kept coordinate of every pair (2g, 2g+1) of x is the one at
    offset bit g of the sub-sampling stream (a stratified sample of exact size ceil(d/2))."""
    return b_q8 == (PRE_ROTATION | 128)


GRID = 0x30000           # flag in b_q8: uniform-grid quantizer of Sec. 4.3 with Delta = (b_q8 & 0xFFFF) / 32768
GRID_MAX_INDEX = 127     # reading: indices are sent as one signed byte each (before any entropy coder); the outermost
                         # intervals extend to infinity


def grid_delta(b_q8: int) -> float:
    """Delta of a uniform-grid budget, 0.0 for every other budget (Sec. 4.3: I_Delta = {[Delta (n - 1/2), Delta (n + 1/2)]})."""
    q = b_q8 & 0xFFFF
    return q / 32768.0 if (b_q8 & ~0xFFFF) == GRID and q >= 1 else 0.0


def grid_centroids(delta: float) -> np.ndarray:
    """c[n], n = 0..127: centre of mass of N(0,1) on [Delta (n - 1/2), Delta (n + 1/2)] (Sec. 3: the optimal value of an
    interval), the last one on [Delta 126.5, inf).  c[0] = 0 by symmetry; the value of index -n is -c[n]."""
    c = np.zeros(GRID_MAX_INDEX + 1)
    for n in range(1, GRID_MAX_INDEX + 1):
        a = delta * (n - 0.5)
        b = delta * (n + 0.5) if n < GRID_MAX_INDEX else math.inf
        m = _mass(a, b)
        c[n] = (_pdf(a) - (_pdf(b) if math.isfinite(b) else 0.0)) / m if m > 0.0 else a   # beyond double range: the edge
    return c


def grid_indices(z: np.ndarray, delta: float) -> np.ndarray:
    """Index of the interval [Delta (n - 1/2), Delta (n + 1/2)] that holds z (Sec. 4.3); a value on an endpoint goes to the
    interval closer to zero (Sec. 2.2.1, footnote): n = sign(z) ceil(|z| / Delta - 1/2), clipped to the byte range."""
    n = np.sign(z) * np.ceil(np.abs(z) / delta - 0.5)
    return np.clip(n, -GRID_MAX_INDEX, GRID_MAX_INDEX).astype(np.int64)


def empirical_entropy_bits(idx: np.ndarray) -> float:
    """-sum f log2 f over the frequencies of the indices: what an ideal entropy coder would spend per coordinate (Sec. 4.3)."""
    _, counts = np.unique(idx, return_counts=True)
    f = counts / idx.size
    return float(-(f * np.log2(f)).sum())


SPARSE = 0x20000         # flag in b_q8: b = m/64 with m = b_q8 & 0xFFFF, sparsification before the rotation
SPARSE_BLOCK = 64


def sparse_m(b_q8: int) -> int:
    """m of an m-of-64 budget, 0 for every other budget."""
    m = b_q8 & 0xFFFF
    return m if (b_q8 & ~0xFFFF) == SPARSE and 1 <= m < SPARSE_BLOCK else 0


def sparse_selection(seed: int, client: int, d: int, m: int) -> np.ndarray:
    """Sec. 4.1 random sparsification with p = m/64, before the rotation: the mask is a uniformly random
    sample of exact size.  reading: a stratified one -- of every 64 consecutive coordinates (the last
    block padded with virtual zeros up to 64) exactly the m with the smallest 16-bit hash keys are kept,
    ties broken by position; key of coordinate i = bits 16 (i & 3) .. +15 of word (i >> 2) of the SPARSE
    stream.  Returns, for every slot r = 64-block * m + rank among the block's kept coordinates in
    position order, the coordinate it holds (>= d for a kept virtual zero)."""
    nblk = (d + SPARSE_BLOCK - 1) // SPARSE_BLOCK
    n = nblk * SPARSE_BLOCK
    words = hash_words(stream_key(seed, STREAM_SPARSE, client), 0, n // 4)
    keys = ((words[:, None] >> (np.uint64(16) * np.arange(4, dtype=np.uint64))) & np.uint64(0xFFFF)).reshape(nblk, SPARSE_BLOCK)
    order = np.argsort(keys.astype(np.int64) * SPARSE_BLOCK + np.arange(SPARSE_BLOCK), axis=1)   # (key, position) ascending
    kept = np.sort(order[:, :m], axis=1)                           # positions of the m smallest, in position order
    return (kept + np.arange(nblk)[:, None] * SPARSE_BLOCK).reshape(-1)


COIN = 0x40000           # flag in b_q8: general non-integer b = (b_q8 & 0xFFFF) / 256 in (1, 4), one coin per coordinate


def fractional(b_q8: int) -> bool:
    """Sec. 4.1, super-bit compression with a non-integer budget, in the paper's own form: every coordinate uses
    I_{floor(b)+1} with probability b - floor(b), independently (see coin_bits), so the message length is random.
    floor(b) = 1, 2, 3 (the finer table is at most I_4)."""
    low = b_q8 & 0xFFFF
    return (b_q8 & ~0xFFFF) == COIN and 256 < low < 1024 and low % 256 != 0


def budget(b_q8: int):
    """-> (bits per kept coordinate, keep-one-in-k).  For non-integer b > 1 the bits are floor(b) (every coordinate
    has floor(b) bits in the first part of the payload; see mixed() and fractional())."""
    if fractional(b_q8):
        return (b_q8 & 0xFFFF) // 256, 1
    if b_q8 >= 256 and b_q8 % 256 == 0 and b_q8 // 256 <= 8:
        return b_q8 // 256, 1
    if b_q8 == 128:
        return 1, 2
    if mixed(b_q8):
        return b_q8 // 256, 1
    if grid_delta(b_q8):
        return 8, 1                                 # one byte per coordinate on the wire (see GRID_MAX_INDEX)
    raise ValueError(f"unsupported bit budget b_q8={b_q8}")


def mixed(b_q8: int) -> bool:
    """b = 1.5, 2.5, 3.5: half of the coordinates use one bit more (Sec. 4.1)."""
    return b_q8 in (384, 640, 896)


def plane_words(D: int, b_q8: int):
    """-> (words of the index part, words of the extra-bit part); each part is rounded up to a
    multiple of two words (reading)."""
    bits, k = budget(b_q8)
    nbits = (D // k if D >= k else 1) * bits
    a = 2 * ((nbits + 63) // 64)
    b = 2 * ((D // 2 + 63) // 64) if mixed(b_q8) else 0
    return a, b


def payload_words(D: int, b_q8: int) -> int:
    """uint32 words of payload."""
    a, b = plane_words(D, b_q8)
    return a + b


def plane_words_fractional(D: int, b_q8: int, extra_bits: int):
    """-> (words of the floor(b)-bit index part, words of the extra-bit part) of a general non-integer budget;
    `extra_bits`: how many coordinates carry the extra bit.  Each part is rounded up to two words (reading)."""
    k, _ = budget(b_q8)
    return 2 * ((D * k + 63) // 64), 2 * ((extra_bits + 63) // 64)


def payload_words_fractional(D: int, b_q8: int, seed: int, client: int) -> int:
    """uint32 words of payload of a general non-integer budget: fixed by the coins alone (never by the data)."""
    up = coin_bits(seed, client, D, b_q8 & 0xFF)
    return sum(plane_words_fractional(D, b_q8, int(up.sum())))


def pack_indices(idx: np.ndarray, bits: int, n_words: int) -> np.ndarray:
    """reading: value j occupies bits [(j*bits) mod 32, +bits) of word floor(j*bits/32),
    least significant first (bits in {1,2,4,8} never straddle a word; other widths are
    packed as one little-endian bit string)."""
    out = np.zeros(n_words * 32, dtype=np.uint8)
    for r in range(bits):
        out[r : idx.size * bits : bits] = (idx >> r) & 1
    weights = (np.uint64(1) << np.arange(32, dtype=np.uint64))
    return (out.reshape(n_words, 32).astype(np.uint64) * weights).sum(axis=1).astype(np.uint32)


def unpack_indices(words: np.ndarray, bits: int, count: int) -> np.ndarray:
    allbits = ((words[:, None].astype(np.uint64) >> np.arange(32, dtype=np.uint64)) & np.uint64(1)).reshape(-1)
    idx = np.zeros(count, dtype=np.int64)
    for r in range(bits):
        idx |= allbits[r : count * bits : bits].astype(np.int64) << r
    return idx


# ----------------------------------------------------------------------------
# Message (Sec. 2.2.1: the sender transmits the quantized rotated vector and the
# scale S; the scale uses a fixed number of bits, e.g. 64).
# reading of the wire layout: 64-byte little-endian header, then the payload words.
# ----------------------------------------------------------------------------
MAGIC = 0x4E454445
HEADER_BYTES = 64
STATUS_ZERO_VECTOR = 1
STATUS_NONFINITE = 2


@dataclass
class Message:
    log2D: int
    d: int
    b_q8: int
    client: int
    status: int
    S: float
    N2: float
    IP: float
    seed: int
    payload: np.ndarray = field(repr=False)
    extra_bits: int = 0    # general non-integer budgets: coordinates that carry the extra bit (length of the second part)

    def to_bytes(self) -> bytes:
        import struct
        head = struct.pack("<IIQIIIIdddQ", MAGIC, self.log2D, self.d, self.b_q8, self.client,
                           self.status, self.extra_bits, self.S, self.N2, self.IP, self.seed & _MASK64)
        assert len(head) == HEADER_BYTES
        return head + self.payload.astype("<u4").tobytes()

    @staticmethod
    def from_bytes(buf: bytes) -> "Message":
        import struct
        magic, log2D, d, b_q8, client, status, extra, S, N2, IP, seed = struct.unpack(
            "<IIQIIIIdddQ", buf[:HEADER_BYTES])
        if magic != MAGIC:
            raise ValueError("bad magic")
        if fractional(b_q8):
            nw = sum(plane_words_fractional(1 << log2D, b_q8, extra))
        else:
            nw = payload_words(1 << log2D, 2048 if grid_delta(b_q8) else 256 if (pre_rotation(b_q8) or sparse_m(b_q8)) else b_q8)
        payload = np.frombuffer(buf, dtype="<u4", count=nw, offset=HEADER_BYTES).copy()
        return Message(log2D, d, b_q8, client, status, S, N2, IP, seed, payload, extra)


def message_bytes(d: int, b_q8: int) -> int:
    """Bytes a buffer must have for one message; for a general non-integer budget the capacity that fits any outcome of
    the coins (the transmitted length is fixed by the coins and stands in the header)."""
    if fractional(b_q8):
        D = padded_dim(d)
        return HEADER_BYTES + 4 * sum(plane_words_fractional(D, b_q8, D))
    if grid_delta(b_q8):
        return HEADER_BYTES + 4 * payload_words(padded_dim(d), 2048)
    if sparse_m(b_q8):
        return HEADER_BYTES + 4 * payload_words(padded_dim(sparse_m(b_q8) * ((d + SPARSE_BLOCK - 1) // SPARSE_BLOCK)), 256)
    if pre_rotation(b_q8):
        return HEADER_BYTES + 4 * payload_words(padded_dim((d + 1) // 2), 256)
    return HEADER_BYTES + 4 * payload_words(padded_dim(d), b_q8)


# ----------------------------------------------------------------------------
# Sender (Sec. 2.2.1 rotation -> quantization -> scale; Sec. 2.3 the scale).
# ----------------------------------------------------------------------------
def quantize_and_scale(y: np.ndarray, N2: float, bits: int):
    """From a rotated vector y = R(x) with |x|^2 = N2: the scaled vector z = eta*y, the
    interval ranks I(z), the quantized vector Q(z), <R(x), Q> and the scale S
    (Sec. 2.2.1 deterministic quantization, Sec. 2.3 scale).  Works for any rotation."""
    thresholds, centroids = tables(bits)
    D = y.size
    eta = math.sqrt(D) / math.sqrt(N2)             # eta_x = sqrt(d)/|x|, d -> padded D
    z = eta * y
    idx = quantize_indices(z, thresholds)          # I(z)
    Q = centroids[idx]                             # Q(eta R(x))
    IP = float(np.dot(y, Q))                       # <R(x), Q(eta R(x))> over all D coordinates
    S = N2 / IP                                    # Sec. 2.3
    return z, idx, Q, IP, S


@dataclass
class EncodeTrace:
    """Intermediates kept for the parity checks (never sent)."""
    z: np.ndarray          # eta * R(x), all D coordinates
    idx: np.ndarray        # interval rank of every coordinate (before sub-sampling)
    kept: np.ndarray       # coordinates whose index is in the payload
    up: np.ndarray | None = None   # b = k + 1/2: True where the coordinate uses the (k+1)-bit quantizer


def upgraded_mask(seed: int, client: int, D: int) -> np.ndarray:
    """True at the coordinate of every pair (2g, 2g+1) that gets the extra bit."""
    off = mix_offsets(seed, client, D // 2).astype(np.int64)
    up = np.zeros(D, dtype=bool)
    up[2 * np.arange(D // 2) + off] = True
    return up


def _encode_mixed(y, N2, d, D, bits, b_q8, seed, client, want_trace):
    """b = k + 1/2 (Sec. 4.1): coordinate i is quantized with I_{k+1} if it is the chosen one of its
    pair, else with I_k; the scale is S = |x|^2 / <R(x), Q> with that coordinate-wise Q (Sec. 2.3).
    reading of the layout: first the low k bits of every coordinate's index, packed as for budget k;
    then one bit per pair, the top bit of the chosen coordinate's (k+1)-bit index."""
    if D < 2:
        raise ValueError("a half-integer budget needs at least one pair of coordinates")
    t_lo, c_lo = tables(bits)
    t_hi, c_hi = tables(bits + 1)
    eta = math.sqrt(D) / math.sqrt(N2)
    z = eta * y
    up = upgraded_mask(seed, client, D)
    idx = np.where(up, quantize_indices(z, t_hi), quantize_indices(z, t_lo))
    Q = np.where(up, c_hi[np.minimum(idx, c_hi.size - 1)], c_lo[np.minimum(idx, c_lo.size - 1)])
    IP = float(np.dot(y, Q))
    S = N2 / IP
    wa, wb = plane_words(D, b_q8)
    low = idx & ((1 << bits) - 1)
    top = (idx[up] >> bits) & 1                    # in pair order: exactly one chosen coordinate per pair
    payload = np.concatenate([pack_indices(low, bits, wa), pack_indices(top, 1, wb)])
    msg = Message(D.bit_length() - 1, d, b_q8, client, 0, S, N2, IP, seed, payload)
    if want_trace:
        return msg, EncodeTrace(z=z, idx=idx, kept=np.arange(D), up=up)
    return msg


def unpack_mixed(payload: np.ndarray, D: int, b_q8: int, up: np.ndarray) -> np.ndarray:
    """The per-coordinate indices of a b = k + 1/2 payload (k+1 bits wide where `up`, else k)."""
    bits, _ = budget(b_q8)
    wa, wb = plane_words(D, b_q8)
    idx = unpack_indices(payload[:wa], bits, D)
    top = unpack_indices(payload[wa:wa + wb], 1, D // 2)
    idx[up] |= top << bits
    return idx


def _encode_fractional(y, N2, d, D, b_q8, seed, client, want_trace):
    """General non-integer b > 1 (Sec. 4.1): coordinate i is quantized with I_{k+1}, k = floor(b), if its coin says so
    (probability b - k), else with I_k; S = |x|^2 / <R(x), Q> with that coordinate-wise Q (Sec. 2.3).
    reading of the layout: first the low k bits of every coordinate's index, packed as for budget k; then one bit for
    every coordinate with a coin, in coordinate order: the top bit of its (k+1)-bit index."""
    k, _ = budget(b_q8)
    t_lo, c_lo = tables(k)
    t_hi, c_hi = tables(k + 1)
    eta = math.sqrt(D) / math.sqrt(N2)
    z = eta * y
    up = coin_bits(seed, client, D, b_q8 & 0xFF)
    idx = np.where(up, quantize_indices(z, t_hi), quantize_indices(z, t_lo))
    Q = np.where(up, c_hi[np.minimum(idx, c_hi.size - 1)], c_lo[np.minimum(idx, c_lo.size - 1)])
    IP = float(np.dot(y, Q))
    S = N2 / IP
    extra = int(up.sum())
    wa, wb = plane_words_fractional(D, b_q8, extra)
    low = idx & ((1 << k) - 1)
    top = (idx[up] >> k) & 1
    payload = np.concatenate([pack_indices(low, k, wa), pack_indices(top, 1, wb)])
    msg = Message(D.bit_length() - 1, d, b_q8, client, 0, S, N2, IP, seed, payload, extra)
    if want_trace:
        return msg, EncodeTrace(z=z, idx=idx, kept=np.arange(D), up=up)
    return msg


def unpack_fractional(payload: np.ndarray, D: int, b_q8: int, up: np.ndarray) -> np.ndarray:
    """The per-coordinate indices of a general non-integer budget's payload (k+1 bits wide where `up`, else k)."""
    k, _ = budget(b_q8)
    extra = int(up.sum())
    wa, wb = plane_words_fractional(D, b_q8, extra)
    idx = unpack_indices(payload[:wa], k, D)
    top = unpack_indices(payload[wa:wa + wb], 1, extra)
    idx[up] |= top << k
    return idx


def sparsify_pairs(x: np.ndarray, seed: int, client: int):
    """(1/p) m o x with p = 1/2, compacted: element g is 2 x[2g + off_g] (0 beyond the end of x).
    Sec. 4.1 random sparsification; its expectation over the offsets is x scattered back."""
    d = x.size
    g = np.arange((d + 1) // 2)
    src = 2 * g + subsample_offsets(seed, client, g.size).astype(np.int64)
    xp = np.concatenate([x, [0.0]])
    return 2.0 * xp[np.minimum(src, d)], src


def encode(x: np.ndarray, seed: int, client: int, b_q8: int, want_trace: bool = False):
    x = np.asarray(x, dtype=np.float64)
    if sparse_m(b_q8):
        # b = m/64: the 1-bit method on the kept coordinates (a vector of m * ceil(d/64) entries).  The factor 1/p
        # of the sparsification is applied by the receiver: the method is scale equivariant, and the sender then
        # works on the values of x themselves.
        src = sparse_selection(seed, client, x.size, sparse_m(b_q8))
        xs = np.concatenate([x, np.zeros(SPARSE_BLOCK)])[src]
        inner = encode(xs, seed, client, 256, want_trace)
        msg, tr = inner if want_trace else (inner, None)
        msg.d = x.size
        msg.b_q8 = b_q8
        return (msg, tr) if want_trace else msg
    if pre_rotation(b_q8):
        # the 1-bit method on the sparsified vector; the message keeps the original d and the flagged budget
        if x.size < 2:
            raise ValueError("sub-sampling in pairs needs at least two coordinates")
        xs, _ = sparsify_pairs(x, seed, client)
        inner = encode(xs, seed, client, 256, want_trace)
        msg, tr = inner if want_trace else (inner, None)
        msg.d = x.size
        msg.b_q8 = b_q8
        return (msg, tr) if want_trace else msg
    d = x.size
    D = padded_dim(d)
    bits, k = budget(b_q8)
    if D < k:
        raise ValueError("sub-bit budget needs at least one whole group of coordinates")
    extra = int(coin_bits(seed, client, D, b_q8 & 0xFF).sum()) if fractional(b_q8) else 0
    nw = sum(plane_words_fractional(D, b_q8, extra)) if fractional(b_q8) else payload_words(D, b_q8)

    N2 = float(np.dot(x, x))                       # |x|^2  (= |R(x)|^2, Sec. 2.2.1)
    if not math.isfinite(N2):
        msg = Message(D.bit_length() - 1, d, b_q8, client, STATUS_NONFINITE, 0.0, N2, 0.0, seed,
                      np.zeros(nw, np.uint32), extra)
        return (msg, None) if want_trace else msg
    if N2 == 0.0:                                  # the x = 0 case the paper sets aside (Sec. 2.1 footnote)
        msg = Message(D.bit_length() - 1, d, b_q8, client, STATUS_ZERO_VECTOR, 0.0, 0.0, 0.0, seed,
                      np.zeros(nw, np.uint32), extra)
        return (msg, None) if want_trace else msg

    y = rotate(x, seed, client)                    # R(x)
    if grid_delta(b_q8):
        # Sec. 4.3: the interval set I_Delta; the scale is S = |x|^2 / <R(x), Q> as for every interval set (Sec. 2.3)
        delta = grid_delta(b_q8)
        z = (math.sqrt(D) / math.sqrt(N2)) * y
        idx = grid_indices(z, delta)
        Q = np.sign(idx) * grid_centroids(delta)[np.abs(idx)]
        IP = float(np.dot(y, Q))
        if IP <= 0.0:                              # every coordinate fell into the interval around 0 (huge Delta)
            msg = Message(D.bit_length() - 1, d, b_q8, client, STATUS_ZERO_VECTOR, 0.0, N2, 0.0, seed, np.zeros(nw, np.uint32))
            return (msg, None) if want_trace else msg
        payload = pack_indices(idx & 0xFF, 8, nw)   # two's complement bytes
        msg = Message(D.bit_length() - 1, d, b_q8, client, 0, N2 / IP, N2, IP, seed, payload)
        return (msg, EncodeTrace(z=z, idx=idx, kept=np.arange(D))) if want_trace else msg
    if mixed(b_q8):
        return _encode_mixed(y, N2, d, D, bits, b_q8, seed, client, want_trace)
    if fractional(b_q8):
        return _encode_fractional(y, N2, d, D, b_q8, seed, client, want_trace)
    z, idx, Q, IP, S = quantize_and_scale(y, N2, bits)

    if k == 1:
        kept = np.arange(D)
    else:                                          # Sec. 4.1 sub-bit; sender's S unchanged (Sec. 4.2)
        groups = max(1, D // k)
        off = subsample_offsets(seed, client, groups).astype(np.int64)
        kept = np.arange(groups) * k + off
        kept = kept[kept < D]
    payload = pack_indices(idx[kept], bits, nw)
    msg = Message(D.bit_length() - 1, d, b_q8, client, 0, S, N2, IP, seed, payload)
    if want_trace:
        return msg, EncodeTrace(z=z, idx=idx, kept=kept)
    return msg


# ----------------------------------------------------------------------------
# Receiver (Sec. 2.2.2: x^_c = S_c R_c^-1(Q(...)), then the plain average;
# Sec. 4.2 / Lemma 4.3: lost coordinates are zero, the rest is multiplied by 1/p
# where p is the fraction of coordinates that arrived, found by counting).
# reading: unsampled coordinates (b<1) and lost packets form one mask with one p.
# ----------------------------------------------------------------------------
def decode_rotated(msg: Message, bitmap: np.ndarray | None = None) -> np.ndarray:
    """(S/p) * m o Q  in the rotated domain, all D coordinates."""
    D = 1 << msg.log2D
    bits, k = budget(msg.b_q8)
    yhat = np.zeros(D, dtype=np.float64)
    if msg.status != 0:
        return yhat
    if grid_delta(msg.b_q8):
        raw = unpack_indices(msg.payload, 8, D)
        idx = np.where(raw >= 128, raw - 256, raw)
        Q = np.sign(idx) * grid_centroids(grid_delta(msg.b_q8))[np.minimum(np.abs(idx), GRID_MAX_INDEX)]
        arrived = np.repeat(bitmap_to_packet_flags(bitmap, D), min(D, PACKET_COORDS))[:D]
        count = int(arrived.sum())
        if count == 0:
            return yhat
        yhat[arrived] = (msg.S / (count / D)) * Q[arrived]
        return yhat
    _, centroids = tables(bits)
    if mixed(msg.b_q8) or fractional(msg.b_q8):
        if mixed(msg.b_q8):
            up = upgraded_mask(msg.seed, msg.client, D)
            idx = unpack_mixed(msg.payload, D, msg.b_q8, up)
        else:
            up = coin_bits(msg.seed, msg.client, D, msg.b_q8 & 0xFF)
            idx = unpack_fractional(msg.payload, D, msg.b_q8, up)
        _, c_hi = tables(bits + 1)
        Q = np.where(up, c_hi[np.minimum(idx, c_hi.size - 1)], centroids[np.minimum(idx, centroids.size - 1)])
        arrived = np.repeat(bitmap_to_packet_flags(bitmap, D), min(D, PACKET_COORDS))[:D]
        count = int(arrived.sum())
        if count == 0:
            return yhat
        yhat[arrived] = (msg.S / (count / D)) * Q[arrived]
        return yhat
    if k == 1:
        kept = np.arange(D)
    else:
        groups = max(1, D // k)
        off = subsample_offsets(msg.seed, msg.client, groups).astype(np.int64)
        kept = np.arange(groups) * k + off
        kept = kept[kept < D]
    idx = unpack_indices(msg.payload, bits, kept.size)
    pk = bitmap_to_packet_flags(bitmap, D)
    arrived = pk[np.minimum(kept // PACKET_COORDS, pk.size - 1)]
    count = int(arrived.sum())
    if count == 0:                                 # nothing arrived: contributes nothing
        return yhat
    p = count / D
    yhat[kept[arrived]] = (msg.S / p) * centroids[idx[arrived]]
    return yhat


def decode(msg: Message, d: int, bitmap: np.ndarray | None = None) -> np.ndarray:
    if sparse_m(msg.b_q8):
        m = sparse_m(msg.b_q8)
        src = sparse_selection(msg.seed, msg.client, d, m)
        inner = Message(msg.log2D, src.size, 256, msg.client, msg.status, msg.S, msg.N2, msg.IP, msg.seed, msg.payload)
        xs_hat = decode(inner, src.size, bitmap) * (SPARSE_BLOCK / m)            # the 1/p of the sparsification
        out = np.zeros(d + SPARSE_BLOCK)
        out[src] = xs_hat
        return out[:d]
    if pre_rotation(msg.b_q8):
        # decode the 1-bit message of dimension ceil(d/2), then put every value back where it was taken from
        dp = (d + 1) // 2
        inner = Message(msg.log2D, dp, 256, msg.client, msg.status, msg.S, msg.N2, msg.IP, msg.seed, msg.payload)
        xs_hat = decode(inner, dp, bitmap)
        src = 2 * np.arange(dp) + subsample_offsets(msg.seed, msg.client, dp).astype(np.int64)
        out = np.zeros(d + 1)
        out[np.minimum(src, d)] = xs_hat
        return out[:d]
    yhat = decode_rotated(msg, bitmap)
    return rotate_inverse(yhat, msg.seed, msg.client)[:d]


def decode_mean(msgs, d: int, bitmaps=None, n: int | None = None) -> np.ndarray:
    """(1/n) sum_c x^_c  (Sec. 2.2.2); n defaults to the number of messages."""
    acc = np.zeros(d, dtype=np.float64)
    for c, m in enumerate(msgs):
        acc += decode(m, d, None if bitmaps is None else bitmaps[c])
    return acc / float(len(msgs) if n is None else n)


# ----------------------------------------------------------------------------
# Error measures (Sec. 2.1 NMSE, Sec. 2.4 vNMSE)
# ----------------------------------------------------------------------------
def vnmse_single(x: np.ndarray, xhat: np.ndarray) -> float:
    return float(np.sum((x - xhat) ** 2) / np.sum(x ** 2))


def nmse(xs, mean_hat: np.ndarray) -> float:
    xs = [np.asarray(v, dtype=np.float64) for v in xs]
    true_mean = sum(xs) / len(xs)
    return float(np.sum((mean_hat - true_mean) ** 2) / (sum(np.dot(v, v) for v in xs) / len(xs)))
