// Lloyd-Max tables of the standard normal for the HIP library (host code, double precision).
//
// EDEN quantizes the scaled rotated coordinates with the optimal 2^b-level scalar quantizer
// of N(0,1), computed offline (Sec. 3 of arXiv 2108.08842); a value is mapped to the centre
// of mass of its interval, q_I = E[z | z in I] (Sec. 2.2.1).  For this quantizer thresholds
// are midpoints of neighbouring levels (Sec. 3, the argmin form).
//
// The solver works on the positive half line only (the interval family is symmetric,
// Sec. 2.2.1 property 1): levels 0 < q_0 < ... < q_{h-1}, thresholds t_0 = 0 < t_1 < ... < t_{h-1},
// h = 2^(b-1).  Up to 16 levels per sign it alternates the two Lloyd conditions until nothing moves; above that it
// solves the same two conditions by shooting from the smallest level (Max 1960).
#include "eden_tables.h"

#include <cmath>
#include <mutex>

namespace {

const double kInvSqrt2 = 0.70710678118654752440;
const double kInvSqrt2Pi = 0.39894228040143267794;

double upper_tail(double t) { return 0.5 * std::erfc(t * kInvSqrt2); }        // P(z > t), t >= 0
double density(double t) { return std::isinf(t) ? 0.0 : kInvSqrt2Pi * std::exp(-0.5 * t * t); }

// centre of mass of [a, b], 0 <= a < b <= inf
double centroid(double a, double b) {
    const double mass = upper_tail(a) - (std::isinf(b) ? 0.0 : upper_tail(b));
    return (density(a) - density(b)) / mass;
}

EdenHalfTable g_tables[EDEN_MAX_TABLE_BITS + 1];
std::once_flag g_once;

// Lloyd's iteration: alternate the two conditions until nothing moves (fast up to 16 levels per sign).
void solve_by_iteration(EdenHalfTable &T, int h) {
    for (int k = 0; k < h; ++k) T.q[k] = 3.5 * (k + 0.5) / h;                  // any increasing start
    T.t[0] = 0.0;
    for (long it = 0; it < 5000000; ++it) {
        for (int k = 1; k < h; ++k) T.t[k] = 0.5 * (T.q[k - 1] + T.q[k]);
        double moved = 0.0;
        for (int k = 0; k < h; ++k) {
            const double hi = (k + 1 < h) ? T.t[k + 1] : INFINITY;
            const double c = centroid(T.t[k], hi);
            moved = std::fmax(moved, std::fabs(c - T.q[k]));
            T.q[k] = c;
        }
        if (moved < 1e-15) break;
    }
    for (int k = 1; k < h; ++k) T.t[k] = 0.5 * (T.q[k - 1] + T.q[k]);
}

// The upper edge b of an interval [a, b] whose centre of mass is `target` (a < target < centroid(a, inf)):
// the centre of mass grows with b, so bisection.
double edge_for_centroid(double a, double target) {
    double lo = target, hi = target + 1.0;
    while (centroid(a, hi) < target) hi += 1.0;
    for (int it = 0; it < 200 && hi - lo > 1e-16 * hi; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (centroid(a, mid) < target) lo = mid; else hi = mid;
    }
    return 0.5 * (lo + hi);
}

// From a guess of the smallest level q_0 the two conditions fix everything else in turn: [0, t_1] must have centre of
// mass q_0, q_1 = 2 t_1 - q_0 puts t_1 at the midpoint, [t_1, t_2] must have centre of mass q_1, ...  Returns how far the
// last level ends from the centre of mass of the last, unbounded interval (+1 / -1 if the chain breaks early because
// the guess is too large / too small).
double chain_from(double q0, int h, EdenHalfTable &T) {
    T.t[0] = 0.0;
    T.q[0] = q0;
    for (int k = 0; k + 1 < h; ++k) {
        const double a = T.t[k], target = T.q[k], open_end = centroid(a, INFINITY);
        if (!(a < target)) return -1.0;
        if (!(target < open_end)) return 1.0;
        T.t[k + 1] = edge_for_centroid(a, target);
        T.q[k + 1] = 2.0 * T.t[k + 1] - target;
    }
    return T.q[h - 1] - centroid(T.t[h - 1], INFINITY);
}

// Many levels: Lloyd's iteration converges too slowly (minutes at 128 levels per sign); bisection on q_0 instead.
void solve_by_shooting(EdenHalfTable &T, int h) {
    double lo = 1e-9, hi = 0.7978845608028654;                                  // q_0 < sqrt(2/pi), the single-level value
    for (int it = 0; it < 200 && hi - lo > 1e-17; ++it) {
        const double mid = 0.5 * (lo + hi);
        if (chain_from(mid, h, T) > 0.0) hi = mid; else lo = mid;
    }
    chain_from(lo, h, T);
}

void solve_all() {
    for (int bits = 1; bits <= EDEN_MAX_TABLE_BITS; ++bits) {
        EdenHalfTable &T = g_tables[bits];
        const int h = 1 << (bits - 1);
        T.half_levels = h;
        if (h <= 16) solve_by_iteration(T, h);
        else solve_by_shooting(T, h);
    }
}

}  // namespace

const EdenHalfTable *eden_half_table(int bits) {
    if (bits < 1 || bits > EDEN_MAX_TABLE_BITS) return nullptr;
    std::call_once(g_once, solve_all);
    return &g_tables[bits];
}
