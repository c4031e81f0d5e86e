// Lloyd-Max tables of the standard normal for the HIP library (host code, double precision).
//
// EDEN quantizes the scaled rotated coordinates with the optimal 2^b-level scalar quantizer
// of N(0,1), computed offline (Sec. 3 of arXiv 2108.08842); a value is mapped to the centre
// of mass of its interval, q_I = E[z | z in I] (Sec. 2.2.1).  For this quantizer thresholds
// are midpoints of neighbouring levels (Sec. 3, the argmin form).
//
// The solver works on the positive half line only (the interval family is symmetric,
// Sec. 2.2.1 property 1): levels 0 < q_0 < ... < q_{h-1}, thresholds t_0 = 0 < t_1 < ... < t_{h-1},
// h = 2^(b-1).  It alternates the two Lloyd conditions until nothing moves.
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

void solve_all() {
    for (int bits = 1; bits <= EDEN_MAX_TABLE_BITS; ++bits) {
        EdenHalfTable &T = g_tables[bits];
        const int h = 1 << (bits - 1);
        T.half_levels = h;
        for (int k = 0; k < h; ++k) T.q[k] = 3.5 * (k + 0.5) / h;              // any increasing start
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
}

}  // namespace

const EdenHalfTable *eden_half_table(int bits) {
    if (bits < 1 || bits > EDEN_MAX_TABLE_BITS) return nullptr;
    std::call_once(g_once, solve_all);
    return &g_tables[bits];
}
