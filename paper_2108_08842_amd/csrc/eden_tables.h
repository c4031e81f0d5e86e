// Positive half of the Lloyd-Max quantizer of N(0,1) for an integer bit budget (Sec. 3).
#ifndef EDEN_TABLES_H
#define EDEN_TABLES_H

#define EDEN_MAX_TABLE_BITS 8
#define EDEN_MAX_HALF_LEVELS 128

struct EdenHalfTable {
    int half_levels;                     // h = 2^(bits-1)
    double t[EDEN_MAX_HALF_LEVELS];      // t[0] = 0 < t[1] < ... : lower edges of the positive intervals
    double q[EDEN_MAX_HALF_LEVELS];      // centres of mass of [t[k], t[k+1])
};

// Solved once per process (thread-safe); nullptr if bits is outside 1..EDEN_MAX_TABLE_BITS.
const EdenHalfTable *eden_half_table(int bits);

#endif
