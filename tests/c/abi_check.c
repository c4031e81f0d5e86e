/* The header must be plain C and the library must link from C: calls only the entry points that need no GPU. */
#include <stdio.h>
#include <math.h>
#include "eden.h"

int main(void) {
    double t[15], q[16];
    if (eden_message_bytes(1024, 256) != 64 + 128) return 1;
    if (eden_message_bytes(1024, 384) != 64 + 128 + 64) return 2;            /* b = 1.5: 1 bit each + 1 bit per pair */
    if (eden_message_bytes(1024, EDEN_B_HALF_PRE) != 64 + 64) return 3;     /* 512 coordinates, b = 1 */
    if (eden_message_bytes(1024, EDEN_B_SPARSE(4)) != 64 + 8) return 4;     /* 4 * 16 = 64 kept coordinates */
    if (eden_message_bytes(0, 256) != 0 || eden_message_bytes(10, 300) != 0) return 5;
    if (eden_get_tables(1, t, q) != EDEN_OK) return 6;
    if (fabs(q[1] - sqrt(2.0 / 3.14159265358979323846)) > 1e-12 || q[0] != -q[1] || t[0] != 0.0) return 7;
    if (eden_get_tables(4, t, q) != EDEN_OK || eden_get_tables(9, t, q) == EDEN_OK) return 8;
    if (!eden_strerror(EDEN_ERR_INVALID_ARG) || !eden_kernel_name(0)) return 9;
    if (eden_encode(NULL, NULL, NULL, NULL, 0, 0, 0, NULL, NULL, NULL) != EDEN_ERR_INVALID_ARG) return 10;
    printf("abi ok\n");
    return 0;
}
