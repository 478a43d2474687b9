// Host-only entry points of libinsum: version, status strings and the group-size rule of
// Section 4.2 (indirect-access count F(g) and the power of two nearest to sqrt(S/n)).
#include <stdint.h>

#include "insum.h"

extern "C" int insum_version(void) { return 100; }

extern "C" const char* insum_status_string(int status) {
    switch (status) {
        case INSUM_OK: return "ok";
        case INSUM_ERR_INVALID_ARG: return "invalid argument";
        case INSUM_ERR_OUT_OF_RANGE: return "coordinate out of range";
        case INSUM_ERR_DUPLICATE: return "duplicate coordinate";
        case INSUM_ERR_CAPACITY: return "output or workspace buffer too small";
        case INSUM_ERR_UNSUPPORTED: return "unsupported dtype or shape";
        case INSUM_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

// g = 2^e with e = round(log2(S/n) / 2).  log2(S/n)/2 rounds to e exactly when
// 4^e / 2 <= S/n < 4^e * 2; we walk e upwards comparing S with n * 2^(2e+1) in 128-bit
// integers, so there is no floating point and no overflow.
extern "C" int32_t insum_default_group_size(int64_t S, int64_t n) {
    if (S <= 0 || n <= 0) return 1;
    int32_t g = 1;
    unsigned __int128 upper = (unsigned __int128)n * 2;  // n * 2^(2e+1) for e = 0
    while ((unsigned __int128)S >= upper && g < (1 << 30)) {
        g *= 2;
        upper *= 4;
    }
    return g;
}

extern "C" int64_t insum_indirect_access_cost(int64_t n, const int64_t* occ, int32_t g) {
    if (n < 0 || g <= 0 || (n > 0 && !occ)) return -1;
    unsigned __int128 groups = 0;   // n * 2^63 at most: no overflow
    for (int64_t i = 0; i < n; ++i) {
        if (occ[i] < 0) return -1;
        groups += (uint64_t)(occ[i] / g + (occ[i] % g != 0));
    }
    if (groups > (unsigned __int128)INT64_MAX / ((uint64_t)g + 1)) return -1;   // F(g) does not fit 64 bits
    return (int64_t)(groups * ((uint64_t)g + 1));
}
