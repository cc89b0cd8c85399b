// Host-only hooks for the CPU test-suite (include/cnnmem_debug.h): the kernels' index arithmetic without a
// GPU.  Built into libcnnmem_testhooks.so, never into libcnnmem.so.
#include "cnnmem_debug.h"
#include "common.hpp"

using namespace cnnmem;

extern "C" {

unsigned cnnmem_debug_fastdiv(unsigned n, unsigned d) {
    if (d == 0) return 0xffffffffu;                // no quotient: the all-ones word, never a valid one for n < 2^31
    return fd_div(n, make_fastdiv(d));
}

// quotients of the small-number division that differ from n / d, over every divisor in [1, max_d] and the
// numerators k*d - 1, k*d, k*d + 1 below max_n (where a quotient can go wrong first); -1 for arguments out of range
long long cnnmem_debug_smalldiv_mismatches(unsigned max_n, unsigned max_d) {
    if (max_n > (1u << 20) || max_d == 0 || max_d >= (1u << 20)) return -1;
    long long bad = 0;
    for (unsigned d = 1; d <= max_d; ++d) {
        const SmallDiv s = make_smalldiv(d);
        for (unsigned m = 0; m < max_n; m += d)
            for (int e = -1; e <= 1; ++e) {
                const long long n = (long long)m + e;
                if (n < 0 || n >= (long long)max_n) continue;
                if (sd_div((unsigned)n, s) != (unsigned)n / d) ++bad;
            }
    }
    return bad;
}

int cnnmem_debug_canonical_permutation(const int* dims, const int* perm, int* rank, long long* canonical_dims,
                                       int* canonical_perm) {
    if (!dims || !perm || !rank || !canonical_dims || !canonical_perm) return 1;
    bool seen[4] = {false, false, false, false};
    for (int i = 0; i < 4; ++i) {
        if (dims[i] <= 0 || perm[i] < 0 || perm[i] > 3 || seen[perm[i]]) return 1;
        seen[perm[i]] = true;
    }
    canonical_permutation(dims, perm, rank, canonical_dims, canonical_perm);
    return 0;
}

unsigned cnnmem_debug_xcd_tile(unsigned block, unsigned nblocks) {
    return xcd_contiguous_tile(block, nblocks);
}

}  // extern "C"
