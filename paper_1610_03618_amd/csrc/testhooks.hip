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
