/*
 * cnnmem_debug.h -- host-only hooks that let the CPU test-suite exercise the
 * library's index arithmetic without a GPU.  They are exported by
 * libcnnmem_testhooks.so, a library of their own: libcnnmem.so does not carry them.
 */
#ifndef CNNMEM_DEBUG_H
#define CNNMEM_DEBUG_H

#ifndef CNNMEM_API
#define CNNMEM_API __attribute__((visibility("default")))
#endif

#ifdef __cplusplus
extern "C" {
#endif

/* n / d through the multiply-shift divider the kernels use for output-index
 * decoding; exact for 0 <= n < 2^31, 1 <= d < 2^31; d = 0 returns 0xffffffff.  Host only. */
CNNMEM_API unsigned cnnmem_debug_fastdiv(unsigned n, unsigned d);

/* The three-instruction divider of indices inside a workgroup's LDS slab (exact for n < 2^20): the number of
 * quotients that differ from n / d over every divisor in [1, max_d] and the numerators k*d - 1, k*d, k*d + 1
 * below max_n; -1 when max_n > 2^20, max_d = 0 or max_d >= 2^20.  Host only. */
CNNMEM_API long long cnnmem_debug_smalldiv_mismatches(unsigned max_n, unsigned max_d);

/* Logical tile that hardware workgroup `block` of an `nblocks`-wide launch
 * processes under the XCD-contiguous ordering (a bijection on [0, nblocks)).
 * Host only. */
CNNMEM_API unsigned cnnmem_debug_xcd_tile(unsigned block, unsigned nblocks);

/* Canonical form cnnmem_permute reduces a permutation to before it picks a
 * kernel: axes of extent 1 dropped, source axes that stay neighbours in the
 * destination merged.  Writes the rank (0..4), the merged source extents and the
 * permutation over them; returns 0, or 1 for invalid arguments.  Host only. */
CNNMEM_API int cnnmem_debug_canonical_permutation(const int *dims, const int *perm, int *rank,
                                                  long long *canonical_dims, int *canonical_perm);

#ifdef __cplusplus
}
#endif
#endif /* CNNMEM_DEBUG_H */
