/*
 * cnnmem_debug.h -- host-only hooks that let the CPU test-suite exercise the
 * library's index arithmetic without a GPU.  Not needed to use the library.
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
 * decoding; exact for 0 <= n < 2^31, 1 <= d < 2^31.  Host only. */
CNNMEM_API unsigned cnnmem_debug_fastdiv(unsigned n, unsigned d);

/* Logical tile that hardware workgroup `block` of an `nblocks`-wide launch
 * processes under the XCD-contiguous ordering (a bijection on [0, nblocks)).
 * Host only. */
CNNMEM_API unsigned cnnmem_debug_xcd_tile(unsigned block, unsigned nblocks);

#ifdef __cplusplus
}
#endif
#endif /* CNNMEM_DEBUG_H */
