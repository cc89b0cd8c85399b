// Memory-system probes for the layout transform (Section IV.C): MEASUREMENT SUPPORT, built into
// libcnnmem_probes.so, never into libcnnmem.so.  `bench.py --workload access_patterns` runs them beside the
// library's own transform and copy on the same tensor.
//
//   * tile pattern: the global addresses of a tiled [R][S] -> [S][R] transpose (R = C*H*W rows of S images, or the
//     inverse), loaded and stored by lanes that keep every value in registers: no LDS, no barrier, and the data
//     is NOT transposed.  What this kernel reaches is what the access order alone allows.
//   * chunk copy: a plain copy whose chunks of 128 B .. 1 MB are read and / or written in a scattered order.
#include "common.hpp"

namespace cnnmem {
namespace {

// One workgroup of 256 lanes moves a tile of TR rows x NS images (TR*NS = 4096*ITERS/4 floats).
//   images_fast_in_src = 1: src is [R][S] (CHWN), dst is [S][R] (NCHW): the strided side is written
//   images_fast_in_src = 0: src is [S][R] (NCHW), dst is [R][S] (CHWN): the strided side is read
//   r_fastest: tiles along R run first (an image group is walked over the whole tensor before the next)
template <int ITERS>
__global__ __launch_bounds__(256) void probe_tile_pattern_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                                 uint32_t R, uint32_t S, uint32_t TR, uint32_t NS,
                                                                 int images_fast_in_src, int r_fastest) {
    const uint32_t tiles_r = R / TR, tiles_s = S / NS;
    const uint32_t tr = r_fastest ? blockIdx.x % tiles_r : blockIdx.x / tiles_s;
    const uint32_t ts = r_fastest ? blockIdx.x / tiles_r : blockIdx.x % tiles_s;
    const size_t r0 = (size_t)tr * TR, n0 = (size_t)ts * NS;
    const uint32_t ns4 = NS / 4, tr4 = TR / 4;
    float4 v[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const uint32_t f = threadIdx.x + it * 256;
        const size_t a_img_fast = (r0 + f / ns4) * S + n0 + 4 * (f % ns4);      // [R][S] side: runs of NS floats
        const size_t a_img_slow = (n0 + f / tr4) * R + r0 + 4 * (f % tr4);      // [S][R] side: runs of TR floats
        v[it] = ld4_stream(src + (images_fast_in_src ? a_img_fast : a_img_slow));
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const uint32_t f = threadIdx.x + it * 256;
        const size_t a_img_fast = (r0 + f / ns4) * S + n0 + 4 * (f % ns4);
        const size_t a_img_slow = (n0 + f / tr4) * R + r0 + 4 * (f % tr4);
        st4_through(dst + (images_fast_in_src ? a_img_slow : a_img_fast), v[it]);
    }
}

// float4 i belongs to chunk i / c4; chunk c is read at (c * rmul) % nchunks and written at (c * wmul) % nchunks
// (a multiplier coprime to nchunks is a bijection; 1 = in place)
__global__ __launch_bounds__(256) void probe_chunk_copy_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                               uint32_t n4, uint32_t c4, uint32_t nchunks, uint32_t rmul,
                                                               uint32_t wmul) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    const uint32_t c = i / c4, w = i % c4;
    const size_t rc = ((uint64_t)c * rmul) % nchunks, wc = ((uint64_t)c * wmul) % nchunks;
    st4_through(dst + 4 * (wc * c4 + w), ld4_stream(src + 4 * (rc * c4 + w)));
}

uint32_t gcd(uint32_t a, uint32_t b) { return b ? gcd(b, a % b) : a; }

}  // namespace
}  // namespace cnnmem

using namespace cnnmem;

extern "C" {

// Tile pattern over a tensor of R x S floats; TR rows x NS images per tile; TR*NS must be 4096, 8192 or 16384,
// S a multiple of NS, NS and TR multiples of 4, pointers 16-byte aligned device pointers.  Rows beyond the last
// whole tile (R % TR of them) are not touched.
// Returns 0, 1 (invalid arguments) or 3 (launch failed).
__attribute__((visibility("default"))) int cnnmem_probe_tile_pattern(const float* src, float* dst, long long R,
                                                                     long long S, int TR, int NS, int images_fast_in_src,
                                                                     int r_fastest, void* stream) {
    if (!src || !dst || R <= 0 || S <= 0 || TR < 4 || NS < 4 || TR % 4 || NS % 4 || R < TR || S % NS) return 1;
    if (R * S >= (1LL << 32) || !aligned16(src) || !aligned16(dst)) return 1;
    const long long tiles = (R / TR) * (S / NS);
    const long long elems = (long long)TR * NS;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)tiles), block(256);
    if (elems == 4096)
        hipLaunchKernelGGL(probe_tile_pattern_kernel<4>, grid, block, 0, st, src, dst, (uint32_t)R, (uint32_t)S, TR, NS, images_fast_in_src, r_fastest);
    else if (elems == 8192)
        hipLaunchKernelGGL(probe_tile_pattern_kernel<8>, grid, block, 0, st, src, dst, (uint32_t)R, (uint32_t)S, TR, NS, images_fast_in_src, r_fastest);
    else if (elems == 16384)
        hipLaunchKernelGGL(probe_tile_pattern_kernel<16>, grid, block, 0, st, src, dst, (uint32_t)R, (uint32_t)S, TR, NS, images_fast_in_src, r_fastest);
    else
        return 1;
    return launch_status();
}

// Copy of n floats (a multiple of chunk_bytes / 4) in chunks; scatter bit 0: reads, bit 1: writes go to
// scattered chunks.  Returns like the function above.
__attribute__((visibility("default"))) int cnnmem_probe_chunk_copy(const float* src, float* dst, long long n,
                                                                   int chunk_bytes, int scatter, void* stream) {
    if (!src || !dst || n <= 0 || chunk_bytes < 16 || chunk_bytes % 16 || (n * 4) % chunk_bytes) return 1;
    if (n >= (1LL << 33) || !aligned16(src) || !aligned16(dst)) return 1;
    const uint32_t c4 = (uint32_t)(chunk_bytes / 16), n4 = (uint32_t)(n / 4), nchunks = n4 / c4;
    uint32_t mul = nchunks / 3 + 12345u;
    mul = nchunks > 1 ? mul % nchunks : 1;
    if (mul < 2) mul = nchunks > 2 ? 2 : 1;
    while (gcd(mul, nchunks) != 1) ++mul;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(probe_chunk_copy_kernel, dim3((n4 + 255) / 256), dim3(256), 0, st, src, dst, n4, c4, nchunks,
                       (scatter & 1) ? mul : 1u, (scatter & 2) ? mul : 1u);
    return launch_status();
}

}  // extern "C"
