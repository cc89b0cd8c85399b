// Layout transformation NCHW <-> CHWN as a 2-D transpose (Section IV.C).
//
// C, H and W keep their relative order in both layouts, so with M = C*H*W the
// NCHW tensor is an [N][M] matrix and the CHWN tensor is the [M][N] matrix: one
// generic kernel src[R][S] -> dst[S][R] serves both directions.
//
// gfx950 design (not the paper's Kepler float2 scheme): every lane moves
// 128-bit words on both the read and the write side.  A workgroup owns a TR x TS
// tile; each lane loads a 4x4 block (four float4 from four consecutive source
// rows), transposes it in registers, and parks the four transposed float4 in an
// LDS tile that is already in destination order.  After one barrier the tile is
// read back row by row with 128-bit LDS reads and written with 128-bit global
// stores, so global reads and writes are both contiguous runs of TS*4 and TR*4
// bytes.  LDS rows are padded by 4 floats and stored in a j-major swizzled order
// so that the 16 lanes that write one 4x4 block column hit distinct bank groups.
#include "common.hpp"

namespace cnnmem {
namespace {

constexpr int kThreads = 256;

// LDS row that holds destination row `s_local` of the tile.  Rows s = 4*bs + j
// are stored at j*(TS/4) + bs: lanes with consecutive bs write consecutive LDS
// rows (pitch 4 floats over a multiple of 16 floats -> distinct bank groups).
template <int TS>
__device__ __forceinline__ int lds_row(int s_local) {
    return (s_local & 3) * (TS / 4) + (s_local >> 2);
}

extern __shared__ float4 dyn_tile[];                // 16-byte aligned dynamic LDS

template <int TR, int TS, int THREADS>
__global__ __launch_bounds__(THREADS) void transpose_vec4_kernel(
    const float* __restrict__ src, float* __restrict__ dst, long long R, long long S,
    uint32_t tiles_s, int xcd_order) {
    static_assert(TR % 4 == 0 && TS % 4 == 0, "tile sides are multiples of 4");
    static_assert((TR * TS / 16) % THREADS == 0, "whole number of 4x4 blocks per lane");
    constexpr int P = TR + 4;                       // LDS pitch in floats (keeps float4 alignment)
    constexpr int NBS = TS / 4;                     // 4x4 blocks along S
    constexpr int LOAD_ITERS = (TR * TS / 16) / THREADS;
    constexpr int NBR = TR / 4;                     // float4 per destination row of the tile
    constexpr int STORE_ITERS = (TS * NBR) / THREADS;

    float* tile = reinterpret_cast<float*>(dyn_tile);   // TS * P floats, sized by the launch

    const uint32_t tile_id = xcd_order ? xcd_contiguous_tile(blockIdx.x, gridDim.x) : blockIdx.x;
    const long long r0 = (long long)(tile_id / tiles_s) * TR;
    const long long s0 = (long long)(tile_id % tiles_s) * TS;
    const int tid = threadIdx.x;

    // Lanes whose 4x4 block falls outside the matrix (edge tiles) re-read the last
    // block instead of branching: every load is unconditional, so all of a lane's
    // loads are in flight together, and what those lanes park in LDS is never
    // written out.  R and S are multiples of 4, hence R - 4 and S - 4 are valid.
    float4 v[LOAD_ITERS][4];
#pragma unroll
    for (int it = 0; it < LOAD_ITERS; ++it) {
        const int b = tid + it * THREADS;
        const int bs = b % NBS;
        const int br = b / NBS;
        long long r = r0 + 4 * br;
        long long s = s0 + 4 * bs;
        r = r < R ? r : R - 4;
        s = s < S ? s : S - 4;
        const float* p = src + (size_t)r * (size_t)S + (size_t)s;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[it][i] = ld4_stream(p + (size_t)i * (size_t)S);
    }
#pragma unroll
    for (int it = 0; it < LOAD_ITERS; ++it) {
        const int b = tid + it * THREADS;
        const int bs = b % NBS;
        const int br = b / NBS;
        const float4 a = v[it][0], bq = v[it][1], c = v[it][2], d = v[it][3];
        float* base = tile + 4 * br;
        *reinterpret_cast<float4*>(base + lds_row<TS>(4 * bs + 0) * P) = make_float4(a.x, bq.x, c.x, d.x);
        *reinterpret_cast<float4*>(base + lds_row<TS>(4 * bs + 1) * P) = make_float4(a.y, bq.y, c.y, d.y);
        *reinterpret_cast<float4*>(base + lds_row<TS>(4 * bs + 2) * P) = make_float4(a.z, bq.z, c.z, d.z);
        *reinterpret_cast<float4*>(base + lds_row<TS>(4 * bs + 3) * P) = make_float4(a.w, bq.w, c.w, d.w);
    }
    __syncthreads();
    // every LDS read first, then the stores: the compiler keeps LDS reads behind the inline-asm store that
    // precedes them in program order, so read / wait / store would repeat STORE_ITERS times
    float4 o[STORE_ITERS];
#pragma unroll
    for (int it = 0; it < STORE_ITERS; ++it) {
        const int f = tid + it * THREADS;
        o[it] = *reinterpret_cast<const float4*>(tile + lds_row<TS>(f / NBR) * P + 4 * (f % NBR));
    }
#pragma unroll
    for (int it = 0; it < STORE_ITERS; ++it) {
        const int f = tid + it * THREADS;
        const int br = f % NBR;
        const int sl = f / NBR;
        const long long s = s0 + sl;
        const long long r = r0 + 4 * br;
        if (s < S && r < R)
            st4_through(dst + (size_t)s * (size_t)R + (size_t)r, o[it]);
    }
}

// One float4 per lane (THREADS = TR*TS/4): the lane scatters its four words into
// the transposed LDS tile with dword writes, and after the barrier reads one
// float4 of a destination row back.  Fewer bytes in flight per lane than the
// 4x4-block kernel; same LDS layout.
template <int TR, int TS>
__global__ __launch_bounds__(TR * TS / 4) void transpose_u1_kernel(
    const float* __restrict__ src, float* __restrict__ dst, long long R, long long S, uint32_t tiles_s,
    int xcd_order) {
    constexpr int P = TR + 4;
    constexpr int NC4 = TS / 4;                     // float4 per source row of the tile
    constexpr int NBR = TR / 4;                     // float4 per destination row of the tile
    __shared__ __attribute__((aligned(16))) float tile[TS * P];

    const uint32_t tile_id = xcd_order ? xcd_contiguous_tile(blockIdx.x, gridDim.x) : blockIdx.x;
    const long long r0 = (long long)(tile_id / tiles_s) * TR;
    const long long s0 = (long long)(tile_id % tiles_s) * TS;
    const int tid = threadIdx.x;
    {
        const int c4 = tid % NC4;
        const int rl = tid / NC4;
        long long r = r0 + rl, s = s0 + 4 * c4;
        r = r < R ? r : R - 1;                      // edge tiles: re-read a valid word, never written out
        s = s < S ? s : S - 4;
        const float4 v = ld4_stream(src + (size_t)r * (size_t)S + (size_t)s);
        tile[lds_row<TS>(4 * c4 + 0) * P + rl] = v.x;
        tile[lds_row<TS>(4 * c4 + 1) * P + rl] = v.y;
        tile[lds_row<TS>(4 * c4 + 2) * P + rl] = v.z;
        tile[lds_row<TS>(4 * c4 + 3) * P + rl] = v.w;
    }
    __syncthreads();
    {
        const int br = tid % NBR;
        const int sl = tid / NBR;
        const long long s = s0 + sl, r = r0 + 4 * br;
        if (s < S && r < R)
            st4_stream(dst + (size_t)s * (size_t)R + (size_t)r,
                       *reinterpret_cast<const float4*>(tile + lds_row<TS>(sl) * P + 4 * br));
    }
}

// Any R, S and any 4-byte alignment: 64x64 tile, dword accesses, pitch 65.
__global__ __launch_bounds__(kThreads) void transpose_scalar_kernel(
    const float* __restrict__ src, float* __restrict__ dst, long long R, long long S,
    uint32_t tiles_s) {
    constexpr int T = 64;
    __shared__ float tile[T * (T + 1)];
    const uint32_t tile_id = blockIdx.x;
    const long long r0 = (long long)(tile_id / tiles_s) * T;
    const long long s0 = (long long)(tile_id % tiles_s) * T;
    const int tx = threadIdx.x % T;
    const int ty = threadIdx.x / T;                 // 0..3
#pragma unroll
    for (int k = 0; k < T / 4; ++k) {
        const int rl = ty + 4 * k;
        const long long r = r0 + rl, s = s0 + tx;
        if (r < R && s < S) tile[rl * (T + 1) + tx] = ld1_stream(src + (size_t)r * (size_t)S + (size_t)s);
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < T / 4; ++k) {
        const int sl = ty + 4 * k;
        const long long s = s0 + sl, r = r0 + tx;
        if (r < R && s < S) st1_stream(dst + (size_t)s * (size_t)R + (size_t)r, tile[tx * (T + 1) + sl]);
    }
}

// One float4 per lane and as many workgroups as it takes: on MI355X this beats
// deeper per-lane unrolling and persistent grids for a pure stream.
__global__ __launch_bounds__(kThreads) void copy_vec4_kernel(const float* __restrict__ src,
                                                             float* __restrict__ dst, size_t n4,
                                                             size_t first) {
    const size_t i = first + (size_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n4) st4_through(dst + 4 * i, ld4_stream(src + 4 * i));
}

__global__ __launch_bounds__(kThreads) void copy_scalar_kernel(const float* __restrict__ src,
                                                               float* __restrict__ dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

template <int TR, int TS, int THREADS = kThreads>
int launch_vec4(const float* src, float* dst, long long R, long long S, hipStream_t st) {
    const long long tiles_r = ceil_div64(R, TR), tiles_s = ceil_div64(S, TS);
    const long long tiles = tiles_r * tiles_s;
    if (tiles > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    constexpr size_t lds_bytes = sizeof(float) * TS * (TR + 4);
    if (lds_bytes > 65536) {                        // above the default per-workgroup limit: opt in (gfx950 has 160 KB)
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&transpose_vec4_kernel<TR, TS, THREADS>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
            return CNNMEM_ERR_RUNTIME;
    }
    hipLaunchKernelGGL((transpose_vec4_kernel<TR, TS, THREADS>), dim3((unsigned)tiles), dim3(THREADS), lds_bytes, st,
                       src, dst, R, S, (uint32_t)tiles_s, env_int("CNNMEM_TRANSFORM_XCD", 0));
    return launch_status();
}

template <int TR, int TS>
int launch_u1(const float* src, float* dst, long long R, long long S, hipStream_t st, int xcd_default = 0) {
    const long long tiles_r = ceil_div64(R, TR), tiles_s = ceil_div64(S, TS);
    const long long tiles = tiles_r * tiles_s;
    if (tiles > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((transpose_u1_kernel<TR, TS>), dim3((unsigned)tiles), dim3(TR * TS / 4), 0, st,
                       src, dst, R, S, (uint32_t)tiles_s, env_int("CNNMEM_TRANSFORM_XCD", xcd_default));
    return launch_status();
}

}  // namespace

int launch_transpose2d(const float* src, float* dst, long long R, long long S, hipStream_t st) {
    if (R == 1 || S == 1) return launch_copy(src, dst, R * S, st);     // a vector: nothing moves
    const bool vec = (R % 4 == 0) && (S % 4 == 0) && aligned16(src) && aligned16(dst);
    // at most 8 rows on one side (batches of 2..8 images): the thin-plane kernels, which idle no lanes
    const bool thin = (R <= 8 || S <= 8) && R * S >= 4 && env_int("CNNMEM_TRANSFORM_TILE", -1) < 0;
    if (vec && !thin) {
        // Tile shape: square by default; when one side of the matrix is short
        // (small batch N) the tile is stretched along the other side so that no
        // lane idles; for the batch sizes of real networks (N >= 128) the tile
        // spans 128 images, which makes the CHWN side of the tile one contiguous
        // run.  Shapes 7 / 8 measured best on MI355X for N = 128 (71 % / 69 % of
        // peak HBM bandwidth against 67 % for the square tile).
        // CNNMEM_TRANSFORM_TILE forces a shape for A/B profiling.
        int shape = env_int("CNNMEM_TRANSFORM_TILE", -1);
        if (shape < 0) {
            if (R <= 16) shape = 3;
            else if (R <= 32) shape = 2;
            else if (S <= 16) shape = 5;
            else if (S <= 32) shape = 4;
            // the short side fits one 128-wide tile side (N = 65..128: one tile spans every image; measured
            // on 100x64x57x57: 36 -> 65 % and 50 -> 63 % against two 64-wide tiles with the second mostly idle)
            // 256 images and more (several tiles along the batch): the one-float4-per-lane tile with neighbouring
            // tiles on one XCD, measured back to back on 256x96x55x55 107.4 -> 97.4 us, 256x64x56x56 77.1 -> 68.1 us,
            // 256x512x14x14 38.7 -> 35.8 us, 384x64x28x28 30.1 -> 28.7 us (192 images: level, left as they are)
            else if (R >= 256 && S >= 4 * R) shape = 12;
            else if (R > 64 && S >= 4 * R) shape = 7;      // few long source rows (NCHW -> CHWN)
            else if (S > 64 && R >= 4 * S) shape = 8;      // many short source rows (CHWN -> NCHW)
            // 48..64 images: the same one-float-per-access LDS tile as shape 8, 64 wide (CHWN -> NCHW on
            // 64x256x56x56: 66.6 -> 71.0 % of peak, 64x64x224x224 65.8 -> 68.3 %, 48x128x56x56 61.1 -> 62.8 %;
            // 40 images lose, 55 x 55 planes are level), and a 128-long tile side along the long source rows
            // (NCHW -> CHWN: 69.6 -> 70.7 %)
            else if (S >= 48 && S <= 64 && R >= 4 * S) shape = 10;
            else if (R == 64 && S >= 4 * R) shape = 6;
            else shape = 0;
        }
        switch (shape) {
            case 1: return launch_vec4<128, 64>(src, dst, R, S, st);
            case 2: return launch_vec4<32, 128>(src, dst, R, S, st);
            case 3: return launch_vec4<16, 256>(src, dst, R, S, st);
            case 4: return launch_vec4<128, 32>(src, dst, R, S, st);
            case 5: return launch_vec4<256, 16>(src, dst, R, S, st);
            case 6: return launch_vec4<64, 128>(src, dst, R, S, st);
            case 7: return launch_vec4<128, 64, 512>(src, dst, R, S, st);
            case 8: return launch_u1<32, 128>(src, dst, R, S, st);
            case 12: return launch_u1<32, 128>(src, dst, R, S, st, 1);
            case 9: return launch_u1<128, 32>(src, dst, R, S, st);
            case 10: return launch_u1<64, 64>(src, dst, R, S, st);
            case 11: return launch_vec4<128, 128, 1024>(src, dst, R, S, st);
            default: return launch_vec4<64, 64>(src, dst, R, S, st);
        }
    }
    // any R, S and any 4-byte alignment: the strided tile kernel of the general permutation,
    // 128-bit accesses at dword alignment (CNNMEM_TRANSFORM_TILE=100 forces the dword kernel for A/B runs)
    if (env_int("CNNMEM_TRANSFORM_TILE", -1) != 100) return launch_transpose2d_any(src, dst, R, S, st);
    const long long tiles_r = ceil_div64(R, 64), tiles_s = ceil_div64(S, 64);
    if (tiles_r * tiles_s > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(transpose_scalar_kernel, dim3((unsigned)(tiles_r * tiles_s)), dim3(kThreads), 0, st,
                       src, dst, R, S, (uint32_t)tiles_s);
    return launch_status();
}

int launch_copy(const float* src, float* dst, long long n, hipStream_t st) {
    if (aligned16(src) && aligned16(dst) && n % 4 == 0) {
        const size_t n4 = (size_t)n / 4;
        const size_t per_launch = (size_t)0x40000000 * kThreads;   // grid.x stays below 2^31
        for (size_t first = 0; first < n4; first += per_launch) {
            const size_t todo = n4 - first < per_launch ? n4 - first : per_launch;
            hipLaunchKernelGGL(copy_vec4_kernel, dim3((unsigned)ceil_div64((long long)todo, kThreads)),
                               dim3(kThreads), 0, st, src, dst, n4, first);
        }
    } else {
        const unsigned blocks = (unsigned)(ceil_div64(n, kThreads) < 16384 ? ceil_div64(n, kThreads) : 16384);
        hipLaunchKernelGGL(copy_scalar_kernel, dim3(blocks), dim3(kThreads), 0, st, src, dst, (size_t)n);
    }
    return launch_status();
}

}  // namespace cnnmem
