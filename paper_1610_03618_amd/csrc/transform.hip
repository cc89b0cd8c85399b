// Layout transformation NCHW <-> CHWN as a 2-D transpose (Section IV.C).
//
// C, H and W keep their relative order in both layouts, so with M = C*H*W the
// NCHW tensor is an [N][M] matrix and the CHWN tensor is the [M][N] matrix: one
// generic kernel src[R][S] -> dst[S][R] serves both directions.
//
// gfx950 design (not the paper's Kepler float2 scheme): every lane moves
// 128-bit words on both the read and the write side, through an LDS tile that
// is already in destination order and free of bank conflicts.  Two kernels:
// 4x4 register blocks (four float4 from four consecutive source rows, transposed
// in registers, parked as four float4 in a padded, j-major LDS tile) for small
// batches, and a one-float4-per-lane tile with an XOR swizzle for the batch
// sizes of real networks.  A pattern-only kernel (the same addresses, no LDS, no
// barrier, data not transposed) runs at the same speed as these kernels, so
// what separates them from a plain copy is the order in which the memory system
// sees the strided side, not the on-chip part.
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
    uint32_t tiles_s) {
    static_assert(TR % 4 == 0 && TS % 4 == 0, "tile sides are multiples of 4");
    static_assert((TR * TS / 16) % THREADS == 0, "whole number of 4x4 blocks per lane");
    constexpr int P = TR + 4;                       // LDS pitch in floats (keeps float4 alignment)
    constexpr int NBS = TS / 4;                     // 4x4 blocks along S
    constexpr int LOAD_ITERS = (TR * TS / 16) / THREADS;
    constexpr int NBR = TR / 4;                     // float4 per destination row of the tile
    constexpr int STORE_ITERS = (TS * NBR) / THREADS;

    float* tile = reinterpret_cast<float*>(dyn_tile);   // TS * P floats, sized by the launch

    const uint32_t tile_id = blockIdx.x;
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

// Swizzled tile, one or a few float4 per lane.  Lanes load float4 of source rows and scatter their four
// words into an LDS tile that is already in destination order; after the barrier a lane reads one
// float4 of a destination row back and stores it.  The tile has no padding: LDS row q = j*(TS/4) + c
// holds destination row 4*c + j, and its float4 slot b sits at physical slot b ^ (c & 7).  A wavefront
// covers 8 float4 columns x 8 source rows per load, so the 32 lanes that scatter together hit 32
// different banks (4*(slot ^ c) + word), and the 16 lanes that read together take two whole 128-byte
// LDS rows: SQ_LDS_BANK_CONFLICT is 0 for every tile shape (a padded, unswizzled tile spent 70 % of its
// LDS cycles on conflicts).  Tile order: 0 = s-tiles fastest, 1 = the same with neighbouring tiles on
// one XCD, 2 = r-tiles fastest.  Order 2 with a tile that spans only 32 images walks the tensor once
// per group of 32 images: fewer rows of the strided side are open at a time, which the memory system
// rewards (CHWN -> NCHW, 256 images: 67.5 -> 72.0 % of peak).
template <int TR, int TS, int THREADS>
__global__ __launch_bounds__(THREADS) void transpose_swz_kernel(
    const float* __restrict__ src, float* __restrict__ dst, long long R, long long S, uint32_t tiles_r,
    uint32_t tiles_s, int order) {
    constexpr int NC4 = TS / 4;                     // float4 per source row of the tile
    constexpr int NBR = TR / 4;                     // float4 per destination row of the tile
    constexpr int ITERS = TR * TS / 4 / THREADS;
    constexpr int CG = NC4 / 8;                     // groups of 8 float4 columns
    static_assert(TR % 32 == 0 && TS % 32 == 0, "tile sides are multiples of 32");
    static_assert((TR * TS / 4) % THREADS == 0 && THREADS % 64 == 0, "whole float4 per lane, whole wavefronts");
    float* tile = reinterpret_cast<float*>(dyn_tile);   // TS rows of TR floats

    uint32_t tr, ts;
    if (order == 2) {
        tr = blockIdx.x % tiles_r;
        ts = blockIdx.x / tiles_r;
    } else {
        const uint32_t t = order == 1 ? xcd_contiguous_tile(blockIdx.x, gridDim.x) : blockIdx.x;
        tr = t / tiles_s;
        ts = t % tiles_s;
    }
    const long long r0 = (long long)tr * TR;
    const long long s0 = (long long)ts * TS;
    const int tid = threadIdx.x;

    // edge tiles: lanes outside the matrix re-read a valid word (never written out), so no load is conditional
    float4 v[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int e = tid + it * THREADS;
        const int c4 = (e & 7) + 8 * ((e >> 6) % CG);
        const int rl = ((e >> 3) & 7) + 8 * ((e >> 6) / CG);
        long long r = r0 + rl, s = s0 + 4 * c4;
        r = r < R ? r : R - 1;
        s = s < S ? s : S - 4;
        v[it] = ld4_stream(src + (size_t)r * (size_t)S + (size_t)s);
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int e = tid + it * THREADS;
        const int c4 = (e & 7) + 8 * ((e >> 6) % CG);
        const int rl = ((e >> 3) & 7) + 8 * ((e >> 6) / CG);
        const int col = 4 * ((rl >> 2) ^ (c4 & 7)) + (rl & 3);
        tile[(0 * NC4 + c4) * TR + col] = v[it].x;
        tile[(1 * NC4 + c4) * TR + col] = v[it].y;
        tile[(2 * NC4 + c4) * TR + col] = v[it].z;
        tile[(3 * NC4 + c4) * TR + col] = v[it].w;
    }
    __syncthreads();
    float4 o[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int e = tid + it * THREADS;
        const int br = e % NBR, q = e / NBR;
        o[it] = *reinterpret_cast<const float4*>(tile + q * TR + 4 * (br ^ (q % NC4 & 7)));
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int e = tid + it * THREADS;
        const int br = e % NBR, q = e / NBR;
        const long long s = s0 + 4 * (q % NC4) + q / NC4, r = r0 + 4 * br;
        if (s < S && r < R) st4_through(dst + (size_t)s * (size_t)R + (size_t)r, o[it]);
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
    // above the default per-workgroup limit (gfx950 has 160 KB): opt in, once per device
    if (lds_bytes > 65536 && !allow_large_lds<&transpose_vec4_kernel<TR, TS, THREADS>>(lds_bytes)) return CNNMEM_ERR_RUNTIME;
    hipLaunchKernelGGL((transpose_vec4_kernel<TR, TS, THREADS>), dim3((unsigned)tiles), dim3(THREADS), lds_bytes, st,
                       src, dst, R, S, (uint32_t)tiles_s);
    return launch_status();
}

template <int TR, int TS, int THREADS>
int launch_swz(const float* src, float* dst, long long R, long long S, hipStream_t st, int order) {
    const long long tiles_r = ceil_div64(R, TR), tiles_s = ceil_div64(S, TS);
    const long long tiles = tiles_r * tiles_s;
    if (tiles > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    constexpr size_t lds_bytes = sizeof(float) * TS * TR;
    if (lds_bytes > 65536 && !allow_large_lds<&transpose_swz_kernel<TR, TS, THREADS>>(lds_bytes)) return CNNMEM_ERR_RUNTIME;
    hipLaunchKernelGGL((transpose_swz_kernel<TR, TS, THREADS>), dim3((unsigned)tiles), dim3(THREADS), lds_bytes, st,
                       src, dst, R, S, (uint32_t)tiles_r, (uint32_t)tiles_s, order);
    return launch_status();
}

// Tile shapes of the 128-bit transpose.  The short side of the matrix is the batch (N images), the long
// side C*H*W.  Measured back to back on MI355X (fraction of 8 TB/s; a copy of the same bytes: 79-82 %):
enum Shape {
    kSquare,        // vec4 64 x 64: neither side short, or 33..47 images
    kRows16,        // vec4 16 x 256: at most 16 source rows, tile stretched along them
    kRows32,        // vec4 32 x 128
    kCols16,        // vec4 256 x 16: at most 16 source columns
    kCols32,        // vec4 128 x 32
    kLongRows64,    // vec4 64 x 128: NCHW -> CHWN, 64 images (74.6 %)
    kLongRows128,   // swz 128 x 32, 512 lanes: NCHW -> CHWN, 65..255 images (128x96x55x55: 75.6 %)
    kLongRows256,   // swz 32 x 128, r-tiles fastest: NCHW -> CHWN from 256 images on (256x512x14x14: 71.2 %)
    kShortRows64,   // swz 64 x 64: CHWN -> NCHW, 48..64 images (64x256x56x56: 74.3 %)
    kShortRows128,  // swz 256 x 32, r-tiles fastest: CHWN -> NCHW, 65..255 images (128x96x55x55: 72.0 %)
    kShortRows256,  // swz 128 x 32, r-tiles fastest: CHWN -> NCHW from 256 images on (256x512x14x14: 72.0 %)
    kLongRowsRagged,   // vec4 128 x 64, 512 lanes: NCHW -> CHWN, 65..127 images that are not a multiple of 32
    kShortRowsRagged,  // swz 32 x 128: CHWN -> NCHW, the same batches (one tile spans every image)
    kLongRowsSmall,    // vec4 128 x 256, 1024 lanes, 135 KB of LDS: NCHW -> CHWN, 65..128 images, at most 24 MB
    kShortRowsSmall,   // swz 256 x 128, 1024 lanes, 128 KB of LDS: CHWN -> NCHW, the same tensors
    kNumShapes
};

// tiles of 256 along the long side (the short side fits one tile): between 128 and 256 of them
bool fat_tiles_fill_one_round(long long long_side) {
    const long long tiles = ceil_div64(long_side, 256);
    return tiles >= 128 && tiles <= 256;
}

Shape choose_shape(long long R, long long S) {
    if (R <= 16) return kRows16;
    if (R <= 32) return kRows32;
    if (S <= 16) return kCols16;
    if (S <= 32) return kCols32;
    if (S >= 4 * R) {                               // few long source rows: NCHW -> CHWN with R images
        if (R >= 256) return kLongRows256;
        // CHWN rows that are not whole 128-byte lines (100 images = 400 B): tiles of 32 images would leave a last
        // group of a few images that walks the whole tensor for them, and the more CHWN rows a tile holds, the
        // fewer lines it shares with its neighbours (100x64x57x57: 55.8 % with 128 x 32 tiles, 65 % with 128 x 64)
        if (R > 64 && R < 128 && R % 32 != 0) return kLongRowsRagged;
        // Small tensors: when fat tiles (128 KB in flight each) make exactly one round of workgroups that keeps at
        // least half of the 256 CUs busy, they beat many small ones (128x256x13x13, 22 MB, 169 tiles: 57 -> 69 % of
        // peak back to back, level with a copy of the same bytes; 36 MB and more: no gain; 5 MB, 36 tiles: slower)
        if (R > 64 && R <= 128 && fat_tiles_fill_one_round(S)) return kLongRowsSmall;
        // NCHW rows whose pitch is a multiple of 8 cache lines start on the same few memory channels: 128 of them
        // read at one column offset collide, 32 rows x 512 B spread (128x256x27x27: 64.7 -> 70.5 % of peak;
        // 128x96x55x55, pitch 9075 lines, prefers the 128-row tile: 75.6 % against 74.1 %)
        if (R > 64 && S % 256 == 0) return kLongRows256;
        if (R > 64) return kLongRows128;
        if (R == 64) return kLongRows64;
    } else if (R >= 4 * S) {                        // many short source rows: CHWN -> NCHW with S images
        if (S >= 256) return kShortRows256;
        if (S > 64 && S < 128 && S % 32 != 0) return kShortRowsRagged;   // 100x64x57x57: 46 % -> 63 %
        if (S > 64 && S <= 128 && fat_tiles_fill_one_round(R)) return kShortRowsSmall;   // 128x256x13x13: 58.6 -> 69 %
        if (S > 64) return kShortRows128;
        if (S >= 48) return kShortRows64;
    }
    return kSquare;
}

}  // namespace

int launch_transpose2d(const float* src, float* dst, long long R, long long S, hipStream_t st) {
    if (R == 1 || S == 1) return launch_copy(src, dst, R * S, st);     // a vector: nothing moves
    const bool vec = (R % 4 == 0) && (S % 4 == 0) && aligned16(src) && aligned16(dst);
    // CNNMEM_TRANSFORM_TILE forces a shape (tests run every shape on small ragged tensors)
    const int forced = env_int("CNNMEM_TRANSFORM_TILE", -1);
    // at most 8 rows on one side (batches of 2..8 images): the thin-plane kernels, which idle no lanes;
    // any other extents or alignment: the strided tile kernel of the general permutation, 128-bit
    // accesses at dword alignment
    const bool thin = (R <= 8 || S <= 8) && R * S >= 4;
    if (!vec || (thin && forced < 0)) return launch_transpose2d_any(src, dst, R, S, st);
    const Shape shape = forced >= 0 && forced < kNumShapes ? (Shape)forced : choose_shape(R, S);
    switch (shape) {
        case kRows16: return launch_vec4<16, 256>(src, dst, R, S, st);
        case kRows32: return launch_vec4<32, 128>(src, dst, R, S, st);
        case kCols16: return launch_vec4<256, 16>(src, dst, R, S, st);
        case kCols32: return launch_vec4<128, 32>(src, dst, R, S, st);
        case kLongRows64: return launch_vec4<64, 128>(src, dst, R, S, st);
        case kLongRows128: return launch_swz<128, 32, 512>(src, dst, R, S, st, 0);
        case kLongRows256: return launch_swz<32, 128, 1024>(src, dst, R, S, st, 2);
        case kShortRows64: return launch_swz<64, 64, 1024>(src, dst, R, S, st, 0);
        case kShortRows128: return launch_swz<256, 32, 1024>(src, dst, R, S, st, 2);
        case kShortRows256: return launch_swz<128, 32, 1024>(src, dst, R, S, st, 2);
        case kLongRowsRagged: return launch_vec4<128, 64, 512>(src, dst, R, S, st);
        case kShortRowsRagged: return launch_swz<32, 128, 1024>(src, dst, R, S, st, 0);
        case kLongRowsSmall: return launch_vec4<128, 256, 1024>(src, dst, R, S, st);
        case kShortRowsSmall: return launch_swz<256, 128, 1024>(src, dst, R, S, st, 0);
        default: return launch_vec4<64, 64>(src, dst, R, S, st);
    }
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
