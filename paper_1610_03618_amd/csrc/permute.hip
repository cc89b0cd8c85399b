// Change between any two of the 24 storage orders of a 4-D tensor (Section I;
// Section IV.A names CHWN and HWCN, the comparison libraries add NHWC).
//
// The host first brings the permutation into a canonical form: axes of extent 1
// are dropped and source axes that stay neighbours, in the same order, in the
// destination are merged.  What is left has rank k <= 4 and is one of
//
//   k <= 1                         a plain copy;
//   k == 2                         the 2-D transpose that also serves NCHW <-> CHWN;
//   fastest axis stays fastest     "row move": contiguous runs of the fastest axis
//                                  are gathered, 128 bits per lane when they allow;
//   fastest axis changes           a batch of strided 2-D transposes over the plane
//                                  spanned by the source's and the destination's
//                                  fastest axes; the other (at most two) axes only
//                                  add an offset on both sides.
//
// The tiled kernel is the strided, batched form of the 2-D transpose: global
// accesses run along the fastest axis of the side they touch, 128 bits per lane
// at any 4-byte alignment (rows of odd length start at every phase), a tile is
// turned through LDS, all loads are unconditional from clamped addresses.
#include "common.hpp"

namespace cnnmem {
namespace {

constexpr int kThreads = 256;

struct TilePlan {
    long long R, S;             // extents: R along the destination's fastest axis, S along the source's
    long long ss_r;             // source stride of r (source stride of s is 1)
    long long ds_s;             // destination stride of s (destination stride of r is 1)
    long long sb0, sb1;         // source strides of the batch axes
    long long db0, db1;         // destination strides of the batch axes
    uint32_t tiles_s, tiles_plane;
    int xcd_order;              // neighbouring tiles on one XCD (they share partly written lines)
};

template <int TS>
__device__ __forceinline__ int lds_row(int s_local) {
    return (s_local & 3) * (TS / 4) + (s_local >> 2);
}

// TR x TS tile, 256 lanes.  Both sides move 128 bits per lane along their own
// fastest axis at whatever 4-byte alignment the rows happen to have (rows of odd
// length start at every phase); only a source narrower than four words (LV =
// false) is read word by word.  LDS holds the tile in destination order: row s
// (swizzled as in the 2-D kernel), pitch TR + 4 floats.
template <int TR, int TS, int THREADS, bool LV>
__global__ __launch_bounds__(THREADS) void permute_tile_kernel(
    const float* __restrict__ src, float* __restrict__ dst, TilePlan p, FastDiv d_plane, FastDiv d_tiles_s,
    FastDiv d_nb1) {
    static_assert(TR % 4 == 0 && TS % 4 == 0, "tile sides are multiples of 4");
    static_assert((TR * TS / 4) % THREADS == 0, "whole number of float4 per lane");
    constexpr int P = TR + 4;
    constexpr int NBR = TR / 4;
    constexpr int WORDS = TR * TS / THREADS;            // dwords per lane
    __shared__ __attribute__((aligned(16))) float tile[(TS + 1) * P];   // one spare row, never read

    const uint32_t tile_id = p.xcd_order ? xcd_contiguous_tile(blockIdx.x, gridDim.x) : blockIdx.x;
    const uint32_t batch = fd_div(tile_id, d_plane);
    const uint32_t in_plane = tile_id - batch * p.tiles_plane;
    const uint32_t tr = fd_div(in_plane, d_tiles_s);
    const uint32_t ts = in_plane - tr * p.tiles_s;
    const uint32_t b0 = fd_div(batch, d_nb1);
    const uint32_t b1 = batch - b0 * d_nb1.d;
    const long long r0 = (long long)tr * TR, s0 = (long long)ts * TS;
    src += (size_t)b0 * (size_t)p.sb0 + (size_t)b1 * (size_t)p.sb1;
    dst += (size_t)b0 * (size_t)p.db0 + (size_t)b1 * (size_t)p.db1;
    const int tid = threadIdx.x;

    if (LV) {
        // One source row per load.  A load that would run past the end of the row starts at S - 4
        // instead (S >= 4 here) and its words are filed under the columns they really are; rows
        // past R re-read the last row and land in tile rows that are never written out.  All
        // loads are unconditional, hence in flight together.
        constexpr int NC4 = TS / 4;
        float4 v[WORDS / 4];
        int col[WORDS / 4];                             // tile column of v[it].x; may be -3..-1 in the last tile
#pragma unroll
        for (int it = 0; it < WORDS / 4; ++it) {
            const int f = tid + it * THREADS;
            const int c4 = f % NC4, rl = f / NC4;
            long long r = r0 + rl, s = s0 + 4 * c4;
            r = r < p.R ? r : p.R - 1;
            s = s + 4 <= p.S ? s : p.S - 4;
            col[it] = (int)(s - s0);
            v[it] = ld4u_stream(src + (size_t)r * (size_t)p.ss_r + (size_t)s);
        }
#pragma unroll
        for (int it = 0; it < WORDS / 4; ++it) {
            const int rl = (tid + it * THREADS) / NC4;
            const int c = col[it];
            const float w[4] = {v[it].x, v[it].y, v[it].z, v[it].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {               // words left of the tile go to the spare row
                const int row = c + j >= 0 ? lds_row<TS>(c + j) : TS;
                tile[row * P + rl] = w[j];
            }
        }
    } else {
        // fewer than four words per source row: dword loads, lanes along s, clamped to valid words
        float v[WORDS];
#pragma unroll
        for (int it = 0; it < WORDS; ++it) {
            const int e = tid + it * THREADS;
            const int sl = e % TS, rl = e / TS;
            long long r = r0 + rl, s = s0 + sl;
            r = r < p.R ? r : p.R - 1;
            s = s < p.S ? s : p.S - 1;
            v[it] = ld1_stream(src + (size_t)r * (size_t)p.ss_r + (size_t)s);
        }
#pragma unroll
        for (int it = 0; it < WORDS; ++it) {
            const int e = tid + it * THREADS;
            const int sl = e % TS, rl = e / TS;
            tile[lds_row<TS>(sl) * P + rl] = v[it];
        }
    }
    __syncthreads();
    // every LDS read first, then the stores (the branches of the ragged end would keep read, wait and store of
    // each iteration together)
    constexpr int STORE_ITERS = (TS * NBR) / THREADS;
    float4 ov[STORE_ITERS];
#pragma unroll
    for (int it = 0; it < STORE_ITERS; ++it) {
        const int f = tid + it * THREADS;
        ov[it] = *reinterpret_cast<const float4*>(tile + lds_row<TS>(f / NBR) * P + 4 * (f % NBR));
    }
#pragma unroll
    for (int it = 0; it < STORE_ITERS; ++it) {
        const int f = tid + it * THREADS;
        const int br = f % NBR, sl = f / NBR;
        const float4 o = ov[it];
        const long long s = s0 + sl, r = r0 + 4 * br;
        if (s < p.S) {
            float* q = dst + (size_t)s * (size_t)p.ds_s + (size_t)r;
            if (r + 4 <= p.R) {
                st4u_stream(q, o);
            } else {                                    // ragged end of a destination row
                if (r < p.R) st1_stream(q, o.x);
                if (r + 1 < p.R) st1_stream(q + 1, o.y);
                if (r + 2 < p.R) st1_stream(q + 2, o.z);
            }
        }
    }
}

// ---- thin planes: one tile axis has at most 8 entries (RGB images between NCHW and NHWC) ----
//
// With T <= 8 rows on one side the square tiles above would idle most lanes.  Here a
// workgroup takes all T entries of the thin axis and kThin entries of the long one; on the
// side where the thin axis is the fastest, that block is one contiguous piece of memory
// (the launcher checks the stride) and is moved as a linear 128-bit stream.

constexpr int kThin = 1024;     // entries of the long axis per workgroup

// The block's kThin * T words sit in LDS in the order of its contiguous side, as 128-bit slots;
// slot f lives at f + f/8.  Eight neighbouring lanes that each own T consecutive slots (stride T),
// and eight lanes that walk consecutive slots, then both touch eight different 16-byte bank groups
// for every T <= 8; with words T apart and no padding, T = 8 put all lanes of a wavefront on two banks.
__device__ __forceinline__ int thin_slot(int f) { return f + (f >> 3); }
__device__ __forceinline__ int thin_word(int i) { return 4 * thin_slot(i >> 2) + (i & 3); }
constexpr int thin_lds_words(int T) { return 4 * (kThin / 4 * T + kThin / 32 * T); }
__device__ __forceinline__ float component(const float4& v, int c) { return c == 0 ? v.x : c == 1 ? v.y : c == 2 ? v.z : v.w; }

// Destination rows are thin: dst[s][r], r < T, rows back to back (ds_s == T).
template <int T>
__global__ __launch_bounds__(kThreads) void permute_thin_dst_kernel(
    const float* __restrict__ src, float* __restrict__ dst, TilePlan p, FastDiv d_plane, FastDiv d_nb1) {
    __shared__ __attribute__((aligned(16))) float tile[thin_lds_words(T)];
    const uint32_t batch = fd_div(blockIdx.x, d_plane);
    const uint32_t ts = blockIdx.x - batch * p.tiles_plane;
    const uint32_t b0 = fd_div(batch, d_nb1);
    const uint32_t b1 = batch - b0 * d_nb1.d;
    src += (size_t)b0 * (size_t)p.sb0 + (size_t)b1 * (size_t)p.sb1;
    dst += (size_t)b0 * (size_t)p.db0 + (size_t)b1 * (size_t)p.db1;
    const long long s0 = (long long)ts * kThin;
    const int ns = (int)(p.S - s0 < kThin ? p.S - s0 : kThin);
    const int tid = threadIdx.x;

    // T source rows of kThin words: one float4 per lane per row; the lanes at the end of the last
    // block re-read the row's last four words instead (S >= 4: launcher)
    long long s = s0 + 4 * tid;
    s = s + 4 <= p.S ? s : p.S - 4;
    const int col = (int)(s - s0);                      // -3 .. kThin - 4
    float4 v[T];
#pragma unroll
    for (int r = 0; r < T; ++r) v[r] = ld4u_stream(src + (size_t)r * (size_t)p.ss_r + (size_t)s);
    if (col == 4 * tid) {
        // four columns x T rows = 4T consecutive destination words = T whole slots
        float w[4 * T];
#pragma unroll
        for (int r = 0; r < T; ++r) {
            w[0 * T + r] = v[r].x;
            w[1 * T + r] = v[r].y;
            w[2 * T + r] = v[r].z;
            w[3 * T + r] = v[r].w;
        }
#pragma unroll
        for (int k = 0; k < T; ++k)
            *reinterpret_cast<float4*>(tile + 4 * thin_slot(tid * T + k)) =
                make_float4(w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3]);
    } else {
        // shifted lanes: word by word; columns left of the block belong to the previous one
#pragma unroll
        for (int r = 0; r < T; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (col + c >= 0) tile[thin_word((col + c) * T + r)] = component(v[r], c);
    }
    __syncthreads();
    // the block's ns * T destination words are contiguous
    float* out = dst + (size_t)s0 * T;
    const int total = ns * T;
    for (int i = 4 * tid; i < total; i += 4 * kThreads) {
        if (i + 4 <= total) {
            st4u_through(out + i, *reinterpret_cast<const float4*>(tile + 4 * thin_slot(i >> 2)));
        } else {
            for (int j = i; j < total; ++j) st1_stream(out + j, tile[thin_word(j)]);
        }
    }
}

// Source rows are thin: src[r][s], s < T, rows back to back (ss_r == T).
template <int T>
__global__ __launch_bounds__(kThreads) void permute_thin_src_kernel(
    const float* __restrict__ src, float* __restrict__ dst, TilePlan p, FastDiv d_plane, FastDiv d_nb1) {
    __shared__ __attribute__((aligned(16))) float tile[thin_lds_words(T)];
    const uint32_t batch = fd_div(blockIdx.x, d_plane);
    const uint32_t tr = blockIdx.x - batch * p.tiles_plane;
    const uint32_t b0 = fd_div(batch, d_nb1);
    const uint32_t b1 = batch - b0 * d_nb1.d;
    src += (size_t)b0 * (size_t)p.sb0 + (size_t)b1 * (size_t)p.sb1;
    dst += (size_t)b0 * (size_t)p.db0 + (size_t)b1 * (size_t)p.db1;
    const long long r0 = (long long)tr * kThin;
    const int nr = (int)(p.R - r0 < kThin ? p.R - r0 : kThin);
    const int tid = threadIdx.x;

    // the block's nr * T source words are contiguous: linear float4 stream, the last one shifted
    // back so that it ends with the block (the whole plane holds R * T >= 4 words: launcher)
    const float* in = src + (size_t)r0 * T;
    const int total = nr * T;
    const long long before = r0 * T;                    // words of this plane in front of the block
    float4 v[T];
    int at[T];
#pragma unroll
    for (int k = 0; k < T; ++k) {
        int i = 4 * (tid + k * kThreads);
        i = i + 4 <= total ? i : total - 4;
        if ((long long)i + before < 0) i = (int)-before;   // tiny first block: start at the plane's first word
        at[k] = i;
        v[k] = ld4u_stream(in + i);
    }
#pragma unroll
    for (int k = 0; k < T; ++k) {
        if (at[k] == 4 * (tid + k * kThreads)) {
            *reinterpret_cast<float4*>(tile + 4 * thin_slot(tid + k * kThreads)) = v[k];
        } else {
            // shifted lanes: word by word; words in front of the block belong to the previous one
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (at[k] + c >= 0) tile[thin_word(at[k] + c)] = component(v[k], c);
        }
    }
    __syncthreads();
    // T destination rows of nr words; a lane's four rows x T columns are T whole slots
    const int r = 4 * tid;
    if (r + 4 <= nr) {
        float w[4 * T];
#pragma unroll
        for (int k = 0; k < T; ++k) {
            const float4 q = *reinterpret_cast<const float4*>(tile + 4 * thin_slot(tid * T + k));
            w[4 * k] = q.x;
            w[4 * k + 1] = q.y;
            w[4 * k + 2] = q.z;
            w[4 * k + 3] = q.w;
        }
#pragma unroll
        for (int sidx = 0; sidx < T; ++sidx)
            st4u_through(dst + (size_t)sidx * (size_t)p.ds_s + (size_t)(r0 + r),
                        make_float4(w[0 * T + sidx], w[1 * T + sidx], w[2 * T + sidx], w[3 * T + sidx]));
    } else {
        for (int sidx = 0; sidx < T; ++sidx)
            for (int j = r; j < nr; ++j)
                st1_stream(dst + (size_t)sidx * (size_t)p.ds_s + (size_t)(r0 + j), tile[thin_word(j * T + sidx)]);
    }
}

struct RowPlan {
    long long t0, t1, t2;       // source strides of the destination's outer axes (slowest first), in floats
    uint32_t L;                 // extent of the fastest axis (the run length)
    uint32_t total;             // all elements
};

__device__ __forceinline__ size_t run_source(uint32_t run, const RowPlan& p, const FastDiv& d_e2, const FastDiv& d_e1) {
    const uint32_t q = fd_div(run, d_e2);
    const uint32_t o2 = run - q * d_e2.d;
    const uint32_t o0 = fd_div(q, d_e1);
    const uint32_t o1 = q - o0 * d_e1.d;
    return (size_t)o0 * (size_t)p.t0 + (size_t)o1 * (size_t)p.t1 + (size_t)o2 * (size_t)p.t2;
}

// The fastest axis is the same on both sides: the destination is a sequence of
// runs of L words, each contiguous in the source too.  A lane owns four
// consecutive destination words (one 128-bit store; DA = the destination is
// 16-byte aligned); when they lie in one run they are one 128-bit load at the
// run's own alignment, else (run boundary inside the four, or the end of the
// tensor) they are fetched one by one.
template <bool DA>
__global__ __launch_bounds__(kThreads) void permute_rows_kernel(
    const float* __restrict__ src, float* __restrict__ dst, RowPlan p, FastDiv d_L, FastDiv d_e2, FastDiv d_e1) {
    const uint32_t e = 4u * (blockIdx.x * kThreads + threadIdx.x);
    if (e >= p.total) return;
    const uint32_t run = fd_div(e, d_L);
    const uint32_t in_run = e - run * p.L;
    if (in_run + 4 <= p.L) {                            // e + 4 <= total follows
        const float4 v = ld4u_stream(src + run_source(run, p, d_e2, d_e1) + in_run);
        if (DA) st4_stream(dst + e, v);
        else st4u_stream(dst + e, v);
        return;
    }
    for (uint32_t j = 0; j < 4 && e + j < p.total; ++j) {
        const uint32_t rj = fd_div(e + j, d_L);
        dst[e + j] = src[run_source(rj, p, d_e2, d_e1) + (e + j - rj * p.L)];
    }
}

template <int TR, int TS, int THREADS = kThreads>
int launch_tile(const float* src, float* dst, const TilePlan& p, long long nb0, long long nb1, hipStream_t st) {
    TilePlan q = p;
    const long long tiles_r = ceil_div64(p.R, TR), tiles_s = ceil_div64(p.S, TS);
    const long long plane = tiles_r * tiles_s;
    if (plane >= 0x7fffffffLL || nb0 * nb1 >= 0x7fffffffLL || plane * nb0 * nb1 >= 0x7fffffffLL)
        return CNNMEM_ERR_UNSUPPORTED;
    q.tiles_s = (uint32_t)tiles_s;
    q.tiles_plane = (uint32_t)plane;
    q.xcd_order = env_int("CNNMEM_PERMUTE_XCD", p.xcd_order);
    const FastDiv d_plane = make_fastdiv((uint32_t)plane), d_tiles_s = make_fastdiv((uint32_t)tiles_s),
                  d_nb1 = make_fastdiv((uint32_t)nb1);
    const dim3 grid((unsigned)(plane * nb0 * nb1)), block(THREADS);
    if (p.S >= 4)
        hipLaunchKernelGGL((permute_tile_kernel<TR, TS, THREADS, true>), grid, block, 0, st, src, dst, q, d_plane,
                           d_tiles_s, d_nb1);
    else
        hipLaunchKernelGGL((permute_tile_kernel<TR, TS, THREADS, false>), grid, block, 0, st, src, dst, q, d_plane,
                           d_tiles_s, d_nb1);
    return launch_status();
}

template <int T>
int launch_thin(bool thin_dst, const float* src, float* dst, const TilePlan& p, long long nb0, long long nb1,
                hipStream_t st) {
    TilePlan q = p;
    const long long plane = ceil_div64(thin_dst ? p.S : p.R, kThin);
    if (plane >= 0x7fffffffLL || nb0 * nb1 >= 0x7fffffffLL || plane * nb0 * nb1 >= 0x7fffffffLL)
        return CNNMEM_ERR_UNSUPPORTED;
    q.tiles_plane = (uint32_t)plane;
    q.tiles_s = thin_dst ? (uint32_t)plane : 1;
    const FastDiv d_plane = make_fastdiv((uint32_t)plane), d_nb1 = make_fastdiv((uint32_t)nb1);
    const dim3 grid((unsigned)(plane * nb0 * nb1)), block(kThreads);
    if (thin_dst)
        hipLaunchKernelGGL((permute_thin_dst_kernel<T>), grid, block, 0, st, src, dst, q, d_plane, d_nb1);
    else
        hipLaunchKernelGGL((permute_thin_src_kernel<T>), grid, block, 0, st, src, dst, q, d_plane, d_nb1);
    return launch_status();
}

int launch_thin_any(int T, bool thin_dst, const float* src, float* dst, const TilePlan& p, long long nb0,
                    long long nb1, hipStream_t st) {
    switch (T) {
        case 2: return launch_thin<2>(thin_dst, src, dst, p, nb0, nb1, st);
        case 3: return launch_thin<3>(thin_dst, src, dst, p, nb0, nb1, st);
        case 4: return launch_thin<4>(thin_dst, src, dst, p, nb0, nb1, st);
        case 5: return launch_thin<5>(thin_dst, src, dst, p, nb0, nb1, st);
        case 6: return launch_thin<6>(thin_dst, src, dst, p, nb0, nb1, st);
        case 7: return launch_thin<7>(thin_dst, src, dst, p, nb0, nb1, st);
        default: return launch_thin<8>(thin_dst, src, dst, p, nb0, nb1, st);
    }
}

int launch_tile_shape(const float* src, float* dst, const TilePlan& p, long long nb0, long long nb1, hipStream_t st) {
    // thin planes (2..8 entries on one tile axis, contiguous on the side where that axis is fastest)
    if (env_int("CNNMEM_PERMUTE_TILE", -1) < 0) {
        if (p.R >= 2 && p.R <= 8 && p.ds_s == p.R && p.S >= 4)
            return launch_thin_any((int)p.R, true, src, dst, p, nb0, nb1, st);
        if (p.S >= 2 && p.S <= 8 && p.ss_r == p.S && p.R * p.S >= 4)
            return launch_thin_any((int)p.S, false, src, dst, p, nb0, nb1, st);
    }
    // Tile shape.  Rows whose length is not a whole number of 128-byte lines start at every
    // phase, so each segment a tile reads or writes ends in partly used lines: the side with
    // such rows gets the long side of the tile (measured on MI355X, 128x96x55x55:
    // NHWC -> NCHW 38 % of peak with 64 x 64, 63 % with 256 x 32).  A short side stretches the
    // tile along the other one.  CNNMEM_PERMUTE_TILE forces a shape for A/B profiling.
    int shape = env_int("CNNMEM_PERMUTE_TILE", -1);
    if (shape < 0) {
        const bool ragged_dst = p.R % 32 != 0, ragged_src = p.S % 32 != 0;
        if (p.R <= 16) shape = 3;
        else if (p.R <= 32) shape = ragged_src && p.S >= 256 ? 8 : 1;
        else if (p.S <= 16) shape = 4;
        else if (p.S <= 32) shape = ragged_dst && p.R >= 256 ? 11 : 2;
        else if (ragged_dst && !ragged_src && p.R > 128) shape = 11;   // 13x13 and 14x14 planes included
        else if (ragged_src && !ragged_dst && p.S > 128) shape = 8;
        else shape = 0;
    }
    switch (shape) {
        case 1: return launch_tile<32, 128>(src, dst, p, nb0, nb1, st);
        case 2: return launch_tile<128, 32>(src, dst, p, nb0, nb1, st);
        case 3: return launch_tile<16, 256>(src, dst, p, nb0, nb1, st);
        case 4: return launch_tile<256, 16>(src, dst, p, nb0, nb1, st);
        case 5: return launch_tile<128, 64, 512>(src, dst, p, nb0, nb1, st);
        case 6: return launch_tile<64, 128, 512>(src, dst, p, nb0, nb1, st);
        case 7: return launch_tile<256, 32, 512>(src, dst, p, nb0, nb1, st);
        case 8: return launch_tile<32, 256, 512>(src, dst, p, nb0, nb1, st);
        case 9: return launch_tile<128, 64, 256>(src, dst, p, nb0, nb1, st);
        case 10: return launch_tile<64, 128, 256>(src, dst, p, nb0, nb1, st);
        case 11: return launch_tile<256, 32, 256>(src, dst, p, nb0, nb1, st);
        case 12: return launch_tile<32, 256, 256>(src, dst, p, nb0, nb1, st);
        default: return launch_tile<64, 64>(src, dst, p, nb0, nb1, st);
    }
}

}  // namespace

// src[R][S] -> dst[S][R] for any R, S and any 4-byte alignment (the 2-D transpose's general path).
int launch_transpose2d_any(const float* src, float* dst, long long R, long long S, hipStream_t st) {
    TilePlan p;
    p.R = R; p.S = S; p.ss_r = S; p.ds_s = R;
    p.sb0 = p.sb1 = p.db0 = p.db1 = 0;
    p.xcd_order = 0;
    return launch_tile_shape(src, dst, p, 1, 1, st);
}

void canonical_permutation(const int* dims, const int* perm, int* rank, long long* cdims, int* cperm) {
    // source axes of extent > 1, in destination order
    int order[4], n = 0;
    for (int i = 0; i < 4; ++i)
        if (dims[perm[i]] > 1) order[n++] = perm[i];
    // groups of source axes that are consecutive (a, a+1, ...) in this order, skipping over
    // extent-1 axes in between, stay one block of memory on both sides
    int first[4], last[4], groups = 0;
    for (int i = 0; i < n; ++i) {
        bool joins = false;
        if (groups > 0 && order[i] > last[groups - 1]) {
            joins = true;
            for (int a = last[groups - 1] + 1; a < order[i]; ++a)
                if (dims[a] > 1) joins = false;
        }
        if (joins) {
            last[groups - 1] = order[i];
        } else {
            first[groups] = last[groups] = order[i];
            ++groups;
        }
    }
    // relabel groups by their place in the source
    for (int g = 0; g < groups; ++g) {
        int place = 0;
        for (int h = 0; h < groups; ++h)
            if (first[h] < first[g]) ++place;
        cperm[g] = place;
        long long e = 1;
        for (int a = first[g]; a <= last[g]; ++a) e *= dims[a];
        cdims[place] = e;
    }
    *rank = groups;
}

PermutePlan plan_permutation(const int* dims, const int* perm) {
    PermutePlan pl = {};
    int k;
    long long d[4];
    int pm[4];
    canonical_permutation(dims, perm, &k, d, pm);
    pl.total = 1;
    for (int i = 0; i < 4; ++i) pl.total *= dims[i];
    if (k <= 1) { pl.kind = PermutePlan::kCopy; return pl; }
    if (k == 2) { pl.kind = PermutePlan::kTranspose2d; pl.R = d[0]; pl.S = d[1]; return pl; }

    long long ss[4], ds[4], e[4];                   // source strides by source axis; destination strides / extents by position
    ss[k - 1] = 1;
    for (int a = k - 2; a >= 0; --a) ss[a] = ss[a + 1] * d[a + 1];
    for (int i = 0; i < k; ++i) e[i] = d[pm[i]];
    ds[k - 1] = 1;
    for (int i = k - 2; i >= 0; --i) ds[i] = ds[i + 1] * e[i + 1];
    if (pm[k - 1] == k - 1) {
        // the fastest axis stays: its runs are gathered; outer destination axes padded at the slow end to three
        pl.kind = PermutePlan::kRows;
        pl.L = d[k - 1];
        for (int i = 0; i < 3; ++i) { pl.oe[i] = 1; pl.ot[i] = 0; }
        for (int i = 0; i < k - 1; ++i) {
            pl.oe[3 - (k - 1) + i] = e[i];
            pl.ot[3 - (k - 1) + i] = ss[pm[i]];
        }
        pl.slow = 3 - (k - 1);
        return pl;
    }
    // the fastest axis changes: tiles over (destination's fastest axis r, source's fastest axis s)
    pl.kind = PermutePlan::kTiles;
    const int ar = pm[k - 1];                       // source axis that is fastest in the destination
    int pos_s = 0;                                  // destination position of the source's fastest axis
    for (int i = 0; i < k; ++i)
        if (pm[i] == k - 1) pos_s = i;
    pl.R = d[ar];
    pl.S = d[k - 1];
    pl.ss_r = ss[ar];
    pl.ds_s = ds[pos_s];
    pl.nb0 = pl.nb1 = 1;
    pl.sb0 = pl.sb1 = pl.db0 = pl.db1 = 0;
    // When every batch axis is slower than both tile axes on both sides, each batch entry is a
    // contiguous block and tiles run in plain order.  Otherwise a batch axis sits between the
    // tile axes in memory (NCHW <-> HWCN: the channel axis), the segments of neighbouring
    // tiles interleave, and keeping neighbours on one XCD measured 5-10 points better.
    pl.xcd_order = 0;
    int nbatch = 0;
    for (int i = 0; i < k; ++i) {                   // remaining axes, in destination order
        if (i == k - 1 || i == pos_s) continue;
        if (i > pos_s || pm[i] > ar) pl.xcd_order = 1;
        if (nbatch == 0 && k == 4) { pl.nb0 = e[i]; pl.sb0 = ss[pm[i]]; pl.db0 = ds[i]; }
        else { pl.nb1 = e[i]; pl.sb1 = ss[pm[i]]; pl.db1 = ds[i]; }
        ++nbatch;
    }
    return pl;
}

int launch_permute(const float* src, float* dst, const int* dims, const int* perm, hipStream_t st) {
    const PermutePlan pl = plan_permutation(dims, perm);
    if (pl.kind == PermutePlan::kCopy) return launch_copy(src, dst, pl.total, st);
    if (pl.kind == PermutePlan::kTranspose2d) return launch_transpose2d(src, dst, pl.R, pl.S, st);
    if (pl.kind == PermutePlan::kRows) {
        // The kernel addresses elements with 32 bits; larger tensors go slice by slice along the
        // destination's slowest axis.
        const long long slice = pl.total / pl.oe[pl.slow];      // elements per entry of that axis
        const long long limit = 0x7fffffffLL;
        if (slice >= limit) return CNNMEM_ERR_UNSUPPORTED;
        const long long per_launch = pl.total < limit ? pl.oe[pl.slow] : limit / slice;
        const FastDiv d_L = make_fastdiv((uint32_t)pl.L);
        for (long long first = 0; first < pl.oe[pl.slow]; first += per_launch) {
            const long long count = pl.oe[pl.slow] - first < per_launch ? pl.oe[pl.slow] - first : per_launch;
            long long ce[3] = {pl.oe[0], pl.oe[1], pl.oe[2]};
            ce[pl.slow] = count;
            RowPlan p;
            p.t0 = pl.ot[0]; p.t1 = pl.ot[1]; p.t2 = pl.ot[2];
            p.L = (uint32_t)pl.L;
            p.total = (uint32_t)(count * slice);
            const FastDiv d_e2 = make_fastdiv((uint32_t)ce[2]), d_e1 = make_fastdiv((uint32_t)ce[1]);
            const float* sp = src + (size_t)first * (size_t)pl.ot[pl.slow];
            float* dp = dst + (size_t)first * (size_t)slice;
            const dim3 grid((unsigned)ceil_div64(ceil_div64(count * slice, 4), kThreads)), block(kThreads);
            if (aligned16(dp))
                hipLaunchKernelGGL((permute_rows_kernel<true>), grid, block, 0, st, sp, dp, p, d_L, d_e2, d_e1);
            else
                hipLaunchKernelGGL((permute_rows_kernel<false>), grid, block, 0, st, sp, dp, p, d_L, d_e2, d_e1);
        }
        return launch_status();
    }
    TilePlan p;
    p.R = pl.R; p.S = pl.S; p.ss_r = pl.ss_r; p.ds_s = pl.ds_s;
    p.sb0 = pl.sb0; p.sb1 = pl.sb1; p.db0 = pl.db0; p.db1 = pl.db1;
    p.xcd_order = pl.xcd_order;
    return launch_tile_shape(src, dst, p, pl.nb0, pl.nb1, st);
}

}  // namespace cnnmem
