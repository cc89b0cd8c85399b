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
// accesses run along the fastest axis of the side they touch (128-bit where
// extents and alignment allow, else dwords, independently per side), a tile is
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
};

template <int TS>
__device__ __forceinline__ int lds_row(int s_local) {
    return (s_local & 3) * (TS / 4) + (s_local >> 2);
}

// TR x TS tile, 256 lanes.  VL / VS: 128-bit accesses on the load / store side.
// LDS holds the tile in destination order: row s (swizzled as in the 2-D kernel),
// pitch TR + 4 floats.
template <int TR, int TS, bool VL, bool VS>
__global__ __launch_bounds__(kThreads) void permute_tile_kernel(
    const float* __restrict__ src, float* __restrict__ dst, TilePlan p, FastDiv d_plane, FastDiv d_tiles_s,
    FastDiv d_nb1) {
    static_assert(TR % 4 == 0 && TS % 4 == 0, "tile sides are multiples of 4");
    static_assert((TR * TS / 4) % kThreads == 0, "whole number of float4 per lane");
    constexpr int P = TR + 4;
    constexpr int NBR = TR / 4;
    constexpr int WORDS = TR * TS / kThreads;           // dwords per lane
    __shared__ __attribute__((aligned(16))) float tile[TS * P];

    const uint32_t batch = fd_div(blockIdx.x, d_plane);
    const uint32_t in_plane = blockIdx.x - batch * p.tiles_plane;
    const uint32_t tr = fd_div(in_plane, d_tiles_s);
    const uint32_t ts = in_plane - tr * p.tiles_s;
    const uint32_t b0 = fd_div(batch, d_nb1);
    const uint32_t b1 = batch - b0 * d_nb1.d;
    const long long r0 = (long long)tr * TR, s0 = (long long)ts * TS;
    src += (size_t)b0 * (size_t)p.sb0 + (size_t)b1 * (size_t)p.sb1;
    dst += (size_t)b0 * (size_t)p.db0 + (size_t)b1 * (size_t)p.db1;
    const int tid = threadIdx.x;

    if (VL) {
        // 128-bit loads along s, one source row per load; the four words of a load belong to
        // four destination rows and are scattered into the tile with dword writes
        constexpr int NC4 = TS / 4;
        float4 v[WORDS / 4];
#pragma unroll
        for (int it = 0; it < WORDS / 4; ++it) {
            const int f = tid + it * kThreads;
            const int c4 = f % NC4, rl = f / NC4;
            long long r = r0 + rl, s = s0 + 4 * c4;
            r = r < p.R ? r : p.R - 1;              // edge tiles re-read valid words that are never written out
            s = s < p.S ? s : p.S - 4;              // S is a multiple of 4 on this path
            v[it] = ld4_stream(src + (size_t)r * (size_t)p.ss_r + (size_t)s);
        }
#pragma unroll
        for (int it = 0; it < WORDS / 4; ++it) {
            const int f = tid + it * kThreads;
            const int c4 = f % NC4, rl = f / NC4;
            tile[lds_row<TS>(4 * c4 + 0) * P + rl] = v[it].x;
            tile[lds_row<TS>(4 * c4 + 1) * P + rl] = v[it].y;
            tile[lds_row<TS>(4 * c4 + 2) * P + rl] = v[it].z;
            tile[lds_row<TS>(4 * c4 + 3) * P + rl] = v[it].w;
        }
    } else {
        // dword loads, consecutive lanes along s; out-of-range lanes re-read the last valid word
        float v[WORDS];
#pragma unroll
        for (int it = 0; it < WORDS; ++it) {
            const int e = tid + it * kThreads;
            const int sl = e % TS, rl = e / TS;
            long long r = r0 + rl, s = s0 + sl;
            r = r < p.R ? r : p.R - 1;
            s = s < p.S ? s : p.S - 1;
            v[it] = ld1_stream(src + (size_t)r * (size_t)p.ss_r + (size_t)s);
        }
#pragma unroll
        for (int it = 0; it < WORDS; ++it) {
            const int e = tid + it * kThreads;
            const int sl = e % TS, rl = e / TS;
            tile[lds_row<TS>(sl) * P + rl] = v[it];
        }
    }
    __syncthreads();
    if (VS) {
#pragma unroll
        for (int it = 0; it < (TS * NBR) / kThreads; ++it) {
            const int f = tid + it * kThreads;
            const int br = f % NBR, sl = f / NBR;
            const float4 o = *reinterpret_cast<const float4*>(tile + lds_row<TS>(sl) * P + 4 * br);
            const long long s = s0 + sl, r = r0 + 4 * br;
            if (s < p.S && r < p.R) st4_stream(dst + (size_t)s * (size_t)p.ds_s + (size_t)r, o);
        }
    } else {
#pragma unroll
        for (int it = 0; it < WORDS; ++it) {
            const int e = tid + it * kThreads;
            const int rl = e % TR, sl = e / TR;
            const long long s = s0 + sl, r = r0 + rl;
            if (s < p.S && r < p.R) st1_stream(dst + (size_t)s * (size_t)p.ds_s + (size_t)r, tile[lds_row<TS>(sl) * P + rl]);
        }
    }
}

struct RowPlan {
    long long t0, t1, t2;       // source strides of the destination's outer axes (slowest first), in floats
    uint32_t per_row;           // items (float4 or floats) per run of the fastest axis
    uint32_t items;             // all items
};

// The fastest axis is the same on both sides: item i of the destination (a
// float4 or a float of a run) comes from the run's place in the source.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void permute_rows_kernel(
    const float* __restrict__ src, float* __restrict__ dst, RowPlan p, FastDiv d_row, FastDiv d_e2, FastDiv d_e1) {
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= p.items) return;
    const uint32_t run = fd_div(i, d_row);
    const uint32_t in_run = i - run * p.per_row;
    const uint32_t q = fd_div(run, d_e2);
    const uint32_t o2 = run - q * d_e2.d;
    const uint32_t o0 = fd_div(q, d_e1);
    const uint32_t o1 = q - o0 * d_e1.d;
    const size_t from = (size_t)o0 * (size_t)p.t0 + (size_t)o1 * (size_t)p.t1 + (size_t)o2 * (size_t)p.t2;
    if (VEC)
        st4_stream(dst + 4 * (size_t)i, ld4_stream(src + from + 4 * (size_t)in_run));
    else
        st1_stream(dst + (size_t)i, ld1_stream(src + from + in_run));
}

template <int TR, int TS>
int launch_tile(const float* src, float* dst, const TilePlan& p, long long nb0, long long nb1, bool vl, bool vs,
                hipStream_t st) {
    TilePlan q = p;
    const long long tiles_r = ceil_div64(p.R, TR), tiles_s = ceil_div64(p.S, TS);
    const long long plane = tiles_r * tiles_s;
    if (plane >= 0x7fffffffLL || nb0 * nb1 >= 0x7fffffffLL || plane * nb0 * nb1 >= 0x7fffffffLL)
        return CNNMEM_ERR_UNSUPPORTED;
    q.tiles_s = (uint32_t)tiles_s;
    q.tiles_plane = (uint32_t)plane;
    const FastDiv d_plane = make_fastdiv((uint32_t)plane), d_tiles_s = make_fastdiv((uint32_t)tiles_s),
                  d_nb1 = make_fastdiv((uint32_t)nb1);
    const dim3 grid((unsigned)(plane * nb0 * nb1)), block(kThreads);
    if (vl && vs)
        hipLaunchKernelGGL((permute_tile_kernel<TR, TS, true, true>), grid, block, 0, st, src, dst, q, d_plane,
                           d_tiles_s, d_nb1);
    else if (vl)
        hipLaunchKernelGGL((permute_tile_kernel<TR, TS, true, false>), grid, block, 0, st, src, dst, q, d_plane,
                           d_tiles_s, d_nb1);
    else if (vs)
        hipLaunchKernelGGL((permute_tile_kernel<TR, TS, false, true>), grid, block, 0, st, src, dst, q, d_plane,
                           d_tiles_s, d_nb1);
    else
        hipLaunchKernelGGL((permute_tile_kernel<TR, TS, false, false>), grid, block, 0, st, src, dst, q, d_plane,
                           d_tiles_s, d_nb1);
    return launch_status();
}

}  // namespace

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

int launch_permute(const float* src, float* dst, const int* dims, const int* perm, hipStream_t st) {
    int k;
    long long d[4];
    int pm[4];
    canonical_permutation(dims, perm, &k, d, pm);
    long long total = 1;
    for (int i = 0; i < 4; ++i) total *= dims[i];
    if (k <= 1) return launch_copy(src, dst, total, st);
    if (k == 2) return launch_transpose2d(src, dst, d[0], d[1], st);

    long long ss[4], ds[4], e[4];                   // source strides by source axis; destination strides / extents by position
    ss[k - 1] = 1;
    for (int a = k - 2; a >= 0; --a) ss[a] = ss[a + 1] * d[a + 1];
    for (int i = 0; i < k; ++i) e[i] = d[pm[i]];
    ds[k - 1] = 1;
    for (int i = k - 2; i >= 0; --i) ds[i] = ds[i + 1] * e[i + 1];
    const bool a16 = aligned16(src) && aligned16(dst);

    if (pm[k - 1] == k - 1) {
        // the fastest axis stays: gather its runs
        const long long L = d[k - 1];
        const bool vec = a16 && L % 4 == 0;
        const long long per_row = vec ? L / 4 : L;
        const long long runs = total / L;
        if (per_row * runs >= 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
        RowPlan p;
        // outer destination axes, padded at the slow end to three
        long long oe[3] = {1, 1, 1}, ot[3] = {0, 0, 0};
        for (int i = 0; i < k - 1; ++i) {
            oe[3 - (k - 1) + i] = e[i];
            ot[3 - (k - 1) + i] = ss[pm[i]];
        }
        p.t0 = ot[0]; p.t1 = ot[1]; p.t2 = ot[2];
        p.per_row = (uint32_t)per_row;
        p.items = (uint32_t)(per_row * runs);
        const FastDiv d_row = make_fastdiv((uint32_t)per_row), d_e2 = make_fastdiv((uint32_t)oe[2]),
                      d_e1 = make_fastdiv((uint32_t)oe[1]);
        const dim3 grid((unsigned)ceil_div64(p.items, kThreads)), block(kThreads);
        if (vec)
            hipLaunchKernelGGL((permute_rows_kernel<true>), grid, block, 0, st, src, dst, p, d_row, d_e2, d_e1);
        else
            hipLaunchKernelGGL((permute_rows_kernel<false>), grid, block, 0, st, src, dst, p, d_row, d_e2, d_e1);
        return launch_status();
    }

    // the fastest axis changes: tiles over (destination's fastest axis r, source's fastest axis s)
    const int ar = pm[k - 1];                       // source axis that is fastest in the destination
    int pos_s = 0;                                  // destination position of the source's fastest axis
    for (int i = 0; i < k; ++i)
        if (pm[i] == k - 1) pos_s = i;
    TilePlan p;
    p.R = d[ar];
    p.S = d[k - 1];
    p.ss_r = ss[ar];
    p.ds_s = ds[pos_s];
    long long nb[2] = {1, 1};
    p.sb0 = p.sb1 = p.db0 = p.db1 = 0;
    int nbatch = 0;
    for (int i = 0; i < k; ++i) {                   // remaining axes, in destination order
        if (i == k - 1 || i == pos_s) continue;
        if (nbatch == 0 && k == 4) { nb[0] = e[i]; p.sb0 = ss[pm[i]]; p.db0 = ds[i]; }
        else { nb[1] = e[i]; p.sb1 = ss[pm[i]]; p.db1 = ds[i]; }
        ++nbatch;
    }
    // every source stride is a multiple of S and every destination stride a multiple of R, so each side
    // can use 128-bit accesses on its own as soon as its fastest extent is a multiple of 4
    const bool vl = a16 && p.S % 4 == 0;
    const bool vs = a16 && p.R % 4 == 0;
    // tile shape: stretch along the longer side when the other is short
    if (p.R <= 16) return launch_tile<16, 256>(src, dst, p, nb[0], nb[1], vl, vs, st);
    if (p.R <= 32) return launch_tile<32, 128>(src, dst, p, nb[0], nb[1], vl, vs, st);
    if (p.S <= 16) return launch_tile<256, 16>(src, dst, p, nb[0], nb[1], vl, vs, st);
    if (p.S <= 32) return launch_tile<128, 32>(src, dst, p, nb[0], nb[1], vl, vs, st);
    return launch_tile<64, 64>(src, dst, p, nb[0], nb[1], vl, vs, st);
}

}  // namespace cnnmem
