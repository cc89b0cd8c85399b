// Max / average pooling computed directly in NCHW or CHWN (Equation 2 of
// Section II.A; Section IV.B on layouts; Section V.A on removing the redundant
// loads of overlapped windows).
//
// gfx950 design, by layout:
//   CHWN  -- N is contiguous, so a lane owns four consecutive images (one
//            float4) of one output column and walks down OY output rows.  Every
//            input row it touches is reduced horizontally once and that row
//            result is reused by all the output rows whose windows contain it
//            (the paper's register working set, applied along H); neighbouring
//            columns are neighbouring lanes, so their shared taps hit in L1.
//   NCHW  -- (n,c) planes are contiguous.  Instead of the strided
//            one-lane-per-output scheme the paper measures, a workgroup streams a
//            contiguous slab (several whole planes, or a strip of rows of a big
//            plane) into LDS with 128-bit loads, then every lane pools from LDS
//            and the outputs, contiguous as well, go out coalesced.  For the
//            non-overlapping 2x2/stride-2 case with even H no staging is needed:
//            rows pair up across the whole tensor and a lane turns 2 x 8 inputs
//            into 4 outputs with 128-bit accesses on both sides.
//   Anything else (odd alignment, N not a multiple of 4, huge extents) runs a
//   one-lane-per-output kernel that relies on the caches.
#include "common.hpp"

namespace cnnmem {
namespace {

constexpr int kThreads = 256;
constexpr float kNegInf = -__builtin_huge_valf();

template <int MODE>
struct Acc {
    static __device__ __forceinline__ float identity() { return MODE == CNNMEM_POOL_MAX ? kNegInf : 0.f; }
    static __device__ __forceinline__ float op(float a, float b) {
        return MODE == CNNMEM_POOL_MAX ? fmaxf(a, b) : a + b;
    }
    static __device__ __forceinline__ float4 identity4() {
        const float i = identity();
        return make_float4(i, i, i, i);
    }
    static __device__ __forceinline__ float4 op4(const float4& a, const float4& b) {
        return make_float4(op(a.x, b.x), op(a.y, b.y), op(a.z, b.z), op(a.w, b.w));
    }
    // Equation 2's division by the window area.  The compiler's correctly rounded fp32 division is about ten
    // instructions per output, which the padded NCHW kernels, bound by vector instruction issue, cannot afford.
    // The reciprocal is formed once (loop invariant; at compile time for the fixed windows) and one residual step on
    // the product gives the correctly rounded quotient again: q = a r, e = a - q d exactly by fma, q + e r.  The
    // fix-up instruction restores the quotient of infinities and NaNs.
    static __device__ __forceinline__ float finish(float a, float divisor) {
        if (MODE == CNNMEM_POOL_MAX) return a;
        const float r = 1.0f / divisor;
        float q = a * r;
        const float e = __builtin_fmaf(-q, divisor, a);
        q = __builtin_fmaf(e, r, q);
        return __builtin_amdgcn_div_fixupf(q, divisor, a);
    }
    static __device__ __forceinline__ float4 finish4(const float4& a, float divisor) {
        return make_float4(finish(a.x, divisor), finish(a.y, divisor), finish(a.z, divisor),
                           finish(a.w, divisor));
    }
};

// ---------------------------------------------------------------------------
// Fallback: one lane per output element, any layout through strides.
// ---------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(kThreads) void pool_generic_kernel(
    const float* __restrict__ src, float* __restrict__ dst, PoolGeom g, int chwn, size_t total) {
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t o = (size_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += stride) {
        // decode the output index in its own layout
        int n, c, i, j;
        size_t t = o;
        if (chwn) {
            n = (int)(t % g.N); t /= g.N;
            j = (int)(t % g.Wo); t /= g.Wo;
            i = (int)(t % g.Ho); c = (int)(t / g.Ho);
        } else {
            j = (int)(t % g.Wo); t /= g.Wo;
            i = (int)(t % g.Ho); t /= g.Ho;
            c = (int)(t % g.C); n = (int)(t / g.C);
        }
        float acc = Acc<MODE>::identity();
        for (int y = 0; y < g.kh; ++y) {
            const int r = i * g.sh - g.ph + y;
            if (r < 0 || r >= g.H) continue;
            for (int x = 0; x < g.kw; ++x) {
                const int q = j * g.sw - g.pw + x;
                if (q < 0 || q >= g.W) continue;
                const size_t idx = chwn ? (((size_t)c * g.H + r) * g.W + q) * g.N + n
                                        : (((size_t)n * g.C + c) * g.H + r) * g.W + q;
                acc = Acc<MODE>::op(acc, src[idx]);
            }
        }
        dst[o] = Acc<MODE>::finish(acc, (float)(g.kh * g.kw));
    }
}

// ---------------------------------------------------------------------------
// CHWN: float4 over four images; a lane owns an OY x OX block of outputs (the
// per-thread working set of Section V.A, expanded in both directions).  Every
// input tap the block needs is loaded once; each input row is reduced
// horizontally once per output column and that row result is reused by all
// output rows whose windows contain it.  KH/KW/SH/SW are compile-time so the
// window loops unroll into registers.
// ---------------------------------------------------------------------------
template <int MODE, int KH, int KW, int SH, int SW, int OY, int OX, bool PADDED>
__global__ __launch_bounds__(kThreads) void pool_chwn_vec4_kernel(
    const float* __restrict__ src, float* __restrict__ dst, PoolGeom g, uint32_t row_items,
    uint32_t blocks_x, uint32_t blocks_y, FastDiv div_n4, uint32_t flat_items, FastDiv div_row_items,
    FastDiv div_blocks_y) {
    constexpr int ROWS_IN = (OY - 1) * SH + KH;     // input rows one lane walks
    constexpr int COLS_IN = (OX - 1) * SW + KW;     // input columns it touches in each of them
    const uint32_t nblocks = gridDim.x;
    const uint32_t tile = xcd_contiguous_tile(blockIdx.x, nblocks);
    uint32_t u, by, c;                              // position in the output row (jb*N4 + n4), strip, feature map
    if (flat_items) {
        // short rows: lanes are dealt over (c, strip, position) without padding every row to a
        // whole workgroup (13 columns x 32 float4 fill 1.6 workgroups)
        const uint32_t f = tile * kThreads + threadIdx.x;
        if (f >= flat_items) return;
        const uint32_t rest = fd_div(f, div_row_items);
        u = f - rest * row_items;
        c = fd_div(rest, div_blocks_y);
        by = rest - c * blocks_y;
    } else {
        // tile -> (bx fastest, then by, then c): vertically adjacent strips are close in tile order
        const uint32_t bx = tile % blocks_x;
        const uint32_t rest = tile / blocks_x;
        by = rest % blocks_y;
        c = rest / blocks_y;
        u = bx * kThreads + threadIdx.x;
        if (u >= row_items) return;
    }
    const uint32_t jb = fd_div(u, div_n4);
    const uint32_t n4 = u - jb * div_n4.d;
    const int j0 = (int)jb * OX;
    const int i0 = (int)by * OY;
    const int N = g.N;

    float4 acc[OY][OX];
#pragma unroll
    for (int oy = 0; oy < OY; ++oy)
#pragma unroll
        for (int ox = 0; ox < OX; ++ox) acc[oy][ox] = Acc<MODE>::identity4();

    const int q0 = j0 * SW - g.pw;
    const int r_base = i0 * SH - g.ph;
    const float* plane = src + (size_t)c * g.H * g.W * N + 4 * n4;
    // Overlapping windows re-read taps that a neighbouring lane or strip has just
    // fetched, so those loads stay cacheable; disjoint windows stream.
    constexpr bool kStream = (KH <= SH) && (KW <= SW);
    // Every load is unconditional (a branch per row would make the compiler wait
    // for each row before asking for the next): taps outside the image are read
    // from a clamped, valid address.  Without padding
    // the only rows past H and columns past W belong to outputs beyond Ho x Wo,
    // which are never stored, so clamping alone is enough there.
#pragma unroll
    for (int rr = 0; rr < ROWS_IN; ++rr) {
        const int r = r_base + rr;
        const bool row_ok = !PADDED || (r >= 0 && r < g.H);
        const int rc = r < 0 ? 0 : (r < g.H ? r : g.H - 1);
        const float* rowp = plane + (size_t)rc * g.W * N;
        float4 h[OX];
#pragma unroll
        for (int ox = 0; ox < OX; ++ox) h[ox] = Acc<MODE>::identity4();
#pragma unroll
        for (int x = 0; x < COLS_IN; ++x) {
            const int q = q0 + x;
            const bool ok = row_ok && (!PADDED || (q >= 0 && q < g.W));
            const int qc = q < 0 ? 0 : (q < g.W ? q : g.W - 1);
            float4 t = kStream ? ld4_stream(rowp + (size_t)qc * N)
                               : *reinterpret_cast<const float4*>(rowp + (size_t)qc * N);
            // A tap in the padding was read from the nearest in-image position, which lies in every window
            // that holds the tap: the maximum needs nothing more.  The average clears it with a bit mask,
            // not with `if (!ok) t = 0`: the compiler turns that into a branch around the load and waits for
            // each load before issuing the next (3x3/s2/p1 had 53 branches and one load in flight).
            if (PADDED && MODE != CNNMEM_POOL_MAX) {
                const uint32_t keep = ok ? 0xffffffffu : 0u;
                t.x = __uint_as_float(__float_as_uint(t.x) & keep);
                t.y = __uint_as_float(__float_as_uint(t.y) & keep);
                t.z = __uint_as_float(__float_as_uint(t.z) & keep);
                t.w = __uint_as_float(__float_as_uint(t.w) & keep);
            }
#pragma unroll
            for (int ox = 0; ox < OX; ++ox)
                if (x >= ox * SW && x < ox * SW + KW) h[ox] = Acc<MODE>::op4(h[ox], t);
        }
#pragma unroll
        for (int oy = 0; oy < OY; ++oy)
            if (rr >= oy * SH && rr < oy * SH + KH) {
#pragma unroll
                for (int ox = 0; ox < OX; ++ox) acc[oy][ox] = Acc<MODE>::op4(acc[oy][ox], h[ox]);
            }
    }
    float* outp = dst + ((size_t)c * g.Ho * g.Wo + j0) * N + 4 * n4;
#pragma unroll
    for (int oy = 0; oy < OY; ++oy) {
        const int i = i0 + oy;
#pragma unroll
        for (int ox = 0; ox < OX; ++ox)
            if (i < g.Ho && j0 + ox < g.Wo)
                st4_through(outp + ((size_t)i * g.Wo + ox) * N, Acc<MODE>::finish4(acc[oy][ox], (float)(KH * KW)));
    }
}

// ---------------------------------------------------------------------------
// CHWN, any window: float4 over four images, the window walked with run-time loops
// (global 7x7 pooling, 5x5 / stride 3, rectangular windows ...).
// ---------------------------------------------------------------------------
// OY vertically adjacent outputs per lane: each input row under them is read and reduced along W once and
// serves every output whose window holds it.  With one output per lane the rows that two windows share were
// fetched from HBM twice (counters: 1.75x the tensor for 5x5 / stride 3): the workgroups of neighbouring
// output rows run at the same time, but each streams 64 KB and the shared rows have left L2 by the time the
// neighbour asks for them.
template <int MODE, int OY>
__global__ __launch_bounds__(kThreads) void pool_chwn_vec4_any_kernel(
    const float* __restrict__ src, float* __restrict__ dst, PoolGeom g, uint32_t items, FastDiv div_n4, FastDiv div_wo,
    FastDiv div_hb) {
    // neighbouring workgroups run on one XCD, so columns that neighbouring lanes' windows share are L2 hits
    const uint32_t u = xcd_contiguous_tile(blockIdx.x, gridDim.x) * kThreads + threadIdx.x;   // ((c*HB + ib)*Wo + j)*N4 + n4
    if (u >= items) return;
    uint32_t t = fd_div(u, div_n4);
    const uint32_t n4 = u - t * div_n4.d;
    uint32_t t2 = fd_div(t, div_wo);
    const int j = (int)(t - t2 * div_wo.d);
    const uint32_t c = fd_div(t2, div_hb);
    const int i0 = (int)(t2 - c * div_hb.d) * OY;              // first output row of the lane
    const int N = g.N;
    int q_lo = j * g.sw - g.pw, q_hi = q_lo + g.kw;
    if (q_lo < 0) q_lo = 0;
    if (q_hi > g.W) q_hi = g.W;
    const int i_last = i0 + OY - 1 < g.Ho - 1 ? i0 + OY - 1 : g.Ho - 1;
    int r_lo = i0 * g.sh - g.ph, r_hi = i_last * g.sh - g.ph + g.kh;
    if (r_lo < 0) r_lo = 0;
    if (r_hi > g.H) r_hi = g.H;
    const float* plane = src + (size_t)c * g.H * g.W * N + 4 * n4;
    float4 acc[OY];
#pragma unroll
    for (int k = 0; k < OY; ++k) acc[k] = Acc<MODE>::identity4();
    for (int r = r_lo; r < r_hi; ++r) {
        const float* rowp = plane + (size_t)r * g.W * N;
        float4 h = Acc<MODE>::identity4();
#pragma unroll 4
        for (int q = q_lo; q < q_hi; ++q)
            h = Acc<MODE>::op4(h, *reinterpret_cast<const float4*>(rowp + (size_t)q * N));
#pragma unroll
        for (int k = 0; k < OY; ++k) {
            const int top = (i0 + k) * g.sh - g.ph;            // first row of output k's window
            if (OY == 1 || (r >= top && r < top + g.kh)) acc[k] = Acc<MODE>::op4(acc[k], h);
        }
    }
    float* out = dst + (((size_t)c * g.Ho + i0) * g.Wo + j) * N + 4 * n4;
#pragma unroll
    for (int k = 0; k < OY; ++k)
        if (i0 + k < g.Ho) st4_stream(out + (size_t)k * g.Wo * N, Acc<MODE>::finish4(acc[k], (float)(g.kh * g.kw)));
}

// The same kernel for tensors with few outputs and large windows (global 7x7 pooling of 128x2048x7x7 has
// 65536 float4 outputs: one wavefront per SIMD, each walking 49 taps one after the other).  The rows of a
// window are dealt over P lanes (row r_lo + part, + P, ...), which puts P times as many loads in flight, and
// the P partial results meet in LDS.  A workgroup is P parts x 256/P outputs; part 0 stores.
template <int MODE, int P>
__global__ __launch_bounds__(kThreads) void pool_chwn_vec4_split_kernel(
    const float* __restrict__ src, float* __restrict__ dst, PoolGeom g, uint32_t items, FastDiv div_n4, FastDiv div_wo,
    FastDiv div_ho) {
    constexpr int PER = kThreads / P;                           // outputs (float4) per workgroup
    __shared__ float4 part_acc[P][PER];
    const int part = threadIdx.x / PER, slot = threadIdx.x % PER;
    const uint32_t u = blockIdx.x * PER + slot;                 // ((c*Ho + i)*Wo + j)*N4 + n4
    const bool live = u < items;
    float4 acc = Acc<MODE>::identity4();
    if (live) {
        const uint32_t t = fd_div(u, div_n4);
        const uint32_t n4 = u - t * div_n4.d;
        const uint32_t t2 = fd_div(t, div_wo);
        const int j = (int)(t - t2 * div_wo.d);
        const uint32_t c = fd_div(t2, div_ho);
        const int i = (int)(t2 - c * div_ho.d);
        const int N = g.N;
        int q_lo = j * g.sw - g.pw, q_hi = q_lo + g.kw;
        if (q_lo < 0) q_lo = 0;
        if (q_hi > g.W) q_hi = g.W;
        int r_lo = i * g.sh - g.ph, r_hi = r_lo + g.kh;
        if (r_lo < 0) r_lo = 0;
        if (r_hi > g.H) r_hi = g.H;
        const float* plane = src + (size_t)c * g.H * g.W * N + 4 * n4;
        for (int r = r_lo + part; r < r_hi; r += P) {
            const float* rowp = plane + (size_t)r * g.W * N;
            int q = q_lo;
            for (; q + 4 <= q_hi; q += 4) {                     // four loads in flight before the first is used
                const float4 v0 = *reinterpret_cast<const float4*>(rowp + (size_t)q * N),
                             v1 = *reinterpret_cast<const float4*>(rowp + (size_t)(q + 1) * N),
                             v2 = *reinterpret_cast<const float4*>(rowp + (size_t)(q + 2) * N),
                             v3 = *reinterpret_cast<const float4*>(rowp + (size_t)(q + 3) * N);
                acc = Acc<MODE>::op4(Acc<MODE>::op4(acc, v0), Acc<MODE>::op4(Acc<MODE>::op4(v1, v2), v3));
            }
            if (q + 2 <= q_hi) {
                const float4 v0 = *reinterpret_cast<const float4*>(rowp + (size_t)q * N),
                             v1 = *reinterpret_cast<const float4*>(rowp + (size_t)(q + 1) * N);
                acc = Acc<MODE>::op4(acc, Acc<MODE>::op4(v0, v1));
                q += 2;
            }
            if (q < q_hi) acc = Acc<MODE>::op4(acc, *reinterpret_cast<const float4*>(rowp + (size_t)q * N));
        }
    }
    part_acc[part][slot] = acc;
    __syncthreads();
    if (part == 0 && live) {
#pragma unroll
        for (int k = 1; k < P; ++k) acc = Acc<MODE>::op4(acc, part_acc[k][slot]);
        st4_stream(dst + 4 * (size_t)u, Acc<MODE>::finish4(acc, (float)(g.kh * g.kw)));
    }
}

// ---------------------------------------------------------------------------
// NCHW, 2x2 window, stride 2, no padding, even H: the tensor is a list of
// N*C*H rows of W floats and output row k is made of input rows 2k and 2k+1.
// A lane reads one float4 of both rows and writes two outputs: a wavefront's
// load is one contiguous 1 KB run (two float4 per row per lane, 32 B apart
// between lanes, measured 60 % against 76 % on 64x256x56x56).
// ---------------------------------------------------------------------------
template <int MODE>
__global__ __launch_bounds__(kThreads) void pool_nchw_2x2s2_kernel(
    const float* __restrict__ src, float* __restrict__ dst, uint32_t items, uint32_t W,
    FastDiv div_per_row) {
    // item I: output floats [2I, 2I + 2); output row = I / (W/4).  Rows that are not whole 128-byte lines
    // (W = 112, 56, 28) leave lines shared between neighbouring workgroups: with neighbours on one XCD the
    // second request for such a line is an L2 hit (counters: 1.022-1.030x the tensor fetched before, W = 224: 1.000x).
    const uint32_t I = xcd_contiguous_tile(blockIdx.x, gridDim.x) * kThreads + threadIdx.x;
    if (I >= items) return;
    const uint32_t orow = fd_div(I, div_per_row);
    const size_t in0 = (size_t)I * 4 + (size_t)orow * W;       // = 2*orow*W + 4*(I % per_row)
    const float4 a = ld4_stream(src + in0), b = ld4_stream(src + in0 + W);
    float o0, o1;
    if (MODE == CNNMEM_POOL_MAX) {
        o0 = fmaxf(fmaxf(a.x, a.y), fmaxf(b.x, b.y));
        o1 = fmaxf(fmaxf(a.z, a.w), fmaxf(b.z, b.w));
    } else {
        o0 = ((a.x + a.y) + (b.x + b.y)) * 0.25f;
        o1 = ((a.z + a.w) + (b.z + b.w)) * 0.25f;
    }
    st2_through(dst + (size_t)I * 2, o0, o1);
}

// ---------------------------------------------------------------------------
// NCHW through LDS.  One workgroup = `planes` consecutive (n,c) planes (all
// their rows) or one strip of `rows_out` output rows of a single plane.
// ---------------------------------------------------------------------------
constexpr int kSlabFloats = 8192;                   // 32 KB of LDS per workgroup

struct SlabPlan {
    int planes_per_wg;      // >= 1 (whole planes) ...
    int rows_per_wg;        // ... or output rows per strip when a plane is split
    int strips;             // strips per plane (1 when whole planes)
    long long total_planes;
};

// OY > 1 (compile-time windows only): a lane owns OY vertically adjacent outputs.  Each of the (OY-1)*SH + KH input
// rows they touch is reduced along W once and that row result serves every output whose window holds the row (the
// CHWN kernel's reuse, taken from LDS here); lanes stay adjacent along W, so the LDS reads stay conflict-free.
// div_blk divides by the number of row blocks per plane, ceil(rows_out / OY).
template <int MODE, int KH, int KW, int SH, int SW, int OY, bool PADDED, int THREADS>
__global__ __launch_bounds__(THREADS) void pool_nchw_slab_kernel(
    const float* __restrict__ src, float* __restrict__ dst, PoolGeom g, SlabPlan plan,
    FastDiv div_wo, FastDiv div_plane_out, FastDiv div_blk, int rt_kh, int rt_kw, int rt_sh, int rt_sw) {
    constexpr int kSlabThreads = THREADS;
    constexpr int kSlabVecPerLane = kSlabFloats / 4 / THREADS + 1;   // float4 per lane, worst case
    __shared__ __attribute__((aligned(16))) float slab[kSlabFloats + 8];
    const int kh = KH ? KH : rt_kh, kw = KW ? KW : rt_kw;
    const int sh = SH ? SH : rt_sh, sw = SW ? SW : rt_sw;

    const uint32_t tile = xcd_contiguous_tile(blockIdx.x, gridDim.x);
    const int plane_in = g.H * g.W;
    const int plane_out = g.Ho * g.Wo;

    long long p0;
    int planes, i0, rows_out;
    if (plan.strips == 1) {
        p0 = (long long)tile * plan.planes_per_wg;
        const long long left = plan.total_planes - p0;
        planes = left < plan.planes_per_wg ? (int)left : plan.planes_per_wg;
        i0 = 0;
        rows_out = g.Ho;
    } else {
        p0 = tile / (uint32_t)plan.strips;
        const int strip = (int)(tile % (uint32_t)plan.strips);
        planes = 1;
        i0 = strip * plan.rows_per_wg;
        rows_out = g.Ho - i0 < plan.rows_per_wg ? g.Ho - i0 : plan.rows_per_wg;
    }
    // input rows this workgroup needs: [r_lo, r_hi) of its first ... last plane
    int r_lo = i0 * sh - g.ph;
    if (r_lo < 0) r_lo = 0;
    int r_hi = (i0 + rows_out - 1) * sh - g.ph + kh;
    if (r_hi > g.H) r_hi = g.H;
    if (planes > 1) { r_lo = 0; r_hi = g.H; }
    const size_t g_lo = (size_t)p0 * plane_in + (size_t)r_lo * g.W;
    const size_t g_hi = (size_t)(p0 + planes - 1) * plane_in + (size_t)r_hi * g.W;
    // The float4 stream starts on a 128-byte line of src when src itself is line
    // aligned (always at least on a float4): wavefronts then fetch whole lines.
    const size_t in_mask = (reinterpret_cast<uintptr_t>(src) & 127u) == 0 ? 31 : 3;
    const size_t a_lo = g_lo & ~in_mask;
    const size_t total_in = (size_t)plan.total_planes * plane_in;
    const int nvec = (int)((g_hi - a_lo + 3) >> 2);

    // ---- load phase: issue every 128-bit load, then park them in LDS ----
    // All loads are unconditional so that they are in flight together: lanes past
    // the slab, and the one float4 in the whole tensor that would cross its end,
    // re-read the last complete float4 instead (total_in >= 4 is a dispatch
    // condition) and simply do not park it.  The up to three floats of a ragged
    // tensor end are then fetched one by one by the lane that owns them.
    const size_t a_last = (total_in - 4) & ~(size_t)3;
    // (a round wholly past the slab is skipped by the whole workgroup: small planes leave most rounds empty)
    float4 v[kSlabVecPerLane];
    if (a_lo + 4 * (size_t)(nvec - 1) <= a_last) {
        // Every workgroup but the one at the tensor's end: no float4 of the slab can cross the end, so the
        // lane's address is a uniform base plus a 32-bit offset and needs no 64-bit clamp (the 64-bit
        // compares and selects of the general form below were a third of the kernel's vector instructions).
        const float* sbase = src + a_lo;
#pragma unroll
        for (int k = 0; k < kSlabVecPerLane; ++k) {
            if (k * kSlabThreads >= nvec) break;
            const uint32_t q = threadIdx.x + k * kSlabThreads;
            v[k] = ld4_stream(sbase + 4u * (q < (uint32_t)nvec ? q : 0u));
        }
#pragma unroll
        for (int k = 0; k < kSlabVecPerLane; ++k) {
            if (k * kSlabThreads >= nvec) break;
            const uint32_t q = threadIdx.x + k * kSlabThreads;
            if (q < (uint32_t)nvec) *reinterpret_cast<float4*>(slab + 4 * q) = v[k];
        }
    } else {
#pragma unroll
        for (int k = 0; k < kSlabVecPerLane; ++k) {
            if (k * kSlabThreads >= nvec) break;
            const int q = threadIdx.x + k * kSlabThreads;
            size_t a = a_lo + 4 * (size_t)(q < nvec ? q : 0);
            a = a <= a_last ? a : a_last;
            v[k] = ld4_stream(src + a);
        }
#pragma unroll
        for (int k = 0; k < kSlabVecPerLane; ++k) {
            if (k * kSlabThreads >= nvec) break;
            const int q = threadIdx.x + k * kSlabThreads;
            const size_t a = a_lo + 4 * (size_t)q;
            if (q < nvec && a <= a_last) *reinterpret_cast<float4*>(slab + 4 * q) = v[k];
        }
        for (int k = 0; k < kSlabVecPerLane; ++k) {
            const int q = threadIdx.x + k * kSlabThreads;
            const size_t a = a_lo + 4 * (size_t)q;
            if (q < nvec && a > a_last) {           // ragged end of the tensor (at most one lane, once)
                for (int j = 0; j < 4; ++j)
                    if (a + j < total_in) slab[4 * q + j] = src[a + j];
            }
        }
    }
    __syncthreads();

    // ---- pool from LDS; outputs of the workgroup are contiguous in dst ----
    // Everything below indexes the workgroup's own slab and outputs: numbers below 2^20, divided in three
    // instructions (sd_div) and multiplied at full rate (24-bit multiply); the padded kernels are bound by the
    // issue of vector instructions, and 32-bit multiplies issue at a quarter of the rate.
    const SmallDiv sd_wo = make_smalldiv(div_wo.d), sd_plane_out = make_smalldiv(div_plane_out.d),
                   sd_blk = make_smalldiv(div_blk.d);
    const int n_out = planes * rows_out * g.Wo;     // planes > 1 implies rows_out == Ho
    const size_t out0 = (size_t)p0 * plane_out + (size_t)i0 * g.Wo;
    // LDS index of element (plane p0, row 0, col 0); may be negative when r_lo > 0
    const int lds0 = (int)((long long)((size_t)p0 * plane_in) - (long long)a_lo);
    // Lane -> output assignment is shifted so that every wavefront's 256-byte
    // store starts on a 128-byte line of dst (no line is written in two pieces).
    if constexpr (OY > 1 && KH != 0) {
        constexpr int ROWS = (OY - 1) * SH + KH;
        constexpr int MAXIT = 4;                     // blocks of OY outputs a lane may hold in registers
        const int nblk = (int)div_blk.d;             // row blocks per plane
        const int n_items = planes * nblk * g.Wo;
        const int r_last = r_hi - 1;                 // rows of the slab: [r_lo, r_hi)
        // Results stay in registers until every lane has finished reading the slab, are then parked in the slab
        // in output order, and leave as one contiguous run of line-aligned wavefront stores.  Stored straight
        // from the lanes, OY row pieces per wavefront, the outputs cost 1.15x their bytes in write traffic
        // (counters, 3x3/s1/p1 on 64x256x56x56) and the kernel 57 % of peak (68 % staged; the average 56 -> 62 %).
        // Stride 1 only: with two rows per lane at stride 2 the staging costs more than the 9 % of extra write
        // traffic it removes (3x3/s2/p1 average on 256x64x112x112: 71 % of peak direct, 68 % staged).
        const bool staged = SH == 1 && n_items <= MAXIT * kSlabThreads && n_out <= kSlabFloats;
        float res[MAXIT][OY];
#pragma unroll
        for (int round = 0; round < MAXIT; ++round) {
            for (int it = (int)threadIdx.x + round * kSlabThreads; it < n_items;
                 it += staged ? n_items : kSlabThreads) {          // staged: one block per round
                const int pb = (int)sd_div((uint32_t)it, sd_wo);      // plane * nblk + block
                const int j = it - __mul24(pb, g.Wo);
                const int pl = (int)sd_div((uint32_t)pb, sd_blk);
                const int blk = pb - __mul24(pl, nblk);
                const int il0 = blk * OY;                               // first output row of the lane, strip-local
                const int rb = (i0 + il0) * SH - g.ph;
                const int qb = j * SW - g.pw;
                const int base = lds0 + __mul24(pl, plane_in);
                // Rows and columns are clamped into the slab: a clamped tap of a real output lies in the same
                // window (so the maximum is unchanged; the average drops it by a select), and the rows of outputs
                // past the strip's end only feed results that are never stored.
                int qc[KW];
                bool q_in[KW];
#pragma unroll
                for (int x = 0; x < KW; ++x) {
                    const int q = qb + x;
                    q_in[x] = !PADDED || (q >= 0 && q < g.W);
                    qc[x] = !PADDED ? q : (q < 0 ? 0 : (q < g.W ? q : g.W - 1));
                }
                float hr[ROWS];
#pragma unroll
                for (int y = 0; y < ROWS; ++y) {
                    const int r = rb + y;
                    int rc = r < r_last ? r : r_last;
                    if (PADDED) rc = rc > r_lo ? rc : r_lo;
                    const float* row = slab + base + __mul24(rc, g.W);
                    float acc = Acc<MODE>::identity();
#pragma unroll
                    for (int x = 0; x < KW; ++x) {
                        const float v = row[qc[x]];
                        if (MODE == CNNMEM_POOL_MAX) acc = fmaxf(acc, v);
                        else acc += q_in[x] ? v : 0.f;
                    }
                    if (MODE != CNNMEM_POOL_MAX && PADDED && (r < 0 || r >= g.H)) acc = 0.f;
                    hr[y] = acc;
                }
#pragma unroll
                for (int k = 0; k < OY; ++k) {
                    float acc = hr[k * SH];
#pragma unroll
                    for (int y = 1; y < KH; ++y) acc = Acc<MODE>::op(acc, hr[k * SH + y]);
                    res[round][k] = Acc<MODE>::finish(acc, (float)(KH * KW));
                }
                if (!staged) {
                    float* out = dst + out0 + (size_t)(__mul24(__mul24(pl, rows_out) + il0, g.Wo) + j);
#pragma unroll
                    for (int k = 0; k < OY; ++k)
                        if (il0 + k < rows_out) st1_stream(out + __mul24(k, g.Wo), res[round][k]);
                }
            }
            if (!staged) return;                     // the unstaged walk did every block in its first round
        }
        __syncthreads();                             // every tap has been read: the slab can take the results
#pragma unroll
        for (int round = 0; round < MAXIT; ++round) {
            const int it = (int)threadIdx.x + round * kSlabThreads;
            if (it < n_items) {
                const int pb = (int)sd_div((uint32_t)it, sd_wo);
                const int j = it - __mul24(pb, g.Wo);
                const int pl = (int)sd_div((uint32_t)pb, sd_blk);
                const int il0 = (pb - __mul24(pl, nblk)) * OY;
#pragma unroll
                for (int k = 0; k < OY; ++k)
                    if (il0 + k < rows_out) slab[__mul24(__mul24(pl, rows_out) + il0 + k, g.Wo) + j] = res[round][k];
            }
        }
        __syncthreads();
        const int lead_s = (int)(((reinterpret_cast<uintptr_t>(dst) >> 2) + out0) & 31);
        for (int o = (int)threadIdx.x - lead_s; o < n_out; o += kSlabThreads)
            if (o >= 0) st1_stream(dst + out0 + o, slab[o]);
        return;
    }
    const int lead = (int)(((reinterpret_cast<uintptr_t>(dst) >> 2) + out0) & 31);
    for (int o = (int)threadIdx.x - lead; o < n_out; o += kSlabThreads) {
        if (o < 0) continue;
        int pl = 0, rem = o;
        if (planes > 1) {
            pl = (int)sd_div((uint32_t)o, sd_plane_out);
            rem = o - __mul24(pl, plane_out);
        }
        const int il = (int)sd_div((uint32_t)rem, sd_wo);
        const int j = rem - __mul24(il, g.Wo);
        const int rb = (i0 + il) * sh - g.ph;
        const int qb = j * sw - g.pw;
        const int base = lds0 + __mul24(pl, plane_in);     // LDS index of this plane's element (0, 0)
        float acc = Acc<MODE>::identity();
        if (KH != 0) {
            // With padding, a tap outside the image is read from the nearest in-image position, which
            // lies in the same window (every window keeps a tap): the maximum does not change, the
            // average drops it by a select.  No branches either way.
#pragma unroll
            for (int y = 0; y < (KH ? KH : 1); ++y) {
                const int r = rb + y;
                const bool r_in = !PADDED || (r >= 0 && r < g.H);
                const int rc = !PADDED ? r : (r < 0 ? 0 : (r < g.H ? r : g.H - 1));
#pragma unroll
                for (int x = 0; x < (KW ? KW : 1); ++x) {
                    const int q = qb + x;
                    const bool in = r_in && (!PADDED || (q >= 0 && q < g.W));
                    const int qc = !PADDED ? q : (q < 0 ? 0 : (q < g.W ? q : g.W - 1));
                    const float v = slab[base + __mul24(rc, g.W) + qc];
                    if (MODE == CNNMEM_POOL_MAX) acc = fmaxf(acc, v);
                    else acc += in ? v : 0.f;
                }
            }
        } else {
            // run-time window: the in-image part of the window, loop bounds clipped once, no test or
            // select per tap (5x5/s3/p2 on 64x64x150x150: average 49 -> 60 % of peak against skipping
            // taps one by one)
            const int r_lo = rb < 0 ? 0 : rb, r_hi = rb + kh < g.H ? rb + kh : g.H;
            const int q_lo = qb < 0 ? 0 : qb, q_hi = qb + kw < g.W ? qb + kw : g.W;
            for (int r = r_lo; r < r_hi; ++r) {
                const int row = base + __mul24(r, g.W);
#pragma unroll 4
                for (int q = q_lo; q < q_hi; ++q) acc = Acc<MODE>::op(acc, slab[row + q]);
            }
        }
        st1_stream(dst + out0 + o, Acc<MODE>::finish(acc, (float)(kh * kw)));
    }
}

// ---- NCHW, 3x3 / stride 2 without padding (the overlapped pooling of the paper's networks): rows kernel -----
// The lanes of a wavefront are the output columns of one output row (of 64 / LW rows for planes of fewer than 33
// output columns, LW the next power of two); what depends on the row - where its three input rows and its
// result sit in LDS - is computed once per workgroup into a table of descriptors, so the inner loop is a
// descriptor read, nine taps and eight operations.  The input rows are requested before the table is built;
// results are staged in LDS and leave as one line-aligned run.
// LDS: [ input rows | staged outputs | trash row | descriptors ]
constexpr int kRowThreads = 256;
constexpr int kRowXVecs = 8;                        // float4 per lane a workgroup's input rows may take
constexpr int kRowLdsFloats = 15360;
struct PoolRowsLds {
    int stage_at, trash_at, desc_at;
    int ntab;                   // descriptors: output rows, whole rounds of the workgroup
    int lanes_per_row;          // LW
};
extern __shared__ float4 pool_dyn_lds[];

template <int MODE>
__global__ __launch_bounds__(kRowThreads) void pool_nchw_k3s2_rows_kernel(
    const float* __restrict__ src, float* __restrict__ dst, PoolGeom g, SlabPlan plan, PoolRowsLds at, FastDiv div_ho) {
    constexpr int THREADS = kRowThreads, kWaves = THREADS / 64, XV = kRowXVecs;
    float* slab = reinterpret_cast<float*>(pool_dyn_lds);
    const int W = g.W, Ho = g.Ho, Wo = g.Wo;
    const int plane_in = g.H * W, plane_out = Ho * Wo;
    const uint32_t total_planes = (uint32_t)plan.total_planes;         // the tensors have fewer than 2^31 elements (launcher)
    const uint32_t tile = xcd_contiguous_tile(blockIdx.x, gridDim.x);
    // whole planes per workgroup (planes that do not fit stay with the slab kernel, whose strips of output rows
    // measured 15 % faster than strips here: 64x96x110x110 60.7 against 71.5 us)
    const uint32_t p0 = tile * (uint32_t)plan.planes_per_wg;
    const uint32_t left = total_planes - p0;
    const int planes = left < (uint32_t)plan.planes_per_wg ? (int)left : plan.planes_per_wg;
    const int n_out = planes * plane_out;
    const uint32_t out0 = p0 * (uint32_t)plane_out;
    const int lead = (int)((((uint32_t)reinterpret_cast<uintptr_t>(dst) >> 2) + out0) & 31u);
    const int stage_at = at.stage_at + (lead & 3);
    int4* desc = reinterpret_cast<int4*>(slab + at.desc_at);

    // ---- input rows on their way (element e lands at slab[e - a_lo], a_lo the line-aligned start) ----
    const uint32_t total_in = total_planes * (uint32_t)plane_in;
    const uint32_t x_lo = p0 * (uint32_t)plane_in;
    const uint32_t x_hi = (p0 + planes) * (uint32_t)plane_in;
    const uint32_t a_lo = x_lo & ~((reinterpret_cast<uintptr_t>(src) & 127u) == 0 ? 31u : 3u);
    const uint32_t nvec = (x_hi - a_lo + 3) >> 2, a_last = (total_in - 4) & ~3u;
    float4 xv[XV];
#pragma unroll
    for (int k = 0; k < XV; ++k) {
        if ((uint32_t)(k * THREADS) >= nvec) break;              // uniform
        const uint32_t q = threadIdx.x + k * THREADS;
        const uint32_t a = a_lo + 4 * (q < nvec ? q : nvec - 1);
        xv[k] = ld4_stream(src + (a <= a_last ? a : a_last));
    }
    // ---- descriptors while the loads are in flight: { first input row of the window row, staged output row } ----
    const int x_base = (int)(p0 * (uint32_t)plane_in - a_lo);                  // slab index of (plane p0, row 0, col 0)
    const int n_rows = planes * Ho;
    for (int t = threadIdx.x; t < at.ntab; t += THREADS) {
        const bool valid = t < n_rows;
        const int tv = valid ? t : 0;
        const int pl = (int)fd_div((uint32_t)tv, div_ho);
        const int i = tv - pl * Ho;
        int4 d;
        d.x = x_base + pl * plane_in + 2 * i * W;
        d.y = valid ? stage_at + tv * Wo : at.trash_at;
        d.z = 0; d.w = 0;
        desc[t] = d;
    }
#pragma unroll
    for (int k = 0; k < XV; ++k) {
        if ((uint32_t)(k * THREADS) >= nvec) break;
        const uint32_t q = threadIdx.x + k * THREADS;
        const uint32_t a = a_lo + 4 * q;
        if (q < nvec) {
            if (a <= a_last) *reinterpret_cast<float4*>(slab + 4 * q) = xv[k];
            else
                for (uint32_t e = 0; e < 4; ++e)
                    if (a + e < total_in) slab[4 * q + e] = src[a + e];
        }
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int LW = at.lanes_per_row;
    const int SUB = 64 / LW, sub = lane / LW, step = kWaves * SUB;
    for (int j = lane & (LW - 1); j < ((Wo + 63) & ~63); j += 64) {
        if (j < Wo) {
            for (int base = wave * SUB; base < at.ntab; base += step) {
                const int4 d = desc[base + sub];
                const float* xp = slab + d.x + 2 * j;
                float acc = Acc<MODE>::identity();
#pragma unroll
                for (int y = 0; y < 3; ++y)
#pragma unroll
                    for (int x = 0; x < 3; ++x) acc = Acc<MODE>::op(acc, xp[y * W + x]);
                slab[d.y + j] = Acc<MODE>::finish(acc, 9.0f);
            }
        }
    }
    __syncthreads();
    // the workgroup's outputs leave as one contiguous run, 128 bits per lane, each wavefront's 1 KB starting on a
    // line of dst
    const float* stage = slab + stage_at;
    for (int o = 4 * (int)threadIdx.x - lead; o < n_out; o += 4 * THREADS) {
        float* q = dst + out0 + o;
        if (o >= 0 && o + 4 <= n_out) {
            st4_stream(q, *reinterpret_cast<const float4*>(stage + o));
        } else {
            for (int e = 0; e < 4; ++e)
                if (o + e >= 0 && o + e < n_out) q[e] = stage[o + e];
        }
    }
}

template <int MODE>
int launch_nchw_k3s2_rows(const float* src, float* dst, const PoolGeom& g, hipStream_t st) {
    constexpr int kWaves = kRowThreads / 64;
    const long long planes = (long long)g.N * g.C;
    const long long plane_in = (long long)g.H * g.W, plane_out = (long long)g.Ho * g.Wo;
    auto part = [](long long floats) { return (long long)((floats + 32 + 3) / 4 * 4); };
    auto round_up = [](long long v, long long m) { return (v + m - 1) / m * m; };
    int lanes_per_row = 64;
    while (lanes_per_row / 2 >= g.Wo) lanes_per_row /= 2;
    const long long step = kWaves * (64 / lanes_per_row);          // output rows per round of the workgroup
    auto layout = [&](long long x_f, long long out_f, long long tasks, PoolRowsLds& at) {
        long long o = part(x_f);
        at.stage_at = (int)o; o += part(out_f);
        at.trash_at = (int)o; o += round_up(g.Wo + 4, 4);
        at.desc_at = (int)o;
        at.ntab = (int)round_up(tasks, step);
        at.lanes_per_row = lanes_per_row;
        if (part(x_f) > 4LL * kRowThreads * kRowXVecs) return 1LL << 40;          // more than the lanes' registers take
        return o + 4LL * at.ntab;
    };
    auto planes_need = [&](long long q, PoolRowsLds& at) { return layout(q * plane_in, q * plane_out, q * g.Ho, at); };
    SlabPlan plan;
    plan.total_planes = planes;
    PoolRowsLds at, probe;
    long long blocks = 0, lds_floats = 0;
    // 16 KB: eight 256-lane workgroups per CU with room to spare (20 KB measured level, 32 KB and 60 KB 3-10 % slower)
    int budget = env_int("CNNMEM_POOL_ROWS_FLOATS", 4096);
    if (budget < 1024 || budget > kRowLdsFloats) budget = kRowLdsFloats;
    if (planes_need(1, probe) > kRowLdsFloats) return CNNMEM_ERR_UNSUPPORTED;
    long long p = 1;
    while (p + 1 <= planes && planes_need(p + 1, probe) <= budget && planes / (p + 1) >= 1024) ++p;
    plan.planes_per_wg = (int)p;
    plan.rows_per_wg = g.Ho;
    plan.strips = 1;
    blocks = ceil_div64(planes, p);
    lds_floats = planes_need(p, at);
    if (blocks > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((pool_nchw_k3s2_rows_kernel<MODE>), dim3((unsigned)blocks), dim3(kRowThreads),
                       sizeof(float) * (size_t)lds_floats, st, src, dst, g, plan, at, make_fastdiv((uint32_t)g.Ho));
    return launch_status();
}

// ---- host-side dispatch ------------------------------------------------------

template <int MODE>
int launch_generic(const float* src, float* dst, const PoolGeom& g, int chwn, hipStream_t st) {
    const size_t total = (size_t)g.N * g.C * g.Ho * g.Wo;
    const long long want = ceil_div64((long long)total, kThreads);
    const unsigned blocks = (unsigned)(want < 65536 ? want : 65536);
    hipLaunchKernelGGL((pool_generic_kernel<MODE>), dim3(blocks), dim3(kThreads), 0, st, src, dst, g, chwn, total);
    return launch_status();
}

template <int MODE, int KH, int KW, int SH, int SW, int OY, int OX>
int launch_chwn_vec4(const float* src, float* dst, const PoolGeom& g, const PoolTuning& tune, hipStream_t st) {
    const long long row_items = (long long)(g.N / 4) * ceil_div64(g.Wo, OX);
    const long long bx = ceil_div64(row_items, kThreads), by = ceil_div64(g.Ho, OY);
    long long blocks = bx * by * g.C;
    if (row_items >= 0x7fffffffLL || blocks > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    const FastDiv dn4 = make_fastdiv((uint32_t)(g.N / 4));
    // rows that do not fill whole workgroups: deal lanes over the flattened (c, strip, position) space
    const long long all_items = row_items * by * g.C;
    const bool flat = row_items % kThreads != 0 && all_items < 0x7fffffffLL && env_int("CNNMEM_POOL_FLAT", 1) != 0;
    const uint32_t flat_items = flat ? (uint32_t)all_items : 0;
    if (flat) blocks = ceil_div64(all_items, kThreads);
    const FastDiv d_row = make_fastdiv((uint32_t)row_items), d_by = make_fastdiv((uint32_t)by);
    // disjoint windows, one output per lane: 64 B in flight per lane, best at 4 workgroups per CU for the
    // maximum and at 3 for the average (five tensors of 411-1644 MB, back to back: the average 1-2 % faster
    // at 3 than at 4 on every one, the maximum 3-6 % slower); larger working sets already keep plenty in
    // flight and are left alone unless asked
    const bool light = OY == 1 && OX == 1 && KH <= SH && KW <= SW;
    const long long in_bytes = 4LL * g.N * g.C * g.H * g.W;
    int cap = light || tune.workgroups_per_cu != 0 ? tune.workgroups_per_cu : -1;
    if (!light && tune.workgroups_per_cu == 0) {
        // Overlapping windows: a lane has 9 (one output) to 15 (two rows) 128-bit loads in flight.  Four
        // resident workgroups per CU measured 1-2 points above the full eight from 96 MB of input up
        // (128x96x55x55: 66.7 -> 68.3 % of peak, 512x96x55x55: 71.9 -> 73.7 %); two-row blocks are best uncapped.
        if (OY * OX == 1 && in_bytes >= (64LL << 20)) cap = 4;
        else if (OY * OX >= 3 && in_bytes >= (64LL << 20)) cap = 5;    // 3x3/s1, four rows: 59.8 -> 62.2 % at 206 MB
    }
    const size_t lds = throttle_lds(cap, in_bytes, light && MODE == CNNMEM_POOL_AVG ? 3 : 4);
    if (g.ph > 0 || g.pw > 0)
        hipLaunchKernelGGL((pool_chwn_vec4_kernel<MODE, KH, KW, SH, SW, OY, OX, true>), dim3((unsigned)blocks),
                           dim3(kThreads), lds, st, src, dst, g, (uint32_t)row_items, (uint32_t)bx,
                           (uint32_t)by, dn4, flat_items, d_row, d_by);
    else
        hipLaunchKernelGGL((pool_chwn_vec4_kernel<MODE, KH, KW, SH, SW, OY, OX, false>), dim3((unsigned)blocks),
                           dim3(kThreads), lds, st, src, dst, g, (uint32_t)row_items, (uint32_t)bx,
                           (uint32_t)by, dn4, flat_items, d_row, d_by);
    return launch_status();
}

// Working-set shapes that are compiled: rows per lane 1..4, columns per lane 1..2.
template <int MODE, int KH, int KW, int SH, int SW>
int launch_chwn_window(int oy, int ox, const float* src, float* dst, const PoolGeom& g, const PoolTuning& tune,
                       hipStream_t st) {
#define CNNMEM_WS(Y, X) \
    if (oy == Y && ox == X) return launch_chwn_vec4<MODE, KH, KW, SH, SW, Y, X>(src, dst, g, tune, st)
    CNNMEM_WS(1, 1); CNNMEM_WS(2, 1); CNNMEM_WS(3, 1); CNNMEM_WS(4, 1);
    CNNMEM_WS(1, 2); CNNMEM_WS(2, 2); CNNMEM_WS(3, 2); CNNMEM_WS(4, 2);
#undef CNNMEM_WS
    return CNNMEM_ERR_UNSUPPORTED;
}

template <int MODE>
int dispatch_chwn(const float* src, float* dst, const PoolGeom& g, const PoolTuning& tune, hipStream_t st) {
    const bool vec = (g.N % 4 == 0) && aligned16(src) && aligned16(dst);
    const int ox = tune.cols_per_lane ? tune.cols_per_lane : env_int("CNNMEM_CHWN_COLS", 1);
    int rc = CNNMEM_ERR_UNSUPPORTED;
    if (vec && g.kh == 3 && g.kw == 3 && g.sh == 2 && g.sw == 2) {
        // Outputs per lane along H.  More rows per lane reuse row results (7 input rows feed 3 outputs
        // instead of 9) but put 21 loads and 3 stores in one lane.  Measured on MI355X with write-through
        // stores, 128x96x55x55: 67.1 % of peak with one row, 64.7 % with two, 63.9 % with three (three was the
        // best before the stores were write-through).  The same holds with padding since the padded taps
        // stopped being branches (256x64x112x112 p1: 74.2 % with one row, 71.8 % with two, 71.4 % with three).
        const int rows = 1;
        rc = launch_chwn_window<MODE, 3, 3, 2, 2>(tune.rows_per_lane ? tune.rows_per_lane : env_int("CNNMEM_CHWN_ROWS", rows), ox, src, dst, g, tune, st);
    } else if (vec && g.kh == 2 && g.kw == 2 && g.sh == 2 && g.sw == 2) {
        // disjoint windows: nothing to reuse, one output per lane is fastest
        rc = launch_chwn_window<MODE, 2, 2, 2, 2>(tune.rows_per_lane ? tune.rows_per_lane : 1, ox, src, dst, g, tune, st);
    } else if (vec && g.kh == 3 && g.kw == 3 && g.sh == 1 && g.sw == 1) {
        rc = launch_chwn_window<MODE, 3, 3, 1, 1>(tune.rows_per_lane ? tune.rows_per_lane : env_int("CNNMEM_CHWN_ROWS", 4), ox, src, dst, g, tune, st);
    }
    if (rc != CNNMEM_ERR_UNSUPPORTED) return rc;
    // Output rows per lane, measured on MI355X (% of peak with 1 / 2 / 3 rows): 5x5/s1 24 / 33 / 37, 5x5/s2
    // 45 / 50 / 51, 5x5/s3 52 / 55 / 55, 4x4/s2 52 / 51 / 50.  Windows more than twice the stride take three,
    // windows between one and two strides two, the rest one.
    int rows = 1;
    if (g.Ho >= 3 && g.kh > 2 * g.sh) rows = 3;
    else if (g.Ho >= 2 && g.kh > g.sh && g.kh < 2 * g.sh) rows = 2;
    // the caller's tuning (the auto-tuner's search over outputs per lane along H) reaches this kernel too
    const int oy = tune.rows_per_lane ? (tune.rows_per_lane > 3 ? 3 : tune.rows_per_lane)
                                      : env_int("CNNMEM_CHWN_ANY_ROWS", rows);
    const long long hb = ceil_div64(g.Ho, oy == 3 ? 3 : (oy == 2 ? 2 : 1));
    const long long items = (long long)g.C * hb * g.Wo * (g.N / 4);
    if (vec && items < 0x7fffffffLL && items > 0) {
        const FastDiv dn4 = make_fastdiv((uint32_t)(g.N / 4)), dwo = make_fastdiv((uint32_t)g.Wo),
                      dhb = make_fastdiv((uint32_t)hb);
        // Few outputs, tall windows: fewer lanes than half the chip holds (256 CUs x 2048) would each walk
        // 16 taps or more one after the other; the window's rows are dealt over 4 or 8 lanes instead
        // (global 7x7 on 128x2048x7x7: 21.9 -> 13.4 us, global 14x14 on 32x512x14x14: 30.6 -> 13.0 us).
        int split = 0;
        if (oy == 1 && items < 262144 && g.kh >= 4 && g.kh * g.kw >= 16) split = g.kh >= 7 ? 8 : 4;
        split = env_int("CNNMEM_CHWN_SPLIT", split);
        if (oy == 1 && (split == 4 || split == 8)) {
            const dim3 sgrid((unsigned)ceil_div64(items, kThreads / split)), sblock(kThreads);
            if (split == 8)
                hipLaunchKernelGGL((pool_chwn_vec4_split_kernel<MODE, 8>), sgrid, sblock, 0, st, src, dst, g, (uint32_t)items, dn4, dwo, dhb);
            else
                hipLaunchKernelGGL((pool_chwn_vec4_split_kernel<MODE, 4>), sgrid, sblock, 0, st, src, dst, g, (uint32_t)items, dn4, dwo, dhb);
            return launch_status();
        }
        const dim3 grid((unsigned)ceil_div64(items, kThreads)), block(kThreads);
        if (oy == 3)
            hipLaunchKernelGGL((pool_chwn_vec4_any_kernel<MODE, 3>), grid, block, 0, st, src, dst, g, (uint32_t)items, dn4, dwo, dhb);
        else if (oy == 2)
            hipLaunchKernelGGL((pool_chwn_vec4_any_kernel<MODE, 2>), grid, block, 0, st, src, dst, g, (uint32_t)items, dn4, dwo, dhb);
        else
            hipLaunchKernelGGL((pool_chwn_vec4_any_kernel<MODE, 1>), grid, block, 0, st, src, dst, g, (uint32_t)items, dn4, dwo, dhb);
        return launch_status();
    }
    return launch_generic<MODE>(src, dst, g, 1, st);
}

template <int MODE, int KH, int KW, int SH, int SW, int OY, int THREADS>
int launch_slab_threads(const float* src, float* dst, const PoolGeom& g, const SlabPlan& plan, long long blocks,
                        hipStream_t st) {
    const FastDiv dwo = make_fastdiv((uint32_t)g.Wo);
    const FastDiv dpo = make_fastdiv((uint32_t)(g.Ho * g.Wo));
    const int rows_out = plan.strips == 1 ? g.Ho : plan.rows_per_wg;
    const FastDiv dblk = make_fastdiv((uint32_t)ceil_div(rows_out, OY));
    if (g.ph > 0 || g.pw > 0 || KH == 0)
        hipLaunchKernelGGL((pool_nchw_slab_kernel<MODE, KH, KW, SH, SW, OY, true, THREADS>), dim3((unsigned)blocks),
                           dim3(THREADS), 0, st, src, dst, g, plan, dwo, dpo, dblk, g.kh, g.kw, g.sh, g.sw);
    else
        hipLaunchKernelGGL((pool_nchw_slab_kernel<MODE, KH, KW, SH, SW, OY, false, THREADS>), dim3((unsigned)blocks),
                           dim3(THREADS), 0, st, src, dst, g, plan, dwo, dpo, dblk, g.kh, g.kw, g.sh, g.sw);
    return launch_status();
}

template <int MODE, int KH, int KW, int SH, int SW, int OY = 1>
int launch_slab(const float* src, float* dst, const PoolGeom& g, const SlabPlan& plan, long long blocks,
                const PoolTuning& tune, hipStream_t st) {
    // lanes per slab: more lanes = fewer 128-bit loads in flight per lane for the same 32 KB;
    // 512 measured best (68 % of peak against 64 % with 256 and 49 % with 1024)
    const int threads = tune.slab_lanes ? tune.slab_lanes : 512;
    if (threads >= 1024) return launch_slab_threads<MODE, KH, KW, SH, SW, OY, 1024>(src, dst, g, plan, blocks, st);
    if (threads >= 512) return launch_slab_threads<MODE, KH, KW, SH, SW, OY, 512>(src, dst, g, plan, blocks, st);
    return launch_slab_threads<MODE, KH, KW, SH, SW, OY, 256>(src, dst, g, plan, blocks, st);
}

template <int MODE>
int dispatch_nchw(const float* src, float* dst, const PoolGeom& g, const PoolTuning& tune, hipStream_t st) {
    const long long planes = (long long)g.N * g.C;
    const bool a16 = aligned16(src) && aligned16(dst);

    // (1) non-overlapping 2x2 / stride 2 on even H: row pairs, no staging
    if (a16 && g.kh == 2 && g.kw == 2 && g.sh == 2 && g.sw == 2 && g.ph == 0 && g.pw == 0 &&
        g.H % 2 == 0 && g.W % 4 == 0 && tune.nchw_kernel != 2) {
        const long long per_row = g.W / 4;
        const long long items = planes * g.Ho * per_row;
        if (items < 0x7fffffffLL) {
            const FastDiv d = make_fastdiv((uint32_t)per_row);
            const unsigned blocks = (unsigned)ceil_div64(items, kThreads);
            // 32 B in flight per lane: best at 5 workgroups per CU on large tensors (64x64x224x224 with
            // write-through stores: 82.7 % of peak at 5, 80.4 % at 6, 78.7 % at 4, 76.0 % uncapped)
            const size_t lds = throttle_lds(tune.workgroups_per_cu, 4LL * planes * g.H * g.W, 5);
            hipLaunchKernelGGL((pool_nchw_2x2s2_kernel<MODE>), dim3(blocks), dim3(kThreads), lds, st, src, dst,
                               (uint32_t)items, (uint32_t)g.W, d);
            return launch_status();
        }
    }

    const long long plane_in = (long long)g.H * g.W;
    // (2a) 3x3 / stride 2 without padding on planes of 12 output columns and more that fit LDS whole: the rows kernel
    // (128x96x55x55 33.0 -> 32.7 us, 128x256x27x27 23.7 -> 22.9 us, back to back 31.5 -> 30.8 and 22.3 -> 21.3 us; planes of
    // 24x24 and 13x13 are better off in the slab kernel's many planes per workgroup: 6.1 against 6.5, 7.2 against 8.0 us)
    if (a16 && g.kh == 3 && g.kw == 3 && g.sh == 2 && g.sw == 2 && g.ph == 0 && g.pw == 0 && g.Wo >= 12 &&
        plane_in * planes < (1LL << 31) && plane_in * planes >= 4 && tune.nchw_kernel == 0 &&
        env_int("CNNMEM_POOL_ROWS", 1) != 0) {
        const int rc = launch_nchw_k3s2_rows<MODE>(src, dst, g, st);
        if (rc != CNNMEM_ERR_UNSUPPORTED) return rc;
    }
    // (2) LDS slab: whole planes when they fit, else strips of output rows
    if (aligned16(src) && plane_in * planes < (1LL << 40) && plane_in * planes >= 4) {
        SlabPlan plan;
        plan.total_planes = planes;
        bool ok = false;
        long long blocks = 0;
        const int budget = kSlabFloats - 32;        // room for the line-aligned head
        if (plane_in <= budget) {
            long long p = budget / plane_in;
            // Small tensors: at least 1024 workgroups when the planes allow, i.e. about one resident round
            // of the chip (5 x 32 KB of LDS per CU).  With 2048 the Table 1 layers of 2-27 MB needed a second
            // round for a handful of lanes each: PL2 8.9 -> 6.8 us, PL4 9.1 -> 7.0, PL10 9.5 -> 7.5, PL7 10.7 -> 9.4.
            const long long min_blocks = 1024;
            if (planes / p < min_blocks) p = planes / min_blocks > 0 ? planes / min_blocks : 1;
            if (p * (long long)g.Ho * g.Wo < (1 << 20)) {         // the kernel's small-number divider
                plan.planes_per_wg = (int)p;
                plan.rows_per_wg = g.Ho;
                plan.strips = 1;
                blocks = ceil_div64(planes, p);
                ok = true;
            }
        } else {
            // rows_out output rows need (rows_out-1)*sh + kh input rows
            const long long max_in_rows = budget / g.W;
            long long rows_out = (max_in_rows - g.kh) / g.sh + 1;
            if (max_in_rows >= g.kh && rows_out >= 1 && rows_out * g.Wo < (1 << 20)) {
                if (rows_out > g.Ho) rows_out = g.Ho;
                plan.planes_per_wg = 1;
                plan.rows_per_wg = (int)rows_out;
                plan.strips = ceil_div(g.Ho, rows_out);
                blocks = planes * plan.strips;
                ok = true;
            }
        }
        if (ok && blocks <= 0x7fffffffLL) {
            // Rows per lane.  Several rows share row results and, with padding, the clamping arithmetic, but
            // break the workgroup's contiguous output run into row pieces: measured better only with padding
            // (3x3/s1/p1 64x256x56x56: 43 -> 57 % max, 34 -> 55 % avg; 3x3/s2/p1 avg 63 -> 70 %) and worse
            // without (3x3/s1: 68 -> 49 %; 3x3/s2: 75 -> 70 %).
            const bool padded = g.ph > 0 || g.pw > 0;
            int oy = env_int("CNNMEM_SLAB_ROWS", 0);
            if (oy == 0) oy = !padded ? 1 : (g.sh == 1 ? 4 : (MODE == CNNMEM_POOL_AVG ? 2 : 1));
            if (g.kh == 3 && g.kw == 3 && g.sh == 2 && g.sw == 2) {
                if (oy == 3) return launch_slab<MODE, 3, 3, 2, 2, 3>(src, dst, g, plan, blocks, tune, st);
                if (oy == 2) return launch_slab<MODE, 3, 3, 2, 2, 2>(src, dst, g, plan, blocks, tune, st);
                return launch_slab<MODE, 3, 3, 2, 2>(src, dst, g, plan, blocks, tune, st);
            }
            if (g.kh == 3 && g.kw == 3 && g.sh == 1 && g.sw == 1) {
                if (oy == 1) return launch_slab<MODE, 3, 3, 1, 1>(src, dst, g, plan, blocks, tune, st);
                if (oy == 2) return launch_slab<MODE, 3, 3, 1, 1, 2>(src, dst, g, plan, blocks, tune, st);
                return launch_slab<MODE, 3, 3, 1, 1, 4>(src, dst, g, plan, blocks, tune, st);
            }
            if (g.kh == 2 && g.kw == 2 && g.sh == 2 && g.sw == 2)
                return launch_slab<MODE, 2, 2, 2, 2>(src, dst, g, plan, blocks, tune, st);
            return launch_slab<MODE, 0, 0, 0, 0>(src, dst, g, plan, blocks, tune, st);
        }
    }
    return launch_generic<MODE>(src, dst, g, 0, st);
}

}  // namespace

int launch_pool_nchw(const float* src, float* dst, const PoolGeom& g, const PoolTuning& tune, hipStream_t st) {
    return g.mode == CNNMEM_POOL_MAX ? dispatch_nchw<CNNMEM_POOL_MAX>(src, dst, g, tune, st)
                                     : dispatch_nchw<CNNMEM_POOL_AVG>(src, dst, g, tune, st);
}

int launch_pool_chwn(const float* src, float* dst, const PoolGeom& g, const PoolTuning& tune, hipStream_t st) {
    return g.mode == CNNMEM_POOL_MAX ? dispatch_chwn<CNNMEM_POOL_MAX>(src, dst, g, tune, st)
                                     : dispatch_chwn<CNNMEM_POOL_AVG>(src, dst, g, tune, st);
}

}  // namespace cnnmem
