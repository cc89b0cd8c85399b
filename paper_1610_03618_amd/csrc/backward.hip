// Backward passes of pooling and softmax (training; Section II.A's footnote: the same
// data structures serve both passes).  Both are as memory-bound as their forward passes.
//
// Pooling backward is written as a gather, one lane per INPUT element (or four images of
// it in CHWN), so no two lanes ever add into the same word and no atomics are needed: the
// lane visits the few windows that contain its element and, for the maximum, re-scans
// each of them to see whether its element is the first maximum in scan order (rows, then
// columns).  Nothing but the forward input and the incoming gradient is read; no index
// tensor has to be kept from the forward pass.
//
// Softmax backward keeps a row of probabilities and a row of incoming gradients in
// registers, reduces their dot product with the forward pass's reductions, and writes
// p * (dp - dot): one read of both inputs, one write.
#include "common.hpp"
#include "rowmath.hpp"

namespace cnnmem {
namespace {

constexpr int kThreads = 256;
constexpr float kNegInf = kRowNegInf;

// Pins a loaded value in registers.  A load whose only use is one arm of a select gets moved under a
// branch by the compiler, and a branch per load means a full wait per load; after this the value
// has an unconditional use, so the loads stay where they are written, back to back.
__device__ __forceinline__ void keep(float4& v) {
    asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
}

// windows (along one axis) that contain input coordinate x: lo <= i <= hi
__device__ __forceinline__ void window_range(int x, int k, int s, int p, int n_out, int& lo, int& hi) {
    const int a = x + p - k + 1;                    // first window start that still reaches x, times s
    lo = a > 0 ? (a + s - 1) / s : 0;
    hi = (x + p) / s;
    if (hi > n_out - 1) hi = n_out - 1;
}

// ---- one lane per input element, any layout ------------------------------------------
template <int MODE>
__global__ __launch_bounds__(kThreads) void pool_bwd_generic_kernel(
    const float* __restrict__ src, const float* __restrict__ ddst, float* __restrict__ dsrc, PoolGeom g, int chwn,
    size_t total) {
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t o = (size_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += stride) {
        int n, c, h, w;
        size_t t = o;
        if (chwn) {
            n = (int)(t % g.N); t /= g.N;
            w = (int)(t % g.W); t /= g.W;
            h = (int)(t % g.H); c = (int)(t / g.H);
        } else {
            w = (int)(t % g.W); t /= g.W;
            h = (int)(t % g.H); t /= g.H;
            c = (int)(t % g.C); n = (int)(t / g.C);
        }
        int i_lo, i_hi, j_lo, j_hi;
        window_range(h, g.kh, g.sh, g.ph, g.Ho, i_lo, i_hi);
        window_range(w, g.kw, g.sw, g.pw, g.Wo, j_lo, j_hi);
        float acc = 0.f;
        for (int i = i_lo; i <= i_hi; ++i)
            for (int j = j_lo; j <= j_hi; ++j) {
                const size_t oidx = chwn ? (((size_t)c * g.Ho + i) * g.Wo + j) * g.N + n
                                         : (((size_t)n * g.C + c) * g.Ho + i) * g.Wo + j;
                if (MODE == CNNMEM_POOL_AVG) {
                    acc += ddst[oidx];
                } else {
                    float best = kNegInf;
                    bool mine = false, any = false;
                    for (int y = 0; y < g.kh; ++y) {
                        const int r = i * g.sh - g.ph + y;
                        if (r < 0 || r >= g.H) continue;
                        for (int x = 0; x < g.kw; ++x) {
                            const int q = j * g.sw - g.pw + x;
                            if (q < 0 || q >= g.W) continue;
                            const size_t idx = chwn ? (((size_t)c * g.H + r) * g.W + q) * g.N + n
                                                    : (((size_t)n * g.C + c) * g.H + r) * g.W + q;
                            const float v = src[idx];
                            if (!any || v > best) { best = v; mine = (r == h && q == w); any = true; }
                        }
                    }
                    if (mine) acc += ddst[oidx];
                }
            }
        dsrc[o] = MODE == CNNMEM_POOL_AVG ? acc / (float)(g.kh * g.kw) : acc;
    }
}

// ---- CHWN: a lane owns four images (one float4) of one input element -------------------
template <int MODE, int KH, int KW, int SH, int SW>
__global__ __launch_bounds__(kThreads) void pool_bwd_chwn_vec4_kernel(
    const float* __restrict__ src, const float* __restrict__ ddst, float* __restrict__ dsrc, PoolGeom g,
    uint32_t items, FastDiv div_n4, FastDiv div_w, FastDiv div_h) {
    const int kh = KH ? KH : g.kh, kw = KW ? KW : g.kw, sh = SH ? SH : g.sh, sw = SW ? SW : g.sw;
    const uint32_t u = blockIdx.x * kThreads + threadIdx.x;
    if (u >= items) return;
    // u = ((c*H + h)*W + w)*N4 + n4
    uint32_t t = fd_div(u, div_n4);
    const uint32_t n4 = u - t * div_n4.d;
    uint32_t t2 = fd_div(t, div_w);
    const int w = (int)(t - t2 * div_w.d);
    const uint32_t c = fd_div(t2, div_h);
    const int h = (int)(t2 - c * div_h.d);
    const int N = g.N;
    int i_lo, i_hi, j_lo, j_hi;
    window_range(h, kh, sh, g.ph, g.Ho, i_lo, i_hi);
    window_range(w, kw, sw, g.pw, g.Wo, j_lo, j_hi);
    const float* plane = src + (size_t)c * g.H * g.W * N + 4 * n4;
    const float* gplane = ddst + (size_t)c * g.Ho * g.Wo * N + 4 * n4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i = i_lo; i <= i_hi; ++i)
        for (int j = j_lo; j <= j_hi; ++j) {
            const float4 gy = *reinterpret_cast<const float4*>(gplane + ((size_t)i * g.Wo + j) * N);
            if (MODE == CNNMEM_POOL_AVG) {
                acc.x += gy.x; acc.y += gy.y; acc.z += gy.z; acc.w += gy.w;
            } else {
                // scan the window in the forward order; `mine` tracks, per image, whether the
                // running first maximum sits on this lane's element
                float4 best = make_float4(kNegInf, kNegInf, kNegInf, kNegInf);
                bool mx = false, my = false, mz = false, mw = false, any = false;
#pragma unroll
                for (int y = 0; y < (KH ? KH : 8); ++y) {
                    if (y >= kh) break;
                    const int r = i * sh - g.ph + y;
                    if (r < 0 || r >= g.H) continue;
#pragma unroll
                    for (int x = 0; x < (KW ? KW : 8); ++x) {
                        if (x >= kw) break;
                        const int q = j * sw - g.pw + x;
                        if (q < 0 || q >= g.W) continue;
                        const float4 v = *reinterpret_cast<const float4*>(plane + ((size_t)r * g.W + q) * N);
                        const bool me = (r == h && q == w);
                        if (!any || v.x > best.x) { best.x = v.x; mx = me; }
                        if (!any || v.y > best.y) { best.y = v.y; my = me; }
                        if (!any || v.z > best.z) { best.z = v.z; mz = me; }
                        if (!any || v.w > best.w) { best.w = v.w; mw = me; }
                        any = true;
                    }
                }
                if (mx) acc.x += gy.x;
                if (my) acc.y += gy.y;
                if (mz) acc.z += gy.z;
                if (mw) acc.w += gy.w;
            }
        }
    if (MODE == CNNMEM_POOL_AVG) {
        const float d = (float)(kh * kw);
        acc = make_float4(acc.x / d, acc.y / d, acc.z / d, acc.w / d);
    }
    st4_stream(dsrc + 4 * (size_t)u, acc);
}

// ---- CHWN, no padding, square window K and stride S known at compile time ---------------
// A lane owns four images of one S x S cell of inputs (the inputs that share their set of
// windows).  The NW x NW windows that touch the cell span RR x RR taps, RR = S*(NW-1) + K:
// the lane loads them once (25 float4 for 3x3 / stride 2 instead of the 81 that four
// separate lanes would ask for), finds the first maximum of each window once, and hands
// each window's gradient to the cell element that holds it.
template <int MODE, int K, int S>
__global__ __launch_bounds__(kThreads) void pool_bwd_chwn_cell_kernel(
    const float* __restrict__ src, const float* __restrict__ ddst, float* __restrict__ dsrc, PoolGeom g,
    uint32_t items, FastDiv div_n4, FastDiv div_cw, FastDiv div_ch) {
    constexpr int NW = (K - 1) / S + 1;             // windows per axis that touch a cell
    constexpr int RR = S * (NW - 1) + K;            // taps per axis they span
    // Overlapping windows: every incoming gradient serves NW x NW cells, most of them in other workgroups.  With
    // neighbouring workgroups on one XCD the second request is an L2 hit (counters, 3x3 / stride 2 average on
    // 128x96x55x55: the gradients were fetched from memory 2.2 times over, 1.24x the algorithmic traffic).
    const uint32_t blk = K > S ? xcd_contiguous_tile(blockIdx.x, gridDim.x) : blockIdx.x;
    const uint32_t u = blk * kThreads + threadIdx.x;
    if (u >= items) return;
    // u = ((c*cells_h + ci)*cells_w + cj)*N4 + n4
    uint32_t t = fd_div(u, div_n4);
    const uint32_t n4 = u - t * div_n4.d;
    uint32_t t2 = fd_div(t, div_cw);
    const int cj = (int)(t - t2 * div_cw.d);
    const uint32_t c = fd_div(t2, div_ch);
    const int ci = (int)(t2 - c * div_ch.d);
    const int N = g.N;
    const int i0 = ci - (NW - 1), j0 = cj - (NW - 1);          // first window of the cell, may be negative
    const int r0 = S * i0, q0 = S * j0;                        // first tap row / column, may be negative

    // incoming gradients of the NW x NW windows; windows outside the output contribute nothing
    float4 gy[NW][NW];
    const float* gplane = ddst + (size_t)c * g.Ho * g.Wo * N + 4 * n4;
#pragma unroll
    for (int a = 0; a < NW; ++a)
#pragma unroll
        for (int b = 0; b < NW; ++b) {
            const int i = i0 + a, j = j0 + b;
            const int ic = i < 0 ? 0 : (i < g.Ho ? i : g.Ho - 1), jc = j < 0 ? 0 : (j < g.Wo ? j : g.Wo - 1);
            gy[a][b] = *reinterpret_cast<const float4*>(gplane + ((size_t)ic * g.Wo + jc) * N);
        }

    // called once every load of the lane has been issued: pins the gradients (see keep) and zeroes
    // those of windows outside the output
    auto settle_gradients = [&]() {
#pragma unroll
        for (int a = 0; a < NW; ++a)
#pragma unroll
            for (int b = 0; b < NW; ++b) keep(gy[a][b]);
#pragma unroll
        for (int a = 0; a < NW; ++a)
#pragma unroll
            for (int b = 0; b < NW; ++b) {
                const int i = i0 + a, j = j0 + b;
                if (!(i >= 0 && i < g.Ho && j >= 0 && j < g.Wo)) gy[a][b] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
    };

    float4 dx[S][S];
#pragma unroll
    for (int ey = 0; ey < S; ++ey)
#pragma unroll
        for (int ex = 0; ex < S; ++ex) dx[ey][ex] = make_float4(0.f, 0.f, 0.f, 0.f);

    if (MODE == CNNMEM_POOL_AVG) {
        settle_gradients();
#pragma unroll
        for (int a = 0; a < NW; ++a)
#pragma unroll
            for (int b = 0; b < NW; ++b)
#pragma unroll
                for (int ey = 0; ey < S; ++ey)
#pragma unroll
                    for (int ex = 0; ex < S; ++ex) {
                        // cell element (ey, ex) is tap (y, x) of window (a, b) when 0 <= y, x < K
                        const int y = S * (NW - 1 - a) + ey, x = S * (NW - 1 - b) + ex;
                        if (y < K && x < K) {
                            dx[ey][ex].x += gy[a][b].x; dx[ey][ex].y += gy[a][b].y;
                            dx[ey][ex].z += gy[a][b].z; dx[ey][ex].w += gy[a][b].w;
                        }
                    }
        const float inv = 1.0f / (float)(K * K);
#pragma unroll
        for (int ey = 0; ey < S; ++ey)
#pragma unroll
            for (int ex = 0; ex < S; ++ex)
                dx[ey][ex] = make_float4(dx[ey][ex].x * inv, dx[ey][ex].y * inv, dx[ey][ex].z * inv, dx[ey][ex].w * inv);
    } else {
        // every tap the windows span, loaded once from clamped addresses (a clamped tap only ever
        // belongs to a window outside the output, whose gradient is zero)
        const float* plane = src + (size_t)c * g.H * g.W * N + 4 * n4;
        float4 xv[RR][RR];
#pragma unroll
        for (int y = 0; y < RR; ++y) {
            const int r = r0 + y;
            const int rc = r < 0 ? 0 : (r < g.H ? r : g.H - 1);
#pragma unroll
            for (int x = 0; x < RR; ++x) {
                const int q = q0 + x;
                const int qc = q < 0 ? 0 : (q < g.W ? q : g.W - 1);
                xv[y][x] = *reinterpret_cast<const float4*>(plane + ((size_t)rc * g.W + qc) * N);
            }
        }
        settle_gradients();
#pragma unroll
        for (int y = 0; y < RR; ++y)
#pragma unroll
            for (int x = 0; x < RR; ++x) keep(xv[y][x]);
#pragma unroll
        for (int a = 0; a < NW; ++a)
#pragma unroll
            for (int b = 0; b < NW; ++b) {
                // first maximum of window (a, b) in scan order, per image: index y*K + x
                float4 best = xv[S * a][S * b];
                int kx = 0, ky = 0, kz = 0, kw = 0;
#pragma unroll
                for (int y = 0; y < K; ++y)
#pragma unroll
                    for (int x = 0; x < K; ++x) {
                        if (y == 0 && x == 0) continue;
                        const float4 v = xv[S * a + y][S * b + x];
                        const int idx = y * K + x;
                        if (v.x > best.x) { best.x = v.x; kx = idx; }
                        if (v.y > best.y) { best.y = v.y; ky = idx; }
                        if (v.z > best.z) { best.z = v.z; kz = idx; }
                        if (v.w > best.w) { best.w = v.w; kw = idx; }
                    }
#pragma unroll
                for (int ey = 0; ey < S; ++ey)
#pragma unroll
                    for (int ex = 0; ex < S; ++ex) {
                        const int y = S * (NW - 1 - a) + ey, x = S * (NW - 1 - b) + ex;
                        if (y < K && x < K) {
                            const int idx = y * K + x;
                            if (kx == idx) dx[ey][ex].x += gy[a][b].x;
                            if (ky == idx) dx[ey][ex].y += gy[a][b].y;
                            if (kz == idx) dx[ey][ex].z += gy[a][b].z;
                            if (kw == idx) dx[ey][ex].w += gy[a][b].w;
                        }
                    }
            }
    }
    float* oplane = dsrc + (size_t)c * g.H * g.W * N + 4 * n4;
#pragma unroll
    for (int ey = 0; ey < S; ++ey) {
        const int h = S * ci + ey;
#pragma unroll
        for (int ex = 0; ex < S; ++ex) {
            const int w = S * cj + ex;
            if (h < g.H && w < g.W) {
                // the average only writes (a quarter as much is read): write-through stores gain 3 % there
                if (MODE == CNNMEM_POOL_AVG) st4_through(oplane + ((size_t)h * g.W + w) * N, dx[ey][ex]);
                else st4_stream(oplane + ((size_t)h * g.W + w) * N, dx[ey][ex]);
            }
        }
    }
}

// ---- CHWN maximum, overlapping windows, through LDS ------------------------------------------
// The cell kernel above asks L1 for RR x RR taps per cell although only S x S of them are new: with
// 3x3 / stride 2 the vector L1 passes 4-5 times the tensor, and that, not HBM, bounds it.  Here a
// workgroup owns a patch of CR x CQ cells of 4*NB4 images: the patch's taps (its inputs plus a halo of
// RR - S rows and columns) go from global memory into LDS once, with all loads in flight together, and
// every lane then takes the taps of its cell's windows from LDS.  Patches that share a halo run on the
// same XCD, so the halo is an L2 hit.  One lane per (cell, four images): 256 = CR * CQ * NB4.
// SHARED: the first maximum of every window of the patch is found once, by one lane per (window, four images),
// and left in LDS as four 8-bit tap indices; the NW x NW cells that share the window read it from there
// instead of each scanning the window's K x K taps again.
template <int K, int S, int CR, int CQ, int NB4, bool SHARED>
__global__ __launch_bounds__(CR * CQ * NB4) void pool_bwd_chwn_patch_kernel(
    const float* __restrict__ src, const float* __restrict__ ddst, float* __restrict__ dsrc, PoolGeom g,
    uint32_t patches_w, uint32_t patches_h, uint32_t chunks, FastDiv div_chunks, FastDiv div_pw, FastDiv div_ph) {
    constexpr int THREADS = CR * CQ * NB4;
    constexpr int NW = (K - 1) / S + 1;
    constexpr int RR = S * (NW - 1) + K;
    constexpr int PR = S * (CR - 1) + RR, PQ = S * (CQ - 1) + RR;      // taps per patch
    constexpr int SLOTS = PR * PQ;                                     // tap positions, NB4 float4 each
    constexpr int ROUNDS = (SLOTS * NB4 + THREADS - 1) / THREADS;
    __shared__ float4 taps[SLOTS * NB4];

    const uint32_t tile = xcd_contiguous_tile(blockIdx.x, gridDim.x);
    // tile = ((c * patches_h + pr) * patches_w + pq) * chunks + chunk
    uint32_t t = fd_div(tile, div_chunks);
    const uint32_t chunk = tile - t * chunks;
    uint32_t t2 = fd_div(t, div_pw);
    const int pq = (int)(t - t2 * patches_w);
    const uint32_t c = fd_div(t2, div_ph);
    const int pr = (int)(t2 - c * patches_h);
    const int N = g.N;
    const int tid = threadIdx.x;
    const int n4 = tid % NB4;
    const size_t n_off = (size_t)chunk * (4 * NB4) + 4 * n4;
    const int r_first = S * (pr * CR - (NW - 1)), q_first = S * (pq * CQ - (NW - 1));   // may be negative

    // ---- all loads first: the patch's taps (clamped into the image: a clamped tap only ever belongs
    // to a window outside the output, whose gradient is zero) and the lane's NW x NW gradients ----
    const float* plane = src + (size_t)c * g.H * g.W * N + n_off;
    float4 v[ROUNDS];
#pragma unroll
    for (int k = 0; k < ROUNDS; ++k) {
        int slot = tid / NB4 + k * (THREADS / NB4);
        slot = slot < SLOTS ? slot : SLOTS - 1;
        const int y = slot / PQ, x = slot - y * PQ;
        const int r = r_first + y, q = q_first + x;
        const int rc = r < 0 ? 0 : (r < g.H ? r : g.H - 1), qc = q < 0 ? 0 : (q < g.W ? q : g.W - 1);
        v[k] = *reinterpret_cast<const float4*>(plane + ((size_t)rc * g.W + qc) * N);
    }
    const int cell = tid / NB4;
    const int cy = cell / CQ, cx = cell - cy * CQ;
    const int ci = pr * CR + cy, cj = pq * CQ + cx;                    // the lane's cell in the image
    const int i0 = ci - (NW - 1), j0 = cj - (NW - 1);
    float4 gy[NW][NW];
    const float* gplane = ddst + (size_t)c * g.Ho * g.Wo * N + n_off;
#pragma unroll
    for (int a = 0; a < NW; ++a)
#pragma unroll
        for (int b = 0; b < NW; ++b) {
            const int i = i0 + a, j = j0 + b;
            const int ic = i < 0 ? 0 : (i < g.Ho ? i : g.Ho - 1), jc = j < 0 ? 0 : (j < g.Wo ? j : g.Wo - 1);
            gy[a][b] = *reinterpret_cast<const float4*>(gplane + ((size_t)ic * g.Wo + jc) * N);
        }
#pragma unroll
    for (int k = 0; k < ROUNDS; ++k) {
        const int slot = tid / NB4 + k * (THREADS / NB4);
        if (slot < SLOTS) taps[slot * NB4 + n4] = v[k];
    }
#pragma unroll
    for (int a = 0; a < NW; ++a)
#pragma unroll
        for (int b = 0; b < NW; ++b) {
            keep(gy[a][b]);
            const int i = i0 + a, j = j0 + b;
            if (!(i >= 0 && i < g.Ho && j >= 0 && j < g.Wo)) gy[a][b] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    __syncthreads();

    float4 dx[S][S];
#pragma unroll
    for (int ey = 0; ey < S; ++ey)
#pragma unroll
        for (int ex = 0; ex < S; ++ex) dx[ey][ex] = make_float4(0.f, 0.f, 0.f, 0.f);
    // first maximum of the window whose first tap is at w0, in scan order, per image: index y*K + x
    auto first_max = [&](const float4* w0, int& kx, int& ky, int& kz, int& kw) {
        float4 best = w0[0];
        kx = ky = kz = kw = 0;
#pragma unroll
        for (int y = 0; y < K; ++y)
#pragma unroll
            for (int x = 0; x < K; ++x) {
                if (y == 0 && x == 0) continue;
                const float4 u = w0[(y * PQ + x) * NB4];
                const int idx = y * K + x;
                if (u.x > best.x) { best.x = u.x; kx = idx; }
                if (u.y > best.y) { best.y = u.y; ky = idx; }
                if (u.z > best.z) { best.z = u.z; kz = idx; }
                if (u.w > best.w) { best.w = u.w; kw = idx; }
            }
    };
    constexpr int WR = CR + NW - 1, WQ = CQ + NW - 1;          // windows that touch the patch
    __shared__ uint32_t widx[SHARED ? WR * WQ * NB4 : 1];
    if constexpr (SHARED) {
        for (int it = tid; it < WR * WQ * NB4; it += THREADS) {
            const int win = it / NB4, wn4 = it - win * NB4;
            const int wy = win / WQ, wx = win - wy * WQ;
            int kx, ky, kz, kw;
            first_max(taps + ((S * wy) * PQ + S * wx) * NB4 + wn4, kx, ky, kz, kw);
            widx[it] = (uint32_t)kx | ((uint32_t)ky << 8) | ((uint32_t)kz << 16) | ((uint32_t)kw << 24);
        }
        __syncthreads();
    }
    // Window by window, taps straight from LDS (holding all RR x RR taps in registers, or finding the
    // maximum first and then its first occurrence, both measured slower: 84 us against 81 us on
    // 128x96x55x55).
#pragma unroll
    for (int a = 0; a < NW; ++a)
#pragma unroll
        for (int b = 0; b < NW; ++b) {
            int kx, ky, kz, kw;
            if constexpr (SHARED) {
                const uint32_t packed = widx[((cy + a) * WQ + (cx + b)) * NB4 + n4];
                kx = (int)(packed & 0xffu); ky = (int)((packed >> 8) & 0xffu);
                kz = (int)((packed >> 16) & 0xffu); kw = (int)(packed >> 24);
            } else {
                first_max(taps + ((S * (cy + a)) * PQ + S * (cx + b)) * NB4 + n4, kx, ky, kz, kw);
            }
#pragma unroll
            for (int ey = 0; ey < S; ++ey)
#pragma unroll
                for (int ex = 0; ex < S; ++ex) {
                    // cell element (ey, ex) is tap (y, x) of window (a, b) when 0 <= y, x < K
                    const int y = S * (NW - 1 - a) + ey, x = S * (NW - 1 - b) + ex;
                    if (y < K && x < K) {
                        const int idx = y * K + x;
                        if (kx == idx) dx[ey][ex].x += gy[a][b].x;
                        if (ky == idx) dx[ey][ex].y += gy[a][b].y;
                        if (kz == idx) dx[ey][ex].z += gy[a][b].z;
                        if (kw == idx) dx[ey][ex].w += gy[a][b].w;
                    }
                }
        }
    float* oplane = dsrc + (size_t)c * g.H * g.W * N + n_off;
#pragma unroll
    for (int ey = 0; ey < S; ++ey) {
        const int h = S * ci + ey;
#pragma unroll
        for (int ex = 0; ex < S; ++ex) {
            const int w = S * cj + ex;
            if (h < g.H && w < g.W) st4_stream(oplane + ((size_t)h * g.W + w) * N, dx[ey][ex]);
        }
    }
}

// ---- NCHW through LDS --------------------------------------------------------------------
// A workgroup takes whole (n, c) planes, or a strip of input rows of one plane, streams
// the incoming gradients of every window that touches them (and, for the maximum, the
// input rows those windows span) into LDS with line-aligned 128-bit loads, and then one
// lane per input element gathers from LDS.  The strip's gradients leave as one
// contiguous run with line-aligned wavefront stores.
constexpr int kBwdSlabFloats = 15360;               // at most 60 KB of LDS per workgroup (sized per launch)
constexpr int kBwdThreads = 512;

struct BwdSlabPlan {
    int planes_per_wg;      // whole planes per workgroup ...
    int rows_per_wg;        // ... or input rows per strip
    int strips;
    long long total_planes;
};

// streams floats [lo, hi) of `p` (16-byte aligned base, `total` floats long) into dst_lds so that
// element e sits at dst_lds[e - a_lo]; returns a_lo, the aligned start.  All loads unconditional.
template <int VEC, int THREADS = kBwdThreads>
__device__ __forceinline__ size_t stream_to_lds(const float* __restrict__ p, size_t lo, size_t hi, size_t total,
                                                float* dst_lds) {
    const size_t mask = (reinterpret_cast<uintptr_t>(p) & 127u) == 0 ? 31 : 3;
    const size_t a_lo = lo & ~mask;
    const int nvec = (int)((hi - a_lo + 3) >> 2);
    const size_t a_last = (total - 4) & ~(size_t)3;            // total >= 4 (dispatch)
    // rounds of THREADS vectors; a round past the end of the part is skipped by the whole
    // workgroup (uniform), inside a round every load is unconditional
    float4 v[VEC];
    if (a_lo + 4 * (size_t)(nvec - 1) <= a_last) {
        // every workgroup but the one at the tensor's end: no float4 can cross the end; uniform base plus a
        // 32-bit lane offset instead of 64-bit compares and selects per load
        const float* base = p + a_lo;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if (k * THREADS >= nvec) break;
            const uint32_t q = threadIdx.x + k * THREADS;
            v[k] = ld4_stream(base + 4u * (q < (uint32_t)nvec ? q : 0u));
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if (k * THREADS >= nvec) break;
            const uint32_t q = threadIdx.x + k * THREADS;
            if (q < (uint32_t)nvec) *reinterpret_cast<float4*>(dst_lds + 4 * q) = v[k];
        }
        return a_lo;
    }
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        if (k * THREADS >= nvec) break;
        const int q = threadIdx.x + k * THREADS;
        size_t a = a_lo + 4 * (size_t)(q < nvec ? q : 0);
        a = a <= a_last ? a : a_last;
        v[k] = ld4_stream(p + a);
    }
    for (int k = 0; k < VEC; ++k) {
        if (k * THREADS >= nvec) break;
        const int q = threadIdx.x + k * THREADS;
        const size_t a = a_lo + 4 * (size_t)q;
        if (q < nvec && a <= a_last) *reinterpret_cast<float4*>(dst_lds + 4 * q) = v[k];
        if (q < nvec && a > a_last)
            for (int j = 0; j < 4; ++j)
                if (a + j < total) dst_lds[4 * q + j] = p[a + j];
    }
    return a_lo;
}

extern __shared__ float4 bwd_dyn_lds[];             // 16-byte aligned dynamic LDS, sized by the launch

// LDS: [ input rows, later the results | gradient rows | position of each window's first maximum (maximum only) ]
// Phase A (maximum): one lane per window finds its first maximum once.  Phase B: a lane takes four
// consecutive input elements, adds up the gradients of the windows that own each (one LDS compare per
// window instead of a re-scan), and stores 128 bits.
template <int MODE, int KH, int KW, int SH, int SW>
__global__ __launch_bounds__(kBwdThreads) void pool_bwd_nchw_slab_kernel(
    const float* __restrict__ src, const float* __restrict__ ddst, float* __restrict__ dsrc, PoolGeom g,
    BwdSlabPlan plan, int x_floats, int gy_floats, FastDiv div_w, FastDiv div_plane_in, FastDiv div_wo,
    FastDiv div_plane_out, FastDiv div_cells_w, FastDiv div_cells_plane) {
    constexpr int VEC = kBwdSlabFloats / 4 / kBwdThreads + 1;
    float* slab = reinterpret_cast<float*>(bwd_dyn_lds);
    const int kh = KH ? KH : g.kh, kw = KW ? KW : g.kw, sh = SH ? SH : g.sh, sw = SW ? SW : g.sw;
    const uint32_t tile = xcd_contiguous_tile(blockIdx.x, gridDim.x);
    const int plane_in = g.H * g.W, plane_out = g.Ho * g.Wo;

    long long p0;
    int planes, h0, rows;
    if (plan.strips == 1) {
        p0 = (long long)tile * plan.planes_per_wg;
        const long long left = plan.total_planes - p0;
        planes = left < plan.planes_per_wg ? (int)left : plan.planes_per_wg;
        h0 = 0;
        rows = g.H;
    } else {
        p0 = tile / (uint32_t)plan.strips;
        planes = 1;
        h0 = (int)(tile % (uint32_t)plan.strips) * plan.rows_per_wg;
        rows = g.H - h0 < plan.rows_per_wg ? g.H - h0 : plan.rows_per_wg;
    }
    // windows (rows of ddst) that touch input rows [h0, h0 + rows)
    int i_lo, i_hi, tmp;
    window_range(h0, kh, sh, g.ph, g.Ho, i_lo, tmp);
    window_range(h0 + rows - 1, kh, sh, g.ph, g.Ho, tmp, i_hi);
    if (planes > 1) { i_lo = 0; i_hi = g.Ho - 1; }
    const bool have_windows = i_hi >= i_lo;
    float* gy_lds = slab + x_floats;                  // x_floats and gy_floats are multiples of 4
    int* amax_lds = reinterpret_cast<int*>(slab + x_floats + gy_floats);
    size_t gy_a_lo = 0, x_a_lo = 0;
    if (have_windows) {
        const size_t lo = (size_t)p0 * plane_out + (size_t)i_lo * g.Wo;
        const size_t hi = (size_t)(p0 + planes - 1) * plane_out + (size_t)(i_hi + 1) * g.Wo;
        gy_a_lo = stream_to_lds<VEC>(ddst, lo, hi, (size_t)plan.total_planes * plane_out, gy_lds);
        if (MODE == CNNMEM_POOL_MAX) {
            int xr_lo = i_lo * sh - g.ph, xr_hi = i_hi * sh - g.ph + kh;
            if (xr_lo < 0) xr_lo = 0;
            if (xr_hi > g.H) xr_hi = g.H;
            if (planes > 1) { xr_lo = 0; xr_hi = g.H; }
            const size_t xlo = (size_t)p0 * plane_in + (size_t)xr_lo * g.W;
            const size_t xhi = (size_t)(p0 + planes - 1) * plane_in + (size_t)xr_hi * g.W;
            x_a_lo = stream_to_lds<VEC>(src, xlo, xhi, (size_t)plan.total_planes * plane_in, slab);
        }
    }
    __syncthreads();
    // LDS index of element (plane p0, row 0, col 0) of x and of ddst
    const long long x_base = (long long)((size_t)p0 * plane_in) - (long long)x_a_lo;
    const long long gy_base = (long long)((size_t)p0 * plane_out) - (long long)gy_a_lo;

    if (MODE == CNNMEM_POOL_MAX && have_windows) {
        // phase A: window (pl, i, j), i in [i_lo, i_hi], flattened like its place in ddst
        const int win_rows = i_hi - i_lo + 1;
        const int n_win = planes > 1 ? planes * plane_out : win_rows * g.Wo;
        for (int v = threadIdx.x; v < n_win; v += kBwdThreads) {
            int pl = 0, rem = v;
            if (planes > 1) {
                pl = (int)fd_div((uint32_t)v, div_plane_out);
                rem = v - pl * plane_out;
            }
            const int il = (int)fd_div((uint32_t)rem, div_wo);
            const int j = rem - il * g.Wo;
            const int i = i_lo + il;
            const float* xs = slab + (x_base + (long long)pl * plane_in);
            float best = kNegInf;
            int where = -1;
            if (KH != 0 && g.ph == 0 && g.pw == 0) {
                // compile-time window without padding: every tap is inside the image
                const int base = (i * sh) * g.W + j * sw;
                best = xs[base];
                where = base;
#pragma unroll
                for (int y = 0; y < (KH ? KH : 1); ++y)
#pragma unroll
                    for (int x = 0; x < (KW ? KW : 1); ++x) {
                        if (y == 0 && x == 0) continue;
                        const float val = xs[base + y * g.W + x];
                        if (val > best) { best = val; where = base + y * g.W + x; }
                    }
            } else
            for (int y = 0; y < kh; ++y) {
                const int r = i * sh - g.ph + y;
                if (r < 0 || r >= g.H) continue;
                for (int x = 0; x < kw; ++x) {
                    const int q = j * sw - g.pw + x;
                    if (q < 0 || q >= g.W) continue;
                    const float val = xs[r * g.W + q];
                    if (where < 0 || val > best) { best = val; where = r * g.W + q; }
                }
            }
            amax_lds[gy_base + (long long)pl * plane_out + i * g.Wo + j] = where;
        }
        __syncthreads();
    }

    const int n_elems = planes * rows * g.W;          // planes > 1 implies rows == H
    const size_t out0 = (size_t)p0 * plane_in + (size_t)h0 * g.W;
    // phase B writes the input gradients into LDS over the input rows, which phase A was the last to read
    float* stage = slab;
    if (KH != 0 && KH == KW && SH == SW && g.ph == 0 && g.pw == 0) {
        // Compile-time square window without padding: a lane takes one S x S cell of inputs, the
        // inputs that share their NW x NW windows, reads those windows' gradients (and owners)
        // once, and writes S runs of S words.  Strips start on cell boundaries (launcher).
        constexpr int K = KH ? KH : 1, S = SH ? SH : 1;
        constexpr int NW = (K - 1) / S + 1;
        const int cells_w = (g.W + S - 1) / S;
        const int cell_rows = (rows + S - 1) / S;
        const int n_cells = planes * cell_rows * cells_w;
        const int ci0 = h0 / S;
        for (int v = threadIdx.x; v < n_cells; v += kBwdThreads) {
            // per_plane = cells of a whole plane (planes > 1 implies whole planes)
            const int pl = planes > 1 ? (int)fd_div((uint32_t)v, div_cells_plane) : 0;
            const int rem = v - pl * (int)div_cells_plane.d;
            const int cil = (int)fd_div((uint32_t)rem, div_cells_w);
            const int cj = rem - cil * cells_w;
            const int ci = ci0 + cil;
            const long long gofs = gy_base + (long long)pl * plane_out;
            float gyv[NW][NW];
            int own[NW][NW];
#pragma unroll
            for (int a = 0; a < NW; ++a)
#pragma unroll
                for (int b = 0; b < NW; ++b) {
                    const int i = ci - (NW - 1) + a, j = cj - (NW - 1) + b;
                    const bool ok = i >= 0 && i < g.Ho && j >= 0 && j < g.Wo;
                    gyv[a][b] = ok ? gy_lds[gofs + i * g.Wo + j] : 0.f;
                    own[a][b] = (ok && MODE == CNNMEM_POOL_MAX) ? amax_lds[gofs + i * g.Wo + j] : -1;
                }
            float* oplane = stage + (long long)pl * plane_in - (long long)h0 * g.W;
#pragma unroll
            for (int ey = 0; ey < S; ++ey) {
                const int h = S * ci + ey;
                if (h >= g.H) continue;
#pragma unroll
                for (int ex = 0; ex < S; ++ex) {
                    const int w = S * cj + ex;
                    if (w >= g.W) continue;
                    const int me = h * g.W + w;
                    float acc = 0.f;
#pragma unroll
                    for (int a = 0; a < NW; ++a)
#pragma unroll
                        for (int b = 0; b < NW; ++b) {
                            const int y = S * (NW - 1 - a) + ey, x = S * (NW - 1 - b) + ex;
                            if (y < K && x < K) {
                                if (MODE == CNNMEM_POOL_AVG) acc += gyv[a][b];
                                else if (own[a][b] == me) acc += gyv[a][b];
                            }
                        }
                    oplane[me] = MODE == CNNMEM_POOL_AVG ? acc * (1.0f / (float)(K * K)) : acc;
                }
            }
        }
    } else {
        // any window: one lane per input element
        for (int o = threadIdx.x; o < n_elems; o += kBwdThreads) {
            int pl = 0, rem = o;
            if (planes > 1) {
                pl = (int)fd_div((uint32_t)o, div_plane_in);
                rem = o - pl * plane_in;
            }
            const int hl = (int)fd_div((uint32_t)rem, div_w);
            const int w = rem - hl * g.W;
            const int h = h0 + hl;
            int a_lo, a_hi, b_lo, b_hi;
            window_range(h, kh, sh, g.ph, g.Ho, a_lo, a_hi);
            window_range(w, kw, sw, g.pw, g.Wo, b_lo, b_hi);
            const long long gofs = gy_base + (long long)pl * plane_out;
            const int me = h * g.W + w;
            float acc = 0.f;
            for (int i = a_lo; i <= a_hi; ++i)
                for (int j = b_lo; j <= b_hi; ++j) {
                    const float gyv = gy_lds[gofs + i * g.Wo + j];
                    if (MODE == CNNMEM_POOL_AVG) acc += gyv;
                    else if (amax_lds[gofs + i * g.Wo + j] == me) acc += gyv;
                }
            stage[o] = MODE == CNNMEM_POOL_AVG ? acc / (float)(kh * kw) : acc;
        }
    }
    __syncthreads();
    // phase C: the workgroup's gradients leave as one contiguous run, 128 bits per lane, each
    // wavefront's 1 KB starting on a line of dsrc
    const int lead = (int)(((reinterpret_cast<uintptr_t>(dsrc) >> 2) + out0) & 31);
    for (int o = 4 * (int)threadIdx.x - lead; o < n_elems; o += 4 * kBwdThreads) {
        float* q = dsrc + out0 + o;
        if (o >= 0 && o + 4 <= n_elems) {
            st4_stream(q, make_float4(stage[o], stage[o + 1], stage[o + 2], stage[o + 3]));
        } else {
            for (int e = 0; e < 4; ++e)
                if (o + e >= 0 && o + e < n_elems) q[e] = stage[o + e];
        }
    }
}

// ---- NCHW average, 3x3 / stride 2 without padding (the overlapped pooling of the paper's networks) -------
// The slab kernel above is bound by instruction issue, not by memory: a division and a dozen clamps per element
// on the vector side, and as much loop and address arithmetic on the scalar side.  Here
//   * the lanes of a wavefront are the columns of one row (of 64 / LW rows for planes narrower than 33 columns,
//     LW the next power of two), so what depends on the column is computed once per lane;
//   * what depends on the row is computed once per workgroup, 64 rows per instruction, and left in LDS as a
//     table of descriptors (LDS indices): the inner loop reads a descriptor, adds the lane's column and goes.
//     Window rows that do not exist point at a row of zeros, results that must not be kept at a trash row: the
//     loop has no conditions (14 vector, 5 scalar and 5 LDS instructions per pair of rows);
//   * a lane gathers one pair of input rows (2u, 2u+1) of its column: both rows lie in window row u, the even one
//     also in u-1, so four gradients serve two elements.
// The maximum takes the same structure with a lane per window (pool_bwd_max_nchw_k3s2_kernel below).
constexpr int kRowThreads = 256;
constexpr int kRowGyVecs = 3, kRowXVecs = 8;      // float4 per lane a workgroup's gradient rows / input rows may take
struct RowsLds {                // LDS layout in floats; the staged result starts at 0
    int gy_at;                  // gradient rows
    int zero_at, trash_at;      // a row of zeros (Wo + 35 floats), a row nobody reads (W + 4 floats)
    int desc_at;                // descriptors, four ints each
    int ntab;                   // descriptors: row pairs, whole rounds of the workgroup
    int lanes_per_row;          // LW
};

__global__ __launch_bounds__(kRowThreads) void pool_bwd_avg_nchw_k3s2_kernel(
    const float* __restrict__ ddst, float* __restrict__ dsrc, PoolGeom g, BwdSlabPlan plan, RowsLds at, FastDiv div_pairs,
    FastDiv div_strips) {
    constexpr int kWaves = kRowThreads / 64;
    float* slab = reinterpret_cast<float*>(bwd_dyn_lds);
    const int H = g.H, W = g.W, Ho = g.Ho, Wo = g.Wo;
    const int plane_in = H * W, plane_out = Ho * Wo;
    const uint32_t total_planes = (uint32_t)plan.total_planes;         // the tensors have fewer than 2^31 elements (launcher)
    // neighbours share cache lines of the gradients (planes are not whole lines, strips share rows): one XCD
    const uint32_t tile = xcd_contiguous_tile(blockIdx.x, gridDim.x);
    uint32_t p0;
    int planes, h0, rows;
    if (plan.strips == 1) {
        p0 = tile * (uint32_t)plan.planes_per_wg;
        const uint32_t left = total_planes - p0;
        planes = left < (uint32_t)plan.planes_per_wg ? (int)left : plan.planes_per_wg;
        h0 = 0;
        rows = H;
    } else {
        p0 = fd_div(tile, div_strips);
        planes = 1;
        h0 = (int)(tile - p0 * (uint32_t)plan.strips) * plan.rows_per_wg;        // even (launcher)
        rows = H - h0 < plan.rows_per_wg ? H - h0 : plan.rows_per_wg;
    }
    // window rows that touch input rows [h0, h0 + rows): at least one (H >= 3, h0 even)
    const int i_lo = h0 >= 2 ? (h0 >> 1) - 1 : 0;
    const int i_hi = ((h0 + rows - 1) >> 1) < Ho - 1 ? (h0 + rows - 1) >> 1 : Ho - 1;
    const int n_elems = planes * rows * W;
    const uint32_t out0 = p0 * (uint32_t)plane_in + (uint32_t)(h0 * W);
    // element o of the workgroup's run sits at stage[o], placed so that the float4 a lane stores at the end
    // (o = 4*lane - lead) is one aligned 128-bit LDS read
    const int lead = (int)((((uint32_t)reinterpret_cast<uintptr_t>(dsrc) >> 2) + out0) & 31u);
    const int stage_at = lead & 3;
    int4* desc = reinterpret_cast<int4*>(slab + at.desc_at);

    // ---- gradient rows on their way: floats [lo, hi) of ddst land so that element e sits at slab[gy_at + e - a_lo],
    // a_lo the 128-byte (else 16-byte) aligned start at or below lo; up to kRowGyVecs float4 per lane ----
    const uint32_t total_out = total_planes * (uint32_t)plane_out;
    const uint32_t lo = p0 * (uint32_t)plane_out + (uint32_t)(i_lo * Wo);
    const uint32_t hi = (p0 + planes - 1) * (uint32_t)plane_out + (uint32_t)((i_hi + 1) * Wo);
    const uint32_t a_lo = lo & ~((reinterpret_cast<uintptr_t>(ddst) & 127u) == 0 ? 31u : 3u);
    const uint32_t nvec = (hi - a_lo + 3) >> 2;                    // <= kRowGyVecs * kRowThreads (launcher)
    const uint32_t a_last = (total_out - 4) & ~3u;                 // the last float4 that ends inside the tensor
    float4 v[kRowGyVecs];
#pragma unroll
    for (int k = 0; k < kRowGyVecs; ++k) {
        if ((uint32_t)(k * kRowThreads) >= nvec) break;             // uniform
        const uint32_t q = threadIdx.x + k * kRowThreads;
        const uint32_t a = a_lo + 4 * (q < nvec ? q : nvec - 1);
        v[k] = ld4_stream(ddst + (a <= a_last ? a : a_last));
    }

    // ---- descriptors and the row of zeros while the loads are in flight ----
    // slab index of element (plane p0, window row 0, column 0) of ddst
    const int gy_base = at.gy_at + (int)(p0 * (uint32_t)plane_out - a_lo);
    const int pairs = (rows + 1) >> 1, n_pairs = planes * pairs, u0 = h0 >> 1;
    for (int t = threadIdx.x; t < at.ntab; t += kRowThreads) {
        const bool valid = t < n_pairs;
        const int tv = valid ? t : 0;
        const int pl = planes > 1 ? (int)fd_div((uint32_t)tv, div_pairs) : 0;
        const int ul = tv - pl * pairs, u = u0 + ul;
        const int rows_at = gy_base + pl * plane_out;
        int4 d;
        d.x = u >= 1 ? rows_at + (u - 1) * Wo : at.zero_at + 1;         // window row u-1 (u-1 < Ho always)
        d.y = u < Ho ? rows_at + u * Wo : at.zero_at + 1;               // window row u
        d.z = valid ? stage_at + (pl * rows + 2 * ul) * W : at.trash_at;
        d.w = valid && 2 * ul + 1 < rows ? d.z + W : at.trash_at;
        desc[t] = d;
    }
    for (int q = threadIdx.x; q < Wo + 3; q += kRowThreads) slab[at.zero_at + q] = 0.f;
#pragma unroll
    for (int k = 0; k < kRowGyVecs; ++k) {
        if ((uint32_t)(k * kRowThreads) >= nvec) break;
        const uint32_t q = threadIdx.x + k * kRowThreads;
        const uint32_t a = a_lo + 4 * q;
        if (q < nvec) {
            if (a <= a_last) {
                *reinterpret_cast<float4*>(slab + at.gy_at + 4 * q) = v[k];
            } else {                                                // the float4 that crosses the end of the tensor
                for (uint32_t e = 0; e < 4; ++e)
                    if (a + e < total_out) slab[at.gy_at + 4 * q + e] = ddst[a + e];
            }
        }
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int LW = at.lanes_per_row;
    const int SUB = 64 / LW, sub = lane / LW, step = kWaves * SUB;
    const float inv = 1.0f / 9.0f;
    for (int w = lane & (LW - 1); w < ((W + 63) & ~63); w += 64) {
        // column w lies in window column (w-1)>>1 and, when even, in the next one; both are read whatever they
        // are (the float before a row and the one after it are inside the LDS allocation)
        const int jb = (w - 1) >> 1;
        const bool j0_ok = jb >= 0 && jb < Wo, j1_ok = (w & 1) == 0 && jb + 1 < Wo;
        if (w < W) {
            for (int base = wave * SUB; base < at.ntab; base += step) {
                const int4 d = desc[base + sub];
                const float* pa = slab + d.x + jb;
                const float* pb = slab + d.y + jb;
                const float a0 = pa[0], a1 = pa[1], b0 = pb[0], b1 = pb[1];
                const float ta = (j0_ok ? a0 : 0.f) + (j1_ok ? a1 : 0.f);
                const float tb = (j0_ok ? b0 : 0.f) + (j1_ok ? b1 : 0.f);
                slab[d.z + w] = (ta + tb) * inv;
                slab[d.w + w] = tb * inv;
            }
        }
    }
    __syncthreads();
    // the workgroup's gradients leave as one contiguous run, 128 bits per lane, each wavefront's 1 KB starting
    // on a line of dsrc
    const float* stage = slab + stage_at;
    for (int o = 4 * (int)threadIdx.x - lead; o < n_elems; o += 4 * kRowThreads) {
        float* q = dsrc + out0 + o;
        if (o >= 0 && o + 4 <= n_elems) {
            st4_stream(q, *reinterpret_cast<const float4*>(stage + o));
        } else {
            for (int e = 0; e < 4; ++e)
                if (o + e >= 0 && o + e < n_elems) q[e] = stage[o + e];
        }
    }
}

// ---- NCHW maximum, 3x3 / stride 2 without padding: the same shape of kernel -----------------------------
// A lane owns a window: it finds the window's first maximum among the nine taps in LDS and adds the window's
// gradient to that element of the staged result.  Windows two rows (or two columns) apart share no input, so even
// window rows go first, a barrier, then odd ones; inside a row the even columns go first, then the odd ones (same
// wavefront, program order): no atomics, and the order of the at most four additions of an element is fixed.
// Both streams (input rows, gradient rows) are requested before the table is built.  128x96x55x55: 65-69 us in the
// slab kernel, 61 us here (256 lanes, one plane per workgroup; 512 lanes 63 us; strips of 28 rows 64 us, of 14 rows
// 98 us: a workgroup's piece must not get small).
// LDS: [ input rows | gradient rows | staged result | descriptors ]
struct MaxRowsLds {
    int gy_at, stage_at, desc_at;
    int ntab0, ntab1;           // descriptors of the even and of the odd window rows, whole rounds of the workgroup
    int lanes_per_row;          // LW, for window rows
};

__global__ __launch_bounds__(kRowThreads) void pool_bwd_max_nchw_k3s2_kernel(
    const float* __restrict__ src, const float* __restrict__ ddst, float* __restrict__ dsrc, PoolGeom g, BwdSlabPlan plan,
    MaxRowsLds at, FastDiv div_even, FastDiv div_odd, FastDiv div_strips) {
    constexpr int THREADS = kRowThreads, kWaves = THREADS / 64;
    constexpr int GV = kRowGyVecs, XV = kRowXVecs;                // float4 per lane that a workgroup's streams may take
    float* slab = reinterpret_cast<float*>(bwd_dyn_lds);
    const int H = g.H, W = g.W, Ho = g.Ho, Wo = g.Wo;
    const int plane_in = H * W, plane_out = Ho * Wo;
    const uint32_t total_planes = (uint32_t)plan.total_planes;         // the tensors have fewer than 2^31 elements (launcher)
    const uint32_t tile = xcd_contiguous_tile(blockIdx.x, gridDim.x);
    uint32_t p0;
    int planes, h0, rows;
    if (plan.strips == 1) {
        p0 = tile * (uint32_t)plan.planes_per_wg;
        const uint32_t left = total_planes - p0;
        planes = left < (uint32_t)plan.planes_per_wg ? (int)left : plan.planes_per_wg;
        h0 = 0;
        rows = H;
    } else {
        p0 = fd_div(tile, div_strips);
        planes = 1;
        h0 = (int)(tile - p0 * (uint32_t)plan.strips) * plan.rows_per_wg;        // even (launcher)
        rows = H - h0 < plan.rows_per_wg ? H - h0 : plan.rows_per_wg;
    }
    // window rows that touch input rows [h0, h0 + rows): at least one (H >= 3, h0 even)
    const int i_lo = h0 >= 2 ? (h0 >> 1) - 1 : 0;
    const int i_hi = ((h0 + rows - 1) >> 1) < Ho - 1 ? (h0 + rows - 1) >> 1 : Ho - 1;
    const int xr_lo = planes > 1 ? 0 : 2 * i_lo, xr_hi = planes > 1 ? H : 2 * i_hi + 3;         // inside the image
    const int n_elems = planes * rows * W;
    const uint32_t out0 = p0 * (uint32_t)plane_in + (uint32_t)(h0 * W);
    const int lead = (int)((((uint32_t)reinterpret_cast<uintptr_t>(dsrc) >> 2) + out0) & 31u);
    const int stage_at = at.stage_at + (lead & 3);
    int4* desc = reinterpret_cast<int4*>(slab + at.desc_at);

    // ---- both streams on their way (element e of a stream lands at its part's start + e - a_lo) ----
    const uint32_t total_out = total_planes * (uint32_t)plane_out, total_in = total_planes * (uint32_t)plane_in;
    const uint32_t g_lo = p0 * (uint32_t)plane_out + (uint32_t)(i_lo * Wo);
    const uint32_t g_hi = (p0 + planes - 1) * (uint32_t)plane_out + (uint32_t)((i_hi + 1) * Wo);
    const uint32_t g_alo = g_lo & ~((reinterpret_cast<uintptr_t>(ddst) & 127u) == 0 ? 31u : 3u);
    const uint32_t g_nvec = (g_hi - g_alo + 3) >> 2, g_alast = (total_out - 4) & ~3u;
    const uint32_t x_lo = p0 * (uint32_t)plane_in + (uint32_t)(xr_lo * W);
    const uint32_t x_hi = (p0 + planes - 1) * (uint32_t)plane_in + (uint32_t)(xr_hi * W);
    const uint32_t x_alo = x_lo & ~((reinterpret_cast<uintptr_t>(src) & 127u) == 0 ? 31u : 3u);
    const uint32_t x_nvec = (x_hi - x_alo + 3) >> 2, x_alast = (total_in - 4) & ~3u;
    float4 gv[GV], xv[XV];
#pragma unroll
    for (int k = 0; k < GV; ++k) {
        if ((uint32_t)(k * THREADS) >= g_nvec) break;             // uniform
        const uint32_t q = threadIdx.x + k * THREADS;
        const uint32_t a = g_alo + 4 * (q < g_nvec ? q : g_nvec - 1);
        gv[k] = ld4_stream(ddst + (a <= g_alast ? a : g_alast));
    }
#pragma unroll
    for (int k = 0; k < XV; ++k) {
        if ((uint32_t)(k * THREADS) >= x_nvec) break;
        const uint32_t q = threadIdx.x + k * THREADS;
        const uint32_t a = x_alo + 4 * (q < x_nvec ? q : x_nvec - 1);
        xv[k] = ld4_stream(src + (a <= x_alast ? a : x_alast));
    }

    // ---- descriptors and the cleared stage while the loads are in flight ----
    const int gy_base = at.gy_at + (int)(p0 * (uint32_t)plane_out - g_alo);       // slab index of (plane p0, window row 0, col 0)
    const int x_base = (int)(p0 * (uint32_t)plane_in - x_alo);
    for (int t = threadIdx.x; t < at.ntab0 + at.ntab1; t += THREADS) {
        const int parity = t >= at.ntab0 ? 1 : 0;
        const int k_flat = t - (parity ? at.ntab0 : 0);
        // window rows i_lo <= i <= i_hi with i % 2 == parity, of every plane
        const int first = i_lo + (((i_lo & 1) != parity) ? 1 : 0);
        const int count = first <= i_hi ? (i_hi - first) / 2 + 1 : 0;
        const bool valid = k_flat < planes * count;
        const int kv = valid ? k_flat : 0;
        const int pl = planes > 1 ? (int)fd_div((uint32_t)kv, parity ? div_odd : div_even) : 0;
        const int i = (count > 0 ? first : i_lo) + 2 * (kv - pl * count);
        int4 d;
        d.x = x_base + pl * plane_in + 2 * i * W;                       // first tap row of the window row
        d.y = gy_base + pl * plane_out + i * Wo;
        d.z = stage_at + (pl * rows - h0 + 2 * i) * W;                  // that tap row in the staged result
        d.w = valid ? (2 * i - h0) * W : -(1 << 30);                    // ... and inside the plane's part of the run
        desc[t] = d;
    }
    {
        const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int q = threadIdx.x; q < (n_elems + 6) / 4; q += THREADS) reinterpret_cast<float4*>(slab + at.stage_at)[q] = zero;
    }
#pragma unroll
    for (int k = 0; k < GV; ++k) {
        if ((uint32_t)(k * THREADS) >= g_nvec) break;
        const uint32_t q = threadIdx.x + k * THREADS;
        const uint32_t a = g_alo + 4 * q;
        if (q < g_nvec) {
            if (a <= g_alast) *reinterpret_cast<float4*>(slab + at.gy_at + 4 * q) = gv[k];
            else
                for (uint32_t e = 0; e < 4; ++e)
                    if (a + e < total_out) slab[at.gy_at + 4 * q + e] = ddst[a + e];
        }
    }
#pragma unroll
    for (int k = 0; k < XV; ++k) {
        if ((uint32_t)(k * THREADS) >= x_nvec) break;
        const uint32_t q = threadIdx.x + k * THREADS;
        const uint32_t a = x_alo + 4 * q;
        if (q < x_nvec) {
            if (a <= x_alast) *reinterpret_cast<float4*>(slab + 4 * q) = xv[k];
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
    const unsigned run_of_plane = (unsigned)(rows * W);
    for (int parity = 0; parity < 2; ++parity) {
        const int tab = parity ? at.ntab0 : 0, ntab = parity ? at.ntab1 : at.ntab0;
        for (int j = lane & (LW - 1); j < ((Wo + 63) & ~63); j += 64) {
            const bool col_ok = j < Wo;
            const int jc = col_ok ? j : Wo - 1;
            const bool even_col = (j & 1) == 0;
            for (int base = wave * SUB; base < ntab; base += step) {
                const int4 d = desc[tab + base + sub];
                const float* xp = slab + d.x + 2 * jc;
                float best = xp[0];
                int off = 0;
#pragma unroll
                for (int y = 0; y < 3; ++y)
#pragma unroll
                    for (int x = 0; x < 3; ++x) {
                        if (y == 0 && x == 0) continue;
                        const float val = xp[y * W + x];
                        if (val > best) { best = val; off = y * W + x; }
                    }
                const float gyv = slab[d.y + jc];
                const int t = 2 * jc + off;
                const bool ok = col_ok && (unsigned)(d.w + t) < run_of_plane;
                // neighbouring lanes may name the same element: even columns first, then odd ones, as two separate
                // LDS read-modify-writes of the wavefront (the fences keep the compiler from merging them or moving
                // the second read above the first write)
                float* out = slab + d.z + t;
                if (ok && even_col) *out += gyv;
                asm volatile("" ::: "memory");
                __builtin_amdgcn_wave_barrier();
                asm volatile("" ::: "memory");
                if (ok && !even_col) *out += gyv;
            }
        }
        __syncthreads();
    }
    const float* stage = slab + stage_at;
    for (int o = 4 * (int)threadIdx.x - lead; o < n_elems; o += 4 * THREADS) {
        float* q = dsrc + out0 + o;
        if (o >= 0 && o + 4 <= n_elems) {
            st4_stream(q, *reinterpret_cast<const float4*>(stage + o));
        } else {
            for (int e = 0; e < 4; ++e)
                if (o + e >= 0 && o + e < n_elems) q[e] = stage[o + e];
        }
    }
}

// ---- NCHW, 2x2 / stride 2, no padding, even H, W a multiple of 4 ------------------------
// Rows pair up across the whole tensor, every input belongs to exactly one window: a lane
// takes one float4 of both rows of a pair (two windows) and the two gradients above them.
template <int MODE>
__global__ __launch_bounds__(kThreads) void pool_bwd_nchw_2x2s2_kernel(
    const float* __restrict__ src, const float* __restrict__ ddst, float* __restrict__ dsrc, uint32_t items,
    uint32_t W, FastDiv div_per_row) {
    const uint32_t I = blockIdx.x * kThreads + threadIdx.x;
    if (I >= items) return;
    const uint32_t orow = fd_div(I, div_per_row);
    const size_t in0 = (size_t)I * 4 + (size_t)orow * W;       // = 2*orow*W + 4*(I % per_row)
    const v2f_t gy = __builtin_nontemporal_load(reinterpret_cast<const v2f_t*>(ddst + (size_t)I * 2));
    float4 da, db;
    if (MODE == CNNMEM_POOL_AVG) {
        const float g0 = gy.x * 0.25f, g1 = gy.y * 0.25f;
        da = make_float4(g0, g0, g1, g1);
        db = da;
    } else {
        const float4 a = ld4_stream(src + in0), b = ld4_stream(src + in0 + W);
        // scan order inside a window: a.x, a.y, b.x, b.y (then a.z, a.w, b.z, b.w); the first maximum wins
        {
            float best = a.x; int k = 0;
            if (a.y > best) { best = a.y; k = 1; }
            if (b.x > best) { best = b.x; k = 2; }
            if (b.y > best) { best = b.y; k = 3; }
            da.x = k == 0 ? gy.x : 0.f; da.y = k == 1 ? gy.x : 0.f;
            db.x = k == 2 ? gy.x : 0.f; db.y = k == 3 ? gy.x : 0.f;
        }
        {
            float best = a.z; int k = 0;
            if (a.w > best) { best = a.w; k = 1; }
            if (b.z > best) { best = b.z; k = 2; }
            if (b.w > best) { best = b.w; k = 3; }
            da.z = k == 0 ? gy.y : 0.f; da.w = k == 1 ? gy.y : 0.f;
            db.z = k == 2 ? gy.y : 0.f; db.w = k == 3 ? gy.y : 0.f;
        }
    }
    if (MODE == CNNMEM_POOL_AVG) {                  // write-heavy: write-through stores, 179 -> 159 us on 64x64x224x224
        st4_through(dsrc + in0, da);
        st4_through(dsrc + in0 + W, db);
    } else {
        st4_stream(dsrc + in0, da);
        st4_stream(dsrc + in0 + W, db);
    }
}

template <int MODE>
int launch_bwd_generic(const float* src, const float* ddst, float* dsrc, const PoolGeom& g, int chwn, hipStream_t st) {
    const size_t total = (size_t)g.N * g.C * g.H * g.W;
    const long long want = ceil_div64((long long)total, kThreads);
    const unsigned blocks = (unsigned)(want < (1 << 20) ? want : (1 << 20));
    hipLaunchKernelGGL((pool_bwd_generic_kernel<MODE>), dim3(blocks), dim3(kThreads), 0, st, src, ddst, dsrc, g, chwn,
                       total);
    return launch_status();
}

template <int MODE, int KH, int KW, int SH, int SW>
int launch_bwd_chwn(const float* src, const float* ddst, float* dsrc, const PoolGeom& g, hipStream_t st) {
    const long long items = (long long)g.C * g.H * g.W * (g.N / 4);
    const FastDiv dn4 = make_fastdiv((uint32_t)(g.N / 4)), dw = make_fastdiv((uint32_t)g.W),
                  dh = make_fastdiv((uint32_t)g.H);
    hipLaunchKernelGGL((pool_bwd_chwn_vec4_kernel<MODE, KH, KW, SH, SW>), dim3((unsigned)ceil_div64(items, kThreads)),
                       dim3(kThreads), 0, st, src, ddst, dsrc, g, (uint32_t)items, dn4, dw, dh);
    return launch_status();
}

template <int MODE, int K, int S>
int launch_bwd_chwn_cell(const float* src, const float* ddst, float* dsrc, const PoolGeom& g, hipStream_t st) {
    const long long cells_h = ceil_div64(g.H, S), cells_w = ceil_div64(g.W, S);
    const long long items = (long long)g.C * cells_h * cells_w * (g.N / 4);
    if (items >= 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    // occupancy cap on large tensors with disjoint windows (64x64x224x224 2x2/s2: the average goes from 74.7 % of
    // peak uncapped to 84.9 % at 4 workgroups per CU, the maximum from 71.1 % to 72.8 % at 3)
    const size_t lds = K <= S ? throttle_lds(env_int("CNNMEM_BWD_WPC", 0), 4LL * g.N * g.C * g.H * g.W,
                                             MODE == CNNMEM_POOL_AVG ? 4 : 3) : 0;
    hipLaunchKernelGGL((pool_bwd_chwn_cell_kernel<MODE, K, S>), dim3((unsigned)ceil_div64(items, kThreads)),
                       dim3(kThreads), lds, st, src, ddst, dsrc, g, (uint32_t)items, make_fastdiv((uint32_t)(g.N / 4)),
                       make_fastdiv((uint32_t)cells_w), make_fastdiv((uint32_t)cells_h));
    return launch_status();
}

// maximum, overlapping windows, N a multiple of 32: patches of 4 x 8 cells of 32 images through LDS (patches of
// 4 x 4 or 4 x 8 cells of 64 images and 2 x 4 cells of 128 images measured the same or 5 % slower)
template <int K, int S>
int launch_bwd_chwn_patch(const float* src, const float* ddst, float* dsrc, const PoolGeom& g, hipStream_t st) {
    constexpr int CR = 4, CQ = 8, NB4 = 8;
    const long long cells_h = ceil_div64(g.H, S), cells_w = ceil_div64(g.W, S);
    const long long ph = ceil_div64(cells_h, CR), pw = ceil_div64(cells_w, CQ), chunks = g.N / (4 * NB4);
    const long long blocks = (long long)g.C * ph * pw * chunks;
    if (blocks >= 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    if (env_int("CNNMEM_BWD_PATCH", 2) == 2)
        hipLaunchKernelGGL((pool_bwd_chwn_patch_kernel<K, S, CR, CQ, NB4, true>), dim3((unsigned)blocks),
                           dim3(CR * CQ * NB4), 0, st, src, ddst, dsrc, g, (uint32_t)pw, (uint32_t)ph, (uint32_t)chunks,
                           make_fastdiv((uint32_t)chunks), make_fastdiv((uint32_t)pw), make_fastdiv((uint32_t)ph));
    else
        hipLaunchKernelGGL((pool_bwd_chwn_patch_kernel<K, S, CR, CQ, NB4, false>), dim3((unsigned)blocks),
                           dim3(CR * CQ * NB4), 0, st, src, ddst, dsrc, g, (uint32_t)pw, (uint32_t)ph, (uint32_t)chunks,
                           make_fastdiv((uint32_t)chunks), make_fastdiv((uint32_t)pw), make_fastdiv((uint32_t)ph));
    return launch_status();
}

template <int MODE, int KH, int KW, int SH, int SW>
int launch_bwd_slab(const float* src, const float* ddst, float* dsrc, const PoolGeom& g, const BwdSlabPlan& plan,
                    int x_floats, int gy_floats, long long blocks, hipStream_t st) {
    const size_t lds = sizeof(float) * (size_t)(x_floats + gy_floats * (MODE == CNNMEM_POOL_MAX ? 2 : 1));
    hipLaunchKernelGGL((pool_bwd_nchw_slab_kernel<MODE, KH, KW, SH, SW>), dim3((unsigned)blocks), dim3(kBwdThreads), lds,
                       st, src, ddst, dsrc, g, plan, x_floats, gy_floats, make_fastdiv((uint32_t)g.W),
                       make_fastdiv((uint32_t)(g.H * g.W)), make_fastdiv((uint32_t)g.Wo),
                       make_fastdiv((uint32_t)(g.Ho * g.Wo)), make_fastdiv((uint32_t)ceil_div(g.W, g.sw)),
                       make_fastdiv((uint32_t)(ceil_div(g.W, g.sw) * ceil_div(g.H, g.sh))));
    return launch_status();
}

// average, 3x3 / stride 2 without padding in NCHW: whole planes per workgroup, or strips of an even number of rows
int launch_bwd_avg_k3s2(const float* ddst, float* dsrc, const PoolGeom& g, hipStream_t st) {
    constexpr int kWaves = kRowThreads / 64;
    const long long planes = (long long)g.N * g.C;
    const long long plane_in = (long long)g.H * g.W, plane_out = (long long)g.Ho * g.Wo;
    // the streamed and the staged part may start up to 31 floats before their first element and are padded to float4
    auto part = [](long long floats) { return (long long)((floats + 32 + 3) / 4 * 4); };
    auto round_up = [](long long v, long long m) { return (v + m - 1) / m * m; };
    int lanes_per_row = 64;
    while (lanes_per_row / 2 >= g.W) lanes_per_row /= 2;
    const long long step = kWaves * (64 / lanes_per_row);          // row pairs per round of the workgroup
    // LDS layout for a staged result of out_f floats, gy_f gradient floats and `tasks` row pairs; the floats needed
    auto layout = [&](long long out_f, long long gy_f, long long tasks, RowsLds& at) {
        long long o = part(out_f);
        at.gy_at = (int)o; o += part(gy_f);
        at.zero_at = (int)o; o += round_up(g.Wo + 3, 4);
        at.trash_at = (int)o; o += round_up(g.W + 4, 4);
        at.desc_at = (int)o;
        at.ntab = (int)round_up(tasks, step);
        at.lanes_per_row = lanes_per_row;
        if (part(gy_f) > 4LL * kRowThreads * kRowGyVecs) return 1LL << 40;        // more than the lanes' registers take
        return o + 4LL * at.ntab;
    };
    auto planes_need = [&](long long q, RowsLds& at) {
        return layout(q * plane_in, q * plane_out, q * ((g.H + 1) / 2), at);
    };
    // a strip of r input rows (r even): its windows span at most r / 2 + 2 gradient rows
    auto strip_need = [&](long long r, RowsLds& at) {
        const long long gr = r / 2 + 2 < g.Ho ? r / 2 + 2 : g.Ho;
        return layout(r * g.W, gr * g.Wo, (r + 1) / 2, at);
    };
    auto busy = [](long long work, long long slots) {
        return (double)work / (double)(ceil_div64(work, slots) * slots);
    };
    BwdSlabPlan plan;
    plan.total_planes = planes;
    RowsLds at, probe;
    long long blocks = 0, lds_floats = 0;
    int preferred = env_int("CNNMEM_BWD_SLAB_FLOATS", 8192);
    if (preferred < 1024 || preferred > kBwdSlabFloats) preferred = kBwdSlabFloats;
    if (planes_need(1, probe) <= kBwdSlabFloats) {
        // Planes per workgroup: among the counts that fit the preferred size (32 KB) and leave at least 2048
        // workgroups, the one that keeps the lanes busiest over the passes (more LDS per workgroup means fewer
        // wavefronts per CU: 128x96x55x55 runs in 39 us with one or two planes, in 46 us with three).
        const long long budget = planes_need(1, probe) <= preferred ? preferred : kBwdSlabFloats;
        long long p = 1;
        double best = -1.0;
        for (long long q = 1; q <= planes && planes_need(q, probe) <= budget; ++q) {
            if (q > 1 && planes / q < 2048) break;
            const double score = busy(q * plane_in / 4 + 1, kRowThreads) * busy(q * ((g.H + 1) / 2), step);
            if (score > best + 0.02) { best = score; p = q; }         // prefer the smaller count on near ties
        }
        plan.planes_per_wg = (int)p;
        plan.rows_per_wg = g.H;
        plan.strips = 1;
        blocks = ceil_div64(planes, p);
        lds_floats = planes_need(p, at);
    } else {
        long long r = g.H / 2 * 2;
        while (r > 2 && strip_need(r, probe) > preferred) r -= 2;
        if (r < 8) {                                    // wide rows: take the large size
            r = g.H / 2 * 2;
            while (r > 2 && strip_need(r, probe) > kBwdSlabFloats) r -= 2;
        }
        if (r < 2 || strip_need(r, probe) > kBwdSlabFloats) return CNNMEM_ERR_UNSUPPORTED;
        plan.planes_per_wg = 1;
        plan.rows_per_wg = (int)r;
        plan.strips = ceil_div(g.H, r);
        blocks = planes * plan.strips;
        lds_floats = strip_need(r, at);
    }
    if (blocks > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(pool_bwd_avg_nchw_k3s2_kernel, dim3((unsigned)blocks), dim3(kRowThreads),
                       sizeof(float) * (size_t)lds_floats, st, ddst, dsrc, g, plan, at,
                       make_fastdiv((uint32_t)((g.H + 1) / 2)), make_fastdiv((uint32_t)plan.strips));
    return launch_status();
}

// maximum, 3x3 / stride 2 without padding in NCHW: whole planes per workgroup, or strips of an even number of rows
int launch_bwd_max_k3s2(const float* src, const float* ddst, float* dsrc, const PoolGeom& g, hipStream_t st) {
    constexpr int THREADS = kRowThreads, kWaves = THREADS / 64;
    const long long planes = (long long)g.N * g.C;
    const long long plane_in = (long long)g.H * g.W, plane_out = (long long)g.Ho * g.Wo;
    auto part = [](long long floats) { return (long long)((floats + 32 + 3) / 4 * 4); };
    auto round_up = [](long long v, long long m) { return (v + m - 1) / m * m; };
    int lanes_per_row = 64;
    while (lanes_per_row / 2 >= g.Wo) lanes_per_row /= 2;
    const long long step = kWaves * (64 / lanes_per_row);          // window rows per round of the workgroup
    auto layout = [&](long long out_f, long long gy_f, long long x_f, long long tasks0, long long tasks1, MaxRowsLds& at) {
        long long o = part(x_f);
        at.gy_at = (int)o; o += part(gy_f);
        at.stage_at = (int)o; o += part(out_f);
        at.desc_at = (int)o;
        at.ntab0 = (int)round_up(tasks0, step);
        at.ntab1 = (int)round_up(tasks1, step);
        at.lanes_per_row = lanes_per_row;
        // more than the lanes' registers take
        if (part(gy_f) > 4LL * THREADS * kRowGyVecs || part(x_f) > 4LL * THREADS * kRowXVecs) return 1LL << 40;
        return o + 4LL * (at.ntab0 + at.ntab1);
    };
    auto planes_need = [&](long long q, MaxRowsLds& at) {
        return layout(q * plane_in, q * plane_out, q * plane_in, q * ((g.Ho + 1) / 2), q * (g.Ho / 2), at);
    };
    // a strip of r input rows (r even): its windows span at most r + 4 input rows and r / 2 + 2 gradient rows, at most
    // r / 4 + 1 of them of one parity
    auto strip_need = [&](long long r, MaxRowsLds& at) {
        const long long xr = r + 4 < g.H ? r + 4 : g.H, gr = r / 2 + 2 < g.Ho ? r / 2 + 2 : g.Ho;
        return layout(r * g.W, gr * g.Wo, xr * g.W, r / 4 + 1, r / 4 + 1, at);
    };
    BwdSlabPlan plan;
    plan.total_planes = planes;
    MaxRowsLds at, probe;
    long long blocks = 0, lds_floats = 0;
    if (planes_need(1, probe) <= kBwdSlabFloats) {
        plan.planes_per_wg = 1;
        plan.rows_per_wg = g.H;
        plan.strips = 1;
        blocks = planes;
        lds_floats = planes_need(1, at);
    } else {
        long long r = g.H / 2 * 2;
        while (r > 2 && strip_need(r, probe) > kBwdSlabFloats) r -= 2;
        if (r < 2 || strip_need(r, probe) > kBwdSlabFloats) return CNNMEM_ERR_UNSUPPORTED;
        plan.planes_per_wg = 1;
        plan.rows_per_wg = (int)r;
        plan.strips = ceil_div(g.H, r);
        blocks = planes * plan.strips;
        lds_floats = strip_need(r, at);
    }
    if (blocks > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(pool_bwd_max_nchw_k3s2_kernel, dim3((unsigned)blocks), dim3(THREADS),
                       sizeof(float) * (size_t)lds_floats, st, src, ddst, dsrc, g, plan, at,
                       make_fastdiv((uint32_t)((g.Ho + 1) / 2)), make_fastdiv((uint32_t)(g.Ho / 2 > 0 ? g.Ho / 2 : 1)),
                       make_fastdiv((uint32_t)plan.strips));
    return launch_status();
}

template <int MODE>
int dispatch_pool_backward(const float* src, const float* ddst, float* dsrc, const PoolGeom& g, int layout,
                           hipStream_t st) {
    const bool a16 = aligned16(ddst) && aligned16(dsrc) && (MODE == CNNMEM_POOL_AVG || aligned16(src));
    const bool square = g.kh == g.kw && g.sh == g.sw && g.ph == 0 && g.pw == 0;
    if (layout == CNNMEM_CHWN) {
        const long long items = (long long)g.C * g.H * g.W * (g.N / 4);
        if (a16 && g.N % 4 == 0 && items < 0x7fffffffLL && g.kh <= 8 && g.kw <= 8) {
            if (square && g.kh == 3 && g.sh == 2) {
                if (MODE == CNNMEM_POOL_MAX && g.N % 32 == 0 && env_int("CNNMEM_BWD_PATCH", 1) != 0) {
                    const int rc = launch_bwd_chwn_patch<3, 2>(src, ddst, dsrc, g, st);
                    if (rc != CNNMEM_ERR_UNSUPPORTED) return rc;
                }
                return launch_bwd_chwn_cell<MODE, 3, 2>(src, ddst, dsrc, g, st);
            }
            if (square && g.kh == 2 && g.sh == 2) return launch_bwd_chwn_cell<MODE, 2, 2>(src, ddst, dsrc, g, st);
            if (g.kh == 3 && g.kw == 3 && g.sh == 2 && g.sw == 2)
                return launch_bwd_chwn<MODE, 3, 3, 2, 2>(src, ddst, dsrc, g, st);
            if (g.kh == 2 && g.kw == 2 && g.sh == 2 && g.sw == 2)
                return launch_bwd_chwn<MODE, 2, 2, 2, 2>(src, ddst, dsrc, g, st);
            return launch_bwd_chwn<MODE, 0, 0, 0, 0>(src, ddst, dsrc, g, st);
        }
        return launch_bwd_generic<MODE>(src, ddst, dsrc, g, 1, st);
    }
    const long long planes = (long long)g.N * g.C;
    if (a16 && g.kh == 2 && g.kw == 2 && g.sh == 2 && g.sw == 2 && g.ph == 0 && g.pw == 0 && g.H % 2 == 0 &&
        g.W % 4 == 0) {
        const long long per_row = g.W / 4;
        const long long items = planes * g.Ho * per_row;
        if (items < 0x7fffffffLL) {
            // the row-pair kernel gains at most a point from a cap (78.3 -> 79.4 %): left uncapped
            const size_t lds = throttle_lds(env_int("CNNMEM_BWD_WPC", -1), 4LL * planes * g.H * g.W, 5);
            hipLaunchKernelGGL((pool_bwd_nchw_2x2s2_kernel<MODE>), dim3((unsigned)ceil_div64(items, kThreads)),
                               dim3(kThreads), lds, st, src, ddst, dsrc, (uint32_t)items, (uint32_t)g.W,
                               make_fastdiv((uint32_t)per_row));
            return launch_status();
        }
    }
    const long long plane_in = (long long)g.H * g.W, plane_out = (long long)g.Ho * g.Wo;
    if (a16 && g.kh == 3 && g.kw == 3 && g.sh == 2 && g.sw == 2 && g.ph == 0 && g.pw == 0 &&
        plane_in * planes < (1LL << 31) && plane_out * planes >= 4 && env_int("CNNMEM_BWD_ROWS", 1) != 0) {
        const int rc = MODE == CNNMEM_POOL_AVG ? launch_bwd_avg_k3s2(ddst, dsrc, g, st)
                                               : launch_bwd_max_k3s2(src, ddst, dsrc, g, st);
        if (rc != CNNMEM_ERR_UNSUPPORTED) return rc;
    }
    // LDS slab: input rows, gradient rows and (maximum) one position per window share 60 KB
    if (a16 && plane_in * planes < (1LL << 40) && plane_in * planes >= 4 && plane_out * planes >= 4) {
        constexpr bool kMax = MODE == CNNMEM_POOL_MAX;
        // each streamed part may start up to 31 floats before its first element and is padded to float4
        auto part = [](long long floats) { return (int)((floats + 32 + 3) / 4 * 4); };
        BwdSlabPlan plan;
        plan.total_planes = planes;
        bool ok = false;
        long long blocks = 0;
        int x_floats = 0, gy_floats = 0;
        // the x part also stages the results, so the average needs it as well
        // 32 KB per workgroup measured best on MI355X (four 512-lane workgroups per CU); up to 60 KB
        // is accepted for planes that need it (CNNMEM_BWD_SLAB_FLOATS overrides for A/B runs)
        int cap = env_int("CNNMEM_BWD_SLAB_FLOATS", 8192);
        if (cap < 1024 || cap > kBwdSlabFloats) cap = kBwdSlabFloats;
        if (part(plane_in) + part(plane_out) * (kMax ? 2 : 1) > cap && g.H * (long long)g.W <= kBwdSlabFloats)
            cap = kBwdSlabFloats;                   // a whole plane does not fit the preferred size: take the large one
        auto fits = [&](long long xf, long long gf) { return part(xf) + part(gf) * (kMax ? 2 : 1) <= cap; };
        if (fits(plane_in, plane_out)) {
            // Planes per workgroup: among the counts that fit (up to 48 KB when the caller did not
            // ask otherwise) and leave at least 2048 workgroups, the one that keeps the 512 lanes
            // busiest over the phases (windows, cells or elements, 128-bit loads and stores).
            const int env_cap = env_int("CNNMEM_BWD_SLAB_FLOATS", 0);
            const long long roomy = env_cap > 0 ? cap : (cap > 12288 ? cap : 12288);
            auto fits_roomy = [&](long long q) {
                return part(q * plane_in) + part(q * plane_out) * (kMax ? 2 : 1) <= roomy;
            };
            auto busy = [&](long long work) {
                const long long rounds = ceil_div64(work, kBwdThreads);
                return (double)work / (double)(rounds * kBwdThreads);
            };
            const long long cells = (long long)ceil_div(g.H, g.sh) * ceil_div(g.W, g.sw);
            long long p = 1;
            double best = -1.0;
            for (long long q = 1; fits_roomy(q) && q <= planes; ++q) {
                if (q > 1 && planes / q < 2048) break;
                double score = busy(q * cells) * busy(q * plane_in / 4 + 1);
                if (kMax) score *= busy(q * plane_out);
                if (score > best + 0.02) { best = score; p = q; }     // prefer the smaller count on near ties
            }
            plan.planes_per_wg = (int)p;
            plan.rows_per_wg = g.H;
            plan.strips = 1;
            blocks = ceil_div64(planes, p);
            x_floats = part(p * plane_in);
            gy_floats = part(p * plane_out);
            ok = true;
        } else {
            // a strip of r input rows: its windows span at most r + 2*(kh - 1) input rows and
            // (r + kh - 2) / sh + 1 gradient rows
            auto xrows = [&](long long r) { return r + 2LL * (g.kh - 1) < g.H ? r + 2LL * (g.kh - 1) : (long long)g.H; };
            auto grows = [&](long long r) {
                const long long n = (r + g.kh - 2) / g.sh + 2;
                return n < g.Ho ? n : (long long)g.Ho;
            };
            long long rows = g.H;
            while (rows > 1 && !fits(xrows(rows) * g.W, grows(rows) * g.Wo)) rows = rows * 3 / 4;
            // whole cells of sh input rows per strip (the compile-time-window kernels work on cells)
            if (rows >= g.sh) rows = rows / g.sh * g.sh;
            if (fits(xrows(rows) * g.W, grows(rows) * g.Wo) && (rows % g.sh == 0 || rows == g.H)) {
                plan.planes_per_wg = 1;
                plan.rows_per_wg = (int)rows;
                plan.strips = ceil_div(g.H, rows);
                blocks = planes * plan.strips;
                x_floats = part(xrows(rows) * g.W);
                gy_floats = part(grows(rows) * g.Wo);
                ok = true;
            }
        }
        if (ok && blocks <= 0x7fffffffLL && (long long)plan.planes_per_wg * plane_in < (1 << 30)) {
            if (g.kh == 3 && g.kw == 3 && g.sh == 2 && g.sw == 2)
                return launch_bwd_slab<MODE, 3, 3, 2, 2>(src, ddst, dsrc, g, plan, x_floats, gy_floats, blocks, st);
            if (g.kh == 2 && g.kw == 2 && g.sh == 2 && g.sw == 2)
                return launch_bwd_slab<MODE, 2, 2, 2, 2>(src, ddst, dsrc, g, plan, x_floats, gy_floats, blocks, st);
            return launch_bwd_slab<MODE, 0, 0, 0, 0>(src, ddst, dsrc, g, plan, x_floats, gy_floats, blocks, st);
        }
    }
    return launch_bwd_generic<MODE>(src, ddst, dsrc, g, 0, st);
}

// =============================================================================
// Softmax backward: dz = p * (dp - sum_k dp_k p_k), row by row
// =============================================================================
template <int TPR, int ITEMS>
__global__ __launch_bounds__(TPR < 256 ? 256 : TPR) void softmax_bwd_rows_kernel(
    const float* probs, const float* dprobs, float* dlogits, int N, int classes, int base_mis, int align) {
    constexpr int BLOCK = TPR < 256 ? 256 : TPR;
    constexpr int ROWS = BLOCK / TPR;
    __shared__ float slots[BLOCK / kWave];
    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const int row_in_block = tid / TPR;
    const int lane = tid % TPR;
    const int first_wave = row_in_block * (TPR / kWave);
    const long long row_raw = (long long)blockIdx.x * ROWS + row_in_block;
    const bool live = row_raw < N;
    const long long row = live ? row_raw : (long long)N - 1;
    const size_t row_off = (size_t)row * (size_t)classes;
    // the row layout of the forward kernel: head up to the next boundary, aligned float4 body, tail
    const int mis = (int)((row_off + (size_t)base_mis) & (size_t)(align - 1));
    const int h = (align - mis) & (align - 1);
    const int nbody = (classes - h) >> 2;
    const int t = classes - h - 4 * nbody;
    const float* p = probs + row_off;
    const float* d = dprobs + row_off;
    float* z = dlogits + row_off;

    float4 pv[ITEMS], dv[ITEMS];
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int q = lane + k * TPR;
        const int qc = q < nbody ? q : nbody - 1;
        pv[k] = ld4_stream(p + h + 4 * qc);
        dv[k] = ld4_stream(d + h + 4 * qc);
    }
    const bool is_edge = lane < h + t;
    const int edge_idx = lane < h ? lane : h + 4 * nbody + (lane - h);
    float pe = 0.f, de = 0.f;
    if (is_edge) { pe = ld1_stream(p + edge_idx); de = ld1_stream(d + edge_idx); }

    float dot = pe * de;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        if (lane + k * TPR >= nbody) pv[k] = make_float4(0.f, 0.f, 0.f, 0.f);     // slots past the row add nothing
        dot += (pv[k].x * dv[k].x + pv[k].y * dv[k].y) + (pv[k].z * dv[k].z + pv[k].w * dv[k].w);
    }
    dot = row_reduce<SumOp, TPR>(dot, slots, wave, first_wave);
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int q = lane + k * TPR;
        if (live && q < nbody)
            st4_stream(z + h + 4 * q, make_float4(pv[k].x * (dv[k].x - dot), pv[k].y * (dv[k].y - dot),
                                                  pv[k].z * (dv[k].z - dot), pv[k].w * (dv[k].w - dot)));
    }
    if (live && is_edge) st1_stream(z + edge_idx, pe * (de - dot));
}

// Any alignment, any length: one workgroup per row, two sweeps (the second mostly from L2).
__global__ __launch_bounds__(256) void softmax_bwd_stream_kernel(const float* probs, const float* dprobs, float* dlogits,
                                                                 int classes) {
    constexpr int TPR = 256;
    __shared__ float slots[TPR / kWave];
    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const size_t row_off = (size_t)blockIdx.x * (size_t)classes;
    const float* p = probs + row_off;
    const float* d = dprobs + row_off;
    float* z = dlogits + row_off;
    float dot = 0.f;
    for (int c = tid; c < classes; c += TPR) dot += p[c] * d[c];
    dot = row_reduce<SumOp, TPR>(dot, slots, wave, 0);
    for (int c = tid; c < classes; c += TPR) z[c] = p[c] * (d[c] - dot);
}

template <int TPR, int ITEMS>
int launch_bwd_rows(const float* p, const float* d, float* z, int N, int classes, int base_mis, int align,
                    hipStream_t st) {
    constexpr int BLOCK = TPR < 256 ? 256 : TPR;
    constexpr int ROWS = BLOCK / TPR;
    hipLaunchKernelGGL((softmax_bwd_rows_kernel<TPR, ITEMS>), dim3((unsigned)ceil_div64(N, ROWS)), dim3(BLOCK), 0, st, p,
                       d, z, N, classes, base_mis, align);
    return launch_status();
}

template <int TPR>
int launch_bwd_rows_items(int items, const float* p, const float* d, float* z, int N, int classes, int base_mis,
                          int align, hipStream_t st) {
#define CNNMEM_CASE(I) \
    if (items <= I) return launch_bwd_rows<TPR, I>(p, d, z, N, classes, base_mis, align, st)
    CNNMEM_CASE(1);
    CNNMEM_CASE(2);
    CNNMEM_CASE(3);
    CNNMEM_CASE(4);
    CNNMEM_CASE(6);
    CNNMEM_CASE(8);
#undef CNNMEM_CASE
    return CNNMEM_ERR_UNSUPPORTED;
}

}  // namespace

int launch_pool_backward(const float* src, const float* ddst, float* dsrc, const PoolGeom& g, int layout,
                         hipStream_t st) {
    return g.mode == CNNMEM_POOL_MAX ? dispatch_pool_backward<CNNMEM_POOL_MAX>(src, ddst, dsrc, g, layout, st)
                                     : dispatch_pool_backward<CNNMEM_POOL_AVG>(src, ddst, dsrc, g, layout, st);
}

int launch_softmax_backward(const float* probs, const float* dprobs, float* dlogits, int N, int classes,
                            hipStream_t st) {
    const uintptr_t pa = reinterpret_cast<uintptr_t>(probs), pb = reinterpret_cast<uintptr_t>(dprobs),
                    pc = reinterpret_cast<uintptr_t>(dlogits);
    const bool same_phase = (((pa ^ pb) | (pa ^ pc)) & 15u) == 0;
    const int align = ((((pa ^ pb) | (pa ^ pc)) & 127u) == 0 && classes >= 64) ? 32 : 4;
    const int base_mis = (int)((pa & (uintptr_t)(4 * align - 1)) >> 2);
    const long long nq = classes / 4;
    // two rows of float4 per lane: at most 4 + 4 of them below 1024 lanes, 8 + 8 at 1024
    int tpr = 64;
    while (tpr < 1024 && nq > (long long)tpr * 4) tpr *= 2;
    const long long items = ceil_div64(nq, tpr);
    // lanes 0 .. h + t - 1 carry the head and tail words: h + t <= 34 with line alignment
    if (same_phase && classes >= 2 * align && classes >= 8 && items <= 8) {
        switch (tpr) {
            case 64: return launch_bwd_rows_items<64>((int)items, probs, dprobs, dlogits, N, classes, base_mis, align, st);
            case 128: return launch_bwd_rows_items<128>((int)items, probs, dprobs, dlogits, N, classes, base_mis, align, st);
            case 256: return launch_bwd_rows_items<256>((int)items, probs, dprobs, dlogits, N, classes, base_mis, align, st);
            case 512: return launch_bwd_rows_items<512>((int)items, probs, dprobs, dlogits, N, classes, base_mis, align, st);
            default: return launch_bwd_rows_items<1024>((int)items, probs, dprobs, dlogits, N, classes, base_mis, align, st);
        }
    }
    hipLaunchKernelGGL(softmax_bwd_stream_kernel, dim3((unsigned)N), dim3(256), 0, st, probs, dprobs, dlogits, classes);
    return launch_status();
}

}  // namespace cnnmem
