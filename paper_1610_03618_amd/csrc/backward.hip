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

// Windows larger than 8 x 8 in the compiled-for-any-window instance fall back to the generic kernel (host).

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
    st4_stream(dsrc + in0, da);
    st4_stream(dsrc + in0 + W, db);
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

template <int MODE>
int dispatch_pool_backward(const float* src, const float* ddst, float* dsrc, const PoolGeom& g, int layout,
                           hipStream_t st) {
    const bool a16 = aligned16(ddst) && aligned16(dsrc) && (MODE == CNNMEM_POOL_AVG || aligned16(src));
    if (layout == CNNMEM_CHWN) {
        const long long items = (long long)g.C * g.H * g.W * (g.N / 4);
        if (a16 && g.N % 4 == 0 && items < 0x7fffffffLL && g.kh <= 8 && g.kw <= 8) {
            if (g.kh == 3 && g.kw == 3 && g.sh == 2 && g.sw == 2)
                return launch_bwd_chwn<MODE, 3, 3, 2, 2>(src, ddst, dsrc, g, st);
            if (g.kh == 2 && g.kw == 2 && g.sh == 2 && g.sw == 2)
                return launch_bwd_chwn<MODE, 2, 2, 2, 2>(src, ddst, dsrc, g, st);
            return launch_bwd_chwn<MODE, 0, 0, 0, 0>(src, ddst, dsrc, g, st);
        }
        return launch_bwd_generic<MODE>(src, ddst, dsrc, g, 1, st);
    }
    if (a16 && g.kh == 2 && g.kw == 2 && g.sh == 2 && g.sw == 2 && g.ph == 0 && g.pw == 0 && g.H % 2 == 0 &&
        g.W % 4 == 0) {
        const long long per_row = g.W / 4;
        const long long items = (long long)g.N * g.C * g.Ho * per_row;
        if (items < 0x7fffffffLL) {
            hipLaunchKernelGGL((pool_bwd_nchw_2x2s2_kernel<MODE>), dim3((unsigned)ceil_div64(items, kThreads)),
                               dim3(kThreads), 0, st, src, ddst, dsrc, (uint32_t)items, (uint32_t)g.W,
                               make_fastdiv((uint32_t)per_row));
            return launch_status();
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
