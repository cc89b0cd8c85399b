// Fused softmax (Section II.A steps 1-5 in one kernel, Section V.B).
//
// The paper's fused kernel stages a row in shared memory, which capped it at
// about 11K categories on its GPU.  Here a row lives in registers: a group of
// TPR lanes (one or more wavefronts) owns one row, each lane holds ITEMS float4,
// the row is read from HBM exactly once and written exactly once.  The max and
// the sum are reduced inside a wavefront with DPP lane permutes and across the
// wavefronts of a row through a few LDS words.
//
// Rows need not be 16-byte aligned (21841 floats = 87364 bytes): the lanes walk
// the row as the aligned float4 stream that covers it and mask the (at most
// three) elements before the row's first and after its last element, so every
// interior access is still a 128-bit one.
#include <cmath>

#include "common.hpp"
#include "rowmath.hpp"

namespace cnnmem {
namespace {

constexpr float kNegInf = kRowNegInf;

// One row per TPR lanes, ITEMS float4 per lane held in registers.
//
// A row of `classes` floats starts `mis` floats past a boundary of `align` floats
// (align = 32, a 128-byte cache line, when both buffers sit at the same offset in
// their lines, else 4, one float4).  It is split into a head (the
// h = (align - mis) % align floats up to the next boundary), a body of nbody
// float4 and a tail of t < 4 floats.  Body slot q = lane + k*TPR is one
// unconditional 128-bit access (lanes past the end re-read the last slot and
// discard it), so the compiler issues all ITEMS loads back to back, and with
// align = 32 every wavefront reads and writes whole cache lines: no line is
// fetched by two wavefronts or written in two pieces.  The at most align + 2
// head/tail floats are carried by lanes 0..h+t-1 in one extra register.
// Requires classes >= 2*align (then nbody >= 1).
template <int TPR, int ITEMS>
__global__ __launch_bounds__(TPR < 256 ? 256 : TPR) void softmax_rows_kernel(
    const float* logits, float* probs, int N, int classes, int base_mis, int align) {
    constexpr int BLOCK = TPR < 256 ? 256 : TPR;
    constexpr int ROWS = BLOCK / TPR;
    __shared__ float slots[BLOCK / kWave], slots_sum[BLOCK / kWave];

    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const int row_in_block = tid / TPR;
    const int lane = tid % TPR;
    const int first_wave = row_in_block * (TPR / kWave);
    const long long row_raw = (long long)blockIdx.x * ROWS + row_in_block;
    const bool live = row_raw < N;
    const long long row = live ? row_raw : (long long)N - 1;        // idle lane groups shadow the last row
    const size_t row_off = (size_t)row * (size_t)classes;
    const int mis = (int)((row_off + (size_t)base_mis) & (size_t)(align - 1));
    const int h = (align - mis) & (align - 1);
    const int nbody = (classes - h) >> 2;
    const int t = classes - h - 4 * nbody;
    const float* x = logits + row_off;
    float* y = probs + row_off;
    const float* xb = x + h;                                        // 16-byte aligned
    float* yb = y + h;

    float4 v[ITEMS];
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int q = lane + k * TPR;
        const int qc = q < nbody ? q : nbody - 1;
        v[k] = ld4_stream(xb + 4 * qc);
    }
    // head / tail element of this lane, if any
    const bool is_head = lane < h;
    const bool is_edge = lane < h + t;
    const int edge_idx = is_head ? lane : h + 4 * nbody + (lane - h);
    float e = kNegInf;
    if (is_edge) e = ld1_stream(x + edge_idx);

    // step 1: row maximum (slots past the body are masked to -inf first)
    float m = e;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        if (lane + k * TPR >= nbody) v[k] = make_float4(kNegInf, kNegInf, kNegInf, kNegInf);
        m = fmaxf(fmaxf(m, fmaxf(v[k].x, v[k].y)), fmaxf(v[k].z, v[k].w));
    }
    m = row_reduce<MaxOp, TPR, true>(m, slots, wave, first_wave);

    // steps 2-4: shift, exponentiate, sum (masked slots hold -inf and give 0)
    e = exp_nonpos(e - m);
    float s = e;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        v[k].x = exp_nonpos(v[k].x - m);
        v[k].y = exp_nonpos(v[k].y - m);
        v[k].z = exp_nonpos(v[k].z - m);
        v[k].w = exp_nonpos(v[k].w - m);
        s += (v[k].x + v[k].y) + (v[k].z + v[k].w);
    }
    s = row_reduce<SumOp, TPR, true>(s, slots_sum, wave, first_wave);

    // step 5: normalise
    const float inv = 1.0f / s;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int q = lane + k * TPR;
        if (live && q < nbody)
            st4_stream(yb + 4 * q, make_float4(v[k].x * inv, v[k].y * inv, v[k].z * inv, v[k].w * inv));
    }
    if (live && is_edge) st1_stream(y + edge_idx, e * inv);
}

// Rows of fewer than 4 categories: one lane per row, everything in registers.
__global__ __launch_bounds__(256) void softmax_tiny_kernel(const float* logits, float* probs, int N, int classes) {
    const long long row = (long long)blockIdx.x * 256 + threadIdx.x;
    if (row >= N) return;
    const float* x = logits + (size_t)row * classes;
    float* y = probs + (size_t)row * classes;
    float v[3];
    float m = kNegInf;
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        v[c] = c < classes ? x[c] : kNegInf;
        m = fmaxf(m, v[c]);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        v[c] = exp_nonpos(v[c] - m);
        s += v[c];
    }
    const float inv = 1.0f / s;
#pragma unroll
    for (int c = 0; c < 3; ++c)
        if (c < classes) y[c] = v[c] * inv;
}

// Short rows (4 .. 159 categories; works up to 512): a whole wavefront per row would idle most lanes, so a
// row gets G = 4 .. 32 lanes and a workgroup 256 / G rows.  Rows start at any dword, hence
// 128-bit accesses at dword alignment; a row's last, partial float4 is loaded as the row's last
// four words and shifted into place, so every load is unconditional.
template <int G, int ITEMS>
__global__ __launch_bounds__(256) void softmax_short_kernel(const float* logits, float* probs, int N, int classes) {
    constexpr int ROWS = 256 / G;
    const int lane = threadIdx.x % G;
    const long long row_raw = (long long)blockIdx.x * ROWS + threadIdx.x / G;
    const bool live = row_raw < N;
    const long long row = live ? row_raw : (long long)N - 1;       // idle groups shadow the last row
    const float* x = logits + (size_t)row * (size_t)classes;
    float* y = probs + (size_t)row * (size_t)classes;

    float t[ITEMS][4];
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int e0 = 4 * (lane + k * G);
        const int ec = e0 + 4 <= classes ? e0 : classes - 4;        // classes >= 4; may be far left of e0
        const float4 v = ld4u_stream(x + (ec > 0 ? ec : 0));
        const float a[4] = {v.x, v.y, v.z, v.w};
        const int d = e0 - ec;                                      // 0 for whole slots, 1..3 in the last one, >= 4 past the row
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float val = kNegInf;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (j + d == u) val = a[u];
            t[k][j] = val;
        }
    }
    float m = kNegInf;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) m = fmaxf(fmaxf(m, fmaxf(t[k][0], t[k][1])), fmaxf(t[k][2], t[k][3]));
    m = group_reduce<MaxOp, G>(m);
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
#pragma unroll
        for (int j = 0; j < 4; ++j) t[k][j] = exp_nonpos(t[k][j] - m);
        s += (t[k][0] + t[k][1]) + (t[k][2] + t[k][3]);
    }
    s = group_reduce<SumOp, G>(s);
    const float inv = 1.0f / s;
    if (!live) return;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int e0 = 4 * (lane + k * G);
        if (e0 + 4 <= classes) {
            st4u_stream(y + e0, make_float4(t[k][0] * inv, t[k][1] * inv, t[k][2] * inv, t[k][3] * inv));
        } else {
            for (int j = 0; j < 4; ++j)
                if (e0 + j < classes) y[e0 + j] = t[k][j] * inv;
        }
    }
}

template <int G>
int launch_short(int items, const float* logits, float* probs, int N, int classes, hipStream_t st) {
    const dim3 grid((unsigned)ceil_div64(N, 256 / G)), block(256);
    switch (items) {
        case 1: hipLaunchKernelGGL((softmax_short_kernel<G, 1>), grid, block, 0, st, logits, probs, N, classes); break;
        case 2: hipLaunchKernelGGL((softmax_short_kernel<G, 2>), grid, block, 0, st, logits, probs, N, classes); break;
        case 3: hipLaunchKernelGGL((softmax_short_kernel<G, 3>), grid, block, 0, st, logits, probs, N, classes); break;
        default: hipLaunchKernelGGL((softmax_short_kernel<G, 4>), grid, block, 0, st, logits, probs, N, classes); break;
    }
    return launch_status();
}

// Rows too long for registers, or buffers whose 16-byte phases differ: one 1024-lane workgroup
// per row, two sweeps of 128-bit accesses at dword alignment (so no head / tail bookkeeping).
// Sweep 1 keeps a running maximum and a running sum of exponentials per lane, rescaling the sum
// whenever the maximum grows (the "online" form of steps 1-4); sweep 2 reads the row again, by
// then mostly from L2, and writes the normalised values.  In place is allowed: a word is read
// by the lane that writes it, just before.
// Both sweeps move U float4 per lane and trip, loaded back to back from clamped addresses (a loop
// with one load per trip keeps a single 128-bit load in flight per lane).  CACHED: the first sweep
// uses ordinary loads, so that the row may still sit in L2 or the memory-side cache when the second
// sweep, which streams, comes back for it.
template <bool CACHED>
__global__ __launch_bounds__(1024) void softmax_stream_kernel(const float* logits, float* probs,
                                                              int classes) {
    constexpr int TPR = 1024;
    constexpr int U = 8;
    __shared__ float slots[TPR / kWave];
    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const size_t row_off = (size_t)blockIdx.x * (size_t)classes;
    const float* x = logits + row_off;
    float* y = probs + row_off;
    const int nvec = classes >> 2;                  // whole float4 of the row (>= 1); the last 0..3 words go one by one
    const int tail0 = nvec << 2;

    float m = kNegInf, s = 0.f;
    for (int q0 = tid; q0 < nvec; q0 += TPR * U) {
        float4 v[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int q = q0 + k * TPR;
            const float* p = x + 4 * (size_t)(q < nvec ? q : nvec - 1);
            if (CACHED) {
                const v4f_unaligned_t t = *reinterpret_cast<const v4f_unaligned_t*>(p);
                v[k] = make_float4(t.x, t.y, t.z, t.w);
            } else {
                v[k] = ld4u_stream(p);
            }
        }
        float vm = kNegInf;
#pragma unroll
        for (int k = 0; k < U; ++k) {
            if (q0 + k * TPR >= nvec) v[k] = make_float4(kNegInf, kNegInf, kNegInf, kNegInf);
            vm = fmaxf(fmaxf(vm, fmaxf(v[k].x, v[k].y)), fmaxf(v[k].z, v[k].w));
        }
        if (vm > m) {                               // rare after the first few trips
            s *= exp_nonpos(m - vm);                // m = -inf at first: exp gives 0, s stays 0
            m = vm;
        }
#pragma unroll
        for (int k = 0; k < U; ++k)
            s += (exp_nonpos(v[k].x - m) + exp_nonpos(v[k].y - m)) + (exp_nonpos(v[k].z - m) + exp_nonpos(v[k].w - m));
    }
    if (tid < classes - tail0) {
        const float v = x[tail0 + tid];
        if (v > m) { s *= exp_nonpos(m - v); m = v; }
        s += exp_nonpos(v - m);
    }
    // combine the lanes: rescale every lane's sum to the row maximum, then add
    const float row_m = row_reduce<MaxOp, TPR>(m, slots, wave, 0);
    s *= exp_nonpos(m - row_m);                     // lanes that saw nothing: m = -inf, s = 0
    const float row_s = row_reduce<SumOp, TPR>(s, slots, wave, 0);
    const float inv = 1.0f / row_s;

    for (int q0 = tid; q0 < nvec; q0 += TPR * U) {
        float4 v[U];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int q = q0 + k * TPR;
            v[k] = ld4u_stream(x + 4 * (size_t)(q < nvec ? q : nvec - 1));
        }
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int q = q0 + k * TPR;
            if (q < nvec)
                st4u_stream(y + 4 * (size_t)q, make_float4(exp_nonpos(v[k].x - row_m) * inv, exp_nonpos(v[k].y - row_m) * inv,
                                                           exp_nonpos(v[k].z - row_m) * inv, exp_nonpos(v[k].w - row_m) * inv));
        }
    }
    if (tid < classes - tail0) y[tail0 + tid] = exp_nonpos(x[tail0 + tid] - row_m) * inv;
}

template <int TPR, int ITEMS>
int launch_rows(const float* logits, float* probs, int N, int classes, int base_mis, int align, int rows_per_cu,
                hipStream_t st) {
    constexpr int BLOCK = TPR < 256 ? 256 : TPR;
    constexpr int ROWS = BLOCK / TPR;
    const unsigned blocks = (unsigned)ceil_div64(N, ROWS);
    // resident workgroups per CU, capped by asking for LDS that the kernel never touches (0 = no cap)
    const int wpc = env_int("CNNMEM_SOFTMAX_WPC", rows_per_cu);
    const size_t lds = wpc > 0 ? throttle_lds(wpc, 0, wpc) : 0;
    hipLaunchKernelGGL((softmax_rows_kernel<TPR, ITEMS>), dim3(blocks), dim3(BLOCK), lds, st, logits, probs, N,
                       classes, base_mis, align);
    return launch_status();
}

template <int TPR>
int launch_rows_items(int items, const float* logits, float* probs, int N, int classes, int base_mis,
                      int align, int rows_per_cu, hipStream_t st) {
#define CNNMEM_CASE(I) \
    if (items <= I) return launch_rows<TPR, I>(logits, probs, N, classes, base_mis, align, rows_per_cu, st)
    CNNMEM_CASE(1);
    CNNMEM_CASE(2);
    CNNMEM_CASE(3);
    CNNMEM_CASE(4);
    CNNMEM_CASE(6);
    CNNMEM_CASE(8);
    CNNMEM_CASE(9);
    CNNMEM_CASE(10);
    CNNMEM_CASE(11);
    CNNMEM_CASE(12);
    CNNMEM_CASE(14);
    CNNMEM_CASE(16);
    CNNMEM_CASE(24);
    CNNMEM_CASE(32);
#undef CNNMEM_CASE
    return CNNMEM_ERR_UNSUPPORTED;
}

}  // namespace

int launch_softmax(const float* logits, float* probs, int N, int classes, hipStream_t st) {
    // The register kernel needs both buffers to share their 16-byte phase.
    const uintptr_t pa = reinterpret_cast<uintptr_t>(logits), pb = reinterpret_cast<uintptr_t>(probs);
    const bool same_phase = ((pa ^ pb) & 15u) == 0;
    // whole-line accesses need both buffers at the same offset inside their 128-byte lines
    const int align = (((pa ^ pb) & 127u) == 0 && classes >= 64 && env_int("CNNMEM_SOFTMAX_ALIGN", 32) == 32) ? 32 : 4;
    const int base_mis = (int)((pa & (uintptr_t)(4 * align - 1)) >> 2);
    if (classes < 4) {
        hipLaunchKernelGGL(softmax_tiny_kernel, dim3((unsigned)ceil_div64(N, 256)), dim3(256), 0, st, logits, probs,
                           N, classes);
        return launch_status();
    }
    // measured on MI355X: 44 % against 28 % of peak at 64 categories, 56 % against 44 % at 128, but
    // 52 % against 61 % at 200, where the 64-lane register kernel below takes over
    const int short_below = env_int("CNNMEM_SOFTMAX_SHORT_BELOW", 160);
    // (rows of fewer than 8 categories always: the register kernel needs one whole float4 after the row's head)
    if (classes < 8 || (classes < (short_below < 513 ? short_below : 513) && env_int("CNNMEM_SOFTMAX_TPR", 0) == 0)) {
        // G lanes per row, at most four float4 per lane
        const int slots = (classes + 3) / 4;
        int g = 4;
        while (g < 32 && slots > 4 * g) g *= 2;
        const int items = (slots + g - 1) / g;
        switch (g) {
            case 4: return launch_short<4>(items, logits, probs, N, classes, st);
            case 8: return launch_short<8>(items, logits, probs, N, classes, st);
            case 16: return launch_short<16>(items, logits, probs, N, classes, st);
            default: return launch_short<32>(items, logits, probs, N, classes, st);
        }
    }
    const long long nq = classes / 4;                             // most aligned float4 a row can hold
    int tpr = env_int("CNNMEM_SOFTMAX_TPR", 0);
    int rows_per_cu = 0;
    if (tpr != 64 && tpr != 128 && tpr != 256 && tpr != 512 && tpr != 1024) {
        // smallest lane group that keeps at most 8 float4 per lane, else 1024
        tpr = 64;
        while (tpr < 1024 && nq > (long long)tpr * 8) tpr *= 2;
        // Rows of 64-128 KB: two resident rows per CU on few wavefronts.  4096 x 21841 back to back: 1024 lanes
        // per row (two workgroups fill a CU) 73.5 % of peak; 256 to 640 lanes per row with the CU capped at
        // two workgroups 75.0-75.3 %; the same lane counts uncapped (three or four rows per CU) 70.5-72 %.
        if (classes >= 16384 && classes <= 32768) {
            tpr = 512;
            rows_per_cu = 2;
        }
    }
    const long long items = ceil_div64(nq, tpr);
    // 1024 lanes leave 128 VGPRs per lane: beyond 16 float4 the row would spill
    const long long max_items = tpr == 1024 ? 16 : 32;
    if (same_phase && items <= max_items) {
        switch (tpr) {
            case 64: return launch_rows_items<64>((int)items, logits, probs, N, classes, base_mis, align, rows_per_cu, st);
            case 128: return launch_rows_items<128>((int)items, logits, probs, N, classes, base_mis, align, rows_per_cu, st);
            case 256: return launch_rows_items<256>((int)items, logits, probs, N, classes, base_mis, align, rows_per_cu, st);
            case 512: return launch_rows_items<512>((int)items, logits, probs, N, classes, base_mis, align, rows_per_cu, st);
            default: return launch_rows_items<1024>((int)items, logits, probs, N, classes, base_mis, align, rows_per_cu, st);
        }
    }
    // measured on MI355X: 512 x 128256 46 -> 56 % of peak, 2048 x 151936 45 -> 57 %, 1024 x 70001 42 -> 52 %,
    // 256 x 262144 48 -> 51 % with the cacheable first sweep
    if (env_int("CNNMEM_SOFTMAX_STREAM_CACHED", 1) != 0)
        hipLaunchKernelGGL(softmax_stream_kernel<true>, dim3((unsigned)N), dim3(1024), 0, st, logits, probs, classes);
    else
        hipLaunchKernelGGL(softmax_stream_kernel<false>, dim3((unsigned)N), dim3(1024), 0, st, logits, probs, classes);
    return launch_status();
}

}  // namespace cnnmem
