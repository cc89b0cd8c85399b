/*
 * cnnmem_ref.c -- CPU oracle for the memory-bound CNN layers.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * obviously-correct host implementation of what the GPU library computes.
 * Only the tests, the smoke check and the benchmark's "cpu_baseline" leg may
 * call it.  It shares no code with the HIP path and includes none of its
 * headers.  All pointers are HOST pointers.
 *
 * What follows the paper:
 *   - layouts: Section II.A (NCHW: W contiguous, H strides by W, C by H*W, N by
 *     C*H*W) and Section IV.C (CHWN: N contiguous; NCHW == [N][C*H*W],
 *     CHWN == [C*H*W][N], so the layout change is a 2-D transpose).
 *   - pooling: Equation 2 (average) and the prose of Section II.A (max).
 *   - softmax: the five steps of Section II.A, in the paper's order.
 *   - layout choice: the (Ct, Nt) heuristic of Section IV.A and the one-scan plan
 *     of Section IV.D.
 *   - the other storage orders: Section I (a 4-D tensor has 24), Section IV.A
 *     (HWCN beside CHWN), the NHWC order of the comparison libraries: a general
 *     axis permutation and a change between two spelled layouts.
 *
 * Readings taken where the paper is silent or garbled (each is pinned or
 * listed as a reading in the design notes):
 *   - pooled extent = floor((L + 2*pad - k) / stride) + 1  (Fig. 8: 12 inputs,
 *     window 4, stride 2 -> 5 outputs);
 *   - Eq. 2's sums run over X*Y taps (upper bounds exclusive: the divisor is
 *     /Y/X);
 *   - padding is not in Eq. 2: a tap outside the image is skipped by max and
 *     adds 0 to the average, whose divisor stays kh*kw;
 *   - the doubled summation signs printed in front of each softmax step are
 *     typesetting debris: step 1 is a max over categories of one image, step 4
 *     a sum over categories of one image.
 *
 * Precision: transforms move 32-bit words untouched; max-pool compares fp32
 * values; average pooling and softmax accumulate in fp64 and round once to
 * fp32.
 *
 * Parity pins: every function here is pinned by tests that do not go through
 * it (worked examples, closed forms, invariants, library routines).  The only
 * unpinned behaviour is pooling with pad > 0, which the paper does not define:
 * it is pinned to the common library routine's convention only.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { REF_OK = 0, REF_ERR_INVALID_ARG = 1, REF_ERR_NOMEM = 3 };
enum { REF_NCHW = 0, REF_CHWN = 1 };
enum { REF_POOL_MAX = 0, REF_POOL_AVG = 1 };

/* Linear index of element (n, c, h, w) of an N x C x H x W tensor.
 * Section II.A gives the NCHW strides; CHWN moves N to the fastest position. */
static size_t at(int layout, int N, int C, int H, int W, int n, int c, int h, int w)
{
    if (layout == REF_NCHW)
        return (((size_t)n * C + c) * H + h) * W + w;
    return (((size_t)c * H + h) * W + w) * N + n;
}

/* Linear index of element (n, c, h, w) in `layout`, for checks on sampled
 * elements of tensors too large to run through the loops below. */
unsigned long long cnnmem_ref_index(int layout, int N, int C, int H, int W, int n, int c, int h, int w)
{
    return (unsigned long long)at(layout, N, C, H, W, n, c, h, w);
}

/* Caps the threads of the loops below (timing aid; results do not depend on it). */
int cnnmem_ref_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#endif
    (void)n;
    return REF_OK;
}

int cnnmem_ref_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Layout change (Section IV.C): the same (n, c, h, w) element is read at its
 * source index and written at its destination index.  Words are moved as
 * 32-bit integers so every bit pattern survives. */
int cnnmem_ref_transform(const float *src, float *dst, int N, int C, int H, int W,
                         int src_layout, int dst_layout)
{
    if (!src || !dst || N <= 0 || C <= 0 || H <= 0 || W <= 0)
        return REF_ERR_INVALID_ARG;
    if ((src_layout != REF_NCHW && src_layout != REF_CHWN) ||
        (dst_layout != REF_NCHW && dst_layout != REF_CHWN))
        return REF_ERR_INVALID_ARG;
    const uint32_t *s = (const uint32_t *)src;
    uint32_t *d = (uint32_t *)dst;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    d[at(dst_layout, N, C, H, W, n, c, h, w)] =
                        s[at(src_layout, N, C, H, W, n, c, h, w)];
    return REF_OK;
}

/* Pooled extent along one axis: number of window positions i with
 * i*stride - pad + k <= L + pad, i.e. floor((L + 2*pad - k)/stride) + 1. */
static int pooled_extent(int L, int k, int s, int p)
{
    return (L + 2 * p - k) / s + 1;
}

static int pool_args_ok(int N, int C, int H, int W, int layout, int mode,
                        int kh, int kw, int sh, int sw, int ph, int pw)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return 0;
    if (layout != REF_NCHW && layout != REF_CHWN) return 0;
    if (mode != REF_POOL_MAX && mode != REF_POOL_AVG) return 0;
    if (kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0) return 0;
    if (ph > kh / 2 || pw > kw / 2) return 0;       /* every window keeps a tap */
    if (H + 2 * ph < kh || W + 2 * pw < kw) return 0;
    return 1;
}

int cnnmem_ref_pool_out_dims(int H, int W, int kh, int kw, int sh, int sw, int ph, int pw,
                             int *Ho, int *Wo)
{
    if (!Ho || !Wo || !pool_args_ok(1, 1, H, W, REF_NCHW, REF_POOL_MAX, kh, kw, sh, sw, ph, pw))
        return REF_ERR_INVALID_ARG;
    *Ho = pooled_extent(H, kh, sh, ph);
    *Wo = pooled_extent(W, kw, sw, pw);
    return REF_OK;
}

/* Pooling (Equation 2 for the average; "max" replaces the sum by a maximum).
 * Output element (n, c, i, j) looks at input rows i*sh - ph + y, y < kh, and
 * columns j*sw - pw + x, x < kw.  The output has the layout of the input. */
int cnnmem_ref_pool(const float *src, float *dst, int N, int C, int H, int W, int layout,
                    int mode, int kh, int kw, int sh, int sw, int ph, int pw)
{
    if (!src || !dst || !pool_args_ok(N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw))
        return REF_ERR_INVALID_ARG;
    const int Ho = pooled_extent(H, kh, sh, ph);
    const int Wo = pooled_extent(W, kw, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    float best = -INFINITY;
                    double sum = 0.0;
                    for (int y = 0; y < kh; ++y)
                        for (int x = 0; x < kw; ++x) {
                            const int r = i * sh - ph + y;
                            const int q = j * sw - pw + x;
                            if (r < 0 || r >= H || q < 0 || q >= W)
                                continue;
                            const float v = src[at(layout, N, C, H, W, n, c, r, q)];
                            if (v > best) best = v;
                            sum += (double)v;
                        }
                    float out;
                    if (mode == REF_POOL_MAX)
                        out = best;
                    else
                        out = (float)(sum / (double)(kh * kw));   /* Eq. 2: /Y/X */
                    dst[at(layout, N, C, Ho, Wo, n, c, i, j)] = out;
                }
    return REF_OK;
}

/* Softmax over the categories of each image (Section II.A, steps 1-5), on a
 * row-major [N][classes] matrix. */
int cnnmem_ref_softmax(const float *logits, float *probs, int N, int classes)
{
    if (!logits || !probs || N <= 0 || classes <= 0)
        return REF_ERR_INVALID_ARG;
    int failed = 0;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const float *in = logits + (size_t)n * classes;
        float *out = probs + (size_t)n * classes;
        double *mid = (double *)malloc((size_t)classes * sizeof(double));
        if (!mid) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        /* step 1: Maxv[n] = max over categories */
        float maxv = in[0];
        for (int c = 1; c < classes; ++c)
            if (in[c] > maxv) maxv = in[c];
        /* step 2: Midv1 = In - Maxv */
        for (int c = 0; c < classes; ++c)
            mid[c] = (double)in[c] - (double)maxv;
        /* step 3: Midv2 = exp(Midv1) */
        for (int c = 0; c < classes; ++c)
            mid[c] = exp(mid[c]);
        /* step 4: Sumv[n] = sum over categories */
        double sumv = 0.0;
        for (int c = 0; c < classes; ++c)
            sumv += mid[c];
        /* step 5: Out = Midv2 / Sumv */
        for (int c = 0; c < classes; ++c)
            out[c] = (float)(mid[c] / sumv);
        free(mid);
    }
    return failed ? REF_ERR_NOMEM : REF_OK;
}

/* Layout heuristic (Section IV.A): a convolution prefers CHWN when it has fewer
 * than Ct input feature maps or a batch of at least Nt images, NCHW otherwise;
 * pooling prefers CHWN (Section IV.B).  kind: 0 convolution, 1 pooling, 2 other
 * (no preference: returns -1). */
int cnnmem_ref_choose_layout(int kind, int N, int C, int Ct, int Nt)
{
    if (kind == 0) {
        if (C < Ct) return REF_CHWN;
        if (N >= Nt) return REF_CHWN;
        return REF_NCHW;
    }
    if (kind == 1) return REF_CHWN;
    return -1;
}

/* Layout plan (Section IV.D): scan the layers once, give each its preferred
 * layout, and mark a transform wherever the layout changes.  Layers without a
 * preference keep the layout their input has; with pool_keeps != 0 so does
 * pooling.  kinds/Ns/Cs have n entries; returns the number of transforms. */
int cnnmem_ref_plan_layouts(const int *kinds, const int *Ns, const int *Cs, int n, int Ct, int Nt,
                            int input_layout, int pool_keeps, int *layouts, int *transform_before)
{
    int current = input_layout, count = 0;
    for (int i = 0; i < n; ++i) {
        int want = cnnmem_ref_choose_layout(kinds[i], Ns[i], Cs[i], Ct, Nt);
        if (want < 0 || (kinds[i] == 1 && pool_keeps)) want = current;
        layouts[i] = want;
        transform_before[i] = (want != current);
        count += transform_before[i];
        current = want;
    }
    return count;
}

/* Number of input loads a one-output-per-thread pooling of an L-long 1-D
 * signal issues (Section V.A, Fig. 8): outputs * window. */
int cnnmem_ref_naive_pool_loads_1d(int L, int k, int s)
{
    if (L < k || k <= 0 || s <= 0) return -1;
    return pooled_extent(L, k, s, 0) * k;
}

/* ---- any of the 24 storage orders of a 4-D tensor (Section I counts 24; Section IV.A
 * names CHWN and HWCN as the batch-fastest candidates; NHWC is the third order the
 * libraries of the paper's comparison offer) ---- */

/* General axis permutation.  `dims` are the source extents, slowest axis first;
 * destination axis i is source axis perm[i] (so the destination extents are
 * dims[perm[0..3]]).  Words move as 32-bit integers. */
int cnnmem_ref_permute(const float *src, float *dst, const int *dims, const int *perm)
{
    if (!src || !dst || !dims || !perm) return REF_ERR_INVALID_ARG;
    int seen[4] = {0, 0, 0, 0};
    for (int i = 0; i < 4; ++i) {
        if (dims[i] <= 0 || perm[i] < 0 || perm[i] > 3 || seen[perm[i]]) return REF_ERR_INVALID_ARG;
        seen[perm[i]] = 1;
    }
    size_t ss[4];                                   /* source strides in words */
    ss[3] = 1;
    for (int a = 2; a >= 0; --a) ss[a] = ss[a + 1] * (size_t)dims[a + 1];
    const int e0 = dims[perm[0]], e1 = dims[perm[1]], e2 = dims[perm[2]], e3 = dims[perm[3]];
    const size_t t0 = ss[perm[0]], t1 = ss[perm[1]], t2 = ss[perm[2]], t3 = ss[perm[3]];
    const uint32_t *s = (const uint32_t *)src;
    uint32_t *d = (uint32_t *)dst;
#pragma omp parallel for schedule(static)
    for (int i0 = 0; i0 < e0; ++i0)
        for (int i1 = 0; i1 < e1; ++i1)
            for (int i2 = 0; i2 < e2; ++i2)
                for (int i3 = 0; i3 < e3; ++i3)
                    d[(((size_t)i0 * e1 + i1) * e2 + i2) * e3 + i3] = s[i0 * t0 + i1 * t1 + i2 * t2 + i3 * t3];
    return REF_OK;
}

/* Stride, in words, of the axis called `letter` when an N x C x H x W tensor is
 * stored in the order spelled by `layout` (four letters, slowest first). */
static int letter_stride(const char *layout, char letter, int N, int C, int H, int W, size_t *stride)
{
    size_t st = 1;
    for (int i = 3; i >= 0; --i) {
        const char l = layout[i];
        if (l == letter) { *stride = st; return 1; }
        st *= (size_t)(l == 'N' ? N : l == 'C' ? C : l == 'H' ? H : W);
    }
    return 0;
}

static int layout_ok(const char *layout)
{
    if (!layout || strlen(layout) != 4) return 0;
    int n = 0, c = 0, h = 0, w = 0;
    for (int i = 0; i < 4; ++i) {
        n += layout[i] == 'N'; c += layout[i] == 'C'; h += layout[i] == 'H'; w += layout[i] == 'W';
    }
    return n == 1 && c == 1 && h == 1 && w == 1;
}

/* Storage-order change between two spelled layouts, e.g. "NCHW" -> "NHWC":
 * element (n, c, h, w) is read where the source order puts it and written where
 * the destination order puts it. */
int cnnmem_ref_relayout(const float *src, float *dst, int N, int C, int H, int W,
                        const char *src_layout, const char *dst_layout)
{
    if (!src || !dst || N <= 0 || C <= 0 || H <= 0 || W <= 0 || !layout_ok(src_layout) || !layout_ok(dst_layout))
        return REF_ERR_INVALID_ARG;
    size_t sn, sc, sh, sw, dn, dc, dh, dw;
    letter_stride(src_layout, 'N', N, C, H, W, &sn); letter_stride(dst_layout, 'N', N, C, H, W, &dn);
    letter_stride(src_layout, 'C', N, C, H, W, &sc); letter_stride(dst_layout, 'C', N, C, H, W, &dc);
    letter_stride(src_layout, 'H', N, C, H, W, &sh); letter_stride(dst_layout, 'H', N, C, H, W, &dh);
    letter_stride(src_layout, 'W', N, C, H, W, &sw); letter_stride(dst_layout, 'W', N, C, H, W, &dw);
    const uint32_t *s = (const uint32_t *)src;
    uint32_t *d = (uint32_t *)dst;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    d[n * dn + c * dc + h * dh + w * dw] = s[n * sn + c * sc + h * sh + w * sw];
    return REF_OK;
}

/* ---- 16-bit storage (the paper's closing remarks expect FP16 hardware to matter for
 * these layers; bf16 is the other 16-bit format of current GPUs) ----
 *
 * Only the storage changes: a stored value is widened exactly, every result is
 * computed as above in fp64 and rounded ONCE, to nearest with ties to even, to the
 * storage format.  fp16 is IEEE binary16 (1 + 5 + 10 bits, bias 15); bf16 is the
 * upper half of binary32 (1 + 8 + 7 bits, bias 127).  Both have subnormals,
 * infinities and NaNs. */
enum { REF_F32 = 0, REF_F16 = 1, REF_BF16 = 2 };

static int frac_bits_of(int dtype) { return dtype == REF_F16 ? 10 : 7; }
static int exp_bits_of(int dtype) { return dtype == REF_F16 ? 5 : 8; }

/* Exact value of a 16-bit pattern. */
static double widen16(uint16_t h, int dtype)
{
    const int fb = frac_bits_of(dtype), eb = exp_bits_of(dtype);
    const int bias = (1 << (eb - 1)) - 1;
    const int sign = h >> 15;
    const int e = (h >> fb) & ((1 << eb) - 1);
    const int f = h & ((1 << fb) - 1);
    double v;
    if (e == (1 << eb) - 1)
        v = f ? NAN : INFINITY;
    else if (e == 0)
        v = ldexp((double)f, 1 - bias - fb);                  /* subnormal: f * 2^(emin - fb) */
    else
        v = ldexp((double)((1 << fb) + f), e - bias - fb);    /* (1 + f/2^fb) * 2^(e - bias) */
    return sign ? -v : v;
}

/* Nearest 16-bit pattern to x, ties to even; overflow gives infinity. */
static uint16_t narrow16(double x, int dtype)
{
    const int fb = frac_bits_of(dtype), eb = exp_bits_of(dtype);
    const int bias = (1 << (eb - 1)) - 1;
    const int emax_field = (1 << eb) - 1;
    const uint16_t sign = (uint16_t)(signbit(x) ? 0x8000 : 0);
    if (isnan(x)) return (uint16_t)(sign | (emax_field << fb) | (1 << (fb - 1)));
    const double a = fabs(x);
    if (isinf(a)) return (uint16_t)(sign | (emax_field << fb));
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                                       /* a = m * 2^e, m in [0.5, 1) */
    e -= 1;                                                   /* a in [2^e, 2^(e+1)) */
    if (e < 1 - bias) e = 1 - bias;                           /* subnormal range: fixed spacing */
    /* a / spacing, spacing = 2^(e - fb); nearbyint rounds to nearest even in the default mode */
    double q = nearbyint(ldexp(a, fb - e));
    if (q >= (double)(2 << fb)) {                             /* rounded up into the next binade */
        q = (double)(1 << fb);
        e += 1;
    }
    int field = e + bias;
    long long frac = (long long)q;
    if (frac < (1 << fb))
        field = 0;                                            /* stayed subnormal */
    else
        frac -= (1 << fb);
    if (field >= emax_field) return (uint16_t)(sign | (emax_field << fb));
    return (uint16_t)(sign | (field << fb) | (int)frac);
}

/* The conversions themselves, exported so that tests can pin them against library conversions. */
double cnnmem_ref_widen16(unsigned h, int dtype) { return widen16((uint16_t)h, dtype); }
unsigned cnnmem_ref_narrow16(double x, int dtype) { return narrow16(x, dtype); }

static int dtype16_ok(int dtype) { return dtype == REF_F16 || dtype == REF_BF16; }

/* Layout change of a tensor of 16-bit words (Section IV.C): words move untouched. */
int cnnmem_ref_transform16(const uint16_t *src, uint16_t *dst, int N, int C, int H, int W,
                           int src_layout, int dst_layout)
{
    if (!src || !dst || N <= 0 || C <= 0 || H <= 0 || W <= 0)
        return REF_ERR_INVALID_ARG;
    if ((src_layout != REF_NCHW && src_layout != REF_CHWN) ||
        (dst_layout != REF_NCHW && dst_layout != REF_CHWN))
        return REF_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    dst[at(dst_layout, N, C, H, W, n, c, h, w)] =
                        src[at(src_layout, N, C, H, W, n, c, h, w)];
    return REF_OK;
}

/* Pooling (Equation 2) on 16-bit storage: the maximum is one of the inputs, the
 * average is the exact sum over kh*kw, rounded once. */
int cnnmem_ref_pool16(const uint16_t *src, uint16_t *dst, int N, int C, int H, int W, int layout,
                      int mode, int kh, int kw, int sh, int sw, int ph, int pw, int dtype)
{
    if (!src || !dst || !dtype16_ok(dtype) || !pool_args_ok(N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw))
        return REF_ERR_INVALID_ARG;
    const int Ho = pooled_extent(H, kh, sh, ph);
    const int Wo = pooled_extent(W, kw, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    double best = -INFINITY, sum = 0.0;
                    uint16_t best_bits = (uint16_t)(0x8000 | (((1 << exp_bits_of(dtype)) - 1) << frac_bits_of(dtype)));
                    for (int y = 0; y < kh; ++y)
                        for (int x = 0; x < kw; ++x) {
                            const int r = i * sh - ph + y;
                            const int q = j * sw - pw + x;
                            if (r < 0 || r >= H || q < 0 || q >= W)
                                continue;
                            const uint16_t bits = src[at(layout, N, C, H, W, n, c, r, q)];
                            const double v = widen16(bits, dtype);
                            if (v > best) { best = v; best_bits = bits; }
                            sum += v;                          /* exact: few terms of <= 11 significant bits */
                        }
                    dst[at(layout, N, C, Ho, Wo, n, c, i, j)] =
                        mode == REF_POOL_MAX ? best_bits : narrow16(sum / (double)(kh * kw), dtype);
                }
    return REF_OK;
}

/* Softmax (Section II.A, steps 1-5) on 16-bit storage. */
int cnnmem_ref_softmax16(const uint16_t *logits, uint16_t *probs, int N, int classes, int dtype)
{
    if (!logits || !probs || N <= 0 || classes <= 0 || !dtype16_ok(dtype))
        return REF_ERR_INVALID_ARG;
    int failed = 0;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const uint16_t *in = logits + (size_t)n * classes;
        uint16_t *out = probs + (size_t)n * classes;
        double *mid = (double *)malloc((size_t)classes * sizeof(double));
        if (!mid) {
#pragma omp atomic write
            failed = 1;
            continue;
        }
        double maxv = widen16(in[0], dtype);                   /* step 1 */
        for (int c = 1; c < classes; ++c) {
            const double v = widen16(in[c], dtype);
            if (v > maxv) maxv = v;
        }
        double sumv = 0.0;
        for (int c = 0; c < classes; ++c) {                    /* steps 2-4 */
            mid[c] = exp(widen16(in[c], dtype) - maxv);
            sumv += mid[c];
        }
        for (int c = 0; c < classes; ++c)                      /* step 5 */
            out[c] = narrow16(mid[c] / sumv, dtype);
        free(mid);
    }
    return failed ? REF_ERR_NOMEM : REF_OK;
}

/* ---- backward passes (training; the paper's footnote in Section II.A notes that the same
 * data structures serve the forward and the backward pass).  The paper defines only the
 * forward operations; these are their textbook derivatives, written as scatters over the
 * forward definition above. ---- */

/* Pooling backward.  Every output (n, c, i, j) sends its incoming gradient ddst back over
 * its window: the average gives each in-image tap 1/(kh*kw) of it (Equation 2's divisor);
 * the maximum gives all of it to the tap that holds the maximum, the first one in scan
 * order (rows, then columns) when several taps tie.  Gradients are accumulated in fp64
 * and rounded once.  `src` is the forward input (unused for the average, may be NULL),
 * `dsrc` has the shape and layout of `src`, `ddst` those of the forward output. */
int cnnmem_ref_pool_backward(const float *src, const float *ddst, float *dsrc, int N, int C, int H, int W,
                             int layout, int mode, int kh, int kw, int sh, int sw, int ph, int pw)
{
    if (!ddst || !dsrc || (mode == REF_POOL_MAX && !src) ||
        !pool_args_ok(N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw))
        return REF_ERR_INVALID_ARG;
    const int Ho = pooled_extent(H, kh, sh, ph);
    const int Wo = pooled_extent(W, kw, sw, pw);
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double *acc = (double *)calloc((size_t)H * W, sizeof(double));
            if (!acc) {
#pragma omp atomic write
                failed = 1;
                continue;
            }
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    const double g = (double)ddst[at(layout, N, C, Ho, Wo, n, c, i, j)];
                    int best_r = -1, best_q = -1;
                    float best = -INFINITY;
                    for (int y = 0; y < kh; ++y)
                        for (int x = 0; x < kw; ++x) {
                            const int r = i * sh - ph + y;
                            const int q = j * sw - pw + x;
                            if (r < 0 || r >= H || q < 0 || q >= W)
                                continue;
                            if (mode == REF_POOL_AVG) {
                                acc[(size_t)r * W + q] += g / (double)(kh * kw);
                            } else {
                                const float v = src[at(layout, N, C, H, W, n, c, r, q)];
                                if (best_r < 0 || v > best) { best = v; best_r = r; best_q = q; }
                            }
                        }
                    if (mode == REF_POOL_MAX)
                        acc[(size_t)best_r * W + best_q] += g;
                }
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    dsrc[at(layout, N, C, H, W, n, c, h, w)] = (float)acc[(size_t)h * W + w];
            free(acc);
        }
    return failed ? REF_ERR_NOMEM : REF_OK;
}

/* Softmax backward: with p = softmax(z) row by row, dz_c = p_c * (dp_c - sum_k dp_k p_k)
 * (the Jacobian diag(p) - p p^T applied to dp). */
int cnnmem_ref_softmax_backward(const float *probs, const float *dprobs, float *dlogits, int N, int classes)
{
    if (!probs || !dprobs || !dlogits || N <= 0 || classes <= 0)
        return REF_ERR_INVALID_ARG;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const float *p = probs + (size_t)n * classes;
        const float *dp = dprobs + (size_t)n * classes;
        float *dz = dlogits + (size_t)n * classes;
        double dot = 0.0;
        for (int c = 0; c < classes; ++c)
            dot += (double)dp[c] * (double)p[c];
        for (int c = 0; c < classes; ++c)
            dz[c] = (float)((double)p[c] * ((double)dp[c] - dot));
    }
    return REF_OK;
}

/* General axis permutation of a tensor of 16-bit words (see cnnmem_ref_permute). */
int cnnmem_ref_permute16(const uint16_t *src, uint16_t *dst, const int *dims, const int *perm)
{
    if (!src || !dst || !dims || !perm) return REF_ERR_INVALID_ARG;
    int seen[4] = {0, 0, 0, 0};
    for (int i = 0; i < 4; ++i) {
        if (dims[i] <= 0 || perm[i] < 0 || perm[i] > 3 || seen[perm[i]]) return REF_ERR_INVALID_ARG;
        seen[perm[i]] = 1;
    }
    size_t ss[4];
    ss[3] = 1;
    for (int a = 2; a >= 0; --a) ss[a] = ss[a + 1] * (size_t)dims[a + 1];
    const int e0 = dims[perm[0]], e1 = dims[perm[1]], e2 = dims[perm[2]], e3 = dims[perm[3]];
    const size_t t0 = ss[perm[0]], t1 = ss[perm[1]], t2 = ss[perm[2]], t3 = ss[perm[3]];
#pragma omp parallel for schedule(static)
    for (int i0 = 0; i0 < e0; ++i0)
        for (int i1 = 0; i1 < e1; ++i1)
            for (int i2 = 0; i2 < e2; ++i2)
                for (int i3 = 0; i3 < e3; ++i3)
                    dst[(((size_t)i0 * e1 + i1) * e2 + i2) * e3 + i3] = src[i0 * t0 + i1 * t1 + i2 * t2 + i3 * t3];
    return REF_OK;
}
