// C ABI of libcnnmem: argument validation and dispatch.  No HIP call is made
// before the arguments of a call have been found valid, and none at load time,
// so the library loads (and rejects bad calls) on a machine without a GPU.
#include "cnnmem.h"
#include "common.hpp"

using namespace cnnmem;

namespace {

bool layout_ok(int l) { return l == CNNMEM_NCHW || l == CNNMEM_CHWN; }

bool window_ok(int H, int W, int kh, int kw, int sh, int sw, int ph, int pw) {
    if (H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0) return false;
    if (ph > kh / 2 || pw > kw / 2) return false;               // every window keeps at least one tap
    if ((long long)H + 2LL * ph < kh || (long long)W + 2LL * pw < kw) return false;
    return true;
}

int pooled_extent(int L, int k, int s, int p) { return (int)(((long long)L + 2LL * p - k) / s + 1); }

}  // namespace

extern "C" {

int cnnmem_transform(const float* src, float* dst, int N, int C, int H, int W, int src_layout,
                     int dst_layout, void* hip_stream) {
    if (!src || !dst || N <= 0 || C <= 0 || H <= 0 || W <= 0) return CNNMEM_ERR_INVALID_ARG;
    if (!layout_ok(src_layout) || !layout_ok(dst_layout)) return CNNMEM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 3u) return CNNMEM_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const long long limit = 1LL << 46;                         // element-count ceiling, far above any HBM
    const long long CH = (long long)C * H;                     // < 2^62
    if (CH > limit / W || CH * W > limit / N) return CNNMEM_ERR_UNSUPPORTED;
    const long long M = CH * W;
    if (src_layout == dst_layout) return launch_copy(src, dst, M * N, st);
    // NCHW is [N][M], CHWN is [M][N] (Section IV.C): a 2-D transpose either way.
    if (src_layout == CNNMEM_NCHW) return launch_transpose2d(src, dst, N, M, st);
    return launch_transpose2d(src, dst, M, N, st);
}

int cnnmem_permute(const float* src, float* dst, const int* dims, const int* perm, void* hip_stream) {
    if (!src || !dst || !dims || !perm) return CNNMEM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 3u) return CNNMEM_ERR_INVALID_ARG;
    bool seen[4] = {false, false, false, false};
    long long total = 1;
    const long long limit = 1LL << 46;
    for (int i = 0; i < 4; ++i) {
        if (dims[i] <= 0 || perm[i] < 0 || perm[i] > 3 || seen[perm[i]]) return CNNMEM_ERR_INVALID_ARG;
        seen[perm[i]] = true;
        if (total > limit / dims[i]) return CNNMEM_ERR_UNSUPPORTED;
        total *= dims[i];
    }
    return launch_permute(src, dst, dims, perm, static_cast<hipStream_t>(hip_stream));
}

int cnnmem_permute_dtype(const void* src, void* dst, const int* dims, const int* perm, int dtype, void* hip_stream) {
    if (dtype == CNNMEM_F32)
        return cnnmem_permute(static_cast<const float*>(src), static_cast<float*>(dst), dims, perm, hip_stream);
    if (dtype != CNNMEM_F16 && dtype != CNNMEM_BF16) return CNNMEM_ERR_INVALID_ARG;
    if (!src || !dst || !dims || !perm) return CNNMEM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 1u) return CNNMEM_ERR_INVALID_ARG;
    bool seen[4] = {false, false, false, false};
    long long total = 1;
    const long long limit = 1LL << 46;
    for (int i = 0; i < 4; ++i) {
        if (dims[i] <= 0 || perm[i] < 0 || perm[i] > 3 || seen[perm[i]]) return CNNMEM_ERR_INVALID_ARG;
        seen[perm[i]] = true;
        if (total > limit / dims[i]) return CNNMEM_ERR_UNSUPPORTED;
        total *= dims[i];
    }
    return launch_permute16(src, dst, dims, perm, static_cast<hipStream_t>(hip_stream));
}

int cnnmem_relayout(const float* src, float* dst, int N, int C, int H, int W, const char* src_layout,
                    const char* dst_layout, void* hip_stream) {
    return cnnmem_relayout_dtype(src, dst, N, C, H, W, src_layout, dst_layout, CNNMEM_F32, hip_stream);
}

int cnnmem_relayout_dtype(const void* src, void* dst, int N, int C, int H, int W, const char* src_layout,
                          const char* dst_layout, int dtype, void* hip_stream) {
    if (!src || !dst || N <= 0 || C <= 0 || H <= 0 || W <= 0 || !src_layout || !dst_layout)
        return CNNMEM_ERR_INVALID_ARG;
    // a layout is the four letters N, C, H, W, each once, slowest axis first
    auto letter = [](char c) { return c == 'N' ? 0 : c == 'C' ? 1 : c == 'H' ? 2 : c == 'W' ? 3 : -1; };
    const int extent[4] = {N, C, H, W};
    int where_in_src[4] = {-1, -1, -1, -1};                    // letter -> axis of the source
    int dims[4], perm[4];
    for (int i = 0; i < 4; ++i) {
        const int l = src_layout[i] ? letter(src_layout[i]) : -1;
        if (l < 0 || where_in_src[l] >= 0) return CNNMEM_ERR_INVALID_ARG;
        where_in_src[l] = i;
        dims[i] = extent[l];
    }
    if (src_layout[4] != 0) return CNNMEM_ERR_INVALID_ARG;
    bool used[4] = {false, false, false, false};
    for (int i = 0; i < 4; ++i) {
        const int l = dst_layout[i] ? letter(dst_layout[i]) : -1;
        if (l < 0 || used[l]) return CNNMEM_ERR_INVALID_ARG;
        used[l] = true;
        perm[i] = where_in_src[l];
    }
    if (dst_layout[4] != 0) return CNNMEM_ERR_INVALID_ARG;
    return cnnmem_permute_dtype(src, dst, dims, perm, dtype, hip_stream);
}

int cnnmem_pool_out_dims(int H, int W, int kh, int kw, int sh, int sw, int ph, int pw, int* Ho, int* Wo) {
    if (!Ho || !Wo || !window_ok(H, W, kh, kw, sh, sw, ph, pw)) return CNNMEM_ERR_INVALID_ARG;
    *Ho = pooled_extent(H, kh, sh, ph);
    *Wo = pooled_extent(W, kw, sw, pw);
    return CNNMEM_OK;
}

int cnnmem_pool_tuned(const float* src, float* dst, int N, int C, int H, int W, int layout, int mode, int kh,
                      int kw, int sh, int sw, int ph, int pw, const cnnmem_pool_tuning* tuning, void* hip_stream) {
    if (!src || !dst || N <= 0 || C <= 0) return CNNMEM_ERR_INVALID_ARG;
    if (!window_ok(H, W, kh, kw, sh, sw, ph, pw)) return CNNMEM_ERR_INVALID_ARG;
    if (!layout_ok(layout)) return CNNMEM_ERR_INVALID_ARG;
    if (mode != CNNMEM_POOL_MAX && mode != CNNMEM_POOL_AVG) return CNNMEM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 3u) return CNNMEM_ERR_INVALID_ARG;
    PoolTuning tune;
    if (tuning) {
        if (tuning->rows_per_lane < 0 || tuning->rows_per_lane > 4) return CNNMEM_ERR_INVALID_ARG;
        if (tuning->cols_per_lane < 0 || tuning->cols_per_lane > 2) return CNNMEM_ERR_INVALID_ARG;
        if (tuning->workgroups_per_cu < -1 || tuning->workgroups_per_cu == 1 || tuning->workgroups_per_cu > 8)
            return CNNMEM_ERR_INVALID_ARG;
        if (tuning->nchw_kernel < 0 || tuning->nchw_kernel > 2) return CNNMEM_ERR_INVALID_ARG;
        if (tuning->slab_lanes != 0 && tuning->slab_lanes != 256 && tuning->slab_lanes != 512 &&
            tuning->slab_lanes != 1024)
            return CNNMEM_ERR_INVALID_ARG;
        tune.rows_per_lane = tuning->rows_per_lane;
        tune.cols_per_lane = tuning->cols_per_lane;
        tune.workgroups_per_cu = tuning->workgroups_per_cu;
        tune.nchw_kernel = tuning->nchw_kernel;
        tune.slab_lanes = tuning->slab_lanes;
    }
    if ((long long)H * W > (1LL << 30) || (long long)kh * kw > (1 << 24)) return CNNMEM_ERR_UNSUPPORTED;
    PoolGeom g;
    g.N = N; g.C = C; g.H = H; g.W = W;
    g.kh = kh; g.kw = kw; g.sh = sh; g.sw = sw; g.ph = ph; g.pw = pw;
    g.mode = mode;
    g.Ho = pooled_extent(H, kh, sh, ph);
    g.Wo = pooled_extent(W, kw, sw, pw);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return layout == CNNMEM_NCHW ? launch_pool_nchw(src, dst, g, tune, st) : launch_pool_chwn(src, dst, g, tune, st);
}

int cnnmem_pool(const float* src, float* dst, int N, int C, int H, int W, int layout, int mode, int kh,
                int kw, int sh, int sw, int ph, int pw, void* hip_stream) {
    return cnnmem_pool_tuned(src, dst, N, C, H, W, layout, mode, kh, kw, sh, sw, ph, pw, nullptr, hip_stream);
}

int cnnmem_softmax(const float* logits, float* probs, int N, int classes, void* hip_stream) {
    if (!logits || !probs || N <= 0 || classes <= 0) return CNNMEM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(logits) | reinterpret_cast<uintptr_t>(probs)) & 3u)
        return CNNMEM_ERR_INVALID_ARG;
    return launch_softmax(logits, probs, N, classes, static_cast<hipStream_t>(hip_stream));
}

int cnnmem_pool_backward(const float* src, const float* ddst, float* dsrc, int N, int C, int H, int W, int layout,
                         int mode, int kh, int kw, int sh, int sw, int ph, int pw, void* hip_stream) {
    if (!ddst || !dsrc || N <= 0 || C <= 0) return CNNMEM_ERR_INVALID_ARG;
    if (!window_ok(H, W, kh, kw, sh, sw, ph, pw)) return CNNMEM_ERR_INVALID_ARG;
    if (!layout_ok(layout)) return CNNMEM_ERR_INVALID_ARG;
    if (mode != CNNMEM_POOL_MAX && mode != CNNMEM_POOL_AVG) return CNNMEM_ERR_INVALID_ARG;
    if (mode == CNNMEM_POOL_MAX && !src) return CNNMEM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(ddst) | reinterpret_cast<uintptr_t>(dsrc)) & 3u)
        return CNNMEM_ERR_INVALID_ARG;
    if ((long long)H * W > (1LL << 30) || (long long)kh * kw > (1 << 24)) return CNNMEM_ERR_UNSUPPORTED;
    PoolGeom g;
    g.N = N; g.C = C; g.H = H; g.W = W;
    g.kh = kh; g.kw = kw; g.sh = sh; g.sw = sw; g.ph = ph; g.pw = pw;
    g.mode = mode;
    g.Ho = pooled_extent(H, kh, sh, ph);
    g.Wo = pooled_extent(W, kw, sw, pw);
    return launch_pool_backward(src, ddst, dsrc, g, layout, static_cast<hipStream_t>(hip_stream));
}

int cnnmem_softmax_backward(const float* probs, const float* dprobs, float* dlogits, int N, int classes,
                            void* hip_stream) {
    if (!probs || !dprobs || !dlogits || N <= 0 || classes <= 0) return CNNMEM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(probs) | reinterpret_cast<uintptr_t>(dprobs) |
         reinterpret_cast<uintptr_t>(dlogits)) & 3u)
        return CNNMEM_ERR_INVALID_ARG;
    return launch_softmax_backward(probs, dprobs, dlogits, N, classes, static_cast<hipStream_t>(hip_stream));
}

int cnnmem_transform_dtype(const void* src, void* dst, int N, int C, int H, int W, int src_layout, int dst_layout,
                           int dtype, void* hip_stream) {
    if (dtype == CNNMEM_F32)
        return cnnmem_transform(static_cast<const float*>(src), static_cast<float*>(dst), N, C, H, W, src_layout,
                                dst_layout, hip_stream);
    if (dtype != CNNMEM_F16 && dtype != CNNMEM_BF16) return CNNMEM_ERR_INVALID_ARG;
    if (!src || !dst || N <= 0 || C <= 0 || H <= 0 || W <= 0) return CNNMEM_ERR_INVALID_ARG;
    if (!layout_ok(src_layout) || !layout_ok(dst_layout)) return CNNMEM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 1u) return CNNMEM_ERR_INVALID_ARG;
    const long long limit = 1LL << 46;
    const long long CH = (long long)C * H;
    if (CH > limit / W || CH * W > limit / N) return CNNMEM_ERR_UNSUPPORTED;
    return launch_transform16(src, dst, N, CH * W, src_layout, dst_layout, static_cast<hipStream_t>(hip_stream));
}

int cnnmem_pool_dtype(const void* src, void* dst, int N, int C, int H, int W, int layout, int mode, int kh, int kw,
                      int sh, int sw, int ph, int pw, int dtype, void* hip_stream) {
    if (dtype == CNNMEM_F32)
        return cnnmem_pool(static_cast<const float*>(src), static_cast<float*>(dst), N, C, H, W, layout, mode, kh, kw,
                           sh, sw, ph, pw, hip_stream);
    if (dtype != CNNMEM_F16 && dtype != CNNMEM_BF16) return CNNMEM_ERR_INVALID_ARG;
    if (!src || !dst || N <= 0 || C <= 0) return CNNMEM_ERR_INVALID_ARG;
    if (!window_ok(H, W, kh, kw, sh, sw, ph, pw)) return CNNMEM_ERR_INVALID_ARG;
    if (!layout_ok(layout)) return CNNMEM_ERR_INVALID_ARG;
    if (mode != CNNMEM_POOL_MAX && mode != CNNMEM_POOL_AVG) return CNNMEM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 1u) return CNNMEM_ERR_INVALID_ARG;
    if ((long long)H * W > (1LL << 30) || (long long)kh * kw > (1 << 24)) return CNNMEM_ERR_UNSUPPORTED;
    PoolGeom g;
    g.N = N; g.C = C; g.H = H; g.W = W;
    g.kh = kh; g.kw = kw; g.sh = sh; g.sw = sw; g.ph = ph; g.pw = pw;
    g.mode = mode;
    g.Ho = pooled_extent(H, kh, sh, ph);
    g.Wo = pooled_extent(W, kw, sw, pw);
    return launch_pool16(src, dst, g, layout, dtype, static_cast<hipStream_t>(hip_stream));
}

int cnnmem_softmax_dtype(const void* logits, void* probs, int N, int classes, int dtype, void* hip_stream) {
    if (dtype == CNNMEM_F32)
        return cnnmem_softmax(static_cast<const float*>(logits), static_cast<float*>(probs), N, classes, hip_stream);
    if (dtype != CNNMEM_F16 && dtype != CNNMEM_BF16) return CNNMEM_ERR_INVALID_ARG;
    if (!logits || !probs || N <= 0 || classes <= 0) return CNNMEM_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(logits) | reinterpret_cast<uintptr_t>(probs)) & 1u)
        return CNNMEM_ERR_INVALID_ARG;
    return launch_softmax16(logits, probs, N, classes, dtype, static_cast<hipStream_t>(hip_stream));
}

int cnnmem_choose_layout(int layer_kind, int N, int C, int Ct, int Nt, int* layout) {
    if (!layout || N <= 0 || C <= 0 || Ct < 0 || Nt < 0) return CNNMEM_ERR_INVALID_ARG;
    switch (layer_kind) {
        case CNNMEM_LAYER_CONV:
            // Section IV.A: few input maps make the NCHW unroll expensive; a large batch gives CHWN
            // both coalescing and register reuse.
            *layout = (C < Ct || N >= Nt) ? CNNMEM_CHWN : CNNMEM_NCHW;
            return CNNMEM_OK;
        case CNNMEM_LAYER_POOL:
            *layout = CNNMEM_CHWN;                              // Section IV.B
            return CNNMEM_OK;
        case CNNMEM_LAYER_OTHER:
            return CNNMEM_OK;
        default:
            return CNNMEM_ERR_INVALID_ARG;
    }
}

int cnnmem_plan_layouts(const cnnmem_layer* layers, int n_layers, int Ct, int Nt, int input_layout,
                        int pool_policy, int* layouts, int* transform_before, int* n_transforms) {
    if (!layers || !layouts || !transform_before || n_layers <= 0) return CNNMEM_ERR_INVALID_ARG;
    if (!layout_ok(input_layout)) return CNNMEM_ERR_INVALID_ARG;
    if (pool_policy != CNNMEM_POOL_PREFERS_CHWN && pool_policy != CNNMEM_POOL_KEEPS_LAYOUT)
        return CNNMEM_ERR_INVALID_ARG;
    for (int i = 0; i < n_layers; ++i) {                        // validate everything before writing anything
        int probe = CNNMEM_NCHW;
        if (cnnmem_choose_layout(layers[i].kind, layers[i].N, layers[i].C, Ct, Nt, &probe) != CNNMEM_OK)
            return CNNMEM_ERR_INVALID_ARG;
    }
    int current = input_layout, count = 0;
    for (int i = 0; i < n_layers; ++i) {
        int want = current;                                     // no preference: inherit
        const bool inherits = layers[i].kind == CNNMEM_LAYER_OTHER ||
                              (layers[i].kind == CNNMEM_LAYER_POOL && pool_policy == CNNMEM_POOL_KEEPS_LAYOUT);
        if (!inherits) cnnmem_choose_layout(layers[i].kind, layers[i].N, layers[i].C, Ct, Nt, &want);
        layouts[i] = want;
        transform_before[i] = want != current;
        count += transform_before[i];
        current = want;
    }
    if (n_transforms) *n_transforms = count;
    return CNNMEM_OK;
}

const char* cnnmem_status_string(int status) {
    switch (status) {
        case CNNMEM_OK: return "ok";
        case CNNMEM_ERR_INVALID_ARG: return "invalid argument";
        case CNNMEM_ERR_UNSUPPORTED: return "unsupported request";
        case CNNMEM_ERR_RUNTIME: return "HIP runtime error at kernel launch";
        default: return "unknown status";
    }
}

int cnnmem_version(void) { return 200; }   // 0.2.0: storage orders, 16-bit storage, backward passes

}  // extern "C"
