/*
 * cnnmem.h -- C ABI of the MI355X (gfx950) library for the memory-bound CNN
 * layers: 4-D layout transformation, pooling in either layout, fused softmax.
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers to fp32 data owned by the caller;
 *     they must be 4-byte aligned (16-byte alignment enables the fastest
 *     kernels, anything else takes a slower but equally exact path).
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default
 *     stream).  Calls only enqueue work on that stream: they never
 *     synchronise, never allocate device memory and keep no state.
 *   - Every function returns a CNNMEM_* status.  Arguments are validated on
 *     the host before any HIP call; an invalid call enqueues nothing.
 *   - Source and destination must not overlap unless stated otherwise.
 *   - Tensors may hold more than 2^31 elements; every extent fits an int.
 */
#ifndef CNNMEM_H
#define CNNMEM_H

#ifndef CNNMEM_API
#define CNNMEM_API __attribute__((visibility("default")))
#endif

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CNNMEM_OK = 0,
    CNNMEM_ERR_INVALID_ARG = 1, /* null pointer, non-positive extent, bad enum, bad window */
    CNNMEM_ERR_UNSUPPORTED = 2, /* legal request no kernel covers (e.g. extent overflow)  */
    CNNMEM_ERR_RUNTIME = 3      /* HIP reported an error when the kernel was launched     */
};

/* Layout tag of a logical N x C x H x W tensor (Section II.A, Section IV.A).
 *   NCHW: element (n,c,h,w) at ((n*C + c)*H + h)*W + w   (W contiguous)
 *   CHWN: element (n,c,h,w) at ((c*H + h)*W + w)*N + n   (N contiguous)   */
enum { CNNMEM_NCHW = 0, CNNMEM_CHWN = 1 };

/* Pooling operation (Section II.A: "average or max"). */
enum { CNNMEM_POOL_MAX = 0, CNNMEM_POOL_AVG = 1 };

/*
 * Layout transformation (Section IV.C).  Copies the N*C*H*W elements of `src`
 * (stored in `src_layout`) to `dst` in `dst_layout`.  Because C, H and W keep
 * their relative order, this is the transpose of an [N][C*H*W] matrix into
 * [C*H*W][N] or back.  Words are moved bit for bit (NaN payloads and signed
 * zeros survive).  Equal layouts give a plain device copy.
 *   src, dst : device, N*C*H*W floats each, not overlapping.
 * Errors: INVALID_ARG for null pointers, extents <= 0 or unknown layout tags.
 */
CNNMEM_API int cnnmem_transform(const float *src, float *dst, int N, int C, int H, int W,
                     int src_layout, int dst_layout, void *hip_stream);

/*
 * General storage-order change.  A 4-D tensor can be stored in 24 orders
 * (Section I); besides NCHW and CHWN the paper names HWCN (Section IV.A) and the
 * NHWC order of the libraries it compares with.  `dims` holds the four source
 * extents, slowest axis first; destination axis i is source axis perm[i], so the
 * destination extents are dims[perm[0]], ..., dims[perm[3]]
 * (dst[i0][i1][i2][i3] = src at the coordinates j with j[perm[k]] = ik).
 * Words are moved bit for bit.
 *   src, dst   : device, dims[0]*dims[1]*dims[2]*dims[3] floats each, not
 *                overlapping, 4-byte aligned (16-byte alignment enables 128-bit
 *                accesses).
 *   dims, perm : host, four ints each, read before the call returns.
 * Errors: INVALID_ARG for null pointers, extents <= 0 or a perm that is not a
 * permutation of 0..3; UNSUPPORTED beyond 2^31 - 1 tiles in one launch (far above any HBM).
 */
CNNMEM_API int cnnmem_permute(const float *src, float *dst, const int *dims, const int *perm, void *hip_stream);

/*
 * The same between two spelled layouts: `src_layout` and `dst_layout` are
 * strings of the four letters N, C, H, W, each once, slowest axis first
 * ("NCHW", "CHWN", "NHWC", "HWCN", ... all 24).  Equal layouts give a device copy.
 *   src, dst : device, N*C*H*W floats each, not overlapping.
 * Errors: INVALID_ARG for null pointers, extents <= 0 or a malformed layout string.
 */
CNNMEM_API int cnnmem_relayout(const float *src, float *dst, int N, int C, int H, int W,
                               const char *src_layout, const char *dst_layout, void *hip_stream);

/*
 * Backward passes (fp32).  The paper's forward definitions (Equation 2, the softmax
 * steps of Section II.A) differentiated; its footnote in Section II.A notes that the
 * same data structures serve both passes.
 *
 * cnnmem_pool_backward: gradient of cnnmem_pool with respect to its input.
 *   src  : device, the forward input, N*C*H*W floats in `layout`; needed for
 *          CNNMEM_POOL_MAX only (may be null for CNNMEM_POOL_AVG).
 *   ddst : device, the gradient arriving at the forward output, N*C*Ho*Wo floats in `layout`.
 *   dsrc : device, out, N*C*H*W floats in `layout`; every element is written (inputs that
 *          no window covers get 0).  Must not overlap src or ddst.
 *   Average: each in-image tap of a window receives ddst / (kh*kw).  Maximum: the whole
 *   ddst of a window goes to the tap holding the maximum, the first in scan order (rows,
 *   then columns) when several tie.  No index tensor from the forward pass is needed: the
 *   windows are re-scanned.
 * cnnmem_softmax_backward: dlogits[n][c] = probs[n][c] * (dprobs[n][c] - sum_k dprobs[n][k]*probs[n][k]).
 *   probs : device, the forward output; dprobs: device, the gradient arriving at it;
 *   dlogits: device, out; N*classes floats each.  dlogits may alias dprobs or probs.
 * Errors as for the forward entry points.
 */
CNNMEM_API int cnnmem_pool_backward(const float *src, const float *ddst, float *dsrc, int N, int C, int H, int W,
                                    int layout, int mode, int kh, int kw, int sh, int sw, int ph, int pw,
                                    void *hip_stream);
CNNMEM_API int cnnmem_softmax_backward(const float *probs, const float *dprobs, float *dlogits, int N, int classes,
                                       void *hip_stream);

/*
 * Storage formats.  CNNMEM_F32 is what every entry point above works on.  With
 * CNNMEM_F16 (IEEE binary16) or CNNMEM_BF16 (the upper half of binary32) a tensor
 * element is 16 bits: the paper's closing remarks expect half precision to push
 * these layers further towards the memory bound, and it halves the bytes they move.
 * Only storage changes: stored values are widened exactly, pooling sums and the
 * softmax are computed in fp32 as for CNNMEM_F32, and each result is rounded once,
 * to nearest even, to the storage format.  The transform moves 16-bit words bit for
 * bit, the maximum of a window is one of its inputs bit for bit.
 */
enum { CNNMEM_F32 = 0, CNNMEM_F16 = 1, CNNMEM_BF16 = 2 };

/*
 * cnnmem_transform / cnnmem_pool / cnnmem_softmax on tensors of `dtype`.  Arguments,
 * layouts, ownership and errors are those of the fp32 entry points; pointers must be
 * aligned to the element size (16-byte alignment enables the 128-bit kernels), and
 * an unknown dtype is an INVALID_ARG.  With CNNMEM_F32 they are the fp32 calls.
 */
CNNMEM_API int cnnmem_transform_dtype(const void *src, void *dst, int N, int C, int H, int W, int src_layout,
                                      int dst_layout, int dtype, void *hip_stream);
CNNMEM_API int cnnmem_pool_dtype(const void *src, void *dst, int N, int C, int H, int W, int layout, int mode,
                                 int kh, int kw, int sh, int sw, int ph, int pw, int dtype, void *hip_stream);
CNNMEM_API int cnnmem_softmax_dtype(const void *logits, void *probs, int N, int classes, int dtype,
                                    void *hip_stream);
/* cnnmem_permute / cnnmem_relayout on tensors of `dtype` (words move bit for bit). */
CNNMEM_API int cnnmem_permute_dtype(const void *src, void *dst, const int *dims, const int *perm, int dtype,
                                    void *hip_stream);
CNNMEM_API int cnnmem_relayout_dtype(const void *src, void *dst, int N, int C, int H, int W, const char *src_layout,
                                     const char *dst_layout, int dtype, void *hip_stream);

/*
 * Pooled output extent (host only, no GPU work):
 *   Ho = floor((H + 2*ph - kh) / sh) + 1,  Wo likewise
 * -- the rule Fig. 8 of Section V.A implies (12 inputs, window 4, stride 2 give
 * 5 outputs).  Errors: INVALID_ARG under the same window rules as cnnmem_pool,
 * or if Ho / Wo is null.
 */
CNNMEM_API int cnnmem_pool_out_dims(int H, int W, int kh, int kw, int sh, int sw, int ph, int pw,
                         int *Ho, int *Wo);

/*
 * Pooling (Equation 2 of Section II.A for the average; the maximum for MAX),
 * computed directly in the layout the tensor is stored in (Section IV.B,
 * Section V.A).  Output element (n,c,i,j) covers input rows i*sh - ph + y,
 * y < kh, and columns j*sw - pw + x, x < kw.  Taps that fall outside the image
 * are ignored by MAX and add zero to AVG, whose divisor is always kh*kw.
 *   src : device, N*C*H*W floats in `layout`.
 *   dst : device, N*C*Ho*Wo floats, written in the same `layout`.
 * MAX returns one of the inputs exactly (inputs are assumed NaN-free; the sign
 * of a zero maximum is unspecified when +0 and -0 tie).  AVG accumulates in
 * fp32.
 * Errors: INVALID_ARG for null pointers; N, C, H, W, kh, kw, sh, sw <= 0;
 * ph, pw < 0; ph > kh/2 or pw > kw/2; H + 2*ph < kh or W + 2*pw < kw; unknown
 * layout or mode.
 */
CNNMEM_API int cnnmem_pool(const float *src, float *dst, int N, int C, int H, int W, int layout, int mode,
                int kh, int kw, int sh, int sw, int ph, int pw, void *hip_stream);

/*
 * Launch-shape choices for one pooling call: the knobs the paper's auto-tuner
 * searches (Section V.A: how many outputs a thread computes in each direction,
 * traded against the parallelism left) plus this part's occupancy cap.  A zero
 * field means "library default"; fields that do not apply to the kernel that
 * serves the call are ignored.  Results never depend on the tuning.
 */
typedef struct cnnmem_pool_tuning {
    int rows_per_lane;     /* CHWN: output rows per lane, 1..4 (run-time windows: at most 3) */
    int cols_per_lane;     /* CHWN: output columns per lane, 1..2                           */
    int workgroups_per_cu; /* cap on resident 256-lane workgroups per CU, 2..8; -1 = no cap */
    int nchw_kernel;       /* NCHW: 1 = row-pair kernel where it applies, 2 = LDS-slab kernel */
    int slab_lanes;        /* NCHW LDS-slab kernel: 256, 512 or 1024 lanes per slab         */
} cnnmem_pool_tuning;

/*
 * cnnmem_pool with explicit launch-shape choices (`tuning` is a HOST pointer and
 * may be null = all defaults).  Same tensors, same results, same errors as
 * cnnmem_pool, plus INVALID_ARG for a field outside the ranges above.
 * `python -m paper_1610_03618_amd.autotune` searches these fields for a shape.
 */
CNNMEM_API int cnnmem_pool_tuned(const float *src, float *dst, int N, int C, int H, int W, int layout, int mode,
                                 int kh, int kw, int sh, int sw, int ph, int pw,
                                 const cnnmem_pool_tuning *tuning, void *hip_stream);

/*
 * Softmax over the categories of each image (Section II.A steps 1-5, fused
 * into one kernel as in Section V.B): for every row n of the row-major
 * [N][classes] matrix, m = max_c x[n][c], e_c = exp(x[n][c] - m),
 * probs[n][c] = e_c / sum_c e_c.  The matrix is read once and written once.
 *   logits, probs : device, N*classes floats each.  probs == logits (exactly
 *                   in place) is allowed; any other overlap is not.
 * fp32 arithmetic; inputs are assumed finite.
 * Errors: INVALID_ARG for null pointers or N, classes <= 0.
 */
CNNMEM_API int cnnmem_softmax(const float *logits, float *probs, int N, int classes, void *hip_stream);

/* ---- layout selection (host only; every pointer below is a HOST pointer) ---- */

/* Kind of layer, as far as layout selection cares. */
enum { CNNMEM_LAYER_CONV = 0, CNNMEM_LAYER_POOL = 1, CNNMEM_LAYER_OTHER = 2 };

/* What a pooling layer asks for.  The paper's GPUs pooled far faster in CHWN
 * (Section IV.B: "CHWN is always preferred"); on MI355X this library pools at the
 * same bandwidth in both layouts, so a pooling layer can simply keep the layout
 * its input arrives in and save the transform. */
enum { CNNMEM_POOL_PREFERS_CHWN = 0, CNNMEM_POOL_KEEPS_LAYOUT = 1 };

/*
 * Layout heuristic of Section IV.A for one layer.  Convolution with batch N and
 * C input feature maps: CHWN if C < Ct or N >= Nt, otherwise NCHW ((Ct, Nt) is
 * a property of the GPU: (32, 128) and (128, 64) on the paper's two).  Pooling:
 * CHWN.  Other layers have no preference: *layout is left untouched and the
 * function returns CNNMEM_OK.
 * Errors: INVALID_ARG for a null pointer, an unknown kind, N, C <= 0 or
 * Ct, Nt < 0.
 */
CNNMEM_API int cnnmem_choose_layout(int layer_kind, int N, int C, int Ct, int Nt, int *layout);

/* One layer of a network for cnnmem_plan_layouts. */
typedef struct cnnmem_layer {
    int kind; /* CNNMEM_LAYER_* */
    int N;    /* batch size */
    int C;    /* input feature maps */
} cnnmem_layer;

/*
 * Layout plan of Section IV.D: one scan over the network sets the layout field
 * of every layer from the heuristic, and a transform is needed wherever a layer's
 * layout differs from the layout its input arrives in.  `input_layout` is the
 * layout of the network input.  Layers without a preference (and pooling under
 * CNNMEM_POOL_KEEPS_LAYOUT) inherit the incoming layout.
 *   layouts          : out, n_layers entries, the layout each layer runs in.
 *   transform_before : out, n_layers entries, 1 if a cnnmem_transform is needed
 *                      in front of layer i, else 0.
 *   n_transforms     : out, optional (may be null), the number of ones above.
 * Errors: INVALID_ARG for null arrays, n_layers <= 0, a bad layer, layout tag or
 * policy.
 */
CNNMEM_API int cnnmem_plan_layouts(const cnnmem_layer *layers, int n_layers, int Ct, int Nt, int input_layout,
                                   int pool_policy, int *layouts, int *transform_before, int *n_transforms);

/* Text for a status code; static storage, never null. */
CNNMEM_API const char *cnnmem_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
CNNMEM_API int cnnmem_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CNNMEM_H */
