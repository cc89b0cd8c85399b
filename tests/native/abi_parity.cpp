// Native check of the C ABI: no Python, no PyTorch.  The program owns its device buffers (hipMalloc) and its
// stream, calls the library's entry points and compares every result with the CPU oracle under the same bars
// as the Python parity tests: transforms and max-pooling bit for bit, average pooling to 1e-6 of the mean tap
// magnitude, softmax to max(2e-6 |ref|, 1e-7).  TEST INFRASTRUCTURE: it links the oracle, the product does not.
// Exit code 0 = every check passed.  Built by __graft_entry__.build(), run by tests/test_gpu_native_abi.py.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "cnnmem.h"

extern "C" {
int cnnmem_ref_transform(const float* src, float* dst, int N, int C, int H, int W, int src_layout, int dst_layout);
int cnnmem_ref_pool(const float* src, float* dst, int N, int C, int H, int W, int layout, int mode, int kh, int kw,
                    int sh, int sw, int ph, int pw);
int cnnmem_ref_softmax(const float* logits, float* probs, int N, int classes);
}

namespace {

int failures = 0;

#define HIP_OK(call)                                                                          \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            std::printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
            std::exit(2);                                                                     \
        }                                                                                     \
    } while (0)

void expect(bool ok, const char* what) {
    std::printf("%-58s %s\n", what, ok ? "ok" : "MISMATCH");
    std::fflush(stdout);
    if (!ok) ++failures;
}

// inputs only: a 64-bit linear congruential generator, uniform in [-1, 1)
struct Rng {
    uint64_t s;
    float next() {
        s = s * 6364136223846793005ULL + 1442695040888963407ULL;
        return (float)((s >> 40) * (1.0 / 8388608.0) - 1.0);
    }
};

struct DeviceBuffer {
    float* p = nullptr;
    size_t n = 0;
    explicit DeviceBuffer(size_t count) : n(count) { HIP_OK(hipMalloc(reinterpret_cast<void**>(&p), count * sizeof(float))); }
    ~DeviceBuffer() { (void)hipFree(p); }
    void upload(const std::vector<float>& h, hipStream_t st) {
        HIP_OK(hipMemcpyAsync(p, h.data(), h.size() * sizeof(float), hipMemcpyHostToDevice, st));
    }
    std::vector<float> download(size_t count, hipStream_t st) {
        std::vector<float> h(count);
        HIP_OK(hipMemcpyAsync(h.data(), p, count * sizeof(float), hipMemcpyDeviceToHost, st));
        HIP_OK(hipStreamSynchronize(st));
        return h;
    }
};

bool same_bits(const std::vector<float>& a, const std::vector<float>& b) {
    return a.size() == b.size() && std::memcmp(a.data(), b.data(), a.size() * sizeof(float)) == 0;
}

void check_layers(int N, int C, int H, int W, hipStream_t st) {
    char what[128];
    const size_t n = (size_t)N * C * H * W;
    Rng rng{(uint64_t)(N * 1000003 + C * 10007 + H * 101 + W)};
    std::vector<float> x(n), xc(n), back(n);
    for (auto& v : x) { const float u = rng.next(); v = u > 0.f ? u : 0.f; }       // what a ReLU layer emits
    DeviceBuffer d_x(n), d_xc(n), d_back(n);
    d_x.upload(x, st);

    cnnmem_ref_transform(x.data(), xc.data(), N, C, H, W, CNNMEM_NCHW, CNNMEM_CHWN);
    int rc = cnnmem_transform(d_x.p, d_xc.p, N, C, H, W, CNNMEM_NCHW, CNNMEM_CHWN, st);
    std::snprintf(what, sizeof what, "transform NCHW->CHWN %dx%dx%dx%d", N, C, H, W);
    expect(rc == CNNMEM_OK && same_bits(d_xc.download(n, st), xc), what);
    rc = cnnmem_transform(d_xc.p, d_back.p, N, C, H, W, CNNMEM_CHWN, CNNMEM_NCHW, st);
    std::snprintf(what, sizeof what, "transform CHWN->NCHW %dx%dx%dx%d (round trip)", N, C, H, W);
    expect(rc == CNNMEM_OK && same_bits(d_back.download(n, st), x), what);

    const int windows[2][2] = {{3, 2}, {2, 2}};
    for (const auto& ws : windows) {
        const int k = ws[0], s = ws[1];
        int Ho = 0, Wo = 0;
        if (cnnmem_pool_out_dims(H, W, k, k, s, s, 0, 0, &Ho, &Wo) != CNNMEM_OK) { expect(false, "pool_out_dims"); continue; }
        const size_t no = (size_t)N * C * Ho * Wo;
        DeviceBuffer d_out(no);
        for (int layout = 0; layout < 2; ++layout) {
            const std::vector<float>& src = layout == CNNMEM_NCHW ? x : xc;
            const float* d_src = layout == CNNMEM_NCHW ? d_x.p : d_xc.p;
            std::vector<float> want(no);
            cnnmem_ref_pool(src.data(), want.data(), N, C, H, W, layout, CNNMEM_POOL_MAX, k, k, s, s, 0, 0);
            rc = cnnmem_pool(d_src, d_out.p, N, C, H, W, layout, CNNMEM_POOL_MAX, k, k, s, s, 0, 0, st);
            std::snprintf(what, sizeof what, "max-pool %dx%d/s%d %s %dx%dx%dx%d", k, k, s, layout ? "CHWN" : "NCHW", N, C, H, W);
            expect(rc == CNNMEM_OK && same_bits(d_out.download(no, st), want), what);
            cnnmem_ref_pool(src.data(), want.data(), N, C, H, W, layout, CNNMEM_POOL_AVG, k, k, s, s, 0, 0);
            rc = cnnmem_pool(d_src, d_out.p, N, C, H, W, layout, CNNMEM_POOL_AVG, k, k, s, s, 0, 0, st);
            const std::vector<float> got = d_out.download(no, st);
            bool ok = rc == CNNMEM_OK;
            for (size_t i = 0; i < no && ok; ++i)       // inputs are >= 0: the result is the mean tap magnitude
                ok = std::fabs((double)got[i] - (double)want[i]) <= 1e-6 * std::fabs((double)want[i]) + 1e-45;
            std::snprintf(what, sizeof what, "avg-pool %dx%d/s%d %s %dx%dx%dx%d", k, k, s, layout ? "CHWN" : "NCHW", N, C, H, W);
            expect(ok, what);
        }
    }
}

void check_softmax(int N, int classes, hipStream_t st) {
    char what[128];
    const size_t n = (size_t)N * classes;
    Rng rng{(uint64_t)(N * 7919 + classes)};
    std::vector<float> z(n), want(n);
    for (auto& v : z) v = 6.f * rng.next();
    for (int r = 0; r < N; r += 8) z[(size_t)r * classes + (size_t)(r % classes)] = 50.f;   // planted outliers
    DeviceBuffer d_z(n), d_p(n);
    d_z.upload(z, st);
    cnnmem_ref_softmax(z.data(), want.data(), N, classes);
    const int rc = cnnmem_softmax(d_z.p, d_p.p, N, classes, st);
    const std::vector<float> got = d_p.download(n, st);
    bool ok = rc == CNNMEM_OK;
    for (size_t i = 0; i < n && ok; ++i) {
        const double bar = std::fmax(2e-6 * std::fabs((double)want[i]), 1e-7);
        ok = std::fabs((double)got[i] - (double)want[i]) <= bar;
    }
    std::snprintf(what, sizeof what, "softmax %d x %d", N, classes);
    expect(ok, what);
}

}  // namespace

int main() {
    int devices = 0;
    if (hipGetDeviceCount(&devices) != hipSuccess || devices < 1) {
        std::printf("no GPU\n");
        return 3;
    }
    HIP_OK(hipSetDevice(0));
    hipStream_t st;
    HIP_OK(hipStreamCreate(&st));
    std::printf("cnnmem version %d\n", cnnmem_version());
    // invalid calls are rejected on the host and enqueue nothing
    expect(cnnmem_transform(nullptr, nullptr, 1, 1, 1, 1, 0, 1, st) == CNNMEM_ERR_INVALID_ARG, "null pointers are rejected");
    check_layers(16, 8, 27, 27, st);        // AlexNet-like plane, small batch
    check_layers(128, 4, 55, 55, st);       // batch of 128: the wide-tile transposes, odd planes
    check_layers(5, 3, 12, 14, st);         // batch not a multiple of 4: the general paths
    check_layers(64, 2, 224, 224, st);      // VGG-like plane: row pairs, strips of rows
    check_softmax(64, 1000, st);
    check_softmax(33, 21841, st);
    check_softmax(1000, 10, st);
    HIP_OK(hipStreamSynchronize(st));
    HIP_OK(hipStreamDestroy(st));
    std::printf(failures ? "FAILED: %d check(s)\n" : "all checks passed\n", failures);
    return failures ? 1 : 0;
}
