// Host cost of the C ABI's launch path, measured from a plain C++ program (no Python, no PyTorch).
//
//   1. host microseconds per call: 2000 calls of one entry point are enqueued without a synchronisation
//      and the host clock is read around the loop;
//   2. a whole step of many small launches, eager (the library called launch by launch, one
//      synchronisation per 50 steps) against the same step captured once into a HIP graph and replayed:
//      the pooling and classifier layers of Table 1 (25 launches) and a batch x categories sweep of the
//      softmax (16 launches).
//
// MEASUREMENT SUPPORT: prints a table, checks nothing against the oracle.  Built by __graft_entry__.build(),
// run by tests/test_gpu_native_abi.py.
#include <hip/hip_runtime.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <functional>
#include <vector>

#include "cnnmem.h"

namespace {

#define HIP_OK(call)                                                                          \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            std::printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); \
            std::exit(2);                                                                     \
        }                                                                                     \
    } while (0)

double now_us() {
    return std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

float* device_floats(size_t n) {
    float* p = nullptr;
    HIP_OK(hipMalloc(reinterpret_cast<void**>(&p), n * sizeof(float)));
    HIP_OK(hipMemset(p, 0, n * sizeof(float)));
    return p;
}

using Launch = std::function<int()>;

void host_cost(const char* what, const Launch& launch, hipStream_t st) {
    for (int i = 0; i < 100; ++i) launch();
    HIP_OK(hipStreamSynchronize(st));
    const int calls = 2000;
    const double t0 = now_us();
    int bad = 0;
    for (int i = 0; i < calls; ++i) bad |= launch();
    const double host = (now_us() - t0) / calls;
    HIP_OK(hipStreamSynchronize(st));
    std::printf("host cost  %-44s %6.2f us per call%s\n", what, host, bad ? "  (a call failed)" : "");
    std::fflush(stdout);
}

double eager_vs_graph(const char* what, const std::vector<Launch>& step, hipStream_t st) {
    const int steps = 200;
    for (int s = 0; s < 10; ++s)
        for (const auto& l : step) l();
    HIP_OK(hipStreamSynchronize(st));
    double t0 = now_us();
    for (int s = 0; s < steps; ++s) {
        for (const auto& l : step) l();
        if (s % 50 == 49) HIP_OK(hipStreamSynchronize(st));
    }
    HIP_OK(hipStreamSynchronize(st));
    const double eager = (now_us() - t0) / steps;

    hipGraph_t graph;
    hipGraphExec_t exec;
    HIP_OK(hipStreamBeginCapture(st, hipStreamCaptureModeGlobal));
    for (const auto& l : step) l();
    HIP_OK(hipStreamEndCapture(st, &graph));
    HIP_OK(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));
    for (int s = 0; s < 10; ++s) HIP_OK(hipGraphLaunch(exec, st));
    HIP_OK(hipStreamSynchronize(st));
    t0 = now_us();
    for (int s = 0; s < steps; ++s) HIP_OK(hipGraphLaunch(exec, st));
    HIP_OK(hipStreamSynchronize(st));
    const double replay = (now_us() - t0) / steps;
    HIP_OK(hipGraphExecDestroy(exec));
    HIP_OK(hipGraphDestroy(graph));
    std::printf("step       %-44s eager %8.2f us   graph replay %8.2f us   ratio %.2f   (%zu launches)\n", what, eager,
                replay, eager / replay, step.size());
    std::fflush(stdout);
    return eager / replay;
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

    // ---- Table 1: pooling layers PL1..PL10 (N, H = W, window, C, stride) in both layouts, classifiers ----
    const int pools[10][5] = {{128, 28, 2, 16, 2}, {128, 14, 2, 16, 2}, {128, 24, 3, 64, 2}, {128, 12, 3, 64, 2},
                              {128, 55, 3, 96, 2}, {128, 27, 3, 192, 2}, {128, 13, 3, 256, 2}, {64, 110, 3, 96, 2},
                              {64, 26, 3, 256, 2}, {64, 13, 3, 256, 2}};
    const int classifiers[5][2] = {{128, 10}, {128, 10}, {128, 1000}, {64, 1000}, {32, 1000}};
    std::vector<Launch> table1;
    for (const auto& p : pools) {
        const int N = p[0], hw = p[1], k = p[2], C = p[3], s = p[4];
        int Ho = 0, Wo = 0;
        if (cnnmem_pool_out_dims(hw, hw, k, k, s, s, 0, 0, &Ho, &Wo) != CNNMEM_OK) return 2;
        const float* x = device_floats((size_t)N * C * hw * hw);
        float* y = device_floats((size_t)N * C * Ho * Wo);
        for (int layout : {CNNMEM_NCHW, CNNMEM_CHWN})
            table1.push_back([=] { return cnnmem_pool(x, y, N, C, hw, hw, layout, CNNMEM_POOL_MAX, k, k, s, s, 0, 0, st); });
    }
    for (const auto& c : classifiers) {
        const int n = c[0], classes = c[1];
        const float* z = device_floats((size_t)n * classes);
        float* pr = device_floats((size_t)n * classes);
        table1.push_back([=] { return cnnmem_softmax(z, pr, n, classes, st); });
    }
    // ---- softmax sweep: batch 32..256 x categories 10..10000 ----
    std::vector<Launch> sweep;
    for (int n : {32, 64, 128, 256})
        for (int classes : {10, 100, 1000, 10000}) {
            const float* z = device_floats((size_t)n * classes);
            float* pr = device_floats((size_t)n * classes);
            sweep.push_back([=] { return cnnmem_softmax(z, pr, n, classes, st); });
        }
    // ---- one transform of a small tensor ----
    const float* tx = device_floats(16 * 64 * 32 * 32);
    float* ty = device_floats(16 * 64 * 32 * 32);
    const Launch small_transform = [=] { return cnnmem_transform(tx, ty, 16, 64, 32, 32, CNNMEM_NCHW, CNNMEM_CHWN, st); };

    std::printf("cnnmem version %d\n", cnnmem_version());
    host_cost("cnnmem_pool 128x16x14x14 2x2/s2 NCHW", table1[2], st);
    host_cost("cnnmem_pool 128x16x14x14 2x2/s2 CHWN", table1[3], st);
    host_cost("cnnmem_pool 128x64x12x12 3x3/s2 NCHW", table1[6], st);
    host_cost("cnnmem_softmax 128x10", table1[20], st);
    host_cost("cnnmem_softmax 128x1000", table1[22], st);
    host_cost("cnnmem_transform 16x64x32x32 NCHW->CHWN", small_transform, st);
    const double r1 = eager_vs_graph("Table 1 pooling + classifier layers", table1, st);
    const double r2 = eager_vs_graph("softmax sweep batch x categories", sweep, st);
    HIP_OK(hipStreamSynchronize(st));
    HIP_OK(hipStreamDestroy(st));
    std::printf("eager / graph: %.2f and %.2f\n", r1, r2);
    return 0;
}
