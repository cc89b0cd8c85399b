// Internal helpers shared by the HIP translation units of libcnnmem.
// Nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <cstdlib>

#include "cnnmem.h"

namespace cnnmem {

constexpr int kWave = 64;       // CDNA wavefront width
constexpr int kNumXcd = 8;      // MI355X: 8 accelerator dies, workgroups are dealt to them round-robin

inline int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }
inline long long ceil_div64(long long a, long long b) { return (a + b - 1) / b; }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Status of the launch that was just enqueued.
inline int launch_status() {
    return hipGetLastError() == hipSuccess ? CNNMEM_OK : CNNMEM_ERR_RUNTIME;
}

// Integer tuning knobs from the environment, for A/B profiling and for tests that force every kernel
// variant.  They are dead unless the process was started with CNNMEM_KNOBS=1: that switch is read once,
// at the first launch, so a production call pays one load of a static flag and no getenv; with the
// switch on, each knob is re-read on every call (a test may change it between calls).
inline bool knobs_enabled() {
    static const bool on = [] {
        const char* s = std::getenv("CNNMEM_KNOBS");
        return s && s[0] == '1';
    }();
    return on;
}
inline int env_int(const char* name, int fallback) {
    if (!knobs_enabled()) return fallback;
    const char* s = std::getenv(name);
    if (!s || !*s) return fallback;
    return std::atoi(s);
}

// Kernels that need more than 64 KB of dynamic LDS opt in once per device and kernel, not once per launch.
template <auto kernel>
inline bool allow_large_lds(size_t bytes) {
    static bool done[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
    if (done[dev]) return true;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)bytes) != hipSuccess)
        return false;
    done[dev] = true;
    return true;
}

// Exact unsigned division of any n < 2^31 by a fixed d in [1, 2^31):
// q = (n * magic) >> shift with magic = floor(2^(31+s)/d) + 1, s = ceil(log2 d).
// The error term magic*d - 2^(31+s) is at most d <= 2^s, so n * error < 2^(31+s).
struct FastDiv {
    uint32_t magic;
    uint32_t shift;
    uint32_t d;
};

inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f;
    f.d = d;
    uint32_t s = 0;
    while ((1ull << s) < d) ++s;
    f.shift = 31 + s;
    f.magic = (uint32_t)(((1ull << f.shift) / d) + 1ull);
    return f;
}

__host__ __device__ __forceinline__ uint32_t fd_div(uint32_t n, const FastDiv& f) {
    return (uint32_t)(((uint64_t)n * f.magic) >> f.shift);
}

// Exact unsigned division of a small n (n < 2^20: indices inside a workgroup's LDS slab) by a fixed d in [1, 2^20) in
// three full-rate vector instructions; the 64-bit multiply and shift of fd_div cost about ten issue slots.
// (n + 1/2) / d is at least 1/(2d) away from the next integer, which the two roundings (n/d * 2^-23 at most) cannot
// bridge while n < 2^21.
struct SmallDiv {
    float inv;
    uint32_t d;
};
__host__ __device__ __forceinline__ SmallDiv make_smalldiv(uint32_t d) {
    SmallDiv s;
    s.inv = 1.0f / (float)d;
    s.d = d;
    return s;
}
__host__ __device__ __forceinline__ uint32_t sd_div(uint32_t n, const SmallDiv& s) {
    return (uint32_t)(((float)n + 0.5f) * s.inv);
}

// Workgroups are handed to the 8 XCDs round-robin by linear id, and each XCD has
// its own L2.  This maps the hardware block id to a logical tile id such that
// consecutive logical tiles run on the same XCD (tiles that share halo rows then
// share an L2).  A bijection on [0, nblocks) for any nblocks.
__host__ __device__ __forceinline__ uint32_t xcd_contiguous_tile(uint32_t block, uint32_t nblocks) {
    const uint32_t xcd = block % kNumXcd;
    const uint32_t q = nblocks / kNumXcd;
    const uint32_t rem = nblocks % kNumXcd;
    const uint32_t start = xcd * q + (xcd < rem ? xcd : rem);
    return start + block / kNumXcd;
}

// ---- streaming global accesses ---------------------------------------------
// Every tensor here is read once and written once, so loads and stores carry the
// non-temporal hint (the `nt` bit of global_load/global_store): lines are not kept
// in L2 / the memory-side cache at the expense of data that will be reused.  On
// MI355X a plain float4 copy gains 6-8 % from it.
typedef float v4f_t __attribute__((ext_vector_type(4)));
typedef float v2f_t __attribute__((ext_vector_type(2)));

// Write-through stores: `sc1 nt`, i.e. device scope on top of the non-temporal hint, so that the line
// is written through L2 towards memory at once instead of lingering there dirty until it is evicted.
// Measured on MI355X (same process, alternating builds): a float4 copy of 2 x 512 MB 80.2 -> 82.4 % of
// 8 TB/s; CHWN 2x2 pooling 166 -> 161 us; the write-heavy 2x2 average-pooling backward 179 -> 159 us.
// Kernels whose stores are interleaved with LDS phases or long register-resident rows lose 2-10 % with
// it (softmax, the LDS slab backward kernel, HWCN -> NCHW), so it is a separate helper used only by the
// kernels that gain, not a global switch.  The compiler has no way to ask for that bit on a plain
// vector store, so the store is one line of inline asm that takes the address and the data as inputs and
// needs no wait.  It carries no "memory" clobber on purpose, so that loads of later iterations may be
// scheduled above it: no kernel here reads back global memory it has written, and a value being stored
// depends on the loads it was computed from.  The compiler cannot look inside the asm, so the one
// software hazard of this instruction is handled here: on gfx940-class hardware a vector-memory store
// of more than 64 bits must be followed by two wait states before a vector ALU instruction overwrites
// its data registers (the compiler inserts them for its own stores); without them a few lanes stored
// the next loop index instead of their result.  The address form `off` reads no scalar registers, and
// stores of up to 64 bits have no such hazard.

__device__ __forceinline__ float4 ld4_stream(const float* p) {
    const v4f_t v = __builtin_nontemporal_load(reinterpret_cast<const v4f_t*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st4_stream(float* p, const float4& a) {
    const v4f_t v = {a.x, a.y, a.z, a.w};
    __builtin_nontemporal_store(v, reinterpret_cast<v4f_t*>(p));
}
// 128-bit accesses at any 4-byte aligned address (gfx950 global memory accepts dword-aligned
// multi-dword accesses; the type's alignment tells the compiler, which picks the instruction).
typedef v4f_t v4f_unaligned_t __attribute__((aligned(4)));
__device__ __forceinline__ float4 ld4u_stream(const float* p) {
    const v4f_unaligned_t v = __builtin_nontemporal_load(reinterpret_cast<const v4f_unaligned_t*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st4u_stream(float* p, const float4& a) {
    const v4f_unaligned_t v = {a.x, a.y, a.z, a.w};
    __builtin_nontemporal_store(v, reinterpret_cast<v4f_unaligned_t*>(p));
}
__device__ __forceinline__ void st2_stream(float* p, float a, float b) {
    const v2f_t v = {a, b};
    __builtin_nontemporal_store(v, reinterpret_cast<v2f_t*>(p));
}
__device__ __forceinline__ float ld1_stream(const float* p) {
    return __builtin_nontemporal_load(p);
}
__device__ __forceinline__ void st1_stream(float* p, float a) {
    __builtin_nontemporal_store(a, p);
}

// 128-bit (16-byte aligned) and 64-bit write-through stores, see above
__device__ __forceinline__ void st4_through(float* p, const float4& a) {
    const v4f_t v = {a.x, a.y, a.z, a.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v));
}
// the same at any 4-byte aligned address
__device__ __forceinline__ void st4u_through(float* p, const float4& a) {
    const v4f_t v = {a.x, a.y, a.z, a.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v));
}
__device__ __forceinline__ void st2_through(float* p, float a, float b) {
    const v2f_t v = {a, b};
    asm volatile("global_store_dwordx2 %0, %1, off sc1 nt" : : "v"(p), "v"(v));
}

// Occupancy throttle.  On tensors of hundreds of MB, HBM throughput on MI355X is
// best with about 48-64 KB of loads in flight per CU; a full complement of eight
// 256-lane workgroups per CU keeps 64-128 KB in flight and loses 2-3 points.
// Asking for dynamic LDS that the kernel never touches caps the workgroups per CU
// (160 KB of LDS per CU).  Smaller tensors want all the parallelism they can get,
// so by default the throttle only applies from 384 MB of input (measured: it gains 2-4 points at 411 MB and
// 822 MB of input and loses 2-5 at 206 MB and below).
//   requested: the caller's tuning (0 = this default rule, -1 = never, 1..8 = that many)
inline size_t throttle_lds(int requested, long long in_bytes, int default_workgroups_per_cu) {
    int wpc = requested;
    if (wpc == 0) wpc = in_bytes >= (384LL << 20) ? default_workgroups_per_cu : -1;
    if (wpc < 0 || wpc >= 8) return 0;
    const size_t bytes = (size_t)(160 * 1024 / wpc) - 1024;
    return bytes > 65536 ? 65536 : bytes;           // 64 KB needs no opt-in and already means two per CU
}

// ---- launchers implemented in the .hip files (host side, C++ linkage, hidden) ----
int launch_transpose2d(const float* src, float* dst, long long R, long long S, hipStream_t st);
int launch_copy(const float* src, float* dst, long long n, hipStream_t st);
int launch_transpose2d_any(const float* src, float* dst, long long R, long long S, hipStream_t st);
// General 4-D axis permutation: dims = source extents (slowest first), destination axis i = source axis perm[i].
int launch_permute(const float* src, float* dst, const int* dims, const int* perm, hipStream_t st);
// What a 4-D permutation comes down to once it is in canonical form (host only; extents and
// strides in elements, independent of the element size).
struct PermutePlan {
    enum Kind { kCopy, kTranspose2d, kRows, kTiles } kind;
    long long total;                        // all elements
    // kTranspose2d, kTiles: R along the destination's fastest axis, S along the source's
    long long R, S;
    long long ss_r, ds_s;                   // kTiles: source stride of r, destination stride of s
    long long nb0, nb1, sb0, sb1, db0, db1; // kTiles: batch extents and strides on both sides
    int xcd_order;                          // kTiles: keep neighbouring tiles on one XCD
    // kRows: run length, extents and source strides of the (up to three) outer destination axes
    long long L, oe[3], ot[3];
    int slow;                               // index of the slowest real outer axis
};
PermutePlan plan_permutation(const int* dims, const int* perm);
// Canonical form of a permutation: extent-1 axes dropped, axes that stay neighbours merged (host only).
void canonical_permutation(const int* dims, const int* perm, int* rank, long long* cdims, int* cperm);

struct PoolGeom {
    int N, C, H, W, Ho, Wo;
    int kh, kw, sh, sw, ph, pw;
    int mode;
};
// Launch-shape choices of a pooling call; 0 everywhere = the library's defaults.
struct PoolTuning {
    int rows_per_lane = 0;      // CHWN working set along H (1..4)
    int cols_per_lane = 0;      // CHWN working set along W (1..2)
    int workgroups_per_cu = 0;  // occupancy cap (2..8), -1 = none
    int nchw_kernel = 0;        // 1 = row pairs when applicable, 2 = LDS slab
    int slab_lanes = 0;         // 256 / 512 / 1024
};
int launch_pool_nchw(const float* src, float* dst, const PoolGeom& g, const PoolTuning& tune, hipStream_t st);
int launch_pool_chwn(const float* src, float* dst, const PoolGeom& g, const PoolTuning& tune, hipStream_t st);

int launch_softmax(const float* logits, float* probs, int N, int classes, hipStream_t st);

// backward passes (fp32)
int launch_pool_backward(const float* src, const float* ddst, float* dsrc, const PoolGeom& g, int layout,
                         hipStream_t st);
int launch_softmax_backward(const float* probs, const float* dprobs, float* dlogits, int N, int classes,
                            hipStream_t st);

// 16-bit storage (dtype CNNMEM_F16 / CNNMEM_BF16); the transform sees the tensor as an [N][M] / [M][N] matrix
int launch_transform16(const void* src, void* dst, long long N, long long M, int src_layout, int dst_layout,
                       hipStream_t st);
int launch_permute16(const void* src, void* dst, const int* dims, const int* perm, hipStream_t st);
int launch_pool16(const void* src, void* dst, const PoolGeom& g, int layout, int dtype, hipStream_t st);
int launch_softmax16(const void* logits, void* probs, int N, int classes, int dtype, hipStream_t st);

}  // namespace cnnmem
