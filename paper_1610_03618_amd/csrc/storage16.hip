// The hot path on 16-bit storage: fp16 (IEEE binary16) and bf16 tensors.
//
// The paper's closing remarks expect half precision to shift these layers further
// towards memory: every element is 2 bytes, so the same 8 TB/s moves twice the
// elements.  Arithmetic does not change: values are widened exactly to fp32,
// pooling sums and the softmax run in fp32 exactly as in the fp32 kernels, and a
// result is rounded once, to nearest even, to the storage format.  A lane still
// moves 128 bits per access, which is now 8 elements:
//   transform -- 2-D transpose of 16-bit words; a lane loads 8 words of two
//                neighbouring source rows and files the eight (row, row+1) pairs
//                as dwords in an LDS tile that is already in destination order;
//   pooling   -- CHWN: a lane owns 8 images; NCHW: row pairs for 2x2 / stride 2,
//                else contiguous slabs through LDS, as for fp32;
//   softmax   -- a row in registers, 8 categories per 128-bit access, rows split
//                into head / line-aligned body / tail.
#include "common.hpp"
#include "rowmath.hpp"

namespace cnnmem {
namespace {

constexpr int kThreads = 256;
constexpr float kNegInf = kRowNegInf;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_unaligned __attribute__((aligned(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ u32x4 ld16_stream(const uint16_t* p) {       // 16-byte aligned
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
__device__ __forceinline__ u32x4 ld16_cached(const uint16_t* p) {
    return *reinterpret_cast<const u32x4*>(p);
}
__device__ __forceinline__ u32x4 ld16u_stream(const uint16_t* p) {      // 4-byte aligned
    const u32x4_unaligned v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_unaligned*>(p));
    return v;
}
__device__ __forceinline__ void st16_stream(uint16_t* p, u32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}
// write-through 128-bit store (device scope on top of the non-temporal hint; see st4_through)
__device__ __forceinline__ void st16_through(uint16_t* p, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v));
}
__device__ __forceinline__ void st16u_stream(uint16_t* p, u32x4 v) {
    const u32x4_unaligned w = v;
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4_unaligned*>(p));
}
__device__ __forceinline__ void st8_stream(uint16_t* p, u32x2 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(p));
}

// Eight consecutive 16-bit words at any 2-byte aligned address of a dword-aligned buffer.  On a
// dword boundary this is one 128-bit access; one word off, the load takes the enclosing aligned
// 128 bits plus the eighth word and shifts, the store writes word, three dwords, word.
__device__ __forceinline__ u32x4 load8_any(const uint16_t* p) {
    if ((reinterpret_cast<uintptr_t>(p) & 2u) == 0) return ld16u_stream(p);
    const u32x4 d = ld16u_stream(p - 1);            // words p-1 .. p+6
    const uint32_t last = p[7];
    u32x4 o;
    o.x = (d.x >> 16) | (d.y << 16);
    o.y = (d.y >> 16) | (d.z << 16);
    o.z = (d.z >> 16) | (d.w << 16);
    o.w = (d.w >> 16) | (last << 16);
    return o;
}
// the same with ordinary (cacheable) loads, for data that is read again soon
__device__ __forceinline__ u32x4 load8_any_keep(const uint16_t* p) {
    if ((reinterpret_cast<uintptr_t>(p) & 2u) == 0) {
        const u32x4_unaligned v = *reinterpret_cast<const u32x4_unaligned*>(p);
        return v;
    }
    const u32x4_unaligned d = *reinterpret_cast<const u32x4_unaligned*>(p - 1);
    const uint32_t last = p[7];
    u32x4 o;
    o.x = (d.x >> 16) | (d.y << 16);
    o.y = (d.y >> 16) | (d.z << 16);
    o.z = (d.z >> 16) | (d.w << 16);
    o.w = (d.w >> 16) | (last << 16);
    return o;
}
__device__ __forceinline__ void store8_any(uint16_t* q, const u32x4& o) {
    if ((reinterpret_cast<uintptr_t>(q) & 2u) == 0) {
        st16u_stream(q, o);
        return;
    }
    q[0] = (uint16_t)o.x;
    uint32_t* d = reinterpret_cast<uint32_t*>(q + 1);
    d[0] = (o.x >> 16) | (o.y << 16);
    d[1] = (o.y >> 16) | (o.z << 16);
    d[2] = (o.z >> 16) | (o.w << 16);
    q[7] = (uint16_t)(o.w >> 16);
}

// ---- the two storage formats -------------------------------------------------
struct Half {                                       // IEEE binary16
    // Both conversions are single instructions written as inline asm on purpose.  Given the
    // _Float16 type, the compiler notices that a maximum of widened halves is itself a half,
    // rewrites the fp32 max chain into v_max_f16 / v_max3_f16, and then ORs the 16-bit result
    // into a dword assuming its upper half is zero; on this target v_max3_f16 leaves the upper
    // half of its destination untouched, and the neighbouring output came out corrupted
    // (2x2 max-pooling, caught by the parity test).  Opaque conversions keep every
    // operation in fp32, and the explicit mask makes the packing independent of what the
    // conversion leaves in the upper half.
    static __device__ __forceinline__ float widen(uint32_t bits16) {
        float f;
        asm("v_cvt_f32_f16_e32 %0, %1" : "=v"(f) : "v"(bits16));    // reads the low 16 bits
        return f;
    }
    static __device__ __forceinline__ uint32_t narrow(float x) {       // nearest even (default rounding mode)
        uint32_t h;
        asm("v_cvt_f16_f32_e32 %0, %1" : "=v"(h) : "v"(x));
        return h & 0xffffu;
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) { return narrow(lo) | (narrow(hi) << 16); }
    // The maximum of two pairs without widening them: exact, subnormals included (16-bit subnormals are
    // never flushed), and it writes the whole destination register.
    static constexpr bool kPairMax = true;
    static constexpr uint32_t kNegInfPair = 0xfc00fc00u;
    // v[0..7] += the eight halves of w, in fp32: the mixed-precision fused multiply-add widens one half of
    // a register exactly, multiplies by 1 and adds with a single rounding, i.e. the fp32 sum, in one
    // instruction per value instead of three (mask or shift, widen, add).  It honours subnormals.
    static __device__ __forceinline__ void add8(float* v, const u32x4& w) {
        const uint32_t d[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "+v"(v[2 * k]) : "v"(d[k]));
            asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(v[2 * k + 1]) : "v"(d[k]));
        }
    }
    static __device__ __forceinline__ uint32_t max2(uint32_t a, uint32_t b) {
        uint32_t r;
        asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
        return r;
    }
};
struct BFloat {                                     // upper half of binary32
    static constexpr bool kPairMax = false;         // no packed bfloat16 arithmetic on this target
    static constexpr uint32_t kNegInfPair = 0xff80ff80u;
    static __device__ __forceinline__ void add8(float* v, const u32x4& w) {
        v[0] += widen(w.x & 0xffffu); v[1] += widen(w.x >> 16);
        v[2] += widen(w.y & 0xffffu); v[3] += widen(w.y >> 16);
        v[4] += widen(w.z & 0xffffu); v[5] += widen(w.z >> 16);
        v[6] += widen(w.w & 0xffffu); v[7] += widen(w.w >> 16);
    }
    static __device__ __forceinline__ float widen(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
    static __device__ __forceinline__ uint32_t narrow(float x) {
        const uint32_t u = __float_as_uint(x);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;                  // nearest even; overflow carries into infinity
    }
    // two values at once with the gfx950 conversion instruction (nearest even): low half = lo, high half = hi
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
        uint32_t w;
        asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(w) : "v"(lo), "v"(hi));
        return w;
    }
};

// Tells the compiler that the four registers may have changed, without emitting anything: values derived
// from them before this point cannot be kept for use after it and must be computed again.
__device__ __forceinline__ void forget_derived(u32x4& w) {
    asm volatile("" : "+v"(w.x), "+v"(w.y), "+v"(w.z), "+v"(w.w));
}
template <class E>
__device__ __forceinline__ void unpack8(const u32x4& w, float* f) {
    f[0] = E::widen(w.x & 0xffffu); f[1] = E::widen(w.x >> 16);
    f[2] = E::widen(w.y & 0xffffu); f[3] = E::widen(w.y >> 16);
    f[4] = E::widen(w.z & 0xffffu); f[5] = E::widen(w.z >> 16);
    f[6] = E::widen(w.w & 0xffffu); f[7] = E::widen(w.w >> 16);
}
template <class E>
__device__ __forceinline__ u32x4 pack8(const float* f) {
    u32x4 w;
    w.x = E::pack2(f[0], f[1]);
    w.y = E::pack2(f[2], f[3]);
    w.z = E::pack2(f[4], f[5]);
    w.w = E::pack2(f[6], f[7]);
    return w;
}

// =============================================================================
// Transform (Section IV.C): src[R][S] -> dst[S][R], 16-bit words.
// =============================================================================

// R and S even (rows then start on dword boundaries), S >= 8.  Work item = two
// neighbouring source rows x 8 columns: two 128-bit loads, eight dword LDS writes
// (each dword is the pair (r, r+1) of one destination row), and after the barrier a
// lane reads four dwords of a destination row and stores 128 bits.  LDS rows have
// an odd pitch in dwords, which spreads both the column-wise writes and the
// row-wise reads over the banks.
template <int TR, int TS>
__global__ __launch_bounds__(kThreads) void transpose16_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, long long R, long long S, uint32_t tiles_s,
    int xcd_order) {
    static_assert(TR % 16 == 0 && TS % 8 == 0 && (TR * TS / 16) % kThreads == 0, "tile shape");
    constexpr int PD = TR / 2 + 1;                  // LDS pitch in dwords
    constexpr int NC8 = TS / 8;
    constexpr int NB8 = TR / 8;
    constexpr int LOADS = (TR * TS / 16) / kThreads;
    constexpr int STORES = (TS * NB8) / kThreads;
    __shared__ uint32_t tile[(TS + 1) * PD];        // one spare row for words left of the tile

    // xcd_order: neighbouring tiles run on one XCD, so a cache line that two of them share (rows that are not a
    // whole number of lines) is fetched from memory once and found in that XCD's L2 the second time
    const uint32_t t = xcd_order ? xcd_contiguous_tile(blockIdx.x, gridDim.x) : blockIdx.x;
    const long long r0 = (long long)(t / tiles_s) * TR;
    const long long s0 = (long long)(t % tiles_s) * TS;
    const int tid = threadIdx.x;

    u32x4 a[LOADS], b[LOADS];
    int col[LOADS];
#pragma unroll
    for (int it = 0; it < LOADS; ++it) {
        const int w = tid + it * kThreads;
        const int c8 = w % NC8, rp = w / NC8;
        long long r = r0 + 2 * rp, s = s0 + 8 * c8;
        r = r < R ? r : R - 2;                      // R is even: row r + 1 exists whenever r does
        s = s + 8 <= S ? s : S - 8;
        col[it] = (int)(s - s0);                    // even, >= -6
        const uint16_t* q = src + (size_t)r * (size_t)S + (size_t)s;
        a[it] = ld16u_stream(q);
        b[it] = ld16u_stream(q + S);
    }
#pragma unroll
    for (int it = 0; it < LOADS; ++it) {
        const int rp = (tid + it * kThreads) / NC8;
        const uint32_t lo[4] = {a[it].x, a[it].y, a[it].z, a[it].w};
        const uint32_t hi[4] = {b[it].x, b[it].y, b[it].z, b[it].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = col[it] + 2 * j;          // columns c and c + 1 have the same sign (c is even)
            const int row0 = c >= 0 ? c : TS, row1 = c >= 0 ? c + 1 : TS;
            tile[row0 * PD + rp] = (lo[j] & 0xffffu) | (hi[j] << 16);
            tile[row1 * PD + rp] = (lo[j] >> 16) | (hi[j] & 0xffff0000u);
        }
    }
    __syncthreads();
    // every LDS read first, then the stores: the branches of the ragged end otherwise keep each iteration's
    // read, wait and store in a block of their own, STORES LDS round trips in a row
    u32x4 ov[STORES];
#pragma unroll
    for (int it = 0; it < STORES; ++it) {
        const int f = tid + it * kThreads;
        const uint32_t* t = tile + (f / NB8) * PD + 4 * (f % NB8);
        ov[it].x = t[0]; ov[it].y = t[1]; ov[it].z = t[2]; ov[it].w = t[3];
    }
#pragma unroll
    for (int it = 0; it < STORES; ++it) {
        const int f = tid + it * kThreads;
        const int b8 = f % NB8, sl = f / NB8;
        const u32x4 o = ov[it];
        const long long s = s0 + sl, r = r0 + 8 * b8;
        if (s < S) {
            uint16_t* q = dst + (size_t)s * (size_t)R + (size_t)r;
            if (r + 8 <= R) {
                st16u_stream(q, o);
            } else {                                // ragged end of a destination row (R is even: whole dwords)
                const uint32_t w[4] = {o.x, o.y, o.z, o.w};
                for (int j = 0; j < 4; ++j)
                    if (r + 2 * j < R) *reinterpret_cast<uint32_t*>(q + 2 * j) = w[j];
            }
        }
    }
}

// The same transpose with 8 x 8 register blocks: a lane loads 8 words of eight consecutive
// source rows (eight 128-bit loads in flight), transposes the block in registers and parks eight
// 128-bit vectors, one per destination row, in an LDS tile that is already in destination
// order; after the barrier it reads 128 bits of a destination row back and stores them.  Four
// times fewer LDS instructions per byte than the pair-packing kernel.  LDS rows are stored
// j-major (destination row s = 8*c + j at j*(TS/8) + c) with a pitch of an odd number of 16-byte
// units, so the eight lanes that write one column of blocks hit distinct bank groups.
template <int TR, int TS, bool ANY>
__global__ __launch_bounds__(kThreads) void transpose16_block_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, long long R, long long S, uint32_t tiles_s) {
    static_assert(TR % 8 == 0 && TS % 8 == 0 && TR * TS == 64 * kThreads, "one 8x8 block per lane");
    constexpr int NC8 = TS / 8;                     // blocks along s
    constexpr int NB8 = TR / 8;                     // 128-bit vectors per destination row of the tile
    constexpr int PV = NB8 + 1 + (NB8 % 2);         // LDS pitch in 16-byte units, odd
    __shared__ u32x4 tile[TS * PV];

    const long long r0 = (long long)(blockIdx.x / tiles_s) * TR;
    const long long s0 = (long long)(blockIdx.x % tiles_s) * TS;
    const int tid = threadIdx.x;
    const int c8 = tid % NC8, rb = tid / NC8;

    long long s = s0 + 8 * c8;
    s = s + 8 <= S ? s : S - 8;                     // S >= 8 (launcher); the shifted block is filed under its true columns
    const int col = (int)(s - s0);                  // >= -7
    u32x4 a[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        long long r = r0 + 8 * rb + i;
        r = r < R ? r : R - 1;                      // rows past R re-read the last one and are never written out
        const uint16_t* q = src + (size_t)r * (size_t)S + (size_t)s;
        a[i] = ANY ? load8_any(q) : ld16u_stream(q);
    }
    // 8 x 8 transpose: o[j] = column j of the block = words (row 0 .. row 7)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t w[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const uint32_t lo = j < 2 ? a[2 * m].x : j < 4 ? a[2 * m].y : j < 6 ? a[2 * m].z : a[2 * m].w;
            const uint32_t hi = j < 2 ? a[2 * m + 1].x : j < 4 ? a[2 * m + 1].y : j < 6 ? a[2 * m + 1].z : a[2 * m + 1].w;
            w[m] = (j & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
        }
        const int c = col + j;                      // tile column of this vector; left of the tile: spare slot
        u32x4 o;
        o.x = w[0]; o.y = w[1]; o.z = w[2]; o.w = w[3];
        const int row = c >= 0 ? (c & 7) * NC8 + (c >> 3) : 0;
        const int slot = c >= 0 ? rb : NB8;         // column NB8 of a row is padding, never read
        tile[row * PV + slot] = o;
    }
    __syncthreads();
    // TS destination rows x NB8 vectors = TS * NB8 = 8 * kThreads stores; every LDS read first (the branches
    // of the store paths would otherwise keep read, wait and store of each iteration together)
    u32x4 ov[8];
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int f = tid + it * kThreads;
        const int sl = f / NB8;
        ov[it] = tile[((sl & 7) * NC8 + (sl >> 3)) * PV + f % NB8];
    }
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int f = tid + it * kThreads;
        const int b8 = f % NB8, sl = f / NB8;
        const u32x4 o = ov[it];
        const long long sd = s0 + sl, r = r0 + 8 * b8;
        if (sd < S) {
            uint16_t* q = dst + (size_t)sd * (size_t)R + (size_t)r;
            if (r + 8 <= R) {
                if (ANY) store8_any(q, o);
                else st16u_stream(q, o);
            } else {
                const uint32_t w[4] = {o.x, o.y, o.z, o.w};
                for (int j = 0; j < 8; ++j)
                    if (r + j < R) q[j] = (uint16_t)(w[j >> 1] >> (16 * (j & 1)));
            }
        }
    }
}

// Any R, S: word by word through a 64 x 64 tile.
__global__ __launch_bounds__(kThreads) void transpose16_scalar_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, long long R, long long S, uint32_t tiles_s) {
    constexpr int T = 64;
    __shared__ uint16_t tile[T * (T + 2)];
    const long long r0 = (long long)(blockIdx.x / tiles_s) * T;
    const long long s0 = (long long)(blockIdx.x % tiles_s) * T;
    const int tx = threadIdx.x % T, ty = threadIdx.x / T;
#pragma unroll
    for (int k = 0; k < T / 4; ++k) {
        const int rl = ty + 4 * k;
        const long long r = r0 + rl, s = s0 + tx;
        if (r < R && s < S) tile[rl * (T + 2) + tx] = src[(size_t)r * (size_t)S + (size_t)s];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < T / 4; ++k) {
        const int sl = ty + 4 * k;
        const long long s = s0 + sl, r = r0 + tx;
        if (r < R && s < S) dst[(size_t)s * (size_t)R + (size_t)r] = tile[tx * (T + 2) + sl];
    }
}

__global__ __launch_bounds__(kThreads) void copy16_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst,
                                                          size_t n) {
    // 8 words per lane where the pointers allow it, the rest word by word
    const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    const bool vec = ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) == 0;
    if (vec) {
        if (8 * i + 8 <= n) st16_stream(dst + 8 * i, ld16_stream(src + 8 * i));
        else for (size_t j = 8 * i; j < n; ++j) dst[j] = src[j];
    } else {
        for (size_t j = 8 * i; j < n && j < 8 * i + 8; ++j) dst[j] = src[j];
    }
}

template <int TR, int TS>
int launch_t16_block(const uint16_t* src, uint16_t* dst, long long R, long long S, bool any, hipStream_t st) {
    const long long tiles_r = ceil_div64(R, TR), tiles_s = ceil_div64(S, TS);
    if (tiles_r * tiles_s > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)(tiles_r * tiles_s)), block(kThreads);
    if (any)
        hipLaunchKernelGGL((transpose16_block_kernel<TR, TS, true>), grid, block, 0, st, src, dst, R, S, (uint32_t)tiles_s);
    else
        hipLaunchKernelGGL((transpose16_block_kernel<TR, TS, false>), grid, block, 0, st, src, dst, R, S, (uint32_t)tiles_s);
    return launch_status();
}

template <int TR, int TS>
int launch_t16(const uint16_t* src, uint16_t* dst, long long R, long long S, hipStream_t st) {
    const long long tiles_r = ceil_div64(R, TR), tiles_s = ceil_div64(S, TS);
    if (tiles_r * tiles_s > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((transpose16_kernel<TR, TS>), dim3((unsigned)(tiles_r * tiles_s)), dim3(kThreads), 0, st, src,
                       dst, R, S, (uint32_t)tiles_s,
                       // source rows that are not whole 128-byte lines: neighbouring tiles share lines (counters showed
                       // 1.25x the tensor fetched from memory); 256x96x55x55 NCHW -> CHWN 61.8 -> 65.7 % of peak.  With
                       // line-aligned source rows the plain order is 1-3 points better.
                       env_int("CNNMEM_TRANSFORM16_XCD", (S * 2) % 128 != 0 ? 1 : 0));
    return launch_status();
}

struct Tile16Plan {
    long long R, S, ss_r, ds_s, sb0, sb1, db0, db1;
    uint32_t tiles_s, tiles_plane;
    int xcd_order = 0;          // tile kernel: neighbouring tiles on one XCD
};

// ---- thin planes: one tile axis has 2..8 entries (batches of 2..8 images, RGB input) ----------
// A workgroup takes all T entries of the thin axis and kThin16 entries of the long one.  On the side
// where the thin axis is fastest that block is one contiguous run and moves as a linear 128-bit stream;
// in LDS it is kept in that order as 128-bit slots, slot f at f + f/8 (a lane's eight entries of the
// long axis times T are T whole slots; the padding spreads neighbouring lanes over all bank groups).
constexpr int kThin16 = 2048;
__device__ __forceinline__ int thin16_slot(int f) { return f + (f >> 3); }
__device__ __forceinline__ int thin16_word(int i) { return 8 * thin16_slot(i >> 3) + (i & 7); }
constexpr int thin16_lds_words(int T) { return 8 * (kThin16 / 8 * T + kThin16 / 64 * T); }
__device__ __forceinline__ uint32_t word_of(const u32x4& v, int c) {        // c-th 16-bit word of eight
    const uint32_t d = c < 2 ? v.x : c < 4 ? v.y : c < 6 ? v.z : v.w;
    return (c & 1) ? d >> 16 : d & 0xffffu;
}

// Destination rows are thin: dst[s][r], r < T, rows back to back (ds_s == T).  S >= 8.
template <int T>
__global__ __launch_bounds__(kThreads) void permute16_thin_dst_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, Tile16Plan p, FastDiv d_plane, FastDiv d_nb1) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[thin16_lds_words(T)];
    const uint32_t batch = fd_div(blockIdx.x, d_plane);
    const uint32_t ts = blockIdx.x - batch * p.tiles_plane;
    const uint32_t b0 = fd_div(batch, d_nb1);
    const uint32_t b1 = batch - b0 * d_nb1.d;
    src += (size_t)b0 * (size_t)p.sb0 + (size_t)b1 * (size_t)p.sb1;
    dst += (size_t)b0 * (size_t)p.db0 + (size_t)b1 * (size_t)p.db1;
    const long long s0 = (long long)ts * kThin16;
    const int ns = (int)(p.S - s0 < kThin16 ? p.S - s0 : kThin16);
    const int tid = threadIdx.x;

    long long s = s0 + 8 * tid;
    s = s + 8 <= p.S ? s : p.S - 8;                     // lanes past the end re-read the row's last eight words
    const int col = (int)(s - s0);                      // -7 .. kThin16 - 8
    u32x4 v[T];
#pragma unroll
    for (int r = 0; r < T; ++r) v[r] = load8_any(src + (size_t)r * (size_t)p.ss_r + (size_t)s);
    if (col == 8 * tid) {
        // eight columns x T rows = 8T consecutive destination words = T whole slots; word h of them is
        // column h / T of row h % T
#pragma unroll
        for (int k = 0; k < T; ++k) {
            uint32_t d[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int lo = 8 * k + 2 * j, hi = lo + 1;
                d[j] = word_of(v[lo % T], lo / T) | (word_of(v[hi % T], hi / T) << 16);
            }
            u32x4 o;
            o.x = d[0]; o.y = d[1]; o.z = d[2]; o.w = d[3];
            *reinterpret_cast<u32x4*>(tile + 8 * thin16_slot(tid * T + k)) = o;
        }
    } else {
        // shifted lanes: word by word; columns left of the block belong to the previous one
#pragma unroll
        for (int r = 0; r < T; ++r)
#pragma unroll
            for (int c = 0; c < 8; ++c)
                if (col + c >= 0) tile[thin16_word((col + c) * T + r)] = (uint16_t)word_of(v[r], c);
    }
    __syncthreads();
    uint16_t* out = dst + (size_t)s0 * T;               // the block's ns * T destination words are contiguous
    const int total = ns * T;
    for (int i = 8 * tid; i < total; i += 8 * kThreads) {
        if (i + 8 <= total) {
            store8_any(out + i, *reinterpret_cast<const u32x4*>(tile + 8 * thin16_slot(i >> 3)));
        } else {
            for (int j = i; j < total; ++j) out[j] = tile[thin16_word(j)];
        }
    }
}

// Source rows are thin: src[r][s], s < T, rows back to back (ss_r == T).  R * T >= 8.
template <int T>
__global__ __launch_bounds__(kThreads) void permute16_thin_src_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, Tile16Plan p, FastDiv d_plane, FastDiv d_nb1) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[thin16_lds_words(T)];
    const uint32_t batch = fd_div(blockIdx.x, d_plane);
    const uint32_t tr = blockIdx.x - batch * p.tiles_plane;
    const uint32_t b0 = fd_div(batch, d_nb1);
    const uint32_t b1 = batch - b0 * d_nb1.d;
    src += (size_t)b0 * (size_t)p.sb0 + (size_t)b1 * (size_t)p.sb1;
    dst += (size_t)b0 * (size_t)p.db0 + (size_t)b1 * (size_t)p.db1;
    const long long r0 = (long long)tr * kThin16;
    const int nr = (int)(p.R - r0 < kThin16 ? p.R - r0 : kThin16);
    const int tid = threadIdx.x;

    // the block's nr * T source words are contiguous: a linear stream, the last vector shifted back so
    // that it ends with the block (or, in a tiny first block, starts with the plane)
    const uint16_t* in = src + (size_t)r0 * T;
    const int total = nr * T;
    const long long before = r0 * T;
    u32x4 v[T];
    int at[T];
#pragma unroll
    for (int k = 0; k < T; ++k) {
        int i = 8 * (tid + k * kThreads);
        i = i + 8 <= total ? i : total - 8;
        if ((long long)i + before < 0) i = (int)-before;
        at[k] = i;
        v[k] = load8_any(in + i);
    }
#pragma unroll
    for (int k = 0; k < T; ++k) {
        if (at[k] == 8 * (tid + k * kThreads)) {
            *reinterpret_cast<u32x4*>(tile + 8 * thin16_slot(tid + k * kThreads)) = v[k];
        } else {
#pragma unroll
            for (int c = 0; c < 8; ++c)
                if (at[k] + c >= 0) tile[thin16_word(at[k] + c)] = (uint16_t)word_of(v[k], c);
        }
    }
    __syncthreads();
    // T destination rows of nr words; a lane's eight rows x T columns are T whole slots, word h of them
    // is row h / T, column h % T
    const int r = 8 * tid;
    if (r + 8 <= nr) {
        u32x4 q[T];
#pragma unroll
        for (int k = 0; k < T; ++k) q[k] = *reinterpret_cast<const u32x4*>(tile + 8 * thin16_slot(tid * T + k));
#pragma unroll
        for (int sidx = 0; sidx < T; ++sidx) {
            uint32_t d[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int lo = (2 * j) * T + sidx, hi = (2 * j + 1) * T + sidx;
                d[j] = word_of(q[lo / 8], lo % 8) | (word_of(q[hi / 8], hi % 8) << 16);
            }
            u32x4 o;
            o.x = d[0]; o.y = d[1]; o.z = d[2]; o.w = d[3];
            store8_any(dst + (size_t)sidx * (size_t)p.ds_s + (size_t)(r0 + r), o);
        }
    } else {
        for (int sidx = 0; sidx < T; ++sidx)
            for (int j = r; j < nr; ++j)
                dst[(size_t)sidx * (size_t)p.ds_s + (size_t)(r0 + j)] = tile[thin16_word(j * T + sidx)];
    }
}

template <int T>
int launch_thin16(bool thin_dst, const uint16_t* src, uint16_t* dst, Tile16Plan p, long long nb0, long long nb1,
                  hipStream_t st) {
    const long long plane = ceil_div64(thin_dst ? p.S : p.R, kThin16);
    if (plane >= 0x7fffffffLL || nb0 * nb1 >= 0x7fffffffLL || plane * nb0 * nb1 >= 0x7fffffffLL)
        return CNNMEM_ERR_UNSUPPORTED;
    p.tiles_plane = (uint32_t)plane;
    p.tiles_s = thin_dst ? (uint32_t)plane : 1;
    const FastDiv d_plane = make_fastdiv((uint32_t)plane), d_nb1 = make_fastdiv((uint32_t)nb1);
    const dim3 grid((unsigned)(plane * nb0 * nb1)), block(kThreads);
    if (thin_dst)
        hipLaunchKernelGGL((permute16_thin_dst_kernel<T>), grid, block, 0, st, src, dst, p, d_plane, d_nb1);
    else
        hipLaunchKernelGGL((permute16_thin_src_kernel<T>), grid, block, 0, st, src, dst, p, d_plane, d_nb1);
    return launch_status();
}

// CNNMEM_ERR_UNSUPPORTED when the plane is not thin (the caller then takes the tile kernels).
int launch_thin16_any(const uint16_t* src, uint16_t* dst, const Tile16Plan& p, long long nb0, long long nb1,
                      hipStream_t st) {
    const bool dword_ok = ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 3u) == 0;
    if (!dword_ok || env_int("CNNMEM_THIN16", 1) == 0) return CNNMEM_ERR_UNSUPPORTED;
    bool thin_dst;
    int T;
    if (p.R >= 2 && p.R <= 8 && p.ds_s == p.R && p.S >= 8) { thin_dst = true; T = (int)p.R; }
    else if (p.S >= 2 && p.S <= 8 && p.ss_r == p.S && p.R * p.S >= 8) { thin_dst = false; T = (int)p.S; }
    else return CNNMEM_ERR_UNSUPPORTED;
    switch (T) {
        case 2: return launch_thin16<2>(thin_dst, src, dst, p, nb0, nb1, st);
        case 3: return launch_thin16<3>(thin_dst, src, dst, p, nb0, nb1, st);
        case 4: return launch_thin16<4>(thin_dst, src, dst, p, nb0, nb1, st);
        case 5: return launch_thin16<5>(thin_dst, src, dst, p, nb0, nb1, st);
        case 6: return launch_thin16<6>(thin_dst, src, dst, p, nb0, nb1, st);
        case 7: return launch_thin16<7>(thin_dst, src, dst, p, nb0, nb1, st);
        default: return launch_thin16<8>(thin_dst, src, dst, p, nb0, nb1, st);
    }
}

int launch_transpose16(const uint16_t* src, uint16_t* dst, long long R, long long S, hipStream_t st) {
    if (R == 1 || S == 1) {                             // a vector: nothing moves
        const long long blocks = ceil_div64(ceil_div64(R * S, 8), kThreads);
        if (blocks > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, src, dst, (size_t)(R * S));
        return launch_status();
    }
    if (env_int("CNNMEM_TRANSFORM16_TILE", -1) < 0) {
        Tile16Plan tp;
        tp.R = R; tp.S = S; tp.ss_r = S; tp.ds_s = R;
        tp.sb0 = tp.sb1 = tp.db0 = tp.db1 = 0;
        tp.tiles_s = tp.tiles_plane = 0;
        const int rc = launch_thin16_any(src, dst, tp, 1, 1, st);
        if (rc != CNNMEM_ERR_UNSUPPORTED) return rc;
    }
    const bool dword_ok = ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 3u) == 0;
    const int forced = env_int("CNNMEM_TRANSFORM16_TILE", -1);
    const bool odd = R % 2 != 0 || S % 2 != 0;
    if (dword_ok && S >= 8 && (forced >= 10 || (odd && forced < 0))) {
        // 8 x 8 register blocks.  On even extents they measure the same as the pair-packing kernel
        // below (both sit at ~85 % of a copy of the same bytes), so that one stays the default;
        // odd extents need the shifted 128-bit accesses, which only this kernel has.
        const bool any = odd;
        int shape = forced;
        if (shape < 0) {
            if (R <= 8) shape = 16;
            else if (R <= 16) shape = 15;
            else if (R <= 32) shape = 13;
            else if (R <= 64) shape = 11;
            else if (S <= 32) shape = 14;
            else if (S <= 64) shape = 12;
            else shape = 10;
        }
        switch (shape) {
            case 11: return launch_t16_block<64, 256>(src, dst, R, S, any, st);
            case 12: return launch_t16_block<256, 64>(src, dst, R, S, any, st);
            case 13: return launch_t16_block<32, 512>(src, dst, R, S, any, st);
            case 14: return launch_t16_block<512, 32>(src, dst, R, S, any, st);
            case 15: return launch_t16_block<16, 1024>(src, dst, R, S, any, st);
            case 16: return launch_t16_block<8, 2048>(src, dst, R, S, any, st);
            default: return launch_t16_block<128, 128>(src, dst, R, S, any, st);
        }
    }
    if (dword_ok && R % 2 == 0 && S % 2 == 0 && S >= 8 && R >= 2) {
        int shape = forced;
        if (shape < 0) {
            if (R <= 16) shape = 3;
            else if (R <= 32) shape = 2;
            else if (S <= 16) shape = 5;
            else if (S <= 32) shape = 4;
            else if (R > 64 && S > 64) shape = 1;       // 65..127 images: one 128-wide tile spans the batch
            // 64 images: the tile side along the long axis stretched (64x256x56x56 fp16: NCHW -> CHWN
            // 61.5 -> 65.2 % of peak, CHWN -> NCHW 62.8 -> 64.8 %; 64x64x224x224: 65.8 -> 70.6 %, 65.3 -> 70.0 %)
            else if (R == 64 && S >= 256) shape = 6;
            else if (S == 64 && R >= 256) shape = 9;
            else shape = 0;
        }
        switch (shape) {
            case 1: return launch_t16<128, 128>(src, dst, R, S, st);
            case 2: return launch_t16<32, 128>(src, dst, R, S, st);
            case 3: return launch_t16<16, 256>(src, dst, R, S, st);
            case 4: return launch_t16<128, 32>(src, dst, R, S, st);
            case 5: return launch_t16<256, 16>(src, dst, R, S, st);
            case 6: return launch_t16<64, 128>(src, dst, R, S, st);
            case 7: return launch_t16<128, 64>(src, dst, R, S, st);
            case 8: return launch_t16<64, 256>(src, dst, R, S, st);
            case 9: return launch_t16<256, 64>(src, dst, R, S, st);
            default: return launch_t16<64, 64>(src, dst, R, S, st);
        }
    }
    const long long tiles_r = ceil_div64(R, 64), tiles_s = ceil_div64(S, 64);
    if (tiles_r * tiles_s > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(transpose16_scalar_kernel, dim3((unsigned)(tiles_r * tiles_s)), dim3(kThreads), 0, st, src, dst,
                       R, S, (uint32_t)tiles_s);
    return launch_status();
}

// ---- any storage order of 16-bit tensors (Section I: 24 orders) --------------------------
// The strided, batched forms of the two kernels above, driven by the same canonical plan as
// the fp32 permutation.


// S >= 8, R >= 2, dword-aligned buffers.  ANY = false: R and S even, so every stride is even and
// rows start on dword boundaries on both sides.  ANY = true: odd extents as well (rows start on
// either half of a dword: load8_any / store8_any; the last row of an odd R pairs with itself).
template <int TR, int TS, bool ANY>
__global__ __launch_bounds__(kThreads) void permute16_tile_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, Tile16Plan p, FastDiv d_plane, FastDiv d_tiles_s,
    FastDiv d_nb1) {
    static_assert(TR % 16 == 0 && TS % 8 == 0 && (TR * TS / 16) % kThreads == 0, "tile shape");
    constexpr int PD = TR / 2 + 1;
    constexpr int NC8 = TS / 8;
    constexpr int NB8 = TR / 8;
    constexpr int LOADS = (TR * TS / 16) / kThreads;
    constexpr int STORES = (TS * NB8) / kThreads;
    __shared__ uint32_t tile[(TS + 1) * PD];

    const uint32_t lin = p.xcd_order ? xcd_contiguous_tile(blockIdx.x, gridDim.x) : blockIdx.x;
    const uint32_t batch = fd_div(lin, d_plane);
    const uint32_t in_plane = lin - batch * p.tiles_plane;
    const uint32_t tr = fd_div(in_plane, d_tiles_s);
    const uint32_t ts = in_plane - tr * p.tiles_s;
    const uint32_t b0 = fd_div(batch, d_nb1);
    const uint32_t b1 = batch - b0 * d_nb1.d;
    const long long r0 = (long long)tr * TR, s0 = (long long)ts * TS;
    src += (size_t)b0 * (size_t)p.sb0 + (size_t)b1 * (size_t)p.sb1;
    dst += (size_t)b0 * (size_t)p.db0 + (size_t)b1 * (size_t)p.db1;
    const int tid = threadIdx.x;

    u32x4 a[LOADS], b[LOADS];
    int col[LOADS];
#pragma unroll
    for (int it = 0; it < LOADS; ++it) {
        const int w = tid + it * kThreads;
        const int c8 = w % NC8, rp = w / NC8;
        long long r = r0 + 2 * rp, s = s0 + 8 * c8;
        s = s + 8 <= p.S ? s : p.S - 8;
        col[it] = (int)(s - s0);                    // >= -7 (even extents: even, >= -6)
        if (ANY) {
            r = r < p.R ? r : p.R - 1;
            const long long r1 = r + 1 < p.R ? r + 1 : p.R - 1;
            a[it] = load8_any(src + (size_t)r * (size_t)p.ss_r + (size_t)s);
            b[it] = load8_any(src + (size_t)r1 * (size_t)p.ss_r + (size_t)s);
        } else {
            r = r < p.R ? r : p.R - 2;
            const uint16_t* q = src + (size_t)r * (size_t)p.ss_r + (size_t)s;
            a[it] = ld16u_stream(q);
            b[it] = ld16u_stream(q + p.ss_r);
        }
    }
#pragma unroll
    for (int it = 0; it < LOADS; ++it) {
        const int rp = (tid + it * kThreads) / NC8;
        const uint32_t lo[4] = {a[it].x, a[it].y, a[it].z, a[it].w};
        const uint32_t hi[4] = {b[it].x, b[it].y, b[it].z, b[it].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int c = col[it] + 2 * j;          // with odd extents c may be -1: only column c + 1 is in the tile
            const int row0 = c >= 0 ? c : TS, row1 = c + 1 >= 0 ? c + 1 : TS;
            tile[row0 * PD + rp] = (lo[j] & 0xffffu) | (hi[j] << 16);
            tile[row1 * PD + rp] = (lo[j] >> 16) | (hi[j] & 0xffff0000u);
        }
    }
    __syncthreads();
    u32x4 ov[STORES];                               // every LDS read first, then the stores (see transpose16_kernel)
#pragma unroll
    for (int it = 0; it < STORES; ++it) {
        const int f = tid + it * kThreads;
        const uint32_t* t = tile + (f / NB8) * PD + 4 * (f % NB8);
        ov[it].x = t[0]; ov[it].y = t[1]; ov[it].z = t[2]; ov[it].w = t[3];
    }
#pragma unroll
    for (int it = 0; it < STORES; ++it) {
        const int f = tid + it * kThreads;
        const int b8 = f % NB8, sl = f / NB8;
        const u32x4 o = ov[it];
        const long long s = s0 + sl, r = r0 + 8 * b8;
        if (s < p.S) {
            uint16_t* q = dst + (size_t)s * (size_t)p.ds_s + (size_t)r;
            if (r + 8 <= p.R) {
                if (ANY) store8_any(q, o);
                else st16u_stream(q, o);
            } else if (ANY) {
                const uint32_t w[4] = {o.x, o.y, o.z, o.w};
                for (int j = 0; j < 8; ++j)
                    if (r + j < p.R) q[j] = (uint16_t)(w[j >> 1] >> (16 * (j & 1)));
            } else {
                const uint32_t w[4] = {o.x, o.y, o.z, o.w};
                for (int j = 0; j < 4; ++j)
                    if (r + 2 * j < p.R) *reinterpret_cast<uint32_t*>(q + 2 * j) = w[j];
            }
        }
    }
}

// Any extents, strides and alignment: word by word through a TR x TS tile (4096 words; stretched
// along the long side when the other has only a few entries, e.g. three feature maps).
template <int TR, int TS>
__global__ __launch_bounds__(kThreads) void permute16_tile_scalar_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, Tile16Plan p, FastDiv d_plane, FastDiv d_tiles_s,
    FastDiv d_nb1) {
    static_assert(TR * TS == 4096, "4096 words per tile");
    constexpr int P = TS + 2;
    __shared__ uint16_t tile[TR * P];
    const uint32_t batch = fd_div(blockIdx.x, d_plane);
    const uint32_t in_plane = blockIdx.x - batch * p.tiles_plane;
    const uint32_t tr = fd_div(in_plane, d_tiles_s);
    const uint32_t ts = in_plane - tr * p.tiles_s;
    const uint32_t b0 = fd_div(batch, d_nb1);
    const uint32_t b1 = batch - b0 * d_nb1.d;
    const long long r0 = (long long)tr * TR, s0 = (long long)ts * TS;
    src += (size_t)b0 * (size_t)p.sb0 + (size_t)b1 * (size_t)p.sb1;
    dst += (size_t)b0 * (size_t)p.db0 + (size_t)b1 * (size_t)p.db1;
#pragma unroll
    for (int k = 0; k < 4096 / kThreads; ++k) {
        const int e = threadIdx.x + k * kThreads;
        const int sl = e % TS, rl = e / TS;
        const long long r = r0 + rl, s = s0 + sl;
        if (r < p.R && s < p.S) tile[rl * P + sl] = src[(size_t)r * (size_t)p.ss_r + (size_t)s];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4096 / kThreads; ++k) {
        const int e = threadIdx.x + k * kThreads;
        const int rl = e % TR, sl = e / TR;
        const long long s = s0 + sl, r = r0 + rl;
        if (r < p.R && s < p.S) dst[(size_t)s * (size_t)p.ds_s + (size_t)r] = tile[rl * P + sl];
    }
}

template <int TR, int TS>
int launch_p16_scalar(const uint16_t* src, uint16_t* dst, Tile16Plan p, long long nb0, long long nb1, hipStream_t st) {
    const long long tiles_r = ceil_div64(p.R, TR), tiles_s = ceil_div64(p.S, TS);
    const long long plane = tiles_r * tiles_s;
    if (plane >= 0x7fffffffLL || nb0 * nb1 >= 0x7fffffffLL || plane * nb0 * nb1 >= 0x7fffffffLL)
        return CNNMEM_ERR_UNSUPPORTED;
    p.tiles_s = (uint32_t)tiles_s;
    p.tiles_plane = (uint32_t)plane;
    hipLaunchKernelGGL((permute16_tile_scalar_kernel<TR, TS>), dim3((unsigned)(plane * nb0 * nb1)), dim3(kThreads), 0, st,
                       src, dst, p, make_fastdiv((uint32_t)plane), make_fastdiv((uint32_t)tiles_s),
                       make_fastdiv((uint32_t)nb1));
    return launch_status();
}

struct Row16Plan {
    long long t0, t1, t2;
    uint32_t L, total;
};

// The fastest axis stays: a lane owns 8 consecutive destination words.  VEC: both buffers are
// dword aligned; 8 words inside one run are one 128-bit load wherever the run happens to start
// (load8_any), and the destination, being linear, is always on a dword boundary.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void permute16_rows_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, Row16Plan p, FastDiv d_L, FastDiv d_e2, FastDiv d_e1) {
    const uint32_t e = 8u * (blockIdx.x * kThreads + threadIdx.x);
    if (e >= p.total) return;
    auto run_source = [&](uint32_t run) {
        const uint32_t q = fd_div(run, d_e2);
        const uint32_t o2 = run - q * d_e2.d;
        const uint32_t o0 = fd_div(q, d_e1);
        const uint32_t o1 = q - o0 * d_e1.d;
        return (size_t)o0 * (size_t)p.t0 + (size_t)o1 * (size_t)p.t1 + (size_t)o2 * (size_t)p.t2;
    };
    const uint32_t run = fd_div(e, d_L);
    const uint32_t in_run = e - run * p.L;
    if (VEC && in_run + 8 <= p.L) {
        st16u_stream(dst + e, load8_any(src + run_source(run) + in_run));
        return;
    }
    for (uint32_t j = 0; j < 8 && e + j < p.total; ++j) {
        const uint32_t rj = fd_div(e + j, d_L);
        dst[e + j] = src[run_source(rj) + (e + j - rj * p.L)];
    }
}

template <int TR, int TS>
int launch_p16_tile(const uint16_t* src, uint16_t* dst, Tile16Plan p, long long nb0, long long nb1, bool any,
                    hipStream_t st) {
    const long long tiles_r = ceil_div64(p.R, TR), tiles_s = ceil_div64(p.S, TS);
    const long long plane = tiles_r * tiles_s;
    if (plane >= 0x7fffffffLL || nb0 * nb1 >= 0x7fffffffLL || plane * nb0 * nb1 >= 0x7fffffffLL)
        return CNNMEM_ERR_UNSUPPORTED;
    p.tiles_s = (uint32_t)tiles_s;
    p.tiles_plane = (uint32_t)plane;
    p.xcd_order = env_int("CNNMEM_PERMUTE16_XCD", p.xcd_order);
    const dim3 grid((unsigned)(plane * nb0 * nb1)), block(kThreads);
    const FastDiv d_plane = make_fastdiv((uint32_t)plane), d_ts = make_fastdiv((uint32_t)tiles_s),
                  d_nb1 = make_fastdiv((uint32_t)nb1);
    if (any)
        hipLaunchKernelGGL((permute16_tile_kernel<TR, TS, true>), grid, block, 0, st, src, dst, p, d_plane, d_ts, d_nb1);
    else
        hipLaunchKernelGGL((permute16_tile_kernel<TR, TS, false>), grid, block, 0, st, src, dst, p, d_plane, d_ts, d_nb1);
    return launch_status();
}

int launch_permute16_impl(const uint16_t* src, uint16_t* dst, const int* dims, const int* perm, hipStream_t st) {
    const PermutePlan pl = plan_permutation(dims, perm);
    const bool dword_ok = ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 3u) == 0;
    if (pl.kind == PermutePlan::kCopy) {
        const long long blocks = ceil_div64(ceil_div64(pl.total, 8), kThreads);
        if (blocks > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, src, dst, (size_t)pl.total);
        return launch_status();
    }
    if (pl.kind == PermutePlan::kTranspose2d) return launch_transpose16(src, dst, pl.R, pl.S, st);
    if (pl.kind == PermutePlan::kRows) {
        const long long slice = pl.total / pl.oe[pl.slow];
        const long long limit = 0x7fffffffLL;
        if (slice >= limit) return CNNMEM_ERR_UNSUPPORTED;
        const long long per_launch = pl.total < limit ? pl.oe[pl.slow] : limit / slice;
        // slices start a multiple of 8 words into the destination when they are not the first one only if
        // the slice length is even; an odd slice length keeps the word-by-word kernel for the later slices
        const bool vec = dword_ok && (pl.total < limit || slice % 2 == 0);
        for (long long first = 0; first < pl.oe[pl.slow]; first += per_launch) {
            const long long count = pl.oe[pl.slow] - first < per_launch ? pl.oe[pl.slow] - first : per_launch;
            long long ce[3] = {pl.oe[0], pl.oe[1], pl.oe[2]};
            ce[pl.slow] = count;
            Row16Plan p;
            p.t0 = pl.ot[0]; p.t1 = pl.ot[1]; p.t2 = pl.ot[2];
            p.L = (uint32_t)pl.L;
            p.total = (uint32_t)(count * slice);
            const uint16_t* sp = src + (size_t)first * (size_t)pl.ot[pl.slow];
            uint16_t* dp = dst + (size_t)first * (size_t)slice;
            const dim3 grid((unsigned)ceil_div64(ceil_div64(count * slice, 8), kThreads)), block(kThreads);
            if (vec)
                hipLaunchKernelGGL((permute16_rows_kernel<true>), grid, block, 0, st, sp, dp, p,
                                   make_fastdiv((uint32_t)pl.L), make_fastdiv((uint32_t)ce[2]),
                                   make_fastdiv((uint32_t)ce[1]));
            else
                hipLaunchKernelGGL((permute16_rows_kernel<false>), grid, block, 0, st, sp, dp, p,
                                   make_fastdiv((uint32_t)pl.L), make_fastdiv((uint32_t)ce[2]),
                                   make_fastdiv((uint32_t)ce[1]));
        }
        return launch_status();
    }
    Tile16Plan p;
    p.R = pl.R; p.S = pl.S; p.ss_r = pl.ss_r; p.ds_s = pl.ds_s;
    p.sb0 = pl.sb0; p.sb1 = pl.sb1; p.db0 = pl.db0; p.db1 = pl.db1;
    p.tiles_s = p.tiles_plane = 0;
    // Neighbouring tiles on one XCD (a line two tiles share is then an L2 hit) when a batch axis lies between
    // the tile axes, as for fp32; when the source rows are short and not whole 128-byte lines (NHWC -> NCHW
    // with 96 channels: 192-byte rows); and when only the destination rows are not whole lines (NHWC -> NCHW of
    // 27 x 27 planes with 256 channels).  Measured in fp16: 128x96x55x55 NHWC -> NCHW 38.5 -> 46.1 % of peak,
    // NCHW -> HWCN 38.2 -> 41.7 %, HWCN -> NCHW 31.7 -> 43.0 %; 128x256x27x27 NHWC -> NCHW 36.4 -> 43.6 %.
    // Long misaligned source rows (NCHW -> NHWC) lose 1-3 points with it and keep the plain order.
    const bool src_ragged = (p.S * 2) % 128 != 0, dst_ragged = (p.R * 2) % 128 != 0;
    p.xcd_order = pl.xcd_order || (src_ragged && p.S < 256) || (dst_ragged && !src_ragged) ? 1 : 0;
    {
        const int rc = launch_thin16_any(src, dst, p, pl.nb0, pl.nb1, st);
        if (rc != CNNMEM_ERR_UNSUPPORTED) return rc;
    }
    if (dword_ok && p.S >= 8 && p.R > 4) {
        // even extents: every stride is a multiple of S (source side) or R (destination side), hence even
        const bool any = p.R % 2 != 0 || p.S % 2 != 0;
        if (p.R <= 16) return launch_p16_tile<16, 256>(src, dst, p, pl.nb0, pl.nb1, any, st);
        if (p.R <= 32) return launch_p16_tile<32, 128>(src, dst, p, pl.nb0, pl.nb1, any, st);
        if (p.S <= 16) return launch_p16_tile<256, 16>(src, dst, p, pl.nb0, pl.nb1, any, st);
        if (p.S <= 32) return launch_p16_tile<128, 32>(src, dst, p, pl.nb0, pl.nb1, any, st);
        // rows that are not whole 128-byte lines (64 words) get the long side of the tile, as for fp32
        const bool ragged_dst = p.R % 64 != 0, ragged_src = p.S % 64 != 0;
        if (ragged_dst && p.R >= 256) return launch_p16_tile<256, 32>(src, dst, p, pl.nb0, pl.nb1, any, st);
        if (ragged_src && p.S >= 256) return launch_p16_tile<32, 256>(src, dst, p, pl.nb0, pl.nb1, any, st);
        if (p.R >= 128 && p.S >= 128) return launch_p16_tile<128, 128>(src, dst, p, pl.nb0, pl.nb1, any, st);
        return launch_p16_tile<64, 64>(src, dst, p, pl.nb0, pl.nb1, any, st);
    }
    if (p.S <= 4) return launch_p16_scalar<1024, 4>(src, dst, p, pl.nb0, pl.nb1, st);
    if (p.R <= 4) return launch_p16_scalar<4, 1024>(src, dst, p, pl.nb0, pl.nb1, st);
    if (p.S <= 16) return launch_p16_scalar<256, 16>(src, dst, p, pl.nb0, pl.nb1, st);
    if (p.R <= 16) return launch_p16_scalar<16, 256>(src, dst, p, pl.nb0, pl.nb1, st);
    return launch_p16_scalar<64, 64>(src, dst, p, pl.nb0, pl.nb1, st);
}

// =============================================================================
// Pooling (Equation 2; Section IV.B, V.A)
// =============================================================================
// fmaxf() on a value that comes straight from memory costs two instructions: the compiler first quiets a
// possible signalling NaN (v_max_f32 x, x, x).  With eight widened values per 128-bit load that doubled the
// arithmetic of maximum pooling and made it slower than the average (256x64x112x112 3x3/s2/p1 CHWN fp16:
// 48 % of peak against 56 %).  The instruction itself returns the other operand for a quiet NaN and a quiet
// NaN for a signalling one, which is all that is wanted here.
__device__ __forceinline__ float max_plain(float a, float b) {
    float r;
    asm("v_max_f32_e32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
template <int MODE>
struct Acc {
    static __device__ __forceinline__ float identity() { return MODE == CNNMEM_POOL_MAX ? kNegInf : 0.f; }
    static __device__ __forceinline__ float op(float a, float b) {
        return MODE == CNNMEM_POOL_MAX ? max_plain(a, b) : a + b;
    }
    // Equation 2's division by the window area.  A correctly rounded fp32 division is about ten instructions
    // per output, as much as the taps of a 3x3 window now that those are one instruction each.  The
    // reciprocal is formed once per lane (at compile time for the fixed windows); one residual step on the
    // product then gives the correctly rounded quotient again (q = a r, e = a - q d exactly by fma,
    // q + e r), which matters: with 16-bit data the exact average often lies exactly on a rounding tie of
    // the storage format (window sums are small integers in units of the data's last place), and the bare
    // product a * (1/15) landed on the wrong side of 0.9 % of them.  The fix-up instruction restores the
    // quotient of infinities and NaNs.
    static __device__ __forceinline__ float finish(float a, float divisor) {
        if (MODE == CNNMEM_POOL_MAX) return a;
        const float r = 1.0f / divisor;
        float q = a * r;
        const float e = __builtin_fmaf(-q, divisor, a);
        q = __builtin_fmaf(e, r, q);
        return __builtin_amdgcn_div_fixupf(q, divisor, a);
    }
};

// The eight accumulators of a lane that owns eight images (one 128-bit word group).  In general they are
// fp32 values; for the maximum of binary16 data they stay packed, because the packed maximum is exact and
// takes 4 instructions per tap instead of 24 (mask or shift, widen, maximum for each of 8 values).
template <class E, int MODE, bool PAIRS = (MODE == CNNMEM_POOL_MAX && E::kPairMax)>
struct Lane8 {
    float v[8];
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = Acc<MODE>::identity();
    }
    __device__ __forceinline__ void tap(const u32x4& w) {
        if (MODE == CNNMEM_POOL_AVG) {
            E::add8(v, w);
        } else {
            float t[8];
            unpack8<E>(w, t);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = Acc<MODE>::op(v[e], t[e]);
        }
    }
    __device__ __forceinline__ void tap_if(const u32x4& w, bool ok) {     // a tap in the padding counts as the identity
        constexpr uint32_t id = MODE == CNNMEM_POOL_MAX ? E::kNegInfPair : 0u;
        u32x4 m;
        m.x = ok ? w.x : id; m.y = ok ? w.y : id; m.z = ok ? w.z : id; m.w = ok ? w.w : id;
        tap(m);
    }
    __device__ __forceinline__ void merge(const Lane8& o) {
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = Acc<MODE>::op(v[e], o.v[e]);
    }
    __device__ __forceinline__ u32x4 result(float divisor) const {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = Acc<MODE>::finish(v[e], divisor);
        return pack8<E>(o);
    }
};
template <class E, int MODE>
struct Lane8<E, MODE, true> {
    u32x4 w;
    __device__ __forceinline__ void clear() { w.x = w.y = w.z = w.w = E::kNegInfPair; }
    __device__ __forceinline__ void tap(const u32x4& t) {
        w.x = E::max2(w.x, t.x); w.y = E::max2(w.y, t.y); w.z = E::max2(w.z, t.z); w.w = E::max2(w.w, t.w);
    }
    __device__ __forceinline__ void tap_if(const u32x4& t, bool ok) {
        u32x4 m;
        m.x = ok ? t.x : E::kNegInfPair; m.y = ok ? t.y : E::kNegInfPair;
        m.z = ok ? t.z : E::kNegInfPair; m.w = ok ? t.w : E::kNegInfPair;
        tap(m);
    }
    __device__ __forceinline__ void merge(const Lane8& o) { tap(o.w); }
    __device__ __forceinline__ u32x4 result(float) const { return w; }
};

// Fallback: one lane per output, any layout through strides.
template <class E, int MODE>
__global__ __launch_bounds__(kThreads) void pool16_generic_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, PoolGeom g, int chwn, size_t total) {
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t o = (size_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += stride) {
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
                acc = Acc<MODE>::op(acc, E::widen(src[idx]));
            }
        }
        dst[o] = (uint16_t)E::narrow(Acc<MODE>::finish(acc, (float)(g.kh * g.kw)));
    }
}

// CHWN, any window: eight images per lane (one 128-bit access), the in-image part of the window walked with
// run-time loops (global 7x7 pooling, 5x5 / stride 3, rectangular windows).  A lane owns OY vertically adjacent
// outputs: each input row under them is read and reduced along W once and serves every output whose window
// holds it, instead of being fetched again by the lanes of the neighbouring output rows.
template <class E, int MODE, int OY>
__global__ __launch_bounds__(kThreads) void pool16_chwn_any_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, PoolGeom g, uint32_t items, FastDiv div_n8,
    FastDiv div_wo, FastDiv div_hb) {
    // neighbouring workgroups on one XCD: output rows that share input rows find them in L2
    const uint32_t u = xcd_contiguous_tile(blockIdx.x, gridDim.x) * kThreads + threadIdx.x;   // ((c*HB + ib)*Wo + j)*N8 + n8
    if (u >= items) return;
    const uint32_t t = fd_div(u, div_n8);
    const uint32_t n8 = u - t * div_n8.d;
    const uint32_t t2 = fd_div(t, div_wo);
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
    const uint16_t* plane = src + (size_t)c * g.H * g.W * N + 8 * n8;
    Lane8<E, MODE> acc[OY];
#pragma unroll
    for (int o = 0; o < OY; ++o) acc[o].clear();
    for (int r = r_lo; r < r_hi; ++r) {
        const uint16_t* rowp = plane + (size_t)r * g.W * N;
        Lane8<E, MODE> h;
        h.clear();
        int q = q_lo;
        for (; q + 4 <= q_hi; q += 4) {                         // four loads in flight before the first is used
            const u32x4 w0 = ld16_cached(rowp + (size_t)q * N), w1 = ld16_cached(rowp + (size_t)(q + 1) * N),
                        w2 = ld16_cached(rowp + (size_t)(q + 2) * N), w3 = ld16_cached(rowp + (size_t)(q + 3) * N);
            h.tap(w0); h.tap(w1); h.tap(w2); h.tap(w3);
        }
        for (; q < q_hi; ++q) h.tap(ld16_cached(rowp + (size_t)q * N));
#pragma unroll
        for (int o = 0; o < OY; ++o) {
            const int top = (i0 + o) * g.sh - g.ph;            // first row of output o's window
            if (OY == 1 || (r >= top && r < top + g.kh)) acc[o].merge(h);
        }
    }
    uint16_t* out = dst + (((size_t)c * g.Ho + i0) * g.Wo + j) * N + 8 * n8;
#pragma unroll
    for (int o = 0; o < OY; ++o)
        if (i0 + o < g.Ho) st16_stream(out + (size_t)o * g.Wo * N, acc[o].result((float)(g.kh * g.kw)));
}

// The same for tensors with few outputs and tall windows (global 7x7 pooling): the rows of a window are
// dealt over P lanes (row r_lo + part, + P, ...), which puts P times as many loads in flight, and the P
// partial results meet in LDS.  A workgroup is P parts x 256/P outputs; part 0 stores.
template <class E, int MODE, int P>
__global__ __launch_bounds__(kThreads) void pool16_chwn_split_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, PoolGeom g, uint32_t items, FastDiv div_n8,
    FastDiv div_wo, FastDiv div_ho) {
    constexpr int PER = kThreads / P;
    __shared__ Lane8<E, MODE> part_acc[P][PER];
    const int part = threadIdx.x / PER, slot = threadIdx.x % PER;
    const uint32_t u = blockIdx.x * PER + slot;                 // ((c*Ho + i)*Wo + j)*N8 + n8
    const bool live = u < items;
    Lane8<E, MODE> acc;
    acc.clear();
    if (live) {
        const uint32_t t = fd_div(u, div_n8);
        const uint32_t n8 = u - t * div_n8.d;
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
        const uint16_t* plane = src + (size_t)c * g.H * g.W * N + 8 * n8;
        for (int r = r_lo + part; r < r_hi; r += P) {
            const uint16_t* rowp = plane + (size_t)r * g.W * N;
            int q = q_lo;
            for (; q + 4 <= q_hi; q += 4) {
                const u32x4 w0 = ld16_cached(rowp + (size_t)q * N), w1 = ld16_cached(rowp + (size_t)(q + 1) * N),
                            w2 = ld16_cached(rowp + (size_t)(q + 2) * N), w3 = ld16_cached(rowp + (size_t)(q + 3) * N);
                acc.tap(w0); acc.tap(w1); acc.tap(w2); acc.tap(w3);
            }
            if (q + 2 <= q_hi) {
                const u32x4 w0 = ld16_cached(rowp + (size_t)q * N), w1 = ld16_cached(rowp + (size_t)(q + 1) * N);
                acc.tap(w0); acc.tap(w1);
                q += 2;
            }
            if (q < q_hi) acc.tap(ld16_cached(rowp + (size_t)q * N));
        }
    }
    part_acc[part][slot] = acc;
    __syncthreads();
    if (part == 0 && live) {
#pragma unroll
        for (int k = 1; k < P; ++k) acc.merge(part_acc[k][slot]);
        st16_stream(dst + 8 * (size_t)u, acc.result((float)(g.kh * g.kw)));
    }
}

// CHWN: a lane owns 8 consecutive images of one output column and walks down OY
// output rows; each input row it touches is reduced horizontally once and that row
// result is reused by every output row whose window contains it (Section V.A's
// working set, in registers).  Loads are unconditional from clamped addresses.
template <class E, int MODE, int KH, int KW, int SH, int SW, int OY, bool PADDED>
__global__ __launch_bounds__(kThreads) void pool16_chwn_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, PoolGeom g, uint32_t row_items,
    uint32_t blocks_x, uint32_t blocks_y, FastDiv div_n8) {
    constexpr int ROWS_IN = (OY - 1) * SH + KH;
    const uint32_t tile = xcd_contiguous_tile(blockIdx.x, gridDim.x);
    const uint32_t bx = tile % blocks_x;
    const uint32_t rest = tile / blocks_x;
    const uint32_t by = rest % blocks_y;
    const uint32_t c = rest / blocks_y;
    const uint32_t u = bx * kThreads + threadIdx.x;           // position in the output row: j * N8 + n8
    if (u >= row_items) return;
    const uint32_t j = fd_div(u, div_n8);
    const uint32_t n8 = u - j * div_n8.d;
    const int i0 = (int)by * OY;
    const int N = g.N;

    Lane8<E, MODE> acc[OY];
#pragma unroll
    for (int oy = 0; oy < OY; ++oy) acc[oy].clear();

    const int q0 = (int)j * SW - g.pw;
    const int r_base = i0 * SH - g.ph;
    const uint16_t* plane = src + (size_t)c * g.H * g.W * N + 8 * n8;
    constexpr bool kStream = (KH <= SH) && (KW <= SW);        // disjoint windows: every tap is read once
    // The taps of input row rr + 1 are requested before those of row rr are reduced.  The order is written
    // out because the reductions are inline-asm instructions, across which the compiler does not move
    // loads: left to it, the bfloat16 maximum waited for every single load before issuing the next
    // (256x96x55x55: 54 % of peak against 62 % for the average).
    int qcol[KW];
    bool qok[KW];
#pragma unroll
    for (int x = 0; x < KW; ++x) {
        const int q = q0 + x;
        qok[x] = !PADDED || (q >= 0 && q < g.W);
        qcol[x] = !PADDED ? q : (q < 0 ? 0 : (q < g.W ? q : g.W - 1));
    }
    auto load_row = [&](int rr, u32x4* w) {
        const int r = r_base + rr;
        const int rc = r < 0 ? 0 : (r < g.H ? r : g.H - 1);    // also the rows under a ragged last block of outputs
        const uint16_t* rowp = plane + (size_t)rc * g.W * N;
#pragma unroll
        for (int x = 0; x < KW; ++x)
            w[x] = kStream ? ld16_stream(rowp + (size_t)qcol[x] * N) : ld16_cached(rowp + (size_t)qcol[x] * N);
    };
    u32x4 wrow[2][KW];
    load_row(0, wrow[0]);
#pragma unroll
    for (int rr = 0; rr < ROWS_IN; ++rr) {
        if (rr + 1 < ROWS_IN) load_row(rr + 1, wrow[(rr + 1) & 1]);
        const int r = r_base + rr;
        const bool row_ok = !PADDED || (r >= 0 && r < g.H);
        Lane8<E, MODE> h;
        h.clear();
#pragma unroll
        for (int x = 0; x < KW; ++x) {
            if (PADDED) h.tap_if(wrow[rr & 1][x], row_ok && qok[x]);
            else h.tap(wrow[rr & 1][x]);
        }
#pragma unroll
        for (int oy = 0; oy < OY; ++oy)
            if (rr >= oy * SH && rr < oy * SH + KH) acc[oy].merge(h);
    }
    uint16_t* outp = dst + ((size_t)c * g.Ho * g.Wo + j) * N + 8 * n8;
#pragma unroll
    for (int oy = 0; oy < OY; ++oy) {
        const int i = i0 + oy;
        if (i < g.Ho) st16_through(outp + (size_t)i * g.Wo * N, acc[oy].result((float)(KH * KW)));
    }
}

// NCHW, 2x2 / stride 2, no padding, even H, W a multiple of 8: the tensor is a list
// of rows of W words and output row k is made of input rows 2k, 2k + 1.  A lane
// reads 8 words of both rows and writes 4 outputs.
template <class E, int MODE>
__global__ __launch_bounds__(kThreads) void pool16_nchw_2x2s2_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, uint32_t items, uint32_t W, FastDiv div_per_row) {
    const uint32_t I = blockIdx.x * kThreads + threadIdx.x;
    if (I >= items) return;
    const uint32_t orow = fd_div(I, div_per_row);
    const size_t in0 = (size_t)I * 8 + (size_t)orow * W;       // = 2*orow*W + 8*(I % per_row)
    float a[8], b[8], o[4];
    unpack8<E>(ld16_stream(src + in0), a);
    unpack8<E>(ld16_stream(src + in0 + W), b);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (MODE == CNNMEM_POOL_MAX) o[k] = fmaxf(fmaxf(a[2 * k], a[2 * k + 1]), fmaxf(b[2 * k], b[2 * k + 1]));
        else o[k] = ((a[2 * k] + a[2 * k + 1]) + (b[2 * k] + b[2 * k + 1])) * 0.25f;
    }
    u32x2 w;
    w.x = E::pack2(o[0], o[1]);
    w.y = E::pack2(o[2], o[3]);
    st8_stream(dst + (size_t)I * 4, w);
}

// NCHW through LDS: a workgroup streams a contiguous slab (whole planes, or a strip
// of rows of one plane with its halo) into 32 KB of LDS with line-aligned 128-bit
// loads, pools from LDS, and writes its outputs, which are contiguous too.
constexpr int kSlabWords = 16384;                   // 32 KB
constexpr int kSlabThreads = 512;

struct Slab16Plan {
    int planes_per_wg, rows_per_wg, strips;
    long long total_planes;
};

// OY > 1 (compile-time windows only): a lane owns a block of 2 x OY outputs.  Each of the (OY-1)*SH + KH
// input rows they touch is read once (SW + KW columns) and reduced along W once per output column; that
// row result serves every output row whose window holds it.  div_blk divides by the row blocks per plane
// (ceil(rows_out / OY)), div_pair by the column pairs per row (ceil(Wo / 2)).
template <class E, int MODE, int KH, int KW, int SH, int SW, int OY, bool PADDED>
__global__ __launch_bounds__(kSlabThreads) void pool16_nchw_slab_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, PoolGeom g, Slab16Plan plan, FastDiv div_wo,
    FastDiv div_plane_out, FastDiv div_blk, FastDiv div_pair) {
    constexpr int VEC = kSlabWords / 8 / kSlabThreads + 1;      // 128-bit loads per lane, worst case
    __shared__ __attribute__((aligned(16))) uint16_t slab[kSlabWords + 16];
    const int kh = KH ? KH : g.kh, kw = KW ? KW : g.kw, sh = SH ? SH : g.sh, sw = SW ? SW : g.sw;
    const uint32_t tile = xcd_contiguous_tile(blockIdx.x, gridDim.x);
    const int plane_in = g.H * g.W, plane_out = g.Ho * g.Wo;

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
    int r_lo = i0 * sh - g.ph;
    if (r_lo < 0) r_lo = 0;
    int r_hi = (i0 + rows_out - 1) * sh - g.ph + kh;
    if (r_hi > g.H) r_hi = g.H;
    if (planes > 1) { r_lo = 0; r_hi = g.H; }
    const size_t g_lo = (size_t)p0 * plane_in + (size_t)r_lo * g.W;
    const size_t g_hi = (size_t)(p0 + planes - 1) * plane_in + (size_t)r_hi * g.W;
    // the 128-bit stream starts on a 128-byte line of src when src is line aligned (src is 16-byte aligned)
    const size_t in_mask = (reinterpret_cast<uintptr_t>(src) & 127u) == 0 ? 63 : 7;
    const size_t a_lo = g_lo & ~in_mask;
    const size_t total_in = (size_t)plan.total_planes * plane_in;
    const int nvec = (int)((g_hi - a_lo + 7) >> 3);
    // every load is unconditional: lanes past the slab, and the one vector of the whole tensor that would
    // cross its end, re-read the last complete vector (total_in >= 8 is a dispatch condition)
    const size_t a_last = (total_in - 8) & ~(size_t)7;
    u32x4 v[VEC];
    if (a_lo + 8 * (size_t)(nvec - 1) <= a_last) {
        // every workgroup but the one at the tensor's end: no vector of the slab can cross the end, so a
        // lane's address is a uniform base plus a 32-bit offset, without the 64-bit clamp of the general form
        const uint16_t* sbase = src + a_lo;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if (k * kSlabThreads >= nvec) break;    // uniform: small planes leave most rounds empty
            const uint32_t q = threadIdx.x + k * kSlabThreads;
            v[k] = ld16_stream(sbase + 8u * (q < (uint32_t)nvec ? q : 0u));
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if (k * kSlabThreads >= nvec) break;
            const uint32_t q = threadIdx.x + k * kSlabThreads;
            if (q < (uint32_t)nvec) *reinterpret_cast<u32x4*>(slab + 8 * q) = v[k];
        }
    } else {
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if (k * kSlabThreads >= nvec) break;
            const int q = threadIdx.x + k * kSlabThreads;
            size_t a = a_lo + 8 * (size_t)(q < nvec ? q : 0);
            a = a <= a_last ? a : a_last;
            v[k] = ld16_stream(src + a);
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            if (k * kSlabThreads >= nvec) break;
            const int q = threadIdx.x + k * kSlabThreads;
            const size_t a = a_lo + 8 * (size_t)q;
            if (q < nvec && a <= a_last) *reinterpret_cast<u32x4*>(slab + 8 * q) = v[k];
        }
        for (int k = 0; k < VEC; ++k) {
            const int q = threadIdx.x + k * kSlabThreads;
            const size_t a = a_lo + 8 * (size_t)q;
            if (q < nvec && a > a_last) {           // ragged end of the tensor (at most one lane, once)
                for (int j = 0; j < 8; ++j)
                    if (a + j < total_in) slab[8 * q + j] = src[a + j];
            }
        }
    }
    __syncthreads();

    const int n_out = planes * rows_out * g.Wo;
    const size_t out0 = (size_t)p0 * plane_out + (size_t)i0 * g.Wo;
    const int lds0 = (int)((long long)((size_t)p0 * plane_in) - (long long)a_lo);
    if constexpr (OY > 1 && KH != 0) {
        constexpr int ROWS = (OY - 1) * SH + KH;
        constexpr int COLS = SW + KW;                // columns under two neighbouring windows
        const int nblk = (int)div_blk.d, npair = (int)div_pair.d;
        const int n_items = planes * nblk * npair;
        const int r_last = r_hi - 1;                 // rows of the slab: [r_lo, r_hi)
        const size_t dst_word = reinterpret_cast<uintptr_t>(dst) >> 1;
        for (int it = (int)threadIdx.x; it < n_items; it += kSlabThreads) {
            const int pb = (int)fd_div((uint32_t)it, div_pair);    // plane * nblk + block
            const int j = 2 * (it - pb * npair);
            const int pl = (int)fd_div((uint32_t)pb, div_blk);
            const int il0 = (pb - pl * nblk) * OY;                  // first output row of the lane, strip-local
            const int rb = (i0 + il0) * SH - g.ph;
            const int qb = j * SW - g.pw;
            const int base = lds0 + pl * plane_in;
            // Rows and columns are clamped into the slab.  A clamped tap of a real output lies in the same
            // window (the maximum is unchanged, the average drops it by a select); rows and columns of
            // outputs past the strip's or the row's end only feed results that are never stored.  Without
            // padding the columns of a real output need no clamp, and those of the missing second output of
            // a ragged pair run at most SW words past the row (the slab array has 16 spare words): the
            // taps of a row are then at constant offsets from one address.
            int qc[COLS];
            bool q_in[COLS];
#pragma unroll
            for (int x = 0; x < COLS; ++x) {
                const int q = qb + x;
                q_in[x] = !PADDED || (q >= 0 && q < g.W);
                int c = q;
                if (PADDED) {
                    c = q < g.W ? q : g.W - 1;
                    c = c > 0 ? c : 0;
                }
                qc[x] = c;
            }
            const size_t o_first = out0 + (size_t)(pl * rows_out + il0) * g.Wo + j;
            if constexpr (MODE == CNNMEM_POOL_MAX && E::kPairMax) {
                // binary16 maximum: the taps of the two outputs are paired in one register (tap x of the
                // left output with tap x of the right one, SW columns on) and reduced with the packed
                // maximum, so a row costs 2 KW - 1 instructions instead of COLS widenings and 2 (KW - 1)
                // maxima, and the result already is the dword to store.  Clamped taps repeat a tap of the
                // same window, which a maximum ignores.
                uint32_t hp[ROWS];
#pragma unroll
                for (int y = 0; y < ROWS; ++y) {
                    const int r = rb + y;
                    int rc = r < r_last ? r : r_last;
                    if (PADDED) rc = rc > r_lo ? rc : r_lo;
                    // Odd columns are read through a second index the compiler cannot relate to the first:
                    // left alone it fuses neighbouring words into 64-bit LDS reads at 2-byte alignment, which
                    // ran a quarter slower than five 16-bit reads.
                    const int row = base + rc * g.W;
                    int row_odd = row + 1;
                    if (!PADDED) asm("" : "+v"(row_odd));      // clamped columns are not fused anyway
                    uint32_t t[COLS];
#pragma unroll
                    for (int x = 0; x < COLS; ++x) t[x] = (x & 1) ? slab[row_odd + qc[x] - 1] : slab[row + qc[x]];
                    uint32_t acc = t[0] | (t[SW] << 16);
#pragma unroll
                    for (int x = 1; x < KW; ++x) acc = E::max2(acc, t[x] | (t[SW + x] << 16));
                    hp[y] = acc;
                }
#pragma unroll
                for (int k = 0; k < OY; ++k) {
                    uint32_t pair = hp[k * SH];
#pragma unroll
                    for (int y = 1; y < KH; ++y) pair = E::max2(pair, hp[k * SH + y]);
                    if (il0 + k >= rows_out) continue;
                    const size_t a = o_first + (size_t)k * g.Wo;
                    const bool second = j + 1 < g.Wo;
                    if (second && ((dst_word + a) & 1) == 0) {
                        *reinterpret_cast<uint32_t*>(dst + a) = pair;
                    } else {
                        dst[a] = (uint16_t)pair;
                        if (second) dst[a + 1] = (uint16_t)(pair >> 16);
                    }
                }
                continue;
            }
            float hr[2][ROWS];
#pragma unroll
            for (int y = 0; y < ROWS; ++y) {
                const int r = rb + y;
                int rc = r < r_last ? r : r_last;
                if (PADDED) rc = rc > r_lo ? rc : r_lo;
                // odd columns through a second index the compiler cannot relate to the first, so that it does
                // not fuse neighbouring words into slow 64-bit LDS reads at 2-byte alignment (see above)
                const int row = base + rc * g.W;
                int row_odd = row + 1;
                if (!PADDED) asm("" : "+v"(row_odd));
                float t[COLS];
#pragma unroll
                for (int x = 0; x < COLS; ++x) {
                    t[x] = E::widen((x & 1) ? slab[row_odd + qc[x] - 1] : slab[row + qc[x]]);
                    if (MODE != CNNMEM_POOL_MAX && PADDED) t[x] = q_in[x] ? t[x] : 0.f;
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    float acc = t[h * SW];
#pragma unroll
                    for (int x = 1; x < KW; ++x) acc = Acc<MODE>::op(acc, t[h * SW + x]);
                    if (MODE != CNNMEM_POOL_MAX && PADDED && (r < 0 || r >= g.H)) acc = 0.f;
                    hr[h][y] = acc;
                }
            }
#pragma unroll
            for (int k = 0; k < OY; ++k) {
                float a0 = hr[0][k * SH], a1 = hr[1][k * SH];
#pragma unroll
                for (int y = 1; y < KH; ++y) {
                    a0 = Acc<MODE>::op(a0, hr[0][k * SH + y]);
                    a1 = Acc<MODE>::op(a1, hr[1][k * SH + y]);
                }
                if (il0 + k >= rows_out) continue;
                const uint32_t b0 = E::narrow(Acc<MODE>::finish(a0, (float)(KH * KW)));
                const uint32_t b1 = E::narrow(Acc<MODE>::finish(a1, (float)(KH * KW)));
                const size_t a = o_first + (size_t)k * g.Wo;
                const bool second = j + 1 < g.Wo;
                if (second && ((dst_word + a) & 1) == 0) {
                    *reinterpret_cast<uint32_t*>(dst + a) = b0 | (b1 << 16);
                } else {
                    dst[a] = (uint16_t)b0;
                    if (second) dst[a + 1] = (uint16_t)b1;
                }
            }
        }
        return;
    }
    // a lane computes two neighbouring outputs and stores them as one dword; the pairs are laid so that
    // dwords (and each wavefront's 256-byte store) are aligned in dst
    const int lead = (int)(((reinterpret_cast<uintptr_t>(dst) >> 1) + out0) & 63);
    for (int o = 2 * (int)threadIdx.x - lead; o < n_out; o += 2 * kSlabThreads) {
        uint32_t bits[2] = {0, 0};
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int oo = o + half;
            if (oo < 0 || oo >= n_out) continue;
            int pl = 0, rem = oo;
            if (planes > 1) {
                pl = (int)fd_div((uint32_t)oo, div_plane_out);
                rem = oo - pl * plane_out;
            }
            const int il = (int)fd_div((uint32_t)rem, div_wo);
            const int j = rem - il * g.Wo;
            const int rb = (i0 + il) * sh - g.ph, qb = j * sw - g.pw;
            const int base = lds0 + pl * plane_in;
            float acc = Acc<MODE>::identity();
            if (KH != 0) {
                // compile-time window, no branches: with padding a tap outside the image is read from the
                // nearest in-image position, which lies in the same window (the maximum does not change,
                // the average drops it by a select)
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
                        const float t = E::widen(slab[base + rc * g.W + qc]);
                        if (MODE == CNNMEM_POOL_MAX) acc = fmaxf(acc, t);
                        else acc += in ? t : 0.f;
                    }
                }
            } else {
                // run-time window: the in-image part of the window, loop bounds clipped once (no test per tap)
                const int r_lo = rb < 0 ? 0 : rb, r_hi = rb + kh < g.H ? rb + kh : g.H;
                const int q_lo = qb < 0 ? 0 : qb, q_hi = qb + kw < g.W ? qb + kw : g.W;
                for (int r = r_lo; r < r_hi; ++r) {
                    const int row = base + r * g.W;
                    int q = q_lo;
                    for (; q + 4 <= q_hi; q += 4) {
                        const float t0 = E::widen(slab[row + q]), t1 = E::widen(slab[row + q + 1]),
                                    t2 = E::widen(slab[row + q + 2]), t3 = E::widen(slab[row + q + 3]);
                        acc = Acc<MODE>::op(Acc<MODE>::op(acc, t0), Acc<MODE>::op(t1, Acc<MODE>::op(t2, t3)));
                    }
                    for (; q < q_hi; ++q) acc = Acc<MODE>::op(acc, E::widen(slab[row + q]));
                }
            }
            bits[half] = E::narrow(Acc<MODE>::finish(acc, (float)(kh * kw)));
        }
        const bool lo_ok = o >= 0;                  // o < n_out by the loop condition
        const bool hi_ok = o + 1 >= 0 && o + 1 < n_out;
        if (lo_ok && hi_ok) *reinterpret_cast<uint32_t*>(dst + out0 + o) = bits[0] | (bits[1] << 16);
        else if (lo_ok) dst[out0 + o] = (uint16_t)bits[0];
        else if (hi_ok) dst[out0 + o + 1] = (uint16_t)bits[1];
    }
}

template <class E, int MODE>
int launch_pool16_generic(const uint16_t* src, uint16_t* dst, const PoolGeom& g, int chwn, hipStream_t st) {
    const size_t total = (size_t)g.N * g.C * g.Ho * g.Wo;
    const long long want = ceil_div64((long long)total, kThreads);
    const unsigned blocks = (unsigned)(want < 65536 ? want : 65536);
    hipLaunchKernelGGL((pool16_generic_kernel<E, MODE>), dim3(blocks), dim3(kThreads), 0, st, src, dst, g, chwn, total);
    return launch_status();
}

template <class E, int MODE, int KH, int KW, int SH, int SW, int OY>
int launch_pool16_chwn(const uint16_t* src, uint16_t* dst, const PoolGeom& g, hipStream_t st) {
    const long long row_items = (long long)(g.N / 8) * g.Wo;
    const long long bx = ceil_div64(row_items, kThreads), by = ceil_div64(g.Ho, OY);
    const long long blocks = bx * by * g.C;
    if (row_items >= 0x7fffffffLL || blocks > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
    const FastDiv dn8 = make_fastdiv((uint32_t)(g.N / 8));
    // occupancy cap for disjoint windows on large tensors, as for fp32: 64x64x224x224 fp16 73.4 % of peak
    // uncapped, 76.6-76.9 % at 3-5 workgroups per CU (CNNMEM_POOL16_WPC: -1 = never, 1..8 = that many)
    const bool light = OY == 1 && KH <= SH && KW <= SW;
    const size_t lds = light ? throttle_lds(env_int("CNNMEM_POOL16_WPC", 0), 2LL * g.N * g.C * g.H * g.W, 4)
                             : throttle_lds(env_int("CNNMEM_POOL16_WPC", -1), 2LL * g.N * g.C * g.H * g.W, 4);
    if (g.ph > 0 || g.pw > 0)
        hipLaunchKernelGGL((pool16_chwn_kernel<E, MODE, KH, KW, SH, SW, OY, true>), dim3((unsigned)blocks),
                           dim3(kThreads), lds, st, src, dst, g, (uint32_t)row_items, (uint32_t)bx, (uint32_t)by, dn8);
    else
        hipLaunchKernelGGL((pool16_chwn_kernel<E, MODE, KH, KW, SH, SW, OY, false>), dim3((unsigned)blocks),
                           dim3(kThreads), lds, st, src, dst, g, (uint32_t)row_items, (uint32_t)bx, (uint32_t)by, dn8);
    return launch_status();
}

template <class E, int MODE, int KH, int KW, int SH, int SW, int OY = 1>
int launch_pool16_slab(const uint16_t* src, uint16_t* dst, const PoolGeom& g, const Slab16Plan& plan, long long blocks,
                       hipStream_t st) {
    const FastDiv dwo = make_fastdiv((uint32_t)g.Wo), dpo = make_fastdiv((uint32_t)(g.Ho * g.Wo));
    const int rows_out = plan.strips == 1 ? g.Ho : plan.rows_per_wg;
    const FastDiv dblk = make_fastdiv((uint32_t)ceil_div(rows_out, OY)), dpair = make_fastdiv((uint32_t)((g.Wo + 1) / 2));
    if (g.ph > 0 || g.pw > 0 || KH == 0)
        hipLaunchKernelGGL((pool16_nchw_slab_kernel<E, MODE, KH, KW, SH, SW, OY, true>), dim3((unsigned)blocks),
                           dim3(kSlabThreads), 0, st, src, dst, g, plan, dwo, dpo, dblk, dpair);
    else
        hipLaunchKernelGGL((pool16_nchw_slab_kernel<E, MODE, KH, KW, SH, SW, OY, false>), dim3((unsigned)blocks),
                           dim3(kSlabThreads), 0, st, src, dst, g, plan, dwo, dpo, dblk, dpair);
    return launch_status();
}

template <class E, int MODE>
int dispatch_pool16(const uint16_t* src, uint16_t* dst, const PoolGeom& g, int layout, hipStream_t st) {
    const bool a16 = aligned16(src) && aligned16(dst);
    if (layout == CNNMEM_CHWN) {
        if (a16 && g.N % 8 == 0 && (long long)g.H * g.W * g.N < (1LL << 40)) {
            if (g.kh == 3 && g.kw == 3 && g.sh == 2 && g.sw == 2)
            {
                // outputs per lane along H: three without padding (256x96x55x55 fp16: 58 % of peak against 55 %
                // with one), two with padding (256x64x112x112 p1: 68 % against 48 % with three)
                const int rows = env_int("CNNMEM_CHWN16_ROWS", g.ph > 0 || g.pw > 0 ? 2 : 3);
                if (rows == 1) return launch_pool16_chwn<E, MODE, 3, 3, 2, 2, 1>(src, dst, g, st);
                if (rows == 2) return launch_pool16_chwn<E, MODE, 3, 3, 2, 2, 2>(src, dst, g, st);
                return launch_pool16_chwn<E, MODE, 3, 3, 2, 2, 3>(src, dst, g, st);
            }
            if (g.kh == 2 && g.kw == 2 && g.sh == 2 && g.sw == 2)
                return launch_pool16_chwn<E, MODE, 2, 2, 2, 2, 1>(src, dst, g, st);
            if (g.kh == 3 && g.kw == 3 && g.sh == 1 && g.sw == 1)
                return launch_pool16_chwn<E, MODE, 3, 3, 1, 1, 3>(src, dst, g, st);
        }
        // output rows per lane as in the 32-bit kernel: three when the window is taller than two strides, two
        // when it is between one and two strides, else one
        int rows = 1;
        if (g.Ho >= 3 && g.kh > 2 * g.sh) rows = 3;
        else if (g.Ho >= 2 && g.kh > g.sh && g.kh < 2 * g.sh) rows = 2;
        const int oy = env_int("CNNMEM_CHWN16_ANY_ROWS", rows);
        const long long hb = ceil_div64(g.Ho, oy == 3 ? 3 : (oy == 2 ? 2 : 1));
        const long long items = (long long)g.C * hb * g.Wo * (g.N / 8);
        if (a16 && g.N % 8 == 0 && items < 0x7fffffffLL && items > 0) {
            const dim3 grid((unsigned)ceil_div64(items, kThreads)), block(kThreads);
            const FastDiv dn8 = make_fastdiv((uint32_t)(g.N / 8)), dwo = make_fastdiv((uint32_t)g.Wo),
                          dhb = make_fastdiv((uint32_t)hb);
            // few outputs, tall windows (global pooling): the window's rows are dealt over 4 or 8 lanes
            int split = 0;
            if (oy == 1 && items < 262144 && g.kh >= 4 && g.kh * g.kw >= 16) split = g.kh >= 7 ? 8 : 4;
            split = env_int("CNNMEM_CHWN_SPLIT", split);
            if (oy == 1 && (split == 4 || split == 8)) {
                const dim3 sgrid((unsigned)ceil_div64(items, kThreads / split));
                if (split == 8)
                    hipLaunchKernelGGL((pool16_chwn_split_kernel<E, MODE, 8>), sgrid, block, 0, st, src, dst, g, (uint32_t)items, dn8, dwo, dhb);
                else
                    hipLaunchKernelGGL((pool16_chwn_split_kernel<E, MODE, 4>), sgrid, block, 0, st, src, dst, g, (uint32_t)items, dn8, dwo, dhb);
                return launch_status();
            }
            if (oy == 3)
                hipLaunchKernelGGL((pool16_chwn_any_kernel<E, MODE, 3>), grid, block, 0, st, src, dst, g, (uint32_t)items, dn8, dwo, dhb);
            else if (oy == 2)
                hipLaunchKernelGGL((pool16_chwn_any_kernel<E, MODE, 2>), grid, block, 0, st, src, dst, g, (uint32_t)items, dn8, dwo, dhb);
            else
                hipLaunchKernelGGL((pool16_chwn_any_kernel<E, MODE, 1>), grid, block, 0, st, src, dst, g, (uint32_t)items, dn8, dwo, dhb);
            return launch_status();
        }
        return launch_pool16_generic<E, MODE>(src, dst, g, 1, st);
    }
    const long long planes = (long long)g.N * g.C;
    if (a16 && g.kh == 2 && g.kw == 2 && g.sh == 2 && g.sw == 2 && g.ph == 0 && g.pw == 0 && g.H % 2 == 0 &&
        g.W % 8 == 0) {
        const long long per_row = g.W / 8;
        const long long items = planes * g.Ho * per_row;
        if (items < 0x7fffffffLL) {
            const FastDiv d = make_fastdiv((uint32_t)per_row);
            // the row-pair kernel is best uncapped in 16 bits (77.3 % of peak; 71.7 % at 4, 76.6 % at 5)
            const size_t lds = throttle_lds(env_int("CNNMEM_POOL16_WPC", -1), 2LL * planes * g.H * g.W, 5);
            hipLaunchKernelGGL((pool16_nchw_2x2s2_kernel<E, MODE>), dim3((unsigned)ceil_div64(items, kThreads)),
                               dim3(kThreads), lds, st, src, dst, (uint32_t)items, (uint32_t)g.W, d);
            return launch_status();
        }
    }
    const long long plane_in = (long long)g.H * g.W;
    // the slab kernel stores dwords: dst must be 4-byte aligned (a16 covers it)
    if (a16 && plane_in * planes < (1LL << 40) && plane_in * planes >= 8) {
        Slab16Plan plan;
        plan.total_planes = planes;
        bool ok = false;
        long long blocks = 0;
        const int budget = kSlabWords - 64;         // room for the line-aligned head
        if (plane_in <= budget) {
            long long p = budget / plane_in;
            const long long min_blocks = 1024;      // about one resident round of the chip (see the fp32 kernel)
            if (planes / p < min_blocks) p = planes / min_blocks > 0 ? planes / min_blocks : 1;
            if (p * (long long)g.Ho * g.Wo < (1 << 30)) {
                plan.planes_per_wg = (int)p;
                plan.rows_per_wg = g.Ho;
                plan.strips = 1;
                blocks = ceil_div64(planes, p);
                ok = true;
            }
        } else {
            const long long max_in_rows = budget / g.W;
            long long rows_out = (max_in_rows - g.kh) / g.sh + 1;
            if (max_in_rows >= g.kh && rows_out >= 1) {
                if (rows_out > g.Ho) rows_out = g.Ho;
                plan.planes_per_wg = 1;
                plan.rows_per_wg = (int)rows_out;
                plan.strips = ceil_div(g.Ho, rows_out);
                blocks = planes * plan.strips;
                ok = true;
            }
        }
        if (ok && blocks <= 0x7fffffffLL) {
            // Rows per lane (0 = default).  With 2-byte elements the per-tap work (16-bit LDS read, widening,
            // clamps) weighs twice as much against the bytes moved as in fp32, so sharing row results pays
            // even without padding: 3x3/s1 on 64x256x56x56 39 -> 52 % of peak (p1: 21 -> 52 %), 3x3/s2/p1 on
            // 256x64x112x112 53 -> 69 %, 3x3/s2 on 256x96x55x55 59 -> 61 %.
            int oy = env_int("CNNMEM_SLAB16_ROWS", 0);
            if (oy == 0) oy = g.sh == 1 ? 4 : (g.ph > 0 || g.pw > 0 ? 3 : 2);
            if (g.kh == 3 && g.kw == 3 && g.sh == 2 && g.sw == 2) {
                if (oy == 2) return launch_pool16_slab<E, MODE, 3, 3, 2, 2, 2>(src, dst, g, plan, blocks, st);
                if (oy == 3) return launch_pool16_slab<E, MODE, 3, 3, 2, 2, 3>(src, dst, g, plan, blocks, st);
                return launch_pool16_slab<E, MODE, 3, 3, 2, 2>(src, dst, g, plan, blocks, st);
            }
            if (g.kh == 2 && g.kw == 2 && g.sh == 2 && g.sw == 2)
                return launch_pool16_slab<E, MODE, 2, 2, 2, 2>(src, dst, g, plan, blocks, st);
            if (g.kh == 3 && g.kw == 3 && g.sh == 1 && g.sw == 1) {
                if (oy == 2) return launch_pool16_slab<E, MODE, 3, 3, 1, 1, 2>(src, dst, g, plan, blocks, st);
                if (oy == 4) return launch_pool16_slab<E, MODE, 3, 3, 1, 1, 4>(src, dst, g, plan, blocks, st);
                return launch_pool16_slab<E, MODE, 3, 3, 1, 1>(src, dst, g, plan, blocks, st);
            }
            return launch_pool16_slab<E, MODE, 0, 0, 0, 0>(src, dst, g, plan, blocks, st);
        }
    }
    return launch_pool16_generic<E, MODE>(src, dst, g, 0, st);
}

// =============================================================================
// Softmax (Section II.A steps 1-5, Section V.B)
// =============================================================================

// One row per TPR lanes, ITEMS 128-bit vectors (8 categories each) per lane, kept in
// registers as fp32.  A row starts `mis` words past a boundary of `align` words
// (64 = a 128-byte line when both buffers share their offset inside lines, else 8)
// and is split into a head of h = (align - mis) % align words, a body of nbody
// aligned vectors and a tail of t < 8 words; head and tail words ride in one extra
// register of lanes 0 .. h + t - 1 (h + t <= 70 <= TPR).
template <class E, int TPR, int ITEMS>
__global__ __launch_bounds__(TPR < 256 ? 256 : TPR, (ITEMS > 4 && TPR == 1024) ? 8 : 1) void softmax16_rows_kernel(
    const uint16_t* logits, uint16_t* probs, int N, int classes, int base_mis, int align) {
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
    const int mis = (int)((row_off + (size_t)base_mis) & (size_t)(align - 1));
    const int h = (align - mis) & (align - 1);
    const int nbody = (classes - h) >> 3;
    const int t = classes - h - 8 * nbody;
    const uint16_t* x = logits + row_off;
    uint16_t* y = probs + row_off;

    u32x4 raw[ITEMS];
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int q = lane + k * TPR;
        const int qc = q < nbody ? q : nbody - 1;
        raw[k] = ld16_stream(x + h + 8 * qc);
    }
    const bool is_edge = lane < h + t;
    const int edge_idx = lane < h ? lane : h + 8 * nbody + (lane - h);
    float e = kNegInf;
    if (is_edge) e = E::widen(x[edge_idx]);

    if constexpr (ITEMS > 4) {
        // Long rows: only the 16-bit words stay in registers (4 per 8 categories instead of 8) and every
        // step widens them again, the exponential being taken twice.  That halves the registers of the
        // 1024-lane kernel, which lets two rows share a CU instead of one; the arithmetic is still far
        // from what bounds the kernel, and the results are the same bit for bit.
        float m = e;
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            float a[8];
            unpack8<E>(raw[k], a);
#pragma unroll
            for (int c = 0; c < 8; ++c) m = fmaxf(m, lane + k * TPR < nbody ? a[c] : kNegInf);
            __builtin_amdgcn_sched_barrier(0);
        }
        m = row_reduce<MaxOp, TPR>(m, slots, wave, first_wave);
        e = exp_nonpos(e - m);
        float s = e;
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            float a[8];
            forget_derived(raw[k]);
            unpack8<E>(raw[k], a);
            float part = 0.f;
#pragma unroll
            for (int c = 0; c < 8; ++c) part += exp_nonpos(a[c] - m);
            s += lane + k * TPR < nbody ? part : 0.f;   // slots past the row re-read its last vector: not counted
            __builtin_amdgcn_sched_barrier(0);      // one vector at a time: widening all of them first would undo the saving
        }
        s = row_reduce<SumOp, TPR>(s, slots, wave, first_wave);
        const float inv = 1.0f / s;
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            const int q = lane + k * TPR;
            forget_derived(raw[k]);
            if (live && q < nbody) {
                float a[8];
                unpack8<E>(raw[k], a);
#pragma unroll
                for (int c = 0; c < 8; ++c) a[c] = exp_nonpos(a[c] - m) * inv;
                st16_stream(y + h + 8 * q, pack8<E>(a));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (live && is_edge) y[edge_idx] = (uint16_t)E::narrow(e * inv);
        return;
    }
    float v[ITEMS][8];
    float m = e;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        unpack8<E>(raw[k], v[k]);
        const bool in_row = lane + k * TPR < nbody;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            if (!in_row) v[k][c] = kNegInf;
            m = fmaxf(m, v[k][c]);
        }
    }
    m = row_reduce<MaxOp, TPR>(m, slots, wave, first_wave);

    e = exp_nonpos(e - m);
    float s = e;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        float part = 0.f;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            v[k][c] = exp_nonpos(v[k][c] - m);
            part += v[k][c];
        }
        s += part;
    }
    s = row_reduce<SumOp, TPR>(s, slots, wave, first_wave);

    const float inv = 1.0f / s;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int q = lane + k * TPR;
        if (live && q < nbody) {
            float o[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) o[c] = v[k][c] * inv;
            st16_stream(y + h + 8 * q, pack8<E>(o));
        }
    }
    if (live && is_edge) y[edge_idx] = (uint16_t)E::narrow(e * inv);
}

// Rows of fewer than 8 categories: one lane per row.
template <class E>
__global__ __launch_bounds__(256) void softmax16_tiny_kernel(const uint16_t* logits, uint16_t* probs, int N, int classes) {
    const long long row = (long long)blockIdx.x * 256 + threadIdx.x;
    if (row >= N) return;
    const uint16_t* x = logits + (size_t)row * classes;
    uint16_t* y = probs + (size_t)row * classes;
    float v[7];
    float m = kNegInf;
#pragma unroll
    for (int c = 0; c < 7; ++c) {
        v[c] = c < classes ? E::widen(x[c]) : kNegInf;
        m = fmaxf(m, v[c]);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < 7; ++c) {
        v[c] = exp_nonpos(v[c] - m);
        s += v[c];
    }
    const float inv = 1.0f / s;
#pragma unroll
    for (int c = 0; c < 7; ++c)
        if (c < classes) y[c] = (uint16_t)E::narrow(v[c] * inv);
}

// Short rows (8 .. 255 categories; works up to 1024) in dword-aligned buffers: G = 4 .. 32 lanes per row, 256 / G
// rows per workgroup, 8 categories per 128-bit access wherever the row happens to start
// (load8_any / store8_any); a row's last, partial vector is loaded as the row's last eight words
// and shifted into place, so every load is unconditional.
template <class E, int G, int ITEMS>
__global__ __launch_bounds__(256) void softmax16_short_kernel(const uint16_t* logits, uint16_t* probs, int N,
                                                              int classes) {
    constexpr int ROWS = 256 / G;
    const int lane = threadIdx.x % G;
    const long long row_raw = (long long)blockIdx.x * ROWS + threadIdx.x / G;
    const bool live = row_raw < N;
    const long long row = live ? row_raw : (long long)N - 1;
    const uint16_t* x = logits + (size_t)row * (size_t)classes;
    uint16_t* y = probs + (size_t)row * (size_t)classes;

    float t[ITEMS][8];
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int e0 = 8 * (lane + k * G);
        const int ec = e0 + 8 <= classes ? e0 : classes - 8;        // classes >= 8
        float a[8];
        unpack8<E>(load8_any(x + ec), a);
        const int d = e0 - ec;                                      // 0, 1..7 in the last vector, >= 8 past the row
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float val = kNegInf;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (j + d == u) val = a[u];
            t[k][j] = val;
        }
    }
    float m = kNegInf;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k)
#pragma unroll
        for (int j = 0; j < 8; ++j) m = fmaxf(m, t[k][j]);
    m = group_reduce<MaxOp, G>(m);
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        float part = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            t[k][j] = exp_nonpos(t[k][j] - m);
            part += t[k][j];
        }
        s += part;
    }
    s = group_reduce<SumOp, G>(s);
    const float inv = 1.0f / s;
    if (!live) return;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int e0 = 8 * (lane + k * G);
        if (e0 + 8 <= classes) {
            float o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = t[k][j] * inv;
            store8_any(y + e0, pack8<E>(o));
        } else {
            for (int j = 0; j < 8; ++j)
                if (e0 + j < classes) y[e0 + j] = (uint16_t)E::narrow(t[k][j] * inv);
        }
    }
}

// Rows too long for registers, buffers that are only 2-byte aligned or whose 16-byte phases
// differ: one 1024-lane workgroup per row, two sweeps (running maximum and rescaled running sum,
// then the normalised values; the second read mostly hits in L2).  VEC: dword-aligned buffers,
// 8 categories per access at any 2-byte phase.
template <class E, bool VEC>
__global__ __launch_bounds__(1024) void softmax16_stream_kernel(const uint16_t* logits, uint16_t* probs, int classes) {
    constexpr int TPR = 1024;
    __shared__ float slots[TPR / kWave];
    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const size_t row_off = (size_t)blockIdx.x * (size_t)classes;
    const uint16_t* x = logits + row_off;
    uint16_t* y = probs + row_off;
    const int nvec = VEC ? classes >> 3 : 0;
    const int tail0 = nvec << 3;

    // the first sweep's loads are cacheable: the second sweep then finds most of the row in L2 or the
    // memory-side cache (fp32, 512 x 128256: 46 -> 56 % of peak)
    float m = kNegInf, s = 0.f;
    for (int q = tid; q < nvec; q += TPR) {
        float a[8];
        unpack8<E>(load8_any_keep(x + 8 * q), a);
        float vm = a[0];
#pragma unroll
        for (int j = 1; j < 8; ++j) vm = fmaxf(vm, a[j]);
        if (vm > m) { s *= exp_nonpos(m - vm); m = vm; }
        float part = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) part += exp_nonpos(a[j] - m);
        s += part;
    }
    for (int c = tail0 + tid; c < classes; c += TPR) {
        const float v = E::widen(x[c]);
        if (v > m) { s *= exp_nonpos(m - v); m = v; }
        s += exp_nonpos(v - m);
    }
    const float row_m = row_reduce<MaxOp, TPR>(m, slots, wave, 0);
    s *= exp_nonpos(m - row_m);
    const float row_s = row_reduce<SumOp, TPR>(s, slots, wave, 0);
    const float inv = 1.0f / row_s;
    for (int q = tid; q < nvec; q += TPR) {
        float a[8];
        unpack8<E>(load8_any(x + 8 * q), a);
#pragma unroll
        for (int j = 0; j < 8; ++j) a[j] = exp_nonpos(a[j] - row_m) * inv;
        store8_any(y + 8 * q, pack8<E>(a));
    }
    for (int c = tail0 + tid; c < classes; c += TPR)
        y[c] = (uint16_t)E::narrow(exp_nonpos(E::widen(x[c]) - row_m) * inv);
}

template <class E, int G>
int launch_short16(int items, const uint16_t* logits, uint16_t* probs, int N, int classes, hipStream_t st) {
    const dim3 grid((unsigned)ceil_div64(N, 256 / G)), block(256);
    switch (items) {
        case 1: hipLaunchKernelGGL((softmax16_short_kernel<E, G, 1>), grid, block, 0, st, logits, probs, N, classes); break;
        case 2: hipLaunchKernelGGL((softmax16_short_kernel<E, G, 2>), grid, block, 0, st, logits, probs, N, classes); break;
        case 3: hipLaunchKernelGGL((softmax16_short_kernel<E, G, 3>), grid, block, 0, st, logits, probs, N, classes); break;
        default: hipLaunchKernelGGL((softmax16_short_kernel<E, G, 4>), grid, block, 0, st, logits, probs, N, classes); break;
    }
    return launch_status();
}

template <class E, int TPR, int ITEMS>
int launch_rows16(const uint16_t* logits, uint16_t* probs, int N, int classes, int base_mis, int align,
                  hipStream_t st) {
    constexpr int BLOCK = TPR < 256 ? 256 : TPR;
    constexpr int ROWS = BLOCK / TPR;
    hipLaunchKernelGGL((softmax16_rows_kernel<E, TPR, ITEMS>), dim3((unsigned)ceil_div64(N, ROWS)), dim3(BLOCK), 0, st,
                       logits, probs, N, classes, base_mis, align);
    return launch_status();
}

template <class E, int TPR>
int launch_rows16_items(int items, const uint16_t* logits, uint16_t* probs, int N, int classes, int base_mis, int align,
                        hipStream_t st) {
#define CNNMEM_CASE(I) \
    if (items <= I) return launch_rows16<E, TPR, I>(logits, probs, N, classes, base_mis, align, st)
    CNNMEM_CASE(1);
    CNNMEM_CASE(2);
    CNNMEM_CASE(3);
    CNNMEM_CASE(4);
    CNNMEM_CASE(6);
    CNNMEM_CASE(8);
#undef CNNMEM_CASE
    return CNNMEM_ERR_UNSUPPORTED;
}

template <class E>
int dispatch_softmax16(const uint16_t* logits, uint16_t* probs, int N, int classes, hipStream_t st) {
    const uintptr_t pa = reinterpret_cast<uintptr_t>(logits), pb = reinterpret_cast<uintptr_t>(probs);
    const bool same_phase = ((pa ^ pb) & 15u) == 0;
    const bool dword_ok = ((pa | pb) & 3u) == 0;
    if (classes < 8) {
        hipLaunchKernelGGL((softmax16_tiny_kernel<E>), dim3((unsigned)ceil_div64(N, 256)), dim3(256), 0, st, logits, probs,
                           N, classes);
        return launch_status();
    }
    // from 256 categories on the register kernel below is faster (72 % against 52 % at 1000 categories)
    const int short_below = env_int("CNNMEM_SOFTMAX_SHORT_BELOW", 256);
    if (classes < (short_below < 1025 ? short_below : 1025) && dword_ok) {
        // G lanes per row, at most four 128-bit vectors per lane
        const int vecs = (classes + 7) / 8;
        int g = 4;
        while (g < 32 && vecs > 4 * g) g *= 2;
        const int items = (vecs + g - 1) / g;
        switch (g) {
            case 4: return launch_short16<E, 4>(items, logits, probs, N, classes, st);
            case 8: return launch_short16<E, 8>(items, logits, probs, N, classes, st);
            case 16: return launch_short16<E, 16>(items, logits, probs, N, classes, st);
            default: return launch_short16<E, 32>(items, logits, probs, N, classes, st);
        }
    }
    // lanes 0 .. h + t - 1 carry the edges: whole-line alignment (h < 64) needs at least 128 lanes per row
    int tpr = 64;
    const long long nq = classes / 8;
    while (tpr < 1024 && nq > (long long)tpr * 4) tpr *= 2;
    const int align = (((pa ^ pb) & 127u) == 0 && classes >= 256 && tpr >= 128) ? 64 : 8;
    const int base_mis = (int)((pa & (uintptr_t)(2 * align - 1)) >> 1);
    const long long items = ceil_div64(nq, tpr);
    if (same_phase && classes >= 32 && items <= 8) {
        switch (tpr) {
            case 64: return launch_rows16_items<E, 64>((int)items, logits, probs, N, classes, base_mis, align, st);
            case 128: return launch_rows16_items<E, 128>((int)items, logits, probs, N, classes, base_mis, align, st);
            case 256: return launch_rows16_items<E, 256>((int)items, logits, probs, N, classes, base_mis, align, st);
            case 512: return launch_rows16_items<E, 512>((int)items, logits, probs, N, classes, base_mis, align, st);
            default: return launch_rows16_items<E, 1024>((int)items, logits, probs, N, classes, base_mis, align, st);
        }
    }
    if (dword_ok)
        hipLaunchKernelGGL((softmax16_stream_kernel<E, true>), dim3((unsigned)N), dim3(1024), 0, st, logits, probs, classes);
    else
        hipLaunchKernelGGL((softmax16_stream_kernel<E, false>), dim3((unsigned)N), dim3(1024), 0, st, logits, probs, classes);
    return launch_status();
}

}  // namespace

// ---- entry points for api.hip (dtype: CNNMEM_F16 or CNNMEM_BF16) ----------------
int launch_transform16(const void* src, void* dst, long long N, long long M, int src_layout, int dst_layout,
                       hipStream_t st) {
    const uint16_t* s = static_cast<const uint16_t*>(src);
    uint16_t* d = static_cast<uint16_t*>(dst);
    if (src_layout == dst_layout) {
        const long long n = N * M;
        const long long blocks = ceil_div64(ceil_div64(n, 8), kThreads);
        if (blocks > 0x7fffffffLL) return CNNMEM_ERR_UNSUPPORTED;
        hipLaunchKernelGGL(copy16_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, st, s, d, (size_t)n);
        return launch_status();
    }
    if (src_layout == CNNMEM_NCHW) return launch_transpose16(s, d, N, M, st);
    return launch_transpose16(s, d, M, N, st);
}

int launch_permute16(const void* src, void* dst, const int* dims, const int* perm, hipStream_t st) {
    return launch_permute16_impl(static_cast<const uint16_t*>(src), static_cast<uint16_t*>(dst), dims, perm, st);
}

int launch_pool16(const void* src, void* dst, const PoolGeom& g, int layout, int dtype, hipStream_t st) {
    const uint16_t* s = static_cast<const uint16_t*>(src);
    uint16_t* d = static_cast<uint16_t*>(dst);
    if (dtype == CNNMEM_F16)
        return g.mode == CNNMEM_POOL_MAX ? dispatch_pool16<Half, CNNMEM_POOL_MAX>(s, d, g, layout, st)
                                         : dispatch_pool16<Half, CNNMEM_POOL_AVG>(s, d, g, layout, st);
    return g.mode == CNNMEM_POOL_MAX ? dispatch_pool16<BFloat, CNNMEM_POOL_MAX>(s, d, g, layout, st)
                                     : dispatch_pool16<BFloat, CNNMEM_POOL_AVG>(s, d, g, layout, st);
}

int launch_softmax16(const void* logits, void* probs, int N, int classes, int dtype, hipStream_t st) {
    const uint16_t* x = static_cast<const uint16_t*>(logits);
    uint16_t* y = static_cast<uint16_t*>(probs);
    return dtype == CNNMEM_F16 ? dispatch_softmax16<Half>(x, y, N, classes, st)
                               : dispatch_softmax16<BFloat>(x, y, N, classes, st);
}

}  // namespace cnnmem
