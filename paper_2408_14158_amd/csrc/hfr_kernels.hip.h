// Device code of libhfr: streaming reduction kernels for CDNA4 (gfx950).
//
// All kernels are pure HBM streams: each lane moves 16-byte vectors, keeps
// K x U independent loads in flight before the first add, and owns every
// output element it writes (so `out` may be one of the inputs). Loads and
// stores carry the non-temporal hint: every byte is touched once.
//
// Two launch shapes exist for each operation:
//   * "wide"  - many workgroups, one tile each (grid-stride beyond a cap): the
//               shape for small and medium inputs, where latency matters;
//   * "bulk"  - one workgroup per compute unit walking the buffers in lock
//               step, results of R trips parked in registers and written in
//               one burst: HBM then sees long read phases over a narrow window
//               and few, long write bursts instead of a constant read/write
//               mix, which is worth more than 10 % of bandwidth on MI355X.
// The arithmetic is the in-order binary32 sum of Algorithm 1's inner loop and
// the add-then-scale of Algorithm 2 pass 1; the translation unit is compiled
// with -ffp-contract=off so no add/multiply pair is ever fused.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <tuple>
#include <type_traits>
#include <utility>

namespace hfr {

// Host side: enqueue `kernel` and return THIS launch's status. The triple-chevron
// form reports through the thread's last-error slot, which may still hold an
// older, unrelated failure that the library would then blame on its own launch.
template <typename... Params, typename... Args, size_t... I>
inline hipError_t launch_kernel_impl(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds_bytes,
                                     hipStream_t stream, std::index_sequence<I...>, Args&&... args) {
    std::tuple<Params...> vals(std::forward<Args>(args)...);  // each argument converted to its parameter type
    void* ptrs[] = {static_cast<void*>(&std::get<I>(vals))...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, stream);
}
template <typename... Params, typename... Args>
inline hipError_t launch_kernel(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream,
                                Args&&... args) {
    static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
    return launch_kernel_impl(kernel, grid, block, 0, stream, std::index_sequence_for<Params...>{},
                              std::forward<Args>(args)...);
}
// The same with `lds_bytes` of LDS reserved per workgroup. No kernel here uses
// LDS; a reservation only bounds how many workgroups the dispatcher places on
// one compute unit at a time (160 KiB of LDS each on gfx950).
template <typename... Params, typename... Args>
inline hipError_t launch_kernel_lds(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds_bytes,
                                    hipStream_t stream, Args&&... args) {
    static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
    return launch_kernel_impl(kernel, grid, block, lds_bytes, stream, std::index_sequence_for<Params...>{},
                              std::forward<Args>(args)...);
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// K device pointers, passed by value in the kernel-argument segment so the
// kernel reads them with scalar loads and no pointer table lives in HBM.
template <int K>
struct PtrPack {
    const void* p[K];
};

// f(integral_constant<int, I>) for I = FROM .. TO-1, unrolled at compile time
// whatever the body's size.
template <int FROM, int TO, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (FROM < TO) {
        f(std::integral_constant<int, FROM>{});
        static_for<FROM + 1, TO>(f);
    }
}

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// binary32 -> bfloat16 bits, round to nearest, ties to even. Adding 0x7FFF plus
// the kept LSB carries exactly when the discarded half is above the tie point,
// or at it with an odd kept LSB; the carry may run into the exponent, which is
// the correct overflow to infinity. NaNs are kept NaN (quiet bit forced).
__device__ __forceinline__ uint32_t bf16_rne(float f) {
    const uint32_t u = as_u32(f);
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    const uint32_t quieted = (u >> 16) | 0x0040u;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? quieted : rounded;
}

// ---- element traits: how a 16-byte vector is widened, summed and narrowed ----

struct F32Traits {
    typedef float elem_t;
    static constexpr int kVec = 4;  // elements per 16-byte vector
    static constexpr int kAcc = 4;  // fp32 accumulators per vector
    __device__ static __forceinline__ void widen(const u32x4& v, float (&a)[4]) {
#pragma unroll
        for (int c = 0; c < 4; ++c) a[c] = as_f32(v[c]);
    }
    __device__ static __forceinline__ u32x4 narrow(const float (&a)[4]) {
        u32x4 v;
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = as_u32(a[c]);
        return v;
    }
    __device__ static __forceinline__ float widen1(float x) { return x; }
    __device__ static __forceinline__ float narrow1(float x) { return x; }
};

struct BF16Traits {
    typedef uint16_t elem_t;
    static constexpr int kVec = 8;
    static constexpr int kAcc = 8;
    // A dword holds elements 2c (low half) and 2c+1 (high half); widening is
    // a shift or a mask, both exact.
    __device__ static __forceinline__ void widen(const u32x4& v, float (&a)[8]) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            a[2 * c] = as_f32(v[c] << 16);
            a[2 * c + 1] = as_f32(v[c] & 0xFFFF0000u);
        }
    }
    __device__ static __forceinline__ u32x4 narrow(const float (&a)[8]) {
        u32x4 v;
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = bf16_rne(a[2 * c]) | (bf16_rne(a[2 * c + 1]) << 16);
        return v;
    }
    __device__ static __forceinline__ float widen1(uint16_t x) { return as_f32(uint32_t(x) << 16); }
    __device__ static __forceinline__ uint16_t narrow1(float x) { return uint16_t(bf16_rne(x)); }
};

// Keeps `x` as a materialised binary32 value. Without it the compiler folds
// "multiply, then convert to fp16" into one mixed-precision instruction
// (v_fma_mixlo_f16) that rounds the exact product ONCE, straight to fp16 -
// not the two roundings (binary32, then fp16) of the arithmetic contract.
__device__ __forceinline__ float rounded_f32(float x) {
    asm volatile("" : "+v"(x));
    return x;
}

// IEEE binary16 storage: the hardware converts (v_cvt_f32_f16 is exact,
// v_cvt_f16_f32 rounds to nearest even in the default rounding mode, fp16
// subnormals are never flushed); the GPU tests check every pattern pair
// against the CPU oracle.
struct F16Traits {
    typedef uint16_t elem_t;
    typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
    static constexpr int kVec = 8;
    static constexpr int kAcc = 8;
    __device__ static __forceinline__ void widen(const u32x4& v, float (&a)[8]) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const half2_t h = __builtin_bit_cast(half2_t, uint32_t(v[c]));
            a[2 * c] = float(h[0]);
            a[2 * c + 1] = float(h[1]);
        }
    }
    __device__ static __forceinline__ u32x4 narrow(const float (&a)[8]) {
        u32x4 v;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            half2_t h;
            h[0] = _Float16(rounded_f32(a[2 * c]));
            h[1] = _Float16(rounded_f32(a[2 * c + 1]));
            v[c] = __builtin_bit_cast(uint32_t, h);
        }
        return v;
    }
    __device__ static __forceinline__ float widen1(uint16_t x) { return float(__builtin_bit_cast(_Float16, x)); }
    __device__ static __forceinline__ uint16_t narrow1(float x) {
        return __builtin_bit_cast(uint16_t, _Float16(rounded_f32(x)));
    }
};

// OCP 8-bit floats: sixteen elements per 16-byte vector. Widening uses the
// single-element hardware conversion with a byte select (the packed widening
// instruction returned the low byte's value in both results on this chip and
// is not used); narrowing uses the packed conversion, which rounds to nearest
// even, keeps subnormals and turns what does not fit into NaN (E4M3) or
// infinity (E5M2). Both were checked against the format definitions on every
// rounding boundary before use, and the GPU tests repeat that through the ABI.
template <bool E5M2>
struct FP8Traits {
    typedef uint8_t elem_t;
    static constexpr int kVec = 16;
    static constexpr int kAcc = 16;
    __device__ static __forceinline__ float cvt1(uint32_t word, int byte) {
        if constexpr (E5M2) {
            switch (byte) {
                case 0: return __builtin_amdgcn_cvt_f32_bf8(word, 0);
                case 1: return __builtin_amdgcn_cvt_f32_bf8(word, 1);
                case 2: return __builtin_amdgcn_cvt_f32_bf8(word, 2);
                default: return __builtin_amdgcn_cvt_f32_bf8(word, 3);
            }
        } else {
            switch (byte) {
                case 0: return __builtin_amdgcn_cvt_f32_fp8(word, 0);
                case 1: return __builtin_amdgcn_cvt_f32_fp8(word, 1);
                case 2: return __builtin_amdgcn_cvt_f32_fp8(word, 2);
                default: return __builtin_amdgcn_cvt_f32_fp8(word, 3);
            }
        }
    }
    __device__ static __forceinline__ uint32_t pack2(float a, float b, uint32_t old, bool high) {
        if constexpr (E5M2) {
            return high ? uint32_t(__builtin_amdgcn_cvt_pk_bf8_f32(a, b, int(old), true))
                        : uint32_t(__builtin_amdgcn_cvt_pk_bf8_f32(a, b, int(old), false));
        } else {
            return high ? uint32_t(__builtin_amdgcn_cvt_pk_fp8_f32(a, b, int(old), true))
                        : uint32_t(__builtin_amdgcn_cvt_pk_fp8_f32(a, b, int(old), false));
        }
    }
    __device__ static __forceinline__ void widen(const u32x4& v, float (&a)[16]) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            a[4 * c] = cvt1(v[c], 0);
            a[4 * c + 1] = cvt1(v[c], 1);
            a[4 * c + 2] = cvt1(v[c], 2);
            a[4 * c + 3] = cvt1(v[c], 3);
        }
    }
    __device__ static __forceinline__ u32x4 narrow(const float (&a)[16]) {
        u32x4 v;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t lo = pack2(a[4 * c], a[4 * c + 1], 0u, false);
            v[c] = pack2(a[4 * c + 2], a[4 * c + 3], lo, true);
        }
        return v;
    }
    __device__ static __forceinline__ float widen1(uint8_t x) { return cvt1(uint32_t(x), 0); }
    __device__ static __forceinline__ uint8_t narrow1(float x) { return uint8_t(pack2(x, x, 0u, false) & 0xFFu); }
};
typedef FP8Traits<false> E4M3Traits;
typedef FP8Traits<true> E5M2Traits;

// ---- 16-byte vector access ----
// ALIGNED: natural 16-byte alignment. Otherwise the access is declared with the
// element's alignment only and the compiler picks what the target allows.
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));
typedef u32x4 u32x4_a1 __attribute__((aligned(1)));

template <int ALIGN>
__device__ __forceinline__ u32x4 load_vec(const void* p) {
    if constexpr (ALIGN >= 16) {
        return __builtin_nontemporal_load(static_cast<const u32x4*>(p));
    } else if constexpr (ALIGN == 4) {
        return __builtin_nontemporal_load(static_cast<const u32x4_a4*>(p));
    } else if constexpr (ALIGN == 2) {
        return __builtin_nontemporal_load(static_cast<const u32x4_a2*>(p));
    } else {
        return __builtin_nontemporal_load(static_cast<const u32x4_a1*>(p));
    }
}

template <int ALIGN>
__device__ __forceinline__ void store_vec(void* p, u32x4 v) {
    if constexpr (ALIGN >= 16) {
        __builtin_nontemporal_store(v, static_cast<u32x4*>(p));
    } else if constexpr (ALIGN == 4) {
        __builtin_nontemporal_store(v, static_cast<u32x4_a4*>(p));
    } else if constexpr (ALIGN == 2) {
        __builtin_nontemporal_store(v, static_cast<u32x4_a2*>(p));
    } else {
        __builtin_nontemporal_store(v, static_cast<u32x4_a1*>(p));
    }
}

// Byte offset of lane `tid`'s u-th vector inside a tile. Kept 32-bit so the
// access is "uniform 64-bit base + 32-bit lane offset" (scalar base register
// plus one offset VGPR) instead of a 64-bit address per lane.
template <int BLOCK>
__device__ __forceinline__ uint32_t lane_off(int u, unsigned tid) {
    return (uint32_t(u) * BLOCK + tid) * 16u;
}

// ---------------------------------------------------------------------------
// K-way in-order sum (Algorithm 1, inner loop).
//
// Work decomposition: the n elements are nvec = n / kVec whole 16-byte vectors
// plus a scalar tail of n % kVec elements. A tile is BLOCK * U consecutive
// vectors; workgroup b takes tiles b, b + gridDim.x, ... (consecutive
// workgroups touch consecutive tiles, which spreads one wavefront of tiles over
// all HBM channels). Inside a tile lane t handles vectors t, t + BLOCK, ...,
// so each load instruction of a wavefront covers 1 KiB of contiguous memory.
// All K * U loads of a trip are issued before the first add.
// ---------------------------------------------------------------------------
// In-order sum of one 16-byte vector position across the K loaded vectors.
// What happens to the fp32 sum before it is narrowed and stored:
//   kEpiNone     nothing (the K-way sum);
//   kEpiScale    one multiply by `scale` (the fused K-way average);
//   kEpiCombine  the LAST input is not a peer buffer but the partial received
//                from the neighbouring node: the sum of the first K - 1 inputs
//                is rounded to the storage type exactly as a stored node
//                partial would be, widened again, the last input is added and
//                the result multiplied by `scale` - Algorithm 1's inner loop
//                and Algorithm 2's pass 1 in one pass over memory, bit for bit
//                what the two separate kernels produce.
constexpr int kEpiNone = 0, kEpiScale = 1, kEpiCombine = 2;

template <typename T, int K, int EPI>
__device__ __forceinline__ u32x4 sum_vectors(const u32x4 (&v)[K], float scale) {
    constexpr int kAcc = T::kAcc;
    float acc[kAcc];
    T::widen(v[0], acc);
#pragma unroll
    for (int j = 1; j < K; ++j) {
        if constexpr (EPI == kEpiCombine) {
            if (j == K - 1) {
                const u32x4 stored = T::narrow(acc);  // the node partial as it would sit in memory
                T::widen(stored, acc);
            }
        }
        float x[kAcc];
        T::widen(v[j], x);
#pragma unroll
        for (int c = 0; c < kAcc; ++c) acc[c] = acc[c] + x[c];
    }
    if constexpr (EPI != kEpiNone) {
#pragma unroll
        for (int c = 0; c < kAcc; ++c) acc[c] = acc[c] * scale;
    }
    return T::narrow(acc);
}

// One element of the scalar tail.
template <typename T, int K, int EPI>
__device__ __forceinline__ void sum_scalar(const PtrPack<K>& in, void* out, size_t i, float scale) {
    typedef typename T::elem_t E;
    float acc = T::widen1(static_cast<const E*>(in.p[0])[i]);
#pragma unroll
    for (int j = 1; j < K; ++j) {
        if constexpr (EPI == kEpiCombine) {
            if (j == K - 1) acc = T::widen1(T::narrow1(acc));
        }
        acc = acc + T::widen1(static_cast<const E*>(in.p[j])[i]);
    }
    if constexpr (EPI != kEpiNone) acc = acc * scale;
    static_cast<E*>(out)[i] = T::narrow1(acc);
}

template <typename T, int K, int U, int BLOCK, int ALIGN, int EPI>
__global__ __launch_bounds__(BLOCK) void reduce_sum_kernel(PtrPack<K> in, void* out, size_t n, float scale) {
    constexpr int kVec = T::kVec;
    constexpr size_t kTileVecs = size_t(BLOCK) * U;
    const size_t nvec = n / kVec;
    const size_t ntiles = (nvec + kTileVecs - 1) / kTileVecs;
    const unsigned tid = threadIdx.x;

    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const size_t base = tile * kTileVecs;  // first vector of the tile (uniform)
        if (base + kTileVecs <= nvec) {
            u32x4 v[U][K];
#pragma unroll
            for (int j = 0; j < K; ++j) {
                const char* pj = static_cast<const char*>(in.p[j]) + base * 16;
#pragma unroll
                for (int u = 0; u < U; ++u) v[u][j] = load_vec<ALIGN>(pj + lane_off<BLOCK>(u, tid));
            }
            // every load of the trip is in flight before the first add
            __builtin_amdgcn_sched_barrier(0);
            char* po = static_cast<char*>(out) + base * 16;
#pragma unroll
            for (int u = 0; u < U; ++u)
                store_vec<ALIGN>(po + lane_off<BLOCK>(u, tid), sum_vectors<T, K, EPI>(v[u], scale));
        } else {
            // last, partial tile: one bounded vector at a time
#pragma unroll 1
            for (int u = 0; u < U; ++u) {
                const size_t idx = base + size_t(u) * BLOCK + tid;
                if (idx < nvec) {
                    u32x4 w[K];
#pragma unroll
                    for (int j = 0; j < K; ++j)
                        w[j] = load_vec<ALIGN>(static_cast<const char*>(in.p[j]) + idx * 16);
                    store_vec<ALIGN>(static_cast<char*>(out) + idx * 16, sum_vectors<T, K, EPI>(w, scale));
                }
            }
        }
    }

    // scalar tail: fewer than kVec elements, done by the first lanes of block 0
    const size_t tail0 = nvec * kVec;
    if (blockIdx.x == 0 && tail0 + tid < n) {
        sum_scalar<T, K, EPI>(in, out, tail0 + tid, scale);
    }
}

// ---------------------------------------------------------------------------
// Two-operand combine and average (Algorithm 2, pass 1, then one multiply):
// out = fl(fl(a + b) * scale). Same decomposition as above with K = 2.
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ u32x4 combine_vectors(const u32x4& va, const u32x4& vb, float scale) {
    constexpr int kAcc = T::kAcc;
    float x[kAcc], y[kAcc];
    T::widen(va, x);
    T::widen(vb, y);
#pragma unroll
    for (int c = 0; c < kAcc; ++c) {
        const float t = x[c] + y[c];  // first rounding
        x[c] = t * scale;             // second rounding (never an fma)
    }
    return T::narrow(x);
}

template <typename T, int U, int BLOCK, int ALIGN>
__global__ __launch_bounds__(BLOCK) void combine_avg_kernel(const void* a, const void* b, void* out,
                                                            size_t n, float scale) {
    constexpr int kVec = T::kVec;
    constexpr size_t kTileVecs = size_t(BLOCK) * U;
    const size_t nvec = n / kVec;
    const size_t ntiles = (nvec + kTileVecs - 1) / kTileVecs;
    const unsigned tid = threadIdx.x;

    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const size_t base = tile * kTileVecs;
        if (base + kTileVecs <= nvec) {
            const char* pa = static_cast<const char*>(a) + base * 16;
            const char* pb = static_cast<const char*>(b) + base * 16;
            char* po = static_cast<char*>(out) + base * 16;
            u32x4 va[U], vb[U];
#pragma unroll
            for (int u = 0; u < U; ++u) va[u] = load_vec<ALIGN>(pa + lane_off<BLOCK>(u, tid));
#pragma unroll
            for (int u = 0; u < U; ++u) vb[u] = load_vec<ALIGN>(pb + lane_off<BLOCK>(u, tid));
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < U; ++u)
                store_vec<ALIGN>(po + lane_off<BLOCK>(u, tid),
                                     combine_vectors<T>(va[u], vb[u], scale));
        } else {
#pragma unroll 1
            for (int u = 0; u < U; ++u) {
                const size_t idx = base + size_t(u) * BLOCK + tid;
                if (idx < nvec) {
                    const u32x4 wa = load_vec<ALIGN>(static_cast<const char*>(a) + idx * 16);
                    const u32x4 wb = load_vec<ALIGN>(static_cast<const char*>(b) + idx * 16);
                    store_vec<ALIGN>(static_cast<char*>(out) + idx * 16,
                                         combine_vectors<T>(wa, wb, scale));
                }
            }
        }
    }

    const size_t tail0 = nvec * kVec;
    if (blockIdx.x == 0 && tail0 + tid < n) {
        typedef typename T::elem_t E;
        const size_t i = tail0 + tid;
        const float t = T::widen1(static_cast<const E*>(a)[i]) + T::widen1(static_cast<const E*>(b)[i]);
        static_cast<E*>(out)[i] = T::narrow1(t * scale);
    }
}


// ---------------------------------------------------------------------------
// Bulk shape of the K-way sum: launched with one workgroup per compute unit.
//
// A tile is blockDim.x * U vectors. Workgroup b visits tiles b, b + G, b + 2G, ...
// (G = gridDim.x), so at any moment the whole chip reads one narrow window
// (G tiles) of each input, which keeps DRAM rows open. The results of R
// consecutive trips stay in registers (R * U vectors per lane) and are stored
// together, so reads and writes reach HBM in long alternating phases.
// A burst holds `trips` <= R trips; the host splits a workgroup's trips evenly
// over its bursts (a last burst of only a few trips is a short read phase that
// ends in a store burst with nothing to overlap it).
// Whole tiles only; the remaining vectors and the scalar tail are done by the
// last and the first workgroup.
// ---------------------------------------------------------------------------
// Stream skew. The K loads of a trip hit the same offset of K buffers; when
// the buffers lie a "bad" distance apart, those K addresses fall into the same
// DRAM bank of the same channel and the loads serialise on row activations
// (measured: 5.9 instead of 6.7 TB/s). A skew pattern lets some streams run a
// few trips ahead of the trip being summed, which moves them a few MiB away;
// what they load early waits in registers. The sum itself is unchanged: each
// result still adds the same K operands in the same order. Which pattern helps
// depends on the placement and is found by measurement (host side).
//   0: no skew   1: leads 0,1,0,1,...   2: leads 0,2,0,2,...   3: leads 3,2,1,0,3,...
constexpr int kSkewPatterns = 4;
template <int SKEW>
__host__ __device__ constexpr int skew_lead(int j) {
    return SKEW == 1 ? (j & 1) : (SKEW == 2 ? 2 * (j & 1) : (SKEW == 3 ? 3 - (j & 3) : 0));
}
constexpr int kMaxSkewLead = 3;

// Request pacing. Throughput of the bulk shape depends on how many loads a
// compute unit keeps in flight: with too few HBM idles, with too many the
// requests of fast workgroups run ahead into later tiles, the window the chip
// reads at any instant widens and DRAM rows are closed before they are used up
// (measured: the best count is some 25 to 40 KiB per compute unit, and every
// element type and input count has its own optimum because the arithmetic of a
// trip is itself a pause between two rounds of loads). Two run-time knobs set
// it, both chosen on the host from a measured table: the workgroup size (a tile
// is blockDim.x * U vectors; BLOCK is only its upper bound) and `pace`, a pause
// of pace * 64 clocks after each trip's arithmetic.
__device__ __forceinline__ void pace_trip(unsigned pace) {
    for (unsigned i = 0; i < pace; ++i) __builtin_amdgcn_s_sleep(1);
}

// Byte offset of lane `tid`'s u-th vector inside a tile of `block` * U vectors.
__device__ __forceinline__ uint32_t lane_off_rt(int u, unsigned tid, unsigned block) {
    return (uint32_t(u) * block + tid) * 16u;
}

template <typename T, int K, int U, int R, int BLOCK, int ALIGN, int EPI, int SKEW = 0>
__global__ __launch_bounds__(BLOCK) void reduce_sum_bulk_kernel(PtrPack<K> in, void* out, size_t n, size_t ntiles,
                                                                float scale, unsigned trips, unsigned pace) {
    static_assert(SKEW == 0 || U == 1, "skewed streams are built for one vector per lane and trip");
    constexpr int kVec = T::kVec;
    const unsigned block = blockDim.x;  // <= BLOCK
    const size_t kTileVecs = size_t(block) * U;
    const size_t nvec = n / kVec;
    // ntiles = nvec / kTileVecs, the whole tiles, comes from the host: the tile size is
    // a run-time value here and a 64-bit division by it would be a long sequence
    const unsigned tid = threadIdx.x;
    const size_t G = gridDim.x;
    trips = trips < 1u ? 1u : (trips > unsigned(R) ? unsigned(R) : trips);  // the loop below must advance

    if constexpr (SKEW == 0) {
        for (size_t t0 = blockIdx.x; t0 < ntiles; t0 += G * trips) {
            u32x4 res[R][U];
            auto load_and_sum = [&](const int r) {
                const size_t tile = t0 + G * r;  // uniform
                if (unsigned(r) < trips && tile < ntiles) {
                    u32x4 v[U][K];
#pragma unroll
                    for (int j = 0; j < K; ++j) {
                        const char* pj = static_cast<const char*>(in.p[j]) + tile * (kTileVecs * 16);
#pragma unroll
                        for (int u = 0; u < U; ++u) v[u][j] = load_vec<ALIGN>(pj + lane_off_rt(u, tid, block));
                    }
                    __builtin_amdgcn_sched_barrier(0);  // the trip's loads go out before its first add
#pragma unroll
                    for (int u = 0; u < U; ++u) res[r][u] = sum_vectors<T, K, EPI>(v[u], scale);
                    pace_trip(pace);
                }
                __builtin_amdgcn_sched_barrier(0);  // trips stay in program order
            };
            auto store = [&](const int r) {
                const size_t tile = t0 + G * r;
                if (unsigned(r) < trips && tile < ntiles) {
                    char* po = static_cast<char*>(out) + tile * (kTileVecs * 16);
#pragma unroll
                    for (int u = 0; u < U; ++u) store_vec<ALIGN>(po + lane_off_rt(u, tid, block), res[r][u]);
                }
            };
            // From five inputs on (where this shape is the default) the trips are
            // unrolled through templates. With a pragma the compiler hoists the
            // thirty-two "does this trip exist" tests out of the trips and spills
            // the flags to vector lanes, which costs each trip a few dozen cycles
            // that the pacing table was not measured with (fp32, 8 to 10 inputs:
            // 3 to 5 % slower), and for the largest bodies it gives up unrolling, so
            // that res[], indexed by a loop variable, ends up in scratch. The
            // template form compiles several times slower; the small input counts,
            // which take this shape only when a knob forces it, keep the pragma.
            if constexpr (K >= 5) {
                static_for<0, R>([&](auto rc) { load_and_sum(decltype(rc)::value); });
                static_for<0, R>([&](auto rc) { store(decltype(rc)::value); });
            } else {
#pragma unroll
                for (int r = 0; r < R; ++r) load_and_sum(r);
#pragma unroll
                for (int r = 0; r < R; ++r) store(r);
            }
        }
    } else {
        // Before trip c is summed, held[j][i] is stream j's vector for this
        // workgroup's trip c + i (i < lead of j). A workgroup's trips are the
        // tiles blockIdx.x, blockIdx.x + G, ... in order, across bursts. Every
        // index below is a compile-time constant, so held[] and res[] live in
        // registers and moving held[] along costs no instruction.
        u32x4 held[K][kMaxSkewLead];
        static_for<0, K>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            static_for<0, skew_lead<SKEW>(j)>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                const size_t tile = blockIdx.x + G * i;
                if (tile < ntiles)
                    held[j][i] = load_vec<ALIGN>(static_cast<const char*>(in.p[j]) + tile * (kTileVecs * 16) +
                                                 lane_off_rt(0, tid, block));
            });
        });
        for (size_t t0 = blockIdx.x; t0 < ntiles; t0 += G * trips) {
            u32x4 res[R];
            static_for<0, R>([&](auto rc) {
                constexpr int r = decltype(rc)::value;
                const size_t tile = t0 + G * r;  // uniform
                if (unsigned(r) < trips && tile < ntiles) {
                    u32x4 v[K];
                    // The streams without a lead first: their vectors are the only ones this trip's
                    // sum has to wait for, and loads return in issue order. The leading streams' loads
                    // follow without a branch: a tile index past the end is clamped to the last tile
                    // (in bounds; what it loads is never summed), so the trip's loads go out back to
                    // back and the arithmetic overlaps with the leading loads still in flight.
                    static_for<0, K>([&](auto jc) {
                        constexpr int j = decltype(jc)::value;
                        if constexpr (skew_lead<SKEW>(j) == 0)
                            v[j] = load_vec<ALIGN>(static_cast<const char*>(in.p[j]) + tile * (kTileVecs * 16) +
                                                   lane_off_rt(0, tid, block));
                    });
                    static_for<0, K>([&](auto jc) {
                        constexpr int j = decltype(jc)::value;
                        constexpr int d = skew_lead<SKEW>(j);
                        if constexpr (d > 0) {
                            const size_t want = tile + G * d;  // the tile stream j will need d trips from now
                            const size_t tj = want < ntiles ? want : ntiles - 1;
                            v[j] = load_vec<ALIGN>(static_cast<const char*>(in.p[j]) + tj * (kTileVecs * 16) +
                                                   lane_off_rt(0, tid, block));
                        }
                    });
                    __builtin_amdgcn_sched_barrier(0);
                    u32x4 x[K];
                    static_for<0, K>([&](auto jc) {
                        constexpr int j = decltype(jc)::value;
                        constexpr int d = skew_lead<SKEW>(j);
                        if constexpr (d == 0) {
                            x[j] = v[j];
                        } else {
                            x[j] = held[j][0];
                            static_for<0, d - 1>([&](auto ic) {
                                held[j][decltype(ic)::value] = held[j][decltype(ic)::value + 1];
                            });
                            held[j][d - 1] = v[j];  // some other tile's data when past the end: never summed
                        }
                    });
                    res[r] = sum_vectors<T, K, EPI>(x, scale);
                    pace_trip(pace);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            static_for<0, R>([&](auto rc) {
                constexpr int r = decltype(rc)::value;
                const size_t tile = t0 + G * r;
                if (unsigned(r) < trips && tile < ntiles)
                    store_vec<ALIGN>(static_cast<char*>(out) + tile * (kTileVecs * 16) + lane_off_rt(0, tid, block),
                                     res[r]);
            });
        }
    }

    // vectors beyond the last whole tile: fewer than a tile, last workgroup
    if (blockIdx.x == G - 1) {
        for (size_t idx = ntiles * kTileVecs + tid; idx < nvec; idx += block) {
            u32x4 w[K];
#pragma unroll
            for (int j = 0; j < K; ++j) w[j] = load_vec<ALIGN>(static_cast<const char*>(in.p[j]) + idx * 16);
            store_vec<ALIGN>(static_cast<char*>(out) + idx * 16, sum_vectors<T, K, EPI>(w, scale));
        }
    }
    // scalar tail: fewer than kVec elements, first lanes of workgroup 0
    const size_t tail0 = nvec * kVec;
    if (blockIdx.x == 0 && tail0 + tid < n) {
        sum_scalar<T, K, EPI>(in, out, tail0 + tid, scale);
    }
}

// ---------------------------------------------------------------------------
// The bulk shape over a LIST of chunks in one launch (plain sum, one vector per
// lane and trip, 16-byte aligned buffers). Every workgroup walks the list in
// the same order and does, chunk after chunk, exactly what reduce_sum_bulk_kernel
// does for one chunk, so the chip never drains between chunks: a workgroup that
// has finished its tiles of one chunk goes on with the next while its
// neighbours are still storing. For chunks that lie apart in memory (which the
// host cannot merge into one longer sum) and are too short to amortise a launch
// of their own: measured against one bulk launch per chunk +21 % at 8 MiB per
// buffer, +7 % at 16 MiB, +3 % at 24 MiB (K = 8 bf16). The chunk table travels
// in the kernel arguments. SKEW as in reduce_sum_bulk_kernel (patterns 0 and 3
// are built).
template <int K>
struct ListEntry {
    const void* in[K];
    void* out;
    size_t n;        // elements
    size_t ntiles;   // whole tiles of blockDim.x vectors
    unsigned trips;  // trips per burst, 1 .. R (host: bulk_trips_per_burst)
    unsigned pad;
};
template <int K>
constexpr int list_capacity() {
    return int((3840 - 16) / sizeof(ListEntry<K>));
}
template <int K>
struct ListTable {
    ListEntry<K> e[list_capacity<K>()];
    int count;
};

template <typename T, int K, int R, int BLOCK, int SKEW = 0>
__global__ __launch_bounds__(BLOCK) void reduce_sum_bulk_list_kernel(ListTable<K> tab, unsigned pace) {
    constexpr int kVec = T::kVec;
    const unsigned block = blockDim.x;  // <= BLOCK
    const size_t kTileVecs = size_t(block);
    const unsigned tid = threadIdx.x;
    const size_t G = gridDim.x;
    for (int c = 0; c < tab.count; ++c) {  // uniform
        const ListEntry<K>& e = tab.e[c];
        const size_t n = e.n, ntiles = e.ntiles, nvec = n / kVec;
        const unsigned trips = e.trips < 1u ? 1u : (e.trips > unsigned(R) ? unsigned(R) : e.trips);
        if constexpr (SKEW == 0) {
            for (size_t t0 = blockIdx.x; t0 < ntiles; t0 += G * trips) {
                u32x4 res[R];
                static_for<0, R>([&](auto rc) {
                    constexpr int r = decltype(rc)::value;
                    const size_t tile = t0 + G * r;  // uniform
                    if (unsigned(r) < trips && tile < ntiles) {
                        u32x4 v[K];
#pragma unroll
                        for (int j = 0; j < K; ++j)
                            v[j] = load_vec<16>(static_cast<const char*>(e.in[j]) + tile * (kTileVecs * 16) +
                                                lane_off_rt(0, tid, block));
                        __builtin_amdgcn_sched_barrier(0);  // the trip's loads go out before its first add
                        res[r] = sum_vectors<T, K, kEpiNone>(v, 1.0f);
                        pace_trip(pace);
                    }
                    __builtin_amdgcn_sched_barrier(0);  // trips stay in program order
                });
                static_for<0, R>([&](auto rc) {
                    constexpr int r = decltype(rc)::value;
                    const size_t tile = t0 + G * r;
                    if (unsigned(r) < trips && tile < ntiles)
                        store_vec<16>(static_cast<char*>(e.out) + tile * (kTileVecs * 16) + lane_off_rt(0, tid, block),
                                      res[r]);
                });
            }
        } else {
            // the skewed trips of reduce_sum_bulk_kernel, chunk by chunk: held[j][i] is stream j's
            // vector for this workgroup's trip c + i of the chunk (i < lead of j)
            u32x4 held[K][kMaxSkewLead];
            static_for<0, K>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                static_for<0, skew_lead<SKEW>(j)>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    const size_t tile = blockIdx.x + G * i;
                    if (tile < ntiles)
                        held[j][i] = load_vec<16>(static_cast<const char*>(e.in[j]) + tile * (kTileVecs * 16) +
                                                  lane_off_rt(0, tid, block));
                });
            });
            for (size_t t0 = blockIdx.x; t0 < ntiles; t0 += G * trips) {
                u32x4 res[R];
                static_for<0, R>([&](auto rc) {
                    constexpr int r = decltype(rc)::value;
                    const size_t tile = t0 + G * r;  // uniform
                    if (unsigned(r) < trips && tile < ntiles) {
                        u32x4 v[K];
                        static_for<0, K>([&](auto jc) {
                            constexpr int j = decltype(jc)::value;
                            if constexpr (skew_lead<SKEW>(j) == 0)
                                v[j] = load_vec<16>(static_cast<const char*>(e.in[j]) + tile * (kTileVecs * 16) +
                                                    lane_off_rt(0, tid, block));
                        });
                        static_for<0, K>([&](auto jc) {
                            constexpr int j = decltype(jc)::value;
                            constexpr int d = skew_lead<SKEW>(j);
                            if constexpr (d > 0) {
                                const size_t want = tile + G * d;
                                const size_t tj = want < ntiles ? want : ntiles - 1;  // in bounds; never summed when clamped
                                v[j] = load_vec<16>(static_cast<const char*>(e.in[j]) + tj * (kTileVecs * 16) +
                                                    lane_off_rt(0, tid, block));
                            }
                        });
                        __builtin_amdgcn_sched_barrier(0);
                        u32x4 x[K];
                        static_for<0, K>([&](auto jc) {
                            constexpr int j = decltype(jc)::value;
                            constexpr int d = skew_lead<SKEW>(j);
                            if constexpr (d == 0) {
                                x[j] = v[j];
                            } else {
                                x[j] = held[j][0];
                                static_for<0, d - 1>([&](auto ic) {
                                    held[j][decltype(ic)::value] = held[j][decltype(ic)::value + 1];
                                });
                                held[j][d - 1] = v[j];
                            }
                        });
                        res[r] = sum_vectors<T, K, kEpiNone>(x, 1.0f);
                        pace_trip(pace);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
                static_for<0, R>([&](auto rc) {
                    constexpr int r = decltype(rc)::value;
                    const size_t tile = t0 + G * r;
                    if (unsigned(r) < trips && tile < ntiles)
                        store_vec<16>(static_cast<char*>(e.out) + tile * (kTileVecs * 16) + lane_off_rt(0, tid, block),
                                      res[r]);
                });
            }
        }
        // vectors beyond the last whole tile: fewer than a tile, last workgroup
        if (blockIdx.x == G - 1) {
            for (size_t idx = ntiles * kTileVecs + tid; idx < nvec; idx += block) {
                u32x4 w[K];
#pragma unroll
                for (int j = 0; j < K; ++j) w[j] = load_vec<16>(static_cast<const char*>(e.in[j]) + idx * 16);
                store_vec<16>(static_cast<char*>(e.out) + idx * 16, sum_vectors<T, K, kEpiNone>(w, 1.0f));
            }
        }
        // scalar tail: fewer than kVec elements, first lanes of workgroup 0
        const size_t tail0 = nvec * kVec;
        if (blockIdx.x == 0 && tail0 + tid < n) {
            PtrPack<K> pk;
#pragma unroll
            for (int j = 0; j < K; ++j) pk.p[j] = e.in[j];
            sum_scalar<T, K, kEpiNone>(pk, e.out, tail0 + tid, 1.0f);
        }
    }
}

// Bulk shape of the combine: two read streams, U vectors of each per trip.
template <typename T, int U, int R, int BLOCK, int ALIGN>
__global__ __launch_bounds__(BLOCK) void combine_avg_bulk_kernel(const void* a, const void* b, void* out,
                                                                 size_t n, float scale, unsigned trips) {
    constexpr int kVec = T::kVec;
    constexpr size_t kTileVecs = size_t(BLOCK) * U;
    const size_t nvec = n / kVec;
    const size_t ntiles = nvec / kTileVecs;
    const unsigned tid = threadIdx.x;
    const size_t G = gridDim.x;
    trips = trips < 1u ? 1u : (trips > unsigned(R) ? unsigned(R) : trips);  // the loop below must advance

    for (size_t t0 = blockIdx.x; t0 < ntiles; t0 += G * trips) {
        u32x4 res[R][U];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const size_t tile = t0 + G * r;
            if (unsigned(r) < trips && tile < ntiles) {
                const char* pa = static_cast<const char*>(a) + tile * (kTileVecs * 16);
                const char* pb = static_cast<const char*>(b) + tile * (kTileVecs * 16);
                u32x4 va[U], vb[U];
#pragma unroll
                for (int u = 0; u < U; ++u) va[u] = load_vec<ALIGN>(pa + lane_off<BLOCK>(u, tid));
#pragma unroll
                for (int u = 0; u < U; ++u) vb[u] = load_vec<ALIGN>(pb + lane_off<BLOCK>(u, tid));
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < U; ++u) res[r][u] = combine_vectors<T>(va[u], vb[u], scale);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const size_t tile = t0 + G * r;
            if (unsigned(r) < trips && tile < ntiles) {
                char* po = static_cast<char*>(out) + tile * (kTileVecs * 16);
#pragma unroll
                for (int u = 0; u < U; ++u) store_vec<ALIGN>(po + lane_off<BLOCK>(u, tid), res[r][u]);
            }
        }
    }

    if (blockIdx.x == G - 1) {
        for (size_t idx = ntiles * kTileVecs + tid; idx < nvec; idx += BLOCK) {
            const u32x4 wa = load_vec<ALIGN>(static_cast<const char*>(a) + idx * 16);
            const u32x4 wb = load_vec<ALIGN>(static_cast<const char*>(b) + idx * 16);
            store_vec<ALIGN>(static_cast<char*>(out) + idx * 16, combine_vectors<T>(wa, wb, scale));
        }
    }
    const size_t tail0 = nvec * kVec;
    if (blockIdx.x == 0 && tail0 + tid < n) {
        typedef typename T::elem_t E;
        const size_t i = tail0 + tid;
        const float t = T::widen1(static_cast<const E*>(a)[i]) + T::widen1(static_cast<const E*>(b)[i]);
        static_cast<E*>(out)[i] = T::narrow1(t * scale);
    }
}


// ---------------------------------------------------------------------------
// Batched K-way sum: many small buckets in ONE launch. The descriptor table
// (K + 1 pointers, the element count and the first tile index per bucket)
// travels in the kernel-argument segment, so nothing is allocated or copied on
// the device. A workgroup finds its bucket from the table's tile prefix
// (lanes compare in parallel) and then handles one tile (256 * U vectors) of it;
// the workgroup that owns a bucket's last tile also does its scalar tail.
// This removes the per-launch host cost (a few microseconds) that dominates
// when buckets or chunks are small.
// ---------------------------------------------------------------------------
template <int K>
struct BatchEntry {
    const void* in[K];
    void* out;
    size_t n;             // elements
    unsigned tile_begin;  // first tile of this bucket in the launch
    unsigned tile_count;  // >= 1 (a bucket shorter than one vector still owns a tile for its tail)
};

// As many entries as fit a 4 KiB kernel-argument segment with room to spare.
template <int K>
constexpr int batch_capacity() {
    return int((3840 - 16) / sizeof(BatchEntry<K>));
}

template <int K>
struct BatchTable {
    BatchEntry<K> e[batch_capacity<K>()];
    int count;
};

template <typename T, int K, int U, int BLOCK, int ALIGN>
__global__ __launch_bounds__(BLOCK) void reduce_sum_batched_kernel(BatchTable<K> tab) {
    constexpr int kVec = T::kVec;
    const unsigned tile = blockIdx.x;
    const unsigned tid = threadIdx.x;
    // Entries are sorted by tile_begin and entry 0 starts at tile 0: the bucket
    // is (number of entries with tile_begin <= tile) - 1. Every wave counts them
    // with its lanes in parallel (one entry per lane, one or two passes) instead
    // of walking the table with dependent scalar loads.
    const unsigned lane = tid & 63u;
    unsigned le_count = 0;
    for (int first = 0; first < tab.count; first += 64) {
        const int i = first + int(lane);
        const bool le = i < tab.count && tab.e[i].tile_begin <= tile;
        le_count += unsigned(__popcll(__ballot(le)));
    }
    const int b = __builtin_amdgcn_readfirstlane(int(le_count) - 1);
    PtrPack<K> in;
#pragma unroll
    for (int j = 0; j < K; ++j) in.p[j] = tab.e[b].in[j];
    void* out = tab.e[b].out;
    const size_t n = tab.e[b].n;
    const unsigned local = tile - tab.e[b].tile_begin;
    const size_t nvec = n / kVec;
    const size_t base = size_t(local) * BLOCK * U;
    if (base + size_t(BLOCK) * U <= nvec) {
        u32x4 v[U][K];
#pragma unroll
        for (int j = 0; j < K; ++j) {
            const char* pj = static_cast<const char*>(in.p[j]) + base * 16;
#pragma unroll
            for (int u = 0; u < U; ++u) v[u][j] = load_vec<ALIGN>(pj + lane_off<BLOCK>(u, tid));
        }
        __builtin_amdgcn_sched_barrier(0);
        char* po = static_cast<char*>(out) + base * 16;
#pragma unroll
        for (int u = 0; u < U; ++u)
            store_vec<ALIGN>(po + lane_off<BLOCK>(u, tid), sum_vectors<T, K, kEpiNone>(v[u], 1.0f));
    } else {
#pragma unroll 1
        for (int u = 0; u < U; ++u) {
            const size_t idx = base + size_t(u) * BLOCK + tid;
            if (idx < nvec) {
                u32x4 w[K];
#pragma unroll
                for (int j = 0; j < K; ++j) w[j] = load_vec<ALIGN>(static_cast<const char*>(in.p[j]) + idx * 16);
                store_vec<ALIGN>(static_cast<char*>(out) + idx * 16, sum_vectors<T, K, kEpiNone>(w, 1.0f));
            }
        }
    }
    const size_t tail0 = nvec * kVec;
    if (local + 1 == tab.e[b].tile_count && tail0 + tid < n) sum_scalar<T, K, kEpiNone>(in, out, tail0 + tid, 1.0f);
}


// ---------------------------------------------------------------------------
// Chunk table in device memory: the same K-way sum for a list of chunks whose
// descriptors the host never reads - one launch whatever the number of chunks,
// and the table may be written by a producer on the GPU. blockIdx.y walks the
// table, blockIdx.x the tiles of a chunk (both with a stride loop, so neither
// the table length nor a chunk's length is bounded by the grid). Alignment is
// decided per chunk on the device: all K + 1 pointers 16-byte aligned selects
// the vector path with natural alignment, anything else the element-aligned one.
// ---------------------------------------------------------------------------
struct ChunkDesc {            // layout of hfr_chunk
    const void* in[16];
    void* out;
    size_t n;
};

template <typename T, int K, int U, int BLOCK, int ALIGN>
__device__ __forceinline__ void sum_chunk_tiles(const PtrPack<K>& in, void* out, size_t n, unsigned tid) {
    constexpr int kVec = T::kVec;
    constexpr size_t kTileVecs = size_t(BLOCK) * U;
    const size_t nvec = n / kVec;
    size_t ntiles = (nvec + kTileVecs - 1) / kTileVecs;
    if (ntiles == 0) ntiles = 1;  // a chunk shorter than one vector still has a tail
    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const size_t base = tile * kTileVecs;
        if (base + kTileVecs <= nvec) {
            u32x4 v[U][K];
#pragma unroll
            for (int j = 0; j < K; ++j) {
                const char* pj = static_cast<const char*>(in.p[j]) + base * 16;
#pragma unroll
                for (int u = 0; u < U; ++u) v[u][j] = load_vec<ALIGN>(pj + lane_off<BLOCK>(u, tid));
            }
            __builtin_amdgcn_sched_barrier(0);
            char* po = static_cast<char*>(out) + base * 16;
#pragma unroll
            for (int u = 0; u < U; ++u)
                store_vec<ALIGN>(po + lane_off<BLOCK>(u, tid), sum_vectors<T, K, kEpiNone>(v[u], 1.0f));
        } else {
#pragma unroll 1
            for (int u = 0; u < U; ++u) {
                const size_t idx = base + size_t(u) * BLOCK + tid;
                if (idx < nvec) {
                    u32x4 w[K];
#pragma unroll
                    for (int j = 0; j < K; ++j) w[j] = load_vec<ALIGN>(static_cast<const char*>(in.p[j]) + idx * 16);
                    store_vec<ALIGN>(static_cast<char*>(out) + idx * 16, sum_vectors<T, K, kEpiNone>(w, 1.0f));
                }
            }
        }
        const size_t tail0 = nvec * kVec;
        if (tile + 1 == ntiles && tail0 + tid < n) sum_scalar<T, K, kEpiNone>(in, out, tail0 + tid, 1.0f);
    }
}

template <typename T, int K, int U, int BLOCK, int ELEM_ALIGN>
__global__ __launch_bounds__(BLOCK) void reduce_sum_table_kernel(const ChunkDesc* __restrict__ table,
                                                                 unsigned n_chunks) {
    const unsigned tid = threadIdx.x;
    for (unsigned c = blockIdx.y; c < n_chunks; c += gridDim.y) {
        const ChunkDesc* d = table + c;  // the same address in every lane: scalar loads
        const size_t n = d->n;
        if (n == 0) continue;
        PtrPack<K> in;
        void* out = d->out;
        uintptr_t bits = reinterpret_cast<uintptr_t>(out);
#pragma unroll
        for (int j = 0; j < K; ++j) {
            in.p[j] = d->in[j];
            bits |= reinterpret_cast<uintptr_t>(in.p[j]);
        }
        if ((bits & 15) == 0)
            sum_chunk_tiles<T, K, U, BLOCK, 16>(in, out, n, tid);
        else
            sum_chunk_tiles<T, K, U, BLOCK, ELEM_ALIGN>(in, out, n, tid);
    }
}

// ---------------------------------------------------------------------------
// Broadcast (Algorithm 2, pass 2: the reduced chunk is copied to every GPU of
// the node): one read of src, K writes. Type-agnostic: bytes are moved as
// 16-byte vectors plus a tail of single bytes. One read instead of the K reads of K separate copies.
// ---------------------------------------------------------------------------
template <int K>
struct DstPack {
    void* p[K];
};

template <int K, int U, int BLOCK, int ALIGN>
__global__ __launch_bounds__(BLOCK) void broadcast_kernel(const void* src, DstPack<K> dst, size_t nbytes) {
    constexpr size_t kTileVecs = size_t(BLOCK) * U;
    const size_t nvec = nbytes / 16;
    const size_t ntiles = (nvec + kTileVecs - 1) / kTileVecs;
    const unsigned tid = threadIdx.x;
    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const size_t base = tile * kTileVecs;
        if (base + kTileVecs <= nvec) {
            u32x4 v[U];
            const char* ps = static_cast<const char*>(src) + base * 16;
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = load_vec<ALIGN>(ps + lane_off<BLOCK>(u, tid));
#pragma unroll
            for (int j = 0; j < K; ++j) {
                char* pd = static_cast<char*>(dst.p[j]) + base * 16;
#pragma unroll
                for (int u = 0; u < U; ++u) store_vec<ALIGN>(pd + lane_off<BLOCK>(u, tid), v[u]);
            }
        } else {
#pragma unroll 1
            for (int u = 0; u < U; ++u) {
                const size_t idx = base + size_t(u) * BLOCK + tid;
                if (idx < nvec) {
                    const u32x4 w = load_vec<ALIGN>(static_cast<const char*>(src) + idx * 16);
#pragma unroll
                    for (int j = 0; j < K; ++j) store_vec<ALIGN>(static_cast<char*>(dst.p[j]) + idx * 16, w);
                }
            }
        }
    }
    // tail: fewer than sixteen bytes
    const size_t tail0 = nvec * 16;
    if (blockIdx.x == 0 && tail0 + tid < nbytes) {
        const uint8_t x = static_cast<const uint8_t*>(src)[tail0 + tid];
#pragma unroll
        for (int j = 0; j < K; ++j) static_cast<uint8_t*>(dst.p[j])[tail0 + tid] = x;
    }
}

// Bulk shape of the broadcast, launched with one workgroup per compute unit:
// a workgroup reads `trips` <= R tiles into registers (tiles b, b + G, ... in
// lock step with the other workgroups) and then writes them to one
// destination after the other, so that at any moment the whole chip writes a
// narrow window of ONE destination instead of K windows at once (measured on
// 128 MiB buffers: 5.2 to 5.4 TB/s against 4.8 to 5.0 for K >= 3). Whole tiles
// only here; the last workgroup moves the remaining vectors and workgroup 0
// the byte tail. 16-byte aligned buffers.
template <int K, int R, int BLOCK>
__global__ __launch_bounds__(BLOCK) void broadcast_bulk_kernel(const void* src, DstPack<K> dst, size_t nbytes,
                                                               unsigned trips) {
    constexpr size_t kTileBytes = size_t(BLOCK) * 16;
    const size_t nvec = nbytes / 16;
    const size_t ntiles = nvec / BLOCK;  // whole tiles
    const unsigned tid = threadIdx.x;
    const size_t G = gridDim.x;
    trips = trips < 1u ? 1u : (trips > unsigned(R) ? unsigned(R) : trips);  // the loop below must advance
    for (size_t t0 = blockIdx.x; t0 < ntiles; t0 += G * trips) {
        u32x4 v[R];
        // one bound for "this burst's trips" and "whole tiles": tile t0 + G * r belongs to the burst
        // exactly when it lies below t0 + G * trips
        const size_t burst_end = t0 + G * trips < ntiles ? t0 + G * trips : ntiles;
        static_for<0, R>([&](auto rc) {
            constexpr int r = decltype(rc)::value;
            const size_t tile = t0 + G * r;
            if (tile < burst_end)
                v[r] = load_vec<16>(static_cast<const char*>(src) + tile * kTileBytes + lane_off<BLOCK>(0, tid));
        });
        __builtin_amdgcn_sched_barrier(0);
        // Every load of the burst has landed before the first store (s_waitcnt vmcnt(0)). Without
        // this the compiler, which cannot match a load's condition with that of the stores that
        // consume it, assumes loads may still be pending when the loop comes round and waits
        // before EVERY load of the next burst, one load in flight at a time.
        __builtin_amdgcn_s_waitcnt(0x0F70);
        static_for<0, K>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            static_for<0, R>([&](auto rc) {
                constexpr int r = decltype(rc)::value;
                const size_t tile = t0 + G * r;
                if (tile < burst_end)
                    store_vec<16>(static_cast<char*>(dst.p[j]) + tile * kTileBytes + lane_off<BLOCK>(0, tid), v[r]);
            });
            __builtin_amdgcn_sched_barrier(0);  // one destination after the other
        });
    }
    if (blockIdx.x == G - 1) {
        for (size_t idx = ntiles * BLOCK + tid; idx < nvec; idx += BLOCK) {
            const u32x4 w = load_vec<16>(static_cast<const char*>(src) + idx * 16);
#pragma unroll
            for (int j = 0; j < K; ++j) store_vec<16>(static_cast<char*>(dst.p[j]) + idx * 16, w);
        }
    }
    const size_t tail0 = nvec * 16;
    if (blockIdx.x == 0 && tail0 + tid < nbytes) {
        const uint8_t x = static_cast<const uint8_t*>(src)[tail0 + tid];
#pragma unroll
        for (int j = 0; j < K; ++j) static_cast<uint8_t*>(dst.p[j])[tail0 + tid] = x;
    }
}

}  // namespace hfr
