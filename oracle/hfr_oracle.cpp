// CPU oracle for the HFReduce reduction arithmetic.
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. Only the test-suite, the smoke
// check and the benchmark's cpu_baseline leg may call it. It shares no code,
// header, table or helper with the HIP library, and neither includes the other.
//
// What it computes follows the paper's two reduction statements:
//   * Algorithm 1 (intra-node reduce), inner loop over the GPUs of a node:
//     the node's chunk is the running sum of every GPU's copy of that chunk,
//     taken in GPU-index order.
//   * Algorithm 2 (inter-node reduce), pass 1: the local partial has the
//     partial received from the neighbouring node added to it.
//   * Section IV-D.1 lists the element types (FP32 / FP16 / BF16 / FP8);
//     all of them are covered here (fp8 as the two OCP formats E4M3 and E5M2).
// The paper never divides; the averaging factor of the combine step is a
// caller-supplied fp32 multiplier applied once, after the add.
//
// Readings taken where the paper is silent (kept deliberately simple so a
// reader can check them by eye):
//   * order      : ascending buffer index j = 0..K-1, accumulator starts from
//                  buffer 0 (no "0 +" in front);
//   * precision  : every add and the multiply are IEEE-754 binary32 operations,
//                  each rounded to nearest-even on its own (no fusing);
//                  16-bit elements are widened exactly, accumulated in binary32
//                  and rounded ONCE to the storage type when stored;
//   * no flush   : subnormals are honoured on input and output.
//
// Build: g++ -O2 -ffp-contract=off -fno-fast-math (x86-64 SSE2 scalar math,
// FLT_EVAL_METHOD == 0). Single-threaded, plain loops, no intrinsics.
//
// Pins (tests/test_oracle_pins.py): closed forms (K=1 identity, sums of
// constants, +x/-x cancellation to +0), an order discriminator, exact rational
// brute force on tiny inputs, an integer-arithmetic model of binary32 rounding,
// tie / carry / overflow tables for the bf16 narrowing, signed zeros and
// subnormals. No function here is unpinned.

#include <cstddef>
#include <cstdint>
#include <cstring>

namespace {

// binary32 <-> raw bits, without aliasing tricks.
inline float bits_to_f32(uint32_t u) {
    float f;
    std::memcpy(&f, &u, sizeof f);
    return f;
}
inline uint32_t f32_to_bits(float f) {
    uint32_t u;
    std::memcpy(&u, &f, sizeof u);
    return u;
}

// bfloat16 is the upper half of a binary32: widening appends sixteen zero bits
// and is exact for every pattern.
inline float widen_bf16(uint16_t h) { return bits_to_f32(static_cast<uint32_t>(h) << 16); }

// binary32 -> bfloat16, round to nearest, ties to the even kept bit.
// Written from the IEEE-754 definition of roundTiesToEven on the discarded
// sixteen bits; a carry out of the kept fraction correctly moves into the
// exponent (largest finite values become infinity).
inline uint16_t narrow_bf16(float f) {
    const uint32_t u = f32_to_bits(f);
    const uint32_t expo = (u >> 23) & 0xFFu;
    const uint32_t frac = u & 0x7FFFFFu;
    if (expo == 0xFFu && frac != 0u) {
        // NaN stays a NaN: keep the sign and top payload bits, force quiet bit.
        return static_cast<uint16_t>((u >> 16) | 0x0040u);
    }
    uint32_t kept = u >> 16;
    const uint32_t dropped = u & 0xFFFFu;
    if (dropped > 0x8000u) {
        kept += 1u;
    } else if (dropped == 0x8000u) {
        if (kept & 1u) kept += 1u;
    }
    return static_cast<uint16_t>(kept);
}

// IEEE binary16 (1 sign, 5 exponent, 10 fraction bits, bias 15) -> binary32,
// exact for every pattern: normal numbers are re-biased, subnormals are
// f * 2^-24 (normalised by shifting), infinities and NaNs keep their class.
inline float widen_f16(uint16_t h) {
    const uint32_t sign = static_cast<uint32_t>(h & 0x8000u) << 16;
    const uint32_t expo = (h >> 10) & 0x1Fu;
    uint32_t frac = h & 0x3FFu;
    if (expo == 0x1Fu) return bits_to_f32(sign | 0x7F800000u | (frac << 13));  // inf / NaN
    if (expo != 0u) return bits_to_f32(sign | ((expo + 112u) << 23) | (frac << 13));
    if (frac == 0u) return bits_to_f32(sign);                                  // +-0
    // subnormal: value = frac * 2^-24; shift the leading one up to bit 10
    uint32_t e = 113u;  // biased binary32 exponent of 2^-14
    while ((frac & 0x400u) == 0u) {
        frac <<= 1;
        --e;
    }
    return bits_to_f32(sign | (e << 23) | ((frac & 0x3FFu) << 13));
}

// binary32 -> binary16, round to nearest, ties to even, from the definition:
// the value is expressed in units of the target's quantum at its magnitude
// (2^(e-10) for normal results, 2^-24 in the subnormal range) and the
// discarded part is compared with half a quantum. Overflow gives infinity.
inline uint16_t narrow_f16(float f) {
    const uint32_t u = f32_to_bits(f);
    const uint16_t sign = static_cast<uint16_t>((u >> 16) & 0x8000u);
    const uint32_t expo = (u >> 23) & 0xFFu;
    const uint32_t frac = u & 0x7FFFFFu;
    if (expo == 0xFFu) {
        if (frac == 0u) return static_cast<uint16_t>(sign | 0x7C00u);                      // inf
        return static_cast<uint16_t>(sign | 0x7C00u | 0x0200u | (frac >> 13));             // quiet NaN
    }
    const int e = static_cast<int>(expo) - 127;  // unbiased (subnormal binary32 inputs are far below 2^-24)
    if (expo == 0u || e < -25) return sign;      // below half of the smallest subnormal: rounds to zero
    // 24-bit significand with the hidden one; result quantum is 2^(max(e,-14) - 10)
    const uint32_t sig = frac | 0x800000u;
    const int drop = (e >= -14) ? 13 : (13 + (-14 - e));  // low bits of sig that fall below the quantum
    uint32_t kept = sig >> drop;
    const uint32_t rest = sig & ((1u << drop) - 1u);
    const uint32_t half = 1u << (drop - 1);
    if (rest > half || (rest == half && (kept & 1u))) kept += 1u;
    if (e >= -14) {
        // kept is in [2^10, 2^11]; 2^11 means the carry moved to the next exponent
        uint32_t he = static_cast<uint32_t>(e + 15);
        if (kept == 0x800u) {
            kept = 0x400u;
            he += 1u;
        }
        if (he >= 0x1Fu) return static_cast<uint16_t>(sign | 0x7C00u);  // overflow
        return static_cast<uint16_t>(sign | (he << 10) | (kept & 0x3FFu));
    }
    // subnormal result: kept in [0, 2^10]; 2^10 is the smallest normal number
    return static_cast<uint16_t>(sign | kept);
}

// ---- 8-bit floating point (the OCP FP8 formats) ----------------------------
// E5M2: 1 sign, 5 exponent (bias 15), 2 fraction bits; IEEE-like: exponent 31
// is infinity / NaN. E4M3: 1 sign, 4 exponent (bias 7), 3 fraction bits; no
// infinity: exponent 15 holds ordinary numbers up to 448 and only S.1111.111
// is NaN. Both have subnormals. Widening is exact. Narrowing rounds to nearest,
// ties to even, on the discarded significand bits; what does not fit becomes
// infinity where the format has one (E5M2) and NaN where it has none (E4M3) -
// the reading "as IEEE as the format allows", no saturation.
template <int EB, int MB, int BIAS>
inline float widen_small(uint8_t b, bool ieee_like) {
    const uint32_t sign = static_cast<uint32_t>(b & 0x80u) << 24;
    const uint32_t expo = (b >> MB) & ((1u << EB) - 1u);
    uint32_t frac = b & ((1u << MB) - 1u);
    const uint32_t emax_field = (1u << EB) - 1u;
    if (ieee_like && expo == emax_field) {
        return bits_to_f32(sign | 0x7F800000u | (frac << (23 - MB)));  // inf (frac 0) or NaN
    }
    if (!ieee_like && expo == emax_field && frac == ((1u << MB) - 1u)) {
        return bits_to_f32(sign | 0x7FC00000u);                       // the single NaN pattern
    }
    if (expo != 0u) return bits_to_f32(sign | ((expo + 127u - BIAS) << 23) | (frac << (23 - MB)));
    if (frac == 0u) return bits_to_f32(sign);
    // subnormal: frac * 2^(1 - BIAS - MB); normalise
    uint32_t e = 127u + 1u - BIAS;  // biased binary32 exponent of 2^(1-BIAS)
    while ((frac & (1u << MB)) == 0u) {
        frac <<= 1;
        --e;
    }
    return bits_to_f32(sign | (e << 23) | ((frac & ((1u << MB) - 1u)) << (23 - MB)));
}

template <int EB, int MB, int BIAS>
inline uint8_t narrow_small(float f, bool ieee_like) {
    const uint32_t u = f32_to_bits(f);
    const uint8_t sign = static_cast<uint8_t>((u >> 24) & 0x80u);
    const uint32_t expo = (u >> 23) & 0xFFu;
    const uint32_t frac = u & 0x7FFFFFu;
    const uint8_t emax_field = static_cast<uint8_t>((1u << EB) - 1u);
    const uint8_t nan_pattern = ieee_like ? static_cast<uint8_t>((emax_field << MB) | (1u << (MB - 1)))
                                          : static_cast<uint8_t>((emax_field << MB) | ((1u << MB) - 1u));
    const uint8_t inf_or_nan = ieee_like ? static_cast<uint8_t>(emax_field << MB) : nan_pattern;
    if (expo == 0xFFu) return static_cast<uint8_t>(sign | (frac == 0u ? inf_or_nan : nan_pattern));
    const int emin = 1 - BIAS;                    // exponent of the smallest normal number
    const int e = static_cast<int>(expo) - 127;
    if (expo == 0u || e < emin - MB - 1) return sign;   // below half of the smallest subnormal
    const uint32_t sig = frac | 0x800000u;
    const int drop = (e >= emin) ? (23 - MB) : (23 - MB + (emin - e));
    uint32_t kept = sig >> drop;
    const uint32_t rest = sig & ((1u << drop) - 1u);
    const uint32_t half = 1u << (drop - 1);
    if (rest > half || (rest == half && (kept & 1u))) kept += 1u;
    uint32_t enc;
    if (e >= emin) {
        uint32_t field = static_cast<uint32_t>(e + BIAS);
        if (kept == (2u << MB)) {   // carry into the next binade
            kept = 1u << MB;
            field += 1u;
        }
        if (field > emax_field) return static_cast<uint8_t>(sign | inf_or_nan);
        enc = (field << MB) | (kept & ((1u << MB) - 1u));
    } else {
        enc = kept;                  // subnormal, or exactly the smallest normal
    }
    if (ieee_like) {
        if (enc >= (static_cast<uint32_t>(emax_field) << MB)) return static_cast<uint8_t>(sign | inf_or_nan);
    } else {
        if (enc >= nan_pattern) return static_cast<uint8_t>(sign | nan_pattern);  // beyond 448
    }
    return static_cast<uint8_t>(sign | enc);
}

inline float widen_e4m3(uint8_t b) { return widen_small<4, 3, 7>(b, false); }
inline uint8_t narrow_e4m3(float f) { return narrow_small<4, 3, 7>(f, false); }
inline float widen_e5m2(uint8_t b) { return widen_small<5, 2, 15>(b, true); }
inline uint8_t narrow_e5m2(float f) { return narrow_small<5, 2, 15>(f, true); }

// One element of Algorithm 1's inner loop: acc starts as buffer 0's value and
// receives buffers 1..K-1 in index order, each add rounded to binary32.
template <typename Load>
inline float sum_in_order(int K, Load load) {
    float acc = load(0);
    for (int j = 1; j < K; ++j) {
        acc = acc + load(j);  // one binary32 add, rounded on its own
    }
    return acc;
}

}  // namespace

extern "C" {

// dtype codes of the oracle's own interface (they happen to be small integers;
// the test harness maps names to them).
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2, ORACLE_FP8_E4M3 = 3, ORACLE_FP8_E5M2 = 4 };

static size_t elem_size_of(int dtype) {
    switch (dtype) {
        case ORACLE_F32: return 4;
        case ORACLE_BF16: case ORACLE_F16: return 2;
        case ORACLE_FP8_E4M3: case ORACLE_FP8_E5M2: return 1;
        default: return 0;
    }
}

// Algorithm 1, inner loop, for one chunk of n elements.
// in: K host pointers, each to n elements of the given type. out: n elements.
// out may be identical to any in[j] (the paper's form is in place).
// Returns 0, or -1 on a bad argument.
int oracle_reduce_sum(const void* const* in, int K, void* out, size_t n, int dtype) {
    if (K < 1 || (n > 0 && (in == nullptr || out == nullptr))) return -1;
    if (dtype == ORACLE_F32) {
        float* o = static_cast<float*>(out);
        for (size_t i = 0; i < n; ++i) {
            o[i] = sum_in_order(K, [&](int j) { return static_cast<const float*>(in[j])[i]; });
        }
        return 0;
    }
    if (dtype == ORACLE_BF16) {
        uint16_t* o = static_cast<uint16_t*>(out);
        for (size_t i = 0; i < n; ++i) {
            const float acc = sum_in_order(
                K, [&](int j) { return widen_bf16(static_cast<const uint16_t*>(in[j])[i]); });
            o[i] = narrow_bf16(acc);
        }
        return 0;
    }
    if (dtype == ORACLE_F16) {
        uint16_t* o = static_cast<uint16_t*>(out);
        for (size_t i = 0; i < n; ++i) {
            const float acc = sum_in_order(
                K, [&](int j) { return widen_f16(static_cast<const uint16_t*>(in[j])[i]); });
            o[i] = narrow_f16(acc);
        }
        return 0;
    }
    if (dtype == ORACLE_FP8_E4M3 || dtype == ORACLE_FP8_E5M2) {
        const bool e4 = dtype == ORACLE_FP8_E4M3;
        uint8_t* o = static_cast<uint8_t*>(out);
        for (size_t i = 0; i < n; ++i) {
            const float acc = sum_in_order(K, [&](int j) {
                const uint8_t b = static_cast<const uint8_t*>(in[j])[i];
                return e4 ? widen_e4m3(b) : widen_e5m2(b);
            });
            o[i] = e4 ? narrow_e4m3(acc) : narrow_e5m2(acc);
        }
        return 0;
    }
    return -1;
}

// Algorithm 2, pass 1 ("local += received"), followed by the averaging
// multiply: out = fl( fl(a + b) * scale ), both operations in binary32.
// out may be identical to a or b.
int oracle_combine_avg(const void* a, const void* b, void* out, size_t n, float scale, int dtype) {
    if (n > 0 && (a == nullptr || b == nullptr || out == nullptr)) return -1;
    if (dtype == ORACLE_F32) {
        const float* x = static_cast<const float*>(a);
        const float* y = static_cast<const float*>(b);
        float* o = static_cast<float*>(out);
        for (size_t i = 0; i < n; ++i) {
            const float t = x[i] + y[i];  // first rounding
            o[i] = t * scale;             // second rounding
        }
        return 0;
    }
    if (dtype == ORACLE_BF16) {
        const uint16_t* x = static_cast<const uint16_t*>(a);
        const uint16_t* y = static_cast<const uint16_t*>(b);
        uint16_t* o = static_cast<uint16_t*>(out);
        for (size_t i = 0; i < n; ++i) {
            const float t = widen_bf16(x[i]) + widen_bf16(y[i]);  // first rounding
            const float u = t * scale;                            // second rounding
            o[i] = narrow_bf16(u);                                // third, to storage
        }
        return 0;
    }
    if (dtype == ORACLE_F16) {
        const uint16_t* x = static_cast<const uint16_t*>(a);
        const uint16_t* y = static_cast<const uint16_t*>(b);
        uint16_t* o = static_cast<uint16_t*>(out);
        for (size_t i = 0; i < n; ++i) {
            const float t = widen_f16(x[i]) + widen_f16(y[i]);
            const float u = t * scale;
            o[i] = narrow_f16(u);
        }
        return 0;
    }
    if (dtype == ORACLE_FP8_E4M3 || dtype == ORACLE_FP8_E5M2) {
        const bool e4 = dtype == ORACLE_FP8_E4M3;
        const uint8_t* x = static_cast<const uint8_t*>(a);
        const uint8_t* y = static_cast<const uint8_t*>(b);
        uint8_t* o = static_cast<uint8_t*>(out);
        for (size_t i = 0; i < n; ++i) {
            const float t = (e4 ? widen_e4m3(x[i]) : widen_e5m2(x[i])) + (e4 ? widen_e4m3(y[i]) : widen_e5m2(y[i]));
            const float u = t * scale;
            o[i] = e4 ? narrow_e4m3(u) : narrow_e5m2(u);
        }
        return 0;
    }
    return -1;
}

// Algorithm 1's chunk loop over a list of gradient buckets: each bucket is
// reduced on its own; how a bucket is cut into chunks cannot change a result
// that is defined element by element, so no chunk size appears here.
// in_table holds n_buckets * K pointers (bucket-major), out_table and n_table
// one entry per bucket.
int oracle_reduce_buckets(const void* const* in_table, void* const* out_table, const size_t* n_table,
                          size_t n_buckets, int K, int dtype) {
    for (size_t b = 0; b < n_buckets; ++b) {
        const int rc = oracle_reduce_sum(in_table + b * static_cast<size_t>(K), K, out_table[b],
                                         n_table[b], dtype);
        if (rc != 0) return rc;
    }
    return 0;
}

// K-way sum with the averaging factor folded in, for an allreduce that has no
// inter-node stage (one node: Algorithm 1 alone, then the data-parallel mean):
// out = narrow( fl( sum_in_order * scale ) ). The sum is not rounded to the
// storage type before the multiply.
int oracle_reduce_avg(const void* const* in, int K, void* out, size_t n, float scale, int dtype) {
    if (K < 1 || (n > 0 && (in == nullptr || out == nullptr))) return -1;
    if (dtype == ORACLE_F32) {
        float* o = static_cast<float*>(out);
        for (size_t i = 0; i < n; ++i) {
            const float acc = sum_in_order(K, [&](int j) { return static_cast<const float*>(in[j])[i]; });
            o[i] = acc * scale;
        }
        return 0;
    }
    if (dtype == ORACLE_BF16) {
        uint16_t* o = static_cast<uint16_t*>(out);
        for (size_t i = 0; i < n; ++i) {
            const float acc = sum_in_order(
                K, [&](int j) { return widen_bf16(static_cast<const uint16_t*>(in[j])[i]); });
            const float avg = acc * scale;
            o[i] = narrow_bf16(avg);
        }
        return 0;
    }
    if (dtype == ORACLE_F16) {
        uint16_t* o = static_cast<uint16_t*>(out);
        for (size_t i = 0; i < n; ++i) {
            const float acc = sum_in_order(
                K, [&](int j) { return widen_f16(static_cast<const uint16_t*>(in[j])[i]); });
            const float avg = acc * scale;
            o[i] = narrow_f16(avg);
        }
        return 0;
    }
    if (dtype == ORACLE_FP8_E4M3 || dtype == ORACLE_FP8_E5M2) {
        const bool e4 = dtype == ORACLE_FP8_E4M3;
        uint8_t* o = static_cast<uint8_t*>(out);
        for (size_t i = 0; i < n; ++i) {
            const float acc = sum_in_order(K, [&](int j) {
                const uint8_t b = static_cast<const uint8_t*>(in[j])[i];
                return e4 ? widen_e4m3(b) : widen_e5m2(b);
            });
            const float avg = acc * scale;
            o[i] = e4 ? narrow_e4m3(avg) : narrow_e5m2(avg);
        }
        return 0;
    }
    return -1;
}

// Slice `rank` of `world` nearly equal contiguous slices of [0, n): the first
// n % world slices hold one element more. (The paper's NVLink variant, Section
// IV-C, has each GPU of a pair reduce and keep its own part of the data.)
void oracle_slice_bounds(size_t n, int rank, int world, size_t* begin, size_t* end) {
    const size_t w = static_cast<size_t>(world), r = static_cast<size_t>(rank);
    const size_t q = n / w, m = n % w;
    *begin = r * q + (r < m ? r : m);
    *end = *begin + q + (r < m ? 1 : 0);
}

// Reduce only slice `rank`: out[i] for i inside the slice gets the in-order
// K-way sum; elements of out outside the slice are not touched.
int oracle_reduce_scatter_slice(const void* const* in, int K, void* out, size_t n, int rank, int world,
                                int dtype) {
    if (world < 1 || rank < 0 || rank >= world) return -1;
    if (K < 1 || (n > 0 && (in == nullptr || out == nullptr))) return -1;
    size_t b = 0, e = 0;
    oracle_slice_bounds(n, rank, world, &b, &e);
    const size_t es = elem_size_of(dtype);
    if (es == 0) return -1;
    const void* shifted[64];
    if (K > 64) return -1;
    for (int j = 0; j < K; ++j) shifted[j] = static_cast<const char*>(in[j]) + b * es;
    return oracle_reduce_sum(shifted, K, static_cast<char*>(out) + b * es, e - b, dtype);
}

// Algorithm 2, pass 2: the reduced data is copied to every GPU of the node.
// dst: K host pointers to n elements each; every one receives an exact copy
// of src.
int oracle_broadcast(const void* src, void* const* dst, int K, size_t n, int dtype) {
    if (K < 1 || (n > 0 && (src == nullptr || dst == nullptr))) return -1;
    const size_t es = elem_size_of(dtype);
    if (es == 0) return -1;
    const unsigned char* s = static_cast<const unsigned char*>(src);
    for (int j = 0; j < K; ++j) {
        unsigned char* d = static_cast<unsigned char*>(dst[j]);
        for (size_t i = 0; i < n * es; ++i) d[i] = s[i];
    }
    return 0;
}

// Test hooks: the two type conversions on their own, so that the pins can
// check them over whole bit-pattern ranges.
void oracle_narrow_bf16(const float* in, uint16_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = narrow_bf16(in[i]);
}
void oracle_widen_bf16(const uint16_t* in, float* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = widen_bf16(in[i]);
}
void oracle_narrow_fp8(const float* in, uint8_t* out, size_t n, int dtype) {
    for (size_t i = 0; i < n; ++i) out[i] = dtype == ORACLE_FP8_E4M3 ? narrow_e4m3(in[i]) : narrow_e5m2(in[i]);
}
void oracle_widen_fp8(const uint8_t* in, float* out, size_t n, int dtype) {
    for (size_t i = 0; i < n; ++i) out[i] = dtype == ORACLE_FP8_E4M3 ? widen_e4m3(in[i]) : widen_e5m2(in[i]);
}
void oracle_narrow_f16(const float* in, uint16_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = narrow_f16(in[i]);
}
void oracle_widen_f16(const uint16_t* in, float* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = widen_f16(in[i]);
}

}  // extern "C"
