// Device-side random draws: worker delays (Sec. 3.1: one i.i.d. delay per worker
// and mini-batch) and mini-batch sample ids (Sec. 1.1: randomly chosen subsets).
//
// Every draw is a pure function of (seed, stream, aux, replica, worker, ordinal,
// version) through Philox4x32-10 (Salmon et al., SC'11), so kernels may evaluate
// them in any order.  The delay is an fp32 value defined by a fixed sequence of
// correctly rounded single-precision operations, which makes it reproducible bit for
// bit by any IEEE-754 implementation; every function that takes part switches
// floating-point contraction off, because the compiler would otherwise fuse the
// multiply-add pairs (the __fmul_rn / __fadd_rn wrappers do not prevent that).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssgd {

enum Stream : uint32_t { kDelay = 1, kBatch = 2, kInit = 3, kMonteCarlo = 4 };

struct Dist {
    int32_t kind;   // 0 exp, 1 shifted exp, 2 pareto, 3 table
    float shift, rate, alpha, scale;
    const float* table;  // device copy
    int64_t table_len;
};

struct u32x4 { uint32_t x, y, z, w; };

__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
    constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
        const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return {c0, c1, c2, c3};
}

__device__ __forceinline__ u32x4 draw(uint64_t seed, uint32_t stream, uint32_t aux, uint32_t replica,
                                      uint32_t worker, uint32_t ordinal, uint32_t version) {
    return philox4x32_10(version, (worker & 0xFFFFu) | (ordinal << 16), replica, (stream & 0xFFu) | (aux << 8),
                         (uint32_t)seed, (uint32_t)(seed >> 32));
}

// (top 23 bits + 1/2) / 2^23: strictly inside (0, 1), all steps exact.
__device__ __forceinline__ float uniform_open(uint32_t bits) {
#pragma clang fp contract(off)
    const float h = (float)(bits >> 9) + 0.5f;
    return h * 0x1p-23f;
}

// -ln(u), u a normal float in (0,1): ln m = 2 atanh((m-1)/(m+1)) on m in (sqrt(1/2), sqrt(2)],
// odd series to the 9th power, plus e*ln2 with ln2 in a short high and a low part.
__device__ __forceinline__ float neg_log(float u) {
#pragma clang fp contract(off)
    const uint32_t b = __float_as_uint(u);
    int e = (int)(b >> 23) - 127;
    float m = __uint_as_float((b & 0x007FFFFFu) | 0x3F800000u);
    if (m > 1.41421354f) { m = m * 0.5f; e += 1; }
    const float num = m - 1.0f, den = m + 1.0f;
    const float s = num / den;
    const float s2 = s * s;
    float p = 0.222222224f;
    p = p * s2; p = p + 0.285714298f;
    p = p * s2; p = p + 0.400000006f;
    p = p * s2; p = p + 0.666666687f;
    p = p * s2; p = p + 2.0f;
    const float r = p * s;
    const float ef = (float)e;
    const float hi = ef * 0.693359375f;
    const float lo = ef * -2.12194440e-4f;
    const float t = r + lo;
    const float ln = hi + t;
    return -ln;
}

// exp(y), y >= 0: y = n ln2 + r, degree-7 Taylor polynomial, scale through the exponent field.
__device__ __forceinline__ float exp_nonneg(float y) {
#pragma clang fp contract(off)
    const float t = y * 1.44269502f;
    const float th = t + 0.5f;
    if (!(th < 128.0f)) return __uint_as_float(0x7F800000u);
    const int n = (int)th;
    const float nf = (float)n;
    const float a = nf * 0.693359375f;
    float r = y - a;
    const float c = nf * -2.12194440e-4f;
    r = r - c;
    float p = 1.98412701e-4f;
    p = p * r; p = p + 1.38888892e-3f;
    p = p * r; p = p + 8.33333377e-3f;
    p = p * r; p = p + 4.16666679e-2f;
    p = p * r; p = p + 0.166666672f;
    p = p * r; p = p + 0.5f;
    p = p * r; p = p + 1.0f;
    p = p * r; p = p + 1.0f;
    return p * __uint_as_float((uint32_t)(n + 127) << 23);
}

__device__ __forceinline__ float delay_from_bits(const Dist& d, uint32_t bits) {
#pragma clang fp contract(off)
    const float E = neg_log(uniform_open(bits));
    if (d.kind == 0) return E / d.rate;
    if (d.kind == 1) { const float q = E / d.rate; return d.shift + q; }
    const float q = E / d.alpha;
    const float x = exp_nonneg(q);
    return d.scale * x;
}

// Delay of the ordinal-th mini-batch that `worker` starts after reading `version`.
__device__ __forceinline__ float delay(const Dist& d, uint64_t seed, uint32_t stream, uint32_t aux,
                                       uint32_t replica, int P, int table_ord, uint32_t worker,
                                       uint32_t ordinal, uint32_t version) {
    if (d.kind == 3) {
        const int64_t idx = ((int64_t)version * P + worker) * table_ord + ordinal;
        return d.table[idx % d.table_len];
    }
    return delay_from_bits(d, draw(seed, stream, aux, replica, worker, ordinal, version).x);
}

// Sample id of slot `slot` of a mini-batch: uniform on [0, N) with replacement.
__device__ __forceinline__ uint32_t batch_index(uint64_t seed, uint32_t replica, uint32_t worker,
                                                uint32_t ordinal, uint32_t version, uint32_t slot, uint32_t N) {
    const u32x4 b = draw(seed, kBatch, slot >> 2, replica, worker, ordinal, version);
    const uint32_t w = (slot & 2u) ? ((slot & 1u) ? b.w : b.z) : ((slot & 1u) ? b.y : b.x);
    return __umulhi(w, N);
}

}  // namespace ssgd
