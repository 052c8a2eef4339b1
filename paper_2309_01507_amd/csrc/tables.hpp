// Host-side construction of the quantization maps and of the lookup tables the kernels keep in LDS.
//
// Maps (paper App. D.2, Sec. 4.1):
//   signed 4-bit dynamic-exponent map: 1 sign bit, E leading zeros, 1 indicator bit, F fraction
//   bits, value 10^-E * (bin midpoint of an even partition of [0.1, 1] into 2^F bins); the bit
//   patterns +000 and -000 stand for 0 and +1 (so -1 does not exist); the code is the rank in the
//   increasingly sorted list.  Linear map: (i+1)/16.
//
// Nearest-entry search M(n) = argmin_i |n - T(i)| (Sec. 2.2), lowest index on a tie, is done in
// the kernels as   code = #{k : n > thr_k},  thr_k = largest float <= (T(k)+T(k+1))/2,
// which is the same function of a float n.  To avoid 15 compares per element the float line is cut
// into buckets by the top 11 bits of n (sign, exponent, two mantissa bits); every bucket holds at
// most one threshold, so   code = base[bucket] + (n > thr[bucket]).
#pragma once

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>

namespace lpmm {

constexpr int kCodes = 16;
constexpr int kBucketBits = 11;
constexpr int kBuckets = 1 << kBucketBits;   // 2048
constexpr int kBucketShift = 32 - kBucketBits;

// Buckets without a threshold compare against a value no normalized input reaches (|n| <= 1 up to
// rounding); it is finite so that distance arithmetic on it stays finite.
constexpr float kNoThreshold = 8.0f;

struct SearchEntry {
    float thr;       // the one decision threshold inside this bucket, kNoThreshold if none
    uint32_t base;   // number of thresholds below the bucket
};

inline uint32_t f2u(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float u2f(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

// ---- the two maps -------------------------------------------------------------------------------

inline void build_de_signed(float T[kCodes]) {
    // magnitudes by (E, F): (0,2) four entries, (1,1) two, (2,0) one
    double mag[7];
    int n = 0;
    for (int E = 2; E >= 0; --E) {
        const int F = 2 - E;
        const int bins = 1 << F;
        const double width = 0.9 / bins;
        for (int k = 0; k < bins; ++k) {
            const double mid = 0.1 + width * (k + 0.5);
            mag[n++] = mid * std::pow(10.0, -E);
        }
    }
    // mag is increasing: 0.0055, 0.0325, 0.0775, 0.2125, 0.4375, 0.6625, 0.8875
    for (int i = 0; i < 7; ++i) {
        T[6 - i] = float(-mag[i]);
        T[8 + i] = float(mag[i]);
    }
    T[7] = 0.0f;
    T[15] = 1.0f;   // the -000 pattern
}

inline void build_linear(float T[kCodes]) {
    for (int i = 0; i < kCodes; ++i) T[i] = float(i + 1) * 0.0625f;
}

// thr[k], k = 0..14: largest float not above the exact midpoint of T[k] and T[k+1].
inline void build_thresholds(const float T[kCodes], float thr[kCodes - 1]) {
    for (int k = 0; k + 1 < kCodes; ++k) {
        const double mid = (double(T[k]) + double(T[k + 1])) * 0.5;   // exact in double
        float f = float(mid);
        if (double(f) > mid) f = std::nextafterf(f, -std::numeric_limits<float>::infinity());
        thr[k] = f;
    }
}

// Bucket table over all float bit patterns.  Returns false if some bucket would need two
// thresholds (then the bucket width is too coarse for this map).
inline bool build_search(const float thr[kCodes - 1], SearchEntry tab[kBuckets]) {
    const float inf = std::numeric_limits<float>::infinity();
    for (int b = 0; b < kBuckets; ++b) {
        const uint32_t lo_bits = uint32_t(b) << kBucketShift;
        const uint32_t hi_bits = lo_bits | ((1u << kBucketShift) - 1u);
        const bool neg = (b >> (kBucketBits - 1)) != 0;
        const int expo = (b >> 2) & 0xFF;
        SearchEntry e{kNoThreshold, 0};
        if (expo == 0xFF) {           // inf / NaN patterns: behave like the brute-force argmin -> code 0
            e.thr = inf;
            tab[b] = e;
            continue;
        }
        // value interval [a, z] covered by the bucket (bit patterns grow away from zero)
        const float a = neg ? u2f(hi_bits) : u2f(lo_bits);
        const float z = neg ? u2f(lo_bits) : u2f(hi_bits);
        int own = 0;
        for (int k = 0; k + 1 < kCodes; ++k) {
            if (thr[k] < a) e.base++;
            else if (thr[k] <= z) { e.thr = thr[k]; own++; }
        }
        if (own > 1) return false;
        tab[b] = e;
    }
    return true;
}

inline int search_code(const SearchEntry tab[kBuckets], float n) {
    const SearchEntry& e = tab[f2u(n) >> kBucketShift];
    return int(e.base) + (n > e.thr ? 1 : 0);
}

// Byte-indexed decode table for the first moment: entry b = {T[b & 15], T[b >> 4]}.
inline void build_byte_decode(const float T[kCodes], float tab[512]) {
    for (int b = 0; b < 256; ++b) {
        tab[2 * b] = T[b & 15];
        tab[2 * b + 1] = T[b >> 4];
    }
}

}  // namespace lpmm
