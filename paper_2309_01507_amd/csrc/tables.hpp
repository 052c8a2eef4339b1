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
// which is the same function of a float n.  To avoid 15 compares per element the interval [-1, 1]
// is cut into 513 buckets, bucket(n) = round-to-nearest-even(256 n) + 256, computed by one fused
// multiply-add with a constant whose unit in the last place is 1 (the rounding of that operation is
// the rounding to an integer, and the integer sits in the low bits of the result).  bucket() is a
// non-decreasing function of n and no bucket holds two thresholds, so
//   code = base[bucket] + (n > thr[bucket]).
#pragma once

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>

namespace lpmm {

constexpr int kCodes = 16;
constexpr int kBucketHalf = 256;                    // buckets per unit of n
constexpr int kBuckets = 2 * kBucketHalf + 1;       // 513: n = -1 ... +1
constexpr int kBucketsPadded = 520;                 // table length (multiple of 8 entries)
constexpr float kBucketScale = float(kBucketHalf);
constexpr float kBucketMagic = 12582912.0f;         // 1.5 * 2^23: floats in [2^23, 2^24) are the integers
constexpr uint32_t kBucketMagicBits = 0x4B400000u;  // its bit pattern

// Buckets without a threshold compare against a value no normalized input reaches (|n| <= 1 up to
// rounding); it is finite so that distance arithmetic on it stays finite.
constexpr float kNoThreshold = 8.0f;

struct SearchEntry {
    float thr;       // the one decision threshold inside this bucket, kNoThreshold if none
    uint32_t base;   // number of thresholds below the bucket
};

inline uint32_t f2u(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }

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

// Unsigned 4-bit dynamic-exponent map (App. D.2; used by the ablation quantizers of Sec. 4.1 / Tab. 1): no sign
// bit, so one more bit for the fraction in every decade: 8 bins with E = 0, 4 with E = 1, 2 with E = 2; the single
// bin of E = 3 is the bit pattern 0001, which the map assigns the value 1, and 0000 is 0.
inline void build_de_unsigned(float T[kCodes]) {
    int n = 0;
    T[n++] = 0.0f;
    for (int E = 2; E >= 0; --E) {
        const int bins = 1 << (3 - E);
        const double width = 0.9 / bins;
        for (int k = 0; k < bins; ++k) T[n++] = float((0.1 + width * (k + 0.5)) * std::pow(10.0, -E));
    }
    T[n++] = 1.0f;      // n == 16; increasing by construction
}

// thr[k], k = 0..n-2, for any increasing table of n entries (see build_thresholds)
inline void build_thresholds_n(const float* T, int n, float* thr) {
    for (int k = 0; k + 1 < n; ++k) {
        const double mid = (double(T[k]) + double(T[k + 1])) * 0.5;
        float f = float(mid);
        if (double(f) > mid) f = std::nextafterf(f, -std::numeric_limits<float>::infinity());
        thr[k] = f;
    }
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

// Bucket of a normalized value.  The kernels only ever look up |n| <= 1 + 2^-22 and skip the
// clamp; the host version clamps so that any finite n gets the code of the nearest end bucket.
inline int search_bucket(float n) {
    const float x = std::fmaf(n, kBucketScale, kBucketMagic);
    if (!(x >= kBucketMagic - kBucketScale)) return 0;
    if (x > kBucketMagic + kBucketScale) return kBuckets - 1;
    return int(f2u(x) - kBucketMagicBits) + kBucketHalf;
}

// Returns false if some bucket would need two thresholds (then the buckets are too coarse for this
// map) or a threshold lies outside [-1, 1].
inline bool build_search(const float thr[kCodes - 1], SearchEntry tab[kBucketsPadded]) {
    int owner[kBuckets];
    for (int b = 0; b < kBuckets; ++b) owner[b] = -1;
    for (int k = 0; k + 1 < kCodes; ++k) {
        if (!(std::fabs(thr[k]) <= 1.0f)) return false;
        const int b = search_bucket(thr[k]);
        if (owner[b] >= 0) return false;
        // The step kernels look up the bucket of an approximate n' that may be a few units in the last place away
        // from the exact n; their guard only compares n' with the threshold of its own bucket.  That is sound as
        // long as no threshold lies so close to a bucket edge (k + 0.5) / 256 that n and n' could straddle the
        // edge next to it: demand a distance of 2^-20 relative, thousands of times the guard's reach.
        const double pos = double(thr[k]) * kBucketHalf + 0.5;
        const double to_edge = std::fabs(pos - std::nearbyint(pos));
        if (to_edge < std::ldexp(std::fabs(double(thr[k])) * kBucketHalf, -20)) return false;
        owner[b] = k;
    }
    uint32_t below = 0;
    for (int b = 0; b < kBucketsPadded; ++b) {
        SearchEntry e{kNoThreshold, below};
        if (b < kBuckets && owner[b] >= 0) {
            e.thr = thr[owner[b]];
            below++;
        }
        tab[b] = e;
    }
    return true;
}

inline int search_code(const SearchEntry tab[kBucketsPadded], float n) {
    if (!std::isfinite(n)) return 0;    // every distance is inf or NaN: the brute-force argmin keeps index 0
    const SearchEntry& e = tab[search_bucket(n)];
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
