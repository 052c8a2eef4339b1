// Device-side building blocks of the 4-bit AdamW step for gfx950 (wave64).
//
// Everything that decides a 4-bit code (the moments, the two normalizing divisions) is evaluated
// in IEEE fp32 with a fixed operation order: one rounding per written operation, fused
// multiply-add only where __builtin_fmaf is written (the translation unit is compiled with
// -ffp-contract=off), denormals kept, correctly rounded division.  The parameter update decides no
// integer and uses the hardware's approximate sqrt / reciprocal.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tables.hpp"

namespace lpmm {

struct Hyper {
    float beta1, beta2;
    float omb1, omb2;     // 1 - beta, rounded once in fp32
    float eps;
    float step_size;      // lr / (1 - beta1^t)
    float inv_sqrt_bc2;   // 1 / sqrt(1 - beta2^t)
    float lr_wd;          // lr * weight_decay
};

// ---- cross-lane reductions inside one DPP row (16 lanes = one 128-element block) ----------------

// Maximum over the 16 lanes of a row of a value that is >= +0 in every lane, result in every lane
// of the row.  Non-negative floats order like their bit patterns, so the unsigned integer maximum is
// used: 0 is its identity, which lets each step fold into one v_max_u32 with a DPP operand, and no
// NaN canonicalization is needed.  All 16 lanes of the row must be active.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_umax(uint32_t x) {
    const uint32_t y = uint32_t(__builtin_amdgcn_update_dpp(0, int(x), CTRL, 0xF, 0xF, false));
    return x > y ? x : y;
}
__device__ __forceinline__ float row16_allmax(float v) {
    uint32_t x = __float_as_uint(v);
    x = dpp_umax<0xB1>(x);    // quad_perm [1,0,3,2]: lane ^ 1
    x = dpp_umax<0x4E>(x);    // quad_perm [2,3,0,1]: lane ^ 2
    x = dpp_umax<0x141>(x);   // row_half_mirror: other quad of the half row
    x = dpp_umax<0x140>(x);   // row_mirror: other half of the row
    return __uint_as_float(x);
}

// ---- gradient element access ---------------------------------------------------------------------

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

template <bool BF16>
__device__ __forceinline__ void load_grad8(const void* g, int64_t idx, float out[8]) {
    if constexpr (BF16) {
        const uint4 w = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(g) + idx);
        out[0] = bf16_lo(w.x); out[1] = bf16_hi(w.x);
        out[2] = bf16_lo(w.y); out[3] = bf16_hi(w.y);
        out[4] = bf16_lo(w.z); out[5] = bf16_hi(w.z);
        out[6] = bf16_lo(w.w); out[7] = bf16_hi(w.w);
    } else {
        const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(g) + idx);
        const float4 a = p[0], b = p[1];
        out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
        out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
    }
}

template <bool BF16>
__device__ __forceinline__ float load_grad1(const void* g, int64_t idx) {
    if constexpr (BF16)
        return __uint_as_float(uint32_t(reinterpret_cast<const uint16_t*>(g)[idx]) << 16);
    else
        return reinterpret_cast<const float*>(g)[idx];
}

// ---- decompress ----------------------------------------------------------------------------------

// second moment: T_LIN[q] * min(r_i, c_j), T_LIN[q] = (q+1)/16 exactly
__device__ __forceinline__ float dequant_v(uint32_t q, float sc) {
    return (float(q + 1u) * 0.0625f) * sc;
}

// ---- the Adam rule of Eq. 1 on one element -------------------------------------------------------

__device__ __forceinline__ float moment_m(const Hyper& h, float m_prev, float g) {
    return __builtin_fmaf(h.beta1, m_prev, h.omb1 * g);
}
__device__ __forceinline__ float moment_v(const Hyper& h, float v_prev, float g) {
    return __builtin_fmaf(h.beta2, v_prev, (h.omb2 * g) * g);
}
// w - lr*( m^/(sqrt(v^)+eps) + wd*w ), to a few ulp (no integer depends on it)
__device__ __forceinline__ float param_update(const Hyper& h, float w, float mt, float vt) {
    const float denom = __builtin_fmaf(__builtin_amdgcn_sqrtf(vt), h.inv_sqrt_bc2, h.eps);
    const float x = mt * __builtin_amdgcn_rcpf(denom);
    const float wdec = __builtin_fmaf(-h.lr_wd, w, w);
    return __builtin_fmaf(-h.step_size, x, wdec);
}

// ---- SGD with momentum (App. E Alg. 2) on one element: h.beta1 is the momentum, h.step_size the rate ----

__device__ __forceinline__ float moment_sgdm(const Hyper& h, float m_prev, float g) {
    return __builtin_fmaf(h.beta1, m_prev, g);
}
__device__ __forceinline__ float param_sgdm(const Hyper& h, float w, float mt) {
    return __builtin_fmaf(-h.step_size, mt, w);
}

// ---- compress ------------------------------------------------------------------------------------

// bucket table entry of a normalized value with |n| <= 1 + 2^-22 (block absmax normalization
// guarantees it for finite input; a wild index could only come from non-finite input and reads LDS,
// which cannot fault): round(256 n) lands in the low bits of the fused multiply-add's result
__device__ __forceinline__ SearchEntry search_entry(const SearchEntry* s_search, float n) {
    const float x = __builtin_fmaf(n, kBucketScale, kBucketMagic);
    return s_search[int(__float_as_uint(x) - kBucketMagicBits) + kBucketHalf];
}

// first moment: n = m_t / s (0 when the block is all zero), code from the bucket table in LDS
__device__ __forceinline__ uint32_t quant_m_code(const SearchEntry* s_search, float mt, float s) {
    const float n = (s == 0.0f) ? 0.0f : mt / s;
    const SearchEntry e = search_entry(s_search, n);
    return e.base + (n > e.thr ? 1u : 0u);
}

// second moment: n = v_t / min(r_i, c_j) (0 when the scale is zero); nearest (k+1)/16 with ties
// down is ceil(16 n - 1.5) clamped to 0..15 (16 n and the subtraction are exact where it matters)
__device__ __forceinline__ uint32_t quant_v_code(float vt, float sc) {
    const float n = (sc == 0.0f) ? 0.0f : vt / sc;
    const float f = ceilf(__builtin_fmaf(16.0f, n, -1.5f));
    return uint32_t(fminf(fmaxf(f, 0.0f), 15.0f));
}

// ---- approximate compress with a guard ---------------------------------------------------------------
//
// The exact functions above cost one IEEE division per element.  The fast variants multiply by an
// approximate reciprocal (v_rcp_f32, 1 ulp) instead and keep track of how close the approximate
// normalized value came to a decision boundary.  The approximate n' and the exact n = RN(x/s)
// differ by at most 2^-22 |n| (1 ulp of the reciprocal, half an ulp each for the product and for
// the exact quotient), so whenever n' stays further than twice that from every boundary both give
// the same code.  `slack` accumulates the margin over a lane's elements; if it ends up negative in
// any lane, the wave recomputes that row's codes with the exact functions.  Scales outside
// [2^-100, 2^100] (where the reciprocal or scale/16 may lose bits) always take the exact path.

constexpr float kScaleLo = 0x1p-100f;
constexpr float kScaleHi = 0x1p100f;

// branch-free: zero, or bits inside [bits(2^-100), bits(2^100)] (scales are never negative)
__device__ __forceinline__ bool scale_is_tame(float s) {
    const uint32_t u = __float_as_uint(s);
    constexpr uint32_t lo = 0x0D800000u, hi = 0x71800000u;     // 2^-100, 2^100
    return bool(int(u - lo <= hi - lo) | int(u == 0u));
}
__device__ __forceinline__ float approx_inv(float s) {
    return s == 0.0f ? 0.0f : __builtin_amdgcn_rcpf(s);
}

// first moment: `dist` = |bits(n') - bits(thr)| for the one threshold of the bucket, i.e. their
// distance in units in the last place (a bucket that holds a threshold lies on one side of zero, so
// the two have the same sign and bit patterns order like magnitudes; buckets without one compare
// against a far-away constant).  The
// exact n can lie at most 4 ulp of thr away from n' (2^-22 |thr|, an ulp being at least 2^-24 |thr|),
// so 16 or more -- which stays at least 8 ulp of thr when the two straddle a power of two -- is safe.
constexpr uint32_t kMinDistM = 16;

__device__ __forceinline__ uint32_t quant_m_code_fast(const SearchEntry* s_search, float mt, float inv_s,
                                                      uint32_t& dist) {
    const float n = mt * inv_s;
    const SearchEntry e = search_entry(s_search, n);
    dist = __usad(__float_as_uint(n), __float_as_uint(e.thr), 0u);
    return e.base + (n > e.thr ? 1u : 0u);
}

// second moment: boundaries of the Linear map are the integers of f = 16 n - 1.5 and the code is
// ceil(f).  The approximate f' is within 2^-17 of the exact one; away from integers
// round-to-nearest(f' + 0.5) equals ceil(f), and the saturating byte convert both rounds that way and
// clamps below at 0 (above, n <= 1 keeps the code at 15).  `off` returns fract(f' + 0.5) - 0.5, the
// signed distance of f' from the integer it is closest to when that distance is small: a magnitude
// below 2^-16 sends the row to the exact path.
constexpr float kMarginV = 0x1p-16f;

template <int BYTE>
__device__ __forceinline__ uint32_t quant_v_code_fast(float vt, float inv_sc, uint32_t packed, float& off) {
    const float x = __builtin_fmaf(16.0f, vt * inv_sc, -1.0f);      // f' + 0.5
    off = __builtin_amdgcn_fractf(x) - 0.5f;                       // 0 when f' sits on an integer
    return __builtin_amdgcn_cvt_pk_u8_f32(x, BYTE, packed);
}

// second-moment decompress with the scale already divided by 16 (exact for tame scales):
// (q+1) * s16 in one rounding == T_LIN[q] * scale
__device__ __forceinline__ float dequant_v16(float qf, float s16) { return __builtin_fmaf(qf, s16, s16); }

// ---- float maximum through an integer atomic (values >= +0 only: bit order == value order) --------

__device__ __forceinline__ void atomic_max_nonneg(float* addr, float v) {
    atomicMax(reinterpret_cast<unsigned int*>(addr), __float_as_uint(v));
}

}  // namespace lpmm
