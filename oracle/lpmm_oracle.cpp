// lpmm_oracle.cpp -- plain, slow, single-threaded CPU oracle for the 4-bit AdamW step of
// "Memory Efficient Optimizers with 4-bit States" (arXiv 2309.01507).
//
// THIS IS TEST INFRASTRUCTURE.  It exists so that the GPU library can be checked against
// something written straight from the paper.  It shares no code, header, table or constant
// with the GPU path, and nothing in the product may call it.  Only the test-suite, the smoke
// check and the benchmark's "cpu_baseline" leg load it.
//
// What it follows (section / equation / algorithm of the paper):
//   * Sec. 2.1, Alg. 1 and App. E Alg. 3: decompress -> Adam update -> compress, per tensor.
//   * Eq. 1: the Adam moment, bias-correction and parameter formulas.
//   * Sec. 2.2: quantizer = mapping o normalization, mapping = argmin_i |n - T(i)|,
//     dequantizer = N^-1 o T; block-wise normalization over the row-major flattening.
//   * Sec. 3: block size 128 for the first moment.
//   * Sec. 4.1 and App. D.2: the zero-excluding Linear map T(i) = (i+1)/2^b.
//   * Sec. 4.2: rank-1 normalization, r_i = max_j x_ij, c_j = max_i x_ij, n_ij = x_ij / min(r_i, c_j).
//   * Sec. 4.2, last paragraph: for 1-dimensional tensors rank-1 normalization degenerates, and
//     block-wise normalization with block size 128 is used for the second moment instead (the
//     mapping stays the Linear one).  App. C.1 (LLaMA): FSDP packs parameters into 1-dimensional
//     arrays, so that run used this form for every tensor.  Functions *_v_block / *_b128_*.
//   * App. F Alg. 4: rank-1 normalization of a tensor with p dimensions: one statistic per index of
//     every dimension (the maximum of |x| over all other indices), an element's scale is the minimum
//     of its p statistics.  Functions *_v_nd / *_nd_*.  (The second moment is >= 0, so |x| = x.)
//   * App. E Alg. 2: compression-based SGD with momentum: m_t = beta m_{t-1} + g, theta -= alpha m_t,
//     the momentum compressed like Adam's first moment (B128 + signed DE map).  Functions *_sgdm*.
//   * Sec. 4.3 and Sec. 5 ("4-bit Factor"): for tensors with two dimensions the second moment is
//     not stored per element but factorized the way the cited Adafactor method does it: one
//     statistic per row and one per column, v_ij reconstructed as row_i * col_j / sum(row).  The
//     first moment stays B128/DE.  Functions *_factor_*.
//   * Sec. 4.1, Tab. 1 and App. D.3 (ablation quantizers, not on any optimizer step's path): block-wise
//     normalization with block size 2048 ("B2048", the 8-bit optimizer's), the unsigned 4-bit DE map, the same
//     map with its zero removed ("DE-0", 15 points, smallest 0.0033), and stochastic rounding between the two
//     neighbouring table entries.  Functions *_ablation.
//   * App. D.1: signed normalization n = sign(x) N(|x|).
//   * App. D.2: the dynamic-exponent (DE) map: sign bit, E leading zeros, indicator bit,
//     F fraction bits; value 10^-E * fraction[k]; two special bit patterns; sorted list.
//
// Precision.  The moments m_t, v_t and the two normalizing divisions are evaluated in IEEE fp32
// (round-to-nearest-even, no contraction except the two explicit fmaf calls, denormals kept),
// because they decide integer codes and both sides must take that decision in the same precision.
// The nearest-entry search takes its differences in double, which is exact for fp32 operands.
// The parameter update, which decides no integer, is evaluated in double from the fp32 moments
// and rounded once to fp32 for storage.
//
// Readings where the paper is silent or inconsistent (each also listed in the design notes):
//   * Alg. 3 prints (1-beta1) in the second-moment line; Eq. 1 has (1-beta2).  Eq. 1 is used.
//   * AdamW = Adam plus decoupled decay: w <- w - lr*( m^/(sqrt(v^)+eps) + wd*w ).
//   * The parameter update uses the precise m_t, v_t (compress is the last line of Alg. 3).
//   * A stored code is the rank of the value in the sorted table (App. D.2, last sentence).
//   * argmin ties go to the lowest index.
//   * A zero scale (all-zero block, untouched row/column, the zero initial state) gives n := 0.
//   * Scales are fp32.  Two codes per byte: element 2k in bits 0..3, element 2k+1 in bits 4..7.
//   * Blocks are [128k, 128k+127] of the row-major flattening; the last one may be short.
//   * Stochastic rounding (App. D.3) needs one uniform number per element.  It is drawn from a counter-based
//     generator so that both sides can produce it on their own: u = (top 24 bits of SplitMix64's output number
//     idx+1 for the state `seed`) * 2^-24, idx the element's flat index; the upper candidate is taken iff
//     u < p, with p = (n - T[q1]) / (T[q2] - T[q1]) evaluated in fp32 (two subtractions, one division).
//   * 4-bit Factor: the paper gives no formulas, only the citation.  Reading: the optimizer stays the
//     AdamW of Eq. 1 (same beta2, same bias correction, same eps; none of the cited method's own extras:
//     no update clipping, no relative step size, no decay-rate schedule, no 1e-30 added to g^2);
//     R_t = beta2 R_{t-1} + (1-beta2) rowsum(g^2), C_t likewise with column sums, and
//     v_t[i][j] = R_t[i] C_t[j] / sum_i R_t[i] (0 when the sum is 0) takes the place of v_t.
//     R and C are stored in fp32; nothing integer depends on them, so they are computed in double.
//
// Parity status: every function below is pinned by the CPU tests against values the paper prints,
// closed forms, brute force, invariants or an fp64 library AdamW, EXCEPT the multi-step trajectory
// of the full quantized step (any second-moment form), for which the paper prints nothing:
// "parity unpinned" beyond its parts.
//
// Build: g++ -O2 -std=c++17 -ffp-contract=off -fPIC -shared lpmm_oracle.cpp -o liblpmm_oracle.so

#include <cmath>
#include <cstdint>
#include <cstring>
#include <algorithm>
#include <vector>

namespace {

constexpr int kBits = 4;
constexpr int kCodes = 1 << kBits;   // 16 quantization points (Sec. 4.1)
constexpr int64_t kBlock = 128;      // B128 (Sec. 3)

// ---------------------------------------------------------------------------------------------
// Quantization mappings (App. D.2)
// ---------------------------------------------------------------------------------------------

// Linear map: T(i) = (i+1)/2^b, i.e. linspace(0,1,2^b+1) without its first point.
void table_linear(int bits, std::vector<double>& out) {
    const int n = 1 << bits;
    out.resize(n);
    for (int i = 0; i < n; ++i) out[i] = double(i + 1) / double(n);
}

// fraction[k] for F fraction bits: p_j = 0.9/2^F * j + 0.1, fraction[k] = (p_k + p_{k+1})/2.
double de_fraction(int F, int k) {
    const double step = (1.0 - 0.1) / double(1 << F);
    const double pk = step * k + 0.1;
    const double pk1 = step * (k + 1) + 0.1;
    return (pk + pk1) / 2.0;
}

// Dynamic-exponent map with `bits` total bits.  Every bit pattern is decoded by the rule of
// App. D.2; the two special patterns are overridden; the values are then sorted increasingly.
void table_de(int bits, bool is_signed, std::vector<double>& out) {
    const int n = 1 << bits;
    const int mag_bits = is_signed ? bits - 1 : bits;   // bits after the sign bit
    out.clear();
    for (int pat = 0; pat < n; ++pat) {
        const int sign = is_signed ? (pat >> mag_bits) & 1 : 0;
        const int mag = pat & ((1 << mag_bits) - 1);
        double val;
        if (mag == 0) {
            // All-zero magnitude field: no indicator bit.  0...0 -> 0; in the signed case the
            // pattern 10...0 is assigned +1 (so -1 does not exist and the map is not symmetric).
            val = (sign == 0) ? 0.0 : 1.0;
        } else if (!is_signed && mag == 1) {
            // Unsigned special pattern 0...01 -> 1.
            val = 1.0;
        } else {
            int E = 0;   // leading zeros of the magnitude field
            while (((mag >> (mag_bits - 1 - E)) & 1) == 0) ++E;
            const int F = mag_bits - E - 1;             // bits after the indicator
            const int k = mag & ((1 << F) - 1);
            val = std::pow(10.0, -double(E)) * de_fraction(F, k);
            if (sign) val = -val;
        }
        out.push_back(val);
    }
    std::sort(out.begin(), out.end());
}

struct Tables {
    float lin[kCodes];
    float de[kCodes];
    Tables() {
        std::vector<double> t;
        table_linear(kBits, t);
        for (int i = 0; i < kCodes; ++i) lin[i] = float(t[i]);
        table_de(kBits, true, t);
        for (int i = 0; i < kCodes; ++i) de[i] = float(t[i]);
    }
};
const Tables& tables() { static const Tables t; return t; }

// Mapping M(n) = argmin_i |n - T(i)| (Sec. 2.2); brute force over all entries, differences in
// double (exact for fp32 inputs), first minimum wins.
int nearest_code(const float* T, int n_entries, float n) {
    int best = 0;
    double best_d = std::fabs(double(n) - double(T[0]));
    for (int i = 1; i < n_entries; ++i) {
        const double d = std::fabs(double(n) - double(T[i]));
        if (d < best_d) { best_d = d; best = i; }
    }
    return best;
}

inline int get_code(const uint8_t* codes, int64_t idx) {
    const uint8_t b = codes[idx >> 1];
    return (idx & 1) ? (b >> 4) : (b & 0x0F);
}
inline void put_code(uint8_t* codes, int64_t idx, int q) {
    uint8_t& b = codes[idx >> 1];
    if (idx & 1) b = uint8_t((b & 0x0F) | (q << 4));
    else         b = uint8_t((b & 0xF0) | q);
}

// ---------------------------------------------------------------------------------------------
// First moment: B128 normalization (Sec. 2.2, 3; signed form App. D.1) + signed DE map
// ---------------------------------------------------------------------------------------------

void quant_m(const float* x, int64_t P, uint8_t* codes, float* scales) {
    const float* T = tables().de;
    std::memset(codes, 0, size_t((P + 1) / 2));
    const int64_t nblk = (P + kBlock - 1) / kBlock;
    for (int64_t k = 0; k < nblk; ++k) {
        const int64_t lo = k * kBlock, hi = std::min(P, lo + kBlock);
        float s = 0.0f;
        for (int64_t i = lo; i < hi; ++i) s = std::max(s, std::fabs(x[i]));
        scales[k] = s;
        for (int64_t i = lo; i < hi; ++i) {
            const float n = (s == 0.0f) ? 0.0f : x[i] / s;   // sign(x) * |x| / s == x / s
            put_code(codes, i, nearest_code(T, kCodes, n));
        }
    }
}

void dequant_m(const uint8_t* codes, const float* scales, int64_t P, float* out) {
    const float* T = tables().de;
    for (int64_t i = 0; i < P; ++i) out[i] = T[get_code(codes, i)] * scales[i / kBlock];
}

// ---------------------------------------------------------------------------------------------
// Second moment: rank-1 normalization (Sec. 4.2) + Linear map (Sec. 4.1)
// ---------------------------------------------------------------------------------------------

void quant_v(const float* x, int64_t rows, int64_t cols, uint8_t* codes, float* r, float* c) {
    const float* T = tables().lin;
    const int64_t P = rows * cols;
    std::memset(codes, 0, size_t((P + 1) / 2));
    for (int64_t i = 0; i < rows; ++i) r[i] = 0.0f;
    for (int64_t j = 0; j < cols; ++j) c[j] = 0.0f;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            const float v = x[i * cols + j];
            r[i] = std::max(r[i], v);
            c[j] = std::max(c[j], v);
        }
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            const float sc = std::min(r[i], c[j]);
            const float n = (sc == 0.0f) ? 0.0f : x[i * cols + j] / sc;
            put_code(codes, i * cols + j, nearest_code(T, kCodes, n));
        }
}

void dequant_v(const uint8_t* codes, const float* r, const float* c, int64_t rows, int64_t cols,
               float* out) {
    const float* T = tables().lin;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j)
            out[i * cols + j] = T[get_code(codes, i * cols + j)] * std::min(r[i], c[j]);
}

// ---------------------------------------------------------------------------------------------
// Second moment of a tensor with p >= 1 dimensions: rank-1 normalization in its general form
// (App. F Alg. 4) + Linear map.  dims[0..p) is the shape (row-major: the last index runs fastest),
// stats holds mu_1 (dims[0] floats), then mu_2 (dims[1] floats), ... one after the other.
// ---------------------------------------------------------------------------------------------

// the p indices of flat element e
void unravel(int64_t e, const int64_t* dims, int p, int64_t* idx) {
    for (int r = p - 1; r >= 0; --r) {
        idx[r] = e % dims[r];
        e /= dims[r];
    }
}

void quant_v_nd(const float* x, const int64_t* dims, int p, uint8_t* codes, float* stats) {
    const float* T = tables().lin;
    int64_t P = 1, n_stats = 0;
    std::vector<int64_t> first(static_cast<size_t>(p));          // where mu_r starts inside stats
    for (int r = 0; r < p; ++r) { first[size_t(r)] = n_stats; n_stats += dims[r]; P *= dims[r]; }
    std::memset(codes, 0, size_t((P + 1) / 2));
    for (int64_t k = 0; k < n_stats; ++k) stats[k] = 0.0f;
    std::vector<int64_t> idx(static_cast<size_t>(p));
    for (int64_t e = 0; e < P; ++e) {                            // Alg. 4, first loop: the statistics
        unravel(e, dims, p, idx.data());
        for (int r = 0; r < p; ++r) {
            float& mu = stats[first[size_t(r)] + idx[size_t(r)]];
            mu = std::max(mu, x[e]);
        }
    }
    for (int64_t e = 0; e < P; ++e) {                            // second loop: M = min over the dimensions
        unravel(e, dims, p, idx.data());
        float M = stats[first[0] + idx[0]];
        for (int r = 1; r < p; ++r) M = std::min(M, stats[first[size_t(r)] + idx[size_t(r)]]);
        const float n = (M == 0.0f) ? 0.0f : x[e] / M;
        put_code(codes, e, nearest_code(T, kCodes, n));
    }
}

void dequant_v_nd(const uint8_t* codes, const float* stats, const int64_t* dims, int p, float* out) {
    const float* T = tables().lin;
    int64_t P = 1, n_stats = 0;
    std::vector<int64_t> first(static_cast<size_t>(p)), idx(static_cast<size_t>(p));
    for (int r = 0; r < p; ++r) { first[size_t(r)] = n_stats; n_stats += dims[r]; P *= dims[r]; }
    for (int64_t e = 0; e < P; ++e) {
        unravel(e, dims, p, idx.data());
        float M = stats[first[0] + idx[0]];
        for (int r = 1; r < p; ++r) M = std::min(M, stats[first[size_t(r)] + idx[size_t(r)]]);
        out[e] = T[get_code(codes, e)] * M;
    }
}

// ---------------------------------------------------------------------------------------------
// Second moment of 1-dimensional (or flattened) tensors: B128 normalization (Sec. 2.2 block-wise
// normalization with the block size of Sec. 3, chosen by Sec. 4.2 for this case) + Linear map.
// The moment is non-negative, so the block's scale max|x| is max x.
// ---------------------------------------------------------------------------------------------

void quant_v_block(const float* x, int64_t P, uint8_t* codes, float* scales) {
    const float* T = tables().lin;
    std::memset(codes, 0, size_t((P + 1) / 2));
    const int64_t nblk = (P + kBlock - 1) / kBlock;
    for (int64_t k = 0; k < nblk; ++k) {
        const int64_t lo = k * kBlock, hi = std::min(P, lo + kBlock);
        float s = 0.0f;
        for (int64_t i = lo; i < hi; ++i) s = std::max(s, std::fabs(x[i]));
        scales[k] = s;
        for (int64_t i = lo; i < hi; ++i) {
            const float n = (s == 0.0f) ? 0.0f : x[i] / s;
            put_code(codes, i, nearest_code(T, kCodes, n));
        }
    }
}

void dequant_v_block(const uint8_t* codes, const float* scales, int64_t P, float* out) {
    const float* T = tables().lin;
    for (int64_t i = 0; i < P; ++i) out[i] = T[get_code(codes, i)] * scales[i / kBlock];
}

// ---------------------------------------------------------------------------------------------
// The optimizer rule A of Alg. 1: Adam (Eq. 1) with decoupled weight decay, on precise states.
// m and v are updated in place (m_{t-1} -> m_t); w is updated in place.
// ---------------------------------------------------------------------------------------------

void adamw_rule(float* w, float* m, float* v, const float* g, int64_t P, float lr, float beta1,
                float beta2, float eps, float wd, int64_t t) {
    const float omb1 = 1.0f - beta1;
    const float omb2 = 1.0f - beta2;
    const double bc1 = 1.0 - std::pow(double(beta1), double(t));
    const double bc2 = 1.0 - std::pow(double(beta2), double(t));
    for (int64_t i = 0; i < P; ++i) {
        // fp32 moments; the operation order is part of the definition both sides implement
        const float mt = std::fmaf(beta1, m[i], omb1 * g[i]);
        const float vt = std::fmaf(beta2, v[i], (omb2 * g[i]) * g[i]);
        m[i] = mt;
        v[i] = vt;
        const double mhat = double(mt) / bc1;
        const double vhat = double(vt) / bc2;
        const double wi = double(w[i]);
        w[i] = float(wi - double(lr) * (mhat / (std::sqrt(vhat) + double(eps)) + double(wd) * wi));
    }
}

// The rule of Alg. 2 on a precise momentum buffer: m_t = beta m_{t-1} + g_t, theta_t = theta_{t-1} - alpha m_t.
// The momentum decides integer codes afterwards, so it is one fused multiply-add in fp32 on both sides;
// the parameter is evaluated in double and rounded once.  No weight decay, no dampening: Alg. 2 has none.
void sgdm_rule(float* w, float* m, const float* g, int64_t P, float lr, float beta) {
    for (int64_t i = 0; i < P; ++i) {
        const float mt = std::fmaf(beta, m[i], g[i]);
        m[i] = mt;
        w[i] = float(double(w[i]) - double(lr) * double(mt));
    }
}

// ---------------------------------------------------------------------------------------------
// Ablation quantizers of the second moment (Sec. 4.1, Tab. 1) and stochastic rounding (App. D.3).
// norm: 0 = B128, 1 = B2048 (block-wise normalization, Sec. 2.2, with the two block sizes the paper
// compares), 2 = rank-1 (Sec. 4.2).  map: 0 = 4-bit DE (unsigned variant for non-negative input, signed
// variant for signed input), 1 = DE-0 (unsigned DE without its zero: 15 points), 2 = Linear.
// Signed input (the first moment of Tab. 1's first line, "B2048/DE for both moments") takes block-wise
// normalization and the signed DE map only.
// ---------------------------------------------------------------------------------------------

bool ablation_table(int map, bool is_signed, std::vector<float>& T) {
    std::vector<double> t;
    if (map == 0) {
        table_de(kBits, is_signed, t);
    } else if (map == 1 && !is_signed) {
        table_de(kBits, false, t);
        t.erase(std::remove(t.begin(), t.end(), 0.0), t.end());      // "simply remove zero" (Sec. 4.1)
    } else if (map == 2 && !is_signed) {
        table_linear(kBits, t);
    } else {
        return false;
    }
    T.resize(t.size());
    for (size_t i = 0; i < t.size(); ++i) T[i] = float(t[i]);
    return true;
}

// SplitMix64 (Steele, Lea, Flood 2014): output number idx+1 of the generator whose state starts at `seed`.
uint64_t splitmix64_at(uint64_t seed, uint64_t idx) {
    uint64_t z = seed + (idx + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
float uniform_at(uint64_t seed, uint64_t idx) { return float(splitmix64_at(seed, idx) >> 40) * 0x1p-24f; }

// App. D.3: the candidate set M(n) holds the nearest entry at or below n and the nearest entry at or
// above n (one point when n is an entry or lies outside the table's range); between two candidates
// q1 < q2 the upper one is chosen with probability (n - T(q1)) / (T(q2) - T(q1)).
int round_stochastic(const float* T, int n_entries, float n, float u) {
    int q1 = -1, q2 = -1;
    for (int i = 0; i < n_entries; ++i) if (T[i] <= n) q1 = i;                // largest entry <= n
    for (int i = n_entries - 1; i >= 0; --i) if (T[i] >= n) q2 = i;           // smallest entry >= n
    if (q1 < 0 && q2 < 0) return 0;     // n is not a number
    if (q1 < 0) return q2;
    if (q2 < 0) return q1;
    if (q1 == q2) return q1;
    const float p = (n - T[q1]) / (T[q2] - T[q1]);
    return u < p ? q2 : q1;
}

// per-element scale of the chosen normalization; sa / sb receive the statistics
void ablation_scales(const float* x, int64_t rows, int64_t cols, int norm, float* sa, float* sb,
                     std::vector<float>& scale) {
    const int64_t P = rows * cols;
    scale.assign(size_t(P), 0.0f);
    if (norm == 2) {
        for (int64_t i = 0; i < rows; ++i) sa[i] = 0.0f;
        for (int64_t j = 0; j < cols; ++j) sb[j] = 0.0f;
        for (int64_t i = 0; i < rows; ++i)
            for (int64_t j = 0; j < cols; ++j) {
                sa[i] = std::max(sa[i], x[i * cols + j]);
                sb[j] = std::max(sb[j], x[i * cols + j]);
            }
        for (int64_t i = 0; i < rows; ++i)
            for (int64_t j = 0; j < cols; ++j) scale[size_t(i * cols + j)] = std::min(sa[i], sb[j]);
    } else {
        const int64_t B = norm == 0 ? 128 : 2048;
        const int64_t nblk = (P + B - 1) / B;
        for (int64_t k = 0; k < nblk; ++k) {
            const int64_t lo = k * B, hi = std::min(P, lo + B);
            float s = 0.0f;
            for (int64_t i = lo; i < hi; ++i) s = std::max(s, std::fabs(x[i]));
            sa[k] = s;
            for (int64_t i = lo; i < hi; ++i) scale[size_t(i)] = s;
        }
    }
}

}  // namespace

extern "C" {

// ---- ablation quantizers (Sec. 4.1, Tab. 1, App. D.3) ------------------------------------------
// Number of entries of the map (16, or 15 for DE-0), 0 for an invalid combination; out (may be null)
// receives the entries.
int oracle_ablation_table(int map, int is_signed, float* out) {
    std::vector<float> T;
    if (!ablation_table(map, is_signed != 0, T)) return 0;
    if (out) for (size_t i = 0; i < T.size(); ++i) out[i] = T[i];
    return int(T.size());
}
uint64_t oracle_splitmix64_at(uint64_t seed, uint64_t idx) { return splitmix64_at(seed, idx); }
float oracle_uniform_at(uint64_t seed, uint64_t idx) { return uniform_at(seed, idx); }
int oracle_round_stochastic(const float* table, int n_entries, float n, float u) {
    return round_stochastic(table, n_entries, n, u);
}
// Compress x (rows x cols, row-major; block-wise normalizations take it flat).  codes: (P+1)/2 bytes.
// sa: block scales (ceil(P/128) or ceil(P/2048) floats) or row maxima (rows floats); sb: column maxima
// (cols floats, rank-1 only).  rounding: 0 = nearest (Sec. 2.2), 1 = stochastic (App. D.3) with `seed`.
// Returns 0, or -1 for a combination that does not exist.
int oracle_quant_ablation(int norm, int map, int is_signed, int rounding, uint64_t seed, const float* x,
                          int64_t rows, int64_t cols, uint8_t* codes, float* sa, float* sb) {
    std::vector<float> T, scale;
    if (!ablation_table(map, is_signed != 0, T) || norm < 0 || norm > 2 || (norm == 2 && is_signed)) return -1;
    const int64_t P = rows * cols;
    ablation_scales(x, rows, cols, norm, sa, sb, scale);
    std::memset(codes, 0, size_t((P + 1) / 2));
    for (int64_t e = 0; e < P; ++e) {
        const float s = scale[size_t(e)];
        const float n = (s == 0.0f) ? 0.0f : x[e] / s;
        const int q = rounding ? round_stochastic(T.data(), int(T.size()), n, uniform_at(seed, uint64_t(e)))
                               : nearest_code(T.data(), int(T.size()), n);
        put_code(codes, e, q);
    }
    return 0;
}
int oracle_dequant_ablation(int norm, int map, int is_signed, const uint8_t* codes, const float* sa,
                            const float* sb, int64_t rows, int64_t cols, float* out) {
    std::vector<float> T;
    if (!ablation_table(map, is_signed != 0, T) || norm < 0 || norm > 2 || (norm == 2 && is_signed)) return -1;
    const int64_t B = norm == 0 ? 128 : 2048;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            const int64_t e = i * cols + j;
            const float s = norm == 2 ? std::min(sa[i], sb[j]) : sa[e / B];
            const int q = get_code(codes, e);
            out[e] = (q < int(T.size()) ? T[size_t(q)] : 0.0f) * s;
        }
    return 0;
}

// ---- tables --------------------------------------------------------------------------------
// out must hold 2^bits floats (table_de) / doubles (table_de_f64).
void oracle_table_linear(int bits, float* out) {
    std::vector<double> t; table_linear(bits, t);
    for (size_t i = 0; i < t.size(); ++i) out[i] = float(t[i]);
}
void oracle_table_de(int bits, int is_signed, float* out) {
    std::vector<double> t; table_de(bits, is_signed != 0, t);
    for (size_t i = 0; i < t.size(); ++i) out[i] = float(t[i]);
}
void oracle_table_de_f64(int bits, int is_signed, double* out) {
    std::vector<double> t; table_de(bits, is_signed != 0, t);
    for (size_t i = 0; i < t.size(); ++i) out[i] = t[i];
}
// The two 16-entry tables the step actually uses (what=0: signed DE, what=1: Linear).
void oracle_step_table(int what, float* out) {
    const float* T = what == 0 ? tables().de : tables().lin;
    for (int i = 0; i < kCodes; ++i) out[i] = T[i];
}

// ---- mapping -------------------------------------------------------------------------------
int oracle_nearest_code(const float* table, int n_entries, float n) {
    return nearest_code(table, n_entries, n);
}
void oracle_nearest_codes(const float* table, int n_entries, const float* n, int64_t count,
                          uint8_t* out) {
    for (int64_t i = 0; i < count; ++i) out[i] = uint8_t(nearest_code(table, n_entries, n[i]));
}

// ---- quantizers (compress / decompress of Alg. 1) --------------------------------------------
// codes: (P+1)/2 bytes; scales: ceil(P/128) floats; r: rows floats; c: cols floats.
void oracle_quant_m(const float* x, int64_t P, uint8_t* codes, float* scales) {
    quant_m(x, P, codes, scales);
}
void oracle_dequant_m(const uint8_t* codes, const float* scales, int64_t P, float* out) {
    dequant_m(codes, scales, P, out);
}
void oracle_quant_v(const float* x, int64_t rows, int64_t cols, uint8_t* codes, float* r, float* c) {
    quant_v(x, rows, cols, codes, r, c);
}
void oracle_dequant_v(const uint8_t* codes, const float* r, const float* c, int64_t rows,
                      int64_t cols, float* out) {
    dequant_v(codes, r, c, rows, cols, out);
}

// ---- optimizer steps -------------------------------------------------------------------------
// Adam/AdamW on uncompressed fp32 states: Alg. 3 with compress = decompress = identity.  Also the
// path for tensors that are not quantized (App. C.1: size <= 4096).
void oracle_adamw32_step(float* w, const float* g, float* m, float* v, int64_t P, float lr,
                         float beta1, float beta2, float eps, float wd, int64_t t) {
    adamw_rule(w, m, v, g, P, lr, beta1, beta2, eps, wd, t);
}

// One step of 4-bit AdamW on one rows x cols tensor (Alg. 3): decompress both moments, apply the
// rule on the precise states, compress both.  All state buffers are updated in place.
// m_t_out / v_t_out (each rows*cols floats, may be null) receive the precise moments before
// compression, so that a test can tell how close a value was to a decision boundary.
void oracle_adamw4_step(float* w, const float* g, uint8_t* m_codes, float* m_scales,
                        uint8_t* v_codes, float* v_r, float* v_c, int64_t rows, int64_t cols,
                        float lr, float beta1, float beta2, float eps, float wd, int64_t t,
                        float* m_t_out, float* v_t_out) {
    const int64_t P = rows * cols;
    std::vector<float> m(static_cast<size_t>(P)), v(static_cast<size_t>(P));
    dequant_m(m_codes, m_scales, P, m.data());                    // Alg. 3: decompress
    dequant_v(v_codes, v_r, v_c, rows, cols, v.data());
    adamw_rule(w, m.data(), v.data(), g, P, lr, beta1, beta2, eps, wd, t);   // Eq. 1
    if (m_t_out) std::memcpy(m_t_out, m.data(), sizeof(float) * size_t(P));
    if (v_t_out) std::memcpy(v_t_out, v.data(), sizeof(float) * size_t(P));
    quant_m(m.data(), P, m_codes, m_scales);                      // Alg. 3: compress
    quant_v(v.data(), rows, cols, v_codes, v_r, v_c);
}

// The same step for a 1-dimensional or flattened tensor of P elements: the second moment is
// compressed block-wise (B128/Linear) instead of rank-1 (Sec. 4.2, last paragraph).  Everything is
// local to a block of 128 elements.
void oracle_quant_v_block(const float* x, int64_t P, uint8_t* codes, float* scales) {
    quant_v_block(x, P, codes, scales);
}
void oracle_dequant_v_block(const uint8_t* codes, const float* scales, int64_t P, float* out) {
    dequant_v_block(codes, scales, P, out);
}
void oracle_adamw4_b128_step(float* w, const float* g, uint8_t* m_codes, float* m_scales,
                             uint8_t* v_codes, float* v_scales, int64_t P, float lr, float beta1,
                             float beta2, float eps, float wd, int64_t t, float* m_t_out,
                             float* v_t_out) {
    std::vector<float> m(static_cast<size_t>(P)), v(static_cast<size_t>(P));
    dequant_m(m_codes, m_scales, P, m.data());                    // Alg. 3: decompress
    dequant_v_block(v_codes, v_scales, P, v.data());
    adamw_rule(w, m.data(), v.data(), g, P, lr, beta1, beta2, eps, wd, t);   // Eq. 1
    if (m_t_out) std::memcpy(m_t_out, m.data(), sizeof(float) * size_t(P));
    if (v_t_out) std::memcpy(v_t_out, v.data(), sizeof(float) * size_t(P));
    quant_m(m.data(), P, m_codes, m_scales);                      // Alg. 3: compress
    quant_v_block(v.data(), P, v_codes, v_scales);
}
void oracle_state_zero_b128(uint8_t* m_codes, float* m_scales, uint8_t* v_codes, float* v_scales,
                            int64_t P) {
    std::vector<float> z(static_cast<size_t>(P), 0.0f);
    quant_m(z.data(), P, m_codes, m_scales);
    quant_v_block(z.data(), P, v_codes, v_scales);
}

// One step of 4-bit AdamW on a tensor with p dimensions (Alg. 3 with the rank-1 normalization of
// App. F Alg. 4 for the second moment).  v_stats: the p statistics vectors one after the other.
void oracle_quant_v_nd(const float* x, const int64_t* dims, int p, uint8_t* codes, float* stats) {
    quant_v_nd(x, dims, p, codes, stats);
}
void oracle_dequant_v_nd(const uint8_t* codes, const float* stats, const int64_t* dims, int p, float* out) {
    dequant_v_nd(codes, stats, dims, p, out);
}
void oracle_adamw4_nd_step(float* w, const float* g, uint8_t* m_codes, float* m_scales, uint8_t* v_codes,
                           float* v_stats, const int64_t* dims, int p, float lr, float beta1, float beta2,
                           float eps, float wd, int64_t t, float* m_t_out, float* v_t_out) {
    int64_t P = 1;
    for (int r = 0; r < p; ++r) P *= dims[r];
    std::vector<float> m(static_cast<size_t>(P)), v(static_cast<size_t>(P));
    dequant_m(m_codes, m_scales, P, m.data());                    // Alg. 3: decompress
    dequant_v_nd(v_codes, v_stats, dims, p, v.data());
    adamw_rule(w, m.data(), v.data(), g, P, lr, beta1, beta2, eps, wd, t);   // Eq. 1
    if (m_t_out) std::memcpy(m_t_out, m.data(), sizeof(float) * size_t(P));
    if (v_t_out) std::memcpy(v_t_out, v.data(), sizeof(float) * size_t(P));
    quant_m(m.data(), P, m_codes, m_scales);                      // Alg. 3: compress
    quant_v_nd(v.data(), dims, p, v_codes, v_stats);
}
void oracle_state_zero_nd(uint8_t* m_codes, float* m_scales, uint8_t* v_codes, float* v_stats,
                          const int64_t* dims, int p) {
    int64_t P = 1;
    for (int r = 0; r < p; ++r) P *= dims[r];
    std::vector<float> z(static_cast<size_t>(P), 0.0f);
    quant_m(z.data(), P, m_codes, m_scales);
    quant_v_nd(z.data(), dims, p, v_codes, v_stats);
}

// SGD with momentum (Alg. 2) on an uncompressed fp32 momentum buffer (tensors that are not quantized), and
// with the momentum compressed to 4 bits (B128 + signed DE map, the first-moment quantizer of Sec. 3).
void oracle_sgdm32_step(float* w, const float* g, float* m, int64_t P, float lr, float beta) {
    sgdm_rule(w, m, g, P, lr, beta);
}
void oracle_sgdm4_step(float* w, const float* g, uint8_t* m_codes, float* m_scales, int64_t P, float lr,
                       float beta, float* m_t_out) {
    std::vector<float> m(static_cast<size_t>(P));
    dequant_m(m_codes, m_scales, P, m.data());                    // Alg. 2: decompress
    sgdm_rule(w, m.data(), g, P, lr, beta);
    if (m_t_out) std::memcpy(m_t_out, m.data(), sizeof(float) * size_t(P));
    quant_m(m.data(), P, m_codes, m_scales);                      // Alg. 2: compress
}

// One step of "4-bit Factor" on one rows x cols tensor (Sec. 4.3; Alg. 3 with the second moment kept
// as row and column statistics instead of a compressed tensor).  R (rows floats) and C (cols floats)
// are updated in place.  v_t_out (rows*cols floats, may be null) receives the reconstructed second
// moment the update used, m_t_out the precise first moment.
void oracle_adamw4_factor_step(float* w, const float* g, uint8_t* m_codes, float* m_scales, float* R,
                               float* C, int64_t rows, int64_t cols, float lr, float beta1,
                               float beta2, float eps, float wd, int64_t t, float* m_t_out,
                               float* v_t_out) {
    const int64_t P = rows * cols;
    std::vector<float> m(static_cast<size_t>(P));
    dequant_m(m_codes, m_scales, P, m.data());                    // Alg. 3: decompress

    // row and column sums of the squared gradient, then their moving averages (the role v_t has in Eq. 1)
    std::vector<double> row_sq(static_cast<size_t>(rows), 0.0), col_sq(static_cast<size_t>(cols), 0.0);
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            const double sq = double(g[i * cols + j]) * double(g[i * cols + j]);
            row_sq[size_t(i)] += sq;
            col_sq[size_t(j)] += sq;
        }
    const double b2 = double(beta2);
    for (int64_t i = 0; i < rows; ++i) R[i] = float(b2 * double(R[i]) + (1.0 - b2) * row_sq[size_t(i)]);
    for (int64_t j = 0; j < cols; ++j) C[j] = float(b2 * double(C[j]) + (1.0 - b2) * col_sq[size_t(j)]);
    double total = 0.0;
    for (int64_t i = 0; i < rows; ++i) total += double(R[i]);

    const float omb1 = 1.0f - beta1;
    const double bc1 = 1.0 - std::pow(double(beta1), double(t));
    const double bc2 = 1.0 - std::pow(b2, double(t));
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            const int64_t e = i * cols + j;
            const float mt = std::fmaf(beta1, m[size_t(e)], omb1 * g[e]);      // Eq. 1, as in adamw_rule
            m[size_t(e)] = mt;
            const double vt = total > 0.0 ? double(R[i]) * double(C[j]) / total : 0.0;
            if (v_t_out) v_t_out[e] = float(vt);
            const double mhat = double(mt) / bc1;
            const double vhat = vt / bc2;
            const double wi = double(w[e]);
            w[e] = float(wi - double(lr) * (mhat / (std::sqrt(vhat) + double(eps)) + double(wd) * wi));
        }
    if (m_t_out) std::memcpy(m_t_out, m.data(), sizeof(float) * size_t(P));
    quant_m(m.data(), P, m_codes, m_scales);                      // Alg. 3: compress
}
// zero state of the factorized form: m as everywhere, R = C = 0
void oracle_state_zero_factor(uint8_t* m_codes, float* m_scales, float* R, float* C, int64_t rows,
                              int64_t cols) {
    const int64_t P = rows * cols;
    std::vector<float> z(static_cast<size_t>(P), 0.0f);
    quant_m(z.data(), P, m_codes, m_scales);
    for (int64_t i = 0; i < rows; ++i) R[i] = 0.0f;
    for (int64_t j = 0; j < cols; ++j) C[j] = 0.0f;
}

// The zero initial state of Alg. 3 (m_0 = v_0 = 0): m codes all point at the table's 0 entry with
// zero scales; the Linear map has no zero, so v = 0 is carried by r = c = 0.
void oracle_state_zero(uint8_t* m_codes, float* m_scales, uint8_t* v_codes, float* v_r, float* v_c,
                       int64_t rows, int64_t cols) {
    const int64_t P = rows * cols;
    std::vector<float> z(static_cast<size_t>(P), 0.0f);
    quant_m(z.data(), P, m_codes, m_scales);
    quant_v(z.data(), rows, cols, v_codes, v_r, v_c);
}

}  // extern "C"
