// Kernels of the 4-bit AdamW step (gfx950, wave64, 256-thread workgroups).
//
// Work unit: a "group" of 16 consecutive lanes (one DPP row) owns one 128-element block of the
// row-major flattening; each lane owns 8 consecutive elements, i.e. one 32-bit word of 4-bit codes
// of each moment, one 128-bit word of bf16 gradient and two 128-bit words of fp32 parameter.
//
// One step is two launches, because every v code needs the complete row and column maxima of the
// updated second moment (rank-1 normalization, paper Sec. 4.2):
//   pass 1: decompress m, v -> Adam moments (Eq. 1) -> parameter update -> block absmax of m_t,
//           compress m_t (B128 + signed dynamic-exponent map) -> row/column maxima of v_t into
//           the workspace (LDS combine, then integer atomic max on the float bits).
//   pass 2: recompute v_t with the identical operation sequence, compress it against
//           min(r'_i, c'_j) (Linear map), and let the last workgroup publish r', c' as the new
//           state and clear the workspace.
#pragma once

#include "device_math.hpp"

namespace lpmm {

// Lookup tables, uploaded once per device at init.
__device__ float d_byte_decode[512];          // entry b: {T_DE[b & 15], T_DE[b >> 4]}
__device__ SearchEntry d_search[kBuckets];    // nearest-entry search for the DE map

struct Tensor4 {
    float* p;               // parameters, fp32 [P]
    const void* g;          // gradient, fp32 or bf16 [P]
    uint32_t* mq;           // first-moment codes, 8 per word
    float* ms;              // first-moment block scales
    uint32_t* vq;           // second-moment codes
    float* r;               // row maxima (state)
    float* c;               // column maxima (state)
    float* r_new;           // workspace: row maxima of v_t (zero between steps)
    float* c_new;           // workspace: column maxima of v_t (zero between steps)
    unsigned int* counter;  // workspace: finished-workgroup counter of pass 2 (zero between steps)
    int64_t rows, cols, P;
    // geometry of the fast path (cols % 128 == 0)
    int nb;                 // column blocks per row = cols / 128
    int gx, gy;             // a workgroup's 16 groups: gx column blocks x gy row phases
    int rw;                 // rows per workgroup tile
    int strips;             // ceil(nb / gx)
    int n_wg;               // strips * ceil(rows / rw)
};

constexpr int kThreads = 256;
constexpr int kXcds = 8;

// Workgroups are dealt to the 8 XCDs round-robin by their id.  Remap so that consecutive logical
// ids -- which touch neighbouring memory -- run on the same XCD and share its L2.
__device__ __forceinline__ int logical_wg() {
    const int per_xcd = gridDim.x / kXcds;   // the grid is padded to a multiple of 8
    return (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
}

__device__ __forceinline__ void load_tables(float2* s_deq, SearchEntry* s_search) {
    const float2* gd = reinterpret_cast<const float2*>(d_byte_decode);
    for (int i = threadIdx.x; i < 256; i += kThreads) s_deq[i] = gd[i];
    const uint2* gs = reinterpret_cast<const uint2*>(d_search);
    uint2* ss = reinterpret_cast<uint2*>(s_search);
    for (int i = threadIdx.x; i < kBuckets; i += kThreads) ss[i] = gs[i];
}

// =====================================================================================================
// Fast path: cols % 128 == 0, so a block never straddles a row and a group can walk down the rows
// of one column block with the 8 old and 8 running new column maxima of its lane in registers.
// The loads of the next row are issued before the current row is computed.
// =====================================================================================================

struct Geo {            // where this group works
    int strip, tile, grp, l, gxi, gyi, cb;
    int64_t row0, row1, col0;
    bool active;
};

__device__ __forceinline__ Geo geometry(const Tensor4& a, int wg) {
    Geo g;
    g.strip = wg % a.strips;
    g.tile = wg / a.strips;
    g.grp = threadIdx.x >> 4;
    g.l = threadIdx.x & 15;
    g.gxi = g.grp % a.gx;
    g.gyi = g.grp / a.gx;
    g.cb = g.strip * a.gx + g.gxi;
    g.row0 = int64_t(g.tile) * a.rw;
    g.row1 = (g.row0 + a.rw < a.rows) ? g.row0 + a.rw : a.rows;
    g.col0 = int64_t(g.cb) * 128 + g.l * 8;
    g.active = g.cb < a.nb;
    return g;
}

__device__ __forceinline__ void load8(const float* p, float out[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
    out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}

template <bool BF16> struct GradRegs;
template <> struct GradRegs<true> { uint4 w; };
template <> struct GradRegs<false> { float4 a, b; };

template <bool BF16>
__device__ __forceinline__ GradRegs<BF16> load_grad_regs(const void* g, int64_t idx) {
    GradRegs<BF16> r;
    if constexpr (BF16) {
        r.w = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(g) + idx);
    } else {
        const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(g) + idx);
        r.a = p[0];
        r.b = p[1];
    }
    return r;
}
template <bool BF16>
__device__ __forceinline__ void unpack_grad(const GradRegs<BF16>& r, float out[8]) {
    if constexpr (BF16) {
        out[0] = bf16_lo(r.w.x); out[1] = bf16_hi(r.w.x);
        out[2] = bf16_lo(r.w.y); out[3] = bf16_hi(r.w.y);
        out[4] = bf16_lo(r.w.z); out[5] = bf16_hi(r.w.z);
        out[6] = bf16_lo(r.w.w); out[7] = bf16_hi(r.w.w);
    } else {
        out[0] = r.a.x; out[1] = r.a.y; out[2] = r.a.z; out[3] = r.a.w;
        out[4] = r.b.x; out[5] = r.b.y; out[6] = r.b.z; out[7] = r.b.w;
    }
}

// float(code) of a lane's 8 codes: split the word into low and high nibbles, then byte converts
__device__ __forceinline__ void codes_to_float(uint32_t w, float qf[8]) {
    const uint32_t lo = w & 0x0F0F0F0Fu, hi = (w >> 4) & 0x0F0F0F0Fu;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        qf[2 * k] = float((lo >> (8 * k)) & 255u);
        qf[2 * k + 1] = float((hi >> (8 * k)) & 255u);
    }
}

template <bool BF16>
struct Row1 {                      // everything pass 1 reads for one row of one lane
    float4 p0, p1;
    GradRegs<BF16> g;
    uint32_t mq, vq;
    float s_old, r_old;
};

template <bool BF16>
__device__ __forceinline__ Row1<BF16> load_row1(const Tensor4& a, const Geo& g, int64_t i) {
    Row1<BF16> r;
    const int64_t e0 = i * a.cols + g.col0;
    const float4* pp = reinterpret_cast<const float4*>(a.p + e0);
    r.p0 = pp[0];
    r.p1 = pp[1];
    r.g = load_grad_regs<BF16>(a.g, e0);
    r.mq = a.mq[e0 >> 3];
    r.vq = a.vq[e0 >> 3];
    r.s_old = a.ms[i * a.nb + g.cb];
    r.r_old = a.r[i];
    return r;
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void pass1_fast(const Tensor4 a, const Hyper h) {
    __shared__ float2 s_deq[256];
    __shared__ SearchEntry s_search[kBuckets];
    __shared__ float s_col[16 * 128];

    const int wg = logical_wg();
    if (wg >= a.n_wg) return;
    load_tables(s_deq, s_search);
    __syncthreads();

    const Geo geo = geometry(a, wg);
    float cmax[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) cmax[e] = 0.0f;

    if (geo.active) {
        float cold[8], cold16[8];
        load8(a.c + geo.col0, cold);
        bool cols_tame = true;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            cols_tame = cols_tame && scale_is_tame(cold[e]);
            cold16[e] = cold[e] * 0.0625f;
        }
        const int64_t stride = a.gy;
        int64_t i = geo.row0 + geo.gyi;
        Row1<BF16> cur;
        if (i < geo.row1) cur = load_row1<BF16>(a, geo, i);
        while (i < geo.row1) {
            const int64_t inext = i + stride;
            Row1<BF16> nxt;
            if (inext < geo.row1) nxt = load_row1<BF16>(a, geo, inext);

            const int64_t e0 = i * a.cols + geo.col0;
            float w[8] = {cur.p0.x, cur.p0.y, cur.p0.z, cur.p0.w, cur.p1.x, cur.p1.y, cur.p1.z, cur.p1.w};
            float g[8];
            unpack_grad<BF16>(cur.g, g);
            float mt[8], vt[8], amax = 0.0f, rmax = 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float2 t = s_deq[(cur.mq >> (8 * k)) & 255u];
                mt[2 * k] = t.x * cur.s_old;          // decompress: T_DE[code] * block scale
                mt[2 * k + 1] = t.y * cur.s_old;
            }
            // the wave takes the exact route for this row if any of its scales is extreme
            const bool tame_in = cols_tame && scale_is_tame(cur.r_old);
            if (__builtin_expect(__ballot(!tame_in) == 0, 1)) {
                float qf[8];
                codes_to_float(cur.vq, qf);
                const float r16 = cur.r_old * 0.0625f;
#pragma unroll
                for (int e = 0; e < 8; ++e) vt[e] = dequant_v16(qf[e], fminf(r16, cold16[e]));
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) vt[e] = dequant_v((cur.vq >> (4 * e)) & 15u, fminf(cur.r_old, cold[e]));
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                mt[e] = moment_m(h, mt[e], g[e]);
                vt[e] = moment_v(h, vt[e], g[e]);
                w[e] = param_update(h, w[e], mt[e], vt[e]);
                amax = fmaxf(amax, fabsf(mt[e]));
                rmax = fmaxf(rmax, vt[e]);
                cmax[e] = fmaxf(cmax[e], vt[e]);
            }
            const float s_new = row16_allmax(amax);     // block absmax of m_t
            rmax = row16_allmax(rmax);

            uint32_t mq_new = 0;
            float slack = 1.0f;
            if (scale_is_tame(s_new)) {
                const float inv_s = approx_inv(s_new);
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    float sa, sb;
                    mq_new |= quant_m_code_fast(s_search, mt[e], inv_s, sa) << (4 * e);
                    mq_new |= quant_m_code_fast(s_search, mt[e + 1], inv_s, sb) << (4 * e + 4);
                    slack = fminf(fminf(slack, sa), sb);
                }
            } else {
                slack = -1.0f;
            }
            if (__builtin_expect(__ballot(slack < 0.0f) != 0, 0)) {
                mq_new = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) mq_new |= quant_m_code(s_search, mt[e], s_new) << (4 * e);
            }

            float4* pp = reinterpret_cast<float4*>(a.p + e0);
            pp[0] = make_float4(w[0], w[1], w[2], w[3]);
            pp[1] = make_float4(w[4], w[5], w[6], w[7]);
            a.mq[e0 >> 3] = mq_new;
            if (geo.l == 0) {
                a.ms[i * a.nb + geo.cb] = s_new;
                if (rmax > 0.0f) atomic_max_nonneg(a.r_new + i, rmax);
            }
            cur = nxt;
            i = inext;
        }
    }

    // column maxima: combine the gy groups that share a column block, then one atomic per column
#pragma unroll
    for (int e = 0; e < 8; ++e) s_col[geo.grp * 128 + geo.l * 8 + e] = cmax[e];
    __syncthreads();
    for (int t = threadIdx.x; t < a.gx * 128; t += kThreads) {
        const int gi = t >> 7;
        float m = 0.0f;
        for (int y = 0; y < a.gy; ++y) m = fmaxf(m, s_col[((y * a.gx + gi) << 7) + (t & 127)]);
        const int cbi = geo.strip * a.gx + gi;
        if (cbi < a.nb && m > 0.0f) atomic_max_nonneg(a.c_new + int64_t(cbi) * 128 + (t & 127), m);
    }
}

// The last workgroup of pass 2 to finish makes r', c' the state and clears the workspace.  Every
// other workgroup has read the old r, c before it took its ticket, so overwriting them is safe.
// Tickets are taken in two levels (kTicketLanes first-level counters, one cache line apart, then
// one top counter) so that thousands of workgroups do not queue up on a single address.
constexpr int kTicketLanes = 32;
constexpr int kTicketStride = 32;   // in 32-bit words: 128 bytes

__device__ __forceinline__ void publish_if_last(const Tensor4& a) {
    __shared__ int s_last;
    __syncthreads();
    if (threadIdx.x == 0) {
        // No fence: the ticket orders nothing but "this workgroup's loads of r, c have returned",
        // which holds once its waves have computed their codes and reached the barrier above.  (An
        // agent-scope release here would write back the XCD's whole L2 once per workgroup.)
        const unsigned int n_wg = gridDim.x;
        const unsigned int lane = blockIdx.x % kTicketLanes;
        const unsigned int in_lane = n_wg / kTicketLanes + (lane < n_wg % kTicketLanes ? 1u : 0u);
        int last = 0;
        if (atomicAdd(a.counter + (1 + lane) * kTicketStride, 1u) == in_lane - 1) {
            a.counter[(1 + lane) * kTicketStride] = 0u;      // this lane is complete: reset it
            const unsigned int lanes_used = n_wg < kTicketLanes ? n_wg : kTicketLanes;
            last = atomicAdd(a.counter, 1u) == lanes_used - 1;
        }
        s_last = last;
    }
    __syncthreads();
    if (!s_last) return;
    for (int64_t i = threadIdx.x; i < a.rows; i += kThreads) { a.r[i] = a.r_new[i]; a.r_new[i] = 0.0f; }
    for (int64_t j = threadIdx.x; j < a.cols; j += kThreads) { a.c[j] = a.c_new[j]; a.c_new[j] = 0.0f; }
    if (threadIdx.x == 0) *a.counter = 0u;
}

template <bool BF16>
struct Row2 {                      // everything pass 2 reads for one row of one lane
    GradRegs<BF16> g;
    uint32_t vq;
    float r_old, r_new;
};

template <bool BF16>
__device__ __forceinline__ Row2<BF16> load_row2(const Tensor4& a, const Geo& g, int64_t i) {
    Row2<BF16> r;
    const int64_t e0 = i * a.cols + g.col0;
    r.g = load_grad_regs<BF16>(a.g, e0);
    r.vq = a.vq[e0 >> 3];
    r.r_old = a.r[i];
    r.r_new = a.r_new[i];
    return r;
}

template <bool BF16>
__device__ __forceinline__ uint32_t pass2_row(const Hyper& h, const Row2<BF16>& row, const float cold[8],
                                              const float cold16[8], const float cnew[8],
                                              const float inv_cnew[8], bool cols_tame) {
    float g[8], vt[8];
    unpack_grad<BF16>(row.g, g);
    const bool tame = cols_tame && scale_is_tame(row.r_old) && scale_is_tame(row.r_new);
    const bool fast = __ballot(!tame) == 0;
    if (__builtin_expect(fast, 1)) {
        float qf[8];
        codes_to_float(row.vq, qf);
        const float r16 = row.r_old * 0.0625f;
#pragma unroll
        for (int e = 0; e < 8; ++e) vt[e] = moment_v(h, dequant_v16(qf[e], fminf(r16, cold16[e])), g[e]);
        const float inv_r = approx_inv(row.r_new);
        // even elements collect in the bytes of `lo`, odd ones in `hi`; word = lo | hi << 4
        uint32_t lo = 0, hi = 0;
        float fmin_ = 0.5f, fmax_ = 0.5f, fa, fb;
#define LPMM_V2(K)                                                                                        \
        lo = quant_v_code_fast<K>(vt[2 * K], fmaxf(inv_r, inv_cnew[2 * K]), lo, fa);                      \
        hi = quant_v_code_fast<K>(vt[2 * K + 1], fmaxf(inv_r, inv_cnew[2 * K + 1]), hi, fb);              \
        fmin_ = fminf(fminf(fmin_, fa), fb);                                                              \
        fmax_ = fmaxf(fmaxf(fmax_, fa), fb);
        LPMM_V2(0) LPMM_V2(1) LPMM_V2(2) LPMM_V2(3)
#undef LPMM_V2
        const bool near = fmin_ < kMarginV || fmax_ > 1.0f - kMarginV;
        if (__builtin_expect(__ballot(near) == 0, 1)) return lo | (hi << 4);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            vt[e] = moment_v(h, dequant_v((row.vq >> (4 * e)) & 15u, fminf(row.r_old, cold[e])), g[e]);
    }
    uint32_t out = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) out |= quant_v_code(vt[e], fminf(row.r_new, cnew[e])) << (4 * e);
    return out;
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void pass2_fast(const Tensor4 a, const Hyper h) {
    const int wg = logical_wg();
    if (wg < a.n_wg) {
        const Geo geo = geometry(a, wg);
        if (geo.active) {
            float cold[8], cold16[8], cnew[8], inv_cnew[8];
            load8(a.c + geo.col0, cold);
            load8(a.c_new + geo.col0, cnew);
            bool cols_tame = true;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                cols_tame = cols_tame && scale_is_tame(cold[e]) && scale_is_tame(cnew[e]);
                cold16[e] = cold[e] * 0.0625f;
                inv_cnew[e] = approx_inv(cnew[e]);
            }
            // two rows per stage, the next stage's loads in flight while this one is computed
            const int64_t stride = a.gy;
            int64_t i = geo.row0 + geo.gyi;
            Row2<BF16> c0, c1;
            if (i < geo.row1) c0 = load_row2<BF16>(a, geo, i);
            if (i + stride < geo.row1) c1 = load_row2<BF16>(a, geo, i + stride);
            while (i < geo.row1) {
                const int64_t j0 = i + 2 * stride, j1 = i + 3 * stride;
                Row2<BF16> n0, n1;
                if (j0 < geo.row1) n0 = load_row2<BF16>(a, geo, j0);
                if (j1 < geo.row1) n1 = load_row2<BF16>(a, geo, j1);
                a.vq[(i * a.cols + geo.col0) >> 3] = pass2_row<BF16>(h, c0, cold, cold16, cnew, inv_cnew, cols_tame);
                if (i + stride < geo.row1)
                    a.vq[((i + stride) * a.cols + geo.col0) >> 3] =
                        pass2_row<BF16>(h, c1, cold, cold16, cnew, inv_cnew, cols_tame);
                c0 = n0;
                c1 = n1;
                i = j0;
            }
        }
    }
    publish_if_last(a);
}

// =====================================================================================================
// General path: any rows x cols.  Lane t owns flat elements [8t, 8t+8); a group is still one block
// of 128, but a lane's elements may lie in different rows, so row and column indices are tracked
// per element and the maxima go straight to atomics (skipped when they cannot raise the value).
// =====================================================================================================

__device__ __forceinline__ void raise_max(float* addr, float v) {
    if (v > 0.0f && __float_as_uint(v) > __hip_atomic_load(reinterpret_cast<unsigned int*>(addr),
                                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomic_max_nonneg(addr, v);
}

struct LaneIo {
    int64_t base;   // first flat element of the lane
    int nv;         // valid elements, 0..8
    int64_t i;      // row of the first element
    int64_t j;      // column of the first element
};

__device__ __forceinline__ LaneIo lane_io(const Tensor4& a, int64_t lane_global) {
    LaneIo io;
    io.base = lane_global * 8;
    const int64_t left = a.P - io.base;
    io.nv = left >= 8 ? 8 : (left > 0 ? int(left) : 0);
    io.i = io.nv ? io.base / a.cols : 0;
    io.j = io.nv ? io.base - io.i * a.cols : 0;
    return io;
}

// code word of a lane: full lanes read one aligned word, the tail lane reads bytes
__device__ __forceinline__ uint32_t load_codes(const uint32_t* q, const LaneIo& io) {
    if (io.nv == 8) return q[io.base >> 3];
    const uint8_t* b = reinterpret_cast<const uint8_t*>(q) + (io.base >> 1);
    uint32_t w = 0;
    for (int k = 0; k < (io.nv + 1) / 2; ++k) w |= uint32_t(b[k]) << (8 * k);
    return w;
}
__device__ __forceinline__ void store_codes(uint32_t* q, const LaneIo& io, uint32_t w) {
    if (io.nv == 8) { q[io.base >> 3] = w; return; }
    uint8_t* b = reinterpret_cast<uint8_t*>(q) + (io.base >> 1);
    for (int k = 0; k < (io.nv + 1) / 2; ++k) b[k] = uint8_t(w >> (8 * k));
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void pass1_general(const Tensor4 a, const Hyper h) {
    __shared__ float2 s_deq[256];
    __shared__ SearchEntry s_search[kBuckets];
    load_tables(s_deq, s_search);
    __syncthreads();

    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const int64_t block = t >> 4;                       // uniform over the group
    if (block * 128 >= a.P) return;                     // whole group past the end
    const LaneIo io = lane_io(a, t);

    float w[8], g[8];
    if (io.nv == 8) {
        const float4* pp = reinterpret_cast<const float4*>(a.p + io.base);
        const float4 p0 = pp[0], p1 = pp[1];
        w[0] = p0.x; w[1] = p0.y; w[2] = p0.z; w[3] = p0.w;
        w[4] = p1.x; w[5] = p1.y; w[6] = p1.z; w[7] = p1.w;
        load_grad8<BF16>(a.g, io.base, g);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            w[e] = e < io.nv ? a.p[io.base + e] : 0.0f;
            g[e] = e < io.nv ? load_grad1<BF16>(a.g, io.base + e) : 0.0f;
        }
    }
    const uint32_t mq = load_codes(a.mq, io);
    const uint32_t vq = load_codes(a.vq, io);
    const float s_old = a.ms[block];

    float mt[8], amax = 0.0f;
    int64_t i = io.i, j = io.j;
    int64_t run_row = io.i;
    float run_max = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (e < io.nv) {
            const float2 tt = s_deq[(mq >> (8 * (e >> 1))) & 255u];
            const float m_prev = ((e & 1) ? tt.y : tt.x) * s_old;
            const float v_prev = dequant_v((vq >> (4 * e)) & 15u, fminf(a.r[i], a.c[j]));
            mt[e] = moment_m(h, m_prev, g[e]);
            const float vt = moment_v(h, v_prev, g[e]);
            w[e] = param_update(h, w[e], mt[e], vt);
            amax = fmaxf(amax, fabsf(mt[e]));
            if (i != run_row) { raise_max(a.r_new + run_row, run_max); run_row = i; run_max = 0.0f; }
            run_max = fmaxf(run_max, vt);
            raise_max(a.c_new + j, vt);
            if (++j == a.cols) { j = 0; ++i; }
        } else {
            mt[e] = 0.0f;
        }
    }
    if (io.nv) raise_max(a.r_new + run_row, run_max);

    const float s_new = row16_allmax(amax);
    uint32_t mq_new = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (e < io.nv) mq_new |= quant_m_code(s_search, mt[e], s_new) << (4 * e);

    if (io.nv == 8) {
        float4* pp = reinterpret_cast<float4*>(a.p + io.base);
        pp[0] = make_float4(w[0], w[1], w[2], w[3]);
        pp[1] = make_float4(w[4], w[5], w[6], w[7]);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (e < io.nv) a.p[io.base + e] = w[e];
    }
    if (io.nv) store_codes(a.mq, io, mq_new);
    if ((threadIdx.x & 15) == 0) a.ms[block] = s_new;
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void pass2_general(const Tensor4 a, const Hyper h) {
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(a, t);
    if (io.nv) {
        float g[8];
        if (io.nv == 8) {
            load_grad8<BF16>(a.g, io.base, g);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) g[e] = e < io.nv ? load_grad1<BF16>(a.g, io.base + e) : 0.0f;
        }
        const uint32_t vq = load_codes(a.vq, io);
        uint32_t vq_new = 0;
        int64_t i = io.i, j = io.j;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (e < io.nv) {
                const float v_prev = dequant_v((vq >> (4 * e)) & 15u, fminf(a.r[i], a.c[j]));
                const float vt = moment_v(h, v_prev, g[e]);
                vq_new |= quant_v_code(vt, fminf(a.r_new[i], a.c_new[j])) << (4 * e);
                if (++j == a.cols) { j = 0; ++i; }
            }
        }
        store_codes(a.vq, io, vq_new);
    }
    publish_if_last(a);
}

// =====================================================================================================
// Uncompressed fp32 states (tensors that are not quantized): Alg. 3 with identity compression.
// =====================================================================================================

template <bool BF16>
__global__ __launch_bounds__(kThreads) void adamw32_kernel(float* p, const void* g, float* m, float* v,
                                                           int64_t n, const Hyper h) {
    const int64_t stride = int64_t(gridDim.x) * kThreads;
    for (int64_t idx = int64_t(blockIdx.x) * kThreads + threadIdx.x; idx < n; idx += stride) {
        const float gi = load_grad1<BF16>(g, idx);
        const float mt = moment_m(h, m[idx], gi);
        const float vt = moment_v(h, v[idx], gi);
        m[idx] = mt;
        v[idx] = vt;
        p[idx] = param_update(h, p[idx], mt, vt);
    }
}

// =====================================================================================================
// Stand-alone decompress / compress of one moment, and the zero state.
// =====================================================================================================

struct QuantArgs {
    const uint32_t* q_in;   // dequant: codes
    uint32_t* q_out;        // quant: codes
    const float* x_in;      // quant: fp32 moment
    float* x_out;           // dequant: fp32 moment
    float* sa;              // block scales or row maxima
    float* sb;              // column maxima (second moment)
    int64_t rows, cols, P;
};

__device__ __forceinline__ Tensor4 as_tensor(const QuantArgs& q) {
    Tensor4 a{};
    a.rows = q.rows; a.cols = q.cols; a.P = q.P;
    return a;
}

__global__ __launch_bounds__(kThreads) void dequant_m_kernel(const QuantArgs q) {
    const Tensor4 a = as_tensor(q);
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(a, t);
    if (!io.nv) return;
    const uint32_t w = load_codes(q.q_in, io);
    const float s = q.sa[t >> 4];
    for (int e = 0; e < io.nv; ++e)
        q.x_out[io.base + e] = d_byte_decode[2 * ((w >> (4 * e)) & 15u)] * s;   // entry b<16: {T[b], T[0]}
}

__global__ __launch_bounds__(kThreads) void dequant_v_kernel(const QuantArgs q) {
    const Tensor4 a = as_tensor(q);
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(a, t);
    if (!io.nv) return;
    const uint32_t w = load_codes(q.q_in, io);
    int64_t i = io.i, j = io.j;
    for (int e = 0; e < io.nv; ++e) {
        q.x_out[io.base + e] = dequant_v((w >> (4 * e)) & 15u, fminf(q.sa[i], q.sb[j]));
        if (++j == q.cols) { j = 0; ++i; }
    }
}

__global__ __launch_bounds__(kThreads) void quant_m_kernel(const QuantArgs q) {
    __shared__ float2 s_deq[256];
    __shared__ SearchEntry s_search[kBuckets];
    load_tables(s_deq, s_search);
    __syncthreads();
    const Tensor4 a = as_tensor(q);
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    if ((t >> 4) * 128 >= q.P) return;
    const LaneIo io = lane_io(a, t);
    float x[8], amax = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        x[e] = e < io.nv ? q.x_in[io.base + e] : 0.0f;
        amax = fmaxf(amax, fabsf(x[e]));
    }
    const float s = row16_allmax(amax);
    uint32_t w = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (e < io.nv) w |= quant_m_code(s_search, x[e], s) << (4 * e);
    if (io.nv) store_codes(q.q_out, io, w);
    if ((threadIdx.x & 15) == 0) q.sa[t >> 4] = s;
}

// second moment, stage 1: row / column maxima into sa / sb (which must be zero on entry)
__global__ __launch_bounds__(kThreads) void quant_v_max_kernel(const QuantArgs q) {
    const Tensor4 a = as_tensor(q);
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(a, t);
    int64_t i = io.i, j = io.j;
    for (int e = 0; e < io.nv; ++e) {
        const float x = q.x_in[io.base + e];
        raise_max(q.sa + i, x);
        raise_max(q.sb + j, x);
        if (++j == q.cols) { j = 0; ++i; }
    }
}

// second moment, stage 2: codes against min(r_i, c_j)
__global__ __launch_bounds__(kThreads) void quant_v_code_kernel(const QuantArgs q) {
    const Tensor4 a = as_tensor(q);
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(a, t);
    if (!io.nv) return;
    uint32_t w = 0;
    int64_t i = io.i, j = io.j;
    for (int e = 0; e < io.nv; ++e) {
        w |= quant_v_code(q.x_in[io.base + e], fminf(q.sa[i], q.sb[j])) << (4 * e);
        if (++j == q.cols) { j = 0; ++i; }
    }
    store_codes(q.q_out, io, w);
}

// fill `n` bytes at dst with `value`, and force the byte at index `last_index` (if >= 0) to `last`
__global__ __launch_bounds__(kThreads) void fill_bytes_kernel(uint8_t* dst, int64_t n, uint8_t value,
                                                              int64_t last_index, uint8_t last) {
    const int64_t stride = int64_t(gridDim.x) * kThreads;
    for (int64_t i = int64_t(blockIdx.x) * kThreads + threadIdx.x; i < n; i += stride)
        dst[i] = (i == last_index) ? last : value;
}

}  // namespace lpmm
