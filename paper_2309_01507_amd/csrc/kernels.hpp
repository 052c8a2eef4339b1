// Kernels of the 4-bit AdamW step (gfx950, wave64, 256-thread workgroups).
//
// Work unit: a group of lanes owns one 128-element block of the row-major flattening.  On the fast
// path (cols % 128 == 0) that is 32 lanes with 4 consecutive elements each; on the general path 16
// lanes (one DPP row) with 8 consecutive elements each.
//
// One step is two passes, because every v code needs the complete row and column maxima of the
// updated second moment (rank-1 normalization, paper Sec. 4.2):
//   pass 1: decompress m, v -> Adam moments (Eq. 1) -> parameter update -> block absmax of m_t,
//           compress m_t (B128 + signed dynamic-exponent map) -> row/column maxima of v_t into
//           the workspace (LDS combine, then integer atomic max on the float bits).
//   pass 2: recompute v_t with the identical operation sequence, compress it against
//           min(r'_i, c'_j) (Linear map), and let the last workgroup publish r', c' as the new
//           state and clear the workspace.
// For 1-dimensional or flattened tensors the second moment is block-wise like the first (Sec. 4.2,
// last paragraph); then nothing crosses a block and the step is ONE pass (b128_*).  The same one-pass
// code without a second moment is SGD with momentum (App. E Alg. 2).  With a factorized second
// moment (Sec. 4.3, factor_*) the two passes are: row / column sums of g^2, then the update.  Tensors
// with more than two dimensions (App. F Alg. 4, nd_*) run the two matrix passes on derived column scales.
// The bodies are "tile" functions; thin __global__ wrappers run them for one tensor (two launches
// per step, one for the block-wise form), and the phase kernels run pass 1 of one set of tensors
// next to pass 2 of the previous set, so that the arithmetic-heavy pass 2 hides under the
// memory-bound pass 1.
#pragma once

#include <cstddef>

#include "device_math.hpp"

namespace lpmm {

// Lookup tables, uploaded once per device at init.
__device__ float d_byte_decode[512];          // entry b: {T_DE[b & 15], T_DE[b >> 4]}
__device__ SearchEntry d_search[kBucketsPadded];    // nearest-entry search for the DE map

enum TensorKind : int { kQuantFast = 0, kQuantGeneral = 1, kFp32State = 2, kQuantBlockV = 3, kFactorFast = 4, kFactorGeneral = 5,
                        kSgdmBlock = 6, kSgdmFp32 = 7 };

struct Tensor4 {
    float* p;               // parameters, fp32 [P]
    const void* g;          // gradient, fp32 or bf16 [P]
    uint32_t* mq;           // first-moment codes, 8 per word   (kFp32State: float* m)
    float* ms;              // first-moment block scales
    uint32_t* vq;           // second-moment codes              (kFp32State: float* v)
    float* r;               // row maxima (state)               (kQuantBlockV: block scales of v; kFactor*: row statistics)
    float* c;               // column maxima (state)            (kFactor*: column statistics)
    float* r_new;           // workspace: row maxima of v_t (zero between steps)      (kFactor*: row sums of g^2)
    float* c_new;           // workspace: column maxima of v_t (zero between steps)   (kFactor*: column sums of g^2)
    unsigned int* counter;  // workspace: ticket counters of pass 2 (zero between steps); kFactor*: also two float sums
    int64_t rows, cols, P;
    // geometry of the fast path (cols % 128 == 0)
    int nb;                 // column blocks per row = cols / 128    (kQuantBlockV: whole blocks of the tensor)
    int gx, gy;             // a workgroup's 8 groups: gx column blocks x gy row phases
    int rw;                 // rows per workgroup tile; rw * cols < 2^29   (kQuantBlockV, kSgdmBlock: blocks a group takes in
                            // a row; general path: chunks of 2048 elements a workgroup of the first pass takes)
    int strips;             // nb / gx
    int n_wg;               // workgroups of pass 1 (kQuantBlockV, kSgdmBlock: of the step;
                            // kFactor*: of the statistics pass, which is tiled like pass 2)
    int kind;
    // pass 2 of the fast path has its own tiling: strips of 256 columns, rw2 rows per workgroup
    int strips2;            // ceil(nb / 2)
    int rw2;                // rw2 * cols < 2^29
    int n_wg2;              // workgroups of pass 2                 (kQuantBlockV: workgroups on whole blocks;
                            // kFactor*: of the update pass, which is tiled like pass 1)
    // log2 of the row spacing of pass 1 / pass 2: the 2^rs (2^rs2) rows that a group (a wave) takes in a
    // row are consecutive, and the groups (waves) that run side by side are 2^rs rows apart
    int rs, rs2;
    int tot_slots;          // kFactor*: slots that each of the two float sums is spread over (1, 2, 4 or 8)
    int flat;               // kQuantFast: pass 1 uses the flat tiling (a group walks along a row)
    int no_decay;           // plans: this tensor takes no weight decay
    int c_extra;            // floats behind c_new (and room behind c) that the publishing workgroup moves and clears
                            // along with the column maxima (tensors with more than two dimensions)
    int nd_index;           // plans: index into the plan's table of inner dimensions, -1 for matrices
    int det;                // kFactorFast in a plan: the sums of g^2 are reduced in a fixed order (no float atomics);
                            // vq then points at the partial sums: float[strips2][round_up(rows, 64)] per strip and row,
                            // then float[tiles][round_up(cols, 64)] per row tile and column
};

// The tensor table of a plan lives in device memory.  A pointer read from memory is a generic
// pointer to the compiler, and accesses through it would become flat instructions: slower, and
// counted together with LDS traffic, so that every wait for a table lookup would also wait for the
// rows being prefetched.  On the device the table is therefore read through a twin of Tensor4 whose
// pointer members are typed as global memory (same layout), and converted member by member.
#if defined(__HIP_DEVICE_COMPILE__)
#define LPMM_AS_GLOBAL __attribute__((address_space(1)))
struct Tensor4Table {
    float LPMM_AS_GLOBAL* p;
    const void LPMM_AS_GLOBAL* g;
    uint32_t LPMM_AS_GLOBAL* mq;
    float LPMM_AS_GLOBAL* ms;
    uint32_t LPMM_AS_GLOBAL* vq;
    float LPMM_AS_GLOBAL* r;
    float LPMM_AS_GLOBAL* c;
    float LPMM_AS_GLOBAL* r_new;
    float LPMM_AS_GLOBAL* c_new;
    unsigned int LPMM_AS_GLOBAL* counter;
    int64_t rows, cols, P;
    int nb, gx, gy, rw, strips, n_wg, kind, strips2, rw2, n_wg2, rs, rs2, tot_slots, flat, no_decay, c_extra, nd_index, det;
};
static_assert(sizeof(Tensor4Table) == sizeof(Tensor4), "the table twin must mirror Tensor4");
__device__ __forceinline__ Tensor4 from_table(const Tensor4Table& t) {
    Tensor4 a;
    a.p = (float*)t.p;
    a.g = (const void*)t.g;
    a.mq = (uint32_t*)t.mq;
    a.ms = (float*)t.ms;
    a.vq = (uint32_t*)t.vq;
    a.r = (float*)t.r;
    a.c = (float*)t.c;
    a.r_new = (float*)t.r_new;
    a.c_new = (float*)t.c_new;
    a.counter = (unsigned int*)t.counter;
    a.rows = t.rows; a.cols = t.cols; a.P = t.P;
    a.nb = t.nb; a.gx = t.gx; a.gy = t.gy; a.rw = t.rw; a.strips = t.strips; a.n_wg = t.n_wg; a.kind = t.kind;
    a.strips2 = t.strips2; a.rw2 = t.rw2; a.n_wg2 = t.n_wg2; a.rs = t.rs; a.rs2 = t.rs2;
    a.tot_slots = t.tot_slots; a.flat = t.flat; a.no_decay = t.no_decay; a.c_extra = t.c_extra; a.nd_index = t.nd_index; a.det = t.det;
    return a;
}
#else
typedef Tensor4 Tensor4Table;
__host__ __device__ inline Tensor4 from_table(const Tensor4& t) { return t; }   // host pass: only parsed, never run
#endif

constexpr int kThreads = 256;
constexpr int kXcds = 8;
constexpr int kElemsPerWg32 = kThreads * 16;   // fp32-state path: elements per workgroup

// Workgroups are dealt to the 8 XCDs round-robin by their id.  Remap so that consecutive logical
// ids -- which touch neighbouring memory -- run on the same XCD and share its L2.
__device__ __forceinline__ int logical_wg() {
    const int per_xcd = gridDim.x / kXcds;   // the grid is padded to a multiple of 8
    return (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
}

constexpr int kWaitVmcnt0 = 0x0F70;   // s_waitcnt vmcnt(0) only: expcnt and lgkmcnt fields at their maxima
constexpr int kMaxRowSlots = 512;    // rows of a pass-1 tile x column blocks of its strip (rw * gx)

struct Lds {
    float2 deq[256];
    SearchEntry search[kBucketsPadded];
    float col[8 * 128];
    float cold[8 * 128];        // flat tiling of pass 1: the strip's old column maxima / 16
    // per row and column block of the tile: new block scale of m and the block's maximum of v_t.
    // They leave for global memory at the end of the tile, so that the row loop issues the same
    // memory instructions on every path (loads, the parameter store, the code store) and nothing
    // that depends on the lane.
    float blk_scale[kMaxRowSlots];
    float blk_vmax[kMaxRowSlots];
};

__device__ __forceinline__ void load_tables(Lds& s) {
    const float2* gd = reinterpret_cast<const float2*>(d_byte_decode);
    for (int i = threadIdx.x; i < 256; i += kThreads) s.deq[i] = gd[i];
    const uint2* gs = reinterpret_cast<const uint2*>(d_search);
    uint2* ss = reinterpret_cast<uint2*>(s.search);
    for (int i = threadIdx.x; i < kBucketsPadded; i += kThreads) ss[i] = gs[i];
    __syncthreads();
}

// ---- small helpers -----------------------------------------------------------------------------------

// min / max of two floats that are both >= +0, through the integer units (no NaN canonicalization)
__device__ __forceinline__ float min_nonneg(float a, float b) {
    const uint32_t x = __float_as_uint(a), y = __float_as_uint(b);
    return __uint_as_float(x < y ? x : y);
}
__device__ __forceinline__ float max_nonneg(float a, float b) {
    const uint32_t x = __float_as_uint(a), y = __float_as_uint(b);
    return __uint_as_float(x > y ? x : y);
}

// Streaming 128-bit access for the parameters: they are read and written exactly once per step.
// The loads carry the non-temporal hint; the stores go out with the nt and sc1 cache-policy bits (write
// through, do not keep the line).  Measured on the 7B-shaped set: about 9 % less time per step than plain
// accesses for nt on both, and a further 2-3 % of pass 1 for sc1 on the store.
typedef float v4f_t __attribute__((ext_vector_type(4)));
typedef uint32_t v4u_t __attribute__((ext_vector_type(4)));
constexpr int kPolicyNtSc1 = 2 | 16;            // gfx94x/gfx950 cache-policy bits: 1 = sc0, 2 = nt, 16 = sc1
constexpr int kRawBufferWord3 = 0x00020000;     // untyped 32-bit data format, no swizzle, offsets in bytes

// Bounds-checked loads of the fast path.  A tile's arrays are described by raw buffer resources
// whose length is the tile's; a load beyond it returns zero and touches no memory.  The row
// prefetch can therefore run unconditionally past the end of a tile: no branch around the loads, so
// the compiler counts outstanding loads exactly and never waits for a row it has just requested.
typedef uint32_t v2u_t __attribute__((ext_vector_type(2)));
typedef __amdgpu_buffer_rsrc_t Rsrc;
constexpr int kPolicyNt = 2;
__device__ __forceinline__ Rsrc tile_rsrc(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, int(bytes), kRawBufferWord3);
}
__device__ __forceinline__ float4 buf_ld_f4_stream(Rsrc r, uint32_t off) {
    const v4f_t v = __builtin_bit_cast(v4f_t, __builtin_amdgcn_raw_buffer_load_b128(r, int(off), 0, kPolicyNt));
    return make_float4(v.x, v.y, v.z, v.w);
}
template <int POLICY = 0>
__device__ __forceinline__ float4 buf_ld_f4(Rsrc r, uint32_t off) {
    const v4f_t v = __builtin_bit_cast(v4f_t, __builtin_amdgcn_raw_buffer_load_b128(r, int(off), 0, POLICY));
    return make_float4(v.x, v.y, v.z, v.w);
}
template <int POLICY = 0>
__device__ __forceinline__ uint2 buf_ld_u2(Rsrc r, uint32_t off) {
    const v2u_t v = __builtin_amdgcn_raw_buffer_load_b64(r, int(off), 0, POLICY);
    return make_uint2(v.x, v.y);
}
// Kept 16 bits wide until it is used: widening right here would put an instruction that needs the
// value directly behind the load, and with it a wait for a row that was only just requested.
__device__ __forceinline__ uint16_t buf_ld_u16(Rsrc r, uint32_t off) {
    return uint16_t(__builtin_amdgcn_raw_buffer_load_b16(r, int(off), 0, 0));
}
__device__ __forceinline__ float buf_ld_f(Rsrc r, uint32_t off) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, int(off), 0, 0));
}

template <typename T>
__device__ __forceinline__ T ld(const void* base, uint32_t byte_off) {
    return *reinterpret_cast<const T*>(reinterpret_cast<const char*>(base) + byte_off);
}
template <typename T>
__device__ __forceinline__ void st(void* base, uint32_t byte_off, T v) {
    *reinterpret_cast<T*>(reinterpret_cast<char*>(base) + byte_off) = v;
}

__device__ __forceinline__ void load8(const float* p, float out[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
    out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}

// =====================================================================================================
// Fast path: cols % 128 == 0, so a block never straddles a row.  Here a lane owns FOUR consecutive
// elements of a row and a group of 32 lanes (half a wave) owns one 128-element block: a group's
// 128-bit parameter access is 512 contiguous bytes, and the per-lane register footprint lets five
// waves share a SIMD.  A group walks down rows of one column block with the old and the running new
// column maxima of its 4 columns in registers.  Loads go through bounds-checked buffer resources of
// the tile (uniform base, 32-bit lane offsets); the loads of the next two rows are in flight while a
// row is computed.
// =====================================================================================================

constexpr int kGroups = 8;          // 32-lane groups per workgroup

// maximum over the 32 lanes of a group of a value that is >= +0 everywhere, result in all 32 lanes
__device__ __forceinline__ float group32_allmax(float v) {
    uint32_t x = __float_as_uint(row16_allmax(v));
    // lane ^ 16 inside each half wave: swizzle in bit mode (and 0x1F, or 0, xor 0x10)
    const uint32_t y = uint32_t(__builtin_amdgcn_ds_swizzle(int(x), 0x401F));
    return __uint_as_float(x > y ? x : y);
}

template <bool BF16> struct GradRegs4;
template <> struct GradRegs4<true> { uint2 w; };
template <> struct GradRegs4<false> { float4 a; };

// gradient of a lane's 4 elements; off4 is the byte offset the elements have in an fp32 array.
// POLICY = kPolicyNt where the gradient is read for the last time in the step.
template <bool BF16, int POLICY = 0>
__device__ __forceinline__ GradRegs4<BF16> load_grad_regs4(Rsrc g_tile, uint32_t off4) {
    GradRegs4<BF16> r;
    if constexpr (BF16) r.w = buf_ld_u2<POLICY>(g_tile, off4 >> 1);
    else r.a = buf_ld_f4<POLICY>(g_tile, off4);
    return r;
}
template <bool BF16>
__device__ __forceinline__ void unpack_grad4(const GradRegs4<BF16>& r, float out[4]) {
    if constexpr (BF16) {
        out[0] = bf16_lo(r.w.x); out[1] = bf16_hi(r.w.x);
        out[2] = bf16_lo(r.w.y); out[3] = bf16_hi(r.w.y);
    } else {
        out[0] = r.a.x; out[1] = r.a.y; out[2] = r.a.z; out[3] = r.a.w;
    }
}

// float(code) of a lane's 4 codes (16 bits): split into low and high nibbles (kept opaque so that
// the byte-to-float converts are used), then one convert per element
__device__ __forceinline__ void codes_to_float4(uint32_t w, float qf[4]) {
    uint32_t lo = w & 0x0F0Fu, hi = (w >> 4) & 0x0F0Fu;
    asm("" : "+v"(lo));
    asm("" : "+v"(hi));
    qf[0] = float(lo & 255u);
    qf[1] = float(hi & 255u);
    qf[2] = float((lo >> 8) & 255u);
    qf[3] = float((hi >> 8) & 255u);
}

// il * pitch + x for a row index and a pitch that both fit 24 bits (rows of a tile; cols <= 2^24).
// The 24-bit multiply-add is a single 32-bit instruction; a full 32-bit multiply-add would go through
// the 64-bit one, whose unused upper addend register the compiler may alias with a register that a
// prefetch is still loading into, which turns into a wait for that prefetch.
__device__ __forceinline__ uint32_t row_offset(int il, int64_t pitch, uint32_t x) {
    return __umul24(uint32_t(il), uint32_t(pitch)) + x;
}

struct Geo {            // where this group works
    int strip, grp, l, gxi, gyi, cb;
    int64_t row0;
    int n_rows;         // rows of this tile
    uint32_t col0;      // first of the lane's 4 columns
    bool active;
};

__device__ __forceinline__ Geo geometry(const Tensor4& a, int wg) {
    Geo g;
    g.strip = wg % a.strips;
    const int tile = wg / a.strips;
    g.grp = threadIdx.x >> 5;
    g.l = threadIdx.x & 31;
    g.gxi = g.grp % a.gx;
    g.gyi = g.grp / a.gx;
    g.cb = g.strip * a.gx + g.gxi;
    g.row0 = int64_t(tile) * a.rw;
    const int64_t left = a.rows - g.row0;
    g.n_rows = left < a.rw ? int(left) : a.rw;
    g.col0 = uint32_t(g.cb) * 128u + uint32_t(g.l) * 4u;
    g.active = g.cb < a.nb;
    return g;
}

// uniform base pointers of a tile (row0 folded in), so that lane offsets fit 32 bits
struct TileBase {
    float* p;
    const char* g;
    uint8_t* mq;
    uint8_t* vq;
    float* ms;
    const float* r;
    float* r_new;
    // the same arrays as bounds-checked resources of n_rows rows, for the loads and the row stores
    Rsrc rp, rg, rmq, rvq, rr, rr_new;
};

template <bool BF16>
__device__ __forceinline__ TileBase tile_base(const Tensor4& a, int64_t row0, int n_rows) {
    TileBase b;
    const int64_t e = row0 * a.cols;
    const uint32_t elems = uint32_t(n_rows) * uint32_t(a.cols);       // < 2^29
    b.p = a.p + e;
    b.g = reinterpret_cast<const char*>(a.g) + e * (BF16 ? 2 : 4);
    b.mq = reinterpret_cast<uint8_t*>(a.mq) + (e >> 1);
    b.vq = reinterpret_cast<uint8_t*>(a.vq) + (e >> 1);
    b.ms = a.ms + row0 * a.nb;
    b.r = a.r + row0;
    b.r_new = a.r_new + row0;
    b.rp = tile_rsrc(b.p, elems * 4u);
    b.rg = tile_rsrc(b.g, elems * (BF16 ? 2u : 4u));
    b.rmq = tile_rsrc(b.mq, elems >> 1);
    b.rvq = tile_rsrc(b.vq, elems >> 1);
    b.rr = tile_rsrc(b.r, uint32_t(n_rows) * 4u);
    b.rr_new = tile_rsrc(b.r_new, uint32_t(n_rows) * 4u);
    return b;
}

__device__ __forceinline__ void load4(const float* p, float out[4]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
}

template <bool BF16>
struct Row1 {                      // everything pass 1 prefetches for one row of one lane
    float4 p;
    GradRegs4<BF16> g;
    uint16_t mq, vq;               // the lane's 4 codes of each moment
};

// The old block scales of m and the old row maxima of v of a tile are not prefetched per row (each would be a
// load of 4 bytes that all 32 lanes of a group share): the tile stages them in LDS once, in the slots that
// later take the new block scales and the new row maxima (s.blk_scale, s.blk_vmax).  A slot's old value is
// read by the same group that replaces it, earlier in program order.

// parameters and first-moment codes of a lane's 4 elements, through the tile's bounds-checked resources (no
// registers for a second set of base addresses)
__device__ __forceinline__ void store_row1(const TileBase& tb, uint32_t off4, const float w[4], uint32_t mq_new);

// il = row index inside the tile; rows at or beyond the tile's end read as zeros
template <bool BF16>
__device__ __forceinline__ Row1<BF16> load_row1(const TileBase& b, const Tensor4& a, const Geo& g, int il) {
    Row1<BF16> r;
    const uint32_t off4 = row_offset(il, a.cols, g.col0) * 4u;   // byte offset, fp32 array
    r.p = buf_ld_f4_stream(b.rp, off4);
    r.g = load_grad_regs4<BF16>(b.rg, off4);
    r.mq = buf_ld_u16(b.rmq, off4 >> 3);
    r.vq = buf_ld_u16(b.rvq, off4 >> 3);
    return r;
}

__device__ __forceinline__ void store_row1(const TileBase& tb, uint32_t off4, const float w[4], uint32_t mq_new) {
    const v4f_t v = {w[0], w[1], w[2], w[3]};
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u_t, v), tb.rp, int(off4), 0, kPolicyNtSc1);
    __builtin_amdgcn_raw_buffer_store_b16(short(mq_new), tb.rmq, int(off4 >> 3), 0, 0);
}

// Raise a running maximum in global memory, reading it first: the value only grows during a kernel,
// so an atomic that cannot change it is skipped.  For the general path, which would otherwise send
// an atomic per element.
__device__ __forceinline__ void raise_max(float* addr, float v) {
    if (v > 0.0f && __float_as_uint(v) > __hip_atomic_load(reinterpret_cast<unsigned int*>(addr),
                                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
        atomic_max_nonneg(addr, v);
}

// One row of pass 1 for one lane: `cur` holds what was loaded for row `il` of the tile.
template <bool BF16, class Mid>
__device__ __forceinline__ void pass1_row(const Tensor4& a, const Hyper& h, const TileBase& tb, const Geo& geo,
                                          Lds& s, const Row1<BF16>& cur, int il, const float cold16[4],
                                          bool cols_tame, float cmax[4], Mid mid) {
    float w[4] = {cur.p.x, cur.p.y, cur.p.z, cur.p.w};
    float g[4];
    unpack_grad4<BF16>(cur.g, g);
    float mt[4], vt[4], amax = 0.0f, rmax = 0.0f;
    const int slot = il * a.gx + geo.gxi;
    const float s_old = s.blk_scale[slot], r_old = s.blk_vmax[slot];     // staged by the tile
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const float2 t = s.deq[(uint32_t(cur.mq) >> (8 * k)) & 255u];
        mt[2 * k] = t.x * s_old;              // decompress: T_DE[code] * block scale
        mt[2 * k + 1] = t.y * s_old;
    }
    // the wave takes the exact route for this row if any of its scales is extreme
    const bool tame_in = bool(int(cols_tame) & int(scale_is_tame(r_old)));
    if (__builtin_expect(__ballot(!tame_in) == 0, 1)) {
        float qf[4];
        codes_to_float4(cur.vq, qf);
        const float r16 = r_old * 0.0625f;
#pragma unroll
        for (int e = 0; e < 4; ++e) vt[e] = dequant_v16(qf[e], min_nonneg(r16, cold16[e]));
    } else {
        float cold[4];
        load4(a.c + geo.col0, cold);
#pragma unroll
        for (int e = 0; e < 4; ++e) vt[e] = dequant_v((uint32_t(cur.vq) >> (4 * e)) & 15u, fminf(r_old, cold[e]));
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        mt[e] = moment_m(h, mt[e], g[e]);
        vt[e] = moment_v(h, vt[e], g[e]);
        w[e] = param_update(h, w[e], mt[e], vt[e]);
        amax = fmaxf(amax, fabsf(mt[e]));
        rmax = max_nonneg(rmax, vt[e]);
        cmax[e] = max_nonneg(cmax[e], vt[e]);
    }
    // the caller's prefetch of a later row is issued here, in the middle of the row's arithmetic:
    // by now the previous row's stores have been acknowledged, and loads queue behind older stores
    __builtin_amdgcn_sched_barrier(0);
    mid();
    __builtin_amdgcn_sched_barrier(0);
    const float s_new = group32_allmax(amax);     // block absmax of m_t
    rmax = group32_allmax(rmax);

    uint32_t mq_new = 0;
    uint32_t dist = scale_is_tame(s_new) ? 0xFFFFFFFFu : 0u;     // an extreme block scale forces the exact route
    {
        const float inv_s = approx_inv(s_new);
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
            uint32_t da, db;
            mq_new |= quant_m_code_fast(s.search, mt[e], inv_s, da) << (4 * e);
            mq_new |= quant_m_code_fast(s.search, mt[e + 1], inv_s, db) << (4 * e + 4);
            dist = min(min(dist, da), db);
        }
    }
    if (__builtin_expect(__ballot(dist < kMinDistM) != 0, 0)) {
        mq_new = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) mq_new |= quant_m_code(s.search, mt[e], s_new) << (4 * e);
    }

    store_row1(tb, row_offset(il, a.cols, geo.col0) * 4u, w, mq_new);
    if (geo.l == 0) {
        s.blk_scale[slot] = s_new;
        s.blk_vmax[slot] = rmax;
    }
}

// TABLES_READY: the caller has loaded the lookup tables into `s` (and synchronized) already.
template <bool BF16, bool TABLES_READY>
__device__ __forceinline__ void pass1_fast_tile(const Tensor4& a, const Hyper& h, int wg, Lds& s) {
    const Geo geo = geometry(a, wg);
    const TileBase tb = tile_base<BF16>(a, geo.row0, geo.n_rows);
    float cmax[4] = {0.0f, 0.0f, 0.0f, 0.0f};

    // old block scales and old row maxima of the tile into the slots of the new ones
    for (int t = threadIdx.x; t < geo.n_rows * a.gx; t += kThreads) {
        const int il = t / a.gx, cbi = geo.strip * a.gx + t % a.gx;
        s.blk_scale[t] = cbi < a.nb ? tb.ms[row_offset(il, a.nb, uint32_t(cbi))] : 0.0f;
        s.blk_vmax[t] = tb.r[il];
    }
    if (geo.active) {
        float cold16[4];
        load4(a.c + geo.col0, cold16);
        bool cols_tame = true;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            cols_tame = bool(int(cols_tame) & int(scale_is_tame(cold16[e])));
            cold16[e] *= 0.0625f;
        }
        // Rows of this group, in the order it takes them: row(k) = gyi * S + k % S + (k / S) * gy * S with
        // S = 2^rs.  With S = 1 these are gyi, gyi + gy, ...; in general the gy groups that work side by
        // side are S rows apart.  The memory system likes the rows in flight at one time to lie 32 KiB
        // apart (measured: up to 10 % more bandwidth than neighbouring rows for 4096-column tensors, whose
        // rows are 16 KiB long), so the host picks S to make S rows a multiple of 32 KiB where it can.
        // The loads of two rows are in flight while a third is computed (three register sets take turns,
        // the loop is unrolled by three); the prefetch is unconditional, rows past the tile come back as
        // zeros and are never used.
        const int n = geo.n_rows, rs = a.rs;
        const int row_g = geo.gyi << rs, hop = a.gy << rs, low = (1 << rs) - 1;
        auto row = [&](int k) { return row_g + (k & low) + (k >> rs) * hop; };    // increasing in k
        int k = 0;
        Row1<BF16> r0 = load_row1<BF16>(tb, a, geo, row(0));
        Row1<BF16> r1 = load_row1<BF16>(tb, a, geo, row(1));
        Row1<BF16> r2;
        // the first rows' loads are in flight meanwhile; the barrier also publishes the staged scales
        if constexpr (!TABLES_READY) load_tables(s);
        else __syncthreads();
        // Everything requested so far has to be here before the first row anyway.  Saying so with an
        // explicit wait gives the loop a start-up state with nothing outstanding; otherwise the
        // start-up's own (tight) wait counts are merged into the loop head and drain the prefetch
        // in every round.
        __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
        // Rounds of three rows while all three exist; the loop has no exit in its middle, so that
        // every path through it sees the same queue of outstanding loads and the compiler's wait
        // counts are exact (an early exit would join a path on which the newest prefetch is still
        // pending, and the loop head would then wait for it).  At most two rows remain afterwards.
        auto none = [] {};
        while (row(k + 2) < n) {
            pass1_row<BF16>(a, h, tb, geo, s, r0, row(k), cold16, cols_tame, cmax,
                            [&] { r2 = load_row1<BF16>(tb, a, geo, row(k + 2)); });
            pass1_row<BF16>(a, h, tb, geo, s, r1, row(k + 1), cold16, cols_tame, cmax,
                            [&] { r0 = load_row1<BF16>(tb, a, geo, row(k + 3)); });
            pass1_row<BF16>(a, h, tb, geo, s, r2, row(k + 2), cold16, cols_tame, cmax,
                            [&] { r1 = load_row1<BF16>(tb, a, geo, row(k + 4)); });
            k += 3;
        }
        if (row(k) < n) {
            pass1_row<BF16>(a, h, tb, geo, s, r0, row(k), cold16, cols_tame, cmax, none);
            if (row(k + 1) < n) pass1_row<BF16>(a, h, tb, geo, s, r1, row(k + 1), cold16, cols_tame, cmax, none);
        }
    } else {
        if constexpr (!TABLES_READY) load_tables(s);   // keeps the workgroup's barriers matched
        else __syncthreads();
    }

    // column maxima: combine the gy groups that share a column block, then one atomic per column
#pragma unroll
    for (int e = 0; e < 4; ++e) s.col[geo.grp * 128 + geo.l * 4 + e] = cmax[e];
    __syncthreads();
    // block scales to the state, block maxima of v_t into the row maxima
    for (int t = threadIdx.x; t < geo.n_rows * a.gx; t += kThreads) {
        const int il = t / a.gx, cbi = geo.strip * a.gx + t % a.gx;
        if (cbi < a.nb) {
            st<float>(tb.ms, row_offset(il, a.nb, uint32_t(cbi)) * 4u, s.blk_scale[t]);
            const float m = s.blk_vmax[t];
            if (m > 0.0f) atomic_max_nonneg(tb.r_new + il, m);     // unconditionally: reading the running
            // maximum first (to skip atomics that cannot raise it) costs a round trip at the end of every tile
            // and was measured to be slower
        }
    }
    for (int t = threadIdx.x; t < a.gx * 128; t += kThreads) {
        const int gi = t >> 7;
        float m = 0.0f;
        for (int y = 0; y < a.gy; ++y) m = fmaxf(m, s.col[((y * a.gx + gi) << 7) + (t & 127)]);
        const int cbi = geo.strip * a.gx + gi;
        if (cbi < a.nb && m > 0.0f) atomic_max_nonneg(a.c_new + int64_t(cbi) * 128 + (t & 127), m);
    }
}

// =====================================================================================================
// Pass 1, "flat" tiling: a workgroup's tile is rw rows x up to 8 column blocks (4 KiB of parameters
// per row), and a group walks ALONG a row -- the strip's blocks one after the other, then its next
// row -- so that each of the 8 groups reads and writes runs of 4 KiB instead of 512 bytes per row.
// The price: a lane's 4 columns change with every block, so the old column maxima of the strip sit in
// LDS (read per block) and the running new ones are raised there with LDS atomics.  Rows are dealt to
// the groups as in the tiling above (spacing 2^rs).  Everything else is pass1_row's arithmetic.
// =====================================================================================================

constexpr int kFlatBlocks = 8;

template <bool BF16>
__device__ __forceinline__ Row1<BF16> load_unit(const TileBase& b, const Tensor4& a, int il, int cb, int l) {
    Row1<BF16> r;
    const uint32_t off4 = row_offset(il, a.cols, uint32_t(cb) * 128u + uint32_t(l) * 4u) * 4u;
    r.p = buf_ld_f4_stream(b.rp, off4);
    // non-temporal although pass 2 reads the gradient again: the re-read comes from HBM either way (the set is far
    // larger than the caches), and not keeping the line is 0.35 % per step on the 7B-shaped set (five A/B pairs)
    r.g = load_grad_regs4<BF16, kPolicyNt>(b.rg, off4);
    r.mq = buf_ld_u16(b.rmq, off4 >> 3);
    r.vq = buf_ld_u16(b.rvq, off4 >> 3);
    return r;
}

// One block of one row.  j = block inside the strip, cb = its column block in the tensor; row_run carries the
// row's maximum of v_t from block to block.
template <bool BF16, class Mid>
__device__ __forceinline__ void flat_unit(const Tensor4& a, const Hyper& h, const TileBase& tb, Lds& s,
                                          const Row1<BF16>& cur, int il, int j, int cb, int l, int nbk,
                                          bool cols_tame, float& row_run, Mid mid) {
    float w[4] = {cur.p.x, cur.p.y, cur.p.z, cur.p.w};
    float g[4];
    unpack_grad4<BF16>(cur.g, g);
    float mt[4], vt[4], amax = 0.0f, rmax = 0.0f;
    const float s_old = s.blk_scale[il * kFlatBlocks + j];     // staged by the tile; replaced below
    const float r_old = s.blk_vmax[il];                        // likewise; replaced after the row's last block
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const float2 t = s.deq[(uint32_t(cur.mq) >> (8 * k)) & 255u];
        mt[2 * k] = t.x * s_old;
        mt[2 * k + 1] = t.y * s_old;
    }
    const uint32_t col0 = uint32_t(cb) * 128u + uint32_t(l) * 4u;
    const bool tame_in = bool(int(cols_tame) & int(scale_is_tame(r_old)));
    if (__builtin_expect(__ballot(!tame_in) == 0, 1)) {
        float qf[4];
        codes_to_float4(cur.vq, qf);
        const float r16 = r_old * 0.0625f;
        const float4 c16 = *reinterpret_cast<const float4*>(&s.cold[j * 128 + l * 4]);
        const float cold16[4] = {c16.x, c16.y, c16.z, c16.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) vt[e] = dequant_v16(qf[e], min_nonneg(r16, cold16[e]));
    } else {
        float cold[4];
        load4(a.c + col0, cold);
#pragma unroll
        for (int e = 0; e < 4; ++e) vt[e] = dequant_v((uint32_t(cur.vq) >> (4 * e)) & 15u, fminf(r_old, cold[e]));
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        mt[e] = moment_m(h, mt[e], g[e]);
        vt[e] = moment_v(h, vt[e], g[e]);
        w[e] = param_update(h, w[e], mt[e], vt[e]);
        amax = fmaxf(amax, fabsf(mt[e]));
        rmax = max_nonneg(rmax, vt[e]);
    }
    __builtin_amdgcn_sched_barrier(0);
    mid();
    __builtin_amdgcn_sched_barrier(0);
    // running column maxima of the strip: LDS atomics on the float bits (values are >= +0)
    unsigned int* cbits = reinterpret_cast<unsigned int*>(&s.col[j * 128 + l * 4]);
#pragma unroll
    for (int e = 0; e < 4; ++e)
        (void)__hip_atomic_fetch_max(cbits + e, __float_as_uint(vt[e]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    const float s_new = group32_allmax(amax);
    rmax = group32_allmax(rmax);
    row_run = j == 0 ? rmax : max_nonneg(row_run, rmax);

    uint32_t mq_new = 0;
    uint32_t dist = scale_is_tame(s_new) ? 0xFFFFFFFFu : 0u;
    {
        const float inv_s = approx_inv(s_new);
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
            uint32_t da, db;
            mq_new |= quant_m_code_fast(s.search, mt[e], inv_s, da) << (4 * e);
            mq_new |= quant_m_code_fast(s.search, mt[e + 1], inv_s, db) << (4 * e + 4);
            dist = min(min(dist, da), db);
        }
    }
    if (__builtin_expect(__ballot(dist < kMinDistM) != 0, 0)) {
        mq_new = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) mq_new |= quant_m_code(s.search, mt[e], s_new) << (4 * e);
    }
    store_row1(tb, row_offset(il, a.cols, col0) * 4u, w, mq_new);
    if (l == 0) {
        s.blk_scale[il * kFlatBlocks + j] = s_new;
        if (j == nbk - 1) s.blk_vmax[il] = row_run;
    }
}

// a.strips = ceil(nb / 8) strips, a.rw rows per tile (at most 64), a.rs the row spacing, a.n_wg workgroups
template <bool BF16>
__device__ __forceinline__ void pass1_flat_tile(const Tensor4& a, const Hyper& h, int wg, Lds& s) {
    const int strip = wg % a.strips, tile = wg / a.strips;
    const int grp = threadIdx.x >> 5, l = threadIdx.x & 31;
    const int cb0 = strip * kFlatBlocks;
    const int left_b = a.nb - cb0;
    const int nbk = left_b < kFlatBlocks ? left_b : kFlatBlocks;         // blocks of this strip, 1..8
    const int64_t row0 = int64_t(tile) * a.rw;
    const int64_t left = a.rows - row0;
    const int n = left < a.rw ? int(left) : a.rw;
    const TileBase tb = tile_base<BF16>(a, row0, n);
    // units of this group in the order it takes them: unit q = block q % nbk of its row number q / nbk
    const int rs = a.rs;
    const int row_g = grp << rs, hop = kGroups << rs, low = (1 << rs) - 1;
    auto row = [&](int k) { return row_g + (k & low) + (k >> rs) * hop; };
    const uint32_t inv_nbk = (65536u + uint32_t(nbk) - 1u) / uint32_t(nbk);   // q / nbk == (q * inv_nbk) >> 16 for q < 9000
    auto krow = [&](int q) { return int((uint32_t(q) * inv_nbk) >> 16); };
    auto blk = [&](int q) { return q - krow(q) * nbk; };
    auto fetch = [&](int q) { return load_unit<BF16>(tb, a, row(krow(q)), cb0 + blk(q), l); };
    int q = 0;
    Row1<BF16> r0 = fetch(0);
    Row1<BF16> r1 = fetch(1);
    Row1<BF16> r2;
    // the strip's old column maxima (scaled) and zeroed running maxima into LDS, then the tables
    bool tame = true;
    for (int t = threadIdx.x; t < nbk * 128; t += kThreads) {
        const float c = a.c[cb0 * 128 + t];
        tame = bool(int(tame) & int(scale_is_tame(c)));
        s.cold[t] = c * 0.0625f;
        s.col[t] = 0.0f;
    }
    // old block scales and old row maxima of the tile into the slots of the new ones
    for (int t = threadIdx.x; t < n * kFlatBlocks; t += kThreads) {
        const int il = t / kFlatBlocks, j = t % kFlatBlocks;
        s.blk_scale[t] = j < nbk ? tb.ms[row_offset(il, a.nb, uint32_t(cb0 + j))] : 0.0f;
    }
    for (int t = threadIdx.x; t < n; t += kThreads) s.blk_vmax[t] = tb.r[t];
    const bool cols_tame = !__syncthreads_or(int(!tame));
    load_tables(s);
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
    float row_run = 0.0f;
    auto none = [] {};
    auto unit = [&](const Row1<BF16>& cur, int qq, auto mid) {
        flat_unit<BF16>(a, h, tb, s, cur, row(krow(qq)), blk(qq), cb0 + blk(qq), l, nbk, cols_tame, row_run, mid);
    };
    while (row(krow(q + 2)) < n) {
        unit(r0, q, [&] { r2 = fetch(q + 2); });
        unit(r1, q + 1, [&] { r0 = fetch(q + 3); });
        unit(r2, q + 2, [&] { r1 = fetch(q + 4); });
        q += 3;
    }
    if (row(krow(q)) < n) {
        unit(r0, q, none);
        if (row(krow(q + 1)) < n) unit(r1, q + 1, none);
    }
    __syncthreads();
    for (int t = threadIdx.x; t < n * kFlatBlocks; t += kThreads) {
        const int il = t / kFlatBlocks, j = t % kFlatBlocks;
        if (j < nbk) st<float>(tb.ms, row_offset(il, a.nb, uint32_t(cb0 + j)) * 4u, s.blk_scale[t]);
    }
    for (int t = threadIdx.x; t < n; t += kThreads) {
        const float m = s.blk_vmax[t];
        if (m > 0.0f) atomic_max_nonneg(tb.r_new + t, m);
    }
    for (int t = threadIdx.x; t < nbk * 128; t += kThreads) {
        const float m = s.col[t];
        if (m > 0.0f) atomic_max_nonneg(a.c_new + cb0 * 128 + t, m);
    }
}

// The last workgroup of a tensor's pass 2 to finish makes r', c' the state and clears the
// workspace.  Every other workgroup has read the old r, c before it took its ticket, so
// overwriting them is safe.  Tickets are taken in two levels (kTicketLanes first-level counters, one
// cache line apart, then one top counter) so that thousands of workgroups do not queue up on a
// single address.  `me` / `participants`: this workgroup's index among, and the number of,
// workgroups that call this for the tensor.
constexpr int kTicketLanes = 32;
constexpr int kTicketStride = 32;                                  // in 32-bit words: 128 bytes
constexpr int kMaxTotSlots = 8;                                    // lines behind the ticket counters, for the
                                                                   // factorized step's two float sums
constexpr int kCounterWords = (1 + kTicketLanes + kMaxTotSlots) * kTicketStride;  // per tensor

// dst[i] = src[i]; src[i] = 0 by one workgroup.  It runs alone at the end of a tensor's pass 2, so
// what counts is latency: 16 loads per thread are in flight before the first store.
__device__ __forceinline__ void move_and_clear(float* dst, float* src, int64_t n) {
    constexpr int kDepth = 16;
    for (int64_t base = threadIdx.x; base < n; base += int64_t(kThreads) * kDepth) {
        float v[kDepth];
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int64_t i = base + int64_t(u) * kThreads;
            v[u] = i < n ? src[i] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int64_t i = base + int64_t(u) * kThreads;
            if (i < n) { dst[i] = v[u]; src[i] = 0.0f; }
        }
    }
}

// true in every thread of the one workgroup that arrives last
__device__ __forceinline__ bool last_to_arrive(const Tensor4& a, unsigned int me, unsigned int participants,
                                               int& s_last) {
    __syncthreads();
    if (threadIdx.x == 0) {
        // No fence: the ticket orders nothing but "this workgroup's loads of r, c have returned",
        // which holds once its waves have computed their codes and reached the barrier above.  (An
        // agent-scope release here would write back the XCD's whole L2 once per workgroup.)
        const unsigned int lane = me % kTicketLanes;
        const unsigned int in_lane = participants / kTicketLanes + (lane < participants % kTicketLanes ? 1u : 0u);
        int last = 0;
        if (atomicAdd(a.counter + (1 + lane) * kTicketStride, 1u) == in_lane - 1) {
            a.counter[(1 + lane) * kTicketStride] = 0u;      // this lane is complete: reset it
            const unsigned int lanes_used = participants < kTicketLanes ? participants : kTicketLanes;
            last = atomicAdd(a.counter, 1u) == lanes_used - 1;
        }
        s_last = last;
    }
    __syncthreads();
    return s_last != 0;
}

__device__ __forceinline__ void publish_if_last(const Tensor4& a, unsigned int me, unsigned int participants,
                                                int& s_last) {
    if (!last_to_arrive(a, me, participants, s_last)) return;
    move_and_clear(a.r, a.r_new, a.rows);
    move_and_clear(a.c, a.c_new, a.cols + a.c_extra);
    if (threadIdx.x == 0) *a.counter = 0u;
}

// Pass 2 of the fast path.  Nothing here is reduced over a block, so the layout is chosen for the
// memory system and for cheap row bookkeeping instead: a wave works on 256 consecutive columns of
// ONE row (lane l owns columns 4l .. 4l+3 of the strip; 128 contiguous bytes of codes, 512 of bf16
// gradient), the four waves of a workgroup take rows w, w+4, ... of the tile.  The row index, the two
// row maxima and everything derived from them are wave-uniform and live in scalar registers.
template <bool BF16>
struct Row2 {                      // what pass 2 reads per element for one row of one lane
    GradRegs4<BF16> g;
    uint16_t vq;                   // the lane's 4 codes
};

// row_elems = il * cols, wave-uniform: it travels as the scalar offset of the buffer instructions, so a row costs no
// vector arithmetic for its addresses.  lane_g / lane_q: the lane's byte offsets inside a row of the gradient / of the
// codes, fixed for the tile.  (Callers pass rows inside the tile only: the scalar offset may not take part in the
// range check of the resource.)
template <bool BF16>
__device__ __forceinline__ Row2<BF16> load_row2(const TileBase& b, uint32_t row_elems, uint32_t lane_g, uint32_t lane_q) {
    Row2<BF16> r;
    if constexpr (BF16) {                                       // last use of the gradient in this step
        const v2u_t w = __builtin_amdgcn_raw_buffer_load_b64(b.rg, int(lane_g), int(row_elems * 2u), kPolicyNt);
        r.g.w = make_uint2(w.x, w.y);
    } else {
        const v4f_t v = __builtin_bit_cast(v4f_t, __builtin_amdgcn_raw_buffer_load_b128(b.rg, int(lane_g), int(row_elems * 4u), kPolicyNt));
        r.g.a = make_float4(v.x, v.y, v.z, v.w);
    }
    r.vq = uint16_t(__builtin_amdgcn_raw_buffer_load_b16(b.rvq, int(lane_q), int(row_elems >> 1), 0));
    return r;
}

__device__ __forceinline__ float lane_value(float v, int lane) {      // lane: wave-uniform
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// The scalars of a wave's rows of one pass-2 tile, one row per lane (row k of the wave in lane k): the old and the new
// row maximum, the old one / 16, the approximate reciprocal of the new one (0 for 0), and `wild`, the mask of the
// rows that must take the exact route whatever their elements (a scale of the row or of the strip's columns outside
// the range in which scale / 16 and the reciprocal keep all their bits).
struct RowScalars {
    float r_old, r_new, r16, inv;
    uint64_t wild;
};

// New codes of the lane's 4 elements of row k of the wave.  The usual route multiplies by approximate reciprocals and
// keeps track of how close it came to a decision boundary; if the row is marked wild, or some lane came too close, the
// whole wave computes the row again from its inputs with exact arithmetic (same bits where both apply).  The second
// route shares no value with the first, so that nothing has to be kept in registers for it.
template <bool BF16>
__device__ __forceinline__ uint32_t pass2_row(const Tensor4& a, const Hyper& h, uint32_t col0, const Row2<BF16>& row,
                                              const RowScalars& rs, int k, const float cold16[4],
                                              const float inv_cnew[4]) {
    float g[4];
    unpack_grad4<BF16>(row.g, g);
    // wave-uniform: the whole wave takes one route
    if (__builtin_expect(((rs.wild >> k) & 1u) == 0u, 1)) {
        float qf[4], vt[4];
        codes_to_float4(row.vq, qf);
        const float r16 = lane_value(rs.r16, k), inv_r = lane_value(rs.inv, k);
#pragma unroll
        for (int e = 0; e < 4; ++e) vt[e] = moment_v(h, dequant_v16(qf[e], min_nonneg(r16, cold16[e])), g[e]);
        // even elements collect in the bytes of `lo`, odd ones in `hi`; word = lo | hi << 4
        uint32_t lo = 0, hi = 0;
        float closest = 0.5f, fa, fb;
#define LPMM_V2(K)                                                                                        \
        lo = quant_v_code_fast<K>(vt[2 * K], max_nonneg(inv_r, inv_cnew[2 * K]), lo, fa);                 \
        hi = quant_v_code_fast<K>(vt[2 * K + 1], max_nonneg(inv_r, inv_cnew[2 * K + 1]), hi, fb);         \
        closest = fminf(fminf(closest, fabsf(fa)), fabsf(fb));
        LPMM_V2(0) LPMM_V2(1)
#undef LPMM_V2
        if (__builtin_expect(__ballot(closest < kMarginV) == 0, 1)) return lo | (hi << 4);
    }
    const float r_old = lane_value(rs.r_old, k), r_new = lane_value(rs.r_new, k);
    float cold[4], cnew[4];
    load4(a.c + col0, cold);
    load4(a.c_new + col0, cnew);
    uint32_t out = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float vt = moment_v(h, dequant_v((uint32_t(row.vq) >> (4 * e)) & 15u, fminf(r_old, cold[e])), g[e]);
        out |= quant_v_code(vt, fminf(r_new, cnew[e])) << (4 * e);
    }
    return out;
}

constexpr int kWaves = kThreads / 64;
constexpr int kMaxRw2 = 64 * kWaves;      // rows of a pass-2 tile: a wave keeps its rows' scalars one per lane

template <bool BF16>
__device__ __forceinline__ void pass2_fast_tile(const Tensor4& a, const Hyper& h, int wg) {
    const int strip = wg % a.strips2, tile = wg / a.strips2;
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    const int lane = threadIdx.x & 63;
    // With an odd number of column blocks the upper half-wave of the last strip has no columns.  Those lanes stay
    // in the loop all the same, because every lane of the wave holds the scalars of one of its rows (below): they
    // work on the lower half's columns a second time and only their stores are left out.
    const uint32_t col_own = uint32_t(strip) * 256u + uint32_t(lane) * 4u;
    const bool live = col_own < uint32_t(a.cols);
    const uint32_t col0 = live ? col_own : col_own - 128u;
    const int64_t row0 = int64_t(tile) * a.rw2;
    const int64_t left = a.rows - row0;
    const int n = left < a.rw2 ? int(left) : a.rw2;
    const TileBase tb = tile_base<BF16>(a, row0, n);
    // rows of this wave in the order it takes them, as in pass 1: the four waves are 2^rs2 rows apart
    const int rs = a.rs2;
    const int row_w = wave << rs, hop = kWaves << rs, low = (1 << rs) - 1;
    auto row = [&](int k) { return row_w + (k & low) + (k >> rs) * hop; };
    // The scalars of the wave's rows (at most 64 per tile), one row per lane; the row loop fetches what it needs
    // with v_readlane instead of two loads, a reciprocal, a select and two range checks per row.  Rows past the
    // tile read as zeros through the bounds-checked resources.
    RowScalars sc;
    {
        const uint32_t il_l = uint32_t(row(lane));
        sc.r_old = buf_ld_f(tb.rr, il_l * 4u);
        sc.r_new = buf_ld_f(tb.rr_new, il_l * 4u);
        sc.r16 = sc.r_old * 0.0625f;
        sc.inv = approx_inv(sc.r_new);
        const bool row_tame = bool(int(scale_is_tame(sc.r_old)) & int(scale_is_tame(sc.r_new)));
        sc.wild = __ballot(!row_tame);
    }
    float cold16[4], inv_cnew[4];
    load4(a.c + col0, cold16);
    load4(a.c_new + col0, inv_cnew);
    bool lane_tame = true;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        lane_tame = bool(int(lane_tame) & int(scale_is_tame(cold16[e])) & int(scale_is_tame(inv_cnew[e])));
        cold16[e] *= 0.0625f;
        inv_cnew[e] = approx_inv(inv_cnew[e]);
    }
    if (__ballot(!lane_tame) != 0) sc.wild = ~uint64_t(0);        // a wild column scale: every row takes the exact route
    // the loads of two rows are in flight while a third is computed (three register sets take turns, the loop is
    // unrolled by three); a prefetch past the tile takes the tile's last row again and is never used
    const uint32_t cols = uint32_t(a.cols);
    const uint32_t lane_g = col0 * (BF16 ? 2u : 4u), lane_q = col0 >> 1;
    const int last = n - 1;
    auto fetch = [&](int il) { return load_row2<BF16>(tb, uint32_t(il < last ? il : last) * cols, lane_g, lane_q); };   // il * cols < 2^29
    auto put = [&](int il, uint32_t codes) {
        if (live) __builtin_amdgcn_raw_buffer_store_b16(short(codes), tb.rvq, int(lane_q), int((uint32_t(il) * cols) >> 1), 0);
    };
    auto codes_of = [&](const Row2<BF16>& r, int k) { return pass2_row<BF16>(a, h, col0, r, sc, k, cold16, inv_cnew); };
    int k = 0;
    Row2<BF16> r0 = fetch(row(0));
    Row2<BF16> r1 = fetch(row(1));
    Row2<BF16> r2 = fetch(row(2));
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);     // loop start-up state: nothing outstanding (see pass 1)
    // Rounds of three rows, no exit in the middle (see pass 1).  A register set is reloaded right after the row it
    // held has been processed, two rows ahead of its next use; the loads are pinned there, after the last use of
    // the values they replace.
    if (row(k + 2) < n) do {
        put(row(k), codes_of(r0, k));
        __builtin_amdgcn_sched_barrier(0);
        r0 = fetch(row(k + 3));
        __builtin_amdgcn_sched_barrier(0);
        put(row(k + 1), codes_of(r1, k + 1));
        __builtin_amdgcn_sched_barrier(0);
        r1 = fetch(row(k + 4));
        __builtin_amdgcn_sched_barrier(0);
        put(row(k + 2), codes_of(r2, k + 2));
        __builtin_amdgcn_sched_barrier(0);
        r2 = fetch(row(k + 5));
        __builtin_amdgcn_sched_barrier(0);
        k += 3;
    } while (row(k + 2) < n);
    if (row(k) < n) {
        put(row(k), codes_of(r0, k));
        if (row(k + 1) < n) put(row(k + 1), codes_of(r1, k + 1));
    }
}

// =====================================================================================================
// Block-wise second moment (1-dimensional or flattened tensors; Sec. 4.2, last paragraph): both
// moments are normalized per block of 128 elements, nothing crosses a block, and the whole step is
// ONE pass.  Same lane layout as pass 1 (4 elements per lane, 32 lanes per block).  The 8 groups of a
// workgroup work 64 blocks = 32 KiB of parameters apart (the distance the memory system serves
// fastest, as for the rows of pass 1): the tensor is cut into super-tiles of 8 x 64 blocks, group g
// owns blocks [64 g, 64 g + 64) of a super-tile, and a workgroup takes `rounds` consecutive blocks of
// each of the 8 ranges, so 64 / rounds workgroups share a super-tile.  The tensor is a.P elements,
// a.r holds the second moment's block scales.  The tile routine covers whole blocks; a ragged last
// block is done by b128_tail_block.
// =====================================================================================================

struct TileB {
    float* p;
    uint8_t* mq;
    uint8_t* vq;
    float* ms;
    float* vs;
    Rsrc rp, rg, rmq, rvq;                // bounds-checked views of the tile, for the loads and stores
};

template <bool BF16>
__device__ __forceinline__ TileB tile_b128(const Tensor4& a, int64_t blk0, int n_blk) {
    TileB b;
    const int64_t e = blk0 * 128;
    const uint32_t elems = uint32_t(n_blk) * 128u;
    b.p = a.p + e;
    b.mq = reinterpret_cast<uint8_t*>(a.mq) + (e >> 1);
    b.vq = reinterpret_cast<uint8_t*>(a.vq) + (e >> 1);
    b.ms = a.ms + blk0;
    b.vs = a.r + blk0;
    b.rp = tile_rsrc(b.p, elems * 4u);
    b.rg = tile_rsrc(reinterpret_cast<const char*>(a.g) + e * (BF16 ? 2 : 4), elems * (BF16 ? 2u : 4u));
    b.rmq = tile_rsrc(b.mq, elems >> 1);
    b.rvq = tile_rsrc(b.vq, elems >> 1);
    return b;
}

template <bool BF16>
struct RowB {                      // everything the step reads for one block, per lane
    float4 p;
    GradRegs4<BF16> g;
    uint16_t mq, vq;               // the lane's 4 codes of each moment
};                                 // (the block's two old scales come from LDS, staged by the tile as in pass 1)

constexpr int kNoBlock = 1 << 22;     // a block index whose offsets lie beyond any tile: loads return zeros

// ib = block index inside the (super-)tile; blocks at or beyond its end read as zeros
// SGDM: the tensor has no second moment (SGD with momentum, App. E Alg. 2)
template <bool BF16, bool SGDM = false>
__device__ __forceinline__ RowB<BF16> load_rowb(const TileB& b, int ib, int l) {
    RowB<BF16> r;
    const uint32_t off4 = (uint32_t(ib) * 128u + uint32_t(l) * 4u) * 4u;
    r.p = buf_ld_f4_stream(b.rp, off4);
    r.g = load_grad_regs4<BF16, kPolicyNt>(b.rg, off4);              // read once per step
    r.mq = buf_ld_u16(b.rmq, off4 >> 3);
    if constexpr (SGDM) r.vq = 0;
    else r.vq = buf_ld_u16(b.rvq, off4 >> 3);
    return r;
}

template <bool BF16, bool SGDM, class Mid>
__device__ __forceinline__ void b128_row(const Hyper& h, const TileB& tb, Lds& s, const RowB<BF16>& cur,
                                         int ib, int slot, int l, Mid mid) {
    float w[4] = {cur.p.x, cur.p.y, cur.p.z, cur.p.w};
    float g[4];
    unpack_grad4<BF16>(cur.g, g);
    float mt[4], vt[4], amax = 0.0f, vmax = 0.0f;
    const float sm_old = s.blk_scale[slot];
    const float sv_old = SGDM ? 0.0f : s.blk_vmax[slot];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const float2 t = s.deq[(uint32_t(cur.mq) >> (8 * k)) & 255u];
        mt[2 * k] = t.x * sm_old;             // decompress: T_DE[code] * block scale
        mt[2 * k + 1] = t.y * sm_old;
    }
    if constexpr (SGDM) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            mt[e] = moment_sgdm(h, mt[e], g[e]);
            w[e] = param_sgdm(h, w[e], mt[e]);
            amax = fmaxf(amax, fabsf(mt[e]));
            vt[e] = 0.0f;
        }
    } else {
        if (__builtin_expect(__ballot(!scale_is_tame(sv_old)) == 0, 1)) {
            float qf[4];
            codes_to_float4(cur.vq, qf);
            const float s16 = sv_old * 0.0625f;
#pragma unroll
            for (int e = 0; e < 4; ++e) vt[e] = dequant_v16(qf[e], s16);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) vt[e] = dequant_v((uint32_t(cur.vq) >> (4 * e)) & 15u, sv_old);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            mt[e] = moment_m(h, mt[e], g[e]);
            vt[e] = moment_v(h, vt[e], g[e]);
            w[e] = param_update(h, w[e], mt[e], vt[e]);
            amax = fmaxf(amax, fabsf(mt[e]));
            vmax = max_nonneg(vmax, vt[e]);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    mid();                                        // the caller's prefetch of a later block
    __builtin_amdgcn_sched_barrier(0);
    const float sm_new = group32_allmax(amax);    // block absmax of m_t
    const float sv_new = SGDM ? 0.0f : group32_allmax(vmax);    // block maximum of v_t

    uint32_t mq_new = 0;
    uint32_t dist = scale_is_tame(sm_new) ? 0xFFFFFFFFu : 0u;
    {
        const float inv_s = approx_inv(sm_new);
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
            uint32_t da, db;
            mq_new |= quant_m_code_fast(s.search, mt[e], inv_s, da) << (4 * e);
            mq_new |= quant_m_code_fast(s.search, mt[e + 1], inv_s, db) << (4 * e + 4);
            dist = min(min(dist, da), db);
        }
    }
    if (__builtin_expect(__ballot(dist < kMinDistM) != 0, 0)) {
        mq_new = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) mq_new |= quant_m_code(s.search, mt[e], sm_new) << (4 * e);
    }

    uint32_t vq_new = 0;
    if constexpr (!SGDM) {
        const float inv_s = approx_inv(sv_new);
        uint32_t lo = 0, hi = 0;
        float closest = scale_is_tame(sv_new) ? 0.5f : 0.0f, fa, fb;
#define LPMM_VB(K)                                                               \
        lo = quant_v_code_fast<K>(vt[2 * K], inv_s, lo, fa);                     \
        hi = quant_v_code_fast<K>(vt[2 * K + 1], inv_s, hi, fb);                 \
        closest = fminf(fminf(closest, fabsf(fa)), fabsf(fb));
        LPMM_VB(0) LPMM_VB(1)
#undef LPMM_VB
        vq_new = lo | (hi << 4);
        if (__builtin_expect(__ballot(closest < kMarginV) != 0, 0)) {
            vq_new = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) vq_new |= quant_v_code(vt[e], sv_new) << (4 * e);
        }
    }

    const uint32_t off4 = (uint32_t(ib) * 128u + uint32_t(l) * 4u) * 4u;
    {   // through the tile's bounds-checked resources: no registers for a second set of base addresses
        const v4f_t v = {w[0], w[1], w[2], w[3]};
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u_t, v), tb.rp, int(off4), 0, kPolicyNtSc1);
        __builtin_amdgcn_raw_buffer_store_b16(short(mq_new), tb.rmq, int(off4 >> 3), 0, 0);
        if constexpr (!SGDM) __builtin_amdgcn_raw_buffer_store_b16(short(vq_new), tb.rvq, int(off4 >> 3), 0, 0);
    }
    if (l == 0) {
        s.blk_scale[slot] = sm_new;
        if constexpr (!SGDM) s.blk_vmax[slot] = sv_new;
    }
}

constexpr int kB128Stride = 64;                            // blocks between the groups of a workgroup
constexpr int kB128Super = kGroups * kB128Stride;          // blocks of a super-tile
constexpr int kB128MaxRounds = kB128Stride;                // block results of a tile are staged in LDS
static_assert(kGroups * kB128MaxRounds <= kMaxRowSlots, "LDS staging of block results");

// workgroup `wg` of a tensor: super-tile wg / slices, slice wg % slices of each group's range, where
// slices = 64 / a.rw and a.rw = rounds (a power of two); a.nb = whole blocks of the tensor
template <bool BF16, bool SGDM = false>
__device__ __forceinline__ void b128_tile(const Tensor4& a, const Hyper& h, int wg, Lds& s) {
    const int rounds = a.rw, slices = kB128Stride / rounds;
    const int64_t sup0 = int64_t(wg / slices) * kB128Super;
    const int64_t left = int64_t(a.nb) - sup0;
    const int n_sup = left < kB128Super ? int(left) : kB128Super;      // blocks of this super-tile that exist
    const TileB tb = tile_b128<BF16>(a, sup0, n_sup > 0 ? n_sup : 0);
    const int grp = threadIdx.x >> 5, l = threadIdx.x & 31;
    const int slice0 = (wg % slices) * rounds;
    const int first = grp * kB128Stride + slice0;                      // the group's first block in the super-tile
    int nv = n_sup - first;                                            // the group's blocks: 0 .. rounds
    nv = nv < 0 ? 0 : (nv > rounds ? rounds : nv);
    // blocks past the group's share must not be fetched (inside the super-tile they are real blocks,
    // another workgroup's): they get an index beyond every tile
    auto blk = [&](int k) { return k < nv ? first + k : kNoBlock; };
    const int slot0 = grp * rounds;
    int k = 0;
    RowB<BF16> r0 = load_rowb<BF16, SGDM>(tb, blk(0), l);
    RowB<BF16> r1 = load_rowb<BF16, SGDM>(tb, blk(1), l);
    RowB<BF16> r2;
    for (int t = threadIdx.x; t < kGroups * rounds; t += kThreads) {   // old block scales into the slots of the new ones
        const int b = (t / rounds) * kB128Stride + slice0 + t % rounds;
        s.blk_scale[t] = b < n_sup ? tb.ms[b] : 0.0f;
        if constexpr (!SGDM) s.blk_vmax[t] = b < n_sup ? tb.vs[b] : 0.0f;
    }
    load_tables(s);                                // the first blocks' loads are in flight meanwhile; its barrier
                                                   // also publishes the staged scales
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);       // loop start-up state: nothing outstanding (see pass 1)
    auto none = [] {};
    while (k + 2 < nv) {                           // rounds of three blocks, no exit in the middle
        b128_row<BF16, SGDM>(h, tb, s, r0, first + k, slot0 + k, l, [&] { r2 = load_rowb<BF16, SGDM>(tb, blk(k + 2), l); });
        b128_row<BF16, SGDM>(h, tb, s, r1, first + k + 1, slot0 + k + 1, l, [&] { r0 = load_rowb<BF16, SGDM>(tb, blk(k + 3), l); });
        b128_row<BF16, SGDM>(h, tb, s, r2, first + k + 2, slot0 + k + 2, l, [&] { r1 = load_rowb<BF16, SGDM>(tb, blk(k + 4), l); });
        k += 3;
    }
    if (k < nv) {
        b128_row<BF16, SGDM>(h, tb, s, r0, first + k, slot0 + k, l, none);
        if (k + 1 < nv) b128_row<BF16, SGDM>(h, tb, s, r1, first + k + 1, slot0 + k + 1, l, none);
    }
    __syncthreads();
    for (int t = threadIdx.x; t < kGroups * rounds; t += kThreads) {   // new block scales: 8 contiguous runs
        const int b = (t / rounds) * kB128Stride + slice0 + t % rounds;
        if (b < n_sup) {
            tb.ms[b] = s.blk_scale[t];
            if constexpr (!SGDM) tb.vs[b] = s.blk_vmax[t];
        }
    }
}

// The last, partial block of a tensor whose size is not a multiple of 128 (a.P - 128 * a.nb
// elements, an even number).  One lane per element pair, exact arithmetic, reductions through LDS.
template <bool BF16, bool SGDM = false>
__device__ __forceinline__ void b128_tail_block(const Tensor4& a, const Hyper& h, Lds& s) {
    const int64_t e0 = int64_t(a.nb) * 128;
    const int n = int(a.P - e0);                   // 1..127
    const int t = threadIdx.x;
    const bool on = t < (n + 1) / 2;               // this lane's pair: elements e0 + 2t, e0 + 2t + 1
    float mt[2] = {0.0f, 0.0f}, vt[2] = {0.0f, 0.0f};
    const float sm_old = a.ms[a.nb], sv_old = SGDM ? 0.0f : a.r[a.nb];
    uint32_t bm = 0, bv = 0;
    if (on) {
        bm = reinterpret_cast<const uint8_t*>(a.mq)[(e0 >> 1) + t];
        if constexpr (!SGDM) bv = reinterpret_cast<const uint8_t*>(a.vq)[(e0 >> 1) + t];
    }
    for (int k = 0; k < 2; ++k) {
        const int64_t e = e0 + 2 * t + k;
        if (on && e < a.P) {
            const float2 dq = s.deq[bm];
            const float g = load_grad1<BF16>(a.g, e);
            if constexpr (SGDM) {
                mt[k] = moment_sgdm(h, (k ? dq.y : dq.x) * sm_old, g);
                a.p[e] = param_sgdm(h, a.p[e], mt[k]);
            } else {
                mt[k] = moment_m(h, (k ? dq.y : dq.x) * sm_old, g);
                vt[k] = moment_v(h, dequant_v((bv >> (4 * k)) & 15u, sv_old), g);
                a.p[e] = param_update(h, a.p[e], mt[k], vt[k]);
            }
        }
    }
    s.col[t] = fmaxf(fabsf(mt[0]), fabsf(mt[1]));
    s.col[kThreads + t] = fmaxf(vt[0], vt[1]);
    __syncthreads();
    float sm_new = 0.0f, sv_new = 0.0f;
    for (int i = 0; i < 64; ++i) {                 // every lane reduces the 64 pairs itself
        sm_new = fmaxf(sm_new, s.col[i]);
        sv_new = fmaxf(sv_new, s.col[kThreads + i]);
    }
    if (on) {
        uint32_t qm = 0, qv = 0;
        for (int k = 0; k < 2; ++k)
            if (e0 + 2 * t + k < a.P) {
                qm |= quant_m_code(s.search, mt[k], sm_new) << (4 * k);
                if constexpr (!SGDM) qv |= quant_v_code(vt[k], sv_new) << (4 * k);
            }
        reinterpret_cast<uint8_t*>(a.mq)[(e0 >> 1) + t] = uint8_t(qm);
        if constexpr (!SGDM) reinterpret_cast<uint8_t*>(a.vq)[(e0 >> 1) + t] = uint8_t(qv);
    }
    if (t == 0) {
        a.ms[a.nb] = sm_new;
        if constexpr (!SGDM) a.r[a.nb] = sv_new;
    }
}

// workgroups [0, n_wg2) run tiles of whole blocks, workgroup n_wg2 (if n_wg > n_wg2) the partial block
template <bool BF16, bool SGDM = false>
__device__ __forceinline__ void b128_work(const Tensor4& a, const Hyper& h, int wg, Lds& s) {
    if (wg < a.n_wg2) {
        b128_tile<BF16, SGDM>(a, h, wg, s);
    } else {
        load_tables(s);
        b128_tail_block<BF16, SGDM>(a, h, s);
    }
}

// =====================================================================================================
// General path: any rows x cols.  Lane t owns flat elements [8t, 8t+8); a group is still one block
// of 128, but a lane's elements may lie in different rows, so row and column indices are tracked
// per element and the maxima go straight to atomics (skipped when they cannot raise the value).
// =====================================================================================================


struct LaneIo {
    int64_t base;   // first flat element of the lane
    int nv;         // valid elements, 0..8
    int64_t i;      // row of the first element
    int64_t j;      // column of the first element
};

__device__ __forceinline__ LaneIo lane_io(int64_t P, int64_t cols, int64_t lane_global) {
    LaneIo io;
    io.base = lane_global * 8;
    const int64_t left = P - io.base;
    io.nv = left >= 8 ? 8 : (left > 0 ? int(left) : 0);
    io.i = io.nv ? io.base / cols : 0;
    io.j = io.nv ? io.base - io.i * cols : 0;
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

// A workgroup of the general pass 1 takes a.rw (1..16, chosen by the host) consecutive chunks of 2048 elements.  The maxima of v_t
// are first combined in LDS (integer atomics on the float bits), indexed by the column -- possible when the
// tensor has at most kGenColsLds columns, which is the usual case for shapes that miss the fast path (narrow
// matrices) -- and by the row relative to the workgroup's first row; one global atomic per column and row
// that the workgroup touched follows at its end.  Wider tensors, or rows shorter than 9 elements, send their
// maxima to global atomics directly (read first, skipped when they cannot raise the value).
constexpr int kGenChunkElems = kThreads * 8;             // a.rw chunks of this many elements per workgroup
constexpr int kGenMaxChunks = 16;
constexpr int kGenColsLds = 2048;                        // s.col and s.cold together
constexpr int kGenRowsLds = 2 * kMaxRowSlots;            // s.blk_scale and s.blk_vmax together

template <bool BF16>
__device__ __forceinline__ void pass1_general_tile(const Tensor4& a, const Hyper& h, int wg, Lds& s) {
    static_assert(offsetof(Lds, cold) == offsetof(Lds, col) + sizeof(float) * 1024, "col and cold are one array here");
    static_assert(offsetof(Lds, blk_vmax) == offsetof(Lds, blk_scale) + sizeof(float) * kMaxRowSlots, "row slots");
    unsigned int* col_l = reinterpret_cast<unsigned int*>(s.col);          // [kGenColsLds]
    unsigned int* row_l = reinterpret_cast<unsigned int*>(s.blk_scale);    // [kGenRowsLds]
    const int n_chunks = a.rw;
    const int64_t e_first = int64_t(wg) * n_chunks * kGenChunkElems;
    const int64_t e_end = e_first + int64_t(n_chunks) * kGenChunkElems < a.P ? e_first + int64_t(n_chunks) * kGenChunkElems : a.P;
    const int64_t i0 = e_first / a.cols;                                   // first row this workgroup touches
    const int64_t n_rows_wg = (e_end - 1) / a.cols - i0 + 1;
    const bool cols_in_lds = a.cols <= kGenColsLds;
    const bool rows_in_lds = n_rows_wg <= kGenRowsLds;
    if (cols_in_lds)
        for (int t = threadIdx.x; t < int(a.cols); t += kThreads) col_l[t] = 0u;
    if (rows_in_lds)
        for (int t = threadIdx.x; t < int(n_rows_wg); t += kThreads) row_l[t] = 0u;
    load_tables(s);                                                        // its barrier covers the zeroing too
    auto raise_col = [&](int64_t j, float v) {
        if (cols_in_lds) (void)__hip_atomic_fetch_max(col_l + j, __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        else raise_max(a.c_new + j, v);
    };
    auto raise_row = [&](int64_t i, float v) {
        if (rows_in_lds) (void)__hip_atomic_fetch_max(row_l + (i - i0), __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        else raise_max(a.r_new + i, v);
    };
    for (int c = 0; c < n_chunks; ++c) {
        const int64_t t = (int64_t(wg) * n_chunks + c) * kThreads + threadIdx.x;
        const int64_t block = t >> 4;                       // uniform over the 16 lanes of a block
        const bool alive = block * 128 < a.P;               // dead lanes are the highest of the last chunk
        const LaneIo io = lane_io(a.P, a.cols, t);
        float w[8], g[8];
        if (io.nv == 8) {
            load8(a.p + io.base, w);
            load_grad8<BF16>(a.g, io.base, g);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                w[e] = e < io.nv ? a.p[io.base + e] : 0.0f;
                g[e] = e < io.nv ? load_grad1<BF16>(a.g, io.base + e) : 0.0f;
            }
        }
        const uint32_t mq = io.nv ? load_codes(a.mq, io) : 0u;
        const uint32_t vq = io.nv ? load_codes(a.vq, io) : 0u;
        const float s_old = alive ? a.ms[block] : 0.0f;

        float mt[8], amax = 0.0f;
        int64_t i = io.i, j = io.j;
        int64_t run_row = io.i;
        float run_max = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (e < io.nv) {
                const float2 tt = s.deq[(mq >> (8 * (e >> 1))) & 255u];
                const float m_prev = ((e & 1) ? tt.y : tt.x) * s_old;
                const float v_prev = dequant_v((vq >> (4 * e)) & 15u, fminf(a.r[i], a.c[j]));
                mt[e] = moment_m(h, m_prev, g[e]);
                const float vt = moment_v(h, v_prev, g[e]);
                w[e] = param_update(h, w[e], mt[e], vt);
                amax = fmaxf(amax, fabsf(mt[e]));
                if (i != run_row) { raise_row(run_row, run_max); run_row = i; run_max = 0.0f; }
                run_max = fmaxf(run_max, vt);
                raise_col(j, vt);
                if (++j == a.cols) { j = 0; ++i; }
            } else {
                mt[e] = 0.0f;
            }
        }
        // The lane's last row usually is its neighbours' too (rows are contiguous runs of lanes): combine
        // over the wave first, one atomic per row and wave.
        {
            const int lane = threadIdx.x & 63;
            long long rr = io.nv ? (long long)run_row : -1ll - lane;
            float rm = run_max;
            for (int d = 1; d < 64; d <<= 1) {
                const float om = __shfl_down(rm, d);
                const long long orow = __shfl_down(rr, d);
                if (lane + d < 64 && orow == rr) rm = fmaxf(rm, om);
            }
            const long long prev = __shfl_up(rr, 1);
            if (io.nv && (lane == 0 || prev != rr)) raise_row(rr, rm);
        }

        const float s_new = row16_allmax(amax);
        uint32_t mq_new = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (e < io.nv) mq_new |= quant_m_code(s.search, mt[e], s_new) << (4 * e);

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
        if (alive && (threadIdx.x & 15) == 0) a.ms[block] = s_new;
    }
    __syncthreads();
    if (cols_in_lds)
        for (int t = threadIdx.x; t < int(a.cols); t += kThreads) {
            const unsigned int m = col_l[t];
            if (m) atomicMax(reinterpret_cast<unsigned int*>(a.c_new) + t, m);
        }
    if (rows_in_lds)
        for (int t = threadIdx.x; t < int(n_rows_wg); t += kThreads) {
            const unsigned int m = row_l[t];
            if (m) atomicMax(reinterpret_cast<unsigned int*>(a.r_new) + i0 + t, m);
        }
}

template <bool BF16>
__device__ __forceinline__ void pass2_general_tile(const Tensor4& a, const Hyper& h, int wg) {
    const int64_t t = int64_t(wg) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(a.P, a.cols, t);
    if (!io.nv) return;
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

// =====================================================================================================
// Factorized second moment ("4-bit Factor", Sec. 4.3): for a rows x cols tensor the second moment is
// kept as row statistics R and column statistics C, moving averages (with beta2, as v_t in Eq. 1) of
// the row and column sums of g^2, and v_t[i][j] = R_i C_j / sum_i R_i takes the place of Eq. 1's v_t.
// The first moment is compressed as everywhere (B128 + signed dynamic-exponent map).
//
// Two passes, because every element's update needs the complete sums of its row and column:
//   statistics pass: reads the gradient only; row and column sums of g^2 into the workspace (float
//                    atomics), plus two scalars: the sum of all g^2 and the sum of the old R.
//   update pass:     R_t[i] = beta2 R[i] + (1-beta2) rowsum_i, C_t[j] likewise, sum R_t = beta2 sum R +
//                    (1-beta2) sum g^2; decompress m, Eq. 1 with the reconstructed v_t, parameter
//                    update, compress m_t.  The last workgroup writes R_t, C_t to the state (the same
//                    expression every workgroup evaluated) and clears the workspace.
// Nothing integer depends on the second moment here, so the sums are plain fp32 in whatever order
// the atomics arrive: R, C and the parameters vary in their last bits from run to run; the first
// moment's codes and scales do not.
// =====================================================================================================

// The two float sums live in the counter block, behind the ticket counters.  Each is spread over
// a.tot_slots slots (a power of two; a workgroup adds to slot = its index modulo the count), one slot
// per 128-byte line, because atomics on one line queue up behind each other even when their addresses
// differ; readers add the slots in a fixed order.  A tensor stepped on its own has all its workgroups
// arrive at once and takes 8 slots; in a plan the tensors' workgroups arrive spread out, one slot
// serves, and the update pass has fewer lines to read.
__device__ __forceinline__ int tot_new_word(int slot) { return (1 + kTicketLanes + slot) * kTicketStride; }      // sum of g^2
__device__ __forceinline__ int tot_old_word(int slot) { return (1 + kTicketLanes + slot) * kTicketStride + 1; }  // sum of the old R

__device__ __forceinline__ void atomic_add_f32(float* addr, float v) { (void)unsafeAtomicAdd(addr, v); }

// new statistic from the old one and this step's sum of squares
__device__ __forceinline__ float stat_ema(const Hyper& h, float old, float sum_sq) {
    return __builtin_fmaf(h.beta2, old, h.omb2 * sum_sq);
}
__device__ __forceinline__ float factor_inv_total(const Tensor4& a, const Hyper& h) {
    const float* tot = reinterpret_cast<const float*>(a.counter);
    float sum_new = 0.0f, sum_old = 0.0f;
    for (int k = 0; k < a.tot_slots; ++k) {
        sum_new += tot[tot_new_word(k)];
        sum_old += tot[tot_old_word(k)];
    }
    const float total = stat_ema(h, sum_old, sum_new);
    return total > 0.0f ? 1.0f / total : 0.0f;          // all-zero statistics: v_t = 0
}

template <int CTRL>
__device__ __forceinline__ float dpp_fadd(float x) {
    return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}
// sum over the 64 lanes of a wave, the same value in every lane (fixed order)
__device__ __forceinline__ float wave_sum(float v) {
    v = dpp_fadd<0xB1>(v);      // lane ^ 1
    v = dpp_fadd<0x4E>(v);      // lane ^ 2
    v = dpp_fadd<0x141>(v);     // other quad of the half row
    v = dpp_fadd<0x140>(v);     // other half of the row of 16
    v += __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), 0x401F));     // lane ^ 16
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0)) +
           __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
}

// Statistics pass, fast path (cols % 128 == 0).  Tiled like pass 2: a wave works on 256 consecutive
// columns of one row, the four waves of a workgroup take rows w, w+4, ... of a tile of rw2 rows.  Row
// sums are staged in LDS, column sums are combined over the four waves in LDS; one atomic per row and
// per column of the tile.
template <bool BF16>
__device__ __forceinline__ void factor_stats_tile(const Tensor4& a, int wg, Lds& s) {
    const int strip = wg % a.strips2, tile = wg / a.strips2;
    const int wave = __builtin_amdgcn_readfirstlane(int(threadIdx.x) >> 6);
    const int lane = threadIdx.x & 63;
    const uint32_t col0 = uint32_t(strip) * 256u + uint32_t(lane) * 4u;
    const bool live = col0 < uint32_t(a.cols);      // odd number of column blocks: upper half of the last strip
    const int64_t row0 = int64_t(tile) * a.rw2;
    const int64_t left = a.rows - row0;
    const int n = left < a.rw2 ? int(left) : a.rw2;
    const Rsrc rg = tile_rsrc(reinterpret_cast<const char*>(a.g) + row0 * a.cols * (BF16 ? 2 : 4),
                              uint32_t(n) * uint32_t(a.cols) * (BF16 ? 2u : 4u));
    float cacc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    auto ld = [&](int il) { return load_grad_regs4<BF16>(rg, row_offset(il, a.cols, col0) * 4u); };
    auto one = [&](const GradRegs4<BF16>& r, int il) {
        float g[4];
        unpack_grad4<BF16>(r, g);
        float sq[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sq[e] = live ? g[e] * g[e] : 0.0f;
            cacc[e] += sq[e];
        }
        const float rsum = wave_sum((sq[0] + sq[1]) + (sq[2] + sq[3]));
        if (lane == 0) s.blk_scale[il] = rsum;
    };
    // rows in the order of pass 2; three register sets take turns: a set is reloaded right after its row has been
    // summed, so the loads of two rows are in flight while a third is summed (more sets in flight measured slower)
    const int rs = a.rs2;
    const int row_w = wave << rs, hop = kWaves << rs, low = (1 << rs) - 1;
    auto row = [&](int k) { return row_w + (k & low) + (k >> rs) * hop; };
    int k = 0;
    constexpr int kDepth = 3;
    GradRegs4<BF16> r[kDepth];
#pragma unroll
    for (int u = 0; u < kDepth; ++u) r[u] = ld(row(u));
    __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
    if (row(k + kDepth - 1) < n) do {
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            one(r[u], row(k + u));
            __builtin_amdgcn_sched_barrier(0);
            r[u] = ld(row(k + kDepth + u));
            __builtin_amdgcn_sched_barrier(0);
        }
        k += kDepth;
    } while (row(k + kDepth - 1) < n);
#pragma unroll
    for (int u = 0; u < kDepth - 1; ++u)
        if (row(k + u) < n) one(r[u], row(k + u));
#pragma unroll
    for (int e = 0; e < 4; ++e) s.col[wave * 256 + lane * 4 + e] = cacc[e];
    __syncthreads();
    if (a.det) {
        // fixed order of summation: this tile's sums go to slots of their own; factor_reduce_one adds the strips
        // of a row and the tiles of a column in index order, factor_totals_one the rows
        const int64_t rows_pad = (a.rows + 63) / 64 * 64, cols_pad = (a.cols + 63) / 64 * 64;
        float* rowpart = reinterpret_cast<float*>(a.vq) + int64_t(strip) * rows_pad + row0;
        float* colpart = reinterpret_cast<float*>(a.vq) + int64_t(a.strips2) * rows_pad + int64_t(tile) * cols_pad;
        for (int t = threadIdx.x; t < n; t += kThreads) rowpart[t] = s.blk_scale[t];
        const int t = threadIdx.x;
        const float csum = (s.col[t] + s.col[256 + t]) + (s.col[512 + t] + s.col[768 + t]);
        const int64_t col = int64_t(strip) * 256 + t;
        if (col < a.cols) colpart[col] = csum;
        return;
    }
    for (int t = threadIdx.x; t < n; t += kThreads) atomic_add_f32(a.r_new + row0 + t, s.blk_scale[t]);
    {
        const int t = threadIdx.x;
        const float csum = (s.col[t] + s.col[256 + t]) + (s.col[512 + t] + s.col[768 + t]);
        const int64_t col = int64_t(strip) * 256 + t;
        if (col < a.cols) atomic_add_f32(a.c_new + col, csum);
    }
    float* tot = reinterpret_cast<float*>(a.counter);
    if (wave == 0) {                 // the tile's share of the sum of all g^2
        float part = 0.0f;
        for (int t = lane; t < n; t += 64) part += s.blk_scale[t];
        part = wave_sum(part);
        if (lane == 0) atomic_add_f32(tot + tot_new_word(wg & (a.tot_slots - 1)), part);
    } else if (wave == 1 && strip == 0) {   // the old statistics of the tile's rows, once per row
        float part = 0.0f;
        for (int t = lane; t < n; t += 64) part += a.r[row0 + t];
        part = wave_sum(part);
        if (lane == 0) atomic_add_f32(tot + tot_old_word(tile & (a.tot_slots - 1)), part);
    }
}

template <bool BF16>
struct RowF {                      // everything the update pass reads for one row of one lane
    float4 p;
    GradRegs4<BF16> g;
    uint16_t mq;
};

template <bool BF16>
__device__ __forceinline__ RowF<BF16> load_rowf(const TileBase& b, const Tensor4& a, const Geo& g, int il) {
    RowF<BF16> r;
    const uint32_t off4 = row_offset(il, a.cols, g.col0) * 4u;
    r.p = buf_ld_f4_stream(b.rp, off4);
    r.g = load_grad_regs4<BF16, kPolicyNt>(b.rg, off4);     // last use of the gradient in this step
    r.mq = buf_ld_u16(b.rmq, off4 >> 3);
    return r;
}

// One row of the update pass for one lane; ct[e] = C_t of the lane's columns.  The row's old block scale and
// R_t[i] / sum R_t come from LDS, where the tile staged them (see pass 1).
template <bool BF16, class Mid>
__device__ __forceinline__ void factor_row(const Tensor4& a, const Hyper& h, const TileBase& tb, const Geo& geo,
                                           Lds& s, const RowF<BF16>& cur, int il, const float ct[4], Mid mid) {
    float w[4] = {cur.p.x, cur.p.y, cur.p.z, cur.p.w};
    float g[4];
    unpack_grad4<BF16>(cur.g, g);
    float mt[4], amax = 0.0f;
    const int slot = il * a.gx + geo.gxi;
    const float s_old = s.blk_scale[slot], rn = s.blk_vmax[slot];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const float2 t = s.deq[(uint32_t(cur.mq) >> (8 * k)) & 255u];
        mt[2 * k] = t.x * s_old;
        mt[2 * k + 1] = t.y * s_old;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        mt[e] = moment_m(h, mt[e], g[e]);
        w[e] = param_update(h, w[e], mt[e], rn * ct[e]);
        amax = fmaxf(amax, fabsf(mt[e]));
    }
    __builtin_amdgcn_sched_barrier(0);
    mid();                                    // the caller's prefetch (see pass 1)
    __builtin_amdgcn_sched_barrier(0);
    const float s_new = group32_allmax(amax);

    uint32_t mq_new = 0;
    uint32_t dist = scale_is_tame(s_new) ? 0xFFFFFFFFu : 0u;
    {
        const float inv_s = approx_inv(s_new);
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
            uint32_t da, db;
            mq_new |= quant_m_code_fast(s.search, mt[e], inv_s, da) << (4 * e);
            mq_new |= quant_m_code_fast(s.search, mt[e + 1], inv_s, db) << (4 * e + 4);
            dist = min(min(dist, da), db);
        }
    }
    if (__builtin_expect(__ballot(dist < kMinDistM) != 0, 0)) {
        mq_new = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) mq_new |= quant_m_code(s.search, mt[e], s_new) << (4 * e);
    }
    store_row1(tb, row_offset(il, a.cols, geo.col0) * 4u, w, mq_new);
    if (geo.l == 0) s.blk_scale[slot] = s_new;
}

// Update pass, fast path: tiled and pipelined like pass 1.
template <bool BF16>
__device__ __forceinline__ void factor_update_tile(const Tensor4& a, const Hyper& h, int wg, Lds& s) {
    const Geo geo = geometry(a, wg);
    const TileBase tb = tile_base<BF16>(a, geo.row0, geo.n_rows);
    const int n = geo.n_rows, rs = a.rs;
    const int row_g = geo.gyi << rs, hop = a.gy << rs, low = (1 << rs) - 1;
    auto row = [&](int k) { return row_g + (k & low) + (k >> rs) * hop; };
    float ct[4] = {0.0f, 0.0f, 0.0f, 0.0f}, csum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    RowF<BF16> r0{}, r1{}, r2;
    if (geo.active) {
        load4(a.c + geo.col0, ct);
        load4(a.c_new + geo.col0, csum);
        r0 = load_rowf<BF16>(tb, a, geo, row(0));
        r1 = load_rowf<BF16>(tb, a, geo, row(1));
    }
    // per row of the tile: the old block scales of m, and R_t[i] / sum R_t once instead of in every lane
    const float inv_total = factor_inv_total(a, h);
    for (int t = threadIdx.x; t < n * a.gx; t += kThreads) {
        const int il = t / a.gx, cbi = geo.strip * a.gx + t % a.gx;
        s.blk_scale[t] = cbi < a.nb ? tb.ms[row_offset(il, a.nb, uint32_t(cbi))] : 0.0f;
        s.blk_vmax[t] = stat_ema(h, tb.r[il], tb.r_new[il]) * inv_total;
    }
    load_tables(s);          // its barrier also publishes the staged values
    if (geo.active) {
#pragma unroll
        for (int e = 0; e < 4; ++e) ct[e] = stat_ema(h, ct[e], csum[e]);
        __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
        int k = 0;
        auto none = [] {};
        while (row(k + 2) < n) {
            factor_row<BF16>(a, h, tb, geo, s, r0, row(k), ct, [&] { r2 = load_rowf<BF16>(tb, a, geo, row(k + 2)); });
            factor_row<BF16>(a, h, tb, geo, s, r1, row(k + 1), ct, [&] { r0 = load_rowf<BF16>(tb, a, geo, row(k + 3)); });
            factor_row<BF16>(a, h, tb, geo, s, r2, row(k + 2), ct, [&] { r1 = load_rowf<BF16>(tb, a, geo, row(k + 4)); });
            k += 3;
        }
        if (row(k) < n) {
            factor_row<BF16>(a, h, tb, geo, s, r0, row(k), ct, none);
            if (row(k + 1) < n) factor_row<BF16>(a, h, tb, geo, s, r1, row(k + 1), ct, none);
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < geo.n_rows * a.gx; t += kThreads) {
        const int il = t / a.gx, cbi = geo.strip * a.gx + t % a.gx;
        if (cbi < a.nb) st<float>(tb.ms, row_offset(il, a.nb, uint32_t(cbi)) * 4u, s.blk_scale[t]);
    }
}

// stat[i] = stat_ema(stat[i], sum[i]); sum[i] = 0, by one workgroup (see move_and_clear)
__device__ __forceinline__ void ema_and_clear(const Hyper& h, float* stat, float* sum, int64_t n) {
    constexpr int kDepth = 8;
    for (int64_t base = threadIdx.x; base < n; base += int64_t(kThreads) * kDepth) {
        float o[kDepth], v[kDepth];
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int64_t i = base + int64_t(u) * kThreads;
            o[u] = i < n ? stat[i] : 0.0f;
            v[u] = i < n ? sum[i] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int64_t i = base + int64_t(u) * kThreads;
            if (i < n) { stat[i] = stat_ema(h, o[u], v[u]); sum[i] = 0.0f; }
        }
    }
}

// The last workgroup of a tensor's update pass makes R_t, C_t the state and clears the workspace;
// every other workgroup has read the old statistics and the sums before it took its ticket.
__device__ __forceinline__ void factor_publish_if_last(const Tensor4& a, const Hyper& h, unsigned int me,
                                                       unsigned int participants, int& s_last) {
    if (!last_to_arrive(a, me, participants, s_last)) return;
    ema_and_clear(h, a.r, a.r_new, a.rows);
    ema_and_clear(h, a.c, a.c_new, a.cols);
    if (threadIdx.x == 0) *a.counter = 0u;
    if (int(threadIdx.x) < a.tot_slots) {
        a.counter[tot_new_word(threadIdx.x)] = 0u;
        a.counter[tot_old_word(threadIdx.x)] = 0u;
    }
}

// Deterministic sums (Tensor4::det): between the statistics pass and the update pass two small kernels turn the
// per-tile partial sums into what the float atomics would have left in the workspace, in a fixed order.
// Layout of the partial sums behind a.vq (rows_pad, cols_pad = rows, cols rounded up to 64):
//   float[strips2][rows_pad]  a row's sum over the columns of one strip
//   float[tiles][cols_pad]    a column's sum over the rows of one tile
//   float[2 * row_wgs]        per 256 rows: the sum of their new row sums, and of their old row statistics
__device__ __forceinline__ const float* det_rowpart(const Tensor4& a) { return reinterpret_cast<const float*>(a.vq); }
__device__ __forceinline__ const float* det_colpart(const Tensor4& a) {
    return det_rowpart(a) + int64_t(a.strips2) * ((a.rows + 63) / 64 * 64);
}
__device__ __forceinline__ float* det_totpart(const Tensor4& a) {
    const int64_t tiles = (a.rows + a.rw2 - 1) / a.rw2;
    return const_cast<float*>(det_colpart(a)) + tiles * ((a.cols + 63) / 64 * 64);
}
// sum over the workgroup, the same value in every thread, combined in a fixed order
__device__ __forceinline__ float wg_sum_fixed(float v, float* s_part) {
    v = wave_sum(v);
    __syncthreads();                                   // s_part may still be read from a previous call
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = v;
    __syncthreads();
    return (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
}

// Workgroup `w` of a tensor's reduce step: 256 rows (w < ceil(rows / 256)) or 64 columns.
__device__ __forceinline__ void factor_reduce_one(const Tensor4& a, int w, float* s_part) {
    const int64_t rows_pad = (a.rows + 63) / 64 * 64, cols_pad = (a.cols + 63) / 64 * 64;
    const int row_wgs = int((a.rows + kThreads - 1) / kThreads);
    if (w < row_wgs) {                                 // uniform over the workgroup
        const float* rowpart = det_rowpart(a);
        const int64_t i = int64_t(w) * kThreads + threadIdx.x;
        float acc = 0.0f, old = 0.0f;
        if (i < a.rows) {
            for (int s0 = 0; s0 < a.strips2; s0 += 8) {        // eight loads in flight, added in index order
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = s0 + u < a.strips2 ? rowpart[int64_t(s0 + u) * rows_pad + i] : 0.0f;
#pragma unroll
                for (int u = 0; u < 8; ++u) acc += v[u];
            }
            a.r_new[i] = acc;
            old = a.r[i];
        }
        const float t_new = wg_sum_fixed(acc, s_part), t_old = wg_sum_fixed(old, s_part);
        if (threadIdx.x == 0) {
            float* tp = det_totpart(a);
            tp[2 * w] = t_new;
            tp[2 * w + 1] = t_old;
        }
    } else {
        // 64 columns per workgroup; a tall tensor has hundreds of row tiles, so four threads share a column: thread
        // (q, c) adds tiles q, q + 4, ... in order, eight loads in flight, and the four sums are added in order of q
        const float* colpart = det_colpart(a);
        const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
        const int64_t j = int64_t(w - row_wgs) * 64 + c;
        const int tiles = int((a.rows + a.rw2 - 1) / a.rw2);
        float acc = 0.0f;
        if (j < a.cols)
            for (int t0 = q; t0 < tiles; t0 += 32) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = t0 + 4 * u < tiles ? colpart[int64_t(t0 + 4 * u) * cols_pad + j] : 0.0f;
#pragma unroll
                for (int u = 0; u < 8; ++u) acc += v[u];
            }
        __shared__ float s_col[kThreads];
        s_col[threadIdx.x] = acc;
        __syncthreads();
        if (q == 0 && j < a.cols) a.c_new[j] = (s_col[c] + s_col[64 + c]) + (s_col[128 + c] + s_col[192 + c]);
    }
}
// One workgroup per tensor, after the reduce step: the two totals (sum of this step's row sums, sum of the old row
// statistics) into slot 0, from the per-256-rows sums dealt to the threads in a fixed pattern.
__device__ __forceinline__ void factor_totals_one(const Tensor4& a, float* s_part) {
    const int row_wgs = int((a.rows + kThreads - 1) / kThreads);
    const float* tp = det_totpart(a);
    float t_new = 0.0f, t_old = 0.0f;
    for (int k = threadIdx.x; k < row_wgs; k += kThreads) {
        t_new += tp[2 * k];
        t_old += tp[2 * k + 1];
    }
    t_new = wg_sum_fixed(t_new, s_part);
    t_old = wg_sum_fixed(t_old, s_part);
    if (threadIdx.x == 0) {
        float* tot = reinterpret_cast<float*>(a.counter);
        tot[tot_new_word(0)] = t_new;
        tot[tot_old_word(0)] = t_old;
    }
}

// General path of the factorized form (any rows x cols): lane t owns flat elements [8t, 8t+8), row and
// column tracked per element.  The statistics pass works like the general pass 1: a.rw consecutive chunks of
// 2048 elements per workgroup, sums combined in LDS (float atomics) by column (tensors of at most 2048
// columns) and by row relative to the workgroup's first row, one global atomic per touched column and row at
// the end; wider tensors add straight to global memory.
template <bool BF16>
__device__ __forceinline__ void factor_stats_general_tile(const Tensor4& a, int wg, int n_wg, Lds& s) {
    float* col_l = s.col;                  // [kGenColsLds] (col and cold)
    float* row_l = s.blk_scale;            // [kGenRowsLds] (blk_scale and blk_vmax)
    const int n_chunks = a.rw;
    const int64_t e_first = int64_t(wg) * n_chunks * kGenChunkElems;
    const int64_t e_end = e_first + int64_t(n_chunks) * kGenChunkElems < a.P ? e_first + int64_t(n_chunks) * kGenChunkElems : a.P;
    const int64_t i0 = e_first / a.cols;
    const int64_t n_rows_wg = (e_end - 1) / a.cols - i0 + 1;
    const bool cols_in_lds = a.cols <= kGenColsLds;
    const bool rows_in_lds = n_rows_wg <= kGenRowsLds;
    if (cols_in_lds)
        for (int t = threadIdx.x; t < int(a.cols); t += kThreads) col_l[t] = 0.0f;
    if (rows_in_lds)
        for (int t = threadIdx.x; t < int(n_rows_wg); t += kThreads) row_l[t] = 0.0f;
    __syncthreads();
    auto add_col = [&](int64_t j, float v) {
        if (cols_in_lds) (void)__hip_atomic_fetch_add(col_l + j, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        else atomic_add_f32(a.c_new + j, v);
    };
    auto add_row = [&](int64_t i, float v) {
        if (rows_in_lds) (void)__hip_atomic_fetch_add(row_l + (i - i0), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        else atomic_add_f32(a.r_new + i, v);
    };
    float part = 0.0f, old = 0.0f;
    const int lane = threadIdx.x & 63;
    for (int c = 0; c < n_chunks; ++c) {
        const int64_t t = (int64_t(wg) * n_chunks + c) * kThreads + threadIdx.x;
        const LaneIo io = lane_io(a.P, a.cols, t);
        float g[8];
        if (io.nv == 8) {
            load_grad8<BF16>(a.g, io.base, g);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) g[e] = e < io.nv ? load_grad1<BF16>(a.g, io.base + e) : 0.0f;
        }
        int64_t i = io.i, j = io.j, run_row = io.i;
        float run = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if (e < io.nv) {
                const float sq = g[e] * g[e];
                if (i != run_row) { add_row(run_row, run); run_row = i; run = 0.0f; }
                run += sq;
                part += sq;
                add_col(j, sq);
                if (++j == a.cols) { j = 0; ++i; }
            }
        }
        // the lane's last row usually is its neighbours' too: add up over the wave first (rows are contiguous
        // runs of lanes, so lane k ends up with the sum over lanes k.. of its row), one atomic per row and wave
        long long rr = io.nv ? (long long)run_row : -1ll - lane;
        float rsum = run;
        for (int d = 1; d < 64; d <<= 1) {
            const float os = __shfl_down(rsum, d);
            const long long orow = __shfl_down(rr, d);
            if (lane + d < 64 && orow == rr) rsum += os;
        }
        const long long prev = __shfl_up(rr, 1);
        if (io.nv && (lane == 0 || prev != rr)) add_row(rr, rsum);
    }
    for (int64_t i = int64_t(wg) * kThreads + threadIdx.x; i < a.rows; i += int64_t(n_wg) * kThreads) old += a.r[i];
    part = wave_sum(part);
    old = wave_sum(old);
    __shared__ float s_tot[2 * kThreads / 64];
    if (lane == 0) { s_tot[threadIdx.x >> 6] = part; s_tot[4 + (threadIdx.x >> 6)] = old; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float* tot = reinterpret_cast<float*>(a.counter);
        atomic_add_f32(tot + tot_new_word(wg & (a.tot_slots - 1)), (s_tot[0] + s_tot[1]) + (s_tot[2] + s_tot[3]));
        atomic_add_f32(tot + tot_old_word(wg & (a.tot_slots - 1)), (s_tot[4] + s_tot[5]) + (s_tot[6] + s_tot[7]));
    }
    if (cols_in_lds)
        for (int t = threadIdx.x; t < int(a.cols); t += kThreads) {
            const float v = col_l[t];
            if (v != 0.0f) atomic_add_f32(a.c_new + t, v);
        }
    if (rows_in_lds)
        for (int t = threadIdx.x; t < int(n_rows_wg); t += kThreads) {
            const float v = row_l[t];
            if (v != 0.0f) atomic_add_f32(a.r_new + i0 + t, v);
        }
}

template <bool BF16>
__device__ __forceinline__ void factor_update_general_tile(const Tensor4& a, const Hyper& h, int wg, Lds& s) {
    const int64_t t = int64_t(wg) * kThreads + threadIdx.x;
    const int64_t block = t >> 4;                       // uniform over the 16 lanes of a block
    if (block * 128 >= a.P) return;
    const LaneIo io = lane_io(a.P, a.cols, t);
    float w[8], g[8];
    if (io.nv == 8) {
        load8(a.p + io.base, w);
        load_grad8<BF16>(a.g, io.base, g);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            w[e] = e < io.nv ? a.p[io.base + e] : 0.0f;
            g[e] = e < io.nv ? load_grad1<BF16>(a.g, io.base + e) : 0.0f;
        }
    }
    const uint32_t mq = load_codes(a.mq, io);
    const float s_old = a.ms[block];
    const float inv_total = factor_inv_total(a, h);
    float mt[8], amax = 0.0f;
    int64_t i = io.i, j = io.j;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (e < io.nv) {
            const float2 tt = s.deq[(mq >> (8 * (e >> 1))) & 255u];
            const float m_prev = ((e & 1) ? tt.y : tt.x) * s_old;
            mt[e] = moment_m(h, m_prev, g[e]);
            const float rn = stat_ema(h, a.r[i], a.r_new[i]) * inv_total;
            const float vt = rn * stat_ema(h, a.c[j], a.c_new[j]);
            w[e] = param_update(h, w[e], mt[e], vt);
            amax = fmaxf(amax, fabsf(mt[e]));
            if (++j == a.cols) { j = 0; ++i; }
        } else {
            mt[e] = 0.0f;
        }
    }
    const float s_new = row16_allmax(amax);
    uint32_t mq_new = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (e < io.nv) mq_new |= quant_m_code(s.search, mt[e], s_new) << (4 * e);
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

// =====================================================================================================
// Uncompressed fp32 states (tensors that are not quantized): Alg. 3 with identity compression.
// One workgroup handles kElemsPerWg32 consecutive elements.
// =====================================================================================================

template <bool BF16>
__device__ __forceinline__ void adamw32_tile(float* p, const void* g, float* m, float* v, int64_t n,
                                             const Hyper& h, int wg) {
    const int64_t base = int64_t(wg) * kElemsPerWg32;
#pragma unroll 4
    for (int k = 0; k < kElemsPerWg32 / kThreads; ++k) {
        const int64_t idx = base + int64_t(k) * kThreads + threadIdx.x;
        if (idx < n) {
            const float gi = load_grad1<BF16>(g, idx);
            const float mt = moment_m(h, m[idx], gi);
            const float vt = moment_v(h, v[idx], gi);
            m[idx] = mt;
            v[idx] = vt;
            p[idx] = param_update(h, p[idx], mt, vt);
        }
    }
}

// SGD with momentum on an uncompressed fp32 buffer (tensors that are not quantized)
template <bool BF16>
__device__ __forceinline__ void sgdm32_tile(float* p, const void* g, float* m, int64_t n, const Hyper& h, int wg) {
    const int64_t base = int64_t(wg) * kElemsPerWg32;
#pragma unroll 4
    for (int k = 0; k < kElemsPerWg32 / kThreads; ++k) {
        const int64_t idx = base + int64_t(k) * kThreads + threadIdx.x;
        if (idx < n) {
            const float mt = moment_sgdm(h, m[idx], load_grad1<BF16>(g, idx));
            m[idx] = mt;
            p[idx] = param_sgdm(h, p[idx], mt);
        }
    }
}

// =====================================================================================================
// Kernels for one tensor: two launches per step.
// =====================================================================================================

template <bool BF16>
__global__ __launch_bounds__(kThreads) void pass1_fast(const Tensor4 a, const Hyper h) {
    __shared__ Lds s;
    const int wg = logical_wg();
    if (wg >= a.n_wg) return;
    if (a.flat) pass1_flat_tile<BF16>(a, h, wg, s);
    else pass1_fast_tile<BF16, false>(a, h, wg, s);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void pass2_fast(const Tensor4 a, const Hyper h) {
    __shared__ int s_last;
    const int wg = logical_wg();
    if (wg < a.n_wg2) pass2_fast_tile<BF16>(a, h, wg);
    publish_if_last(a, blockIdx.x, gridDim.x, s_last);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void b128_kernel(const Tensor4 a, const Hyper h) {
    __shared__ Lds s;
    const int wg = logical_wg();
    if (wg < a.n_wg) b128_work<BF16>(a, h, wg, s);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void factor_stats_fast(const Tensor4 a) {
    __shared__ Lds s;
    const int wg = logical_wg();
    if (wg < a.n_wg) factor_stats_tile<BF16>(a, wg, s);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void factor_update_fast(const Tensor4 a, const Hyper h) {
    __shared__ Lds s;
    __shared__ int s_last;
    const int wg = logical_wg();
    if (wg < a.n_wg2) factor_update_tile<BF16>(a, h, wg, s);
    factor_publish_if_last(a, h, blockIdx.x, gridDim.x, s_last);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void factor_stats_general(const Tensor4 a) {
    __shared__ Lds s;
    factor_stats_general_tile<BF16>(a, blockIdx.x, gridDim.x, s);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void factor_update_general(const Tensor4 a, const Hyper h) {
    __shared__ Lds s;
    __shared__ int s_last;
    load_tables(s);
    factor_update_general_tile<BF16>(a, h, blockIdx.x, s);
    factor_publish_if_last(a, h, blockIdx.x, gridDim.x, s_last);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void sgdm4_kernel(const Tensor4 a, const Hyper h) {
    __shared__ Lds s;
    const int wg = logical_wg();
    if (wg < a.n_wg) b128_work<BF16, true>(a, h, wg, s);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void sgdm32_kernel(float* p, const void* g, float* m, int64_t n, const Hyper h) {
    sgdm32_tile<BF16>(p, g, m, n, h, blockIdx.x);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void pass1_general(const Tensor4 a, const Hyper h) {
    __shared__ Lds s;
    pass1_general_tile<BF16>(a, h, blockIdx.x, s);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void pass2_general(const Tensor4 a, const Hyper h) {
    __shared__ int s_last;
    pass2_general_tile<BF16>(a, h, blockIdx.x);
    publish_if_last(a, blockIdx.x, gridDim.x, s_last);
}

template <bool BF16>
__global__ __launch_bounds__(kThreads) void adamw32_kernel(float* p, const void* g, float* m, float* v,
                                                           int64_t n, const Hyper h) {
    adamw32_tile<BF16>(p, g, m, v, n, h, blockIdx.x);
}

// =====================================================================================================
// Phase kernel of the multi-tensor step.  A phase runs the "A" work of one set of tensors (pass 1
// of quantized tensors, the whole update of fp32-state tensors) together with the "B" work of the
// previous set (pass 2).  The two kinds are interleaved in proportion, so that at any time each CU
// holds memory-bound pass-1 workgroups next to arithmetic-bound pass-2 workgroups.
// =====================================================================================================

// Hyper-parameters of a plan's launches: by value, or -- for a step that is captured into a graph and replayed
// while the learning rate and the step number change -- read from device memory, where a one-thread kernel
// enqueued in front of the step has put them.
struct HyperArg {
    Hyper h;
    const Hyper* dev;       // non-null: use *dev
};
__device__ __forceinline__ Hyper resolve(const HyperArg& a) { return a.dev ? *a.dev : a.h; }

// the host's make_hyper on the device: lr and the step number come from device memory
__global__ void hyper_prepare_kernel(const float* lr_dev, const int64_t* step_dev, float beta1, float beta2, float eps,
                                     float wd, Hyper* out) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const double lr = double(*lr_dev);
    int64_t t = *step_dev;
    if (t < 1) t = 1;
    Hyper h;
    h.beta1 = beta1;
    h.beta2 = beta2;
    h.omb1 = 1.0f - beta1;
    h.omb2 = 1.0f - beta2;
    h.eps = eps;
    const double bc1 = 1.0 - pow(double(beta1), double(t));
    const double bc2 = 1.0 - pow(double(beta2), double(t));
    h.step_size = float(lr / bc1);
    h.inv_sqrt_bc2 = float(1.0 / sqrt(bc2));
    h.lr_wd = float(lr * double(wd));
    *out = h;
}
__global__ void sgdm_hyper_prepare_kernel(const float* lr_dev, float momentum, Hyper* out) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    Hyper h{};
    h.beta1 = momentum;
    h.step_size = *lr_dev;
    *out = h;
}

struct Segment {        // a run of workgroups that work on one tensor
    int wg_begin;       // first workgroup of the run, in its kind's numbering
    int tensor;         // index into the tensor table
};

// Tensors per kind in one phase; the tables travel as kernel arguments (3 KiB of the 4 KiB a launch may carry).
// As many as fit: sets of a few hundred small tensors run fastest as a single group (the 108 M-parameter set of 197
// tensors: 0.361 ms per step as one group against 0.397 as two with their passes overlapped).
constexpr int kMaxSeg = 192;

struct Phase {
    const Tensor4Table* tensors;
    int n_seg_a, n_seg_b;
    int n_a, n_b;           // workgroups of each kind
    Segment seg_a[kMaxSeg];
    Segment seg_b[kMaxSeg];
};

static_assert(sizeof(Phase) + sizeof(HyperArg) <= 4000, "kernel arguments of a phase launch");

// the hyper-parameters as they apply to one tensor of a plan
__device__ __forceinline__ Hyper for_tensor(const Hyper& h, const Tensor4& a) {
    Hyper t = h;
    if (a.no_decay) t.lr_wd = 0.0f;
    return t;
}

// last segment whose first workgroup is <= wg (segments are sorted by wg_begin, seg[0].wg_begin = 0;
// a uniform binary search on scalar registers)
__device__ __forceinline__ Segment find_segment(const Segment* seg, int n_seg, int wg) {
    int lo = 0, hi = n_seg;                 // answer in [lo, hi)
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (seg[mid].wg_begin <= wg) lo = mid; else hi = mid;
    }
    return seg[lo];
}

// ROLES: 0 = A and B work interleaved in one launch; 1 = A work only; 2 = B work only; 3 = A work
// only of a group without rank-1 tensors (block-wise and fp32-state tensors: no pass-1 code).  The
// single-role kernels exist because a kernel's register and LDS footprint is that of its heaviest
// path: launched on their own (on a second stream), the light pass-2 workgroups fit into the
// register space that the resident pass-1 workgroups leave free.
template <bool BF16, int ROLES>
__global__ __launch_bounds__(kThreads) void phase_kernel(const Phase ph, const HyperArg ha) {
    const Hyper h = resolve(ha);
    const int x = logical_wg();
    constexpr bool kOnlyA = ROLES == 1 || ROLES == 3;
    const int n = (ROLES == 2 ? 0 : ph.n_a) + (kOnlyA ? 0 : ph.n_b);
    if (x >= n) return;
    // B workgroups sit at the positions where floor(x * n_b / n) steps up
    const int b_before = kOnlyA ? 0 : (ROLES == 2 ? x : int((int64_t(x) * ph.n_b) / n));
    const int b_after = kOnlyA ? 0 : (ROLES == 2 ? x + 1 : int((int64_t(x + 1) * ph.n_b) / n));
    if (!kOnlyA && b_after > b_before) {
        __shared__ int s_last;
        const Segment sg = find_segment(ph.seg_b, ph.n_seg_b, b_before);
        const Tensor4 a = from_table(ph.tensors[sg.tensor]);
        const int wg = b_before - sg.wg_begin;
        if (a.kind == kQuantFast) pass2_fast_tile<BF16>(a, h, wg);
        else pass2_general_tile<BF16>(a, h, wg);
        publish_if_last(a, wg, a.n_wg2, s_last);
    } else if (ROLES != 2) {
        __shared__ Lds s;
        const int xa = x - b_before;
        const Segment sg = find_segment(ph.seg_a, ph.n_seg_a, xa);
        const Tensor4 a = from_table(ph.tensors[sg.tensor]);
        const Hyper ht = for_tensor(h, a);
        const int wg = xa - sg.wg_begin;
        if (a.kind == kFp32State) {
            adamw32_tile<BF16>(a.p, a.g, reinterpret_cast<float*>(a.mq), reinterpret_cast<float*>(a.vq), a.P, ht, wg);
        } else if (a.kind == kQuantBlockV) {
            b128_work<BF16>(a, ht, wg, s);
        } else if (ROLES == 3) {
            // not reached: the host launches this variant only for groups without rank-1 tensors
        } else if (a.kind == kQuantFast) {
            if (a.flat) pass1_flat_tile<BF16>(a, ht, wg, s);
            else pass1_fast_tile<BF16, false>(a, ht, wg, s);
        } else {
            pass1_general_tile<BF16>(a, ht, wg, s);
        }
    }
}

// =====================================================================================================
// Rank-1 normalization of a tensor with more than two dimensions (App. F Alg. 4): one statistic per
// index of every dimension, an element's scale is the minimum of its statistics.  Seen as a matrix of
// d_1 rows and d_2 * ... * d_p columns, the scale is min(mu_1[i], colscale[col]) with colscale[col] =
// min over the other dimensions of their statistic at the column's index: the two passes of the
// matrix step run unchanged on (mu_1, colscale), and two small kernels between them turn the column
// maxima of v_t into the new statistics (reduce) and those into the new colscale (expand).
// =====================================================================================================

constexpr int kMaxInnerDims = 7;

struct InnerDims {                  // dimensions 2..p
    int n;
    int64_t d[kMaxInnerDims];       // sizes
    int64_t first[kMaxInnerDims];   // where each dimension's statistics start in the statistics array
};

// One workgroup per statistic: mu_new[first[r] + j] = max of colmax over the columns whose index in inner
// dimension r is j (cols / d_r of them: col = a * d_r * inner + j * inner + b).  No atomics: with a small
// dimension (a 3 x 3 kernel) thousands of columns share a statistic, and atomics on one address queue up.
// `stat` = which statistic this workgroup computes (0 .. d_2 + ... + d_p - 1).
__device__ __forceinline__ void nd_reduce_one(const float* colmax, float* mu_new, int64_t cols, const InnerDims& dm,
                                              int64_t stat, float* s_part) {
    int r = 0;
    int64_t j = stat;
    while (r < dm.n - 1 && j >= dm.d[r]) { j -= dm.d[r]; ++r; }
    int64_t inner = 1;
    for (int q = r + 1; q < dm.n; ++q) inner *= dm.d[q];
    const int64_t count = cols / dm.d[r];
    float m = 0.0f;
    for (int64_t k = threadIdx.x; k < count; k += kThreads) {
        const int64_t a = k / inner, b = k - a * inner;
        m = fmaxf(m, colmax[(a * dm.d[r] + j) * inner + b]);
    }
    m = row16_allmax(m);                    // values are >= +0
    m = fmaxf(m, __shfl_xor(m, 16));
    m = fmaxf(m, __shfl_xor(m, 32));
    if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) mu_new[dm.first[r] + j] = fmaxf(fmaxf(s_part[0], s_part[1]), fmaxf(s_part[2], s_part[3]));
}

// colscale[col] = min over the inner dimensions of mu[first[r] + idx_r(col)]
__device__ __forceinline__ void nd_expand_one(const float* mu, float* colscale, int64_t cols, const InnerDims& dm,
                                              int64_t col) {
    if (col >= cols) return;
    int64_t rest = col;
    float m = 0.0f;
    for (int r = dm.n - 1; r >= 0; --r) {
        const int64_t idx = rest % dm.d[r];
        rest /= dm.d[r];
        const float v = mu[dm.first[r] + idx];
        m = (r == dm.n - 1) ? v : fminf(m, v);
    }
    colscale[col] = m;
}

__global__ __launch_bounds__(kThreads) void nd_reduce_kernel(const float* colmax, float* mu_new, int64_t cols,
                                                             const InnerDims dm) {
    __shared__ float s_part[kThreads / 64];
    nd_reduce_one(colmax, mu_new, cols, dm, blockIdx.x, s_part);
}

__global__ __launch_bounds__(kThreads) void nd_expand_kernel(const float* mu, float* colscale, int64_t cols,
                                                             const InnerDims dm) {
    nd_expand_one(mu, colscale, cols, dm, int64_t(blockIdx.x) * kThreads + threadIdx.x);
}

// The two small kernels between the passes for all tensors with more than two dimensions of one group of a plan.
struct NdPhase {
    const Tensor4Table* tensors;
    const InnerDims* dims;          // device table, indexed by Tensor4::nd_index
    int n_seg, n_r, n_e;            // tensors; workgroups of the reduce and of the expand kernel
    Segment seg_r[kMaxSeg];         // per tensor: first workgroup of the reduce kernel (one per statistic)
    Segment seg_e[kMaxSeg];         // per tensor: first workgroup of the expand kernel (one per 256 columns)
};

static_assert(sizeof(NdPhase) <= 4000, "kernel arguments of the reduce / expand launches");

__global__ __launch_bounds__(kThreads) void nd_plan_reduce(const NdPhase ph) {
    __shared__ float s_part[kThreads / 64];
    const int x = blockIdx.x;
    if (x >= ph.n_r) return;
    const Segment sg = find_segment(ph.seg_r, ph.n_seg, x);
    const Tensor4 a = from_table(ph.tensors[sg.tensor]);
    const InnerDims dm = ph.dims[a.nd_index];
    nd_reduce_one(a.c_new, a.c_new + a.cols, a.cols, dm, x - sg.wg_begin, s_part);
}

__global__ __launch_bounds__(kThreads) void nd_plan_expand(const NdPhase ph) {
    const int x = blockIdx.x;
    if (x >= ph.n_e) return;
    const Segment sg = find_segment(ph.seg_e, ph.n_seg, x);
    const Tensor4 a = from_table(ph.tensors[sg.tensor]);
    const InnerDims dm = ph.dims[a.nd_index];
    nd_expand_one(a.c_new + a.cols, a.c_new, a.cols, dm, int64_t(x - sg.wg_begin) * kThreads + threadIdx.x);
}

// The reduce and totals steps for all tensors with deterministic sums of one group of a plan.
struct DetPhase {
    const Tensor4Table* tensors;
    int n_seg, n_r;                 // tensors; workgroups of the reduce kernel
    Segment seg_r[kMaxSeg];         // per tensor: first workgroup of the reduce kernel
};

__global__ __launch_bounds__(kThreads) void factor_plan_reduce(const DetPhase ph) {
    __shared__ float s_part[kThreads / 64];
    const int x = blockIdx.x;
    if (x >= ph.n_r) return;
    const Segment sg = find_segment(ph.seg_r, ph.n_seg, x);
    factor_reduce_one(from_table(ph.tensors[sg.tensor]), x - sg.wg_begin, s_part);
}

__global__ __launch_bounds__(kThreads) void factor_plan_totals(const DetPhase ph) {
    __shared__ float s_part[kThreads / 64];
    if (int(blockIdx.x) >= ph.n_seg) return;
    factor_totals_one(from_table(ph.tensors[ph.seg_r[blockIdx.x].tensor]), s_part);
}

// The same for a plan whose 2-dimensional tensors keep a factorized second moment: "A" work is the
// statistics pass (next to block-wise and fp32-state tensors, which are complete after it), "B" work
// the update pass.  ROLES: 0 = both interleaved, 1 = A only, 2 = B only.  Separate kernels, so that the
// rank-1 kernels above keep their register footprint.
template <bool BF16, int ROLES>
__global__ __launch_bounds__(kThreads) void factor_phase_kernel(const Phase ph, const HyperArg ha) {
    const Hyper h = resolve(ha);
    __shared__ Lds s;
    const int x = logical_wg();
    const int n = (ROLES == 2 ? 0 : ph.n_a) + (ROLES == 1 ? 0 : ph.n_b);
    if (x >= n) return;
    const int b_before = ROLES == 1 ? 0 : (ROLES == 2 ? x : int((int64_t(x) * ph.n_b) / n));
    const int b_after = ROLES == 1 ? 0 : (ROLES == 2 ? x + 1 : int((int64_t(x + 1) * ph.n_b) / n));
    if (ROLES != 1 && b_after > b_before) {
        __shared__ int s_last;
        const Segment sg = find_segment(ph.seg_b, ph.n_seg_b, b_before);
        const Tensor4 a = from_table(ph.tensors[sg.tensor]);
        const Hyper ht = for_tensor(h, a);
        const int wg = b_before - sg.wg_begin;
        if (a.kind == kFactorFast) {
            factor_update_tile<BF16>(a, ht, wg, s);
        } else {
            load_tables(s);
            factor_update_general_tile<BF16>(a, ht, wg, s);
        }
        factor_publish_if_last(a, h, wg, a.n_wg2, s_last);
    } else if (ROLES != 2) {
        const int xa = x - b_before;
        const Segment sg = find_segment(ph.seg_a, ph.n_seg_a, xa);
        const Tensor4 a = from_table(ph.tensors[sg.tensor]);
        const int wg = xa - sg.wg_begin;
        const Hyper ht = for_tensor(h, a);
        if (a.kind == kFp32State)
            adamw32_tile<BF16>(a.p, a.g, reinterpret_cast<float*>(a.mq), reinterpret_cast<float*>(a.vq), a.P, ht, wg);
        else if (a.kind == kQuantBlockV) b128_work<BF16>(a, ht, wg, s);
        else if (a.kind == kFactorFast) factor_stats_tile<BF16>(a, wg, s);
        else factor_stats_general_tile<BF16>(a, wg, a.n_wg, s);
    }
}

// A plan of SGD-with-momentum tensors (App. E Alg. 2): everything is one pass, so only "A" work exists.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void sgdm_phase_kernel(const Phase ph, const HyperArg ha) {
    const Hyper h = resolve(ha);
    __shared__ Lds s;
    const int x = logical_wg();
    if (x >= ph.n_a) return;
    const Segment sg = find_segment(ph.seg_a, ph.n_seg_a, x);
    const Tensor4 a = from_table(ph.tensors[sg.tensor]);
    const int wg = x - sg.wg_begin;
    if (a.kind == kSgdmFp32) sgdm32_tile<BF16>(a.p, a.g, reinterpret_cast<float*>(a.mq), a.P, h, wg);
    else b128_work<BF16, true>(a, h, wg, s);
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

__global__ __launch_bounds__(kThreads) void dequant_m_kernel(const QuantArgs q) {
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(q.P, q.cols, t);
    if (!io.nv) return;
    const uint32_t w = load_codes(q.q_in, io);
    const float s = q.sa[t >> 4];
    for (int e = 0; e < io.nv; ++e)
        q.x_out[io.base + e] = d_byte_decode[2 * ((w >> (4 * e)) & 15u)] * s;   // entry b<16: {T[b], T[0]}
}

__global__ __launch_bounds__(kThreads) void dequant_v_kernel(const QuantArgs q) {
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(q.P, q.cols, t);
    if (!io.nv) return;
    const uint32_t w = load_codes(q.q_in, io);
    int64_t i = io.i, j = io.j;
    for (int e = 0; e < io.nv; ++e) {
        q.x_out[io.base + e] = dequant_v((w >> (4 * e)) & 15u, fminf(q.sa[i], q.sb[j]));
        if (++j == q.cols) { j = 0; ++i; }
    }
}

// second moment with block scales (1-dimensional / flattened tensors)
__global__ __launch_bounds__(kThreads) void dequant_vb_kernel(const QuantArgs q) {
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(q.P, q.cols, t);
    if (!io.nv) return;
    const uint32_t w = load_codes(q.q_in, io);
    const float s = q.sa[t >> 4];
    for (int e = 0; e < io.nv; ++e) q.x_out[io.base + e] = dequant_v((w >> (4 * e)) & 15u, s);
}

__global__ __launch_bounds__(kThreads) void quant_m_kernel(const QuantArgs q) {
    __shared__ Lds s;
    load_tables(s);
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    if ((t >> 4) * 128 >= q.P) return;
    const LaneIo io = lane_io(q.P, q.cols, t);
    float x[8], amax = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        x[e] = e < io.nv ? q.x_in[io.base + e] : 0.0f;
        amax = fmaxf(amax, fabsf(x[e]));
    }
    const float sc = row16_allmax(amax);
    uint32_t w = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (e < io.nv) w |= quant_m_code(s.search, x[e], sc) << (4 * e);
    if (io.nv) store_codes(q.q_out, io, w);
    if ((threadIdx.x & 15) == 0) q.sa[t >> 4] = sc;
}

// block-wise second moment (values >= 0): block maximum, Linear map
__global__ __launch_bounds__(kThreads) void quant_vb_kernel(const QuantArgs q) {
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    if ((t >> 4) * 128 >= q.P) return;
    const LaneIo io = lane_io(q.P, q.cols, t);
    float x[8], vmax = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        x[e] = e < io.nv ? q.x_in[io.base + e] : 0.0f;
        vmax = fmaxf(vmax, fabsf(x[e]));
    }
    const float sc = row16_allmax(vmax);
    uint32_t w = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (e < io.nv) w |= quant_v_code(x[e], sc) << (4 * e);
    if (io.nv) store_codes(q.q_out, io, w);
    if ((threadIdx.x & 15) == 0) q.sa[t >> 4] = sc;
}

// second moment, stage 1: row / column maxima into sa / sb (which must be zero on entry)
__global__ __launch_bounds__(kThreads) void quant_v_max_kernel(const QuantArgs q) {
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(q.P, q.cols, t);
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
    const int64_t t = int64_t(blockIdx.x) * kThreads + threadIdx.x;
    const LaneIo io = lane_io(q.P, q.cols, t);
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
