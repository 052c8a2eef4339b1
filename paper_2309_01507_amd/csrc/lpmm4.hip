// lpmm4.so -- C ABI and launch logic of the 4-bit AdamW step (declared in include/lpmm4.h).
// Host side only: argument checks, launch geometry, bias corrections.  All arithmetic of the
// method runs in the kernels of kernels.hpp.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <memory>
#include <mutex>
#include <unordered_map>
#include <vector>

#include "../../include/lpmm4.h"
#include "kernels.hpp"
#include "ablation.hpp"

namespace {

using namespace lpmm;

constexpr int kMaxDevices = 16;
static_assert(kCounterWords * 4 <= 8192, "counter block");
constexpr size_t kCounterBytes = 8192;  // tail of the workspace: ticket counters of pass 2, one cache line apart

struct DeviceCtx {
    bool ready = false;
    float* ws = nullptr;        // workspace: floats [0, cap) for r', c'; then counters
    int64_t cap_floats = 0;
    unsigned int* counter = nullptr;
    int n_cu = 256;
    unsigned char* scratch = nullptr;   // this device's copy of `scratch` below (its address on this device)
};

// Device memory of the library's own for lpmm_adamw4_step_noalloc: the ticket counters of pass 2, then the row
// and column maxima of the updated second moment.  Every GPU that loads the library holds one copy until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress; the address of a device's
// copy is DeviceCtx::scratch, looked up once per device by lpmm_adamw4_init.
constexpr int64_t kScratchFloats = LPMM_NOALLOC_MAX_ROWS_PLUS_COLS + 128;     // rows and cols each padded to 64
static __device__ __align__(256) unsigned char scratch[kCounterBytes + kScratchFloats * 4];

DeviceCtx g_ctx[kMaxDevices];
std::mutex g_mu;
thread_local int g_last_hip = 0;

// per-kernel timing (lpmm_profile_begin / _end)
struct Profile {
    bool on = false;
    int64_t max_calls = 0, calls = 0;
    std::vector<hipEvent_t> ev;    // 3 per recorded call
};
Profile g_prof;

hipEvent_t prof_event(int64_t call, int which) {
    return g_prof.ev[size_t(call) * 3 + which];
}

// host copies of the tables (also serve the host-only entry points)
struct HostTables {
    float de[kCodes], lin[kCodes], thr[kCodes - 1];
    float byte_decode[512];
    SearchEntry search[kBucketsPadded];
    bool ok;
    HostTables() {
        build_de_signed(de);
        build_linear(lin);
        build_thresholds(de, thr);
        ok = build_search(thr, search);
        build_byte_decode(de, byte_decode);
    }
};
const HostTables& host_tables() { static const HostTables t; return t; }

int hip_fail(hipError_t e) { g_last_hip = int(e); return LPMM_EHIP; }
#define LPMM_HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) return hip_fail(e_); } while (0)

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
bool finite_nonneg(float x) { return std::isfinite(x) && x >= 0.0f; }

int env_int(const char* name, int dflt) {
    const char* s = std::getenv(name);
    return (s && *s) ? std::atoi(s) : dflt;
}

int check_shape(const int64_t* shape, int64_t* rows, int64_t* cols) {
    if (!shape) return LPMM_EINVAL;
    if (shape[0] < 1 || shape[1] < 1) return LPMM_EINVAL;
    if (shape[0] > (int64_t(1) << 31) || shape[1] > (int64_t(1) << 31)) return LPMM_EINVAL;
    if (shape[0] * shape[1] > (int64_t(1) << 40)) return LPMM_EINVAL;
    *rows = shape[0];
    *cols = shape[1];
    return LPMM_OK;
}

int make_hyper(float lr, float beta1, float beta2, float eps, float wd, int64_t step, Hyper* h) {
    if (step < 1) return LPMM_EINVAL;
    if (!finite_nonneg(lr) || !finite_nonneg(eps) || !finite_nonneg(wd)) return LPMM_EINVAL;
    if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f)) return LPMM_EINVAL;
    h->beta1 = beta1;
    h->beta2 = beta2;
    h->omb1 = 1.0f - beta1;
    h->omb2 = 1.0f - beta2;
    h->eps = eps;
    const double bc1 = 1.0 - std::pow(double(beta1), double(step));
    const double bc2 = 1.0 - std::pow(double(beta2), double(step));
    h->step_size = float(double(lr) / bc1);
    h->inv_sqrt_bc2 = float(1.0 / std::sqrt(bc2));
    h->lr_wd = float(double(lr) * double(wd));
    return LPMM_OK;
}

int current_ctx(DeviceCtx** out) {
    int dev = 0;
    LPMM_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices || !g_ctx[dev].ready) return LPMM_ENOTINIT;
    *out = &g_ctx[dev];
    return LPMM_OK;
}

int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
int pad8(int64_t n) { return int(round_up(n, kXcds)); }

// Geometry of the fast path.  gx column blocks share a workgroup (so that one workgroup touches
// whole 128-byte lines of codes and runs of block scales), gy = 8/gx groups walk interleaved
// rows of the same column blocks and combine their column maxima in LDS.  rw_hint > 0 fixes the
// rows per workgroup; otherwise they are chosen so that the tensor alone fills the chip.
// log2 of the smallest S in {1, 2, 4, 8} for which S rows of `row_bytes` bytes are a multiple of 32 KiB; 0 if
// there is none.  Rows in flight side by side then lie 32 KiB apart, which is what the memory system serves
// fastest (measured).  S must divide `per_group`, the rows of a tile that one group (or wave) takes: only
// then does row(k) = g*S + k%S + (k/S)*groups*S enumerate every row of the tile exactly once.
int row_spacing_log2(int64_t row_bytes, int64_t rows_per_tile, int groups, const char* env) {
    if (rows_per_tile % groups) return 0;
    const int64_t per_group = rows_per_tile / groups;
    auto fits = [&](int l) { return l >= 0 && l <= 3 && (per_group % (int64_t(1) << l)) == 0; };
    const int forced = env_int(env, -1);
    if (forced >= 0) return fits(forced) ? forced : 0;
    for (int l = 0; fits(l); ++l)
        if (((row_bytes << l) % 32768) == 0) return l;
    return 0;
}

void fast_geometry(Tensor4* a, int n_cu, int64_t rw_hint, int64_t rw2_hint, int grad_bytes, bool flat_default = false) {
    a->nb = int(a->cols / LPMM_BLOCK);
    int gx = env_int("LPMM_GX", 1);
    if (gx < 1 || gx > kGroups || (gx & (gx - 1))) gx = 1;
    while (gx > 1 && (a->nb % gx) != 0) gx >>= 1;
    a->gx = gx;
    a->gy = kGroups / gx;
    a->strips = a->nb / gx;
    int64_t rw = env_int("LPMM_RW", 0);
    if (rw <= 0) rw = rw_hint < 0 ? 64 : rw_hint;       // rw_hint: 0 = a tensor on its own (sized below), -1 = in a plan
    if (rw <= 0) {
        // tall tiles amortize a workgroup's start-up and its column atomics; shrink them only as
        // far as needed to give every CU a couple of workgroups
        rw = 64;
        while (rw > a->gy && a->strips * ((a->rows + rw - 1) / rw) < 2 * int64_t(n_cu)) rw >>= 1;
    }
    const int64_t cap = (int64_t(1) << 29) / a->cols;     // lane offsets inside a tile stay below 2^31 bytes
    if (rw > cap) rw = cap;
    if (rw * gx > kMaxRowSlots) rw = kMaxRowSlots / gx;    // per-row results of a tile are staged in LDS
    rw = round_up(rw, a->gy);
    if (rw > cap || rw * gx > kMaxRowSlots) rw -= a->gy;
    if (rw > a->rows) rw = round_up(a->rows, a->gy);
    if (rw < a->gy) rw = a->gy;
    a->rw = int(rw);
    a->n_wg = int(a->strips * ((a->rows + rw - 1) / rw));
    a->rs = row_spacing_log2(a->cols * 4, rw, a->gy, "LPMM_RS");      // the parameters' rows
    a->flat = 0;
    // Flat tiling of pass 1 (strips of 8 column blocks, the 8 groups take rows, each walks along its row): the
    // caller decides (flat_default); LPMM_FLAT = 0 / 1 overrides.
    const int flat_env = env_int("LPMM_FLAT", -1);
    const bool want_flat = flat_env >= 0 ? flat_env != 0 : flat_default;
    if (want_flat && a->kind == kQuantFast) {
        a->flat = 1;
        a->gx = 1; a->gy = kGroups;
        a->strips = (a->nb + kFlatBlocks - 1) / kFlatBlocks;
        int64_t rwf = env_int("LPMM_RW", 0);
        if (rwf <= 0) rwf = rw_hint > 0 ? rw_hint : 32;
        if (rwf > 64) rwf = 64;                                   // rw * 8 block results are staged in LDS
        const int64_t capf = (int64_t(1) << 29) / a->cols;
        if (rwf > capf) rwf = capf;
        rwf = round_up(rwf, kGroups);
        if (rwf > capf || rwf > 64) rwf -= kGroups;
        if (rwf > a->rows) rwf = round_up(a->rows, kGroups);
        if (rwf < kGroups) rwf = kGroups;
        a->rw = int(rwf);
        a->n_wg = int(a->strips * ((a->rows + rwf - 1) / rwf));
        a->rs = row_spacing_log2(a->cols * 4, rwf, kGroups, "LPMM_RS");
    }
    // pass 2: strips of 256 columns, a wave per row
    a->strips2 = (a->nb + 1) / 2;
    int64_t rw2 = env_int("LPMM_RW2", 0);
    if (rw2 <= 0) rw2 = rw2_hint;
    if (rw2 <= 0) {
        rw2 = 64;
        while (rw2 > kWaves && a->strips2 * ((a->rows + rw2 - 1) / rw2) < 2 * int64_t(n_cu)) rw2 >>= 1;
    }
    if (rw2 > cap) rw2 = cap;
    if (rw2 > kMaxRw2) rw2 = kMaxRw2;                       // a wave of pass 2 keeps its rows' scalars one per lane
    if (rw2 > a->rows) rw2 = a->rows;
    if (rw2 < 1) rw2 = 1;
    a->rw2 = int(rw2);
    a->n_wg2 = int(a->strips2 * ((a->rows + rw2 - 1) / rw2));
    a->rs2 = row_spacing_log2(a->cols * grad_bytes, rw2, kWaves, "LPMM_RS2");   // pass 2 mostly reads the gradient
}

// Tiling of a tensor whose second moment is block-wise: super-tiles of 8 x 64 blocks, each shared by
// 64 / rounds workgroups (rounds: a power of two, blocks that a group takes in a row), plus one workgroup
// for a partial last block.  rounds_hint > 0 fixes the rounds.
void b128_geometry(Tensor4* a, int n_cu, int64_t rounds_hint) {
    a->nb = int(a->P / LPMM_BLOCK);
    const int64_t supers = (a->nb + kB128Super - 1) / kB128Super;
    int64_t want = env_int("LPMM_B128_ROUNDS", 0);
    if (want <= 0) want = rounds_hint;
    int64_t rounds = 16;
    if (want > 0) {
        rounds = 1;
        while (rounds * 2 <= want && rounds * 2 <= kB128MaxRounds) rounds *= 2;      // round down to a power of two
    } else {
        while (rounds > 1 && supers * (kB128Stride / rounds) < 2 * int64_t(n_cu)) rounds >>= 1;
    }
    a->rw = int(rounds);
    a->n_wg2 = int(supers * (kB128Stride / rounds));
    a->n_wg = a->n_wg2 + ((a->P % LPMM_BLOCK) ? 1 : 0);
    a->gx = 1; a->gy = kGroups; a->strips = 1; a->strips2 = 1; a->rw2 = 1;
}

bool fast_eligible(int64_t cols, const float* v_colmax) {
    return (cols % LPMM_BLOCK) == 0 && cols < (int64_t(1) << 24) && aligned(v_colmax, 16) &&     // 24-bit row offsets
           !env_int("LPMM_FORCE_GENERAL", 0);
}

// general path: pass 2 takes one chunk of 2048 elements per workgroup, pass 1 several consecutive ones (the
// more, the fewer atomics leave the workgroup; few enough that the tensor alone still fills the chip)
void general_geometry(Tensor4* a, int n_cu) {
    const int64_t chunks = (a->P + kGenChunkElems - 1) / kGenChunkElems;
    int64_t per_wg = env_int("LPMM_GEN_CHUNKS", 0);
    if (per_wg <= 0) per_wg = chunks / (4 * int64_t(n_cu));
    if (per_wg < 1) per_wg = 1;
    if (per_wg > kGenMaxChunks) per_wg = kGenMaxChunks;
    a->rw = int(per_wg);
    a->n_wg = int((chunks + per_wg - 1) / per_wg);
    a->n_wg2 = int(chunks);
}

template <bool BF16>
int launch_step(const Tensor4& t, const Hyper& h, bool fast, hipStream_t s) {
    const bool rec = g_prof.on && g_prof.calls < g_prof.max_calls;
    const int64_t call = g_prof.calls;
    if (rec) LPMM_HIP(hipEventRecord(prof_event(call, 0), s));
    const int grid = fast ? pad8(t.n_wg) : t.n_wg;
    if (fast) hipLaunchKernelGGL(pass1_fast<BF16>, dim3(grid), dim3(kThreads), 0, s, t, h);
    else hipLaunchKernelGGL(pass1_general<BF16>, dim3(grid), dim3(kThreads), 0, s, t, h);
    LPMM_HIP(hipGetLastError());
    if (rec) LPMM_HIP(hipEventRecord(prof_event(call, 1), s));
    if (fast) hipLaunchKernelGGL(pass2_fast<BF16>, dim3(pad8(t.n_wg2)), dim3(kThreads), 0, s, t, h);
    else hipLaunchKernelGGL(pass2_general<BF16>, dim3(t.n_wg2), dim3(kThreads), 0, s, t, h);
    LPMM_HIP(hipGetLastError());
    if (rec) {
        LPMM_HIP(hipEventRecord(prof_event(call, 2), s));
        g_prof.calls = call + 1;
    }
    return LPMM_OK;
}

int fill(void* dst, int64_t n, uint8_t value, int64_t last_index, uint8_t last, hipStream_t s);

// Where a single-tensor step keeps its new maxima and ticket counters: the workspace given to lpmm_adamw4_init
// (the default), the library's own device array (lpmm_adamw4_step_noalloc), or a workspace of the caller's
// (lpmm_adamw4_step_ws).
struct WorkspaceChoice {
    bool use_scratch = false;
    void* own = nullptr;
    size_t own_bytes = 0;
};

int step_impl(bool bf16, void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
              uint8_t* v_codes, float* v_rowmax, float* v_colmax, const int64_t* shape, float lr,
              float beta1, float beta2, float eps, float wd, int64_t step, void* stream,
              const WorkspaceChoice& wc = WorkspaceChoice()) {
    int64_t rows, cols;
    int rc = check_shape(shape, &rows, &cols);
    if (rc) return rc;
    if (!param || !grad || !m_codes || !m_blockscale || !v_codes || !v_rowmax || !v_colmax)
        return LPMM_EINVAL;
    if (!aligned(param, 16) || !aligned(grad, 16) || !aligned(m_codes, 4) || !aligned(v_codes, 4) ||
        !aligned(m_blockscale, 4) || !aligned(v_rowmax, 4) || !aligned(v_colmax, 4))
        return LPMM_EINVAL;
    Hyper h;
    rc = make_hyper(lr, beta1, beta2, eps, wd, step, &h);
    if (rc) return rc;
    DeviceCtx* ctx;
    rc = current_ctx(&ctx);
    if (rc) return rc;
    const int64_t rows_pad = round_up(rows, 64), cols_pad = round_up(cols, 64);
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* ws = ctx->ws;
    unsigned int* counter = ctx->counter;
    if (wc.own) {
        // same layout as the workspace of lpmm_adamw4_init: the floats, then the counters in the last 8 KiB
        if (!aligned(wc.own, 256) || wc.own_bytes < kCounterBytes + 256 * sizeof(float)) return LPMM_EINVAL;
        const int64_t cap = int64_t((wc.own_bytes - kCounterBytes) / sizeof(float)) / 64 * 64;
        if (rows_pad + cols_pad > cap) return LPMM_EWORKSPACE;
        ws = static_cast<float*>(wc.own);
        counter = reinterpret_cast<unsigned int*>(static_cast<char*>(wc.own) + size_t(cap) * sizeof(float));
    } else if (wc.use_scratch) {
        if (!ctx->scratch) return LPMM_ENOTINIT;
        if (rows_pad + cols_pad > kScratchFloats) return LPMM_EWORKSPACE;
        // The array keeps what the last call on this device left.  A completed step leaves zeros, a step that
        // was cut short may not have: clear the part this call uses (counters, then the two runs of maxima)
        // with a kernel, so that the call stays capturable.
        rc = fill(ctx->scratch, int64_t(kCounterBytes) + (rows_pad + cols_pad) * int64_t(sizeof(float)), 0, -1, 0, s);
        if (rc) return rc;
        counter = reinterpret_cast<unsigned int*>(ctx->scratch);
        ws = reinterpret_cast<float*>(ctx->scratch + kCounterBytes);
    } else if (rows_pad + cols_pad > ctx->cap_floats) {
        return LPMM_EWORKSPACE;
    }

    Tensor4 t{};
    t.p = static_cast<float*>(param);
    t.g = grad;
    t.mq = reinterpret_cast<uint32_t*>(m_codes);
    t.ms = m_blockscale;
    t.vq = reinterpret_cast<uint32_t*>(v_codes);
    t.r = v_rowmax;
    t.c = v_colmax;
    t.r_new = ws;
    t.c_new = ws + rows_pad;
    t.counter = counter;
    t.rows = rows;
    t.cols = cols;
    t.P = rows * cols;
    const bool fast = fast_eligible(cols, v_colmax);
    t.kind = fast ? kQuantFast : kQuantGeneral;
    if (fast) fast_geometry(&t, ctx->n_cu, 0, 0, bf16 ? 2 : 4);
    else general_geometry(&t, ctx->n_cu);
    return bf16 ? launch_step<true>(t, h, fast, s) : launch_step<false>(t, h, fast, s);
}

int b128_step_impl(bool bf16, void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                   uint8_t* v_codes, float* v_blockscale, int64_t numel, float lr, float beta1, float beta2,
                   float eps, float wd, int64_t step, void* stream) {
    if (numel < 1 || numel > (int64_t(1) << 37)) return LPMM_EINVAL;
    if (!param || !grad || !m_codes || !m_blockscale || !v_codes || !v_blockscale) return LPMM_EINVAL;
    if (!aligned(param, 16) || !aligned(grad, 16) || !aligned(m_codes, 4) || !aligned(v_codes, 4) ||
        !aligned(m_blockscale, 4) || !aligned(v_blockscale, 4))
        return LPMM_EINVAL;
    Hyper h;
    int rc = make_hyper(lr, beta1, beta2, eps, wd, step, &h);
    if (rc) return rc;
    DeviceCtx* ctx;
    rc = current_ctx(&ctx);      // the lookup tables live in device memory filled by init
    if (rc) return rc;
    Tensor4 t{};
    t.p = static_cast<float*>(param);
    t.g = grad;
    t.mq = reinterpret_cast<uint32_t*>(m_codes);
    t.ms = m_blockscale;
    t.vq = reinterpret_cast<uint32_t*>(v_codes);
    t.r = v_blockscale;
    t.rows = 1;
    t.cols = numel;
    t.P = numel;
    t.kind = kQuantBlockV;
    b128_geometry(&t, ctx->n_cu, 0);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool rec = g_prof.on && g_prof.calls < g_prof.max_calls;
    const int64_t call = g_prof.calls;
    if (rec) LPMM_HIP(hipEventRecord(prof_event(call, 0), s));
    if (bf16) hipLaunchKernelGGL(b128_kernel<true>, dim3(pad8(t.n_wg)), dim3(kThreads), 0, s, t, h);
    else hipLaunchKernelGGL(b128_kernel<false>, dim3(pad8(t.n_wg)), dim3(kThreads), 0, s, t, h);
    LPMM_HIP(hipGetLastError());
    if (rec) {
        LPMM_HIP(hipEventRecord(prof_event(call, 1), s));
        LPMM_HIP(hipEventRecord(prof_event(call, 2), s));
        g_prof.calls = call + 1;
    }
    return LPMM_OK;
}

// Workgroups for `items` items at `per_thread` per thread.  Kernels that are not grid-stride loops must
// get the full count (the default cap is the largest grid HIP takes; 2^40 elements stay far below it).
int grid_for(int64_t items, int64_t per_thread, int max_blocks = 0x7FFFFFFF) {
    const int64_t threads = (items + per_thread - 1) / per_thread;
    int64_t blocks = (threads + kThreads - 1) / kThreads;
    if (blocks < 1) blocks = 1;
    if (blocks > max_blocks) blocks = max_blocks;
    return int(blocks);
}

int make_sgdm_hyper(float lr, float momentum, Hyper* h) {
    if (!finite_nonneg(lr) || !(momentum >= 0.0f && momentum < 1.0f)) return LPMM_EINVAL;
    *h = Hyper{};
    h->beta1 = momentum;
    h->step_size = lr;
    return LPMM_OK;
}

int sgdm4_step_impl(bool bf16, void* param, const void* grad, uint8_t* m_codes, float* m_blockscale, int64_t numel,
                    float lr, float momentum, void* stream) {
    if (numel < 1 || numel > (int64_t(1) << 37)) return LPMM_EINVAL;
    if (!param || !grad || !m_codes || !m_blockscale) return LPMM_EINVAL;
    if (!aligned(param, 16) || !aligned(grad, 16) || !aligned(m_codes, 4) || !aligned(m_blockscale, 4))
        return LPMM_EINVAL;
    Hyper h;
    int rc = make_sgdm_hyper(lr, momentum, &h);
    if (rc) return rc;
    DeviceCtx* ctx;
    rc = current_ctx(&ctx);      // the lookup tables live in device memory filled by init
    if (rc) return rc;
    Tensor4 t{};
    t.p = static_cast<float*>(param);
    t.g = grad;
    t.mq = reinterpret_cast<uint32_t*>(m_codes);
    t.ms = m_blockscale;
    t.rows = 1;
    t.cols = numel;
    t.P = numel;
    b128_geometry(&t, ctx->n_cu, 0);
    t.kind = kSgdmBlock;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool rec = g_prof.on && g_prof.calls < g_prof.max_calls;
    const int64_t call = g_prof.calls;
    if (rec) LPMM_HIP(hipEventRecord(prof_event(call, 0), s));
    if (bf16) hipLaunchKernelGGL(sgdm4_kernel<true>, dim3(pad8(t.n_wg)), dim3(kThreads), 0, s, t, h);
    else hipLaunchKernelGGL(sgdm4_kernel<false>, dim3(pad8(t.n_wg)), dim3(kThreads), 0, s, t, h);
    LPMM_HIP(hipGetLastError());
    if (rec) {
        LPMM_HIP(hipEventRecord(prof_event(call, 1), s));
        LPMM_HIP(hipEventRecord(prof_event(call, 2), s));
        g_prof.calls = call + 1;
    }
    return LPMM_OK;
}

// shape of a tensor with p >= 2 dimensions as the matrix the kernels see, plus its inner dimensions
int nd_shape(const int64_t* dims, int ndim, int64_t* rows, int64_t* cols, int64_t* ext, InnerDims* dm) {
    if (!dims || ndim < 2 || ndim > 1 + kMaxInnerDims) return LPMM_EINVAL;
    int64_t c = 1, e = 0;
    InnerDims d{};
    d.n = ndim - 1;
    for (int r = 1; r < ndim; ++r) {
        if (dims[r] < 1 || dims[r] > (int64_t(1) << 31)) return LPMM_EINVAL;
        if (c > (int64_t(1) << 31) / dims[r]) return LPMM_EINVAL;
        c *= dims[r];
        d.d[r - 1] = dims[r];
        d.first[r - 1] = e;
        e += dims[r];
    }
    const int64_t shape[2] = {dims[0], c};
    const int rc = check_shape(shape, rows, cols);
    if (rc) return rc;
    *ext = e;
    if (dm) *dm = d;
    return LPMM_OK;
}

int nd_step_impl(bool bf16, void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                 uint8_t* v_codes, float* v_row, float* v_col, const int64_t* dims, int ndim, float lr,
                 float beta1, float beta2, float eps, float wd, int64_t step, void* stream) {
    int64_t rows, cols, ext;
    InnerDims dm;
    int rc = nd_shape(dims, ndim, &rows, &cols, &ext, &dm);
    if (rc) return rc;
    if (!param || !grad || !m_codes || !m_blockscale || !v_codes || !v_row || !v_col) return LPMM_EINVAL;
    if (!aligned(param, 16) || !aligned(grad, 16) || !aligned(m_codes, 4) || !aligned(v_codes, 4) ||
        !aligned(m_blockscale, 4) || !aligned(v_row, 4) || !aligned(v_col, 4))
        return LPMM_EINVAL;
    Hyper h;
    rc = make_hyper(lr, beta1, beta2, eps, wd, step, &h);
    if (rc) return rc;
    DeviceCtx* ctx;
    rc = current_ctx(&ctx);
    if (rc) return rc;
    const int64_t rows_pad = round_up(rows, 64);
    if (rows_pad + round_up(cols + ext, 64) > ctx->cap_floats) return LPMM_EWORKSPACE;
    Tensor4 t{};
    t.p = static_cast<float*>(param);
    t.g = grad;
    t.mq = reinterpret_cast<uint32_t*>(m_codes);
    t.ms = m_blockscale;
    t.vq = reinterpret_cast<uint32_t*>(v_codes);
    t.r = v_row;
    t.c = v_col;                          // [cols] column scales, then [ext] the inner dimensions' statistics
    t.r_new = ctx->ws;
    t.c_new = ctx->ws + rows_pad;         // [cols] column maxima of v_t, then [ext] the new statistics
    t.c_extra = int(ext);
    t.counter = ctx->counter;
    t.rows = rows;
    t.cols = cols;
    t.P = rows * cols;
    const bool fast = fast_eligible(cols, v_col);
    t.kind = fast ? kQuantFast : kQuantGeneral;
    if (fast) fast_geometry(&t, ctx->n_cu, 0, 0, bf16 ? 2 : 4);
    else general_geometry(&t, ctx->n_cu);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = fast ? pad8(t.n_wg) : t.n_wg;
    const int grid_cols = grid_for(cols, 1);
#define LPMM_ND_LAUNCH(B)                                                                                         \
    if (fast) hipLaunchKernelGGL(pass1_fast<B>, dim3(grid), dim3(kThreads), 0, s, t, h);                          \
    else hipLaunchKernelGGL(pass1_general<B>, dim3(grid), dim3(kThreads), 0, s, t, h);                            \
    LPMM_HIP(hipGetLastError());                                                                                  \
    hipLaunchKernelGGL(nd_reduce_kernel, dim3(int(ext)), dim3(kThreads), 0, s, t.c_new, t.c_new + cols, cols, dm);  \
    LPMM_HIP(hipGetLastError());                                                                                  \
    hipLaunchKernelGGL(nd_expand_kernel, dim3(grid_cols), dim3(kThreads), 0, s, t.c_new + cols, t.c_new, cols, dm); \
    LPMM_HIP(hipGetLastError());                                                                                  \
    if (fast) hipLaunchKernelGGL(pass2_fast<B>, dim3(pad8(t.n_wg2)), dim3(kThreads), 0, s, t, h);                 \
    else hipLaunchKernelGGL(pass2_general<B>, dim3(t.n_wg2), dim3(kThreads), 0, s, t, h);                         \
    LPMM_HIP(hipGetLastError());
    if (bf16) { LPMM_ND_LAUNCH(true) } else { LPMM_ND_LAUNCH(false) }
#undef LPMM_ND_LAUNCH
    return LPMM_OK;
}

// Tiling of a tensor with a factorized second moment: the statistics pass is tiled like pass 2 and is the
// step's first ("A") launch, the update pass is tiled like pass 1 and is the second ("B") one.
// rows per tile of the statistics pass when its sums are reduced in a fixed order: fixed, because the size of the
// partial-sum buffer (part of the plan's memory) follows from it
constexpr int64_t kDetStatRows = 128;

// floats of partial sums of a rows x cols tensor with deterministic sums
int64_t det_partial_floats(int64_t rows, int64_t cols) {
    const int64_t strips2 = (cols / LPMM_BLOCK + 1) / 2, tiles = (rows + kDetStatRows - 1) / kDetStatRows;
    const int64_t row_wgs = (rows + kThreads - 1) / kThreads;
    return strips2 * round_up(rows, 64) + tiles * round_up(cols, 64) + round_up(2 * row_wgs, 64);
}

void factor_geometry(Tensor4* a, int n_cu, int64_t rw_hint, int64_t rw2_hint, int grad_bytes, bool fast,
                     int tot_slots) {
    a->tot_slots = tot_slots;
    a->kind = fast ? kFactorFast : kFactorGeneral;
    if (fast) {
        fast_geometry(a, n_cu, rw_hint, rw2_hint, grad_bytes);
        if (a->det) {
            a->rw2 = int(std::min<int64_t>(kDetStatRows, a->rows));
            a->n_wg2 = int(a->strips2 * ((a->rows + kDetStatRows - 1) / kDetStatRows));
            a->rs2 = row_spacing_log2(a->cols * grad_bytes, a->rw2, kWaves, "LPMM_RS2");
        }
        if (a->rw2 > kMaxRowSlots) {          // row sums of a statistics tile are staged in LDS
            a->rw2 = kMaxRowSlots;
            a->n_wg2 = int(a->strips2 * ((a->rows + a->rw2 - 1) / a->rw2));
            a->rs2 = row_spacing_log2(a->cols * grad_bytes, a->rw2, kWaves, "LPMM_RS2");
        }
        std::swap(a->n_wg, a->n_wg2);
        a->kind = kFactorFast;
    } else {
        general_geometry(a, n_cu);          // statistics pass: several chunks per workgroup; update pass: one
        a->kind = kFactorGeneral;
    }
}

int factor_step_impl(bool bf16, void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                     float* v_row, float* v_col, const int64_t* shape, float lr, float beta1, float beta2,
                     float eps, float wd, int64_t step, void* stream) {
    int64_t rows, cols;
    int rc = check_shape(shape, &rows, &cols);
    if (rc) return rc;
    if (!param || !grad || !m_codes || !m_blockscale || !v_row || !v_col) return LPMM_EINVAL;
    if (!aligned(param, 16) || !aligned(grad, 16) || !aligned(m_codes, 4) || !aligned(m_blockscale, 4) ||
        !aligned(v_row, 4) || !aligned(v_col, 4))
        return LPMM_EINVAL;
    Hyper h;
    rc = make_hyper(lr, beta1, beta2, eps, wd, step, &h);
    if (rc) return rc;
    DeviceCtx* ctx;
    rc = current_ctx(&ctx);
    if (rc) return rc;
    const int64_t rows_pad = round_up(rows, 64), cols_pad = round_up(cols, 64);
    if (rows_pad + cols_pad > ctx->cap_floats) return LPMM_EWORKSPACE;
    Tensor4 t{};
    t.p = static_cast<float*>(param);
    t.g = grad;
    t.mq = reinterpret_cast<uint32_t*>(m_codes);
    t.ms = m_blockscale;
    t.r = v_row;
    t.c = v_col;
    t.r_new = ctx->ws;
    t.c_new = ctx->ws + rows_pad;
    t.counter = ctx->counter;
    t.rows = rows;
    t.cols = cols;
    t.P = rows * cols;
    const bool fast = fast_eligible(cols, v_col);
    factor_geometry(&t, ctx->n_cu, 0, 0, bf16 ? 2 : 4, fast, kMaxTotSlots);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool rec = g_prof.on && g_prof.calls < g_prof.max_calls;
    const int64_t call = g_prof.calls;
    if (rec) LPMM_HIP(hipEventRecord(prof_event(call, 0), s));
#define LPMM_LAUNCH_FACTOR(B)                                                                                      \
    if (fast) hipLaunchKernelGGL(factor_stats_fast<B>, dim3(pad8(t.n_wg)), dim3(kThreads), 0, s, t);               \
    else hipLaunchKernelGGL(factor_stats_general<B>, dim3(t.n_wg), dim3(kThreads), 0, s, t);                       \
    LPMM_HIP(hipGetLastError());                                                                                   \
    if (rec) LPMM_HIP(hipEventRecord(prof_event(call, 1), s));                                                     \
    if (fast) hipLaunchKernelGGL(factor_update_fast<B>, dim3(pad8(t.n_wg2)), dim3(kThreads), 0, s, t, h);          \
    else hipLaunchKernelGGL(factor_update_general<B>, dim3(t.n_wg2), dim3(kThreads), 0, s, t, h);                  \
    LPMM_HIP(hipGetLastError());
    if (bf16) { LPMM_LAUNCH_FACTOR(true) } else { LPMM_LAUNCH_FACTOR(false) }
#undef LPMM_LAUNCH_FACTOR
    if (rec) {
        LPMM_HIP(hipEventRecord(prof_event(call, 2), s));
        g_prof.calls = call + 1;
    }
    return LPMM_OK;
}

// ---- multi-tensor plans ---------------------------------------------------------------------------

struct PhaseLaunch {
    Phase ph;
    int grid;        // both kinds in one launch
    int grid_a;      // A work alone
    int grid_b;      // B work alone
    bool a_has_rank1;   // some A tensor takes pass 1 of the rank-1 path (else the lighter kernel variant runs)
    // tensors with more than two dimensions among the B tensors: two small kernels run before their pass 2
    NdPhase nd;
    bool has_nd;
    // tensors with deterministic sums among the B tensors (factorized plans): two small kernels before their update pass
    DetPhase det;
    bool has_det;
};

struct PlanHost {
    std::vector<char> staging;          // host image of the device tables (kept for the async copy)
    std::vector<PhaseLaunch> phases;
    bool bf16 = false;
    bool factor = false;                // the plan's 2-dimensional tensors keep a factorized second moment
    bool sgdm = false;                  // a plan of SGD-with-momentum tensors (lpmm_sgdm4_step_multi)
    bool flat = false;                  // large tensors, several groups: pass 1 uses the flat tiling
    bool serial = false;                // LPMM_MULTI_STREAMS=0: every pass a launch of its own on the caller's stream
    int64_t params = 0;                 // parameters of all tensors of the plan
    Hyper* d_hyper = nullptr;           // device slot inside the plan for the hyper-parameters of a captured step
    int device = 0;
    // second stream for pass 2 (same priority as any other stream), with its ordering events
    hipStream_t side = nullptr;
    hipStream_t side_a = nullptr;       // optional: pass 1 of odd phases, so that consecutive pass-1 launches overlap their tails
    hipEvent_t ev_join_a = nullptr;
    std::vector<hipEvent_t> ev_a;       // ev_a[j]: phase j's A work is complete
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    ~PlanHost() {
        for (hipEvent_t e : ev_a) (void)hipEventDestroy(e);
        if (ev_fork) (void)hipEventDestroy(ev_fork);
        if (ev_join) (void)hipEventDestroy(ev_join);
        if (ev_join_a) (void)hipEventDestroy(ev_join_a);
        if (side) (void)hipStreamDestroy(side);
        if (side_a) (void)hipStreamDestroy(side_a);
    }
};

// shared ownership: a step copies the pointer out under the lock and keeps the plan's host record (streams, events)
// alive until it has enqueued its work, even if another thread releases the plan meanwhile
std::unordered_map<void*, std::shared_ptr<PlanHost>> g_plans;

struct PlanLayout {
    size_t off_tensors, off_dims, off_hyper, off_counters, off_floats, total;
    int64_t n_nd;
};

bool desc_shape_ok(const lpmm_tensor_desc& d) {
    int64_t shape[2] = {d.rows, d.cols}, r, c;
    return check_shape(shape, &r, &c) == LPMM_OK && (d.kind == LPMM_KIND_4BIT || d.kind == LPMM_KIND_FP32 ||
                                                     d.kind == LPMM_KIND_4BIT_B128 || d.kind == LPMM_KIND_4BIT_FACTOR ||
                                                     d.kind == LPMM_KIND_SGDM_4BIT || d.kind == LPMM_KIND_SGDM_FP32 ||
                                                     d.kind == LPMM_KIND_4BIT_ND);
}

// inner dimensions of tensor i of a plan: inner_dims holds kMaxInnerDims sizes per tensor, inner_ndim their count
// (0 for tensors that are not LPMM_KIND_4BIT_ND).  Fills dm and ext (the number of statistics of those dimensions).
bool plan_inner_dims(const lpmm_tensor_desc& d, int64_t i, const int64_t* inner_dims, const int32_t* inner_ndim,
                     InnerDims* dm, int64_t* ext) {
    if (!inner_dims || !inner_ndim) return false;
    const int k = inner_ndim[i];
    if (k < 1 || k > kMaxInnerDims) return false;
    int64_t dims[1 + kMaxInnerDims];
    dims[0] = d.rows;
    for (int r = 0; r < k; ++r) dims[1 + r] = inner_dims[i * kMaxInnerDims + r];
    int64_t rows, cols;
    if (nd_shape(dims, 1 + k, &rows, &cols, ext, dm) != LPMM_OK) return false;
    return cols == d.cols;
}

bool plan_layout(const lpmm_tensor_desc* descs, int64_t n, const int64_t* inner_dims, const int32_t* inner_ndim,
                 PlanLayout* L) {
    if (!descs || n < 1 || n > (1 << 20)) return false;
    int64_t floats = 0, n_nd = 0;
    bool rank1 = false, factor = false;
    for (int64_t i = 0; i < n; ++i) {
        if (!desc_shape_ok(descs[i])) return false;
        if (descs[i].kind == LPMM_KIND_4BIT || descs[i].kind == LPMM_KIND_4BIT_FACTOR)
            floats += round_up(descs[i].rows, 64) + round_up(descs[i].cols, 64);
        if (descs[i].kind == LPMM_KIND_4BIT_FACTOR && (descs[i].flags & LPMM_FLAG_DETERMINISTIC))
            floats += det_partial_floats(descs[i].rows, descs[i].cols);
        if (descs[i].kind == LPMM_KIND_4BIT_ND) {
            InnerDims dm;
            int64_t ext;
            if (!plan_inner_dims(descs[i], i, inner_dims, inner_ndim, &dm, &ext)) return false;
            floats += round_up(descs[i].rows, 64) + round_up(descs[i].cols + ext, 64);
            ++n_nd;
        }
        if (descs[i].kind == LPMM_KIND_4BIT || descs[i].kind == LPMM_KIND_4BIT_ND) rank1 = true;
        if (descs[i].kind == LPMM_KIND_4BIT_FACTOR) factor = true;
    }
    L->n_nd = n_nd;
    int64_t n_sgdm = 0;
    for (int64_t i = 0; i < n; ++i)
        if (descs[i].kind == LPMM_KIND_SGDM_4BIT || descs[i].kind == LPMM_KIND_SGDM_FP32) ++n_sgdm;
    if (rank1 && factor) return false;       // two different optimizers: one plan holds one of them
    if (n_sgdm != 0 && n_sgdm != n) return false;
    size_t off = 0;
    L->off_tensors = off;   off += size_t(round_up(n * int64_t(sizeof(Tensor4)), 256));
    L->off_dims = off;      off += size_t(round_up(n_nd * int64_t(sizeof(InnerDims)), 256));
    L->off_hyper = off;     off += 256;                       // hyper-parameters of a captured step
    L->off_counters = off;  off += size_t(n) * kCounterWords * sizeof(unsigned int);
    L->off_floats = off;    off += size_t(floats) * sizeof(float);
    L->total = size_t(round_up(int64_t(off), 256));
    return true;
}

int fill(void* dst, int64_t n, uint8_t value, int64_t last_index, uint8_t last, hipStream_t s) {
    if (n <= 0) return LPMM_OK;
    hipLaunchKernelGGL(fill_bytes_kernel, dim3(grid_for(n, 16, 4096)), dim3(kThreads), 0, s,
                       static_cast<uint8_t*>(dst), n, value, last_index, last);
    LPMM_HIP(hipGetLastError());
    return LPMM_OK;
}

}  // namespace

extern "C" {

const char* lpmm_strerror(int code) {
    switch (code) {
        case LPMM_OK: return "ok";
        case LPMM_EINVAL: return "invalid argument (null or misaligned pointer, bad shape, step < 1, or bad hyper-parameter)";
        case LPMM_ENOTINIT: return "lpmm_adamw4_init has not been called for the current device";
        case LPMM_EHIP: return "a HIP call failed (see lpmm_last_hip_error)";
        case LPMM_EWORKSPACE: return "workspace too small for this tensor (rows + cols)";
        default: return "unknown lpmm error code";
    }
}

int lpmm_last_hip_error(void) { return g_last_hip; }

int lpmm_table(int which, float* out) {
    if (!out || (which != 0 && which != 1)) return LPMM_EINVAL;
    const HostTables& t = host_tables();
    for (int i = 0; i < kCodes; ++i) out[i] = which == 0 ? t.de[i] : t.lin[i];
    return LPMM_OK;
}

int lpmm_host_nearest_codes(int which, const float* n, int64_t count, uint8_t* out) {
    if (!n || !out || count < 0 || (which != 0 && which != 1)) return LPMM_EINVAL;
    const HostTables& t = host_tables();
    if (!t.ok) return LPMM_EINVAL;
    for (int64_t i = 0; i < count; ++i) {
        if (which == 0) {
            out[i] = uint8_t(search_code(t.search, n[i]));
        } else {
            const float f = std::ceil(std::fmaf(16.0f, n[i], -1.5f));
            out[i] = uint8_t(std::fmin(std::fmax(f, 0.0f), 15.0f));
        }
    }
    return LPMM_OK;
}

size_t lpmm_adamw4_workspace_bytes(int64_t max_rows_plus_cols) {
    if (max_rows_plus_cols < 2) max_rows_plus_cols = 2;
    // rows and cols are each rounded up to 64 floats inside the workspace
    return size_t(round_up(max_rows_plus_cols, 64) + 128) * sizeof(float) + kCounterBytes;
}

int lpmm_adamw4_init(int device, void* workspace, size_t workspace_bytes, void* stream) {
    if (device < 0 || device >= kMaxDevices) return LPMM_EINVAL;
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < kCounterBytes + 256 * sizeof(float))
        return LPMM_EINVAL;
    const HostTables& t = host_tables();
    if (!t.ok) return LPMM_EINVAL;
    std::lock_guard<std::mutex> lock(g_mu);
    int prev = 0;
    LPMM_HIP(hipGetDevice(&prev));
    LPMM_HIP(hipSetDevice(device));
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyToSymbolAsync(HIP_SYMBOL(d_byte_decode), t.byte_decode, sizeof(t.byte_decode), 0,
                                          hipMemcpyHostToDevice, s);
    if (e == hipSuccess)
        e = hipMemcpyToSymbolAsync(HIP_SYMBOL(d_search), t.search, sizeof(t.search), 0,
                                   hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipMemsetAsync(workspace, 0, workspace_bytes, s);
    int n_cu = 256;
    if (e == hipSuccess) e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, device);
    // where this device keeps its copy of the library's own scratch array (`device` is current here)
    unsigned char* scratch_ptr = nullptr;
    if (e == hipSuccess) e = hipGetSymbolAddress(reinterpret_cast<void**>(&scratch_ptr), HIP_SYMBOL(scratch));
    (void)hipSetDevice(prev);
    if (e != hipSuccess) return hip_fail(e);
    DeviceCtx& c = g_ctx[device];
    c.scratch = scratch_ptr;
    c.ws = static_cast<float*>(workspace);
    c.cap_floats = int64_t((workspace_bytes - kCounterBytes) / sizeof(float)) / 64 * 64;
    c.counter = reinterpret_cast<unsigned int*>(static_cast<char*>(workspace) + size_t(c.cap_floats) * sizeof(float));
    c.n_cu = n_cu > 0 ? n_cu : 256;
    c.ready = true;
    return LPMM_OK;
}

int lpmm_adamw4_state_sizes(const int64_t shape[2], size_t sizes[5]) {
    int64_t rows, cols;
    const int rc = check_shape(shape, &rows, &cols);
    if (rc) return rc;
    if (!sizes) return LPMM_EINVAL;
    const int64_t P = rows * cols;
    sizes[0] = size_t((P + 1) / 2);
    sizes[1] = size_t((P + LPMM_BLOCK - 1) / LPMM_BLOCK) * sizeof(float);
    sizes[2] = size_t((P + 1) / 2);
    sizes[3] = size_t(rows) * sizeof(float);
    sizes[4] = size_t(cols) * sizeof(float);
    return LPMM_OK;
}

int lpmm_adamw4_state_zero(uint8_t* m_codes, float* m_blockscale, uint8_t* v_codes, float* v_rowmax,
                           float* v_colmax, const int64_t shape[2], void* stream) {
    size_t sz[5];
    const int rc = lpmm_adamw4_state_sizes(shape, sz);
    if (rc) return rc;
    if (!m_codes || !m_blockscale || !v_codes || !v_rowmax || !v_colmax) return LPMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t P = shape[0] * shape[1];
    // code 7 is the rank of 0.0 in the DE map; an odd tail leaves its unused high nibble 0
    int r = fill(m_codes, int64_t(sz[0]), 0x77, (P & 1) ? int64_t(sz[0]) - 1 : -1, 0x07, s);
    if (!r) r = fill(m_blockscale, int64_t(sz[1]), 0, -1, 0, s);
    if (!r) r = fill(v_codes, int64_t(sz[2]), 0, -1, 0, s);
    if (!r) r = fill(v_rowmax, int64_t(sz[3]), 0, -1, 0, s);
    if (!r) r = fill(v_colmax, int64_t(sz[4]), 0, -1, 0, s);
    return r;
}

int lpmm_adamw4_step(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                     uint8_t* v_codes, float* v_rowmax, float* v_colmax, const int64_t shape[2],
                     float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step,
                     void* stream) {
    return step_impl(false, param, grad, m_codes, m_blockscale, v_codes, v_rowmax, v_colmax, shape, lr,
                     beta1, beta2, eps, weight_decay, step, stream);
}

int lpmm_adamw4_step_bf16g(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                           uint8_t* v_codes, float* v_rowmax, float* v_colmax, const int64_t shape[2],
                           float lr, float beta1, float beta2, float eps, float weight_decay,
                           int64_t step, void* stream) {
    return step_impl(true, param, grad, m_codes, m_blockscale, v_codes, v_rowmax, v_colmax, shape, lr,
                     beta1, beta2, eps, weight_decay, step, stream);
}

int lpmm_adamw4_step_noalloc(void* param, const void* grad, int grad_dtype, uint8_t* m_codes, float* m_blockscale,
                             uint8_t* v_codes, float* v_rowmax, float* v_colmax, const int64_t shape[2],
                             float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step,
                             void* stream) {
    if (grad_dtype != LPMM_GRAD_F32 && grad_dtype != LPMM_GRAD_BF16) return LPMM_EINVAL;
    return step_impl(grad_dtype == LPMM_GRAD_BF16, param, grad, m_codes, m_blockscale, v_codes, v_rowmax, v_colmax,
                     shape, lr, beta1, beta2, eps, weight_decay, step, stream, WorkspaceChoice{true, nullptr, 0});
}

int lpmm_adamw4_step_ws(void* param, const void* grad, int grad_dtype, uint8_t* m_codes, float* m_blockscale,
                        uint8_t* v_codes, float* v_rowmax, float* v_colmax, const int64_t shape[2], float lr,
                        float beta1, float beta2, float eps, float weight_decay, int64_t step, void* workspace,
                        size_t workspace_bytes, void* stream) {
    if (grad_dtype != LPMM_GRAD_F32 && grad_dtype != LPMM_GRAD_BF16) return LPMM_EINVAL;
    if (!workspace) return LPMM_EINVAL;
    return step_impl(grad_dtype == LPMM_GRAD_BF16, param, grad, m_codes, m_blockscale, v_codes, v_rowmax, v_colmax,
                     shape, lr, beta1, beta2, eps, weight_decay, step, stream,
                     WorkspaceChoice{false, workspace, workspace_bytes});
}

int lpmm_adamw4_b128_state_sizes(int64_t numel, size_t sizes[4]) {
    if (numel < 1 || numel > (int64_t(1) << 37) || !sizes) return LPMM_EINVAL;
    sizes[0] = sizes[2] = size_t((numel + 1) / 2);
    sizes[1] = sizes[3] = size_t((numel + LPMM_BLOCK - 1) / LPMM_BLOCK) * sizeof(float);
    return LPMM_OK;
}

int lpmm_adamw4_b128_state_zero(uint8_t* m_codes, float* m_blockscale, uint8_t* v_codes, float* v_blockscale,
                                int64_t numel, void* stream) {
    size_t sz[4];
    const int rc = lpmm_adamw4_b128_state_sizes(numel, sz);
    if (rc) return rc;
    if (!m_codes || !m_blockscale || !v_codes || !v_blockscale) return LPMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int r = fill(m_codes, int64_t(sz[0]), 0x77, (numel & 1) ? int64_t(sz[0]) - 1 : -1, 0x07, s);
    if (!r) r = fill(m_blockscale, int64_t(sz[1]), 0, -1, 0, s);
    if (!r) r = fill(v_codes, int64_t(sz[2]), 0, -1, 0, s);
    if (!r) r = fill(v_blockscale, int64_t(sz[3]), 0, -1, 0, s);
    return r;
}

int lpmm_adamw4_b128_step(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                          uint8_t* v_codes, float* v_blockscale, int64_t numel, float lr, float beta1,
                          float beta2, float eps, float weight_decay, int64_t step, void* stream) {
    return b128_step_impl(false, param, grad, m_codes, m_blockscale, v_codes, v_blockscale, numel, lr, beta1,
                          beta2, eps, weight_decay, step, stream);
}

int lpmm_adamw4_b128_step_bf16g(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                                uint8_t* v_codes, float* v_blockscale, int64_t numel, float lr, float beta1,
                                float beta2, float eps, float weight_decay, int64_t step, void* stream) {
    return b128_step_impl(true, param, grad, m_codes, m_blockscale, v_codes, v_blockscale, numel, lr, beta1,
                          beta2, eps, weight_decay, step, stream);
}

int lpmm_adamw4_factor_state_sizes(const int64_t shape[2], size_t sizes[4]) {
    int64_t rows, cols;
    const int rc = check_shape(shape, &rows, &cols);
    if (rc) return rc;
    if (!sizes) return LPMM_EINVAL;
    const int64_t P = rows * cols;
    sizes[0] = size_t((P + 1) / 2);
    sizes[1] = size_t((P + LPMM_BLOCK - 1) / LPMM_BLOCK) * sizeof(float);
    sizes[2] = size_t(rows) * sizeof(float);
    sizes[3] = size_t(cols) * sizeof(float);
    return LPMM_OK;
}

int lpmm_adamw4_factor_state_zero(uint8_t* m_codes, float* m_blockscale, float* v_row, float* v_col,
                                  const int64_t shape[2], void* stream) {
    size_t sz[4];
    const int rc = lpmm_adamw4_factor_state_sizes(shape, sz);
    if (rc) return rc;
    if (!m_codes || !m_blockscale || !v_row || !v_col) return LPMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t P = shape[0] * shape[1];
    int r = fill(m_codes, int64_t(sz[0]), 0x77, (P & 1) ? int64_t(sz[0]) - 1 : -1, 0x07, s);
    if (!r) r = fill(m_blockscale, int64_t(sz[1]), 0, -1, 0, s);
    if (!r) r = fill(v_row, int64_t(sz[2]), 0, -1, 0, s);
    if (!r) r = fill(v_col, int64_t(sz[3]), 0, -1, 0, s);
    return r;
}

int lpmm_adamw4_factor_step(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale, float* v_row,
                            float* v_col, const int64_t shape[2], float lr, float beta1, float beta2, float eps,
                            float weight_decay, int64_t step, void* stream) {
    return factor_step_impl(false, param, grad, m_codes, m_blockscale, v_row, v_col, shape, lr, beta1, beta2,
                            eps, weight_decay, step, stream);
}

int lpmm_adamw4_factor_step_bf16g(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                                  float* v_row, float* v_col, const int64_t shape[2], float lr, float beta1,
                                  float beta2, float eps, float weight_decay, int64_t step, void* stream) {
    return factor_step_impl(true, param, grad, m_codes, m_blockscale, v_row, v_col, shape, lr, beta1, beta2,
                            eps, weight_decay, step, stream);
}

int lpmm_adamw4_nd_state_sizes(const int64_t* dims, int ndim, size_t sizes[5]) {
    int64_t rows, cols, ext;
    const int rc = nd_shape(dims, ndim, &rows, &cols, &ext, nullptr);
    if (rc) return rc;
    if (!sizes) return LPMM_EINVAL;
    const int64_t P = rows * cols;
    sizes[0] = size_t((P + 1) / 2);
    sizes[1] = size_t((P + LPMM_BLOCK - 1) / LPMM_BLOCK) * sizeof(float);
    sizes[2] = size_t((P + 1) / 2);
    sizes[3] = size_t(rows) * sizeof(float);
    sizes[4] = size_t(cols + ext) * sizeof(float);
    return LPMM_OK;
}

int lpmm_adamw4_nd_state_zero(uint8_t* m_codes, float* m_blockscale, uint8_t* v_codes, float* v_row, float* v_col,
                              const int64_t* dims, int ndim, void* stream) {
    size_t sz[5];
    const int rc = lpmm_adamw4_nd_state_sizes(dims, ndim, sz);
    if (rc) return rc;
    if (!m_codes || !m_blockscale || !v_codes || !v_row || !v_col) return LPMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int64_t P = 1;
    for (int r = 0; r < ndim; ++r) P *= dims[r];
    int r = fill(m_codes, int64_t(sz[0]), 0x77, (P & 1) ? int64_t(sz[0]) - 1 : -1, 0x07, s);
    if (!r) r = fill(m_blockscale, int64_t(sz[1]), 0, -1, 0, s);
    if (!r) r = fill(v_codes, int64_t(sz[2]), 0, -1, 0, s);
    if (!r) r = fill(v_row, int64_t(sz[3]), 0, -1, 0, s);
    if (!r) r = fill(v_col, int64_t(sz[4]), 0, -1, 0, s);
    return r;
}

int lpmm_adamw4_nd_step(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale, uint8_t* v_codes,
                        float* v_row, float* v_col, const int64_t* dims, int ndim, float lr, float beta1,
                        float beta2, float eps, float weight_decay, int64_t step, void* stream) {
    return nd_step_impl(false, param, grad, m_codes, m_blockscale, v_codes, v_row, v_col, dims, ndim, lr, beta1,
                        beta2, eps, weight_decay, step, stream);
}

int lpmm_adamw4_nd_step_bf16g(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                              uint8_t* v_codes, float* v_row, float* v_col, const int64_t* dims, int ndim,
                              float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step,
                              void* stream) {
    return nd_step_impl(true, param, grad, m_codes, m_blockscale, v_codes, v_row, v_col, dims, ndim, lr, beta1,
                        beta2, eps, weight_decay, step, stream);
}

int lpmm_sgdm4_state_sizes(int64_t numel, size_t sizes[2]) {
    if (numel < 1 || numel > (int64_t(1) << 37) || !sizes) return LPMM_EINVAL;
    sizes[0] = size_t((numel + 1) / 2);
    sizes[1] = size_t((numel + LPMM_BLOCK - 1) / LPMM_BLOCK) * sizeof(float);
    return LPMM_OK;
}

int lpmm_sgdm4_state_zero(uint8_t* m_codes, float* m_blockscale, int64_t numel, void* stream) {
    size_t sz[2];
    const int rc = lpmm_sgdm4_state_sizes(numel, sz);
    if (rc) return rc;
    if (!m_codes || !m_blockscale) return LPMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int r = fill(m_codes, int64_t(sz[0]), 0x77, (numel & 1) ? int64_t(sz[0]) - 1 : -1, 0x07, s);
    if (!r) r = fill(m_blockscale, int64_t(sz[1]), 0, -1, 0, s);
    return r;
}

int lpmm_sgdm4_step(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale, int64_t numel, float lr,
                    float momentum, void* stream) {
    return sgdm4_step_impl(false, param, grad, m_codes, m_blockscale, numel, lr, momentum, stream);
}

int lpmm_sgdm4_step_bf16g(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale, int64_t numel,
                          float lr, float momentum, void* stream) {
    return sgdm4_step_impl(true, param, grad, m_codes, m_blockscale, numel, lr, momentum, stream);
}

int lpmm_sgdm32_step(void* param, const void* grad, float* m, int64_t numel, int grad_dtype, float lr,
                     float momentum, void* stream) {
    if (!param || !grad || !m || numel < 1) return LPMM_EINVAL;
    if (grad_dtype != LPMM_GRAD_F32 && grad_dtype != LPMM_GRAD_BF16) return LPMM_EINVAL;
    if (!aligned(param, 4) || !aligned(m, 4) || !aligned(grad, grad_dtype == LPMM_GRAD_F32 ? 4 : 2)) return LPMM_EINVAL;
    Hyper h;
    const int rc = make_sgdm_hyper(lr, momentum, &h);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = int((numel + kElemsPerWg32 - 1) / kElemsPerWg32);
    if (grad_dtype == LPMM_GRAD_BF16)
        hipLaunchKernelGGL(sgdm32_kernel<true>, dim3(grid), dim3(kThreads), 0, s, static_cast<float*>(param), grad, m, numel, h);
    else
        hipLaunchKernelGGL(sgdm32_kernel<false>, dim3(grid), dim3(kThreads), 0, s, static_cast<float*>(param), grad, m, numel, h);
    LPMM_HIP(hipGetLastError());
    return LPMM_OK;
}

int lpmm_adamw32_step(void* param, const void* grad, float* m, float* v, int64_t numel, int grad_dtype,
                      float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step,
                      void* stream) {
    if (!param || !grad || !m || !v || numel < 1) return LPMM_EINVAL;
    if (grad_dtype != LPMM_GRAD_F32 && grad_dtype != LPMM_GRAD_BF16) return LPMM_EINVAL;
    if (!aligned(param, 4) || !aligned(m, 4) || !aligned(v, 4) ||
        !aligned(grad, grad_dtype == LPMM_GRAD_F32 ? 4 : 2))
        return LPMM_EINVAL;
    Hyper h;
    const int rc = make_hyper(lr, beta1, beta2, eps, weight_decay, step, &h);
    if (rc) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = int((numel + kElemsPerWg32 - 1) / kElemsPerWg32);
    if (grad_dtype == LPMM_GRAD_BF16)
        hipLaunchKernelGGL(adamw32_kernel<true>, dim3(grid), dim3(kThreads), 0, s,
                           static_cast<float*>(param), grad, m, v, numel, h);
    else
        hipLaunchKernelGGL(adamw32_kernel<false>, dim3(grid), dim3(kThreads), 0, s,
                           static_cast<float*>(param), grad, m, v, numel, h);
    LPMM_HIP(hipGetLastError());
    return LPMM_OK;
}

int lpmm_dequant_state(int which, const uint8_t* codes, const float* scale_a, const float* scale_b,
                       const int64_t shape[2], float* out, void* stream) {
    int64_t rows, cols;
    const int rc = check_shape(shape, &rows, &cols);
    if (rc) return rc;
    if ((which != 0 && which != 1 && which != 2) || !codes || !scale_a || !out || (which == 1 && !scale_b))
        return LPMM_EINVAL;
    if (!aligned(codes, 4) || !aligned(out, 4)) return LPMM_EINVAL;
    DeviceCtx* ctx;
    const int rc2 = current_ctx(&ctx);   // the DE table lives in device memory filled by init
    if (rc2) return rc2;
    QuantArgs q{};
    q.q_in = reinterpret_cast<const uint32_t*>(codes);
    q.x_out = out;
    q.sa = const_cast<float*>(scale_a);
    q.sb = const_cast<float*>(scale_b);
    q.rows = rows; q.cols = cols; q.P = rows * cols;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = grid_for(q.P, 8);
    if (which == 0) hipLaunchKernelGGL(dequant_m_kernel, dim3(grid), dim3(kThreads), 0, s, q);
    else if (which == 1) hipLaunchKernelGGL(dequant_v_kernel, dim3(grid), dim3(kThreads), 0, s, q);
    else hipLaunchKernelGGL(dequant_vb_kernel, dim3(grid), dim3(kThreads), 0, s, q);
    LPMM_HIP(hipGetLastError());
    return LPMM_OK;
}

int lpmm_quant_state(int which, const float* in, const int64_t shape[2], uint8_t* codes, float* scale_a,
                     float* scale_b, void* stream) {
    int64_t rows, cols;
    const int rc = check_shape(shape, &rows, &cols);
    if (rc) return rc;
    if ((which != 0 && which != 1 && which != 2) || !codes || !scale_a || !in || (which == 1 && !scale_b))
        return LPMM_EINVAL;
    if (!aligned(codes, 4) || !aligned(in, 4)) return LPMM_EINVAL;
    DeviceCtx* ctx;
    const int rc2 = current_ctx(&ctx);
    if (rc2) return rc2;
    QuantArgs q{};
    q.x_in = in;
    q.q_out = reinterpret_cast<uint32_t*>(codes);
    q.sa = scale_a;
    q.sb = scale_b;
    q.rows = rows; q.cols = cols; q.P = rows * cols;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = grid_for(q.P, 8);
    if (which == 0) {
        hipLaunchKernelGGL(quant_m_kernel, dim3(grid), dim3(kThreads), 0, s, q);
        LPMM_HIP(hipGetLastError());
    } else if (which == 2) {
        hipLaunchKernelGGL(quant_vb_kernel, dim3(grid), dim3(kThreads), 0, s, q);
        LPMM_HIP(hipGetLastError());
    } else {
        int r = fill(scale_a, rows * int64_t(sizeof(float)), 0, -1, 0, s);
        if (!r) r = fill(scale_b, cols * int64_t(sizeof(float)), 0, -1, 0, s);
        if (r) return r;
        hipLaunchKernelGGL(quant_v_max_kernel, dim3(grid), dim3(kThreads), 0, s, q);
        LPMM_HIP(hipGetLastError());
        hipLaunchKernelGGL(quant_v_code_kernel, dim3(grid), dim3(kThreads), 0, s, q);
        LPMM_HIP(hipGetLastError());
    }
    return LPMM_OK;
}

}  // extern "C"

namespace {

// the map of an ablation quantizer, with its decision thresholds; false for a combination that does not exist
bool ablation_map(int map, int is_signed, AblMap* m) {
    float T[kCodes];
    int n = kCodes;
    if (map == LPMM_MAP_DE) {
        if (is_signed) build_de_signed(T); else build_de_unsigned(T);
    } else if (map == LPMM_MAP_DE0 && !is_signed) {
        float U[kCodes];
        build_de_unsigned(U);                 // U[0] is the zero that DE-0 drops
        n = kCodes - 1;
        for (int i = 0; i < n; ++i) T[i] = U[i + 1];
    } else if (map == LPMM_MAP_LINEAR && !is_signed) {
        build_linear(T);
    } else {
        return false;
    }
    *m = AblMap{};
    m->n = n;
    for (int i = 0; i < n; ++i) m->T[i] = T[i];
    build_thresholds_n(T, n, m->thr);
    return true;
}

bool ablation_valid(int norm, int is_signed) {
    return (norm == LPMM_NORM_B128 || norm == LPMM_NORM_B2048 || (norm == LPMM_NORM_RANK1 && !is_signed));
}

}  // namespace

extern "C" {

int lpmm_ablation_table(int map, int is_signed, float out[16]) {
    AblMap m;
    if (!out || !ablation_map(map, is_signed, &m)) return LPMM_EINVAL;
    for (int i = 0; i < kCodes; ++i) out[i] = i < m.n ? m.T[i] : 0.0f;
    return m.n;
}

int lpmm_quant_ablation(int norm, int map, int is_signed, int rounding, uint64_t seed, const float* in,
                        const int64_t shape[2], uint8_t* codes, float* scale_a, float* scale_b, void* stream) {
    int64_t rows, cols;
    const int rc = check_shape(shape, &rows, &cols);
    if (rc) return rc;
    AblMap m;
    if (!ablation_valid(norm, is_signed) || !ablation_map(map, is_signed, &m)) return LPMM_EINVAL;
    if (rounding != LPMM_ROUND_NEAREST && rounding != LPMM_ROUND_STOCHASTIC) return LPMM_EINVAL;
    if (!in || !codes || !scale_a || (norm == LPMM_NORM_RANK1 && !scale_b)) return LPMM_EINVAL;
    if (!aligned(in, 4) || !aligned(codes, 4) || !aligned(scale_a, 4)) return LPMM_EINVAL;
    AblArgs a{};
    a.x_in = in;
    a.q_out = reinterpret_cast<uint32_t*>(codes);
    a.sa = scale_a;
    a.sb = scale_b;
    a.rows = rows; a.cols = cols; a.P = rows * cols;
    a.stochastic = rounding == LPMM_ROUND_STOCHASTIC;
    a.seed = seed;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int grid = grid_for(a.P, 8);
    if (norm == LPMM_NORM_RANK1) {
        int r = fill(scale_a, rows * int64_t(sizeof(float)), 0, -1, 0, s);
        if (!r) r = fill(scale_b, cols * int64_t(sizeof(float)), 0, -1, 0, s);
        if (r) return r;
        QuantArgs q{};
        q.x_in = in; q.sa = scale_a; q.sb = scale_b;
        q.rows = rows; q.cols = cols; q.P = a.P;
        hipLaunchKernelGGL(quant_v_max_kernel, dim3(grid), dim3(kThreads), 0, s, q);
        LPMM_HIP(hipGetLastError());
        hipLaunchKernelGGL(abl_quant_rank1_kernel, dim3(grid), dim3(kThreads), 0, s, a, m);
    } else if (norm == LPMM_NORM_B128) {
        hipLaunchKernelGGL(abl_quant_block_kernel<128>, dim3(grid), dim3(kThreads), 0, s, a, m);
    } else {
        hipLaunchKernelGGL(abl_quant_block_kernel<2048>, dim3(grid), dim3(kThreads), 0, s, a, m);
    }
    LPMM_HIP(hipGetLastError());
    return LPMM_OK;
}

int lpmm_dequant_ablation(int norm, int map, int is_signed, const uint8_t* codes, const float* scale_a,
                          const float* scale_b, const int64_t shape[2], float* out, void* stream) {
    int64_t rows, cols;
    const int rc = check_shape(shape, &rows, &cols);
    if (rc) return rc;
    AblMap m;
    if (!ablation_valid(norm, is_signed) || !ablation_map(map, is_signed, &m)) return LPMM_EINVAL;
    if (!codes || !scale_a || !out || (norm == LPMM_NORM_RANK1 && !scale_b)) return LPMM_EINVAL;
    if (!aligned(codes, 4) || !aligned(out, 4) || !aligned(scale_a, 4)) return LPMM_EINVAL;
    AblArgs a{};
    a.q_in = reinterpret_cast<const uint32_t*>(codes);
    a.x_out = out;
    a.sa = const_cast<float*>(scale_a);
    a.sb = const_cast<float*>(scale_b);
    a.rows = rows; a.cols = cols; a.P = rows * cols;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(abl_dequant_kernel, dim3(grid_for(a.P, 8)), dim3(kThreads), 0, s, a, m, norm);
    LPMM_HIP(hipGetLastError());
    return LPMM_OK;
}

size_t lpmm_adamw4_plan_bytes(const lpmm_tensor_desc* descs, int64_t n) {
    return lpmm_adamw4_plan_bytes_nd(descs, n, nullptr, nullptr);
}

size_t lpmm_adamw4_plan_bytes_nd(const lpmm_tensor_desc* descs, int64_t n, const int64_t* inner_dims,
                                 const int32_t* inner_ndim) {
    PlanLayout L;
    return plan_layout(descs, n, inner_dims, inner_ndim, &L) ? L.total : 0;
}

int lpmm_adamw4_plan_build(const lpmm_tensor_desc* descs, int64_t n, int grad_dtype, void* plan,
                           size_t plan_bytes, void* stream) {
    return lpmm_adamw4_plan_build_nd(descs, n, nullptr, nullptr, grad_dtype, plan, plan_bytes, stream);
}

int lpmm_adamw4_plan_build_nd(const lpmm_tensor_desc* descs, int64_t n, const int64_t* inner_dims,
                              const int32_t* inner_ndim, int grad_dtype, void* plan, size_t plan_bytes,
                              void* stream) {
    PlanLayout L;
    if (!plan_layout(descs, n, inner_dims, inner_ndim, &L)) return LPMM_EINVAL;
    if (!plan || !aligned(plan, 256) || plan_bytes < L.total) return LPMM_EINVAL;
    if (grad_dtype != LPMM_GRAD_F32 && grad_dtype != LPMM_GRAD_BF16) return LPMM_EINVAL;
    DeviceCtx* ctx;
    int rc = current_ctx(&ctx);          // the lookup tables are uploaded by lpmm_adamw4_init
    if (rc) return rc;
    int dev = 0;
    LPMM_HIP(hipGetDevice(&dev));

    auto host = std::make_shared<PlanHost>();
    host->bf16 = grad_dtype == LPMM_GRAD_BF16;
    host->device = dev;
    host->staging.assign(L.off_counters, 0);
    Tensor4* tens = reinterpret_cast<Tensor4*>(host->staging.data() + L.off_tensors);
    InnerDims* h_dims = reinterpret_cast<InnerDims*>(host->staging.data() + L.off_dims);
    int64_t n_nd = 0;
    char* dplan = static_cast<char*>(plan);
    const Tensor4* d_tens = reinterpret_cast<const Tensor4*>(dplan + L.off_tensors);
    float* d_floats = reinterpret_cast<float*>(dplan + L.off_floats);
    const InnerDims* d_dims = reinterpret_cast<const InnerDims*>(dplan + L.off_dims);
    host->d_hyper = reinterpret_cast<Hyper*>(dplan + L.off_hyper);
    unsigned int* d_counters = reinterpret_cast<unsigned int*>(dplan + L.off_counters);

    const int64_t rw_hint = env_int("LPMM_MULTI_RW", -1);      // -1: the plan defaults (64 rows, 32 for the flat tiling)
    const int64_t rw2_hint = env_int("LPMM_MULTI_RW2", 128);
    // Flat tiling of pass 1 for the large tensors of this plan?  Measured: 3-4 % faster on the 7B-shaped set, where
    // pass 1 runs beside pass 2 of the previous group; 4 % slower for one large tensor alone (one group, the passes
    // run one after the other); slower on sets of small tensors, whose tiles become too few; and a launch that
    // mixes many cheap tiles with a few four times more expensive flat ones loses 20 % to imbalance between the
    // XCDs.  So: only in plans with several groups whose rank-1 parameters are at least 90 % in large tensors.
    constexpr int64_t kFlatMinElems = int64_t(1) << 23;
    // parameters per group of consecutive tensors: large groups win (fewer kernel tails); cutting a set that fits
    // one group into three so that its pass 2 has a pass 1 to run beside gave -3 % on the 108 M set, nothing on
    // the 354 M set and +1.4 % on its factorized form, so it is not done
    int64_t group_params = int64_t(env_int("LPMM_PHASE_MPARAMS", 2048)) << 20;
    if (n > kMaxSeg && env_int("LPMM_PHASE_MPARAMS", 0) <= 0) {
        // More tensors than one group's tables hold: cut by parameters, into about equal parts, instead of filling
        // every group up to the table size (292 tensors of 354 M parameters: 190 M + 164 M parameters measured 0.895
        // ms per step, the first 192 tensors + the rest, 254 M + 100 M, 0.905).  The tenth on top keeps the greedy fill
        // below from leaving a small group over.
        int64_t total = 0;
        for (int64_t i = 0; i < n; ++i) total += descs[i].rows * descs[i].cols;
        const int64_t k = (n + kMaxSeg - 1) / kMaxSeg;
        group_params = std::min(group_params, total / k + total / (10 * k) + 1);
    }
    bool plan_flat = false;
    {
        const int64_t gp = group_params;
        int64_t p_rank1 = 0, p_big = 0, acc = 0, in_group = 0, n_groups = 0;
        for (int64_t i = 0; i < n; ++i) {
            const int64_t P = descs[i].rows * descs[i].cols;
            if ((descs[i].kind == LPMM_KIND_4BIT || descs[i].kind == LPMM_KIND_4BIT_ND) &&
                fast_eligible(descs[i].cols, descs[i].v_colmax)) {
                p_rank1 += P;
                if (P >= kFlatMinElems) p_big += P;
            }
            if (in_group == 0 || in_group >= kMaxSeg || acc + P > gp) { ++n_groups; acc = 0; in_group = 0; }
            acc += P;
            ++in_group;
        }
        plan_flat = n_groups > 1 && p_rank1 > 0 && p_big * 10 >= p_rank1 * 9;
    }
    // Tiling of one quantized tensor of the plan.  shrink = 0 gives the plan's default tiles (sized for sets that
    // fill the chip many times over); each further level halves the rows (blocks) a workgroup takes, for groups of
    // tensors that are too small to give every CU a couple of workgroups (see below).
    const int gbytes = grad_dtype == LPMM_GRAD_BF16 ? 2 : 4;
    auto set_geometry = [&](Tensor4& t, const lpmm_tensor_desc& d, int shrink) {
        const int64_t rw_s = std::max<int64_t>((rw_hint < 0 ? 64 : rw_hint) >> shrink, 8);
        const int64_t rw2_s = std::max<int64_t>(rw2_hint >> shrink, 4);
        const int64_t rounds_s = std::max<int64_t>(int64_t(env_int("LPMM_MULTI_B128_ROUNDS", 8)) >> shrink, 1);
        if (d.kind == LPMM_KIND_SGDM_4BIT) {
            b128_geometry(&t, ctx->n_cu, rounds_s);
            t.kind = kSgdmBlock;
        } else if (d.kind == LPMM_KIND_4BIT_B128) {
            b128_geometry(&t, ctx->n_cu, rounds_s);
        } else if (d.kind == LPMM_KIND_4BIT_FACTOR) {
            factor_geometry(&t, ctx->n_cu, shrink ? rw_s : rw_hint, rw2_s, gbytes, fast_eligible(d.cols, d.v_colmax), 1);
        } else if (t.kind == kQuantFast) {
            fast_geometry(&t, ctx->n_cu, shrink ? rw_s : rw_hint, rw2_s, gbytes, plan_flat && t.P >= kFlatMinElems);
        }
    };
    int64_t fofs = 0;
    for (int64_t i = 0; i < n; ++i) {
        const lpmm_tensor_desc& d = descs[i];
        const size_t galign = grad_dtype == LPMM_GRAD_F32 ? 4 : 2;
        Tensor4 t{};
        t.rows = d.rows; t.cols = d.cols; t.P = d.rows * d.cols;
        if (d.flags & ~(LPMM_FLAG_NO_DECAY | LPMM_FLAG_DETERMINISTIC)) return LPMM_EINVAL;
        if ((d.flags & LPMM_FLAG_DETERMINISTIC) &&
            (d.kind != LPMM_KIND_4BIT_FACTOR || !fast_eligible(d.cols, d.v_colmax))) return LPMM_EINVAL;
        t.no_decay = (d.flags & LPMM_FLAG_NO_DECAY) ? 1 : 0;
        t.p = static_cast<float*>(d.param);
        t.g = d.grad;
        t.mq = static_cast<uint32_t*>(d.m_state);
        t.vq = static_cast<uint32_t*>(d.v_state);
        if (!d.param || !d.grad || !d.m_state) return LPMM_EINVAL;
        const bool is_sgdm = d.kind == LPMM_KIND_SGDM_4BIT || d.kind == LPMM_KIND_SGDM_FP32;
        if (!d.v_state && d.kind != LPMM_KIND_4BIT_FACTOR && !is_sgdm) return LPMM_EINVAL;
        if (d.kind == LPMM_KIND_SGDM_FP32) {
            if (!aligned(d.param, 4) || !aligned(d.m_state, 4) || !aligned(d.grad, galign)) return LPMM_EINVAL;
            t.vq = nullptr;
            t.kind = kSgdmFp32;
            t.n_wg = t.n_wg2 = int((t.P + kElemsPerWg32 - 1) / kElemsPerWg32);
            host->sgdm = true;
        } else if (d.kind == LPMM_KIND_SGDM_4BIT) {
            if (!d.m_blockscale) return LPMM_EINVAL;
            if (!aligned(d.param, 16) || !aligned(d.grad, 16) || !aligned(d.m_state, 4) || !aligned(d.m_blockscale, 4))
                return LPMM_EINVAL;
            t.vq = nullptr;
            t.ms = d.m_blockscale;
            set_geometry(t, d, 0);
            host->sgdm = true;
        } else if (d.kind == LPMM_KIND_4BIT_FACTOR) {
            if (!d.m_blockscale || !d.v_rowmax || !d.v_colmax) return LPMM_EINVAL;
            if (!aligned(d.param, 16) || !aligned(d.grad, 16) || !aligned(d.m_state, 4) ||
                !aligned(d.m_blockscale, 4) || !aligned(d.v_rowmax, 4) || !aligned(d.v_colmax, 4))
                return LPMM_EINVAL;
            t.vq = nullptr;
            t.ms = d.m_blockscale;
            t.r = d.v_rowmax;                      // row statistics
            t.c = d.v_colmax;                      // column statistics
            t.r_new = d_floats + fofs;
            fofs += round_up(d.rows, 64);
            t.c_new = d_floats + fofs;
            fofs += round_up(d.cols, 64);
            t.counter = d_counters + i * kCounterWords;
            if (d.flags & LPMM_FLAG_DETERMINISTIC) {
                t.det = 1;
                t.vq = reinterpret_cast<uint32_t*>(d_floats + fofs);      // the partial sums
                fofs += det_partial_floats(d.rows, d.cols);
            }
            set_geometry(t, d, 0);
            host->factor = true;
        } else if (d.kind == LPMM_KIND_FP32) {
            if (!aligned(d.param, 4) || !aligned(d.m_state, 4) || !aligned(d.v_state, 4) || !aligned(d.grad, galign))
                return LPMM_EINVAL;
            t.kind = kFp32State;
            t.n_wg = t.n_wg2 = int((t.P + kElemsPerWg32 - 1) / kElemsPerWg32);
        } else if (d.kind == LPMM_KIND_4BIT_B128) {
            if (!d.m_blockscale || !d.v_rowmax) return LPMM_EINVAL;
            if (!aligned(d.param, 16) || !aligned(d.grad, 16) || !aligned(d.m_state, 4) || !aligned(d.v_state, 4) ||
                !aligned(d.m_blockscale, 4) || !aligned(d.v_rowmax, 4))
                return LPMM_EINVAL;
            t.ms = d.m_blockscale;
            t.r = d.v_rowmax;                      // block scales of the second moment
            t.kind = kQuantBlockV;
            set_geometry(t, d, 0);
        } else {
            if (!d.m_blockscale || !d.v_rowmax || !d.v_colmax) return LPMM_EINVAL;
            if (!aligned(d.param, 16) || !aligned(d.grad, 16) || !aligned(d.m_state, 4) || !aligned(d.v_state, 4) ||
                !aligned(d.m_blockscale, 4) || !aligned(d.v_rowmax, 4) || !aligned(d.v_colmax, 4))
                return LPMM_EINVAL;
            t.ms = d.m_blockscale;
            t.r = d.v_rowmax;
            t.c = d.v_colmax;
            t.nd_index = -1;
            int64_t ext = 0;
            if (d.kind == LPMM_KIND_4BIT_ND) {
                // more than two dimensions: v_colmax holds the column scales and, behind them, the statistics of
                // the inner dimensions; the workspace mirrors that layout (see lpmm_adamw4_nd_step)
                InnerDims dm;
                if (!plan_inner_dims(d, i, inner_dims, inner_ndim, &dm, &ext)) return LPMM_EINVAL;
                h_dims[n_nd] = dm;
                t.nd_index = int(n_nd++);
                t.c_extra = int(ext);
            }
            t.r_new = d_floats + fofs;
            fofs += round_up(d.rows, 64);
            t.c_new = d_floats + fofs;
            fofs += round_up(d.cols + ext, 64);
            t.counter = d_counters + i * kCounterWords;
            if (fast_eligible(d.cols, d.v_colmax)) {
                t.kind = kQuantFast;
                set_geometry(t, d, 0);
                if (t.flat) host->flat = true;
            } else {
                t.kind = kQuantGeneral;
                general_geometry(&t, ctx->n_cu);
            }
        }
        tens[i] = t;
        host->params += t.P;
    }

    // groups of consecutive tensors; phase j = A work of group j + B work of group j-1
    std::vector<std::pair<int64_t, int64_t>> groups;      // [first, last)
    for (int64_t i = 0; i < n;) {
        int64_t j = i, acc = 0;
        while (j < n && j - i < kMaxSeg && (j == i || acc + tens[j].P <= group_params)) acc += tens[j++].P;
        groups.emplace_back(i, j);
        i = j;
    }
    // A group whose tensors are small would put few, long workgroups on the chip (one 1024 x 1024 matrix: 128 for
    // its first pass, 32 for its second, on 256 CUs): halve its tiles until each of its launches has two
    // workgroups per CU (measured on that matrix: 23.5 -> 13.8 us per step).
    for (const auto& gr : groups) {
        for (int shrink = 1; shrink <= 3; ++shrink) {
            int64_t n_a = 0, n_b = 0;
            bool two_pass = false;
            for (int64_t i = gr.first; i < gr.second; ++i) {
                n_a += tens[i].n_wg;
                const bool has_b = tens[i].kind == kQuantFast || tens[i].kind == kQuantGeneral ||
                                   tens[i].kind == kFactorFast || tens[i].kind == kFactorGeneral;
                if (has_b) { n_b += tens[i].n_wg2; two_pass = true; }
            }
            if (n_a >= 2 * int64_t(ctx->n_cu) && (!two_pass || n_b >= 2 * int64_t(ctx->n_cu))) break;
            for (int64_t i = gr.first; i < gr.second; ++i) set_geometry(tens[i], descs[i], shrink);
        }
    }
    for (size_t j = 0; j <= groups.size(); ++j) {
        PhaseLaunch pl{};
        pl.ph.tensors = reinterpret_cast<const Tensor4Table*>(d_tens);
        if (j < groups.size())
            for (int64_t i = groups[j].first; i < groups[j].second; ++i) {
                pl.ph.seg_a[pl.ph.n_seg_a++] = Segment{pl.ph.n_a, int(i)};
                if (tens[i].kind == kQuantFast || tens[i].kind == kQuantGeneral) pl.a_has_rank1 = true;
                pl.ph.n_a += tens[i].n_wg;
            }
        if (j >= 1)
            for (int64_t i = groups[j - 1].first; i < groups[j - 1].second; ++i) {
                if (tens[i].kind == kFp32State || tens[i].kind == kQuantBlockV || tens[i].kind == kSgdmBlock ||
                    tens[i].kind == kSgdmFp32)
                    continue;
                pl.ph.seg_b[pl.ph.n_seg_b++] = Segment{pl.ph.n_b, int(i)};
                pl.ph.n_b += tens[i].n_wg2;
                if (tens[i].det) {
                    pl.has_det = true;
                    pl.det.seg_r[pl.det.n_seg++] = Segment{pl.det.n_r, int(i)};
                    pl.det.n_r += int((tens[i].rows + kThreads - 1) / kThreads + (tens[i].cols + 63) / 64);
                }
                if (tens[i].nd_index >= 0 && (tens[i].kind == kQuantFast || tens[i].kind == kQuantGeneral)) {
                    pl.has_nd = true;
                    pl.nd.seg_r[pl.nd.n_seg] = Segment{pl.nd.n_r, int(i)};
                    pl.nd.seg_e[pl.nd.n_seg] = Segment{pl.nd.n_e, int(i)};
                    ++pl.nd.n_seg;
                    pl.nd.n_r += tens[i].c_extra;                                       // one workgroup per statistic
                    pl.nd.n_e += int((tens[i].cols + kThreads - 1) / kThreads);
                }
            }
        pl.nd.tensors = pl.ph.tensors;
        pl.nd.dims = d_dims;
        pl.det.tensors = pl.ph.tensors;
        if (pl.ph.n_a + pl.ph.n_b == 0) continue;
        if (int64_t(pl.ph.n_a) + pl.ph.n_b > (int64_t(1) << 30)) return LPMM_EINVAL;
        pl.grid = pad8(int64_t(pl.ph.n_a) + pl.ph.n_b);
        pl.grid_a = pad8(pl.ph.n_a);
        pl.grid_b = pad8(pl.ph.n_b);
        host->phases.push_back(pl);
    }
    // A second stream pays only if some pass 2 has a pass 1 of another group to run beside.  Factorized plans take
    // their launches one after the other on the caller's stream by default: the statistics pass (read-only) and the
    // update pass each run at the memory system's rate alone, and side by side they only get in each other's way
    // (7B-shaped set: 14.71 ms per step against 14.84, 354 M set 0.841 against 0.854).
    const int stream_mode = env_int("LPMM_MULTI_STREAMS", host->factor ? 0 : 2);
    host->serial = stream_mode == 0 && !host->sgdm;
    bool any_b = false;
    for (const PhaseLaunch& pl : host->phases) any_b = any_b || pl.ph.n_b > 0;
    if (stream_mode >= 2 && groups.size() > 1 && !host->sgdm && any_b) {
        LPMM_HIP(hipStreamCreateWithFlags(&host->side, hipStreamNonBlocking));
        LPMM_HIP(hipEventCreateWithFlags(&host->ev_fork, hipEventDisableTiming));
        LPMM_HIP(hipEventCreateWithFlags(&host->ev_join, hipEventDisableTiming));
        if (stream_mode >= 3) {
            LPMM_HIP(hipStreamCreateWithFlags(&host->side_a, hipStreamNonBlocking));
            LPMM_HIP(hipEventCreateWithFlags(&host->ev_join_a, hipEventDisableTiming));
        }
        host->ev_a.resize(host->phases.size());
        for (hipEvent_t& e : host->ev_a) LPMM_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    }

    hipStream_t s = static_cast<hipStream_t>(stream);
    LPMM_HIP(hipMemsetAsync(dplan + L.off_counters, 0, L.total - L.off_counters, s));
    LPMM_HIP(hipMemcpyAsync(dplan, host->staging.data(), L.off_counters, hipMemcpyHostToDevice, s));
    std::lock_guard<std::mutex> lock(g_mu);
    g_plans[plan] = std::move(host);
    return LPMM_OK;
}

}  // extern "C"

namespace {

// One-pass kernels (block-wise AdamW, SGDM) of plans of 2^30 parameters or more run with four workgroups per CU
// instead of the seven or eight that their registers allow, by way of unused dynamic LDS: 1 % less time per step on
// the 7B-shaped set (more resident waves only lengthen every wave's queueing), 2-3 % more on the 354 M set, whose
// launches are short, hence the size condition.  LPMM_P3_LDS_PAD overrides the number of bytes.
unsigned one_pass_lds_pad(const PlanHost& host) {
    return unsigned(std::clamp(env_int("LPMM_P3_LDS_PAD", host.params >= (int64_t(1) << 30) ? 14336 : 0), 0, 45056));
}

// lr_dev / step_dev non-null: the capturable form, hyper-parameters prepared on the device
int adamw4_step_multi_impl(void* plan, float lr, const float* lr_dev, float beta1, float beta2, float eps,
                           float weight_decay, int64_t step, const int64_t* step_dev, void* stream) {
#define LPMM_CHECK(call) do { const int rc_ = (call); if (rc_) return rc_; } while (0)
    // column maxima -> new statistics -> new column scales, for the group's tensors with more than two dimensions
    auto launch_nd = [](const PhaseLaunch& pl, hipStream_t on) -> int {
        hipLaunchKernelGGL(nd_plan_reduce, dim3(pl.nd.n_r), dim3(kThreads), 0, on, pl.nd);
        LPMM_HIP(hipGetLastError());
        hipLaunchKernelGGL(nd_plan_expand, dim3(pl.nd.n_e), dim3(kThreads), 0, on, pl.nd);
        LPMM_HIP(hipGetLastError());
        return LPMM_OK;
    };
    // per-tile partial sums -> row / column sums and totals, for the group's tensors with deterministic sums
    auto launch_det = [](const PhaseLaunch& pl, hipStream_t on) -> int {
        hipLaunchKernelGGL(factor_plan_reduce, dim3(pl.det.n_r), dim3(kThreads), 0, on, pl.det);
        LPMM_HIP(hipGetLastError());
        hipLaunchKernelGGL(factor_plan_totals, dim3(pl.det.n_seg), dim3(kThreads), 0, on, pl.det);
        LPMM_HIP(hipGetLastError());
        return LPMM_OK;
    };
    const bool capturable = lr_dev != nullptr;
    HyperArg h{};
    const int rc = make_hyper(capturable ? 0.0f : lr, beta1, beta2, eps, weight_decay, capturable ? 1 : step, &h.h);
    if (rc) return rc;
    if (capturable && !step_dev) return LPMM_EINVAL;
    std::shared_ptr<const PlanHost> host;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        auto it = g_plans.find(plan);
        if (it == g_plans.end()) return LPMM_EINVAL;
        host = it->second;
    }
    int dev = 0;
    LPMM_HIP(hipGetDevice(&dev));
    if (dev != host->device || host->sgdm) return LPMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool bf16 = host->bf16;
    if (capturable) {
        hipLaunchKernelGGL(hyper_prepare_kernel, dim3(1), dim3(64), 0, s, lr_dev, step_dev, beta1, beta2, eps,
                           weight_decay, host->d_hyper);
        LPMM_HIP(hipGetLastError());
        h.dev = host->d_hyper;
    }
    // Plans with the flat tiling of pass 1 run their pass-1 launches with unused dynamic LDS, so that three instead of
    // five workgroups share a CU: two waves per SIMD already saturate pass 1 on large tensors, and more of them only
    // take issue slots and memory queues from the pass 2 that runs beside (measured on the 7B-shaped set: 1 % less
    // time per step with bf16 gradients, 1-3 % with fp32 gradients; sets of small tensors lose 4 %, so not there).
    const unsigned lds_pad = unsigned(std::clamp(env_int("LPMM_P1_LDS_PAD", host->flat ? 22528 : 0), 0, 45056));
    const unsigned pad3 = one_pass_lds_pad(*host);
    // roles: 0 = A and B work in one launch, 1 = A only, 2 = B only, 3 = A only without rank-1 tensors
    auto launch = [&](int roles, int grid, hipStream_t on, const PhaseLaunch& pl) {
#define LPMM_PHASE_CASE(K, R)                                                                               \
        if (bf16) hipLaunchKernelGGL((K<true, R>), dim3(grid), dim3(kThreads), (R == 1 ? lds_pad : R == 3 ? pad3 : 0), on, pl.ph, h);            \
        else hipLaunchKernelGGL((K<false, R>), dim3(grid), dim3(kThreads), (R == 1 ? lds_pad : R == 3 ? pad3 : 0), on, pl.ph, h);
        if (host->factor) {
            if (roles == 0) { LPMM_PHASE_CASE(factor_phase_kernel, 0) }
            else if (roles == 2) { LPMM_PHASE_CASE(factor_phase_kernel, 2) }
            else { LPMM_PHASE_CASE(factor_phase_kernel, 1) }
        } else {
            if (roles == 0) { LPMM_PHASE_CASE(phase_kernel, 0) }
            else if (roles == 1) { LPMM_PHASE_CASE(phase_kernel, 1) }
            else if (roles == 2) { LPMM_PHASE_CASE(phase_kernel, 2) }
            else { LPMM_PHASE_CASE(phase_kernel, 3) }
        }
#undef LPMM_PHASE_CASE
    };
    if (host->side || host->serial) {
        // A work of phase j on the caller's stream, B work (pass 2 of the tensors whose pass 1 ran
        // in phase j-1) on the side stream behind an event; the caller's stream rejoins at the end.
        // Serial plans take the same launches one after the other on the caller's stream, without events.
        const bool two = host->side != nullptr;
        hipStream_t s2 = two ? host->side : s;
        // The side stream's first work waits for the event behind the first A launch, which also puts it behind
        // everything that was on the caller's stream before this call (and into a capture of that stream): no fork
        // event is needed for it.  A second stream for pass 1 starts with work of its own and does need one.
        if (host->side_a) {
            LPMM_HIP(hipEventRecord(host->ev_fork, s));
            LPMM_HIP(hipStreamWaitEvent(host->side_a, host->ev_fork, 0));
        }
        // The last phase holds B work only, with no pass 1 left to run beside: it goes on the caller's stream,
        // straight behind the A work it depends on, and spares the step one hand-over between the streams (a
        // dependent launch on another stream starts 10-15 us later than one on the same stream).
        const size_t n_ph = host->phases.size();
        const bool tail_on_s = two && !host->side_a && n_ph >= 2 && host->phases[n_ph - 1].ph.n_a == 0;
        for (size_t j = 0; j < n_ph; ++j) {
            const PhaseLaunch& pl = host->phases[j];
            const bool tail = tail_on_s && j + 1 == n_ph;
            if (tail) {
                LPMM_HIP(hipEventRecord(host->ev_join, s2));      // everything the side stream was given
                s2 = s;
            }
            if (pl.ph.n_b > 0) {
                if (two && !tail) LPMM_HIP(hipStreamWaitEvent(s2, host->ev_a[j - 1], 0));
                // a factorized plan's heavy kernel is its B work (the update pass): that one is timed
                const bool rec = host->factor && g_prof.on && g_prof.calls < g_prof.max_calls;
                const int64_t call = g_prof.calls;
                if (rec) LPMM_HIP(hipEventRecord(prof_event(call, 0), s2));
                if (pl.has_nd) LPMM_CHECK(launch_nd(pl, s2));
                if (pl.has_det) LPMM_CHECK(launch_det(pl, s2));
                launch(2, pl.grid_b, s2, pl);
                LPMM_HIP(hipGetLastError());
                if (rec) {
                    LPMM_HIP(hipEventRecord(prof_event(call, 1), s2));
                    LPMM_HIP(hipEventRecord(prof_event(call, 2), s2));
                    g_prof.calls = call + 1;
                }
            }
            hipStream_t sa = (host->side_a && (j & 1)) ? host->side_a : s;
            if (pl.ph.n_a > 0) {
                const bool rec = !host->factor && g_prof.on && g_prof.calls < g_prof.max_calls;
                const int64_t call = g_prof.calls;
                if (rec) LPMM_HIP(hipEventRecord(prof_event(call, 0), sa));
                launch(pl.a_has_rank1 ? 1 : 3, pl.grid_a, sa, pl);
                LPMM_HIP(hipGetLastError());
                if (rec) {
                    LPMM_HIP(hipEventRecord(prof_event(call, 1), sa));
                    LPMM_HIP(hipEventRecord(prof_event(call, 2), sa));
                    g_prof.calls = call + 1;
                }
            }
            // an event only where the next phase has B work that waits for it on the side stream (nobody waits
            // for the A work of the last group when its B work follows it on the same stream)
            const bool waited_for = j + 1 < n_ph && host->phases[j + 1].ph.n_b > 0 && !(tail_on_s && j + 2 >= n_ph);
            if (two && waited_for) LPMM_HIP(hipEventRecord(host->ev_a[j], sa));
        }
        if (!two) return LPMM_OK;
        if (!tail_on_s) LPMM_HIP(hipEventRecord(host->ev_join, s2));
        LPMM_HIP(hipStreamWaitEvent(s, host->ev_join, 0));
        if (host->side_a) {
            LPMM_HIP(hipEventRecord(host->ev_join_a, host->side_a));
            LPMM_HIP(hipStreamWaitEvent(s, host->ev_join_a, 0));
        }
        return LPMM_OK;
    }
    for (const PhaseLaunch& pl : host->phases) {
        // as on the two-stream route, only launches that carry pass 1 (factorized plans: the update pass) are timed
        const bool rec = g_prof.on && g_prof.calls < g_prof.max_calls && (host->factor ? pl.ph.n_b > 0 : pl.ph.n_a > 0);
        const int64_t call = g_prof.calls;
        if (rec) LPMM_HIP(hipEventRecord(prof_event(call, 0), s));
        // a launch that holds only one kind of work takes that kind's (lighter) kernel
        if (pl.has_nd) LPMM_CHECK(launch_nd(pl, s));      // the A work of these tensors ran in the previous launch
        if (pl.has_det) LPMM_CHECK(launch_det(pl, s));
        const int roles = pl.ph.n_b == 0 ? (pl.a_has_rank1 ? 1 : 3) : (pl.ph.n_a == 0 ? 2 : 0);
        launch(roles, pl.grid, s, pl);
        LPMM_HIP(hipGetLastError());
        if (rec) {
            LPMM_HIP(hipEventRecord(prof_event(call, 1), s));
            LPMM_HIP(hipEventRecord(prof_event(call, 2), s));
            g_prof.calls = call + 1;
        }
    }
    return LPMM_OK;
}

int sgdm4_step_multi_impl(void* plan, float lr, const float* lr_dev, float momentum, void* stream) {
    HyperArg h{};
    const int rc = make_sgdm_hyper(lr_dev ? 0.0f : lr, momentum, &h.h);
    if (rc) return rc;
    std::shared_ptr<const PlanHost> host;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        auto it = g_plans.find(plan);
        if (it == g_plans.end()) return LPMM_EINVAL;
        host = it->second;
    }
    int dev = 0;
    LPMM_HIP(hipGetDevice(&dev));
    if (dev != host->device || !host->sgdm) return LPMM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (lr_dev) {
        hipLaunchKernelGGL(sgdm_hyper_prepare_kernel, dim3(1), dim3(64), 0, s, lr_dev, momentum, host->d_hyper);
        LPMM_HIP(hipGetLastError());
        h.dev = host->d_hyper;
    }
    for (const PhaseLaunch& pl : host->phases) {
        if (pl.ph.n_a == 0) continue;
        const bool rec = g_prof.on && g_prof.calls < g_prof.max_calls;
        const int64_t call = g_prof.calls;
        if (rec) LPMM_HIP(hipEventRecord(prof_event(call, 0), s));
        const unsigned pads = one_pass_lds_pad(*host);
        if (host->bf16) hipLaunchKernelGGL(sgdm_phase_kernel<true>, dim3(pl.grid_a), dim3(kThreads), pads, s, pl.ph, h);
        else hipLaunchKernelGGL(sgdm_phase_kernel<false>, dim3(pl.grid_a), dim3(kThreads), pads, s, pl.ph, h);
        LPMM_HIP(hipGetLastError());
        if (rec) {
            LPMM_HIP(hipEventRecord(prof_event(call, 1), s));
            LPMM_HIP(hipEventRecord(prof_event(call, 2), s));
            g_prof.calls = call + 1;
        }
    }
    return LPMM_OK;
}

}  // namespace

extern "C" {

int lpmm_adamw4_step_multi(void* plan, float lr, float beta1, float beta2, float eps, float weight_decay,
                           int64_t step, void* stream) {
    return adamw4_step_multi_impl(plan, lr, nullptr, beta1, beta2, eps, weight_decay, step, nullptr, stream);
}

int lpmm_adamw4_step_multi_capturable(void* plan, const float* lr, const int64_t* step, float beta1, float beta2,
                                      float eps, float weight_decay, void* stream) {
    if (!lr || !step) return LPMM_EINVAL;
    return adamw4_step_multi_impl(plan, 0.0f, lr, beta1, beta2, eps, weight_decay, 1, step, stream);
}

int lpmm_sgdm4_step_multi(void* plan, float lr, float momentum, void* stream) {
    return sgdm4_step_multi_impl(plan, lr, nullptr, momentum, stream);
}

int lpmm_sgdm4_step_multi_capturable(void* plan, const float* lr, float momentum, void* stream) {
    if (!lr) return LPMM_EINVAL;
    return sgdm4_step_multi_impl(plan, 0.0f, lr, momentum, stream);
}

int lpmm_adamw4_plan_release(void* plan) {
    std::lock_guard<std::mutex> lock(g_mu);
    return g_plans.erase(plan) ? LPMM_OK : LPMM_EINVAL;
}

int lpmm_profile_begin(int64_t max_calls) {
    if (max_calls < 1 || max_calls > (int64_t(1) << 20)) return LPMM_EINVAL;
    while (int64_t(g_prof.ev.size()) < 3 * max_calls) {
        hipEvent_t e;
        LPMM_HIP(hipEventCreate(&e));
        g_prof.ev.push_back(e);
    }
    g_prof.max_calls = max_calls;
    g_prof.calls = 0;
    g_prof.on = true;
    return LPMM_OK;
}

int lpmm_profile_end(double ms[2], int64_t* n_calls) {
    if (!ms || !n_calls) return LPMM_EINVAL;
    g_prof.on = false;
    ms[0] = ms[1] = 0.0;
    *n_calls = g_prof.calls;
    for (int64_t c = 0; c < g_prof.calls; ++c) {
        LPMM_HIP(hipEventSynchronize(prof_event(c, 2)));
        float a = 0.0f, b = 0.0f;
        LPMM_HIP(hipEventElapsedTime(&a, prof_event(c, 0), prof_event(c, 1)));
        LPMM_HIP(hipEventElapsedTime(&b, prof_event(c, 1), prof_event(c, 2)));
        ms[0] += a;
        ms[1] += b;
    }
    g_prof.calls = 0;
    return LPMM_OK;
}

}  // extern "C"
