/*
 * lpmm4.h -- C ABI of lpmm4.so: the fused 4-bit AdamW optimizer step for AMD MI355X (gfx950).
 *
 * Method: "Memory Efficient Optimizers with 4-bit States" (arXiv 2309.01507).  One step is
 * Alg. 1 lines 3-5 / App. E Alg. 3 for one parameter tensor: decompress the 4-bit first and
 * second moment, apply the Adam rule of Eq. 1 (with AdamW's decoupled weight decay) on the precise
 * moments, compress both moments again.
 *   first moment : block-wise normalization, block 128 over the row-major flattening (Sec. 2.2,
 *                  Sec. 3), signed form n = sign(x) N(|x|) (App. D.1), signed 4-bit
 *                  dynamic-exponent map (App. D.2).
 *   second moment: rank-1 normalization n_ij = x_ij / min(r_i, c_j) with r_i = max_j x_ij,
 *                  c_j = max_i x_ij (Sec. 4.2), Linear map T(i) = (i+1)/16 without zero (Sec. 4.1).
 *
 * Further sections below: the block-wise second moment for 1-dimensional / flattened tensors (Sec. 4.2),
 * the factorized second moment of "4-bit Factor" (Sec. 4.3), rank-1 normalization for more than two
 * dimensions (App. F Alg. 4), SGD with momentum (App. E Alg. 2), stand-alone compress / decompress, the
 * quantizers the paper ablates for the second moment (Sec. 4.1, Tab. 1, App. D.3), plans (many tensors per
 * call), and the plan steps with device-resident learning rate and step number.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers unless the comment says "host".  The caller owns every
 *     buffer; the library allocates no device memory and never frees anything.
 *   - `shape` is a HOST pointer to {rows, cols}; tensors are row-major, P = rows*cols elements.
 *     Calls that take a flat tensor (numel) accept any shape.  A 1-dimensional tensor belongs to
 *     lpmm_adamw4_b128_step, not to the rank-1 step: Sec. 4.2 replaces rank-1 normalization by B128 there.
 *     (The rank-1 calls accept rows == 1 or cols == 1 and then do what Sec. 4.2's formula says literally --
 *     every element is its own column maximum, all codes are 15 and v_colmax is a plain fp32 copy of the
 *     second moment -- which is correct but compresses nothing.)
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue work
 *     and return; they never synchronize.  Work of one call is ordered on `stream`.
 *   - Return value: LPMM_OK or a negative error code; nothing is printed, nothing aborts.
 *     On error nothing has been enqueued, except LPMM_EHIP from a launch in the middle of a call.
 *   - NaN/Inf in gradients or states are not detected; the result is then unspecified.
 *
 * State layout of one quantized tensor (all caller-owned, sizes from lpmm_adamw4_state_sizes)
 *   m_codes      uint8[(P+1)/2]   two codes per byte: element 2k in bits 0..3, element 2k+1 in
 *                                 bits 4..7; a code is the rank of the value in the increasing
 *                                 DE table (code 7 = 0.0, code 15 = +1.0)
 *   m_blockscale float[ceil(P/128)]  absmax of block k = elements [128k, 128k+127]
 *   v_codes      uint8[(P+1)/2]   same packing; code q stands for (q+1)/16
 *   v_rowmax     float[rows]      r_i
 *   v_colmax     float[cols]      c_j
 *   The zero state of Alg. 3 (m_0 = v_0 = 0) is: m codes 7, block scales 0, v codes 0, r = c = 0.
 */
#ifndef LPMM4_H
#define LPMM4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LPMM_OK          0
#define LPMM_EINVAL     (-1)  /* null / misaligned pointer, bad shape, step < 1, bad hyper-parameter */
#define LPMM_ENOTINIT   (-2)  /* lpmm_adamw4_init has not been called for the current device */
#define LPMM_EHIP       (-3)  /* a HIP call failed; see lpmm_last_hip_error() */
#define LPMM_EWORKSPACE (-4)  /* the workspace given to init is too small for this tensor */

#define LPMM_BLOCK 128        /* B128, Sec. 3 */

/* Gradient element types. */
#define LPMM_GRAD_F32  0
#define LPMM_GRAD_BF16 1

/* Human-readable text for an error code (host, static storage). */
const char* lpmm_strerror(int code);
/* hipError_t (as int) of the most recent LPMM_EHIP in the calling host thread, else 0. */
int lpmm_last_hip_error(void);

/* The two 16-entry quantization maps the kernels use (host call, no GPU needed):
 * which = 0: signed dynamic-exponent map of App. D.2; which = 1: Linear map of Sec. 4.1.
 * out: host float[16].  Returns LPMM_EINVAL for another `which` or a null pointer. */
int lpmm_table(int which, float* out);

/* Host model of the kernels' nearest-entry search M(n) = argmin_i |n - T(i)| (Sec. 2.2), ties to
 * the lower index: the same bucket table the kernels read, evaluated on the CPU.  For tests of
 * the host-built table; which as in lpmm_table.  n, out: host arrays of `count` elements. */
int lpmm_host_nearest_codes(int which, const float* n, int64_t count, uint8_t* out);

/* Bytes of workspace lpmm_adamw4_init needs so that steps on tensors with rows + cols <=
 * max_rows_plus_cols can run.  The workspace holds the row/column maxima of the updated second
 * moment (Sec. 4.2) while the old ones are still being read, plus completion counters. */
size_t lpmm_adamw4_workspace_bytes(int64_t max_rows_plus_cols);

/* Registers `workspace` (device memory, 256-byte aligned, workspace_bytes long, owned by the caller
 * and kept alive until the process ends or init is called again) for device `device`, clears it
 * on `stream`, and uploads the quantization tables.  May be called again to replace the
 * workspace.  Steps on one device share this workspace: calls that may overlap in time on one
 * device (different streams) race; calls on one stream are safe.  For steps that overlap, see
 * lpmm_adamw4_step_ws (a workspace per call) and the plans (a workspace per plan). */
int lpmm_adamw4_init(int device, void* workspace, size_t workspace_bytes, void* stream);

/* Sizes in bytes of the five state buffers of a rows x cols tensor, in the order
 * {m_codes, m_blockscale, v_codes, v_rowmax, v_colmax}.  shape, sizes: host. */
int lpmm_adamw4_state_sizes(const int64_t shape[2], size_t sizes[5]);

/* Writes the zero state (m_0 = v_0 = 0 of Alg. 3) into the five buffers. */
int lpmm_adamw4_state_zero(uint8_t* m_codes, float* m_blockscale, uint8_t* v_codes,
                           float* v_rowmax, float* v_colmax, const int64_t shape[2], void* stream);

/* One 4-bit AdamW step on one tensor (Alg. 3 with Eq. 1 and decoupled decay):
 *   m~ = T_DE[m_code] * blockscale,  v~ = T_LIN[v_code] * min(r_i, c_j)          (decompress)
 *   m_t = beta1*m~ + (1-beta1)*g,    v_t = beta2*v~ + (1-beta2)*g^2              (Eq. 1)
 *   w  <- w - lr*( (m_t/(1-beta1^t)) / (sqrt(v_t/(1-beta2^t)) + eps) + weight_decay*w )
 *   m codes/scales <- B128/DE(m_t),  v codes, r, c <- rank-1/Linear(v_t)           (compress)
 * param: float[P], updated in place.  grad: float[P], read only.  The five state buffers are
 * updated in place.  param and grad must be 16-byte aligned, the others 4-byte aligned.
 * step is t >= 1.  Hyper-parameters: lr >= 0, 0 <= beta < 1, eps >= 0, weight_decay >= 0.
 * Two kernels are enqueued (the column maxima of v_t must be complete before any v code can be
 * written).  Needs lpmm_adamw4_init on the current device with rows + cols within the workspace. */
int lpmm_adamw4_step(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                     uint8_t* v_codes, float* v_rowmax, float* v_colmax, const int64_t shape[2],
                     float lr, float beta1, float beta2, float eps, float weight_decay,
                     int64_t step, void* stream);

/* Same step with a bf16 gradient buffer (uint16 bit patterns, upcast exactly in the kernel). */
int lpmm_adamw4_step_bf16g(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                           uint8_t* v_codes, float* v_rowmax, float* v_colmax,
                           const int64_t shape[2], float lr, float beta1, float beta2, float eps,
                           float weight_decay, int64_t step, void* stream);

/* The step of lpmm_adamw4_step / _step_bf16g (Alg. 3, Sec. 4.2) with a workspace of the caller's in place of the
 * one registered by lpmm_adamw4_init, so that steps on different tensors can run on different streams at the same
 * time: give every stream (or every tensor) its own workspace.  workspace: device memory, 256-byte aligned, at
 * least lpmm_adamw4_workspace_bytes(rows + cols) long, owned by the caller, zero-filled once before its first use
 * (hipMemset, or any fill); every completed step leaves it zero-filled again, so it can be passed to the next step
 * as it is.  Two calls that may overlap in time must not share a workspace.  lpmm_adamw4_init must have run on the
 * current device (for the tables), with any workspace.  Other arguments, state layout, alignment and results as
 * lpmm_adamw4_step; grad_dtype is LPMM_GRAD_F32 or LPMM_GRAD_BF16.  Errors: LPMM_EINVAL (null or misaligned
 * workspace, fewer than 8 KiB + 1 KiB), LPMM_EWORKSPACE (too small for this shape); nothing is enqueued then. */
int lpmm_adamw4_step_ws(void* param, const void* grad, int grad_dtype, uint8_t* m_codes, float* m_blockscale,
                        uint8_t* v_codes, float* v_rowmax, float* v_colmax, const int64_t shape[2], float lr,
                        float beta1, float beta2, float eps, float weight_decay, int64_t step, void* workspace,
                        size_t workspace_bytes, void* stream);

/* The step of lpmm_adamw4_step / _step_bf16g for callers that cannot allocate device memory and do not want to
 * size a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * row / column maxima of the updated second moment and the completion counters live in a device array that
 * is part of the library itself (LPMM_NOALLOC_MAX_ROWS_PLUS_COLS + 128 floats + 8 KiB, held by every GPU the
 * library is loaded on until the process ends) instead of the workspace given to lpmm_adamw4_init; init must
 * still have run on the current device (it looks up the array's address there and uploads the tables), with
 * any workspace.  Arguments, state layout, alignment and results as lpmm_adamw4_step; grad_dtype is
 * LPMM_GRAD_F32 or LPMM_GRAD_BF16.  Limit: round_up(rows, 64) + round_up(cols, 64) <=
 * LPMM_NOALLOC_MAX_ROWS_PLUS_COLS + 128, else LPMM_EWORKSPACE and nothing is enqueued.  Enqueues three kernels
 * (one clears the part of the array this call uses), calls no allocating routine, no memset, no
 * synchronization.  All calls on one GPU share the one array: calls that may overlap in time on one GPU
 * (different streams) race; calls on one stream are safe. */
#define LPMM_NOALLOC_MAX_ROWS_PLUS_COLS 131072
int lpmm_adamw4_step_noalloc(void* param, const void* grad, int grad_dtype, uint8_t* m_codes,
                             float* m_blockscale, uint8_t* v_codes, float* v_rowmax, float* v_colmax,
                             const int64_t shape[2], float lr, float beta1, float beta2, float eps,
                             float weight_decay, int64_t step, void* stream);

/* ---- block-wise second moment: 1-dimensional and flattened tensors ---------------------------------
 * Rank-1 normalization needs a 2-dimensional shape; for a 1-dimensional tensor it degenerates and the
 * paper uses block-wise normalization with block size 128 for the second moment as well (Sec. 4.2,
 * last paragraph), keeping the Linear map of Sec. 4.1.  The same holds when a framework hands the
 * optimizer flattened parameters (App. C.1: the LLaMA runs under FSDP).  State of such a tensor of
 * `numel` elements:
 *   m_codes, m_blockscale   as above
 *   v_codes      uint8[(numel+1)/2]        code q stands for (q+1)/16
 *   v_blockscale float[ceil(numel/128)]    maximum of block k = elements [128k, 128k+127]
 * zero state: m codes 7, v codes 0, all scales 0.  Everything is local to a block, so the step is
 * ONE kernel that touches every byte once (no workspace; lpmm_adamw4_init must still have run on the
 * current device: the lookup tables live there).  param, grad 16-byte aligned, the rest 4-byte. */

/* sizes[4] (host, out): bytes of m_codes, m_blockscale, v_codes, v_blockscale. */
int lpmm_adamw4_b128_state_sizes(int64_t numel, size_t sizes[4]);

/* Writes the zero state on `stream`. */
int lpmm_adamw4_b128_state_zero(uint8_t* m_codes, float* m_blockscale, uint8_t* v_codes,
                                float* v_blockscale, int64_t numel, void* stream);

/* One AdamW step (App. E Alg. 3 with the block-wise second moment), in place on param and the four
 * state buffers; grad (float[numel]) is read only.  Hyper-parameters and `step` as lpmm_adamw4_step. */
int lpmm_adamw4_b128_step(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                          uint8_t* v_codes, float* v_blockscale, int64_t numel, float lr, float beta1,
                          float beta2, float eps, float weight_decay, int64_t step, void* stream);

/* Same step with a bf16 gradient buffer. */
int lpmm_adamw4_b128_step_bf16g(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                                uint8_t* v_codes, float* v_blockscale, int64_t numel, float lr,
                                float beta1, float beta2, float eps, float weight_decay, int64_t step,
                                void* stream);

/* ---- factorized second moment ("4-bit Factor") ------------------------------------------------------
 * Sec. 4.3 and Sec. 5: for tensors with two dimensions the second moment is not stored per element
 * but factorized as in the cited Adafactor method: one statistic per row and one per column; the
 * first moment stays B128 / dynamic-exponent, the optimizer stays the AdamW of Eq. 1.  The paper
 * gives no formulas for this variant; the reading implemented here:
 *   R_t[i] = beta2 R_{t-1}[i] + (1-beta2) sum_j g_ij^2      C_t[j] = beta2 C_{t-1}[j] + (1-beta2) sum_i g_ij^2
 *   v_t[i][j] = R_t[i] C_t[j] / sum_i R_t[i]   (0 where that sum is 0)   in place of Eq. 1's v_t,
 * with Eq. 1's bias corrections and eps, and none of the cited method's own extras (update clipping,
 * relative step size, decay-rate schedule, the constant added to g^2).  State of a rows x cols tensor:
 *   m_codes, m_blockscale   as above
 *   v_row  float[rows]      R            v_col  float[cols]      C          zero state: all 0
 * (1-dimensional second moments are quantized instead: lpmm_adamw4_b128_step.)  Two kernels are
 * enqueued: one reads the gradient and accumulates the sums (fp32 atomics: R, C and the parameters
 * may differ in their last bits from run to run; the first moment does not; in a plan, LPMM_FLAG_DETERMINISTIC
 * selects sums in a fixed order instead), one updates.  Needs
 * lpmm_adamw4_init on the current device with rows + cols within the workspace.  param, grad 16-byte
 * aligned, the rest 4-byte. */

/* sizes[4] (host, out): bytes of m_codes, m_blockscale, v_row, v_col. */
int lpmm_adamw4_factor_state_sizes(const int64_t shape[2], size_t sizes[4]);

/* Writes the zero state on `stream`. */
int lpmm_adamw4_factor_state_zero(uint8_t* m_codes, float* m_blockscale, float* v_row, float* v_col,
                                  const int64_t shape[2], void* stream);

/* One step, in place on param and the four state buffers; grad (float[rows*cols]) is read only.
 * Hyper-parameters and `step` as lpmm_adamw4_step. */
int lpmm_adamw4_factor_step(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                            float* v_row, float* v_col, const int64_t shape[2], float lr, float beta1,
                            float beta2, float eps, float weight_decay, int64_t step, void* stream);

/* Same step with a bf16 gradient buffer. */
int lpmm_adamw4_factor_step_bf16g(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                                  float* v_row, float* v_col, const int64_t shape[2], float lr,
                                  float beta1, float beta2, float eps, float weight_decay, int64_t step,
                                  void* stream);

/* ---- rank-1 normalization for tensors with more than two dimensions ------------------------------------
 * App. F Alg. 4: a tensor of shape d_1 x ... x d_p keeps one statistic per index of every dimension
 * (the maximum of the second moment over all other indices); an element's scale is the minimum of
 * its p statistics.  The kernels see the tensor as a matrix of d_1 rows and d_2 * ... * d_p columns.
 * State (2 <= ndim <= 8, row-major, last index fastest):
 *   m_codes, m_blockscale, v_codes   as for lpmm_adamw4_step, with rows*cols = d_1 * ... * d_p
 *   v_row  float[d_1]                         statistics of dimension 1
 *   v_col  float[cols + d_2 + ... + d_p]      first the cols = d_2*...*d_p column scales (for each column the
 *                                             minimum of the other dimensions' statistics at its index; derived,
 *                                             kept so that the step need not rebuild them), then the statistics
 *                                             of dimensions 2..p one after the other
 * zero state: m codes 7, everything else 0.  (v_codes, v_row, v_col) decompress with
 * lpmm_dequant_state(which = 1, shape = {d_1, cols}).  With ndim = 2 the results equal lpmm_adamw4_step's.
 * Four kernels are enqueued (the two passes, and two small ones between them that turn column maxima into
 * the new statistics and column scales).  Needs lpmm_adamw4_init with d_1 + cols + d_2 + ... + d_p (+ 128)
 * floats of workspace, i.e. that number passed as max_rows_plus_cols.  Alignment as lpmm_adamw4_step. */

/* sizes[5] (host, out): bytes of m_codes, m_blockscale, v_codes, v_row, v_col. */
int lpmm_adamw4_nd_state_sizes(const int64_t* dims, int ndim, size_t sizes[5]);

/* Writes the zero state on `stream`. */
int lpmm_adamw4_nd_state_zero(uint8_t* m_codes, float* m_blockscale, uint8_t* v_codes, float* v_row,
                              float* v_col, const int64_t* dims, int ndim, void* stream);

/* One AdamW step (App. E Alg. 3), in place on param and the five state buffers; grad is read only.
 * dims: host array of ndim sizes.  Hyper-parameters and `step` as lpmm_adamw4_step. */
int lpmm_adamw4_nd_step(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                        uint8_t* v_codes, float* v_row, float* v_col, const int64_t* dims, int ndim,
                        float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step,
                        void* stream);

/* Same step with a bf16 gradient buffer. */
int lpmm_adamw4_nd_step_bf16g(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                              uint8_t* v_codes, float* v_row, float* v_col, const int64_t* dims, int ndim,
                              float lr, float beta1, float beta2, float eps, float weight_decay,
                              int64_t step, void* stream);

/* ---- SGD with momentum, 4-bit momentum -------------------------------------------------------------------
 * App. E Alg. 2: m_t = momentum * m_{t-1} + g, param -= lr * m_t (the precise m_t), m compressed like
 * Adam's first moment (block size 128, signed dynamic-exponent map).  No weight decay, no dampening, no
 * bias correction: the algorithm has none.  State of a tensor of `numel` elements (any shape, taken flat):
 *   m_codes uint8[(numel+1)/2], m_blockscale float[ceil(numel/128)]      zero state: codes 7, scales 0
 * One kernel, every byte touched once.  Needs lpmm_adamw4_init on the current device (lookup tables).
 * param, grad 16-byte aligned, the rest 4-byte. */

/* sizes[2] (host, out): bytes of m_codes, m_blockscale. */
int lpmm_sgdm4_state_sizes(int64_t numel, size_t sizes[2]);

/* Writes the zero state on `stream`. */
int lpmm_sgdm4_state_zero(uint8_t* m_codes, float* m_blockscale, int64_t numel, void* stream);

/* One step, in place on param and the two state buffers; grad (float[numel]) is read only.
 * lr >= 0 finite, 0 <= momentum < 1. */
int lpmm_sgdm4_step(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale, int64_t numel,
                    float lr, float momentum, void* stream);

/* Same step with a bf16 gradient buffer. */
int lpmm_sgdm4_step_bf16g(void* param, const void* grad, uint8_t* m_codes, float* m_blockscale,
                          int64_t numel, float lr, float momentum, void* stream);

/* The same rule with an uncompressed fp32 momentum buffer m[numel], for tensors that are not quantized. */
int lpmm_sgdm32_step(void* param, const void* grad, float* m, int64_t numel, int grad_dtype, float lr,
                     float momentum, void* stream);

/* AdamW step with uncompressed fp32 states, for tensors that are not quantized (App. C.1: size
 * <= 4096, biases and normalization vectors): Alg. 3 with compress = decompress = identity.
 * param, m, v: float[numel] in place; grad: float or bf16 [numel] per grad_dtype. */
int lpmm_adamw32_step(void* param, const void* grad, float* m, float* v, int64_t numel,
                      int grad_dtype, float lr, float beta1, float beta2, float eps,
                      float weight_decay, int64_t step, void* stream);

/* Decompress one moment to fp32 (the dequantizer N^-1 o T of Sec. 2.2).
 * which = 0: first moment, scale_a = m_blockscale, scale_b ignored (may be NULL).
 * which = 1: second moment, scale_a = v_rowmax, scale_b = v_colmax.
 * which = 2: block-wise second moment, scale_a = v_blockscale, scale_b ignored (may be NULL).
 * out: float[P]. */
int lpmm_dequant_state(int which, const uint8_t* codes, const float* scale_a, const float* scale_b,
                       const int64_t shape[2], float* out, void* stream);

/* Compress an fp32 moment into 4-bit state (the quantizer M o N of Sec. 2.2), same `which` and
 * scale arguments as lpmm_dequant_state, all outputs.  in: float[P]; for which = 1 and 2 the values
 * must be >= 0.  For which = 1 needs lpmm_adamw4_init (it uses no workspace but the tables). */
int lpmm_quant_state(int which, const float* in, const int64_t shape[2], uint8_t* codes,
                     float* scale_a, float* scale_b, void* stream);

/* ---- the quantizers the paper ablates for the second moment ---------------------------------------------
 * Sec. 4.1 and Tab. 1 compare, for the second moment: block-wise normalization with block size 2048 (the
 * 8-bit optimizer's) or 128, or rank-1 normalization; the 4-bit dynamic-exponent map of App. D.2 ("DE":
 * unsigned variant, 16 points with a zero), the same map with its zero removed ("DE-0", 15 points, the
 * smallest being 0.0033), or the Linear map; and rounding to the nearest entry or stochastic rounding
 * (App. D.3: between the two entries that enclose n, the upper one with probability (n - T(q1)) / (T(q2) -
 * T(q1))).  Tab. 1's first line also compresses the first moment with B2048 / signed DE.  These two calls
 * compress and decompress one tensor with any of those quantizers; they are not on an optimizer step's path.
 *   codes    uint8[(P+1)/2], packed like the states above; a code is the rank in the map (DE-0: 0..14)
 *   scale_a  float[ceil(P/128)] or float[ceil(P/2048)] block scales (absmax, blocks of the row-major
 *            flattening), or float[rows] row maxima for rank-1
 *   scale_b  float[cols] column maxima for rank-1, else ignored (may be NULL)
 * is_signed = 1 (signed input, scale = max |x|, signed DE map) exists for the block-wise normalizations with
 * LPMM_MAP_DE only; rank-1, DE-0 and Linear take non-negative input.  A zero scale gives n = 0.
 * Stochastic rounding draws the uniform number of element idx (its row-major index) from a counter-based
 * generator, so that results do not depend on the launch: u = (top 24 bits of SplitMix64's output number
 * idx + 1 for the initial state `seed`) * 2^-24; the upper entry is taken iff u < p, p evaluated in fp32
 * (two subtractions and one correctly rounded division).  in, codes, scales 4-byte aligned. */
#define LPMM_NORM_B128   0
#define LPMM_NORM_B2048  1
#define LPMM_NORM_RANK1  2
#define LPMM_MAP_DE      0
#define LPMM_MAP_DE0     1
#define LPMM_MAP_LINEAR  2
#define LPMM_ROUND_NEAREST    0
#define LPMM_ROUND_STOCHASTIC 1

/* The entries of one of these maps (host call, no GPU needed): out[0 .. n) increasing, the rest 0; returns n
 * (16, or 15 for DE-0), or LPMM_EINVAL for a combination that does not exist. */
int lpmm_ablation_table(int map, int is_signed, float out[16]);

int lpmm_quant_ablation(int norm, int map, int is_signed, int rounding, uint64_t seed, const float* in,
                        const int64_t shape[2], uint8_t* codes, float* scale_a, float* scale_b, void* stream);

int lpmm_dequant_ablation(int norm, int map, int is_signed, const uint8_t* codes, const float* scale_a,
                          const float* scale_b, const int64_t shape[2], float* out, void* stream);

/* ---- many tensors in one call ---------------------------------------------------------------------
 * The same step for a whole parameter set (Alg. 1: "perform the optimizer steps separately for each
 * layer" -- here all layers are enqueued by one call).  A plan is built once for a list of tensors;
 * lpmm_adamw4_step_multi then enqueues a short sequence of launches: pass 1 of one group of tensors
 * runs on `stream` while pass 2 of the previous group runs beside it on a second stream that the
 * plan owns (same priority; `stream` waits for it before the call's work counts as complete, so the
 * usual stream ordering holds for the caller).  Plans with a single group, plans of factorized tensors and
 * the one-pass kinds enqueue all their launches on `stream`.  Results are identical to calling the
 * single-tensor entry points one tensor at a time. */

#define LPMM_KIND_4BIT 0   /* quantized states as in lpmm_adamw4_step */
#define LPMM_KIND_FP32 1   /* uncompressed fp32 states as in lpmm_adamw32_step */
#define LPMM_KIND_4BIT_B128 2   /* quantized states, block-wise second moment, as in lpmm_adamw4_b128_step:
                                   v_rowmax points at v_blockscale, v_colmax is ignored, the tensor is the
                                   rows*cols elements taken flat */

#define LPMM_KIND_4BIT_FACTOR 3 /* quantized first moment, factorized second moment, as in lpmm_adamw4_factor_step:
                                   v_state is ignored (may be NULL), v_rowmax points at v_row, v_colmax at v_col.
                                   A plan holds LPMM_KIND_4BIT or LPMM_KIND_4BIT_FACTOR tensors, not both (they
                                   are two optimizers); either may be mixed with the other two kinds */

#define LPMM_KIND_SGDM_4BIT 4   /* SGD with momentum, 4-bit momentum, as in lpmm_sgdm4_step: m_state = m_codes,
                                   m_blockscale; the v_* members are ignored; the tensor is taken flat */
#define LPMM_KIND_SGDM_FP32 5   /* SGD with momentum, fp32 momentum, as in lpmm_sgdm32_step: m_state = float m[] */
                                /* SGDM kinds make a plan of their own, stepped by lpmm_sgdm4_step_multi */

#define LPMM_FLAG_NO_DECAY 1    /* this tensor takes no weight decay (biases and normalization weights are commonly
                                   excluded); lpmm_adamw4_step_multi then uses weight_decay = 0 for it */

#define LPMM_FLAG_DETERMINISTIC 2  /* LPMM_KIND_4BIT_FACTOR tensors with cols % 128 == 0 only: the row and column sums of
                                   g^2 (Sec. 4.3) are not accumulated with float atomics, whose order varies from run to
                                   run, but written per tile and added in a fixed order by two small extra kernels per
                                   tensor group: R, C and the parameters are then reproducible bit for bit.  Costs plan
                                   memory (about 0.05 bytes per parameter for the partial sums); other tensors with this
                                   flag make lpmm_adamw4_plan_build return LPMM_EINVAL */

#define LPMM_KIND_4BIT_ND 6     /* quantized states of a tensor with more than two dimensions, as in lpmm_adamw4_nd_step:
                                   rows = d_1, cols = d_2 * ... * d_p, v_rowmax points at v_row, v_colmax at v_col
                                   (cols + d_2 + ... + d_p floats); the sizes d_2 .. d_p come from the side tables of
                                   lpmm_adamw4_plan_bytes_nd / lpmm_adamw4_plan_build_nd.  Counts as LPMM_KIND_4BIT
                                   for the rule about mixing optimizers */

typedef struct lpmm_tensor_desc {
    void* param;            /* float[rows*cols], in place */
    const void* grad;       /* float or bf16 [rows*cols] (one type for the whole plan) */
    void* m_state;          /* 4BIT: uint8 m_codes;  FP32: float m[rows*cols] */
    float* m_blockscale;    /* 4BIT only */
    void* v_state;          /* 4BIT: uint8 v_codes;  FP32: float v[rows*cols] */
    float* v_rowmax;        /* 4BIT only */
    float* v_colmax;        /* 4BIT only */
    int64_t rows, cols;
    int32_t kind;           /* LPMM_KIND_* */
    int32_t flags;          /* LPMM_FLAG_* bits, 0 for none (plan_bytes reads them too) */
} lpmm_tensor_desc;

/* Bytes of device memory a plan for these tensors needs (descriptor tables, per-tensor row/column
 * maxima of the updated second moment, ticket counters).  descs: host array of n entries; only
 * rows, cols, kind and flags are read.  Returns 0 for invalid input. */
size_t lpmm_adamw4_plan_bytes(const lpmm_tensor_desc* descs, int64_t n);

/* Builds the plan into `plan` (device memory, 256-byte aligned, plan_bytes long, owned by the caller
 * and kept alive and unmodified while the plan is in use) on `stream`; the copy is complete when
 * work enqueued on `stream` before this call's return has finished.  Pointer alignment rules are
 * those of the single-tensor calls.  The plan refers to the tensors' buffers by address: rebuild it
 * if any of them moves.  A small host-side record is kept until lpmm_adamw4_plan_release(plan). */
int lpmm_adamw4_plan_build(const lpmm_tensor_desc* descs, int64_t n, int grad_dtype, void* plan,
                           size_t plan_bytes, void* stream);

/* The same two calls for lists that hold LPMM_KIND_4BIT_ND tensors.  inner_dims: host array of 7 sizes per tensor
 * (d_2 .. d_p, unused entries ignored), inner_ndim: host array with p - 1 per tensor, 0 for tensors of other kinds.
 * Two small kernels per tensor group are enqueued in addition (see lpmm_adamw4_nd_step). */
size_t lpmm_adamw4_plan_bytes_nd(const lpmm_tensor_desc* descs, int64_t n, const int64_t* inner_dims,
                                 const int32_t* inner_ndim);
int lpmm_adamw4_plan_build_nd(const lpmm_tensor_desc* descs, int64_t n, const int64_t* inner_dims,
                              const int32_t* inner_ndim, int grad_dtype, void* plan, size_t plan_bytes,
                              void* stream);

/* One step (same t, same hyper-parameters) for every tensor of the plan.  A plan holds its own
 * workspace, so plans (and single-tensor steps) may run concurrently on different streams as long
 * as they share no tensor; two steps of the same plan must not overlap. */
int lpmm_adamw4_step_multi(void* plan, float lr, float beta1, float beta2, float eps,
                           float weight_decay, int64_t step, void* stream);

/* One SGD-with-momentum step for every tensor of a plan built from LPMM_KIND_SGDM_* tensors only
 * (lpmm_adamw4_step_multi rejects such a plan, and this call rejects the others). */
int lpmm_sgdm4_step_multi(void* plan, float lr, float momentum, void* stream);

/* The same steps with the learning rate and the step number read from DEVICE memory when the kernels run (lr:
 * one float, step: one int64, values >= 1), for callers that capture the step into a HIP graph and replay it while
 * a schedule changes the rate and the step counts up: the bias corrections of Eq. 1 are evaluated on the device by
 * a one-thread kernel enqueued in front of the step's launches (into a slot inside the plan).  The other
 * hyper-parameters are captured by value.  Nothing is allocated, copied or synchronized.  The caller guarantees
 * lr >= 0 and step >= 1 (a smaller step is taken as 1); they cannot be checked here. */
int lpmm_adamw4_step_multi_capturable(void* plan, const float* lr, const int64_t* step, float beta1, float beta2,
                                      float eps, float weight_decay, void* stream);
int lpmm_sgdm4_step_multi_capturable(void* plan, const float* lr, float momentum, void* stream);

/* Forgets the host-side record of a plan (the device memory stays the caller's): lpmm_adamw4_plan_build keeps,
 * per plan, a host copy of the launch tables and, for plans with more than one tensor group, up to two HIP streams
 * (default priority, non-blocking) and a handful of events for the ordering between the two passes; they are
 * created by plan_build and destroyed here (or when the last step that is still enqueueing on another host thread
 * returns).  No device memory is allocated or freed by either call.  Work already enqueued is not waited for:
 * synchronize first if the plan's device memory is going to be reused. */
int lpmm_adamw4_plan_release(void* plan);

/* Per-kernel timing for benchmarks, with HIP events recorded on each call's own stream.
 * lpmm_profile_begin(max_calls): from now on every lpmm_adamw4_step / _step_bf16g call in this process
 * records an event before pass 1, between the two passes and after pass 2, and every
 * lpmm_adamw4_step_multi call an event before and after each of its launches, for at most max_calls
 * recorded launches pairs / launches (later ones run unrecorded).  Creates host-side event objects only.
 * lpmm_profile_end: waits for the recorded events and stops recording.  Single-tensor steps: ms[0]
 * = summed duration in milliseconds of the recorded pass-1 launches, ms[1] = of the pass-2 launches,
 * *n_calls = recorded calls.  Multi-tensor steps: ms[0] = summed duration of the recorded launches
 * that carry pass 1 (their pass-2 companions run beside them on the plan's second stream; in a plan of
 * factorized tensors: of the update passes), ms[1] = 0, *n_calls = recorded launches.  (Do not mix the two kinds between one begin and end.)
 * ms, n_calls: host.  Not thread-safe: begin, end and every step between them must come from one host thread. */
int lpmm_profile_begin(int64_t max_calls);
int lpmm_profile_end(double ms[2], int64_t* n_calls);

#ifdef __cplusplus
}
#endif
#endif /* LPMM4_H */
