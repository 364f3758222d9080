/*
 * s2a.h -- C ABI of the MI355X (gfx950) 4-bit GELU activation library.
 *
 * The library implements the non-parametric activation step of S2A
 * (Sec. 3.2 "Non-Parametric Layers", Fig. 3, and the "GeLU layer" paragraph,
 * Eq. 8-12): the forward pass evaluates the sigmoid-form GELU at full
 * precision and keeps only a 4-bit code of the clipped input; the backward
 * pass turns each code back into the derivative the paper fits for it and
 * multiplies by the incoming gradient.
 *
 * Conventions shared by every entry point
 *   - Returns an int: S2A_OK (0) or a negative S2A_ERR_* value.  Nothing
 *     throws, nothing blocks: kernels are enqueued on `stream` and the call
 *     returns.  A call that launches resets the calling thread's HIP last-error
 *     state first (as hipGetLastError does), so that S2A_ERR_LAUNCH reports this
 *     launch only: an error left there by the caller's own earlier runtime calls
 *     is dropped, not reported.  Argument errors are detected on the host before any device
 *     work, in the order NOT_INIT, DTYPE, SIZE, NULL, ALIGN.
 *   - x, y, dy, dx and codes are DEVICE pointers owned by the caller.  The
 *     library allocates no device memory and keeps no reference to them.
 *   - Tensors are flat and contiguous; only the element count n matters.
 *   - `dtype` is an s2a_dtype: the storage type of x/y/dy/dx.  Arithmetic is
 *     fp32 for both; results are rounded once (nearest-even) to the storage
 *     type.
 *   - `codes` holds ceil(n/2) bytes: element 2j in bits 0..3 and element 2j+1
 *     in bits 4..7 of byte j.  For odd n the last high nibble is written as 0.
 *   - `stream` is a hipStream_t passed as void*; NULL is the default stream.
 *   - Pointers need only element alignment.  16-byte aligned x/y/dy/dx with
 *     4-byte aligned codes take the vector kernels; anything else takes a
 *     slower element-wise kernel with identical results.
 *   - Exact aliasing y == x and dx == dy (in place) is allowed; any other
 *     overlap between an input and an output is undefined.
 */
#ifndef S2A_H
#define S2A_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { S2A_F32 = 0, S2A_BF16 = 1 } s2a_dtype;

enum {
    S2A_OK = 0,
    S2A_ERR_NULL = -1,     /* a required pointer is NULL while n > 0 */
    S2A_ERR_SIZE = -2,     /* n < 0 */
    S2A_ERR_DTYPE = -3,    /* dtype is not an s2a_dtype */
    S2A_ERR_LEVELS = -4,   /* s2a_qtable_init: levels != 16 */
    S2A_ERR_NOT_INIT = -5, /* s2a_qtable_init has not succeeded yet */
    S2A_ERR_LAUNCH = -6,   /* the HIP runtime refused the launch */
    S2A_ERR_ALIGN = -7     /* a buffer lacks the alignment its entry point requires */
};

/* Floats of device memory behind a `qstate` pointer (see s2a_act_fwd_dyn). */
#define S2A_QSTATE_FLOATS 544

/*
 * Quantization-table setup (GeLU paragraph: x is clipped to [-2, 2] and
 * quantized as in Eq. 8 with N = 4; backward dequantizes by Eq. 9 and applies
 * Eq. 12).  Because a code takes only 2^N values, Eq. 9 followed by Eq. 12 is
 * a 16-entry table: representatives xhat_k = -2 + k*4/15 and derivatives
 * D[k] = sigma(1.702 xhat_k) + 0.22 sin(1.5 xhat_k).  The table is computed on
 * the host in double precision, rounded once to fp32, and kept in process
 * memory; kernels receive it by value, so there is no per-device state.
 *
 *   levels  number of quantization levels 2^N.  Only 16 is supported (two
 *           codes per byte); anything else returns S2A_ERR_LEVELS and leaves
 *           the library state unchanged.
 *
 * Idempotent.  Must not race with s2a_act_fwd / s2a_act_bwd on other threads.
 */
int s2a_qtable_init(int levels);

/*
 * Read back the table built by s2a_qtable_init (HOST pointers, any may be
 * NULL): the 16 representatives (Eq. 9), the 16 derivatives (Eq. 12 at the
 * representatives) and the 15 decision points half-way between neighbouring
 * representatives.  Returns S2A_ERR_NOT_INIT before a successful init.
 */
int s2a_qtable_get(float xhat[16], float deriv[16], float bounds[15]);

/*
 * Forward pass (Fig. 3 forward; Eq. 10; clip + Eq. 8 applied to x):
 *   y[i]    = x[i] * sigma(1.702 x[i])
 *   code[i] = round_half_even((clip(x[i], -2, 2) + 2) * 15/4)   in 0..15
 * x is read once; y and the packed codes are the only outputs, and the codes
 * are all the backward pass needs.  NaN inputs give y = NaN and code 0;
 * +inf gives y = +inf, code 15; -inf gives y = NaN, code 0.
 *
 *   x      [in]  device, n elements of `dtype`
 *   y      [out] device, n elements of `dtype` (may equal x)
 *   codes  [out] device, ceil(n/2) bytes
 *   n      element count, >= 0; n == 0 returns S2A_OK without a launch
 */
int s2a_act_fwd(const void* x, void* y, uint8_t* codes, int64_t n, int dtype, void* stream);

/*
 * Backward pass (Fig. 3 backward; Eq. 9 then Eq. 12, then the chain rule):
 *   dx[i] = dy[i] * D[code[i]]
 *
 *   dy     [in]  device, n elements of `dtype`
 *   codes  [in]  device, ceil(n/2) bytes as written by s2a_act_fwd
 *   dx     [out] device, n elements of `dtype` (may equal dy)
 */
int s2a_act_bwd(const void* dy, const uint8_t* codes, void* dx, int64_t n, int dtype,
                void* stream);

/*
 * Measured-range variant (GeLU paragraph read literally: Eq. 8's minimum and
 * maximum are those of the clipped tensor rather than the clip limits; Eq. 9
 * then needs the same pair in the backward pass).  One (min, scale) pair per call, kept beside the codes:
 *
 *   lo = min clip(x), hi = max clip(x), scale = (hi - lo) / 15
 *   code[i] = round((clip(x[i]) - lo) / scale)          (all 0 when hi == lo)
 *   dx[i]   = dy[i] * (sigma(1.702 xh) + 0.22 sin(1.5 xh)),  xh = code[i]*scale + lo
 *
 *   qstate  device, S2A_QSTATE_FLOATS floats, 4-byte aligned, caller-owned.
 *           Forward overwrites it and needs no initialisation; backward only
 *           reads entries 16..31.  Contents: [2] = lo, [3] = scale, [16..31] =
 *           the 16 derivative levels; the other entries are working values of
 *           the kernels (binning constants, per-block minima and maxima).  NaN
 *           inputs clip to -2 and take part in the minimum.  n == 0 leaves
 *           lo = scale = 0.
 *
 * Forward enqueues two kernels on `stream` (per-block min/max; the forward
 * kernel proper, which reduces those to the range and leaves the levels in
 * qstate); both run for n == 0 as well.  x is read twice, except that a
 * wavefront of the first kernel stops reading once it has met a value at or
 * beyond each clip limit (min = -2 and max = 2 are then settled), so tensors
 * that exceed both limits throughout cost little more than the fixed-range
 * entry point.  No atomics are used, so the result does not depend on
 * scheduling.
 * Everything else is as for
 * s2a_act_fwd / s2a_act_bwd.  When the tensor has elements beyond both clip
 * limits the results equal the fixed-range entry points'.
 */
int s2a_act_fwd_dyn(const void* x, void* y, uint8_t* codes, float* qstate, int64_t n, int dtype,
                    void* stream);
int s2a_act_bwd_dyn(const void* dy, const uint8_t* codes, const float* qstate, void* dx, int64_t n,
                    int dtype, void* stream);

/*
 * SiLU / Swish with the same 4-bit scheme (GeLU paragraph, last sentence, names
 * both as covered by the design; the paper gives no constants for them).  SiLU(x) = x sigma(x) is the
 * paper's GELU form x sigma(1.702 x) under x -> x / 1.702, so everything
 * transfers by that substitution:
 *   forward   y = x * sigma(x);  code = round((clip(x, -3.404, 3.404) + 3.404) * 15 / 6.808)
 *   backward  dx = dy * (sigma(xh) + 0.22 sin(1.5 xh / 1.702)),  xh = -3.404 + code * 6.808/15
 * Arguments, layout and errors as for s2a_act_fwd / s2a_act_bwd (fixed range
 * only); needs s2a_qtable_init.
 */
int s2a_silu_fwd(const void* x, void* y, uint8_t* codes, int64_t n, int dtype, void* stream);
int s2a_silu_bwd(const void* dy, const uint8_t* codes, void* dx, int64_t n, int dtype, void* stream);

/*
 * ReLU with a 1-bit saved activation (Sec. 3.2, "ReLU layer": the derivative
 * is 0 or 1, so the mask x > 0 is all the backward pass needs).
 *   forward   y[i] = x[i] > 0 ? x[i] : 0;  bit i of `mask` = x[i] > 0
 *   backward  dx[i] = bit i ? dy[i] : 0
 * `mask` holds ceil(n/8) bytes, element 8j+b in bit b of byte j, pad bits 0.
 * The mask is strict (x = 0 and NaN give bit 0 and y = 0).  Needs no
 * s2a_qtable_init.  x/y/dy/dx 16-byte aligned take the vector kernels; y == x
 * and dx == dy are allowed.
 */
int s2a_relu_fwd(const void* x, void* y, uint8_t* mask, int64_t n, int dtype, void* stream);
int s2a_relu_bwd(const void* dy, const uint8_t* mask, void* dx, int64_t n, int dtype, void* stream);

/*
 * Softmax with a 4-bit saved output (Sec. 3.2, "Softmax layer", Eq. 7-9): the
 * gradient of softmax needs only y, so y is quantized between its row minimum
 * and maximum (Eq. 8, N = 4) and dequantized (Eq. 9) before the gradient.
 *   forward   y = softmax(x) along rows of length L (Eq. 7)
 *             lo = min y, s = (max y - min y)/15, code = round((y - lo)/s)
 *   backward  yh = code*s + lo;  dx_i = yh_i * (dy_i - sum_j yh_j dy_j)
 *
 *   x, y, dy, dx  device, rows*L elements of `dtype`, row stride L (y may equal
 *                 x, dx may equal dy)
 *   codes         device, rows * ceil(L/2) bytes: every row starts on a byte,
 *                 element 2j in the low nibble; odd L leaves the last high
 *                 nibble 0
 *   qparams       device, 2*rows floats, 4-byte aligned: (lo, s) of row r at
 *                 [2r], [2r+1].  A row of equal y has s = 0 and codes 0.
 *   L             1 <= L <= S2A_SOFTMAX_MAX_L (else S2A_ERR_SIZE); rows >= 0.  Rows up to
 *                 1024 (every attention of the paper's models) take the tuned
 *                 kernels; longer rows take one block per row, untuned, with at
 *                 most 2^31 - 1 rows per call
 * Inputs of -inf (masked logits) give y = 0.  Needs no s2a_qtable_init.
 * x, y (dy, dx) and codes 16-byte aligned take the LDS-staged kernels; any other
 * alignment takes element-wise kernels with the same results.
 */
#define S2A_SOFTMAX_MAX_L (1 << 20)
int s2a_softmax_fwd(const void* x, void* y, uint8_t* codes, float* qparams, int64_t rows, int64_t L,
                    int dtype, void* stream);
int s2a_softmax_bwd(const void* dy, const uint8_t* codes, const float* qparams, void* dx,
                    int64_t rows, int64_t L, int dtype, void* stream);

/*
 * Channel Average Pooling (Sec. 3.1, "Lite Side Branch" paragraph, Eq. 5), the
 * parameter-free connector between the backbone and the side branch:
 *   forward   y[m] = (1/r) * sum_{j<r} x[m*r + j]
 *   backward  dx[m*r + j] = dy[m] / r
 * Channels are contiguous, so m runs over all (token, channel-group) pairs of
 * the flat tensor.  Nothing is saved for backward.
 *   x, dx   device, n_out * r elements of `dtype`
 *   y, dy   device, n_out elements of `dtype`
 *   r       compression factor, a power of two in 2..64 (else S2A_ERR_SIZE);
 *           the paper's experiments use 8
 * x (dx) 16-byte aligned takes the vector kernel.  Needs no s2a_qtable_init.
 */
int s2a_cap_fwd(const void* x, void* y, int64_t n_out, int r, int dtype, void* stream);
int s2a_cap_bwd(const void* dy, void* dx, int64_t n_out, int r, int dtype, void* stream);

/*
 * Low-Rank Prompt (Sec. 3.1, "Low-Rank Prompt (LRP)" paragraph, Eq. 3-4):
 *   forward   y[b] = x[b] + A B            for every sample b of the batch
 *   backward  dL/dx = dL/dy (alias it; nothing to compute),
 *             dA = sum_b dL/dy[b] B^T,  dB = sum_b A^T dL/dy[b]
 * Neither x nor y is needed in backward.
 *   x, y, dy  device, batch*N*C elements of `dtype` (sample-major, then token,
 *             then channel), 16-byte aligned (else S2A_ERR_ALIGN); y may equal x
 *   A, dA     device, fp32 [N x r] row-major;  B, dB  device, fp32 [r x C]
 *   work      device, N*C floats of scratch owned by the caller (holds the
 *             batch-summed gradient between the kernels of one call)
 *   r         1..128 (the paper uses 30 and scales it up to 100, Sec. 4.3); C a
 *             multiple of 8 (bf16) or 4 (fp32), else S2A_ERR_SIZE
 * Forward is one kernel; backward enqueues two (the batch sum of dL/dy into
 * `work`, then both products).  Needs no s2a_qtable_init.
 */
int s2a_lrp_fwd(const void* x, void* y, const float* A, const float* B, int64_t batch, int64_t N,
                int64_t C, int r, int dtype, void* stream);
int s2a_lrp_bwd(const void* dy, const float* A, const float* B, float* dA, float* dB, float* work,
                int64_t batch, int64_t N, int64_t C, int r, int dtype, void* stream);

/*
 * s2a_lrp_bwd for callers that cannot provide working memory because they cannot
 * allocate any: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and kernels as
 * s2a_lrp_bwd, without `work`: the N*C floats between the two kernels live in
 * a fixed array inside the library's device code (S2A_LRP_NOALLOC_MAX_FLOATS
 * floats = 4 MiB, held on every GPU the library runs on until the process
 * ends).  The call allocates nothing and calls no allocating routine; the first
 * call on a device only looks up the array's address on that device.
 *   - N*C > S2A_LRP_NOALLOC_MAX_FLOATS returns S2A_ERR_SIZE (use s2a_lrp_bwd).
 *   - All calls on one GPU share the array: calls that may overlap there (two
 *     streams, two threads) race on it and must be ordered by the caller.
 *     Nothing in it has to start at zero, and it keeps the last call's contents.
 *   - S2A_ERR_LAUNCH also reports that the array's address could not be found.
 */
#define S2A_LRP_NOALLOC_MAX_FLOATS (1 << 20)
int s2a_lrp_bwd_noalloc(const void* dy, const float* A, const float* B, float* dA, float* dB,
                        int64_t batch, int64_t N, int64_t C, int r, int dtype, void* stream);

/* Static, NUL-terminated description of a return code.  Never NULL. */
const char* s2a_strerror(int code);

#ifdef __cplusplus
}
#endif

#endif /* S2A_H */
