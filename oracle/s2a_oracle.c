/*
 * s2a_oracle.c -- CPU oracle for the 4-bit GELU activation step of S2A.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, scalar, double-precision
 * statement of what the activation path computes.  It exists so that tests,
 * the smoke check and the cpu_baseline leg of the benchmark have something
 * obviously correct to compare the GPU library against.  Product code never
 * links, imports or calls it, and it shares no code, header, table or
 * constant generator with the HIP sources.
 *
 * What it follows (S2A paper, Sec. 3.2 "Non-Parametric Layers"):
 *   - the general scheme of Fig. 3: forward computes y from the full-precision
 *     x and saves only a low-bit activation; backward dequantizes it, forms
 *     dy/dx and multiplies by dL/dy;
 *   - "GeLU layer" paragraph: Eq. 10 (forward), Eq. 11 (exact derivative, used
 *     here for cross-checks only), Eq. 12 (sine-fitted derivative used in the
 *     backward pass), the clip of x to [-2, 2], and the statement that x is
 *     quantized as in Eq. 8 and dequantized by Eq. 9 with N = 4 bits.
 *
 * Readings taken where the paper is silent (each is listed in the design
 * notes of the repository):
 *   - Eq. 8's min/max are the clip limits -2 and 2 (fixed, not measured from
 *     the tensor): after the clip they are the extremes of any tensor that has
 *     one element beyond each limit, and the activation interface carries no
 *     per-tensor scale.
 *   - The rounding function of Eq. 8 is round-half-to-even.
 *   - NaN clips like C's fmax/fmin (the non-NaN operand wins), so NaN -> code 0.
 *   - Two codes per byte, element 2j in bits 0..3 and element 2j+1 in bits
 *     4..7 of byte j; an odd n leaves the last high nibble 0.  The paper only
 *     says a code needs N bits; the packing order is this build's.
 *
 * Parity pins (tests/test_oracle_pins.py), none of which re-type a formula
 * below: Eq. 10 against a library logistic function and the identity
 * y(x) - y(-x) = x; Eq. 11 against automatic differentiation of Eq. 10;
 * Eq. 12 at the points where the sine term is 0 or +-0.22 and the odd
 * symmetry D(x) + D(-x) = 1; the quantizer against exact rational arithmetic
 * over every bf16 bit pattern plus its invariants (monotone, 16 levels,
 * representatives reproduce themselves, mirror symmetry); packing against a
 * little-endian bit stream.  No function here is "parity unpinned".
 *
 * Everything is IEEE double unless a storage type is named.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* Quantizer constants: N = 4 bits (GeLU paragraph), range = the clip limits. */
#define ORACLE_NBITS 4
#define ORACLE_XMIN (-2.0)
#define ORACLE_XMAX (2.0)

static double logistic(double z) { return 1.0 / (1.0 + exp(-z)); }

/* Eq. 10: y = x * sigma(1.702 x). */
double s2a_oracle_gelu(double x) { return x * logistic(1.702 * x); }

/* Eq. 11: sigma(1.702x) + 1.702 x e^{-1.702x} sigma^2(1.702x). Cross-check only. */
double s2a_oracle_gelu_deriv_exact(double x)
{
    double z = 1.702 * x;
    double s = logistic(z);
    return s + z * exp(-z) * s * s;
}

/* Eq. 12: sigma(1.702x) + 0.22 sin(1.5x). */
double s2a_oracle_gelu_deriv_approx(double x)
{
    return logistic(1.702 * x) + 0.22 * sin(1.5 * x);
}

/* Scale of Eq. 8 with max = 2, min = -2, N = 4. */
static double quant_scale(void)
{
    return (ORACLE_XMAX - ORACLE_XMIN) / (double)((1 << ORACLE_NBITS) - 1);
}

/* Clip to [-2, 2] (GeLU paragraph), then Eq. 8 applied to x. */
int s2a_oracle_quantize(double x)
{
    double xc = fmin(fmax(x, ORACLE_XMIN), ORACLE_XMAX);
    double q = nearbyint((xc - ORACLE_XMIN) / quant_scale()); /* half-to-even */
    return (int)q;
}

/* Eq. 9 applied to x_q. */
double s2a_oracle_dequantize(int q) { return (double)q * quant_scale() + ORACLE_XMIN; }

/*
 * The 16 representatives xhat_k (Eq. 9), the derivative the backward pass
 * uses for each (Eq. 12 at xhat_k), and the 15 decision points between
 * neighbouring representatives.
 */
void s2a_oracle_table(double xhat[16], double deriv[16], double bounds[15])
{
    for (int k = 0; k < 16; ++k) {
        xhat[k] = s2a_oracle_dequantize(k);
        deriv[k] = s2a_oracle_gelu_deriv_approx(xhat[k]);
    }
    for (int j = 0; j < 15; ++j)
        bounds[j] = ORACLE_XMIN + ((double)j + 0.5) * quant_scale();
}

/* Storage element i -> the exact double it denotes. */
static double load_elem(const void *p, int dtype, int64_t i)
{
    if (dtype == ORACLE_F32) {
        float f;
        memcpy(&f, (const char *)p + 4 * i, 4);
        return (double)f;
    }
    uint16_t h;
    memcpy(&h, (const char *)p + 2 * i, 2);
    uint32_t w = (uint32_t)h << 16; /* bf16 is the top half of an fp32 */
    float f;
    memcpy(&f, &w, 4);
    return (double)f;
}

/* Distance from x to the nearest of the 15 decision points. */
static double boundary_distance(double x)
{
    double best = INFINITY;
    for (int j = 0; j < 15; ++j) {
        double b = ORACLE_XMIN + ((double)j + 0.5) * quant_scale();
        double d = fabs(x - b);
        if (d < best) best = d;
    }
    return best;
}

/*
 * Forward pass over n elements of x (storage type `dtype`).
 *   y      [n]          Eq. 10 of each element, double           (may be NULL)
 *   code   [n]          unpacked 4-bit codes, one per byte       (may be NULL)
 *   packed [(n+1)/2]    two codes per byte, low nibble first     (may be NULL)
 *   near   [n]          1 where x lies within `band` of a decision point of
 *                       the quantizer, else 0                    (may be NULL)
 * Returns 0, or -1 for a bad dtype / negative n.
 */
int s2a_oracle_fwd(const void *x, int dtype, int64_t n, double *y, uint8_t *code,
                   uint8_t *packed, uint8_t *near, double band)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || n < 0) return -1;
    if (packed) memset(packed, 0, (size_t)((n + 1) / 2));
    for (int64_t i = 0; i < n; ++i) {
        double xi = load_elem(x, dtype, i);
        int q = s2a_oracle_quantize(xi);
        if (y) y[i] = s2a_oracle_gelu(xi);
        if (code) code[i] = (uint8_t)q;
        if (packed) packed[i / 2] |= (uint8_t)(q << (4 * (i & 1)));
        if (near) near[i] = (uint8_t)(boundary_distance(xi) <= band);
    }
    return 0;
}

/*
 * Backward pass: dx[i] = dy[i] * Eq.12(Eq.9(code[i])) with the codes read
 * from the packed bytes (low nibble = even element).
 */
int s2a_oracle_bwd(const void *dy, int dtype, const uint8_t *packed, int64_t n, double *dx)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || n < 0) return -1;
    for (int64_t i = 0; i < n; ++i) {
        int q = (packed[i / 2] >> (4 * (i & 1))) & 0xF;
        double xhat = s2a_oracle_dequantize(q);
        dx[i] = load_elem(dy, dtype, i) * s2a_oracle_gelu_deriv_approx(xhat);
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Data-dependent range (GeLU paragraph read literally): Eq. 8's min and max are
 * measured on the clipped tensor instead of being the clip limits.  One (min, scale) pair per tensor,
 * stored beside the codes, as Eq. 9 needs both in the backward pass.
 *
 * Readings: the extremes are taken over the whole tensor (the paper names no
 * granularity); NaN clips to -2 as above and therefore takes part in the
 * minimum; a tensor whose clipped values are all equal has scale 0 and every
 * code 0, so Eq. 9 returns that value exactly.
 *
 * Pins (tests/test_oracle_dyn_pins.py): equality with the fixed-range oracle
 * whenever the tensor reaches both clip limits; exact rational arithmetic on
 * small tensors; shift invariance of the codes; extremes map to codes 0 and
 * 15; reconstruction within half a step; the degenerate tensor.
 * ---------------------------------------------------------------------- */

static double clip_x(double x) { return fmin(fmax(x, ORACLE_XMIN), ORACLE_XMAX); }

/* min and scale of Eq. 8 for this tensor; returns 0, or -1 on bad arguments. */
int s2a_oracle_range(const void *x, int dtype, int64_t n, double *qmin, double *qscale)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || n < 0) return -1;
    double lo = INFINITY, hi = -INFINITY;
    for (int64_t i = 0; i < n; ++i) {
        double xc = clip_x(load_elem(x, dtype, i));
        if (xc < lo) lo = xc;
        if (xc > hi) hi = xc;
    }
    if (n == 0) { lo = 0.0; hi = 0.0; }
    *qmin = lo;
    *qscale = (hi - lo) / (double)((1 << ORACLE_NBITS) - 1);
    return 0;
}

/* Eq. 8 with a given (min, scale). */
int s2a_oracle_quantize_dyn(double x, double qmin, double qscale)
{
    if (!(qscale > 0.0)) return 0;
    double q = nearbyint((clip_x(x) - qmin) / qscale);
    /* a value outside the range the scale was measured on still gets a valid code */
    if (q < 0.0) q = 0.0;
    if (q > 15.0) q = 15.0;
    return (int)q;
}

/* Eq. 9 with a given (min, scale). */
double s2a_oracle_dequantize_dyn(int q, double qmin, double qscale) { return (double)q * qscale + qmin; }

/*
 * Forward pass with the measured range.  Outputs as in s2a_oracle_fwd, plus
 * the (min, scale) pair.  `near` flags inputs within `band` of a decision
 * point qmin + (j + 1/2) * qscale.
 */
int s2a_oracle_fwd_dyn(const void *x, int dtype, int64_t n, double *y, uint8_t *code,
                       uint8_t *packed, double *qmin, double *qscale, uint8_t *near, double band)
{
    if (s2a_oracle_range(x, dtype, n, qmin, qscale) != 0) return -1;
    if (packed) memset(packed, 0, (size_t)((n + 1) / 2));
    for (int64_t i = 0; i < n; ++i) {
        double xi = load_elem(x, dtype, i);
        int q = s2a_oracle_quantize_dyn(xi, *qmin, *qscale);
        if (y) y[i] = s2a_oracle_gelu(xi);
        if (code) code[i] = (uint8_t)q;
        if (packed) packed[i / 2] |= (uint8_t)(q << (4 * (i & 1)));
        if (near) {
            double best = INFINITY;
            for (int j = 0; j < 15; ++j) {
                double d = fabs(clip_x(xi) - (*qmin + ((double)j + 0.5) * *qscale));
                if (d < best) best = d;
            }
            near[i] = (uint8_t)(best <= band);
        }
    }
    return 0;
}

/* Backward pass: Eq. 9 with the stored (min, scale), then Eq. 12, then the product. */
int s2a_oracle_bwd_dyn(const void *dy, int dtype, const uint8_t *packed, int64_t n, double qmin,
                       double qscale, double *dx)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || n < 0) return -1;
    for (int64_t i = 0; i < n; ++i) {
        int q = (packed[i / 2] >> (4 * (i & 1))) & 0xF;
        double xhat = s2a_oracle_dequantize_dyn(q, qmin, qscale);
        dx[i] = load_elem(dy, dtype, i) * s2a_oracle_gelu_deriv_approx(xhat);
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * ReLU layer (Sec. 3.2, "ReLU layer" paragraph): the derivative takes the two
 * values 0 and 1, so the saved activation is the 1-bit mask "x > 0".
 *
 * Readings: the mask is strict (x = 0 has derivative 0, as in PyTorch); y is
 * x where the mask is set and +0 elsewhere (NaN has no order, so NaN -> 0);
 * eight mask bits per byte, element 8j+b in bit b of byte j, pad bits 0.
 *
 * Pins (tests/test_oracle_relu_pins.py): y against a library ReLU, the mask
 * against numpy's little-endian bit packing of (x > 0), the backward pass
 * against automatic differentiation of a library ReLU, the 32x size ratio.
 * ---------------------------------------------------------------------- */
int s2a_oracle_relu_fwd(const void *x, int dtype, int64_t n, double *y, uint8_t *bit,
                        uint8_t *packed)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || n < 0) return -1;
    if (packed) memset(packed, 0, (size_t)((n + 7) / 8));
    for (int64_t i = 0; i < n; ++i) {
        double xi = load_elem(x, dtype, i);
        int m = xi > 0.0;
        if (y) y[i] = m ? xi : 0.0;
        if (bit) bit[i] = (uint8_t)m;
        if (packed) packed[i / 8] |= (uint8_t)(m << (i & 7));
    }
    return 0;
}

int s2a_oracle_relu_bwd(const void *dy, int dtype, const uint8_t *packed, int64_t n, double *dx)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || n < 0) return -1;
    for (int64_t i = 0; i < n; ++i) {
        int m = (packed[i / 8] >> (i & 7)) & 1;
        dx[i] = m ? load_elem(dy, dtype, i) : 0.0;
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Softmax layer (Sec. 3.2, "Softmax layer" paragraph, Eq. 7-9).  The gradient
 * of softmax needs only y, and y lies in (0, 1) with sum 1, so y is what gets
 * quantized: asymmetric N-bit quantization between its minimum and maximum
 * (Eq. 8), dequantized by Eq. 9 before the gradient of Eq. 7 is formed.
 *
 * Layout: `rows` vectors of length L, contiguous (row stride L).  Codes are
 * packed two per byte within a row, each row starting on a byte:
 * ceil(L/2) bytes per row, element 2j in the low nibble, odd L leaves the last
 * high nibble 0.  One (min, scale) pair per row.
 *
 * Readings: N = 4 as for GELU (Sec. 4.3 quantizes both to 4 bits); min and max
 * are taken per softmax vector (Eq. 8 is written for the vector y); a row
 * whose y are all equal has scale 0 and codes 0; the exponentials are taken
 * relative to the row maximum, which is Eq. 7 in exact arithmetic and avoids
 * overflow (so -inf inputs give y = 0); rounding is half-to-even.
 *
 * Pins (tests/test_oracle_softmax_pins.py): a library softmax; the literal
 * quotient of Eq. 7; sum 1 and shift invariance; exact rational arithmetic for
 * the codes; automatic differentiation of a library softmax on rows whose y sit
 * exactly on the 16 levels; the closed forms for constant rows and for L = 2.
 * ---------------------------------------------------------------------- */
int s2a_oracle_softmax_fwd(const void *x, int dtype, int64_t rows, int64_t L, double *y,
                           uint8_t *code, uint8_t *packed, double *qmin, double *qscale,
                           uint8_t *near, double band_t)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || rows < 0 || L < 1) return -1;
    const int64_t rb = (L + 1) / 2;
    const double levels = (double)((1 << ORACLE_NBITS) - 1);
    if (packed) memset(packed, 0, (size_t)(rows * rb));
    for (int64_t r = 0; r < rows; ++r) {
        double m = -INFINITY, sum = 0.0;
        for (int64_t i = 0; i < L; ++i) m = fmax(m, load_elem(x, dtype, r * L + i));
        for (int64_t i = 0; i < L; ++i) sum += exp(load_elem(x, dtype, r * L + i) - m);
        double lo = INFINITY, hi = -INFINITY;
        for (int64_t i = 0; i < L; ++i) {                       /* Eq. 7 */
            double yi = exp(load_elem(x, dtype, r * L + i) - m) / sum;
            y[r * L + i] = yi;
            lo = fmin(lo, yi);
            hi = fmax(hi, yi);
        }
        double s = (hi - lo) / levels;                          /* Eq. 8 */
        if (qmin) qmin[r] = lo;
        if (qscale) qscale[r] = s;
        for (int64_t i = 0; i < L; ++i) {
            double t = s > 0.0 ? (y[r * L + i] - lo) / s : 0.0;
            int q = (int)nearbyint(t);
            if (code) code[r * L + i] = (uint8_t)q;
            if (packed) packed[r * rb + i / 2] |= (uint8_t)(q << (4 * (i & 1)));
            if (near) near[r * L + i] = (uint8_t)(fabs(t - floor(t) - 0.5) <= band_t);
        }
    }
    return 0;
}

/* Eq. 9, then the product of dL/dy with the Jacobian of Eq. 7 written with y-hat:
 * dx_i = yh_i * (dy_i - sum_j yh_j dy_j). */
int s2a_oracle_softmax_bwd(const void *dy, int dtype, const uint8_t *packed, const double *qmin,
                           const double *qscale, int64_t rows, int64_t L, double *dx)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || rows < 0 || L < 1) return -1;
    const int64_t rb = (L + 1) / 2;
    for (int64_t r = 0; r < rows; ++r) {
        double dot = 0.0;
        for (int64_t i = 0; i < L; ++i) {
            int q = (packed[r * rb + i / 2] >> (4 * (i & 1))) & 0xF;
            double yh = (double)q * qscale[r] + qmin[r];
            dot += yh * load_elem(dy, dtype, r * L + i);
        }
        for (int64_t i = 0; i < L; ++i) {
            int q = (packed[r * rb + i / 2] >> (4 * (i & 1))) & 0xF;
            double yh = (double)q * qscale[r] + qmin[r];
            dx[r * L + i] = yh * (load_elem(dy, dtype, r * L + i) - dot);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * SiLU / Swish (the last sentence of the GeLU paragraph names both as served by
 * the same design).  The paper gives no constants for them.  SiLU(x) = x sigma(x) is Eq. 10 under x -> x / 1.702
 * (SiLU(x) = 1.702 * GELU(x / 1.702)), so the derivative of SiLU at x is the
 * derivative of Eq. 10 at x / 1.702 and the paper's fit, range and bit width
 * carry over by that substitution: derivative sigma(x) + 0.22 sin(1.5 x/1.702),
 * clip to [-2*1.702, 2*1.702], 16 levels.  This reading is this build's.
 *
 * Pins (tests/test_oracle_silu_pins.py): a library SiLU and its automatic
 * differentiation; exact agreement with the GELU functions above under the
 * substitution.
 * ---------------------------------------------------------------------- */
#define ORACLE_SILU_CLIP (2.0 * 1.702)

double s2a_oracle_silu(double x) { return x * logistic(x); }

double s2a_oracle_silu_deriv_approx(double x) { return logistic(x) + 0.22 * sin(1.5 * x / 1.702); }

static double silu_scale(void) { return (2.0 * ORACLE_SILU_CLIP) / (double)((1 << ORACLE_NBITS) - 1); }

int s2a_oracle_silu_quantize(double x)
{
    double xc = fmin(fmax(x, -ORACLE_SILU_CLIP), ORACLE_SILU_CLIP);
    return (int)nearbyint((xc + ORACLE_SILU_CLIP) / silu_scale());
}

double s2a_oracle_silu_dequantize(int q) { return (double)q * silu_scale() - ORACLE_SILU_CLIP; }

int s2a_oracle_silu_fwd(const void *x, int dtype, int64_t n, double *y, uint8_t *code,
                        uint8_t *packed, uint8_t *near, double band)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || n < 0) return -1;
    if (packed) memset(packed, 0, (size_t)((n + 1) / 2));
    for (int64_t i = 0; i < n; ++i) {
        double xi = load_elem(x, dtype, i);
        int q = s2a_oracle_silu_quantize(xi);
        if (y) y[i] = s2a_oracle_silu(xi);
        if (code) code[i] = (uint8_t)q;
        if (packed) packed[i / 2] |= (uint8_t)(q << (4 * (i & 1)));
        if (near) {
            double best = INFINITY;
            for (int j = 0; j < 15; ++j) {
                double d = fabs(xi - (-ORACLE_SILU_CLIP + ((double)j + 0.5) * silu_scale()));
                if (d < best) best = d;
            }
            near[i] = (uint8_t)(best <= band);
        }
    }
    return 0;
}

int s2a_oracle_silu_bwd(const void *dy, int dtype, const uint8_t *packed, int64_t n, double *dx)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || n < 0) return -1;
    for (int64_t i = 0; i < n; ++i) {
        int q = (packed[i / 2] >> (4 * (i & 1))) & 0xF;
        dx[i] = load_elem(dy, dtype, i) * s2a_oracle_silu_deriv_approx(s2a_oracle_silu_dequantize(q));
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Channel Average Pooling (Sec. 3.1, "Lite Side Branch" paragraph, Eq. 5):
 * y_k = (1/r) sum_{j<r} x_{k r + j} along the channel axis, and
 * dL/dx_{k r + j} = dL/dy_k / r.  Channels are contiguous and C is a multiple
 * of r, so on the flat tensor output m averages inputs m*r .. m*r + r - 1.
 *
 * Pins (tests/test_oracle_cap_lrp_pins.py): a library average pooling and its
 * automatic differentiation; the adjoint identity <CAP x, g> = <x, CAP^T g>.
 * ---------------------------------------------------------------------- */
int s2a_oracle_cap_fwd(const void *x, int dtype, int64_t n_out, int r, double *y)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || n_out < 0 || r < 1) return -1;
    for (int64_t m = 0; m < n_out; ++m) {
        double acc = 0.0;
        for (int j = 0; j < r; ++j) acc += load_elem(x, dtype, m * r + j);
        y[m] = acc / (double)r;
    }
    return 0;
}

int s2a_oracle_cap_bwd(const void *dy, int dtype, int64_t n_out, int r, double *dx)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || n_out < 0 || r < 1) return -1;
    for (int64_t m = 0; m < n_out; ++m)
        for (int j = 0; j < r; ++j) dx[m * r + j] = load_elem(dy, dtype, m) / (double)r;
    return 0;
}

/* ------------------------------------------------------------------------
 * Low-Rank Prompt (Sec. 3.1, "Low-Rank Prompt (LRP)" paragraph, Eq. 3-4):
 * y = x + A B with A in R^{N x r}, B in R^{r x C}; dL/dx = dL/dy,
 * dL/dA = dL/dy B^T, dL/dB = A^T dL/dy.  x holds `batch` samples of N x C
 * (row-major), and the same prompt A B is added to each, so the parameter
 * gradients sum over the batch.  A and B are fp32 (they are trained
 * parameters); x, y, dy use the storage type.
 *
 * Pins: a library matmul for the forward pass and automatic differentiation
 * for the three gradients.
 * ---------------------------------------------------------------------- */
int s2a_oracle_lrp_fwd(const void *x, int dtype, const float *A, const float *B, int64_t batch,
                       int64_t N, int64_t C, int r, double *y)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || batch < 0 || N < 0 || C < 0 || r < 0) return -1;
    for (int64_t b = 0; b < batch; ++b)
        for (int64_t i = 0; i < N; ++i)
            for (int64_t c = 0; c < C; ++c) {
                double p = 0.0;
                for (int k = 0; k < r; ++k) p += (double)A[i * r + k] * (double)B[(int64_t)k * C + c];
                y[(b * N + i) * C + c] = load_elem(x, dtype, (b * N + i) * C + c) + p;
            }
    return 0;
}

/* dA [N x r], dB [r x C]; dL/dx = dL/dy needs no arithmetic. */
int s2a_oracle_lrp_bwd(const void *dy, int dtype, const float *A, const float *B, int64_t batch,
                       int64_t N, int64_t C, int r, double *dA, double *dB)
{
    if ((dtype != ORACLE_F32 && dtype != ORACLE_BF16) || batch < 0 || N < 0 || C < 0 || r < 0) return -1;
    for (int64_t i = 0; i < N * r; ++i) dA[i] = 0.0;
    for (int64_t i = 0; i < (int64_t)r * C; ++i) dB[i] = 0.0;
    for (int64_t b = 0; b < batch; ++b)
        for (int64_t i = 0; i < N; ++i)
            for (int64_t c = 0; c < C; ++c) {
                double g = load_elem(dy, dtype, (b * N + i) * C + c);
                for (int k = 0; k < r; ++k) {
                    dA[i * r + k] += g * (double)B[(int64_t)k * C + c];
                    dB[(int64_t)k * C + c] += (double)A[i * r + k] * g;
                }
            }
    return 0;
}
