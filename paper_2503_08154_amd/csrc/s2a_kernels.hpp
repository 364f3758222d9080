// s2a_kernels.hpp -- gfx950 device code of the 4-bit GELU activation path.
//
// Two streaming kernels, each reading every input byte once and writing every
// output byte once (S2A Sec. 3.2, Fig. 3 and the "GeLU layer" paragraph):
//
//   forward   y = x * sigma(1.702 x)                      (Eq. 10)
//             code = bin of clip(x, -2, 2) among 16 uniform levels (Eq. 8, N = 4)
//             two codes per byte, element 2j in the low nibble
//   backward  dx = dy * D[code],  D[k] = Eq. 12 at the k-th representative (Eq. 9)
//
// The path is bound by HBM bandwidth (2e + 0.5 bytes per element and
// direction, e = element size), so the design is: one 128-bit load per lane
// and step, laid out so that a wavefront touches contiguous kilobytes; all
// packing done in registers; several independent loads in flight per lane;
// no LDS except the 64-byte derivative table of the backward pass.
//
// Work unit: a "vector" = 16 bytes of x (8 bf16 or 4 fp32).  Vector v owns
// elements [v*EPV, (v+1)*EPV) and code bytes [v*EPV/2, (v+1)*EPV/2), so no
// code byte is shared between lanes.  A block of S2A_BLOCK lanes handles
// UNROLL consecutive groups of S2A_BLOCK vectors.  Elements past the last
// full vector (fewer than EPV) are handled element-wise by one lane.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s2a {

constexpr int kBlock = 256;

struct QTable {
    float d[16];  // D[k], rounded once from double
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// 1.702 * log2(e) = 2.45546695959301560..., split so that kKhi + kKlo carries
// 48 bits of the product (the fp32 path needs more than one fp32 of it).
constexpr double kKd = 1.702 * 1.4426950408889634074;
constexpr float kKhi = (float)kKd;
constexpr float kKlo = (float)(kKd - (double)kKhi);
constexpr float kLn2 = 0.69314718055994530942f;

// ---------------------------------------------------------------- Eq. 10 ---

// sigma(1.702 x) * x for bf16 storage: the result is rounded to 8 significant
// bits afterwards, so one fp32 exponent argument is enough.  The exponential
// is carried with a 2^-32 bias: E = 2^-32 e^{-1.702x}, sigma = 2^-32 / (2^-32 + E).
// That keeps the quotient representable for x down to about -65, where y has
// already dropped below the smallest bf16 denormal, instead of overflowing at
// x = -52 where y is still a normal number.
__device__ __forceinline__ float gelu_fast(float x)
{
    float u = __builtin_fmaf(x, -kKhi, -32.0f);
    float e = __builtin_amdgcn_exp2f(u);             // v_exp_f32
    float r = __builtin_amdgcn_rcpf(e + 0x1p-32f);   // v_rcp_f32, = 2^32 sigma
    return x * (r * 0x1p-32f);
}

// The same function to a few fp32 ulps over the whole fp32 range.
//  - The exponent argument u = -K x is formed as an exact sum uh + ul (FMA
//    residual plus the low half of K); exp2(uh) is corrected by the factor
//    (1 + ln2 * ul).  Without this the rounding of u alone costs up to
//    ln2 * ulp(u)/2 = 2.6e-6 relative at |x| = 40.
//  - For uh > 64 (x < -26) the "1 +" of the denominator no longer registers in
//    fp32; the quotient is taken as x * 2^-(uh-64) * 2^-64 so that it neither
//    overflows nor loses bits before y itself goes denormal.
//  - |x| is capped at 128 for the exponent only (beyond that sigma is exactly
//    0 or 1 in fp32); the final product uses x itself, so +-inf and NaN behave
//    as the formula says: y(+inf) = +inf, y(-inf) = NaN, y(NaN) = NaN.
__device__ __forceinline__ float gelu_accurate(float x)
{
    float xs = __builtin_amdgcn_fmed3f(x, -128.0f, 128.0f);
    float uh = xs * -kKhi;
    float ul = __builtin_fmaf(xs, -kKhi, -uh);
    ul = __builtin_fmaf(xs, -kKlo, ul);
    bool big = uh > 64.0f;
    float e = __builtin_amdgcn_exp2f(uh - (big ? 64.0f : 0.0f));
    e = e * __builtin_fmaf(ul, kLn2, 1.0f);  // a product, so that e = +inf stays +inf
    float r = __builtin_amdgcn_rcpf(e + (big ? 0.0f : 1.0f));
    float y = (x * r) * (big ? 0x1p-64f : 1.0f);
    return (x <= 128.0f) ? y : x;  // x > 128 or NaN: sigma == 1, or propagate NaN
}

// ------------------------------------------------------- clip + Eq. 8 ------

// code = round((clip(x,-2,2) + 2) * 15/4).  Rounding to nearest equals
// floor(3.75 xc + 8) because the only exact tie of the real-valued expression
// is x = 0 (7.5 -> 8 under ties-to-even, and floor(8) = 8).  One FMA rounds the
// exact value once.  The clip is applied after the conversion instead of
// before it: v_cvt_u32_f32 truncates toward zero (the floor, for t >= 0) and
// saturates -- negative and NaN inputs give 0, huge ones 0xffffffff -- so
// min(c, 15) finishes the clip and NaN lands on code 0 like a value below the
// range.  The instruction is written out because a C float-to-unsigned cast
// leaves exactly those out-of-range cases undefined.
__device__ __forceinline__ uint32_t bin16(float x)
{
    float t = __builtin_fmaf(x, 3.75f, 8.0f);
    uint32_t c;
    asm("v_cvt_u32_f32 %0, %1" : "=v"(c) : "v"(t));
    return c < 15u ? c : 15u;
}

// Shift a 4-bit code into the top of `acc`; after 8 pushes the first code
// sits in bits 0..3.  (v_alignbit_b32: one op, no masking needed.)
__device__ __forceinline__ uint32_t push_nibble(uint32_t acc, uint32_t code)
{
    return __builtin_amdgcn_alignbit(code, acc, 4);
}

// ------------------------------------------------------------- storage ----

// Bit reinterpretation takes its argument BY VALUE: __builtin_bit_cast applied
// directly to an element of an ext_vector lvalue reads element 0 instead.
__device__ __forceinline__ float as_f32(uint32_t w) { return __builtin_bit_cast(float, w); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

__device__ __forceinline__ float bf16_lo(uint32_t w) { return as_f32(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return as_f32(w & 0xffff0000u); }

// Two fp32 -> two bf16, nearest-even (v_cvt_pk_bf16_f32); a in the low half.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    bf16x2 v = __builtin_convertvector((f32x2){a, b}, bf16x2);
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ float load_elem_f32(const void* p, int64_t i) { return ((const float*)p)[i]; }
__device__ __forceinline__ float load_elem_bf16(const void* p, int64_t i)
{
    return as_f32((uint32_t)((const uint16_t*)p)[i] << 16);
}
__device__ __forceinline__ void store_elem_f32(void* p, int64_t i, float v) { ((float*)p)[i] = v; }
__device__ __forceinline__ void store_elem_bf16(void* p, int64_t i, float v)
{
    ((uint16_t*)p)[i] = (uint16_t)pack_bf16(v, 0.0f);
}

template <bool BF16>
__device__ __forceinline__ float load_elem(const void* p, int64_t i)
{
    return BF16 ? load_elem_bf16(p, i) : load_elem_f32(p, i);
}
template <bool BF16>
__device__ __forceinline__ void store_elem(void* p, int64_t i, float v)
{
    if (BF16) store_elem_bf16(p, i, v); else store_elem_f32(p, i, v);
}
template <bool BF16>
__device__ __forceinline__ float gelu(float x) { return BF16 ? gelu_fast(x) : gelu_accurate(x); }

template <bool NT>
__device__ __forceinline__ u32x4 ldg128(const u32x4* p)
{
    return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT>
__device__ __forceinline__ void stg128(u32x4* p, u32x4 v)
{
    if (NT) __builtin_nontemporal_store(v, p); else *p = v;
}
template <bool NT, typename T>
__device__ __forceinline__ T ldg(const T* p)
{
    return NT ? __builtin_nontemporal_load(p) : *p;
}
template <bool NT, typename T>
__device__ __forceinline__ void stg(T* p, T v)
{
    if (NT) __builtin_nontemporal_store(v, p); else *p = v;
}

// ------------------------------------------------- element-wise pieces ----

// Elements [first, n) with first even: one code byte per pair, pad nibble 0.
template <bool BF16>
__device__ __forceinline__ void fwd_pairs(const void* x, void* y, uint8_t* codes, int64_t first,
                                          int64_t n, int64_t pair0, int64_t pair_stride)
{
    int64_t npairs = (n - first + 1) / 2;
    for (int64_t p = pair0; p < npairs; p += pair_stride) {
        int64_t i = first + 2 * p;
        float a = load_elem<BF16>(x, i);
        uint32_t byte = bin16(a);
        store_elem<BF16>(y, i, gelu<BF16>(a));
        if (i + 1 < n) {
            float b = load_elem<BF16>(x, i + 1);
            byte |= bin16(b) << 4;
            store_elem<BF16>(y, i + 1, gelu<BF16>(b));
        }
        codes[i / 2] = (uint8_t)byte;
    }
}

template <bool BF16>
__device__ __forceinline__ void bwd_pairs(const void* dy, const uint8_t* codes, void* dx,
                                          const float* tab, int64_t first, int64_t n,
                                          int64_t pair0, int64_t pair_stride)
{
    int64_t npairs = (n - first + 1) / 2;
    for (int64_t p = pair0; p < npairs; p += pair_stride) {
        int64_t i = first + 2 * p;
        uint32_t byte = codes[i / 2];
        store_elem<BF16>(dx, i, load_elem<BF16>(dy, i) * tab[byte & 15u]);
        if (i + 1 < n) store_elem<BF16>(dx, i + 1, load_elem<BF16>(dy, i + 1) * tab[byte >> 4]);
    }
}

// ------------------------------------------------------------- forward ----

// One vector of 8 bf16: y bits in place, returns the 8 packed codes.
template <bool BF16>
__device__ __forceinline__ uint32_t fwd_vector(u32x4& v)
{
    uint32_t acc = 0;
    if (BF16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = bf16_lo(v[j]), b = bf16_hi(v[j]);
            acc = push_nibble(acc, bin16(a));
            acc = push_nibble(acc, bin16(b));
            v[j] = pack_bf16(gelu_fast(a), gelu_fast(b));
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = as_f32(v[j]);
            acc = push_nibble(acc, bin16(a));
            v[j] = as_u32(gelu_accurate(a));
        }
        acc >>= 16;  // 4 codes -> low 16 bits
    }
    return acc;
}

// Vector kernel.  Requires x, y 16-byte aligned and codes 4-byte aligned.
// x and y may be the same buffer (every lane loads its vectors before it
// stores them), so neither is declared restrict.
//   nvec   number of full vectors, n / EPV
//   grid   ceil((nvec + (n % EPV != 0)) / (kBlock * UNROLL)) blocks
template <bool BF16, int UNROLL, bool NT>
__global__ __launch_bounds__(kBlock) void fwd_kernel(const u32x4* x, u32x4* y,
                                                     uint8_t* __restrict__ codes, int64_t n,
                                                     int64_t nvec)
{
    constexpr int EPV = BF16 ? 8 : 4;
    typedef typename std::conditional<BF16, uint32_t, uint16_t>::type code_t;
    const int64_t base = (int64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;
    code_t* cw = (code_t*)codes;

    if (base + (int64_t)(UNROLL - 1) * kBlock < nvec) {  // whole block strip in range: no per-load checks
        u32x4 v[UNROLL];
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) v[k] = ldg128<NT>(x + base + k * kBlock);
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) {
            uint32_t c = fwd_vector<BF16>(v[k]);
            stg128<NT>(y + base + k * kBlock, v[k]);
            stg<NT, code_t>(cw + base + k * kBlock, (code_t)c);
        }
        return;
    }
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        int64_t i = base + k * kBlock;
        if (i < nvec) {
            u32x4 v = x[i];
            uint32_t c = fwd_vector<BF16>(v);
            y[i] = v;
            cw[i] = (code_t)c;
        } else if (i == nvec) {  // one lane finishes the n % EPV leftover elements
            fwd_pairs<BF16>(x, y, codes, nvec * EPV, n, 0, 1);
        }
    }
}

// Any alignment: one lane per code byte, grid-stride.
template <bool BF16>
__global__ __launch_bounds__(kBlock) void fwd_kernel_unaligned(const void* x, void* y,
                                                               uint8_t* codes, int64_t n)
{
    fwd_pairs<BF16>(x, y, codes, 0, n, (int64_t)blockIdx.x * kBlock + threadIdx.x,
                    (int64_t)gridDim.x * kBlock);
}

// ------------------------------------------------------------ backward ----

template <bool BF16>
__device__ __forceinline__ void bwd_vector(u32x4& v, uint32_t c, const float* tab)
{
    if (BF16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = bf16_lo(v[j]) * tab[(c >> (8 * j)) & 15u];
            float b = bf16_hi(v[j]) * tab[(c >> (8 * j + 4)) & 15u];
            v[j] = pack_bf16(a, b);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = as_f32(v[j]) * tab[(c >> (4 * j)) & 15u];
            v[j] = as_u32(a);
        }
    }
}

template <bool BF16, int UNROLL, bool NT>
__global__ __launch_bounds__(kBlock) void bwd_kernel(const u32x4* dy,
                                                     const uint8_t* __restrict__ codes,
                                                     u32x4* dx, QTable qt, int64_t n,
                                                     int64_t nvec)
{
    constexpr int EPV = BF16 ? 8 : 4;
    typedef typename std::conditional<BF16, uint32_t, uint16_t>::type code_t;
    __shared__ float tab[16];
    if (threadIdx.x < 16) tab[threadIdx.x] = qt.d[threadIdx.x];
    __syncthreads();

    const int64_t base = (int64_t)blockIdx.x * (kBlock * UNROLL) + threadIdx.x;
    const code_t* cw = (const code_t*)codes;

    if (base + (int64_t)(UNROLL - 1) * kBlock < nvec) {
        u32x4 v[UNROLL];
        uint32_t c[UNROLL];
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) {
            v[k] = ldg128<NT>(dy + base + k * kBlock);
            c[k] = ldg<NT, code_t>(cw + base + k * kBlock);
        }
#pragma unroll
        for (int k = 0; k < UNROLL; ++k) {
            bwd_vector<BF16>(v[k], c[k], tab);
            stg128<NT>(dx + base + k * kBlock, v[k]);
        }
        return;
    }
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        int64_t i = base + k * kBlock;
        if (i < nvec) {
            u32x4 v = dy[i];
            bwd_vector<BF16>(v, cw[i], tab);
            dx[i] = v;
        } else if (i == nvec) {
            bwd_pairs<BF16>(dy, codes, dx, tab, nvec * EPV, n, 0, 1);
        }
    }
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void bwd_kernel_unaligned(const void* dy,
                                                               const uint8_t* codes, void* dx,
                                                               QTable qt, int64_t n)
{
    __shared__ float tab[16];
    if (threadIdx.x < 16) tab[threadIdx.x] = qt.d[threadIdx.x];
    __syncthreads();
    bwd_pairs<BF16>(dy, codes, dx, tab, 0, n, (int64_t)blockIdx.x * kBlock + threadIdx.x,
                    (int64_t)gridDim.x * kBlock);
}

}  // namespace s2a
