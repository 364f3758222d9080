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
// no LDS on the vector path (the 64-byte derivative table of the backward pass
// lives in one register per lane and is read with a cross-lane permute).
//
// Work unit: a "vector" = 16 bytes of x (8 bf16 or 4 fp32).  Vector v owns
// elements [v*EPV, (v+1)*EPV) and code bytes [v*EPV/2, (v+1)*EPV/2), so no
// code byte is shared between lanes.  A block is ONE wavefront of 64 lanes and
// every lane handles one vector: a wave reads 1 KiB of x, writes 1 KiB of y and
// 256 B (bf16) or 128 B (fp32) of codes, all contiguous.  Measured on MI355X,
// single-wave blocks with one load in flight per lane beat wider blocks and
// deeper unrolling by 1-10 %: with 8 waves per SIMD the chip already keeps
// about 8 MB of reads in flight, and a larger window only spreads the DRAM
// accesses over more rows.  Elements past the last full vector (fewer than
// EPV) are handled element-wise by one lane.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s2a {

constexpr int kWave = 64;    // lanes per block of the vector kernels
constexpr int kBlock = 256;  // lanes per block of the element-wise kernels

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

// Streaming memory access.  Loads carry the non-temporal hint (nt).  Stores
// carry "sc0 sc1 nt": written through to memory at system scope and not kept
// in L2 or the on-die cache -- the outputs are not read again by this kernel,
// and on MI355X a copy kernel with these stores runs 4 % faster than with nt
// alone (80 % vs 77 % of the HBM peak at 100 MB).  The compiler offers no
// source-level spelling for that combination without also serialising the
// stores, so the three store instructions are written out.
__device__ __forceinline__ u32x4 stream_load128(const u32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ uint32_t stream_load32(const uint32_t* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ uint32_t stream_load16(const uint16_t* p) { return __builtin_nontemporal_load(p); }

__device__ __forceinline__ void stream_store128(u32x4* p, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void stream_store32(uint32_t* p, uint32_t v)
{
    asm volatile("global_store_dword %0, %1, off sc0 sc1 nt" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void stream_store16(uint16_t* p, uint32_t v)
{
    asm volatile("global_store_short %0, %1, off sc0 sc1 nt" ::"v"(p), "v"(v) : "memory");
}

// The packed codes of one vector: a dword (8 bf16 elements) or a half-word (4 fp32 elements).
template <bool BF16>
__device__ __forceinline__ uint32_t load_codes(const uint8_t* codes, int64_t v)
{
    return BF16 ? stream_load32((const uint32_t*)codes + v) : stream_load16((const uint16_t*)codes + v);
}
template <bool BF16>
__device__ __forceinline__ void store_codes(uint8_t* codes, int64_t v, uint32_t c)
{
    if (BF16) stream_store32((uint32_t*)codes + v, c); else stream_store16((uint16_t*)codes + v, c);
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

// `tab` is anything indexable by a code: an LDS array, or the by-value kernel
// argument itself (the compiler then reads the kernarg segment).
template <bool BF16, typename Tab>
__device__ __forceinline__ void bwd_pairs(const void* dy, const uint8_t* codes, void* dx,
                                          const Tab& tab, int64_t first, int64_t n,
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
// x and y may be the same buffer (a lane loads its vector before it stores
// it), so neither is declared restrict.
//   nvec   number of full vectors, n / EPV
//   grid   ceil((nvec + (n % EPV != 0)) / kWave) blocks of kWave lanes
template <bool BF16>
__global__ __launch_bounds__(kWave) void fwd_kernel(const u32x4* x, u32x4* y,
                                                    uint8_t* __restrict__ codes, int64_t n,
                                                    int64_t nvec)
{
    constexpr int EPV = BF16 ? 8 : 4;
    const int64_t i = (int64_t)blockIdx.x * kWave + threadIdx.x;
    if (i < nvec) {
        u32x4 v = stream_load128(x + i);
        uint32_t c = fwd_vector<BF16>(v);
        stream_store128(y + i, v);
        store_codes<BF16>(codes, i, c);
    } else if (i == nvec) {  // one lane finishes the n % EPV leftover elements
        fwd_pairs<BF16>(x, y, codes, nvec * EPV, n, 0, 1);
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

// D[code] for a per-lane code, with the table spread over the wave: lane l
// holds D[l & 15] in `tv`, and ds_bpermute_b32 fetches the register of lane
// `code` (no LDS memory is touched).  Every lane of the wave must be active:
// the permute does not deliver the register of a source lane that is masked off.
__device__ __forceinline__ float lookup_lane(uint32_t code, int tv)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((int)(code << 2), tv));
}

template <bool BF16, typename Lookup>
__device__ __forceinline__ void bwd_vector(u32x4& v, uint32_t c, Lookup D)
{
    if (BF16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = bf16_lo(v[j]) * D((c >> (8 * j)) & 15u);
            float b = bf16_hi(v[j]) * D((c >> (8 * j + 4)) & 15u);
            v[j] = pack_bf16(a, b);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = as_u32(as_f32(v[j]) * D((c >> (4 * j)) & 15u));
    }
}

// Vector kernel of the backward pass; same layout and grid as fwd_kernel.
// dy and dx may be the same buffer.
template <bool BF16>
__global__ __launch_bounds__(kWave) void bwd_kernel(const u32x4* dy,
                                                    const uint8_t* __restrict__ codes, u32x4* dx,
                                                    QTable qt, int64_t n, int64_t nvec)
{
    constexpr int EPV = BF16 ? 8 : 4;
    const int64_t wave0 = (int64_t)blockIdx.x * kWave;
    const int64_t i = wave0 + threadIdx.x;
    if (wave0 + kWave <= nvec) {  // whole wave in range (a scalar branch): permute lookup
        const int tv = __builtin_bit_cast(int, qt.d[threadIdx.x & 15]);
        u32x4 v = stream_load128(dy + i);
        uint32_t c = load_codes<BF16>(codes, i);
        bwd_vector<BF16>(v, c, [tv](uint32_t code) { return lookup_lane(code, tv); });
        stream_store128(dx + i, v);
    } else if (i < nvec) {        // last, partial wave: read the table from the kernel arguments
        u32x4 v = dy[i];
        uint32_t c = load_codes<BF16>(codes, i);
        bwd_vector<BF16>(v, c, [&qt](uint32_t code) { return qt.d[code]; });
        stream_store128(dx + i, v);
    } else if (i == nvec) {
        bwd_pairs<BF16>(dy, codes, dx, qt.d, nvec * EPV, n, 0, 1);
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
