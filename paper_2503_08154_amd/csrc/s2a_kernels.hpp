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
// direction, e = element size), so the design is: one 128-bit load per lane,
// laid out so that a wavefront touches contiguous kilobytes; all packing done
// in registers; no LDS on the vector path (the 64-byte derivative table of the
// backward pass lives in one register per lane and is read with a cross-lane
// permute).  Further down, with the same skeleton where it applies: the
// measured-range quantizer, SiLU, the ReLU bit mask, softmax with 4-bit saved
// output, Channel Average Pooling and the Low-Rank Prompt.
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

// The activation is x * sigma(a x): a = 1.702 for the paper's GELU (Eq. 10),
// a = 1 for SiLU / Swish, which the GeLU paragraph names as covered by the same
// design.  Under the substitution x -> x / 1.702 SiLU(x) = 1.702 * GELU(x/1.702),
// so its derivative at x is Eq. 11 at x / 1.702, the sine fit becomes
// sigma(x) + 0.22 sin(1.5 x / 1.702), and the clip range becomes +-2 * 1.702.
enum { kActGelu = 0, kActSilu = 1 };
template <int ACT>
struct Act {
    static constexpr double slope = ACT == kActGelu ? 1.702 : 1.0;
    static constexpr double clip = ACT == kActGelu ? 2.0 : 2.0 * 1.702;
    // slope * log2(e), split so that hi + lo carries 48 bits of the product
    // (the fp32 path needs more than one fp32 of it)
    static constexpr double kd = slope * 1.4426950408889634074;
    static constexpr float khi = (float)kd;
    static constexpr float klo = (float)(kd - (double)khi);
    // binning: code = floor(x * 7.5/clip + 8)   (3.75 and 8, both exact, for GELU)
    static constexpr float bin_scale = (float)(7.5 / clip);
};
constexpr float kLn2 = 0.69314718055994530942f;

// ---------------------------------------------------------------- Eq. 10 ---

// sigma(1.702 x) * x for bf16 storage: the result is rounded to 8 significant
// bits afterwards, so one fp32 exponent argument is enough.  The exponential
// is carried with a 2^-32 bias: E = 2^-32 e^{-1.702x}, sigma = 2^-32 / (2^-32 + E).
// That keeps the quotient representable for x down to about -65, where y has
// already dropped below the smallest bf16 denormal, instead of overflowing at
// x = -52 where y is still a normal number.
template <int ACT>
__device__ __forceinline__ float gelu_fast(float x)
{
    float u = __builtin_fmaf(x, -Act<ACT>::khi, -32.0f);
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
template <int ACT>
__device__ __forceinline__ float gelu_accurate(float x)
{
    float xs = __builtin_amdgcn_fmed3f(x, -128.0f, 128.0f);
    float uh = xs * -Act<ACT>::khi;
    float ul = __builtin_fmaf(xs, -Act<ACT>::khi, -uh);
    ul = __builtin_fmaf(xs, -Act<ACT>::klo, ul);
    bool big = uh > 64.0f;
    float e = __builtin_amdgcn_exp2f(uh - (big ? 64.0f : 0.0f));
    e = e * __builtin_fmaf(ul, kLn2, 1.0f);  // a product, so that e = +inf stays +inf
    float r = __builtin_amdgcn_rcpf(e + (big ? 0.0f : 1.0f));
    float y = (x * r) * (big ? 0x1p-64f : 1.0f);
    return (x <= 128.0f) ? y : x;  // x > 128 or NaN: sigma == 1, or propagate NaN
}

// ------------------------------------------------------- clip + Eq. 8 ------

// code = round((clip(x, lo, hi) - lo) * 15 / (hi - lo)) as one FMA and one
// convert: t = x * scale + offset with scale = 15/(hi-lo), offset = 1/2 - lo*scale.
// Rounding to nearest equals floor(t) because an exact tie of the real-valued
// expression is itself a decision point (for the fixed range [-2, 2] the only
// one is x = 0: 7.5 -> 8 under ties-to-even, and floor(8) = 8).  One FMA rounds
// the exact value once.  The clip is applied after the conversion instead of
// before it: v_cvt_u32_f32 truncates toward zero (the floor, for t >= 0) and
// saturates -- negative and NaN inputs give 0, huge ones 0xffffffff -- so
// min(c, 15) finishes the clip and NaN lands on code 0 like a value below the
// range.  The instruction is written out because a C float-to-unsigned cast
// leaves exactly those out-of-range cases undefined.
__device__ __forceinline__ uint32_t bin_affine(float x, float scale, float offset)
{
    float t = __builtin_fmaf(x, scale, offset);
    uint32_t c;
    asm("v_cvt_u32_f32 %0, %1" : "=v"(c) : "v"(t));
    return c < 15u ? c : 15u;
}

// Fixed range: lo = -clip, hi = clip (the clip limits): scale = 7.5/clip, offset = 8.
template <int ACT>
struct BinFixed {
    __device__ __forceinline__ uint32_t operator()(float x) const { return bin_affine(x, Act<ACT>::bin_scale, 8.0f); }
};
// Measured range: scale and offset from range_reduce.
struct BinRange {
    float scale, offset;
    __device__ __forceinline__ uint32_t operator()(float x) const { return bin_affine(x, scale, offset); }
};

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
template <bool BF16, int ACT>
__device__ __forceinline__ float gelu(float x) { return BF16 ? gelu_fast<ACT>(x) : gelu_accurate<ACT>(x); }

// Streaming memory access.  Loads carry the non-temporal hint (nt).  The
// 16-byte stores carry "sc0 sc1 nt": written through to memory at system scope
// and not kept in L2 or the on-die cache -- the outputs are not read again by
// this kernel, and on MI355X a copy kernel with these stores runs 4 % faster
// than with nt alone (80 % vs 77 % of the HBM peak at 100 MB).  The small
// stores of the packed codes (4 or 2 bytes per lane) carry "sc1" only: written
// through at device scope but without the streaming hint.  With nt on them the
// forward kernels ran 3-5 % slower (ViT-L bf16 80.3 -> 83.3 % of peak, ViT-G
// fp32 83.3 -> 87.7 %); plain write-back stores come out between the two, and
// the same holds for the softmax codes although those leave as 16-byte vectors
// (forward 2-4 % faster without nt on them).  The
// compiler offers no source-level spelling for these combinations without also
// serialising the stores, so the store instructions are written out.
__device__ __forceinline__ u32x4 stream_load128(const u32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ uint32_t stream_load32(const uint32_t* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ uint32_t stream_load16(const uint16_t* p) { return __builtin_nontemporal_load(p); }

__device__ __forceinline__ void stream_store128(u32x4* p, u32x4 v)
{
    // s_nop 1: a store of more than 64 bits reads its data registers for up to two more wait
    // states, and a VALU write to one of them in that window corrupts the stored value.  The
    // compiler inserts the wait for stores it emits itself, but it cannot see into this string
    // (seen as a few garbage elements per some launches of a loop that refills the registers).
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
// 16 bytes of packed codes (the staged softmax writes its code bytes as whole vectors): the
// codes' policy, with the same wait after a wide store.
__device__ __forceinline__ void stream_store128_codes(u32x4* p, u32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void stream_store32(uint32_t* p, uint32_t v)
{
    asm volatile("global_store_dword %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void stream_store16(uint16_t* p, uint32_t v)
{
    asm volatile("global_store_short %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void stream_store8(uint8_t* p, uint32_t v)  // low byte of v
{
    asm volatile("global_store_byte %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
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

// ---------------------------------------------------------- cross-lane ----

// Cross-lane moves inside a row of 16 lanes as DPP operand modifiers (no LDS
// traffic, one VALU op each): swap with the neighbour (xor 1), with the other
// pair of the quad (xor 2), mirror the 8 / the 16 lanes of a half row / row.
// After the quads agree, the two mirrors pair every lane with one from the
// other half, so for all-reduce purposes they act as xor 4 and xor 8.  Every
// lane of the wave must be active.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, dpp_move<CTRL>(__builtin_bit_cast(int, v)));
}
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v)
{
    uint64_t u = __builtin_bit_cast(uint64_t, v);
    uint32_t lo = (uint32_t)dpp_move<CTRL>((int)(uint32_t)u), hi = (uint32_t)dpp_move<CTRL>((int)(uint32_t)(u >> 32));
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

// v_max_f32 / v_min_f32 as single instructions.  (The portable fmaxf / fminf
// first re-quiet every operand the compiler cannot prove canonical -- here all
// of them, since they come from bit patterns -- which doubles the op count.)
// NaN operands lose against numbers, as with fmaxf / fminf.
__device__ __forceinline__ float vmax(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float vmin(float a, float b)
{
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// Three-operand maximum / minimum: one VALU op takes in both elements of a pair.
__device__ __forceinline__ float vmax3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float vmin3(float a, float b, float c)
{
    float r;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// All-reduce over the G lanes of a row group; F(a, b) is the (commutative) combiner.
template <int G, typename T, typename F>
__device__ __forceinline__ T group_reduce(T v, F f)
{
    v = f(v, dpp_move<kDppXor1>(v));
    v = f(v, dpp_move<kDppXor2>(v));
    if (G >= 8) v = f(v, dpp_move<kDppHalfMirror>(v));
    if (G >= 16) v = f(v, dpp_move<kDppMirror>(v));
    if (G >= 32) v = f(v, __shfl_xor(v, 16, kWave));
    if (G >= 64) v = f(v, __shfl_xor(v, 32, kWave));
    return v;
}
// A DPP operand must not be read within two wait states of the VALU write that produced it.
// The compiler spaces the instructions it emits itself, but it does not look into asm strings,
// so a value that comes out of vmax / vmin / vmax3 / vmin3 passes through this before a
// cross-lane move reads it: the asm both waits and is the value's last definition.
__device__ __forceinline__ float settled(float v)
{
    asm("s_nop 1" : "+v"(v));
    return v;
}
template <int G>
__device__ __forceinline__ float group_max(float v)
{
    return group_reduce<G>(settled(v), [](float a, float b) { return settled(vmax(a, b)); });
}
template <int G>
__device__ __forceinline__ float group_min(float v)
{
    return group_reduce<G>(settled(v), [](float a, float b) { return settled(vmin(a, b)); });
}
template <int G, typename T>
__device__ __forceinline__ T group_sum(T v) { return group_reduce<G>(v, [](T a, T b) { return a + b; }); }

// ------------------------------------------------- element-wise pieces ----

// Elements [first, n) with first even: one code byte per pair, pad nibble 0.
template <bool BF16, int ACT, typename Bin>
__device__ __forceinline__ void fwd_pairs(const void* x, void* y, uint8_t* codes, Bin bin,
                                          int64_t first, int64_t n, int64_t pair0,
                                          int64_t pair_stride)
{
    int64_t npairs = (n - first + 1) / 2;
    for (int64_t p = pair0; p < npairs; p += pair_stride) {
        int64_t i = first + 2 * p;
        float a = load_elem<BF16>(x, i);
        uint32_t byte = bin(a);
        store_elem<BF16>(y, i, gelu<BF16, ACT>(a));
        if (i + 1 < n) {
            float b = load_elem<BF16>(x, i + 1);
            byte |= bin(b) << 4;
            store_elem<BF16>(y, i + 1, gelu<BF16, ACT>(b));
        }
        codes[i / 2] = (uint8_t)byte;
    }
}

// `D` maps a code to its derivative level (an LDS array, the kernel arguments
// or device memory behind it).
template <bool BF16, typename Lookup>
__device__ __forceinline__ void bwd_pairs(const void* dy, const uint8_t* codes, void* dx,
                                          Lookup D, int64_t first, int64_t n,
                                          int64_t pair0, int64_t pair_stride)
{
    int64_t npairs = (n - first + 1) / 2;
    for (int64_t p = pair0; p < npairs; p += pair_stride) {
        int64_t i = first + 2 * p;
        uint32_t byte = codes[i / 2];
        store_elem<BF16>(dx, i, load_elem<BF16>(dy, i) * D(byte & 15u));
        if (i + 1 < n) store_elem<BF16>(dx, i + 1, load_elem<BF16>(dy, i + 1) * D(byte >> 4));
    }
}

// ------------------------------------------------------------- forward ----

// One vector of 8 bf16: y bits in place, returns the 8 packed codes.
template <bool BF16, int ACT, typename Bin>
__device__ __forceinline__ uint32_t fwd_vector(u32x4& v, Bin bin)
{
    uint32_t acc = 0;
    if (BF16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = bf16_lo(v[j]), b = bf16_hi(v[j]);
            acc = push_nibble(acc, bin(a));
            acc = push_nibble(acc, bin(b));
            v[j] = pack_bf16(gelu_fast<ACT>(a), gelu_fast<ACT>(b));
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = as_f32(v[j]);
            acc = push_nibble(acc, bin(a));
            v[j] = as_u32(gelu_accurate<ACT>(a));
        }
        acc >>= 16;  // 4 codes -> low 16 bits
    }
    return acc;
}

// Layout of the per-tensor quantizer state of the measured-range variant
// (kQsFloats floats of caller-owned device memory, written by the forward pass;
// the backward pass reads only the table):
//   [2] min   [3] scale = (max-min)/15   [4] 15/(max-min) (0 if max == min)
//   [5] 1/2 - min * [4]                  [16..31] D[k] = Eq. 12 at min + k*scale
//   [32 .. 32+kRangeBlocks)              per-block minima of clip(x)
//   [32+kRangeBlocks .. 32+2*kRangeBlocks) per-block maxima
// Per-block partial results instead of atomics: 2048 blocks updating one
// address cost 48 us on MI355X (device-scope atomics serialise at about 12 ns
// each), three times the range pass itself; partials also need no reset
// launch and make the result independent of the order blocks finish in.
// Lanes per block by measurement at the ViT-L shape (range pass + forward kernel, 1024 / 512 / 256
// lanes): 38.8 / 38.2 / 37.9 us for activations that reach both clip limits (every wave stops after
// its first loads, so fewer lanes read less), 55.6 / 55.3 / 56.3 us for a tensor that stays inside.
constexpr int kRangeBlocks = 256, kRangeBlock = 512;
constexpr int kQsMin = 2, kQsScale = 3, kQsInv = 4, kQsOff = 5, kQsTable = 16, kQsPartMin = 32,
              kQsPartMax = 32 + kRangeBlocks, kQsFloats = 32 + 2 * kRangeBlocks;

// --------------------------------------------- measured range (Eq. 8) -----

// Block-wide minimum and maximum (all lanes call; lane 0 of the block gets the result).
template <int BLOCK>
__device__ __forceinline__ void block_minmax(float& lo, float& hi)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        lo = fminf(lo, __shfl_xor(lo, off, kWave));
        hi = fmaxf(hi, __shfl_xor(hi, off, kWave));
    }
    __shared__ float slo[BLOCK / kWave], shi[BLOCK / kWave];
    if ((threadIdx.x & (kWave - 1)) == 0) {
        slo[threadIdx.x / kWave] = lo;
        shi[threadIdx.x / kWave] = hi;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < BLOCK / kWave; ++w) {
            lo = fminf(lo, slo[w]);
            hi = fmaxf(hi, shi[w]);
        }
    }
}

// Some lane of the wave has met the lower clip limit and some lane the upper one: nothing the
// wave could still read changes min = -2, max = 2.  Uniform over the active lanes.
// (lo and hi are the unclipped extremes; a NaN counts as -2.)
__device__ __forceinline__ bool wave_saturated(float lo, float hi, bool nan)
{
    return __builtin_amdgcn_ballot_w64(lo <= -2.0f || nan) != 0 && __builtin_amdgcn_ballot_w64(hi >= 2.0f) != 0;
}

// Pass 1 of the measured range: per-block min / max of clip(x).  Each block
// walks its own contiguous share of the 16-byte vectors (of the elements when
// ALIGNED is false) and leaves its pair in qs[kQsPartMin + b] and
// qs[kQsPartMax + b] (+inf / -inf if it saw no element); all kRangeBlocks slots
// are written whatever the grid size.
// The clip bounds the result: a wave whose first round of loads held an
// element at or beyond each clip limit stops reading (wave_saturated), so a
// tensor with values beyond both limits throughout -- the activations of the
// paper's workloads -- costs one round of loads per wave (4 us instead of 21 us
// at the ViT-L shape) and still gives exactly min = -2, max = 2.  Tensors that stay
// inside a limit are read to the end, with ordinary cached loads on purpose: a
// tensor that fits the 256 MB on-die cache is then still there when the
// forward kernel reads it again (measured: the forward kernel takes 32.3 us
// instead of 36.1 us at the ViT-L shape; with streaming loads the two kernels
// together take the same time, the pass gaining what the forward kernel loses).
// That full pass runs at 4.4 TB/s (23 us for 103 MB) whatever was tried on it:
// two or eight loads in flight per lane, 256 .. 1024 lanes per block, a third of
// the arithmetic, the whole grid sweeping the tensor instead of a share per
// block, streaming loads -- all within 1 %.
template <bool BF16, bool ALIGNED>
__global__ __launch_bounds__(kRangeBlock) void range_minmax_kernel(const void* x, float* qs,
                                                                   int64_t n)
{
    constexpr int EPV = BF16 ? 8 : 4;
    // The clip is monotone, so it is applied to the two results instead of to every element; a NaN
    // (which the clip sends to -2) loses against numbers in v_min3 / v_max3 and is remembered by a
    // flag.  Two elements cost one min3, one max3 and one unordered compare.
    float lo = __builtin_inff(), hi = -__builtin_inff();
    bool nan = false;
    auto take2 = [&](float a, float b) {
        lo = vmin3(lo, a, b);
        hi = vmax3(hi, a, b);
        nan |= __builtin_isunordered(a, b);
    };
    auto take1 = [&](float a) { take2(a, a); };
    int64_t done = 0;
    if (ALIGNED) {
        const int64_t nvec = n / EPV;
        const u32x4* xv = (const u32x4*)x;
        const int64_t share = (nvec + gridDim.x - 1) / gridDim.x;
        const int64_t beg = (int64_t)blockIdx.x * share;
        const int64_t end = beg + share < nvec ? beg + share : nvec;
        // Loads are never predicated: a position past the block's share is replaced by the share's
        // last vector (a duplicate changes neither extreme), so the code between the loads and their
        // use is straight-line and the compiler lets them overlap.
        const int64_t last = end - 1;
        auto eat = [&](const u32x4& v) {
#pragma unroll
            for (int j = 0; j < 4; j += 2) {
                if (BF16) {
                    take2(bf16_lo(v[j]), bf16_hi(v[j]));
                    take2(bf16_lo(v[j + 1]), bf16_hi(v[j + 1]));
                } else {
                    take2(as_f32(v[j]), as_f32(v[j + 1]));
                }
            }
        };
        if (beg < end) {
            // first round, two vectors per lane (1024 or 2048 elements per wave); then the question
            // whether the wave can stop is asked once: asked in every round it makes each round's
            // loads wait for the data of the round before
            constexpr int U0 = 2;
            {
                u32x4 v[U0];
#pragma unroll
                for (int k = 0; k < U0; ++k) {
                    const int64_t at = beg + threadIdx.x + k * kRangeBlock;
                    v[k] = xv[at < end ? at : last];
                }
#pragma unroll
                for (int k = 0; k < U0; ++k) eat(v[k]);
            }
            // the rest of the share (tensors that stay inside a clip limit), four vectors per lane
            // and round, the next round's loads requested before this round's are used: two buffers
            // that swap roles, so that no loaded value is copied (a copy would wait for it)
            constexpr int U = 4;
            constexpr int64_t STEP = (int64_t)U * kRangeBlock;
            auto fetch = [&](u32x4(&v)[U], int64_t base) {
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    const int64_t at = base + threadIdx.x + k * kRangeBlock;
                    v[k] = xv[at < end ? at : last];
                }
            };
            int64_t at = beg + U0 * kRangeBlock;  // uniform over the block
            if (at < end && !wave_saturated(lo, hi, nan)) {
                u32x4 a[U], b[U];
                fetch(a, at);
                for (;;) {
                    fetch(b, at + STEP);
#pragma unroll
                    for (int k = 0; k < U; ++k) eat(a[k]);
                    at += STEP;
                    if (at >= end) break;
                    fetch(a, at + STEP);
#pragma unroll
                    for (int k = 0; k < U; ++k) eat(b[k]);
                    at += STEP;
                    if (at >= end) break;
                }
            }
        }
        done = nvec * EPV;
    }
    // leftover (or, unaligned, all) elements one by one, spread over the whole grid
    for (int64_t i = done + (int64_t)blockIdx.x * kRangeBlock + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * kRangeBlock) {
        if (wave_saturated(lo, hi, nan)) break;
        take1(load_elem<BF16>(x, i));
    }
    if (nan) {
        lo = fminf(lo, -2.0f);
        hi = fmaxf(hi, -2.0f);
    }
    if (lo <= hi) {  // the lane has seen an element (otherwise +inf / -inf stay: "no element")
        lo = __builtin_amdgcn_fmed3f(lo, -2.0f, 2.0f);
        hi = __builtin_amdgcn_fmed3f(hi, -2.0f, 2.0f);
    }
    block_minmax<kRangeBlock>(lo, hi);
    if (threadIdx.x == 0) {
        qs[kQsPartMin + blockIdx.x] = lo;
        qs[kQsPartMax + blockIdx.x] = hi;
    }
    // a grid smaller than kRangeBlocks (small tensors): the remaining slots read as "no element"
    for (int p = (int)(gridDim.x + blockIdx.x * kRangeBlock + threadIdx.x); p < kRangeBlocks;
         p += (int)(gridDim.x * kRangeBlock)) {
        qs[kQsPartMin + p] = __builtin_inff();
        qs[kQsPartMax + p] = -__builtin_inff();
    }
}

// Pass 2 has no launch of its own: every wave of the forward kernel reduces
// the kRangeBlocks pairs itself (2 KiB that stay in the vector cache) and turns
// (min, max) into the binning constants, all waves by the same instructions and
// therefore to the same bits.  A launch in between costs 4.6 us at any size
// (kernel boundary plus latency), 8 % of the whole pass at the ViT-L shape.
// The first wave of the grid also leaves min, scale, the constants and the 16
// derivative levels in qs for the backward pass (range_publish).
struct RangeParts {
    float lo[kRangeBlocks / kWave], hi[kRangeBlocks / kWave];
};
struct RangeBin {
    BinRange bin;
    double lo, width;  // min and max - min of the clipped tensor (0, 0 for an empty one)
};
// The loads alone, so that a kernel can put its own first load behind them and
// reduce while that one is in flight (loads return in order).
__device__ __forceinline__ RangeParts range_parts(const float* qs)
{
    const int lane = (int)threadIdx.x & (kWave - 1);
    RangeParts p;
#pragma unroll
    for (int q = 0; q < kRangeBlocks / kWave; ++q) {
        p.lo[q] = qs[kQsPartMin + q * kWave + lane];
        p.hi[q] = qs[kQsPartMax + q * kWave + lane];
    }
    return p;
}
// Every lane of the wave must be active (cross-lane moves).
__device__ __forceinline__ RangeBin range_reduce(const RangeParts& part)
{
    float lo = part.lo[0], hi = part.hi[0];
#pragma unroll
    for (int q = 1; q < kRangeBlocks / kWave; ++q) {
        lo = vmin(lo, part.lo[q]);
        hi = vmax(hi, part.hi[q]);
    }
    lo = group_min<kWave>(lo);
    hi = group_max<kWave>(hi);
    const bool empty = !(lo <= hi);
    RangeBin r;
    r.lo = empty ? 0.0 : (double)lo;
    r.width = (empty ? 0.0 : (double)hi) - r.lo;
    const double inv = r.width > 0.0 ? 15.0 / r.width : 0.0;
    r.bin = BinRange{(float)inv, (float)(0.5 - r.lo * inv)};
    return r;
}
// One wave: min, scale, the binning constants and the levels
// D[k] = sigma(1.702 xhat_k) + 0.22 sin(1.5 xhat_k), xhat_k = min + k * scale
// (Eq. 9, Eq. 12), in double, rounded once.
__device__ __forceinline__ void range_publish(float* qs, const RangeBin& r)
{
    const int lane = (int)threadIdx.x & (kWave - 1);
    const double scale = r.width / 15.0;
    if (lane < 16) {
        const double xh = r.lo + scale * (double)lane;
        qs[kQsTable + lane] = (float)(1.0 / (1.0 + exp(-1.702 * xh)) + 0.22 * sin(1.5 * xh));
    }
    if (lane == 0) {
        qs[kQsMin] = (float)r.lo;
        qs[kQsScale] = (float)scale;
        qs[kQsInv] = r.bin.scale;
        qs[kQsOff] = r.bin.offset;
    }
}

// ------------------------------------------------------ forward kernels ----

// Vector kernel.  Requires x, y 16-byte aligned and codes 4-byte aligned.
// x and y may be the same buffer (a lane loads its vector before it stores
// it), so neither is declared restrict.
//   nvec   number of full vectors, n / EPV
//   grid   ceil((nvec + (n % EPV != 0)) / kWave) blocks of kWave lanes
template <bool BF16, int ACT>
__global__ __launch_bounds__(kWave) void fwd_kernel(const u32x4* x, u32x4* y,
                                                    uint8_t* __restrict__ codes, int64_t n,
                                                    int64_t nvec)
{
    constexpr int EPV = BF16 ? 8 : 4;
    const BinFixed<ACT> bin;
    const int64_t i = (int64_t)blockIdx.x * kWave + threadIdx.x;
    if (i < nvec) {
        // A wave that is about to issue its load or its stores goes ahead of the waves that are
        // in their arithmetic: the memory system is the bottleneck, so its requests should never
        // wait for an issue slot.  Measured: fp32 forward 87.1 -> 85.5 us at the ViT-G shape
        // (82.2 -> 83.7 % of peak); no change for bf16, whose arithmetic is lighter.
        __builtin_amdgcn_s_setprio(3);
        u32x4 v = stream_load128(x + i);
        __builtin_amdgcn_s_setprio(0);
        uint32_t c = fwd_vector<BF16, ACT>(v, bin);
        __builtin_amdgcn_s_setprio(3);
        stream_store128(y + i, v);
        store_codes<BF16>(codes, i, c);
    } else if (i == nvec) {  // one lane finishes the n % EPV leftover elements
        fwd_pairs<BF16, ACT>(x, y, codes, bin, nvec * EPV, n, 0, 1);
    }
}

// The same with the measured range (GELU only): qs holds the partial minima
// and maxima of the range pass.  A wave that lies wholly inside the tensor (a
// scalar branch) requests the first pair and its vector of x; if that pair
// already is (-2, 2) the range is settled, otherwise the wave reads and
// reduces all pairs.  The grid has at least one block, also for n = 0, so
// that qs is always completed.
template <bool BF16>
__global__ __launch_bounds__(kWave) void fwd_dyn_kernel(const u32x4* x, u32x4* y,
                                                        uint8_t* __restrict__ codes,
                                                        float* __restrict__ qs, int64_t n,
                                                        int64_t nvec)
{
    constexpr int EPV = BF16 ? 8 : 4;
    const int64_t wave0 = (int64_t)blockIdx.x * kWave;
    const int64_t i = wave0 + threadIdx.x;
    RangeBin r;
    if (wave0 + kWave <= nvec) {
        // One block of the range pass that met both clip limits settles min = -2, max = 2 for the
        // whole tensor: then the other 255 pairs need not be read (the constants are those the
        // reduction would give: 15/4 and 1/2 + 2 * 15/4).
        const float lo0 = qs[kQsPartMin], hi0 = qs[kQsPartMax];
        __builtin_amdgcn_s_setprio(3);
        u32x4 v = stream_load128(x + i);
        __builtin_amdgcn_s_setprio(0);
        if (lo0 == -2.0f && hi0 == 2.0f) {
            r.bin = BinRange{3.75f, 8.0f};
            r.lo = -2.0;
            r.width = 4.0;
        } else {
            r = range_reduce(range_parts(qs));
        }
        uint32_t c = fwd_vector<BF16, kActGelu>(v, r.bin);
        __builtin_amdgcn_s_setprio(3);
        stream_store128(y + i, v);
        store_codes<BF16>(codes, i, c);
        __builtin_amdgcn_s_setprio(0);
    } else {
        r = range_reduce(range_parts(qs));
        if (i < nvec) {
            u32x4 v = stream_load128(x + i);
            uint32_t c = fwd_vector<BF16, kActGelu>(v, r.bin);
            stream_store128(y + i, v);
            store_codes<BF16>(codes, i, c);
        } else if (i == nvec) {
            fwd_pairs<BF16, kActGelu>(x, y, codes, r.bin, nvec * EPV, n, 0, 1);
        }
    }
    if (blockIdx.x == 0) range_publish(qs, r);
}

// Any alignment: one lane per code byte, grid-stride.  DYN: measured range as above.
template <bool BF16, bool DYN, int ACT>
__global__ __launch_bounds__(kBlock) void fwd_kernel_unaligned(const void* x, void* y,
                                                               uint8_t* codes,
                                                               float* __restrict__ qs,
                                                               int64_t n)
{
    const int64_t pair0 = (int64_t)blockIdx.x * kBlock + threadIdx.x, stride = (int64_t)gridDim.x * kBlock;
    if constexpr (DYN) {
        const RangeBin r = range_reduce(range_parts(qs));
        fwd_pairs<BF16, ACT>(x, y, codes, r.bin, 0, n, pair0, stride);
        if (blockIdx.x == 0 && threadIdx.x < kWave) range_publish(qs, r);
    } else {
        fwd_pairs<BF16, ACT>(x, y, codes, BinFixed<ACT>(), 0, n, pair0, stride);
    }
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

// The packed codes of a whole wave (64 consecutive vectors starting at vector `wave0`: 256 bytes
// for bf16, 128 for fp32) fetched by its first 16 (8) lanes as 16-byte vectors; every lane then
// picks its own dword (half-word) out of the fetching lane's registers with ds_bpermute_b32.
// Same bytes and cache lines as one small load per lane, but a quarter (an eighth) of the lanes
// go through the address path: measured 0.4-0.9 % on the backward kernel at the ViT-L / ViT-G
// shapes (bf16 35.3 -> 35.2 us, 45.5 -> 45.3 us; fp32 84.9 -> 84.2 us).  Needs the codes of the
// wave 16-byte aligned and every lane active.  The choice between this and one load per lane is
// a template parameter set by the launcher, not a branch in the kernel: with a branch the
// compiler waited for the gradient vector before it requested the codes (two memory latencies
// in a row, 4 % on the whole kernel).
template <bool BF16>
__device__ __forceinline__ uint32_t load_codes_wave(const uint8_t* codes, int64_t wave0)
{
    const int lane = (int)threadIdx.x & (kWave - 1);
    constexpr int FETCH = BF16 ? 16 : 8;
    u32x4 cw = {0u, 0u, 0u, 0u};
    if (lane < FETCH) cw = stream_load128((const u32x4*)(codes + wave0 * (BF16 ? 4 : 2)) + lane);
    const int src = (BF16 ? lane >> 2 : lane >> 3) << 2;  // byte index of the lane that fetched this lane's codes
    const uint32_t c0 = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)cw[0]);
    const uint32_t c1 = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)cw[1]);
    const uint32_t c2 = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)cw[2]);
    const uint32_t c3 = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)cw[3]);
    const int k = BF16 ? lane & 3 : (lane >> 1) & 3;     // which dword of the 16 bytes
    // masks instead of a chain of selects: straight-line code whatever the compiler makes of it
    const uint32_t m0 = k == 0 ? ~0u : 0u, m1 = k == 1 ? ~0u : 0u, m2 = k == 2 ? ~0u : 0u, m3 = k == 3 ? ~0u : 0u;
    const uint32_t w = (c0 & m0) | (c1 & m1) | (c2 & m2) | (c3 & m3);
    if (BF16) return w;
    return (lane & 1) ? (w >> 16) : (w & 0xffffu);
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
// dy and dx may be the same buffer.  DYN selects the table: the fixed-range
// levels passed by value, or the 16 levels the forward pass left in qs.
template <bool BF16, bool DYN, bool WAVE_CODES>
__global__ __launch_bounds__(kWave) void bwd_kernel(const u32x4* dy,
                                                    const uint8_t* __restrict__ codes, u32x4* dx,
                                                    QTable qt, const float* __restrict__ qs,
                                                    int64_t n, int64_t nvec)
{
    constexpr int EPV = BF16 ? 8 : 4;
    const int64_t wave0 = (int64_t)blockIdx.x * kWave;
    const int64_t i = wave0 + threadIdx.x;
    auto level = [&](uint32_t code) { return DYN ? qs[kQsTable + code] : qt.d[code]; };
    if (wave0 + kWave <= nvec) {  // whole wave in range (a scalar branch): permute lookup
        const int tv = __builtin_bit_cast(int, level(threadIdx.x & 15));
        u32x4 v = stream_load128(dy + i);
        const uint32_t c = WAVE_CODES ? load_codes_wave<BF16>(codes, wave0) : load_codes<BF16>(codes, i);
        bwd_vector<BF16>(v, c, [tv](uint32_t code) { return lookup_lane(code, tv); });
        stream_store128(dx + i, v);
    } else if (i < nvec) {        // last, partial wave: read the table from memory
        u32x4 v = dy[i];
        uint32_t c = load_codes<BF16>(codes, i);
        bwd_vector<BF16>(v, c, level);
        stream_store128(dx + i, v);
    } else if (i == nvec) {
        bwd_pairs<BF16>(dy, codes, dx, level, nvec * EPV, n, 0, 1);
    }
}

template <bool BF16, bool DYN>
__global__ __launch_bounds__(kBlock) void bwd_kernel_unaligned(const void* dy,
                                                               const uint8_t* codes, void* dx,
                                                               QTable qt,
                                                               const float* __restrict__ qs,
                                                               int64_t n)
{
    __shared__ float tab[16];
    if (threadIdx.x < 16) tab[threadIdx.x] = DYN ? qs[kQsTable + threadIdx.x] : qt.d[threadIdx.x];
    __syncthreads();
    bwd_pairs<BF16>(dy, codes, dx, [&](uint32_t code) { return tab[code]; }, 0, n,
                    (int64_t)blockIdx.x * kBlock + threadIdx.x, (int64_t)gridDim.x * kBlock);
}

// ------------------------------------------------ ReLU 1-bit mask ---------
//
// Sec. 3.2, "ReLU layer": the derivative is 0 or 1, so the saved activation is
// the mask x > 0, one bit per element (element 8j+b in bit b of byte j).
//   forward   y = x > 0 ? x : 0,  bit = x > 0        (2e + 1/8 bytes per element)
//   backward  dx = bit ? dy : 0                       (2e + 1/8 bytes per element)
// Same streaming skeleton as the GELU kernels: single-wave blocks, one 16-byte
// vector per lane.  A bf16 vector owns exactly one mask byte; an fp32 vector
// owns a nibble, and the even lane of each lane pair fetches its neighbour's
// nibble with a cross-lane shuffle and stores the byte.  The lane just past
// the last full vector takes the n % EPV leftover elements, so that a byte is
// still written by exactly one lane.

__device__ __forceinline__ float relu(float x) { return x > 0.0f ? x : 0.0f; }

template <bool BF16>
__global__ __launch_bounds__(kWave) void relu_fwd_kernel(const u32x4* x, u32x4* y,
                                                         uint8_t* __restrict__ mask, int64_t n,
                                                         int64_t nvec)
{
    constexpr int EPV = BF16 ? 8 : 4;
    const int64_t i = (int64_t)blockIdx.x * kWave + threadIdx.x;
    uint32_t bits = 0;
    if (i < nvec) {
        u32x4 v = stream_load128(x + i);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (BF16) {
                // NaN compares false: bit 0, y = 0.  y keeps x's bits where the bit is set.
                float a = bf16_lo(v[j]), b = bf16_hi(v[j]);
                uint32_t ma = a > 0.0f, mb = b > 0.0f;
                bits |= (ma << (2 * j)) | (mb << (2 * j + 1));
                v[j] = (ma ? (v[j] & 0x0000ffffu) : 0u) | (mb ? (v[j] & 0xffff0000u) : 0u);
            } else {
                float a = as_f32(v[j]);
                uint32_t ma = a > 0.0f;
                bits |= ma << j;
                v[j] = ma ? v[j] : 0u;
            }
        }
        stream_store128(y + i, v);
    } else if (i == nvec) {
        for (int64_t e = nvec * EPV; e < n; ++e) {
            float a = load_elem<BF16>(x, e);
            bits |= (uint32_t)(a > 0.0f) << (e - nvec * EPV);
            store_elem<BF16>(y, e, relu(a));
        }
    }
    // every lane of the wave takes part in the shuffle
    if (BF16) {
        if (i * EPV < n) stream_store8(mask + i, bits);  // sc1 like the code stores: 1 % over a plain store
    } else {
        uint32_t other = (uint32_t)__shfl_xor((int)bits, 1, kWave);
        if ((threadIdx.x & 1) == 0 && i * EPV < n) stream_store8(mask + (i >> 1), bits | (other << 4));
    }
}

template <bool BF16>
__global__ __launch_bounds__(kWave) void relu_bwd_kernel(const u32x4* dy,
                                                         const uint8_t* __restrict__ mask,
                                                         u32x4* dx, int64_t n, int64_t nvec)
{
    constexpr int EPV = BF16 ? 8 : 4;
    const int64_t i = (int64_t)blockIdx.x * kWave + threadIdx.x;
    if (i < nvec) {
        u32x4 v = stream_load128(dy + i);
        uint32_t bits = BF16 ? mask[i] : (uint32_t)(mask[i >> 1] >> (4 * (i & 1)));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (BF16)
                v[j] &= (((bits >> (2 * j)) & 1u) ? 0x0000ffffu : 0u) |
                        (((bits >> (2 * j + 1)) & 1u) ? 0xffff0000u : 0u);
            else
                v[j] = ((bits >> j) & 1u) ? v[j] : 0u;
        }
        stream_store128(dx + i, v);
    } else if (i == nvec) {
        for (int64_t e = nvec * EPV; e < n; ++e) {
            uint32_t m = (mask[e >> 3] >> (e & 7)) & 1u;
            store_elem<BF16>(dx, e, m ? load_elem<BF16>(dy, e) : 0.0f);
        }
    }
}

// Any alignment: one lane per mask byte (8 elements), grid-stride.
template <bool BF16>
__global__ __launch_bounds__(kBlock) void relu_fwd_kernel_unaligned(const void* x, void* y,
                                                                    uint8_t* mask, int64_t n)
{
    const int64_t nbytes = (n + 7) / 8;
    for (int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x; b < nbytes;
         b += (int64_t)gridDim.x * kBlock) {
        uint32_t bits = 0;
        for (int k = 0; k < 8 && b * 8 + k < n; ++k) {
            float a = load_elem<BF16>(x, b * 8 + k);
            bits |= (uint32_t)(a > 0.0f) << k;
            store_elem<BF16>(y, b * 8 + k, relu(a));
        }
        mask[b] = (uint8_t)bits;
    }
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void relu_bwd_kernel_unaligned(const void* dy,
                                                                    const uint8_t* mask, void* dx,
                                                                    int64_t n)
{
    const int64_t nbytes = (n + 7) / 8;
    for (int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x; b < nbytes;
         b += (int64_t)gridDim.x * kBlock) {
        uint32_t bits = mask[b];
        for (int k = 0; k < 8 && b * 8 + k < n; ++k)
            store_elem<BF16>(dx, b * 8 + k, ((bits >> k) & 1u) ? load_elem<BF16>(dy, b * 8 + k) : 0.0f);
    }
}

// ------------------------------------------ Softmax with 4-bit y ----------
//
// Sec. 3.2, "Softmax layer", Eq. 7-9.  Per row of length L:
//   forward   y = softmax(x)                                       (Eq. 7)
//             lo = min y, hi = max y, s = (hi - lo)/15
//             code = round((y - lo)/s)                              (Eq. 8, N = 4)
//             saved: codes (row-aligned, ceil(L/2) bytes) and (lo, s) per row
//   backward  yh = code*s + lo                                      (Eq. 9)
//             dx_i = yh_i * (dy_i - sum_j yh_j dy_j)               (Eq. 7's Jacobian)
//
// A row is handled by a group of G lanes, so a wave holds 64/G rows and all
// row reductions are cross-lane moves inside the group.  The kernels for
// 16-byte aligned buffers give each lane element pairs (G = 4 .. 32, see
// below); the element-wise fallback kernels give lane l the elements l, l+G,
// l+2G, ... (G = 8 .. 64, the smallest with ceil(L/G) <= 16): there elements 2j
// and 2j+1 sit in neighbouring lanes at the same step, and the even lane packs
// both codes into the byte it stores.
constexpr int kSoftmaxSlots = 16;    // elements (fallback kernels) or element pairs (staged kernels) per lane at most
constexpr int kSoftmaxShortL = 64 * kSoftmaxSlots;  // rows up to here are held in the registers of one lane group
constexpr int kSoftmaxMaxL = 1 << 20;               // longer rows: one block per row, several passes (below)

// exp(x - m) for x <= m.  The bf16 storage path takes the plain route.  The
// fp32 storage path keeps 1e-6 relative accuracy down to the smallest results:
// the difference x - m is formed exactly as s + err (two-sum), and the exponent
// (s + err) * log2(e) as an exact hi + lo pair; otherwise the rounding of the
// difference alone costs 2e-6 relative at x - m = -36.  Differences below -200
// (e^-200 is 0 in fp32; this includes masked logits of -inf) return 0 there.
template <bool BF16>
__device__ __forceinline__ float exp_diff(float x, float m)
{
    constexpr double kL2e = 1.4426950408889634074;
    constexpr float hi = (float)kL2e, lo = (float)(kL2e - (double)hi);
    float s = x - m;
    if (BF16) return __builtin_amdgcn_exp2f(s * hi);  // -inf -> 0 by itself
    float bb = s - x;
    float err = (x - (s - bb)) + (-m - bb);
    const bool ok = s > -200.0f;  // false for -inf and NaN as well
    s = ok ? s : -200.0f;
    err = ok ? err : 0.0f;
    float t = s * hi;
    float tl = __builtin_fmaf(s, hi, -t);
    tl = __builtin_fmaf(s, lo, tl);
    tl = __builtin_fmaf(err, hi, tl);
    return __builtin_amdgcn_exp2f(t) * __builtin_fmaf(tl, kLn2, 1.0f);
}

// Staging.  A block of BLOCK lanes owns BLOCK/G consecutive rows, i.e. one
// contiguous span of x (and of y, codes).  Row starts are only element-aligned
// (L = 197 bf16 -> 394-byte rows), so per-row global access would be a stream of
// 2-byte loads (24 % of the HBM peak at the ViT-B/16 attention shape); instead
// the span is moved between HBM and LDS with 16-byte vectors (its ragged first
// and last vector element by element), and the row-shaped access pattern hits
// LDS.  The LDS copy keeps the span's offset within its first 16-byte vector,
// so global vectors map onto aligned LDS vectors.
constexpr int kSoftmaxBlock = 256;  // lanes per block of the fallback kernels

// Copy bytes [a, b) of `src` (global, `total` bytes long, 16-byte aligned) to
// lds + (p - (a & ~15)).  Whole 16-byte vectors are moved, including the first
// and last one, which also carry a few bytes of the neighbouring blocks' rows
// (never used); only a vector that would cross the end of the tensor is read
// element by element, one element per lane (UNIT = bytes per element).  Up to
// four loads per lane are in flight before the first LDS write waits for data.
template <int UNIT>
__device__ __forceinline__ void copy_unit(unsigned char* dst, const unsigned char* src)
{
    if (UNIT == 4) *(uint32_t*)dst = *(const uint32_t*)src;
    else if (UNIT == 2) *(uint16_t*)dst = *(const uint16_t*)src;
    else *dst = *src;
}
template <int UNIT, int BLOCK, int U>
struct StageIn {
    const unsigned char* g0;  // uniform over the block
    unsigned char* lds;
    int head, span, nv, nfull, i0;
    bool cut;
    u32x4 t[U];
    __device__ __forceinline__ StageIn(const void* src, unsigned char* lds_, int64_t a, int64_t b, int64_t total)
    {
        const int64_t a_dn = a & ~(int64_t)15;
        g0 = (const unsigned char*)src + a_dn;
        lds = lds_;
        head = (int)(a - a_dn);
        span = (int)(b - a_dn);
        nv = (span + 15) >> 4;
        cut = a_dn + 16 * (int64_t)nv > total;  // the tensor ends inside the last vector
        nfull = cut ? nv - 1 : nv;
        // lane <-> vector mapping relative to a 256-byte aligned window, so that every
        // wave-wide access covers whole, aligned lines except at the two ends of the span
        i0 = (int)(((uintptr_t)g0 >> 4) & 15);
    }
    // One round = U loads per lane starting at vector `base`: request them, then (commit) put them into LDS.
    __device__ __forceinline__ void issue(int base)
    {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = base + u * BLOCK + (int)threadIdx.x;
            if (i >= 0 && i < nfull) t[u] = stream_load128((const u32x4*)(g0 + 16 * i));
        }
    }
    __device__ __forceinline__ void commit(int base)
    {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = base + u * BLOCK + (int)threadIdx.x;
            if (i >= 0 && i < nfull) *(u32x4*)(lds + 16 * i) = t[u];
        }
    }
    // The rounds after the first, and the cut last vector.
    __device__ __forceinline__ void finish()
    {
        for (int base = -i0 + U * BLOCK; base < nfull; base += U * BLOCK) {
            issue(base);
            commit(base);
        }
        const int tid = (int)threadIdx.x;
        if (cut && tid < 16 / UNIT) {
            const int p = 16 * (nv - 1) + tid * UNIT;
            if (p >= head && p < span) copy_unit<UNIT>(lds + p, g0 + p);
        }
    }
};
template <int UNIT, int BLOCK>
__device__ __forceinline__ void stage_in(const void* src, unsigned char* lds, int64_t a, int64_t b,
                                         int64_t total)
{
    StageIn<UNIT, BLOCK, 4> st(src, lds, a, b, total);
    st.issue(-st.i0);
    st.commit(-st.i0);
    st.finish();
}
// Two spans at once (the backward kernel's dL/dy and codes): the first round of both is requested
// before either is waited for, so a block pays the memory latency once.
template <int UNIT_A, int UNIT_B, int BLOCK>
__device__ __forceinline__ void stage_in2(const void* src_a, unsigned char* lds_a, int64_t a0, int64_t a1, int64_t total_a,
                                          const void* src_b, unsigned char* lds_b, int64_t b0, int64_t b1, int64_t total_b)
{
    StageIn<UNIT_A, BLOCK, 4> sa(src_a, lds_a, a0, a1, total_a);
    StageIn<UNIT_B, BLOCK, 2> sb(src_b, lds_b, b0, b1, total_b);
    sa.issue(-sa.i0);
    sb.issue(-sb.i0);
    sa.commit(-sa.i0);
    sb.commit(-sb.i0);
    sa.finish();
    sb.finish();
}
// The reverse copy.  Vectors that lie wholly inside [a, b) are stored as such;
// the ragged first and last vector belong partly to other blocks and are
// written element by element, one element per lane.
template <int UNIT, int BLOCK, bool CODES = false>
__device__ __forceinline__ void stage_out(void* dst, const unsigned char* lds, int64_t a, int64_t b)
{
    const int64_t a_dn = a & ~(int64_t)15;
    unsigned char* g0 = (unsigned char*)dst + a_dn;
    const int head = (int)(a - a_dn), span = (int)(b - a_dn);
    const int first_full = head ? 1 : 0, last_full = span >> 4;  // vectors [first_full, last_full) are whole
    const int tid = (int)threadIdx.x;
    const int i0 = (int)(((uintptr_t)g0 >> 4) & 15);  // 256-byte aligned windows, as in stage_in
    for (int i = tid - i0; i < last_full; i += BLOCK)
        if (i >= first_full) {
            const u32x4 v = *(const u32x4*)(lds + 16 * i);
            if (CODES) stream_store128_codes((u32x4*)(g0 + 16 * i), v); else stream_store128((u32x4*)(g0 + 16 * i), v);
        }
    constexpr int PER = 16 / UNIT;
    if (tid < 2 * PER) {
        const bool tail = tid >= PER;
        const int p = tail ? 16 * last_full + (tid - PER) * UNIT : tid * UNIT;
        const bool want = tail ? !(first_full == 1 && last_full == 0) : first_full == 1;
        if (want && p >= head && p < span && (tail || p < 16)) copy_unit<UNIT>(g0 + p, lds + p);
    }
}

// ---- staged kernels: x, y (dy, dx) and codes 16-byte aligned (the launcher checks) ----
//
// A row is handled by G lanes (4, 8, 16 or 32).  Lane l owns the element PAIRS
// l, l+G, l+2G, ... of its row (pair j = elements 2j and 2j+1), SLOTS pairs at
// most, SLOTS = ceil(ceil(L/2) / G) exactly: the two codes of a pair share one
// byte of the row-aligned code array, so a lane forms and stores whole bytes by
// itself, and two outputs leave through one bf16 conversion.  Only the last
// slot can hold lanes whose pair is half or wholly past the row end, so every
// earlier slot runs without predicates and in straight-line code.  Rows past
// the end of the tensor (last block only) shadow the block's last real row and
// store nothing.  `data_bytes` is the size of the LDS data area; the codes area
// follows it.

template <bool BF16>
__device__ __forceinline__ float lds_in(const unsigned char* p)
{
    return BF16 ? as_f32((uint32_t)(*(const uint16_t*)p) << 16) : *(const float*)p;
}
// Two neighbouring elements to LDS.  Rows of odd length start on odd elements,
// so a bf16 pair is only 2-byte aligned: two 16-bit stores of one packed word,
// volatile so that they are not merged into one misaligned 32-bit store (which
// the LDS accepts but serialises: measured 1.7x on the whole kernel).
template <bool BF16>
__device__ __forceinline__ void lds_out2(unsigned char* p, float a, float b)
{
    if (BF16) {
        const uint32_t w = pack_bf16(a, b);
        typedef volatile __attribute__((address_space(3))) uint16_t lds_u16;
        ((lds_u16*)p)[0] = (uint16_t)w;
        ((lds_u16*)p)[1] = (uint16_t)(w >> 16);
    } else {
        ((float*)p)[0] = a;
        ((float*)p)[1] = b;
    }
}
template <bool BF16>
__device__ __forceinline__ void lds_out(unsigned char* p, float v)
{
    if (BF16) *(uint16_t*)p = (uint16_t)pack_bf16(v, 0.0f); else *(float*)p = v;
}

// exp(x - m) for all elements of one row.  bf16 storage: exp2(x*log2e - m*log2e)
// with the second product formed once per row; its rounding error is the same
// factor on every element of the row and cancels in the normalisation.  fp32
// storage: the compensated difference of exp_diff.
template <bool BF16>
struct RowExp {
    float m, nm;
    __device__ __forceinline__ explicit RowExp(float m_) : m(m_), nm(-m_ * 1.44269504088896340736f) {}
    __device__ __forceinline__ float operator()(float x) const
    {
        if (BF16) return __builtin_amdgcn_exp2f(__builtin_fmaf(x, 1.44269504088896340736f, nm));
        return exp_diff<false>(x, m);
    }
};

// The blocks of a staged kernel live long (load the span, compute, store it) and
// all of the first wave of blocks -- as many as fit the chip at once -- would
// start together and move through the three phases in step: the memory system
// is swamped, then idle while everyone computes, then swamped again, and with
// only two to five such rounds per launch the blocks never drift apart.  So the
// k-th block that a compute unit receives at the start of the launch (blocks
// are handed out round-robin: k = blockIdx / compute units) first sleeps k
// steps of 16 x 64 clocks (0.43 us; eight blocks per unit, up to 3 us).
// Measured at the ViT-B/16 attention shape: 3-5 % on every kernel (steps of
// 8 / 16 / 24 / 32 / 48: +2.5 / +3.5 / +1 / -1 / -5 % for the bf16 forward);
// staggering neighbouring compute units instead of the slots of one unit: no
// gain.  `stagger_units` is 0 for launches of less than two rounds.
constexpr int kStaggerSlots = 8;
__device__ __forceinline__ void stagger_first_round(int stagger_units)
{
    if (stagger_units > 0 && (int)blockIdx.x < kStaggerSlots * stagger_units) {
        const int k = (int)blockIdx.x / stagger_units;
        for (int q = 0; q < k; ++q) __builtin_amdgcn_s_sleep(16);
    }
}

template <bool BF16, int G, int SLOTS, int BLOCK>
__global__ __launch_bounds__(BLOCK) void softmax_fwd_staged(const void* x, void* y,
                                                                    uint8_t* codes,
                                                                    float* __restrict__ qparams,
                                                                    int64_t rows, int L,
                                                                    int data_bytes, int stagger_units)
{
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int RPB = BLOCK / G;           // rows per block
    constexpr int KL = SLOTS - 1;            // the only slot that can be partly empty
    constexpr int PS = 2 * G * ES;           // bytes between a lane's consecutive pairs
    extern __shared__ __align__(16) unsigned char lds[];
    const int l = threadIdx.x % G;
    const int64_t row0 = (int64_t)blockIdx.x * RPB;
    const int nrows = rows - row0 < RPB ? (int)(rows - row0) : RPB;
    const int rb = (L + 1) / 2;
    const int64_t xa = row0 * L * ES, xb = (row0 + nrows) * L * ES;
    const int64_t ca = row0 * rb, cb = (row0 + nrows) * rb;
    const int e0 = 2 * (l + KL * G), e1 = e0 + 1;  // this lane's elements in the last slot
    const bool has0 = e0 < L, has1 = e1 < L;
    // lanes past the row end re-read the row's last element: a duplicate changes neither extreme
    const int o0 = ((has0 ? e0 : L - 1) - 2 * l) * ES, o1 = ((has1 ? e1 : L - 1) - 2 * l) * ES;

    stagger_first_round(stagger_units);
    stage_in<ES, BLOCK>(x, lds, xa, xb, rows * L * ES);
    __syncthreads();

    const int lrow = (int)threadIdx.x / G;
    const bool live = lrow < nrows;
    const int srow = live ? lrow : nrows - 1;
    unsigned char* lx = lds + (int)(xa & 15) + (srow * L + 2 * l) * ES;  // this lane's first pair
    unsigned char* lc = lds + data_bytes + (int)(ca & 15) + srow * rb + l;  // and its code byte

    // pass 1: load, row maximum and minimum
    float a[SLOTS], b[SLOTS];
    float m = -__builtin_inff(), xmin = __builtin_inff();
#pragma unroll
    for (int k = 0; k < KL; ++k) {
        a[k] = lds_in<BF16>(lx + k * PS);
        b[k] = lds_in<BF16>(lx + k * PS + ES);
    }
    a[KL] = lds_in<BF16>(lx + o0);
    b[KL] = lds_in<BF16>(lx + o1);
#pragma unroll
    for (int k = 0; k < SLOTS; ++k) {
        m = vmax3(m, a[k], b[k]);
        xmin = vmin3(xmin, a[k], b[k]);
    }
    m = group_max<G>(m);
    xmin = group_min<G>(xmin);

    // pass 2: exponentials and their sum
    const RowExp<BF16> ex(m);
    typedef typename std::conditional<BF16, float, double>::type acc_t;
    acc_t sum = 0;
#pragma unroll
    for (int k = 0; k < KL; ++k) {
        a[k] = ex(a[k]);
        b[k] = ex(b[k]);
        sum += (acc_t)a[k];
        sum += (acc_t)b[k];
    }
    a[KL] = has0 ? ex(a[KL]) : 0.0f;
    b[KL] = has1 ? ex(b[KL]) : 0.0f;
    sum += (acc_t)a[KL];
    sum += (acc_t)b[KL];
    sum = group_sum<G>(sum);
    // reciprocals by v_rcp_f32 (1 ulp): a full division sequence costs a dozen instructions per lane
    const float inv = BF16 ? __builtin_amdgcn_rcpf((float)sum) : (float)((acc_t)1 / sum);
    // y is monotone in x, so its extremes are the images of the row's extremes
    const float hi = ex(m) * inv;
    const float lo = ex(xmin) * inv;
    const float scale = (hi - lo) * (1.0f / 15.0f);
    const float inv_scale = hi > lo ? 15.0f * __builtin_amdgcn_rcpf(hi - lo) : 0.0f;
    if (live && l == 0) {
        qparams[2 * (row0 + lrow)] = lo;
        qparams[2 * (row0 + lrow) + 1] = scale;
    }

    // pass 3: y and the codes into LDS.  lo <= y <= hi and inv_scale is
    // 15/(hi - lo) to 1 ulp, so (y - lo)*inv_scale + 0.5 stays below 15.5*(1 + 2^-21):
    // the saturating conversion (floor; NaN and negatives -> 0) never exceeds 15.  The
    // offset 0.5 - lo*inv_scale is formed once per row, so a code costs one FMA and one convert.
    const float q_off = __builtin_fmaf(-lo, inv_scale, 0.5f);
    auto quantize = [&](float yk) -> uint32_t {
        float t = __builtin_fmaf(yk, inv_scale, q_off);
        uint32_t c;
        asm("v_cvt_u32_f32 %0, %1" : "=v"(c) : "v"(t));
        return c;
    };
    if (live) {
#pragma unroll
        for (int k = 0; k < KL; ++k) {
            const float ya = a[k] * inv, yb = b[k] * inv;
            lds_out2<BF16>(lx + k * PS, ya, yb);
            lc[k * G] = (uint8_t)(quantize(ya) | (quantize(yb) << 4));
        }
        const float ya = a[KL] * inv, yb = b[KL] * inv;
        if (has1) {
            lds_out2<BF16>(lx + KL * PS, ya, yb);
            lc[KL * G] = (uint8_t)(quantize(ya) | (quantize(yb) << 4));
        } else if (has0) {  // the row's last, unpaired element: the pad nibble is 0
            lds_out<BF16>(lx + KL * PS, ya);
            lc[KL * G] = (uint8_t)quantize(ya);
        }
    }
    __syncthreads();
    stage_out<ES, BLOCK>(y, lds, xa, xb);
    stage_out<1, BLOCK, true>(codes, lds + data_bytes, ca, cb);
}

template <bool BF16, int G, int SLOTS, int BLOCK>
__global__ __launch_bounds__(BLOCK) void softmax_bwd_staged(const void* dy,
                                                                    const uint8_t* codes,
                                                                    const float* __restrict__ qparams,
                                                                    void* dx, int64_t rows, int L,
                                                                    int data_bytes, int stagger_units)
{
    constexpr int ES = BF16 ? 2 : 4;
    constexpr int RPB = BLOCK / G;
    constexpr int KL = SLOTS - 1;
    constexpr int PS = 2 * G * ES;
    extern __shared__ __align__(16) unsigned char lds[];
    const int l = threadIdx.x % G;
    const int64_t row0 = (int64_t)blockIdx.x * RPB;
    const int nrows = rows - row0 < RPB ? (int)(rows - row0) : RPB;
    const int rb = (L + 1) / 2;
    const int64_t xa = row0 * L * ES, xb = (row0 + nrows) * L * ES;
    const int64_t ca = row0 * rb, cb = (row0 + nrows) * rb;
    const int e0 = 2 * (l + KL * G), e1 = e0 + 1;
    const bool has0 = e0 < L, has1 = e1 < L;
    // lanes past the row end read the row's last element and last byte, and drop them
    const int o0 = ((has0 ? e0 : L - 1) - 2 * l) * ES, o1 = ((has1 ? e1 : L - 1) - 2 * l) * ES;
    const int oc = (has0 ? l + KL * G : rb - 1) - l;

    stagger_first_round(stagger_units);
    const int lrow = (int)threadIdx.x / G;
    const bool live = lrow < nrows;
    const int srow = live ? lrow : nrows - 1;
    // the row's (lo, scale) are requested before the staging loads, not after the barrier
    const float lo = qparams[2 * (row0 + srow)];
    const float scale = qparams[2 * (row0 + srow) + 1];
    stage_in2<ES, 1, BLOCK>(dy, lds, xa, xb, rows * L * ES, codes, lds + data_bytes, ca, cb, rows * rb);
    __syncthreads();

    unsigned char* lx = lds + (int)(xa & 15) + (srow * L + 2 * l) * ES;
    const unsigned char* lc = lds + data_bytes + (int)(ca & 15) + srow * rb + l;

    float ya[SLOTS], yb[SLOTS], ga[SLOTS], gb[SLOTS];
#pragma unroll
    for (int k = 0; k < SLOTS; ++k) {
        const uint32_t byte = lc[k < KL ? k * G : oc];
        ya[k] = __builtin_fmaf((float)(byte & 15u), scale, lo);
        yb[k] = __builtin_fmaf((float)(byte >> 4), scale, lo);
        ga[k] = lds_in<BF16>(lx + (k < KL ? k * PS : o0));
        gb[k] = lds_in<BF16>(lx + (k < KL ? k * PS + ES : o1));
    }
    float dot = 0.0f;
#pragma unroll
    for (int k = 0; k < KL; ++k) {
        dot = __builtin_fmaf(ya[k], ga[k], dot);
        dot = __builtin_fmaf(yb[k], gb[k], dot);
    }
    dot = has0 ? __builtin_fmaf(ya[KL], ga[KL], dot) : dot;
    dot = has1 ? __builtin_fmaf(yb[KL], gb[KL], dot) : dot;
    dot = group_sum<G>(dot);

    if (live) {
#pragma unroll
        for (int k = 0; k < KL; ++k)
            lds_out2<BF16>(lx + k * PS, ya[k] * (ga[k] - dot), yb[k] * (gb[k] - dot));
        if (has1)
            lds_out2<BF16>(lx + KL * PS, ya[KL] * (ga[KL] - dot), yb[KL] * (gb[KL] - dot));
        else if (has0)
            lds_out<BF16>(lx + KL * PS, ya[KL] * (ga[KL] - dot));
    }
    __syncthreads();
    stage_out<ES, BLOCK>(dx, lds, xa, xb);
}

// ---- element-wise kernels for buffers that are not 16-byte aligned (same results, not tuned) ----

template <bool BF16, int G>
__global__ __launch_bounds__(kSoftmaxBlock) void softmax_fwd_kernel(const void* x, void* y,
                                                                    uint8_t* codes,
                                                                    float* __restrict__ qparams,
                                                                    int64_t rows, int L)
{
    constexpr int RPB = kSoftmaxBlock / G;
    const int l = threadIdx.x % G, lrow = threadIdx.x / G;
    const int64_t row = (int64_t)blockIdx.x * RPB + lrow;
    const bool live = row < rows;
    const int rb = (L + 1) / 2;
    const float ninf = -__builtin_inff(), pinf = __builtin_inff();

    float v[kSoftmaxSlots];
    float m = ninf, xmin = pinf;
#pragma unroll
    for (int k = 0; k < kSoftmaxSlots; ++k) {
        v[k] = ninf;
        if (k * G < L) {  // uniform over the block
            const int idx = l + k * G;
            if (live && idx < L) {
                v[k] = load_elem<BF16>(x, row * L + idx);
                xmin = vmin(xmin, v[k]);
            }
            m = vmax(m, v[k]);
        }
    }
    m = group_max<G>(m);
    xmin = group_min<G>(xmin);
    typedef typename std::conditional<BF16, float, double>::type acc_t;
    acc_t sum = 0;
#pragma unroll
    for (int k = 0; k < kSoftmaxSlots; ++k)
        if (k * G < L) {
            v[k] = exp_diff<BF16>(v[k], m);
            sum += (acc_t)v[k];
        }
    sum = group_sum<G>(sum);
    const float inv = (float)((acc_t)1 / sum);
    const float hi = exp_diff<BF16>(m, m) * inv;
    const float lo = exp_diff<BF16>(xmin, m) * inv;
    const float scale = (hi - lo) / 15.0f;
    const float inv_scale = scale > 0.0f ? 15.0f / (hi - lo) : 0.0f;
    if (live && l == 0) {
        qparams[2 * row] = lo;
        qparams[2 * row + 1] = scale;
    }
#pragma unroll
    for (int k = 0; k < kSoftmaxSlots; ++k)
        if (k * G < L) {
            const int idx = l + k * G;
            const float yk = v[k] * inv;
            uint32_t c = 0;
            if (idx < L) {
                float t = __builtin_fmaf(yk - lo, inv_scale, 0.5f);
                asm("v_cvt_u32_f32 %0, %1" : "=v"(c) : "v"(t));
                c = c < 15u ? c : 15u;
            }
            const uint32_t other = (uint32_t)dpp_move<kDppXor1>((int)c);  // all lanes take part
            if (live && idx < L) {
                store_elem<BF16>(y, row * L + idx, yk);
                if ((l & 1) == 0) codes[row * rb + (idx >> 1)] = (uint8_t)(c | (other << 4));
            }
        }
}

template <bool BF16, int G>
__global__ __launch_bounds__(kSoftmaxBlock) void softmax_bwd_kernel(const void* dy,
                                                                    const uint8_t* codes,
                                                                    const float* __restrict__ qparams,
                                                                    void* dx, int64_t rows, int L)
{
    constexpr int RPB = kSoftmaxBlock / G;
    const int l = threadIdx.x % G, lrow = threadIdx.x / G;
    const int64_t row = (int64_t)blockIdx.x * RPB + lrow;
    const bool live = row < rows;
    const int rb = (L + 1) / 2;
    const float lo = live ? qparams[2 * row] : 0.0f;
    const float scale = live ? qparams[2 * row + 1] : 0.0f;
    float yh[kSoftmaxSlots], g[kSoftmaxSlots];
    float dot = 0.0f;
#pragma unroll
    for (int k = 0; k < kSoftmaxSlots; ++k) {
        yh[k] = 0.0f;
        g[k] = 0.0f;
        if (k * G < L) {
            const int idx = l + k * G;
            if (live && idx < L) {
                const uint32_t byte = codes[row * rb + (idx >> 1)];
                yh[k] = __builtin_fmaf((float)((byte >> (4 * (idx & 1))) & 15u), scale, lo);
                g[k] = load_elem<BF16>(dy, row * L + idx);
            }
            dot = __builtin_fmaf(yh[k], g[k], dot);
        }
    }
    dot = group_sum<G>(dot);
#pragma unroll
    for (int k = 0; k < kSoftmaxSlots; ++k)
        if (k * G < L) {
            const int idx = l + k * G;
            if (live && idx < L) store_elem<BF16>(dx, row * L + idx, yh[k] * (g[k] - dot));
        }
}

// ---- rows longer than kSoftmaxShortL: one block per row, the row re-read from the caches ----
//
// No attention of the paper's models has such rows (197 .. 577); this path is there so that the
// entry points hold for any L, and is not tuned.  Forward: pass 1 finds max and min of x, pass 2
// the sum of the exponentials (fp64 accumulators: a lane adds up to L / 256 terms), pass 3 forms y
// and the codes pair by pair, so a lane owns whole code bytes.  lo and hi are the images of the
// extreme x (y is monotone in x), as in the other kernels.  x is only overwritten in pass 3, by
// the lane that read the element, so y may be x.  Backward: pass 1 the dot product, pass 2 dx.

// Combine one value per wave over the block's waves; every lane gets the result.  `slots` holds
// one T per wave; two barriers, so it can be used again right away.
template <typename T, typename F>
__device__ __forceinline__ T block_combine(T wave_value, T* slots, F f)
{
    const int wave = threadIdx.x / kWave, waves = blockDim.x / kWave;
    if (threadIdx.x % kWave == 0) slots[wave] = wave_value;
    __syncthreads();
    T v = slots[0];
    for (int w = 1; w < waves; ++w) v = f(v, slots[w]);
    __syncthreads();
    return v;
}

template <bool BF16>
__global__ __launch_bounds__(kSoftmaxBlock) void softmax_fwd_long_kernel(const void* x, void* y, uint8_t* codes,
                                                                         float* __restrict__ qparams, int L)
{
    __shared__ float fslots[kSoftmaxBlock / kWave];
    __shared__ double dslots[kSoftmaxBlock / kWave];
    const int64_t row = blockIdx.x, base = row * L;
    const int rb = (L + 1) / 2;
    float m = -__builtin_inff(), xmin = __builtin_inff();
    for (int idx = threadIdx.x; idx < L; idx += kSoftmaxBlock) {
        const float v = load_elem<BF16>(x, base + idx);
        m = vmax(m, v);
        xmin = vmin(xmin, v);
    }
    m = block_combine(group_max<kWave>(m), fslots, [](float a, float b) { return vmax(a, b); });
    xmin = block_combine(group_min<kWave>(xmin), fslots, [](float a, float b) { return vmin(a, b); });
    double sum = 0.0;
    for (int idx = threadIdx.x; idx < L; idx += kSoftmaxBlock)
        sum += (double)exp_diff<BF16>(load_elem<BF16>(x, base + idx), m);
    sum = block_combine(group_sum<kWave>(sum), dslots, [](double a, double b) { return a + b; });
    const float inv = (float)(1.0 / sum);
    const float hi = exp_diff<BF16>(m, m) * inv;
    const float lo = exp_diff<BF16>(xmin, m) * inv;
    const float scale = (hi - lo) / 15.0f;
    const float inv_scale = scale > 0.0f ? 15.0f / (hi - lo) : 0.0f;
    if (threadIdx.x == 0) {
        qparams[2 * row] = lo;
        qparams[2 * row + 1] = scale;
    }
    for (int pair = threadIdx.x; pair < rb; pair += kSoftmaxBlock) {
        uint32_t byte = 0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int idx = 2 * pair + h;
            if (idx < L) {
                const float yk = exp_diff<BF16>(load_elem<BF16>(x, base + idx), m) * inv;
                const float t = __builtin_fmaf(yk - lo, inv_scale, 0.5f);
                uint32_t c;
                asm("v_cvt_u32_f32 %0, %1" : "=v"(c) : "v"(t));
                c = c < 15u ? c : 15u;
                byte |= c << (4 * h);
                store_elem<BF16>(y, base + idx, yk);
            }
        }
        codes[row * rb + pair] = (uint8_t)byte;
    }
}

template <bool BF16>
__global__ __launch_bounds__(kSoftmaxBlock) void softmax_bwd_long_kernel(const void* dy, const uint8_t* codes,
                                                                         const float* __restrict__ qparams, void* dx,
                                                                         int L)
{
    __shared__ double dslots[kSoftmaxBlock / kWave];
    const int64_t row = blockIdx.x, base = row * L;
    const int rb = (L + 1) / 2;
    const float lo = qparams[2 * row], scale = qparams[2 * row + 1];
    double acc = 0.0;
    for (int idx = threadIdx.x; idx < L; idx += kSoftmaxBlock) {
        const uint32_t byte = codes[row * rb + (idx >> 1)];
        const float yh = __builtin_fmaf((float)((byte >> (4 * (idx & 1))) & 15u), scale, lo);
        acc += (double)(yh * load_elem<BF16>(dy, base + idx));
    }
    const float dot = (float)block_combine(group_sum<kWave>(acc), dslots, [](double a, double b) { return a + b; });
    for (int idx = threadIdx.x; idx < L; idx += kSoftmaxBlock) {
        const uint32_t byte = codes[row * rb + (idx >> 1)];
        const float yh = __builtin_fmaf((float)((byte >> (4 * (idx & 1))) & 15u), scale, lo);
        store_elem<BF16>(dx, base + idx, yh * (load_elem<BF16>(dy, base + idx) - dot));
    }
}

// --------------------------------------- Channel Average Pooling ----------
//
// Sec. 3.1, "Lite Side Branch" paragraph, Eq. 5: y_k = (1/r) sum_{j<r} x_{kr+j}
// along the contiguous channel axis; dL/dx_{kr+j} = dL/dy_k / r.  Parameter
// free and activation free: backward needs only dL/dy and r.  On the flat
// tensor, output m averages inputs m*R .. m*R + R - 1 (R a power of two, 2..64).
// Streaming skeleton as above: single-wave blocks, one 16-byte vector of x (of
// dx) per lane.  R <= EPV: a lane produces EPV/R outputs; R > EPV: R/EPV
// neighbouring lanes add up by DPP moves and the first of them stores.
// Bytes per input element: e + e/R in either direction.

// Lanes per block and vectors per lane of the pooling kernels, by measurement at [64, 197, 4096]
// bf16, r = 8 (forward 116 MB, mostly read; backward the same bytes, mostly written): single-wave
// blocks with one vector per lane, the shape of the activation kernels, reach 59 % / 64 % of the
// HBM peak here -- such waves are so short-lived that the launch rate of waves (about 4.6 per ns)
// limits them.  Forward: 128 lanes x 4 vectors 73 % (x 1: 64 %, x 2: 70 %, x 8: 73 %; 256 lanes
// the same within 1 %; sending a wave's 64 two-byte outputs out through 8 lanes as 16-byte vectors
// gains 2 % there and loses 8 % at the token shapes, where the kernel is a few microseconds long:
// not used).  Backward: 128 lanes 88 %, 256 lanes 86 %.
constexpr int kCapBlock = 128, kCapFwdVectors = 4;

template <bool BF16>
__device__ __forceinline__ void unpack_vector(const u32x4& v, float* f)
{
    if (BF16) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f[2 * j] = bf16_lo(v[j]);
            f[2 * j + 1] = bf16_hi(v[j]);
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = as_f32(v[j]);
    }
}

// V vectors per lane, all requested before the first is used: a kernel that mostly reads needs more
// bytes in flight per wave than the read-and-write kernels above (their waves live long enough on
// their stores).  Lane t of a block takes the vectors t, t + B, t + 2B, ... of the block's chunk.
template <bool BF16, int R, int V>
__global__ __launch_bounds__(kCapBlock) void cap_fwd_kernel(const u32x4* x, void* y, int64_t n_in,
                                                            int64_t nvec)
{
    constexpr int EPV = BF16 ? 8 : 4;
    constexpr float kInv = 1.0f / (float)R;
    const int64_t first = (int64_t)blockIdx.x * (blockDim.x * V) + threadIdx.x;
    u32x4 t[V];
    if (nvec > 0) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int64_t i = first + (int64_t)v * blockDim.x;
            t[v] = stream_load128(x + (i < nvec ? i : nvec - 1));  // lanes past the end re-read the last vector
        }
    }
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const int64_t i = first + (int64_t)v * blockDim.x;
        if constexpr (R <= EPV) {
            constexpr int OUT = EPV / R;  // outputs per lane
            if (i < nvec) {
                float f[EPV], o[OUT];
                unpack_vector<BF16>(t[v], f);
#pragma unroll
                for (int q = 0; q < OUT; ++q) {
                    float acc = f[q * R];
#pragma unroll
                    for (int j = 1; j < R; ++j) acc += f[q * R + j];
                    o[q] = acc * kInv;
                }
#pragma unroll
                for (int q = 0; q < OUT; ++q) store_elem<BF16>(y, i * OUT + q, o[q]);
            } else if (i == nvec) {  // leftover groups past the last full vector
                for (int64_t m = nvec * OUT; m < n_in / R; ++m) {
                    float acc = 0.0f;
                    for (int j = 0; j < R; ++j) acc += load_elem<BF16>(x, m * R + j);
                    store_elem<BF16>(y, m, acc * kInv);
                }
            }
        } else {
            constexpr int K = R / EPV;  // lanes per output, 2..16: stays inside a DPP row
            // every lane takes part in the DPP moves (n_in is a multiple of R > EPV, so nvec > 0 here)
            float f[EPV];
            unpack_vector<BF16>(t[v], f);
            float acc = f[0];
#pragma unroll
            for (int j = 1; j < EPV; ++j) acc += f[j];
            acc += dpp_move<kDppXor1>(acc);
            if (K >= 4) acc += dpp_move<kDppXor2>(acc);
            if (K >= 8) acc += dpp_move<kDppHalfMirror>(acc);
            if (K >= 16) acc += dpp_move<kDppMirror>(acc);
            if (i < nvec && (threadIdx.x % K) == 0) store_elem<BF16>(y, i / K, acc * kInv);
        }
    }
}

template <bool BF16, int R>
__global__ __launch_bounds__(kCapBlock) void cap_bwd_kernel(const void* dy, u32x4* dx, int64_t n_in,
                                                            int64_t nvec)
{
    constexpr int EPV = BF16 ? 8 : 4;
    constexpr float kInv = 1.0f / (float)R;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nvec) {
        float f[EPV];
        if constexpr (R >= EPV) {
            const float g = load_elem<BF16>(dy, i * EPV / R) * kInv;
#pragma unroll
            for (int j = 0; j < EPV; ++j) f[j] = g;
        } else {
            constexpr int OUT = EPV / R;
#pragma unroll
            for (int q = 0; q < OUT; ++q) {
                const float g = load_elem<BF16>(dy, i * OUT + q) * kInv;
#pragma unroll
                for (int j = 0; j < R; ++j) f[q * R + j] = g;
            }
        }
        u32x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = BF16 ? pack_bf16(f[2 * j], f[2 * j + 1]) : as_u32(f[j]);
        stream_store128(dx + i, v);
    } else if (i == nvec) {
        for (int64_t e = nvec * EPV; e < n_in; ++e) store_elem<BF16>(dx, e, load_elem<BF16>(dy, e / R) * kInv);
    }
}

// Any alignment: one lane per output element, grid-stride.
template <bool BF16>
__global__ __launch_bounds__(kBlock) void cap_fwd_kernel_unaligned(const void* x, void* y,
                                                                   int64_t n_out, int r)
{
    const float inv = 1.0f / (float)r;
    for (int64_t m = (int64_t)blockIdx.x * kBlock + threadIdx.x; m < n_out; m += (int64_t)gridDim.x * kBlock) {
        float acc = 0.0f;
        for (int j = 0; j < r; ++j) acc += load_elem<BF16>(x, m * r + j);
        store_elem<BF16>(y, m, acc * inv);
    }
}
template <bool BF16>
__global__ __launch_bounds__(kBlock) void cap_bwd_kernel_unaligned(const void* dy, void* dx,
                                                                   int64_t n_out, int r)
{
    const float inv = 1.0f / (float)r;
    for (int64_t m = (int64_t)blockIdx.x * kBlock + threadIdx.x; m < n_out; m += (int64_t)gridDim.x * kBlock) {
        const float g = load_elem<BF16>(dy, m) * inv;
        for (int j = 0; j < r; ++j) store_elem<BF16>(dx, m * r + j, g);
    }
}

// ------------------------------------------------ Low-Rank Prompt ----------
//
// Sec. 3.1, "Low-Rank Prompt (LRP)" paragraph, Eq. 3-4: y = x + A B with
// A [N x r], B [r x C] (fp32 parameters), the same prompt for every sample of
// the batch; dL/dx = dL/dy, dL/dA = dL/dy B^T, dL/dB = A^T dL/dy, both summed
// over the batch.  Neither x nor y is needed in backward.
//
// Forward: the prompt is never materialised in HBM.  A block is kLrpPos
// 16-byte vector positions of the sample (token i, channels c..c+EPV-1) times
// kLrpGroups lane groups; the positions are 4 token rows x 32 neighbouring
// vectors, so that the block's slab of B (r rows of 32 vectors) serves four
// tokens: with 128 vectors of one row the blocks pulled as many bytes of B out
// of L2 as of x out of HBM (forward 16.2 -> 12.8 us at [32, 257, 1664], 11.0 ->
// 10.1 us at [64, 197, 1024]; 8 x 16 is no better, 2 x 64 in between).  Group g of a position streams the
// samples g, g+G, g+2G, ... from x to y, eight 16-byte loads in flight, so the
// batch is what fills the chip (a sample holds only ~150 k elements).  The EPV
// prompt values of a position, P[i, c..] = sum_k A[i,k] B[k,c..], are shared
// work: group g adds the terms k = g, g+G, ... while its first loads of x are
// in flight, and the G partial sums meet in LDS in fixed order -- every row of
// B is read once per position, not once per lane.  HBM traffic: x once, y once.
//
// Backward: G = sum_b dL/dy[b] comes from one pass over dL/dy (G goes to an N*C
// fp32 workspace), dA = G B^T and dB = A^T G from a second kernel that reads G
// out of the caches; the two products are tiny (2 N C r = 9 MFLOP each at
// ViT-B/16) next to the pass over dL/dy.
constexpr int kLrpPos = 128;
constexpr int kLrpFwdTokens = 4;                         // a block's positions: this many token rows ...
constexpr int kLrpFwdCols = kLrpPos / kLrpFwdTokens;     // ... times this many neighbouring vectors of each
constexpr int kLrpGroups = 8;
constexpr int kLrpFwdBlock = kLrpPos * kLrpGroups;
constexpr int kLrpMaxRank = 128;  // the paper's scaling study goes to rank 100 (Sec. 4.3, Fig. 5)
static_assert(kLrpMaxRank <= 2 * 8 * kLrpGroups, "the forward kernel sums the prompt in at most two rounds of 64 ranks");

template <bool BF16, int ROUNDS>
__global__ __launch_bounds__(kLrpFwdBlock) void lrp_fwd_kernel(const u32x4* x, u32x4* y,
                                                               const float* __restrict__ A,
                                                               const float* __restrict__ B,
                                                               int batch, int N, int C, int r)
{
    constexpr int EPV = BF16 ? 8 : 4;
    constexpr int U = 8;
    __shared__ __align__(16) float part[kLrpGroups][kLrpPos * EPV];
    const int pos = threadIdx.x % kLrpPos, grp = threadIdx.x / kLrpPos;
    const int vpt = C / EPV;                            // vectors per token row (the launcher checks C % EPV)
    const int64_t sample = (int64_t)N * vpt;            // vectors per sample
    const int col_tiles = (vpt + kLrpFwdCols - 1) / kLrpFwdCols;
    const int i = (int)(blockIdx.x / col_tiles) * kLrpFwdTokens + pos / kLrpFwdCols;     // token
    const int q = (int)(blockIdx.x % col_tiles) * kLrpFwdCols + pos % kLrpFwdCols;       // vector inside the token row
    const bool valid = i < N && q < vpt;
    const int64_t at = (int64_t)i * vpt + q;  // this lane's vector inside a sample
    // the first round of x is requested before the prompt values are formed: the latencies overlap
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (valid && grp + u * kLrpGroups < batch) v[u] = stream_load128(x + (int64_t)(grp + u * kLrpGroups) * sample + at);
    float p[EPV];
#pragma unroll
    for (int j = 0; j < EPV; ++j) p[j] = 0.0f;
    if (valid) {
        const int c0 = q * EPV;
        const float* Ai = A + (int64_t)i * r;
        const float* Bc = B + c0;
        const bool b_vectors = ((uintptr_t)B & 15u) == 0;  // C and c0 are multiples of EPV, so rows follow B
        // Rows of B this group has in flight at a time, and how many such stages it takes.  Ranks up
        // to 64 (ROUNDS = 1, the paper's own): 8 rows, one stage.  Above: 4 rows per stage and four
        // stages, each behind the arithmetic of the one before (its addresses are made to depend on
        // that result) -- all 16 rows at once, or 8 and 8, need more registers than a 1024-lane block
        // has, and the compiler spills to memory.  The stage count is fixed at compile time: a
        // run-time loop made the first loads of x wait at its back edge (forward 9.3 -> 13.6 us at
        // ViT-B/16).
        constexpr int KU = ROUNDS == 1 ? 8 : 4, STAGES = ROUNDS * 8 / KU;
#pragma unroll
        for (int stage = 0; stage < STAGES; ++stage) {
            int k_bias = 0;
            if (stage > 0) asm volatile("" : "+v"(k_bias) : "v"(p[0]));
            const int k0 = stage * KU * kLrpGroups + k_bias;
            float a[KU];
            u32x4 bk[KU][EPV / 4];
#pragma unroll
            for (int q = 0; q < KU; ++q) {
                const int k = k0 + grp + q * kLrpGroups;
                if (k < r) {
                    a[q] = Ai[k];
#pragma unroll
                    for (int h = 0; h < EPV / 4; ++h) {
                        const float* src = Bc + (int64_t)k * C + 4 * h;
                        if (b_vectors) bk[q][h] = *(const u32x4*)src;
                        else bk[q][h] = u32x4{as_u32(src[0]), as_u32(src[1]), as_u32(src[2]), as_u32(src[3])};
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < KU; ++q)
                if (k0 + grp + q * kLrpGroups < r) {
#pragma unroll
                    for (int j = 0; j < EPV; ++j) p[j] = __builtin_fmaf(a[q], as_f32(bk[q][j / 4][j % 4]), p[j]);
                }
        }
    }
#pragma unroll
    for (int j = 0; j < EPV; ++j) part[grp][pos * EPV + j] = p[j];
    __syncthreads();
#pragma unroll
    for (int j = 0; j < EPV; ++j) {
        float sum = part[0][pos * EPV + j];
#pragma unroll
        for (int g = 1; g < kLrpGroups; ++g) sum += part[g][pos * EPV + j];
        p[j] = sum;
    }
    if (!valid) return;
    for (int b = grp; b < batch; b += U * kLrpGroups) {
        if (b != grp) {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (b + u * kLrpGroups < batch) v[u] = stream_load128(x + (int64_t)(b + u * kLrpGroups) * sample + at);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (b + u * kLrpGroups < batch) {
                float f[EPV];
                unpack_vector<BF16>(v[u], f);
                u32x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    o[j] = BF16 ? pack_bf16(f[2 * j] + p[2 * j], f[2 * j + 1] + p[2 * j + 1]) : as_u32(f[j] + p[j]);
                stream_store128(y + (int64_t)(b + u * kLrpGroups) * sample + at, o);
            }
    }
}

// Backward, first kernel: G = sum_b dL/dy[b] in fp32, one pass over dL/dy.  A block is
// kLrpSumPos neighbouring 16-byte vector positions of the sample times kLrpSumSlices batch
// slices: slice s of a position adds the samples s, s + S, s + 2S, ... with eight loads in
// flight, and the S partial sums meet in LDS in fixed order (the result does not depend on the
// launch).  Positions, not token rows, are what is spread over the blocks: a few hundred
// 32-position chunks fill the chip evenly whatever N is (one block per token left a quarter of
// the compute units idle at N = 197 and gave one unit two blocks at N = 257).
constexpr int kLrpSumPos = 32, kLrpSumSlices = 8, kLrpSumBlock = kLrpSumPos * kLrpSumSlices;

template <bool BF16>
__global__ __launch_bounds__(kLrpSumBlock) void lrp_batch_sum_kernel(const u32x4* dy, float* __restrict__ G,
                                                                     int batch, int64_t sample)
{
    constexpr int EPV = BF16 ? 8 : 4;
    constexpr int U = 8;
    __shared__ __align__(16) float part[kLrpSumSlices][kLrpSumPos * EPV];
    const int pos = threadIdx.x % kLrpSumPos, slice = threadIdx.x / kLrpSumPos;
    const int64_t at = (int64_t)blockIdx.x * kLrpSumPos + pos;  // this lane's vector inside a sample
    float acc[EPV];
#pragma unroll
    for (int j = 0; j < EPV; ++j) acc[j] = 0.0f;
    if (at < sample) {
        const u32x4* src = dy + at;
        for (int b0 = slice; b0 < batch; b0 += kLrpSumSlices * U) {
            u32x4 t[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (b0 + u * kLrpSumSlices < batch) t[u] = stream_load128(src + (int64_t)(b0 + u * kLrpSumSlices) * sample);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (b0 + u * kLrpSumSlices < batch) {
                    float f[EPV];
                    unpack_vector<BF16>(t[u], f);
#pragma unroll
                    for (int j = 0; j < EPV; ++j) acc[j] += f[j];
                }
        }
    }
#pragma unroll
    for (int j = 0; j < EPV; ++j) part[slice][pos * EPV + j] = acc[j];
    __syncthreads();
    // kLrpSumPos * EPV sums per block, one per lane (fp32 storage: the first half of the lanes)
    const int e = threadIdx.x;
    const int64_t first = (int64_t)blockIdx.x * kLrpSumPos * EPV;
    if (e < kLrpSumPos * EPV && first + e < sample * EPV) {
        float g = part[0][e];
#pragma unroll
        for (int q = 1; q < kLrpSumSlices; ++q) g += part[q][e];
        G[first + e] = g;
    }
}

// Backward, second kernel: the two small products, from G (fp32, N x C), on the matrix cores:
//   dB[k, c] = sum_i A[i, k] G[i, c]        blocks [0, blocks_b):  16 ranks x 64 channels, all tokens
//   dA[i, k] = sum_c G[i, c] B[k, c]        the rest:              16 tokens x 16 ranks, all channels
// 2 N C r flops each (24 MFLOP at ViT-L/16 and rank 30, 100 MFLOP at rank 100): nothing next to
// the pass over dL/dy in arithmetic, but as vector code (a wave per (token, rank) dot product, a
// lane group per column of dB) the two took as long as that pass and twice as long at rank 100:
// every element of G went from L2 to the compute units r / 4 + r / 8 times.  With
// v_mfma_f32_16x16x4_f32 (fp32 in, fp32 accumulate) a tile of G serves 16 ranks at once, a
// block's whole share goes out in one round of 16-byte loads, 8 waves split the contraction index
// and the 8 partial tiles meet in LDS in fixed order (the result does not depend on the launch).
// What is left is latency: G was written a moment ago by other compute units, so its first touch
// here comes from beyond this XCD's L2 (1-2 us), and the launch has only 60-200 blocks.
//
// Operand layout of the instruction, lane l = 16 g + m (g = 0..3, m = 0..15):
//   a: element (row m, contraction index g)        b: element (contraction index g, column m)
//   d[v], v = 0..3: element (row 4 g + v, column m)
// The contraction index may be any bijection of the real one as long as a and b use the same,
// which is what lets a lane feed the four components of one 16-byte vector to four instructions.
//   dB: rows = ranks, contraction = tokens, columns = channels.  A lane loads G[token][c0 + 4 m .. + 3]
//       and instruction t takes component t: column m of accumulator t is channel c0 + 4 m + t, so
//       a wave covers 64 channels and reads 256 contiguous bytes of each of its tokens' rows.
//   dA: rows = tokens, contraction = channels, columns = ranks: instruction (s, t) contracts the
//       channels cb + 16 g + 4 s + t, g = 0..3, of the rows G[i0 + m] and B[k0 + m].
// Rows, columns and contraction indices past the end are fed zeros (both operands where it is the
// contraction index, so that nothing non-finite meets a zero there).  Blocks that share rows of G
// (dA) or a slab of its columns (dB) are numbered so that they run on the same XCD.
constexpr int kXcds = 8;  // accelerator dies; block b of a grid runs on die b % 8
constexpr int kLrpAbWaves = 8, kLrpAbBlock = kLrpAbWaves * kWave;
constexpr int kLrpTile = 16;                 // rows and columns of one matrix-core tile
constexpr int kLrpDbChannels = 4 * kLrpTile; // a dB block's channels: four tiles, interleaved
constexpr int kLrpDaChunk = 64;              // channels a wave contracts per round of four vectors

// Straight-line code matters here: around a load that sits under a run-time condition the
// compiler waits for every outstanding load at the join, which puts the rounds of loads in
// series.  So nothing is loaded conditionally: an address past the end is replaced by one inside
// and the value by zero, the alignment case and the number of rounds are template parameters, and
// the kernel picks the instantiation once, at its top.
template <bool VEC>
__device__ __forceinline__ float4 load_f32x4(const float* p, bool live)
{
    float4 v;
    if constexpr (VEC) v = *(const float4*)p;
    else v = float4{p[0], p[1], p[2], p[3]};
    return float4{live ? v.x : 0.0f, live ? v.y : 0.0f, live ? v.z : 0.0f, live ? v.w : 0.0f};
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 mfma_16x16x4(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

constexpr int kLrpDbQuads = 8;   // token quads in flight per wave: 256 tokens per round of a dB block
constexpr int kLrpDaChunks = 2;  // 64-channel chunks in flight per wave: 1024 channels per round of a dA block
// (9 quads and 4 chunks, which put N = 257 and C = 1664 into one round, gain 4 % there and cost
// 10 % at N = 197, C = 1024: the slots past the end still issue their loads)

// ---- dB: ranks k0 .. k0 + 15, channels c0 .. c0 + 63; wave w takes the token quads w, w + 8, ...
// ROUNDS > 0: that many rounds of 256 tokens, unrolled; 0: as many as N needs.
template <int ROUNDS, bool VEC>
__device__ __forceinline__ void lrp_db_tile(const float* __restrict__ G, const float* __restrict__ A,
                                            float* __restrict__ dB, float (*part)[4][kWave][4], int N, int C, int r,
                                            int k0, int c0)
{
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // the same in every lane: conditions on it are scalar
    const int m = lane % kLrpTile, g = lane / kLrpTile;
    const bool col_live = c0 + 4 * m < C, row_live = k0 + m < r;  // C % 4 == 0: a vector is inside or outside as a whole
    const float* Gc = G + (col_live ? c0 + 4 * m : c0);
    const float* Ak = A + (row_live ? k0 + m : 0);
    const f32x4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
    f32x4 acc[4] = {zero, zero, zero, zero};
    const int quads = (N + 3) / 4;
    constexpr int STEP = kLrpAbWaves * kLrpDbQuads;
    auto one_round = [&](int round) {
        float4 gv[kLrpDbQuads];
        float av[kLrpDbQuads];
#pragma unroll
        for (int u = 0; u < kLrpDbQuads; ++u) {
            const int64_t i = 4 * ((int64_t)round * STEP + wave + kLrpAbWaves * u) + g;
            const bool in = i < N;
            const int64_t ii = in ? i : 0;
            gv[u] = load_f32x4<VEC>(Gc + ii * C, in && col_live);
            const float a = Ak[ii * r];
            av[u] = in && row_live ? a : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < kLrpDbQuads; ++u) {
            if ((int64_t)round * STEP + wave + kLrpAbWaves * u >= quads) continue;  // the whole wave: nothing but zeros
            acc[0] = mfma_16x16x4(av[u], gv[u].x, acc[0]);
            acc[1] = mfma_16x16x4(av[u], gv[u].y, acc[1]);
            acc[2] = mfma_16x16x4(av[u], gv[u].z, acc[2]);
            acc[3] = mfma_16x16x4(av[u], gv[u].w, acc[3]);
        }
    };
    if constexpr (ROUNDS > 0) {
#pragma unroll
        for (int round = 0; round < ROUNDS; ++round) one_round(round);
    } else {
        for (int round = 0; (int64_t)round * STEP < quads; ++round) one_round(round);
    }
    // accumulator t, register v of lane (g, m): rank k0 + 4 g + v, channel c0 + 4 m + t
#pragma unroll
    for (int v = 0; v < 4; ++v) *(float4*)part[wave][v][lane] = float4{acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
    __syncthreads();
    if (tid < 4 * kWave) {
        const int v = tid / kWave, l = tid % kWave, k = k0 + 4 * (l / kLrpTile) + v, cc = c0 + 4 * (l % kLrpTile);
        float4 sum = *(const float4*)part[0][v][l];
#pragma unroll
        for (int w = 1; w < kLrpAbWaves; ++w) {
            const float4 p = *(const float4*)part[w][v][l];
            sum.x += p.x, sum.y += p.y, sum.z += p.z, sum.w += p.w;
        }
        if (k < r && cc < C) {
            float* out = dB + (int64_t)k * C + cc;
            if (((uintptr_t)dB & 15u) == 0) *(float4*)out = sum;
            else out[0] = sum.x, out[1] = sum.y, out[2] = sum.z, out[3] = sum.w;
        }
    }
}

// ---- dA: tokens i0 .. i0 + 15, ranks k0 .. k0 + 15; wave w takes the 64-channel chunks w, w + 8, ...
// ROUNDS > 0: that many rounds of 1024 channels, unrolled; 0: as many as C needs.
// Both operands have the contraction index (channels) along their rows, and the instruction wants
// neighbouring lanes on neighbouring ROWS: fetched that way a wave-wide load is 64 separate 16-byte
// pieces, and the address unit, which takes them one line at a time, becomes what the kernel waits
// for (measured: the kernel's time followed the number of such loads, real or masked).  So a wave
// fetches its 16 x 64 tile the way memory likes it -- 16 lanes along 256 contiguous bytes of a
// row, four rows per load -- and turns it through a strip of LDS of its own (rows padded by 16
// bytes: both the row-wise stores and the operand-wise loads are conflict-free).  LDS
// instructions of one wave complete in order, so the strip needs no barrier, only a compiler
// fence between a store and the load of another lane's data.
constexpr int kLrpStageStride = kLrpDaChunk + 4;                   // floats per staged row
constexpr int kLrpStageFloats = kLrpTile * kLrpStageStride;        // per wave

__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int ROUNDS, bool VEC>
__device__ __forceinline__ void lrp_da_tile(const float* __restrict__ G, const float* __restrict__ B,
                                            float* __restrict__ dA, float* lds, int N, int C, int r, int i0, int k0)
{
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);  // the same in every lane: conditions on it are scalar
    const int m = lane % kLrpTile, g = lane / kLrpTile;
    float* stage = lds + wave * kLrpStageFloats;
    // fetch: lane (g, m) takes rows g, g + 4, g + 8, g + 12 of the tile, channels 4 m .. 4 m + 3 of the chunk
    const float* Grow[4];
    const float* Brow[4];
    bool tok_live[4], rank_live[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        tok_live[j] = i0 + 4 * j + g < N;
        rank_live[j] = k0 + 4 * j + g < r;
        Grow[j] = G + (int64_t)(tok_live[j] ? i0 + 4 * j + g : 0) * C;
        Brow[j] = B + (int64_t)(rank_live[j] ? k0 + 4 * j + g : 0) * C;
    }
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    constexpr int STEP = kLrpAbWaves * kLrpDaChunks * kLrpDaChunk;
    auto one_round = [&](int round) {
        float4 gv[kLrpDaChunks][4], bv[kLrpDaChunks][4];
#pragma unroll
        for (int u = 0; u < kLrpDaChunks; ++u) {
            const int64_t ch = (int64_t)round * STEP + (wave + kLrpAbWaves * u) * kLrpDaChunk + 4 * m;
            const bool in = ch < C;
            const int64_t at = in ? ch : 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                gv[u][j] = load_f32x4<VEC>(Grow[j] + at, in && tok_live[j]);
                bv[u][j] = load_f32x4<VEC>(Brow[j] + at, in && rank_live[j]);
            }
        }
#pragma unroll
        for (int u = 0; u < kLrpDaChunks; ++u) {
            if ((int64_t)round * STEP + (wave + kLrpAbWaves * u) * kLrpDaChunk >= C) continue;  // the whole wave: nothing but zeros
            float4 ga[4], ba[4];
            // operand: lane (g, m) takes row m, channels 16 g + 4 s .. + 3 of the chunk for instruction group s
#pragma unroll
            for (int j = 0; j < 4; ++j) *(float4*)&stage[(4 * j + g) * kLrpStageStride + 4 * m] = gv[u][j];
            wave_lds_fence();
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) ga[s4] = *(const float4*)&stage[m * kLrpStageStride + 16 * g + 4 * s4];
            wave_lds_fence();
#pragma unroll
            for (int j = 0; j < 4; ++j) *(float4*)&stage[(4 * j + g) * kLrpStageStride + 4 * m] = bv[u][j];
            wave_lds_fence();
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) ba[s4] = *(const float4*)&stage[m * kLrpStageStride + 16 * g + 4 * s4];
            wave_lds_fence();
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                acc = mfma_16x16x4(ga[s4].x, ba[s4].x, acc);
                acc = mfma_16x16x4(ga[s4].y, ba[s4].y, acc);
                acc = mfma_16x16x4(ga[s4].z, ba[s4].z, acc);
                acc = mfma_16x16x4(ga[s4].w, ba[s4].w, acc);
            }
        }
    };
    if constexpr (ROUNDS > 0) {
#pragma unroll
        for (int round = 0; round < ROUNDS; ++round) one_round(round);
    } else {
        for (int round = 0; (int64_t)round * STEP < C; ++round) one_round(round);
    }
    // register v of lane (g, m): token i0 + 4 g + v, rank k0 + m
    __syncthreads();  // every wave is done with its strip: the partial tiles go over the same memory
    float(*part)[kWave][4] = (float(*)[kWave][4])lds;
    *(float4*)part[wave][lane] = float4{acc[0], acc[1], acc[2], acc[3]};
    __syncthreads();
    if (tid < 4 * kWave) {
        const int v = tid % 4, l = tid / 4;  // the four registers of a lane side by side, as they lie in LDS
        float sum = part[0][l][v];
#pragma unroll
        for (int w = 1; w < kLrpAbWaves; ++w) sum += part[w][l][v];
        const int i = i0 + 4 * (l / kLrpTile) + v, k = k0 + l % kLrpTile;
        if (i < N && k < r) dA[(int64_t)i * r + k] = sum;
    }
}

__global__ __launch_bounds__(kLrpAbBlock) void lrp_grad_ab_kernel(const float* __restrict__ G,
                                                                  const float* __restrict__ A,
                                                                  const float* __restrict__ B,
                                                                  float* __restrict__ dA, float* __restrict__ dB,
                                                                  int N, int C, int r, int blocks_b)
{
    constexpr int PART = kLrpAbWaves * 4 * kWave * 4, STAGE = kLrpAbWaves * kLrpStageFloats;
    __shared__ __align__(16) float lds[PART > STAGE ? PART : STAGE];  // 34 KB: dB's partial tiles, or dA's strips
    const int ktiles = (r + kLrpTile - 1) / kLrpTile;
    const bool vec = (((uintptr_t)G | (uintptr_t)B) & 15u) == 0;  // rows are whole vectors: C % 4 == 0
    if ((int)blockIdx.x < blocks_b) {
        const int b = blockIdx.x;
        const int k0 = ((b / kXcds) % ktiles) * kLrpTile;
        const int c0 = ((b / kXcds / ktiles) * kXcds + b % kXcds) * kLrpDbChannels;
        if (c0 >= C) return;  // slabs rounded up to whole groups of 8 (the whole block, before any barrier)
        constexpr int TOKENS = 4 * kLrpAbWaves * kLrpDbQuads;  // per round
        if (!vec) lrp_db_tile<0, false>(G, A, dB, (float(*)[4][kWave][4])lds, N, C, r, k0, c0);
        else if (N <= TOKENS) lrp_db_tile<1, true>(G, A, dB, (float(*)[4][kWave][4])lds, N, C, r, k0, c0);
        else if (N <= 2 * TOKENS) lrp_db_tile<2, true>(G, A, dB, (float(*)[4][kWave][4])lds, N, C, r, k0, c0);
        else lrp_db_tile<0, true>(G, A, dB, (float(*)[4][kWave][4])lds, N, C, r, k0, c0);
        return;
    }
    const int ba = blockIdx.x - blocks_b;
    const int k0 = ((ba / kXcds) % ktiles) * kLrpTile;
    const int i0 = ((ba / kXcds / ktiles) * kXcds + ba % kXcds) * kLrpTile;
    if (i0 >= N) return;  // token tiles rounded up to whole groups of 8
    constexpr int CHANNELS = kLrpAbWaves * kLrpDaChunks * kLrpDaChunk;  // per round
    if (!vec) lrp_da_tile<0, false>(G, B, dA, lds, N, C, r, i0, k0);
    else if (C <= CHANNELS) lrp_da_tile<1, true>(G, B, dA, lds, N, C, r, i0, k0);
    else if (C <= 2 * CHANNELS) lrp_da_tile<2, true>(G, B, dA, lds, N, C, r, i0, k0);
    else if (C <= 4 * CHANNELS) lrp_da_tile<4, true>(G, B, dA, lds, N, C, r, i0, k0);
    else lrp_da_tile<0, true>(G, B, dA, lds, N, C, r, i0, k0);
}

// ------------------------------------------------- measurement aid --------
// The activation kernels' skeleton with the arithmetic taken out.
__global__ __launch_bounds__(kWave) void stream_copy_kernel(const u32x4* src, u32x4* dst, int64_t nvec)
{
    const int64_t i = (int64_t)blockIdx.x * kWave + threadIdx.x;
    if (i < nvec) stream_store128(dst + i, stream_load128(src + i));
}
// The same with the packed codes' share of the traffic: SIDE bytes per lane written after the
// vector (forward shape) or read with it (backward shape; folded into the data so that the load
// is not dead).
template <int SIDE, bool SIDE_IN>
__global__ __launch_bounds__(kWave) void stream_copy_shaped_kernel(const u32x4* src, u32x4* dst, uint8_t* side,
                                                                   int64_t nvec)
{
    const int64_t i = (int64_t)blockIdx.x * kWave + threadIdx.x;
    if (i < nvec) {
        u32x4 v = stream_load128(src + i);
        if (SIDE_IN) {
            v[0] ^= load_codes<SIDE == 4>(side, i);
            stream_store128(dst + i, v);
        } else {
            stream_store128(dst + i, v);
            store_codes<SIDE == 4>(side, i, v[0] ^ v[2]);
        }
    }
}

}  // namespace s2a
