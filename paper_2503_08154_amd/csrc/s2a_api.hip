// s2a_api.hip -- host side of the C ABI declared in include/s2a.h: argument
// checks, the quantization table, kernel selection and launch.  No device
// memory is allocated and nothing synchronizes.
#include "s2a.h"
#include "s2a_bench.h"

#include <math.h>

#include <mutex>
#include <type_traits>

#include "s2a_kernels.hpp"

// Library-owned working memory for s2a_lrp_bwd_noalloc: part of the loaded code object, so every
// GPU the library runs on holds its own copy (4 MiB) at its own address until the process ends.
// In host code the name below is only a handle for hipGetSymbolAddress, never an address:
// kernels receive the looked-up pointer (scratch_on_current_device).
static __device__ __align__(256) float scratch[S2A_LRP_NOALLOC_MAX_FLOATS];

namespace {

struct TableState {
    bool ready = false;
    s2a::QTable dev;   // fp32 derivative levels handed to kernels by value
    s2a::QTable silu;  // the same for SiLU: Eq. 12 under x -> x / 1.702
    float xhat[16];
    float bounds[15];
};
TableState g_table;

// Sec. 3.2, GeLU paragraph: representatives of Eq. 9 on the clip range
// [-2, 2] with 2^4 levels, and Eq. 12 evaluated at each of them.
void build_table(TableState& t)
{
    const double lo = -2.0, hi = 2.0;
    const double step = (hi - lo) / 15.0;
    for (int k = 0; k < 16; ++k) {
        double xh = lo + step * (double)k;
        double d = 1.0 / (1.0 + exp(-1.702 * xh)) + 0.22 * sin(1.5 * xh);
        t.xhat[k] = (float)xh;
        t.dev.d[k] = (float)d;
        // SiLU(x) = 1.702 * GELU(x / 1.702): representatives 1.702 * xh, same derivative formula in xh
        // written in the SiLU variable: sigma(xs) + 0.22 sin(1.5 xs / 1.702), xs = 1.702 * xh
        double xs = 1.702 * xh;
        t.silu.d[k] = (float)(1.0 / (1.0 + exp(-xs)) + 0.22 * sin(1.5 * xs / 1.702));
    }
    for (int j = 0; j < 15; ++j) t.bounds[j] = (float)(lo + step * ((double)j + 0.5));
    t.ready = true;
}

int check_args(const void* a, const void* b, const void* c, int64_t n, int dtype)
{
    if (dtype != S2A_F32 && dtype != S2A_BF16) return S2A_ERR_DTYPE;
    if (n < 0) return S2A_ERR_SIZE;
    if (n > 0 && (!a || !b || !c)) return S2A_ERR_NULL;
    return S2A_OK;
}

int check_common(const void* a, const void* b, const void* c, int64_t n, int dtype)
{
    if (!g_table.ready) return S2A_ERR_NOT_INIT;
    return check_args(a, b, c, n, dtype);
}

bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// Blocks of the element-wise kernels: enough to fill the chip, grid-stride beyond.
unsigned pair_grid(int64_t n)
{
    int64_t pairs = (n + 1) / 2;
    int64_t blocks = (pairs + s2a::kBlock - 1) / s2a::kBlock;
    const int64_t cap = 256 * 32;
    return (unsigned)(blocks < cap ? blocks : cap);
}

// Runs `launch` and turns the runtime's verdict into a return code.  Any stale
// error left by earlier, unrelated runtime calls is dropped first.
template <typename F>
int checked_launch(F launch)
{
    (void)hipGetLastError();
    launch();
    return hipGetLastError() == hipSuccess ? S2A_OK : S2A_ERR_LAUNCH;
}

// Blocks of the vector kernels: one wave per 64 vectors (plus one slot for the leftover elements).
template <bool BF16>
bool vector_grid(int64_t n, int64_t* nvec, unsigned* blocks)
{
    constexpr int EPV = BF16 ? 8 : 4;
    *nvec = n / EPV;
    int64_t slots = *nvec + (n % EPV != 0);
    int64_t b = (slots + s2a::kWave - 1) / s2a::kWave;
    if (b > 0x7fffffffLL) return false;
    *blocks = (unsigned)b;
    return true;
}

// DYN: the kernel's first wave also completes qstate, so at least one block runs even for n == 0.
template <bool BF16, bool DYN, int ACT = s2a::kActGelu>
int launch_fwd(const void* x, void* y, uint8_t* codes, float* qs, int64_t n, hipStream_t st)
{
    if (aligned(x, 16) && aligned(y, 16) && aligned(codes, 4)) {
        int64_t nvec;
        unsigned blocks;
        if (!vector_grid<BF16>(n, &nvec, &blocks)) return S2A_ERR_SIZE;
        if (DYN && blocks == 0) blocks = 1;
        return checked_launch([&] {
            if constexpr (DYN)
                s2a::fwd_dyn_kernel<BF16><<<dim3(blocks), dim3(s2a::kWave), 0, st>>>(
                    (const s2a::u32x4*)x, (s2a::u32x4*)y, codes, qs, n, nvec);
            else
                s2a::fwd_kernel<BF16, ACT><<<dim3(blocks), dim3(s2a::kWave), 0, st>>>(
                    (const s2a::u32x4*)x, (s2a::u32x4*)y, codes, n, nvec);
        });
    }
    unsigned blocks = pair_grid(n);
    if (DYN && blocks == 0) blocks = 1;
    return checked_launch([&] {
        s2a::fwd_kernel_unaligned<BF16, DYN, ACT><<<dim3(blocks), dim3(s2a::kBlock), 0, st>>>(x, y, codes, qs, n);
    });
}

template <bool BF16, bool DYN>
int launch_bwd(const void* dy, const uint8_t* codes, void* dx, const float* qs, int64_t n,
               hipStream_t st, const s2a::QTable& table = g_table.dev)
{
    if (aligned(dy, 16) && aligned(dx, 16) && aligned(codes, 4)) {
        int64_t nvec;
        unsigned blocks;
        if (!vector_grid<BF16>(n, &nvec, &blocks)) return S2A_ERR_SIZE;
        // codes that are 16-byte aligned (not only 4) are fetched a wave at a time
        const bool wave_codes = aligned(codes, 16);
        return checked_launch([&] {
            if (wave_codes)
                s2a::bwd_kernel<BF16, DYN, true><<<dim3(blocks), dim3(s2a::kWave), 0, st>>>(
                    (const s2a::u32x4*)dy, codes, (s2a::u32x4*)dx, table, qs, n, nvec);
            else
                s2a::bwd_kernel<BF16, DYN, false><<<dim3(blocks), dim3(s2a::kWave), 0, st>>>(
                    (const s2a::u32x4*)dy, codes, (s2a::u32x4*)dx, table, qs, n, nvec);
        });
    }
    return checked_launch([&] {
        s2a::bwd_kernel_unaligned<BF16, DYN><<<dim3(pair_grid(n)), dim3(s2a::kBlock), 0, st>>>(
            dy, codes, dx, table, qs, n);
    });
}

// The launch that measures the range of x: per-block minima and maxima into qstate.
template <bool BF16>
int launch_range(const void* x, float* qs, int64_t n, hipStream_t st)
{
    constexpr int EPV = BF16 ? 8 : 4;
    const bool al = aligned(x, 16);
    int64_t items = al ? n / EPV + 1 : n;
    int64_t blocks = (items + s2a::kRangeBlock - 1) / s2a::kRangeBlock;
    if (blocks > s2a::kRangeBlocks) blocks = s2a::kRangeBlocks;  // grid-stride beyond
    if (blocks < 1) blocks = 1;
    return checked_launch([&] {
        if (al)
            s2a::range_minmax_kernel<BF16, true><<<dim3((unsigned)blocks), dim3(s2a::kRangeBlock), 0, st>>>(x, qs, n);
        else
            s2a::range_minmax_kernel<BF16, false><<<dim3((unsigned)blocks), dim3(s2a::kRangeBlock), 0, st>>>(x, qs, n);
    });
}

template <bool BF16>
int launch_relu_fwd(const void* x, void* y, uint8_t* mask, int64_t n, hipStream_t st)
{
    if (aligned(x, 16) && aligned(y, 16)) {
        int64_t nvec;
        unsigned blocks;
        if (!vector_grid<BF16>(n, &nvec, &blocks)) return S2A_ERR_SIZE;
        return checked_launch([&] {
            s2a::relu_fwd_kernel<BF16><<<dim3(blocks), dim3(s2a::kWave), 0, st>>>(
                (const s2a::u32x4*)x, (s2a::u32x4*)y, mask, n, nvec);
        });
    }
    return checked_launch([&] {
        s2a::relu_fwd_kernel_unaligned<BF16><<<dim3(pair_grid(n / 4 + 1)), dim3(s2a::kBlock), 0, st>>>(x, y, mask, n);
    });
}

template <bool BF16>
int launch_relu_bwd(const void* dy, const uint8_t* mask, void* dx, int64_t n, hipStream_t st)
{
    if (aligned(dy, 16) && aligned(dx, 16)) {
        int64_t nvec;
        unsigned blocks;
        if (!vector_grid<BF16>(n, &nvec, &blocks)) return S2A_ERR_SIZE;
        return checked_launch([&] {
            s2a::relu_bwd_kernel<BF16><<<dim3(blocks), dim3(s2a::kWave), 0, st>>>(
                (const s2a::u32x4*)dy, mask, (s2a::u32x4*)dx, n, nvec);
        });
    }
    return checked_launch([&] {
        s2a::relu_bwd_kernel_unaligned<BF16><<<dim3(pair_grid(n / 4 + 1)), dim3(s2a::kBlock), 0, st>>>(dy, mask, dx, n);
    });
}

// Lanes per softmax row: the smallest group whose lanes hold at most kSoftmaxSlots elements each.
int softmax_group(int64_t L)
{
    for (int g = 8; g <= 64; g *= 2)
        if ((L + g - 1) / g <= s2a::kSoftmaxSlots) return g;
    return 0;
}

// The staged kernels (16-byte aligned buffers) give each lane element pairs:
// G lanes per row, the smallest of 4 .. 64 whose lanes hold at most
// pair_slots() pairs each, and exactly ceil(pairs / G) slots compiled in.
// Slot limit by measurement at the ViT-B/16 attention shape (197-long rows):
// bf16 runs fastest with 8 lanes x 13 pairs, fp32 with 16 lanes x 7 pairs.
template <bool BF16>
constexpr int pair_slots() { return BF16 ? 16 : 8; }
// How many rows of one wave meet in the same LDS bank (64 banks of 4 bytes) when every lane
// reads one pair: row r of the wave starts r * row_bytes into the span and its G lanes cover
// G * pair_bytes from there.
int lds_row_conflicts(int64_t row_bytes, int g, int pair_bytes)
{
    int hits[64] = {0};
    int worst = 0;
    for (int r = 0; r < 64 / g; ++r) {
        const int64_t a = r * row_bytes, b = a + (int64_t)g * pair_bytes - 1;
        for (int64_t w = a / 4; w <= b / 4; ++w)
            if (++hits[w % 64] > worst) worst = hits[w % 64];
    }
    return worst;
}
template <bool BF16>
int softmax_pair_group(int64_t L)
{
    const int64_t pairs = (L + 1) / 2;
    const int es = BF16 ? 2 : 4, gmax = BF16 ? 32 : 64;
    int g = 4;
    while (g <= gmax && (pairs + g - 1) / g > pair_slots<BF16>()) g *= 2;
    if (g > gmax) return 0;
    // rows whose length puts more than four rows of a wave on the same banks (powers of two and
    // their neighbours) take a group twice as wide, i.e. half the rows per wave.  Measured, bf16:
    // L = 64: 31 -> 25 us for 118 MB; L = 128: 48 -> 33 us for 175 MB; L = 256: 34 -> 31.5 us;
    // a second doubling loses more in per-wave work than it gains.
    if (2 * g <= gmax && lds_row_conflicts(L * es, g, 2 * es) > 4 &&
        lds_row_conflicts(L * es, 2 * g, 2 * es) < lds_row_conflicts(L * es, g, 2 * es))
        g *= 2;
    return g;
}

// LDS bytes of one staged softmax block: the data span (+ up to 15 bytes of
// lead-in and padding to a vector), then the codes span.
// Lanes per block of the staged kernels: 256 measured fastest of 64 .. 1024.
constexpr int kStagedBlock = 256;
template <bool BF16, int G>
void softmax_lds(int L, int* data_bytes, int* total_bytes)
{
    const int rpb = kStagedBlock / G, es = BF16 ? 2 : 4;
    *data_bytes = ((rpb * L * es + 15 + 15) / 16) * 16;
    *total_bytes = *data_bytes + ((rpb * ((L + 1) / 2) + 15 + 15) / 16) * 16;
}

// Compute units of the current device (0 if the runtime does not say), looked up once per device.
// Threads that race on the first call store the same value.
int device_units()
{
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = -1;
        cached[dev] = n;
    }
    return cached[dev] > 0 ? cached[dev] : 0;
}
// The staged kernels stagger their first round of blocks (see stagger_first_round) when the
// launch has at least two rounds of kStaggerSlots blocks per compute unit.
int stagger_units(int64_t blocks)
{
    const int units = device_units();
    return units > 0 && blocks >= 2LL * s2a::kStaggerSlots * units ? units : 0;
}

// Calls f(std::integral_constant<int, SLOTS>) for SLOTS == slots.
template <int G, int MAXS, int S = MAXS, typename F>
void with_slots(int slots, F f)
{
    if (slots == S) f(std::integral_constant<int, S>{});
    else if constexpr (S > 1) with_slots<G, MAXS, S - 1>(slots, f);
}

template <bool BF16, int G>
int launch_softmax_fwd_staged(const void* x, void* y, uint8_t* codes, float* qp, int64_t rows, int L,
                              hipStream_t st)
{
    const int rpb = kStagedBlock / G;
    const int64_t blocks = (rows + rpb - 1) / rpb;
    if (blocks > 0x7fffffffLL) return S2A_ERR_SIZE;
    int data_bytes, total;
    softmax_lds<BF16, G>(L, &data_bytes, &total);
    const int stagger = stagger_units(blocks);
    return checked_launch([&] {
        with_slots<G, pair_slots<BF16>()>(((L + 1) / 2 + G - 1) / G, [&](auto sc) {
            s2a::softmax_fwd_staged<BF16, G, decltype(sc)::value, kStagedBlock>
                <<<dim3((unsigned)blocks), dim3(kStagedBlock), total, st>>>(x, y, codes, qp, rows, L, data_bytes, stagger);
        });
    });
}
template <bool BF16, int G>
int launch_softmax_bwd_staged(const void* dy, const uint8_t* codes, const float* qp, void* dx,
                              int64_t rows, int L, hipStream_t st)
{
    const int rpb = kStagedBlock / G;
    const int64_t blocks = (rows + rpb - 1) / rpb;
    if (blocks > 0x7fffffffLL) return S2A_ERR_SIZE;
    int data_bytes, total;
    softmax_lds<BF16, G>(L, &data_bytes, &total);
    const int stagger = stagger_units(blocks);
    return checked_launch([&] {
        with_slots<G, pair_slots<BF16>()>(((L + 1) / 2 + G - 1) / G, [&](auto sc) {
            s2a::softmax_bwd_staged<BF16, G, decltype(sc)::value, kStagedBlock>
                <<<dim3((unsigned)blocks), dim3(kStagedBlock), total, st>>>(dy, codes, qp, dx, rows, L, data_bytes, stagger);
        });
    });
}

template <bool BF16, int G>
int launch_softmax_fwd_g(const void* x, void* y, uint8_t* codes, float* qp, int64_t rows, int L,
                         hipStream_t st)
{
    const int rpb = s2a::kSoftmaxBlock / G;
    const int64_t blocks = (rows + rpb - 1) / rpb;
    if (blocks > 0x7fffffffLL) return S2A_ERR_SIZE;
    return checked_launch([&] {
        s2a::softmax_fwd_kernel<BF16, G><<<dim3((unsigned)blocks), dim3(s2a::kSoftmaxBlock), 0, st>>>(
            x, y, codes, qp, rows, L);
    });
}
template <bool BF16, int G>
int launch_softmax_bwd_g(const void* dy, const uint8_t* codes, const float* qp, void* dx,
                         int64_t rows, int L, hipStream_t st)
{
    const int rpb = s2a::kSoftmaxBlock / G;
    const int64_t blocks = (rows + rpb - 1) / rpb;
    if (blocks > 0x7fffffffLL) return S2A_ERR_SIZE;
    return checked_launch([&] {
        s2a::softmax_bwd_kernel<BF16, G><<<dim3((unsigned)blocks), dim3(s2a::kSoftmaxBlock), 0, st>>>(
            dy, codes, qp, dx, rows, L);
    });
}
template <bool BF16>
int launch_softmax_fwd(const void* x, void* y, uint8_t* codes, float* qp, int64_t rows, int L,
                       hipStream_t st)
{
    if (L > s2a::kSoftmaxShortL) {
        if (rows > 0x7fffffffLL) return S2A_ERR_SIZE;
        return checked_launch([&] {
            s2a::softmax_fwd_long_kernel<BF16><<<dim3((unsigned)rows), dim3(s2a::kSoftmaxBlock), 0, st>>>(x, y, codes, qp, L);
        });
    }
    if (aligned(x, 16) && aligned(y, 16) && aligned(codes, 16))
        switch (softmax_pair_group<BF16>(L)) {
            case 4: return launch_softmax_fwd_staged<BF16, 4>(x, y, codes, qp, rows, L, st);
            case 8: return launch_softmax_fwd_staged<BF16, 8>(x, y, codes, qp, rows, L, st);
            case 16: return launch_softmax_fwd_staged<BF16, 16>(x, y, codes, qp, rows, L, st);
            case 32: return launch_softmax_fwd_staged<BF16, 32>(x, y, codes, qp, rows, L, st);
            case 64:  // only rows of fp32 reach 64 lanes
                if constexpr (!BF16) return launch_softmax_fwd_staged<BF16, 64>(x, y, codes, qp, rows, L, st);
                return S2A_ERR_SIZE;
            default: return S2A_ERR_SIZE;
        }
    switch (softmax_group(L)) {
        case 8: return launch_softmax_fwd_g<BF16, 8>(x, y, codes, qp, rows, L, st);
        case 16: return launch_softmax_fwd_g<BF16, 16>(x, y, codes, qp, rows, L, st);
        case 32: return launch_softmax_fwd_g<BF16, 32>(x, y, codes, qp, rows, L, st);
        case 64: return launch_softmax_fwd_g<BF16, 64>(x, y, codes, qp, rows, L, st);
        default: return S2A_ERR_SIZE;
    }
}
template <bool BF16>
int launch_softmax_bwd(const void* dy, const uint8_t* codes, const float* qp, void* dx,
                       int64_t rows, int L, hipStream_t st)
{
    if (L > s2a::kSoftmaxShortL) {
        if (rows > 0x7fffffffLL) return S2A_ERR_SIZE;
        return checked_launch([&] {
            s2a::softmax_bwd_long_kernel<BF16><<<dim3((unsigned)rows), dim3(s2a::kSoftmaxBlock), 0, st>>>(dy, codes, qp, dx, L);
        });
    }
    if (aligned(dy, 16) && aligned(dx, 16) && aligned(codes, 16))
        switch (softmax_pair_group<BF16>(L)) {
            case 4: return launch_softmax_bwd_staged<BF16, 4>(dy, codes, qp, dx, rows, L, st);
            case 8: return launch_softmax_bwd_staged<BF16, 8>(dy, codes, qp, dx, rows, L, st);
            case 16: return launch_softmax_bwd_staged<BF16, 16>(dy, codes, qp, dx, rows, L, st);
            case 32: return launch_softmax_bwd_staged<BF16, 32>(dy, codes, qp, dx, rows, L, st);
            case 64:  // only rows of fp32 reach 64 lanes
                if constexpr (!BF16) return launch_softmax_bwd_staged<BF16, 64>(dy, codes, qp, dx, rows, L, st);
                return S2A_ERR_SIZE;
            default: return S2A_ERR_SIZE;
        }
    switch (softmax_group(L)) {
        case 8: return launch_softmax_bwd_g<BF16, 8>(dy, codes, qp, dx, rows, L, st);
        case 16: return launch_softmax_bwd_g<BF16, 16>(dy, codes, qp, dx, rows, L, st);
        case 32: return launch_softmax_bwd_g<BF16, 32>(dy, codes, qp, dx, rows, L, st);
        case 64: return launch_softmax_bwd_g<BF16, 64>(dy, codes, qp, dx, rows, L, st);
        default: return S2A_ERR_SIZE;
    }
}

int check_softmax(const void* a, const void* b, const void* c, const void* d, int64_t rows,
                  int64_t L, int dtype)
{
    if (dtype != S2A_F32 && dtype != S2A_BF16) return S2A_ERR_DTYPE;
    if (rows < 0 || L < 1 || L > s2a::kSoftmaxMaxL) return S2A_ERR_SIZE;
    if (rows > 0 && (!a || !b || !c || !d)) return S2A_ERR_NULL;
    if (((uintptr_t)d & 3u) != 0) return S2A_ERR_ALIGN;
    return S2A_OK;
}

template <bool BF16, int R>
int launch_cap_g(bool fwd, const void* in, void* out, int64_t n_out, hipStream_t st)
{
    constexpr int EPV = BF16 ? 8 : 4;
    const int64_t n_in = n_out * R;
    const int64_t nvec = n_in / EPV;
    const int64_t slots = nvec + (n_in % EPV != 0);
    const int bs = s2a::kCapBlock;
    const int64_t per = fwd ? (int64_t)bs * s2a::kCapFwdVectors : bs;  // vectors per block
    const int64_t blocks = (slots + per - 1) / per;
    if (blocks > 0x7fffffffLL) return S2A_ERR_SIZE;
    return checked_launch([&] {
        if (fwd)
            s2a::cap_fwd_kernel<BF16, R, s2a::kCapFwdVectors><<<dim3((unsigned)blocks), dim3(bs), 0, st>>>(
                (const s2a::u32x4*)in, out, n_in, nvec);
        else
            s2a::cap_bwd_kernel<BF16, R><<<dim3((unsigned)blocks), dim3(bs), 0, st>>>(
                in, (s2a::u32x4*)out, n_in, nvec);
    });
}

// `wide` is the r-times larger tensor (x in forward, dx in backward): it decides the vector path.
template <bool BF16>
int launch_cap(bool fwd, const void* in, void* out, const void* wide, int64_t n_out, int r, hipStream_t st)
{
    if (aligned(wide, 16)) {
        switch (r) {
            case 2: return launch_cap_g<BF16, 2>(fwd, in, out, n_out, st);
            case 4: return launch_cap_g<BF16, 4>(fwd, in, out, n_out, st);
            case 8: return launch_cap_g<BF16, 8>(fwd, in, out, n_out, st);
            case 16: return launch_cap_g<BF16, 16>(fwd, in, out, n_out, st);
            case 32: return launch_cap_g<BF16, 32>(fwd, in, out, n_out, st);
            case 64: return launch_cap_g<BF16, 64>(fwd, in, out, n_out, st);
            default: return S2A_ERR_SIZE;
        }
    }
    return checked_launch([&] {
        if (fwd)
            s2a::cap_fwd_kernel_unaligned<BF16><<<dim3(pair_grid(2 * n_out)), dim3(s2a::kBlock), 0, st>>>(in, out, n_out, r);
        else
            s2a::cap_bwd_kernel_unaligned<BF16><<<dim3(pair_grid(2 * n_out)), dim3(s2a::kBlock), 0, st>>>(in, out, n_out, r);
    });
}

int check_cap(const void* a, const void* b, int64_t n_out, int r, int dtype)
{
    if (dtype != S2A_F32 && dtype != S2A_BF16) return S2A_ERR_DTYPE;
    if (n_out < 0 || r < 2 || r > 64 || (r & (r - 1)) != 0) return S2A_ERR_SIZE;
    if (n_out > 0 && (!a || !b)) return S2A_ERR_NULL;
    return S2A_OK;
}

int check_lrp(int64_t batch, int64_t N, int64_t C, int r, int dtype)
{
    if (dtype != S2A_F32 && dtype != S2A_BF16) return S2A_ERR_DTYPE;
    const int epv = dtype == S2A_BF16 ? 8 : 4;
    if (batch < 0 || N < 0 || C < 0 || r < 1 || r > s2a::kLrpMaxRank) return S2A_ERR_SIZE;
    if (C % epv != 0) return S2A_ERR_SIZE;                       // a row of channels is whole 16-byte vectors
    if (batch > 0x7fffffff || N > 0x7fffffff || C > 0x7fffffff) return S2A_ERR_SIZE;
    if (N * C > 0x7fffffffLL * epv) return S2A_ERR_SIZE;         // vectors per sample fit an int
    return S2A_OK;
}

static_assert(s2a::kQsFloats == S2A_QSTATE_FLOATS, "header and kernels disagree on the qstate size");
static_assert(s2a::kSoftmaxMaxL == S2A_SOFTMAX_MAX_L, "header and kernels disagree on the longest softmax row");

// Both kernels of the Low-Rank-Prompt backward pass; `work` holds N*C floats (the batch-summed
// gradient between the two).  Arguments are checked by the callers.
int launch_lrp_bwd(const void* dy, const float* A, const float* B, float* dA, float* dB, float* work,
                   int64_t batch, int64_t N, int64_t C, int r, int dtype, hipStream_t st)
{
    const int epv = dtype == S2A_BF16 ? 8 : 4;
    const int64_t sample = N * (C / epv);  // vectors per sample
    const int64_t sum_blocks = (sample + s2a::kLrpSumPos - 1) / s2a::kLrpSumPos;
    // token tiles (dA) and 64-channel slabs (dB) in whole groups of 8, one member per XCD
    const int64_t x = s2a::kXcds;
    const int64_t ktiles = (r + s2a::kLrpTile - 1) / s2a::kLrpTile;
    const int64_t itiles = (N + s2a::kLrpTile - 1) / s2a::kLrpTile;
    const int64_t slabs = (C + s2a::kLrpDbChannels - 1) / s2a::kLrpDbChannels;
    const int64_t blocks_a = (itiles + x - 1) / x * x * ktiles;
    const int64_t blocks_b = (slabs + x - 1) / x * x * ktiles;
    if (sum_blocks > 0x7fffffffLL || blocks_a + blocks_b > 0x7fffffffLL) return S2A_ERR_SIZE;
    int rc = checked_launch([&] {
        if (dtype == S2A_BF16)
            s2a::lrp_batch_sum_kernel<true><<<dim3((unsigned)sum_blocks), dim3(s2a::kLrpSumBlock), 0, st>>>(
                (const s2a::u32x4*)dy, work, (int)batch, sample);
        else
            s2a::lrp_batch_sum_kernel<false><<<dim3((unsigned)sum_blocks), dim3(s2a::kLrpSumBlock), 0, st>>>(
                (const s2a::u32x4*)dy, work, (int)batch, sample);
    });
    if (rc != S2A_OK) return rc;
    return checked_launch([&] {
        s2a::lrp_grad_ab_kernel<<<dim3((unsigned)(blocks_a + blocks_b)), dim3(s2a::kLrpAbBlock), 0, st>>>(
            work, A, B, dA, dB, (int)N, (int)C, r, (int)blocks_b);
    });
}

int check_lrp_bwd_ptrs(const void* dy, const float* A, const float* B, float* dA, float* dB, int64_t batch)
{
    if ((batch > 0 && !dy) || !A || !B || !dA || !dB) return S2A_ERR_NULL;
    if (!aligned(dy, 16) || !aligned(A, 4) || !aligned(B, 4) || !aligned(dA, 4) || !aligned(dB, 4))
        return S2A_ERR_ALIGN;
    return S2A_OK;
}

constexpr int kMaxDevices = 64;
float* g_scratch_ptr[kMaxDevices];   // per device, looked up on the first call with that device current
std::mutex g_scratch_mutex;

// The device address of `scratch` on the current device; nullptr if the runtime cannot say.
float* scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = (float*)p;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

int s2a_qtable_init(int levels)
{
    if (levels != 16) return S2A_ERR_LEVELS;
    build_table(g_table);
    return S2A_OK;
}

int s2a_qtable_get(float xhat[16], float deriv[16], float bounds[15])
{
    if (!g_table.ready) return S2A_ERR_NOT_INIT;
    for (int k = 0; k < 16; ++k) {
        if (xhat) xhat[k] = g_table.xhat[k];
        if (deriv) deriv[k] = g_table.dev.d[k];
    }
    for (int j = 0; j < 15; ++j)
        if (bounds) bounds[j] = g_table.bounds[j];
    return S2A_OK;
}

int s2a_act_fwd(const void* x, void* y, uint8_t* codes, int64_t n, int dtype, void* stream)
{
    int rc = check_common(x, y, codes, n, dtype);
    if (rc != S2A_OK || n == 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_fwd<true, false>(x, y, codes, nullptr, n, st)
                             : launch_fwd<false, false>(x, y, codes, nullptr, n, st);
}

int s2a_act_bwd(const void* dy, const uint8_t* codes, void* dx, int64_t n, int dtype, void* stream)
{
    int rc = check_common(dy, codes, dx, n, dtype);
    if (rc != S2A_OK || n == 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_bwd<true, false>(dy, codes, dx, nullptr, n, st)
                             : launch_bwd<false, false>(dy, codes, dx, nullptr, n, st);
}

int s2a_act_fwd_dyn(const void* x, void* y, uint8_t* codes, float* qstate, int64_t n, int dtype,
                    void* stream)
{
    int rc = check_common(x, y, codes, n, dtype);
    if (rc != S2A_OK) return rc;
    if (!qstate) return S2A_ERR_NULL;
    if (((uintptr_t)qstate & 3u) != 0) return S2A_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    // n == 0 still leaves a defined state behind (min = max = 0, scale 0): both launches run
    rc = dtype == S2A_BF16 ? launch_range<true>(x, qstate, n, st) : launch_range<false>(x, qstate, n, st);
    if (rc != S2A_OK) return rc;
    return dtype == S2A_BF16 ? launch_fwd<true, true>(x, y, codes, qstate, n, st)
                             : launch_fwd<false, true>(x, y, codes, qstate, n, st);
}

int s2a_act_bwd_dyn(const void* dy, const uint8_t* codes, const float* qstate, void* dx, int64_t n,
                    int dtype, void* stream)
{
    int rc = check_common(dy, codes, dx, n, dtype);
    if (rc != S2A_OK) return rc;
    if (!qstate) return S2A_ERR_NULL;
    if (((uintptr_t)qstate & 3u) != 0) return S2A_ERR_ALIGN;
    if (n == 0) return S2A_OK;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_bwd<true, true>(dy, codes, dx, qstate, n, st)
                             : launch_bwd<false, true>(dy, codes, dx, qstate, n, st);
}

int s2a_silu_fwd(const void* x, void* y, uint8_t* codes, int64_t n, int dtype, void* stream)
{
    int rc = check_common(x, y, codes, n, dtype);
    if (rc != S2A_OK || n == 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_fwd<true, false, s2a::kActSilu>(x, y, codes, nullptr, n, st)
                             : launch_fwd<false, false, s2a::kActSilu>(x, y, codes, nullptr, n, st);
}

int s2a_silu_bwd(const void* dy, const uint8_t* codes, void* dx, int64_t n, int dtype, void* stream)
{
    int rc = check_common(dy, codes, dx, n, dtype);
    if (rc != S2A_OK || n == 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_bwd<true, false>(dy, codes, dx, nullptr, n, st, g_table.silu)
                             : launch_bwd<false, false>(dy, codes, dx, nullptr, n, st, g_table.silu);
}

int s2a_relu_fwd(const void* x, void* y, uint8_t* mask, int64_t n, int dtype, void* stream)
{
    int rc = check_args(x, y, mask, n, dtype);
    if (rc != S2A_OK || n == 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_relu_fwd<true>(x, y, mask, n, st)
                             : launch_relu_fwd<false>(x, y, mask, n, st);
}

int s2a_relu_bwd(const void* dy, const uint8_t* mask, void* dx, int64_t n, int dtype, void* stream)
{
    int rc = check_args(dy, mask, dx, n, dtype);
    if (rc != S2A_OK || n == 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_relu_bwd<true>(dy, mask, dx, n, st)
                             : launch_relu_bwd<false>(dy, mask, dx, n, st);
}

int s2a_softmax_fwd(const void* x, void* y, uint8_t* codes, float* qparams, int64_t rows, int64_t L,
                    int dtype, void* stream)
{
    int rc = check_softmax(x, y, codes, qparams, rows, L, dtype);
    if (rc != S2A_OK || rows == 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_softmax_fwd<true>(x, y, codes, qparams, rows, (int)L, st)
                             : launch_softmax_fwd<false>(x, y, codes, qparams, rows, (int)L, st);
}

int s2a_softmax_bwd(const void* dy, const uint8_t* codes, const float* qparams, void* dx,
                    int64_t rows, int64_t L, int dtype, void* stream)
{
    int rc = check_softmax(dy, codes, dx, qparams, rows, L, dtype);
    if (rc != S2A_OK || rows == 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_softmax_bwd<true>(dy, codes, qparams, dx, rows, (int)L, st)
                             : launch_softmax_bwd<false>(dy, codes, qparams, dx, rows, (int)L, st);
}

int s2a_cap_fwd(const void* x, void* y, int64_t n_out, int r, int dtype, void* stream)
{
    int rc = check_cap(x, y, n_out, r, dtype);
    if (rc != S2A_OK || n_out == 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_cap<true>(true, x, y, x, n_out, r, st)
                             : launch_cap<false>(true, x, y, x, n_out, r, st);
}

int s2a_cap_bwd(const void* dy, void* dx, int64_t n_out, int r, int dtype, void* stream)
{
    int rc = check_cap(dy, dx, n_out, r, dtype);
    if (rc != S2A_OK || n_out == 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_cap<true>(false, dy, dx, dx, n_out, r, st)
                             : launch_cap<false>(false, dy, dx, dx, n_out, r, st);
}

int s2a_lrp_fwd(const void* x, void* y, const float* A, const float* B, int64_t batch, int64_t N,
                int64_t C, int r, int dtype, void* stream)
{
    int rc = check_lrp(batch, N, C, r, dtype);
    if (rc != S2A_OK) return rc;
    if (batch == 0 || N == 0 || C == 0) return S2A_OK;
    if (!x || !y || !A || !B) return S2A_ERR_NULL;
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(A, 4) || !aligned(B, 4)) return S2A_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const int epv = dtype == S2A_BF16 ? 8 : 4;
    // a block: kLrpFwdTokens token rows x kLrpFwdCols neighbouring vectors of each
    const int64_t blocks = ((N + s2a::kLrpFwdTokens - 1) / s2a::kLrpFwdTokens) * ((C / epv + s2a::kLrpFwdCols - 1) / s2a::kLrpFwdCols);
    if (blocks > 0x7fffffffLL) return S2A_ERR_SIZE;
    const dim3 grid((unsigned)blocks), block(s2a::kLrpFwdBlock);
    const s2a::u32x4* xv = (const s2a::u32x4*)x;
    s2a::u32x4* yv = (s2a::u32x4*)y;
    const bool two = r > 64;  // rounds of 64 ranks in the kernel's prompt sum
    return checked_launch([&] {
        if (dtype == S2A_BF16 && !two) s2a::lrp_fwd_kernel<true, 1><<<grid, block, 0, st>>>(xv, yv, A, B, (int)batch, (int)N, (int)C, r);
        else if (dtype == S2A_BF16) s2a::lrp_fwd_kernel<true, 2><<<grid, block, 0, st>>>(xv, yv, A, B, (int)batch, (int)N, (int)C, r);
        else if (!two) s2a::lrp_fwd_kernel<false, 1><<<grid, block, 0, st>>>(xv, yv, A, B, (int)batch, (int)N, (int)C, r);
        else s2a::lrp_fwd_kernel<false, 2><<<grid, block, 0, st>>>(xv, yv, A, B, (int)batch, (int)N, (int)C, r);
    });
}

int s2a_lrp_bwd(const void* dy, const float* A, const float* B, float* dA, float* dB, float* work,
                int64_t batch, int64_t N, int64_t C, int r, int dtype, void* stream)
{
    int rc = check_lrp(batch, N, C, r, dtype);
    if (rc != S2A_OK) return rc;
    if (N == 0 || C == 0) return S2A_OK;
    rc = check_lrp_bwd_ptrs(dy, A, B, dA, dB, batch);
    if (rc != S2A_OK) return rc;
    if (!work) return S2A_ERR_NULL;
    if (!aligned(work, 4)) return S2A_ERR_ALIGN;
    return launch_lrp_bwd(dy, A, B, dA, dB, work, batch, N, C, r, dtype, (hipStream_t)stream);
}

int s2a_lrp_bwd_noalloc(const void* dy, const float* A, const float* B, float* dA, float* dB,
                        int64_t batch, int64_t N, int64_t C, int r, int dtype, void* stream)
{
    int rc = check_lrp(batch, N, C, r, dtype);
    if (rc != S2A_OK) return rc;
    if (N * C > (int64_t)S2A_LRP_NOALLOC_MAX_FLOATS) return S2A_ERR_SIZE;  // beyond the library's working memory
    if (N == 0 || C == 0) return S2A_OK;
    rc = check_lrp_bwd_ptrs(dy, A, B, dA, dB, batch);
    if (rc != S2A_OK) return rc;
    float* work = scratch_on_current_device();
    if (!work) return S2A_ERR_LAUNCH;
    return launch_lrp_bwd(dy, A, B, dA, dB, work, batch, N, C, r, dtype, (hipStream_t)stream);
}

int s2a_stream_copy(const void* src, void* dst, int64_t nbytes, void* stream)
{
    if (nbytes < 0 || nbytes % 16 != 0) return S2A_ERR_SIZE;
    if (nbytes == 0) return S2A_OK;
    if (!src || !dst) return S2A_ERR_NULL;
    if (!aligned(src, 16) || !aligned(dst, 16)) return S2A_ERR_ALIGN;
    const int64_t nvec = nbytes / 16;
    const int64_t blocks = (nvec + s2a::kWave - 1) / s2a::kWave;
    if (blocks > 0x7fffffffLL) return S2A_ERR_SIZE;
    return checked_launch([&] {
        s2a::stream_copy_kernel<<<dim3((unsigned)blocks), dim3(s2a::kWave), 0, (hipStream_t)stream>>>(
            (const s2a::u32x4*)src, (s2a::u32x4*)dst, nvec);
    });
}

int s2a_stream_copy_shaped(const void* src, void* dst, void* side, int64_t nbytes, int side_bytes,
                           int side_is_input, void* stream)
{
    if (nbytes < 0 || nbytes % 16 != 0 || (side_bytes != 2 && side_bytes != 4)) return S2A_ERR_SIZE;
    if (nbytes == 0) return S2A_OK;
    if (!src || !dst || !side) return S2A_ERR_NULL;
    if (!aligned(src, 16) || !aligned(dst, 16) || !aligned(side, 4)) return S2A_ERR_ALIGN;
    const int64_t nvec = nbytes / 16;
    const int64_t blocks = (nvec + s2a::kWave - 1) / s2a::kWave;
    if (blocks > 0x7fffffffLL) return S2A_ERR_SIZE;
    const dim3 grid((unsigned)blocks), block(s2a::kWave);
    hipStream_t st = (hipStream_t)stream;
    const s2a::u32x4* s = (const s2a::u32x4*)src;
    s2a::u32x4* d = (s2a::u32x4*)dst;
    uint8_t* c = (uint8_t*)side;
    return checked_launch([&] {
        if (side_bytes == 4 && side_is_input) s2a::stream_copy_shaped_kernel<4, true><<<grid, block, 0, st>>>(s, d, c, nvec);
        else if (side_bytes == 4) s2a::stream_copy_shaped_kernel<4, false><<<grid, block, 0, st>>>(s, d, c, nvec);
        else if (side_is_input) s2a::stream_copy_shaped_kernel<2, true><<<grid, block, 0, st>>>(s, d, c, nvec);
        else s2a::stream_copy_shaped_kernel<2, false><<<grid, block, 0, st>>>(s, d, c, nvec);
    });
}

const char* s2a_strerror(int code)
{
    switch (code) {
        case S2A_OK: return "ok";
        case S2A_ERR_NULL: return "a required pointer is NULL";
        case S2A_ERR_SIZE: return "element count is negative or too large for one launch";
        case S2A_ERR_DTYPE: return "dtype is neither S2A_F32 nor S2A_BF16";
        case S2A_ERR_LEVELS: return "only 16 quantization levels (4-bit codes) are supported";
        case S2A_ERR_NOT_INIT: return "s2a_qtable_init has not been called";
        case S2A_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
        case S2A_ERR_ALIGN: return "a buffer does not have the alignment its entry point requires";
        default: return "unknown s2a error code";
    }
}

}  // extern "C"
