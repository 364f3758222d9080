// s2a_api.hip -- host side of the C ABI declared in include/s2a.h: argument
// checks, the quantization table, kernel selection and launch.  No device
// memory is allocated and nothing synchronizes.
#include "s2a.h"

#include <math.h>

#include "s2a_kernels.hpp"

namespace {


struct TableState {
    bool ready = false;
    s2a::QTable dev;   // fp32 derivative levels handed to kernels by value
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
    }
    for (int j = 0; j < 15; ++j) t.bounds[j] = (float)(lo + step * ((double)j + 0.5));
    t.ready = true;
}

int check_common(const void* a, const void* b, const void* c, int64_t n, int dtype)
{
    if (!g_table.ready) return S2A_ERR_NOT_INIT;
    if (dtype != S2A_F32 && dtype != S2A_BF16) return S2A_ERR_DTYPE;
    if (n < 0) return S2A_ERR_SIZE;
    if (n > 0 && (!a || !b || !c)) return S2A_ERR_NULL;
    return S2A_OK;
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

template <bool BF16>
int launch_fwd(const void* x, void* y, uint8_t* codes, int64_t n, hipStream_t st)
{
    constexpr int EPV = BF16 ? 8 : 4;
    (void)hipGetLastError();  // drop any stale error left by earlier, unrelated runtime calls
    if (aligned(x, 16) && aligned(y, 16) && aligned(codes, 4)) {
        int64_t nvec = n / EPV;
        int64_t slots = nvec + (n % EPV != 0);
        int64_t blocks = (slots + s2a::kWave - 1) / s2a::kWave;
        if (blocks > 0x7fffffffLL) return S2A_ERR_SIZE;
        s2a::fwd_kernel<BF16><<<dim3((unsigned)blocks), dim3(s2a::kWave), 0, st>>>(
            (const s2a::u32x4*)x, (s2a::u32x4*)y, codes, n, nvec);
    } else {
        s2a::fwd_kernel_unaligned<BF16><<<dim3(pair_grid(n)), dim3(s2a::kBlock), 0, st>>>(x, y, codes, n);
    }
    return hipGetLastError() == hipSuccess ? S2A_OK : S2A_ERR_LAUNCH;
}

template <bool BF16>
int launch_bwd(const void* dy, const uint8_t* codes, void* dx, int64_t n, hipStream_t st)
{
    constexpr int EPV = BF16 ? 8 : 4;
    (void)hipGetLastError();  // drop any stale error left by earlier, unrelated runtime calls
    if (aligned(dy, 16) && aligned(dx, 16) && aligned(codes, 4)) {
        int64_t nvec = n / EPV;
        int64_t slots = nvec + (n % EPV != 0);
        int64_t blocks = (slots + s2a::kWave - 1) / s2a::kWave;
        if (blocks > 0x7fffffffLL) return S2A_ERR_SIZE;
        s2a::bwd_kernel<BF16><<<dim3((unsigned)blocks), dim3(s2a::kWave), 0, st>>>(
            (const s2a::u32x4*)dy, codes, (s2a::u32x4*)dx, g_table.dev, n, nvec);
    } else {
        s2a::bwd_kernel_unaligned<BF16><<<dim3(pair_grid(n)), dim3(s2a::kBlock), 0, st>>>(
            dy, codes, dx, g_table.dev, n);
    }
    return hipGetLastError() == hipSuccess ? S2A_OK : S2A_ERR_LAUNCH;
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
    return dtype == S2A_BF16 ? launch_fwd<true>(x, y, codes, n, st)
                             : launch_fwd<false>(x, y, codes, n, st);
}

int s2a_act_bwd(const void* dy, const uint8_t* codes, void* dx, int64_t n, int dtype, void* stream)
{
    int rc = check_common(dy, codes, dx, n, dtype);
    if (rc != S2A_OK || n == 0) return rc;
    hipStream_t st = (hipStream_t)stream;
    return dtype == S2A_BF16 ? launch_bwd<true>(dy, codes, dx, n, st)
                             : launch_bwd<false>(dy, codes, dx, n, st);
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
        default: return "unknown s2a error code";
    }
}

}  // extern "C"
