// Half-precision mode with the k loop cut into parts (skinny problems): the parts cannot add to
// an f16 C -- that would round once per part -- so they add, atomically and in f32, to a
// workspace of M x N floats that starts at zero, and a second pass adds the workspace to C with
// the mode's one rounding to nearest even.  This file holds the two small passes around the
// GEMM launch (zero the workspace; C = round(C + workspace)).
#include "gemm_device.h"
#include "../../include/gemm_f16.h"

namespace {

using namespace gemm_dev;

__global__ __launch_bounds__(256) void splitk_zero_kernel(float* __restrict__ ws, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) reinterpret_cast<floatx4*>(ws)[i] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
}

// One thread per element: C is only known to be 2-byte aligned.  clear = leave zeros behind (the
// library's own scratch stays zero between calls).
__global__ __launch_bounds__(256) void splitk_finish_f16_kernel(float* __restrict__ ws, half_t* __restrict__ C, int64_t ldc,
                                                                int M, int N, int clear)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)M * N) return;
    const int64_t r = i / N, c = i - r * N;
    half_t* const p = C + r * ldc + c;
    *p = (half_t)((float)*p + ws[i]);                     // exact widening, f32 addition, one rounding to nearest even
    if (clear) ws[i] = 0.0f;
}

// The library's own scratch memory for gemm_f16_f16acc_static_workspace: 2^20 floats (4 MB) per
// GPU the library runs on, held until the process ends; it covers every problem that the
// workspace form cuts along k.  The name below is a host-side stand-in, not a device address:
// host code uses the pointer that static_scratch() hands out.
constexpr int64_t STATIC_SCRATCH_FLOATS = 1 << 20;
static __device__ __align__(256) float scratch[STATIC_SCRATCH_FLOATS];

constexpr int MAX_DEVICES = 64;
float* g_scratch_ptr[MAX_DEVICES] = {};

}  // namespace

// The current device's copy of the scratch array (its address is asked for once per device, with
// that device current) and its size in floats.
int splitk_f16_static_scratch(float** ptr, int64_t* floats)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return GEMM_F16_ERR_LAUNCH;
    if (!g_scratch_ptr[dev]) {
        float* p = nullptr;
        if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GEMM_F16_ERR_LAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    *floats = STATIC_SCRATCH_FLOATS;
    return GEMM_F16_OK;
}

// n floats (a multiple of 4, 16-byte aligned) to zero
int splitk_f16_zero(float* ws, int64_t n, hipStream_t stream)
{
    const int64_t n4 = n / 4, blocks = (n4 + 255) / 256;
    if (blocks > INT32_MAX) return GEMM_F16_ERR_SIZE;
    if (blocks > 0) hipLaunchKernelGGL(splitk_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, ws, n4);
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}

// C (f16, M x N, pitch ldc) = round(C + ws (f32, M x N, pitch N))
int splitk_f16_finish(float* ws, void* C, int64_t ldc, int64_t M, int64_t N, int clear, hipStream_t stream)
{
    const int64_t blocks = (M * N + 255) / 256;
    if (blocks > INT32_MAX) return GEMM_F16_ERR_SIZE;
    if (blocks > 0) hipLaunchKernelGGL(splitk_finish_f16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, ws, (half_t*)C, ldc, (int)M, (int)N, clear);
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}
