// Measurement aid of bench.py, not part of the GEMM library: what the matrix units sustain when
// NOTHING but MFMAs runs (operands stay in registers: no LDS, no memory traffic), on operand
// DATA handed in by the caller.  Under a dense MFMA load the part is power-limited and the limit
// depends on how much the operands toggle (all-zero operands: 2.4 PFLOP/s; the benchmark's
// N(0,1)/sqrt(K) operands: about 1.85 PFLOP/s), so a GEMM's throughput on given data has to be
// read against this figure measured on the same data, in the same run.
//
// One workgroup per compute unit, 8 wavefronts (two per SIMD: one wavefront alone leaves issue
// gaps), each with the register blocking of the library's large-tile kernel: 8 A fragments x 4 B
// fragments -> 8 x 4 accumulators of v_mfma_f32_16x16x32_f16, 32 MFMAs per iteration.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

__global__ __launch_bounds__(512) void mfma_only_kernel(const half8* __restrict__ frags, float* __restrict__ sink, int iters)
{
    // 12 fragments of 256 lanes x 16 bytes: 8 for A, 4 for B; wavefront w and w + 4 (which share a SIMD) use the same
    half8 a[8], b[4];
    const int t = threadIdx.x & 255;
#pragma unroll
    for (int i = 0; i < 8; i++) a[i] = frags[i * 256 + t];
#pragma unroll
    for (int j = 0; j < 4; j++) b[j] = frags[(8 + j) * 256 + t];
    floatx4 c[8][4];
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) c[i][j] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
            for (int i = 0; i < 8; i++) c[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(b[j], a[i], c[i][j], 0, 0, 0);
        asm volatile("" : "+v"(a[0]), "+v"(b[0]));       // the loop body is not hoisted or merged across iterations
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) s += c[i][j][0] + c[i][j][1] + c[i][j][2] + c[i][j][3];
    if (s == 12345.678f) sink[0] = s;                     // keeps the accumulators alive; practically never taken
}

}  // namespace

extern "C" {

// flops of one launch = workgroups * 8 wavefronts * iters * 32 MFMAs * 16384
int bench_mfma_only(const void* frags /* device, 12 * 256 * 16 bytes */, void* sink /* device, 4 bytes */,
                    int iters, int workgroups, void* stream)
{
    if (!frags || !sink || iters < 0 || workgroups < 1) return -1;
    hipLaunchKernelGGL(mfma_only_kernel, dim3((unsigned)workgroups), dim3(512), 0, (hipStream_t)stream,
                       (const half8*)frags, (float*)sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

}  // extern "C"
