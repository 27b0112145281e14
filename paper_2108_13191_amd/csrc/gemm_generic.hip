// Any-shape, any-alignment kernel: every global access is a predicated
// element access, so nothing outside the M x K, K x N and M x N extents is
// touched and the k tail is zero-filled in both operands.  It follows the
// two-level recipe of the paper's Algorithm "Two-level tiled tensor core
// Matmul" in its plainest form (one LDS buffer, two barriers per step); the
// tuned kernels live in gemm_tiled.hip.
#include "gemm_common.h"
#include "../../include/gemm_f16.h"

namespace {

constexpr int GBM = 64, GBN = 64, GBK = 32, GPAD = 8;

// C_IN_LOOP (a ladder row, never selected): the accumulator goes to C and comes back in every
// k step, as in the paper's Algorithm "Two-level tiled tensor core Matmul" before the load and
// store of C are hoisted out of the k loop (section "Generating WMMA Ops and More").  With f16
// C that rounds the running sum at every step, so the row is built for f32 C only.
// ROUND_PER_SLICE (another ladder row, f16 C only): the literal reading of the paper's half
// precision mode (section Half Precision Performance: the accumulation is done in f16 as well)
// -- the running sum is rounded to binary16, to nearest even, behind every MFMA, i.e. after
// every 16-deep k slice, the depth of the paper's m16n16k16 operation.  The library's own
// reading keeps the sum in f32 and rounds once at the store.
template <typename CT, bool C_IN_LOOP = false, bool ROUND_PER_SLICE = false>
__global__ __launch_bounds__(256) void gemm_generic_kernel(
    int M, int N, int K, const half_t* __restrict__ A, int64_t lda,
    const half_t* __restrict__ B, int64_t ldb, CT* __restrict__ C, int64_t ldc, int tiles_n,
    const CT* __restrict__ bias, int relu)
{
    // A tile as [m][k], B tile transposed to [n][k]: both MFMA operands then
    // read 8 consecutive k per lane with one 16-byte LDS load.
    __shared__ __attribute__((aligned(16))) half_t As[GBM][GBK + GPAD];
    __shared__ __attribute__((aligned(16))) half_t Bt[GBN][GBK + GPAD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t tile = blockIdx.x;
    const int64_t m0 = (tile / tiles_n) * GBM, n0 = (tile % tiles_n) * GBN;

    // v_mfma_f32_32x32x16_f16 accumulator layout: register i of lane l is
    // row 8*(i/4) + 4*(l/32) + i%4, column l%32 of the 32x32 block.
    floatx16 acc;
    const int64_t col = n0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const int64_t row = m0 + wm * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i & 3);
        acc[i] = (row < M && col < N) ? (float)C[row * ldc + col] : 0.0f;
    }

    for (int64_t k0 = 0; k0 < K; k0 += GBK) {
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int r = (tid >> 5) + 8 * i, kk = tid & 31;
            const int64_t gr = m0 + r, gk = k0 + kk;
            As[r][kk] = (gr < M && gk < K) ? A[gr * lda + gk] : (half_t)0;
        }
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int kk = (tid >> 6) + 4 * i, n = tid & 63;
            const int64_t gk = k0 + kk, gn = n0 + n;
            Bt[n][kk] = (gk < K && gn < N) ? B[gk * ldb + gn] : (half_t)0;
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < GBK / 16; ks++) {
            // operand layout: lane l holds row (column) l%32, k = 8*(l/32) .. +7
            const half8 a = *reinterpret_cast<const half8*>(&As[wm * 32 + (lane & 31)][ks * 16 + 8 * (lane >> 5)]);
            const half8 b = *reinterpret_cast<const half8*>(&Bt[wn * 32 + (lane & 31)][ks * 16 + 8 * (lane >> 5)]);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
            if constexpr (ROUND_PER_SLICE) {
#pragma unroll
                for (int i = 0; i < 16; i++) acc[i] = (float)(half_t)acc[i];
            }
        }
        __syncthreads();
        if constexpr (C_IN_LOOP) {
            if (k0 + GBK < K) {
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const int64_t row = m0 + wm * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i & 3);
                    if (row < M && col < N) {
                        volatile CT* c = &C[row * ldc + col];
                        *c = (CT)acc[i];
                        acc[i] = (float)*c;
                    }
                }
            }
        }
    }

    const float bv = (bias && col < N) ? (float)bias[col] : 0.0f;     // fused epilogue: + bias, ReLU (NaN, -0 pass)
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const int64_t row = m0 + wm * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i & 3);
        if (row < M && col < N) {                                  // f16: round to nearest even
            float v = acc[i] + bv;
            C[row * ldc + col] = (CT)((relu && v < 0.0f) ? 0.0f : v);
        }
    }
}

}  // namespace

int64_t grid_generic(int64_t M, int64_t N)
{
    const int64_t tm = (M + GBM - 1) / GBM, tn = (N + GBN - 1) / GBN;
    if (tm > 0 && tn > INT32_MAX / tm) return -1;
    return tm * tn;
}

#ifdef GEMM_F16_LADDER
int launch_generic_c_in_loop(const GemmArgs& a)
{
    if (a.c_is_f16) return launch_generic(a);
    const int64_t g = grid_generic(a.M, a.N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    const int tiles_n = (int)((a.N + GBN - 1) / GBN);
    hipLaunchKernelGGL((gemm_generic_kernel<float, true>), dim3((unsigned)g), dim3(256), 0, a.stream,
                       (int)a.M, (int)a.N, (int)a.K, a.A, a.lda, a.B, a.ldb, (float*)a.C, a.ldc, tiles_n, (const float*)a.bias, a.relu);
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}
const GemmConfigDesc kGenericCInLoop = {
    "generic64x64x32_c_in_loop", 64, 64, 32, 4, 32, 32, 2 * 64 * (32 + 8) * 2, false, launch_generic_c_in_loop, grid_generic};
const GemmConfigDesc* generic_c_in_loop_config() { return &kGenericCInLoop; }

int launch_generic_round_per_slice(const GemmArgs& a)
{
    if (!a.c_is_f16) return launch_generic(a);
    const int64_t g = grid_generic(a.M, a.N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    const int tiles_n = (int)((a.N + GBN - 1) / GBN);
    hipLaunchKernelGGL((gemm_generic_kernel<half_t, false, true>), dim3((unsigned)g), dim3(256), 0, a.stream,
                       (int)a.M, (int)a.N, (int)a.K, a.A, a.lda, a.B, a.ldb, (half_t*)a.C, a.ldc, tiles_n, (const half_t*)a.bias, a.relu);
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}
const GemmConfigDesc kGenericRoundPerSlice = {
    "generic64x64x32_f16_round_per_slice", 64, 64, 32, 4, 32, 32, 2 * 64 * (32 + 8) * 2, false, launch_generic_round_per_slice, grid_generic};
const GemmConfigDesc* generic_round_per_slice_config() { return &kGenericRoundPerSlice; }
#endif

int launch_generic(const GemmArgs& a)
{
    const int64_t g = grid_generic(a.M, a.N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    const int tiles_n = (int)((a.N + GBN - 1) / GBN);
    if (a.c_is_f16)
        hipLaunchKernelGGL((gemm_generic_kernel<half_t>), dim3((unsigned)g), dim3(256), 0, a.stream,
                           (int)a.M, (int)a.N, (int)a.K, a.A, a.lda, a.B, a.ldb, (half_t*)a.C, a.ldc, tiles_n, (const half_t*)a.bias, a.relu);
    else
        hipLaunchKernelGGL((gemm_generic_kernel<float>), dim3((unsigned)g), dim3(256), 0, a.stream,
                           (int)a.M, (int)a.N, (int)a.K, a.A, a.lda, a.B, a.ldb, (float*)a.C, a.ldc, tiles_n, (const float*)a.bias, a.relu);
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}
