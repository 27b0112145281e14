// Measurement aid, not part of the GEMM library: what the matrix units of this
// MI355X sustain when NOTHING but MFMAs runs (operands stay in registers, no
// LDS, no memory), as a function of the operand DATA.  Under a dense MFMA load
// the part is power-limited and the limit depends on how much the operands
// toggle: this program prints the TFLOP/s of a pure MFMA loop for all-zero /
// all-one operands and for the random distributions of the benchmark
// workloads, for both f16 MFMA shapes.  It gives the data-dependent ceiling
// that the GEMM kernels' throughput on the same data has to be read against.
// Build: hipcc -O3 --offload-arch=gfx950 -o probe_mfma_ceiling probe_mfma_ceiling.hip
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#include <cmath>
#include <vector>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));
template <int NF>
__global__ __launch_bounds__(256) void k_mfma16(const half8* fr, float* out, int iters) {
  half8 a[NF], b[NF];
  for (int i = 0; i < NF; i++) { a[i] = fr[(i * 2 + 0) * 256 + threadIdx.x]; b[i] = fr[(i * 2 + 1) * 256 + threadIdx.x]; }
  float4v c[16];
  for (int i = 0; i < 16; i++) for (int e = 0; e < 4; e++) c[i][e] = 0;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < NF; i++) {
#pragma unroll
      for (int j = 0; j < 16; j++) c[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[(i + j) % NF], b[(i * 3 + j) % NF], c[j], 0, 0, 0);
    }
  }
  float s = 0; for (int i = 0; i < 16; i++) for (int e = 0; e < 4; e++) s += c[i][e];
  if (s == 12345.678f) out[0] = s;
}


// each lane loads NF distinct A and B fragments from memory (data pattern set by host), then loops MFMAs cycling through them
template <int NF>
__global__ __launch_bounds__(256) void k_mfma(const half8* fr, float* out, int iters) {
  half8 a[NF], b[NF];
  for (int i = 0; i < NF; i++) { a[i] = fr[(i * 2 + 0) * 256 + threadIdx.x]; b[i] = fr[(i * 2 + 1) * 256 + threadIdx.x]; }
  float16v c[8];
  for (int i = 0; i < 8; i++) for (int e = 0; e < 16; e++) c[i][e] = 0;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < NF; i++) {
#pragma unroll
      for (int j = 0; j < 8; j++) c[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[(i + j) % NF], b[(i * 3 + j) % NF], c[j], 0, 0, 0);
    }
  }
  float s = 0; for (int i = 0; i < 8; i++) for (int e = 0; e < 16; e++) s += c[i][e];
  if (s == 12345.678f) out[0] = s;
}

int main() {
  const int NF = 8;
  std::vector<_Float16> h(NF * 2 * 256 * 8);
  half8* d; float* out; CK(hipMalloc(&d, h.size() * 2)); CK(hipMalloc(&out, 64));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  const char* names[] = {"zeros", "ones", "normal/sqrt(8192)", "normal(0,1)", "uniform(-1,1)", "small ints -2..2"};
  for (int mode = 0; mode < 6; mode++) {
    srand(1);
    for (auto& x : h) {
      float u1 = (rand() + 1.0f) / (RAND_MAX + 2.0f), u2 = (rand() + 1.0f) / (RAND_MAX + 2.0f);
      float n = sqrtf(-2 * logf(u1)) * cosf(6.2831853f * u2);
      float v = mode == 0 ? 0.f : mode == 1 ? 1.f : mode == 2 ? n / 90.5f : mode == 3 ? n : mode == 4 ? (2 * u1 - 1) : (float)(rand() % 5 - 2);
      x = (_Float16)v;
    }
    CK(hipMemcpy(d, h.data(), h.size() * 2, hipMemcpyHostToDevice));
    int iters = 20000;
    k_mfma<NF><<<256, 256>>>(d, out, 100);
    for (int rep = 0; rep < 2; rep++) {
      CK(hipEventRecord(e0)); k_mfma<NF><<<256, 256>>>(d, out, iters); CK(hipEventRecord(e1)); CK(hipDeviceSynchronize());
      float ms; CK(hipEventElapsedTime(&ms, e0, e1));
      double flops = (double)iters * NF * 8 * 32768.0 * 4 * 256;
      printf("MFMA-only 32x32x16, operands %-20s: %.3f ms  %.1f TFLOP/s\n", names[mode], ms, flops / ms / 1e9);
    }
    for (int rep = 0; rep < 2; rep++) {
      CK(hipEventRecord(e0)); k_mfma16<NF><<<256, 256>>>(d, out, iters); CK(hipEventRecord(e1)); CK(hipDeviceSynchronize());
      float ms; CK(hipEventElapsedTime(&ms, e0, e1));
      double flops = (double)iters * NF * 16 * 16384.0 * 4 * 256;
      printf("MFMA-only 16x16x32, operands %-20s: %.3f ms  %.1f TFLOP/s\n", names[mode], ms, flops / ms / 1e9);
    }
  }
  return 0;
}
