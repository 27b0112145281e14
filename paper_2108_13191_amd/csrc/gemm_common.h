// Shared declarations of the HIP GEMM library (device vector types, the
// launcher prototypes behind the C ABI).  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 half_t;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));

// One GEMM call, as validated by the C ABI.  c_is_f16 selects the element
// type of C (f32 otherwise).
struct GemmArgs {
    int64_t M, N, K;
    const half_t* A; int64_t lda;
    const half_t* B; int64_t ldb;
    void* C; int64_t ldc;
    int c_is_f16;
    hipStream_t stream;
    const void* bias;      // N elements of C's type, or nullptr
    int relu;              // 0 / 1
};

// Static description of one kernel configuration.
struct GemmConfigDesc {
    const char* name;
    int block_m, block_n, block_k, waves, wave_m, wave_n, lds_bytes;
    bool needs_aligned;                       // 16-byte aligned A, B; lda, ldb, K, N multiples of 8
    int (*launch)(const GemmArgs&);           // returns a GEMM_F16_* code
    int64_t (*grid)(int64_t M, int64_t N);    // workgroups for a problem (<0: too many)
};

// gemm_generic.hip
int launch_generic(const GemmArgs& a);
int64_t grid_generic(int64_t M, int64_t N);

// gemm_tiled.hip
int tiled_num_configs();
const GemmConfigDesc* tiled_config(int i);

// gemm_pingpong.hip
const GemmConfigDesc* pingpong_config();
const GemmConfigDesc* pingpong16_config(int block_m, int block_n);   // 256x256, 192x256, 128x256, 256x192 or 128x128
const GemmConfigDesc* pingpong16_persistent_config();                 // 256x256, one workgroup per compute unit walks its tiles
const GemmConfigDesc* pingpong16_staggered_config();                  // 256x256, every other compute unit half a tile ahead

// gemm_overlap.hip
const GemmConfigDesc* overlap_config();                              // 256x128, two accumulator sets: C traffic under the next tile's MFMAs

// gemm_api.hip
int compute_units();                                                 // of the current device (256 if there is none)

// gemm_w4.hip
const GemmConfigDesc* w4_config();
