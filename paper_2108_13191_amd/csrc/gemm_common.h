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
    int k_split = 0;       // > 1: the k loop cut into this many parts that add to C atomically (five-stage 128 x 128 kernel, f32 C, no fused epilogue)
};

// Static description of one kernel configuration.
struct GemmConfigDesc {
    const char* name;
    int block_m, block_n, block_k, waves, wave_m, wave_n, lds_bytes;
    bool needs_aligned;                       // 16-byte aligned A, B; lda, ldb, K, N multiples of 8
    int (*launch)(const GemmArgs&);           // returns a GEMM_F16_* code
    int64_t (*grid)(int64_t M, int64_t N);    // workgroups for a problem (<0: too many)
};

// What the launchers and the selector assume about the device, in one place: compute units,
// XCDs (each with its own L2; consecutive workgroup ids are dealt to them in turn), and
// the rate of the constant wall clock the late start counts in.  Queried once per process
// from the current device; without a device the MI355X values (256, 8, 100 MHz).
struct ChipShape {
    int cus;                // compute units: workgroups of the largest tile that run at once
    int xcds;               // 32 compute units each on gfx950 parts (8 on an MI355X, fewer in partitioned modes)
    int wall_clock_khz;
};
const ChipShape& chip();                     // gemm_api.hip

// gemm_generic.hip
int launch_generic(const GemmArgs& a);
int64_t grid_generic(int64_t M, int64_t N);

// gemm_tiled.hip: the plain ring-buffered tiling, 64 x 64 (ladder builds also 128 x 128 and 256 x 256)
const GemmConfigDesc* tiled_config(int block);

// gemm_pingpong.hip
const GemmConfigDesc* pingpong16_config(int block_m, int block_n);   // 256x256, 192x256, 128x256, 256x192 or 128x128
const GemmConfigDesc* pingpong16_persistent_config();                 // 256x256, one workgroup per compute unit walks its tiles
const GemmConfigDesc* pingpong16_staggered_config();                  // 256x256, every other compute unit half a tile ahead

// gemm_w4a.hip
const GemmConfigDesc* long_k_config();                                // 256x256, four wavefronts of 128x128, k loop in assembly

// gemm_w4a128.hip
const GemmConfigDesc* deep_ring_config();                             // 128x128, four wavefronts of 64x64, k loop in assembly over five LDS stages

// gemm_splitk_f16.hip: the passes around a split-k launch in the half-precision mode
int splitk_f16_zero(float* ws, int64_t n, hipStream_t stream);
int splitk_f16_finish(float* ws, void* C, int64_t ldc, int64_t M, int64_t N, int clear, hipStream_t stream);
int splitk_f16_static_scratch(float** ptr, int64_t* floats);            // the library's own scratch memory on the current device

#ifdef GEMM_F16_LADDER
// Comparison kernels and ablation rows: built into libgemm_f16_ladder.so only, never selected.
const GemmConfigDesc* pingpong_config();                             // gemm_pingpong.hip: 256x256 on 32x32x16 MFMAs
const GemmConfigDesc* pingpong16_192x192_config();                   // gemm_pingpong.hip: 192x192 tile (fills 256 compute units where 192x256 fills 192)
const GemmConfigDesc* pingpong16_rowwise_config();                   // gemm_pingpong.hip: 256x256, MFMAs of a phase row by row of blocks
const GemmConfigDesc* pingpong16_no_xcd_order_config();              // gemm_pingpong.hip: tiles dealt to XCDs as the hardware deals workgroups
const GemmConfigDesc* tiled_no_swizzle_config();                     // gemm_tiled.hip: 256x256, LDS image not swizzled
const GemmConfigDesc* generic_c_in_loop_config();                    // gemm_generic.hip: C read and written in every k step
const GemmConfigDesc* generic_round_per_slice_config();              // gemm_generic.hip: f16 mode, running sum rounded to f16 every 16 k
const GemmConfigDesc* interleaved_config();                          // ladder/gemm_interleaved.hip
const GemmConfigDesc* overlap_config();                              // ladder/gemm_overlap.hip
const GemmConfigDesc* w4_config();                                   // ladder/gemm_w4.hip
#endif
