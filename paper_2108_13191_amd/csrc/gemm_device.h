// Device-side helpers shared by the tuned kernels (gemm_tiled.hip,
// gemm_pingpong.hip): the direct global -> LDS copy, the two LDS fragment
// reads, the XCD-aware workgroup -> tile map.  gfx950 only.
#pragma once
#include "gemm_common.h"

namespace gemm_dev {

constexpr int BK = 64;             // k extent per LDS stage (f16 elements)

struct TiledParams {
    int M, N, K;
    const half_t* A; int64_t lda;
    const half_t* B; int64_t ldb;
    void* C; int64_t ldc;
    int tiles_m, tiles_n, group_m;
    int num_xcd;           // XCDs the workgroup ids are dealt to in turn (1: tiles in plain order)
    const void* bias;      // fused epilogue: N elements of C's type or nullptr; relu 0 / 1
    int relu;
    int stagger_ticks;     // late start: workgroups on odd XCDs start this many wall-clock ticks late (0: all at once)
    int first_generation;  // late start: workgroups that begin with the launch (only these wait)
    int k_split;           // five-stage 128 x 128 kernel: > 1 = workgroup b works on tile b % tiles, part b / tiles of the k loop, and adds to C atomically
};

// The fields every launcher fills the same way: the problem, the tile grid for bm x bn tiles,
// and the tile order (group_m tile rows at a time; an XCD's 32 concurrent tiles should form a
// near-square block of C).
inline TiledParams make_tiled_params(const GemmArgs& a, int bm, int bn, int group_m)
{
    TiledParams p = {};
    p.M = (int)a.M; p.N = (int)a.N; p.K = (int)a.K;
    p.A = a.A; p.lda = a.lda; p.B = a.B; p.ldb = a.ldb; p.C = a.C; p.ldc = a.ldc;
    p.bias = a.bias; p.relu = a.relu;
    p.tiles_m = (int)((a.M + bm - 1) / bm);
    p.tiles_n = (int)((a.N + bn - 1) / bn);
    p.group_m = group_m < p.tiles_m ? group_m : p.tiles_m;
    p.num_xcd = chip().xcds;
    return p;
}

// The fused epilogue on one result: + bias, then ReLU written so that NaN and
// -0 pass through.
__device__ __forceinline__ float epilogue_value(float v, float bias, int relu)
{
    v += bias;
    return (relu && v < 0.0f) ? 0.0f : v;
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef __attribute__((address_space(1))) const void* gbl_ptr_t;
typedef __attribute__((address_space(3))) shortx4* lds_s4_ptr_t;

// 16 bytes per lane, global -> LDS at lds_byte_addr (wave-uniform) + 16 * lane.
// The global address is base (wave-uniform, 64 bit) + byte_off (per lane, 32
// bit).  Written as inline assembly on purpose: the compiler cannot tell which
// LDS bytes an LDS-DMA load writes and would wait for ALL outstanding copies
// (vmcnt(0)) in front of every LDS read of the other buffer, serialising the
// prefetch with the MFMA phase.  The kernel orders these copies itself: an
// explicit vmcnt(0) and a barrier before a buffer is read.
__device__ __forceinline__ void async_copy16(const void* base, uint32_t byte_off, uint32_t lds_byte_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\t"
                 "s_nop 0\n\t"
                 "global_load_lds_dwordx4 %0, %1"
                 :: "v"(byte_off), "s"(base), "s"(lds_byte_addr) : "memory", "m0");
}

// The same copy in two instructions that the caller separates by at least one other instruction
// (the wait state between a write of M0 and an LDS-DMA load): set_m0 puts base + imm into M0
// (imm must fold to a compile-time constant), async_copy16_m0 is the load.  Nothing in between
// may write M0; the kernels that use the pair issue nothing but MFMAs there.
__device__ __forceinline__ void set_m0(uint32_t base, uint32_t imm)
{
    asm volatile("s_add_u32 m0, %0, %1" :: "s"(base), "n"(imm) : "m0", "scc");
}
__device__ __forceinline__ void async_copy16_m0(const void* base, uint32_t byte_off)
{
    asm volatile("global_load_lds_dwordx4 %0, %1" :: "v"(byte_off), "s"(base) : "memory");
}

__device__ __forceinline__ half8 lds_read_b128(uint32_t addr)
{
    return *(__attribute__((address_space(3))) const half8*)(uintptr_t)addr;
}

__device__ __forceinline__ half4 lds_read_tr16(uint32_t addr)
{
    shortx4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4_ptr_t)(uintptr_t)addr);
    return __builtin_bit_cast(half4, v);
}

// Workgroup id -> C tile.  Ids are dealt to the XCDs round-robin; give XCD x
// the x-th contiguous slice of a tile order that walks group_m tile rows at a
// time, column by column.
__device__ __forceinline__ void tile_of_block(const TiledParams& p, int pid, int& tile_m, int& tile_n)
{
    const int num = p.tiles_m * p.tiles_n;
    const int q = num / p.num_xcd, r = num % p.num_xcd;
    const int x = pid % p.num_xcd;
    const int l = x * q + (x < r ? x : r) + pid / p.num_xcd;
    const int group_size = p.group_m * p.tiles_n;
    const int g = l / group_size;
    const int first_m = g * p.group_m;
    const int gm = (p.tiles_m - first_m < p.group_m) ? (p.tiles_m - first_m) : p.group_m;
    const int in_group = l % group_size;
    tile_m = first_m + in_group % gm;
    tile_n = in_group / gm;
}

// C tile <-> accumulators of one wavefront: FM x FN blocks of 32 x 32, block
// (fm, fn) at rows row0 + 32 fm, columns col0 + 32 fn (row0, col0 wave-uniform).
// Accumulator register i of lane l is row 8*(i/4) + 4*(l/32) + i%4, column l%32
// of its block.  Addresses are a wave-uniform row pointer plus one per-lane
// 32-bit offset, so that no per-element 64-bit address lives in registers.
// With `edge`, elements at rows >= M or columns >= N are read as 0 / not stored.
template <typename CT, int FM, int FN>
__device__ __forceinline__ void load_c_tile(floatx16 (&acc)[FM][FN], const CT* C, int64_t ldc,
                                            int row0, int col0, int lane, int M, int N, bool edge)
{
    const uint32_t voff = ((uint32_t)(4 * (lane >> 5)) * (uint32_t)ldc + (uint32_t)(lane & 31)) * (uint32_t)sizeof(CT);
    const int lrow = 4 * (lane >> 5), lcol = lane & 31;
#pragma unroll
    for (int fm = 0; fm < FM; fm++)
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int r = row0 + fm * 32 + 8 * (i / 4) + (i & 3);
            const char* rowp = reinterpret_cast<const char*>(C + (int64_t)r * ldc + col0);
#pragma unroll
            for (int fn = 0; fn < FN; fn++) {
                float v = 0.0f;
                if (!edge || (r + lrow < M && col0 + fn * 32 + lcol < N))
                    v = (float)*reinterpret_cast<const CT*>(rowp + voff + fn * 32 * sizeof(CT));
                acc[fm][fn][i] = v;
            }
        }
}

template <typename CT, int FM, int FN>
__device__ __forceinline__ void store_c_tile(const floatx16 (&acc)[FM][FN], CT* C, int64_t ldc,
                                             int row0, int col0, int lane, int M, int N, bool edge,
                                             const CT* bias, int relu)
{
    const uint32_t voff = ((uint32_t)(4 * (lane >> 5)) * (uint32_t)ldc + (uint32_t)(lane & 31)) * (uint32_t)sizeof(CT);
    const int lrow = 4 * (lane >> 5), lcol = lane & 31;
    float b[FN];
#pragma unroll
    for (int fn = 0; fn < FN; fn++) b[fn] = (bias && col0 + fn * 32 + lcol < N) ? (float)bias[col0 + fn * 32 + lcol] : 0.0f;
#pragma unroll
    for (int fm = 0; fm < FM; fm++)
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int r = row0 + fm * 32 + 8 * (i / 4) + (i & 3);
            char* rowp = reinterpret_cast<char*>(C + (int64_t)r * ldc + col0);
#pragma unroll
            for (int fn = 0; fn < FN; fn++)
                if (!edge || (r + lrow < M && col0 + fn * 32 + lcol < N))
                    *reinterpret_cast<CT*>(rowp + voff + fn * 32 * sizeof(CT)) = (CT)epilogue_value(acc[fm][fn][i], b[fn], relu);   // f16: one rounding, to nearest even
        }
}

// Accumulators formed with the operands exchanged (B fragment first) hold their block
// transposed: a lane owns 4 consecutive columns of one row of C per register group, so C moves
// 4 elements per lane and instruction (N is a multiple of 8 in the kernels that do this, so
// such a group lies entirely inside or outside C).  Vector accesses are only element-aligned.
template <typename CT> struct CVec4 {
    typedef CT type __attribute__((ext_vector_type(4), aligned(sizeof(CT))));
};

}  // namespace gemm_dev
