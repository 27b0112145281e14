// The 128 x 128 x 64 form of the four-wavefront kernel with an assembly k loop (gemm_w4a.hip
// describes the structure): wavefront tile 64 x 64 = 4 x 4 accumulators, one workgroup per
// compute unit.  It is for problems of at most one 128 x 128 tile per compute unit, where the
// phase-alternating kernel of that tile runs alone on its compute unit and its k step (a
// quarter of a microsecond of MFMAs) is shorter than the time a copy takes to arrive from L2,
// which its two or three buffers cannot cover.  Here the LDS is a ring of five stages (160 KB:
// copies run four k steps ahead), and a wavefront issues its 32 MFMAs of a k step back to
// back, with the 24 LDS reads and 8 copies of the step in their shadow and one barrier
// (gemm_w4a128_loop.inc, written by gen_w4a128_loop.py).
//
// C is read before the loop (into registers), added and stored behind it.  A k tail (K % 64
// != 0) is one unpipelined step through registers after the loop.  With a split k loop (skinny
// f32 problems) a workgroup multiplies a part of the k steps of its tile and adds the result to
// C atomically instead.  Requirements as for the other tuned kernels: A, B 16-byte aligned;
// lda, ldb, K, N multiples of 8.  Rows >= M / columns >= N are fetched from clamped addresses
// and never stored.
#include "gemm_device.h"
#include "../../include/gemm_f16.h"
#include "gemm_w4a128_loop.inc"

namespace {

using namespace gemm_dev;

constexpr int SBM = 128, SBN = 128;
constexpr int A_BUF = SBM * BK * 2;          // 16 KB
constexpr int B_BUF = BK * SBN * 2;          // 16 KB
constexpr int STAGE = A_BUF + B_BUF;         // a stage of the ring: A, then B
constexpr int STAGES = 5;                    // copies run STAGES - 1 k steps ahead
constexpr int W4A128_LDS = STAGES * STAGE;   // 160 KB
constexpr int B_ROW = SBN * 2;               // bytes per k row of a B stage
constexpr int NCOPY = 4;                     // copies per wavefront per A (or B) stage

// A wave-uniform pointer, said so that it is held in scalar registers (the copies take their
// base address from a scalar register pair).
__device__ __forceinline__ const char* uniform_ptr128(const void* ptr)
{
    const uint64_t v = (uint64_t)(uintptr_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const char*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

template <typename CT>
__global__ __launch_bounds__(256) void gemm_w4a128_kernel(const TiledParams p)
{
    __shared__ __attribute__((aligned(1024))) char smem[W4A128_LDS];
    const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_ptr_t)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm_base = (wave >> 1) * 64, wn_base = (wave & 1) * 64;

    // Split k (f32 C, no fused epilogue, few tiles and a long k loop: every compute unit should
    // stream operands): workgroup b takes tile b % tiles and part b / tiles of the k steps, and
    // adds its sums to C with atomic f32 additions -- C holds the old C already, the order of the
    // additions is not fixed.  K_len = this workgroup's part of K (all of it without a split).
    const bool split = p.k_split > 1;
    const int num_tiles = p.tiles_m * p.tiles_n;
    const int part = split ? (int)blockIdx.x / num_tiles : 0;
    int tile_m, tile_n;
    tile_of_block(p, (int)blockIdx.x - part * num_tiles, tile_m, tile_n);
    const int m0 = tile_m * SBM, n0 = tile_n * SBN;
    const bool edge = (m0 + SBM > p.M) || (n0 + SBN > p.N);

    const int k_steps = p.K / BK + (p.K % BK != 0);
    const int steps_per_part = split ? (k_steps + p.k_split - 1) / p.k_split : 0;
    if (split && part * steps_per_part >= k_steps) return;     // more parts than k steps: nothing to add
    const int k_begin = part * steps_per_part * BK;            // < K
    const int K_len = split ? (p.K - k_begin < steps_per_part * BK ? p.K - k_begin : steps_per_part * BK) : p.K;
    const int kt_full = K_len / BK;

    // ---- copy plan ------------------------------------------------------------------
    // A stage = 16 wave-wide copies of 8 rows x 128 B; wavefront w takes copies q = w + 4t.
    // Lane i writes (row 8q + i/8, chunk position i%8), which holds logical chunk position
    // ^ ((row/2)%8) = 4 (w%2) + i/16, the same for every t.
    const half_t* const a_tile = p.A + (int64_t)m0 * p.lda + k_begin;
    const half_t* const b_tile = p.B + (int64_t)k_begin * p.ldb + n0;
    const int a_chunk = (lane & 7) ^ (4 * (wave & 1) + (lane >> 4));
    uint32_t a_off[NCOPY];
#pragma unroll
    for (int t = 0; t < NCOPY; t++) {
        int row = 8 * (wave + 4 * t) + (lane >> 3);
        row = (m0 + row < p.M) ? row : p.M - 1 - m0;                 // clamp: loaded, never stored
        a_off[t] = ((uint32_t)row * (uint32_t)p.lda + 8 * a_chunk) * 2;
    }
    // B stage = 16 copies of 4 k rows x 256 B; copy q = w + 4t covers k rows 4q .. 4q+3.
    // Lane i writes (k row 4q + i/16, chunk position i%16), which holds logical chunk position
    // ^ swz(k row), swz = 4*(row%4) + 2*((row/8)%2) = 4 (i/16) + 2 ((w/2)%2), the same for every t.
    uint32_t b_off[NCOPY];
    const int b_krow0 = 4 * wave + (lane >> 4);                       // k row of copy t: b_krow0 + 16t
    {
        const int swz = ((lane >> 4) << 2) | (((wave >> 1) & 1) << 1);
        int col = 8 * ((lane & 15) ^ swz);
        if (n0 + col + 8 > p.N) col = 0;                              // clamp: loaded, never stored
#pragma unroll
        for (int t = 0; t < NCOPY; t++) b_off[t] = ((uint32_t)(b_krow0 + 16 * t) * (uint32_t)p.ldb + col) * 2;
    }
    const uint32_t lds_wave = smem_base + 1024 * wave;

    // ---- fragment read addresses ------------------------------------------------------
    // A operand of the 16x16x32 MFMA: lane l holds tile row l%16 of its 16-row block, k =
    // 8*(l/16)..+7 of the 32-wide slice s -> logical chunk 4s + l/16, stored at chunk ^ ((row/2)%8).
    uint32_t a_rd[2];
    {
        const uint32_t row_off = (uint32_t)(wm_base + (lane & 15)) * (BK * 2);
        const int sw = (lane & 15) >> 1;
#pragma unroll
        for (int s = 0; s < 2; s++)
            a_rd[s] = smem_base + row_off + (uint32_t)(((4 * s + (lane >> 4)) ^ sw) * 16);
    }
    // B operand: lane l holds column l%16, the same k.  One transposing read serves 16 lanes:
    // lanes 4r..4r+3 of a 16-lane block point at 16 consecutive columns of k row r and lane i
    // receives column i of rows 0..3.  Block b covers k 8b..8b+7 of the slice in two reads.
    uint32_t b_rd[4];
    {
        const int blk = lane >> 4, j = lane & 15;
        const uint32_t row_off = (uint32_t)(8 * blk + (j >> 2)) * B_ROW;
        const int swz = ((j >> 2) << 2) | ((blk & 1) << 1);           // of k rows 8b + j/4 (+4, +32)
#pragma unroll
        for (int fn = 0; fn < 4; fn++) {
            const int chunk = 2 * ((wn_base >> 4) + fn) + ((j & 3) >> 1);   // 16-byte chunk of columns 4(j%4)..+3
            b_rd[fn] = smem_base + A_BUF + row_off + (uint32_t)((chunk ^ swz) * 16 + 8 * (j & 1));
        }
    }

    // ---- C in: fetched first, so that its way from memory overlaps that of the first k steps
    // (a wavefront alone on its SIMD has the registers: 64 for an f32 tile) ------------------
    // Transposed 16 x 16 blocks (B fragment first): register r of lane l is row l%16, column
    // 4*(l/16) + r of block (fm, fn): one vector access per block.
    CT* const Cbase = (CT*)p.C;
    typedef typename CVec4<CT>::type ctx4;
    const int c_lrow = lane & 15, c_lcol = 4 * (lane >> 4);
    const uint32_t c_voff = ((uint32_t)c_lrow * (uint32_t)p.ldc + (uint32_t)c_lcol) * (uint32_t)sizeof(CT);
    const int c_row0 = m0 + wm_base, c_col0 = n0 + wn_base;
    float bias4[4][4];
#pragma unroll
    for (int fn = 0; fn < 4; fn++)
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int col = c_col0 + fn * 16 + c_lcol + e;
            bias4[fn][e] = (p.bias && col < p.N) ? (float)reinterpret_cast<const CT*>(p.bias)[col] : 0.0f;
        }
    // block (fm, fn): is this lane's group inside C?  (N is a multiple of 8: all 4 columns or none)
    auto c_ok = [&](int fm, int fn) -> bool {
        return !edge || ((c_row0 + fm * 16 + c_lrow < p.M) && (c_col0 + fn * 16 + c_lcol < p.N));
    };
    // a group outside C reads the first four elements of the workgroup's tile instead (always
    // inside C) and is not used
    ctx4 cin[4][4];
    if (!split)
#pragma unroll
    for (int fm = 0; fm < 4; fm++)
#pragma unroll
        for (int fn = 0; fn < 4; fn++) {
            const bool ok = c_ok(fm, fn);
            const char* rowp = ok ? reinterpret_cast<const char*>(Cbase + (int64_t)(c_row0 + fm * 16) * p.ldc + c_col0)
                                  : reinterpret_cast<const char*>(Cbase + (int64_t)m0 * p.ldc + n0);
            const uint32_t off = ok ? c_voff + (uint32_t)(fn * 16 * sizeof(CT)) : 0u;
            cin[fm][fn] = *reinterpret_cast<const ctx4*>(rowp + off);
        }

    floatx4 acc[4][4];
    if (kt_full > 0) {
        // k steps 0..3 into stages 0..3 (a k step beyond the last one: k step 0 once more, which
        // nobody reads; the loop's waits count on 8 copies per stage); the loop copies from k
        // step 4 on.  Only k step 0 (and C, requested before it) is waited for here: the wait
        // in the middle of k step j leaves the 20 copies behind those of step j + 1 in flight,
        // which holds from j = 0 on with steps 2, 3 and half of 4 behind step 1.
#pragma unroll
        for (int s = 0; s < STAGES - 1; s++) {
            const int ks = s < kt_full ? s : 0;
            const char* const a_src = uniform_ptr128(a_tile + (int64_t)ks * BK);
            const char* const b_src = uniform_ptr128(b_tile + (int64_t)ks * BK * p.ldb);
#pragma unroll
            for (int t = 0; t < NCOPY; t++) async_copy16(a_src, a_off[t], lds_wave + s * STAGE + 4096 * t);
#pragma unroll
            for (int t = 0; t < NCOPY; t++) async_copy16(b_src, b_off[t], lds_wave + s * STAGE + A_BUF + 4096 * t);
        }
        asm volatile("s_waitcnt vmcnt(24)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");

        const uint64_t a_base = (uint64_t)(uintptr_t)a_tile, b_base = (uint64_t)(uintptr_t)b_tile;
        const uint32_t b_step = (uint32_t)BK * (uint32_t)p.ldb * 2u;                // bytes per k step of B (ldb <= 2^22)
        const uint64_t a_ptr = a_base + (STAGES - 1) * BK * 2, b_ptr = b_base + (STAGES - 1) * (uint64_t)b_step;
        const uint32_t a_base_lo = __builtin_amdgcn_readfirstlane((uint32_t)a_base), a_base_hi = __builtin_amdgcn_readfirstlane((uint32_t)(a_base >> 32));
        const uint32_t b_base_lo = __builtin_amdgcn_readfirstlane((uint32_t)b_base), b_base_hi = __builtin_amdgcn_readfirstlane((uint32_t)(b_base >> 32));
        const uint32_t a_ptr_lo = __builtin_amdgcn_readfirstlane((uint32_t)a_ptr), a_ptr_hi = __builtin_amdgcn_readfirstlane((uint32_t)(a_ptr >> 32));
        const uint32_t b_ptr_lo = __builtin_amdgcn_readfirstlane((uint32_t)b_ptr), b_ptr_hi = __builtin_amdgcn_readfirstlane((uint32_t)(b_ptr >> 32));
        asm volatile(W4A128_LOOP_ASM : W4A128_LOOP_OUTPUTS(acc) : W4A128_LOOP_INPUTS : W4A128_LOOP_CLOBBERS);
    } else {
#pragma unroll
        for (int fm = 0; fm < 4; fm++)
#pragma unroll
            for (int fn = 0; fn < 4; fn++) acc[fm][fn] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
    }

    // ---- k tail: one unpipelined step through registers, zero beyond K ------------------
    if (K_len % BK != 0) {
        __builtin_amdgcn_s_barrier();                // every wavefront is out of the loop and its copies have landed: stage 0 is free
        const int k0 = kt_full * BK, krem = K_len - k0;
        const char* a_src = (const char*)(a_tile + k0);
        const char* b_src = (const char*)(b_tile + (int64_t)k0 * p.ldb);
#pragma unroll
        for (int t = 0; t < NCOPY; t++) {
            uintx4 va = {0u, 0u, 0u, 0u}, vb = {0u, 0u, 0u, 0u};
            if (8 * a_chunk < krem) va = *reinterpret_cast<const uintx4*>(a_src + a_off[t]);
            if (b_krow0 + 16 * t < krem) vb = *reinterpret_cast<const uintx4*>(b_src + b_off[t]);
            *(__attribute__((address_space(3))) uintx4*)(uintptr_t)(lds_wave + 4096 * t + 16 * lane) = va;
            *(__attribute__((address_space(3))) uintx4*)(uintptr_t)(lds_wave + A_BUF + 4096 * t + 16 * lane) = vb;
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 2; s++) {
            half8 fa[4], fb[4];
#pragma unroll
            for (int fn = 0; fn < 4; fn++) {
                const uint32_t addr = b_rd[fn] + s * 32 * B_ROW;
                fb[fn] = __builtin_shufflevector(lds_read_tr16(addr), lds_read_tr16(addr + 4 * B_ROW), 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int fm = 0; fm < 4; fm++) fa[fm] = lds_read_b128(a_rd[s] + fm * 16 * (BK * 2));
#pragma unroll
            for (int fm = 0; fm < 4; fm++)
#pragma unroll
                for (int fn = 0; fn < 4; fn++)
                    acc[fm][fn] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fb[fn], fa[fm], acc[fm][fn], 0, 0, 0);
        }
    }

    // ---- split k: this part's sums are added to C (only the launcher's f32 instantiation) ----
    // One atomic instruction per row of the wavefront's 64 x 64 block, 64 consecutive floats
    // (measured 190 G additions/s; in the accumulators' own layout -- 16 rows x 4 floats per
    // instruction -- 70 G/s): the block goes through a wavefront-private 17 KB of the LDS, which
    // is free once every wavefront is through its last k step.
    if constexpr (sizeof(CT) == 4) {
        if (split) {
            constexpr uint32_t T_PITCH = 64 * 4 + 16;                 // bytes per row: rows 8 apart share banks, two at a time
            const uint32_t tbuf = smem_base + (uint32_t)wave * (64u * T_PITCH);
            __syncthreads();
#pragma unroll
            for (int fm = 0; fm < 4; fm++)
#pragma unroll
                for (int fn = 0; fn < 4; fn++)
                    *(__attribute__((address_space(3))) floatx4*)(uintptr_t)(tbuf + (uint32_t)(fm * 16 + c_lrow) * T_PITCH + (uint32_t)(fn * 16 + c_lcol) * 4) = acc[fm][fn];
            const int rows_in = p.M - c_row0 < 64 ? p.M - c_row0 : 64;             // rows of the block inside C (may be <= 0)
            const bool col_in = c_col0 + lane < p.N;
            float* const cbase = reinterpret_cast<float*>(Cbase) + (int64_t)c_row0 * p.ldc + c_col0 + lane;
            for (int r = 0; r < rows_in; r++) {
                const float v = *(__attribute__((address_space(3))) const float*)(uintptr_t)(tbuf + (uint32_t)r * T_PITCH + 4u * lane);
                // a part that sums to zero leaves C alone (the memory's adders need not keep a subnormal C + 0)
                if (col_in && v != 0.0f) unsafeAtomicAdd(cbase + (int64_t)r * p.ldc, v);
            }
            return;
        }
    }
    // ---- + C, + bias, ReLU, -> C ------------------------------------------------------
#pragma unroll
    for (int fm = 0; fm < 4; fm++) {
        char* rowp = reinterpret_cast<char*>(Cbase + (int64_t)(c_row0 + fm * 16) * p.ldc + c_col0);
#pragma unroll
        for (int fn = 0; fn < 4; fn++) {
            ctx4 v;
#pragma unroll
            for (int e = 0; e < 4; e++) v[e] = (CT)epilogue_value(acc[fm][fn][e] + (float)cin[fm][fn][e], bias4[fn][e], p.relu);   // f16: one rounding, to nearest even
            if (c_ok(fm, fn))
                *reinterpret_cast<ctx4*>(rowp + c_voff + fn * 16 * sizeof(CT)) = v;
        }
    }
}

int64_t grid_w4a128(int64_t M, int64_t N)
{
    const int64_t tm = (M + SBM - 1) / SBM, tn = (N + SBN - 1) / SBN;
    if (tm > 0 && tn > INT32_MAX / tm) return -1;
    return tm * tn;
}

int launch_w4a128(const GemmArgs& a)
{
    const int64_t g = grid_w4a128(a.M, a.N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    TiledParams p = make_tiled_params(a, SBM, SBN, 8);   // an XCD's 64 concurrent tiles form an 8 x 8 block of C
    // the parts of a split k loop add to C atomically: f32 C and no bias or activation, which would have to wait for the last part
    const int parts = (a.k_split > 1 && !a.c_is_f16 && !a.bias && !a.relu) ? a.k_split : 1;
    if (g * parts > INT32_MAX) return GEMM_F16_ERR_SIZE;
    p.k_split = parts;
    if (a.c_is_f16)
        hipLaunchKernelGGL(gemm_w4a128_kernel<half_t>, dim3((unsigned)g), dim3(256), 0, a.stream, p);
    else
        hipLaunchKernelGGL(gemm_w4a128_kernel<float>, dim3((unsigned)(g * parts)), dim3(256), 0, a.stream, p);
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}

const GemmConfigDesc kW4a128 = {
    "w4a_128x128x64", SBM, SBN, BK, 4, 64, 64, W4A128_LDS, true, launch_w4a128, grid_w4a128};

}  // namespace

const GemmConfigDesc* deep_ring_config() { return &kW4a128; }
