// The long-k kernel: 256 x 256 C tile per workgroup, FOUR wavefronts (one per
// SIMD), each owning a 128 x 128 block -- 8 x 8 accumulators of 16 x 16 = 256
// registers, the whole AccVGPR file -- with its k loop written in assembly.
//
// Why this shape: under a dense MFMA load with random operands the part is
// power-limited, so what counts is energy per flop, and a 128 x 128 wavefront
// tile reads a third less LDS per flop than eight wavefronts of 128 x 64.  Why
// assembly: a wavefront that is alone on its SIMD has nobody to hide the
// compiler's address arithmetic, branches and waits behind (the C++ form of this
// kernel, ladder/gemm_w4.hip, keeps the matrix pipe 43 % busy); here the loop
// body holds MFMAs, LDS reads, copies and scalar pointer arithmetic only
// (gemm_w4a_loop.inc, written by gen_w4a_loop.py, which documents the schedule).
// Against the phase-alternating kernel it is level at four tiles of 128 k steps
// per compute unit and 1-3 % ahead where k loops are longer; the selector takes
// it there.
//
// The steps are those of the paper's recipe (Algorithm "Two-level tiled tensor
// core Matmul"; the copies of later k tiles in flight while the current one is
// multiplied, sections "Global Memory Load Latency Hiding" and "Completing
// Latency Hiding").  C is moved once per tile (section "Generating WMMA Ops and
// More"): in f32 mode, with enough k steps, it is read and added to the running
// sums during the first k steps of the loop (a compute unit takes ~12 us to
// bring a tile of C in from HBM; behind the loop its matrix units would idle
// meanwhile) and stored behind it, both through a range-checked buffer view of
// the wavefront's part of C, so that edge tiles take the same straight-line
// code; otherwise it is read, added and stored behind the loop.
//
// Around the loop, in C++: the copy plan and fragment addresses (the LDS image
// and swizzles of ladder/gemm_w4.hip), the first two k steps' copies, a k tail
// (K % 64 != 0) as one unpipelined step through registers after the loop, and
// the epilogue (+ C where it is not in the sums yet, + bias, ReLU, -> C).
//
// Requirements as for the other tuned kernels: A, B 16-byte aligned; lda, ldb,
// K, N multiples of 8.  Rows >= M / columns >= N are fetched from clamped
// addresses and never stored.
#include <type_traits>
#include "gemm_device.h"
#include "../../include/gemm_f16.h"
#include "gemm_w4a_loop.inc"

namespace {

using namespace gemm_dev;

constexpr int WBM = 256, WBN = 256;
constexpr int A_BUF = WBM * BK * 2;          // 32 KB
constexpr int B_BUF = BK * WBN * 2;          // 32 KB
constexpr int B_REGION = 2 * A_BUF;          // after the two A buffers
constexpr int W4A_LDS = 2 * A_BUF + 3 * B_BUF;  // 160 KB
constexpr int B_ROW = WBN * 2;               // bytes per k row of a B stage
constexpr int NCOPY = 8;                     // copies per wavefront per A (or B) stage

// A wave-uniform pointer, said so that it is held in scalar registers (the copies take their
// base address from a scalar register pair).
__device__ __forceinline__ const char* uniform_ptr(const void* ptr)
{
    const uint64_t v = (uint64_t)(uintptr_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const char*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

template <typename CT>
__global__ __launch_bounds__(256) void gemm_w4a_kernel(const TiledParams p)
{
    __shared__ __attribute__((aligned(1024))) char smem[W4A_LDS];
    const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_ptr_t)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm_base = (wave >> 1) * 128, wn_base = (wave & 1) * 128;

    int tile_m, tile_n;
    tile_of_block(p, blockIdx.x, tile_m, tile_n);
    const int m0 = tile_m * WBM, n0 = tile_n * WBN;
    const bool edge = (m0 + WBM > p.M) || (n0 + WBN > p.N);

    const int kt_full = p.K / BK;

    // ---- copy plan (the LDS image and swizzles of gemm_w4.hip) -----------------
    // A stage = 32 wave-wide copies of 8 rows x 128 B; wavefront w takes copies
    // q = w + 4t.  Lane i writes (row 8q + i/8, chunk position i%8), which holds
    // logical chunk position ^ ((row/2)%8).
    const half_t* const a_tile = p.A + (int64_t)m0 * p.lda;
    const half_t* const b_tile = p.B + n0;
    const int a_chunk = (lane & 7) ^ (4 * (wave & 1) + (lane >> 4));
    uint32_t a_off[NCOPY];
#pragma unroll
    for (int t = 0; t < NCOPY; t++) {
        int row = 8 * (wave + 4 * t) + (lane >> 3);
        row = (m0 + row < p.M) ? row : p.M - 1 - m0;                 // clamp: loaded, never stored
        a_off[t] = ((uint32_t)row * (uint32_t)p.lda + 8 * a_chunk) * 2;
    }
    // B stage = 32 copies of 2 k rows x 512 B; copy q = w + 4t covers k rows 2q,
    // 2q+1.  Lane i writes (k row 2q + i/32, chunk position i%32), which holds
    // logical chunk position ^ swz(k row), swz = 4*(row%4) + 2*((row/8)%2).
    uint32_t b_off[NCOPY];
    const int b_krow0 = 2 * wave + (lane >> 5);                       // k row of copy t: b_krow0 + 8t
#pragma unroll
    for (int t = 0; t < NCOPY; t++) {
        const int swz = ((b_krow0 & 3) << 2) | ((t & 1) << 1);
        int col = 8 * ((lane & 31) ^ swz);
        if (n0 + col + 8 > p.N) col = 0;                              // clamp: loaded, never stored
        b_off[t] = ((uint32_t)(b_krow0 + 8 * t) * (uint32_t)p.ldb + col) * 2;
    }
    const uint32_t lds_wave = smem_base + 1024 * wave;

    // ---- fragment read addresses ------------------------------------------------
    uint32_t a_rd[2];
    {
        const uint32_t row_off = (uint32_t)(wm_base + (lane & 15)) * (BK * 2);
        const int sw = (lane & 15) >> 1;
#pragma unroll
        for (int s = 0; s < 2; s++)
            a_rd[s] = smem_base + row_off + (uint32_t)(((4 * s + (lane >> 4)) ^ sw) * 16);
    }
    uint32_t b_rd[8];
    {
        const int blk = lane >> 4, j = lane & 15;
        const uint32_t row_off = (uint32_t)(8 * blk + (j >> 2)) * B_ROW;
        const int swz = ((j >> 2) << 2) | ((blk & 1) << 1);
#pragma unroll
        for (int fn = 0; fn < 8; fn++) {
            const int chunk = 2 * ((wn_base >> 4) + fn) + ((j & 3) >> 1);
            b_rd[fn] = smem_base + B_REGION + row_off + (uint32_t)((chunk ^ swz) * 16 + 8 * (j & 1));
        }
    }

    // Transposed 16 x 16 blocks (B fragment first): register r of lane l is row
    // l%16, column 4*(l/16) + r of block (fm, fn): one vector access per block.
    CT* const Cbase = (CT*)p.C;
    typedef typename CVec4<CT>::type ctx4;
    const int c_lrow = lane & 15, c_lcol = 4 * (lane >> 4);
    const uint32_t c_voff = ((uint32_t)c_lrow * (uint32_t)p.ldc + (uint32_t)c_lcol) * (uint32_t)sizeof(CT);
    const int c_row0 = m0 + wm_base, c_col0 = n0 + wn_base;
    // C is read and added inside the loop in f32 mode where the loop is long enough; otherwise
    // behind it
    const bool c_in_loop = sizeof(CT) == 4 && kt_full >= W4A_C_STEPS;
    // The loads inside the loop are range-checked buffer loads on this wavefront's part of C:
    // base = its first element, c_bytes = distance to the end of C's last element (0 if the
    // block lies outside C; offsets inside a 128-row block stay below 2^31).  A row beyond C's
    // last is out of range by that; a lane whose 4 columns of block column fn lie beyond C's
    // last gets an offset that is out of range whatever the row.  Out of range = no access, 0.
    uint32_t c_voff_fn[8];
#pragma unroll
    for (int fn = 0; fn < 8; fn++) c_voff_fn[fn] = (c_col0 + fn * 16 + c_lcol < p.N) ? c_voff : 0x80000000u;
    const int64_t c_span = (c_row0 < p.M && c_col0 < p.N)
                               ? ((int64_t)(p.M - 1 - c_row0) * p.ldc + (p.N - c_col0)) * (int64_t)sizeof(CT) : 0;
    const uint32_t c_bytes = __builtin_amdgcn_readfirstlane((uint32_t)(c_span < 0x7fffffff ? c_span : 0x7fffffff));

    floatx4 acc[8][8];
    if (kt_full > 0) {
        // k steps 0 and 1 into A buffers 0, 1 and B buffers 0, 1; the loop copies from k step 2 on
        const int first = kt_full < 2 ? kt_full : 2;
        for (int s = 0; s < first; s++) {
            const char* const a_src = uniform_ptr(a_tile + (int64_t)s * BK);
            const char* const b_src = uniform_ptr(b_tile + (int64_t)s * BK * p.ldb);
#pragma unroll
            for (int t = 0; t < NCOPY; t++) {
                async_copy16(a_src, a_off[t], lds_wave + s * A_BUF + 4096 * t);
                async_copy16(b_src, b_off[t], lds_wave + B_REGION + s * B_BUF + 4096 * t);
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");

        const uint64_t a_base = (uint64_t)(uintptr_t)a_tile, b_base = (uint64_t)(uintptr_t)b_tile;
        const uint32_t b_step = (uint32_t)BK * (uint32_t)p.ldb * 2u;                // bytes per k step of B (ldb <= 2^22)
        const uint64_t a_ptr = a_base + 2 * BK * 2, b_ptr = b_base + 2 * (uint64_t)b_step;
        const uint32_t a_base_lo = __builtin_amdgcn_readfirstlane((uint32_t)a_base), a_base_hi = __builtin_amdgcn_readfirstlane((uint32_t)(a_base >> 32));
        const uint32_t b_base_lo = __builtin_amdgcn_readfirstlane((uint32_t)b_base), b_base_hi = __builtin_amdgcn_readfirstlane((uint32_t)(b_base >> 32));
        const uint32_t a_ptr_lo = __builtin_amdgcn_readfirstlane((uint32_t)a_ptr), a_ptr_hi = __builtin_amdgcn_readfirstlane((uint32_t)(a_ptr >> 32));
        const uint32_t b_ptr_lo = __builtin_amdgcn_readfirstlane((uint32_t)b_ptr), b_ptr_hi = __builtin_amdgcn_readfirstlane((uint32_t)(b_ptr >> 32));
        const uint64_t c_wave = (uint64_t)(uintptr_t)(Cbase + (int64_t)c_row0 * p.ldc + c_col0);
        const uint32_t c_lo = __builtin_amdgcn_readfirstlane((uint32_t)c_wave), c_hi = __builtin_amdgcn_readfirstlane((uint32_t)(c_wave >> 32) & 0xffffu);
        const uint32_t c_rowstep = 16u * (uint32_t)p.ldc * (uint32_t)sizeof(CT);    // bytes from one row of blocks to the next (ldc <= 2^22)
        if (c_in_loop)
            asm volatile(W4A_LOOP_C_ASM : W4A_LOOP_OUTPUTS(acc) : W4A_LOOP_INPUTS : W4A_LOOP_CLOBBERS);
        else
            asm volatile(W4A_LOOP_ASM : W4A_LOOP_OUTPUTS(acc) : W4A_LOOP_INPUTS : W4A_LOOP_CLOBBERS);
    } else {
#pragma unroll
        for (int fm = 0; fm < 8; fm++)
#pragma unroll
            for (int fn = 0; fn < 8; fn++) acc[fm][fn] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
    }

    // ---- k tail: one unpipelined step through registers, zero beyond K ------------
    if (p.K % BK != 0) {
        __builtin_amdgcn_s_barrier();                // every wavefront is out of the loop: the buffers are free
        const int k0 = kt_full * BK, krem = p.K - k0;
        const char* a_src = (const char*)(a_tile + k0);
        const char* b_src = (const char*)(b_tile + (int64_t)k0 * p.ldb);
#pragma unroll
        for (int t = 0; t < NCOPY; t++) {
            uintx4 va = {0u, 0u, 0u, 0u}, vb = {0u, 0u, 0u, 0u};
            if (8 * a_chunk < krem) va = *reinterpret_cast<const uintx4*>(a_src + a_off[t]);
            if (b_krow0 + 8 * t < krem) vb = *reinterpret_cast<const uintx4*>(b_src + b_off[t]);
            *(__attribute__((address_space(3))) uintx4*)(uintptr_t)(lds_wave + 4096 * t + 16 * lane) = va;
            *(__attribute__((address_space(3))) uintx4*)(uintptr_t)(lds_wave + B_REGION + 4096 * t + 16 * lane) = vb;
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 2; s++) {
            half8 fa[8], fb[8];
#pragma unroll
            for (int fn = 0; fn < 8; fn++) {
                const uint32_t addr = b_rd[fn] + s * 32 * B_ROW;
                fb[fn] = __builtin_shufflevector(lds_read_tr16(addr), lds_read_tr16(addr + 4 * B_ROW), 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int fm = 0; fm < 8; fm++) fa[fm] = lds_read_b128(a_rd[s] + fm * 16 * (BK * 2));
#pragma unroll
            for (int fm = 0; fm < 8; fm++)
#pragma unroll
                for (int fn = 0; fn < 8; fn++)
                    acc[fm][fn] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fb[fn], fa[fm], acc[fm][fn], 0, 0, 0);
        }
    }

    // ---- + C, -> C -------------------------------------------------------------------
    // fused epilogue: this lane's 4 columns of the bias for each of its 8 block columns
    float bias4[8][4];
#pragma unroll
    for (int fn = 0; fn < 8; fn++)
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const int col = c_col0 + fn * 16 + c_lcol + e;
            bias4[fn][e] = (p.bias && col < p.N) ? (float)reinterpret_cast<const CT*>(p.bias)[col] : 0.0f;
        }
    auto c_ok = [&](int fm, int fn) -> bool {
        return !edge || ((c_row0 + fm * 16 + c_lrow < p.M) && (c_col0 + fn * 16 + c_lcol < p.N));
    };
    // a group outside C reads the first four elements of the workgroup's tile instead (always
    // inside C; the wavefront's own 128 x 128 block may lie outside altogether) and is not used
    auto c_load = [&](int fm, int fn) -> ctx4 {
        const bool ok = c_ok(fm, fn);
        const char* rowp = ok ? reinterpret_cast<const char*>(Cbase + (int64_t)(c_row0 + fm * 16) * p.ldc + c_col0)
                              : reinterpret_cast<const char*>(Cbase + (int64_t)m0 * p.ldc + n0);
        const uint32_t off = ok ? c_voff + (uint32_t)(fn * 16 * sizeof(CT)) : 0u;
        return *reinterpret_cast<const ctx4*>(rowp + off);
    };
    auto fetch_rows = [&](int fm0, ctx4 (&cin)[2][8]) {
#pragma unroll
        for (int r = 0; r < 2; r++)
#pragma unroll
            for (int fn = 0; fn < 8; fn++) cin[r][fn] = c_load(fm0 + r, fn);
    };
    auto finish_rows = [&](int fm0, const ctx4 (&cin)[2][8]) {
#pragma unroll
        for (int r = 0; r < 2; r++) {
            const int fm = fm0 + r;
            char* rowp = reinterpret_cast<char*>(Cbase + (int64_t)(c_row0 + fm * 16) * p.ldc + c_col0);
#pragma unroll
            for (int fn = 0; fn < 8; fn++) {
                ctx4 v;
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] = (CT)epilogue_value(acc[fm][fn][e] + (float)cin[r][fn][e], bias4[fn][e], p.relu);   // f16: one rounding, to nearest even
                if (c_ok(fm, fn))
                    *reinterpret_cast<ctx4*>(rowp + c_voff + fn * 16 * sizeof(CT)) = v;
            }
        }
    };
    auto fence = [&]() { __builtin_amdgcn_sched_barrier(0); };
    if (c_in_loop) {
        // C is in the sums already: only stores, through the same range-checked view of C as
        // the loads in the loop -- a store to a row or column beyond C's last is dropped by the
        // check, so that edge tiles need no masks either
        const __amdgpu_buffer_rsrc_t c_rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void*)(Cbase + (int64_t)c_row0 * p.ldc + c_col0), 0, c_bytes, 0x20000);
        const uint32_t c_rowstep = 16u * (uint32_t)p.ldc * (uint32_t)sizeof(CT);
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int fm = 0; fm < 8; fm++)
#pragma unroll
            for (int fn = 0; fn < 8; fn++) {
                floatx4 v;
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] = epilogue_value(acc[fm][fn][e], bias4[fn][e], p.relu);
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), c_rsrc, c_voff_fn[fn] + fn * 64, fm * c_rowstep, 0);
            }
        return;
    }
    ctx4 c_q0[2][8], c_q1[2][8], c_q2[2][8];
    fetch_rows(0, c_q0); fetch_rows(2, c_q1); fetch_rows(4, c_q2); fence();
    finish_rows(0, c_q0); fence();
    fetch_rows(6, c_q0); fence();
    finish_rows(2, c_q1); fence();
    finish_rows(4, c_q2); fence();
    finish_rows(6, c_q0);
}

int64_t grid_w4a(int64_t M, int64_t N)
{
    const int64_t tm = (M + WBM - 1) / WBM, tn = (N + WBN - 1) / WBN;
    if (tm > 0 && tn > INT32_MAX / tm) return -1;
    return tm * tn;
}

int launch_w4a(const GemmArgs& a)
{
    const int64_t g = grid_w4a(a.M, a.N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    const TiledParams p = make_tiled_params(a, WBM, WBN, 8);   // an XCD's 32 concurrent tiles form an 8 x 4 block of C
    if (a.c_is_f16)
        hipLaunchKernelGGL(gemm_w4a_kernel<half_t>, dim3((unsigned)g), dim3(256), 0, a.stream, p);
    else
        hipLaunchKernelGGL(gemm_w4a_kernel<float>, dim3((unsigned)g), dim3(256), 0, a.stream, p);
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}

const GemmConfigDesc kW4a = {
    "w4a_256x256x64", WBM, WBN, BK, 4, 128, 128, W4A_LDS, true, launch_w4a, grid_w4a};

}  // namespace

const GemmConfigDesc* long_k_config() { return &kW4a; }
