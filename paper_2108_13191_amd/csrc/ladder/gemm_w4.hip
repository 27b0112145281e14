// The large-problem kernel: 256 x 256 C tile per workgroup, FOUR wavefronts
// (one per SIMD), each owning a 128 x 128 block: 8 x 8 accumulators of 16 x 16
// = 256 registers, the whole AccVGPR file.  k steps of 64, f16 MFMA
// (v_mfma_f32_16x16x32_f16), f32 accumulation.
//
// Why this shape on MI355X: under a dense MFMA load with random operands the
// part is power-bound (an MFMA-only loop on N(0,1) data sustains about 64 % of
// the nominal rate), so what counts is energy per flop.  A 128 x 128 wavefront
// tile reads (128 + 128) x 64 f16 = 32 KB of LDS per k step and wavefront, one
// third less than eight wavefronts of 128 x 64; the 16x16x32 instruction moves
// fewer accumulator bytes per flop than 32x32x16 and measured 6 % faster in
// that MFMA-only loop.
//
// The steps are those of the paper's recipe (Algorithm "Two-level tiled tensor
// core Matmul"; C handled once per tile outside the k loop, section
// "Generating WMMA Ops and More"; the copies of later k tiles in flight while
// the current one is multiplied, sections "Global Memory Load Latency Hiding"
// and "Completing Latency Hiding"), re-timed for one wavefront per SIMD:
//
//   * A k step is two 32-wide k slices of 64 MFMAs per wavefront.  The
//     wavefront is alone on its SIMD and issues in order, so an instruction
//     placed behind an MFMA that waits for the matrix pipe waits with it;
//     therefore every pair of MFMAs is followed by exactly one other
//     instruction -- one of the 24 LDS fragment reads of the NEXT slice
//     (fragments are double buffered in registers) or one of the 8 global ->
//     LDS copies of the slice -- which issues in the shadow of the MFMAs.  The
//     scheduler is told to keep that order.
//   * LDS (160 KB): 2 A buffers (256 x 64 f16, 32 KB) and 3 B buffers (64 x 256
//     f16, 32 KB).  One workgroup barrier per k step, between the two slices:
//     behind it the A buffer just consumed takes the copies of k step +2
//     (issued during the second slice, a whole slice before they are needed)
//     and the B buffer consumed one step earlier takes k step +2's B during
//     the following first slice (more than a k step ahead).
//   * Copies are global_load_lds_dwordx4, XOR-swizzled by the choice of the
//     16-byte chunk each lane fetches; A fragments ds_read_b128, B fragments
//     ds_read_b64_tr_b16 (B is N-contiguous, the MFMA wants K-contiguous
//     lanes).
//   * The MFMA is issued with the B fragment as first operand, i.e. it forms
//     the transposed 16 x 16 block: a lane then owns 4 CONSECUTIVE columns of
//     one row of C, so C moves 16 bytes per lane (f32) instead of 4.
//   * The accumulators start at zero.  C is read once: a quarter of the tile
//     during the last k step (whose copy slots are empty), the rest while the
//     first quarters are added and stored.  C + sum is formed as sum + C.
//
// Requirements as for the other tuned kernels: A, B 16-byte aligned; lda, ldb,
// K, N multiples of 8.  Rows >= M / columns >= N are fetched from clamped
// addresses and never stored; the k tail is zero-filled through registers.
#include "../gemm_device.h"
#include "../../../include/gemm_f16.h"

namespace {

using namespace gemm_dev;

constexpr int WBM = 256, WBN = 256;
constexpr int A_BUF = WBM * BK * 2;          // 32 KB
constexpr int B_BUF = BK * WBN * 2;          // 32 KB
constexpr int B_REGION = 2 * A_BUF;          // after the two A buffers
constexpr int W4_LDS = 2 * A_BUF + 3 * B_BUF;   // 160 KB
constexpr int B_ROW = WBN * 2;               // bytes per k row of a B stage
constexpr int NCOPY = 8;                     // copies per wavefront per A (or B) stage

template <bool B> struct BoolTag { static constexpr bool value = B; };

template <typename CT>
__global__ __launch_bounds__(256) void gemm_w4_kernel(const TiledParams p)
{
    __shared__ __attribute__((aligned(1024))) char smem[W4_LDS];
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
    const int KT = (p.K + BK - 1) / BK;

    // ---- copy plan ----------------------------------------------------------
    // A stage = 32 wave-wide copies of 8 rows x 128 B; wavefront w takes copies
    // q = w + 4t (t = 0..7).  Lane i writes (row 8q + i/8, chunk position i%8),
    // which must hold logical chunk position ^ ((row/2)%8) -- a per-lane
    // constant because q = w (mod 2).
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
    // 2q+1.  Lane i writes (k row 2q + i/32, chunk position i%32), which must
    // hold logical chunk position ^ swz(k row), swz = 4*(row%4) + 2*((row/8)%2):
    // the row%4 term spreads the four k rows of one transposing read over the
    // banks, the (row/8)%2 term those of the two 16-lane blocks (k and k+8)
    // that are served together.  (row/8)%2 = t%2 here.
    uint32_t b_off[NCOPY];
    const int b_krow0 = 2 * wave + (lane >> 5);                       // k row of copy t: b_krow0 + 8t
#pragma unroll
    for (int t = 0; t < NCOPY; t++) {
        const int swz = ((b_krow0 & 3) << 2) | ((t & 1) << 1);
        int col = 8 * ((lane & 31) ^ swz);
        if (n0 + col + 8 > p.N) col = 0;                              // clamp: loaded, never stored
        b_off[t] = ((uint32_t)(b_krow0 + 8 * t) * (uint32_t)p.ldb + col) * 2;
    }
    // copy t of the A stage of k step s into A buffer s%2
    auto copy_a = [&](int s, int t) {
        const uint32_t dst = smem_base + (s & 1) * A_BUF + 1024 * (wave + 4 * t);
        const char* src = (const char*)(a_tile + (int64_t)s * BK);
        if (s < kt_full) {
            async_copy16(src, a_off[t], dst);
        } else {                                                       // k tail: through registers, zero beyond K
            uintx4 v = {0u, 0u, 0u, 0u};
            if (8 * a_chunk < p.K - s * BK) v = *reinterpret_cast<const uintx4*>(src + a_off[t]);
            *(__attribute__((address_space(3))) uintx4*)(uintptr_t)(dst + 16 * lane) = v;
        }
    };
    // copy t of the B stage of k step s into B buffer s%3
    auto copy_b = [&](int s, int t) {
        const uint32_t dst = smem_base + B_REGION + (s % 3) * B_BUF + 1024 * (wave + 4 * t);
        const char* src = (const char*)(b_tile + (int64_t)s * BK * p.ldb);
        if (s < kt_full) {
            async_copy16(src, b_off[t], dst);
        } else {
            uintx4 v = {0u, 0u, 0u, 0u};
            if (b_krow0 + 8 * t < p.K - s * BK) v = *reinterpret_cast<const uintx4*>(src + b_off[t]);
            *(__attribute__((address_space(3))) uintx4*)(uintptr_t)(dst + 16 * lane) = v;
        }
    };

    // ---- prologue: what the steady-state schedule does not cover ---------------
#pragma unroll
    for (int t = 0; t < NCOPY; t++) { copy_a(0, t); copy_b(0, t); }
    if (KT > 1) {
#pragma unroll
        for (int t = 0; t < NCOPY; t++) { copy_a(1, t); copy_b(1, t); }
    }

    // ---- accumulators -------------------------------------------------------
    floatx4 acc[8][8];
#pragma unroll
    for (int fm = 0; fm < 8; fm++)
#pragma unroll
        for (int fn = 0; fn < 8; fn++) acc[fm][fn] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
    CT* const Cbase = (CT*)p.C;
    typedef typename CVec4<CT>::type ctx4;
    // Transposed 16 x 16 blocks (B fragment first): register r of lane l is row
    // l%16, column 4*(l/16) + r of block (fm, fn): one vector access per block.
    const int c_lrow = lane & 15, c_lcol = 4 * (lane >> 4);
    const uint32_t c_voff = ((uint32_t)c_lrow * (uint32_t)p.ldc + (uint32_t)c_lcol) * (uint32_t)sizeof(CT);
    const int c_row0 = m0 + wm_base, c_col0 = n0 + wn_base;
    // block (fm, fn): is this lane's group inside C?  (N is a multiple of 8: all 4 columns or none)
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
    ctx4 c_q0[2][8];               // C of accumulator rows 0, 1: fetched during the last k step

    // ---- fragment read addresses ----------------------------------------------
    // A operand of the 16x16x32 MFMA: lane l holds tile row l%16 of its 16-row
    // block, k = 8*(l/16)..+7 of the 32-wide slice s -> logical chunk 4s + l/16,
    // stored at chunk ^ ((row/2)%8).
    uint32_t a_rd[2];
    {
        const uint32_t row_off = (uint32_t)(wm_base + (lane & 15)) * (BK * 2);
        const int sw = (lane & 15) >> 1;
#pragma unroll
        for (int s = 0; s < 2; s++)
            a_rd[s] = smem_base + row_off + (uint32_t)(((4 * s + (lane >> 4)) ^ sw) * 16);
    }
    // B operand: lane l holds column l%16, the same k.  One transposing read
    // serves 16 lanes: lanes 4r..4r+3 of a 16-lane block point at 16
    // consecutive columns of k row r and lane i receives column i of rows 0..3.
    // Block b covers k 8b..8b+7 of the slice in two reads (+0..3, +4..7).
    uint32_t b_rd[8];
    {
        const int blk = lane >> 4, j = lane & 15;
        const uint32_t row_off = (uint32_t)(8 * blk + (j >> 2)) * B_ROW;
        const int swz = ((j >> 2) << 2) | ((blk & 1) << 1);           // of k rows 8b + j/4 (+4, +32)
#pragma unroll
        for (int fn = 0; fn < 8; fn++) {
            const int chunk = 2 * ((wn_base >> 4) + fn) + ((j & 3) >> 1);   // 16-byte chunk of columns 4(j%4)..+3
            b_rd[fn] = smem_base + B_REGION + row_off + (uint32_t)((chunk ^ swz) * 16 + 8 * (j & 1));
        }
    }

    half8 fa[2][8], fb[2][8];      // fragments of two k slices: [slice & 1][fm], [slice & 1][fn]
    half4 b_lo[8];                 // first half of a B operand until its second read is issued

    // read r (0..23) of slice s of (A buffer at a_base, B buffer at b_base)
    // into fragment set d: the 8 B operands (2 reads each) first, then the 8 A
    auto issue_read = [&](uint32_t a_base, uint32_t b_base, int s, int d, int r) {
        if (r < 16) {
            const int fn = r >> 1;
            const uint32_t addr = b_rd[fn] + b_base + s * 32 * B_ROW;
            if ((r & 1) == 0) b_lo[fn] = lds_read_tr16(addr);
            else fb[d][fn] = __builtin_shufflevector(b_lo[fn], lds_read_tr16(addr + 4 * B_ROW), 0, 1, 2, 3, 4, 5, 6, 7);
        } else {
            const int fm = r - 16;
            fa[d][fm] = lds_read_b128(a_rd[s] + a_base + fm * 16 * (BK * 2));
        }
    };
    // MFMA number i (0..63) of a slice, B fragment first = transposed block
    auto mfma_one = [&](int d, int i) {
        const int fm = i >> 3, fn = i & 7;
        acc[fm][fn] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fb[d][fn], fa[d][fm], acc[fm][fn], 0, 0, 0);
    };
    auto fence = [&]() { __builtin_amdgcn_sched_barrier(0); };

    // prologue copies have landed; publish, then fetch slice 0
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int r = 0; r < 24; r++) issue_read(0, 0, 0, 0, r);

    // ---- main loop -------------------------------------------------------------
    // k step j, unit u of a slice = MFMAs 2u, 2u+1 and one companion:
    //   slice 0: u 0-23 read r = u of slice 1 (same stage); u 24-31 copy B(j+2), copies 0-7
    //   barrier
    //   slice 1: u 0-23 read r = u of slice 0 of stage j+1;  u 24-31 copy A(j+2), copies 0-7
    // The last k step (LAST) has nothing to copy or prefetch; its 16 copy slots
    // fetch a quarter of the C tile instead.
    auto k_step = [&](int j, auto last_tag) {
        constexpr bool LAST = decltype(last_tag)::value;
        const uint32_t a_cur = (uint32_t)(j & 1) * A_BUF, a_nxt = a_cur ^ A_BUF;
        const uint32_t b_cur = (uint32_t)(j % 3) * B_BUF, b_nxt = (uint32_t)((j + 1) % 3) * B_BUF;
#pragma unroll
        for (int u = 0; u < 32; u++) {
            mfma_one(0, 2 * u); mfma_one(0, 2 * u + 1); fence();
            if (u < 24) issue_read(a_cur, b_cur, 1, 1, u);
            else if (LAST) c_q0[0][u - 24] = c_load(0, u - 24);
            else if (j + 2 < KT) copy_b(j + 2, u - 24);
            fence();
        }
        if (LAST) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        } else {
            // Everything but the 8 B copies just issued has landed (A(j+1),
            // B(j+1)) and this wavefront's reads of stage j are complete; after
            // the barrier that holds for all four wavefronts.
            if (j + 2 < kt_full) asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
            else                 asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        fence();
#pragma unroll
        for (int u = 0; u < 32; u++) {
            mfma_one(1, 2 * u); mfma_one(1, 2 * u + 1); fence();
            if (u < 24) { if (!LAST) issue_read(a_nxt, b_nxt, 0, 0, u); }
            else if (LAST) c_q0[1][u - 24] = c_load(1, u - 24);
            else if (j + 2 < KT) copy_a(j + 2, u - 24);
            fence();
        }
    };
    for (int j = 0; j + 1 < KT; j++) k_step(j, BoolTag<false>());
    k_step(KT - 1, BoolTag<true>());

    // ---- + C, -> C ---------------------------------------------------------------
    // Quarter by quarter (two accumulator rows = 16 vector accesses per lane):
    // the next quarter of C is fetched while the current one is added and stored.
    {
        auto finish_rows = [&](int fm0, const ctx4 (&cin)[2][8]) {
#pragma unroll
            for (int r = 0; r < 2; r++) {
                const int fm = fm0 + r;
                char* rowp = reinterpret_cast<char*>(Cbase + (int64_t)(c_row0 + fm * 16) * p.ldc + c_col0);
#pragma unroll
                for (int fn = 0; fn < 8; fn++) {
                    ctx4 v;
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] = (CT)(acc[fm][fn][e] + (float)cin[r][fn][e]);   // f16: one rounding, to nearest even
                    if (c_ok(fm, fn))
                        *reinterpret_cast<ctx4*>(rowp + c_voff + fn * 16 * sizeof(CT)) = v;
                }
            }
        };
        auto fetch_rows = [&](int fm0, ctx4 (&cin)[2][8]) {
#pragma unroll
            for (int r = 0; r < 2; r++)
#pragma unroll
                for (int fn = 0; fn < 8; fn++) cin[r][fn] = c_load(fm0 + r, fn);
        };
        ctx4 c_q1[2][8], c_q2[2][8];
        fetch_rows(2, c_q1); fetch_rows(4, c_q2); fence();
        finish_rows(0, c_q0); fence();
        fetch_rows(6, c_q0); fence();
        finish_rows(2, c_q1); fence();
        finish_rows(4, c_q2); fence();
        finish_rows(6, c_q0);
    }
}

int64_t grid_w4(int64_t M, int64_t N)
{
    const int64_t tm = (M + WBM - 1) / WBM, tn = (N + WBN - 1) / WBN;
    if (tm > 0 && tn > INT32_MAX / tm) return -1;
    return tm * tn;
}

int launch_w4(const GemmArgs& a)
{
    const int64_t g = grid_w4(a.M, a.N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    if (a.bias || a.relu) return GEMM_F16_ERR_CONFIG;      // this comparison kernel has no fused epilogue
    TiledParams p = make_tiled_params(a, WBM, WBN, 8);     // an XCD's 32 concurrent tiles form an 8 x 4 block of C
    p.bias = nullptr; p.relu = 0;
    if (a.c_is_f16)
        hipLaunchKernelGGL(gemm_w4_kernel<half_t>, dim3((unsigned)g), dim3(256), 0, a.stream, p);
    else
        hipLaunchKernelGGL(gemm_w4_kernel<float>, dim3((unsigned)g), dim3(256), 0, a.stream, p);
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}

const GemmConfigDesc kW4 = {
    "w4_256x256x64", WBM, WBN, BK, 4, 128, 128, W4_LDS, true, launch_w4, grid_w4};

}  // namespace

const GemmConfigDesc* w4_config() { return &kW4; }
