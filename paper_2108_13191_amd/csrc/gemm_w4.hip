// The large-problem kernel: 256 x 256 C tile per workgroup, FOUR wavefronts
// (one per SIMD), each owning a 128 x 128 block: 16 accumulators of 32 x 32 =
// 256 registers, the whole AccVGPR file.  k steps of 64, f16 MFMA
// (v_mfma_f32_32x32x16_f16), f32 accumulation.
//
// Why this shape on MI355X: under a dense MFMA load the part is power-bound,
// so what counts is work per flop.  A 128 x 128 wavefront tile reads
// (128 + 128) x 64 f16 = 32 KB of LDS per k step and wavefront, 128 KB per
// workgroup, one third less than eight wavefronts of 128 x 64; and each LDS
// byte is fetched from L2 once per 256 x 256 tile.
//
// The steps are those of the paper's recipe (Algorithm "Two-level tiled tensor
// core Matmul"; C hoisted out of the k loop, section "Generating WMMA Ops and
// More"; the copies of later k tiles in flight while the current one is
// multiplied, sections "Global Memory Load Latency Hiding" and "Completing
// Latency Hiding"), re-timed for one wavefront per SIMD:
//
//   * A k step is 64 MFMAs per wavefront, cut into 16 chunks of 4 MFMAs (one
//     accumulator row of one 16-wide k slice).  Every chunk also carries 3 of
//     the 12 LDS fragment reads of the NEXT slice (fragments are double
//     buffered in registers) and exactly ONE global -> LDS copy, so that the
//     LDS and the texture path see an even load and everything is issued in
//     the shadow of the MFMAs.  The scheduler may not move anything across a
//     chunk boundary.
//   * LDS (160 KB): 2 A buffers (256 x 64 f16, 32 KB) and 3 B buffers (64 x 256
//     f16, 32 KB).  One workgroup barrier per k step, in front of the last
//     slice: behind it the A buffer just consumed takes the copies of k step
//     +2 (issued over the next 8 chunks, at least 8 chunks before they are
//     needed) and the B buffer consumed one step earlier takes k step +3's
//     (issued over the following 8 chunks, more than a k step ahead).
//   * Copies are global_load_lds_dwordx4, XOR-swizzled by the choice of the
//     chunk each lane fetches; A fragments ds_read_b128, B fragments
//     ds_read_b64_tr_b16.
//   * The MFMA is issued with the B fragment as first operand, i.e. it forms
//     the transposed 32 x 32 block: a lane then owns 4 CONSECUTIVE columns of
//     one row of C per register group, so C is loaded and stored 16 bytes per
//     lane (f32) instead of 4.
//
// Requirements as for the other tuned kernels: A, B 16-byte aligned; lda, ldb,
// K, N multiples of 8.  Rows >= M / columns >= N are fetched from clamped
// addresses and never stored; the k tail is zero-filled through registers.
#include "gemm_device.h"
#include "../../include/gemm_f16.h"

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
    // B stage = 32 copies of 2 k rows x 512 B; lane i writes (k row 2q + i/32,
    // chunk position i%32), which must hold the chunk whose 64-byte granule
    // index is XORed with (k row)%4.
    uint32_t b_off[NCOPY];
    const int b_krow0 = 2 * wave + (lane >> 5);                       // k row of copy t: b_krow0 + 8t
    {
        const int sw = 2 * (wave & 1) + (lane >> 5);                  // (2q + i/32) % 4
        int col = 8 * ((lane & 31) ^ (sw << 2));
        if (n0 + col + 8 > p.N) col = 0;                              // clamp: loaded, never stored
#pragma unroll
        for (int t = 0; t < NCOPY; t++)
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
    if (KT > 1) {                  // A(1): the first half only, k step 0 issues the second
#pragma unroll
        for (int t = 0; t < NCOPY; t++) { if (t < 4) copy_a(1, t); copy_b(1, t); }
    }

    // ---- accumulators -------------------------------------------------------
    // They start at zero; the C tile is read once, during the LAST k step (its
    // chunks have no copies left to issue), into otherwise idle registers, and
    // added when the products are complete: C + sum = sum + C.
    floatx16 acc[4][4];
#pragma unroll
    for (int fm = 0; fm < 4; fm++)
#pragma unroll
        for (int fn = 0; fn < 4; fn++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[fm][fn][i] = 0.0f;
    CT* const Cbase = (CT*)p.C;
    typedef typename CVec4<CT>::type ctx4;
    // Transposed 32 x 32 blocks (B fragment first): register i of lane l is row
    // l%32, column 8*(i/4) + 4*(l/32) + i%4 -- group g = i/4 is 4 consecutive
    // columns of one row of C: one vector access per (fm, fn, g).
    const int c_lrow = lane & 31, c_lcol = 4 * (lane >> 5);
    const uint32_t c_voff = ((uint32_t)c_lrow * (uint32_t)p.ldc + (uint32_t)c_lcol) * (uint32_t)sizeof(CT);
    const int c_row0 = m0 + wm_base, c_col0 = n0 + wn_base;
    // group (fm, fn, g) lies inside C?  (N is a multiple of 8: all or nothing)
    auto c_ok = [&](int fm, int fn, int g) -> bool {
        return !edge || ((c_row0 + fm * 32 + c_lrow < p.M) && (c_col0 + fn * 32 + 8 * g + c_lcol < p.N));
    };
    // a group outside C reads the wavefront tile's first group instead (valid)
    auto c_load = [&](int fm, int fn, int g) -> ctx4 {
        const char* base = reinterpret_cast<const char*>(Cbase + (int64_t)c_row0 * p.ldc + c_col0);
        const bool ok = c_ok(fm, fn, g);
        const char* rowp = base + (ok ? (int64_t)fm * 32 * p.ldc * (int64_t)sizeof(CT) : 0);
        const uint32_t off = ok ? c_voff + (uint32_t)((fn * 32 + 8 * g) * sizeof(CT)) : 0u;
        return *reinterpret_cast<const ctx4*>(rowp + off);
    };
    ctx4 c_lo[2][4][4];            // C of accumulator rows 0, 1: fetched during the last k step

    // ---- fragment read addresses ----------------------------------------------
    // A operand: lane l holds tile row (l%32) of its 32-row block, k = 8*(l/32)..+7
    // of slice ks -> logical chunk 2*ks + l/32, stored at chunk ^ ((row/2)%8).
    uint32_t a_rd[4];
    {
        const uint32_t row_off = (uint32_t)(wm_base + (lane & 31)) * (BK * 2);
        const int sw = (lane >> 1) & 7;
#pragma unroll
        for (int ks = 0; ks < 4; ks++)
            a_rd[ks] = smem_base + row_off + (uint32_t)(((2 * ks + (lane >> 5)) ^ sw) * 16);
    }
    // B operand: one transposing read serves 16 lanes -- lanes 4r..4r+3 of a
    // 16-lane block point at 16 consecutive columns of k row r and lane i gets
    // column i of rows 0..3.  Blocks 0,1: the two column halves at k 0..7,
    // blocks 2,3: at k 8..15; two reads (k +0..3, +4..7) make one operand.
    uint32_t b_rd[4];
    {
        const int blk = lane >> 4, j = lane & 15;
        const uint32_t lane_off = (uint32_t)(8 * (blk >> 1) + (j >> 2)) * B_ROW + (uint32_t)(16 * (blk & 1) + 4 * (j & 3)) * 2;
#pragma unroll
        for (int fn = 0; fn < 4; fn++)
            b_rd[fn] = smem_base + B_REGION + lane_off + (uint32_t)((((wn_base >> 5) + fn) ^ (j >> 2)) * 64);
    }

    half8 fa[2][4], fb[2][4];      // fragments of two k slices: [slice & 1][fm], [slice & 1][fn]
    half4 b_lo[4];                 // first half of a B operand until its second read is issued

    // read r (0..11) of slice ks of (A buffer at a_base, B buffer at b_base)
    // into fragment set d: B operands first, then A
    auto issue_read = [&](uint32_t a_base, uint32_t b_base, int ks, int d, int r) {
        if (r < 8) {
            const int fn = r >> 1;
            const uint32_t addr = b_rd[fn] + b_base + ks * 16 * B_ROW;
            if ((r & 1) == 0) b_lo[fn] = lds_read_tr16(addr);
            else fb[d][fn] = __builtin_shufflevector(b_lo[fn], lds_read_tr16(addr + 4 * B_ROW), 0, 1, 2, 3, 4, 5, 6, 7);
        } else {
            const int fm = r - 8;
            fa[d][fm] = lds_read_b128(a_rd[ks] + a_base + fm * 32 * (BK * 2));
        }
    };
    // one MFMA; B fragment first = transposed block
    auto mfma_one = [&](int d, int fm, int fn) {
        acc[fm][fn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[d][fn], fa[d][fm], acc[fm][fn], 0, 0, 0);
    };
    // The wavefront is alone on its SIMD and issues in order: an instruction
    // behind an MFMA that waits for the matrix pipe waits with it.  So every
    // MFMA is followed by exactly one other instruction (an LDS read, a copy, a
    // C load), which issues in the 32-cycle shadow of that MFMA; the scheduler
    // is told to keep this order.
    auto fence = [&]() { __builtin_amdgcn_sched_barrier(0); };

    // prologue copies have landed; publish, then fetch slice 0
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int r = 0; r < 12; r++) issue_read(0, 0, 0, 0, r);

    // ---- main loop -------------------------------------------------------------
    // Chunk q of k step j: MFMA row q%4 of slice q/4; reads 3(q%4)..+2 of the
    // next slice; one copy: q 0-3: A(j+1) copies 4-7, q 4-11: B(j+2) copies
    // 0-7, q 12-15 (behind the barrier): A(j+2) copies 0-3.  The last k step
    // (LAST) has nothing to copy or prefetch and fetches half of the C tile
    // instead, 2 vector loads per chunk.
    auto k_step = [&](int j, auto last_tag) {
        constexpr bool LAST = decltype(last_tag)::value;
        const uint32_t a_cur = (uint32_t)(j & 1) * A_BUF, a_nxt = a_cur ^ A_BUF;
        const uint32_t b_cur = (uint32_t)(j % 3) * B_BUF, b_nxt = (uint32_t)((j + 1) % 3) * B_BUF;
#pragma unroll
        for (int q = 0; q < 12; q++) {
            const int ks = q >> 2, c = q & 3;
#pragma unroll
            for (int i = 0; i < 3; i++) {
                mfma_one(ks & 1, c, i); fence();
                issue_read(a_cur, b_cur, ks + 1, (ks + 1) & 1, 3 * c + i); fence();
            }
            mfma_one(ks & 1, c, 3); fence();
            if (LAST) {
#pragma unroll
                for (int u = 2 * q; u < 2 * q + 2; u++) c_lo[u >> 4][(u >> 2) & 3][u & 3] = c_load(u >> 4, (u >> 2) & 3, u & 3);
            } else {
                if (q < 4) copy_a(j + 1, 4 + q);
                else if (j + 2 < KT) copy_b(j + 2, q - 4);
            }
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
        for (int c = 0; c < 4; c++) {
#pragma unroll
            for (int i = 0; i < 3; i++) {
                mfma_one(1, c, i); fence();
                if (!LAST) { issue_read(a_nxt, b_nxt, 0, 0, 3 * c + i); fence(); }
            }
            mfma_one(1, c, 3); fence();
            if (LAST) {
#pragma unroll
                for (int u = 24 + 2 * c; u < 24 + 2 * c + 2; u++) c_lo[u >> 4][(u >> 2) & 3][u & 3] = c_load(u >> 4, (u >> 2) & 3, u & 3);
            } else {
                if (j + 2 < KT) copy_a(j + 2, c);
            }
            fence();
        }
    };
    for (int j = 0; j + 1 < KT; j++) k_step(j, BoolTag<false>());
    k_step(KT - 1, BoolTag<true>());

    // ---- + C, -> C ---------------------------------------------------------------
    // Rows 2 and 3 of C are fetched while rows 0 and 1 are added and stored (one
    // row of 64 registers at a time, in the registers the previous row frees).
    {
        auto finish_row = [&](int fm, const ctx4 (&cin)[4][4]) {
            char* rowp = reinterpret_cast<char*>(Cbase + (int64_t)(c_row0 + fm * 32) * p.ldc + c_col0);
#pragma unroll
            for (int fn = 0; fn < 4; fn++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    ctx4 v;
#pragma unroll
                    for (int e = 0; e < 4; e++) v[e] = (CT)(acc[fm][fn][4 * g + e] + (float)cin[fn][g][e]);   // f16: one rounding, to nearest even
                    if (c_ok(fm, fn, g))
                        *reinterpret_cast<ctx4*>(rowp + c_voff + (fn * 32 + 8 * g) * sizeof(CT)) = v;
                }
        };
        ctx4 c_r2[4][4], c_r3[4][4];
#pragma unroll
        for (int u = 0; u < 16; u++) c_r2[u >> 2][u & 3] = c_load(2, u >> 2, u & 3);
        __builtin_amdgcn_sched_barrier(0);
        finish_row(0, c_lo[0]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 16; u++) c_r3[u >> 2][u & 3] = c_load(3, u >> 2, u & 3);
        __builtin_amdgcn_sched_barrier(0);
        finish_row(1, c_lo[1]);
        __builtin_amdgcn_sched_barrier(0);
        finish_row(2, c_r2);
        __builtin_amdgcn_sched_barrier(0);
        finish_row(3, c_r3);
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
    TiledParams p;
    p.M = (int)a.M; p.N = (int)a.N; p.K = (int)a.K;
    p.A = a.A; p.lda = a.lda; p.B = a.B; p.ldb = a.ldb; p.C = a.C; p.ldc = a.ldc;
    p.tiles_m = (int)((a.M + WBM - 1) / WBM);
    p.tiles_n = (int)((a.N + WBN - 1) / WBN);
    p.group_m = 8 < p.tiles_m ? 8 : p.tiles_m;     // an XCD's 32 concurrent tiles form an 8 x 4 block of C
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
