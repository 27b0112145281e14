// The kernel for problems whose time goes into reading and writing C (short k
// loops): 256 x 128 C tile per workgroup, 8 wavefronts in two phase-alternating
// groups as in gemm_pingpong.hip, one workgroup per compute unit walking its
// tiles -- and TWO sets of accumulators per wavefront (2 x 64 registers: a
// wavefront's part of the tile is 128 x 32).  While a tile is multiplied into one
// set, the other set, which holds the finished sums of the tile before it, is
// added to C and stored a 32-row slab at a time in the phases in which the
// wavefront only reads fragments.  C traffic (HBM) and MFMA work thus run at the
// same time on every compute unit, instead of all units reading and writing C
// together and then all multiplying together with HBM idle.
//
// The steps are those of the paper's recipe (Algorithm "Two-level tiled tensor
// core Matmul", C hoisted out of the k loop as in section "Generating WMMA Ops and
// More", loads for later k tiles in flight as in section "Completing Latency
// Hiding"); what is added is that the k loops of consecutive tiles form ONE
// software pipeline: the copies issued in k step k are those of k step k + 2 of
// the same tile or, in a tile's last two k steps, of the first two k steps of the
// workgroup's next tile, so the pipeline never drains between tiles.  (After a
// workgroup's last tile those two copies fetch its first two k steps again: valid
// addresses, never read.)
//
// LDS: 2 A buffers (256 x 64 f16 = 32 KB) + 3 B buffers (64 x 128 f16 = 16 KB) =
// 112 KB, XOR-swizzled as in gemm_pingpong.hip, + 36 KB in which each wavefront
// turns a 32 x 32 slab of results from the MFMA's layout (a lane owns 4 consecutive
// columns of one row of a 16 x 16 block) into whole 128-byte rows for the stores.
// C is read in the MFMA's layout directly (64-byte pieces: fine for loads).
//
// The C loads are inline assembly like the global -> LDS copies.  Written as
// ordinary loads the compiler would place a wait in front of their first use that
// allows only the loads it knows of to be outstanding -- it does not count the
// copies, so that wait would also cover copies issued a phase earlier and stall
// every reading phase for a memory latency (measured: 167 us instead of 130 on the
// (16384, 3072, 768) problem).  The pipeline's own waits count what is certain:
// when k step k ends, the loads younger than the copies of k step k - 1 are this k
// step's 6 copies plus the 4 C loads of a slab where one was requested; loads
// complete in order, so with at most that many operations outstanding those copies
// have landed (outstanding stores only make the wait longer) -- and with them every
// C load requested before them.  A slab is therefore complete, without a wait of
// its own, once copies issued behind it have been awaited, and it is used in the k
// step after that; the use goes through an empty asm statement so that the
// compiler cannot move it ahead of that point.  Slabs 0 and 1 of the previous tile
// are requested at the end of k steps 0 and 1 and added in k steps 3 and 4, slabs
// 2 and 3 are requested in k steps 3 and 4 (into the registers just freed) and
// added in k steps 5 and 6.  For the count to be exact every C load is issued
// unconditionally, from a clamped address where the element lies outside C.
//
// Requirements: as for the other tuned kernels, and K a multiple of 64 with at
// least 9 k steps (other problems are passed on to the 256 x 256 kernel).
#include "../gemm_device.h"
#include "../../../include/gemm_f16.h"

namespace {

using namespace gemm_dev;

constexpr int OBM = 256, OBN = 128;
constexpr int OHM = OBM / 2, OWN = OBN / 4;                 // a wavefront's rows (group) and columns
constexpr int OA_BUF = OBM * BK * 2, OB_BUF = BK * OBN * 2, OB_ROW = OBN * 2;
constexpr int ONA = 2, ONB = 3;                             // LDS buffers: copies run two k steps ahead
constexpr int OB_REGION = ONA * OA_BUF;
constexpr int O_STAGE = ONA * OA_BUF + ONB * OB_BUF;        // behind the 112 KB of A and B buffers:
constexpr int O_PITCH = OWN * 4 + 16;                       // a 32 x 32 f32 slab per wavefront, rows 144 B apart
constexpr int O_LDS = O_STAGE + 8 * 32 * O_PITCH;           // 148 KB
constexpr int OTA = OHM / 32, OTB = OBN / 64;               // copies per wavefront, k step and operand: 4 + 2
constexpr int OFM = OHM / 16, OFN = OWN / 16;               // 8 x 2 accumulator blocks of 16 x 16
constexpr int OSLABS = OHM / 32;                            // C moves in 4 slabs of 32 rows x 32 columns per wavefront
constexpr int MIN_KT = 9;

__device__ __forceinline__ void ov_barrier()
{
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

template <int V> struct ITag { static constexpr int value = V; };

template <typename CT>
__global__ __launch_bounds__(512) void gemm_pp_overlap_kernel(const TiledParams p)
{
    __shared__ __attribute__((aligned(1024))) char smem[O_LDS];
    const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_ptr_t)smem;
    typedef typename CVec4<CT>::type ctx4;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2;                 // 0: X (top 128 rows), 1: Y (bottom 128 rows)
    const int wn = wave & 3;                   // column block of 32; also the copy slot within the group
    const int KT = p.K / BK;
    const int tiles = p.tiles_m * p.tiles_n;

    // ---- the tile being copied (runs two k steps ahead of the tile being multiplied) ----
    int next_tile = blockIdx.x;                // next tile index to hand to the copy side
    int cp_m0 = 0, cp_n0 = 0;
    const half_t* a_tile = p.A;
    const half_t* b_tile = p.B;
    uint32_t a_off[OTA], b_off[OTB];
    // Lane offsets of the copies, as in gemm_pingpong.hip: A copy q = wn + 4t covers tile
    // rows 8q .. 8q+7 of the group's half; B copy q covers k rows 4q .. 4q+3 of the k half.
    auto copy_side_to = [&](int tile) {
        int tm, tn;
        tile_of_block(p, tile, tm, tn);
        cp_m0 = tm * OBM; cp_n0 = tn * OBN;
        a_tile = p.A + (int64_t)cp_m0 * p.lda;
        b_tile = p.B + cp_n0;
        int ln = lane;
        asm volatile("" : "+v"(ln));           // recomputed per tile, not kept in registers across tiles
        const int a_chunk = (ln & 7) ^ (4 * (wn & 1) + (ln >> 4));
#pragma unroll
        for (int t = 0; t < OTA; t++) {
            int row = grp * OHM + 8 * (wn + 4 * t) + (ln >> 3);
            row = (cp_m0 + row < p.M) ? row : p.M - 1 - cp_m0;          // clamp: loaded, never stored
            a_off[t] = ((uint32_t)row * (uint32_t)p.lda + 8 * a_chunk) * 2;
        }
#pragma unroll
        for (int t = 0; t < OTB; t++) {
            const int krow = 4 * (wn + 4 * t) + ln / 16;
            const int swz = ((krow & 3) << 2) | (((krow >> 3) & 1) << 1);
            int col = 8 * ((ln % 16) ^ swz);
            if (cp_n0 + col + 8 > p.N) col = 0;                         // clamp: loaded, never stored
            b_off[t] = ((uint32_t)krow * (uint32_t)p.ldb + col) * 2;
        }
    };
    // copies of k slice ck of the tile on the copy side into A buffer abuf (0/1) and B buffer bbuf (0..2)
    auto copy_a_part = [&](int ck, int abuf, int t) {
        async_copy16(a_tile + (int64_t)ck * BK, a_off[t], smem_base + abuf * OA_BUF + grp * (OA_BUF / 2) + 1024 * (wn + 4 * t));
    };
    auto copy_b_part = [&](int ck, int bbuf, int t) {
        async_copy16(b_tile + ((int64_t)ck * BK + grp * 32) * p.ldb, b_off[t],
                     smem_base + OB_REGION + bbuf * OB_BUF + grp * (OB_BUF / 2) + 1024 * (wn + 4 * t));
    };

    // ---- fragment read addresses (16x16x32 MFMA operands; see gemm_pingpong.hip) ----
    uint32_t a_rd[2], b_rd[OFN];
    {
        const int lr = lane & 15, lk = lane >> 4;
        const uint32_t row_off = (uint32_t)(grp * OHM + lr) * (BK * 2);
        const int sw = (lr >> 1) & 7;
#pragma unroll
        for (int sl = 0; sl < 2; sl++) a_rd[sl] = smem_base + row_off + (uint32_t)(((4 * sl + lk) ^ sw) * 16);
        const int blk = lane >> 4, j = lane & 15;
        const int krow = 8 * blk + (j >> 2);
        const int swz = ((krow & 3) << 2) | (((krow >> 3) & 1) << 1);
#pragma unroll
        for (int fn = 0; fn < OFN; fn++) {
            const int col = wn * OWN + fn * 16 + 4 * (j & 3);
            b_rd[fn] = smem_base + OB_REGION + (uint32_t)krow * OB_ROW + (uint32_t)(((col >> 3) ^ swz) * 16 + 2 * (col & 7));
        }
    }
    half8 fa[OFM], fb[OFN];
    auto read_fragments = [&](int abuf, int bbuf, int h) {
        uint32_t a0 = a_rd[h] + (uint32_t)abuf * OA_BUF;
        asm volatile("" : "+v"(a0));
#pragma unroll
        for (int fm = 0; fm < OFM; fm++) fa[fm] = lds_read_b128(a0 + fm * 16 * (BK * 2));
#pragma unroll
        for (int fn = 0; fn < OFN; fn++) {
            uint32_t b0 = b_rd[fn] + (uint32_t)bbuf * OB_BUF;
            asm volatile("" : "+v"(b0));
            const half4 lo = lds_read_tr16(b0 + h * 32 * OB_ROW);
            const half4 hi = lds_read_tr16(b0 + h * 32 * OB_ROW + 4 * OB_ROW);
            fb[fn] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };

    // ---- C side: the tile whose sums wait in the other accumulator set ---------------
    // Block (fm, fn) of a wavefront's part: rows crow0 + 16 fm + l%16, columns ccol0 +
    // 16 fn + 4 (l/16) .. +3 (the MFMA is issued with the B fragment first).
    CT* const Cbase = (CT*)p.C;
    struct CTile { int crow0, ccol0; bool edge; };
    CTile prev = {0, 0, false};
    typedef uint32_t craw_t __attribute__((ext_vector_type(sizeof(CT) == 4 ? 4 : 2)));   // 4 elements of C as loaded
    craw_t cin[2][4];                          // two slabs of C on their way / waiting to be added
    float bias4[OFN][4];
    auto c_ptr = [&](const CTile& t, int fm, int fn, int ln, bool& ok) -> CT* {
        const int row = t.crow0 + 16 * fm + (ln & 15), col = t.ccol0 + 16 * fn + 4 * (ln >> 4);
        ok = !t.edge || (row < p.M && col < p.N);                      // N is a multiple of 8: all 4 columns or none
        return Cbase + (ok ? (int64_t)row * p.ldc + col : (int64_t)0);
    };
    auto request_slab = [&](const CTile& t, int s) {                   // 4 loads, always issued
        int ln = lane;
        asm volatile("" : "+v"(ln));
#pragma unroll
        for (int r = 0; r < 2; r++)
#pragma unroll
            for (int fn = 0; fn < OFN; fn++) {
                bool ok;
                const CT* src = c_ptr(t, 2 * s + r, fn, ln, ok);
                if constexpr (sizeof(CT) == 4) asm volatile("global_load_dwordx4 %0, %1, off ; C slab load" : "=v"(cin[s & 1][2 * r + fn]) : "v"(src) : "memory");
                else                           asm volatile("global_load_dwordx2 %0, %1, off ; C slab load" : "=v"(cin[s & 1][2 * r + fn]) : "v"(src) : "memory");
            }
    };
    // The bias of the tile's columns, through the same kind of load and an immediate
    // wait (only when there is a bias: one short stall per tile).  An ordinary load
    // here would make the compiler wait for every outstanding operation in front of
    // each use of the bias, also when there is none.
    auto load_bias = [&](const CTile& t) {
#pragma unroll
        for (int fn = 0; fn < OFN; fn++)
#pragma unroll
            for (int e = 0; e < 4; e++) bias4[fn][e] = 0.0f;
        if (p.bias) {
            int ln = lane;
            asm volatile("" : "+v"(ln));
            const int col = t.ccol0 + 4 * (ln >> 4);
            craw_t raw[OFN];
#pragma unroll
            for (int fn = 0; fn < OFN; fn++) {
                const int c = col + 16 * fn;
                const CT* src = reinterpret_cast<const CT*>(p.bias) + (c < p.N ? c : 0);
                if constexpr (sizeof(CT) == 4) asm volatile("global_load_dwordx4 %0, %1, off ; bias load" : "=v"(raw[fn]) : "v"(src) : "memory");
                else                           asm volatile("global_load_dwordx2 %0, %1, off ; bias load" : "=v"(raw[fn]) : "v"(src) : "memory");
            }
            static_assert(OFN == 2, "operands of the wait below");
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(raw[0]), "+v"(raw[1]) :: "memory");
#pragma unroll
            for (int fn = 0; fn < OFN; fn++)
                if (col + 16 * fn < p.N) {
                    const ctx4 b4 = __builtin_bit_cast(ctx4, raw[fn]);
#pragma unroll
                    for (int e = 0; e < 4; e++) bias4[fn][e] = (float)b4[e];
                }
        }
    };
    // + C (+ bias, ReLU) in the layout the MFMA leaves (row l%16 of a block, 4 columns at
    // 4 (l/16)), then through this wavefront's 4.5 KB of LDS so that 8 lanes cover one
    // 128-byte row of the slab: stored as it sits in registers, a row would go out as two
    // 64-byte halves from two instructions, which the memory system takes far worse
    // (measured: the stores alone then cost 55 us on the (16384, 3072, 768) problem).
    auto finish_slab = [&](const CTile& t, int s, const floatx4 (&acc)[OFM][OFN]) {
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const uint32_t tbuf = smem_base + O_STAGE + (uint32_t)wave * (32u * O_PITCH);
        const uint32_t w_addr = tbuf + (uint32_t)(ln & 15) * O_PITCH + (uint32_t)(ln >> 4) * 16;
        const uint32_t r_addr = tbuf + (uint32_t)(ln >> 3) * O_PITCH + (uint32_t)(ln & 7) * 16;
        // the slab has arrived (see the file header); nothing may use it before this point
        asm volatile("; C slab arrived %0 %1 %2 %3" : "+v"(cin[s & 1][0]), "+v"(cin[s & 1][1]), "+v"(cin[s & 1][2]), "+v"(cin[s & 1][3]));
#pragma unroll
        for (int r = 0; r < 2; r++)
#pragma unroll
            for (int fn = 0; fn < OFN; fn++) {
                const ctx4 c4 = __builtin_bit_cast(ctx4, cin[s & 1][2 * r + fn]);
                floatx4 v;
#pragma unroll
                for (int e = 0; e < 4; e++) v[e] = epilogue_value(acc[2 * s + r][fn][e] + (float)c4[e], bias4[fn][e], p.relu);
                *(__attribute__((address_space(3))) floatx4*)(uintptr_t)(w_addr + r * 16 * O_PITCH + fn * 16 * 4) = v;
            }
        // back: lane l takes row l/8 (+ 8 per pass), columns 4 (l%8) .. +3
        const int orow = t.crow0 + 32 * s + (ln >> 3), ocol = t.ccol0 + 4 * (ln & 7);
        const bool col_ok = !t.edge || ocol < p.N;                     // N is a multiple of 8: all 4 columns or none
        CT* const dst0 = Cbase + (int64_t)orow * p.ldc + ocol;
#pragma unroll
        for (int ps = 0; ps < 4; ps++) {
            const floatx4 v = *(__attribute__((address_space(3))) const floatx4*)(uintptr_t)(r_addr + 8 * ps * O_PITCH);
            ctx4 o;
#pragma unroll
            for (int e = 0; e < 4; e++) o[e] = (CT)v[e];               // f16: the one rounding, to nearest even
            if (col_ok && (!t.edge || orow + 8 * ps < p.M)) *reinterpret_cast<ctx4*>(dst0 + (int64_t)(8 * ps) * p.ldc) = o;
        }
    };

    // ---- one k step; HOOK = position in the tile's first seven k steps (0..6), 7 = none ----
    // X: read, barrier, multiply, barrier, twice; Y the same one phase later.  The
    // multiplying wavefront issues its copies between its MFMAs: its k half of B in the
    // first half step, its own A rows in the second.
    int g_abuf = 0, g_bbuf = 0;                // buffers of the k step being multiplied
    auto k_step = [&](floatx4 (&acc)[OFM][OFN], const floatx4 (&old)[OFM][OFN], bool have_old, int ck, auto hook) {
        constexpr int J = decltype(hook)::value;
        const int cbbuf = g_bbuf == 0 ? ONB - 1 : g_bbuf - 1;          // (g_bbuf + 2) % 3: B buffer of the k step copied now
#pragma unroll
        for (int h = 0; h < 2; h++) {
            read_fragments(g_abuf, g_bbuf, h);
            if (h == 0) {
                if constexpr (J >= 3 && J <= 6) {
                    if (have_old) {
                        finish_slab(prev, J - 3, old);
                        if constexpr (J <= 4) request_slab(prev, J - 1);      // into the registers just freed
                    }
                }
                if constexpr (J == 0) {
                    if (have_old) load_bias(prev);
#pragma unroll
                    for (int fm = 0; fm < OFM; fm++)
#pragma unroll
                        for (int fn = 0; fn < OFN; fn++)
#pragma unroll
                            for (int e = 0; e < 4; e++) acc[fm][fn][e] = 0.0f;
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            ov_barrier();
#pragma unroll
            for (int fm = 0; fm < OFM; fm++)
#pragma unroll
                for (int fn = 0; fn < OFN; fn++) {
                    acc[fm][fn] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fb[fn], fa[fm], acc[fm][fn], 0, 0, 0);
                    const int idx = fm * OFN + fn;
                    if (idx % 4 == 1) {
                        __builtin_amdgcn_sched_barrier(0);
                        if (h == 0) { if (idx / 4 < OTB) copy_b_part(ck, cbbuf, idx / 4); }
                        else        { if (idx / 4 < OTA) copy_a_part(ck, g_abuf, idx / 4); }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            if (h == 1) {
                __builtin_amdgcn_sched_barrier(0);
                // Slabs 0 and 1 are requested here, behind this k step's copies: a load
                // from HBM returns later than the copies (mostly L2 hits) issued after it
                // would, and loads return in order, so a C load has to be complete only
                // when the copies issued BEHIND it are awaited -- two k steps from now.
                if constexpr (J <= 1) { if (have_old) request_slab(prev, J); }
                // The copies of the k step before this one have landed when at most the
                // loads issued after them are outstanding (see the file header): this k
                // step's 6 copies, plus the slab requested in this k step (J = 0, 3, 4: 4
                // loads), in the k step before and in this one (J = 1: 8), or at the end of
                // the k step before (J = 2: 4).
                constexpr int later_loads = OTA + OTB + ((J == 1) ? 8 : (J <= 4) ? 4 : 0);
                if (have_old) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(later_loads) : "memory");
                else          asm volatile("s_waitcnt vmcnt(%0)" :: "n"(OTA + OTB) : "memory");
            }
            ov_barrier();
        }
        g_abuf = g_abuf == ONA - 1 ? 0 : g_abuf + 1;
        g_bbuf = g_bbuf == ONB - 1 ? 0 : g_bbuf + 1;
    };

    // One tile into `acc` while `old` (the tile before it, if any) goes to C.
    auto run_tile = [&](floatx4 (&acc)[OFM][OFN], const floatx4 (&old)[OFM][OFN], bool have_old) {
        k_step(acc, old, have_old, 2, ITag<0>{});
        k_step(acc, old, have_old, 3, ITag<1>{});
        k_step(acc, old, have_old, 4, ITag<2>{});
        k_step(acc, old, have_old, 5, ITag<3>{});
        k_step(acc, old, have_old, 6, ITag<4>{});
        k_step(acc, old, have_old, 7, ITag<5>{});
        k_step(acc, old, have_old, 8, ITag<6>{});
        int k = 7;
        for (; k + 2 < KT; k++) k_step(acc, old, have_old, k + 2, ITag<7>{});
        // the last two k steps fetch the first two of the next tile (or of this one again)
        if (next_tile < tiles) { copy_side_to(next_tile); next_tile += gridDim.x; }
        k_step(acc, old, have_old, 0, ITag<7>{});
        k_step(acc, old, have_old, 1, ITag<7>{});
    };

    // ---- prologue: the first tile's k steps 0 and 1 ------------------------------------
    int mul_tile = blockIdx.x;                 // the tile being multiplied
    copy_side_to(next_tile);
    next_tile += gridDim.x;
#pragma unroll
    for (int s = 0; s < 2; s++) {
#pragma unroll
        for (int t = 0; t < OTA; t++) copy_a_part(s, s, t);
#pragma unroll
        for (int t = 0; t < OTB; t++) copy_b_part(s, s, t);
    }
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(OTA + OTB) : "memory");
    ov_barrier();
    if (grp == 1) ov_barrier();                // phase 0: X reads, Y has nothing to do yet

    floatx4 acc0[OFM][OFN], acc1[OFM][OFN];
    auto tile_done = [&]() {                   // the tile just multiplied becomes the one that goes to C
        int tm, tn;
        tile_of_block(p, mul_tile, tm, tn);
        prev.crow0 = tm * OBM + grp * OHM;
        prev.ccol0 = tn * OBN + wn * OWN;
        prev.edge = (tm * OBM + OBM > p.M) || (tn * OBN + OBN > p.N);
        mul_tile += gridDim.x;
    };
    // the last tile's sums: nothing is multiplied any more, so C is simply read, added and stored
    auto drain = [&](const floatx4 (&old)[OFM][OFN]) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the copies issued in the last two k steps land in this workgroup's LDS
        load_bias(prev);
        // two slabs in flight; the 4 loads of the younger slab (and stores) may be outstanding
        request_slab(prev, 0);
#pragma unroll
        for (int s = 0; s < OSLABS; s++) {
            if (s + 1 < OSLABS) {
                request_slab(prev, s + 1);
                asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
            } else {
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            finish_slab(prev, s, old);
        }
    };
    bool have_old = false;
    for (;;) {
        run_tile(acc0, acc1, have_old);
        tile_done();
        have_old = true;
        if (mul_tile >= tiles) { if (grp == 0) ov_barrier(); drain(acc0); break; }
        run_tile(acc1, acc0, true);
        tile_done();
        if (mul_tile >= tiles) { if (grp == 0) ov_barrier(); drain(acc1); break; }
    }
}

int64_t grid_overlap(int64_t M, int64_t N)
{
    const int64_t tm = (M + OBM - 1) / OBM, tn = (N + OBN - 1) / OBN;
    if (tm > 0 && tn > INT32_MAX / tm) return -1;
    const int64_t g = tm * tn;
    return g < chip().cus ? g : chip().cus;
}

int launch_overlap(const GemmArgs& a)
{
    const int64_t g = grid_overlap(a.M, a.N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    // k tails and very short k loops: the plain 256 x 256 launch (the selector never sends such problems here)
    if (a.K % BK != 0 || a.K / BK < MIN_KT) return pingpong16_config(256, 256)->launch(a);
    TiledParams p = make_tiled_params(a, OBM, OBN, 8);
    if (a.c_is_f16) hipLaunchKernelGGL((gemm_pp_overlap_kernel<half_t>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
    else            hipLaunchKernelGGL((gemm_pp_overlap_kernel<float>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}

const GemmConfigDesc kOverlap = {
    "ov256x128x64_w2x4_mi16", OBM, OBN, BK, 8, OHM, OWN, O_LDS, true, launch_overlap, grid_overlap};

}  // namespace

const GemmConfigDesc* overlap_config() { return &kOverlap; }
