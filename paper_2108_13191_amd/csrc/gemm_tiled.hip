// Tuned f16 GEMM kernels for gfx950: C = A B + C, row-major, f16 A and B,
// f32 accumulation on the matrix units (v_mfma_f32_32x32x16_f16).
//
// Structure (the two-level tiling of the paper's Algorithm "Two-level tiled
// tensor core Matmul", with the C tile hoisted out of the k loop as in section
// "Generating WMMA Ops and More" and the next k tile fetched while the current
// one is multiplied as in section "Completing Latency Hiding"):
//
//   * a workgroup owns a BM x BN tile of C, a wavefront a WM x WN part of it,
//     kept in registers for the whole k loop (FM x FN accumulators of 32x32);
//   * per k step of BK = 64 the A tile (BM x 64) and B tile (64 x BN) are
//     copied global -> LDS by global_load_lds_dwordx4 (16 bytes per lane,
//     written lane-linearly, no register staging), into one of a ring of LDS
//     buffers (two; four for the 64 x 64 tile); one barrier per k step;
//   * bank conflicts are avoided not by padding (the direct-to-LDS write is
//     lane-linear) but by choosing which 16-byte chunk each lane fetches, so
//     that the tile lands XOR-swizzled: A rows XOR their chunk index with
//     (row/2)%8, B rows XOR their 64-byte granule index with row%4;
//   * A fragments are read with ds_read_b128; B is N-contiguous, so its
//     K-contiguous fragments come from ds_read_b64_tr_b16 (a 4 x 16 transpose
//     across 16 lanes), two per fragment;
//   * workgroup ids are remapped so that each of the 8 XCDs (ids are dealt
//     round-robin to them) works on a compact block of C tiles.
//
// Requirements (checked by the caller in gemm_api.hip): A and B 16-byte
// aligned, lda, ldb, K and N multiples of 8.  M is arbitrary.  Rows beyond M
// and columns beyond N are fetched from clamped (valid) addresses and never
// stored; the k tail (K % 64) is zero-filled through registers.
#include "gemm_device.h"
#include "../../include/gemm_f16.h"

namespace {

using namespace gemm_dev;

// STAGES = LDS buffers (a power of two): the copies of k step kt + STAGES are
// issued in k step kt, so that many k steps of A and B are on their way at any
// time.  Two are enough when a k step's MFMAs outlast the memory latency (large
// tiles); a 64 x 64 tile multiplies a k step in about 60 ns and would otherwise
// spend its time waiting for every k step in turn.
// SWIZZLE = false (a ladder row, never selected) leaves the LDS image as the copies deliver it:
// the fragment reads then run into bank conflicts, which is what the XOR placement is there for
// (the paper pads its shared-memory rows instead: section "Padding to avoid bank conflicts" --
// a direct-to-LDS copy writes lane-linearly and cannot pad).
template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, typename CT, bool SWIZZLE = true>
__global__ __launch_bounds__(WAVES_M * WAVES_N * 64) void gemm_tiled_kernel(const TiledParams p)
{
    static_assert(STAGES >= 2 && (STAGES & (STAGES - 1)) == 0, "stage index is kt & (STAGES - 1)");
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int FM = WM / 32, FN = WN / 32;
    constexpr int A_STAGE = BM * BK * 2;            // bytes
    constexpr int B_STAGE = BK * BN * 2;
    constexpr int STAGE = A_STAGE + B_STAGE;
    constexpr int A_INSTR = A_STAGE / 1024;         // wave-wide 1 KiB copies per stage
    constexpr int B_INSTR = B_STAGE / 1024;
    constexpr int NTA = A_INSTR / NW, NTB = B_INSTR / NW;
    constexpr int B_ROW = BN * 2;                   // bytes per k row of the B tile
    constexpr int B_RPI = 1024 / B_ROW;             // k rows per wave-wide copy
    constexpr int B_LPR = 64 / B_RPI;               // lanes (16-byte chunks) per k row
    static_assert(NW % 2 == 0, "the swizzle of a lane's chunk must not depend on the copy index");
    static_assert(A_INSTR % NW == 0 && B_INSTR % NW == 0, "copies must divide among the waves");
    static_assert(WM % 32 == 0 && WN % 32 == 0 && BN >= 64 && BN <= 512, "tile shape");

    __shared__ __attribute__((aligned(1024))) char smem[STAGES * STAGE];
    const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_ptr_t)smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm_base = (wave / WAVES_N) * WM, wn_base = (wave % WAVES_N) * WN;

    int tile_m, tile_n;
    tile_of_block(p, blockIdx.x, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const bool edge = (m0 + BM > p.M) || (n0 + BN > p.N);

    // ---- global -> LDS copy plan (per lane, constant over k) -----------------
    // A: copy q covers tile rows 8q .. 8q+7 (128 bytes each); lane i writes LDS
    // chunk (row 8q + i/8, position i%8), which must hold logical chunk
    // position ^ ((row/2)%8).
    // Global addresses are a wave-uniform 64-bit base (tile origin, advanced by
    // one k step per iteration) plus a per-lane 32-bit byte offset that never
    // changes.
    const half_t* const a_tile = p.A + (int64_t)m0 * p.lda;
    const half_t* const b_tile = p.B + n0;
    uint32_t a_off[NTA];
    int a_chunk;                                  // logical 16-byte chunk (8 k) this lane fetches
    {
        const int sw = SWIZZLE ? 4 * (wave & 1) + (lane >> 4) : 0;  // (row/2)%8 for row = 8q + lane/8, q = wave mod 2
        a_chunk = (lane & 7) ^ sw;
#pragma unroll
        for (int t = 0; t < NTA; t++) {
            int row = 8 * (wave + NW * t) + (lane >> 3);
            row = (m0 + row < p.M) ? row : p.M - 1 - m0;            // clamp: loaded, never stored
            a_off[t] = ((uint32_t)row * (uint32_t)p.lda + 8 * a_chunk) * 2;
        }
    }
    // B: copy q covers k rows B_RPI*q .. ; lane i writes (row B_RPI*q + i/B_LPR,
    // chunk position i%B_LPR), which must hold the logical chunk whose 64-byte
    // granule index is XORed with row%4 (two granules per row: with (row/2)%2).
    uint32_t b_off[NTB];
    int b_krow[NTB];
    {
        const int pos = lane % B_LPR;
#pragma unroll
        for (int t = 0; t < NTB; t++) {
            const int krow = B_RPI * (wave + NW * t) + lane / B_LPR;
            const int sw = !SWIZZLE ? 0 : (B_ROW >= 256) ? (krow & 3) : ((krow >> 1) & 1);
            const int chunk = pos ^ (sw << 2);
            int col = 8 * chunk;
            col = (n0 + col + 8 <= p.N) ? col : 0;                  // clamp: loaded, never stored
            b_krow[t] = krow;
            b_off[t] = ((uint32_t)krow * (uint32_t)p.ldb + col) * 2;
        }
    }

    const int kt_full = p.K / BK;
    const int KT = (p.K + BK - 1) / BK;

    // copy number idx (0 .. NTA+NTB-1) of this wavefront for k step kt into LDS
    // stage `buf`; the k tail goes through registers and is zero beyond K
    constexpr int NC = NTA + NTB;
    auto issue_copy = [&](int kt, int buf, int idx) {
        const uint32_t a_dst = smem_base + buf * STAGE;
        const uint32_t b_dst = a_dst + A_STAGE;
        const int64_t k0 = (int64_t)kt * BK;
        const bool is_a = idx < NTA;
        const int t = is_a ? idx : idx - NTA;
        const char* src = is_a ? (const char*)(a_tile + k0) : (const char*)(b_tile + k0 * p.ldb);
        const uint32_t off = is_a ? a_off[is_a ? t : 0] : b_off[is_a ? 0 : t];
        const uint32_t dst = (is_a ? a_dst : b_dst) + 1024 * (wave + NW * t);
        if (kt < kt_full) {
            async_copy16(src, off, dst);
        } else {
            const int kvalid = p.K - (int)k0;                       // 8 .. 56, multiple of 8
            uintx4 v = {0u, 0u, 0u, 0u};
            const bool ok = is_a ? (8 * a_chunk < kvalid) : (b_krow[is_a ? 0 : t] < kvalid);
            if (ok) v = *reinterpret_cast<const uintx4*>(src + off);
            *(__attribute__((address_space(3))) uintx4*)(uintptr_t)(dst + 16 * lane) = v;
        }
    };

    // ---- prologue: the first STAGES k steps' copies, then the C tile ----------
#pragma unroll
    for (int s = 0; s < STAGES; s++)
        if (s < KT) {
#pragma unroll
            for (int i = 0; i < NC; i++) issue_copy(s, s, i);
        }

    // accumulator register i of lane l: row 8*(i/4) + 4*(l/32) + i%4, column l%32
    floatx16 acc[FM][FN];
    CT* const Cbase = (CT*)p.C;
    load_c_tile<CT, FM, FN>(acc, Cbase, p.ldc, m0 + wm_base, n0 + wn_base, lane, p.M, p.N, edge);

    // ---- fragment read addresses (per lane, constant over k) -----------------
    // A operand of the 32x32x16 MFMA: lane l holds row l%32, k = 8*(l/32) .. +7
    // of the 16-wide k slice -> logical chunk 2*ks + l/32 of tile row r,
    // stored at position chunk ^ ((r/2)%8).
    uint32_t a_rd[BK / 16];
    {
        const uint32_t row_off = (uint32_t)(wm_base + (lane & 31)) * (BK * 2);
        const int sw = SWIZZLE ? (lane >> 1) & 7 : 0;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ks++)
            a_rd[ks] = smem_base + row_off + (uint32_t)(((2 * ks + (lane >> 5)) ^ sw) * 16);
    }
    // B operand: lane l holds column l%32, the same k.  One transposing read
    // serves 16 lanes: lanes 4r..4r+3 of a 16-lane block point at 16
    // consecutive columns of k row r, and lane i receives column i of rows
    // 0..3.  Blocks 0,1 are the two column halves of k 0..7, blocks 2,3 of
    // k 8..15; two reads (k +0..3, +4..7) make one operand.
    uint32_t b_rd[FN];
    {
        const int blk = lane >> 4, j = lane & 15;
        const uint32_t lane_off = (uint32_t)(8 * (blk >> 1) + (j >> 2)) * B_ROW + (uint32_t)(16 * (blk & 1) + 4 * (j & 3)) * 2;
        const int sw = !SWIZZLE ? 0 : (B_ROW >= 256) ? (j >> 2) : ((j >> 3) & 1);   // swizzle term of this lane's k row
#pragma unroll
        for (int fn = 0; fn < FN; fn++)
            b_rd[fn] = smem_base + A_STAGE + lane_off + (uint32_t)((((wn_base >> 5) + fn) ^ sw) * 64);
    }

    // Fragments are double-buffered by 16-wide k slice: while the MFMAs of slice
    // ks run from fa/fb[ks&1], the reads of slice ks+1 fill fa/fb[(ks+1)&1].
    half8 fa[2][FM], fb[2][FN];
    constexpr int NR = FM + 2 * FN;                 // LDS reads per slice: A b128, B 2 x tr_b64
    half4 b_lo[FN];                                 // first half of a B operand until its second read is issued

    // read number r (0 .. NR-1) of slice ks of LDS stage `buf` into fragment set d:
    // B operands first (every MFMA row needs all of them), then A
    auto issue_read = [&](uint32_t stage_off, int ks, int d, int r) {
        if (r < 2 * FN) {
            const int fn = r >> 1;
            const uint32_t base = b_rd[fn] + stage_off + ks * 16 * B_ROW;
            if ((r & 1) == 0) b_lo[fn] = lds_read_tr16(base);
            else fb[d][fn] = __builtin_shufflevector(b_lo[fn], lds_read_tr16(base + 4 * B_ROW), 0, 1, 2, 3, 4, 5, 6, 7);
        } else {
            const int fm = r - 2 * FN;
            fa[d][fm] = lds_read_b128(a_rd[ks] + stage_off + fm * 32 * (BK * 2));
        }
    };

    // prologue copies and the C tile have landed; publish, then fetch slice 0
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
#pragma unroll
    for (int r = 0; r < NR; r++) issue_read(0, 0, 0, r);

    // ---- main loop -------------------------------------------------------------
    // One barrier per k step, placed in front of the last slice: behind it the
    // stage just consumed is free (copies for k step kt+STAGES go there) and the
    // next stage is complete (its slice 0 is fetched while the last slice is
    // multiplied).  Copies complete in order: with those of k steps kt+2 ..
    // kt+STAGES-1 allowed to be outstanding, k step kt+1 has landed; in the last
    // STAGES-1 k steps fewer are outstanding than that, so everything is awaited.  Every slice is cut into
    // FM chunks {a share of the next slice's LDS reads, a share of the copies,
    // one row of MFMAs}; the scheduler may reorder inside a chunk only, so LDS
    // and copy instructions are issued in the shadow of the MFMAs around them.
    for (int kt = 0; kt < KT; kt++) {
        const uint32_t cur = (uint32_t)(kt & (STAGES - 1)) * STAGE, nxt = (uint32_t)((kt + 1) & (STAGES - 1)) * STAGE;
#pragma unroll
        for (int ks = 0; ks < BK / 16 - 1; ks++) {
#pragma unroll
            for (int c = 0; c < FM; c++) {
#pragma unroll
                for (int r = c * NR / FM; r < (c + 1) * NR / FM; r++) issue_read(cur, ks + 1, (ks + 1) & 1, r);
#pragma unroll
                for (int fn = 0; fn < FN; fn++)
                    acc[c][fn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[ks & 1][c], fb[ks & 1][fn], acc[c][fn], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // this wave's copies of k step kt+1 have landed and its reads of this
        // stage are complete; after the barrier that holds for every wave
        if (STAGES > 2 && kt + STAGES <= kt_full) {      // (a k tail goes through registers, not through the counter's order)
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"((STAGES - 2) * NC) : "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        }
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        const bool more = kt + 1 < KT, copy = kt + STAGES < KT;
#pragma unroll
        for (int c = 0; c < FM; c++) {
            if (more) {
#pragma unroll
                for (int r = c * NR / FM; r < (c + 1) * NR / FM; r++) issue_read(nxt, 0, 0, r);
            }
            if (copy) {
#pragma unroll
                for (int i = c * NC / FM; i < (c + 1) * NC / FM; i++) issue_copy(kt + STAGES, kt & (STAGES - 1), i);
            }
#pragma unroll
            for (int fn = 0; fn < FN; fn++)
                acc[c][fn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[1][c], fb[1][fn], acc[c][fn], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- accumulators -> C -----------------------------------------------------
    {
        // Everything the addresses and bounds are made of is re-derived here
        // (opaque to common-subexpression elimination), so that no per-row
        // address or lane mask of the C load is kept alive across the k loop.
        int Mb = p.M, Nb = p.N, lane2 = lane, row2 = m0 + wm_base, col2 = n0 + wn_base;
        int64_t ldc2 = p.ldc;
        CT* C2 = Cbase;
        asm volatile("" : "+s"(Mb), "+s"(Nb), "+s"(row2), "+s"(col2), "+s"(ldc2), "+s"(C2), "+v"(lane2));
        store_c_tile<CT, FM, FN>(acc, C2, ldc2, row2, col2, lane2, Mb, Nb, edge, (const CT*)p.bias, p.relu);
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
int64_t grid_tiled(int64_t M, int64_t N)
{
    const int64_t tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
    if (tm > 0 && tn > INT32_MAX / tm) return -1;
    return tm * tn;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, bool SWIZZLE = true>
int launch_tiled(const GemmArgs& a)
{
    const int64_t g = grid_tiled<BM, BN, WAVES_M, WAVES_N>(a.M, a.N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    // 32 workgroups of an XCD that run together should form a near-square block of C
    const TiledParams p = make_tiled_params(a, BM, BN, (BM >= 256) ? 8 : 16);
    constexpr int threads = WAVES_M * WAVES_N * 64;
    if (a.c_is_f16)
        hipLaunchKernelGGL((gemm_tiled_kernel<BM, BN, WAVES_M, WAVES_N, STAGES, half_t, SWIZZLE>), dim3((unsigned)g), dim3(threads), 0, a.stream, p);
    else
        hipLaunchKernelGGL((gemm_tiled_kernel<BM, BN, WAVES_M, WAVES_N, STAGES, float, SWIZZLE>), dim3((unsigned)g), dim3(threads), 0, a.stream, p);
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}

#define TILED_CONFIG(NAME, BM, BN, WMS, WNS, ST, SWZ)                                               \
    { NAME, BM, BN, BK, (WMS) * (WNS), (BM) / (WMS), (BN) / (WNS), (ST) * ((BM) + (BN)) * BK * 2,   \
      true, launch_tiled<BM, BN, WMS, WNS, ST, SWZ>, grid_tiled<BM, BN, WMS, WNS> }

const GemmConfigDesc kTiled64 = TILED_CONFIG("t64x64x64_w2x2", 64, 64, 2, 2, 4, true);
#ifdef GEMM_F16_LADDER
const GemmConfigDesc kTiled128 = TILED_CONFIG("t128x128x64_w2x2", 128, 128, 2, 2, 2, true);
const GemmConfigDesc kTiled256 = TILED_CONFIG("t256x256x64_w2x4", 256, 256, 2, 4, 2, true);
const GemmConfigDesc kTiled256NoSwizzle = TILED_CONFIG("t256x256x64_w2x4_noswz", 256, 256, 2, 4, 2, false);
#endif

}  // namespace

// block = 64: the smallest problems.  Ladder builds: 128 and 256, the same kernel at the
// larger tiles (comparison rows; the phase-alternating kernel serves those sizes).
const GemmConfigDesc* tiled_config(int block)
{
#ifdef GEMM_F16_LADDER
    if (block == 128) return &kTiled128;
    if (block == 256) return &kTiled256;
#endif
    (void)block;
    return &kTiled64;
}
#ifdef GEMM_F16_LADDER
const GemmConfigDesc* tiled_no_swizzle_config() { return &kTiled256NoSwizzle; }
#endif
