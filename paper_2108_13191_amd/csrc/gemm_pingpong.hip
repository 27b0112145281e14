// The large-problem kernel: 256 x 256 C tile per workgroup (also built with 192
// and 128 rows), 8 wavefronts, k steps of 64, f16 MFMA with f32 accumulators
// (v_mfma_f32_16x16x32_f16 in the default configuration, v_mfma_f32_32x32x16_f16
// in the other; the text below counts in the latter's 32 x 32 blocks).
//
// The steps are those of the paper's recipe (Algorithm "Two-level tiled tensor
// core Matmul"; C hoisted out of the k loop, section "Generating WMMA Ops and
// More"; global loads for later k tiles in flight while the current one is
// multiplied, section "Completing Latency Hiding"), arranged for CDNA4:
//
//   * Wavefronts 0-3 ("X") own the top 128 rows of the tile, 4-7 ("Y") the
//     bottom 128; each owns a 128 x 64 block (4 x 2 accumulators of 32 x 32,
//     128 registers).  Wavefront w and w+4 share a SIMD.
//   * Time is cut into phases separated by one workgroup barrier.  In a phase
//     one group reads its A/B fragments of half a k step from LDS into
//     registers (48 VGPRs), while the other group issues its 16 MFMAs back to
//     back with every operand already in registers, and between them its 4
//     global -> LDS copies for two k steps ahead; then they swap.  The matrix
//     pipe of a SIMD therefore always has a wavefront that is not waiting on
//     LDS, and the copies (paced by the texture addresser, 16 cycles per 1 KB
//     wave-wide copy) are spread over the phase instead of queueing up in the
//     reading phase, which would then outlast the MFMAs.
//   * 160 KB of LDS hold 2 A buffers (256 x 64 f16 = 32 KB each) and 3 B
//     buffers (64 x 256 f16 = 32 KB each).  Each group brings in the A rows it
//     reads itself (X: A-top, Y: A-bottom) and one k half of B for everybody
//     (X: B-low = k rows 0-31, Y: B-high = k rows 32-63).
//   * Copies are global_load_lds_dwordx4 (no register staging); the LDS image
//     is XOR-swizzled by the choice of the chunk each lane fetches; A
//     fragments are ds_read_b128, B fragments ds_read_b64_tr_b16 (B is
//     N-contiguous, the MFMA wants K-contiguous lanes).
//
// Schedule (k = k step of 64, cut in halves h = 0,1 of two 16-wide k slices;
// phase numbers P):
//   X: P = 4k+2h    read the fragments of (k,h)
//      P = 4k+2h+1  16 MFMAs of (k,h); h=0: issue B-low(k+2), h=1: A-top(k+2)
//   Y: the same one phase later; h=0: issue B-high(k+2), h=1: A-bottom(k+2)
// A-top(k+2) overwrites A-top(k), which X finished reading in the phase
// before; B-low(k+2) overwrites B-low(k-1), last read by Y five phases earlier
// (hence the third B buffer).  At the end of the multiplying phase of (k,1) a
// wavefront waits until its copies for k step k+1 have landed (vmcnt(8): only
// the 8 issued during this k step may be outstanding) and the barrier that
// follows publishes them: a copy has four phases (A) or six (B) to cross L2 /
// Infinity Fabric.  The last two k steps issue no copies and run as a second
// loop (and, when K is not a multiple of 64, the k step that fetches the k
// tail as a third), so that the main loop carries no branch between its MFMAs.
//
// The accumulators start at zero; C is read once per tile in the epilogue,
// where the accumulators pass through LDS so that both the read and the write
// of C are whole row segments, 16 bytes per lane.  The first 32 rows (64 for
// f16 C) of each wavefront's part of C are requested before the last two k
// steps, which issue no copies, so that they arrive under those MFMAs.
//
// Launch forms (same tile body, pp_tile): one workgroup per tile (the hardware
// hands tiles to compute units as they free up); chained -- one workgroup per
// compute unit walks its tiles and requests a tile's first k step before the
// epilogue of the tile before it; staggered -- every other compute unit starts
// on half a tile (the 128-row form), so that the two halves of the chip read and
// write C at different times.
//
// Requirements as for the other tuned kernels: A, B 16-byte aligned; lda, ldb,
// K, N multiples of 8.  Rows >= M / columns >= N are fetched from clamped
// addresses and never stored; the k tail is zero-filled through registers.
#include "gemm_device.h"
#include "../../include/gemm_f16.h"

namespace {

using namespace gemm_dev;

constexpr int A_REGION = 0;                  // two A buffers, then three B buffers

__device__ __forceinline__ void phase_barrier()
{
    // nothing may be scheduled across a phase boundary
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// MI = 32: v_mfma_f32_32x32x16_f16 (4 x 2 accumulators of 32 x 32 per wavefront, two
// 16-wide k slices per phase); MI = 16: v_mfma_f32_16x16x32_f16 (8 x 4 accumulators
// of 16 x 16, one 32-wide k slice per phase).  Same LDS image, schedule and epilogue.
template <int MI> struct AccBlock;
template <> struct AccBlock<32> { typedef floatx16 type; };
template <> struct AccBlock<16> { typedef floatx4 type; };

template <bool V> struct BoolTag { static constexpr bool value = V; };
template <int V> struct IntTag { static constexpr int value = V; };

// TAIL = false is the instantiation for K % 64 == 0.  With TAIL the k step that
// fetches the k tail (through registers, zero-filled) is a loop of its own, so
// the main loop is the same in both.

// BM = rows of the workgroup tile: 256, or 192 / 128 for problems whose tile count
// fills the compute units better that way (the wavefront tile is then 96 x 64 /
// 64 x 64; everything else is unchanged).  BN = its columns: 256, or 128 (wavefront
// tile 32 columns wide) for the small-problem form 128 x 128.
// Where 16-byte chunk `chunk` of k row `krow` of a B stage sits within its row.  Rows
// of 256 or 512 bytes all start at bank 0, so the 4 k rows of a transposing read (and
// the 16-lane blocks that read k and k + 8 together) are spread by XORing the chunk
// index with 4 (k%4) + 2 ((k/8)%2).  Rows of 384 bytes (192 columns) start at bank 0
// and 32 in turn, which already separates k and k + 1; k and k + 2, and k and k + 8,
// are separated by XORing the chunk's low 3 bits with 2 ((k/2)%2) + 4 ((k/8)%2), so a
// chunk never leaves its 128-byte group (a 384-byte row has no 16 chunks to XOR over).
// Both values are even (the two chunks of a 16-column read stay adjacent) and the same
// for k rows 4, 16 and 32 apart (the reads of a fragment differ by instruction offsets).
template <int BN>
__device__ __forceinline__ int b_chunk_position(int chunk, int krow)
{
    if constexpr (BN == 192) return (chunk & ~7) | ((chunk & 7) ^ ((((krow >> 1) & 1) << 1) | (((krow >> 3) & 1) << 2)));
    else                     return chunk ^ (((krow & 3) << 2) | (((krow >> 3) & 1) << 1));
}

template <int BM, int BN>
constexpr int pp_lds_bytes() { return 2 * (BM * BK * 2) + 3 * (BK * BN * 2); }     // 160 KB for 256 x 256

// One BM x BN tile of C with its first row and column at (m0, n0), by the whole
// workgroup; smem_base = LDS address of pp_lds_bytes<BM, BN>() bytes, 1 KB aligned.
// PERSIST: afterwards the tiles next_tile, next_tile + tile_step, ... (indices as
// for tile_of_block) as long as they exist.  The copies of a tile's k step 0 are
// then issued before the epilogue of the tile before it, those of k step 1 right
// after it, so that a tile's first operands cross the memory system while C is
// read and written; the epilogue's transposing buffers lie in the LDS that k step
// 0 does not use.
template <typename CT, int MI, bool TAIL, int BM, int BN, bool PERSIST = false, bool ROWWISE = false>
__device__ __forceinline__ void pp_tile(const TiledParams& p, const uint32_t smem_base, int m0, int n0,
                                        int next_tile = 0, const int tile_step = 0)
{
    static_assert(!PERSIST || (BM == 256 && BN == 256), "the relocated epilogue buffers are laid out for 256 x 256");
    constexpr int HM = BM / 2;                       // rows per wavefront group
    constexpr int WN = BN / 4;                       // columns per wavefront
    constexpr int B_BUF = BK * BN * 2;               // 32 KB for BN = 256
    constexpr int B_ROW = BN * 2;                    // bytes per k row of a B stage
    constexpr int TB = BN / 64;                      // copies per wavefront and B half
    constexpr int A_BUF = BM * BK * 2;               // 32 KB for BM = 256
    constexpr int B_REGION = 2 * A_BUF;
    constexpr int TA = HM / 32;                      // copies per wavefront and A half

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2;                 // 0: X (top rows), 1: Y (bottom rows)
    const int wn = wave & 3;                   // column block of 64; also the copy slot within the group

    const int kt_full = p.K / BK;
    const int KT = (p.K + BK - 1) / BK;

    // ---- copy plan ----------------------------------------------------------
    // A half (128 rows x 128 B = 16 KB) = 16 wave-wide copies of 8 rows; the 4
    // wavefronts of a group take copies q = wn + 4t.  Lane i writes (row
    // 8q + i/8, chunk position i%8), which must hold logical chunk
    // position ^ ((row/2)%8) -- a per-lane constant because q = wn (mod 2).
    // (m0, n0, a_tile, b_tile and the lane offsets describe the tile being copied:
    // under PERSIST they move on to the next tile before the epilogue)
    const half_t* a_tile = p.A + (int64_t)m0 * p.lda;
    const half_t* b_tile = p.B + n0;
    const int a_chunk = (lane & 7) ^ (4 * (wn & 1) + (lane >> 4));
    auto a_offset = [&](int half, int t, int ln) -> uint32_t {
        const int a_chunk = (ln & 7) ^ (4 * (wn & 1) + (ln >> 4));
        int row = half * HM + 8 * (wn + 4 * t) + (ln >> 3);
        row = (m0 + row < p.M) ? row : p.M - 1 - m0;                 // clamp: loaded, never stored
        return ((uint32_t)row * (uint32_t)p.lda + 8 * a_chunk) * 2;
    };
    // B half (32 k rows x B_ROW bytes) = 4 * TB wave-wide copies of 1 KB; copy q = wn +
    // 4t.  Lane i writes chunk 64 q + i of the half, i.e. k row (64 q + i) / CPR, chunk
    // position (64 q + i) % CPR (a copy is 2 k rows for BN = 256, 4 for BN = 128, 2 2/3
    // for BN = 192), and fetches the logical chunk that b_chunk_position puts there
    // (the map is its own inverse).
    constexpr int CPR = B_ROW / 16;                                   // chunks per k row
    auto b_krow = [&](int t) -> int { return (64 * (wn + 4 * t) + lane) / CPR; };   // within the half
    auto b_offset = [&](int t, int ln) -> uint32_t {                  // relative to the half's first k row
        const int g = 64 * (wn + 4 * t) + ln;
        const int krow = g / CPR;
        int col = 8 * b_chunk_position<BN>(g % CPR, krow);
        if (n0 + col + 8 > p.N) col = 0;                              // clamp: loaded, never stored
        return ((uint32_t)krow * (uint32_t)p.ldb + col) * 2;
    };
    // Copy t (of 4 per wavefront) of one A half of k step s into A buffer s%2;
    // `off` = the caller's 4 lane offsets.  A whole k step goes global -> LDS
    // directly; the k tail (the last k step when K is not a multiple of 64) goes
    // through registers, zero beyond K.
    auto copy_a_part = [&](int s, int half, const uint32_t (&off)[4], int t, auto whole_tag) {
        const uint32_t dst = smem_base + A_REGION + (s & 1) * A_BUF + half * (A_BUF / 2) + 1024 * (wn + 4 * t);
        const half_t* src = a_tile + (int64_t)s * BK;
        if constexpr (decltype(whole_tag)::value) {
            async_copy16(src, off[t], dst);
        } else {
            const int kvalid = p.K - s * BK;
            uintx4 v = {0u, 0u, 0u, 0u};
            if (8 * a_chunk < kvalid) v = *reinterpret_cast<const uintx4*>((const char*)src + off[t]);
            *(__attribute__((address_space(3))) uintx4*)(uintptr_t)(dst + 16 * lane) = v;
        }
    };
    // copy t of one B half of k step s into B buffer s%3
    auto copy_b_part = [&](int s, int half, const uint32_t (&off)[4], int t, auto whole_tag) {
        const uint32_t dst = smem_base + B_REGION + (s % 3) * B_BUF + half * (B_BUF / 2) + 1024 * (wn + 4 * t);
        const half_t* src = b_tile + ((int64_t)s * BK + half * 32) * p.ldb;
        if constexpr (decltype(whole_tag)::value) {
            async_copy16(src, off[t], dst);
        } else {
            const int kvalid = p.K - s * BK - half * 32;               // valid k rows of this half (may be <= 0)
            uintx4 v = {0u, 0u, 0u, 0u};
            if (b_krow(t) < kvalid) v = *reinterpret_cast<const uintx4*>((const char*)src + off[t]);
            *(__attribute__((address_space(3))) uintx4*)(uintptr_t)(dst + 16 * lane) = v;
        }
    };

    // The same copies in two steps for the main loop: the LDS destination goes to M0 with one scalar
    // add (a wave-uniform base plus an immediate), and the load follows one MFMA later -- the MFMA
    // between them is the wait state an M0 write needs before an LDS-DMA load, so a copy costs
    // the multiplying wavefront two issue slots instead of four.
    auto a_dst_base = [&](int s, int half) -> uint32_t { return smem_base + A_REGION + (s & 1) * A_BUF + half * (A_BUF / 2) + 1024 * wn; };
    auto b_dst_base = [&](int s, int half) -> uint32_t { return smem_base + B_REGION + (s % 3) * B_BUF + half * (B_BUF / 2) + 1024 * wn; };

    // X copies A-top and B-low, Y copies A-bottom and B-high: each group brings
    // in the A rows it reads itself and one k half of B for both groups.
    uint32_t a_off[4], b_off[4];
#pragma unroll
    for (int t = 0; t < 4; t++) { a_off[t] = t < TA ? a_offset(grp, t, lane) : 0u; b_off[t] = t < TB ? b_offset(t, lane) : 0u; }

    // ---- prologue: k steps 0 and 1 ---------------------------------------------
    auto issue_k_step = [&](int s) {          // all of this wavefront's copies of k step s (0 or 1)
        if (s < KT) {
            if (!TAIL || s < kt_full) {
#pragma unroll
                for (int t = 0; t < 4; t++) { if (t < TA) copy_a_part(s, grp, a_off, t, BoolTag<true>{}); if (t < TB) copy_b_part(s, grp, b_off, t, BoolTag<true>{}); }
            } else {
#pragma unroll
                for (int t = 0; t < 4; t++) { if (t < TA) copy_a_part(s, grp, a_off, t, BoolTag<false>{}); if (t < TB) copy_b_part(s, grp, b_off, t, BoolTag<false>{}); }
            }
        }
    };
    issue_k_step(0);
    issue_k_step(1);

    bool chained = false;
    for (;;) {      // one tile per trip (a single trip unless PERSIST)
    const int cm0 = m0, cn0 = n0;             // the tile being multiplied and stored
    // Per-lane addresses that are the same for every tile are derived again per tile
    // from this copy of the lane number, which the compiler cannot see through:
    // kept across the whole loop they would not fit the register file beside the
    // accumulators and would be spilled, and reloading a spilled value waits for
    // every load and store in flight.
    int lane_t = lane;
    if constexpr (PERSIST) asm volatile("" : "+v"(lane_t));
    const bool edge = (cm0 + BM > p.M) || (cn0 + BN > p.N);
    // ---- accumulators -------------------------------------------------------
    // They start at zero; C is read once, in the epilogue, and added there
    // (C + sum formed as sum + C).  The MFMA is issued with the B fragment
    // first, i.e. it forms the transposed 32 x 32 block: register i of lane l
    // is row l%32, column 8*(i/4) + 4*(l/32) + i%4 -- 4 consecutive columns per
    // register group, which the epilogue moves 16 bytes at a time.  (16 x 16
    // blocks: register r of lane l is row l%16, column 4*(l/16) + r.)
    constexpr int FM = HM / MI, FN = WN / MI;        // accumulator blocks per wavefront tile
    typedef typename AccBlock<MI>::type acc_t;       // 16 (MI = 32) or 4 (MI = 16) registers
    acc_t acc[FM][FN];
#pragma unroll
    for (int fm = 0; fm < FM; fm++)
#pragma unroll
        for (int fn = 0; fn < FN; fn++)
#pragma unroll
            for (int i = 0; i < MI * MI / 64; i++) acc[fm][fn][i] = 0.0f;
    CT* const Cbase = (CT*)p.C;
    const int crow0 = cm0 + grp * HM;
    const int ccol0 = cn0 + wn * WN;

    // ---- fragment read addresses ----------------------------------------------
    // MI = 32: A operand lane l holds tile row l%32 of its block, k = 8*(l/32)..+7 of
    // the 16-wide slice ks -> logical chunk 2*ks + l/32 (4 slices per k step).
    // MI = 16: row l%16, k = 8*(l/16)..+7 of the 32-wide slice h -> chunk 4*h + l/16
    // (2 slices per k step).  Either way stored at chunk ^ ((row/2)%8).
    constexpr int NSL = (MI == 32) ? 4 : 2;          // k slices per k step
    uint32_t a_rd[NSL];
    {
        const int lr = lane_t & (MI - 1), lk = lane_t / MI;
        const uint32_t row_off = (uint32_t)(grp * HM + lr) * (BK * 2);
        const int sw = (lr >> 1) & 7;
#pragma unroll
        for (int sl = 0; sl < NSL; sl++)
            a_rd[sl] = smem_base + A_REGION + row_off + (uint32_t)((((64 / MI) * sl + lk) ^ sw) * 16);
    }
    // B operand: one transposing read serves 16 lanes -- lanes 4r..4r+3 of a
    // 16-lane block point at 16 consecutive columns of k row r and lane i gets
    // column i of rows 0..3; two reads (k +0..3, +4..7) make one operand.
    // MI = 32: blocks 0,1 are the two column halves at k 0..7, blocks 2,3 at k 8..15.
    // MI = 16: block b covers k 8b..8b+7 of the 32-wide slice.
    uint32_t b_rd[FN];
    {
        const int blk = lane_t >> 4, j = lane_t & 15;
        const int krow = (MI == 32) ? 8 * (blk >> 1) + (j >> 2) : 8 * blk + (j >> 2);   // first read; +4 second
#pragma unroll
        for (int fn = 0; fn < FN; fn++) {
            const int col = wn * WN + fn * MI + ((MI == 32) ? 16 * (blk & 1) : 0) + 4 * (j & 3);   // first of 4 columns
            // (the position is the same for k rows 4, 16 and 32 further on)
            b_rd[fn] = smem_base + B_REGION + (uint32_t)krow * B_ROW + (uint32_t)(b_chunk_position<BN>(col >> 3, krow) * 16 + 2 * (col & 7));
        }
    }

    half8 fa[NSL / 2][FM], fb[NSL / 2][FN];          // fragments of half a k step: [slice][fm], [slice][fn]

    auto read_fragments = [&](int k, int h) {
        const uint32_t a_buf = (uint32_t)(k & 1) * A_BUF;
        const uint32_t b_buf = (uint32_t)(k % 3) * B_BUF;
        // one address register per fragment column (fn) / k slice; the rest of
        // each address is an instruction offset
        uint32_t b0[FN];
#pragma unroll
        for (int fn = 0; fn < FN; fn++) { b0[fn] = b_rd[fn] + b_buf; asm volatile("" : "+v"(b0[fn])); }
#pragma unroll
        for (int s = 0; s < NSL / 2; s++) {
            const int sl = (NSL / 2) * h + s;
            uint32_t a0 = a_rd[sl] + a_buf;
            asm volatile("" : "+v"(a0));
#pragma unroll
            for (int fm = 0; fm < FM; fm++)
                fa[s][fm] = lds_read_b128(a0 + fm * MI * (BK * 2));
#pragma unroll
            for (int fn = 0; fn < FN; fn++) {
                const half4 lo = lds_read_tr16(b0[fn] + sl * (64 / NSL) * B_ROW);
                const half4 hi = lds_read_tr16(b0[fn] + sl * (64 / NSL) * B_ROW + 4 * B_ROW);
                fb[s][fn] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        }
    };
    // A multiplying phase: the MFMAs of half a k step (k slices of the fragments
    // just read), with this wavefront's 4 copies for k step k + 2 spread between
    // them (h = 0: its k half of B, h = 1: its own A rows).  The copies are paced
    // by the texture addresser (a wave-wide 1 KB copy occupies it for 16
    // cycles); spread out like this they neither queue up behind each other nor
    // hold up the MFMAs, which wait for the pipe anyway.  After the last MFMA of
    // a k step the wavefront waits for its copies for k step k + 1 (in-order
    // completion: only the 8 issued during this k step may be outstanding), so
    // that the barrier that follows publishes them.
    constexpr int NMFMA = (NSL / 2) * FM * FN;
    constexpr int NPRE = (sizeof(CT) == 2) ? 2 : 1;     // slabs of 32 C rows requested before the last two k steps
    constexpr int LPR = (WN == 48) ? 16 : WN / 4;       // epilogue: lanes per row segment (4 columns each; 48 columns: 12 of 16 lanes used),
    constexpr int RPP = 64 / LPR, PASSES = 32 / RPP;    // rows per pass, passes per slab of 32 rows
    // copy_tag: 0 no copies (last two k steps), 1 k step k + 2 is a whole one,
    // 2 it is the k tail
    auto multiply_phase = [&](int k, int h, auto copy_tag) {
        constexpr bool COPY = decltype(copy_tag)::value != 0;
        typedef BoolTag<decltype(copy_tag)::value == 1> whole_t;
        const uint32_t dst_base = (h == 0) ? b_dst_base(k + 2, grp) : a_dst_base(k + 2, grp);
        if constexpr (decltype(copy_tag)::value == 1 && NMFMA / 8 - 1 == 0) {
            __builtin_amdgcn_sched_barrier(0);
            set_m0(dst_base, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int s = 0; s < NSL / 2; s++)
#pragma unroll
            for (int fm = 0; fm < FM; fm++)
#pragma unroll
                for (int fn = 0; fn < FN; fn++) {
                    // B fragment first: the transposed block.  The blocks of a slice are walked two
                    // rows of blocks at a time, down, right, up, right, ... (and back in the next
                    // pair of rows), so that from one MFMA to the next exactly one operand changes and
                    // the A operand goes back and forth between two fragments.  The part is at its
                    // power limit, and what an MFMA draws depends on how its operands differ from
                    // the last one's: MFMAs alone (operands in registers, the workload's data) run
                    // 1936 TFLOP/s walking row by row (both operands change at every row end), 1960
                    // in serpentine rows, 1985 in this order, 2030 with the same operands every
                    // time; the headline gained 1.3 % from serpentine rows.
                    // (ROWWISE: a ladder row, the blocks row by row.)
                    const int lin = fm * FN + fn, pr = lin / (2 * FN), q = lin % (2 * FN);
                    const int gm = ROWWISE ? fm : 2 * pr + ((q % 4 == 1 || q % 4 == 2) ? 1 : 0);
                    const int gn = ROWWISE ? fn : (pr & 1) ? FN - 1 - q / 2 : q / 2;
                    if constexpr (MI == 32) acc[gm][gn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[s][gn], fa[s][gm], acc[gm][gn], 0, 0, 0);
                    else                    acc[gm][gn] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fb[s][gn], fa[s][gm], acc[gm][gn], 0, 0, 0);
                    const int idx = (s * FM + fm) * FN + fn;
                    if constexpr (decltype(copy_tag)::value == 1) {
                        // whole k step: copy t is loaded behind MFMA t * NMFMA/4 + NMFMA/8 - 1 and its M0 is
                        // set one MFMA earlier (copy 0 of the small tiles: in front of the first MFMA)
                        const int tl = idx / (NMFMA / 4), ts = (idx + 1) / (NMFMA / 4);
                        if (idx % (NMFMA / 4) == NMFMA / 8 - 1 && tl < (h == 0 ? TB : TA)) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (h == 0) async_copy16_m0(b_tile + ((int64_t)(k + 2) * BK + grp * 32) * p.ldb, b_off[tl]);
                            else        async_copy16_m0(a_tile + (int64_t)(k + 2) * BK, a_off[tl]);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        if ((idx + 1) % (NMFMA / 4) == NMFMA / 8 - 1 && ts < (h == 0 ? TB : TA)) {
                            __builtin_amdgcn_sched_barrier(0);
                            set_m0(dst_base, 4096 * ts);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    } else if (COPY && idx % (NMFMA / 4) == NMFMA / 8 - 1) {
                        __builtin_amdgcn_sched_barrier(0);
                        if (h == 0) { if (idx / (NMFMA / 4) < TB) copy_b_part(k + 2, grp, b_off, idx / (NMFMA / 4), whole_t{}); }
                        else        { if (idx / (NMFMA / 4) < TA) copy_a_part(k + 2, grp, a_off, idx / (NMFMA / 4), whole_t{}); }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
        if (h == 1) {
            __builtin_amdgcn_sched_barrier(0);
            if (whole_t::value) {
                asm volatile("s_waitcnt vmcnt(%0)" :: "n"(TA + TB) : "memory");      // this k step's copies may be outstanding
            }
            else if constexpr (decltype(copy_tag)::value == 0) {
                // the last two k steps: only the early C loads (8 per slab) may be outstanding
                asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"(NPRE * PASSES) : "memory");
            } else {
                asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            }
        }
    };
    auto k_step = [&](int k, auto copy_tag) {
#pragma unroll
        for (int h = 0; h < 2; h++) {
            read_fragments(k, h);          // X: phase 4k + 2h,     Y: 4k + 2h + 1
            // lgkmcnt(0), as the builtin: the compiler then knows that the fragments have arrived
            // and puts no waits of its own between the MFMAs that use them
            __builtin_amdgcn_s_waitcnt(0xC07F);
            asm volatile("" ::: "memory");
            phase_barrier();
            multiply_phase(k, h, copy_tag);          // X: phase 4k + 2h + 1, Y: 4k + 2h + 2
            if (decltype(copy_tag)::value != 0 || grp == 0 || h == 0 || k + 1 < KT) phase_barrier();
        }
    };

    // k step 0 has landed before phase 0; the 8 copies of k step 1 (issued
    // behind it, completing in order) may still be on their way -- the wait at
    // the end of k step 0 covers them
    // (A chained tile's k step 0 was requested before the epilogue of the tile
    // before it and that epilogue has since consumed C loads requested later: loads
    // complete in order, so it has landed.  Not waiting here matters: a wait would
    // also count the C stores just issued.)
    if (!PERSIST || !chained) {
        if (1 < kt_full) {
            asm volatile("s_waitcnt vmcnt(%0)" :: "n"(TA + TB) : "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        }
    } else if (TAIL && kt_full < 1) {
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");       // k step 0 went through registers
    }
    phase_barrier();

    // Both groups run the same loop; Y enters it one phase (one barrier) later
    // and leaves out the last barrier, so every wavefront meets the same
    // number of barriers.
    if (grp == 1) phase_barrier();         // phase 0: X reads, Y has nothing to do yet
    // k steps that issue copies for step k + 2, then the last two, which do not
    int k = 0;
    for (; k + 2 < kt_full; k++) k_step(k, IntTag<1>{});
    if constexpr (TAIL) { for (; k + 2 < KT; k++) k_step(k, IntTag<2>{}); }     // at most once: fetches the k tail

    // ---- C: addresses, and the first rows on their way -----------------------------
    // The last two k steps issue no copies; the first 32 rows of this wavefront's
    // part of C (64 for f16 C) are requested here, so that they arrive while those
    // k steps are multiplied (loads complete in order: the waits of those k steps
    // leave exactly these loads outstanding).
    typedef typename CVec4<CT>::type ctx4;
    constexpr int PITCH = LPR * 16 + 16;                     // 272 B for 64 (and 48) columns
    // (PERSIST: in the second A buffer and the second and third B buffers, which the
    // next tile's k step 0 leaves alone)
    const uint32_t tbuf = !PERSIST ? smem_base + (uint32_t)wave * (32u * PITCH)
                        : wave < 3 ? smem_base + A_BUF + (uint32_t)wave * (32u * PITCH)
                                   : smem_base + B_REGION + B_BUF + (uint32_t)(wave - 3) * (32u * PITCH);
    // where this lane's 4 consecutive columns of a block go: row l%MI, column 4*(l/MI) (+ block offsets)
    int lane_e = lane;
    if constexpr (PERSIST) asm volatile("" : "+v"(lane_e));
    const uint32_t w_addr = tbuf + (uint32_t)(lane_e & (MI - 1)) * PITCH + (uint32_t)(lane_e / MI) * 16;
    const uint32_t r_addr = tbuf + (uint32_t)(lane_e / LPR) * PITCH + (uint32_t)(lane_e % LPR) * 16;
    const int orow = lane_e / LPR, ocol = 4 * (lane_e % LPR);     // this lane's row (of RPP) and column in a pass
    const bool col_ok = (LPR * 4 == WN || ocol < WN) && (!edge || (ccol0 + ocol < p.N));   // N is a multiple of 8: all 4 columns or none
    CT* const cptr = Cbase + (int64_t)(crow0 + orow) * p.ldc + ccol0 + ocol;
    float bias4[4] = {0.0f, 0.0f, 0.0f, 0.0f};              // fused epilogue: this lane's 4 columns of the bias
    if (p.bias && col_ok) {
#pragma unroll
        for (int e = 0; e < 4; e++) bias4[e] = (float)reinterpret_cast<const CT*>(p.bias)[ccol0 + ocol + e];
    }
    ctx4 cin[2][PASSES];
    auto fetch = [&](int fm, ctx4 (&dst)[PASSES]) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ps++) {
            const bool ok = col_ok && (!edge || (crow0 + fm * 32 + RPP * ps + orow < p.M));
            // a group outside C reads this lane's first (valid or clamped) group of the tile instead
            const CT* src = ok ? cptr + (int64_t)(fm * 32 + RPP * ps) * p.ldc : Cbase + (int64_t)cm0 * p.ldc + cn0;
            dst[ps] = *reinterpret_cast<const ctx4*>(src);
        }
    };
#pragma unroll
    for (int f = 0; f < NPRE; f++) fetch(f, cin[f]);
    __builtin_amdgcn_sched_barrier(0);
    for (; k < KT; k++) k_step(k, IntTag<0>{});

    // ---- PERSIST: the next tile's k step 0 on its way before this tile's epilogue ----
    bool has_next = false;
    if constexpr (PERSIST) {
        has_next = next_tile < p.tiles_m * p.tiles_n;
        if (has_next) {
            int tm, tn;
            tile_of_block(p, next_tile, tm, tn);
            next_tile += tile_step;
            m0 = tm * BM; n0 = tn * BN;
            a_tile = p.A + (int64_t)m0 * p.lda;
            b_tile = p.B + n0;
            int ln = lane;
            asm volatile("" : "+v"(ln));
#pragma unroll
            for (int t = 0; t < 4; t++) { a_off[t] = t < TA ? a_offset(grp, t, ln) : 0u; b_off[t] = t < TB ? b_offset(t, ln) : 0u; }
            issue_k_step(0);
        }
    }

    // ---- + C, -> C ---------------------------------------------------------------
    // Behind the last barrier nobody reads the A/B buffers any more, so each
    // wavefront takes 8.5 KB of LDS as a private transposing buffer: 32 rows x
    // 64 columns of its accumulators at a time go in as they sit in registers
    // (16 bytes per lane, row pitch 272 B: conflict-free) and come back with 16
    // lanes covering one row, so that C is read and written in whole 256-byte
    // row segments (128 B for f16 C), 16 bytes (8) per lane.
    {
#pragma unroll
        for (int fm = 0; fm < HM / 32; fm++) {
            if (fm + 1 < HM / 32 && fm + 1 >= NPRE) fetch(fm + 1, cin[(fm + 1) & 1]);
            if constexpr (MI == 32) {
#pragma unroll
                for (int fn = 0; fn < FN; fn++)
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        const floatx4 v = {acc[fm][fn][4 * g], acc[fm][fn][4 * g + 1], acc[fm][fn][4 * g + 2], acc[fm][fn][4 * g + 3]};
                        *(__attribute__((address_space(3))) floatx4*)(uintptr_t)(w_addr + (fn * 32 + 8 * g) * 4) = v;
                    }
            } else {
#pragma unroll
                for (int r = 0; r < 2; r++)
#pragma unroll
                    for (int fn = 0; fn < FN; fn++)
                        *(__attribute__((address_space(3))) floatx4*)(uintptr_t)(w_addr + r * 16 * PITCH + fn * 16 * 4) = acc[2 * fm + r][fn];
            }
#pragma unroll
            for (int ps = 0; ps < PASSES; ps++) {
                const floatx4 s4 = *(__attribute__((address_space(3))) const floatx4*)(uintptr_t)(r_addr + RPP * ps * PITCH);
                const ctx4 c4 = cin[fm & 1][ps];
                ctx4 o;
#pragma unroll
                for (int e = 0; e < 4; e++) o[e] = (CT)epilogue_value(s4[e] + (float)c4[e], bias4[e], p.relu);      // f16: one rounding, to nearest even
                if (col_ok && (!edge || (crow0 + fm * 32 + RPP * ps + orow < p.M)))
                    *reinterpret_cast<ctx4*>(cptr + (int64_t)(fm * 32 + RPP * ps) * p.ldc) = o;
            }
        }
    }
    if (!PERSIST || !has_next) break;
    // every wavefront is done with its transposing buffer: k step 1 may overwrite them
    phase_barrier();
    {   // the lane offsets once more (not kept across the epilogue)
        int ln = lane;
        asm volatile("" : "+v"(ln));
#pragma unroll
        for (int t = 0; t < 4; t++) { a_off[t] = t < TA ? a_offset(grp, t, ln) : 0u; b_off[t] = t < TB ? b_offset(t, ln) : 0u; }
    }
    issue_k_step(1);
    chained = true;
    }   // tiles
}

// Short k loops with several tiles per compute unit: the workgroups that start on
// every other XCD (consecutive block indices go to the XCDs in turn, so with an even
// number of XCDs odd indices are odd XCDs) begin 10-15 us late and stay that far behind,
// so that the two halves of the chip read and write C -- which takes all of HBM's
// bandwidth when every unit does it at once -- at different times.  Whole XCDs are
// shifted, so each L2 still serves units that walk k in lockstep.  Only the first
// p.first_generation workgroups wait (those that start when the launch does; the others
// start as units free up and inherit the offset).  The delay is paid once per launch:
// measured +2 ... +4 % at 3 tiles per unit, +4 ... +10 % at 4-8.  The wait is bounded (it
// ends after 20 000 polls whatever the clock says) and changes no result.
__device__ __forceinline__ void late_start(const TiledParams& p)
{
    if (p.stagger_ticks > 0 && (blockIdx.x & 1) && (int)blockIdx.x < p.first_generation) {
        const uint64_t t0 = wall_clock64();
        for (int spins = 0; wall_clock64() - t0 < (uint64_t)p.stagger_ticks && spins < 20000; spins++) __builtin_amdgcn_s_sleep(16);
    }
}
// Host side: the delay in wall-clock ticks, or 0 where the late start does not apply -- the
// device must deal workgroups to an even number (two or more) of XCDs.
inline int late_start_ticks()
{
    const ChipShape& c = chip();
    if (c.xcds < 2 || (c.xcds & 1)) return 0;
    return (int)(12e-6 * 1e3 * c.wall_clock_khz);          // 12 us
}
// workgroups that run at once: one per compute unit, two where the LDS allows
template <int BM, int BN>
int pp_at_once() { return chip().cus * (pp_lds_bytes<BM, BN>() <= 80 * 1024 ? 2 : 1); }

template <typename CT, int MI, bool TAIL, int BM, int BN, bool ROWWISE = false>
__global__ __launch_bounds__(512) void gemm_pp256_kernel(const TiledParams p)
{
    __shared__ __attribute__((aligned(1024))) char smem[pp_lds_bytes<BM, BN>()];
    late_start(p);
    int tile_m, tile_n;
    tile_of_block(p, blockIdx.x, tile_m, tile_n);
    pp_tile<CT, MI, TAIL, BM, BN, false, ROWWISE>(p, (uint32_t)(uintptr_t)(lds_ptr_t)smem, tile_m * BM, tile_n * BN);
}

// One workgroup per compute unit walks the tiles blockIdx.x, blockIdx.x + gridDim.x,
// ... (the same tiles, in the same order, that the hardware would hand that unit
// when every tile is a workgroup of its own and all tiles take equally long).
template <typename CT, int MI, bool TAIL>
__global__ __launch_bounds__(512) void gemm_pp256_persistent_kernel(const TiledParams p)
{
    __shared__ __attribute__((aligned(1024))) char smem[pp_lds_bytes<256, 256>()];
    late_start(p);
    int tile_m, tile_n;
    tile_of_block(p, blockIdx.x, tile_m, tile_n);
    pp_tile<CT, MI, TAIL, 256, 256, true>(p, (uint32_t)(uintptr_t)(lds_ptr_t)smem, tile_m * 256, tile_n * 256,
                                          (int)(blockIdx.x + gridDim.x), (int)gridDim.x);
}

// The 256 x 256 tiling with the first-generation workgroups of every other compute
// unit (block index bit 5: the hardware hands consecutive workgroups to the 8 XCDs
// in turn and, within an XCD, to its 4 shader engines in turn) taking only the top
// 128 rows of their tile; the bottom halves come last in the grid.  Those units
// then stay half a tile ahead of the others for the whole launch, so that at any
// time about half the chip is in its epilogue -- the C read and write, which on
// short-K problems saturates HBM when all units do it at once -- while the other
// half multiplies.  Results do not depend on where workgroups actually land.
constexpr int MIXED_HALVES = 128;
template <typename CT, int MI, bool TAIL>
__global__ __launch_bounds__(512) void gemm_pp_mixed_kernel(const TiledParams p)
{
    __shared__ __attribute__((aligned(1024))) char smem[pp_lds_bytes<256, 256>()];
    const uint32_t smem_base = (uint32_t)(uintptr_t)(lds_ptr_t)smem;
    const int tiles = p.tiles_m * p.tiles_n;
    int b = blockIdx.x, half = -1;
    if (b >= tiles) { const int r = b - tiles; b = ((r >> 5) << 6) | 32 | (r & 31); half = 1; }   // r-th block of the first generation with bit 5 set
    else if (b < p.first_generation && (b & 32)) half = 0;
    int tile_m, tile_n;
    tile_of_block(p, b, tile_m, tile_n);
    if (half < 0) {
        pp_tile<CT, MI, TAIL, 256, 256>(p, smem_base, tile_m * 256, tile_n * 256);
    } else {
        const int m0 = tile_m * 256 + 128 * half;
        if (m0 < p.M) pp_tile<CT, MI, TAIL, 128, 256>(p, smem_base, m0, tile_n * 256);
    }
}

template <int BM, int BN>
int64_t grid_pp(int64_t M, int64_t N)
{
    const int64_t tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
    if (tm > 0 && tn > INT32_MAX / tm) return -1;
    return tm * tn;
}

template <int MI, int BM, int BN>
int launch_pp(const GemmArgs& a, bool xcd_order = true)
{
    const int64_t g = grid_pp<BM, BN>(a.M, a.N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    TiledParams p = make_tiled_params(a, BM, BN, 8);       // an XCD's 32 concurrent tiles form an 8 x 4 block of C
    if (!xcd_order) p.num_xcd = 1;
    // late start of every other XCD (see late_start): short k loops and four or more rounds of workgroups
    // (measured +4 ... +9 % on every tile form; at three rounds of the 128 x 128 form the delay costs more than it gains)
    p.first_generation = pp_at_once<BM, BN>();
    p.stagger_ticks = (a.K <= 2048 && g >= 4 * (int64_t)p.first_generation) ? late_start_ticks() : 0;
    const bool tail = (a.K % BK) != 0;
    if (a.c_is_f16) {
        if (tail) hipLaunchKernelGGL((gemm_pp256_kernel<half_t, MI, true, BM, BN>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
        else      hipLaunchKernelGGL((gemm_pp256_kernel<half_t, MI, false, BM, BN>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
    } else {
        if (tail) hipLaunchKernelGGL((gemm_pp256_kernel<float, MI, true, BM, BN>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
        else      hipLaunchKernelGGL((gemm_pp256_kernel<float, MI, false, BM, BN>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
    }
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}
template <int MI, int BM, int BN> int launch_pp_plain(const GemmArgs& a) { return launch_pp<MI, BM, BN>(a); }

// The staggered form is laid out for 256 compute units (the half tiles are the first-generation
// workgroups with bit 5 of the index set: 128 of them); on any other device, and with fewer
// than two tiles per compute unit, the plain tiling runs.
bool mixed_applies(int64_t tiles) { return chip().cus == 2 * MIXED_HALVES && tiles >= 2 * chip().cus; }

int64_t grid_pp_mixed(int64_t M, int64_t N)
{
    const int64_t g = grid_pp<256, 256>(M, N);
    return (g < 0 || !mixed_applies(g)) ? g : g + MIXED_HALVES;
}

int launch_pp_mixed(const GemmArgs& a)
{
    const int64_t tiles = grid_pp<256, 256>(a.M, a.N);
    if (tiles < 0 || tiles + MIXED_HALVES > INT32_MAX) return GEMM_F16_ERR_SIZE;
    if (!mixed_applies(tiles)) return launch_pp<16, 256, 256>(a);
    const int64_t g = tiles + MIXED_HALVES;
    TiledParams p = make_tiled_params(a, 256, 256, 8);
    p.first_generation = chip().cus;
    const bool tail = (a.K % BK) != 0;
    if (a.c_is_f16) {
        if (tail) hipLaunchKernelGGL((gemm_pp_mixed_kernel<half_t, 16, true>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
        else      hipLaunchKernelGGL((gemm_pp_mixed_kernel<half_t, 16, false>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
    } else {
        if (tail) hipLaunchKernelGGL((gemm_pp_mixed_kernel<float, 16, true>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
        else      hipLaunchKernelGGL((gemm_pp_mixed_kernel<float, 16, false>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
    }
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}

int64_t grid_pp_persistent(int64_t M, int64_t N)
{
    const int64_t g = grid_pp<256, 256>(M, N);
    return g < chip().cus ? g : chip().cus;
}

int launch_pp_persistent(const GemmArgs& a)
{
    const int64_t tiles = grid_pp<256, 256>(a.M, a.N);
    if (tiles < 0) return GEMM_F16_ERR_SIZE;
    if (tiles <= chip().cus) return launch_pp<16, 256, 256>(a);      // one tile each: nothing to chain
    const unsigned g = (unsigned)chip().cus;
    TiledParams p = make_tiled_params(a, 256, 256, 8);
    p.first_generation = (int)g;
    p.stagger_ticks = (a.K <= 2048 && tiles >= 3 * (int64_t)g) ? late_start_ticks() : 0;
    const bool tail = (a.K % BK) != 0;
    if (a.c_is_f16) {
        if (tail) hipLaunchKernelGGL((gemm_pp256_persistent_kernel<half_t, 16, true>), dim3(g), dim3(512), 0, a.stream, p);
        else      hipLaunchKernelGGL((gemm_pp256_persistent_kernel<half_t, 16, false>), dim3(g), dim3(512), 0, a.stream, p);
    } else {
        if (tail) hipLaunchKernelGGL((gemm_pp256_persistent_kernel<float, 16, true>), dim3(g), dim3(512), 0, a.stream, p);
        else      hipLaunchKernelGGL((gemm_pp256_persistent_kernel<float, 16, false>), dim3(g), dim3(512), 0, a.stream, p);
    }
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}

constexpr int lds_pp(int bm, int bn) { return 2 * bm * BK * 2 + 3 * BK * bn * 2; }
const GemmConfigDesc kPingPong16 = {
    "pp256x256x64_w2x4_mi16", 256, 256, BK, 8, 128, 64, lds_pp(256, 256), true, launch_pp_plain<16, 256, 256>, grid_pp<256, 256>};
const GemmConfigDesc kPingPong16_192 = {
    "pp192x256x64_w2x4_mi16", 192, 256, BK, 8, 96, 64, lds_pp(192, 256), true, launch_pp_plain<16, 192, 256>, grid_pp<192, 256>};
const GemmConfigDesc kPingPong16_128 = {
    "pp128x256x64_w2x4_mi16", 128, 256, BK, 8, 64, 64, lds_pp(128, 256), true, launch_pp_plain<16, 128, 256>, grid_pp<128, 256>};
const GemmConfigDesc kPingPong16_256x192 = {
    "pp256x192x64_w2x4_mi16", 256, 192, BK, 8, 128, 48, lds_pp(256, 192), true, launch_pp_plain<16, 256, 192>, grid_pp<256, 192>};
const GemmConfigDesc kPingPong16_128x128 = {
    "pp128x128x64_w2x4_mi16", 128, 128, BK, 8, 64, 32, lds_pp(128, 128), true, launch_pp_plain<16, 128, 128>, grid_pp<128, 128>};
const GemmConfigDesc kPingPong16Mixed = {
    "pp256x256x64_w2x4_mi16_stag", 256, 256, BK, 8, 128, 64, lds_pp(256, 256), true, launch_pp_mixed, grid_pp_mixed};
const GemmConfigDesc kPingPong16Persistent = {
    "pp256x256x64_w2x4_mi16_chain", 256, 256, BK, 8, 128, 64, lds_pp(256, 256), true, launch_pp_persistent, grid_pp_persistent};
#ifdef GEMM_F16_LADDER
// ladder rows: the same kernel on 32x32x16 MFMAs, and with the tiles dealt to the XCDs the way
// the hardware deals workgroups (no XCD-aware order: the 8 L2s then each see tiles from all over C)
int launch_pp_no_xcd_order(const GemmArgs& a) { return launch_pp<16, 256, 256>(a, false); }
// ladder row: the plain 256 x 256 kernel with the MFMAs of a phase issued row by row of blocks
int launch_pp_rowwise(const GemmArgs& a)
{
    const int64_t g = grid_pp<256, 256>(a.M, a.N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    TiledParams p = make_tiled_params(a, 256, 256, 8);
    p.first_generation = pp_at_once<256, 256>();
    p.stagger_ticks = (a.K <= 2048 && g >= 4 * (int64_t)p.first_generation) ? late_start_ticks() : 0;     // as launch_pp
    const bool tail = (a.K % BK) != 0;
    if (a.c_is_f16) {
        if (tail) hipLaunchKernelGGL((gemm_pp256_kernel<half_t, 16, true, 256, 256, true>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
        else      hipLaunchKernelGGL((gemm_pp256_kernel<half_t, 16, false, 256, 256, true>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
    } else {
        if (tail) hipLaunchKernelGGL((gemm_pp256_kernel<float, 16, true, 256, 256, true>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
        else      hipLaunchKernelGGL((gemm_pp256_kernel<float, 16, false, 256, 256, true>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
    }
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}
const GemmConfigDesc kPingPong = {
    "pp256x256x64_w2x4", 256, 256, BK, 8, 128, 64, lds_pp(256, 256), true, launch_pp_plain<32, 256, 256>, grid_pp<256, 256>};
const GemmConfigDesc kPingPong16_192x192 = {
    "pp192x192x64_w2x4_mi16", 192, 192, BK, 8, 96, 48, lds_pp(192, 192), true, launch_pp_plain<16, 192, 192>, grid_pp<192, 192>};
const GemmConfigDesc kPingPong16Rowwise = {
    "pp256x256x64_w2x4_mi16_rowwise", 256, 256, BK, 8, 128, 64, lds_pp(256, 256), true, launch_pp_rowwise, grid_pp<256, 256>};
const GemmConfigDesc kPingPong16NoXcd = {
    "pp256x256x64_w2x4_mi16_noxcd", 256, 256, BK, 8, 128, 64, lds_pp(256, 256), true, launch_pp_no_xcd_order, grid_pp<256, 256>};
#endif

}  // namespace

const GemmConfigDesc* pingpong16_persistent_config() { return &kPingPong16Persistent; }
const GemmConfigDesc* pingpong16_staggered_config() { return &kPingPong16Mixed; }
const GemmConfigDesc* pingpong16_config(int bm, int bn)
{
    if (bn == 128) return &kPingPong16_128x128;
    if (bn == 192) return &kPingPong16_256x192;
    return bm == 128 ? &kPingPong16_128 : bm == 192 ? &kPingPong16_192 : &kPingPong16;
}
#ifdef GEMM_F16_LADDER
const GemmConfigDesc* pingpong_config() { return &kPingPong; }
const GemmConfigDesc* pingpong16_no_xcd_order_config() { return &kPingPong16NoXcd; }
const GemmConfigDesc* pingpong16_192x192_config() { return &kPingPong16_192x192; }
const GemmConfigDesc* pingpong16_rowwise_config() { return &kPingPong16Rowwise; }
#endif
