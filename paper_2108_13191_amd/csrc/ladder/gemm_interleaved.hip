// A ladder row (comparison kernel, never selected): the 256 x 256 tile of the
// phase-alternating kernel (gemm_pingpong.hip) -- same 8 wavefronts of 128 x 64,
// k steps of 64, v_mfma_f32_16x16x32_f16, LDS image, copy plan and epilogue --
// but BOTH wavefronts of a SIMD multiply all the time: every wavefront
// software-pipelines its own fragment reads between its own MFMAs (the paper's
// "Completing Latency Hiding" applied one level further down: LDS -> register
// loads for a later block of MFMAs are in flight while the current block is
// multiplied), and there is one barrier per k step instead of four.
//
// Outcome on the headline workload: 5-8 % slower than the phase-alternating
// kernel (about 2650 against 2400 cycles per k step).  The older wavefront of a
// SIMD wins the issue arbitration and reaches the barrier about 800 cycles
// before the younger one, which finishes its k step alone; every LDS read,
// copy, address add and wait of a wavefront sits between two of its own MFMAs;
// and the part being power-limited, the less busy matrix pipe (0.67 against
// 0.77) only partly turns into a higher clock (1.58 against 1.44 GHz).
//
// A k step of a wavefront is four blocks of 16 MFMAs (k slice s = 0, 1 of 32;
// accumulator rows fm 0-3 or 4-7; all four accumulator columns):
//   block 0: slice 0, rows 0-3   while reading  A(slice 0, rows 4-7)
//   block 1: slice 0, rows 4-7   while reading  A(slice 1, rows 0-3), B(slice 1)
//   block 2: slice 1, rows 0-3   while reading  A(slice 1, rows 4-7)
//   -- wait for own LDS reads and for the copies of k step k+1; barrier --
//   block 3: slice 1, rows 4-7   while reading  A, B(slice 0, rows 0-3) of k step k+1
// Two register sets of 4 A fragments and two of 4 B fragments (64 VGPRs) rotate
// through the blocks.  Behind the barrier of k step k every wavefront has read
// all of A(k) and B(k): the A copies for k step k+2 (into the buffer of A(k);
// two A buffers) are issued in block 3, the B copies for k+2 (three B buffers:
// into the buffer of B(k-1)) in blocks 0 and 1.  Copies complete in order, so
// "at most this k step's B copies outstanding" at the barrier means k+1 has landed.
// K must be a multiple of 64 (k tails run the phase-alternating kernel).
#include "../gemm_device.h"
#include "../../../include/gemm_f16.h"

namespace {

using namespace gemm_dev;

__device__ __forceinline__ void fence_schedule() { __builtin_amdgcn_sched_barrier(0); }

__device__ __forceinline__ void workgroup_barrier()
{
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

template <bool V> struct Flag { static constexpr bool value = V; };

constexpr int IL_BM = 256, IL_BN = 256;
constexpr int IL_A_BUF = IL_BM * BK * 2;            // 32 KB
constexpr int IL_B_BUF = BK * IL_BN * 2;            // 32 KB
constexpr int IL_B_REGION = 2 * IL_A_BUF;
constexpr int IL_LDS = 2 * IL_A_BUF + 3 * IL_B_BUF; // 160 KB
constexpr int IL_B_ROW = IL_BN * 2;                 // bytes per k row of a B stage

// position of 16-byte chunk `chunk` of k row `krow` within its row (see gemm_pingpong.hip)
__device__ __forceinline__ int il_b_chunk_position(int chunk, int krow)
{
    return chunk ^ (((krow & 3) << 2) | (((krow >> 3) & 1) << 1));
}

template <typename CT>
__device__ __forceinline__ void il_tile(const TiledParams& p, const uint32_t smem_base, const int m0, const int n0)
{
    constexpr int HM = IL_BM / 2, WN = IL_BN / 4;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave >> 2;                 // 0: top 128 rows, 1: bottom 128 rows
    const int wn = wave & 3;                   // column block of 64; also the copy slot within the group
    const int KT = p.K / BK;                   // K is a multiple of 64 here
    const bool edge = (m0 + IL_BM > p.M) || (n0 + IL_BN > p.N);

    // ---- copy plan: as in the phase-alternating kernel ---------------------------------
    // group 0 copies the top A rows and k rows 0-31 of B, group 1 the bottom A rows and k
    // rows 32-63 of B; 4 wave-wide 1 KB copies of each per wavefront and k step
    const half_t* const a_tile = p.A + (int64_t)m0 * p.lda;
    const half_t* const b_tile = p.B + n0;
    uint32_t a_off[4], b_off[4];
#pragma unroll
    for (int t = 0; t < 4; t++) {
        const int a_chunk = (lane & 7) ^ (4 * (wn & 1) + (lane >> 4));
        int row = grp * HM + 8 * (wn + 4 * t) + (lane >> 3);
        row = (m0 + row < p.M) ? row : p.M - 1 - m0;                  // clamp: loaded, never stored
        a_off[t] = ((uint32_t)row * (uint32_t)p.lda + 8 * a_chunk) * 2;
        const int g = 64 * (wn + 4 * t) + lane;                       // chunk index within the B half
        const int krow = g / 32;
        int col = 8 * il_b_chunk_position(g % 32, krow);
        if (n0 + col + 8 > p.N) col = 0;                              // clamp: loaded, never stored
        b_off[t] = ((uint32_t)krow * (uint32_t)p.ldb + col) * 2;
    }
    auto copy_a = [&](int s, int t) {
        const uint32_t dst = smem_base + (s & 1) * IL_A_BUF + grp * (IL_A_BUF / 2) + 1024 * (wn + 4 * t);
        async_copy16(a_tile + (int64_t)s * BK, a_off[t], dst);
    };
    auto copy_b = [&](int s, int t) {
        const uint32_t dst = smem_base + IL_B_REGION + (s % 3) * IL_B_BUF + grp * (IL_B_BUF / 2) + 1024 * (wn + 4 * t);
        async_copy16(b_tile + ((int64_t)s * BK + grp * 32) * p.ldb, b_off[t], dst);
    };

    // ---- prologue: k steps 0 and 1 on their way ------------------------------------------
#pragma unroll
    for (int t = 0; t < 4; t++) { copy_a(0, t); copy_b(0, t); }
    if (KT > 1) {
#pragma unroll
        for (int t = 0; t < 4; t++) { copy_a(1, t); copy_b(1, t); }
    }
#define copy_a(s, t) copy_a(s, t)
#define copy_b(s, t) copy_b(s, t)

    // ---- accumulators: 8 x 4 blocks of 16 x 16, formed transposed (B fragment first), so
    // that register r of lane l of a block is row l%16, column 4*(l/16) + r --------------
    floatx4 acc[8][4];
#pragma unroll
    for (int fm = 0; fm < 8; fm++)
#pragma unroll
        for (int fn = 0; fn < 4; fn++) acc[fm][fn] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

    // ---- fragment read addresses (buffer 0; the buffer offset is added per k step) --------
    // A operand: lane l holds row l%16 of its block, k = 8*(l/16)..+7 of the 32-wide slice s
    // -> logical chunk 4 s + l/16, stored at chunk ^ ((row/2)%8); block fm is an instruction offset.
    uint32_t a_rd[2];
    {
        const int lr = lane & 15, lk = lane >> 4;
        const uint32_t row_off = (uint32_t)(grp * HM + lr) * (BK * 2);
        const int sw = (lr >> 1) & 7;
#pragma unroll
        for (int s = 0; s < 2; s++) a_rd[s] = smem_base + row_off + (uint32_t)(((4 * s + lk) ^ sw) * 16);
    }
    // B operand: a transposing read serves 16 lanes (lanes 4r..4r+3 point at 16 consecutive
    // columns of k row r); 16-lane block b covers k 8b..8b+7 of the slice; two reads (k +0..3,
    // +4..7) make one operand.  The slice is an instruction offset.
    uint32_t b_rd[4];
    {
        const int blk = lane >> 4, j = lane & 15;
        const int krow = 8 * blk + (j >> 2);
#pragma unroll
        for (int fn = 0; fn < 4; fn++) {
            const int col = wn * WN + fn * 16 + 4 * (j & 3);
            b_rd[fn] = smem_base + IL_B_REGION + (uint32_t)krow * IL_B_ROW + (uint32_t)(il_b_chunk_position(col >> 3, krow) * 16 + 2 * (col & 7));
        }
    }

    half8 fa[2][4], fb[2][4];                  // two sets of 4 A fragments, two of 4 B fragments
    auto read_a = [&](half8 (&dst)[4], int k, int s, int half) {
        uint32_t a0 = a_rd[s] + (uint32_t)(k & 1) * IL_A_BUF;
        asm volatile("" : "+v"(a0));
#pragma unroll
        for (int i = 0; i < 4; i++) dst[i] = lds_read_b128(a0 + (4 * half + i) * 16 * (BK * 2));
    };
    auto read_b = [&](half8 (&dst)[4], int k, int s) {
        const uint32_t b_buf = (uint32_t)(k % 3) * IL_B_BUF;
#pragma unroll
        for (int fn = 0; fn < 4; fn++) {
            uint32_t b0 = b_rd[fn] + b_buf;
            asm volatile("" : "+v"(b0));
            const half4 lo = lds_read_tr16(b0 + s * 32 * IL_B_ROW);
            const half4 hi = lds_read_tr16(b0 + s * 32 * IL_B_ROW + 4 * IL_B_ROW);
            dst[fn] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    // 16 MFMAs: accumulator rows 4*half..+3, all four columns; the B fragment is held for four
    // MFMAs in a row.  `reads()` runs behind the second MFMA (the fragment reads for a later
    // block: issued here, not in front of the block, so that the wait in front of the block's
    // first MFMA covers exactly the reads of the block before); `copy(c)`, c = 0..3, behind
    // MFMAs 4, 7, 10 and 13.
    auto multiply = [&](const half8 (&a)[4], const half8 (&b)[4], int half, auto reads, auto copy) {
#pragma unroll
        for (int fn = 0; fn < 4; fn++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                acc[4 * half + i][fn] = __builtin_amdgcn_mfma_f32_16x16x32_f16(b[fn], a[i], acc[4 * half + i][fn], 0, 0, 0);
                const int idx = 4 * fn + i;
                if (idx == 1) { fence_schedule(); reads(); fence_schedule(); }
                if (idx >= 4 && idx % 3 == 1) { fence_schedule(); copy(idx / 3 - 1); fence_schedule(); }
            }
    };
    auto none = [](int) {};

    // k step k.  CP: the copies of k step k + 2 exist; NEXT: so does k step k + 1.
    auto k_step = [&](int k, auto cp, auto next) {
        constexpr bool CP = decltype(cp)::value, NEXT = decltype(next)::value;
        fence_schedule();
        multiply(fa[0], fb[0], 0, [&]() { read_a(fa[1], k, 0, 1); },
                 [&](int c) { if (CP && c >= 2) copy_b(k + 2, c - 2); });
        fence_schedule();
        multiply(fa[1], fb[0], 1, [&]() { read_a(fa[0], k, 1, 0); read_b(fb[1], k, 1); },
                 [&](int c) { if (CP && c >= 2) copy_b(k + 2, c); });
        fence_schedule();
        multiply(fa[0], fb[1], 0, [&]() { read_a(fa[1], k, 1, 1); }, none);
        fence_schedule();
        // own reads of A(k), B(k) complete; k step k + 1 has landed (in-order completion: only the
        // B copies issued during this k step may be outstanding); the barrier publishes both
        if (CP) asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
        else    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        workgroup_barrier();
        multiply(fa[1], fb[1], 1, [&]() { if (NEXT) { read_a(fa[0], k + 1, 0, 0); read_b(fb[0], k + 1, 0); } },
                 [&](int c) { if (CP) copy_a(k + 2, c); });
        fence_schedule();
    };

    // k step 0 has landed (the 8 copies of k step 1 behind it may be outstanding)
    if (KT > 1) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    workgroup_barrier();
    read_a(fa[0], 0, 0, 0);
    read_b(fb[0], 0, 0);
    fence_schedule();

    int k = 0;
    for (; k + 2 < KT; k++) k_step(k, Flag<true>{}, Flag<true>{});
    if (k + 1 < KT) { k_step(k, Flag<false>{}, Flag<true>{}); k++; }
    k_step(k, Flag<false>{}, Flag<false>{});

    // ---- + C, -> C: through a per-wavefront transposing buffer in LDS (nobody reads A / B
    // stages any more: every wavefront passed the last barrier after its last read), so that C
    // is read and written as whole 256-byte row segments, 16 bytes (8 for f16 C) per lane ----
    typedef typename CVec4<CT>::type ctx4;
    constexpr int PITCH = 16 * 16 + 16;                       // 272 B
    constexpr int PASSES = 8;                                 // 4 rows per pass, 32 rows per slab
    const uint32_t tbuf = smem_base + (uint32_t)wave * (32u * PITCH);
    const uint32_t w_addr = tbuf + (uint32_t)(lane & 15) * PITCH + (uint32_t)(lane >> 4) * 16;
    const uint32_t r_addr = tbuf + (uint32_t)(lane >> 4) * PITCH + (uint32_t)(lane & 15) * 16;
    const int orow = lane >> 4, ocol = 4 * (lane & 15);
    const int crow0 = m0 + grp * HM, ccol0 = n0 + wn * WN;
    const bool col_ok = !edge || (ccol0 + ocol < p.N);        // N is a multiple of 8: all 4 columns or none
    CT* const Cbase = (CT*)p.C;
    CT* const cptr = Cbase + (int64_t)(crow0 + orow) * p.ldc + ccol0 + ocol;
    float bias4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (p.bias && col_ok) {
#pragma unroll
        for (int e = 0; e < 4; e++) bias4[e] = (float)reinterpret_cast<const CT*>(p.bias)[ccol0 + ocol + e];
    }
    ctx4 cin[2][PASSES];
    auto fetch = [&](int slab, ctx4 (&dst)[PASSES]) {
#pragma unroll
        for (int ps = 0; ps < PASSES; ps++) {
            const bool ok = col_ok && (!edge || (crow0 + slab * 32 + 4 * ps + orow < p.M));
            const CT* src = ok ? cptr + (int64_t)(slab * 32 + 4 * ps) * p.ldc : Cbase + (int64_t)m0 * p.ldc + n0;
            dst[ps] = *reinterpret_cast<const ctx4*>(src);
        }
    };
    fetch(0, cin[0]);
#pragma unroll
    for (int slab = 0; slab < HM / 32; slab++) {
        if (slab + 1 < HM / 32) fetch(slab + 1, cin[(slab + 1) & 1]);
#pragma unroll
        for (int r = 0; r < 2; r++)
#pragma unroll
            for (int fn = 0; fn < 4; fn++)
                *(__attribute__((address_space(3))) floatx4*)(uintptr_t)(w_addr + r * 16 * PITCH + fn * 16 * 4) = acc[2 * slab + r][fn];
#pragma unroll
        for (int ps = 0; ps < PASSES; ps++) {
            const floatx4 s4 = *(__attribute__((address_space(3))) const floatx4*)(uintptr_t)(r_addr + 4 * ps * PITCH);
            const ctx4 c4 = cin[slab & 1][ps];
            ctx4 o;
#pragma unroll
            for (int e = 0; e < 4; e++) o[e] = (CT)epilogue_value(s4[e] + (float)c4[e], bias4[e], p.relu);   // f16: one rounding, to nearest even
            if (col_ok && (!edge || (crow0 + slab * 32 + 4 * ps + orow < p.M)))
                *reinterpret_cast<ctx4*>(cptr + (int64_t)(slab * 32 + 4 * ps) * p.ldc) = o;
        }
    }
}

template <typename CT>
__global__ __launch_bounds__(512) void gemm_il256_kernel(const TiledParams p)
{
    __shared__ __attribute__((aligned(1024))) char smem[IL_LDS];
    int tile_m, tile_n;
    tile_of_block(p, blockIdx.x, tile_m, tile_n);
    il_tile<CT>(p, (uint32_t)(uintptr_t)(lds_ptr_t)smem, tile_m * IL_BM, tile_n * IL_BN);
}

int64_t grid_il(int64_t M, int64_t N)
{
    const int64_t tm = (M + IL_BM - 1) / IL_BM, tn = (N + IL_BN - 1) / IL_BN;
    if (tm > 0 && tn > INT32_MAX / tm) return -1;
    return tm * tn;
}

int launch_il(const GemmArgs& a)
{
    if (a.K % BK != 0) return pingpong16_config(256, 256)->launch(a);     // k tails: the phase-alternating kernel
    const int64_t g = grid_il(a.M, a.N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    TiledParams p = make_tiled_params(a, IL_BM, IL_BN, 8);
    if (a.c_is_f16) hipLaunchKernelGGL((gemm_il256_kernel<half_t>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
    else            hipLaunchKernelGGL((gemm_il256_kernel<float>), dim3((unsigned)g), dim3(512), 0, a.stream, p);
    return hipGetLastError() == hipSuccess ? GEMM_F16_OK : GEMM_F16_ERR_LAUNCH;
}

const GemmConfigDesc kInterleaved = {
    "il256x256x64_w2x4_mi16", IL_BM, IL_BN, BK, 8, 128, 64, IL_LDS, true, launch_il, grid_il};

}  // namespace

const GemmConfigDesc* interleaved_config() { return &kInterleaved; }
