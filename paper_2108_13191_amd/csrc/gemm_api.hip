// The C ABI of the library (include/gemm_f16.h): argument checks, choice of a
// kernel configuration, launch on the caller's stream.  No allocation, no
// synchronisation.
#include "gemm_common.h"
#include "../../include/gemm_f16.h"
#include <string.h>

namespace {

// Configuration table.  The product library holds the any-shape kernel, the phase-alternating
// eight-wavefront kernel (16x16x32 MFMA) in its five tile shapes and its two launch forms for
// several tiles per compute unit (chained, staggered), and the plain ring-buffered 64 x 64 tiling
// for the smallest problems.  A ladder build (GEMM_F16_LADDER, libgemm_f16_ladder.so) appends
// the comparison kernels and ablation rows behind them; the selector never picks those.
enum {
    ID_GENERIC = 0,
    ID_PP256,          // 256 x 256
    ID_PP192,          // 192 x 256
    ID_PP128,          // 128 x 256
    ID_PP256x192,      // 256 x 192
    ID_PP128x128,      // 128 x 128, two workgroups per compute unit
    ID_CHAIN,          // 256 x 256, one workgroup per compute unit walks its tiles
    ID_STAG,           // 256 x 256, every other compute unit starts on half a tile
    ID_T64,            // 64 x 64, four LDS stages
    ID_LONG_K,         // 256 x 256, four wavefronts of 128 x 128, k loop in assembly
    ID_RING128,        // 128 x 128, four wavefronts of 64 x 64, k loop in assembly over five LDS stages
    NUM_PRODUCT
};

const GemmConfigDesc kGeneric = {
    "generic64x64x32", 64, 64, 32, 4, 32, 32, 2 * 64 * (32 + 8) * 2,
    false, launch_generic, grid_generic};

#ifdef GEMM_F16_LADDER
constexpr int NUM_LADDER = 12;
#else
constexpr int NUM_LADDER = 0;
#endif
int num_configs() { return NUM_PRODUCT + NUM_LADDER; }

const GemmConfigDesc* config(int id)
{
    switch (id) {
    case ID_GENERIC:   return &kGeneric;
    case ID_PP256:     return pingpong16_config(256, 256);
    case ID_PP192:     return pingpong16_config(192, 256);
    case ID_PP128:     return pingpong16_config(128, 256);
    case ID_PP256x192: return pingpong16_config(256, 192);
    case ID_PP128x128: return pingpong16_config(128, 128);
    case ID_CHAIN:     return pingpong16_persistent_config();
    case ID_STAG:      return pingpong16_staggered_config();
    case ID_T64:       return tiled_config(64);
    case ID_LONG_K:    return long_k_config();
    case ID_RING128:   return deep_ring_config();
#ifdef GEMM_F16_LADDER
    case NUM_PRODUCT + 0: return tiled_config(128);
    case NUM_PRODUCT + 1: return tiled_config(256);
    case NUM_PRODUCT + 2: return tiled_no_swizzle_config();
    case NUM_PRODUCT + 3: return pingpong_config();
    case NUM_PRODUCT + 4: return pingpong16_no_xcd_order_config();
    case NUM_PRODUCT + 5: return w4_config();
    case NUM_PRODUCT + 6: return overlap_config();
    case NUM_PRODUCT + 7: return interleaved_config();
    case NUM_PRODUCT + 8: return generic_c_in_loop_config();
    case NUM_PRODUCT + 9: return generic_round_per_slice_config();
    case NUM_PRODUCT + 10: return pingpong16_192x192_config();
    case NUM_PRODUCT + 11: return pingpong16_rowwise_config();
#endif
    default: return &kGeneric;
    }
}

int g_forced = -1;

}  // namespace

const ChipShape& chip()
{
    static const ChipShape shape = [] {
        ChipShape c = {256, 8, 100000};
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess) {
            if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) {
                c.cus = v;
                c.xcds = v >= 32 ? v / 32 : 1;
            }
            if (hipDeviceGetAttribute(&v, hipDeviceAttributeWallClockRate, dev) == hipSuccess && v > 0) c.wall_clock_khz = v;
        }
        return c;
    }();
    return shape;
}

namespace {

int check_args(int c_is_f16, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
               const void* B, int64_t ldb, const void* C, int64_t ldc)
{
    const int64_t lim = INT32_MAX;
    if (M < 0 || N < 0 || K < 0 || M > lim || N > lim || K > lim) return GEMM_F16_ERR_SIZE;
    if (lda < K || ldb < N || ldc < N || lda > lim || ldb > lim || ldc > lim) return GEMM_F16_ERR_PITCH;
    if (M == 0 || N == 0) return GEMM_F16_OK;
    if (!C) return GEMM_F16_ERR_NULL;
    if (K > 0 && (!A || !B)) return GEMM_F16_ERR_NULL;
    if (((uintptr_t)A & 1) || ((uintptr_t)B & 1) || ((uintptr_t)C & (c_is_f16 ? 1 : 3))) return GEMM_F16_ERR_ALIGN;
    return GEMM_F16_OK;
}

// Pitches above this take the any-shape kernel, whose addresses are all 64-bit: the tuned
// kernels keep tile-relative byte offsets of A and B (up to 256 rows) in 32 bits, and the
// plain tilings (64 x 64 and the ladder's larger ones) do the same for C.
constexpr int64_t MAX_TUNED_PITCH = 1 << 22;

bool aligned_for_tiled(int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, int64_t ldc)
{
    return ((uintptr_t)A % 16 == 0) && ((uintptr_t)B % 16 == 0) && lda % 8 == 0 && ldb % 8 == 0 &&
           K % 8 == 0 && N % 8 == 0 && K >= 8 &&
           lda <= MAX_TUNED_PITCH && ldb <= MAX_TUNED_PITCH && ldc <= MAX_TUNED_PITCH;
}

// What a call runs: one configuration on all rows, or the 256 x 256 kernel on
// the first rows1 rows and configuration id2 on the rest (second launch on the
// same stream; the row ranges of C are disjoint); k_split > 1: one launch whose
// workgroups each take a part of the k loop of a tile.
struct Plan { int id; int64_t rows1; int id2; int k_split = 0; };

struct Cand { int id; double eff; int per_cu; };
// The 192- and 128-row forms reuse operands less per tile, but e.g. 6144^3 is exactly three
// rounds of 192 x 256 tiles instead of 2.25 of 256 x 256.  The 128 x 128 form runs two
// workgroups per compute unit, which hide each other's prologue and epilogue: the choice for
// problems of a few hundred tiles.  256 x 192 serves N = 768 and the like.  eff = measured
// throughput per unit of tile area relative to the 256 x 256 tile, over whole rounds.
const Cand kCands[] = {{ID_PP256, 1.0, 1}, {ID_PP192, 0.95, 1}, {ID_PP128, 0.85, 1}, {ID_PP256x192, 0.9, 1},
                       {ID_PP128x128, 0.9, 2}, {ID_T64, 0.4, 4}};

// Estimated time of one launch in units of tile area: the rounds the grid needs
// on the device's compute units times the work of one tile, divided by the
// configuration's efficiency (large tiles reuse operands better; small tiles
// fill the chip on small problems -- the trade-off the paper reports in
// section Mixed Precision Performance).  Behind at least one full round, a partial round of
// the one-workgroup-per-unit kernels costs half a round plus half its fill (a problem of less
// than one round pays a whole one, unless it is the second launch of a split: alone it is
// bound by latencies, not by power): the part runs at its power limit, and
// compute units that idle leave their share to the clock of the others (measured on 25
// problems of 100 to 1600 tiles of 256 x 256, in rounds of that tile: 16 tiles left over
// +0.55, 64 +0.6 ... 0.7, 128 +0.8 ... 0.9, 228 +0.9; counting a partial round as a full one
// chose a plan 6 to 10 % slower than the best on 4608^3, 3072 x 8192 x 4096, 6144 x 4096 x
// 2048, 8192 x 2560 x 8192).  With several workgroups per unit, those which would share a
// compute unit and do not have to (the last round has fewer than 256 x per_cu of them) run
// somewhat faster.
// The 128 x 128 form's two workgroups per compute unit hide each other's
// prologue and epilogue, which counts for more the shorter the k loop is.
// The 64 x 64 tiling moves f16 C two bytes per lane: on problems of 512^2 results and more with
// k loops up to 2048 its f16 mode falls behind the 128 x 128 form (measured 25 / 62 / 78 / 123
// against 29 / 75 / 104 / 146 TFLOP/s at 512^3, 768^3, 1024^2 x 512, 1024^3; in f32 mode, and at
// K = 4096 in both, it stays ahead).
double launch_cost(const Cand& c, int c_is_f16, int64_t M, int64_t N, int64_t K, bool behind_full_rounds)
{
    const GemmConfigDesc* d = config(c.id);
    const int64_t g = d->grid(M, N);
    if (g < 0) return -1.0;
    double eff = c.eff;
    if (c.id == ID_PP128x128) { eff = 0.78 + 0.2 * (K < 1024 ? 1.0 : 1024.0 / (double)K); if (eff > 0.92) eff = 0.92; }
    if (c.id == ID_T64 && c_is_f16 && K <= 2048 && M * N >= 512 * 512) eff *= 0.75;
    const int64_t cus = chip().cus, slots = cus * c.per_cu;
    const int64_t full = g / slots, left = g % slots;
    const double sharing = (double)((left + cus - 1) / cus);                   // workgroups per compute unit in the last round
    const double last = !left ? 0.0 : (c.per_cu == 1 && (full >= 1 || behind_full_rounds)) ? 0.5 + 0.5 * (double)left / (double)cus
                                                                   : (0.5 + 0.5 * sharing / c.per_cu) * c.per_cu;
    return ((double)full * c.per_cu + last) * (double)d->block_m * d->block_n / eff;
}

int best_single(int c_is_f16, int64_t M, int64_t N, int64_t K, double* cost_out, bool behind_full_rounds = false)
{
    int best = ID_PP256;
    double best_cost = -1.0;
    for (const Cand& c : kCands) {
        const double cost = launch_cost(c, c_is_f16, M, N, K, behind_full_rounds);
        if (cost < 0) continue;
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = c.id; }
    }
    *cost_out = best_cost;
    return best;
}

// Pick the plan with the lowest estimated time.  Besides the single launches,
// the rows are cut once: whole rounds of 256 x 256 tiles first, and whatever
// configuration suits the left-over rows best behind them -- 5120^3 is one full
// round of 256 x 256 tiles plus one round of 192 x 256 tiles instead of two
// rounds of which the second is 56 % full.
int id_chained() { return ID_CHAIN; }
int id_staggered() { return ID_STAG; }

// The 256 x 256 tiling runs chained when a compute unit gets more than one tile
// (measured 1-5 % faster, more the shorter the k loop; the k-tail form is not:
// it needs a few registers more than there are).
int chained_if_it_pays(int id, int64_t rows, int64_t N, int64_t K)
{
    if (id != ID_PP256 || K % 64 != 0) return id;
    const GemmConfigDesc* c = config(id_chained());
    return c->grid(rows, N) < config(ID_PP256)->grid(rows, N) ? id_chained() : id;
}

// Long k loops take the four-wavefront kernel, and so do f32 problems of at most one 256 x 256
// tile per compute unit: there nothing else hides the read of C, which that kernel does inside
// its k loop (from 36 k steps on).  Measured against the plain / chained 256 x 256 form, all
// alternating in one process at the steady state (f32 / f16 mode): K = 16384: 16384^3 +3.5 ...
// +4.4 / +2.5 %, 8192^2 +1.3 ... +4 / +2 ... +4 %, 6144 x 8192 +2 / +2 %; K = 12288: 12288^3
// +1 ... +5 / +2 %, 16384^2 +1 ... +1.7 / +1 %, 8192 x 16384 0 %, 8192^2 -1 / 0 %; K = 8192:
// 4096^2 (one tile per compute unit) +5 / +0.5 %, 4096 x 8192 (two) +2 / 0 %, 8192^2 -0.5 ... -1 %,
// 12288^2 -1 ... -2 %, 16384^2 0 %; one tile per compute unit, K = 6144 / 4096 / 3072 / 2304: +6.5,
// +8, +8, +10 % in f32 mode (3840 x 4096 x 4096, 240 tiles: +5 %; ragged 4000 x 4000 x 4096 +2.5 %,
// 3900 x 4000 x 3072 +2 %: edge tiles read and store C through range-checked buffer accesses),
// -2 ... -9 % in f16 mode (C read behind the loop); K = 2048 (no C in the loop): -10 %; two tiles
// per compute unit, K = 4096 / 6144: -2 / 0 % (f16 -5 / -2 %).
int long_k_if_it_pays(int id, int c_is_f16, int64_t rows, int64_t N, int64_t K)
{
    if (id != ID_PP256 && id != ID_CHAIN) return id;
    const int64_t tiles = config(ID_PP256)->grid(rows, N), cus = chip().cus;
    // (a k tail is an unpipelined step behind that kernel's loop: 4000^3 +1 %, left where it was)
    const bool pays = K >= 12288 || (K >= 8192 && tiles <= 2 * cus) || (!c_is_f16 && K >= 2304 && K % 64 == 0 && tiles <= cus);
    return pays ? ID_LONG_K : id;
}

// At most one 128 x 128 tile per compute unit and 96 or more k steps: the four-wavefront kernel
// with five LDS stages.  A k step of such a tile is a quarter of a microsecond of MFMAs, less
// than a copy's way from L2, which the phase-alternating kernel's two or three buffers cannot
// cover (0.6 us per k step against 0.42 on a full chip, 0.30 on a quarter of it); that kernel
// in turn starts and ends sooner (80 KB of LDS: the next launch's workgroups start beside the
// last one's).  Measured, alternating in one process on the same operands (they stay in the
// last-level cache), f32 / f16 mode: 2048^2, K = 2048: -6 / -2 %, 3072: +3 / +4 %, 4096: +8 /
// +9 %, 8192: +22 / +21 %; 1536^2 x 3072 +13 / +16 %, 1024 x 2048 x 4096 +22 / +23 %, 1280^2 x
// 5120 +14 / +15 %, ragged 2000^2 x 4096 +5 / +8 %; the strips behind a split: 256 x 7168^2
// +25 / +28 %, 256 x 9216^2 +26 / +27 %, 256 x 15360^2 (bound by the read of B) 0 %.  More than
// one tile per compute unit (2048 x 4096 x 4096, 2560^2 x 4096): -7 ... -9 %.  With operand
// sets rotating so that every launch reads A and B from HBM its k step is 0.50 us against
// 0.56, but its start costs 5 us more: 2048^2, K = 3072: -8 / -4 %, 4096: -3 / 0 %, 6144: -3 /
// -0.5 %, 8192: +3 / +5 %; 1536^2 x 3072 -6 / -5 %; 256 x 7168^2 -3 %.  From K = 6144 on what
// it gains on cached operands (+15 % and more) outweighs what it loses on cold ones.
int deep_ring_if_it_pays(int id, int64_t rows, int64_t N, int64_t K)
{
    if (id != ID_PP128x128) return id;
    return (K >= 6144 && config(ID_RING128)->grid(rows, N) <= chip().cus) ? ID_RING128 : id;
}

Plan select_plan_unchained(int c_is_f16, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, int64_t ldc)
{
    if (!aligned_for_tiled(N, K, A, lda, B, ldb, ldc)) return {ID_GENERIC, M, -1};
    if (g_forced >= 0 && g_forced < num_configs()) return {g_forced, M, -1};
    double cost = 0;
    Plan best = {best_single(c_is_f16, M, N, K, &cost), M, -1};
    const int64_t tiles_m = (M + 255) / 256, tiles_n = (N + 255) / 256, cus = chip().cus;
    if (tiles_n > cus || tiles_m < 2 || cost < 0) return best;
    // Short k loops, two or more full rounds of 256 x 256 tiles and a last round at
    // most half full: the staggered form fills that round with half tiles (and
    // spreads the C traffic, which dominates such problems, over time).  With long
    // k loops the two halves of the chip would no longer share operand panels in L2.
    // Such problems are bound by the traffic of C, and no plan of two launches is tried for
    // them: (16384,2304,768) 80 us against 84 ... 87 on 256 x 192 tiles (three whole rounds),
    // 90 chained, 86 for a row split.
    {
        const int64_t tiles = tiles_m * tiles_n, full = tiles / cus, left = tiles % cus;
        const double staggered = ((double)full + 0.4) * 65536.0;
        if (cus == 256 && K <= 1024 && full >= 2 && left > 0 && left <= 128 && staggered < cost) return {id_staggered(), M, -1};
    }
    const double second_launch = 3000.0;                  // drain and refill between the two launches
    const int64_t total_rounds = (tiles_m * tiles_n + cus - 1) / cus;
    for (int64_t r = total_rounds > 4 ? total_rounds - 3 : 1; r <= total_rounds; r++) {   // the cut is near the end
        const int64_t j = (r * cus) / tiles_n;             // tile rows that fit r rounds
        if (j < 1 || j >= tiles_m) continue;
        double rest = 0;
        const int id2 = best_single(c_is_f16, M - 256 * j, N, K, &rest, true);
        const int64_t t1 = j * tiles_n;                     // tiles of the first launch: whole rounds and a partial one, as in launch_cost
        const double first = ((double)(t1 / cus) + (t1 % cus ? 0.5 + 0.5 * (double)(t1 % cus) / (double)cus : 0.0)) * 65536.0;
        if (rest >= 0 && first + rest + second_launch < cost) { cost = first + rest + second_launch; best = {ID_PP256, 256 * j, id2}; }
    }
    return best;
}

// Few tiles and a long k loop (skinny problems: a few hundred rows, or few columns, against K
// and the other dimension in the thousands): the time goes into streaming the larger operand,
// and a compute unit streams at most the bytes it holds in flight per memory latency (about
// 50 GB/s), so that 64 tiles on 64 compute units reach a fifth of the memory's rate.  In f32
// mode the k loop is cut so that every compute unit gets a part: workgroups of the five-stage
// 128 x 128 kernel, one per tile and part of at least 16 k steps (and no more parts than keep
// the additions under four million), which add their sums to C with atomic f32 additions (C holds the old C; no fused epilogue, which would have to follow
// the last part; f16 C would be rounded once per part: both run unsplit).  The order of the
// additions is not fixed, so results may differ in the last bit from run to run.
int k_split_if_it_pays(int& id, int c_is_f16, int64_t M, int64_t N, int64_t K)
{
    if (c_is_f16 || (id != ID_RING128 && id != ID_PP128x128 && id != ID_T64 && id != ID_PP128)) return 0;
    const int64_t tiles = config(ID_RING128)->grid(M, N), cus = chip().cus, steps = (K + 63) / 64;
    if (tiles <= 0 || 2 * tiles > cus) return 0;
    int64_t parts = cus / tiles < steps / 16 ? cus / tiles : steps / 16;
    if (parts > 16) parts = 16;
    // the additions: M x N per part, a row of 64 floats per instruction, about 5 us per million;
    // measured with at most 4 million of them (before -> after): (64,8192,8192) 49 -> 30 us,
    // (128,8192,8192) 52 -> 37, (256,8192,8192) 54 -> 45, (1024,2048,8192) 57 -> 47,
    // (512,4096,4096) 31 -> 32
    if (parts * M * N > 4194304) parts = 4194304 / (M * N);
    if (parts < 2) return 0;
    id = ID_RING128;
    return (int)parts;
}

Plan select_plan(int c_is_f16, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, int64_t ldc)
{
    Plan pl = select_plan_unchained(c_is_f16, M, N, K, A, lda, B, ldb, ldc);
    if (g_forced >= 0 && g_forced < num_configs()) return pl;        // a forced configuration runs as it is
    pl.id = long_k_if_it_pays(chained_if_it_pays(pl.id, pl.rows1, N, K), c_is_f16, pl.rows1, N, K);
    pl.id = deep_ring_if_it_pays(pl.id, pl.rows1, N, K);
    if (pl.id2 >= 0) pl.id2 = long_k_if_it_pays(chained_if_it_pays(pl.id2, M - pl.rows1, N, K), c_is_f16, M - pl.rows1, N, K);
    if (pl.id2 >= 0) pl.id2 = deep_ring_if_it_pays(pl.id2, M - pl.rows1, N, K);
    if (pl.id2 < 0 && pl.rows1 == M) pl.k_split = k_split_if_it_pays(pl.id, c_is_f16, M, N, K);
    return pl;
}

void fill_desc(int id, int64_t grid, gemm_f16_config* out, int64_t split_rows = 0, int id2 = -1)
{
    const GemmConfigDesc* d = config(id);
    memset(out, 0, sizeof(*out));
    out->id = id; out->block_m = d->block_m; out->block_n = d->block_n; out->block_k = d->block_k;
    out->waves = d->waves; out->wave_m = d->wave_m; out->wave_n = d->wave_n; out->lds_bytes = d->lds_bytes;
    out->grid = grid;
    out->split_rows = (int32_t)split_rows;
    out->id2 = id2;
    strncpy(out->name, d->name, sizeof(out->name) - 1);
}

int run(int c_is_f16, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
        const void* B, int64_t ldb, void* C, int64_t ldc, void* stream,
        const void* bias = nullptr, int act = GEMM_F16_ACT_NONE)
{
    const int rc = check_args(c_is_f16, M, N, K, A, lda, B, ldb, C, ldc);
    if (rc != GEMM_F16_OK) return rc;
    if (act != GEMM_F16_ACT_NONE && act != GEMM_F16_ACT_RELU) return GEMM_F16_ERR_CONFIG;
    if ((uintptr_t)bias & (c_is_f16 ? 1 : 3)) return GEMM_F16_ERR_ALIGN;
    if (M == 0 || N == 0) return GEMM_F16_OK;
    const bool fused = bias != nullptr || act != GEMM_F16_ACT_NONE;
    if (K == 0 && !fused) return GEMM_F16_OK;             // C + empty sum = C
    GemmArgs a;
    a.bias = bias; a.relu = act == GEMM_F16_ACT_RELU;
    if (K == 0) {
        // the epilogue alone: the any-shape kernel with an empty k loop (it never touches A or B then)
        a.M = M; a.N = N; a.K = 0;
        a.A = (const half_t*)A; a.lda = lda; a.B = (const half_t*)B; a.ldb = ldb; a.C = C; a.ldc = ldc;
        a.c_is_f16 = c_is_f16; a.stream = (hipStream_t)stream;
        return config(ID_GENERIC)->launch(a);
    }
    const Plan plan = select_plan(c_is_f16, M, N, K, A, lda, B, ldb, ldc);
    a.M = plan.rows1; a.N = N; a.K = K;
    a.A = (const half_t*)A; a.lda = lda; a.B = (const half_t*)B; a.ldb = ldb; a.C = C; a.ldc = ldc;
    a.c_is_f16 = c_is_f16; a.stream = (hipStream_t)stream;
    a.k_split = fused ? 0 : plan.k_split;                   // a fused epilogue has to follow the whole sum
    const int rc1 = config(plan.id)->launch(a);
    if (rc1 != GEMM_F16_OK || plan.rows1 == M) return rc1;
    a.k_split = 0;
    a.M = M - plan.rows1;                                   // the left-over rows: A and C move down, B stays
    a.A = (const half_t*)A + plan.rows1 * lda;
    a.C = (char*)C + plan.rows1 * ldc * (c_is_f16 ? 2 : 4);
    return config(plan.id2)->launch(a);
}

// Parts of a split k loop for the half-precision mode through a workspace (0: runs unsplit):
// the rule of the f32 mode on the plan the f16 mode would take.
int f16_workspace_parts(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, int64_t ldc)
{
    if (M <= 0 || N <= 0 || K <= 0 || !aligned_for_tiled(N, K, A, lda, B, ldb, ldc) || (g_forced >= 0 && g_forced < num_configs())) return 0;
    const Plan pl = select_plan(1, M, N, K, A, lda, B, ldb, ldc);
    if (pl.id2 >= 0 || pl.rows1 != M) return 0;
    // the two passes over the workspace: (1024,2048,8192), 8 MB, 56 us against 53 unsplit; (256,4096,16384), 4 MB, 52 against 97
    if (M * N > 1048576) return 0;
    int id = pl.id;
    return k_split_if_it_pays(id, 0, M, N, K);
}

// The half-precision mode with `ws` (M x N floats, 16-byte aligned, all zero if ws_is_zero) as the
// f32 sum of the parts; clear_after: leave it all zero again.
int run_f16_split(int parts, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb,
                  void* C, int64_t ldc, float* ws, bool ws_is_zero, bool clear_after, void* stream)
{
    int rc = ws_is_zero ? GEMM_F16_OK : splitk_f16_zero(ws, M * N, (hipStream_t)stream);   // N is a multiple of 8
    if (rc != GEMM_F16_OK) return rc;
    GemmArgs a;
    a.M = M; a.N = N; a.K = K;
    a.A = (const half_t*)A; a.lda = lda; a.B = (const half_t*)B; a.ldb = ldb; a.C = ws; a.ldc = N;
    a.c_is_f16 = 0; a.stream = (hipStream_t)stream; a.bias = nullptr; a.relu = 0; a.k_split = parts;
    rc = config(ID_RING128)->launch(a);
    if (rc != GEMM_F16_OK) return rc;
    return splitk_f16_finish(ws, C, ldc, M, N, clear_after ? 1 : 0, (hipStream_t)stream);
}

}  // namespace

extern "C" {

int64_t gemm_f16_f16acc_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0 || M > INT32_MAX || N > INT32_MAX || K > INT32_MAX) return 0;
    return f16_workspace_parts(M, N, K, (const void*)16, K, (const void*)16, N, N) >= 2 ? M * N * 4 : 0;
}

int gemm_f16_f16acc_workspace(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                              const void* B, int64_t ldb, void* C, int64_t ldc,
                              void* workspace, int64_t workspace_bytes, void* stream)
{
    const int rc = check_args(1, M, N, K, A, lda, B, ldb, C, ldc);
    if (rc != GEMM_F16_OK) return rc;
    if (workspace && ((uintptr_t)workspace & 15)) return GEMM_F16_ERR_ALIGN;
    const int parts = f16_workspace_parts(M, N, K, A, lda, B, ldb, ldc);
    if (parts < 2 || !workspace || workspace_bytes < M * N * 4) return run(1, M, N, K, A, lda, B, ldb, C, ldc, stream);
    return run_f16_split(parts, M, N, K, A, lda, B, ldb, C, ldc, (float*)workspace, false, false, stream);
}

int gemm_f16_f32acc(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                    const void* B, int64_t ldb, float* C, int64_t ldc, void* stream)
{
    return run(0, M, N, K, A, lda, B, ldb, C, ldc, stream);
}

int gemm_f16_f16acc(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                    const void* B, int64_t ldb, void* C, int64_t ldc, void* stream)
{
    return run(1, M, N, K, A, lda, B, ldb, C, ldc, stream);
}

int gemm_f16_f32acc_bias_act(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                             const void* B, int64_t ldb, float* C, int64_t ldc,
                             const float* bias, int act, void* stream)
{
    return run(0, M, N, K, A, lda, B, ldb, C, ldc, stream, bias, act);
}

int gemm_f16_f16acc_bias_act(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                             const void* B, int64_t ldb, void* C, int64_t ldc,
                             const void* bias, int act, void* stream)
{
    return run(1, M, N, K, A, lda, B, ldb, C, ldc, stream, bias, act);
}

int gemm_f16_f16acc_static_workspace(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                                     const void* B, int64_t ldb, void* C, int64_t ldc, void* stream)
{
    const int rc = check_args(1, M, N, K, A, lda, B, ldb, C, ldc);
    if (rc != GEMM_F16_OK) return rc;
    const int parts = f16_workspace_parts(M, N, K, A, lda, B, ldb, ldc);
    if (parts < 2) return run(1, M, N, K, A, lda, B, ldb, C, ldc, stream);      // no scratch memory involved
    float* ws = nullptr;
    int64_t floats = 0;
    const int rc2 = splitk_f16_static_scratch(&ws, &floats);
    if (rc2 != GEMM_F16_OK) return rc2;
    if (M * N > floats) return GEMM_F16_ERR_WORKSPACE;
    return run_f16_split(parts, M, N, K, A, lda, B, ldb, C, ldc, ws, false, false, stream);
}

const char* gemm_strerror(int code)
{
    switch (code) {
    case GEMM_F16_OK: return "success";
    case GEMM_F16_ERR_SIZE: return "a dimension is negative or too large";
    case GEMM_F16_ERR_PITCH: return "a leading dimension is smaller than the row length or too large";
    case GEMM_F16_ERR_NULL: return "a required pointer is NULL";
    case GEMM_F16_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    case GEMM_F16_ERR_CONFIG: return "unknown configuration id, activation or bad query argument";
    case GEMM_F16_ERR_ALIGN: return "a pointer is not aligned to its element size";
    case GEMM_F16_ERR_WORKSPACE: return "the problem needs more scratch memory than the library holds (use gemm_f16_f16acc_workspace or gemm_f16_f16acc)";
    default: return "unknown error code";
    }
}

int gemm_f16_query_config(int c_is_f16, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                          const void* B, int64_t ldb, const void* C, int64_t ldc, gemm_f16_config* out)
{
    if (!out) return GEMM_F16_ERR_CONFIG;
    // pointers are inspected for alignment only; stand-ins for NULL keep the checks uniform
    const void* a = A ? A : (const void*)16;
    const void* b = B ? B : (const void*)16;
    const void* c = C ? C : (const void*)16;
    const int rc = check_args(c_is_f16, M, N, K, a, lda, b, ldb, c, ldc);
    if (rc != GEMM_F16_OK) return rc;
    const Plan plan = select_plan(c_is_f16, M, N, K, a, lda, b, ldb, ldc);
    if (M == 0 || N == 0 || K == 0) { fill_desc(plan.id, 0, out); return GEMM_F16_OK; }
    int64_t g = config(plan.id)->grid(plan.rows1, N);
    if (g < 0) return GEMM_F16_ERR_SIZE;
    if (plan.rows1 < M) {
        const int64_t g2 = config(plan.id2)->grid(M - plan.rows1, N);
        if (g2 < 0) return GEMM_F16_ERR_SIZE;
        g += g2;
    }
    if (plan.k_split > 1) g *= plan.k_split;               // one workgroup per tile and part of the k loop
    fill_desc(plan.id, g, out, plan.rows1 < M ? plan.rows1 : 0, plan.rows1 < M ? plan.id2 : -1);
    return GEMM_F16_OK;
}

int gemm_f16_num_configs(void) { return num_configs(); }

int gemm_f16_describe_config(int id, gemm_f16_config* out)
{
    if (!out || id < 0 || id >= num_configs()) return GEMM_F16_ERR_CONFIG;
    fill_desc(id, 0, out);
    return GEMM_F16_OK;
}

int gemm_f16_force_config(int id)
{
    if (id >= num_configs()) return GEMM_F16_ERR_CONFIG;
    g_forced = id < 0 ? -1 : id;
    return GEMM_F16_OK;
}

}  // extern "C"
