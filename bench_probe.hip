// Measurement aid of bench.py, not part of the GEMM library: what the matrix units sustain when
// NOTHING but MFMAs runs (operands stay in registers: no LDS, no memory traffic), on operand
// DATA handed in by the caller.  Under a dense MFMA load the part is power-limited and the limit
// depends on how much the operands toggle (all-zero operands: 2.4 PFLOP/s; the benchmark's
// N(0,1)/sqrt(K) operands: about 1.85 PFLOP/s), so a GEMM's throughput on given data has to be
// read against this figure measured on the same data, in the same run.
//
// One workgroup per compute unit, 8 wavefronts (two per SIMD: one wavefront alone leaves issue
// gaps), each with the register blocking of the library's large-tile kernel: 8 A fragments x 4 B
// fragments -> 8 x 4 accumulators of v_mfma_f32_16x16x32_f16, 32 MFMAs per iteration, issued in
// the order the library's kernels use (two rows of blocks at a time, down, right, up, right:
// one operand changes from one MFMA to the next; column by column this loop is 2.5 % slower, the
// operands' changes are part of what the matrix units draw).
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

__global__ __launch_bounds__(512) void mfma_only_kernel(const half8* __restrict__ frags, float* __restrict__ sink, int iters)
{
    // 12 fragments of 256 lanes x 16 bytes: 8 for A, 4 for B; wavefront w and w + 4 (which share a SIMD) use the same
    half8 a[8], b[4];
    const int t = threadIdx.x & 255;
#pragma unroll
    for (int i = 0; i < 8; i++) a[i] = frags[i * 256 + t];
#pragma unroll
    for (int j = 0; j < 4; j++) b[j] = frags[(8 + j) * 256 + t];
    floatx4 c[8][4];
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) c[i][j] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int n = 0; n < 32; n++) {
            const int pr = n / 8, q = n % 8;
            const int i = 2 * pr + ((q % 4 == 1 || q % 4 == 2) ? 1 : 0), j = (pr & 1) ? 3 - q / 2 : q / 2;
            c[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(b[j], a[i], c[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);           // in this order
        }
        asm volatile("" : "+v"(a[0]), "+v"(b[0]));       // the loop body is not hoisted or merged across iterations
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) s += c[i][j][0] + c[i][j][1] + c[i][j][2] + c[i][j][3];
    if (s == 12345.678f) sink[0] = s;                     // keeps the accumulators alive; practically never taken
}

// ---- the loop budget: what the main loop of a GEMM costs beyond its MFMAs -----------------------
// Three loops with the register blocking above, hand-scheduled in assembly on fixed registers so
// that nothing but the named ingredient differs (a compiler-scheduled loop adds waits and address
// arithmetic of its own): (0) the 32 MFMAs of half a k step alone; (1) plus the LDS fragment
// reads that feed them in the library's kernels (8 ds_read_b128 + 8 ds_read_b64_tr_b16 per
// wavefront, data discarded); (2) plus the wavefront's share of the global -> LDS copies (4 x 1 KB
// by global_load_lds_dwordx4 from a 32 KB region that stays in L2).  The MFMA operands and the LDS
// contents come from the caller's data, so the three figures show, on the workload's own operand
// distribution, what the LDS reads and the copies take from the matrix units -- in issue and
// register-port time and, the part being power-limited, in energy.
// Registers: v[0:31] A fragments, v[34:49] B fragments, v[64:191] accumulators, v[200:215] read
// targets, v230 / v231 LDS read addresses, v232 the lane's copy offset.
#define MFMA(c0, c1, b0, b1, a0, a1) "v_mfma_f32_16x16x32_f16 v[" #c0 ":" #c1 "], v[" #b0 ":" #b1 "], v[" #a0 ":" #a1 "], v[" #c0 ":" #c1 "]\n\t"
// (the 32 MFMAs in the order of the library's kernels: two rows of blocks at a time, down, right, up, right)
#define LOOP_BODY(R0, R1, R2, R3, R4, R5, R6, R7, R8, R9, R10, R11, R12, R13, R14, R15, S0, S1, S2, S3, G0, G1, G2, G3) \
    MFMA(64, 67, 34, 37, 0, 3) \
    MFMA(80, 83, 34, 37, 4, 7) R0 \
    MFMA(84, 87, 38, 41, 4, 7) \
    MFMA(68, 71, 38, 41, 0, 3) R1 S0 \
    MFMA(72, 75, 42, 45, 0, 3) G0 \
    MFMA(88, 91, 42, 45, 4, 7) R2 \
    MFMA(92, 95, 46, 49, 4, 7) \
    MFMA(76, 79, 46, 49, 0, 3) R3 \
    MFMA(108, 111, 46, 49, 8, 11) \
    MFMA(124, 127, 46, 49, 12, 15) R4 \
    MFMA(120, 123, 42, 45, 12, 15) \
    MFMA(104, 107, 42, 45, 8, 11) R5 S1 \
    MFMA(100, 103, 38, 41, 8, 11) G1 \
    MFMA(116, 119, 38, 41, 12, 15) R6 \
    MFMA(112, 115, 34, 37, 12, 15) \
    MFMA(96, 99, 34, 37, 8, 11) R7 \
    MFMA(128, 131, 34, 37, 16, 19) \
    MFMA(144, 147, 34, 37, 20, 23) R8 \
    MFMA(148, 151, 38, 41, 20, 23) \
    MFMA(132, 135, 38, 41, 16, 19) R9 S2 \
    MFMA(136, 139, 42, 45, 16, 19) G2 \
    MFMA(152, 155, 42, 45, 20, 23) R10 \
    MFMA(156, 159, 46, 49, 20, 23) \
    MFMA(140, 143, 46, 49, 16, 19) R11 \
    MFMA(172, 175, 46, 49, 24, 27) \
    MFMA(188, 191, 46, 49, 28, 31) R12 \
    MFMA(184, 187, 42, 45, 28, 31) \
    MFMA(168, 171, 42, 45, 24, 27) R13 S3 \
    MFMA(164, 167, 38, 41, 24, 27) G3 \
    MFMA(180, 183, 38, 41, 28, 31) R14 \
    MFMA(176, 179, 34, 37, 28, 31) \
    MFMA(160, 163, 34, 37, 24, 27) R15

#define LOOP_MFMA_ONLY LOOP_BODY("", "", "", "", "", "", "", "", "", "", "", "", "", "", "", "", "", "", "", "", "", "", "", "")
#define LOOP_LDS LOOP_BODY("ds_read_b128 v[200:203], v230 offset:0\n\t", "ds_read_b64_tr_b16 v[204:205], v231 offset:1024\n\t", "ds_read_b128 v[208:211], v230 offset:2048\n\t", "ds_read_b64_tr_b16 v[212:213], v231 offset:3072\n\t", "ds_read_b128 v[200:203], v230 offset:4096\n\t", "ds_read_b64_tr_b16 v[204:205], v231 offset:5120\n\t", "ds_read_b128 v[208:211], v230 offset:6144\n\t", "ds_read_b64_tr_b16 v[212:213], v231 offset:7168\n\t", "ds_read_b128 v[200:203], v230 offset:8192\n\t", "ds_read_b64_tr_b16 v[204:205], v231 offset:9216\n\t", "ds_read_b128 v[208:211], v230 offset:10240\n\t", "ds_read_b64_tr_b16 v[212:213], v231 offset:11264\n\t", "ds_read_b128 v[200:203], v230 offset:12288\n\t", "ds_read_b64_tr_b16 v[204:205], v231 offset:13312\n\t", "ds_read_b128 v[208:211], v230 offset:14336\n\t", "ds_read_b64_tr_b16 v[212:213], v231 offset:15360\n\t", "", "", "", "", "", "", "", "") "s_waitcnt lgkmcnt(0)"
#define LOOP_LDS_COPIES LOOP_BODY("ds_read_b128 v[200:203], v230 offset:0\n\t", "ds_read_b64_tr_b16 v[204:205], v231 offset:1024\n\t", "ds_read_b128 v[208:211], v230 offset:2048\n\t", "ds_read_b64_tr_b16 v[212:213], v231 offset:3072\n\t", "ds_read_b128 v[200:203], v230 offset:4096\n\t", "ds_read_b64_tr_b16 v[204:205], v231 offset:5120\n\t", "ds_read_b128 v[208:211], v230 offset:6144\n\t", "ds_read_b64_tr_b16 v[212:213], v231 offset:7168\n\t", "ds_read_b128 v[200:203], v230 offset:8192\n\t", "ds_read_b64_tr_b16 v[204:205], v231 offset:9216\n\t", "ds_read_b128 v[208:211], v230 offset:10240\n\t", "ds_read_b64_tr_b16 v[212:213], v231 offset:11264\n\t", "ds_read_b128 v[200:203], v230 offset:12288\n\t", "ds_read_b64_tr_b16 v[204:205], v231 offset:13312\n\t", "ds_read_b128 v[208:211], v230 offset:14336\n\t", "ds_read_b64_tr_b16 v[212:213], v231 offset:15360\n\t", "s_add_u32 m0, %0, 32768\n\t", "s_add_u32 m0, %0, 33792\n\t", "s_add_u32 m0, %0, 34816\n\t", "s_add_u32 m0, %0, 35840\n\t", "global_load_lds_dwordx4 v232, %1 offset:0\n\t", "global_load_lds_dwordx4 v232, %1 offset:1024\n\t", "global_load_lds_dwordx4 v232, %1 offset:2048\n\t", "global_load_lds_dwordx4 v232, %1 offset:3072\n\t") "s_waitcnt vmcnt(4) lgkmcnt(0)"
#define LOOP_CLOBBERS "v0", "v1", "v2", "v3", "v4", "v5", "v6", "v7", "v8", "v9", "v10", "v11", "v12", "v13", "v14", "v15", "v16", "v17", "v18", "v19", "v20", "v21", "v22", "v23", "v24", "v25", "v26", "v27", "v28", "v29", "v30", "v31", "v32", "v33", "v34", "v35", "v36", "v37", "v38", "v39", "v40", "v41", "v42", "v43", "v44", "v45", "v46", "v47", "v48", "v49", "v50", "v51", "v52", "v53", "v54", "v55", "v56", "v57", "v58", "v59", "v60", "v61", "v62", "v63", "v64", "v65", "v66", "v67", "v68", "v69", "v70", "v71", "v72", "v73", "v74", "v75", "v76", "v77", "v78", "v79", "v80", "v81", "v82", "v83", "v84", "v85", "v86", "v87", "v88", "v89", "v90", "v91", "v92", "v93", "v94", "v95", "v96", "v97", "v98", "v99", "v100", "v101", "v102", "v103", "v104", "v105", "v106", "v107", "v108", "v109", "v110", "v111", "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", "v120", "v121", "v122", "v123", "v124", "v125", "v126", "v127", "v128", "v129", "v130", "v131", "v132", "v133", "v134", "v135", "v136", "v137", "v138", "v139", "v140", "v141", "v142", "v143", "v144", "v145", "v146", "v147", "v148", "v149", "v150", "v151", "v152", "v153", "v154", "v155", "v156", "v157", "v158", "v159", "v160", "v161", "v162", "v163", "v164", "v165", "v166", "v167", "v168", "v169", "v170", "v171", "v172", "v173", "v174", "v175", "v176", "v177", "v178", "v179", "v180", "v181", "v182", "v183", "v184", "v185", "v186", "v187", "v188", "v189", "v190", "v191", "v192", "v193", "v194", "v195", "v196", "v197", "v198", "v199", "v200", "v201", "v202", "v203", "v204", "v205", "v206", "v207", "v208", "v209", "v210", "v211", "v212", "v213", "v214", "v215", "v216", "v217", "v218", "v219", "v220", "v221", "v222", "v223", "v224", "v225", "v226", "v227", "v228", "v229"

#define ZERO_ACCUMULATORS \
    "v_mov_b32 v64, 0\n\tv_mov_b32 v65, 0\n\tv_mov_b32 v66, 0\n\tv_mov_b32 v67, 0\n\tv_mov_b32 v68, 0\n\tv_mov_b32 v69, 0\n\tv_mov_b32 v70, 0\n\tv_mov_b32 v71, 0\n\t" \
    "v_mov_b32 v72, 0\n\tv_mov_b32 v73, 0\n\tv_mov_b32 v74, 0\n\tv_mov_b32 v75, 0\n\tv_mov_b32 v76, 0\n\tv_mov_b32 v77, 0\n\tv_mov_b32 v78, 0\n\tv_mov_b32 v79, 0\n\t" \
    "v_mov_b32 v80, 0\n\tv_mov_b32 v81, 0\n\tv_mov_b32 v82, 0\n\tv_mov_b32 v83, 0\n\tv_mov_b32 v84, 0\n\tv_mov_b32 v85, 0\n\tv_mov_b32 v86, 0\n\tv_mov_b32 v87, 0\n\t" \
    "v_mov_b32 v88, 0\n\tv_mov_b32 v89, 0\n\tv_mov_b32 v90, 0\n\tv_mov_b32 v91, 0\n\tv_mov_b32 v92, 0\n\tv_mov_b32 v93, 0\n\tv_mov_b32 v94, 0\n\tv_mov_b32 v95, 0\n\t" \
    "v_mov_b32 v96, 0\n\tv_mov_b32 v97, 0\n\tv_mov_b32 v98, 0\n\tv_mov_b32 v99, 0\n\tv_mov_b32 v100, 0\n\tv_mov_b32 v101, 0\n\tv_mov_b32 v102, 0\n\tv_mov_b32 v103, 0\n\t" \
    "v_mov_b32 v104, 0\n\tv_mov_b32 v105, 0\n\tv_mov_b32 v106, 0\n\tv_mov_b32 v107, 0\n\tv_mov_b32 v108, 0\n\tv_mov_b32 v109, 0\n\tv_mov_b32 v110, 0\n\tv_mov_b32 v111, 0\n\t" \
    "v_mov_b32 v112, 0\n\tv_mov_b32 v113, 0\n\tv_mov_b32 v114, 0\n\tv_mov_b32 v115, 0\n\tv_mov_b32 v116, 0\n\tv_mov_b32 v117, 0\n\tv_mov_b32 v118, 0\n\tv_mov_b32 v119, 0\n\t" \
    "v_mov_b32 v120, 0\n\tv_mov_b32 v121, 0\n\tv_mov_b32 v122, 0\n\tv_mov_b32 v123, 0\n\tv_mov_b32 v124, 0\n\tv_mov_b32 v125, 0\n\tv_mov_b32 v126, 0\n\tv_mov_b32 v127, 0\n\t" \
    "v_mov_b32 v128, 0\n\tv_mov_b32 v129, 0\n\tv_mov_b32 v130, 0\n\tv_mov_b32 v131, 0\n\tv_mov_b32 v132, 0\n\tv_mov_b32 v133, 0\n\tv_mov_b32 v134, 0\n\tv_mov_b32 v135, 0\n\t" \
    "v_mov_b32 v136, 0\n\tv_mov_b32 v137, 0\n\tv_mov_b32 v138, 0\n\tv_mov_b32 v139, 0\n\tv_mov_b32 v140, 0\n\tv_mov_b32 v141, 0\n\tv_mov_b32 v142, 0\n\tv_mov_b32 v143, 0\n\t" \
    "v_mov_b32 v144, 0\n\tv_mov_b32 v145, 0\n\tv_mov_b32 v146, 0\n\tv_mov_b32 v147, 0\n\tv_mov_b32 v148, 0\n\tv_mov_b32 v149, 0\n\tv_mov_b32 v150, 0\n\tv_mov_b32 v151, 0\n\t" \
    "v_mov_b32 v152, 0\n\tv_mov_b32 v153, 0\n\tv_mov_b32 v154, 0\n\tv_mov_b32 v155, 0\n\tv_mov_b32 v156, 0\n\tv_mov_b32 v157, 0\n\tv_mov_b32 v158, 0\n\tv_mov_b32 v159, 0\n\t" \
    "v_mov_b32 v160, 0\n\tv_mov_b32 v161, 0\n\tv_mov_b32 v162, 0\n\tv_mov_b32 v163, 0\n\tv_mov_b32 v164, 0\n\tv_mov_b32 v165, 0\n\tv_mov_b32 v166, 0\n\tv_mov_b32 v167, 0\n\t" \
    "v_mov_b32 v168, 0\n\tv_mov_b32 v169, 0\n\tv_mov_b32 v170, 0\n\tv_mov_b32 v171, 0\n\tv_mov_b32 v172, 0\n\tv_mov_b32 v173, 0\n\tv_mov_b32 v174, 0\n\tv_mov_b32 v175, 0\n\t" \
    "v_mov_b32 v176, 0\n\tv_mov_b32 v177, 0\n\tv_mov_b32 v178, 0\n\tv_mov_b32 v179, 0\n\tv_mov_b32 v180, 0\n\tv_mov_b32 v181, 0\n\tv_mov_b32 v182, 0\n\tv_mov_b32 v183, 0\n\t" \
    "v_mov_b32 v184, 0\n\tv_mov_b32 v185, 0\n\tv_mov_b32 v186, 0\n\tv_mov_b32 v187, 0\n\tv_mov_b32 v188, 0\n\tv_mov_b32 v189, 0\n\tv_mov_b32 v190, 0\n\tv_mov_b32 v191, 0\n\t"

template <int VARIANT>
__global__ __launch_bounds__(512) void loop_budget_kernel(const char* __restrict__ data /* 64 KB */, float* __restrict__ sink, int iters)
{
    __shared__ __attribute__((aligned(1024))) char smem[65536];       // 32 KB read by the fragment reads, 32 KB written by the copies
    for (int i = threadIdx.x; i < 32768 / 16; i += 512) ((uint4*)smem)[i] = ((const uint4*)data)[i];
    __syncthreads();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const char* frag = data + (threadIdx.x & 255) * 256;              // 16 x 16 bytes per lane: 8 A and 4 B fragments (and 4 unused)
    const unsigned copy_dst = __builtin_amdgcn_readfirstlane(lds) + 4096u * wave;     // + 32768 + 1024 t in the loop
    const char* copy_src = data + 4096 * wave;
    asm volatile("v_and_b32 v230, 63, %0\n\tv_lshlrev_b32 v230, 4, v230\n\tv_add_u32 v230, v230, %1\n\t"
                 "v_and_b32 v231, 63, %0\n\tv_lshlrev_b32 v231, 3, v231\n\tv_add_u32 v231, v231, %1\n\t"
                 "v_and_b32 v232, 63, %0\n\tv_lshlrev_b32 v232, 4, v232"
                 :: "v"(threadIdx.x), "v"(lds) : "v230", "v231", "v232");
    asm volatile("global_load_dwordx4 v[0:3], %0, off\n\tglobal_load_dwordx4 v[4:7], %0, off offset:16\n\t"
                 "global_load_dwordx4 v[8:11], %0, off offset:32\n\tglobal_load_dwordx4 v[12:15], %0, off offset:48\n\t"
                 "global_load_dwordx4 v[16:19], %0, off offset:64\n\tglobal_load_dwordx4 v[20:23], %0, off offset:80\n\t"
                 "global_load_dwordx4 v[24:27], %0, off offset:96\n\tglobal_load_dwordx4 v[28:31], %0, off offset:112\n\t"
                 "global_load_dwordx4 v[34:37], %0, off offset:128\n\tglobal_load_dwordx4 v[38:41], %0, off offset:144\n\t"
                 "global_load_dwordx4 v[42:45], %0, off offset:160\n\tglobal_load_dwordx4 v[46:49], %0, off offset:176\n\t"
                 "s_waitcnt vmcnt(0)"
                 :: "v"(frag) : LOOP_CLOBBERS, "memory");
    // accumulators start at zero (whatever a register held before would otherwise decide how much the adders toggle)
    asm volatile(ZERO_ACCUMULATORS ::: LOOP_CLOBBERS);
    for (int it = 0; it < iters; it++) {
        if constexpr (VARIANT == 0) asm volatile(LOOP_MFMA_ONLY ::: LOOP_CLOBBERS, "memory");
        if constexpr (VARIANT == 1) asm volatile(LOOP_LDS ::: LOOP_CLOBBERS, "memory");
        if constexpr (VARIANT == 2) asm volatile(LOOP_LDS_COPIES :: "s"(copy_dst), "s"(copy_src) : LOOP_CLOBBERS, "m0", "scc", "memory");
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    if (iters < 0) sink[0] = (float)smem[5];
}

}  // namespace

extern "C" {

// variant 0: MFMAs only, 1: + LDS fragment reads, 2: + global -> LDS copies; data: 64 KB of device memory holding f16
// operands (read as fragments, as LDS contents and as the copies' source).  flops as for bench_mfma_only.
int bench_loop_budget(const void* data, void* sink, int variant, int iters, int workgroups, void* stream)
{
    if (!data || !sink || iters < 0 || workgroups < 1 || variant < 0 || variant > 2) return -1;
    const dim3 g((unsigned)workgroups), b(512);
    if (variant == 0) hipLaunchKernelGGL(loop_budget_kernel<0>, g, b, 0, (hipStream_t)stream, (const char*)data, (float*)sink, iters);
    if (variant == 1) hipLaunchKernelGGL(loop_budget_kernel<1>, g, b, 0, (hipStream_t)stream, (const char*)data, (float*)sink, iters);
    if (variant == 2) hipLaunchKernelGGL(loop_budget_kernel<2>, g, b, 0, (hipStream_t)stream, (const char*)data, (float*)sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

// flops of one launch = workgroups * 8 wavefronts * iters * 32 MFMAs * 16384
int bench_mfma_only(const void* frags /* device, 12 * 256 * 16 bytes */, void* sink /* device, 4 bytes */,
                    int iters, int workgroups, void* stream)
{
    if (!frags || !sink || iters < 0 || workgroups < 1) return -1;
    hipLaunchKernelGGL(mfma_only_kernel, dim3((unsigned)workgroups), dim3(512), 0, (hipStream_t)stream,
                       (const half8*)frags, (float*)sink, iters);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

}  // extern "C"
