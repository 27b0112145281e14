#!/usr/bin/env python3
"""Writes gemm_w4a128_loop.inc: the k loop of the 128 x 128 x 64 form of the four-wavefront
kernel (gemm_w4a128.hip) as a hand-scheduled assembly block, plus the operand lists that bind
it to the C++ around it.  The structure is that of gen_w4a_loop.py (which documents it: k steps
unrolled over the period of the LDS buffers, one barrier per k step, copy sources redirected to
the tile's first k step once they would lie beyond KT) at a quarter of the tile:

  wavefront tile 64 x 64 = 4 x 4 accumulators of 16 x 16 (64 AccVGPRs), 16 MFMAs per 32-wide k
  slice; fragments of a slice: 4 A (ds_read_b128) + 4 B (two transposing reads each).

A k step of this tile is 32 MFMAs per wavefront, about 0.25 us, a quarter of what a copy takes
to arrive from L2: the LDS therefore holds a ring of FIVE stages (A 16 KB: 128 rows x 128 B,
then B 16 KB: 64 k rows x 256 B; 160 KB), and the copies of k step j + 4 are issued during
step j (4 + 4 per wavefront) into the stage that step j - 1 used.

Schedule of k step j ("after MFMA i" = in its shadow):

  slice 0 (fragment set 0):
    after MFMA 0..3         scalar: sources of this step's copies, advance
    after MFMA 0..5         two of the 12 fragment reads of slice 1 each (into set 1)
    after MFMA 8 + 2t       M0 for copy t of B(j + 4), after MFMA 9 + 2t the copy
    wait: all copies but those 4 and the 16 of k steps j + 2 and j + 3, all LDS reads; barrier
  slice 1 (fragment set 1):
    after MFMA 0..5         the fragment reads of slice 0 of k step j + 1
    after MFMA 8 + 2t, 9 + 2t   copy t of A(j + 4)
    wait: all LDS reads

Run: python3 gen_w4a128_loop.py   (writes gemm_w4a128_loop.inc beside itself)
"""
import os

from gen_w4a_loop import S_J, S_J2, S_ASRC, S_BSRC, S_APTR, S_BPTR, asm_macro, snake

A_BUF = 16384
B_BUF = 16384
STAGE = A_BUF + B_BUF                             # a stage: A, then B
STAGES = 5
AHEAD = STAGES - 1                                # copies are issued this many k steps ahead
B_ROW = 256
FM = FN = 4
NCOPY = 4
SLOTS = FM * FN
SCALAR_CLOBBERS = [f"s{i}" for i in range(64, 74)]
V_CLOBBERED = 64                                  # two fragment sets of 32 registers


def frag_a(d, fm):
    lo = 32 * d + 4 * fm
    return f"v[{lo}:{lo + 3}]"


def frag_b(d, fn, half=None):
    lo = 32 * d + 16 + 4 * fn
    if half is None:
        return f"v[{lo}:{lo + 3}]"
    return f"v[{lo + 2 * half}:{lo + 2 * half + 1}]"


def acc(fm, fn):
    lo = 4 * (FN * fm + fn)
    return f"a[{lo}:{lo + 3}]"


def mfma(d, i):
    fm, fn = snake(i, FN)                                 # one operand changes per MFMA, A back and forth between two
    return f"v_mfma_f32_16x16x32_f16 {acc(fm, fn)}, {frag_b(d, fn)}, {frag_a(d, fm)}, {acc(fm, fn)}"


def read(stage, s, d, r):
    """Read r (0..11) of k slice s of LDS stage `stage` into fragment set d: the 4 B operands
    (two transposing reads each) first, then the 4 A operands.  Stages 0, 1 are addressed from
    the registers a_rd / b_rd, stages 2, 3 from a_rdm / b_rdm (+ 64 KB), stage 4 from a_rdh /
    b_rdh (+ 128 KB): the instruction's offset has 16 bits.  The B registers point at the B half
    of stage 0."""
    suffix = ("", "", "m", "m", "h")[stage]
    base = (stage % 2) * STAGE
    if r < 2 * FN:
        fn, half = r >> 1, r & 1
        off = base + s * 32 * B_ROW + half * 4 * B_ROW
        assert off < 65536
        return f"ds_read_b64_tr_b16 {frag_b(d, fn, half)}, %[b_rd{suffix}{fn}] offset:{off}"
    fm = r - 2 * FN
    off = base + fm * 16 * 128
    assert off < 65536
    return f"ds_read_b128 {frag_a(d, fm)}, %[a_rd{suffix}{s}] offset:{off}"


NREADS = 2 * FN + FM


def k_step(ph):
    out = []
    nxt = (ph + 1) % STAGES
    a_dst = ((ph + AHEAD) % STAGES) * STAGE
    b_dst = a_dst + A_BUF
    scalar = [
        [f"s_add_u32 {S_J2}, {S_J}, {AHEAD}", f"s_cmp_lt_u32 {S_J2}, %[kt]"],
        [f"s_cselect_b32 s66, {S_APTR[0]}, %[a_base_lo]", f"s_cselect_b32 s67, {S_APTR[1]}, %[a_base_hi]"],
        [f"s_cselect_b32 s68, {S_BPTR[0]}, %[b_base_lo]", f"s_cselect_b32 s69, {S_BPTR[1]}, %[b_base_hi]"],
        [f"s_add_u32 {S_APTR[0]}, {S_APTR[0]}, 128", f"s_addc_u32 {S_APTR[1]}, {S_APTR[1]}, 0",
         f"s_add_u32 {S_BPTR[0]}, {S_BPTR[0]}, %[b_step]", f"s_addc_u32 {S_BPTR[1]}, {S_BPTR[1]}, 0"],
    ]

    def slice_(d, reads, copy_dst, copy_off, copy_src, scalars, last):
        r = 0
        for i in range(SLOTS):
            out.append(mfma(d, i))
            if scalars and i < 4:
                out.extend(scalar[i])
            for _ in range(2):
                if i < 6 and r < NREADS:
                    out.append(reads(r)); r += 1
            if i >= 8 and i % 2 == 0:
                out.append(f"s_add_u32 m0, %[lds_wave], {copy_dst + 4096 * ((i - 8) // 2)}")
            if i >= 8 and i % 2 == 1:
                out.append(f"global_load_lds_dwordx4 %[{copy_off}{(i - 9) // 2}], {copy_src}")
            if last and i == 12:
                out.append(f"s_add_u32 {S_J}, {S_J}, 1")
        assert r == NREADS

    slice_(0, lambda r: read(ph, 1, 1, r), b_dst, "b_off", S_BSRC, True, False)
    # outstanding may stay: this slice's 4 copies and all 8 of each of the k steps j + 2, j + 3
    out.append(f"s_waitcnt vmcnt({NCOPY + 2 * NCOPY * (AHEAD - 2)}) lgkmcnt(0)")
    out.append("s_barrier")
    slice_(1, lambda r: read(nxt, 0, 0, r), a_dst, "a_off", S_ASRC, False, True)
    out.append("s_waitcnt lgkmcnt(0)")
    out.append(f"s_cmp_lt_u32 {S_J}, %[kt]")
    out.append("s_cbranch_scc1 W4A128_TOP_%=" if ph == STAGES - 1 else "s_cbranch_scc0 W4A128_DONE_%=")
    return out


def block():
    out = []
    for i in range(4 * FM * FN):
        out.append(f"v_accvgpr_write_b32 a{i}, 0")
    out += [f"s_mov_b32 {S_J}, 0",
            f"s_mov_b32 {S_APTR[0]}, %[a_ptr_lo]", f"s_mov_b32 {S_APTR[1]}, %[a_ptr_hi]",
            f"s_mov_b32 {S_BPTR[0]}, %[b_ptr_lo]", f"s_mov_b32 {S_BPTR[1]}, %[b_ptr_hi]"]
    for r in range(NREADS):
        out.append(read(0, 0, 0, r))
    out.append("s_waitcnt lgkmcnt(0)")
    out.append("W4A128_TOP_%=:")
    for ph in range(STAGES):
        out += k_step(ph)
    out.append("W4A128_DONE_%=:")
    out.append("s_waitcnt vmcnt(0)")
    return out


def render():
    """The text of gemm_w4a128_loop.inc."""
    text = ["// Generated by gen_w4a128_loop.py -- edit the generator, not this file.",
            "// W4A128_LOOP_ASM: the k loop; W4A128_LOOP_OUTPUTS(acc) / W4A128_LOOP_INPUTS / W4A128_LOOP_CLOBBERS: its operands."]
    text += asm_macro("W4A128_LOOP_ASM", block())
    outs = []
    for fm in range(FM):
        outs.append("    " + ", ".join(f'"=&{{{acc(fm, fn)}}}"(ACC[{fm}][{fn}])' for fn in range(FN)))
    text.append("#define W4A128_LOOP_OUTPUTS(ACC) \\")
    text.append(", \\\n".join(outs))
    vin = []
    for suffix, plus in (("", 0), ("m", 65536), ("h", 131072)):
        vin += [f'[a_rd{suffix}{s}] "v"(a_rd[{s}] + {plus}u)' for s in range(2)]
        vin += [f'[b_rd{suffix}{f}] "v"(b_rd[{f}] + {plus}u)' for f in range(FN)]
    vin += [f'[a_off{t}] "v"(a_off[{t}])' for t in range(NCOPY)]
    vin += [f'[b_off{t}] "v"(b_off[{t}])' for t in range(NCOPY)]
    sin = ['[lds_wave] "s"(lds_wave)', '[kt] "s"(kt_full)', '[b_step] "s"(b_step)',
           '[a_base_lo] "s"(a_base_lo)', '[a_base_hi] "s"(a_base_hi)', '[b_base_lo] "s"(b_base_lo)', '[b_base_hi] "s"(b_base_hi)',
           '[a_ptr_lo] "s"(a_ptr_lo)', '[a_ptr_hi] "s"(a_ptr_hi)', '[b_ptr_lo] "s"(b_ptr_lo)', '[b_ptr_hi] "s"(b_ptr_hi)']
    text.append("#define W4A128_LOOP_INPUTS \\")
    allin = vin + sin
    rows = [", ".join(allin[i:i + 4]) for i in range(0, len(allin), 4)]
    text.append("    " + ", \\\n    ".join(rows))
    clob = [f'"v{i}"' for i in range(V_CLOBBERED)] + [f'"{s}"' for s in SCALAR_CLOBBERS] + ['"m0"', '"scc"', '"memory"']
    text.append("#define W4A128_LOOP_CLOBBERS \\")
    rows = [", ".join(clob[i:i + 16]) for i in range(0, len(clob), 16)]
    text.append("    " + ", \\\n    ".join(rows))
    return "\n".join(text) + "\n"


INC_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "gemm_w4a128_loop.inc")


def main():
    with open(INC_PATH, "w") as f:
        f.write(render())
    print(f"wrote {INC_PATH}: {len(block())} instructions")


if __name__ == "__main__":
    main()
