#!/usr/bin/env python3
"""Writes gemm_w4a_loop.inc: the k loop of the four-wavefront 256 x 256 x 64 kernel
(gemm_w4a.hip) as one hand-scheduled assembly block, plus the operand lists that
bind it to the C++ around it.

Why assembly: the wavefront is alone on its SIMD, so every instruction the
compiler adds to the loop (address arithmetic, branches around the copies,
accumulator moves when the loop is unrolled) is matrix-pipe idle time.  Here the
loop is unrolled six k steps deep -- the period of the 2 A buffers and 3 B
buffers -- so that every LDS address is a register plus an immediate, and the
vector ALU issues nothing but MFMAs.

Schedule of k step j (two 32-wide k slices of 64 MFMAs; "after MFMA i" = in its
shadow; the steps of the paper's recipe -- sections "Global Memory Load Latency
Hiding" and "Completing Latency Hiding" -- at one wavefront per SIMD):

  slice 0 (fragment set 0):
    after MFMA 0..3     scalar: source pointers of this step's copies (k step
                        j + 2, or the tile's first k step once j + 2 >= KT:
                        loaded into a buffer nobody reads any more), advance
    after odd MFMA < 48 the 24 fragment reads of slice 1 into set 1
    after MFMA 8t + 6   copy t of B(j + 2) into B buffer (j + 2) % 3 (M0 is set
                        after MFMA 8t + 4)
    wait: all copies but those 8, all LDS reads; workgroup barrier
  slice 1 (fragment set 1):
    after odd MFMA < 48 the 24 fragment reads of slice 0 of k step j + 1
    after MFMA 8t + 6   copy t of A(j + 2) into A buffer j % 2
    wait: all LDS reads

Run: python3 gen_w4a_loop.py   (writes gemm_w4a_loop.inc beside itself)
"""
import os

A_BUF = 32768
B_BUF = 32768
B_REGION = 2 * A_BUF
B_ROW = 512

# fixed scalar registers of the block (declared as clobbers)
S_J, S_J2 = "s64", "s65"
S_ASRC, S_BSRC = "s[66:67]", "s[68:69]"          # sources of this step's copies
S_APTR, S_BPTR = ("s70", "s71"), ("s72", "s73")  # running: k step j + 2
SCALAR_CLOBBERS = [f"s{i}" for i in range(64, 74)]


def frag_a(d, fm):
    lo = 64 * d + 4 * fm
    return f"v[{lo}:{lo + 3}]"


def frag_b(d, fn, half=None):
    lo = 64 * d + 32 + 4 * fn
    if half is None:
        return f"v[{lo}:{lo + 3}]"
    return f"v[{lo + 2 * half}:{lo + 2 * half + 1}]"


def acc(fm, fn):
    lo = 4 * (8 * fm + fn)
    return f"a[{lo}:{lo + 3}]"


def mfma(d, i):
    fm, fn = i >> 3, i & 7
    return f"v_mfma_f32_16x16x32_f16 {acc(fm, fn)}, {frag_b(d, fn)}, {frag_a(d, fm)}, {acc(fm, fn)}"


def read(step_phase, s, d, r):
    """Read r (0..23) of k slice s of the stage of phase step_phase into fragment set d:
    the 8 B operands (two transposing reads each) first, then the 8 A operands."""
    abuf, bbuf = step_phase % 2, step_phase % 3
    if r < 16:
        fn, half = r >> 1, r & 1
        if bbuf < 2:
            reg, off = f"%[b_rd{fn}]", bbuf * B_BUF
        else:
            reg, off = f"%[b_rdh{fn}]", 0
        off += s * 32 * B_ROW + half * 4 * B_ROW
        assert off < 65536
        return f"ds_read_b64_tr_b16 {frag_b(d, fn, half)}, {reg} offset:{off}"
    fm = r - 16
    off = abuf * A_BUF + fm * 16 * 128
    assert off < 65536
    return f"ds_read_b128 {frag_a(d, fm)}, %[a_rd{s}] offset:{off}"


def k_step(ph):
    out = []
    nxt = (ph + 1) % 6
    b_dst = B_REGION + ((ph + 2) % 3) * B_BUF
    a_dst = (ph % 2) * A_BUF
    scalar = [
        [f"s_add_u32 {S_J2}, {S_J}, 2", f"s_cmp_lt_u32 {S_J2}, %[kt]"],
        [f"s_cselect_b32 s66, {S_APTR[0]}, %[a_base_lo]", f"s_cselect_b32 s67, {S_APTR[1]}, %[a_base_hi]"],
        [f"s_cselect_b32 s68, {S_BPTR[0]}, %[b_base_lo]", f"s_cselect_b32 s69, {S_BPTR[1]}, %[b_base_hi]"],
        [f"s_add_u32 {S_APTR[0]}, {S_APTR[0]}, 128", f"s_addc_u32 {S_APTR[1]}, {S_APTR[1]}, 0",
         f"s_add_u32 {S_BPTR[0]}, {S_BPTR[0]}, %[b_step]", f"s_addc_u32 {S_BPTR[1]}, {S_BPTR[1]}, 0"],
    ]
    # ---- slice 0
    r = 0
    for i in range(64):
        out.append(mfma(0, i))
        if i < 4:
            out += scalar[i]
        if i % 2 == 1 and r < 24:
            out.append(read(ph, 1, 1, r)); r += 1
        if i % 8 == 4:
            out.append(f"s_add_u32 m0, %[lds_wave], {b_dst + 4096 * (i // 8)}")
        if i % 8 == 6:
            out.append(f"global_load_lds_dwordx4 %[b_off{i // 8}], {S_BSRC}")
    assert r == 24
    out.append("s_waitcnt vmcnt(8) lgkmcnt(0)")
    out.append("s_barrier")
    # ---- slice 1
    r = 0
    for i in range(64):
        out.append(mfma(1, i))
        if i % 2 == 1 and r < 24:
            out.append(read(nxt, 0, 0, r)); r += 1
        if i % 8 == 4:
            out.append(f"s_add_u32 m0, %[lds_wave], {a_dst + 4096 * (i // 8)}")
        if i % 8 == 6:
            out.append(f"global_load_lds_dwordx4 %[a_off{i // 8}], {S_ASRC}")
        if i == 60:
            out += [f"s_add_u32 {S_J}, {S_J}, 1"]
    out.append("s_waitcnt lgkmcnt(0)")
    out.append(f"s_cmp_lt_u32 {S_J}, %[kt]")
    out.append("s_cbranch_scc1 W4A_TOP_%=" if ph == 5 else "s_cbranch_scc0 W4A_DONE_%=")
    return out


def block():
    out = []
    for i in range(256):
        out.append(f"v_accvgpr_write_b32 a{i}, 0")
    out += [f"s_mov_b32 {S_J}, 0",
            f"s_mov_b32 {S_APTR[0]}, %[a_ptr_lo]", f"s_mov_b32 {S_APTR[1]}, %[a_ptr_hi]",
            f"s_mov_b32 {S_BPTR[0]}, %[b_ptr_lo]", f"s_mov_b32 {S_BPTR[1]}, %[b_ptr_hi]"]
    for r in range(24):
        out.append(read(0, 0, 0, r))
    out.append("s_waitcnt lgkmcnt(0)")
    out.append("W4A_TOP_%=:")
    for ph in range(6):
        out += k_step(ph)
    out.append("W4A_DONE_%=:")
    out.append("s_waitcnt vmcnt(0)")
    return out


def render():
    """The text of gemm_w4a_loop.inc."""
    lines = block()
    text = ["// Generated by gen_w4a_loop.py -- edit the generator, not this file.",
            "// W4A_LOOP_ASM: the k loop; W4A_LOOP_OUTPUTS(acc) / W4A_LOOP_INPUTS / W4A_LOOP_CLOBBERS: its operands.",
            "#define W4A_LOOP_ASM \\"]
    for ln in lines:
        text.append(f'    "{ln}\\n\\t" \\')
    text[-1] = text[-1][:-2]
    outs = []
    for fm in range(8):
        outs.append("    " + ", ".join(f'"=&{{{acc(fm, fn)}}}"(ACC[{fm}][{fn}])' for fn in range(8)))
    text.append("#define W4A_LOOP_OUTPUTS(ACC) \\")
    text.append(", \\\n".join(outs))
    vin = [f'[a_rd{s}] "v"(a_rd[{s}])' for s in range(2)]
    vin += [f'[b_rd{f}] "v"(b_rd[{f}])' for f in range(8)]
    vin += [f'[b_rdh{f}] "v"(b_rd[{f}] + {2 * B_BUF}u)' for f in range(8)]
    vin += [f'[a_off{t}] "v"(a_off[{t}])' for t in range(8)]
    vin += [f'[b_off{t}] "v"(b_off[{t}])' for t in range(8)]
    sin = ['[lds_wave] "s"(lds_wave)', '[kt] "s"(kt_full)', '[b_step] "s"(b_step)',
           '[a_base_lo] "s"(a_base_lo)', '[a_base_hi] "s"(a_base_hi)', '[b_base_lo] "s"(b_base_lo)', '[b_base_hi] "s"(b_base_hi)',
           '[a_ptr_lo] "s"(a_ptr_lo)', '[a_ptr_hi] "s"(a_ptr_hi)', '[b_ptr_lo] "s"(b_ptr_lo)', '[b_ptr_hi] "s"(b_ptr_hi)']
    text.append("#define W4A_LOOP_INPUTS \\")
    allin = vin + sin
    rows = [", ".join(allin[i:i + 4]) for i in range(0, len(allin), 4)]
    text.append("    " + ", \\\n    ".join(rows))
    clob = [f'"v{i}"' for i in range(128)] + [f'"{s}"' for s in SCALAR_CLOBBERS] + ['"m0"', '"scc"', '"memory"']
    text.append("#define W4A_LOOP_CLOBBERS \\")
    rows = [", ".join(clob[i:i + 16]) for i in range(0, len(clob), 16)]
    text.append("    " + ", \\\n    ".join(rows))
    return "\n".join(text) + "\n"


INC_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "gemm_w4a_loop.inc")


def main():
    with open(INC_PATH, "w") as f:
        f.write(render())
    print(f"wrote {INC_PATH}: {len(block())} instructions")


if __name__ == "__main__":
    main()
