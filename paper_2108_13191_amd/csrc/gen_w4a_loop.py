#!/usr/bin/env python3
"""Writes gemm_w4a_loop.inc: the k loop of the four-wavefront 256 x 256 x 64 kernel
(gemm_w4a.hip) as hand-scheduled assembly blocks, plus the operand lists that bind
them to the C++ around them.

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
    wait: all copies but those 8 (and the C loads of the step before), all LDS
    reads; workgroup barrier
  slice 1 (fragment set 1):
    after odd MFMA < 48 the 24 fragment reads of slice 0 of k step j + 1
    after MFMA 8t + 6   copy t of A(j + 2) into A buffer j % 2
    wait: all LDS reads

Two blocks are written.  W4A_LOOP_ASM is the loop alone (accumulators start at
zero; C is added by the caller afterwards).  W4A_LOOP_C_ASM reads C inside the
loop: a compute unit moves its 256 KB of C from HBM at a rate set by latency and
by how many requests it may have in flight, about 12 us per tile, during which
the matrix units would idle if it were done behind the loop.  Its first
C_STEPS k steps are a straight-line section in which, besides the schedule above,

    after MFMA 63 of slice 1 of step j        C_PER_STEP 16 x 16 blocks of C are loaded (one 16-byte
                                              load per lane and block) into one of three register sets;
                                              buffer loads, whose range check returns 0 for rows beyond
                                              C's last (the caller puts lanes whose columns lie beyond
                                              C's last out of range through their offset register)
    in slice 1 of step j + 2 (they have       those blocks are added to their accumulators: read the
    landed: the wait in the middle of that    AccVGPR, add, write it back, three instructions in the
    step leaves only younger loads out)       shadow of an MFMA, never next to an MFMA of that block

after which the loop proper takes over (C_STEPS is a multiple of six).  C + sum
is then formed as (partial sum + C) + rest of the sum.

Run: python3 gen_w4a_loop.py   (writes gemm_w4a_loop.inc beside itself)
"""
import os

A_BUF = 32768
B_BUF = 32768
B_REGION = 2 * A_BUF
B_ROW = 512

C_PER_STEP = 2                      # blocks of C loaded per k step in the C section
C_LOAD_STEPS = 64 // C_PER_STEP     # k steps that load C
C_STEPS = ((C_LOAD_STEPS + 2 + 5) // 6) * 6   # length of the section: the last loads are added two steps later

# fixed registers of the blocks (declared as clobbers)
S_J, S_J2 = "s64", "s65"
S_ASRC, S_BSRC = "s[66:67]", "s[68:69]"          # sources of this step's copies
S_APTR, S_BPTR = ("s70", "s71"), ("s72", "s73")  # running: k step j + 2
S_CSOFF = "s74"                                  # running: byte offset of the row of blocks fm in this wavefront's C
S_CRSRC = "s[76:79]"                             # buffer descriptor of this wavefront's part of C
SCALAR_CLOBBERS = [f"s{i}" for i in range(64, 80)]
V_CTMP = 128                                     # 3 sets x C_PER_STEP blocks x 4 registers of C
V_T = V_CTMP + 3 * C_PER_STEP * 4                # 3 scratch registers for the adds
V_CLOBBERED = V_T + 3


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


def snake(i, width):
    """(fm, fn) of MFMA i of a slice over blocks of `width` columns: two rows of blocks at a time,
    down, right, up, right, ... and back in the next pair of rows.  From one MFMA to the next
    exactly one of the two operands changes, and the A operand goes back and forth between two
    fragments: the part runs at its power limit, and MFMAs alone draw the less the less their
    operands differ from the last one's (1936 TFLOP/s walking row by row, 1960 in serpentine
    rows, 1985 in this order, 2030 with the same operands every time)."""
    pr, q = divmod(i, 2 * width)
    fm = 2 * pr + (1 if q % 4 in (1, 2) else 0)
    fn = q // 2 if pr % 2 == 0 else width - 1 - q // 2
    return fm, fn


def block_at(i):
    return snake(i, 8)


SLOT_OF = {8 * fm + fn: i for i in range(64) for fm, fn in [snake(i, 8)]}


def slot_of(b):
    """The MFMA of a slice that works on block b = 8 fm + fn."""
    return SLOT_OF[b]


def mfma(d, i):
    fm, fn = block_at(i)
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


def c_tmp(tset, n):
    lo = V_CTMP + (tset * C_PER_STEP + n) * 4
    return lo


# slots of slice 1 (an MFMA's shadow) that hold no LDS read, copy or M0 write, and not the last one
CLEAN_SLOTS = [i for i in range(63) if (i < 48 and i % 8 in (0, 2)) or (i >= 48 and i % 8 not in (4, 6))]


def add_plan(blocks):
    """slot -> instructions that add the loaded C blocks (block, first register of its C data) to
    their accumulators, one accumulator register per slot: read it, add, write it back.  The
    MFMA of block b is number slot_of(b) of every slice of 64: a slot qualifies for b if the last
    such MFMA was issued at least 6 MFMAs before it (its result is there) and the next one comes
    at least 3 MFMAs after it (the write is seen)."""
    plan, free = {}, list(CLEAN_SLOTS)
    for b, reg in blocks:
        ok = [s for s in free if (s - slot_of(b)) % 64 >= 6 and (slot_of(b) - s) % 64 >= 3]
        assert len(ok) >= 4, (b, free)
        for e, s in enumerate(ok[:4]):
            free.remove(s)
            t = f"v{V_T + e % 3}"
            plan[s] = [f"v_accvgpr_read_b32 {t}, a{4 * b + e}", f"v_add_f32 {t}, {t}, v{reg + e}", f"v_accvgpr_write_b32 a{4 * b + e}, {t}"]
    return plan


def k_step(ph, exits=True, loads=(), adds=(), loads_before=0):
    """One k step at phase ph = j mod 6.  loads: (block, first register) of the C blocks to load at
    its end; adds: those to add in its second slice; loads_before: C loads the step before issued."""
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
    out.append(f"s_waitcnt vmcnt({8 + loads_before}) lgkmcnt(0)")
    out.append("s_barrier")
    # ---- slice 1
    plan = add_plan(adds)
    r = 0
    for i in range(64):
        out.append(mfma(1, i))
        if i % 2 == 1 and r < 24:
            out.append(read(nxt, 0, 0, r)); r += 1
        if i % 8 == 4:
            out.append(f"s_add_u32 m0, %[lds_wave], {a_dst + 4096 * (i // 8)}")
        if i % 8 == 6:
            out.append(f"global_load_lds_dwordx4 %[a_off{i // 8}], {S_ASRC}")
        out += plan.get(i, [])
        if i == 60:
            out += [f"s_add_u32 {S_J}, {S_J}, 1"]
    for b, reg in loads:
        out.append(f"buffer_load_dwordx4 v[{reg}:{reg + 3}], %[c_voff{b & 7}], {S_CRSRC}, {S_CSOFF} offen offset:{(b & 7) * 64}")
        if b & 7 == 7:
            out.append(f"s_add_u32 {S_CSOFF}, {S_CSOFF}, %[c_rowstep]")
    out.append("s_waitcnt lgkmcnt(0)")
    if exits:
        out.append(f"s_cmp_lt_u32 {S_J}, %[kt]")
        out.append("s_cbranch_scc1 W4A_TOP_%=" if ph == 5 else "s_cbranch_scc0 W4A_DONE_%=")
    return out


def head(with_c):
    out = []
    for i in range(256):
        out.append(f"v_accvgpr_write_b32 a{i}, 0")
    out += [f"s_mov_b32 {S_J}, 0",
            f"s_mov_b32 {S_APTR[0]}, %[a_ptr_lo]", f"s_mov_b32 {S_APTR[1]}, %[a_ptr_hi]",
            f"s_mov_b32 {S_BPTR[0]}, %[b_ptr_lo]", f"s_mov_b32 {S_BPTR[1]}, %[b_ptr_hi]"]
    if with_c:
        # raw buffer (stride 0): base, number of bytes that may be read from it, 32-bit data format
        out += ["s_mov_b32 s76, %[c_lo]", "s_mov_b32 s77, %[c_hi]", "s_mov_b32 s78, %[c_bytes]", "s_mov_b32 s79, 0x20000",
                f"s_mov_b32 {S_CSOFF}, 0"]
    for r in range(24):
        out.append(read(0, 0, 0, r))
    out.append("s_waitcnt lgkmcnt(0)")
    return out


def loop():
    out = ["W4A_TOP_%=:"]
    for ph in range(6):
        out += k_step(ph)
    out.append("W4A_DONE_%=:")
    out.append("s_waitcnt vmcnt(0)")
    return out


def block():
    """The loop alone."""
    return head(False) + loop()


def c_loads_of_step(j):
    """(block, first register of its C data) of the blocks loaded at the end of k step j of the C section."""
    if j < 0 or j >= C_LOAD_STEPS:
        return []
    return [(C_PER_STEP * j + n, c_tmp(j % 3, n)) for n in range(C_PER_STEP)]


def block_c():
    """The C section (needs KT >= C_STEPS), then the loop."""
    out = head(True)
    for j in range(C_STEPS):
        out += k_step(j % 6, exits=False, loads=c_loads_of_step(j), adds=c_loads_of_step(j - 2),
                      loads_before=len(c_loads_of_step(j - 1)))
    out += [f"s_cmp_lt_u32 {S_J}, %[kt]", "s_cbranch_scc0 W4A_DONE_%="]
    return out + loop()


def asm_macro(name, lines):
    text = [f"#define {name} \\"]
    for ln in lines:
        text.append(f'    "{ln}\\n\\t" \\')
    text[-1] = text[-1][:-2]
    return text


def render():
    """The text of gemm_w4a_loop.inc."""
    text = ["// Generated by gen_w4a_loop.py -- edit the generator, not this file.",
            "// W4A_LOOP_ASM: the k loop; W4A_LOOP_C_ASM: the same with C read and added during its first W4A_C_STEPS",
            "// k steps; W4A_LOOP_OUTPUTS(acc) / W4A_LOOP_INPUTS / W4A_LOOP_CLOBBERS: their operands.",
            f"#define W4A_C_STEPS {C_STEPS}"]
    text += asm_macro("W4A_LOOP_ASM", block())
    text += asm_macro("W4A_LOOP_C_ASM", block_c())
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
    vin += [f'[c_voff{f}] "v"(c_voff_fn[{f}])' for f in range(8)]
    sin = ['[lds_wave] "s"(lds_wave)', '[kt] "s"(kt_full)', '[b_step] "s"(b_step)',
           '[a_base_lo] "s"(a_base_lo)', '[a_base_hi] "s"(a_base_hi)', '[b_base_lo] "s"(b_base_lo)', '[b_base_hi] "s"(b_base_hi)',
           '[a_ptr_lo] "s"(a_ptr_lo)', '[a_ptr_hi] "s"(a_ptr_hi)', '[b_ptr_lo] "s"(b_ptr_lo)', '[b_ptr_hi] "s"(b_ptr_hi)',
           '[c_lo] "s"(c_lo)', '[c_hi] "s"(c_hi)', '[c_bytes] "s"(c_bytes)', '[c_rowstep] "s"(c_rowstep)']
    text.append("#define W4A_LOOP_INPUTS \\")
    allin = vin + sin
    rows = [", ".join(allin[i:i + 4]) for i in range(0, len(allin), 4)]
    text.append("    " + ", \\\n    ".join(rows))
    clob = [f'"v{i}"' for i in range(V_CLOBBERED)] + [f'"{s}"' for s in SCALAR_CLOBBERS] + ['"m0"', '"scc"', '"memory"']
    text.append("#define W4A_LOOP_CLOBBERS \\")
    rows = [", ".join(clob[i:i + 16]) for i in range(0, len(clob), 16)]
    text.append("    " + ", \\\n    ".join(rows))
    return "\n".join(text) + "\n"


INC_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "gemm_w4a_loop.inc")


def main():
    with open(INC_PATH, "w") as f:
        f.write(render())
    print(f"wrote {INC_PATH}: {len(block())} + {len(block_c())} instructions, C section of {C_STEPS} k steps")


if __name__ == "__main__":
    main()
