"""CPU checks of the generated assembly k loop of the long-k kernel
(csrc/gen_w4a_loop.py -> gemm_w4a_loop.inc): the committed file is what the generator
writes, and an emulation of the loop's scalar side (pointer arithmetic with carries, selects,
branches) for 1..40 k steps shows that every copy fetches a k step below KT from the right
address into the right LDS buffer, that every fragment read touches the buffer that holds its
k step, and that the waits and barriers order copies and reads of a buffer; for the block that
reads C inside the loop, that every 16 x 16 block of C is loaded once from its address and added
once to each of its four accumulator registers, after the load has landed, before the register
set is loaded again, and never next to an MFMA of that block."""
import importlib.util
import os
import re
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2108_13191_amd", "csrc")


def _generator(name="gen_w4a_loop"):
    if CSRC not in sys.path:
        sys.path.insert(0, CSRC)             # the 128 x 128 generator imports the other one
    spec = importlib.util.spec_from_file_location(name, os.path.join(CSRC, name + ".py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


@pytest.mark.parametrize("name", ["gen_w4a_loop", "gen_w4a128_loop"])
def test_committed_include_is_what_the_generator_writes(name):
    gen = _generator(name)
    with open(gen.INC_PATH) as f:
        assert f.read() == gen.render()


# What differs between the two tile forms: MFMAs per 32-wide k slice, bytes of an A / a B buffer,
# copies per wavefront and buffer, how many k steps ahead the copies run, whether the C++ prologue
# waits for all of its copies or only for those of k step 0 (`waited`), and the LDS map:
# buffer_of(kind, k step) -> (buffer key, its byte offset in the LDS); reg_base(register name) ->
# the LDS offset that the address register points at.
def _w4a_buffer(kind, step):
    return (("A", step % 2), (step % 2) * 32768) if kind == "A" else (("B", step % 3), 65536 + (step % 3) * 32768)


def _w4a_reg_base(reg):
    return 0 if reg.startswith("%[a_rd") else 65536 + (65536 if reg.startswith("%[b_rdh") else 0)


def _w4a128_buffer(kind, step):
    return ((kind, step % 5), (step % 5) * 32768 + (0 if kind == "A" else 16384))


def _w4a128_reg_base(reg):
    name = reg[2:-1].rstrip("0123456789")
    return {"a_rd": 0, "a_rdm": 65536, "a_rdh": 131072, "b_rd": 16384, "b_rdm": 16384 + 65536, "b_rdh": 16384 + 131072}[name]


GEOMETRY = {"gen_w4a_loop": dict(slice=64, a_buf=32768, b_buf=32768, ncopy=8, ahead=2, waited="all", buffer_of=_w4a_buffer, reg_base=_w4a_reg_base),
            "gen_w4a128_loop": dict(slice=16, a_buf=16384, b_buf=16384, ncopy=4, ahead=4, waited="first", buffer_of=_w4a128_buffer, reg_base=_w4a128_reg_base)}


A_BASE = 0x100000000 - 4096        # the running A pointer crosses a 32-bit carry
B_BASE = 0x7000000000
B_STEP = 64 * 8192 * 2
C_BASE = 0x300000000 - 3 * 16 * 8192 * 4 - 64
C_ROWSTEP = 16 * 8192 * 4
C_BYTES = 0x12345678
LDS_WAVE = 3072


def _run(lines, kt, ahead):
    """Execute the block's scalar instructions; return the trace of copies, reads, barriers."""
    labels = {ln[:-1]: i for i, ln in enumerate(lines) if ln.endswith(":")}
    S = {"%[kt]": kt, "%[b_step]": B_STEP, "%[lds_wave]": LDS_WAVE,
         "%[a_base_lo]": A_BASE & 0xffffffff, "%[a_base_hi]": A_BASE >> 32,
         "%[b_base_lo]": B_BASE & 0xffffffff, "%[b_base_hi]": B_BASE >> 32}
    ap, bp = A_BASE + ahead * 128, B_BASE + ahead * B_STEP
    S.update({"%[a_ptr_lo]": ap & 0xffffffff, "%[a_ptr_hi]": ap >> 32, "%[b_ptr_lo]": bp & 0xffffffff, "%[b_ptr_hi]": bp >> 32})
    S.update({"%[c_lo]": C_BASE & 0xffffffff, "%[c_hi]": C_BASE >> 32, "%[c_rowstep]": C_ROWSTEP, "%[c_bytes]": C_BYTES})

    def val(x):
        return S[x] if x in S else int(x)

    scc, pc, t, nmfma = 0, 0, 0, 0
    trace = []                      # (time, kind, ...)
    while pc < len(lines):
        ln = lines[pc]
        pc += 1
        if ln.endswith(":"):
            continue
        t += 1
        assert t < 400 * (kt + 2), "the loop does not end"
        op, _, rest = ln.partition(" ")
        a = [x.strip() for x in rest.split(",")]
        if op == "s_mov_b32":
            S[a[0]] = int(a[1], 16) if a[1].startswith("0x") else val(a[1])
        elif op == "s_add_u32":
            r = val(a[1]) + val(a[2]); S[a[0]] = r & 0xffffffff; scc = r >> 32
        elif op == "s_addc_u32":
            r = val(a[1]) + val(a[2]) + scc; S[a[0]] = r & 0xffffffff; scc = r >> 32
        elif op == "s_cmp_lt_u32":
            scc = int(val(a[0]) < val(a[1]))
        elif op == "s_cselect_b32":
            S[a[0]] = val(a[1]) if scc else val(a[2])
        elif op == "s_cbranch_scc0":
            pc = pc if scc else labels[a[0]]
        elif op == "s_cbranch_scc1":
            pc = labels[a[0]] if scc else pc
        elif op == "global_load_lds_dwordx4":
            m = re.match(r"s\[(\d+):(\d+)\]", a[1])
            src = S[f"s{m.group(1)}"] | (S[f"s{m.group(2)}"] << 32)
            trace.append((t, "copy", a[0], src, S["m0"], nmfma))
        elif op == "buffer_load_dwordx4":
            # v[..], per-lane offset of block column fn, descriptor s[76:79] (base in s76, s77), scalar offset, immediate
            m = re.match(r"v\[(\d+):(\d+)\]", a[0])
            m2 = re.match(r"(s\d+) offen offset:(\d+)", a[3])
            assert a[2] == "s[76:79]" and int(m.group(2)) == int(m.group(1)) + 3
            assert S["s78"] == C_BYTES and S["s79"] == 0x20000 and S["s77"] < 0x10000
            assert a[1] == f"%[c_voff{int(m2.group(2)) // 64}]", "the offset register of another block column"
            off = S[m2.group(1)] + int(m2.group(2))
            assert off < 2 ** 31
            src = (S["s76"] | (S["s77"] << 32)) + off
            trace.append((t, "cload", int(m.group(1)), src, nmfma))
        elif op == "v_accvgpr_read_b32":
            trace.append((t, "accread", a[0], int(a[1][1:]), nmfma))
        elif op == "v_add_f32":
            assert a[0] == a[1]
            trace.append((t, "add", a[0], int(a[2][1:]), nmfma))
        elif op == "v_accvgpr_write_b32" and a[1] != "0":
            trace.append((t, "accwrite", int(a[0][1:]), a[1], nmfma))
        elif op.startswith("ds_read"):
            m = re.match(r"(%\[\w+\]) offset:(\d+)", a[1])
            trace.append((t, "read", m.group(1), int(m.group(2)), nmfma))
        elif op.startswith("v_mfma"):
            m = re.match(r"a\[(\d+):", a[0])
            trace.append((t, "mfma", int(m.group(1)) // 4))
            nmfma += 1
        elif op == "s_barrier":
            trace.append((t, "barrier"))
        elif op == "s_waitcnt":
            vm = re.search(r"vmcnt\((\d+)\)", rest)
            lg = re.search(r"lgkmcnt\((\d+)\)", rest)
            trace.append((t, "wait", int(vm.group(1)) if vm else None, int(lg.group(1)) if lg else None))
        else:
            assert op == "v_accvgpr_write_b32", ln
    return trace, nmfma


@pytest.mark.parametrize("name,with_c", [("gen_w4a_loop", False), ("gen_w4a_loop", True), ("gen_w4a128_loop", False)])
def test_scalar_side_of_the_loop_for_every_trip_count(name, with_c):
    gen = _generator(name)
    geo = GEOMETRY[name]
    SL, A_BUF, B_BUF, NCOPY, AHEAD = geo["slice"], geo["a_buf"], geo["b_buf"], geo["ncopy"], geo["ahead"]
    buffer_of, reg_base = geo["buffer_of"], geo["reg_base"]
    lines = gen.block_c() if with_c else gen.block()
    for kt in range(gen.C_STEPS if with_c else 1, gen.C_STEPS + 14 if with_c else 41):
        trace, nmfma = _run(lines, kt, AHEAD)
        _check_c(gen, trace, with_c)
        assert nmfma == 2 * SL * kt
        # every slice multiplies every block of the wavefront's tile once, and from one MFMA of a
        # slice to the next exactly one operand changes (same block row or same block column)
        order = [e[2] for e in trace if e[1] == "mfma"]
        width = 8 if SL == 64 else 4
        for i in range(0, len(order), SL):
            assert sorted(order[i:i + SL]) == list(range(SL)), ("blocks of a slice", kt, i // SL)
            for a, b in zip(order[i:i + SL - 1], order[i + 1:i + SL]):
                assert (a // width == b // width) != (a % width == b % width), ("both operands change", a, b)
        barriers = [e[0] for e in trace if e[1] == "barrier"]
        assert len(barriers) == kt
        # --- copies: (time, buffer, k step), where they come from and where they land
        copies = []
        for e in trace:
            if e[1] != "copy":
                continue
            t, _, voff, src, m0, at = e
            j = (at - 1) // (2 * SL)                        # issued in the shadow of MFMA at - 1: its k step
            want = j + AHEAD if j + AHEAD < kt else 0
            d = m0 - LDS_WAVE
            n = int(voff[-2])
            kind = "A" if voff.startswith("%[a_off") else "B"
            buf, where = buffer_of(kind, j + AHEAD)
            assert src == (A_BASE + 128 * want if kind == "A" else B_BASE + B_STEP * want), (kind, "source", kt, j)
            assert d == where + 4096 * n and n < NCOPY, (kind, "target", kt, j)
            copies.append((t, buf, want if j + AHEAD < kt else None))
        assert len(copies) == 2 * NCOPY * kt
        issued_in_block = len(copies)
        # The copies the C++ prologue issues before the block: all complete and behind a barrier
        # ("all": k steps 0 .. min(kt, AHEAD) - 1), or ("first") only those of k step 0, the
        # others -- always AHEAD - 1 further k steps, beyond the last one k step 0 once more --
        # still in flight in front of the block's own copies, A then B of each k step.
        landed = {}
        in_flight = []
        for step in range(AHEAD if geo["waited"] == "first" else min(kt, AHEAD)):
            for kind in ("A", "B"):
                if step == 0 or geo["waited"] == "all":
                    landed[buffer_of(kind, step)[0]] = step
                else:
                    in_flight += [(buffer_of(kind, step)[0], step if step < kt else None)] * NCOPY
        copies = [(i - len(in_flight), buf, step) for i, (buf, step) in enumerate(in_flight)] + copies
        # --- a copy has landed for every wavefront once a wait that leaves fewer vector-memory
        # operations outstanding than were issued after it is followed by a barrier
        vmem = [c[0] for c in copies[:len(copies) - issued_in_block]] + [e[0] for e in trace if e[1] in ("copy", "cload")]

        def landed_at(copy_index):
            t_issue = copies[copy_index][0]
            for e in trace:
                if e[1] == "wait" and e[2] is not None and e[0] > t_issue:
                    later = sum(1 for v in vmem if t_issue < v < e[0])
                    if later >= e[2]:
                        nxt = [b for b in barriers if b > e[0]]
                        return nxt[0] if nxt else None
            return None
        land_time = [landed_at(i) for i in range(len(copies))]
        # --- reads: which buffer, which k step they expect
        for e in trace:
            if e[1] != "read":
                continue
            t, _, reg, off, at = e
            h = -1 if at == 0 else (at - 1) // SL           # issued during slice h: a read of slice h + 1
            step, sl = (h + 1) // 2, (h + 1) % 2
            kind = "A" if reg.startswith("%[a_rd") else "B"
            buf, where = buffer_of(kind, step)
            within = reg_base(reg) + off - where             # the read lies in the buffer of its k step
            if kind == "A":
                # 16-row blocks of 128-byte rows: 2 KB apart, inside the wavefront's half of the buffer
                assert int(reg[-2]) == sl and within % 2048 == 0 and 0 <= within < A_BUF // 2
            else:
                # slice s = k rows 32s.. of the buffer, second transposing read 4 k rows further
                assert within in (sl * (B_BUF // 2), sl * (B_BUF // 2) + B_BUF // 16)
            if step >= kt:
                continue                                    # fragments nobody multiplies
            # the last copy into this buffer issued before the read holds this k step and has landed
            before = [i for i, c in enumerate(copies) if c[1] == buf and c[0] < t]
            if before:
                i = before[-1]
                assert copies[i][2] == step, ("stale buffer", kt, step, buf)
                assert land_time[i] is not None and land_time[i] < t, ("read before the copy landed", kt, step, buf)
            else:
                assert landed.get(buf) == step, ("buffer never filled", kt, step, buf)
            # the next copy into this buffer is issued behind a barrier that follows a wait for this read
            after = [c for c in copies if c[1] == buf and c[0] > t]
            if after:
                waits = [w[0] for w in trace if w[1] == "wait" and w[3] == 0 and w[0] > t]
                assert waits and any(waits[0] < b < after[0][0] for b in barriers), ("buffer overwritten while read", kt, step, buf)


def _check_c(gen, trace, with_c):
    """The loads of C and their additions to the accumulators."""
    loads = [e for e in trace if e[1] == "cload"]
    if not with_c:
        assert not loads and not any(e[1] in ("accread", "add", "accwrite") for e in trace)
        return
    assert len(loads) == 64
    vmem = [e[0] for e in trace if e[1] in ("copy", "cload")]
    waits = [e for e in trace if e[1] == "wait" and e[2] is not None]
    mfmas = [e for e in trace if e[1] == "mfma"]
    adds_seen = set()
    for b, (t_load, _, reg, src, _) in enumerate(loads):
        assert src == C_BASE + (b >> 3) * C_ROWSTEP + (b & 7) * 64, ("C source", b)
        # landed: a wait behind the load that leaves no more outstanding than were issued after the load
        t_landed = min(w[0] for w in waits if w[0] > t_load and sum(1 for v in vmem if t_load < v < w[0]) >= w[2])
        # the next load into these registers
        again = [l[0] for l in loads if l[2] == reg and l[0] > t_load]
        t_again = again[0] if again else float("inf")
        for e in range(4):
            a_reg = 4 * b + e
            rd = [x for x in trace if x[1] == "accread" and x[3] == a_reg]
            wr = [x for x in trace if x[1] == "accwrite" and x[2] == a_reg]
            assert len(rd) == 1 and len(wr) == 1, ("one addition per accumulator register", a_reg)
            ad = [x for x in trace if x[1] == "add" and x[0] == rd[0][0] + 1]
            assert len(ad) == 1 and ad[0][2] == rd[0][2] and ad[0][3] == reg + e and wr[0][0] == ad[0][0] + 1 and wr[0][3] == rd[0][2]
            assert t_landed < ad[0][0] < t_again, ("C data not there / overwritten", b, e)
            # no MFMA of block b between the read and the write, none issued within 5 MFMAs before the
            # read, none within 2 MFMAs after the write
            own = [m[0] for m in mfmas if m[2] == b]
            before = [m[0] for m in mfmas if m[0] < rd[0][0]][-5:]
            after = [m[0] for m in mfmas if m[0] > wr[0][0]][:2]
            assert not any(before[0] <= o <= after[-1] for o in own), ("addition next to an MFMA of its block", b, e)
            adds_seen.add(a_reg)
    assert adds_seen == set(range(256))
