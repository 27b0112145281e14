"""CPU checks of the generated assembly k loop of the four-wavefront ladder kernel
(csrc/ladder/gen_w4a_loop.py -> gemm_w4a_loop.inc): the committed file is what the generator
writes, and an emulation of the loop's scalar side (pointer arithmetic with carries, selects,
branches) for 1..40 k steps shows that every copy fetches a k step below KT from the right
address into the right LDS buffer, that every fragment read touches the buffer that holds its
k step, and that the waits and barriers order copies and reads of a buffer."""
import importlib.util
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GEN = os.path.join(ROOT, "paper_2108_13191_amd", "csrc", "ladder", "gen_w4a_loop.py")


def _generator():
    spec = importlib.util.spec_from_file_location("gen_w4a_loop", GEN)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_committed_include_is_what_the_generator_writes():
    gen = _generator()
    with open(gen.INC_PATH) as f:
        assert f.read() == gen.render()


A_BASE = 0x100000000 - 4096        # the running A pointer crosses a 32-bit carry
B_BASE = 0x7000000000
B_STEP = 64 * 8192 * 2
LDS_WAVE = 3072


def _run(lines, kt):
    """Execute the block's scalar instructions; return the trace of copies, reads, barriers."""
    labels = {ln[:-1]: i for i, ln in enumerate(lines) if ln.endswith(":")}
    S = {"%[kt]": kt, "%[b_step]": B_STEP, "%[lds_wave]": LDS_WAVE,
         "%[a_base_lo]": A_BASE & 0xffffffff, "%[a_base_hi]": A_BASE >> 32,
         "%[b_base_lo]": B_BASE & 0xffffffff, "%[b_base_hi]": B_BASE >> 32}
    ap, bp = A_BASE + 2 * 128, B_BASE + 2 * B_STEP
    S.update({"%[a_ptr_lo]": ap & 0xffffffff, "%[a_ptr_hi]": ap >> 32, "%[b_ptr_lo]": bp & 0xffffffff, "%[b_ptr_hi]": bp >> 32})

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
            S[a[0]] = val(a[1])
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
        elif op.startswith("ds_read"):
            m = re.match(r"(%\[\w+\]) offset:(\d+)", a[1])
            trace.append((t, "read", m.group(1), int(m.group(2)), nmfma))
        elif op.startswith("v_mfma"):
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


def test_scalar_side_of_the_loop_for_every_trip_count():
    lines = _generator().block()
    for kt in range(1, 41):
        trace, nmfma = _run(lines, kt)
        assert nmfma == 128 * kt
        barriers = [e[0] for e in trace if e[1] == "barrier"]
        assert len(barriers) == kt
        # --- copies: (time, buffer, k step), where they come from and where they land
        copies = []
        for e in trace:
            if e[1] != "copy":
                continue
            t, _, voff, src, m0, at = e
            j = at // 128                                   # the k step during which it is issued
            want = j + 2 if j + 2 < kt else 0
            d = m0 - LDS_WAVE
            n = int(voff[-2])
            if voff.startswith("%[a_off"):
                assert src == A_BASE + 128 * want, ("A source", kt, j)
                assert d == (j % 2) * 32768 + 4096 * n, ("A target", kt, j)
                copies.append((t, ("A", j % 2), want if j + 2 < kt else None))
            else:
                assert src == B_BASE + B_STEP * want, ("B source", kt, j)
                assert d == 65536 + ((j + 2) % 3) * 32768 + 4096 * n, ("B target", kt, j)
                copies.append((t, ("B", (j + 2) % 3), want if j + 2 < kt else None))
        assert len(copies) == 16 * kt
        # the copies the C++ prologue issues before the block (complete, behind a barrier)
        landed = {("A", 0): 0, ("B", 0): 0}
        if kt > 1:
            landed.update({("A", 1): 1, ("B", 1): 1})
        # --- a copy has landed for every wavefront once a wait that leaves fewer copies
        # outstanding than were issued after it is followed by a barrier
        def landed_at(copy_index):
            t_issue = copies[copy_index][0]
            for e in trace:
                if e[1] == "wait" and e[2] is not None and e[0] > t_issue:
                    later = sum(1 for c in copies if t_issue < c[0] < e[0])
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
            h = -1 if at == 0 else (at - 1) // 64           # issued during slice h: a read of slice h + 1
            step, sl = (h + 1) // 2, (h + 1) % 2
            if reg.startswith("%[a_rd"):
                assert int(reg[-2]) == sl and off % 2048 == 0 and off % 32768 < 16384
                buf = ("A", off // 32768)
                assert buf[1] == step % 2
            else:
                full = off + (65536 if reg.startswith("%[b_rdh") else 0)
                assert full % 32768 in (sl * 16384, sl * 16384 + 2048)
                buf = ("B", full // 32768)
                assert buf[1] == step % 3
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
