"""Guards on the generated code of the decode kernel (no GPU needed).

The decode kernel issues its loads through hand-written instructions that the compiler does not
track (so that it places no wait for them inside the tile loop); the waits are explicit.  That is
only correct while the compiler never reads a destination register of such a load between the load
and the next wait - e.g. through a register-to-register copy that joins two definitions.  This test
compiles the file to assembly and checks exactly that, for every instantiation of the kernel
(and the same for the scalar loads of the table entries in the prologue of both decode kernels).
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _registers(text):
    used = set()
    for m in re.finditer(r"v\[(\d+):(\d+)\]", text):
        used.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        used.add(int(m.group(1)))
    return used


HAND = "  ;hand"        # suffix of an instruction that comes from an inline-assembly block


def _instructions(lines):
    """Instruction and label lines of a function, comments dropped; instructions between the
    compiler's markers of an inline-assembly block carry the suffix HAND.  The kernel's landing
    marks (an assembly comment `; landed <register>` right behind an explicit wait) are kept as
    pseudo-instructions `landed <register>`."""
    out, hand = [], False
    for raw in lines:
        if "#ASMSTART" in raw:
            hand = True
        elif "#ASMEND" in raw:
            hand = False
        m = re.match(r"\s*; landed (\S+)", raw)
        if hand and m:
            out.append("landed " + m.group(1) + HAND)
            continue
        l = raw.split(";")[0].strip()
        if l:
            out.append(l + HAND if hand else l)
    return out


def reads_of_inflight_registers(body):
    """(load line, offending line) pairs: instructions that touch (read or write) a destination
    register of a hand-written vector-memory load (one from an inline-assembly block, which the
    compiler neither sees nor waits for) before the place the source names as the point where the
    load has landed.

    The control-flow graph of the function is explored with a small abstract state:
      * the registers with such a load possibly outstanding - a hand-written load (or an atomic
        that returns a value) adds its destination; a landing mark (the kernel puts one right
        behind the explicit wait that covers the load) or a wait for all vector-memory operations
        removes it;
      * the 64-bit scalar flags the compiler's structurizer sets to -1 or 0 and branches on later
        (`s_mov_b64 s[a:b], -1` or `s_cselect_b64 s[a:b], -1, 0` ... `s_and_b64 vcc, exec, s[a:b]`
        ... `s_cbranch_vccz`), so that several branches on one flag are not taken in
        contradictory ways.
    States that differ are followed separately; every (instruction, state) pair is visited once.
    Whether the count of a partial wait is right is not checked here: that is the kernel's own
    bookkeeping, which the parity tests exercise."""
    n = len(body)
    hand = [l.endswith(HAND) for l in body]
    body = [l[:-len(HAND)] if l.endswith(HAND) else l for l in body]
    labels = {l[:-1]: i for i, l in enumerate(body) if l.endswith(":")}
    found = set()

    def first_operand_sgprs(line, op):
        first = line[len(op):].split(",")[0]
        regs = set(int(x) for x in re.findall(r"\bs(\d+)\b", first))
        for m in re.finditer(r"s\[(\d+):(\d+)\]", first):
            regs.update(range(int(m.group(1)), int(m.group(2)) + 1))
        return regs

    def step(i, state):
        """-> list of (next index, next state); state = (outstanding, flags, vcc)"""
        out_regs, flags, vcc = state
        line = body[i]
        op = line.split()[0]
        nxt = [i + 1] if i + 1 < n else []
        if op.endswith(":") or op.startswith("."):
            return [(j, state) for j in nxt]
        if op == "s_endpgm":
            return []
        if op == "s_waitcnt":
            if "vmcnt(0)" in line:
                out_regs = frozenset()
            return [(j, (out_regs, flags, vcc)) for j in nxt]
        if op == "landed":
            regs = _registers(line[len(op):])
            out_regs = frozenset(x for x in out_regs if x[0] not in regs)
            return [(j, (out_regs, flags, vcc)) for j in nxt]
        m = re.match(r"s_branch (\S+)$", line)
        if m:
            return [(labels[m.group(1)], state)]
        m = re.match(r"s_cbranch_(\w+) (\S+)$", line)
        if m:
            kind, target = m.group(1), labels[m.group(2)]
            # The lane mask can only be empty right behind an instruction that narrows it (the
            # compiler then skips the masked region with `s_cbranch_execz`).  Anywhere else - behind
            # the `s_or_b64 exec, exec, saved` that closes a region, or in a block that does not
            # write the mask - it is the non-empty mask the wave arrived with, and the branches
            # the structurizer puts there are decided: execz never taken, execnz always.
            narrowed = False
            for k in range(i - 1, -1, -1):      # the last write of the mask in this basic block
                if body[k].endswith(":") or body[k].startswith(("s_branch", "s_cbranch")):
                    break
                if re.search(r"\bexec\b", body[k].split(",")[0]) or "saveexec" in body[k] or body[k].startswith("v_cmpx"):
                    narrowed = not re.match(r"s_or_b64 exec, exec, s\[\d+:\d+\]$", body[k])
                    break
            if kind == "execz" and not narrowed:
                return [(j, state) for j in nxt]
            if kind == "execnz" and not narrowed:
                return [(target, state)]
            if kind in ("vccz", "vccnz") and isinstance(vcc, int):
                taken = (vcc == 0) == (kind == "vccz")
                return [(target, state)] if taken else [(j, state) for j in nxt]
            if kind in ("vccz", "vccnz") and vcc is not None:
                # vcc mirrors a flag whose value (-1 or 0) is not known yet: each way out of the
                # branch learns it
                key, same = vcc
                def learned(vcc_value):
                    val = vcc_value if same else -1 - vcc_value
                    fl = frozenset(f for f in flags if f[0] != key) | {(key, val)}
                    return (out_regs, fl, vcc_value)
                vcc_if_taken = 0 if kind == "vccz" else -1
                return [(target, learned(vcc_if_taken))] + [(j, learned(-1 - vcc_if_taken)) for j in nxt]
            return [(j, state) for j in nxt] + [(target, state)]
        # ordinary instruction: hazards first
        is_hand_load = hand[i] and op.startswith(("global_load", "global_atomic")) and not op.startswith("global_load_lds")
        # (a hand-written load may be issued again to the registers of one that is still
        # outstanding - an early request repeated with other addresses: loads return in order, the
        # later one wins - so only its address operands count as touched)
        touched = _registers(",".join(line[len(op):].split(",")[1:]) if is_hand_load else line[len(op):])
        for reg, k in out_regs:
            if reg in touched:
                found.add((body[k], line))
        if is_hand_load:
            dst = set()
            m = re.match(r"global_load_\w+ (v\[\d+:\d+\]|v\d+),", line)
            if m:
                dst = _registers(m.group(1))
            m = re.match(r"global_atomic_\w+ (v\d+), v", line)       # an atomic that returns a value
            if m and " sc0" in line:
                dst = _registers(m.group(1))
            out_regs = frozenset(x for x in out_regs if x[0] not in dst) | frozenset((r, i) for r in dst)
        # flags and vcc
        m = re.match(r"s_mov_b64 s\[(\d+):(\d+)\], (-1|0)$", line)
        m1 = re.match(r"s_cselect_b64 s\[(\d+):(\d+)\], (-1, 0|0, -1)$", line)
        m2 = re.match(r"s_(and|andn2)_b64 vcc, exec, s\[(\d+):(\d+)\]$", line)
        if m:
            key = (int(m.group(1)), int(m.group(2)))
            flags = frozenset(f for f in flags if f[0] != key) | {(key, int(m.group(3)))}
        elif m1:      # -1 or 0, not known which: "U"
            key = (int(m1.group(1)), int(m1.group(2)))
            flags = frozenset(f for f in flags if f[0] != key) | {(key, "U")}
        elif m2:
            key = (int(m2.group(2)), int(m2.group(3)))
            val = dict(flags).get(key)
            if val is None:
                vcc = None
            elif val == "U":
                vcc = (key, m2.group(1) == "and")
            else:
                vcc = val if m2.group(1) == "and" else -1 - val
        else:
            if "vcc" in line:
                vcc = None
            if flags:
                killed = first_operand_sgprs(line, op)
                if killed:
                    flags = frozenset(f for f in flags if not (set(range(f[0][0], f[0][1] + 1)) & killed))
        return [(j, (out_regs, flags, vcc)) for j in nxt]

    start = (0, (frozenset(), frozenset(), None))
    seen, work = {start}, [start]
    while work:
        i, state = work.pop()
        for nxt in step(i, state):
            if nxt not in seen:
                seen.add(nxt)
                work.append(nxt)
        assert len(seen) < 2000000, "state explosion"
    return sorted(found)


def reads_of_inflight_scalars(body):
    """The same for the hand-written scalar table loads (s_load_dword[x2] ..., 0x0 from a pointer other
    than the kernel-argument segment s[0:1]): reads of their destinations before the next
    s_waitcnt lgkmcnt(0)."""
    found, pending = [], set()
    for line in body:
        op = line.split()[0]
        if pending and "lgkmcnt(0)" in line:
            pending = set()
            continue
        if pending and not op.endswith(":") and not op.startswith("."):
            operands = line[len(op):].split(",")
            whole = op.startswith(("s_cmp", "s_cbranch", "s_bitcmp", "global_", "ds_write", "v_cmp"))
            reads = line[len(op):] if whole else ",".join(operands[1:])
            used = set(int(x) for x in re.findall(r"\bs(\d+)\b", reads))
            for m in re.finditer(r"s\[(\d+):(\d+)\]", reads):
                used.update(range(int(m.group(1)), int(m.group(2)) + 1))
            if used & pending:
                found.append(line)
        m = re.match(r"s_load_dword(x2)? (?:s(\d+)|s\[(\d+):(\d+)\]), s\[(\d+):\d+\], 0x0$", line)
        if m and m.group(5) != "0":
            if m.group(2) is not None:
                pending.add(int(m.group(2)))
            else:
                pending.update(range(int(m.group(3)), int(m.group(4)) + 1))
    return found


def test_checker_flags_a_copy_of_an_inflight_register():
    bad_s = ["s_load_dword s7, s[4:5], 0x0", "s_add_i32 s9, s7, 1", "s_waitcnt lgkmcnt(0)"]
    good_s = ["s_load_dword s7, s[4:5], 0x0", "s_add_i32 s9, s8, 1", "s_waitcnt lgkmcnt(0)",
              "s_add_i32 s9, s7, 1"]
    assert reads_of_inflight_scalars(bad_s) and not reads_of_inflight_scalars(good_s)
    H = lambda lines: [l + HAND if l.startswith(("global_", "landed")) else l for l in lines]
    check = lambda lines: reads_of_inflight_registers(H(lines))
    bad = ["global_load_dwordx4 v[8:11], v[2:3], off", "v_mov_b32_e32 v20, v9", "s_waitcnt vmcnt(0)"]
    good = ["global_load_dwordx4 v[8:11], v[2:3], off", "v_mov_b32_e32 v21, v20", "s_waitcnt vmcnt(0)",
            "ds_write_b128 v1, v[8:11]"]
    assert check(bad) and not check(good)
    assert not reads_of_inflight_registers(bad)          # a load the compiler knows about is its business
    # a partial wait covers what the landing marks behind it name, nothing else
    partial = ["global_load_dwordx4 v[8:11], v[2:3], off", "global_load_lds_dwordx4 v[4:5], off",
               "global_load_dwordx4 v[12:15], v[2:3], off", "s_waitcnt vmcnt(1)", "landed v[8:11]",
               "v_mov_b32_e32 v20, v9"]
    assert not check(partial)
    assert check(partial + ["v_mov_b32_e32 v21, v13"])
    assert check(partial[:4] + ["v_mov_b32_e32 v20, v9"])
    # overwriting a register whose load is outstanding is flagged as well
    assert check(["global_load_dwordx4 v[8:11], v[2:3], off", "v_mov_b32_e32 v9, v20"])
    # an atomic that returns a value is a load
    assert check(["global_atomic_add v7, v[4:5], v2, off sc0", "v_readfirstlane_b32 s0, v7"])
    assert not check(["global_atomic_add v7, v[4:5], v2, off sc0", "s_waitcnt vmcnt(0)", "landed v7",
                      "v_readfirstlane_b32 s0, v7"])
    # across the back-edge of a loop: loaded at the bottom of a pass, read at the top of the next
    loop = [".LBB0_1:", "v_add_f32_e32 v30, v30, v8", "s_waitcnt vmcnt(0)",
            "global_load_dwordx4 v[8:11], v[2:3], off", "s_cbranch_scc1 .LBB0_1", "s_waitcnt vmcnt(0)"]
    assert check(loop)
    assert not check([loop[0], loop[2], loop[1]] + loop[3:])
    # the two arms of a branch do not see each other's loads, the code behind the join sees both
    arms = ["s_cbranch_scc1 .LBB0_2", "global_load_dwordx4 v[8:11], v[2:3], off", "s_branch .LBB0_3",
            ".LBB0_2:", "v_mov_b32_e32 v8, 0", ".LBB0_3:", "s_waitcnt vmcnt(0)", "v_mov_b32_e32 v20, v8"]
    assert not check(arms)
    assert check(arms[:6] + ["v_mov_b32_e32 v20, v8"])
    # the marks survive the reading of the compiler's output
    got = _instructions(["\t;;#ASMSTART", "\ts_waitcnt vmcnt(4)", "\t;;#ASMEND", "\t;;#ASMSTART",
                         "\t; landed v[62:65]", "\t;;#ASMEND", "\tv_mov_b32_e32 v1, v62 ; comment"])
    assert got == ["s_waitcnt vmcnt(4)" + HAND, "landed v[62:65]" + HAND, "v_mov_b32_e32 v1, v62"]


def test_decode_kernel_never_reads_a_register_whose_load_is_in_flight(tmp_path):
    import __graft_entry__ as G
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc")
    src = os.path.join(ROOT, "paper_2510_13797_amd", "csrc", "bc_decode.hip")
    out = str(tmp_path / "bc_decode.s")
    flags = [f for f in G.HIPCC_FLAGS if f not in ("-shared", "-Wall")] + G.FILE_FLAGS.get("bc_decode.hip", [])
    subprocess.check_call([hipcc] + flags + ["-w", "-I", os.path.join(ROOT, "include"), "-S",
                                             "--cuda-device-only", src, "-o", out])
    text = open(out).read().split("\n")
    starts = [i for i, l in enumerate(text) if re.match(r"^_ZN2bc1[78]decode_(lds|valu)_kernel\w+:", l)]
    assert len(starts) >= 10 + 20
    for s in starts:
        e = next(i for i in range(s, len(text)) if text[i].startswith(".Lfunc_end"))
        marked = _instructions(text[s:e])
        body = [l[:-len(HAND)] if l.endswith(HAND) else l for l in marked]
        if "decode_lds_kernel" in text[s]:
            assert any(l.startswith("global_load_lds_dwordx4") for l in body)
            # M0 (the LDS address of a DMA load) is set by the hand-written sequence itself, right in
            # front of every such load, and nothing else in the kernel touches it
            for i, l in enumerate(body):
                if l.startswith("global_load_lds"):
                    assert body[i - 2].startswith("s_mov_b32 m0, s") and body[i - 1].startswith("s_nop"), body[i - 2:i + 1]
                elif re.search(r"\bm0\b", l):
                    assert l.startswith("s_mov_b32 m0, s"), l
            # the landing marks are there, each behind one of the explicit waits
            marks = [i for i, l in enumerate(body) if l.startswith("landed ")]
            assert len(marks) >= 6, text[s][:80]
            for i in marks:
                back = [l for l in body[max(0, i - 40):i] if not l.startswith("landed ")]
                assert any(l.startswith("s_waitcnt vmcnt(") for l in back[-24:]), (text[s][:80], body[i])
            assert not reads_of_inflight_registers(marked), (text[s][:80], reads_of_inflight_registers(marked)[:3])
        # the six table entries of the prologue (both kernels)
        assert sum(1 for l in body if re.match(r"s_load_dword(x2)? \S+ s\[(?!0:1)\d+:\d+\], 0x0$", l)) >= 6, text[s][:80]
        assert not reads_of_inflight_scalars(body), (text[s][:80], reads_of_inflight_scalars(body)[:3])
