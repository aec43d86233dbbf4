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


def reads_of_inflight_registers(body):
    """(load line, reader line) pairs: instructions after a register load and before the next vmcnt
    wait (in program order) that read the load's destination registers."""
    found = []
    for i, line in enumerate(body):
        m = re.match(r"global_load_dwordx4 v\[(\d+):(\d+)\],", line)
        if not m:
            continue
        dst = set(range(int(m.group(1)), int(m.group(2)) + 1))
        for later in body[i + 1:]:
            if "vmcnt" in later:
                break
            op = later.split()[0]
            if op.startswith(".") or op.endswith(":"):
                continue
            operands = later[len(op):].split(",")
            all_read = op.startswith(("ds_write", "global_store", "global_load_lds", "global_atomic"))
            reads = ",".join(operands if all_read else operands[1:])
            if _registers(reads) & dst:
                found.append((line, later))
    return found


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
    good_s = ["s_load_dword s7, s[4:5], 0x0", "s_add_i32 s7, s9, 1"[:0] + "s_add_i32 s9, s8, 1", "s_waitcnt lgkmcnt(0)",
              "s_add_i32 s9, s7, 1"]
    assert reads_of_inflight_scalars(bad_s) and not reads_of_inflight_scalars(good_s)
    bad = ["global_load_dwordx4 v[8:11], v[2:3], off", "v_mov_b32_e32 v20, v9", "s_waitcnt vmcnt(0)"]
    good = ["global_load_dwordx4 v[8:11], v[2:3], off", "v_mov_b32_e32 v9, v20", "s_waitcnt vmcnt(0)",
            "ds_write_b128 v1, v[8:11]"]
    assert reads_of_inflight_registers(bad) and not reads_of_inflight_registers(good)


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
    assert len(starts) >= 13 + 20
    for s in starts:
        e = next(i for i in range(s, len(text)) if text[i].startswith(".Lfunc_end"))
        body = [l.strip() for l in text[s:e] if l.strip() and not l.strip().startswith(";")]
        if "decode_lds_kernel" in text[s]:
            assert any(l.startswith("global_load_lds_dwordx4") for l in body)
            # M0 (the LDS address of a DMA load) is set by the hand-written sequence itself, right in
            # front of every such load, and nothing else in the kernel touches it
            for i, l in enumerate(body):
                if l.startswith("global_load_lds"):
                    assert body[i - 2].startswith("s_mov_b32 m0, s") and body[i - 1].startswith("s_nop"), body[i - 2:i + 1]
                elif re.search(r"\bm0\b", l):
                    assert l.startswith("s_mov_b32 m0, s"), l
            assert not reads_of_inflight_registers(body), (text[s][:80], reads_of_inflight_registers(body)[:3])
        # the six table entries of the prologue (both kernels)
        assert sum(1 for l in body if re.match(r"s_load_dword(x2)? \S+ s\[(?!0:1)\d+:\d+\], 0x0$", l)) >= 6, text[s][:80]
        assert not reads_of_inflight_scalars(body), (text[s][:80], reads_of_inflight_scalars(body)[:3])
