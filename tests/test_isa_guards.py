"""Guards on the generated code of the decode kernel (no GPU needed).

The decode kernel issues its loads through hand-written instructions that the compiler does not
track (so that it places no wait for them inside the tile loop); the waits are explicit.  That is
only correct while the compiler never reads a destination register of such a load between the load
and the next wait - e.g. through a register-to-register copy that joins two definitions.  This test
compiles the file to assembly and checks exactly that, for every instantiation of the kernel.
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


def test_checker_flags_a_copy_of_an_inflight_register():
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
    starts = [i for i, l in enumerate(text) if re.match(r"^_ZN2bc17decode_lds_kernel\w+:", l)]
    assert len(starts) >= 13
    for s in starts:
        e = next(i for i in range(s, len(text)) if text[i].startswith(".Lfunc_end"))
        body = [l.strip() for l in text[s:e] if l.strip() and not l.strip().startswith(";")]
        assert any(l.startswith("global_load_lds_dwordx4") for l in body)
        assert not reads_of_inflight_registers(body), (text[s][:80], reads_of_inflight_registers(body)[:3])
