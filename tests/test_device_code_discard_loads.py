"""Generated-code check for the loads whose data is thrown away (load16_discard: they pull the next launch's
weights and the old K,V blocks into the L2).  Such a load writes its destination registers when it RETURNS, long
after it was issued; if the compiler hands those registers to anything else in the meantime (it did, to the next
address computation, when the destination was a write-only operand), the returning data corrupts that value and the
next load goes to a wild address.  The statement therefore reads and writes one reserved register group; this test
reads the compiler's assembly and checks that between every such load and the wait that follows it no other
instruction names a register of that group."""
import os
import re
import shutil

import pytest

from paper_2512_15176_amd import build


def _regs(line):
    out = set()
    for m in re.finditer(r"\bv(\d+)\b", line):
        out.add(int(m.group(1)))
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", line):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    return out


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_nothing_touches_a_discarded_loads_registers_before_the_wait(tmp_path):
    text = open(build.device_assembly(str(tmp_path / "deer_device.s"))).read().split("\n")
    starts = [i for i, l in enumerate(text) if re.match(r"^_ZN4deer\w+:", l)]
    kernels_with_discards = 0
    for s in starts:
        e = next(i for i in range(s, len(text)) if text[i].startswith(".Lfunc_end"))
        body = text[s:e]
        loads = [i for i, l in enumerate(body) if "global_load_dwordx4" in l and "; discard" in l]
        if not loads:
            continue
        kernels_with_discards += 1
        labels = {m.group(1): i for i, l in enumerate(body) for m in [re.match(r"^(\.LBB\w+):", l)] if m}
        for i in loads:
            sink = _regs(body[i].split(",")[0])
            assert len(sink) == 4
            # every path from the load to the wait behind it (branches followed, both ways where conditional)
            todo, seen = [i + 1], set()
            while todo:
                j = todo.pop()
                while j not in seen:
                    seen.add(j)
                    line = body[j].split(";")[0].strip() if not body[j].lstrip().startswith(";") else ""
                    if "s_waitcnt vmcnt(0)" in line:
                        break
                    assert "s_endpgm" not in line, (text[s], "a discarded load is not waited for")
                    if j not in loads and line and not line.startswith("."):
                        assert not (_regs(line) & sink), (text[s], body[i].strip(), line)
                    m = re.match(r"s_(c?branch)\w*\s+(\.LBB\w+)", line)
                    if m:
                        todo.append(labels[m.group(2)])
                        if m.group(1) == "branch":
                            break
                    j += 1
    # the split GEMMs (QKV, O / down projections, each in several instantiations) and per-head attention fetch ahead
    assert kernels_with_discards >= 6
