"""Generated-code check for the loads whose data is thrown away (load16_discard: idle workgroups pull the next
launch's weights and the old K,V blocks into the L2).  They write to LDS, not to registers: a register that waits for
a load must be kept away from the register allocator until the data is back, and an earlier form with a register
destination had that register handed to the next address computation while the load was still on its way (wild
addresses).  What remains to be guaranteed is that the workgroup still owns its LDS when the data arrives: on every
path from such a load to the end of the program there must be a wait for all outstanding loads."""
import os
import re
import shutil

import pytest

from paper_2512_15176_amd import build


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
def test_every_discarded_load_is_waited_for_before_the_program_ends(tmp_path):
    text = open(build.device_assembly(str(tmp_path / "deer_device.s"))).read().split("\n")
    starts = [i for i, l in enumerate(text) if re.match(r"^_ZN4deer\w+:", l)]
    kernels = 0
    for s in starts:
        e = next(i for i in range(s, len(text)) if text[i].startswith(".Lfunc_end"))
        body = text[s:e]
        marks = [i for i, l in enumerate(body) if "; fetch ahead" in l]
        if not marks:
            continue
        kernels += 1
        labels = {m.group(1): i for i, l in enumerate(body) for m in [re.match(r"^(\.LBB\w+):", l)] if m}
        for i in marks:
            # the statement behind the marker is a load to LDS, with no register destination
            nxt = next(l for l in body[i + 1:] if "global_load" in l)
            assert "global_load_lds_dwordx4" in nxt, (text[s], nxt)
            todo, seen = [i + 1], set()
            while todo:
                j = todo.pop()
                while j not in seen and j < len(body):
                    seen.add(j)
                    line = body[j].split(";")[0].strip() if not body[j].lstrip().startswith(";") else ""
                    if "s_waitcnt vmcnt(0)" in line:
                        break
                    assert "s_endpgm" not in line, (text[s], "a discarded load is not waited for")
                    m = re.match(r"s_(c?branch)\w*\s+(\.LBB\w+)", line)
                    if m:
                        todo.append(labels[m.group(2)])
                        if m.group(1) == "branch":
                            break
                    j += 1
    # the split GEMMs (QKV, O / down projections, each in several instantiations) and per-head attention fetch ahead
    assert kernels >= 6
