"""The explicit 128-bit device-scope loads of RowAgent128 are not counted by the compiler's
own wait insertion: the kernel waits for them itself (P::wait_all) before the first use
(P::settle).  That discipline only holds if the compiler puts no instruction that touches a
load's destination registers between the load and the wait -- no copy, no spill.  The explicit
128-bit stores likewise carry their own two wait states (s_nop 1), which the compiler cannot add
to an instruction it does not see.  This test
compiles the two translation units that instantiate the SGD kernel to assembly (device pass
only, no GPU needed) and checks exactly that, for every RowAgent128 instantiation."""
import os
import re
import subprocess

import pytest

from paper_2008_12336_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def registers(token):
    m = re.match(r"v\[(\d+):(\d+)\]$", token)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", token)
    return {int(m.group(1))} if m else set()


def violations(path):
    """(kernels checked, explicit loads seen, list of offending lines) for one .s file."""
    kernels = loads = 0
    bad = []
    inside = False
    pending = {}
    stores = []  # line of the last explicit store while its s_nop has not been seen, else None
    for number, line in enumerate(open(path), 1):
        text = line.strip()
        m = re.match(r"^(_ZN4gosh10sgd_kernel\S*):", text)
        if m:
            inside = "RowAgent128" in m.group(1)
            kernels += inside
            pending = {}
            continue
        if not inside or not text or text[0] in ";." or re.match(r"^\.?LBB", text):
            continue
        op = text.split()[0]
        if op == "s_endpgm":
            pending = {}
            continue
        tokens = re.findall(r"v\[\d+:\d+\]|v\d+", text)
        if op == "global_store_dwordx4" and " sc1" in text:
            stores.append(number)
            continue
        if stores and stores[-1] is not None and op != "s_nop":
            bad.append(f"{os.path.basename(path)}:{number}: explicit store not followed by its wait states: {text}")
            stores[-1] = None
            continue
        if op == "s_nop" and stores and stores[-1] is not None:
            if text.split()[1] != "1":
                bad.append(f"{os.path.basename(path)}:{number}: {text} after an explicit 128-bit store (two wait states are needed)")
            stores[-1] = None
            continue
        if op == "global_load_dwordx4" and " sc1" in text:
            loads += 1
            for reg in registers(tokens[0]):
                pending[reg] = number
            continue
        if op == "s_waitcnt" and "vmcnt(0)" in text:
            pending = {}
            continue
        used = set()
        for token in tokens:
            used |= registers(token)
        if used & set(pending):
            bad.append(f"{os.path.basename(path)}:{number}: {text}")
    return kernels, loads, bad


@pytest.mark.timeout(900)
def test_nothing_touches_an_explicit_load_before_its_wait(tmp_path):
    jobs = []
    for unit in ("gosh_train.hip", "gosh_parts.hip"):
        out = str(tmp_path / (unit + ".s"))
        flags = [f for f in B.FLAGS if f not in ("-shared", "-fPIC")]
        cmd = [B.hipcc(), *flags, "--cuda-device-only", "-S", "-I" + os.path.join(ROOT, "include"), "-I" + B.CSRC,
               "-x", "hip", os.path.join(B.CSRC, unit), "-o", out]
        jobs.append((out, subprocess.Popen(cmd, stdout=subprocess.DEVNULL, stderr=subprocess.PIPE)))
    total_kernels = total_loads = 0
    for out, job in jobs:
        _, err = job.communicate()
        assert job.returncode == 0, err.decode()[-2000:]
        kernels, loads, bad = violations(out)
        assert not bad, "\n".join(bad[:20])
        total_kernels += kernels
        total_loads += loads
    # epoch work with 32- and 64-bit offsets and pair work, concurrent and sequential, five group sizes
    assert total_kernels >= 30 and total_loads >= 5 * total_kernels
