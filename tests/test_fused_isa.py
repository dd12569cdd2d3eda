"""Static check of the fused kernel's machine code (no GPU needed).

The fused multi-round kernel issues its tile prefetch as asm statements that the
compiler does not track, and waits for them itself (one `s_waitcnt vmcnt(0)`
before the registers are used).  That is only correct if the compiler never
reads, copies or overwrites a prefetch register between the load that targets it
and that wait.  This test compiles the kernel file to gfx950 assembly with the
library's flags and checks every instantiation:

* no instruction uses a register that has a prefetch load pending (linear scan);
* in the steady-state loop (everything after the first tile has entered LDS) the
  prefetch registers appear only as load destinations and as sources of the LDS
  writes that follow the wait;
* no kernel uses scratch memory (a spill would count as vector memory traffic and
  serialise the prefetch).

The expected counts follow from the kernel's constant kPrefetch, read from the
source.  A toolchain change that breaks any of this fails here (also when hipcc is
missing: the check must not be skipped silently); behind it, the GPU tests that
compare fused passes with single rounds bit for bit are the gate for any compiler
change.
"""
import os
import re
import shutil
import subprocess

import pytest

import __graft_entry__ as entry

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _regs(line: str) -> set[int]:
    body = line.split(";")[0]
    out: set[int] = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", body):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", body):
        out.add(int(m.group(1)))
    return out


LOAD = re.compile(r"global_load_dwordx4 v\[(\d+):(\d+)\], v\[(\d+):(\d+)\]")


def test_prefetch_registers_untouched_until_the_wait(tmp_path):
    if shutil.which(HIPCC) is None and not os.path.exists(HIPCC):
        pytest.fail("hipcc is needed: the fused kernel's untracked prefetch loads must be checked in the machine code")
    src = open(os.path.join(entry.CSRC, "fused_rounds.hip")).read()
    slots = int(re.search(r"constexpr int kPrefetch = (\d+);", src).group(1))      # prefetch registers per thread
    variants = 2 * len(re.findall(r"fused_rounds_kernel<DT, \w+, \d, \d, \d, BPC>", src))   # x 2 storage types
    asm = tmp_path / "fused_rounds.s"
    flags = [f for f in entry.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    subprocess.check_call([HIPCC, *flags, "-I", os.path.join(entry.ROOT, "include"), "-S", "--cuda-device-only",
                           os.path.join(entry.CSRC, "fused_rounds.hip"), "-o", str(asm)],
                          stderr=subprocess.DEVNULL)
    text = asm.read_text().split("\n")
    starts = [i for i, l in enumerate(text) if re.match(r"^_ZN7moshpit.*fused_rounds_kernel.*:", l)]
    assert len(starts) >= variants, "expected every instantiation of the fused kernel in the assembly"
    for s in starts:
        e = s
        while "s_endpgm" not in text[e]:
            e += 1
        K = text[s:e + 1]
        name = text[s].split(":")[0]
        assert not any("scratch_" in l for l in K), f"{name}: uses scratch memory"
        # the prefetch loads are the asm statements (the compiler marks them); its own, tracked
        # 128-bit loads (gradients of a Moshpit SGD pass) are waited for by the compiler
        loads = [i for i, l in enumerate(K) if "global_load_dwordx4" in l and "#ASMSTART" in K[i - 1]]
        tracked = [i for i, l in enumerate(K) if "global_load_dwordx4" in l and "#ASMSTART" not in K[i - 1]]
        # one load per slot for the first tile, one before the rounds of a tile, one spread over its rounds
        assert len(loads) == 3 * slots, f"{name}: expected three groups of {slots} prefetch loads"
        pre: set[int] = set()
        for i in loads:
            m = LOAD.search(K[i])
            assert m, K[i]
            pre.update(range(int(m.group(1)), int(m.group(2)) + 1))
        assert len(pre) == 4 * slots, f"{name}: prefetch registers are not the same in both places"
        # (a) linear scan: nothing touches a register whose load is pending
        pending: set[int] = set()
        for li, l in enumerate(K):
            m = LOAD.search(l)
            if m and li in tracked:
                assert not (_regs(l) & pending), f"{name}: a tracked load touches a pending prefetch register: {l.strip()}"
            elif m:
                assert not (set(range(int(m.group(3)), int(m.group(4)) + 1)) & pending), f"{name}: {l}"
                pending.update(range(int(m.group(1)), int(m.group(2)) + 1))
            elif "s_waitcnt vmcnt(0)" in l:
                pending = set()
            else:
                assert not (_regs(l) & pending), f"{name}: touches a pending prefetch register: {l.strip()}"
        # (b) steady state: from the barrier after the first tile's LDS writes to the end
        w0 = next(i for i in range(loads[slots - 1], len(K)) if "s_waitcnt vmcnt(0)" in K[i])
        b0 = next(i for i in range(w0, len(K)) if "s_barrier" in K[i])
        w1 = next((i for i in range(loads[-1], len(K)) if "s_waitcnt vmcnt(0)" in K[i]), None)
        assert w1 is not None, f"{name}: no wait after the loop's prefetch loads"
        for i in range(b0, len(K)):
            if not (_regs(K[i]) & pre) or i in loads:
                continue
            assert "ds_write_b128" in K[i] and i > w1, f"{name}: line {i}: {K[i].strip()}"
