"""Static check of the fused kernel's machine code (no GPU needed).

The fused multi-round kernel moves its tiles between HBM and its slot registers
with asm statements that the compiler does not track, and waits for them itself
(one `s_waitcnt vmcnt(0)` before the registers are used).  That is only correct if
the compiler never reads, copies or overwrites a slot register between the load
that targets it and that wait.  This test compiles the kernel file to gfx950
assembly with the library's flags and checks every instantiation:

* no instruction uses a register that has a load pending (linear scan);
* in the steady-state loop (everything after the first tile has entered LDS) the
  slot registers appear only as load destinations and as data of the stores to
  HBM until the wait; the swap with LDS (and any register copies) come after it;
* every slot's store to HBM precedes the load into the same register;
* no kernel uses scratch memory (a spill would count as vector memory traffic and
  serialise the loads).

The counts below follow from the kernel's constant kPrefetch (slots per thread),
read from the source.  A toolchain change that breaks any of this fails here; the
fused-versus-single-round bit-identity tests on the GPU are the gate behind it.
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


STORE = re.compile(r"global_store_dwordx4 v\[(\d+):(\d+)\], v\[(\d+):(\d+)\]")


def test_prefetch_registers_untouched_until_the_wait(tmp_path):
    if shutil.which(HIPCC) is None and not os.path.exists(HIPCC):
        pytest.fail("hipcc is needed: the fused kernel's untracked loads must be checked in the machine code")
    src = open(os.path.join(entry.CSRC, "fused_rounds.hip")).read()
    slots = int(re.search(r"constexpr int kPrefetch = (\d+);", src).group(1))
    variants = len(re.findall(r"fused_rounds_kernel<DT, \w+, \d, \d, \d, BPC>", src))
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
        loads = [i for i, l in enumerate(K) if "global_load_dwordx4" in l]
        stores = [i for i, l in enumerate(K) if "global_store_dwordx4" in l]
        # one load per slot for the first tile and one in the loop; one store per slot in the
        # loop and one for the last tile
        assert len(loads) == 2 * slots, f"{name}: expected two groups of {slots} slot loads, found {len(loads)}"
        assert len(stores) == 2 * slots, f"{name}: expected two groups of {slots} slot stores, found {len(stores)}"
        pre: set[int] = set()
        for i in loads:
            m = LOAD.search(K[i])
            assert m, K[i]
            pre.update(range(int(m.group(1)), int(m.group(2)) + 1))
        assert len(pre) == 4 * slots, f"{name}: slot registers are not the same in both places"
        for i in stores[:slots]:                    # the loop's stores send slot registers
            m = STORE.search(K[i])
            assert m and set(range(int(m.group(3)), int(m.group(4)) + 1)) <= pre, f"{name}: {K[i].strip()}"
        # (a) linear scan: nothing touches a register whose load is pending
        pending: set[int] = set()
        for l in K:
            m = LOAD.search(l)
            if m:
                assert not (set(range(int(m.group(3)), int(m.group(4)) + 1)) & pending), f"{name}: {l}"
                pending.update(range(int(m.group(1)), int(m.group(2)) + 1))
            elif "s_waitcnt vmcnt(0)" in l:
                pending = set()
            else:
                assert not (_regs(l) & pending), f"{name}: touches a pending slot register: {l.strip()}"
        # (b) steady state: from the barrier after the first tile's LDS writes to the end
        w0 = next(i for i in range(loads[slots - 1], len(K)) if "s_waitcnt vmcnt(0)" in K[i])
        b0 = next(i for i in range(w0, len(K)) if "s_barrier" in K[i])
        w1 = max(i for i in range(len(K)) if "s_waitcnt vmcnt(0)" in K[i])
        assert w1 > loads[-1], f"{name}: no wait after the loop's slot loads"
        # the rounds of a tile run between b0 and w1, over and over, with loads pending: there the
        # slot registers may appear in the slot loads and stores only
        for i in range(b0, w1):
            if not (_regs(K[i]) & pre) or "global_load_dwordx4" in K[i] or "global_store_dwordx4" in K[i]:
                continue
            raise AssertionError(f"{name}: line {i} touches a slot register inside the tile loop: {K[i].strip()}")
        assert stores[slots] > w1, f"{name}: the last tile's stores must follow the loop"
        # (c) in the loop a slot's store comes before the load into the same registers
        loop_loads = {int(LOAD.search(K[i]).group(1)): i for i in loads[slots:]}
        loop_stores = {int(STORE.search(K[i]).group(3)): i for i in stores[:slots]}
        assert set(loop_loads) == set(loop_stores), f"{name}: loop stores and loads use different registers"
        for reg, at in loop_loads.items():
            assert loop_stores[reg] < at, f"{name}: load into v{reg} precedes the store of its old content"
