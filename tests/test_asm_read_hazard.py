"""Build-time guard for the kernels that issue LDS reads as inline assembly (the compiler takes such a statement's output
as valid at once; the hardware delivers it later).  Nothing may read, copy or overwrite a result register between the
read and the `s_waitcnt lgkmcnt` that covers it.  The check compiles the two kernels to gfx950 assembly and walks the
listing in order (branches are not followed: the listing order visits every instruction once, and LDS reads complete in
issue order, so a wait for "at most n outstanding" releases all but the n youngest reads)."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2111_09389_amd", "csrc")


def _regs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def _violations(listing):
    pending, reads, bad = {}, 0, []
    for no, line in enumerate(listing.splitlines(), 1):
        t = line.strip()
        if not t or t[0] in ";.":
            continue
        if t.startswith("s_waitcnt") and "lgkmcnt" in t:
            n = int(re.search(r"lgkmcnt\((\d+)\)", t).group(1))
            order = sorted(set(pending.values()))
            keep = set(order[-n:]) if n > 0 else set()
            pending = {r: at for r, at in pending.items() if at in keep}
            continue
        if t.startswith("ds_read_b64_tr_b8"):
            reads += 1
            for r in _regs(t.split()[1]):
                pending[r] = no
            continue
        if t.startswith("s_"):
            continue
        if _regs(t) & set(pending):
            bad.append((no, t))
    return reads, bad


@pytest.mark.parametrize("source", ["qconv_wgrad_rows.hip", "qconv_wgrad_gemm.hip"])
def test_nothing_touches_an_assembly_lds_read_before_its_wait(tmp_path, source):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    out = tmp_path / (source + ".s")
    cmd = [hipcc, "-x", "hip", "-S", "--cuda-device-only", os.path.join(CSRC, source), "-o", str(out), "--offload-arch=gfx950", "-O3",
           "-std=c++17", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    subprocess.run(cmd, check=True, capture_output=True)
    reads, bad = _violations(out.read_text())
    assert reads > 0, "the kernel no longer issues its transposing reads as assembly: this guard checks nothing"
    assert not bad, bad[:5]


def test_the_checker_sees_a_planted_copy():
    listing = """
	ds_read_b64_tr_b8 v[4:5], v9
	ds_read_b64_tr_b8 v[6:7], v9 offset:256
	v_mov_b32_e32 v20, v6
	s_waitcnt lgkmcnt(0)
	v_mfma_i32_32x32x32_i8 v[32:47], v[4:7], v[10:13], v[32:47]
"""
    reads, bad = _violations(listing)
    assert reads == 2 and len(bad) == 1 and "v_mov_b32" in bad[0][1]
    ok = listing.replace("	v_mov_b32_e32 v20, v6\n", "")
    assert _violations(ok) == (2, [])
    # a wait that leaves the youngest read outstanding releases only the older one
    partial = listing.replace("s_waitcnt lgkmcnt(0)", "s_waitcnt lgkmcnt(1)").replace("	v_mov_b32_e32 v20, v6\n", "")
    reads, bad = _violations(partial)
    assert len(bad) == 1 and "v_mfma" in bad[0][1]


def _full_waits_between_loads_and_products(listing):
    """(function, line) of every `s_waitcnt vmcnt(0)` that stands, in listing order, between a direct-to-LDS load and the
    next matrix instruction with no barrier after it: such a wait takes the loads that were meant to stay in flight out
    of flight.  (The designed wait of a pipeline step is followed by the step's barrier, and the loads of the following
    step are issued after that.)"""
    func, after_load, waits, found = None, False, [], []
    for no, line in enumerate(listing.splitlines(), 1):
        m = re.match(r"^(_Z\w+):", line)
        if m:
            func, after_load, waits = m.group(1), False, []
            continue
        t = line.strip()
        if t.startswith("buffer_load") and t.endswith("lds"):
            after_load = True
        elif t.startswith("s_barrier"):
            after_load, waits = False, []
        elif t.startswith("v_mfma"):
            found += waits
            after_load, waits = False, []
        elif after_load and t.startswith("s_waitcnt") and re.search(r"vmcnt\(0\)", t):
            waits.append((func, no))
    return found


@pytest.mark.parametrize("source", ["qconv_patch.hip", "qconv_wgrad_rows.hip", "qconv_wgrad_gemm.hip", "qconv_igemm_dma.hip"])
def test_no_full_wait_between_direct_to_lds_loads_and_the_products_they_run_under(tmp_path, source):
    """A performance guard, not a correctness one: the kernels that load operands straight into LDS keep the loads of the
    following steps in flight under the products of the current one.  The compiler's own wait insertion has broken that
    three times (an inline-assembly wait it could not see, a transposing-read builtin without alias information); each
    showed up as a `vmcnt(0)` between the loads and the next matrix instruction."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    out = tmp_path / (source + ".s")
    cmd = [hipcc, "-x", "hip", "-S", "--cuda-device-only", os.path.join(CSRC, source), "-o", str(out), "--offload-arch=gfx950", "-O3",
           "-std=c++17", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    subprocess.run(cmd, check=True, capture_output=True)
    listing = out.read_text()
    assert "lds" in listing and "v_mfma" in listing
    assert _full_waits_between_loads_and_products(listing) == []


def test_the_performance_guard_sees_a_planted_wait():
    good = """
_Zkernel:
	s_waitcnt vmcnt(3) lgkmcnt(0)
	s_barrier
	buffer_load_dwordx4 v2, s[24:27], 0 offen lds
	ds_read_b128 v[4:7], v9
	v_mfma_i32_32x32x32_i8 v[32:47], v[4:7], v[10:13], v[32:47]
	buffer_load_dwordx4 v2, s[24:27], 0 offen lds
	s_waitcnt vmcnt(0)
	s_barrier
"""
    assert _full_waits_between_loads_and_products(good) == []
    bad = good.replace("	ds_read_b128 v[4:7], v9\n", "	s_waitcnt vmcnt(0)\n	ds_read_b128 v[4:7], v9\n")
    assert _full_waits_between_loads_and_products(bad) == [("_Zkernel", 6)]
