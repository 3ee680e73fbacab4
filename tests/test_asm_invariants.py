"""Structural checks of compiled kernels (no GPU needed): the streaming GEMM's hand-counted
waits, and the split-K hand-over of the projection's partial sums.

The kernel issues its ring loads as inline assembly and waits for them with hand-counted
`s_waitcnt vmcnt(N)`.  That is only correct while the compiler (a) adds no vector-memory
operation of its own to the loop, (b) never copies a ring register between its load and its
wait, and (c) does not hand a register of a load still in flight to other code behind the loop.
These properties are read off the generated assembly."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2605_00422_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# (channel tiles per wavefront, wavefronts along the tokens, wavefronts along K, ring depth) of
# every instantiation that is launched
# every instantiation that is launched; the last entry: codes nibble-packed (4 code copies per slice instead of 8)
SHAPES = [(1, 1, 1, 4), (1, 1, 4, 4), (2, 1, 4, 4), (4, 4, 1, 4), (5, 4, 1, 4), (4, 4, 1, 2), (2, 1, 2, 4), (5, 1, 1, 4)]
VARIANTS = [(*v, a4) for a4 in (0, 1) for v in SHAPES]


@pytest.fixture(scope="module")
def kernels():
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "gemm_prefill.s")
        cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-w", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only",
               "-o", out, os.path.join(CSRC, "gemm_prefill.hip")]
        subprocess.run(cmd, check=True, capture_output=True)
        text = open(out).read().split("\n")
    found = {}
    for ntl, wm, wk, nb, a4 in VARIANTS:
        # (the two trailing template arguments: not gated, nibble-packed or not)
        pat = re.compile(rf"^_ZN.*gemm_prefill_direct_kernelILi{ntl}ELi{wm}ELi{wk}ELi{nb}ELb0ELb{a4}E.*:")
        start = next(i for i, l in enumerate(text) if pat.match(l))
        end = next(i for i in range(start, len(text)) if "s_endpgm" in text[i])
        found[(ntl, wm, wk, nb, a4)] = text[start:end + 1]
    return found


def _main_loop(lines):
    start = next(i for i, l in enumerate(lines) if "Loop Header" in l)
    label = lines[start].split(":")[0].strip()
    end = next(i for i in range(start + 1, len(lines)) if re.search(rf"s_cbranch\S*\s+{re.escape(label)}$", lines[i]))
    return start, end


@pytest.mark.parametrize("ntl,wm,wk,nb,a4", VARIANTS)
def test_streaming_gemm_loop_structure(kernels, ntl, wm, wk, nb, a4):
    lines = kernels[(ntl, wm, wk, nb, a4)]
    copies = 4 if a4 else 8
    start, end = _main_loop(lines)
    loop = lines[start:end + 1]
    code = [l.strip() for l in loop if l.strip() and not l.strip().startswith((";", "."))]
    # nb slices per trip: nb x (NTL weight loads + 8 asynchronous code copies), nb x 4 x 2 NTL MFMAs
    assert sum(l.startswith("global_load_lds_dwordx4") for l in code) == copies * nb
    assert sum(l.startswith("global_load_dwordx4") for l in code) == nb * ntl
    assert sum(l.startswith("v_mfma_i32_32x32x32_i8") for l in code) == nb * 4 * 2 * ntl
    # the only vector-memory waits are the hand-counted ones, with the documented count
    waits = [l for l in code if l.startswith("s_waitcnt") and "vmcnt" in l]
    assert waits == [f"s_waitcnt vmcnt({(nb - 2) * (ntl + copies)})"] * nb
    # no other memory traffic and no register shuffling of ring or accumulator registers
    assert not any(l.startswith(("scratch_", "global_store", "buffer_", "flat_")) for l in code)
    assert not any(l.startswith(("v_mov_b32", "v_accvgpr")) for l in code)


@pytest.mark.parametrize("ntl,wm,wk,nb,a4", VARIANTS)
def test_registers_of_loads_in_flight_stay_reserved(kernels, ntl, wm, wk, nb, a4):
    lines = kernels[(ntl, wm, wk, nb, a4)]
    start, end = _main_loop(lines)
    dest = set()
    for l in lines[start:end]:
        m = re.match(r"\s*global_load_dwordx4 v\[(\d+):(\d+)\]", l)
        if m:
            dest.update(range(int(m.group(1)), int(m.group(2)) + 1))
    assert len(dest) == 4 * nb * ntl
    drain = next(i for i in range(end, len(lines)) if "s_waitcnt vmcnt(0)" in lines[i])
    for l in lines[end + 1:drain]:
        l = l.strip()
        if not l or l.startswith((";", ".", "s_", "global_store", "ds_write", "scratch_store")):
            continue
        m = re.match(r"\S+\s+v\[(\d+):(\d+)\]", l) or re.match(r"\S+\s+v(\d+)()", l)
        if m:
            lo = int(m.group(1))
            hi = int(m.group(2)) if m.group(2) else lo
            assert not any(r in dest for r in range(lo, hi + 1)), f"writes a register of a load in flight: {l}"


def _device_asm(src):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "out.s")
        cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-w", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-S", "--cuda-device-only",
               "-o", out, os.path.join(CSRC, src)]
        subprocess.run(cmd, check=True, capture_output=True)
        return [l.strip() for l in open(out).read().split("\n")]


@pytest.mark.parametrize("src,min_sites", [("psp_prefill.hip", 1), ("rotate_quant.hip", 2)])
def test_partial_sums_are_acknowledged_before_the_arrival_count(src, min_sites):
    """The workgroup that arrives last at the counter reads the other workgroups' partial tiles.
    Nothing but an explicit wait orders a workgroup's device-scope stores before its counter bump
    (a workgroup-scope fence emits none), so between the last such store and the returning atomic
    add there must be: a wait for all vector-memory operations, then the barrier, then the add."""
    lines = _device_asm(src)
    sites = 0
    for i, l in enumerate(lines):
        if not (l.startswith("global_atomic_add") and l.endswith("sc0")):
            continue                                   # (adds without return value are code sums)
        bar = next(j for j in range(i, 0, -1) if lines[j] == "s_barrier")
        st = next((j for j in range(bar, max(bar - 400, 0), -1)
                   if lines[j].startswith("global_store_dword") and lines[j].endswith("sc1")), None)
        if st is None:
            continue
        sites += 1
        waits = [j for j in range(st + 1, bar) if lines[j].startswith("s_waitcnt") and "vmcnt(0)" in lines[j]]
        assert waits, f"{src}: no vmcnt(0) wait between the partial stores (line {st}) and the barrier (line {bar})"
        assert not any(lines[j].startswith("global_store") for j in range(waits[-1], bar))
    assert sites >= min_sites
