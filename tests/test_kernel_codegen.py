"""Properties of the compiled gfx950 code that the kernels' timing rests on and that a change
elsewhere in the source can silently undo (the compiler decides them, not the source text).

The device code of the library is compiled to assembly text (no GPU needed, about half a minute) and
read as text:

* the GEMM kernels that feed B fragments through LDS issue their global -> LDS transfers from
  assembly statements the compiler cannot see.  A wait for outstanding vector memory operations that
  the compiler places BETWEEN two such transfers (for a load of its own that it moved up) makes the
  wave wait for every transfer in turn; the kernels start their filling code with a wait the compiler
  does see, so that it has nothing left to wait for.  Measured cost when it went wrong: 49 -> 65 us per
  gate/up launch at 56 rows.
* the GEMM kernels of the per-layer hot path use no scratch memory (register spills cost about 3 us per
  launch on the 8-row kernels).  For the persistent whole-step kernel this is the property that decides
  whether it works at all: a reload from scratch is a vector memory operation that returns behind every
  weight fragment the wave has in flight, and what forced its descriptors and loop-invariant per-lane
  values into scratch (a descriptor copied out of global memory, a load through a selected address,
  values hoisted out of the loop over phases) is invisible in the source.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def device_asm(tmp_path_factory):
    if not (os.path.exists(HIPCC) or shutil.which(HIPCC)):
        pytest.skip("hipcc not available")
    from paper_2603_17573_amd import build as b
    out = str(tmp_path_factory.mktemp("asm") / "heisd_device.s")
    flags = [f for f in b.HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    cmd = [HIPCC] + flags + ["--cuda-device-only", "-S"] + b.SOURCES + ["-o", out]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert proc.returncode == 0, proc.stdout
    return open(out).read()


def kernel_bodies(asm, pattern):
    """{mangled name: [instructions]} of the kernels whose name matches pattern."""
    out = {}
    for m in re.finditer(r"^(_Z\w+):", asm, flags=re.M):
        name = m.group(1)
        if not re.search(pattern, name):
            continue
        end = asm.find("s_endpgm", m.end())
        lines = [ln.strip() for ln in asm[m.end():end].split("\n")]
        out[name] = [ln for ln in lines if ln and not ln.startswith(";") and not ln.startswith(".")]
    return out


def waits_between_transfers(instr):
    """Count the vector-memory waits that are followed, within a few instructions, by another
    global -> LDS transfer of the same run of transfers."""
    bad = 0
    for i, ins in enumerate(instr):
        if not ins.startswith("global_load_lds"):
            continue
        nxt = instr[i + 1:i + 12]
        for k, t in enumerate(nxt):
            if t.startswith("global_load_lds"):
                break
            if t.startswith("s_waitcnt") and "vmcnt" in t:
                if any(x.startswith("global_load_lds") for x in nxt[k + 1:k + 8]):
                    bad += 1
                break
    return bad


def test_scanner_sees_a_planted_wait():
    good = ["s_mov_b32 m0, s1", "global_load_lds_dwordx4 v[0:1], off", "s_mov_b32 m0, s2",
            "global_load_lds_dwordx4 v[2:3], off", "s_waitcnt vmcnt(0)", "s_barrier"]
    bad = good[:2] + ["s_waitcnt vmcnt(0)"] + good[2:]
    assert waits_between_transfers(good) == 0
    assert waits_between_transfers(bad) == 1


def test_no_compiler_wait_between_lds_transfers(device_asm):
    bodies = kernel_bodies(device_asm, r"bat_gemm_(ns|wide)|persist_forward")
    assert len(bodies) >= 10, sorted(bodies)
    for name, instr in bodies.items():
        assert any(i.startswith("global_load_lds") for i in instr), name
        assert waits_between_transfers(instr) == 0, name


def test_hot_kernels_use_no_scratch(device_asm):
    strict = r"(fast_gemm_kernel|fast_gemm_stream_kernel|fast_attn_kernel|persist_forward|bat_gemm_ns|bat_gemm_wide|bat_split_finish|retrieve_scores)"
    lenient = r"heisd8bat_gemmILi"          # a few set-up values outside the loop of products: at most 64 bytes
    seen = 0
    for m in re.finditer(r"\.amdhsa_kernel (\S+)(.*?)\.end_amdhsa_kernel", device_asm, flags=re.S):
        name, block = m.group(1), m.group(2)
        size = int(re.search(r"\.amdhsa_private_segment_fixed_size\s+(\d+)", block).group(1))
        if re.search(strict, name):
            seen += 1
            assert size == 0, (name, size)
        elif re.search(lenient, name):
            seen += 1
            assert size <= 64, (name, size)
    assert seen >= 20, seen
