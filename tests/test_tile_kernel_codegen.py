"""Host-side check of the LDS-tiled GEMM's generated code (no GPU needed).

The tile kernel loads its weight fragments with hand-issued asynchronous loads into a ring of
registers and waits for them with explicit counters, so its correctness rests on three
properties of the compiled code that the C++ source cannot state:
  * between the first per-block wait and the final drain, nothing but those loads writes a
    ring register and nothing but an MFMA (as its weight operand; with MXFP4 weights also the
    shift that extracts a block's scale byte) reads one -- a register copied or reused while a
    load is still in flight would hold stale or clobbered data;
  * the only vector-memory waits inside that region are the two the source writes
    (vmcnt(9) or vmcnt(10) per K block, vmcnt(0) at the drain) -- an extra compiler-inserted wait means it
    modelled one of the hand-issued operations and the counting no longer holds;
  * the kernel uses no scratch memory (a spill inside the loop would add vector-memory
    operations that break the in-order count).
The test compiles gemm_tile.hip to gfx950 assembly with the product flags and checks them.
"""
import os
import re
import subprocess

import pytest

from paper_2604_01621_amd import build as dwdp_build

SRC = os.path.join(dwdp_build.CSRC, "gemm_tile.hip")
# weight loads into the ring: 16 bytes per lane (FP8 codes, MXFP4 codes) or, for the MXFP4 scale
# dwords, 4 bytes per lane into a single register
RING_LOAD = re.compile(r"\s*global_load_dword(?:x4 v\[(\d+):(\d+)\]| v(\d+)), v(\d+), s\[\d+:\d+\](?: offset:\d+)?(?: nt)?$")


def _ring_regs(m):
    """Destination registers and address register of a ring load."""
    if m.group(1) is not None:
        return set(range(int(m.group(1)), int(m.group(2)) + 1)), int(m.group(4))
    return {int(m.group(3))}, int(m.group(4))


def _regs(text):
    used = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        used.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        used.add(int(m.group(1)))
    return used


@pytest.fixture(scope="module")
def tile_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("asm") / "gemm_tile.s"
    flags = [f for f in dwdp_build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [dwdp_build.hipcc_path()] + flags + ["--cuda-device-only", "-S", SRC, "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    return out.read_text()


def _kernels(asm):
    parts = re.split(r"\n(?=_ZN4dwdp20gemm_fp8_tile_kernel\w+:)", asm)[1:]
    assert len(parts) == 4, "expected GEMM-1 and GEMM-2, each for FP8 and MXFP4 weights"
    for k in parts:
        body = k.split(".end_amdhsa_kernel")[0]
        meta = k[len(body):]
        lines = [l for l in body.split("\n") if l.strip() and not l.strip().startswith((";", ".", "//"))]
        name = k.split(":")[0]
        yield name, lines, k


def _is_mx(name):
    # template arguments <G1, MX> are mangled as ILb<G1>ELb<MX>E
    return re.search(r"ILb[01]ELb1E", name) is not None


def test_ring_registers_are_left_alone(tile_asm):
    for name, lines, _ in _kernels(tile_asm):
        loads = [i for i, l in enumerate(lines) if RING_LOAD.match(l)]
        # prologue: 2 blocks x 4 loads; loop: 3 unrolled blocks x 4 loads
        assert len(loads) == 20, (name, len(loads))
        ring = set()
        for i in loads:
            ring |= _ring_regs(RING_LOAD.match(lines[i]))[0]
        # 3 fragments: FP8 16 registers of codes; MXFP4 8 of codes and 2 scale dwords
        assert len(ring) == (30 if _is_mx(name) else 48), (name, sorted(ring))
        first = next(i for i, l in enumerate(lines) if "vmcnt(9)" in l)
        drain = next(i for i, l in enumerate(lines) if "vmcnt(0)" in l and i > loads[-1])
        bad = []
        for l in lines[first:drain + 1]:
            t = l.strip()
            m = RING_LOAD.match(l)
            if m:
                if _ring_regs(m)[1] in ring:
                    bad.append(t)       # an address offset held in a ring register
                continue
            if not (_regs(t) & ring):
                continue
            if t.startswith("v_lshrrev_b32") and _is_mx(name):
                # MXFP4: this block's scale byte is shifted out of its (landed) scale dword into
                # another register; a read after the wait, like the MFMA's
                if int(re.match(r"v_lshrrev_b32_e32 v(\d+),", t).group(1)) not in ring:
                    continue
            if t.startswith("v_mfma"):
                ops = re.findall(r"v\[(\d+):(\d+)\]", t)
                dst = set(range(int(ops[0][0]), int(ops[0][1]) + 1))
                if not (dst & ring):
                    continue            # read as an operand only
            bad.append(t)
        assert not bad, (name, bad[:10])


def test_only_the_written_vector_memory_waits(tile_asm):
    for name, lines, _ in _kernels(tile_asm):
        loads = [i for i, l in enumerate(lines) if RING_LOAD.match(l)]
        first = next(i for i, l in enumerate(lines) if "vmcnt(9)" in l)
        drain = next(i for i, l in enumerate(lines) if "vmcnt(0)" in l and i > loads[-1])
        waits = set()
        for l in lines[first:drain + 1]:
            waits.update(re.findall(r"vmcnt\((\d+)\)", l))
        assert waits == {"9", "10", "0"}, (name, waits)
        # one wait per unrolled K block: the block after the first two has no scale copy (9
        # operations may be outstanding), the one after the third has (10)
        assert sum("vmcnt(9)" in l for l in lines[first:drain]) == 2, name
        assert sum("vmcnt(10)" in l for l in lines[first:drain]) == 1, name
        # 3 blocks of 5 token copies and one scale copy in the loop, 2 x 5 + 1 in the prologue
        assert sum("global_load_lds_dwordx4" in l for l in lines) == 25, name
        assert sum("global_load_lds_dwordx3" in l for l in lines) == 2, name
        # the drain is the only vmcnt(0) after the first per-block wait
        assert sum("vmcnt(0)" in l for l in lines[first:drain + 1]) == 1, name


def test_no_scratch_and_two_waves_per_simd(tile_asm):
    for name, lines, full in _kernels(tile_asm):
        assert not any("scratch_" in l for l in lines), name
        m = re.search(r"\.amdhsa_next_free_vgpr (\d+)", full)
        assert m and int(m.group(1)) <= 256, (name, m and m.group(1))   # 8 waves on 4 SIMDs: 256 registers each
