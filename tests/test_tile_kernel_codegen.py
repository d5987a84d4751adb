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
  * no spill or reload inside a K loop (it would be one more vector-memory operation in the
    in-order queue: the waits stay safe, since more outstanding operations only make a wait for
    "at most n outstanding" stricter, but every such wait would drain the queue).
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
    parts = re.split(r"\n(?=_ZN4dwdp\d+gemm_tile_(?:persistent|item)_kernel\w+:)", asm)[1:]
    # the persistent kernel for FP8 and MXFP4 weights (two item functions each) and the
    # one-workgroup-per-item kernels: GEMM-1 and GEMM-2, each for FP8 and MXFP4
    assert len(parts) == 6, len(parts)
    for k in parts:
        body = k.split(".end_amdhsa_kernel")[0].split(".Lfunc_end")[0]
        name = k.split(":")[0]
        yield name, body.split("\n"), k


def _is_mx(name):
    # template arguments <MX> / <G1, MX> are mangled as ILb<MX>E / ILb<G1>ELb<MX>E
    if "item_kernel" in name:
        return re.search(r"ILb[01]ELb1E", name) is not None
    return re.search(r"kernelILb1E", name) is not None


def _n_loops(name):
    return 1 if "item_kernel" in name else 2


LABEL = re.compile(r"^(\.LBB\d+_\d+):")
FALLTHROUGH = re.compile(r"^; %bb\.\d+:")


def _blocks(raw_lines, depth):
    """Basic blocks of a kernel as (label or None, header of the loop of the given depth the block
    belongs to or None, instruction lines).  The compiler annotates every block with its loop
    ("in Loop: Header=BBx_y Depth=d", "This Inner Loop Header: Depth=d").  The K loops are at
    depth 2 in the persistent kernel (inside the loop over work items) and at depth 1 otherwise."""
    blocks, cur = [], [None, None, []]
    for n, l in enumerate(raw_lines):
        m, f = LABEL.match(l), FALLTHROUGH.match(l)
        if m or f:
            blocks.append(tuple(cur))
            hdr = None
            # the annotation may continue on the comment lines that follow the label
            note = l
            for nxt in raw_lines[n + 1:n + 4]:
                if not nxt.strip().startswith(";") or FALLTHROUGH.match(nxt):
                    break
                note += nxt
            h = re.search(r"Header=(BB\d+_\d+) Depth=%d" % depth, note)
            if h:
                hdr = "." + "L" + h.group(1)
            elif m and re.search(r"This Inner Loop Header: Depth=%d" % depth, note):
                hdr = m.group(1)
            cur = [m.group(1) if m else None, hdr, []]
            continue
        t = l.strip()
        if t and not t.startswith((";", ".", "//")):
            cur[2].append(t)
    blocks.append(tuple(cur))
    return blocks


def _k_loops(name, raw_lines):
    """The two K loops of a kernel (of the GEMM-1 and of the GEMM-2 item function): for each, the
    instructions of all its blocks and, for every block the loop exits to, the instructions up to
    and including the first full vector-memory wait (the drain)."""
    blocks = _blocks(raw_lines, _n_loops(name))
    headers = []
    for lab, hdr, ins in blocks:
        if hdr and hdr not in headers:
            headers.append(hdr)
    loops = []
    for h in headers:
        members = [b for b in blocks if b[1] == h]
        body = [t for b in members for t in b[2]]
        if not any(t.startswith("v_mfma") for t in body):
            continue                      # ticket loop, polling loop, index fill loops
        inside = {b[0] for b in members if b[0]}
        targets = set()
        for t in body:
            m = re.match(r"s_c?branch\w* (\.LBB\d+_\d+)", t)
            if m and m.group(1) not in inside:
                targets.add(m.group(1))
        exits = []
        for lab, hdr, ins in blocks:
            if lab in targets:
                k = next((i for i, t in enumerate(ins) if "vmcnt(0)" in t), None)
                assert k is not None, (name, lab, "a loop exit that does not drain first")
                exits.append(ins[:k + 1])
        # a loop whose last block falls through to its exit: the textually following block
        loops.append((body, exits))
    assert len(loops) == _n_loops(name), (name, len(loops), headers)
    return loops


def _ring(body):
    ring = set()
    for t in body:
        m = RING_LOAD.match("\t" + t)
        if m:
            ring |= _ring_regs(m)[0]
    return ring


def test_ring_registers_are_left_alone(tile_asm):
    for name, raw, _ in _kernels(tile_asm):
        for body, exits in _k_loops(name, raw):
            ring = _ring(body)
            # 3 fragments: FP8 16 registers of codes; MXFP4 8 of codes and 2 scale dwords
            assert len(ring) == (30 if _is_mx(name) else 48), (name, sorted(ring))
            bad = []
            for t in body + [t for e in exits for t in e]:
                m = RING_LOAD.match("\t" + t)
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
    for name, raw, _ in _kernels(tile_asm):
        for body, exits in _k_loops(name, raw):
            waits = []
            for t in body:
                waits += re.findall(r"vmcnt\((\d+)\)", t)
            # one wait per unrolled K block: the block after the first two has no scale copy (9
            # operations may be outstanding), the one after the third has (10); nothing else
            assert sorted(waits) == ["10", "9", "9"], (name, waits)
            # no other vector-memory operation inside the loop: in particular no spill or reload, which
            # would be counted by the waits (harmless for the data, but it drains the queue every time)
            assert not any(t.startswith(("scratch_", "buffer_", "flat_")) for t in body), name
            # 3 blocks of 5 token copies and one scale copy
            assert sum(t.startswith("global_load_lds_dwordx4") for t in body) == 15, name
            assert sum(t.startswith("global_load_lds_dwordx3") for t in body) == 1, name
            # 3 blocks x 4 weight loads (a load whose address depends on a branch appears once per side)
            n_ring = sum(bool(RING_LOAD.match("\t" + t)) for t in body)
            assert 12 <= n_ring <= 16, (name, n_ring)
            for e in exits:
                assert sum("vmcnt(" in t for t in e) == 1, (name, e)     # the drain is the first wait on the way out


def test_lds_reads_stay_lds_reads_and_two_waves_per_simd(tile_asm):
    for name, raw, full in _kernels(tile_asm):
        # the item functions get their LDS arrays as pointers: after inlining every access must
        # still be an LDS instruction, none may have become a generic (flat) access
        assert not any(l.strip().startswith("flat_") for l in raw), name
        m = re.search(r"\.amdhsa_next_free_vgpr (\d+)", full)
        assert m and int(m.group(1)) <= 256, (name, m and m.group(1))   # 8 waves on 4 SIMDs: 256 registers each
        # a few values may be spilled around an item (checked above: never inside a K loop)
        m = re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", full)
        assert m and int(m.group(1)) <= 128, (name, m and m.group(1))
