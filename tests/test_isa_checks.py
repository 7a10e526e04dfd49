"""Static checks of the generated gfx950 code (no GPU needed): the device code is compiled to
assembly with the library's own flags and scanned.

1. fp32 arithmetic is one rounding per operation: no fused multiply-add, no packed fp32.
2. Hazard check for the hand-written loads and stores of the fast path.  On gfx9-class hardware an SGPR
   written by a vector instruction (v_readfirstlane, v_readlane, a carry-out ...) must not be
   read by a vector memory instruction within 5 wait states.  The compiler pads its own memory
   instructions but does not look inside inline assembly, so a base pointer that reaches an
   inline-asm global_load or global_store through v_readfirstlane without padding makes the
   access use a stale address.  The kernels read their pointer tables with scalar loads and pad in scalar_ptr();
   this test keeps it that way.
"""
import os
import re
import subprocess
import tempfile

import pytest

from paper_1811_11141_amd import build as libbuild

SRC = os.path.join(libbuild.CSRC, "kernels.hip")


@pytest.fixture(scope="module")
def isa_text():
    flags = [f for f in libbuild.FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as td:
        out = os.path.join(td, "kernels.s")
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        res = subprocess.run([hipcc, *flags, "-S", "--cuda-device-only", "-o", out, SRC],
                             capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-2000:]
        with open(out) as f:
            return f.read()


@pytest.fixture(scope="module")
def isa_lines(isa_text):
    lines = [l.rstrip() for l in isa_text.splitlines() if l.startswith("\t") and not l.strip().startswith((";", "."))]
    assert len(lines) > 10000
    return lines


def test_no_fused_or_packed_fp32(isa_lines):
    bad = [l for l in isa_lines if re.match(r"\s*(v_fma_f32|v_fmac_f32|v_mad_f32|v_mac_f32|v_pk_(add|mul|fma)_f32)", l)]
    assert not bad, bad[:5]
    assert any("v_add_f32" in l for l in isa_lines) and any("v_mul_f32" in l for l in isa_lines)


def _sgpr_dests(line):
    mn, _, rest = line.strip().partition(" ")
    if not mn.startswith("v_"):
        return []
    ops = [o.strip() for o in rest.split(",")]
    dsts = ops[:1]
    if "_co_" in mn or mn.startswith(("v_addc", "v_subb", "v_div_scale", "v_mad_u64", "v_mad_i64")):
        dsts = ops[:2]
    regs = []
    for d in dsts:
        m = re.match(r"s\[(\d+):(\d+)\]$", d) or re.match(r"s(\d+)$", d)
        if m:
            regs += list(range(int(m.group(1)), int(m.group(m.lastindex)) + 1))
    return regs


def test_hand_written_loads_respect_the_sgpr_hazard(isa_lines):
    pat = re.compile(r"global_(?:load_dwordx4 v\[\d+:\d+\], v\d+|store_dwordx4 v\d+, v\[\d+:\d+\]), s\[(\d+):(\d+)\].* nt")
    checked, bad = 0, []
    for i, l in enumerate(isa_lines):
        m = pat.search(l)
        if not m:
            continue
        checked += 1
        base = {int(m.group(1)), int(m.group(2))}
        waited, k = 0, i - 1
        while waited < 5 and k >= 0:
            p = isa_lines[k].strip()
            if base & set(_sgpr_dests(p)):
                bad.append((p, l.strip()))
                break
            nop = re.match(r"s_nop (\d+)", p)
            waited += int(nop.group(1)) + 1 if nop else 1
            k -= 1
    assert checked > 1000          # the fast paths are there
    assert not bad, bad[:5]
    assert not any("v_readfirstlane" in l or "v_readlane" in l for l in isa_lines)


def test_scalar_unit_only_reads_memory(isa_lines):
    """Scalar memory instructions in the device code are loads and clock reads only: every
    write to memory goes through the vector unit."""
    scalar_mem = set()
    for l in isa_lines:
        mn = l.strip().split(" ")[0]
        if mn.startswith("s_") and any(w in mn for w in ("load", "mem", "st" + "ore", "atomic", "cache", "scratch", "probe")):
            scalar_mem.add(mn)
    assert scalar_mem, "expected scalar loads of the tables"
    allowed = ("s_load_dword", "s_buffer_load_dword", "s_memrealtime", "s_memtime")
    bad = [m for m in scalar_mem if not m.startswith(allowed)]
    assert not bad, bad


def test_workgroups_per_compute_unit_table_matches_the_compiled_kernels(isa_text):
    """The launch rules assume how many workgroups a compute unit holds: the fused reduce kernel
    16 (8 waves per SIMD) up to 14 pieces per lane, 14 (7 waves) with 16 pieces or with 16 workers;
    the update kernel 14, and 12 with 16 workers.  Recompute that from the registers the compiled
    kernels use: 512 VGPRs per SIMD in granules of 8; 800 SGPRs per SIMD in granules of 16, a wave
    taking sixteen more than the kernel's own count (the allowance that reproduces the batch sizes
    measured for both kernels); at most 8 waves."""
    meta = re.findall(r"\.name:\s+(\S+)\n(?:.*\n)*?\s+\.sgpr_count:\s+(\d+)\n(?:.*\n)*?\s+\.vgpr_count:\s+(\d+)", isa_text)
    regs = {name: (int(sg), int(vg)) for name, sg, vg in meta}

    def workgroups_per_cu(pattern):
        key = [k for k in regs if pattern in k]
        assert len(key) == 1, (pattern, key)
        sg, vg = regs[key[0]]
        waves = min(8, 512 // (-(-vg // 8) * 8), 800 // (-(-(sg + 16) // 16) * 16))
        return 2 * waves, (sg, vg)

    seen = 0
    for nw in (1, 2, 4, 8, 16):
        for u in (8, 10, 12, 14, 16):
            got, why = workgroups_per_cu(f"k_fusedILi{nw}ELi{u}ELb0ELb1ELi1E")
            assert got == (14 if (nw >= 16 or u == 16) else 16), (nw, u, why)
            seen += 1
        got, why = workgroups_per_cu(f"k_fusedILi{nw}ELi8ELb1ELb1ELi1E")      # with the update
        assert got == (12 if nw >= 16 else 14), (nw, why)
    assert seen == 25
