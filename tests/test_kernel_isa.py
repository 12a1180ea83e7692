"""The tiled GEMM reads LDS through inline assembly that the compiler cannot see through: it does
not know that the destination registers are written asynchronously.  The kernel is written so that
this is safe (every read is waited for, with its registers named, before they are used; the main
loop is one straight-line body), but a register copy, a spill or a queue drain that a different
compiler version slipped into that loop would silently break or slow it.  This test compiles the
kernel for gfx950 exactly as the build does and inspects the generated main loop."""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2507_17769_amd import build as B


@pytest.fixture(scope="module")
def gemm_asm():
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "gemm.s")
        flags = [f for f in B.FLAGS if f != "-fPIC"]
        cmd = [B.HIPCC] + flags + ["--cuda-device-only", "-S", os.path.join(B.CSRC, "gemm.hip"), "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        return open(out).read()


def _kernels(asm):
    """name -> body text of every gemm_dma_kernel instantiation"""
    out = {}
    for m in re.finditer(r"^(_ZN2ps15gemm_dma_kernel\w+):\s*;.*?\n(.*?)s_endpgm", asm, re.S | re.M):
        out[m.group(1)] = m.group(2)
    return out


def test_tiled_gemm_main_loop_is_clean(gemm_asm):
    ks = _kernels(gemm_asm)
    assert len(ks) == 4, sorted(ks)          # two tiles x two epilogues
    for name, body in ks.items():
        lines = [l.strip() for l in body.splitlines()]
        # the main loop: from the label that carries the loop-header comment to the backward branch
        start = next(i for i, l in enumerate(lines) if "Inner Loop Header" in l)
        label = next(l.split(":")[0] for l in reversed(lines[:start + 1]) if re.match(r"\.LBB\d+_\d+:", l))
        end = next(i for i in range(start, len(lines)) if lines[i].startswith("s_cbranch") and lines[i].endswith(label))
        loop = [l for l in lines[start:end + 1] if l and not l.startswith(";")]
        ops = [l.split()[0] for l in loop]
        n_mfma = sum(o.startswith("v_mfma") for o in ops)
        n_read = sum(o == "ds_read_b128" for o in ops)
        n_load = sum(o.startswith("global_load_lds") for o in ops)
        assert n_mfma in (8, 32) and n_read == (8 if n_mfma == 8 else 16) and n_load == (4 if n_mfma == 8 else 8), (name, n_mfma, n_read, n_load)
        # nothing that moves, spills or copies registers, and no full drain of the load queue
        bad = [l for l in loop if re.match(r"(v_mov|v_accvgpr|scratch_|buffer_|v_swap|v_perm)", l) or "vmcnt(0)" in l]
        assert not bad, (name, bad)
        assert ops.count("s_barrier") == 1, name


def test_tiled_gemm_does_not_spill(gemm_asm):
    for m in re.finditer(r"^\s*\.amdhsa_kernel (_ZN2ps15gemm_dma_kernel\w+)(.*?)\.end_amdhsa_kernel", gemm_asm, re.S | re.M):
        body = m.group(2)
        scratch = re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", body)
        assert scratch and int(scratch.group(1)) == 0, (m.group(1), scratch and scratch.group(1))
