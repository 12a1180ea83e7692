"""The tiled GEMM reads LDS through inline assembly that the compiler cannot see through: it does
not know that the destination registers are written asynchronously, nor that the matrix instructions
(assembly too, to pin the accumulators to the accumulation registers) have hazards.  The kernel is
written so that this is safe (every read is waited for, with its registers named, before they are used;
the main loop is one straight-line body of two stages; every accumulator is reused 16 or 64 instructions
later), but a register copy, a spill or a queue drain that a different compiler version slipped into
that loop would silently break or slow it.  This test compiles the kernel for gfx950 exactly as the
build does and inspects the generated code."""
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
    """name -> body text of every gemm_sk_kernel instantiation"""
    out = {}
    for m in re.finditer(r"^(_ZN2ps14gemm_sk_kernel\w+):\s*;.*?\n(.*?)s_endpgm", asm, re.S | re.M):
        out[m.group(1)] = m.group(2)
    return out


def _main_loop(lines):
    """the innermost loop that holds the matrix instructions: from its label to the backward branch"""
    labels = {m.group(1): i for i, l in enumerate(lines) for m in [re.match(r"(\.LBB\d+_\d+):", l)] if m}
    best = None
    for i, l in enumerate(lines):
        m = re.match(r"s_cbranch\w+ (\.LBB\d+_\d+)", l)
        if m and m.group(1) in labels and labels[m.group(1)] < i:
            body = [x for x in lines[labels[m.group(1)]:i + 1] if x and not x.startswith(";")]
            if any(x.startswith("v_mfma") for x in body) and (best is None or len(body) < len(best)):
                best = body
    return best


def test_tiled_gemm_main_loop_is_clean(gemm_asm):
    ks = _kernels(gemm_asm)
    assert len(ks) == 4, sorted(ks)          # two tiles x two epilogues
    for name, body in ks.items():
        lines = [l.strip() for l in body.splitlines()]
        loop = _main_loop(lines)
        assert loop, name
        ops = [l.split()[0] for l in loop]
        n_mfma = sum(o == "v_mfma_f32_16x16x32_bf16" for o in ops)
        n_read = sum(o == "ds_read_b128" for o in ops)
        n_load = sum(o.startswith("global_load_lds") for o in ops)
        # two stages per trip: 2 x 64 (16) MFMAs, 2 x 16 (8) operand reads, 2 x 8 (4) copies per wavefront
        assert (n_mfma, n_read, n_load) in ((128, 32, 16), (32, 16, 8)), (name, n_mfma, n_read, n_load)
        # nothing that moves, spills or copies registers, and no full drain of the load queue
        bad = [l for l in loop if re.match(r"(v_mov|v_accvgpr|scratch_|buffer_|v_swap|v_perm)", l) or "vmcnt(0)" in l]
        assert not bad, (name, bad)
        assert ops.count("s_barrier") == 2, name
        # every matrix instruction accumulates in place, in the accumulation registers, on vector-register operands
        for l in loop:
            if l.startswith("v_mfma"):
                m = re.match(r"v_mfma_f32_16x16x32_bf16 (a\[\d+:\d+\]), v\[\d+:\d+\], v\[\d+:\d+\], (a\[\d+:\d+\])$", l)
                assert m and m.group(1) == m.group(2), (name, l)
        # the operands a stage consumes were all waited for at the end of the stage before: the first instruction after
        # each barrier's matrix work starts is never a read into a register the same stage's MFMAs use
        waits = [i for i, l in enumerate(loop) if l.startswith("s_waitcnt lgkmcnt(0)")]
        assert len(waits) == 2, (name, waits)


def test_tiled_gemm_does_not_spill(gemm_asm):
    n = 0
    for m in re.finditer(r"^\s*\.amdhsa_kernel (_ZN2ps14gemm_sk_kernel\w+)(.*?)\.end_amdhsa_kernel", gemm_asm, re.S | re.M):
        body = m.group(2)
        scratch = re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", body)
        assert scratch and int(scratch.group(1)) == 0, (m.group(1), scratch and scratch.group(1))
        n += 1
    assert n == 4


def test_accumulators_are_not_read_right_behind_the_last_matrix_instruction(gemm_asm):
    """The compiler inserts no hazard waits around the assembly: after the main loop the kernel itself must wait before
    stores or LDS writes take the accumulation registers as data."""
    for name, body in _kernels(gemm_asm).items():
        lines = [l.strip() for l in body.splitlines() if l.strip() and not l.strip().startswith(";")]
        last = max(i for i, l in enumerate(lines) if l.startswith("v_mfma"))
        nops = [i for i, l in enumerate(lines) if l == "s_nop 15"]
        assert len(nops) == 2 and nops[1] == nops[0] + 1 and nops[0] > last, (name, nops, last)
        users = [i for i, l in enumerate(lines) if i > last and re.match(r"(global_store|ds_write|v_accvgpr_read)", l) and re.search(r"\ba\[?\d", l)]
        assert users and min(users) > nops[1], (name, min(users) if users else None, nops)


@pytest.fixture(scope="module")
def attn_asm():
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "attention.s")
        flags = [f for f in B.FLAGS if f != "-fPIC"]
        cmd = [B.HIPCC] + flags + ["--cuda-device-only", "-S", os.path.join(B.CSRC, "attention.hip"), "-o", out]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        return open(out).read()


def test_attention_kernel_keeps_two_blocks_per_compute_unit(attn_asm):
    """The attention plan counts on every block of the launch being resident at once: two blocks of four wavefronts per
    compute unit, i.e. at most 256 registers per lane and no more than half the LDS per block, and nothing spilled inside the loops.  The
    teams' LDS reads are assembly whose waits the kernel places itself: the loop that holds the barrier must not drain
    the copy queue (a wait for all outstanding loads would undo the two pairs kept in flight)."""
    n = 0
    for m in re.finditer(r"^\s*\.amdhsa_kernel (_ZN2ps11attn_kernel\w+)(.*?)\.end_amdhsa_kernel", attn_asm, re.S | re.M):
        body = m.group(2)
        get = lambda key: int(re.search(key + r" (\d+)", body).group(1))
        # a few lane constants of the store epilogues may live in scratch between a work item's start and its end;
        # the loops are checked for scratch accesses below
        assert get(r"\.amdhsa_private_segment_fixed_size") <= 64, m.group(1)
        assert get(r"\.amdhsa_next_free_vgpr") <= 256, (m.group(1), get(r"\.amdhsa_next_free_vgpr"))
        assert get(r"\.amdhsa_group_segment_fixed_size") <= 80 * 1024, m.group(1)
        n += 1
    assert n == 10          # head dims 64 and 128 x group sizes 1, 2, 4, 8, 16
    for m in re.finditer(r"^(_ZN2ps11attn_kernelILi128E\w+):\s*;.*?\n(.*?)s_endpgm", attn_asm, re.S | re.M):
        lines = [l.strip() for l in m.group(2).splitlines() if l.strip() and not l.strip().startswith(";")]
        labels = {mm.group(1): i for i, l in enumerate(lines) for mm in [re.match(r"(\.LBB\d+_\d+):", l)] if mm}
        loops = []
        for i, l in enumerate(lines):
            mm = re.match(r"s_c?branch\w* (\.LBB\d+_\d+)$", l)
            if mm and mm.group(1) in labels and labels[mm.group(1)] < i:
                body = lines[labels[mm.group(1)]:i + 1]
                if any(x == "s_barrier" for x in body) and any(x.startswith("v_mfma") for x in body):
                    loops.append(body)
        assert loops, m.group(1)
        for i, l in enumerate(lines):                # no loop that holds matrix instructions touches scratch
            mm = re.match(r"s_c?branch\w* (\.LBB\d+_\d+)$", l)
            if mm and mm.group(1) in labels and labels[mm.group(1)] < i:
                body = lines[labels[mm.group(1)]:i + 1]
                if any(x.startswith("v_mfma") for x in body) and len(body) < 900:
                    assert not any(x.startswith("scratch_") for x in body), (m.group(1), mm.group(1))
        team = min(loops, key=len)           # the innermost loop with a barrier and matrix instructions: a team's pair loop
        ops = [l.split()[0] for l in team]
        assert ops.count("s_barrier") == 1, (m.group(1), ops.count("s_barrier"))
        assert sum(o.startswith("global_load_lds") for o in ops) == 4, m.group(1)       # a quarter of a pair per wavefront
        assert sum(o == "v_mfma_f32_16x16x32_bf16" for o in ops) == 51, m.group(1)      # three tiles: 8 for the scores, 8 + 1 for P.V and the row sums each
        assert not any(o.startswith("scratch_") for o in ops), m.group(1)
        # the only full drain of the load queue sits in the rarely taken branch that reloads the page-id table
        drains = [i for i, l in enumerate(team) if l.startswith("s_waitcnt") and "vmcnt(0)" in l]
        assert len(drains) <= 1, (m.group(1), drains)


def _regs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]", text):
        out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    for m in re.finditer(r"\bv(\d+)\b", text):
        out.add(int(m.group(1)))
    return out


def _touched_before_their_wait(lines):
    """Vector registers that an LDS read is still writing when another instruction names them.  LDS operations retire
    in order, so `s_waitcnt lgkmcnt(n)` leaves the last n outstanding; the scan follows the code in layout order."""
    pending, bad = [], []
    for i, l in enumerate(lines):
        if not l or l.startswith(".LBB") or l.startswith(";"):
            continue
        op = l.split()[0]
        if op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", l)
            if m:
                n = int(m.group(1))
                pending = pending[len(pending) - n:] if n > 0 else []
            continue
        is_read = op.startswith("ds_read")
        touched = _regs(",".join(l.split(",")[1:])) if is_read else _regs(l)
        if any(p & touched for p in pending):
            bad.append((i, l))
        if op.startswith("ds_"):
            pending.append(_regs(l.split(",")[0]) if is_read else set())
    return bad


def test_the_scan_for_early_uses_finds_a_planted_one():
    ok = ["ds_read_b128 v[4:7], v2 offset:16", "v_add_f32_e32 v9, v8, v8", "s_waitcnt lgkmcnt(0)", "v_mov_b32_e32 v9, v5"]
    assert not _touched_before_their_wait(ok)
    early = ["ds_read_b128 v[4:7], v2 offset:16", "v_mov_b32_e32 v9, v5", "s_waitcnt lgkmcnt(0)"]
    assert _touched_before_their_wait(early) == [(1, early[1])]
    partial = ["ds_read_b64 v[4:5], v2", "ds_read_b64 v[6:7], v2 offset:8", "s_waitcnt lgkmcnt(1)", "v_mov_b32_e32 v9, v4", "v_mov_b32_e32 v9, v6"]
    assert _touched_before_their_wait(partial) == [(4, partial[4])]


def test_no_register_is_used_while_an_lds_read_is_still_writing_it(gemm_asm, attn_asm):
    """The tiled GEMM and the attention teams read LDS through assembly whose results the compiler believes valid at
    once; the kernels wait for them with statements that name the registers.  Anywhere in these kernels, loop or not, a
    register copy or an operand use that the compiler slipped in between a read and its wait would read stale data."""
    n = 0
    for asm, pat in ((gemm_asm, "gemm_sk_kernel"), (gemm_asm, "gemm_wstream_kernel"), (attn_asm, "attn_kernel")):
        for m in re.finditer(r"^(\S*" + pat + r"\S*):\s*;.*?\n(.*?)s_endpgm", asm, re.S | re.M):
            lines = [x.strip() for x in m.group(2).splitlines()]
            bad = _touched_before_their_wait(lines)
            assert not bad, (m.group(1), bad[:3])
            n += 1
    assert n >= 4 + 10
