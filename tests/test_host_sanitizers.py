"""The library's host code (step planner, profile consumers, cluster simulator) under AddressSanitizer and
UndefinedBehaviorSanitizer: tests/host_sanitize_driver.cpp is built with both, together with planner.cpp, policy.cpp
and sim.cpp, and replays seeded inputs written here to a file; any report aborts it.  What it prints is compared with
what the regular library returns for the same inputs, so the replay is known to exercise the same code paths."""
import os
import subprocess
import tempfile

import numpy as np
import pytest

from paper_2507_17769_amd import binding as B
from paper_2507_17769_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2507_17769_amd", "csrc")
MASK = (1 << 64) - 1


def _mix(h, v):
    return (h * 1000003 + (int(v) & 0xFFFFFFFF)) & MASK


@pytest.fixture(scope="module")
def driver():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "driver")
        cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
               "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I", CSRC, os.path.join(ROOT, "tests", "host_sanitize_driver.cpp")] + \
              [os.path.join(CSRC, f) for f in ("planner.cpp", "policy.cpp", "sim.cpp")] + ["-o", exe]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        yield exe, tmp


def _run(driver, mode, text):
    exe, tmp = driver
    path = os.path.join(tmp, mode + ".txt")
    with open(path, "w") as f:
        f.write(text)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe, mode, path], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, (r.returncode, r.stderr[-4000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout.strip().splitlines()


def test_planner_under_sanitizers_matches_the_library(driver):
    rng = np.random.default_rng(5)
    cases, lines = [], []
    for it in range(120):
        n_kv, group = [(2, 2), (8, 4), (1, 16), (4, 1)][it % 4]
        max_pos = int(rng.integers(900, 5000))
        n_workers = int(rng.choice([0, 1, 3, 64, 2048]))
        n_seqs = int(rng.integers(0, 40))
        shapes = []
        for s in range(n_seqs):
            n_new = 1 if rng.random() < 0.6 else int(rng.integers(1, 200))
            kv_len = n_new + int(rng.integers(0, 700))
            shapes.append((n_new, kv_len, (kv_len + 15) // 16 + int(rng.integers(0, 3))))
        n_pool = sum(sh[2] for sh in shapes) + int(rng.integers(1, 50))
        free = list(rng.permutation(n_pool))
        seqs = [[1000 + s, n_new, kv_len, [int(free.pop()) for _ in range(n_pages)]] for s, (n_new, kv_len, n_pages) in enumerate(shapes)]
        bad = rng.random()
        if seqs and bad < 0.25:    # one defect: each kind must be refused the way the library refuses it
            s = seqs[int(rng.integers(0, len(seqs)))]
            k = int(rng.integers(0, 6))
            if k == 0: s[1] = 0
            elif k == 1: s[2] = s[1] - 1
            elif k == 2: s[2] = max_pos + 1 + s[1]
            elif k == 3: s[3] = s[3][:max(0, (s[2] + 15) // 16 - 1)]
            elif k == 4 and s[3]: s[3][0] = n_pool + 3
            elif k == 5 and len(seqs) > 1: seqs[0][0] = seqs[-1][0]
            if k == 4 and len(seqs) > 1 and s[3] and rng.random() < 0.5: s[3][0] = seqs[0][3][-1] if seqs[0] is not s and seqs[0][3] else n_pool + 3   # a shared page
        cases.append((n_kv, group, max_pos, n_pool, n_workers, seqs))
        lines.append(f"{n_kv} {group} {max_pos} {n_pool} {n_workers} 512 {12 * (16 // group)} 22 {len(seqs)}")
        for rid, n_new, kv_len, pages in seqs:
            lines.append(f"{rid} {n_new} {kv_len} {len(pages)} " + " ".join(str(p) for p in pages))
    out = _run(driver, "plan", f"{len(cases)}\n" + "\n".join(lines) + "\n")
    assert len(out) == len(cases)
    n_ok = 0
    for (n_kv, group, max_pos, n_pool, n_workers, seqs), line in zip(cases, out):
        got = line.split()
        ctx = B.Context(64 * n_kv * group, n_kv * group, n_kv, 64, 128, 1, max_pos, host_only=True)
        ctx.kv_alloc(n_pool, 1, 0)
        ctx.set_option("attn_workers", n_workers)
        sa = [(rid, n_new, kv_len, np.array(pages, dtype=np.int32)) for rid, n_new, kv_len, pages in seqs]
        try:
            cu, pos, slots = ctx.step_indices(sa)
            items = ctx.plan_attention(sa)
        except B.PolystepError as e:
            assert int(got[0]) == e.status, (got, str(e))
            ctx.destroy()
            continue
        ctx.destroy()
        assert got[0] == "0", (got, seqs)
        h_idx = 0
        for v in list(cu) + list(pos) + list(slots):
            h_idx = _mix(h_idx, v)
        h_items = 0
        for v in items.reshape(-1):
            h_items = _mix(h_items, v)
        assert [int(x) for x in got[1:]] == [int(sum(s[1] for s in seqs)), int(sum(s[2] for s in seqs)), len(items), h_idx, h_items], (got, seqs)
        n_ok += 1
    assert 60 <= n_ok < len(cases)          # both accepted and refused batches were replayed


def test_simulator_and_policy_under_sanitizers_match_the_library(driver):
    batch_sizes, kv_sizes = [1, 16, 64, 256, 1024, 4096], [4096, 32768, 131072, 524288]
    ms = np.array([[4.0 + 0.013 * b + 2.2e-5 * k for k in kv_sizes] for b in batch_sizes], dtype=np.float32)
    tpots = list(W.SIM_TPOTS_MS)
    runs = []
    for seed, mode, n, rate, max_p, max_o, servers in ((1, 0, 400, 0.08, 1024, 1024, 6), (2, 1, 400, 0.05, 1024, 512, 6), (3, 0, 250, 0.02, 8192, 2048, 5),
                                                      (4, 1, 250, 0.02, 8192, 2048, 5)):
        tr = W.sim_trace(seed, n, rate, max_p, max_o, burst=seed == 3)
        runs.append((mode, servers, tr, (1 + max_o) // 2))
    text = [f"{len(batch_sizes)} {len(kv_sizes)}", " ".join(map(str, batch_sizes)), " ".join(map(str, kv_sizes)),
            " ".join(repr(float(v)) for v in ms.reshape(-1)), str(len(runs))]
    for mode, servers, tr, avg in runs:
        text.append(f"{mode} {servers} {len(tpots)} " + " ".join(repr(t) for t in tpots) + f" {avg} 2000000.0 1000 1000000000 2048")
        text.append(str(len(tr["arrival"])))
        for i in range(len(tr["arrival"])):
            text.append(f"{tr['arrival'][i]!r} {tr['prompt'][i]} {tr['output'][i]} {tr['ttft'][i]!r} {tr['tier'][i]}")
    out = _run(driver, "sim", "\n".join(text) + "\n")
    prof = B.Profile(batch_sizes, kv_sizes, ms)
    at = 0
    for mode, servers, tr, avg in runs:
        r = prof.simulate(tr["arrival"], tr["prompt"], tr["output"], tr["ttft"], tr["tier"], tpots, servers, avg, 2e6, 1000,
                          disaggregated=mode == 1, prefill_budget=2048)
        h = 0
        for i in range(len(tr["arrival"])):
            a = int(np.float64(r["first_token_ms"][i]).view(np.uint64))
            b = int(np.float64(r["finish_ms"][i]).view(np.uint64))
            for v in (r["attained"][i], a & 0xFFFFFFFF, a >> 32, b & 0xFFFFFFFF, b >> 32, r["server"][i], r["decode_server"][i]):
                h = _mix(h, v)
        got = out[at].split()
        want = [0, r["end_ms"], r["cost_ms"], r["scale_ups"], r["scale_downs"], r["promotions"], r["dropped"], r["iterations"], r["admission_tests"], h]
        assert [float(x) for x in got] == [float(x) for x in want], (got, want)
        assert int(got[-1]) == h
        at += 1
        for i in range(min(8, len(tr["arrival"]))):
            run = [(tr["prompt"][i] + 5, 5), (1000, 100), (17, 1)]
            admit, pred, kv = prof.predict_admit(run, tr["prompt"][i], avg, tpots[tr["tier"][i]], 1.5)
            admit2, chunk, iters, ft = prof.predict_chunked_prefill(run, tr["prompt"][i], avg, tpots[tr["tier"][i]], tr["ttft"][i], 0.5)
            got = out[at].split()
            assert [float(x) for x in got] == [float(admit), pred, float(kv), float(admit2), float(chunk), float(iters), ft], (got, i)
            at += 1
    assert at == len(out)
    prof.close()
