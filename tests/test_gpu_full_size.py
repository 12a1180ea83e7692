"""GPU parity at the benchmark's full sizes (8B-shaped layer), in the launch configuration
bench.py times.  The oracle runs the whole layer on the host (seconds), so every output
element is compared, not a sample."""
import numpy as np
import pytest

from paper_2507_17769_amd import workloads as W
from gpu_harness import TOL, Case, f32

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg", [1, 2])
def test_8b_layer_full_size(cfg):
    b = W.config_batch(cfg, seed=0)
    print(f"cfg{cfg}: T={b.n_tokens} total_kv={b.total_kv} pool={b.n_pool_pages}", flush=True)
    c = Case(b)
    errs = c.run()
    print(f"cfg{cfg} errors {errs} stats ms_total={c.stats.ms_total:.3f} stages={[round(x, 3) for x in c.stats.ms_stage]}", flush=True)
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, bad
    # appended K/V of the new tokens only (reading the whole pool back is the tiny tests' job)
    eng = c.eng
    from gpu_harness import bf16_ulp_distance
    for s in b.seqs[:8]:
        k, v = eng.read_kv(0, s.pages, s.prefix, s.n_new)
        ok, ov = c.pool_b.gather(0, [int(p) for p in s.pages], s.kv_len)
        for got, want in ((k, ok[s.prefix:]), (v, ov[s.prefix:])):
            g, w = f32(got).astype(np.float64), want.astype(np.float64)
            assert np.all(np.abs(g - w) <= 2.0 ** -7 * np.abs(w) + 1e-3 * np.sqrt(np.mean(w * w)))
    c.close()


def test_largest_latency_grid_cell_full_size():
    """The largest cell of the latency grid (2048-token chunk at its drawn prefix + 256 decodes, 8B-shaped layer): the
    tiled GEMMs with 256x256 tiles, the longest prefill work items and the decode items in one attention launch."""
    b = W.grid_cell_batch(2048, 256, seed=0)
    print(f"grid cell: T={b.n_tokens} total_kv={b.total_kv} pool={b.n_pool_pages}", flush=True)
    c = Case(b)
    errs = c.run()
    print(f"grid cell errors {errs}", flush=True)
    bad = {k: v for k, v in errs.items() if not v <= TOL}
    assert not bad, bad
    c.close()


def test_70b_shaped_two_layer_stack_full_batch_teacher_forced(capsys):
    """The 70B-shaped configuration at its real batch (1024-token chunk at prefix 4096 + 256 decodes,
    660 k KV tokens per layer) on two layers, each checked on its own against the oracle from the
    layer's actual input: the code path bench.py times and checks on the 80-layer stack."""
    import argparse
    import json
    import bench
    a = argparse.Namespace(layers=2, kv_slots=2, check_layers="0,1", seed=0, steps=2, warmup=1, option=[])
    bench.run_cfg4(a)
    res = json.loads(capsys.readouterr().out.strip().splitlines()[-1])
    assert res["output_finite"]
    checks = {c["layer"]: c for c in res["layer_checks"]}
    assert set(checks) == {0, 1} and all(c["pass"] for c in checks.values()), checks
    # layer 1 sits on a residual stream that dominates its branches: the plain bar against the definition holds
    assert checks[1]["judged_against"] == "definition" and checks[1]["max_err_over_rms"] <= TOL
    # layer 0 of this shape is the ill-conditioned one: the definition itself moves by more than the bar when its
    # stored activations are rounded to bf16, and the kernels stay within the bar of that variant
    assert checks[0]["max_err_over_rms_vs_bf16_variant"] <= TOL
    assert checks[0]["max_err_over_rms"] <= checks[0]["oracle_gap_definition_vs_bf16_variant"] + TOL


def test_prompt_start_chunk_is_judged_against_the_bf16_activation_variant():
    """The first tokens of a prompt attend to a handful of keys; on the 8B shape rounding the stored activations to
    bf16 then moves the definition itself by more than the bar (the two oracle variants against each other, no kernel
    involved).  The kernels are held to the bar against the definition evaluated with those roundings, and to the
    bar plus that gap against the definition."""
    from gpu_harness import rel_err
    b = W.custom_batch("8b", 3, 96, 0, [], name="prompt_start")
    c = Case(b)
    errs = c.run()
    gap = rel_err(c.want_b, c.want)
    vs_variant = rel_err(c.out32, c.want_b)
    print(f"prompt start: definition moved by {gap:.4f} x RMS; kernels {vs_variant:.4f} from the variant, {errs['out']:.4f} from the definition", flush=True)
    assert vs_variant <= TOL
    assert errs["out"] <= gap + TOL
    bad = {k: v for k, v in errs.items() if k.endswith("|bf16:score") and not v <= 1.6 * TOL}
    assert not bad, bad   # per-row intermediates against the variant: the gated activation of such rows reaches 1.5 x the bar
    c.close()
