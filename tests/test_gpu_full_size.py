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
