"""bench.py --workload sim on a stored table runs on the host alone: the JSON line keeps its shape and the C++ simulator
agrees with the oracle on the sample it times."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_sim_workload_on_a_stored_table(tmp_path):
    bs, ks = [1, 16, 64, 256, 512, 1024, 2048, 4096], [4096, 32768, 131072, 524288]
    ms = [[round(4.0 + 0.013 * b + 2.2e-5 * k, 4) for k in ks] for b in bs]
    table = tmp_path / "table.json"
    table.write_text(json.dumps({"batch_sizes": bs, "kv_sizes": ks, "ms": ms, "ms_filled": ms, "n_layers": 32, "vocab": 128256,
                                 "kv_capacity_tokens": 2000000}))
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "sim", "--table", str(table), "--requests", "400"],
                       capture_output=True, text=True, cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    d = json.loads(r.stdout.strip().splitlines()[-1])
    assert d["metric"] == "cluster_simulation_dslo_goodput" and d["n_gpus"] == 1 and d["vs_baseline"] is None
    assert set(d["goodput"]) == set(d["optimal"]) and len(d["goodput"]) == 6
    assert all(run["attained"] <= 1.0 and len(run["attained_by_tier"]) == 4 for run in d["runs"])
    assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["identical_outputs"] is True
