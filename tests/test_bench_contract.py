"""bench.py's command-line contract: what can be checked without a GPU, and the JSON line on one."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args, env=None):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          env={**os.environ, **(env or {})}, timeout=600)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _bench("--gpus", "2")
    assert r.returncode != 0 and "single-GPU" in r.stderr and r.stdout.strip() == ""
    r = _bench(env={"WORLD_SIZE": "2"})
    assert r.returncode != 0 and "single-GPU" in r.stderr


def test_the_rotary_bench_shapes_are_shapes_the_library_takes():
    # (descriptor checks run on the host: no GPU needed)
    import ctypes
    sys.path.insert(0, ROOT)
    import bench
    import paper_2412_11741_amd as csr
    from paper_2412_11741_amd import binding as B
    for sh in bench.ROPE_SHAPES:
        d = B.DecodeDesc(B=sh["B"], Hq=sh["Hq"], Hkv=sh["Hkv"], T=sh["T"], d=128, N=sh["N"], sK=sh["sK"], sV=sh["sV"], snK=1,
                         snV=sh["snV"], scale=0.0, q_dtype=B.CSR_F16, dict_dtype=B.CSR_F16, coef_dtype=B.CSR_F16,
                         idx_dtype=B.CSR_I16, out_dtype=B.CSR_F16, flags=0, rope_base=10000.0, rope_layout=0, rope_pos0=0)
        need = csr.lib().csr_decode_workspace_bytes(ctypes.byref(d))
        assert 0 < need < 1 << 32, (sh, csr.last_error())


def test_recorded_counter_traffic_names_a_committed_profile_summary():
    # `traffic` in the JSON line is a recorded rocprofv3 --pmc figure, labelled as such: its source must exist
    sys.path.insert(0, ROOT)
    import bench
    for table in (bench.PMC_TRAFFIC_BYTES, bench.PMC_DECODE_TRAFFIC_BYTES):
        for key in table:
            rec = bench.recorded_traffic(table, key)
            assert rec["traffic"] > 0 and "recorded" in rec["traffic_source"]
            assert os.path.isfile(os.path.join(ROOT, rec["traffic_source"].split(" ")[0])), rec
    assert bench.recorded_traffic(bench.PMC_TRAFFIC_BYTES, "no such workload") == {"traffic": None, "traffic_source": None}
    assert bench.median([3.0, 1.0, 2.0]) == 2.0 and bench.median([4.0, 1.0, 2.0, 3.0]) == 2.5


@pytest.mark.gpu
def test_the_json_line_carries_the_contracts_fields():
    r = _bench("--steps", "3", "--warmup", "1", "--no-extra-decode", "--no-extra-encode")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 3 and out["warmup"] == 1 and out["vs_baseline"] is None
    assert out["config"]["workload"] == "llama7b_layer" and "model" not in out["config"]
    roof = out["roofline"]
    assert roof["bound"] == "mfma" and roof["peak"] == 2500.0 and roof["unit"] == "TFLOP/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-4 and roof["traffic"] > 0
    assert roof["traffic_source"].startswith("profiles/") and "recorded" in roof["traffic_source"]
    # achieved = algorithmic flop per launch / launch time, value = vectors per second over the whole step
    assert abs(roof["achieved"] - out["config"]["vectors_per_step"] * roof["flop_per_vector"] / (roof["median_launch_ms"] * 1e-3) / 1e12) < 0.01 * roof["achieved"]
    assert abs(out["value"] - out["config"]["vectors_per_step"] / (out["ms_per_step"] * 1e-3)) < 0.01 * out["value"]
    cpu = out["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    for leg in ("roofline_decode", "chunked_step", "paper_sized_step", "decode_step", "reconstruct", "rope_decode"):
        assert leg in out, leg
    assert out["paper_sized_step"]["atoms"] == 256 and out["paper_sized_step"]["rope_base"] == 10000.0
    step = out["decode_step"]   # appended with the Gram matrices, and without them: the same atoms, faster
    assert step["same_atoms_as_without_gram"] and 0 < step["append_ms"] < step["append_ms_without_gram"]
    for r_ in out["rope_decode"]:
        assert r_["bound"] == "alu" and r_["peak"] == 157.3 and abs(r_["frac"] - r_["achieved"] / r_["peak"]) < 1e-4
