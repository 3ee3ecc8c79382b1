"""bench.py's contract with the driver: any --steps >= 1 and --warmup >= 0 are accepted and exactly that many
steps are timed; the JSON line carries the roofline and the CPU baseline."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_graph_schedule_times_exactly_the_requested_steps():
    import bench

    for per_graph in (1, 3, 8):
        for steps in range(1, 50):
            full, rem = bench.graph_schedule(steps, per_graph)
            assert full >= 0 and 0 <= rem < per_graph
            assert full * per_graph + rem == steps            # nothing rounded away, nothing added
    assert bench.graph_schedule(20, 8) == (2, 4)               # the driver's command line
    assert bench.graph_schedule(200, 8) == (25, 0)
    assert bench.graph_schedule(1, 8) == (0, 1)
    with pytest.raises(ValueError):
        bench.graph_schedule(0, 8)


def test_profile_traffic_follows_the_launch_configuration(tmp_path, monkeypatch):
    """The counter figure is reported only while the library still picks the launch configurations it was measured
    with; anything else reads as null rather than as a stale number."""
    import bench

    prof = tmp_path / "p.txt"
    prof.write_text("some text\ntraffic_bytes_per_launch: 3.0e7 config: qkv=64/192,o=16/64\nmore text\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    monkeypatch.setattr(bench, "TRAFFIC_PROFILES", {"w": "p.txt", "gone": "missing.txt"})
    assert bench.profile_traffic("w", "qkv=64/192,o=16/64") == (3.0e7, "p.txt")
    assert bench.profile_traffic("w", "qkv=65/96,o=16/64") == (None, None)
    assert bench.profile_traffic("gone", "qkv=64/192,o=16/64") == (None, None)
    assert bench.profile_traffic("other", "x") == (None, None)


def test_algorithmic_bytes_formula():
    import bench

    # packed codes + 1.5 B of level-2 metadata per group + FP16 channel scales + INT8 activations + FP16 token
    # scales + FP16 output, for the QKV layer of the decode workload: 27.6 MB
    M, N, K = 64, 12288, 4096
    want = K * N // 2 + 3 * N * (K // 128) // 2 + 2 * N + M * K + 2 * M + 2 * M * N
    assert bench.algorithmic_bytes(M, N, K) == want
    assert abs(want - 27.6e6) < 0.1e6


@pytest.mark.gpu
@pytest.mark.timeout(900)
def test_driver_command_line_prints_one_complete_json_line():
    """`python bench.py --gpus 1 --steps 20 --warmup 5`, as the driver runs it, in a fresh process."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--steps", "20", "--warmup", "5"],
                       cwd=ROOT, capture_output=True, text=True, timeout=850)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    assert d["steps"] == 20 and d["warmup"] == 5 and d["n_gpus"] == 1
    assert d["unit"] == "TOPS" and d["value"] > 0 and d["ms_per_step"] > 0 and d["higher_is_better"] is True
    assert d["config"]["workload"].startswith("llama2_7b_decode_m64")
    roof = d["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    assert "traffic" in roof
    # the plain read of the same weights, timed beside the GEMM: between the launch floor and the GEMM's own time
    floor = roof["read_floor"]
    assert 1.0 < floor["avg_launch_us"] < roof["avg_launch_us"] * 1.5 and 0 < floor["frac_of_peak"] < 1
    assert abs(roof["gemm_time_over_read_floor"] - roof["avg_launch_us"] / floor["avg_launch_us"]) < 0.02
    fused = d["fused_producer_step"]        # the same GEMMs fed by the producers with the quantizer fused in
    assert fused["unit"] == "TOPS" and fused["value"] > 0 and 0.5 * d["ms_per_step"] < fused["ms_per_step"] < 3 * d["ms_per_step"]
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
    leg = d["compute_leg"]
    assert leg["workload"] == "llama3_70b_prefill_m2048"
    assert leg["roofline"]["bound"] == "mfma" and leg["roofline"]["peak"] == 5033.0 and 0 < leg["roofline"]["frac"] < 1
    # the matrix cores' own sustained rates, measured in the same run: constant operands close to the published peak,
    # random operands below it, the GEMM below the ceiling with the dequantizer's vector work attached
    ceil = leg["roofline"]["mfma_ceiling"]
    # (loose bounds: the sustained rates depend on the machine's power management)
    assert 0.6 < ceil["constant_operands"] <= 1.05
    assert ceil["random_operands_with_dequant_valu"] <= ceil["random_operands"] * 1.1 <= ceil["constant_operands"] * 1.2
    assert leg["roofline"]["frac"] < ceil["constant_operands"]


def test_read_probe_library_exports_its_entry_point():
    import ctypes

    from paper_2405_04532_amd import build as qbuild
    assert os.path.exists(qbuild.PROBE_LIB), "run `python -m paper_2405_04532_amd.build` first"
    lib = ctypes.CDLL(qbuild.PROBE_LIB)
    assert hasattr(lib, "qoq_probe_read") and hasattr(lib, "qoq_probe_mfma")
    lib.qoq_probe_mfma.restype = ctypes.c_int
    lib.qoq_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.qoq_probe_mfma(4, 10, 256, ctypes.c_void_p(4096), None) == 1
    assert lib.qoq_probe_mfma(0, 0, 256, ctypes.c_void_p(4096), None) == 1
    assert lib.qoq_probe_mfma(0, 10, 256, None, None) == 1
    lib.qoq_probe_read.restype = ctypes.c_int
    lib.qoq_probe_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    # argument checks run before anything touches a device
    assert lib.qoq_probe_read(None, 1024, None, 256, None) == 1
    assert lib.qoq_probe_read(ctypes.c_void_p(4096), 1000, ctypes.c_void_p(4096), 256, None) == 1
    assert lib.qoq_probe_read(ctypes.c_void_p(4096), 1024, ctypes.c_void_p(4096), 0, None) == 1


@pytest.mark.gpu
def test_read_probe_reads_what_it_is_given():
    """Contract of the probe: the call succeeds for sizes around the slab boundaries and any grid, stays inside the
    buffer (the sizes below end exactly at the end of the allocation's used part), and leaves the sink untouched
    for ordinary data."""
    import ctypes

    import torch

    import bench
    lib = bench.load_read_probe()
    src = torch.zeros(1 << 20, dtype=torch.int32, device="cuda:0")
    sink = torch.full((4096,), -1, dtype=torch.int32, device="cuda:0")
    for nbytes in (16, 4096 + 16, (1 << 22) - 16, 1 << 22):
        for nwg in (1, 7, 256, 4096):
            assert lib.qoq_probe_read(src.data_ptr(), nbytes, sink.data_ptr(), nwg, None) == 0
    torch.cuda.synchronize()
    assert bool((sink == -1).all())


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], cwd=ROOT, capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
