"""Host-side checks of bench.py's command line and of the tables it shares with the tests (no GPU)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stderr + p.stdout)


def test_layer_and_sweep_tables_are_well_formed():
    sys.path.insert(0, ROOT)
    import bench

    names = [layer[0] for layer in bench.LAYERS]
    assert len(set(names)) == len(names)
    for idx in range(len(bench.LAYERS)):
        c = bench.layer_case(idx, n_images=1)
        assert c["Ho"] >= 1 and c["Wo"] >= 1 and c["x"].shape[0] == 1
        assert (c["w"] is None) == (c["kind"] in ("max", "avg"))
    assert list(bench.SWEEP_FILTERS) == sorted(set(bench.SWEEP_FILTERS)) and all(k % 2 == 1 for k in bench.SWEEP_FILTERS)
    assert max(bench.SWEEP_1D) <= 64 and min(bench.SWEEP_1D) >= 2
    # every launch of the step has its buffers and its traffic entry keyed to an existing source file
    for name in bench.BUFFERS:
        assert name in bench.TRAFFIC
        assert os.path.exists(os.path.join(ROOT, "paper_2310_05218_amd", "csrc", bench.TRAFFIC[name][1]))
