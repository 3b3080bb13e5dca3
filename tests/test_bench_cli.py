"""bench.py without a GPU: what it refuses, and that the pieces of its line that need no device are right."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                         stderr=subprocess.STDOUT, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stdout


def test_algorithmic_bytes_of_the_named_workload():
    """The roofline's numerator: bytes per weight b/8 + 4/128, plus x and y once per layer, on the 7B shapes."""
    sys.path.insert(0, ROOT)
    import pmpd_synth as synth

    shape = synth.LLAMA_7B
    n = shape.n_weights()
    assert n == 6_476_005_376
    x_y = sum(2 * i + 4 * o for (_, _, _, o, i) in shape.layers())
    for b, want in ((4, 3_448_094_720), (3, 2_638_594_048), (2, 1_829_093_376)):
        assert n * b // 8 + n * 4 // 128 + x_y == want
