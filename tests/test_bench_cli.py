"""Host-side behaviour of bench.py that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and not r.stdout.strip()


def test_a_multi_rank_launch_is_refused_too():
    env = dict(os.environ, WORLD_SIZE="2", RANK="0", LOCAL_RANK="0")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True,
                       timeout=120, env=env)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_buffer_sets_make_whole_passes_of_exactly_the_requested_steps():
    import importlib.util
    import types
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    per_set = 32 * 196 * (256 * 4 * 2 + 128 + 4)          # config 2: fp32 in and out, codes, pixel sums
    for steps, warmup, serial, streams in ((2000, 200, False, 4), (2000, 200, True, 4), (1000, 100, False, 4),
                                           (600, 60, False, 3), (2000, 200, False, 0), (777, 50, False, 4)):
        n = bench.choose_sets(per_set, types.SimpleNamespace(steps=steps, warmup=warmup, serial=serial, streams=streams))
        chains = 1 if serial else (streams or 2)
        assert n * per_set >= 2 * 256e6                   # beyond the last-level cache
        assert n % chains == 0                            # every chain gets the same number of steps
        if steps != 777:                                  # (no divisor of 777 is in range: rounded up instead)
            assert steps % n == 0 and warmup % n == 0
