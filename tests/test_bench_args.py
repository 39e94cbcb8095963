"""Host logic of bench.py that needs no GPU: how --steps / --warmup are turned into what is run."""
import subprocess
import sys

import pytest

import bench


@pytest.mark.parametrize("steps,warmup,want", [
    (20, 5, (100, 100)),            # the values the harness passes
    (2000, 200, (2000, 200)),       # the defaults
    (1, 0, (100, 0)),
    (100, 100, (100, 100)),
    (101, 199, (200, 200)),
    (1234, 1, (1300, 100)),
])
def test_steps_are_rounded_up_to_whole_cycles(steps, warmup, want):
    K, W = bench.normalise_steps(steps, warmup)
    assert (K, W) == want
    assert K % bench.EVICT_EVERY == 0 and W % bench.EVICT_EVERY == 0 and K >= steps and W >= warmup
    assert K - steps < bench.EVICT_EVERY and W - warmup < bench.EVICT_EVERY
    assert bench.EVICT_EVERY % bench.ADD_EVERY == 0     # a cycle holds whole add windows


@pytest.mark.parametrize("steps,warmup", [(0, 5), (-3, 0), (10, -1)])
def test_bad_counts_are_refused(steps, warmup):
    with pytest.raises(ValueError):
        bench.normalise_steps(steps, warmup)


def test_more_than_one_gpu_is_refused_before_anything_runs():
    r = subprocess.run([sys.executable, bench.__file__, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout == ""


def test_one_byte_model():
    assert bench.STEP_ALGORITHMIC_BYTES == 512 * 57030
    assert 1.0 < bench.RECORDED_STEP_TRAFFIC_BYTES / bench.STEP_ALGORITHMIC_BYTES < 1.1
    model, n = bench.host_cpu()
    assert isinstance(model, str) and model and n >= 1
