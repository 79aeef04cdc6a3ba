"""Host logic of bench.py that runs without a GPU: the cpu_baseline leg on the tiny shape."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import bench
from paper_2604_18396_amd import configs, inputs


def test_cpu_baseline_with_fewer_scheduled_steps_than_its_budget():
    """The driver runs `--steps 20 --warmup 5` with a 24-step CPU budget: the schedule handed
    to the CPU leg is shorter than the budget and must simply bound the sample."""
    cfg = configs.TINY.with_(min_exit_layer=1)     # the schedule law draws from L/4 = 1 upwards
    w = inputs.make_weights(cfg, 1)
    sched = inputs.make_exit_schedule(cfg.n_layers, 3, 2)
    r = bench.cpu_baseline(cfg, w, sched, 24)
    assert r["kind"] == "oracle" and r["unit"] == "tokens/s" and r["value"] > 0 and r["cores"] >= 1
    assert r["sample"].startswith("3 decode steps")
    r = bench.cpu_baseline(cfg, w, inputs.make_exit_schedule(cfg.n_layers, 40, 2), 5)
    assert r["sample"].startswith("5 decode steps")
