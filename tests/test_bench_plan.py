"""bench.py accepts any --steps / --warmup / --queue on every workload: the planning code never refuses, times
exactly the requested number of steps, and never drives a sample beyond its cache."""
import pytest

import bench
from paper_2505_18164_amd import synth as S


@pytest.mark.parametrize("workload", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("steps,warmup", [(20, 5), (1600, 80), (7, 3), (1, 0), (5000, 5000)])
@pytest.mark.parametrize("queue", [0, 1, 5, 64])
def test_any_step_count_is_planned(workload, steps, warmup, queue):
    wl = S.WORKLOADS[workload]
    cfg = wl["cfg"]()
    n, prompt, max_ctx = wl["n_seqs"], wl["prompt"], cfg["max_ctx"]
    q, windows = bench.plan_windows(n, prompt, max_ctx, steps, warmup, queue)
    assert 1 <= q <= n
    assert sum(t for _, t in windows) == steps                    # exactly the requested steps are timed
    assert windows[0][0] <= warmup
    for wu, timed in windows:
        assert timed >= 1
        # replay the calls of this window against the caches' capacity
        length = [prompt] * n
        calls = bench.calls_of(0, wu, q, n) + bench.calls_of(wu, timed, q, n)
        assert sum(len(c) for c in calls) == wu + timed
        for ids in calls:
            assert 1 <= len(ids) <= q and len(set(ids)) == len(ids)   # a sample has one message per call
            for s in ids:
                length[s] += 1
                assert length[s] <= max_ctx


def test_the_drivers_command_line_parses():
    a = bench.parse(["--gpus", "1", "--steps", "20", "--warmup", "5"])
    assert (a.gpus, a.steps, a.warmup, a.workload, a.queue) == (1, 20, 5, 4, 0)


def test_round_robin_calls_continue_where_the_warm_up_stopped():
    assert bench.calls_of(5, 20, 8, 8) == [[5, 6, 7, 0, 1, 2, 3, 4], [5, 6, 7, 0, 1, 2, 3, 4], [5, 6, 7, 0]]
    assert bench.calls_of(0, 3, 1, 2) == [[0], [1], [0]]


def test_paper_run_flag_parses():
    a = bench.parse(["--paper-run", "tinyllama", "--paper-tokens", "50"])
    assert a.paper_run == "tinyllama" and a.paper_tokens == 50 and a.gpus == 1
    assert bench.parse([]).paper_run is None
