"""The heterogeneity-aware partitioner (Sec. III-C) on the CPU: the dynamic programme against the exhaustive
evaluation of Eq. 3 / Eq. 4 in oracle/partition.py, and that definition against hand-worked values."""
import numpy as np
import pytest

from oracle import partition as opart
from paper_2012_13846_amd import partition as part


def recs(times, act, par):
    return [part.LayerRecord(f"l{i}", t, a, p) for i, (t, a, p) in enumerate(zip(times, act, par))]


def test_eq3_hand_worked():
    # two layers, two processors: slowest compute 3 + 5 = 8 s; all-reduce 2 * (2-1) * (10 + 30) / 20 = 4 s; / 2
    t = [[1.0, 2.0], [3.0, 5.0]]
    p = [10.0, 30.0]
    assert opart.Q(t, p, 20.0, 0, 1, [0, 1]) == pytest.approx((8.0 + 4.0) / 2)
    assert opart.Q(t, p, 20.0, 0, 1, [0]) == pytest.approx(3.0)          # one processor: no synchronisation
    assert opart.Q(t, p, 20.0, 1, 1, [1]) == pytest.approx(5.0)
    assert part.get_comp_time(t, p, 20.0, 0, 1, [0, 1]) == pytest.approx(6.0)


def test_eq4_hand_worked():
    # 3 layers of 4, 4, 8 s on two equal processors, no parameters, tiny activations.
    # one stage on both: 16 / 2 = 8;  split after layer 1: max(8, 0, 8) = 8;  after layer 0: max(4, 12) = 12 -> 8
    t = [[4.0, 4.0, 8.0]] * 2
    time, stages = opart.C(t, [0, 0, 0], [0, 0, 0], 1.0, 0, 2, [0, 1])
    assert time == pytest.approx(8.0)
    # with a parameter-heavy model the single replicated stage pays the all-reduce and the pipeline wins
    p = [0.0, 0.0, 8.0]
    time, stages = opart.C(t, p, [0, 0, 0], 1.0, 0, 2, [0, 1])
    assert opart.Q(t, p, 1.0, 0, 2, [0, 1]) == pytest.approx((16 + 16) / 2)
    assert time == pytest.approx(8.0) and stages == [(0, 1, [0]), (2, 2, [1])]
    # a boundary transfer of 10 s after layer 1 sets the time of that split: max(8, 10, 8) = 10, still the best
    time, stages = opart.C(t, p, [0.0, 10.0, 0.0], 1.0, 0, 2, [0, 1])
    assert time == pytest.approx(10.0) and stages == [(0, 1, [0]), (2, 2, [1])]
    # at 13 s the split moves to the cheap boundary after layer 0: max(4, 0, 12) = 12
    time, stages = opart.C(t, p, [0.0, 13.0, 0.0], 1.0, 0, 2, [0, 1])
    assert time == pytest.approx(12.0) and stages == [(0, 0, [0]), (1, 2, [1])]


@pytest.mark.parametrize("seed", range(12))
def test_dynamic_programme_equals_exhaustive_definition(seed):
    rng = np.random.default_rng(seed)
    L, M = int(rng.integers(2, 7)), int(rng.integers(1, 5))
    base = rng.uniform(0.5, 5.0, L)
    speeds = {"a": 1.0, "b": float(rng.uniform(1.1, 3.0)), "c": float(rng.uniform(0.3, 0.9))}
    act = rng.uniform(0.0, 4.0, L).tolist()
    par = rng.uniform(0.0, 6.0, L).tolist()
    profiles = {k: recs((base * s).tolist(), [int(a * 1000) for a in act], [int(p * 1000) for p in par])
                for k, s in speeds.items()}
    procs = [str(x) for x in rng.choice(list(speeds), M)]
    bw = float(rng.uniform(500, 5000))
    plan = part.partition(profiles, procs, bw)
    # the same search space, written out: processors sorted by total time, stages take consecutive ones
    order = plan.order
    t = [[r.time_s for r in profiles[procs[a]]] for a in order]
    p = [r.param_bytes for r in profiles["a"]]
    a_ = [r.activation_bytes for r in profiles["a"]]
    want_t, want_stages = opart.C(t, p, a_, bw, 0, L - 1, list(range(M)))
    assert plan.pipeline_time_s == pytest.approx(want_t, rel=1e-12)
    assert plan.data_parallel_time_s == pytest.approx(opart.Q(t, p, bw, 0, L - 1, list(range(M))), rel=1e-12)
    assert plan.pipeline_time_s <= plan.data_parallel_time_s + 1e-15
    # the plan is a valid cover: consecutive layer ranges, every processor once, stage times as Eq. 3 gives them
    assert plan.stages[0].first_layer == 0 and plan.stages[-1].last_layer == L - 1
    used = []
    for s0, s1 in zip(plan.stages, plan.stages[1:]):
        assert s1.first_layer == s0.last_layer + 1
    worst = 0.0
    for k, s in enumerate(plan.stages):
        used += s.processors
        pos = [order.index(a) for a in s.processors]
        assert pos == list(range(pos[0], pos[0] + len(pos)))             # consecutive in the sorted list
        assert s.time_s == pytest.approx(opart.Q(t, p, bw, s.first_layer, s.last_layer, pos), rel=1e-12)
        worst = max(worst, s.time_s)
        if k + 1 < len(plan.stages):
            worst = max(worst, a_[s.last_layer] / bw)
    assert sorted(used) == list(range(M))
    assert worst == pytest.approx(plan.pipeline_time_s, rel=1e-12)


def test_closed_forms():
    # one processor: everything is one stage and takes the sum of the layer times
    prof = {"x": recs([1.0, 2.0, 3.0], [5, 5, 5], [7, 7, 7])}
    plan = part.partition(prof, ["x"], 10.0)
    assert len(plan.stages) == 1 and plan.pipeline_time_s == pytest.approx(6.0)
    # 4 equal layers, 4 equal processors, huge parameters, free activations: one layer per processor
    prof = {"x": recs([1.0] * 4, [0] * 4, [10 ** 9] * 4)}
    plan = part.partition(prof, ["x"] * 4, 1.0)
    assert [(s.first_layer, s.last_layer, len(s.processors)) for s in plan.stages] == [(l, l, 1) for l in range(4)]
    assert plan.pipeline_time_s == pytest.approx(1.0)
    # no parameters and expensive activations: plain data parallel is best
    prof = {"x": recs([1.0] * 4, [10 ** 9] * 4, [0] * 4)}
    plan = part.partition(prof, ["x"] * 4, 1.0)
    assert len(plan.stages) == 1 and plan.pipeline_time_s == pytest.approx(1.0)
    # heterogeneous: a processor twice as fast gets twice the layers (8 equal layers, parameters forbid replication)
    prof = {"fast": recs([1.0] * 9, [0] * 9, [10 ** 9] * 9), "slow": recs([2.0] * 9, [0] * 9, [10 ** 9] * 9)}
    plan = part.partition(prof, ["slow", "fast"], 1.0)
    sizes = {tuple(s.processors): s.last_layer - s.first_layer + 1 for s in plan.stages}
    assert sizes == {(1,): 6, (0,): 3} and plan.pipeline_time_s == pytest.approx(6.0)


def test_profile_files_round_trip(tmp_path):
    r = recs([0.00123, 0.5], [1024, 4096], [0, 27 * 64 * 64 * 2])
    path = str(tmp_path / "p.txt")
    part.write_profile(path, "MI355X", r, {"batch": 4})
    gpu, back = part.read_profile(path)
    assert gpu == "MI355X" and [b.name for b in back] == ["l0", "l1"]
    assert back[0].time_s == pytest.approx(0.00123) and back[1].param_bytes == 27 * 64 * 64 * 2
    assert [b.time_s for b in part.scaled(back, 2.0)] == pytest.approx([0.00246, 1.0])
