"""SmartProfile on the GPU at hand (short warm-up and profile stages), its text file, and a plan from it for a
machine with two processor types (the second one synthesised as a slower copy: there is one GPU here)."""
import pytest

pytestmark = pytest.mark.gpu


def test_profile_partition_round_trip(tmp_path):
    from paper_2012_13846_amd import partition, smartprofile
    rec = smartprofile.profile_stack(scale=0.05, warmup=3, iters=5)
    assert len(rec) == 11 and all(r.time_s > 0 for r in rec[:10]) and rec[10].time_s >= 0
    assert rec[0].param_bytes == 27 * 32 * 32 * 2 + 2 * 32 * 4 and rec[7].param_bytes == 27 * 256 * 256 * 2 + 2 * 256 * 4
    assert rec[3].activation_bytes < rec[2].activation_bytes * 2      # the stride-2 layer has fewer rows
    path = str(tmp_path / "mi355x.txt")
    partition.write_profile(path, "MI355X", rec)
    gpu, back = partition.read_profile(path)
    assert gpu == "MI355X" and len(back) == 11
    profiles = {"MI355X": back, "half_speed": partition.scaled(back, 2.0)}
    plan = partition.partition(profiles, ["half_speed", "MI355X", "MI355X", "half_speed"], 50e9)
    assert plan.pipeline_time_s <= plan.data_parallel_time_s
    assert plan.stages[0].first_layer == 0 and plan.stages[-1].last_layer == 10
    assert sorted(a for s in plan.stages for a in s.processors) == [0, 1, 2, 3]
    print("plan:", [(s.first_layer, s.last_layer, s.processors, round(s.time_s * 1e3, 3)) for s in plan.stages],
          "pipeline ms", plan.pipeline_time_s * 1e3, "data parallel ms", plan.data_parallel_time_s * 1e3)
