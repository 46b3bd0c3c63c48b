"""Heterogeneity-aware pipeline partition (Sec. III-C: Alg. 1, Alg. 2, Eq. 3, Eq. 4) as a host-side tool.

Input: per-layer records of SmartProfile (smartprofile.py) for every processor type -- compute time (forward +
backward), activation bytes, parameter bytes -- a processor list and the bandwidth between processors.
Output: the layer-to-stage assignment and the processors of every stage (a stage with several processors is
replicated: data parallel inside the stage), minimising the time of the slowest stage.

The recursion is Eq. 4 with Eq. 3 as the cost of a replicated stage; processors are sorted by capability and a
stage takes consecutive processors of that list (the paper's heuristic, which cuts the 2^n subsets to n prefixes).
Dynamic programming over (first layer, last layer, prefix length) with back-pointers; O(L^3 M^2).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple


@dataclass
class LayerRecord:
    name: str
    time_s: float          # forward + backward compute time of the layer on this processor type
    activation_bytes: int  # output of the layer (what crosses a stage boundary placed after it)
    param_bytes: int


@dataclass
class Stage:
    first_layer: int
    last_layer: int
    processors: List[int]  # indices into the caller's processor list
    time_s: float          # Eq. 3 for this stage


@dataclass
class Plan:
    stages: List[Stage]
    pipeline_time_s: float       # time of the slowest stage or boundary transfer (what Eq. 4 minimises)
    data_parallel_time_s: float  # all layers as one stage replicated on all processors (the baseline of Alg. 1)
    order: List[int]             # the processor list as sorted


def get_comp_time(times: Sequence[Sequence[float]], params: Sequence[float], bw: float, i: int, j: int,
                  procs: Sequence[int]) -> float:
    """Alg. 2 = Eq. 3: layers i..j as one stage replicated on `procs`: the slowest processor's compute time plus
    the all-reduce of the stage's parameters, 2 (m-1) sum(p) / BW, all divided by m."""
    m = len(procs)
    comp_sum = max(sum(times[a][i:j + 1]) for a in procs)
    comm = 2.0 * (m - 1) * sum(params[i:j + 1]) / bw
    return (comp_sum + comm) / m


def partition(profiles: Dict[str, List[LayerRecord]], processors: Sequence[str], bandwidth_bytes_per_s: float,
              fastest_first: bool = True) -> Plan:
    """profiles: processor type -> its SmartProfile records (same layers in the same order for every type).
    processors: the type of every processor available.  Returns the plan of Alg. 1."""
    if not processors:
        raise ValueError("no processors")
    layer_sets = [profiles[t] for t in processors]
    L = len(layer_sets[0])
    if L == 0 or any(len(ls) != L for ls in layer_sets):
        raise ValueError("every processor type needs a record for every layer")
    ref = layer_sets[0]
    params = [float(r.param_bytes) for r in ref]
    act = [float(r.activation_bytes) for r in ref]
    # sorted by capability = by the total profiled time
    total = [sum(r.time_s for r in ls) for ls in layer_sets]
    order = sorted(range(len(processors)), key=lambda a: (total[a], a), reverse=not fastest_first)
    times = [[r.time_s for r in layer_sets[a]] for a in order]      # times[position in sorted list][layer]
    M, bw = len(order), float(bandwidth_bytes_per_s)

    # prefix sums of layer times per processor and of parameters; Eq. 3 in O(m)
    pt = [[0.0] * (L + 1) for _ in range(M)]
    for a in range(M):
        for l in range(L):
            pt[a][l + 1] = pt[a][l] + times[a][l]
    pp = [0.0] * (L + 1)
    for l in range(L):
        pp[l + 1] = pp[l] + params[l]

    def q(i, j, lo, hi):       # layers i..j on sorted processors lo..hi-1
        m = hi - lo
        comp = max(pt[a][j + 1] - pt[a][i] for a in range(lo, hi))
        return (comp + 2.0 * (m - 1) * (pp[j + 1] - pp[i]) / bw) / m

    # c[i][j][m]: best time for layers i..j on the first m sorted processors (Eq. 4); choice = (k, n) or None
    # Only i = 0 is reachable from C(0, L-1, M): the left part of every split keeps the first layer.
    INF = float("inf")
    c = [[INF] * (M + 1) for _ in range(L)]
    choice: List[List[Tuple[int, int] | None]] = [[None] * (M + 1) for _ in range(L)]
    for j in range(L):
        for m in range(1, M + 1):
            best, how = q(0, j, 0, m), None                  # the range as one replicated stage (data parallel)
            for k in range(0, j):
                comm = act[k] / bw
                for n in range(1, m):
                    cand = max(c[k][n], comm, q(k + 1, j, n, m))
                    if cand < best:
                        best, how = cand, (k, n)
            c[j][m], choice[j][m] = best, how

    stages: List[Stage] = []
    j, m = L - 1, M
    while True:
        how = choice[j][m]
        if how is None:
            stages.append(Stage(0, j, [order[a] for a in range(0, m)], q(0, j, 0, m)))
            break
        k, n = how
        stages.append(Stage(k + 1, j, [order[a] for a in range(n, m)], q(k + 1, j, n, m)))
        j, m = k, n
    stages.reverse()
    return Plan(stages, c[L - 1][M], q(0, L - 1, 0, M), [int(a) for a in order])


# ---- SmartProfile's text files -----------------------------------------------------------------------------------
def write_profile(path: str, gpu_type: str, records: Sequence[LayerRecord], meta: Dict[str, object] | None = None):
    """One line per layer: index, name, compute time in ms (forward + backward), activation bytes, parameter bytes."""
    with open(path, "w") as f:
        f.write(f"# SmartProfile gpu_type={gpu_type}\n")
        for k, v in (meta or {}).items():
            f.write(f"# {k}={v}\n")
        f.write("# layer name time_ms activation_bytes param_bytes\n")
        for i, r in enumerate(records):
            f.write(f"{i} {r.name} {r.time_s * 1e3:.6f} {r.activation_bytes} {r.param_bytes}\n")


def read_profile(path: str) -> Tuple[str, List[LayerRecord]]:
    gpu_type, records = "", []
    for line in open(path):
        line = line.strip()
        if line.startswith("# SmartProfile gpu_type="):
            gpu_type = line.split("=", 1)[1]
        if not line or line.startswith("#"):
            continue
        idx, name, ms, act, par = line.split()
        assert int(idx) == len(records)
        records.append(LayerRecord(name, float(ms) * 1e-3, int(act), int(par)))
    return gpu_type, records


def scaled(records: Sequence[LayerRecord], slowdown: float) -> List[LayerRecord]:
    """Records of a hypothetical processor type `slowdown` times slower (for planning without that hardware)."""
    return [LayerRecord(r.name, r.time_s * slowdown, r.activation_bytes, r.param_bytes) for r in records]
