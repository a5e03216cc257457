"""Oracle of the paper's strategy-selection problem (Section III-B steps 2-4, Section III-C;
Algorithm 1, "profile", "estimate communication overhead", "solve optimization").
Test infrastructure: the objective written out by its definition and minimised by enumerating
every assignment.  Shares no code with paper_2503_23186_amd/asa.py.

The paper prints  min_{s_i in {DP, MP, HP}} sum_i max(t_comp(c_i) + t_comm(c_i, s_i))  subject to
sum_{i: device(c_i) = j} mem(c_i, s_i) <= M_j for every device j, and gives no formula for t_comm or
mem.  The reading taken (each point is a reading, listed in the design notes):

  * components c_1..c_L form a chain (the layer order of the network); the step time is the sum
    over components of the time the slowest device spends on that component ("sum max": the
    devices synchronise between components), plus what it costs to change the data layout between
    consecutive components;
  * a strategy is DP (all K devices, batch split K ways), HP (groups of d devices split the
    component's model dimension, K/d groups split the batch) or MP on device j (the whole
    component on one device, full batch): K + 2 choices per component;
  * per-device time of component i:
      DP    : t_i / K + ring all-reduce of its G_i gradient bytes over K devices
      HP    : t_i / K + ring all-reduce of G_i / d bytes over the K/d replicas
                      + all-gather of its O_i output bytes inside a group of d
      MP(j) : t_i   (the other devices idle)
    ring all-reduce of n bytes over r devices = 2 (r-1)/r * n / bw + 2 (r-1) * lat  (0 for r = 1);
    all-gather of n bytes over d devices = (d-1)/d * n / bw + (d-1) * lat, once forward and once
    for the gradient in the backward pass;
  * layout change between consecutive components (output O_i forward, its gradient backward):
      same layout           : 0
      MP(j) -> MP(k), k != j: 2 * (O_i / bw + lat)
      MP <-> DP or HP       : 2 * ((K-1)/K * O_i / bw + lat)   (gather to / scatter from one device)
      DP <-> HP             : 2 * ((d-1)/d * O_i / bw + lat)
  * memory of component i on device j:  S_i = state bytes (weights, gradients, momentum, copies),
    A_i = activations kept for the backward pass at the full batch:
      DP    : S_i + A_i / K      on every device
      HP    : S_i / d + A_i / K  on every device
      MP(j) : S_i + A_i          on device j only.
"""
from __future__ import annotations
import itertools


def layouts(K, d):
    """All choices for one component: ("DP",), ("HP",) if 1 < d < K and d divides K, ("MP", j)."""
    out = [("DP",)]
    if 1 < d < K and K % d == 0:
        out.append(("HP",))
    out += [("MP", j) for j in range(K)]
    return out


def ring_allreduce(n, r, bw, lat):
    return 0.0 if r <= 1 else 2.0 * (r - 1) / r * n / bw + 2.0 * (r - 1) * lat


def allgather(n, d, bw, lat):
    return 0.0 if d <= 1 else (d - 1) / d * n / bw + (d - 1) * lat


def component_time(c, s, K, d, bw, lat):
    """The slowest device's time for component c under choice s."""
    if s[0] == "DP":
        return c["t"] / K + ring_allreduce(c["G"], K, bw, lat)
    if s[0] == "HP":
        return c["t"] / K + ring_allreduce(c["G"] / d, K // d, bw, lat) + 2.0 * allgather(c["O"], d, bw, lat)
    return c["t"]


def transition(c, a, b, K, d, bw, lat):
    """Cost of handing component c's output (and, backward, its gradient) from layout a to layout b."""
    if a == b:
        return 0.0
    if a[0] == "MP" and b[0] == "MP":
        return 2.0 * (c["O"] / bw + lat)
    if a[0] == "MP" or b[0] == "MP":
        return 2.0 * ((K - 1) / K * c["O"] / bw + lat)
    return 2.0 * ((d - 1) / d * c["O"] / bw + lat)


def memory(c, s, K, d):
    """Bytes per device (list of K) that component c occupies under choice s."""
    if s[0] == "DP":
        return [c["S"] + c["A"] / K] * K
    if s[0] == "HP":
        return [c["S"] / d + c["A"] / K] * K
    return [c["S"] + c["A"] if j == s[1] else 0.0 for j in range(K)]


def objective(comps, assign, K, d, bw, lat):
    total = 0.0
    for i, c in enumerate(comps):
        total += component_time(c, assign[i], K, d, bw, lat)
        if i + 1 < len(comps):
            total += transition(c, assign[i], assign[i + 1], K, d, bw, lat)
    return total


def feasible(comps, assign, K, d, mem_cap):
    used = [0.0] * K
    for c, s in zip(comps, assign):
        for j, m in enumerate(memory(c, s, K, d)):
            used[j] += m
    return all(u <= cap for u, cap in zip(used, mem_cap))


def solve_brute_force(comps, K, d, bw, lat, mem_cap):
    """Minimum of the objective over every feasible assignment.  Returns (time, assignment) or
    (inf, None) when nothing fits.  (K+2)^L assignments: tiny instances only."""
    best, best_a = float("inf"), None
    for assign in itertools.product(layouts(K, d), repeat=len(comps)):
        if not feasible(comps, assign, K, d, mem_cap):
            continue
        t = objective(comps, assign, K, d, bw, lat)
        if t < best:
            best, best_a = t, assign
    return best, best_a
