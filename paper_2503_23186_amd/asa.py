"""Strategy selection of the paper's Adaptive Scheduling Algorithm on the host (Section III-B steps
1-4 and 6, Section III-C; Algorithm 1: "partition model into L logical components", "profile
execution time t_comp(c_i)", "estimate communication overhead t_comm(c_i, s)", "solve
optimization", "re-profile and update strategy").

Control plane only: no kernels, no device memory.  The measured input is `Trainer.profile()` (the
per-call times of cnnk_train_step on this GPU); the byte counts come from the layer list.  With one
GPU there is nothing to apply the chosen plan to: the module answers "what would the algorithm
choose for K devices of this kind", which is the part of the method that one device can show.

The paper prints the objective as  min sum_i max(t_comp(c_i) + t_comm(c_i, s_i))  under a
per-device memory constraint and gives no formula for t_comm or mem.  Reading taken:

  step time  = sum over components (in layer order) of the slowest device's time for the component
               + the cost of changing the data layout between consecutive components
  choices    = DP (all K devices, batch split K ways) | HP (groups of d devices split the model
               dimension, K/d groups split the batch) | MP on device j (whole component, full batch)
  times      DP: t/K + allreduce(G over K)      HP: t/K + allreduce(G/d over K/d) + 2 allgather(O in d)
             MP(j): t
  allreduce(n over r) = 2 (r-1)/r n/bw + 2 (r-1) lat,  allgather(n in d) = (d-1)/d n/bw + (d-1) lat
  layout change with output bytes O: same 0 | MP(j)->MP(k) 2 (O/bw + lat)
             | MP <-> DP/HP 2 ((K-1)/K O/bw + lat) | DP <-> HP 2 ((d-1)/d O/bw + lat)
  memory     DP: S + A/K on every device | HP: S/d + A/K on every device | MP(j): S + A on device j
  (t: measured time of the component on one device at the full batch; G: gradient bytes; O: bytes of
  the component's output; S: bytes of weights + gradients + momentum + low-precision copies; A:
  activation bytes kept for the backward pass.)

The chain structure makes the unconstrained problem a shortest path (one pass of dynamic
programming over the components); the memory constraint couples the components, so the solver is a
depth-first branch and bound whose bound is that unconstrained optimum of the remaining suffix.
Exact; exponential only in how much of the tree the memory constraint forces it to visit.
"""
from __future__ import annotations
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

DP, HP, MP = "DP", "HP", "MP"


@dataclass
class Component:
    name: str
    t: float          # seconds on one device at the full batch (forward + backward + update)
    G: float          # gradient bytes exchanged by data parallelism
    O: float          # bytes of the component's output activation (same for its gradient)
    S: float          # parameter state bytes
    A: float          # activation bytes kept for the backward pass
    layers: Tuple[int, ...] = ()


@dataclass
class Cluster:
    K: int                      # devices
    mem: Sequence[float]        # bytes available per device (length K)
    bw: float                   # bytes / s per device of the collectives and transfers
    lat: float = 5e-6           # seconds per message
    d: int = 2                  # group size of the hybrid strategy (ignored unless 1 < d < K, d | K)

    def __post_init__(self):
        if isinstance(self.mem, (int, float)):
            self.mem = [float(self.mem)] * self.K
        if len(self.mem) != self.K or self.K < 1 or self.bw <= 0:
            raise ValueError("bad cluster description")

    @property
    def hybrid(self):
        return 1 < self.d < self.K and self.K % self.d == 0


@dataclass
class Plan:
    time: float                                   # predicted seconds per step (inf: nothing fits)
    assignment: List[Tuple] = field(default_factory=list)   # per component: ("DP",) | ("HP",) | ("MP", j)
    mem_used: List[float] = field(default_factory=list)     # bytes per device
    nodes: int = 0                                # search nodes visited


def _choices(cl: Cluster):
    out = [(DP,)]
    if cl.hybrid:
        out.append((HP,))
    return out + [(MP, j) for j in range(cl.K)]


def _allreduce(n, r, cl):
    return 0.0 if r <= 1 else 2.0 * (r - 1) / r * n / cl.bw + 2.0 * (r - 1) * cl.lat


def _allgather(n, d, cl):
    return 0.0 if d <= 1 else (d - 1) / d * n / cl.bw + (d - 1) * cl.lat


def t_comm(c: Component, s, cl: Cluster) -> float:
    """Communication overhead of component c under choice s (Algorithm 1, t_comm(c_i, s))."""
    if s[0] == DP:
        return _allreduce(c.G, cl.K, cl)
    if s[0] == HP:
        return _allreduce(c.G / cl.d, cl.K // cl.d, cl) + 2.0 * _allgather(c.O, cl.d, cl)
    return 0.0


def t_device(c: Component, s, cl: Cluster) -> float:
    """Time the slowest device spends on component c: its share of t_comp plus t_comm."""
    share = c.t if s[0] == MP else c.t / cl.K
    return share + t_comm(c, s, cl)


def t_relayout(c: Component, a, b, cl: Cluster) -> float:
    if a == b:
        return 0.0
    if a[0] == MP and b[0] == MP:
        f = 1.0
    elif a[0] == MP or b[0] == MP:
        f = (cl.K - 1) / cl.K
    else:
        f = (cl.d - 1) / cl.d
    return 2.0 * (f * c.O / cl.bw + cl.lat)


def mem_per_device(c: Component, s, cl: Cluster) -> List[float]:
    if s[0] == DP:
        return [c.S + c.A / cl.K] * cl.K
    if s[0] == HP:
        return [c.S / cl.d + c.A / cl.K] * cl.K
    return [c.S + c.A if j == s[1] else 0.0 for j in range(cl.K)]


def predict(comps: Sequence[Component], assignment, cl: Cluster) -> float:
    """Step time of a given assignment under the model above."""
    total = 0.0
    for i, c in enumerate(comps):
        total += t_device(c, assignment[i], cl)
        if i + 1 < len(comps):
            total += t_relayout(c, assignment[i], assignment[i + 1], cl)
    return total


def solve(comps: Sequence[Component], cl: Cluster) -> Plan:
    """The assignment that minimises the step time subject to the per-device memory limits."""
    L = len(comps)
    if L == 0:
        return Plan(0.0, [], [0.0] * cl.K, 0)
    ch = _choices(cl)
    n = len(ch)
    T = [[t_device(c, s, cl) for s in ch] for c in comps]
    X = [[[t_relayout(c, a, b, cl) for b in ch] for a in ch] for c in comps]
    Mm = [[mem_per_device(c, s, cl) for s in ch] for c in comps]
    # unconstrained optimum of the suffix i.. given the layout of component i (shortest path)
    lb = [[0.0] * n for _ in range(L)]
    lb[L - 1] = list(T[L - 1])
    for i in range(L - 2, -1, -1):
        for a in range(n):
            lb[i][a] = T[i][a] + min(X[i][a][b] + lb[i + 1][b] for b in range(n))
    # least memory any choice leaves on the busiest device, summed over a suffix: a cheap test that
    # the remaining components can fit at all
    min_total = [0.0] * (L + 1)
    for i in range(L - 1, -1, -1):
        min_total[i] = min_total[i + 1] + min(sum(m) for m in Mm[i])
    cap_total = float(sum(cl.mem))
    same_caps = all(m == cl.mem[0] for m in cl.mem)
    first_mp = 2 if cl.hybrid else 1

    best = Plan(float("inf"))
    used = [0.0] * cl.K
    cur = [0] * L
    nodes = 0

    def dfs(i, prev, cost, mp_devices):
        nonlocal best, nodes
        nodes += 1
        if i == L:
            if cost < best.time:
                best = Plan(cost, [ch[k] for k in cur], list(used), 0)
            return
        if sum(used) + min_total[i] > cap_total:
            return
        order = sorted(range(n), key=lambda b: (X[i - 1][prev][b] if i else 0.0) + lb[i][b])
        for b in order:
            step = (X[i - 1][prev][b] if i else 0.0)
            if cost + step + lb[i][b] >= best.time:
                break                      # sorted by this very bound: no later choice can win
            # identical devices are interchangeable: a component may open at most the next unused one
            if same_caps and b >= first_mp and (b - first_mp) > mp_devices:
                continue
            m = Mm[i][b]
            if any(used[j] + m[j] > cl.mem[j] for j in range(cl.K)):
                continue
            for j in range(cl.K):
                used[j] += m[j]
            cur[i] = b
            opened = mp_devices + 1 if (b >= first_mp and (b - first_mp) == mp_devices) else mp_devices
            dfs(i + 1, b, cost + step + T[i][b], opened if same_caps else mp_devices)
            for j in range(cl.K):
                used[j] -= m[j]

    dfs(0, 0, 0.0, 0)
    best.nodes = nodes
    return best


def components_from_tape(layers, rows, dtype="bf16", group="conv") -> List[Component]:
    """Logical components out of a layer list and `Trainer.profile()` rows [(layer, phase, ms)].

    group="conv": a component is a convolution (or the classifier head) together with the layers
    that follow it up to the next convolution (its batch norm, activation, pooling, residual add):
    the granularity at which a layer's weights can be replicated, split or placed.
    The update phase's time (one row for all parameters) is spread in proportion to parameter bytes."""
    esz = 2 if dtype == "bf16" else 4
    t_layer = [0.0] * len(layers)
    t_update = 0.0
    for li, phase, ms in rows:
        if li < 0:
            t_update += ms * 1e-3
        else:
            t_layer[li] += ms * 1e-3
    groups, cur = [], []
    for i, L in enumerate(layers):
        if L["op"] in ("conv", "fc_loss") and cur and group == "conv":
            groups.append(cur)
            cur = []
        cur.append(i)
    if cur:
        groups.append(cur)

    def params_of(L):
        if L["op"] == "conv":
            return L["Cout"] * L["R"] * L["S"] * L["Cin"], True
        if L["op"] == "bn":
            return 2 * L["C"], False
        if L["op"] == "fc_loss":
            return L["classes"] * L["F"] + L["classes"], False
        return 0, False

    def out_elems(L):
        if L["op"] == "conv":
            Ho = (L["H"] + 2 * L["pad"] - L["R"]) // L["stride"] + 1
            Wo = (L["W"] + 2 * L["pad"] - L["S"]) // L["stride"] + 1
            return L["N"] * Ho * Wo * L["Cout"]
        if L["op"] == "pool":
            return L["N"] * L["C"] * ((L["H"] // 2) * (L["W"] // 2) if L["mode"] == "max2" else 1)
        if L["op"] == "fc_loss":
            return L["N"] * L["classes"]
        return L["N"] * L["H"] * L["W"] * L["C"]

    comps = []
    total_p = sum(params_of(L)[0] for L in layers) or 1
    for g in groups:
        n_p, state, kept = 0, 0.0, 0.0
        for i in g:
            p, low = params_of(layers[i])
            n_p += p
            state += p * (12 + (2 if (low and dtype == "bf16") else 0))   # fp32 weight, gradient, momentum (+ bf16 copy)
            kept += out_elems(layers[i]) * (4 if layers[i]["op"] == "fc_loss" else esz)
        last = layers[g[-1]]
        comps.append(Component(name="%s%d" % (layers[g[0]]["op"], g[0]),
                               t=sum(t_layer[i] for i in g) + t_update * n_p / total_p,
                               G=4.0 * n_p, O=float(out_elems(last) * (4 if last["op"] == "fc_loss" else esz)),
                               S=state, A=kept, layers=tuple(g)))
    return comps


def components_from_vit(net, call_names, times_ms) -> List[Component]:
    """Logical components of a Vision Transformer out of the per-call times of cnnk_vit_train_step
    (names as cnnk_vit_step_call_name lists them): the embedding, per block its attention half
    (first norm, QKV, attention, projection) and its MLP half (second norm, two linear layers), and
    the head.  The update's time is spread in proportion to parameter bytes."""
    esz = 2 if net.dtype == "bf16" else 4
    d, m, T, B = net.dim, net.mlp, net.tokens, net.batch
    rows = B * T
    t = {}
    t_update = 0.0
    for name, ms in zip(call_names, times_ms):
        if name == "update":
            t_update += ms * 1e-3
            continue
        if name.startswith("block"):
            blk, rest = name.split(".", 1)
            half = "attention" if rest.split(".")[0] in ("ln1", "qkv", "attn", "proj") else "mlp"
            key = "%s.%s" % (blk, half)
        else:
            key = name.split(".")[0]
        t[key] = t.get(key, 0.0) + ms * 1e-3
    n_emb = d * net.patch * net.patch * 3 + 2 * d + T * d
    n_att = 2 * d + 3 * d * d + 3 * d + d * d + d
    n_mlp = 2 * d + 2 * d * m + m + d
    n_head = 2 * d + net.classes * d + net.classes
    total = n_emb + net.layers * (n_att + n_mlp) + n_head
    out = []

    def comp(name, n_p, n_matrix, kept_elems, out_elems):
        return Component(name=name, t=t.get(name, 0.0) + t_update * n_p / total, G=4.0 * n_p, O=float(out_elems * esz),
                         S=12.0 * n_p + (2.0 * n_matrix if net.dtype == "bf16" else 0.0), A=float(kept_elems * esz))

    out.append(comp("embed", n_emb, d * net.patch * net.patch * 3, B * (T - 1) * net.patch * net.patch * 3 + rows * d, rows * d))
    for l in range(net.layers):
        out.append(comp("block%d.attention" % l, n_att, 4 * d * d, rows * (d + 3 * d + d + d), rows * d))
        out.append(comp("block%d.mlp" % l, n_mlp, 2 * d * m, rows * (d + 2 * m + d), rows * d))
    out.append(comp("head", n_head, 0, B * d, B * net.classes))
    return out


def changed_significantly(old_times: Sequence[float], new_times: Sequence[float], rel=0.1) -> bool:
    """Algorithm 1's "if communication patterns changed significantly: re-profile and update
    strategy".  The paper names no criterion; reading: some component's measured time moved by more
    than `rel` of the step time since the plan was made."""
    if len(old_times) != len(new_times):
        return True
    total = sum(old_times) or 1.0
    return any(abs(a - b) > rel * total for a, b in zip(old_times, new_times))
