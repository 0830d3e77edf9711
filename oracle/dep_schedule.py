"""Oracle for the disaggregated-expert-parallel schedule and the configuration search --
TEST INFRASTRUCTURE (plain Python, double).  Only tests may import this module.

What it follows (paper notation: m_a samples per attention micro-batch, r_1 micro-batches, m_e
tokens per expert and chunk, r_2 chunks, T layers, ag attention-group size, S sequence length):

  * task times are linear in their workload (Sec. 4.1):  t_a(m_a), t_s(m_a), t_e(m_e), t_a2e(m_e)
    = t_e2a(m_e); `layer_models` builds their coefficients from the GEMM / attention / link
    primitives the way "Performance models of different layers" does;
  * token conservation, last rule of Eq. limitation:  m_e * r_2 * E = m_a * ag * top_k * S;
  * `replay` starts every task as early as the rules of Eq. limitation allow: four resources
    (attention-group GPU, A2E link, expert-group GPU, E2A link) each run one task at a time
    (rules 1-5), shared expert and A2E of a micro-batch wait for its attention (rule 6), expert
    compute for its A2E (rule 7), E2A for its expert compute (rule 8), the next layer's attention
    for all E2A chunks and the shared expert of the same micro-batch (rule 9).  The order in which
    a resource takes its tasks is fixed: links and expert group by (layer, micro-batch, chunk); the
    attention group by layer and inside a layer ASAS (a_0 s_0 a_1 s_1 ...) or AASS (a_0 a_1 ... s_0
    s_1 ...), Sec. 4.2 "Determine the order of Attention and Shared Expert";
  * `replay_one_gpu` is NOT in the paper: it is the same set of rules plus one more, for the stand-in
    in which the attention group's shared experts and the expert group's routed experts run on the
    compute units of one GPU (a shared-expert task and an expert task do not overlap).  The rules then
    no longer fix the schedule (which of two waiting tasks takes the compute units first is a
    choice), so it is defined by a procedure: of the next unscheduled task of each of the four task
    sequences, those whose predecessors have been placed are candidates; the one that can start
    earliest (ties: attention group, A2E, experts, E2A) is placed at that time; repeat;
  * `layer0_times` are the layer-0 start times Sec. 4.2 prints for ASAS, with
    X = t_a + t_s,  Y = max(t_e, t_a2e),  F = max(X, r_2 Y);
  * `objective` is the denominator of Eq. simplify-objective / Eq. solver_r2 for ASAS:
        (T - 1) max(G, r_1 F) + max(X, G) + (r_1 - 1) F,
        G = t_a + 2 t_a2e + t_e + (r_2 - 1) Y.
    Reading: the equation as printed adds (r_2 - 1) Y once more outside G.  With G defined as above
    (the paper's own definition, the one the layer offset max(G, r_1 F) needs) that term is counted
    twice: the last E2A of layer 0 ends at G + (r_1 - 1) F by the printed layer-0 start times.  The
    duplicate is dropped here; `objective_as_printed` keeps it for the record;
  * `search` takes the steps of Algorithm 1: m_a downwards, r_1 = the largest the memory bound
    allows, pairs with an r_1 already seen skipped, both orders scored, r_2 by minimising the
    makespan.  Readings: getMaxR1 is never defined in the paper; its complexity paragraph states
    the memory rule r_1 * m_a <= cap, so getMaxR1(m_a) = min(r1_cap, cap // m_a).  The paper prints
    no closed form for AASS; it is scored by `replay`, ASAS by `objective`.  "Solve" is exhaustive
    over r_2 in 1..r2_max here (the product uses the convexity in 1/r_2).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

ASAS = 0
AASS = 1


@dataclass(frozen=True)
class Linear:
    alpha: float
    beta: float

    def __call__(self, x: float) -> float:
        return self.alpha + self.beta * x


@dataclass(frozen=True)
class TaskModels:
    a: Linear  # attention of one micro-batch, argument m_a
    s: Linear  # shared experts of one micro-batch, argument m_a
    e: Linear  # routed experts of one chunk on one expert-group GPU, argument m_e
    c: Linear  # A2E (= E2A) transfer of one chunk, argument m_e


@dataclass(frozen=True)
class Problem:
    ag: int         # attention-group size
    n_experts: int  # E
    top_k: int
    seq_len: int    # S
    n_layers: int   # T


def layer_models(*, alpha_gm: float, beta_gm: float, alpha_attn: float, beta_attn: float,
                 alpha_c: float, beta_c: float, S: int, M: int, H: int, n_h: int, d_k: int, d_v: int,
                 n_shared: int, E: int, eg: int) -> TaskModels:
    """Sec. 4.1, "Performance models of different layers".  alpha_e carries the factor 3 of
    Eq. moe_detail (three projections per expert), which the printed definition drops."""
    a = Linear(4 * alpha_gm + alpha_attn,
               beta_gm * (2 * S * M * n_h * d_k + 2 * S * M * n_h * d_v) + beta_attn * S * S * n_h * (d_k + d_v))
    s = Linear(3 * n_shared * alpha_gm, 3 * n_shared * beta_gm * S * M * H)
    e = Linear(3 * (E / eg) * alpha_gm, 3 * (E / eg) * beta_gm * M * H)
    c = Linear(alpha_c, beta_c * E * M / eg)
    return TaskModels(a, s, e, c)


def tokens_per_expert(p: Problem, m_a: int, r_2: int) -> float:
    """m_e from the conservation rule of Eq. limitation."""
    return m_a * p.ag * p.top_k * p.seq_len / (r_2 * p.n_experts)


def replay(mod: TaskModels, p: Problem, m_a: int, r_1: int, r_2: int, order: int) -> Dict[str, object]:
    """Earliest-start schedule under Eq. limitation.  Returns start times tau_a[t][i], tau_s[t][i],
    tau_a2e[t][i][j], tau_e[t][i][j], tau_e2a[t][i][j] and the makespan
    max(last shared end, last E2A end) of Eq. final-objective."""
    m_e = tokens_per_expert(p, m_a, r_2)
    t_a, t_s, t_e, t_c = mod.a(m_a), mod.s(m_a), mod.e(m_e), mod.c(m_e)
    T = p.n_layers
    tau_a = [[0.0] * r_1 for _ in range(T)]
    tau_s = [[0.0] * r_1 for _ in range(T)]
    tau_a2e = [[[0.0] * r_2 for _ in range(r_1)] for _ in range(T)]
    tau_e = [[[0.0] * r_2 for _ in range(r_1)] for _ in range(T)]
    tau_e2a = [[[0.0] * r_2 for _ in range(r_1)] for _ in range(T)]
    free_ag = free_a2e = free_eg = free_e2a = 0.0
    for t in range(T):
        # attention group, in its fixed order
        def ready(i: int) -> float:  # rule 9
            if t == 0:
                return 0.0
            return max(max(tau_e2a[t - 1][i][j] + t_c for j in range(r_2)), tau_s[t - 1][i] + t_s)
        if order == ASAS:
            for i in range(r_1):
                tau_a[t][i] = max(free_ag, ready(i))
                free_ag = tau_a[t][i] + t_a
                tau_s[t][i] = free_ag                       # rule 6, same resource: starts right away
                free_ag = tau_s[t][i] + t_s
        else:
            for i in range(r_1):
                tau_a[t][i] = max(free_ag, ready(i))
                free_ag = tau_a[t][i] + t_a
            for i in range(r_1):
                tau_s[t][i] = free_ag                       # after every attention of the layer
                free_ag = tau_s[t][i] + t_s
        # links and expert group
        for i in range(r_1):
            for j in range(r_2):
                tau_a2e[t][i][j] = max(free_a2e, tau_a[t][i] + t_a)   # rule 6
                free_a2e = tau_a2e[t][i][j] + t_c
                tau_e[t][i][j] = max(free_eg, free_a2e)               # rule 7
                free_eg = tau_e[t][i][j] + t_e
                tau_e2a[t][i][j] = max(free_e2a, free_eg)             # rule 8
                free_e2a = tau_e2a[t][i][j] + t_c
    makespan = max(tau_s[T - 1][r_1 - 1] + t_s, tau_e2a[T - 1][r_1 - 1][r_2 - 1] + t_c)
    return {"tau_a": tau_a, "tau_s": tau_s, "tau_a2e": tau_a2e, "tau_e": tau_e, "tau_e2a": tau_e2a,
            "makespan": makespan, "t": (t_a, t_s, t_e, t_c)}


def ag_sequence(r_1: int, order: int) -> List[Tuple[str, int]]:
    """One layer of the attention group's fixed task order: ("a" | "s", micro-batch)."""
    if order == ASAS:
        return [(kind, i) for i in range(r_1) for kind in ("a", "s")]
    return [("a", i) for i in range(r_1)] + [("s", i) for i in range(r_1)]


def replay_one_gpu(mod: TaskModels, p: Problem, m_a: int, r_1: int, r_2: int, order: int) -> Dict[str, object]:
    """The schedule of `replay` with one rule more -- shared-expert and expert tasks share one GPU's
    compute units and do not overlap -- built by the procedure the module header states."""
    m_e = tokens_per_expert(p, m_a, r_2)
    t_a, t_s, t_e, t_c = mod.a(m_a), mod.s(m_a), mod.e(m_e), mod.c(m_e)
    T = p.n_layers
    seq_ag = [(t, kind, i) for t in range(T) for kind, i in ag_sequence(r_1, order)]
    seq_ch = [(t, i, j) for t in range(T) for i in range(r_1) for j in range(r_2)]
    start: Dict[Tuple, float] = {}          # ("a" | "s", t, i) and ("a2e" | "e" | "e2a", t, i, j) -> start time
    dur = {"a": t_a, "s": t_s, "a2e": t_c, "e": t_e, "e2a": t_c}
    end = lambda key: start[key] + dur[key[0]]
    cursor = {"ag": 0, "a2e": 0, "e": 0, "e2a": 0}
    free = {"ag": 0.0, "a2e": 0.0, "e": 0.0, "e2a": 0.0}
    free_cu = 0.0                           # the compute units: shared-expert and expert tasks

    def candidate(res: str):
        """(earliest start, key) of the next task of a sequence, or None if it is exhausted or a
        predecessor has not been placed."""
        if res == "ag":
            if cursor["ag"] == len(seq_ag):
                return None
            t, kind, i = seq_ag[cursor["ag"]]
            if kind == "a":
                before = [] if t == 0 else [("s", t - 1, i)] + [("e2a", t - 1, i, j) for j in range(r_2)]
            else:
                before = [("a", t, i)]
            key = (kind, t, i)
        else:
            if cursor[res] == len(seq_ch):
                return None
            t, i, j = seq_ch[cursor[res]]
            before = {"a2e": [("a", t, i)], "e": [("a2e", t, i, j)], "e2a": [("e", t, i, j)]}[res]
            key = (res, t, i, j)
        if any(b not in start for b in before):
            return None
        at = max([free[res]] + [end(b) for b in before])
        if key[0] in ("s", "e"):
            at = max(at, free_cu)
        return at, key

    n_tasks = len(seq_ag) + 3 * len(seq_ch)
    while len(start) < n_tasks:
        best = None
        for res in ("ag", "a2e", "e", "e2a"):       # this order breaks ties
            c = candidate(res)
            if c is not None and (best is None or c[0] < best[0][0]):
                best = (c, res)
        (at, key), res = best
        start[key] = at
        free[res] = at + dur[key[0]]
        if key[0] in ("s", "e"):
            free_cu = at + dur[key[0]]
        cursor[res] += 1
    grid2 = lambda kind: [[start[(kind, t, i)] for i in range(r_1)] for t in range(T)]
    grid3 = lambda kind: [[[start[(kind, t, i, j)] for j in range(r_2)] for i in range(r_1)] for t in range(T)]
    out = {"tau_a": grid2("a"), "tau_s": grid2("s"), "tau_a2e": grid3("a2e"), "tau_e": grid3("e"),
           "tau_e2a": grid3("e2a"), "t": (t_a, t_s, t_e, t_c)}
    out["makespan"] = max(out["tau_s"][T - 1][r_1 - 1] + t_s, out["tau_e2a"][T - 1][r_1 - 1][r_2 - 1] + t_c)
    return out


def check_schedule(sch: Dict[str, object], r_1: int, r_2: int, T: int, tol: float = 1e-9,
                   one_gpu: bool = False) -> List[str]:
    """Every rule of Eq. limitation, checked directly on a set of start times (no knowledge of how
    they were produced).  one_gpu: also that no shared-expert task overlaps an expert task.
    Returns the list of violated rules (empty = valid)."""
    t_a, t_s, t_e, t_c = sch["t"]
    bad: List[str] = []

    def exclusive(name: str, spans: List[Tuple[float, float]]) -> None:
        spans = sorted(spans)
        for (s0, e0), (s1, _) in zip(spans, spans[1:]):
            if s1 < e0 - tol:
                bad.append(f"{name}: overlap {s0}..{e0} / {s1}")

    ag = [(sch["tau_a"][t][i], sch["tau_a"][t][i] + t_a) for t in range(T) for i in range(r_1)]
    ag += [(sch["tau_s"][t][i], sch["tau_s"][t][i] + t_s) for t in range(T) for i in range(r_1)]
    exclusive("rules 1-2 (attention group)", ag)
    idx = [(t, i, j) for t in range(T) for i in range(r_1) for j in range(r_2)]
    exclusive("rule 3 (A2E)", [(sch["tau_a2e"][t][i][j], sch["tau_a2e"][t][i][j] + t_c) for t, i, j in idx])
    exclusive("rule 4 (E2A)", [(sch["tau_e2a"][t][i][j], sch["tau_e2a"][t][i][j] + t_c) for t, i, j in idx])
    exclusive("rule 5 (expert group)", [(sch["tau_e"][t][i][j], sch["tau_e"][t][i][j] + t_e) for t, i, j in idx])
    if one_gpu:
        exclusive("one GPU (shared experts / experts)",
                  [(sch["tau_e"][t][i][j], sch["tau_e"][t][i][j] + t_e) for t, i, j in idx] +
                  [(sch["tau_s"][t][i], sch["tau_s"][t][i] + t_s) for t in range(T) for i in range(r_1)])
    for t in range(T):
        for i in range(r_1):
            end_a = sch["tau_a"][t][i] + t_a
            if sch["tau_s"][t][i] < end_a - tol:
                bad.append(f"rule 6: shared ({t},{i}) before its attention ends")
            for j in range(r_2):
                if sch["tau_a2e"][t][i][j] < end_a - tol:
                    bad.append(f"rule 6: A2E ({t},{i},{j}) before its attention ends")
                if sch["tau_e"][t][i][j] < sch["tau_a2e"][t][i][j] + t_c - tol:
                    bad.append(f"rule 7: expert ({t},{i},{j}) before its A2E ends")
                if sch["tau_e2a"][t][i][j] < sch["tau_e"][t][i][j] + t_e - tol:
                    bad.append(f"rule 8: E2A ({t},{i},{j}) before its expert ends")
                if t + 1 < T and sch["tau_a"][t + 1][i] < sch["tau_e2a"][t][i][j] + t_c - tol:
                    bad.append(f"rule 9: attention ({t + 1},{i}) before E2A ({t},{i},{j}) ends")
            if t + 1 < T and sch["tau_a"][t + 1][i] < sch["tau_s"][t][i] + t_s - tol:
                bad.append(f"rule 9: attention ({t + 1},{i}) before shared ({t},{i}) ends")
    return bad


def _xyfg(mod: TaskModels, p: Problem, m_a: int, r_1: int, r_2: int) -> Tuple[float, float, float, float, Tuple]:
    m_e = tokens_per_expert(p, m_a, r_2)
    t_a, t_s, t_e, t_c = mod.a(m_a), mod.s(m_a), mod.e(m_e), mod.c(m_e)
    X = t_a + t_s
    Y = max(t_e, t_c)
    F = max(X, r_2 * Y)
    G = t_a + t_c + t_e + t_c + (r_2 - 1) * Y
    return X, Y, F, G, (t_a, t_s, t_e, t_c)


def layer0_times(mod: TaskModels, p: Problem, m_a: int, r_1: int, r_2: int) -> Dict[str, object]:
    """The layer-0 start times Sec. 4.2 prints (ASAS)."""
    X, Y, F, _, (t_a, t_s, t_e, t_c) = _xyfg(mod, p, m_a, r_1, r_2)
    return {
        "tau_a": [i * X for i in range(r_1)],
        "tau_s": [i * X + t_a for i in range(r_1)],
        "tau_a2e": [[t_a + i * F + j * t_c for j in range(r_2)] for i in range(r_1)],
        "tau_e": [[t_a + t_c + i * F + j * Y for j in range(r_2)] for i in range(r_1)],
        "tau_e2a": [[t_a + t_c + t_e + i * F + j * Y for j in range(r_2)] for i in range(r_1)],
    }


def objective(mod: TaskModels, p: Problem, m_a: int, r_1: int, r_2: int) -> float:
    """Makespan model of ASAS over T layers (denominator of Eq. simplify-objective, see header)."""
    X, _, F, G, _ = _xyfg(mod, p, m_a, r_1, r_2)
    return (p.n_layers - 1) * max(G, r_1 * F) + max(X, G) + (r_1 - 1) * F


def objective_as_printed(mod: TaskModels, p: Problem, m_a: int, r_1: int, r_2: int) -> float:
    X, Y, F, G, _ = _xyfg(mod, p, m_a, r_1, r_2)
    return (p.n_layers - 1) * max(G, r_1 * F) + max(X, G) + (r_2 - 1) * Y + (r_1 - 1) * F


def score(mod: TaskModels, p: Problem, m_a: int, r_1: int, r_2: int, order: int) -> float:
    """Makespan used by the search: the closed form for ASAS, the replay for AASS."""
    if order == ASAS:
        return objective(mod, p, m_a, r_1, r_2)
    return replay(mod, p, m_a, r_1, r_2, AASS)["makespan"]


def solve_r2(mod: TaskModels, p: Problem, m_a: int, r_1: int, order: int, r2_max: int) -> Tuple[int, float]:
    """Smallest r_2 in 1..r2_max with the smallest makespan, by trying all of them."""
    best, best_t = 1, score(mod, p, m_a, r_1, 1, order)
    for r_2 in range(2, r2_max + 1):
        t = score(mod, p, m_a, r_1, r_2, order)
        if t < best_t:
            best, best_t = r_2, t
    return best, best_t


def max_r1(m_a: int, mem_cap: int, r1_cap: int) -> int:
    return min(r1_cap, mem_cap // m_a)


def search(mod: TaskModels, p: Problem, m_a_max: int, mem_cap: int, r1_cap: int,
           r2_max: int) -> Optional[Dict[str, object]]:
    """Algorithm 1.  Throughput = r_1 m_a ag / makespan (Eq. final-objective).  Returns the best
    (m_a, r_1, m_e, r_2, order) with its makespan and throughput, or None if nothing fits."""
    best: Optional[Dict[str, object]] = None
    prev_r1 = 0
    for m_a in range(m_a_max, 0, -1):
        r_1 = max_r1(m_a, mem_cap, r1_cap)
        if r_1 == 0 or r_1 == prev_r1:
            continue
        for order in (ASAS, AASS):
            r_2, span = solve_r2(mod, p, m_a, r_1, order, r2_max)
            tps = r_1 * m_a * p.ag / span
            if best is None or tps > best["throughput"]:
                best = {"m_a": m_a, "r_1": r_1, "r_2": r_2, "order": order,
                        "m_e": tokens_per_expert(p, m_a, r_2), "makespan": span, "throughput": tps}
        prev_r1 = r_1
    return best


def search_exhaustive(mod: TaskModels, p: Problem, m_a_max: int, mem_cap: int, r1_cap: int,
                      r2_max: int, orders=(ASAS, AASS)) -> Optional[Dict[str, object]]:
    """Every (m_a, r_1, r_2, order) with r_1 m_a <= mem_cap, no pruning: what Algorithm 1's skipping
    of non-Pareto pairs must not lose."""
    best: Optional[Dict[str, object]] = None
    for m_a in range(m_a_max, 0, -1):
        for r_1 in range(1, max_r1(m_a, mem_cap, r1_cap) + 1):
            for order in orders:
                for r_2 in range(1, r2_max + 1):
                    span = score(mod, p, m_a, r_1, r_2, order)
                    tps = r_1 * m_a * p.ag / span
                    if best is None or tps > best["throughput"]:
                        best = {"m_a": m_a, "r_1": r_1, "r_2": r_2, "order": order, "makespan": span,
                                "throughput": tps}
    return best
