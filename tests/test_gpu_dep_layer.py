"""moe_ep_forward_dep on the GPU: the layer run as the disaggregated schedule of Sec. 2.3 (micro-batches,
attention stand-ins, shared experts on the attention-group stream in ASAS / AASS order) gives the bits of
the plain forward, its routing matches the oracle chunk by chunk, and its measured timeline obeys the
rules of Eq. limitation."""
import numpy as np
import pytest

import oracle
from workloads import CONFIGS, bf16_bits_to_f32, make_inputs, tiny_workload
from helpers import rel_err_rows

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

ASAS, AASS = 0, 1


def _gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def _wl():
    return tiny_workload(name="dep_layer", n_tokens=700, hidden=256, inter=192, n_experts=16, local_begin=2,
                         n_local=12, top_k=3, n_shared=1, shared_inter=256)


@pytest.mark.parametrize("pinned", [False, True])
def test_same_bits_as_the_plain_forward_for_every_schedule(pinned):
    g = _gpu()
    wl = _wl()
    inp = make_inputs(wl, seed=51)
    ctx = g.make_ctx(wl, max_chunks=12, pinned=pinned)
    d = g.DeviceInputs(wl, inp, pinned=pinned)
    base = g.run_forward(ctx, wl, d, r=1)
    ref = oracle.forward(inp["tokens"], inp["gate_logits"], inp["routed_w"], inp["shared_w"], hidden=wl.hidden,
                         inter=wl.inter, n_experts=wl.n_experts, local_begin=wl.local_begin, n_local=wl.n_local,
                         n_shared=wl.n_shared, shared_inter=wl.shared_inter, top_k=wl.top_k, r_chunks=1)
    assert rel_err_rows(bf16_bits_to_f32(base), ref["out"]) <= 2e-2
    for r_1, r_2, order, attn_us in ((1, 1, ASAS, 0.0), (3, 2, ASAS, 50.0), (3, 2, AASS, 50.0), (4, 3, AASS, 0.0),
                                     (2, 1, ASAS, 200.0), (12, 1, AASS, 5.0)):
        print(f"[case] dep r_1={r_1} r_2={r_2} order={order} attn_us={attn_us} pinned={pinned}", flush=True)
        out = g.run_forward_dep(ctx, wl, d, r_1, r_2, order, attn_us)
        assert np.array_equal(out, base), (r_1, r_2, order)
    # routing of chunk (i, j) = the oracle's routing of the same token range
    g.run_forward_dep(ctx, wl, d, 3, 2, ASAS, 0.0)
    import paper_2512_21487_amd as pkg
    for c in range(6):
        t0, Tn = pkg.binding.chunk_range(wl.n_tokens, 3, 2, c)
        got = ctx.get_routing(c)
        assert np.array_equal(got["idx"], ref["idx"][t0:t0 + Tn])
        assert got["idx"].shape[0] == Tn and got["count"].sum() == (got["pos"] >= 0).sum()
    ctx.destroy()


def test_no_shared_experts_and_more_micro_batches_than_tokens():
    g = _gpu()
    wl = tiny_workload(name="dep_small", n_tokens=5, hidden=64, inter=64, n_experts=8, n_local=8, top_k=2)
    inp = make_inputs(wl, seed=52)
    ctx = g.make_ctx(wl, max_chunks=16)
    d = g.DeviceInputs(wl, inp)
    base = g.run_forward(ctx, wl, d, r=1)
    for r_1, r_2, order in ((8, 2, ASAS), (1, 16, AASS), (16, 1, ASAS)):
        print(f"[case] dep_small r_1={r_1} r_2={r_2} order={order}", flush=True)
        assert np.array_equal(g.run_forward_dep(ctx, wl, d, r_1, r_2, order, 10.0), base)
    ctx.destroy()


def test_bad_schedule_arguments_are_rejected():
    g = _gpu()
    import paper_2512_21487_amd as pkg
    wl = CONFIGS["tiny"]
    ctx = g.make_ctx(wl, max_chunks=8)
    d = g.DeviceInputs(wl, make_inputs(wl))
    for r_1, r_2, order, attn_us in ((0, 1, ASAS, 0.0), (1, 0, ASAS, 0.0), (3, 3, ASAS, 0.0), (1, 1, 2, 0.0),
                                     (1, 1, ASAS, -1.0), (1, 1, ASAS, 2e6), (1, 1, ASAS, float("nan"))):
        with pytest.raises(pkg.MoeEpError) as ei:
            g.run_forward_dep(ctx, wl, d, r_1, r_2, order, attn_us)
        assert ei.value.code == -1
    ctx.destroy()


@pytest.mark.parametrize("order", [ASAS, AASS])
def test_measured_timeline_obeys_the_rules(order):
    """Eq. limitation on the measured schedule (moe_ep_get_timeline) of a pinned-host run with r_1 = 3,
    r_2 = 2: the attention group runs one task at a time in the order asked for (rules 1, 2), a
    micro-batch's inbound copies start after its attention (rule 6), a chunk's experts after its inbound
    copy (rule 7), its outbound copy after its aggregation (rule 8), its aggregation after the
    micro-batch's shared experts, links and experts take their chunks in order (rules 3-5), and the
    attention stand-ins last about as long as asked."""
    g = _gpu()
    wl = _wl()
    r_1, r_2, attn_us = 3, 2, 300.0
    ctx = g.make_ctx(wl, max_chunks=8, pinned=True)
    d = g.DeviceInputs(wl, make_inputs(wl, seed=53), pinned=True)
    g.run_forward_dep(ctx, wl, d, r_1, r_2, order, attn_us)
    ctx.set_profiling(1)
    g.run_forward_dep(ctx, wl, d, r_1, r_2, order, attn_us)
    tl = ctx.get_timeline()
    ctx.get_stage_ms()
    ctx.set_profiling(0)
    by = {}
    for name, fwd, b, e in tl:
        assert fwd == 0 and e >= b >= 0.0
        by.setdefault(name, []).append((b, e))
    eps = 2e-3
    assert len(by["attention"]) == r_1 and len(by["shared_gate_up_gemm"]) == r_1 and len(by["shared_down_gemm"]) == r_1
    for b, e in by["attention"]:
        assert 0.8 * attn_us <= (e - b) * 1e3 <= 2.0 * attn_us + 50.0
    for name in ("copy_in", "router", "routed_gate_up_gemm", "routed_down_gemm", "aggregation", "copy_out"):
        assert len(by[name]) == r_1 * r_2, name
        for (b0, e0), (b1, e1) in zip(by[name], by[name][1:]):
            assert b1 >= e0 - eps, f"{name}: two tasks overlap on one resource"
    # the attention group's sequence
    ag = []
    for i in range(r_1):
        ag.append(("a", i, by["attention"][i]))
        ag.append(("s", i, (by["shared_gate_up_gemm"][i][0], by["shared_down_gemm"][i][1])))
    want = [("a", i) if x == 0 else ("s", i) for i in range(r_1) for x in (0, 1)] if order == ASAS else \
           [("a", i) for i in range(r_1)] + [("s", i) for i in range(r_1)]
    ag.sort(key=lambda t: t[2][0])
    assert [(k, i) for k, i, _ in ag] == want
    for (_, _, (b0, e0)), (_, _, (b1, e1)) in zip(ag, ag[1:]):
        assert b1 >= e0 - eps
    for i in range(r_1):
        for j in range(r_2):
            c = i * r_2 + j
            assert by["copy_in"][c][0] >= by["attention"][i][1] - eps            # rule 6
            # rule 7: the experts wait for the chunk's token rows; gate and partition only for its gate
            # scores, which head the transfer
            assert by["routed_gate_up_gemm"][c][0] >= by["copy_in"][c][1] - eps
            assert by["router"][c][0] >= by["copy_in"][c][0] - eps
            assert by["aggregation"][c][0] >= by["shared_down_gemm"][i][1] - eps
            assert by["copy_out"][c][0] >= by["aggregation"][c][1] - eps         # rule 8
    assert by["forward"][0][1] >= max(by["copy_out"][-1][1], by["shared_down_gemm"][-1][1]) - eps
    ctx.destroy()


@pytest.mark.parametrize("seed", list(range(10)))
def test_seeded_random_layers_match_the_oracle(seed):
    """Ten seeded random layer shapes (K extents from one to nine 64-wide steps, experts with and
    without tokens, local subsets, zero to two shared experts, Zipf skew or none) through
    moe_ep_forward with a random chunk count and through moe_ep_forward_dep with a random schedule:
    routing bit-exact, outputs within the tolerance, and the two entry points give the same bits."""
    g = _gpu()
    rng = np.random.default_rng(1000 + seed)
    n_experts = int(rng.choice([4, 8, 24, 64]))
    n_local = int(rng.integers(1, n_experts + 1))
    local_begin = int(rng.integers(0, n_experts - n_local + 1))
    n_shared = int(rng.integers(0, 3))
    wl = tiny_workload(name=f"random{seed}", n_tokens=int(rng.integers(1, 900)), hidden=64 * int(rng.integers(1, 10)),
                       inter=64 * int(rng.integers(1, 7)), n_experts=n_experts, local_begin=local_begin,
                       n_local=n_local, top_k=int(rng.integers(1, min(n_experts, 8) + 1)), n_shared=n_shared,
                       shared_inter=64 * int(rng.integers(1, 5)) if n_shared else 0,
                       zipf_s=float(rng.choice([0.0, 1.2])))
    inp = make_inputs(wl, seed=seed)
    r = int(rng.integers(1, 7))
    r_1, r_2 = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    pinned = bool(rng.integers(0, 2))
    print(f"[case] {wl} r={r} r_1={r_1} r_2={r_2} pinned={pinned}", flush=True)
    ref = oracle.forward(inp["tokens"], inp["gate_logits"], inp["routed_w"], inp["shared_w"], hidden=wl.hidden,
                         inter=wl.inter, n_experts=wl.n_experts, local_begin=wl.local_begin, n_local=wl.n_local,
                         n_shared=wl.n_shared, shared_inter=wl.shared_inter, top_k=wl.top_k, r_chunks=1)
    ctx = g.make_ctx(wl, max_chunks=9, pinned=pinned)
    d = g.DeviceInputs(wl, inp, pinned=pinned)
    out = g.run_forward(ctx, wl, d, r=r, order=int(rng.integers(0, 2)))
    import paper_2512_21487_amd as pkg
    for c in range(r):
        t0, Tn = pkg.binding.chunk_range(wl.n_tokens, 1, r, c)
        assert np.array_equal(ctx.get_routing(c)["idx"], ref["idx"][t0:t0 + Tn])
    assert rel_err_rows(bf16_bits_to_f32(out), ref["out"]) <= 2e-2
    out_dep = g.run_forward_dep(ctx, wl, d, r_1, r_2, int(rng.integers(0, 2)), float(rng.choice([0.0, 20.0])))
    assert np.array_equal(out_dep, out)
    ctx.destroy()


@pytest.mark.parametrize("order", [ASAS, AASS])
def test_measured_makespan_lies_between_the_replay_for_two_groups_and_the_replay_for_one_gpu(order):
    """The schedule model against the GPU, both ways (DeepSeek-V2-Lite-shaped layer, two micro-batches of two
    chunks, 100 us attention stand-ins).  Fed with what the shared-expert and expert tasks take alone, the
    replay of Eq. limitation is a lower bound of the measured makespan -- its two groups do not slow each
    other down -- and the replay with the rule "shared experts and experts never overlap"
    (moe_ep_dep_replay_one_gpu) an upper bound: on one GPU they do overlap, each at a part of the rate."""
    import time
    import paper_2512_21487_amd as pkg
    g = _gpu()
    wl = CONFIGS["dsv2_lite"]
    r_1, r_2, attn_us = 2, 2, 100.0
    ctx = g.make_ctx(wl, max_chunks=r_1 * r_2)
    d = g.DeviceInputs(wl, make_inputs(wl))
    T_mb = -(-wl.n_tokens // r_1)
    # the tasks alone: one micro-batch through the plain forward, shared experts first, then its chunks
    plain = lambda: ctx.forward(d.tokens, d.logits, d.routed, d.shared, wl.top_k, r_2, 0, n_tokens=T_mb, out=d.out)
    for _ in range(3):
        plain()
    ctx.set_profiling(10)
    for _ in range(10):
        plain()
    st = ctx.get_stage_ms()
    ctx.set_profiling(0)
    t_s = st["shared_gate_up_gemm"] + st["shared_down_gemm"]
    t_e = sum(st[n] for n in ("router", "partition", "routed_gate_up_gemm", "routed_down_gemm", "aggregation")) / r_2
    run = lambda: ctx.forward_dep(d.tokens, d.logits, d.routed, d.shared, wl.top_k, r_1, r_2, order, attn_us,
                                  n_tokens=wl.n_tokens, out=d.out)
    for _ in range(3):
        run()
    spans = []
    for _ in range(5):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            run()
        torch.cuda.synchronize()
        spans.append((time.perf_counter() - t0) / 10 * 1e3)
    measured = float(np.median(spans))
    mod = pkg.DepModels(attn_us * 1e-3, 0.0, t_s, 0.0, t_e, 0.0, 0.0, 0.0)
    prob = pkg.DepProblem(ag=1, n_experts=wl.n_experts, top_k=wl.top_k, seq_len=1, n_layers=1)
    lower = pkg.dep_replay(mod, prob, 1, r_1, r_2, order)[0]
    upper = pkg.dep_replay(mod, prob, 1, r_1, r_2, order, one_gpu=True)[0]
    print(f"       order={order}: tasks alone t_s {t_s:.4f} t_e {t_e:.4f} ms; two groups {lower:.4f} <= measured "
          f"{measured:.4f} <= one GPU without overlap {upper:.4f} ms", flush=True)
    assert lower <= upper
    assert 0.93 * lower <= measured <= 1.07 * upper
    ctx.destroy()


@pytest.mark.parametrize("dep", [False, True])
def test_layers_back_to_back_give_the_bits_of_lone_forwards(dep):
    """Steady state over several layers (Sec. 4.2, the per-layer offset of the multi-layer timeline): L
    layers with their own weights and gate scores are enqueued back to back on one stream, layer l
    reading what layer l - 1 wrote, with no host synchronisation in between and one context whose
    workspaces every layer reuses.  Each layer's output must be the bits of a lone, synchronised forward
    on the same input; the measured period per layer is held against the schedule model's per-layer
    term max(G, r_1 F) fed with the task times the timeline shows."""
    import time
    import paper_2512_21487_amd as pkg
    g = _gpu()
    wl = _wl()
    L, r_1, r_2, attn_us = 4, 2, 2, 40.0
    layers = [make_inputs(wl, seed=70 + l) for l in range(L)]
    ctx = g.make_ctx(wl, max_chunks=r_1 * r_2)
    d = [g.DeviceInputs(wl, inp) for inp in layers]
    x0 = d[0].tokens.clone()

    def run_layer(l, x, out):
        if dep:
            ctx.forward_dep(x, d[l].logits, d[l].routed, d[l].shared, wl.top_k, r_1, r_2, ASAS, attn_us,
                            n_tokens=wl.n_tokens, out=out)
        else:
            ctx.forward(x, d[l].logits, d[l].routed, d[l].shared, wl.top_k, r_2, 1, n_tokens=wl.n_tokens, out=out)

    # lone forwards, one at a time
    lone, x = [], x0
    for l in range(L):
        out = torch.zeros_like(x0)
        run_layer(l, x, out)
        torch.cuda.synchronize()
        lone.append(out)
        x = out
    # the same chain enqueued at once, every layer's weights now read from a tile-order copy
    for l in range(L):
        ctx.prepare_weights(d[l].routed, d[l].shared)
    outs = [torch.zeros_like(x0) for _ in range(L)]

    def chain():
        x = x0
        for l in range(L):
            run_layer(l, x, outs[l])
            x = outs[l]

    chain()
    torch.cuda.synchronize()
    for l in range(L):
        assert torch.equal(outs[l], lone[l]), f"layer {l} of the chain differs from its lone forward"
    assert any(bool(o.any()) for o in outs)
    # period per layer against the model: task times from the measured timeline of one lone layer
    for _ in range(3):
        chain()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(10):
        chain()
    torch.cuda.synchronize()
    period_ms = (time.perf_counter() - t0) / (10 * L) * 1e3
    ctx.set_profiling(1)
    run_layer(0, x0, outs[0])
    by = {}
    for n, _, b, e in ctx.get_timeline():
        by.setdefault(n, []).append((b, e))
    ctx.get_stage_ms()
    ctx.set_profiling(0)
    mean = lambda xs: float(np.mean(xs)) if len(xs) else 0.0
    t_a = mean([e - b for b, e in by.get("attention", [])])
    t_s = mean([e2 - b1 for (b1, _), (_, e2) in zip(by["shared_gate_up_gemm"], by["shared_down_gemm"])])
    t_e = mean([e2 - b1 for (b1, _), (_, e2) in zip(by["router"], by["routed_down_gemm"])]) + \
        mean([e - b for b, e in by["aggregation"]])
    lone_ms = by["forward"][0][1] - by["forward"][0][0]
    mod = pkg.DepModels(t_a, 0.0, t_s, 0.0, t_e, 0.0, 0.0, 0.0)
    prob = pkg.DepProblem(ag=1, n_experts=wl.n_experts, top_k=wl.top_k, seq_len=1, n_layers=L)
    rr1 = r_1 if dep else 1
    span_L = pkg.dep_makespan(mod, prob, 1, rr1, r_2)
    prob1 = pkg.DepProblem(ag=1, n_experts=wl.n_experts, top_k=wl.top_k, seq_len=1, n_layers=1)
    per_layer_model = (span_L - pkg.dep_makespan(mod, prob1, 1, rr1, r_2)) / (L - 1)   # (T-1) max(G, r_1 F) / (T-1)
    print(f"       dep={dep}: period {period_ms:.4f} ms per layer, lone layer {lone_ms:.4f} ms, "
          f"model per-layer term {per_layer_model:.4f} ms (t_a {t_a:.4f} t_s {t_s:.4f} t_e {t_e:.4f})", flush=True)
    # layers depend on each other, so the chain cannot beat the model's per-layer term; it also must
    # not cost more than lone layers do (no hidden synchronisation, no re-allocation)
    assert period_ms >= 0.5 * per_layer_model
    assert period_ms <= 1.25 * lone_ms + 0.05
    ctx.destroy()
