"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integer results (selected experts, counts, offsets, permutation) must be
bit-exact; outputs must satisfy max_i |gpu_i - ref_i| / max(|ref_i|, rms(ref row)) <= 2e-2, the
floor being the rms of the token's own output row (helpers.rel_err_rows; bf16 inputs, fp32
accumulation, activation and expert outputs rounded to bf16 once).  The same figure with one floor
over all rows is printed beside it and bounded at twice the tolerance."""
import numpy as np
import pytest

import oracle
import os

from helpers import load_tiny_golden, rel_err, rel_err_rows
from workloads import CONFIGS, bf16_bits_to_f32, make_inputs, tiny_workload

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 2e-2
W_TOL = 2e-6  # routing weights: fp32 exp and division against the fp64 oracle


def _gpu():
    import gpu_util
    return gpu_util


def _oracle_full(inp, wl, r=1):
    return oracle.forward(inp["tokens"], inp["gate_logits"], inp["routed_w"], inp["shared_w"],
                          hidden=wl.hidden, inter=wl.inter, n_experts=wl.n_experts,
                          local_begin=wl.local_begin, n_local=wl.n_local, n_shared=wl.n_shared,
                          shared_inter=wl.shared_inter, top_k=wl.top_k, r_chunks=r)


def _check_routing(ctx, ref, r, T, k):
    """Every chunk's routing against the oracle run with the same r: bit-exact."""
    Tc = (T + r - 1) // r
    for c in range(r):
        got = ctx.get_routing(c)
        t0 = c * Tc
        Tn = 0 if t0 >= T else min(Tc, T - t0)
        assert np.array_equal(got["idx"], ref["idx"][t0:t0 + Tn]), f"idx differs in chunk {c}"
        assert np.array_equal(got["count"], ref["count"][c]), f"count differs in chunk {c}"
        assert np.array_equal(got["offset"], ref["offset"][c]), f"offset differs in chunk {c}"
        A = int(ref["offset"][c][-1])
        assert np.array_equal(got["perm"], ref["perm"][c][:A]), f"perm differs in chunk {c}"
        assert np.array_equal(got["pos"], ref["pos"][t0:t0 + Tn]), f"pos differs in chunk {c}"
        if Tn:
            assert np.max(np.abs(got["w"].astype(np.float64) - ref["w"][t0:t0 + Tn])) <= W_TOL


def _full_parity(wl, seed=0, r=1, order=0, mutate=None, prepared=False):
    """prepared: the forward reads tile-order copies of the weights (moe_ep_prepare_weights)."""
    g = _gpu()
    inp = make_inputs(wl, seed=seed)
    if mutate:
        mutate(inp)
    print(f"[case] {wl.name} T={wl.n_tokens} M={wl.hidden} H={wl.inter} E={wl.n_experts} "
          f"El={wl.n_local}@{wl.local_begin} k={wl.top_k} Ns={wl.n_shared} r={r} order={order} "
          f"seed={seed}", flush=True)
    ref = _oracle_full(inp, wl, r)
    ctx = g.make_ctx(wl, max_chunks=max(r, 1))
    d = g.DeviceInputs(wl, inp)
    if prepared:
        ctx.prepare_weights(d.routed, d.shared)
    out = g.run_forward(ctx, wl, d, r=r, order=order)
    _check_routing(ctx, ref, r, wl.n_tokens, wl.top_k)
    err, err_all = rel_err_rows(bf16_bits_to_f32(out), ref["out"]), rel_err(bf16_bits_to_f32(out), ref["out"])
    print(f"       rel_err={err:.3e} (one floor over all rows: {err_all:.3e})", flush=True)
    assert err <= TOL and err_all <= 2 * TOL
    ctx.destroy()
    return out, ref


class _env:
    """Environment knobs of the library (read at moe_ep_create) set for a with-block."""

    def __init__(self, **kv):
        self.kv = kv

    def __enter__(self):
        self.old = {k: os.environ.get(k) for k in self.kv}
        for k, v in self.kv.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = str(v)

    def __exit__(self, *exc):
        for k, v in self.old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v


# ------------------------------------------------------------------ element by element
def test_tiny_config_matches_oracle():
    _full_parity(CONFIGS["tiny"])


def test_tiny_against_stored_oracle_values():
    """The GPU output against oracle values stored in tests/golden (no oracle run needed)."""
    g = _gpu()
    path = os.path.join(os.path.dirname(__file__), "golden", "tiny_oracle_values.txt")
    count, routing, samples, rms = load_tiny_golden(path)
    wl = CONFIGS["tiny"]
    ctx = g.make_ctx(wl)
    d = g.DeviceInputs(wl, make_inputs(wl))
    out = bf16_bits_to_f32(g.run_forward(ctx, wl, d))
    got = ctx.get_routing(0)
    assert got["count"].tolist() == count
    for t, i0, i1, w0, w1 in routing:
        assert got["idx"][t].tolist() == [i0, i1]
        assert abs(got["w"][t, 0] - w0) <= W_TOL and abs(got["w"][t, 1] - w1) <= W_TOL
    for t, c, v in samples:
        assert abs(out[t, c] - v) / max(abs(v), rms) <= TOL
    ctx.destroy()


@pytest.mark.parametrize("r,order", [(1, 0), (3, 1), (8, 0)])
def test_ragged_multi_tile_local_share(r, order):
    """Several row tiles per expert with ragged tails, a column tail, a local share that
    starts at expert 2, E not a multiple of 64, two shared experts."""
    wl = tiny_workload(name="ragged", n_tokens=777, hidden=192, inter=320, n_experts=10,
                       local_begin=2, n_local=6, top_k=3, n_shared=2, shared_inter=192)
    _full_parity(wl, seed=21, r=r, order=order)


def test_skewed_load_with_empty_experts():
    wl = tiny_workload(name="skew", n_tokens=600, hidden=128, inter=128, n_experts=70,
                       n_local=70, top_k=4)

    def mutate(inp):
        inp["gate_logits"][:, 5] += 30.0      # one expert takes every token
        inp["gate_logits"][:, 40:60] -= 30.0  # twenty experts get none

    out, ref = _full_parity(wl, seed=22, mutate=mutate)
    assert ref["count"][0][5] == 600 and np.all(ref["count"][0][40:60] == 0)


def test_quantised_logits_ties_are_bit_exact():
    wl = tiny_workload(name="ties", n_tokens=500, hidden=64, inter=64, n_experts=160,
                       local_begin=0, n_local=160, top_k=6)

    def mutate(inp):
        inp["gate_logits"][:] = np.round(inp["gate_logits"] * 2.0) / 2.0
        inp["gate_logits"][::7] = 0.0          # all-equal rows, signed zeros included
        inp["gate_logits"][::14, ::2] = -0.0

    _full_parity(wl, seed=23, mutate=mutate)


@pytest.mark.parametrize("k,E", [(1, 8), (8, 8), (1, 1)])
def test_top_k_extremes(k, E):
    wl = tiny_workload(name=f"k{k}E{E}", n_tokens=130, hidden=64, inter=128, n_experts=E,
                       n_local=E, top_k=k)
    _full_parity(wl, seed=24)


def test_no_token_selects_a_local_expert():
    wl = tiny_workload(name="none_local", n_tokens=100, hidden=64, inter=64, n_experts=8,
                       local_begin=6, n_local=2, top_k=2)

    def mutate(inp):
        inp["gate_logits"][:, 6:] = -40.0

    out, ref = _full_parity(wl, seed=25, mutate=mutate)
    assert ref["count"].sum() == 0 and not out.any()       # exact zeros


def test_single_token_and_empty_call():
    g = _gpu()
    wl = tiny_workload(name="one", n_tokens=1, hidden=64, inter=64, n_experts=8, n_local=8,
                       top_k=2, n_shared=1, shared_inter=64)
    _full_parity(wl, seed=26)
    ctx = g.make_ctx(wl)
    d = g.DeviceInputs(wl, make_inputs(wl, seed=26))
    ctx.forward(d.tokens, d.logits, d.routed, d.shared, 2, 1, 0, n_tokens=0, out=d.out)
    torch.cuda.synchronize()
    assert not d.out.cpu().numpy().any()
    ctx.destroy()


def test_more_chunks_than_tokens():
    wl = tiny_workload(name="r_gt_T", n_tokens=5, hidden=64, inter=64, n_experts=8, n_local=8,
                       top_k=2, n_shared=1, shared_inter=64)
    _full_parity(wl, seed=27, r=8)


def test_maximum_expert_count_and_top_k():
    """The limits of the boundary: 512 experts, all local, 64 experts per token."""
    wl = tiny_workload(name="E512k64", n_tokens=96, hidden=64, inter=64, n_experts=512, n_local=512,
                       top_k=64)
    _full_parity(wl, seed=28)


@pytest.mark.parametrize("prepared", [False, True])
@pytest.mark.parametrize("variant", [0, 1, 2, 6, 8, 9, 11, 12, 13, 14, 21, 22, 31])
@pytest.mark.parametrize("hidden", [64, 128, 192, 320])
def test_every_tile_variant_matches_oracle(variant, hidden, prepared):
    """Each instantiated tile shape / ring depth of the grouped GEMM (11, 12: 160-row tiles held by 1 x 4
    and 1 x 2 wavefronts; 13, 14: 224- and 256-row tiles held by 1 x 4), for the routed and the shared experts, on K extents of one, two, three and five 64-wide
    steps (shortest pipelines, fallbacks to the 32-wide variants included) with ragged row and column
    tails.  prepared: with tile-order copies of the weights, which variants 1, 2 and 11 read (with a
    column tail: 320 and 192 output columns in tiles of 128 and 256) and the others, and every fallback
    for a short K, ignore."""
    wl = tiny_workload(name=f"v{variant}_M{hidden}", n_tokens=333, hidden=hidden, inter=320, n_experts=6,
                       n_local=6, top_k=2, n_shared=1, shared_inter=192)
    old = {k: os.environ.get(k) for k in ("MOE_EP_GEMM_VARIANT", "MOE_EP_SHARED_VARIANT")}
    os.environ["MOE_EP_GEMM_VARIANT"] = os.environ["MOE_EP_SHARED_VARIANT"] = str(variant)
    try:
        _full_parity(wl, seed=29, prepared=prepared)
    finally:
        for k, v in old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v


@pytest.mark.parametrize("n_experts", [297, 298, 512])
def test_deepest_ring_at_the_lds_limit(n_experts):
    """The 160-row tiles keep a 156 KB ring; the per-expert tables behind it fit the 160 KB of a
    workgroup for up to 297 experts (8 bytes to spare), beyond that the launch falls back to the
    two-slot variant with the same row tile."""
    wl = tiny_workload(name=f"lds_limit_E{n_experts}", n_tokens=700, hidden=192, inter=192, n_experts=n_experts,
                       n_local=n_experts, top_k=8)
    old = os.environ.get("MOE_EP_GEMM_VARIANT")
    os.environ["MOE_EP_GEMM_VARIANT"] = "11"
    try:
        _full_parity(wl, seed=43)
    finally:
        if old is None:
            os.environ.pop("MOE_EP_GEMM_VARIANT", None)
        else:
            os.environ["MOE_EP_GEMM_VARIANT"] = old


def test_tile_shape_does_not_change_a_bit():
    """Every output element is accumulated over K in the same order whatever tile it falls in, so the
    tile shape the library picks (or is told to use) never shows in the result."""
    g = _gpu()
    wl = tiny_workload(name="tile_bits", n_tokens=1500, hidden=320, inter=256, n_experts=6, n_local=6, top_k=2,
                       n_shared=1, shared_inter=192)
    d = g.DeviceInputs(wl, make_inputs(wl, seed=44))
    old = os.environ.get("MOE_EP_GEMM_VARIANT")
    outs = {}
    try:
        for variant in (None, 0, 1, 2, 6, 11, 12, 13, 14, 21, 22, 31):
            if variant is None:
                os.environ.pop("MOE_EP_GEMM_VARIANT", None)
            else:
                os.environ["MOE_EP_GEMM_VARIANT"] = str(variant)
            ctx = g.make_ctx(wl)
            outs[variant] = g.run_forward(ctx, wl, d)
            ctx.destroy()
    finally:
        if old is None:
            os.environ.pop("MOE_EP_GEMM_VARIANT", None)
        else:
            os.environ["MOE_EP_GEMM_VARIANT"] = old
    assert outs[None].any()
    for variant, out in outs.items():
        assert np.array_equal(out, outs[None]), f"tile variant {variant} changed output bits"


def test_weights_in_tile_order_give_the_same_bits():
    """moe_ep_prepare_weights: the copy only changes where the weight tiles are read from, so the bits are
    those of the forward that reads the caller's layout -- routed weights alone, shared alone, both, a
    second set of weights beside the first, a refresh after the caller has rewritten the weights in
    place, and after moe_ep_forget_weights."""
    g = _gpu()
    wl = tiny_workload(name="tile_order", n_tokens=900, hidden=320, inter=192, n_experts=10, local_begin=3,
                       n_local=5, top_k=3, n_shared=2, shared_inter=192)
    inp = make_inputs(wl, seed=51)
    d = g.DeviceInputs(wl, inp)
    ctx = g.make_ctx(wl, max_chunks=4)
    base = g.run_forward(ctx, wl, d)
    ref = _oracle_full(inp, wl)
    assert rel_err_rows(bf16_bits_to_f32(base), ref["out"]) <= TOL
    assert ctx.prepared_weight_bytes() > 0 and ctx.last_tile_shape("routed_gate_up_gemm")["tile_order"] == 0
    for what in ("routed", "shared", "both"):
        ctx.prepare_weights(d.routed if what != "shared" else None, d.shared if what != "routed" else None)
        for r, order in ((1, 0), (3, 1)):
            assert np.array_equal(g.run_forward(ctx, wl, d, r=r, order=order), base), f"{what} r={r} changed the bits"
        assert ctx.last_tile_shape("routed_down_gemm")["tile_order"] == (what != "shared")
        assert ctx.last_tile_shape("shared_gate_up_gemm")["tile_order"] == (what != "routed")
        assert np.array_equal(g.run_forward_dep(ctx, wl, d, r_1=2, r_2=2, dep_order=0, attn_us=20.0), base)
        ctx.forget_weights()
    # a second set of weights prepared beside the first: each forward reads the copy of its own pointer
    inp2 = make_inputs(wl, seed=52)
    d2 = g.DeviceInputs(wl, inp2)
    base2 = g.run_forward(ctx, wl, d2)
    assert not np.array_equal(base2, base)
    ctx.prepare_weights(d.routed, d.shared)
    ctx.prepare_weights(d2.routed, d2.shared)
    assert np.array_equal(g.run_forward(ctx, wl, d), base)
    assert np.array_equal(g.run_forward(ctx, wl, d2), base2)
    # the caller rewrites the first set in place and prepares it again: the copy follows
    d.routed.copy_(d2.routed)
    d.shared.copy_(d2.shared)
    ctx.prepare_weights(d.routed, d.shared)
    d.tokens.copy_(d2.tokens)
    d.logits.copy_(d2.logits)
    assert np.array_equal(g.run_forward(ctx, wl, d), base2)
    ctx.forget_weights(d.routed, d.shared)
    assert np.array_equal(g.run_forward(ctx, wl, d), base2)
    assert np.array_equal(g.run_forward(ctx, wl, d2), base2)
    with pytest.raises(pkg_error()):               # nothing to prepare
        ctx.prepare_weights(None, None)
    ctx.destroy()


def pkg_error():
    import paper_2512_21487_amd as pkg
    return pkg.MoeEpError


@pytest.mark.parametrize("variant,units", [(14, 0), (14, 7), (14, 3), (14, 1), (2, 0), (2, 3), (2, 1), (13, 5), (11, 2),
                                           (1, 1), (31, 0), (31, 2), (22, 0), (22, 3), (21, 1)])
def test_row_tiles_cut_to_fit_the_experts(variant, units):
    """Row tiles are cut per expert to equal heights in units of 32 rows per row of wavefronts, at most
    `units` of them (0: as many as the variant holds): expert loads that are empty, one row, exact
    multiples of a unit and of a full tile, one row more, and several tiles with a remainder must all
    match the oracle, with 1 x 4 and with 2 x 2 wavefronts, and with the same bits as the default."""
    g = _gpu()
    wl = tiny_workload(name=f"cut_v{variant}_u{units}", n_tokens=2400, hidden=192, inter=320, n_experts=12, n_local=12,
                       top_k=1, n_shared=0)
    loads = [0, 1, 32, 33, 64, 65, 256, 257, 512, 700, 31, 0]      # rows of the 12 experts
    loads[-1] = wl.n_tokens - sum(loads)

    def exact_loads(inp):
        lg = np.full((wl.n_tokens, 12), -30.0, dtype=np.float32)
        t = 0
        for e, n in enumerate(loads):
            lg[t:t + n, e] = 5.0
            t += n
        inp["gate_logits"][:] = lg[np.random.default_rng(7).permutation(wl.n_tokens)]

    with _env(MOE_EP_GEMM_VARIANT=variant, MOE_EP_UP_UNITS=units or None, MOE_EP_DOWN_UNITS=units or None):
        out, ref = _full_parity(wl, seed=41, mutate=exact_loads)
    assert sorted(ref["count"][0].tolist()) == sorted(loads)
    inp = make_inputs(wl, seed=41)
    exact_loads(inp)
    with _env(MOE_EP_GEMM_VARIANT=None, MOE_EP_UP_UNITS=None, MOE_EP_DOWN_UNITS=None):
        ctx = g.make_ctx(wl)
        base = g.run_forward(ctx, wl, g.DeviceInputs(wl, inp))
        ctx.destroy()
    assert np.array_equal(out, base)


@pytest.mark.parametrize("mode", ["fp32", "scaled"])
@pytest.mark.parametrize("variant", [None, 1, 14])
def test_other_forms_of_the_expert_outputs_match_the_oracle(mode, variant):
    """MOE_EP_EXPERT_OUT: the routed experts' outputs reach the aggregation as fp32, or as bf16 already
    multiplied by the routing weight.  Both move a rounding point, so the bits differ from the default;
    the oracle bar is the same, and chunking still changes nothing."""
    g = _gpu()
    wl = tiny_workload(name=f"y_{mode}", n_tokens=777, hidden=192, inter=320, n_experts=10, local_begin=2,
                       n_local=6, top_k=3, n_shared=2, shared_inter=192)
    with _env(MOE_EP_EXPERT_OUT=mode, MOE_EP_GEMM_VARIANT=variant):
        out, ref = _full_parity(wl, seed=37, r=1)
        out3, _ = _full_parity(wl, seed=37, r=3, order=1)
    assert np.array_equal(out, out3)
    if mode == "fp32":   # one rounding less: never further from the oracle than the default path
        with _env(MOE_EP_EXPERT_OUT=None, MOE_EP_GEMM_VARIANT=variant):
            base, _ = _full_parity(wl, seed=37, r=1)
        e_new = np.abs(bf16_bits_to_f32(out).astype(np.float64) - ref["out"]).mean()
        e_old = np.abs(bf16_bits_to_f32(base).astype(np.float64) - ref["out"]).mean()
        assert e_new <= e_old


def test_grouped_copy_of_token_rows_matches_too():
    """MOE_EP_FUSED_GATHER=0: the token rows are first copied into expert-grouped order and the gate/up
    projection reads that copy (the path kept for comparison and for chunks of 4 GB and more)."""
    wl = tiny_workload(name="grouped_copy", n_tokens=333, hidden=192, inter=320, n_experts=10, local_begin=2,
                       n_local=6, top_k=3, n_shared=1, shared_inter=192)
    old = os.environ.get("MOE_EP_FUSED_GATHER")
    os.environ["MOE_EP_FUSED_GATHER"] = "0"
    try:
        _full_parity(wl, seed=35, r=2)
    finally:
        if old is None:
            os.environ.pop("MOE_EP_FUSED_GATHER", None)
        else:
            os.environ["MOE_EP_FUSED_GATHER"] = old


# ------------------------------------------------------------------ invariants on the GPU
def test_chunking_and_order_do_not_change_a_bit():
    g = _gpu()
    wl = CONFIGS["tiny"]
    inp = make_inputs(wl)
    ctx = g.make_ctx(wl, max_chunks=64)
    d = g.DeviceInputs(wl, inp)
    base = g.run_forward(ctx, wl, d, r=1, order=0)
    for r, order in [(1, 1), (2, 0), (4, 1), (7, 0), (64, 1)]:
        print(f"[case] tiny r={r} order={order}", flush=True)
        out = g.run_forward(ctx, wl, d, r=r, order=order)
        assert np.array_equal(out, base), f"r={r} order={order} changed the output bits"
    ctx.destroy()


def test_context_reuse_with_fewer_tokens():
    """A context sized for more tokens serves a smaller call; stale workspace rows do not leak."""
    g = _gpu()
    wl = CONFIGS["tiny"]
    inp = make_inputs(wl)
    ctx = g.make_ctx(wl)
    d = g.DeviceInputs(wl, inp)
    full = g.run_forward(ctx, wl, d)
    part = g.run_forward(ctx, wl, d, n_tokens=50)
    assert np.array_equal(part, full[:50])
    ctx.destroy()


@pytest.mark.parametrize("fused_out", [1, 0])
def test_pinned_host_pipeline_matches_device_mode(fused_out):
    """Pinned-host I/O, with the outbound transfer fused into the aggregation (default) and as a copy on
    a link stream of its own: the bits of the device-resident forward, shared experts included (their
    rows reach the host through the aggregation also where a token keeps no routed expert)."""
    g = _gpu()
    wl = tiny_workload(name="pinned", n_tokens=700, hidden=256, inter=192, n_experts=16,
                       local_begin=4, n_local=8, top_k=4, n_shared=1, shared_inter=128)
    inp = make_inputs(wl, seed=27)
    ctx = g.make_ctx(wl)
    base = g.run_forward(ctx, wl, g.DeviceInputs(wl, inp))
    ctx.destroy()
    with _env(MOE_EP_FUSED_OUT=fused_out):
        pctx = g.make_ctx(wl, pinned=True)
    pd = g.DeviceInputs(wl, inp, pinned=True)
    for r, order in [(1, 0), (4, 1), (8, 0)]:
        print(f"[case] pinned r={r} order={order} fused_out={fused_out}", flush=True)
        out = g.run_forward(pctx, wl, pd, r=r, order=order)
        assert np.array_equal(out, base)
    pctx.destroy()


def test_pinned_host_chunks_that_start_off_16_byte_boundaries():
    """7 experts and 15-token chunks: a chunk's gate scores start 420 bytes into the buffer, so the
    inbound copy takes its 4-byte path; the result must still match the oracle."""
    g = _gpu()
    wl = tiny_workload(name="pinned_odd", n_tokens=75, hidden=64, inter=64, n_experts=7, n_local=7,
                       top_k=3, n_shared=1, shared_inter=64)
    inp = make_inputs(wl, seed=31)
    ref = _oracle_full(inp, wl, 5)
    pctx = g.make_ctx(wl, pinned=True)
    pd = g.DeviceInputs(wl, inp, pinned=True)
    out = g.run_forward(pctx, wl, pd, r=5, order=1)
    _check_routing(pctx, ref, 5, wl.n_tokens, wl.top_k)
    assert rel_err_rows(bf16_bits_to_f32(out), ref["out"]) <= TOL
    pctx.destroy()


def test_device_mode_forward_can_be_captured_in_a_graph():
    """Device mode enqueues kernels on the caller's stream and nothing else (no allocation, no memset,
    no host synchronisation), so a forward can be captured once and replayed; every replay, with
    eager work and synchronisations in between, must reproduce the eager bits."""
    g = _gpu()
    wl = tiny_workload(name="graph", n_tokens=300, hidden=128, inter=192, n_experts=12, local_begin=2,
                       n_local=8, top_k=3, n_shared=1, shared_inter=64)
    inp = make_inputs(wl, seed=34)
    ctx = g.make_ctx(wl)
    d = g.DeviceInputs(wl, inp)
    eager = g.run_forward(ctx, wl, d, r=2, order=1)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    d.out.zero_()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        ctx.forward(d.tokens, d.logits, d.routed, d.shared, wl.top_k, 2, 1, n_tokens=wl.n_tokens, out=d.out,
                    stream=torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for rep in range(4):
        d.out.zero_()
        scratch = torch.randn(1 << 16, device="cuda").sum().item()  # eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        got = d.out.cpu().numpy().view(np.uint16)
        assert np.array_equal(got, eager), f"replay {rep} differs from the eager forward"
    ctx.destroy()


_DIGEST_SCRIPT = r"""
import hashlib, sys
sys.path.insert(0, {tests!r}); sys.path.insert(0, {root!r})
import gpu_util as g
from workloads import make_inputs, tiny_workload
wl = tiny_workload(name="serial", n_tokens=700, hidden=256, inter=192, n_experts=16, local_begin=4, n_local=8,
                   top_k=4, n_shared=1, shared_inter=128)
inp = make_inputs(wl, seed=36)
for pinned in (False, True):
    ctx = g.make_ctx(wl, pinned=pinned)
    d = g.DeviceInputs(wl, inp, pinned=pinned)
    for r, order in ((1, 0), (4, 1)):
        out = g.run_forward(ctx, wl, d, r=r, order=order)
        print(hashlib.sha256(out.tobytes()).hexdigest())
    for r_1, r_2, dep_order in ((2, 2, 0), (4, 2, 1)):
        out = g.run_forward_dep(ctx, wl, d, r_1, r_2, dep_order, 30.0)
        print(hashlib.sha256(out.tobytes()).hexdigest())
    ctx.destroy()
"""


def test_serialised_launches_give_the_same_bits():
    """The event graph between the streams is the race surface: with every launch made blocking
    (HIP_LAUNCH_BLOCKING=1, AMD_SERIALIZE_KERNEL=3) the outputs must be the bits of the asynchronous
    run, in device and pinned-host mode, chunked and not, through moe_ep_forward and through
    moe_ep_forward_dep (attention-group stream, both orders)."""
    import subprocess
    import sys
    here = os.path.dirname(os.path.abspath(__file__))
    script = _DIGEST_SCRIPT.format(tests=here, root=os.path.dirname(here))
    digests = []
    for extra in ({}, {"HIP_LAUNCH_BLOCKING": "1", "AMD_SERIALIZE_KERNEL": "3"}):
        env = dict(os.environ, **extra)
        p = subprocess.run([sys.executable, "-c", script], capture_output=True, text=True, env=env, timeout=300)
        assert p.returncode == 0, p.stderr[-2000:]
        digests.append([l for l in p.stdout.split() if len(l) == 64])
    assert len(digests[0]) == 8 and digests[0] == digests[1]
    assert len(set(digests[0])) == 1  # and chunking, order and I/O mode change nothing either


@pytest.mark.parametrize("fused_out", [False, True])
def test_measured_timeline_obeys_the_precedence_rules(fused_out):
    """The measured schedule of a pinned-host forward with r_2 = 3 (moe_ep_get_timeline): every stage
    appears once per chunk, a chunk's compute starts after its inbound copy ends and its outbound copy
    after its aggregation ends (Sec. 3.2, Eq. limitation, rules 7-8), each resource runs its tasks in
    chunk order without overlap (rules 3-5).  With the outbound transfer fused into the aggregation (the
    default of moe_ep_forward) there is no outbound copy and the aggregation is the chunk's last task."""
    g = _gpu()
    wl = tiny_workload(name="timeline", n_tokens=600, hidden=256, inter=192, n_experts=16, n_local=16, top_k=2)
    with _env(MOE_EP_FUSED_OUT=1 if fused_out else 0):
        pctx = g.make_ctx(wl, pinned=True)
    pd = g.DeviceInputs(wl, make_inputs(wl, seed=33), pinned=True)
    base = g.run_forward(pctx, wl, pd, r=3)
    pctx.set_profiling(1)
    out = g.run_forward(pctx, wl, pd, r=3)
    assert np.array_equal(out, base)
    tl = pctx.get_timeline()
    pctx.get_stage_ms()
    pctx.set_profiling(0)
    by = {}
    for name, fwd, b, e in tl:
        assert fwd == 0 and e >= b >= 0.0
        by.setdefault(name, []).append((b, e))
    stages = ["copy_in", "router", "partition", "routed_gate_up_gemm", "routed_down_gemm", "aggregation"]
    if not fused_out:
        stages.append("copy_out")
    else:
        assert "copy_out" not in by
    for name in stages:
        assert len(by[name]) == 3, name
        for (b0, e0), (b1, e1) in zip(by[name], by[name][1:]):
            assert b1 >= e0 - 1e-3, f"{name}: chunks overlap on one resource"
    eps = 2e-3  # event timestamps resolve to about a microsecond
    for c in range(3):
        assert by["routed_gate_up_gemm"][c][0] >= by["copy_in"][c][1] - eps
        assert by["router"][c][0] >= by["copy_in"][c][0] - eps   # gate and partition need the scores only
        if not fused_out:
            assert by["copy_out"][c][0] >= by["aggregation"][c][1] - eps
        assert by["routed_down_gemm"][c][0] >= by["routed_gate_up_gemm"][c][1] - eps
    last = by["aggregation" if fused_out else "copy_out"][2][1]
    assert len(by["forward"]) == 1 and by["forward"][0][1] >= last - eps
    pctx.destroy()


def test_auto_chunks_from_timing_model():
    """r_chunks = 0 takes r_2 from the context's timing model (Sec. 4.2) and changes no output bit."""
    g = _gpu()
    import paper_2512_21487_amd as pkg
    wl = CONFIGS["tiny"]
    ctx = g.make_ctx(wl, max_chunks=8)
    d = g.DeviceInputs(wl, make_inputs(wl))
    base = g.run_forward(ctx, wl, d, r=1)
    with pytest.raises(pkg.MoeEpError) as ei:       # no model yet
        g.run_forward(ctx, wl, d, r=0)
    assert ei.value.code == -4
    # transfers dominate and scale with tokens, start-up costs are small: chunking pays off
    model = pkg.PipelineModel(0.001, 0.01, 0.001, 0.005, 0.001, 0.01)
    ctx.set_pipeline_model(model)
    out = g.run_forward(ctx, wl, d, r=0)
    want = pkg.choose_chunks(model, wl.n_tokens, 8)
    assert ctx.last_chunks() == want and want > 1
    assert np.array_equal(out, base)
    ctx.set_pipeline_model(pkg.PipelineModel(1.0, 0.0, 1.0, 0.0, 1.0, 0.0))   # start-up only -> 1
    g.run_forward(ctx, wl, d, r=0)
    assert ctx.last_chunks() == 1
    ctx.destroy()


def test_errors_surface_as_status_codes():
    g = _gpu()
    import paper_2512_21487_amd as pkg
    wl = CONFIGS["tiny"]
    ctx = g.make_ctx(wl)
    d = g.DeviceInputs(wl, make_inputs(wl))
    with pytest.raises(pkg.MoeEpError) as ei:
        ctx.forward(d.tokens, d.logits, d.routed, d.shared, 3, 1, 0, out=d.out)
    assert ei.value.code == -1 and "top_k" in str(ei.value)
    with pytest.raises(pkg.MoeEpError):
        ctx.forward(d.tokens, d.logits, d.routed, None, 2, 1, 0, out=d.out)
    g.run_forward(ctx, wl, d)  # still usable afterwards
    ctx.destroy()


def test_pointers_the_gpu_cannot_use_are_rejected_before_any_launch():
    """Raw addresses (which the binding passes through unchecked) of pageable host memory, of pinned
    memory in the wrong mode and of a device allocation that ends before the forward's extent give
    MOE_EP_EINVAL naming the argument; nothing is enqueued and the context stays usable."""
    import ctypes
    g = _gpu()
    import paper_2512_21487_amd as pkg
    wl = CONFIGS["tiny"]
    inp = make_inputs(wl)
    ctx = g.make_ctx(wl)
    d = g.DeviceInputs(wl, inp)
    good = g.run_forward(ctx, wl, d)
    args = dict(tokens=d.tokens.data_ptr(), logits=d.logits.data_ptr(), routed=d.routed.data_ptr(),
                shared=d.shared.data_ptr(), out=d.out.data_ptr())

    def call(**swap):
        a = dict(args, **swap)
        ctx.forward(a["tokens"], a["logits"], a["routed"], a["shared"], wl.top_k, 1, 0,
                    n_tokens=wl.n_tokens, out=a["out"])

    pageable = np.ascontiguousarray(inp["tokens"])
    with pytest.raises(pkg.MoeEpError) as ei:
        call(tokens=pageable.ctypes.data)
    assert ei.value.code == -1 and "tokens" in str(ei.value)
    host_w = np.ascontiguousarray(inp["routed_w"])
    with pytest.raises(pkg.MoeEpError) as ei:
        call(routed=host_w.ctypes.data)
    assert ei.value.code == -1 and "routed_w" in str(ei.value)
    # a device allocation of its own that is too short for [T, M] bf16
    hip = ctypes.CDLL("libamdhip64.so")
    small = ctypes.c_void_p()
    assert hip.hipMalloc(ctypes.byref(small), ctypes.c_size_t(4096)) == 0
    try:
        base, size = ctypes.c_void_p(), ctypes.c_size_t()
        assert hip.hipMemGetAddressRange(ctypes.byref(base), ctypes.byref(size), small) == 0
        assert (base.value, size.value) == (small.value, 4096)  # what the library will be told
        with pytest.raises(pkg.MoeEpError) as ei:
            call(out=small.value)
        assert ei.value.code == -1 and "out" in str(ei.value) and "smaller" in str(ei.value)
    finally:
        assert hip.hipFree(small) == 0
    assert np.array_equal(g.run_forward(ctx, wl, d), good)
    ctx.destroy()
    # pinned-host mode wants pinned host memory for the three streamed buffers
    pctx = g.make_ctx(wl, pinned=True)
    pd = g.DeviceInputs(wl, inp, pinned=True)
    with pytest.raises(pkg.MoeEpError) as ei:
        pctx.forward(d.tokens.data_ptr(), pd.logits.data_ptr(), pd.routed.data_ptr(), pd.shared.data_ptr(),
                     wl.top_k, 1, 0, n_tokens=wl.n_tokens, out=pd.out.data_ptr())
    assert ei.value.code == -1 and "tokens" in str(ei.value) and "pinned" in str(ei.value)
    assert np.array_equal(g.run_forward(pctx, wl, pd), good)
    pctx.destroy()


def test_binding_rejects_tensors_of_the_wrong_size_or_place():
    g = _gpu()
    wl = CONFIGS["tiny"]
    ctx = g.make_ctx(wl)
    d = g.DeviceInputs(wl, make_inputs(wl))
    with pytest.raises(ValueError, match="out holds"):
        ctx.forward(d.tokens, d.logits, d.routed, d.shared, wl.top_k, 1, 0, out=d.out[: wl.n_tokens // 2])
    with pytest.raises(ValueError, match="tokens must be contiguous"):
        ctx.forward(d.tokens.t(), d.logits, d.routed, d.shared, wl.top_k, 1, 0, n_tokens=wl.n_tokens, out=d.out)
    with pytest.raises(ValueError, match="gate_logits must be a device tensor"):
        ctx.forward(d.tokens, d.logits.cpu(), d.routed, d.shared, wl.top_k, 1, 0, out=d.out)
    ctx.destroy()


def test_device_probe_reports_plausible_rates():
    """The measurement aid: the register-only MFMA loop stays below the vendor peak, all-zero operands
    (less switching, more clock) are not slower than random ones, and the copy moves a few TB/s."""
    import paper_2512_21487_amd as pkg
    rnd = pkg.probe_device(0, zero_operands=False)
    zero = pkg.probe_device(0, zero_operands=True)
    print(f"       random {rnd}  zero {zero}", flush=True)
    assert 500.0 < rnd["mfma_tflops"] <= 2600.0 and 0.5 < rnd["mfma_ghz"] <= 2.6
    assert zero["mfma_tflops"] >= 0.98 * rnd["mfma_tflops"] and zero["mfma_tflops"] <= 2600.0
    assert 1000.0 < rnd["copy_gbs"] < 8000.0


# ------------------------------------------------------------------ full-size configurations
def _full_size_parity(name, variants, pinned=False, seed=0, tile_variants=()):
    """At the benchmark's sizes and in the launch configuration bench.py times (weights prepared in tile
    order): the whole layer is
    run once on the CPU oracle and EVERY output element is compared with it (so every expert's first
    and last row and every row-tile edge is covered, whatever tile the library picks); routing of
    every token and chunk bit-exact; every (r, order) variant and every listed tile variant
    bit-identical to the first forward."""
    g = _gpu()
    wl = CONFIGS[name]
    inp = make_inputs(wl, seed=seed)
    T, k = wl.n_tokens, wl.top_k
    print(f"[case] {name} seed={seed}: oracle over all {T} tokens on {oracle.threads()} threads", flush=True)
    ref = _oracle_full(inp, wl, 1)
    idx, w = ref["idx"], ref["w"]
    local = (idx >= wl.local_begin) & (idx < wl.local_begin + wl.n_local)
    assert int(ref["offset"][0][-1]) == int(local.sum())
    ctx = g.make_ctx(wl, pinned=pinned)
    d = g.DeviceInputs(wl, inp, pinned=pinned)
    ctx.prepare_weights(d.routed, d.shared)        # as bench.py does: the weights are read in tile order
    first = None
    for r, order in variants:
        print(f"[case] {name} r={r} order={order} pinned={pinned}", flush=True)
        out = g.run_forward(ctx, wl, d, r=r, order=order)
        Tc = (T + r - 1) // r
        kept_total = 0
        for c in range(r):
            t0 = c * Tc
            Tn = 0 if t0 >= T else min(Tc, T - t0)
            got = ctx.get_routing(c)
            part = oracle.dispatch(idx[t0:t0 + Tn], wl.local_begin, wl.n_local)
            assert np.array_equal(got["idx"], idx[t0:t0 + Tn])
            for key in ("count", "offset", "perm", "pos"):
                assert np.array_equal(got[key], part[key]), f"{key} differs in chunk {c}"
            assert np.max(np.abs(got["w"].astype(np.float64) - w[t0:t0 + Tn])) <= W_TOL
            kept_total += int(part["offset"][-1])
        assert kept_total == int(local.sum())      # token conservation over the chunks
        if first is None:
            got_f = bf16_bits_to_f32(out)
            err, err_all = rel_err_rows(got_f, ref["out"]), rel_err(got_f, ref["out"])
            # the same figure over the rows most exposed to a tiling mistake: first and last row of
            # every local expert (their tokens), reported so that a failure names where it is
            off = ref["offset"][0]
            rows = np.concatenate([off[:-1][off[1:] > off[:-1]], off[1:][off[1:] > off[:-1]] - 1])
            edge_tok = np.unique(ref["perm"][0][rows] // k)
            edge_err = rel_err_rows(got_f[edge_tok], ref["out"][edge_tok])
            print(f"       rel_err={err:.3e} over all {T} x {wl.hidden} elements (expert edge rows: "
                  f"{edge_err:.3e}; one floor over all rows: {err_all:.3e}), kept={kept_total}", flush=True)
            assert err <= TOL and err_all <= 2 * TOL
            if wl.n_shared == 0:                   # rows with nothing kept are exact zeros
                assert not out[~local.any(axis=1)].any()
            first = out
        else:
            assert np.array_equal(out, first), f"r={r} order={order} changed the output bits"
    ctx.forget_weights()                           # the weights read where the caller keeps them: the same bits
    print(f"[case] {name} weights in the caller's layout", flush=True)
    assert np.array_equal(g.run_forward(ctx, wl, d, r=variants[0][0], order=variants[0][1]), first)
    ctx.destroy()
    for tv in tile_variants:                       # told to use one tile shape: the same bits
        print(f"[case] {name} tile variant {tv}", flush=True)
        with _env(MOE_EP_GEMM_VARIANT=tv):
            vctx = g.make_ctx(wl, pinned=pinned)
            out = g.run_forward(vctx, wl, d, r=1, order=0)
            vctx.destroy()
        assert np.array_equal(out, first), f"tile variant {tv} changed the output bits"
    if tile_variants:                              # every projection out of the 32 x 32 x 16 instruction: the same bits
        print(f"[case] {name} MOE_EP_MFMA=32", flush=True)
        with _env(MOE_EP_MFMA=32):
            vctx = g.make_ctx(wl, pinned=pinned)
            out = g.run_forward(vctx, wl, d, r=1, order=0)
            assert vctx.last_tile_shape("routed_gate_up_gemm")["mfma_rows"] == 32
            vctx.destroy()
        assert np.array_equal(out, first), "the 32 x 32 x 16 kernels changed the output bits"


def _sweep(wl, orders=(0,)):
    """Every r of the workload's sweep; with shared experts both orders at the ends of the sweep."""
    cases = [(r, 0) for r in wl.r_sweep]
    if wl.n_shared > 0:
        cases += [(wl.r_sweep[-1], 1), (wl.r_sweep[0], 1)]
        if len(wl.r_sweep) > 2:
            cases.append((wl.r_sweep[1], 1))
    return cases


def test_dsv2_lite_full_size():
    _full_size_parity("dsv2_lite", _sweep(CONFIGS["dsv2_lite"]), tile_variants=(1, 11, 21, 31))


def test_qwen3_30b_full_size_skewed():
    _full_size_parity("qwen3_30b", _sweep(CONFIGS["qwen3_30b"]), tile_variants=(1, 11, 21, 31))


def test_dsv2_expert_group_share_full_size():
    _full_size_parity("dsv2_eg", _sweep(CONFIGS["dsv2_eg"]), tile_variants=(1, 11, 21, 31))


@pytest.mark.parametrize("name", ["qwen3_235b_eg_256", "qwen3_235b_eg_1024", "qwen3_235b_eg_4096"])
def test_qwen3_235b_expert_group_share_decode_pinned(name):
    _full_size_parity(name, _sweep(CONFIGS[name]), pinned=True, tile_variants=(1, 11, 21, 31))


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_decode_share_other_seeds_keep_the_margin(seed):
    """The configuration with the least margin against the tolerance, on other draws of the inputs."""
    _full_size_parity("qwen3_235b_eg_4096", [(1, 0)], pinned=False, seed=seed)


@pytest.mark.parametrize("name", ["qwen3_235b_eg_256", "qwen3_235b_eg_4096"])
def test_chosen_chunk_count_is_as_fast_as_the_best_measured(name):
    """r_chunks = 0 with task models fitted on this GPU (Sec. 4.1), including the second set for tasks
    that run beside others: the r_2 the library picks must run within 5 % of the fastest r_2 of the
    measured sweep (Sec. 4.2, "Determine r_2 and m_e")."""
    g = _gpu()
    import bench
    wl = CONFIGS[name]
    inp = make_inputs(wl)
    ctx = g.make_ctx(wl, pinned=True, max_chunks=8)
    d = g.DeviceInputs(wl, inp, pinned=True)
    stream = torch.cuda.current_stream().cuda_stream
    res = bench.fit_pipeline(ctx, d.tokens, d.logits, d.routed, d.shared, d.out, wl.n_tokens, wl.top_k, 0, stream)
    print(f"       chosen r = {res['chosen_r']} (independent resources: {res['chosen_r_independent_resources']}), "
          f"measured {res['measured_ms']}, predicted {res['predicted_ms']}", flush=True)
    best = min(res["measured_ms"].values())
    assert res["measured_ms"][str(res["chosen_r"])] <= 1.05 * best
    ctx.destroy()
