"""moe_ep_forward_noalloc, the entry point for callers that cannot allocate: the same forward on the
library's static workspace.  Its output must be the bits moe_ep_forward gives (which the parity tests
hold against the oracle), on two calls in a row that share the workspace, the second with a smaller
input, and its limits must come back as errors before anything is launched."""
import ctypes

import numpy as np
import pytest

from workloads import make_inputs, tiny_workload

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _cfg(pkg, wl, max_tokens, max_chunks=2):
    return pkg.MoeEpConfig(wl.hidden, wl.inter, wl.n_experts, wl.local_begin, wl.n_local, wl.n_shared,
                           wl.shared_inter, max_tokens, wl.top_k, max_chunks, pkg.IO_DEVICE, 0)


def test_noalloc_forward_gives_the_bits_of_the_context_forward():
    import gpu_util as g
    import paper_2512_21487_amd as pkg
    # several row tiles per expert with ragged tails, a local share, two shared experts
    wl = tiny_workload(name="noalloc", n_tokens=900, hidden=256, inter=320, n_experts=12, local_begin=3,
                       n_local=7, top_k=3, n_shared=2, shared_inter=192)
    inp = make_inputs(wl, seed=61)
    d = g.DeviceInputs(wl, inp)
    ctx = g.make_ctx(wl)
    want_full = g.run_forward(ctx, wl, d, r=1, order=0)
    want_small = g.run_forward(ctx, wl, d, r=1, order=0, n_tokens=333)
    ctx.destroy()
    assert want_full.any()

    cfg = _cfg(pkg, wl, wl.n_tokens)
    assert 0 < pkg.workspace_bytes(cfg) <= pkg.NOALLOC_SCRATCH_BYTES
    print(f"[case] noalloc T={wl.n_tokens} then T=333, workspace {pkg.workspace_bytes(cfg)} bytes", flush=True)
    before = torch.cuda.memory_allocated()
    d.out.zero_()
    torch.cuda.synchronize()
    pkg.forward_noalloc(cfg, d.tokens, d.logits, d.routed, d.shared, wl.top_k, 1, 0, n_tokens=wl.n_tokens, out=d.out)
    torch.cuda.synchronize()
    got_full = d.out.cpu().numpy().view(np.uint16).copy()
    assert np.array_equal(got_full, want_full)
    # second call in a row on the same workspace, fewer tokens, chunked and interleaved this time
    d.out.zero_()
    torch.cuda.synchronize()
    pkg.forward_noalloc(cfg, d.tokens, d.logits, d.routed, d.shared, wl.top_k, 2, 1, n_tokens=333, out=d.out)
    torch.cuda.synchronize()
    got_small = d.out.cpu().numpy().view(np.uint16).copy()
    assert np.array_equal(got_small[:333], want_small)
    assert not got_small[333:].any()                 # rows beyond the call's tokens are untouched
    assert torch.cuda.memory_allocated() == before


def test_noalloc_forward_rejects_what_it_cannot_serve():
    import gpu_util as g
    import paper_2512_21487_amd as pkg
    wl = tiny_workload(name="noalloc_err", n_tokens=64, hidden=64, inter=64, n_experts=8, n_local=8, top_k=2)
    d = g.DeviceInputs(wl, make_inputs(wl, seed=62))
    args = (d.tokens, d.logits, d.routed, None, wl.top_k)
    big = _cfg(pkg, wl, 1 << 20)                      # a workspace far beyond the static array
    assert pkg.workspace_bytes(big) > pkg.NOALLOC_SCRATCH_BYTES
    with pytest.raises(pkg.MoeEpError) as ei:
        pkg.forward_noalloc(big, *args, 1, 0, n_tokens=64, out=d.out)
    assert ei.value.code == -1 and "MOE_EP_NOALLOC_SCRATCH_BYTES" in str(ei.value)
    ok = _cfg(pkg, wl, 64)
    with pytest.raises(pkg.MoeEpError) as ei:         # no context, no timing model
        pkg.forward_noalloc(ok, *args, 0, 0, n_tokens=64, out=d.out)
    assert ei.value.code == -1 and "r_chunks" in str(ei.value)
    pinned = _cfg(pkg, wl, 64)
    pinned.io_mode = pkg.IO_PINNED_HOST
    with pytest.raises(pkg.MoeEpError) as ei:
        pkg.forward_noalloc(pinned, *args, 1, 0, n_tokens=64, out=d.out)
    assert ei.value.code == -1 and "MOE_EP_IO_DEVICE" in str(ei.value)
    with pytest.raises(pkg.MoeEpError) as ei:         # more tokens than the configuration was sized for
        pkg.forward_noalloc(_cfg(pkg, wl, 32), *args, 1, 0, n_tokens=64, out=d.out)
    assert ei.value.code == -1
    pkg.forward_noalloc(ok, *args, 1, 0, n_tokens=64, out=d.out)   # and the valid call still runs
    torch.cuda.synchronize()
    assert d.out.cpu().numpy().any()
