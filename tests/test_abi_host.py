"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects
bad arguments before touching HIP (no compute call is made here)."""
import ctypes
import os
import re

import pytest

import paper_2512_21487_amd as pkg
from paper_2512_21487_amd import MoeEpConfig

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _good(**kw):
    base = dict(hidden=256, inter=512, n_experts=8, local_begin=0, n_local=8, n_shared=1,
                shared_inter=512, max_tokens=128, max_top_k=2, max_chunks=8, io_mode=0, device=0)
    base.update(kw)
    return MoeEpConfig(**base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "moe_ep.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(moe_ep_[a-z_]+)\s*\(", header))
    assert {"moe_ep_create", "moe_ep_forward", "moe_ep_destroy"} <= names
    lib = pkg.load_library()
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in moe_ep.h but not exported"
    assert lib.moe_ep_version().decode().count(".") == 1
    assert not hasattr(lib, "moe_ep_probe_device")   # the benchmark's aid is not in the layer's library
    probe_header = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "moe_ep_probe.h")).read(), flags=re.S)
    probe_names = set(re.findall(r"\b(moe_ep_[a-z_]+)\s*\(", probe_header))
    assert probe_names == {"moe_ep_probe_device"}
    assert hasattr(pkg.load_probe_library(), "moe_ep_probe_device")


def test_config_struct_matches_header():
    header = open(os.path.join(ROOT, "include", "moe_ep.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} moe_ep_config;", header, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"int32_t\s+(\w+)\s*;", body)
    assert fields == [f[0] for f in MoeEpConfig._fields_]
    assert ctypes.sizeof(MoeEpConfig) == 4 * len(fields)


def test_valid_config_and_workspace_size():
    cfg = _good()
    assert pkg.validate_config(cfg) == (0, "ok")
    ws = pkg.workspace_bytes(cfg)
    # the experts' outputs alone: A_max * M * 2 bytes (the grouped copy of the token rows is not part of
    # the default workspace: the gate/up projection gathers them itself)
    assert ws >= 128 * 2 * 256 * 2
    assert pkg.workspace_bytes(_good(hidden=100)) == 0


def test_size_of_the_tile_order_weight_copies():
    """Per expert and projection: output rows rounded up to whole weight tiles (gate/up: 128 activation
    columns = 256 weight rows per tile; down: 256 rows) times the reduction length, bf16."""
    from paper_2512_21487_amd.binding import prepared_weight_bytes
    cfg = _good(hidden=320, inter=192, n_experts=8, n_local=5, n_shared=2, shared_inter=192)
    up = 5 * 2 * 256 * 320 * 2          # 192 activation columns = 2 tiles of 128
    down = 5 * 2 * 256 * 192 * 2        # 320 output columns = 2 tiles of 256
    s_up = 2 * 2 * 256 * 320 * 2
    s_down = 2 * 256 * (2 * 192) * 2    # one group over the concatenated intermediate
    assert prepared_weight_bytes(cfg, True, False) == up + down
    assert prepared_weight_bytes(cfg, False, True) == s_up + s_down
    assert prepared_weight_bytes(cfg, True, True) == up + down + s_up + s_down
    assert prepared_weight_bytes(_good(n_shared=0, shared_inter=0), False, True) == 0
    assert prepared_weight_bytes(_good(hidden=100)) == 0
    # full tiles: exactly the size of the weights
    big = _good(hidden=5120, inter=1536, n_experts=160, n_local=20, n_shared=2, shared_inter=1536, max_tokens=16384, max_top_k=6)
    assert prepared_weight_bytes(big) == (20 + 2) * 3 * 1536 * 5120 * 2


@pytest.mark.parametrize("kw,word", [
    (dict(hidden=100), "hidden"), (dict(hidden=0), "hidden"), (dict(inter=96), "inter"),
    (dict(n_experts=0), "n_experts"), (dict(n_experts=513, n_local=8), "n_experts"),
    (dict(n_local=0), "local"), (dict(local_begin=4, n_local=5), "local"),
    (dict(local_begin=-1), "local"), (dict(n_shared=-1), "n_shared"),
    (dict(n_shared=1, shared_inter=0), "shared_inter"), (dict(max_tokens=0), "max_tokens"),
    (dict(max_top_k=0), "max_top_k"), (dict(max_top_k=9), "max_top_k"),
    (dict(max_top_k=65, n_experts=128, n_local=8), "max_top_k"),
    (dict(max_chunks=0), "max_chunks"), (dict(max_chunks=65), "max_chunks"),
    (dict(io_mode=2), "io_mode"), (dict(device=-1), "device"),
    (dict(hidden=32768, inter=32768), "2^30"), (dict(hidden=32768, n_shared=1, shared_inter=32768), "2^30"),
])
def test_bad_config_is_rejected_with_a_reason(kw, word):
    rc, why = pkg.validate_config(_good(**kw))
    assert rc == -1 and word in why


def test_create_rejects_bad_config_without_touching_hip():
    lib = pkg.load_library()
    ctx = ctypes.c_void_p()
    cfg = _good(hidden=100)
    assert lib.moe_ep_create(ctypes.byref(cfg), ctypes.byref(ctx)) == -1
    assert not ctx.value
    assert lib.moe_ep_create(ctypes.byref(_good()), None) == -1
    assert lib.moe_ep_destroy(None) == 0
    assert lib.moe_ep_forward(None, None, None, None, None, 1, 1, 0, 0, None, None) == -1


@pytest.mark.parametrize("kw,word", [
    (dict(top_k=0), "top_k"), (dict(top_k=3), "top_k"), (dict(r_chunks=-1), "r_chunks"),
    (dict(r_chunks=9), "r_chunks"), (dict(n_tokens=-1), "n_tokens"),
    (dict(n_tokens=129), "n_tokens"), (dict(order=2), "order"), (dict(routed_w=None), "routed_w"),
    (dict(shared_w=None), "shared_w"), (dict(tokens=None), "tokens"), (dict(out=None), "tokens"),
    (dict(gate_logits=None), "tokens"),
])
def test_bad_forward_arguments_are_rejected(kw, word):
    args = dict(tokens=0x1000, gate_logits=0x2000, routed_w=0x3000, shared_w=0x4000, top_k=2,
                r_chunks=1, order=0, n_tokens=128, out=0x5000)
    assert pkg.validate_forward(_good(), **args) == (0, "ok")
    args.update(kw)
    rc, why = pkg.validate_forward(_good(), **args)
    assert rc == -1 and word in why


def test_forward_edge_arguments_that_are_legal():
    base = dict(tokens=0x1000, gate_logits=0x2000, routed_w=0x3000, shared_w=0x4000, top_k=2,
                r_chunks=8, order=1, n_tokens=3, out=0x5000)
    assert pkg.validate_forward(_good(), **base)[0] == 0          # r_chunks > n_tokens
    assert pkg.validate_forward(_good(), **dict(base, r_chunks=0))[0] == 0   # 0 = from the timing model
    base.update(n_tokens=0, tokens=None, gate_logits=None, out=None)
    assert pkg.validate_forward(_good(), **base)[0] == 0          # empty call is a no-op
    noshared = _good(n_shared=0, shared_inter=0)
    args = dict(base, shared_w=None, order=77)                     # order ignored without shared
    assert pkg.validate_forward(noshared, **args)[0] == 0
    assert pkg.validate_forward(noshared, **dict(args, shared_w=0x4000))[0] == -1


def test_chunk_ranges_partition_the_tokens():
    """moe_ep_chunk_range (host only): the r_1 * r_2 chunks tile [0, n_tokens) in order, a micro-batch
    holds ceil(n_tokens / r_1) tokens except the last ones, a chunk ceil(micro-batch / r_2) except the
    last ones of its micro-batch, chunks never straddle micro-batches, and r_1 = 1 is the ceil(n / r)
    cut moe_ep_forward documents (Sec. 2.3)."""
    from paper_2512_21487_amd.binding import chunk_range
    for T in (0, 1, 5, 64, 700, 4097):
        for r_1 in (1, 2, 3, 7, 16):
            for r_2 in (1, 2, 5):
                Tm = -(-T // r_1) if T else 0
                Tc = -(-Tm // r_2) if Tm else 0
                pos = 0
                for c in range(r_1 * r_2):
                    t0, n = chunk_range(T, r_1, r_2, c)
                    i, j = divmod(c, r_2)
                    assert 0 <= n <= Tc
                    if n:
                        assert t0 == pos and i * Tm <= t0 and t0 + n <= min(T, (i + 1) * Tm)
                        assert t0 == i * Tm + j * Tc
                        pos = t0 + n
                    else:
                        assert t0 <= T
                assert pos == T
                if r_1 == 1:
                    for c in range(r_2):
                        want0 = min(c * Tc, T)
                        assert chunk_range(T, 1, r_2, c) == (want0, min(Tc, T - want0))
    lib = pkg.load_library()
    a, b = ctypes.c_int32(), ctypes.c_int32()
    for args in ((-1, 1, 1, 0), (8, 0, 1, 0), (8, 1, 0, 0), (8, 2, 2, 4), (8, 2, 2, -1)):
        assert lib.moe_ep_chunk_range(*args, ctypes.byref(a), ctypes.byref(b)) == -1
    assert lib.moe_ep_chunk_range(8, 1, 1, 0, None, ctypes.byref(b)) == -1


def test_tensor_marshalling_checks():
    """The binding's tensor checks (size, density, placement) need no GPU."""
    torch = pytest.importorskip("torch")
    from paper_2512_21487_amd.binding import _check_tensor
    t = torch.zeros((8, 64), dtype=torch.int16)
    _check_tensor(None, "shared_w", 0, False)
    _check_tensor(12345, "tokens", 1 << 20, False)          # raw addresses are the library's to check
    with pytest.raises(ValueError, match="holds 1024 bytes"):
        _check_tensor(t, "tokens", 1025, True)
    with pytest.raises(ValueError, match="contiguous"):
        _check_tensor(t.t(), "tokens", 16, True)
    with pytest.raises(ValueError, match="pinned host tensor"):
        _check_tensor(t, "tokens", 1024, True)
    with pytest.raises(ValueError, match="device tensor"):
        _check_tensor(t, "tokens", 1024, False)


def test_row_tile_of_the_routed_projections():
    """The tallest row tile follows from expected rounds of tiles x measured time per tile of each shape
    (128 / 160 / 224 / 256 rows: 1 / 1.15 / 1.74 / 1.79 for a long K): worked by hand for the benchmark
    shapes on 256 compute units."""
    from paper_2512_21487_amd import routed_tile_rows
    dsv2_eg = _good(hidden=5120, inter=1536, n_experts=160, n_local=20, shared_inter=1536, n_shared=2,
                    max_tokens=16384, max_top_k=6)
    # 614 rows per expert: 5.15 tiles of 128, 4.15 of 160, 3.01 of 224, 3 of 256; gate/up 12 column
    # tiles: 5, 4, 3, 3 rounds = 5.0, 4.59, 5.23, 5.38 in units of a 128-row tile
    assert routed_tile_rows(dsv2_eg, 16384, 6, False) == 160
    # down, 20 column tiles: 9, 7, 5, 5 rounds = 9.0, 7.95, 8.55, 8.82
    assert routed_tile_rows(dsv2_eg, 16384, 6, True) == 160
    decode = _good(hidden=4096, inter=1536, n_experts=128, n_local=16, n_shared=0, shared_inter=0,
                   max_tokens=4096, max_top_k=8)
    # 256 +- 16 rows per expert: 2.5 tiles of 128 or 2 of 160; gate/up 480 or 384 tiles: 2 rounds both
    assert routed_tile_rows(decode, 4096, 8, False) == 128
    # down, 16 column tiles: 640 tiles = 3 rounds against 512 = 2 rounds
    assert routed_tile_rows(decode, 4096, 8, True) == 160
    for T in (1, 256, 1024):   # one tile per expert with every shape: the cheapest one
        assert routed_tile_rows(decode, T, 8, False) == routed_tile_rows(decode, T, 8, True) == 128
    # 180 +- 13 rows per expert, 8 experts x 32 column tiles = 256 columns of tiles: one 224-row tile each
    # would be one round (1.71) against two rounds of 128-row tiles (2.0), but the tall shapes are not
    # candidates (measured slower wherever they win on paper)
    few = _good(hidden=8192, inter=1536, n_experts=8, n_local=8, n_shared=0, shared_inter=0, max_tokens=1440,
                max_top_k=1)
    assert routed_tile_rows(few, 1440, 1, True) == 128
