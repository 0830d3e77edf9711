"""ctypes binding of include/moe_ep.h -- same names, argument marshalling only."""
from __future__ import annotations

import ctypes
import os
import sys
from typing import Dict, Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmoe_ep.so")
_lib: Optional[ctypes.CDLL] = None

ORDER_SHARED_FIRST = 0
ORDER_INTERLEAVED = 1
IO_DEVICE = 0
IO_PINNED_HOST = 1
STAGES = ("router", "partition", "routed_gate_up_gemm", "routed_down_gemm",
          "shared_gate_up_gemm", "shared_down_gemm", "aggregation", "forward", "copy_in",
          "copy_out", "attention")

_STATUS = {0: "OK", -1: "EINVAL", -2: "ENOMEM", -3: "EHIP", -4: "ESTATE"}


def chunk_range(T: int, r_1: int, r_2: int, c: int):
    """moe_ep_chunk_range: (first token, tokens) of chunk c = i * r_2 + j."""
    first, count = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = load_library().moe_ep_chunk_range(T, r_1, r_2, c, ctypes.byref(first), ctypes.byref(count))
    if rc != 0:
        raise ValueError("moe_ep_chunk_range: arguments out of range")
    return first.value, count.value


class MoeEpError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"moe_ep: {_STATUS.get(code, code)}: {msg}")
        self.code = code


class PipelineModel(ctypes.Structure):
    """Mirror of ``moe_ep_pipeline_model`` (alpha + beta * tokens-per-chunk for each resource; the
    ``*_beside`` coefficients, all zero when absent, price the tasks while other resources are active)."""
    _fields_ = [(n, ctypes.c_double) for n in (
        "alpha_in", "beta_in", "alpha_e", "beta_e", "alpha_out", "beta_out",
        "alpha_in_beside", "beta_in_beside", "alpha_e_beside", "beta_e_beside", "alpha_out_beside",
        "beta_out_beside")]


class DepModels(ctypes.Structure):
    """Mirror of ``moe_ep_dep_models`` (linear task models of attention, shared experts, experts, link)."""
    _fields_ = [(n, ctypes.c_double) for n in (
        "alpha_a", "beta_a", "alpha_s", "beta_s", "alpha_e", "beta_e", "alpha_c", "beta_c")]


class DepProblem(ctypes.Structure):
    """Mirror of ``moe_ep_dep_problem``."""
    _fields_ = [(n, ctypes.c_int32) for n in ("ag", "n_experts", "top_k", "seq_len", "n_layers")]


class DepConfig(ctypes.Structure):
    """Mirror of ``moe_ep_dep_config``."""
    _fields_ = [("m_a", ctypes.c_int32), ("r_1", ctypes.c_int32), ("r_2", ctypes.c_int32),
                ("order", ctypes.c_int32), ("m_e", ctypes.c_double), ("makespan", ctypes.c_double),
                ("throughput", ctypes.c_double)]


class DepPrimitives(ctypes.Structure):
    """Mirror of ``moe_ep_dep_primitives``."""
    _fields_ = [(n, ctypes.c_double) for n in (
        "alpha_gm", "beta_gm", "alpha_attn", "beta_attn", "alpha_c", "beta_c")] + [
        (n, ctypes.c_int32) for n in (
            "seq_len", "hidden", "inter", "n_heads", "d_k", "d_v", "n_shared", "n_experts", "eg")]


DEP_ASAS, DEP_AASS = 0, 1


class MoeEpConfig(ctypes.Structure):
    """Mirror of ``moe_ep_config``."""
    _fields_ = [(n, ctypes.c_int32) for n in (
        "hidden", "inter", "n_experts", "local_begin", "n_local", "n_shared", "shared_inter",
        "max_tokens", "max_top_k", "max_chunks", "io_mode", "device")]


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libmoe_ep.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2512_21487_amd.build` "
                          "(hipcc, gfx950) first")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    cfgp = ctypes.POINTER(MoeEpConfig)
    lib.moe_ep_version.restype = ctypes.c_char_p
    lib.moe_ep_version.argtypes = []
    lib.moe_ep_validate_config.restype = ctypes.c_int
    lib.moe_ep_validate_config.argtypes = [cfgp, ctypes.POINTER(ctypes.c_char_p)]
    lib.moe_ep_validate_forward.restype = ctypes.c_int
    lib.moe_ep_validate_forward.argtypes = [cfgp, vp, vp, vp, vp, i32, i32, i32, i32, vp,
                                            ctypes.POINTER(ctypes.c_char_p)]
    lib.moe_ep_workspace_bytes.restype = ctypes.c_size_t
    lib.moe_ep_workspace_bytes.argtypes = [cfgp]
    lib.moe_ep_create.restype = ctypes.c_int
    lib.moe_ep_create.argtypes = [cfgp, ctypes.POINTER(vp)]
    lib.moe_ep_forward.restype = ctypes.c_int
    lib.moe_ep_forward.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp]
    lib.moe_ep_prepare_weights.restype = ctypes.c_int
    lib.moe_ep_prepare_weights.argtypes = [vp, vp, vp, vp]
    lib.moe_ep_forget_weights.restype = ctypes.c_int
    lib.moe_ep_forget_weights.argtypes = [vp, vp, vp]
    lib.moe_ep_prepared_weight_bytes.restype = ctypes.c_size_t
    lib.moe_ep_prepared_weight_bytes.argtypes = [cfgp, i32, i32]
    lib.moe_ep_forward_noalloc.restype = ctypes.c_int
    lib.moe_ep_forward_noalloc.argtypes = [cfgp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp,
                                           ctypes.POINTER(ctypes.c_char_p)]
    lib.moe_ep_forward_dep.restype = ctypes.c_int
    lib.moe_ep_forward_dep.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, ctypes.c_double, i32, vp, vp]
    lib.moe_ep_chunk_range.restype = ctypes.c_int
    lib.moe_ep_chunk_range.argtypes = [i32, i32, i32, i32, vp, vp]
    lib.moe_ep_routed_tile_rows.restype = i32
    lib.moe_ep_routed_tile_rows.argtypes = [cfgp, i32, i32, i32, i32]
    lib.moe_ep_last_tile_shape.restype = ctypes.c_int
    lib.moe_ep_last_tile_shape.argtypes = [vp, i32, i32] + [ctypes.POINTER(i32)] * 8
    lib.moe_ep_get_routing.restype = ctypes.c_int
    lib.moe_ep_get_routing.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
    lib.moe_ep_set_profiling.restype = ctypes.c_int
    lib.moe_ep_set_profiling.argtypes = [vp, i32]
    lib.moe_ep_set_profiling_stages.restype = ctypes.c_int
    lib.moe_ep_set_profiling_stages.argtypes = [vp, ctypes.c_uint32]
    lib.moe_ep_get_timeline.restype = ctypes.c_int
    lib.moe_ep_get_timeline.argtypes = [vp, vp, vp, vp, vp, i32, ctypes.POINTER(i32)]
    lib.moe_ep_get_stage_ms.restype = ctypes.c_int
    lib.moe_ep_get_stage_ms.argtypes = [vp, vp, i32]
    dp = ctypes.POINTER(ctypes.c_double)
    lib.moe_ep_fit_linear.restype = ctypes.c_int
    lib.moe_ep_fit_linear.argtypes = [dp, dp, i32, dp, dp, dp]
    lib.moe_ep_pipeline_makespan.restype = ctypes.c_double
    lib.moe_ep_pipeline_makespan.argtypes = [ctypes.POINTER(PipelineModel), i32, i32]
    lib.moe_ep_choose_chunks.restype = i32
    lib.moe_ep_choose_chunks.argtypes = [ctypes.POINTER(PipelineModel), i32, i32]
    lib.moe_ep_set_pipeline_model.restype = ctypes.c_int
    lib.moe_ep_set_pipeline_model.argtypes = [vp, ctypes.POINTER(PipelineModel)]
    lib.moe_ep_last_chunks.restype = i32
    lib.moe_ep_last_chunks.argtypes = [vp]
    mp, pp = ctypes.POINTER(DepModels), ctypes.POINTER(DepProblem)
    lib.moe_ep_dep_layer_models.restype = ctypes.c_int
    lib.moe_ep_dep_layer_models.argtypes = [ctypes.POINTER(DepPrimitives), mp]
    lib.moe_ep_dep_tokens_per_expert.restype = ctypes.c_double
    lib.moe_ep_dep_tokens_per_expert.argtypes = [pp, i32, i32]
    lib.moe_ep_dep_replay.restype = ctypes.c_int
    lib.moe_ep_dep_replay.argtypes = [mp, pp, i32, i32, i32, i32, dp, dp, dp, dp, dp, dp]
    lib.moe_ep_dep_replay_one_gpu.restype = ctypes.c_int
    lib.moe_ep_dep_replay_one_gpu.argtypes = [mp, pp, i32, i32, i32, i32, dp, dp, dp, dp, dp, dp]
    lib.moe_ep_dep_makespan.restype = ctypes.c_double
    lib.moe_ep_dep_makespan.argtypes = [mp, pp, i32, i32, i32]
    lib.moe_ep_dep_solve_r2.restype = ctypes.c_int
    lib.moe_ep_dep_solve_r2.argtypes = [mp, pp, i32, i32, i32, i32, ctypes.POINTER(i32), dp]
    lib.moe_ep_dep_search.restype = ctypes.c_int
    lib.moe_ep_dep_search.argtypes = [mp, pp, i32, i32, i32, i32, ctypes.POINTER(DepConfig)]
    lib.moe_ep_last_error.restype = ctypes.c_char_p
    lib.moe_ep_last_error.argtypes = [vp]
    lib.moe_ep_destroy.restype = ctypes.c_int
    lib.moe_ep_destroy.argtypes = [vp]
    _lib = lib
    return lib


def _ptr(x) -> Optional[int]:
    """Raw address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    raise TypeError(f"cannot take the address of {type(x)}")


def _check_tensor(x, name: str, n_bytes: int, want_pinned: bool) -> None:
    """Marshalling check of a torch tensor argument: dense, at least ``n_bytes`` long and resident where
    the call will read it (raw addresses pass through; the library queries those itself)."""
    if x is None or not hasattr(x, "is_contiguous"):
        return
    if not x.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    have = x.numel() * x.element_size()
    if have < n_bytes:
        raise ValueError(f"{name} holds {have} bytes, the forward needs {n_bytes}")
    if want_pinned and not (x.device.type == "cpu" and x.is_pinned()):
        raise ValueError(f"{name} must be a pinned host tensor in IO_PINNED_HOST mode")
    if not want_pinned and not (x.is_cuda or x.is_pinned()):
        raise ValueError(f"{name} must be a device tensor")


def prepared_weight_bytes(cfg: MoeEpConfig, routed: bool = True, shared: bool = True) -> int:
    """moe_ep_prepared_weight_bytes: device bytes moe_ep_prepare_weights takes for these sets of weights."""
    return int(load_library().moe_ep_prepared_weight_bytes(ctypes.byref(cfg), int(routed), int(shared)))


def validate_config(cfg: MoeEpConfig) -> Tuple[int, str]:
    why = ctypes.c_char_p()
    rc = load_library().moe_ep_validate_config(ctypes.byref(cfg), ctypes.byref(why))
    return rc, (why.value or b"").decode()


def validate_forward(cfg: MoeEpConfig, tokens, gate_logits, routed_w, shared_w, top_k: int,
                     r_chunks: int, order: int, n_tokens: int, out) -> Tuple[int, str]:
    why = ctypes.c_char_p()
    rc = load_library().moe_ep_validate_forward(
        ctypes.byref(cfg), _ptr(tokens), _ptr(gate_logits), _ptr(routed_w), _ptr(shared_w),
        top_k, r_chunks, order, n_tokens, _ptr(out), ctypes.byref(why))
    return rc, (why.value or b"").decode()


NOALLOC_SCRATCH_BYTES = 32 << 20   # MOE_EP_NOALLOC_SCRATCH_BYTES


def forward_noalloc(cfg: MoeEpConfig, tokens, gate_logits, routed_w, shared_w, top_k: int, r_chunks: int = 1,
                    order: int = ORDER_SHARED_FIRST, n_tokens: Optional[int] = None, out=None,
                    stream: Optional[int] = None) -> int:
    """moe_ep_forward_noalloc: the forward without a context, on the library's static workspace."""
    if n_tokens is None:
        n_tokens = int(tokens.shape[0])
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    why = ctypes.c_char_p()
    rc = load_library().moe_ep_forward_noalloc(ctypes.byref(cfg), _ptr(tokens), _ptr(gate_logits), _ptr(routed_w),
                                               _ptr(shared_w), top_k, r_chunks, order, n_tokens, _ptr(out), stream,
                                               ctypes.byref(why))
    if rc != 0:
        raise MoeEpError(rc, (why.value or b"").decode())
    return rc


def routed_tile_rows(cfg: MoeEpConfig, n_tokens: int, top_k: int, down: bool, n_cu: int = 256) -> int:
    """moe_ep_routed_tile_rows: tallest row tile (128 or 160 rows) of a routed projection of a chunk."""
    rows = int(load_library().moe_ep_routed_tile_rows(ctypes.byref(cfg), n_tokens, top_k, int(down), n_cu))
    if rows < 0:
        raise ValueError("moe_ep_routed_tile_rows: bad arguments")
    return rows


_PROBE_LIB_PATH = os.path.join(_HERE, "libmoe_ep_probe.so")
_probe_lib: Optional[ctypes.CDLL] = None


def load_probe_library() -> ctypes.CDLL:
    """libmoe_ep_probe.so (include/moe_ep_probe.h): the benchmark's measurement aid, a library of its own."""
    global _probe_lib
    if _probe_lib is None:
        if not os.path.exists(_PROBE_LIB_PATH):
            raise ImportError(f"{_PROBE_LIB_PATH} is missing: run `python -m paper_2512_21487_amd.build` first")
        lib = ctypes.CDLL(_PROBE_LIB_PATH)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.moe_ep_probe_device.restype = ctypes.c_int
        lib.moe_ep_probe_device.argtypes = [ctypes.c_int32, ctypes.c_int32, dp, dp, dp]
        _probe_lib = lib
    return _probe_lib


def probe_device(device: int = 0, zero_operands: bool = False) -> Dict[str, float]:
    """moe_ep_probe_device: register-only MFMA rate and clock, streaming copy rate of the GPU."""
    tf, ghz, gbs = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    rc = load_probe_library().moe_ep_probe_device(device, int(zero_operands), ctypes.byref(tf), ctypes.byref(ghz),
                                                  ctypes.byref(gbs))
    if rc != 0:
        raise MoeEpError(rc, "moe_ep_probe_device failed")
    return {"mfma_tflops": tf.value, "mfma_ghz": ghz.value, "copy_gbs": gbs.value}


def workspace_bytes(cfg: MoeEpConfig) -> int:
    return int(load_library().moe_ep_workspace_bytes(ctypes.byref(cfg)))


def fit_linear(x, t) -> Tuple[float, float, float]:
    """moe_ep_fit_linear: (alpha, beta, R^2) of t = alpha + beta x."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    t = np.ascontiguousarray(t, dtype=np.float64)
    a, b, r2 = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    dp = ctypes.POINTER(ctypes.c_double)
    rc = load_library().moe_ep_fit_linear(x.ctypes.data_as(dp), t.ctypes.data_as(dp), int(x.size),
                                          ctypes.byref(a), ctypes.byref(b), ctypes.byref(r2))
    if rc != 0:
        raise MoeEpError(rc, "moe_ep_fit_linear: need >= 2 samples with distinct workloads")
    return a.value, b.value, r2.value


def pipeline_makespan(model: PipelineModel, n_tokens: int, r_chunks: int) -> float:
    return float(load_library().moe_ep_pipeline_makespan(ctypes.byref(model), n_tokens, r_chunks))


def choose_chunks(model: PipelineModel, n_tokens: int, r_max: int) -> int:
    r = int(load_library().moe_ep_choose_chunks(ctypes.byref(model), n_tokens, r_max))
    if r < 1:
        raise MoeEpError(r, "moe_ep_choose_chunks: bad arguments")
    return r


def dep_layer_models(prim: DepPrimitives) -> DepModels:
    out = DepModels()
    rc = load_library().moe_ep_dep_layer_models(ctypes.byref(prim), ctypes.byref(out))
    if rc != 0:
        raise MoeEpError(rc, "moe_ep_dep_layer_models: bad arguments")
    return out


def dep_tokens_per_expert(problem: DepProblem, m_a: int, r_2: int) -> float:
    return float(load_library().moe_ep_dep_tokens_per_expert(ctypes.byref(problem), m_a, r_2))


def dep_replay(models: DepModels, problem: DepProblem, m_a: int, r_1: int, r_2: int, order: int,
               one_gpu: bool = False):
    """moe_ep_dep_replay (one_gpu: moe_ep_dep_replay_one_gpu): (makespan, dict of start-time arrays
    shaped [T, r_1] / [T, r_1, r_2])."""
    T = problem.n_layers
    tau = {"tau_a": np.empty((T, r_1)), "tau_s": np.empty((T, r_1)), "tau_a2e": np.empty((T, r_1, r_2)),
           "tau_e": np.empty((T, r_1, r_2)), "tau_e2a": np.empty((T, r_1, r_2))}
    span = ctypes.c_double()
    dp = ctypes.POINTER(ctypes.c_double)
    fn = load_library().moe_ep_dep_replay_one_gpu if one_gpu else load_library().moe_ep_dep_replay
    rc = fn(
        ctypes.byref(models), ctypes.byref(problem), m_a, r_1, r_2, order, ctypes.byref(span),
        *(tau[k].ctypes.data_as(dp) for k in ("tau_a", "tau_s", "tau_a2e", "tau_e", "tau_e2a")))
    if rc != 0:
        raise MoeEpError(rc, "moe_ep_dep_replay: bad arguments")
    return span.value, tau


def dep_makespan(models: DepModels, problem: DepProblem, m_a: int, r_1: int, r_2: int) -> float:
    return float(load_library().moe_ep_dep_makespan(ctypes.byref(models), ctypes.byref(problem), m_a, r_1, r_2))


def dep_solve_r2(models: DepModels, problem: DepProblem, m_a: int, r_1: int, order: int,
                 r2_max: int) -> Tuple[int, float]:
    r2, span = ctypes.c_int32(), ctypes.c_double()
    rc = load_library().moe_ep_dep_solve_r2(ctypes.byref(models), ctypes.byref(problem), m_a, r_1, order,
                                            r2_max, ctypes.byref(r2), ctypes.byref(span))
    if rc != 0:
        raise MoeEpError(rc, "moe_ep_dep_solve_r2: bad arguments")
    return r2.value, span.value


def dep_search(models: DepModels, problem: DepProblem, m_a_max: int, mem_cap: int, r1_cap: int,
               r2_max: int) -> Optional[DepConfig]:
    """moe_ep_dep_search (Algorithm 1); None when no (m_a, r_1) pair fits the memory rule."""
    best = DepConfig()
    rc = load_library().moe_ep_dep_search(ctypes.byref(models), ctypes.byref(problem), m_a_max, mem_cap,
                                          r1_cap, r2_max, ctypes.byref(best))
    if rc == -4:
        return None
    if rc != 0:
        raise MoeEpError(rc, "moe_ep_dep_search: bad arguments")
    return best


class MoeEp:
    """Owns one ``moe_ep_ctx``.  Tensors are torch tensors (or raw addresses) that the caller
    allocated; nothing is computed on the Python side."""

    def __init__(self, *, hidden: int, inter: int, n_experts: int, n_local: int, max_tokens: int,
                 max_top_k: int, local_begin: int = 0, n_shared: int = 0, shared_inter: int = 0,
                 max_chunks: int = 8, io_mode: int = IO_DEVICE, device: int = 0):
        self._lib = load_library()
        self.cfg = MoeEpConfig(hidden, inter, n_experts, local_begin, n_local, n_shared,
                               shared_inter, max_tokens, max_top_k, max_chunks, io_mode, device)
        self._ctx = ctypes.c_void_p()
        rc, why = validate_config(self.cfg)
        if rc != 0:
            raise MoeEpError(rc, why)
        rc = self._lib.moe_ep_create(ctypes.byref(self.cfg), ctypes.byref(self._ctx))
        if rc != 0:
            self._ctx = ctypes.c_void_p()
            raise MoeEpError(rc, "moe_ep_create failed (no usable HIP device or out of memory)")
        self._last = (0, 0, 0, 1)

    def _check_forward_tensors(self, tokens, gate_logits, routed_w, shared_w, n_tokens, out) -> None:
        c = self.cfg
        pinned = c.io_mode == IO_PINNED_HOST
        T = max(int(n_tokens), 0)
        _check_tensor(tokens, "tokens", T * c.hidden * 2, pinned)
        _check_tensor(gate_logits, "gate_logits", T * c.n_experts * 4, pinned)
        _check_tensor(out, "out", T * c.hidden * 2, pinned)
        _check_tensor(routed_w, "routed_w", c.n_local * 3 * c.inter * c.hidden * 2, False)
        _check_tensor(shared_w, "shared_w", c.n_shared * 3 * c.shared_inter * c.hidden * 2, False)

    # -- moe_ep_forward -------------------------------------------------------------------
    def forward(self, tokens, gate_logits, routed_w, shared_w, top_k: int, r_chunks: int = 1,
                order: int = ORDER_SHARED_FIRST, n_tokens: Optional[int] = None, out=None,
                stream: Optional[int] = None) -> int:
        if n_tokens is None:
            n_tokens = int(tokens.shape[0])
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        self._check_forward_tensors(tokens, gate_logits, routed_w, shared_w, n_tokens, out)
        rc = self._lib.moe_ep_forward(self._ctx, _ptr(tokens), _ptr(gate_logits), _ptr(routed_w),
                                      _ptr(shared_w), top_k, r_chunks, order, n_tokens, _ptr(out),
                                      stream)
        if rc != 0:
            raise MoeEpError(rc, self.last_error())
        self._last = (n_tokens, top_k, int(self._lib.moe_ep_last_chunks(self._ctx)), 1)
        return rc

    # -- moe_ep_prepare_weights / moe_ep_forget_weights -------------------------------------
    def prepare_weights(self, routed_w=None, shared_w=None, stream: Optional[int] = None) -> int:
        """Tile-order copies of the weights at these pointers; later forwards given the same tensors use them."""
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        c = self.cfg
        _check_tensor(routed_w, "routed_w", c.n_local * 3 * c.inter * c.hidden * 2, False)
        _check_tensor(shared_w, "shared_w", c.n_shared * 3 * c.shared_inter * c.hidden * 2, False)
        rc = self._lib.moe_ep_prepare_weights(self._ctx, _ptr(routed_w), _ptr(shared_w), stream)
        if rc != 0:
            raise MoeEpError(rc, self.last_error())
        return rc

    def forget_weights(self, routed_w=None, shared_w=None) -> int:
        rc = self._lib.moe_ep_forget_weights(self._ctx, _ptr(routed_w), _ptr(shared_w))
        if rc != 0:
            raise MoeEpError(rc, self.last_error())
        return rc

    def prepared_weight_bytes(self, routed: bool = True, shared: bool = True) -> int:
        return int(self._lib.moe_ep_prepared_weight_bytes(ctypes.byref(self.cfg), int(routed), int(shared)))

    # -- moe_ep_forward_dep ---------------------------------------------------------------
    def forward_dep(self, tokens, gate_logits, routed_w, shared_w, top_k: int, r_1: int = 1, r_2: int = 1,
                    dep_order: int = 0, attn_us: float = 0.0, n_tokens: Optional[int] = None, out=None,
                    stream: Optional[int] = None) -> int:
        if n_tokens is None:
            n_tokens = int(tokens.shape[0])
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        self._check_forward_tensors(tokens, gate_logits, routed_w, shared_w, n_tokens, out)
        rc = self._lib.moe_ep_forward_dep(self._ctx, _ptr(tokens), _ptr(gate_logits), _ptr(routed_w),
                                          _ptr(shared_w), top_k, r_1, r_2, dep_order, float(attn_us),
                                          n_tokens, _ptr(out), stream)
        if rc != 0:
            raise MoeEpError(rc, self.last_error())
        self._last = (n_tokens, top_k, r_1 * r_2, r_1)
        return rc

    # -- moe_ep_get_routing ---------------------------------------------------------------
    def get_routing(self, chunk: int = 0) -> Dict[str, np.ndarray]:
        T, k, r, r_1 = self._last
        t0, Tn = chunk_range(T, r_1, r // r_1 if r_1 else 1, chunk) if r else (0, 0)
        El = self.cfg.n_local
        idx = np.zeros((Tn, k), dtype=np.int32)
        w = np.zeros((Tn, k), dtype=np.float32)
        pos = np.full((Tn, k), -1, dtype=np.int32)
        count = np.zeros(El, dtype=np.int32)
        offset = np.zeros(El + 1, dtype=np.int32)
        perm = np.full(max(Tn * k, 1), -1, dtype=np.int32)
        rc = self._lib.moe_ep_get_routing(self._ctx, chunk, _ptr(idx), _ptr(w), _ptr(pos),
                                          _ptr(count), _ptr(offset), _ptr(perm))
        if rc != 0:
            raise MoeEpError(rc, self.last_error())
        return {"idx": idx, "w": w, "pos": pos, "count": count, "offset": offset,
                "perm": perm[:offset[-1]].copy()}

    # -- moe_ep_last_tile_shape -----------------------------------------------------------
    def last_tile_shape(self, stage: str, chunk: int = 0) -> Optional[Dict[str, int]]:
        """Tile shape of the kernel the last forward launched for `stage` (an entry of STAGES naming a
        projection); None if the layer has no such stage."""
        v = [ctypes.c_int32() for _ in range(8)]
        rc = self._lib.moe_ep_last_tile_shape(self._ctx, chunk, STAGES.index(stage), *[ctypes.byref(x) for x in v])
        if rc == -4:
            return None
        if rc != 0:
            raise MoeEpError(rc, "moe_ep_last_tile_shape: bad arguments")
        return dict(zip(("rows", "cols", "k_step", "ring_slots", "waves_m", "waves_n", "tile_order", "mfma_rows"),
                        (x.value for x in v)))

    # -- timing model ---------------------------------------------------------------------
    def set_pipeline_model(self, model: Optional[PipelineModel]) -> None:
        rc = self._lib.moe_ep_set_pipeline_model(self._ctx, ctypes.byref(model) if model else None)
        if rc != 0:
            raise MoeEpError(rc, self.last_error())

    def last_chunks(self) -> int:
        return int(self._lib.moe_ep_last_chunks(self._ctx))

    # -- profiling ------------------------------------------------------------------------
    def set_profiling(self, depth: int) -> None:
        rc = self._lib.moe_ep_set_profiling(self._ctx, depth)
        if rc != 0:
            raise MoeEpError(rc, self.last_error())

    def set_profiling_stages(self, names=None) -> None:
        """Time only the named stages (entries of STAGES); None = every stage."""
        mask = 0xFFFFFFFF if names is None else sum(1 << STAGES.index(n) for n in names)
        rc = self._lib.moe_ep_set_profiling_stages(self._ctx, mask)
        if rc != 0:
            raise MoeEpError(rc, self.last_error())

    def get_timeline(self, max_spans: int = 4096):
        """moe_ep_get_timeline: list of (stage name, forward index, begin ms, end ms)."""
        st = (ctypes.c_int32 * max_spans)(); fw = (ctypes.c_int32 * max_spans)()
        b = (ctypes.c_float * max_spans)(); e = (ctypes.c_float * max_spans)()
        n = ctypes.c_int32()
        rc = self._lib.moe_ep_get_timeline(self._ctx, ctypes.cast(st, ctypes.c_void_p), ctypes.cast(fw, ctypes.c_void_p),
                                           ctypes.cast(b, ctypes.c_void_p), ctypes.cast(e, ctypes.c_void_p),
                                           max_spans, ctypes.byref(n))
        if rc != 0:
            raise MoeEpError(rc, self.last_error())
        return [(STAGES[st[i]], int(fw[i]), float(b[i]), float(e[i])) for i in range(n.value)]

    def get_stage_ms(self) -> Dict[str, float]:
        ms = (ctypes.c_float * len(STAGES))()
        rc = self._lib.moe_ep_get_stage_ms(self._ctx, ctypes.cast(ms, ctypes.c_void_p), len(STAGES))
        if rc != 0:
            raise MoeEpError(rc, self.last_error())
        return {name: float(ms[i]) for i, name in enumerate(STAGES)}

    def last_error(self) -> str:
        return (self._lib.moe_ep_last_error(self._ctx) or b"").decode()

    def destroy(self) -> None:
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            self._lib.moe_ep_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        # At interpreter shutdown the HIP runtime, a preloaded profiler and torch's allocators are being
        # torn down in an order this object does not control: calling into the library then could touch
        # streams and events that are already gone.  The process is ending; the driver reclaims the memory.
        try:
            if sys is None or sys.is_finalizing():
                return
            self.destroy()
        except Exception:
            pass
