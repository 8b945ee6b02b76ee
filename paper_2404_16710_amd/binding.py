"""ctypes binding of libls.so: same names and argument order as include/ls.h.

Only marshalling happens here.  If the library has not been built the import of `lib()`
raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

LS_F32, LS_BF16 = 0, 1
LS_MAX_ROWS = 16
_HERE = os.path.dirname(os.path.abspath(__file__))

EXPORTS = (
    "ls_workspace_bytes", "ls_load_weights", "ls_prefill", "ls_draft", "ls_verify", "ls_generate",
    "ls_generate_no_reuse", "ls_generate_dynamic", "ls_generate_early_exit", "ls_score", "ls_probe_layers", "ls_get_state", "ls_peek_round", "ls_debug_capture",
    "ls_debug_timeline", "ls_debug_copy", "ls_debug_read", "ls_set_launch", "ls_set_prompt_tiles", "ls_debug_spin_limit", "ls_debug_kv_policy", "ls_strerror", "ls_destroy",
    "ls_generate_static", "ls_static_workspace_limit",
)


class LsError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {code} ({lib().ls_strerror(code).decode()})")


class ls_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "ffn_dim", "vocab")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float),
                ("dtype", C.c_int32), ("max_seq", C.c_int32), ("max_draft", C.c_int32)]


_PP = C.POINTER(C.c_void_p)


class ls_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p)] + \
               [(n, _PP) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "attn_norm", "ffn_norm")] + \
               [("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


class ls_stats(C.Structure):
    _fields_ = [("rounds", C.c_int64), ("drafted", C.c_int64), ("accepted", C.c_int64),
                ("generated", C.c_int64), ("ms_prefill", C.c_float), ("ms_decode", C.c_float)]


@dataclass
class Stats:
    rounds: int
    drafted: int
    accepted: int
    generated: int
    ms_prefill: float
    ms_decode: float

    @property
    def acceptance(self) -> float:
        return self.accepted / self.drafted if self.drafted else 0.0


def lib_path() -> str:
    return os.path.join(_HERE, "libls.so")


_LIB = None


def lib() -> C.CDLL:
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2404_16710_amd.build`")
    L = C.CDLL(path)
    vp, i32, i32p, f32p = C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_float)
    L.ls_workspace_bytes.restype = C.c_size_t
    L.ls_workspace_bytes.argtypes = [C.POINTER(ls_config)]
    L.ls_load_weights.restype = C.c_int
    L.ls_load_weights.argtypes = [C.POINTER(ls_config), C.POINTER(ls_weights), vp, C.c_size_t, C.POINTER(vp)]
    L.ls_prefill.restype = C.c_int
    L.ls_prefill.argtypes = [vp, vp, i32, vp]
    L.ls_draft.restype = C.c_int
    L.ls_draft.argtypes = [vp, i32, i32, vp]
    L.ls_verify.restype = C.c_int
    L.ls_verify.argtypes = [vp, i32, i32, vp]
    L.ls_generate.restype = C.c_int
    L.ls_generate.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, C.POINTER(ls_stats), vp]
    L.ls_generate_dynamic.restype = C.c_int
    L.ls_generate_dynamic.argtypes = [vp, vp, i32, i32, i32, i32, i32, C.c_float, i32, vp, vp, C.POINTER(ls_stats),
                                      C.POINTER(C.c_int64), vp]
    L.ls_generate_no_reuse.restype = C.c_int
    L.ls_generate_no_reuse.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, C.POINTER(ls_stats), vp]
    L.ls_generate_early_exit.restype = C.c_int
    L.ls_generate_early_exit.argtypes = [vp, vp, i32, i32, i32, vp, C.POINTER(ls_stats), vp]
    L.ls_probe_layers.restype = C.c_int
    L.ls_probe_layers.argtypes = [vp, vp, i32, vp, vp, vp]
    L.ls_score.restype = C.c_int
    L.ls_score.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    L.ls_get_state.restype = C.c_int
    L.ls_get_state.argtypes = [vp, i32p, i32p, i32p, vp]
    L.ls_peek_round.restype = C.c_int
    L.ls_peek_round.argtypes = [vp, i32p, i32p, f32p, f32p, i32p, vp]
    L.ls_debug_capture.restype = C.c_int
    L.ls_debug_capture.argtypes = [vp, vp]
    L.ls_debug_timeline.restype = C.c_int
    L.ls_debug_timeline.argtypes = [vp, vp, i32, i32]
    L.ls_debug_copy.restype = C.c_int
    L.ls_debug_copy.argtypes = [vp, vp, C.c_size_t, vp]
    L.ls_set_launch.restype = C.c_int
    L.ls_set_launch.argtypes = [vp, i32]
    L.ls_set_prompt_tiles.restype = C.c_int
    L.ls_set_prompt_tiles.argtypes = [vp, i32]
    L.ls_debug_read.restype = C.c_int
    L.ls_debug_read.argtypes = [vp, C.c_size_t, vp, i32, vp]
    L.ls_debug_spin_limit.restype = C.c_int
    L.ls_debug_spin_limit.argtypes = [vp, i32]
    L.ls_debug_kv_policy.restype = C.c_int
    L.ls_debug_kv_policy.argtypes = [vp, i32]
    L.ls_generate_static.restype = C.c_int
    L.ls_generate_static.argtypes = [C.POINTER(ls_config), C.POINTER(ls_weights), vp, i32, i32, i32, i32, i32, vp,
                                     C.POINTER(ls_stats), vp]
    L.ls_static_workspace_limit.restype = C.c_size_t
    L.ls_static_workspace_limit.argtypes = []
    L.ls_strerror.restype = C.c_char_p
    L.ls_strerror.argtypes = [C.c_int]
    L.ls_destroy.restype = None
    L.ls_destroy.argtypes = [vp]
    _LIB = L
    return L


def config_struct(model_cfg, max_seq: int, max_draft: int = 15) -> ls_config:
    """model_cfg: any object with the fields of workloads.ModelConfig."""
    m = model_cfg
    return ls_config(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn_dim, m.vocab,
                     float(m.rope_base), float(m.rms_eps), LS_BF16 if m.dtype == "bf16" else LS_F32,
                     int(max_seq), int(max_draft))


def _check(code: int, what: str) -> None:
    if code != 0:
        raise LsError(code, what)


class DeviceWeights:
    """The tensors of a model on the GPU (torch owns the memory) and the ls_weights struct that
    points at them.  weights: dict as produced by workloads.make_weights."""

    def __init__(self, model_cfg, weights: dict, device):
        import torch
        self.tensors = []   # keeps device memory alive
        self.by_name = {}   # (name, layer) -> tensor; layer -1 for the global tensors

        def up(a: np.ndarray):
            if a.dtype == np.uint16:
                t = torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
            else:
                t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
            self.tensors.append(t)
            return t.data_ptr()

        L = model_cfg.n_layers
        w = ls_weights()
        for name in ("embed", "final_norm", "lm_head"):
            setattr(w, name, up(weights[name]))
            self.by_name[(name, -1)] = self.tensors[-1]
        self.ptr_arrays = {}
        for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "attn_norm", "ffn_norm"):
            ptrs = []
            for l in range(L):
                ptrs.append(up(weights["layers"][l][name]))
                self.by_name[(name, l)] = self.tensors[-1]
            arr = (C.c_void_p * L)(*ptrs)
            self.ptr_arrays[name] = arr
            setattr(w, name, C.cast(arr, _PP))
        self.struct = w

    def replace(self, name: str, layer: int, a: np.ndarray) -> None:
        """Overwrites one tensor in place (same shape and dtype): the device address stays valid."""
        import torch
        t = self.by_name[(name, layer)]
        src = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16) if a.dtype == np.uint16 else torch.from_numpy(a)
        assert src.shape == t.shape and src.dtype == t.dtype
        t.copy_(src)


def generate_static(model_cfg, dev_weights: DeviceWeights, max_seq: int, prompt: Sequence[int], max_new: int,
                    exit_layer: int, d: int, eos_id: int = -1, max_draft: int = 15, device: str = "cuda:0"):
    """ls_generate_static: the whole job with the library's own fixed workspace (no context, no
    caller workspace).  Returns (tokens, stats) like LsModel.generate."""
    import torch
    cfg_c = config_struct(model_cfg, max_seq, max_draft)
    dev = torch.device(device)
    p = torch.as_tensor(np.asarray(prompt, dtype=np.int32), device=dev)
    out = torch.empty(max_new, dtype=torch.int32, device=dev)
    st = ls_stats()
    stream = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    _check(lib().ls_generate_static(C.byref(cfg_c), C.byref(dev_weights.struct), C.c_void_p(p.data_ptr()), len(prompt),
                                    max_new, exit_layer, d, eos_id, C.c_void_p(out.data_ptr()), C.byref(st), stream),
           "ls_generate_static")
    stats = Stats(st.rounds, st.drafted, st.accepted, st.generated, st.ms_prefill, st.ms_decode)
    return out.cpu().numpy()[: stats.generated].tolist(), stats


class LsModel:
    """One model + one sequence on the current CUDA(HIP) device.

    weights: dict as produced by workloads.make_weights (uint16 bf16 bit patterns or float32).
    """

    def __init__(self, model_cfg, weights: dict, max_seq: int, max_draft: int = 15, device: str = "cuda:0"):
        import torch
        self.torch = torch
        self.lib = lib()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the HIP path has no CPU fallback")
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = model_cfg
        self.max_seq, self.max_draft = int(max_seq), int(max_draft)
        self._cfg_c = config_struct(model_cfg, max_seq, max_draft)
        self._dev_weights = DeviceWeights(model_cfg, weights, self.device)
        self._tensors = self._dev_weights.tensors
        w = self._w = self._dev_weights.struct
        nbytes = self.lib.ls_workspace_bytes(C.byref(self._cfg_c))
        if nbytes == 0:
            raise LsError(-1, "ls_workspace_bytes")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        ctx = C.c_void_p()
        _check(self.lib.ls_load_weights(C.byref(self._cfg_c), C.byref(w), C.c_void_p(base), nbytes, C.byref(ctx)),
               "ls_load_weights")
        self.ctx = ctx
        self.workspace_bytes = nbytes
        self._capture = None

    # -- helpers
    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def _dev_i32(self, ids: Sequence[int]):
        t = self.torch.as_tensor(np.asarray(ids, dtype=np.int32), device=self.device)
        return t

    def replace_tensor(self, name: str, layer: int, a: np.ndarray) -> None:
        """New values for one weight tensor (same shape); no call may be in flight."""
        self.torch.cuda.synchronize(self.device)
        self._dev_weights.replace(name, layer, a)
        self.torch.cuda.synchronize(self.device)

    def close(self):
        if getattr(self, "ctx", None):
            self.torch.cuda.synchronize(self.device)
            self.lib.ls_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the C ABI, one method per entry point
    def set_launch(self, wg_per_cu: int) -> int:
        g = self.lib.ls_set_launch(self.ctx, wg_per_cu)
        if g < 0:
            raise LsError(g, "ls_set_launch")
        return g

    def debug_spin_limit(self, polls: int) -> None:
        _check(self.lib.ls_debug_spin_limit(self.ctx, polls), "ls_debug_spin_limit")

    def debug_kv_policy(self, policy: int) -> None:
        _check(self.lib.ls_debug_kv_policy(self.ctx, policy), "ls_debug_kv_policy")

    def set_prompt_tiles(self, rows: int) -> None:
        _check(self.lib.ls_set_prompt_tiles(self.ctx, rows), "ls_set_prompt_tiles")

    def prefill(self, prompt: Sequence[int]) -> None:
        self._prompt = self._dev_i32(prompt)
        _check(self.lib.ls_prefill(self.ctx, C.c_void_p(self._prompt.data_ptr()), len(prompt), self._stream()), "ls_prefill")

    def draft(self, exit_layer: int, d: int) -> None:
        _check(self.lib.ls_draft(self.ctx, exit_layer, d, self._stream()), "ls_draft")

    def verify(self, exit_layer: int, d: int) -> None:
        _check(self.lib.ls_verify(self.ctx, exit_layer, d, self._stream()), "ls_verify")

    def generate(self, prompt: Sequence[int], max_new: int, exit_layer: int, d: int, eos_id: int = -1):
        p = self._dev_i32(prompt)
        out = self.torch.empty(max_new, dtype=self.torch.int32, device=self.device)
        st = ls_stats()
        _check(self.lib.ls_generate(self.ctx, C.c_void_p(p.data_ptr()), len(prompt), max_new, exit_layer, d, eos_id,
                                    C.c_void_p(out.data_ptr()), C.byref(st), self._stream()), "ls_generate")
        stats = Stats(st.rounds, st.drafted, st.accepted, st.generated, st.ms_prefill, st.ms_decode)
        return out.cpu().numpy()[: stats.generated].tolist(), stats

    def generate_no_reuse(self, prompt: Sequence[int], max_new: int, exit_layer: int, d: int, eos_id: int = -1):
        p = self._dev_i32(prompt)
        out = self.torch.empty(max_new, dtype=self.torch.int32, device=self.device)
        st = ls_stats()
        _check(self.lib.ls_generate_no_reuse(self.ctx, C.c_void_p(p.data_ptr()), len(prompt), max_new, exit_layer, d,
                                             eos_id, C.c_void_p(out.data_ptr()), C.byref(st), self._stream()),
               "ls_generate_no_reuse")
        stats = Stats(st.rounds, st.drafted, st.accepted, st.generated, st.ms_prefill, st.ms_decode)
        return out.cpu().numpy()[: stats.generated].tolist(), stats

    def generate_dynamic(self, prompt: Sequence[int], max_new: int, exit_low: int, exit_high: int, d: int, tau: float,
                         eos_id: int = -1):
        """Per-token exit layer.  Returns (tokens, stats, exit layer of every draft as rows of d, drafts that left
        at exit_low)."""
        p = self._dev_i32(prompt)
        out = self.torch.empty(max_new, dtype=self.torch.int32, device=self.device)
        exits = self.torch.zeros(max_new * d, dtype=self.torch.int32, device=self.device)
        st = ls_stats()
        low = C.c_int64(0)
        _check(self.lib.ls_generate_dynamic(self.ctx, C.c_void_p(p.data_ptr()), len(prompt), max_new, exit_low, exit_high,
                                            d, C.c_float(tau), eos_id, C.c_void_p(out.data_ptr()),
                                            C.c_void_p(exits.data_ptr()), C.byref(st), C.byref(low), self._stream()),
               "ls_generate_dynamic")
        stats = Stats(st.rounds, st.drafted, st.accepted, st.generated, st.ms_prefill, st.ms_decode)
        ex = exits.cpu().numpy()[: stats.rounds * d].reshape(stats.rounds, d).tolist()
        return out.cpu().numpy()[: stats.generated].tolist(), stats, ex, int(low.value)

    def generate_early_exit(self, prompt: Sequence[int], max_new: int, exit_layer: int):
        p = self._dev_i32(prompt)
        out = self.torch.empty(max_new, dtype=self.torch.int32, device=self.device)
        st = ls_stats()
        _check(self.lib.ls_generate_early_exit(self.ctx, C.c_void_p(p.data_ptr()), len(prompt), max_new, exit_layer,
                                               C.c_void_p(out.data_ptr()), C.byref(st), self._stream()),
               "ls_generate_early_exit")
        stats = Stats(st.rounds, st.drafted, st.accepted, st.generated, st.ms_prefill, st.ms_decode)
        return out.cpu().numpy()[: stats.generated].tolist(), stats

    def score(self, tokens: Sequence[int], n_layers_used: Optional[int] = None):
        t = self._dev_i32(tokens)
        n = len(tokens)
        am = self.torch.empty(n, dtype=self.torch.int32, device=self.device)
        mg = self.torch.empty(n, dtype=self.torch.float32, device=self.device)
        _check(self.lib.ls_score(self.ctx, C.c_void_p(t.data_ptr()), n, n_layers_used or self.cfg.n_layers,
                                 C.c_void_p(am.data_ptr()), C.c_void_p(mg.data_ptr()), self._stream()), "ls_score")
        return am.cpu().numpy(), mg.cpu().numpy()

    def probe_layers(self, tokens: Sequence[int]):
        """argmax and margin of g(x_l) for every layer l = 1..L and every row: arrays [L][n]."""
        t = self._dev_i32(tokens)
        n, L = len(tokens), self.cfg.n_layers
        am = self.torch.empty((L, n), dtype=self.torch.int32, device=self.device)
        mg = self.torch.empty((L, n), dtype=self.torch.float32, device=self.device)
        _check(self.lib.ls_probe_layers(self.ctx, C.c_void_p(t.data_ptr()), n, C.c_void_p(am.data_ptr()),
                                        C.c_void_p(mg.data_ptr()), self._stream()), "ls_probe_layers")
        return am.cpu().numpy(), mg.cpu().numpy()

    def get_state(self):
        pos, last, n_gen = C.c_int32(), C.c_int32(), C.c_int32()
        _check(self.lib.ls_get_state(self.ctx, C.byref(pos), C.byref(last), C.byref(n_gen), self._stream()), "ls_get_state")
        return pos.value, last.value, n_gen.value

    def peek_round(self, d: int):
        D = (C.c_int32 * LS_MAX_ROWS)()
        V = (C.c_int32 * LS_MAX_ROWS)()
        dm = (C.c_float * LS_MAX_ROWS)()
        vm = (C.c_float * LS_MAX_ROWS)()
        n = C.c_int32()
        _check(self.lib.ls_peek_round(self.ctx, D, V, dm, vm, C.byref(n), self._stream()), "ls_peek_round")
        return list(D[:d]), list(V[:d + 1]), list(dm[:d]), list(vm[:d + 1]), n.value

    def debug_timeline(self, capacity: int = 0, workgroup: int = 0):
        """capacity > 0: returns the device tensor (uint64 as int64) later launches append events to."""
        if capacity > 0:
            self._timeline = self.torch.zeros(capacity, dtype=self.torch.int64, device=self.device)
            _check(self.lib.ls_debug_timeline(self.ctx, C.c_void_p(self._timeline.data_ptr()), capacity, workgroup),
                   "ls_debug_timeline")
        else:
            _check(self.lib.ls_debug_timeline(self.ctx, None, 0, 0), "ls_debug_timeline")
            self._timeline = None
        return self._timeline

    def debug_copy(self, nbytes: int) -> None:
        """Runs the library's plain copy kernel over nbytes (counter calibration for profilers)."""
        src = self.torch.zeros(nbytes, dtype=self.torch.uint8, device=self.device)
        dst = self.torch.empty_like(src)
        _check(self.lib.ls_debug_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()), nbytes, self._stream()),
               "ls_debug_copy")
        self.torch.cuda.synchronize(self.device)

    def debug_capture(self, on: bool = True):
        """Returns the device tensor [n_layers, max_seq, d_model] that later passes fill."""
        if on:
            self._capture = self.torch.zeros((self.cfg.n_layers, self.max_seq, self.cfg.d_model),
                                             dtype=self.torch.float32, device=self.device)
            _check(self.lib.ls_debug_capture(self.ctx, C.c_void_p(self._capture.data_ptr())), "ls_debug_capture")
        else:
            _check(self.lib.ls_debug_capture(self.ctx, None), "ls_debug_capture")
            self._capture = None
        return self._capture
