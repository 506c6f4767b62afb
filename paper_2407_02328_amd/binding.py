"""ctypes binding of libadore.so: the same calls as include/adore.h, argument marshalling only.

torch is used for device memory and the stream; every step of the path runs in
the library's HIP kernels.  There is no fallback: if the library is missing or
a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libadore.so")

ADORE_F32, ADORE_BF16 = 0, 1
KERNELS = ["attend", "attend_combine", "ctrl_input", "ctrl_cell", "release", "rebuild_select", "rebuild_gemm",
           "rescore", "fwd_qkv", "fwd_qkv_cur", "fwd_attend", "fwd_oproj", "fwd_oproj_cur", "rope", "h2o_release",
           "h2o_choice", "h2o_place"]
SCORE_STATIC, SCORE_RESCORE, SCORE_H2O = 0, 1, 2

EXPORTS = [
    "adore_workspace_bytes", "adore_create", "adore_destroy", "adore_init_cache", "adore_attend",
    "adore_schedule", "adore_rebuild", "adore_decode_step", "adore_forward_step", "adore_get_state", "adore_set_state",
    "adore_set_input_order", "adore_check_guards", "adore_set_timing", "adore_read_timing", "adore_kernel_name", "adore_strerror", "adore_abi_version",
    "adore_topk_attention_workspace_bytes", "adore_topk_attention", "adore_topk_attention_static",
]


class AdoreConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("layers", "batch", "heads", "head_dim", "hidden", "cache_slots", "rebuild_budget",
                 "max_positions", "ctrl_hidden", "dtype")] + [("pos_scale", ctypes.c_float),
                                                              ("score_mode", ctypes.c_int32),
                                                              ("rope_base", ctypes.c_float)]


_WEIGHT_FIELDS = ["w_kv", "gru_w_ih", "gru_w_hh", "gru_b_ih", "gru_b_hh", "pos_w", "pos_b", "mlp_w1",
                  "mlp_b1", "out_w", "out_b"]


class AdoreWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in _WEIGHT_FIELDS]


class AdoreForwardWeights(ctypes.Structure):
    _fields_ = [("w_q", ctypes.c_void_p), ("w_o", ctypes.c_void_p)]


class AdoreError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"adore error {code}: {msg}")
        self.code = code


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libadore.so from the package directory.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2407_02328_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.adore_workspace_bytes.restype = sz
    lib.adore_workspace_bytes.argtypes = [ctypes.POINTER(AdoreConfig)]
    lib.adore_create.restype = ctypes.c_int
    lib.adore_create.argtypes = [ctypes.POINTER(AdoreConfig), ctypes.POINTER(AdoreWeights), vp, sz, vp,
                                 ctypes.POINTER(vp)]
    lib.adore_destroy.restype = ctypes.c_int
    lib.adore_destroy.argtypes = [vp]
    lib.adore_init_cache.restype = ctypes.c_int
    lib.adore_init_cache.argtypes = [vp, vp, vp, vp, vp, vp, i32]
    lib.adore_attend.restype = ctypes.c_int
    lib.adore_attend.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.adore_schedule.restype = ctypes.c_int
    lib.adore_schedule.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.adore_rebuild.restype = ctypes.c_int
    lib.adore_rebuild.argtypes = [vp, i32, vp]
    lib.adore_decode_step.restype = ctypes.c_int
    lib.adore_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.adore_forward_step.restype = ctypes.c_int
    lib.adore_forward_step.argtypes = [vp, ctypes.POINTER(AdoreForwardWeights), vp, vp, vp, vp, vp, vp, vp]
    lib.adore_get_state.restype = ctypes.c_int
    lib.adore_get_state.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.POINTER(i32)]
    lib.adore_set_state.restype = ctypes.c_int
    lib.adore_set_state.argtypes = [vp, vp, vp, vp, vp, vp, i32]
    lib.adore_set_input_order.restype = ctypes.c_int
    lib.adore_set_input_order.argtypes = [vp, i32]
    lib.adore_set_timing.restype = ctypes.c_int
    lib.adore_set_timing.argtypes = [vp, i32]
    lib.adore_read_timing.restype = ctypes.c_int
    lib.adore_read_timing.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
    lib.adore_kernel_name.restype = ctypes.c_char_p
    lib.adore_kernel_name.argtypes = [i32]
    lib.adore_strerror.restype = ctypes.c_char_p
    lib.adore_strerror.argtypes = [ctypes.c_int]
    lib.adore_check_guards.restype = ctypes.c_int
    lib.adore_check_guards.argtypes = [vp, ctypes.POINTER(ctypes.c_int32)]
    lib.adore_abi_version.restype = ctypes.c_int
    lib.adore_abi_version.argtypes = []
    lib.adore_topk_attention_workspace_bytes.restype = sz
    lib.adore_topk_attention_workspace_bytes.argtypes = [i32, i32, i32]
    lib.adore_topk_attention.restype = ctypes.c_int
    lib.adore_topk_attention.argtypes = [vp, vp, vp, vp, vp, sz, i32, i32, i32, i32, vp]
    lib.adore_topk_attention_static.restype = ctypes.c_int
    lib.adore_topk_attention_static.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp]
    _lib = lib
    return lib


def _check(lib, rc: int):
    if rc != 0:
        raise AdoreError(rc, lib.adore_strerror(rc).decode())


def make_config(*, layers, batch, heads, head_dim, hidden, cache_slots, rebuild_budget, max_positions,
                ctrl_hidden, dtype, pos_scale, score_mode=0, rope_base=0.0) -> AdoreConfig:
    code = {"f32": ADORE_F32, "bf16": ADORE_BF16}[dtype] if isinstance(dtype, str) else int(dtype)
    return AdoreConfig(layers, batch, heads, head_dim, hidden, cache_slots, rebuild_budget, max_positions,
                       ctrl_hidden, code, pos_scale, int(score_mode), float(rope_base))


def topk_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, top_k: int, out: torch.Tensor = None,
                   workspace: torch.Tensor = None) -> torch.Tensor:
    """adore_topk_attention on torch's current stream.  q, k, v: [rows, seq, head_dim] bf16, contiguous, on the GPU;
    out and workspace (uint8) are allocated here unless given."""
    lib = load_library()
    for name, t in (("q", q), ("k", k), ("v", v)):
        if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous() or t.shape != q.shape or t.dim() != 3:
            raise ValueError(f"{name}: expected a contiguous bf16 GPU tensor [rows, seq, head_dim]")
    rows, seq, d = q.shape
    if out is None:
        out = torch.empty_like(q)
    elif out.dtype != torch.bfloat16 or not out.is_contiguous() or out.shape != q.shape or out.device != q.device:
        raise ValueError("out: expected a contiguous bf16 tensor like q")
    need = lib.adore_topk_attention_workspace_bytes(rows, seq, d)
    if workspace is None:
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=q.device)
    elif workspace.dtype != torch.uint8 or not workspace.is_contiguous() or workspace.device != q.device:
        raise ValueError("workspace: expected a contiguous uint8 tensor on q's device")
    stream = torch.cuda.current_stream(q.device).cuda_stream
    _check(lib, lib.adore_topk_attention(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), workspace.data_ptr(),
                                         workspace.numel(), rows, seq, d, int(top_k), stream))
    return out


def topk_attention_static(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, top_k: int, out: torch.Tensor) -> torch.Tensor:
    """adore_topk_attention_static on torch's current stream: no workspace, nothing allocated (out is the caller's)."""
    lib = load_library()
    for name, t in (("q", q), ("k", k), ("v", v), ("out", out)):
        if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous() or t.shape != q.shape or t.dim() != 3:
            raise ValueError(f"{name}: expected a contiguous bf16 GPU tensor [rows, seq, head_dim]")
    rows, seq, d = q.shape
    stream = torch.cuda.current_stream(q.device).cuda_stream
    _check(lib, lib.adore_topk_attention_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), rows, seq, d,
                                                int(top_k), stream))
    return out


class Adore:
    """One decode job.  Method names and argument order follow include/adore.h."""

    def __init__(self, cfg: AdoreConfig, weights: Dict[str, torch.Tensor], device="cuda:0"):
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        self.storage = torch.bfloat16 if cfg.dtype == ADORE_BF16 else torch.float32
        c = cfg
        dp, Hd = c.ctrl_hidden, c.heads * c.head_dim
        shapes = {"w_kv": (c.layers, 2 * Hd, c.hidden), "gru_w_ih": (3 * dp, c.hidden), "gru_w_hh": (3 * dp, dp),
                  "gru_b_ih": (3 * dp,), "gru_b_hh": (3 * dp,), "pos_w": (dp,), "pos_b": (dp,),
                  "mlp_w1": (dp, dp), "mlp_b1": (dp,), "out_w": (dp,), "out_b": (1,)}
        self._weights = {}
        w = AdoreWeights()
        for name in _WEIGHT_FIELDS:
            dt = self.storage if name in ("w_kv", "gru_w_ih", "gru_w_hh") else torch.float32
            setattr(w, name, self._ptr(weights[name], shapes[name], dt, name))
            self._weights[name] = weights[name]          # keep alive
        nbytes = self.lib.adore_workspace_bytes(ctypes.byref(cfg))
        if nbytes == 0:
            raise AdoreError(-1, "invalid configuration")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        self.stream = torch.cuda.current_stream(self.device)
        handle = ctypes.c_void_p()
        _check(self.lib, self.lib.adore_create(ctypes.byref(cfg), ctypes.byref(w), base, nbytes,
                                               self.stream.cuda_stream, ctypes.byref(handle)))
        self.handle = handle

    # -- marshalling ---------------------------------------------------------
    def _ptr(self, t: Optional[torch.Tensor], shape: Sequence[int], dtype: torch.dtype, name: str,
             optional: bool = False):
        if t is None:
            if optional:
                return None
            raise ValueError(f"{name} is required")
        if t.device.type != "cuda" or t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous():
            raise ValueError(f"{name}: expected contiguous cuda {dtype} tensor of shape {tuple(shape)}, got "
                             f"{t.device} {t.dtype} {tuple(t.shape)} contiguous={t.is_contiguous()}")
        if t.data_ptr() % 16:
            raise ValueError(f"{name}: base not 16-byte aligned")
        return t.data_ptr()

    def close(self):
        if getattr(self, "handle", None):
            self.lib.adore_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the ABI -------------------------------------------------------------
    def init_cache(self, prompt_k, prompt_v, hidden_store, ctrl_input, score_override, S: int):
        c, st = self.cfg, self.storage
        _check(self.lib, self.lib.adore_init_cache(
            self.handle,
            self._ptr(prompt_k, (c.layers, c.batch, c.heads, S, c.head_dim), st, "prompt_k"),
            self._ptr(prompt_v, (c.layers, c.batch, c.heads, S, c.head_dim), st, "prompt_v"),
            self._ptr(hidden_store, (c.layers, c.batch, c.max_positions, c.hidden), st, "hidden_store",
                      optional=True),                    # None: prepare for forward_step
            self._ptr(ctrl_input, (c.batch, S, c.hidden), st, "ctrl_input"),
            self._ptr(score_override, (c.batch, c.heads, S) if c.score_mode == SCORE_H2O else (c.batch, S),
                      torch.float32, "score_override", optional=True), S))

    def attend(self, layer: int, q, k_new, v_new, out):
        c, st = self.cfg, self.storage
        shp = (c.batch, c.heads, c.head_dim)
        _check(self.lib, self.lib.adore_attend(
            self.handle, layer, self._ptr(q, shp, st, "q"), self._ptr(k_new, shp, st, "k_new"),
            self._ptr(v_new, shp, st, "v_new"), self._ptr(out, shp, torch.float32, "out")))

    def schedule(self, x_n, score_override=None, slot_map=None, released_pos=None, rebuilt_pos=None):
        c = self.cfg
        _check(self.lib, self.lib.adore_schedule(
            self.handle, self._ptr(x_n, (c.batch, c.hidden), self.storage, "x_n", optional=c.score_mode == SCORE_H2O),
            self._ptr(score_override, (c.batch,), torch.float32, "score_override", optional=True),
            self._ptr(slot_map, (c.batch, c.heads, c.cache_slots), torch.int32, "slot_map", optional=True),
            self._ptr(released_pos, (c.batch, c.heads, c.rebuild_budget + 1), torch.int32, "released_pos",
                      optional=True),
            self._ptr(rebuilt_pos, (c.batch, max(c.rebuild_budget, 1)), torch.int32, "rebuilt_pos",
                      optional=True)))

    def rebuild(self, layer: int, hidden_store_layer):
        c = self.cfg
        _check(self.lib, self.lib.adore_rebuild(
            self.handle, layer,
            self._ptr(hidden_store_layer, (c.batch, c.max_positions, c.hidden), self.storage, "hidden_store_layer")))

    def decode_step(self, q, k_new, v_new, hidden_store, x_n, score_override, out, slot_map=None):
        c, st = self.cfg, self.storage
        shp = (c.batch, c.heads, c.head_dim)
        _check(self.lib, self.lib.adore_decode_step(
            self.handle, self._ptr(q, shp, st, "q"), self._ptr(k_new, shp, st, "k_new"),
            self._ptr(v_new, shp, st, "v_new"),
            self._ptr(hidden_store, (c.batch, c.max_positions, c.hidden), st, "hidden_store"),
            self._ptr(x_n, (c.batch, c.hidden), st, "x_n", optional=c.score_mode == SCORE_H2O),
            self._ptr(score_override, (c.batch,), torch.float32, "score_override", optional=True),
            self._ptr(out, shp, torch.float32, "out"),
            self._ptr(slot_map, (c.batch, c.heads, c.cache_slots), torch.int32, "slot_map", optional=True)))

    def forward_step(self, w_q, w_o, embed, score_override, rows_out, slot_map=None, released_pos=None,
                     rebuilt_pos=None, layer_rows=None):
        c, st = self.cfg, self.storage
        Hd = c.heads * c.head_dim
        fw = AdoreForwardWeights(self._ptr(w_q, (c.layers, Hd, c.hidden), st, "w_q"),
                                 self._ptr(w_o, (c.layers, c.hidden, Hd), st, "w_o"))
        _check(self.lib, self.lib.adore_forward_step(
            self.handle, ctypes.byref(fw),
            self._ptr(embed, (c.batch, c.max_positions, c.hidden), st, "embed"),
            self._ptr(score_override, (c.batch,), torch.float32, "score_override", optional=True),
            self._ptr(rows_out, (c.batch, c.rebuild_budget + 1, c.hidden), st, "rows_out"),
            self._ptr(layer_rows, (c.layers, c.batch, c.rebuild_budget + 1, c.hidden), st, "layer_rows", optional=True),
            self._ptr(slot_map, (c.batch, c.heads, c.cache_slots), torch.int32, "slot_map", optional=True),
            self._ptr(released_pos, (c.batch, c.heads, c.rebuild_budget + 1), torch.int32, "released_pos",
                      optional=True),
            self._ptr(rebuilt_pos, (c.batch, max(c.rebuild_budget, 1)), torch.int32, "rebuilt_pos",
                      optional=True)))

    def _state_ptrs(self, slot_pos, scores, z, cache_k, cache_v):
        c, st = self.cfg, self.storage
        cs = (c.layers, c.batch, c.heads, c.cache_slots, c.head_dim)
        return (self._ptr(slot_pos, (c.batch, c.heads, c.cache_slots), torch.int32, "slot_pos", optional=True),
                self._ptr(scores, self._score_shape(), torch.float32, "scores", optional=True),
                self._ptr(z, (c.batch, c.ctrl_hidden), torch.float32, "z", optional=True),
                self._ptr(cache_k, cs, st, "cache_k", optional=True),
                self._ptr(cache_v, cs, st, "cache_v", optional=True))

    def _score_shape(self):
        c = self.cfg
        return (c.batch, c.heads, c.max_positions) if c.score_mode == SCORE_H2O else (c.batch, c.max_positions)

    def get_state(self, slot_pos=None, scores=None, z=None, cache_k=None, cache_v=None) -> int:
        step = ctypes.c_int32(-1)
        _check(self.lib, self.lib.adore_get_state(self.handle, *self._state_ptrs(slot_pos, scores, z, cache_k, cache_v),
                                                  ctypes.byref(step)))
        return step.value

    def set_state(self, slot_pos, scores, z, cache_k, cache_v, step: int):
        _check(self.lib, self.lib.adore_set_state(self.handle, *self._state_ptrs(slot_pos, scores, z, cache_k, cache_v),
                                                  step))

    def set_input_order(self, ordered: bool):
        _check(self.lib, self.lib.adore_set_input_order(self.handle, int(ordered)))

    def check_guards(self) -> int:
        """Damaged guard words of the debug layout (ADORE_GUARD_WORDS=1 at create), or -1 if there are none."""
        bad = ctypes.c_int32(0)
        _check(self.lib, self.lib.adore_check_guards(self.handle, ctypes.byref(bad)))
        return int(bad.value)

    def set_timing(self, enable: bool):
        _check(self.lib, self.lib.adore_set_timing(self.handle, int(enable)))

    def read_timing(self):
        ms = (ctypes.c_float * len(KERNELS))()
        cnt = (ctypes.c_int32 * len(KERNELS))()
        _check(self.lib, self.lib.adore_read_timing(self.handle, ms, cnt))
        return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(KERNELS)}

    # -- convenience (allocation only) ----------------------------------------
    def empty_state(self):
        c, st, dev = self.cfg, self.storage, self.device
        cs = (c.layers, c.batch, c.heads, c.cache_slots, c.head_dim)
        return dict(slot_pos=torch.empty((c.batch, c.heads, c.cache_slots), dtype=torch.int32, device=dev),
                    scores=torch.empty(self._score_shape(), dtype=torch.float32, device=dev),
                    z=torch.empty((c.batch, c.ctrl_hidden), dtype=torch.float32, device=dev),
                    cache_k=torch.empty(cs, dtype=st, device=dev), cache_v=torch.empty(cs, dtype=st, device=dev))
