"""Workload shapes and seeded tensors for the ADORE decode path.

Everything returned is a float32 numpy array whose values are exactly
representable in the workload's storage type (bf16 or fp32), so an upload to
the GPU in that type and an upcast to fp64 on the CPU start from the same
bits.  Random streams are counter based (numpy's Philox) and keyed by
(seed + 1000*layer, tensor id, step), so any tensor can be regenerated alone.

Symbols follow the paper: m persistent cache rows and R rebuilt rows per step
(Sec. 3.1 "Experimental Protocols"); K = m + R + 1 physical slots is the
number of rows attention sees (Sec. 2.3); d' is the controller's hidden size
(App. "Implementation Details").
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np

BASE_SEED = 20240702

# tensor ids (second Philox key word, high half)
_T_Q, _T_K, _T_V, _T_PK, _T_PV, _T_HID, _T_WKV = 1, 2, 3, 4, 5, 6, 7
_T_GRU_IH, _T_GRU_HH, _T_GRU_BIH, _T_GRU_BHH = 8, 9, 10, 11
_T_POS_W, _T_POS_B, _T_W1, _T_B1, _T_WO, _T_BO = 12, 13, 14, 15, 16, 17
_T_SAL_PERM, _T_SAL_DIR = 18, 19
_T_WQ, _T_WOUT = 20, 21


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even), kept as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) & np.uint32(0xFFFF0000)).view(np.float32)


@dataclass(frozen=True)
class Workload:
    name: str
    L: int          # layers
    B: int          # batch (sequences)
    H: int          # heads
    d: int          # head_dim
    D: int          # hidden size
    K: int          # physical cache slots per (sequence, head) = m + R + 1
    R: int          # rebuild budget, tokens / step / sequence
    S: int          # prompt length
    T: int          # decode steps
    dtype: str      # "f32" | "bf16": storage of cache, q/k/v, hidden, W_kv, GRU matrices
    dprime: int = 128
    pos_scale: float = 2.0 ** -12
    act_std: float = 1.0     # q, k, v, hidden
    w_std: float = 0.02      # W_kv
    salience: bool = False   # heavy-tailed per-token offset (long-context workload)
    rescore: bool = False    # controller scores every token again at every step (relative position)
    rope_base: float = 0.0   # > 0: rotary position embedding with this base on keys/queries made from hidden states
    h2o: bool = False        # scores are the attention each head has given a token so far (the H2O(Rebuilt) baseline)
    seed: int = BASE_SEED

    @property
    def m(self) -> int:
        return self.K - self.R - 1

    @property
    def N_max(self) -> int:
        return self.S + self.T

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


def _tiny_std(d: int) -> float:
    return 1.0 / np.sqrt(d)


WORKLOADS: Dict[str, Workload] = {
    # The five benchmark workloads.  Where no rebuild budget is specified, R = 32 is used.
    "tiny": Workload("tiny", L=1, B=1, H=4, d=64, D=256, K=64, R=8, S=128, T=256, dtype="f32",
                     act_std=_tiny_std(64), w_std=_tiny_std(64)),
    "llama7b_layer": Workload("llama7b_layer", L=1, B=16, H=32, d=128, D=4096, K=512, R=32,
                              S=1024, T=512, dtype="bf16"),
    "long_context": Workload("long_context", L=1, B=4, H=32, d=128, D=4096, K=1024, R=32,
                             S=8192, T=1024, dtype="bf16", salience=True),
    "high_batch": Workload("high_batch", L=1, B=128, H=32, d=128, D=4096, K=256, R=16,
                           S=512, T=256, dtype="bf16"),
    "stack32": Workload("stack32", L=32, B=32, H=32, d=128, D=4096, K=512, R=32,
                        S=2048, T=512, dtype="bf16"),
}


def workload(name: str) -> Workload:
    return WORKLOADS[name]


class SyntheticInputs:
    """All tensors of one workload, generated on demand from the seed."""

    def __init__(self, w: Workload):
        self.w = w
        self._sal = None

    # -- random streams -------------------------------------------------------
    def _rng(self, tensor_id: int, layer: int = 0, step: int = 0) -> np.random.Generator:
        key = [self.w.seed + 1000 * layer, (tensor_id << 32) | step]
        return np.random.Generator(np.random.Philox(key=key))

    def _store(self, a: np.ndarray) -> np.ndarray:
        a = np.ascontiguousarray(a, dtype=np.float32)
        return round_bf16(a) if self.w.dtype == "bf16" else a

    def _normal(self, shape, std, tensor_id, layer=0, step=0, storage=True) -> np.ndarray:
        a = self._rng(tensor_id, layer, step).standard_normal(shape, dtype=np.float32)
        a *= np.float32(std)
        return self._store(a) if storage else a

    # -- salience (long-context workload) -------------------------------------
    def salience(self) -> np.ndarray:
        """[B, N_max] logit offsets s_i = c * rank_i^-1.1, top token gets +8."""
        if self._sal is None:
            w = self.w
            s = np.zeros((w.B, w.N_max), dtype=np.float64)
            if w.salience:
                for b in range(w.B):
                    perm = self._rng(_T_SAL_PERM, 0, b).permutation(w.N_max) + 1
                    s[b] = 8.0 * perm.astype(np.float64) ** -1.1
            self._sal = s
        return self._sal

    # -- weights --------------------------------------------------------------
    def weights(self) -> Dict[str, np.ndarray]:
        w = self.w
        dp = w.dprime
        out = {
            "w_kv": np.stack([self._normal((2 * w.H * w.d, w.D), w.w_std, _T_WKV, l)
                              for l in range(w.L)]),
            "gru_w_ih": self._normal((3 * dp, w.D), 1.0 / np.sqrt(w.D), _T_GRU_IH),
            "gru_w_hh": self._normal((3 * dp, dp), 1.0 / np.sqrt(dp), _T_GRU_HH),
            # fp32 parameters (never stored in bf16)
            "gru_b_ih": self._normal((3 * dp,), 0.1, _T_GRU_BIH, storage=False),
            "gru_b_hh": self._normal((3 * dp,), 0.1, _T_GRU_BHH, storage=False),
            "pos_w": self._normal((dp,), 1.0, _T_POS_W, storage=False),
            "pos_b": self._normal((dp,), 0.1, _T_POS_B, storage=False),
            "mlp_w1": self._normal((dp, dp), 1.0 / np.sqrt(dp), _T_W1, storage=False),
            "mlp_b1": self._normal((dp,), 0.1, _T_B1, storage=False),
            "out_w": self._normal((dp,), 4.0 / np.sqrt(dp), _T_WO, storage=False),
            "out_b": self._normal((1,), 0.1, _T_BO, storage=False),
        }
        return out

    def forward_weights(self) -> Dict[str, np.ndarray]:
        """Query and output projections of every layer, for the rebuild forward through a layer stack:
        w_q [L, H*d, D], w_o [L, D, H*d] (rows of w_q grouped by head like W_k)."""
        w = self.w
        return {
            "w_q": np.stack([self._normal((w.H * w.d, w.D), w.w_std, _T_WQ, l) for l in range(w.L)]),
            "w_o": np.stack([self._normal((w.D, w.H * w.d), w.w_std, _T_WOUT, l) for l in range(w.L)]),
        }

    # -- activations ----------------------------------------------------------
    def hidden_store_layer(self, layer: int) -> np.ndarray:
        """[B, N_max, D]: the hidden state entering `layer` for every position.

        Layer 0's rows are the token embeddings the controller reads (x_i).
        """
        w = self.w
        hs = self._rng(_T_HID, layer).standard_normal((w.B, w.N_max, w.D), dtype=np.float32)
        hs *= np.float32(w.act_std)
        if w.salience and layer == 0:
            u = self._rng(_T_SAL_DIR).standard_normal(w.D)
            u /= np.linalg.norm(u)
            kappa = 4.0
            hs += (kappa * self.salience()[:, :, None] * u[None, None, :]).astype(np.float32)
        return self._store(hs)

    def hidden_store(self) -> np.ndarray:
        """[L, B, N_max, D].  Only for workloads small enough to hold at once."""
        return np.stack([self.hidden_store_layer(l) for l in range(self.w.L)])

    def prompt_kv(self) -> Tuple[np.ndarray, np.ndarray]:
        """prompt_k, prompt_v: [L, B, H, S, d]."""
        w = self.w
        ks, vs = [], []
        for l in range(w.L):
            k = self._rng(_T_PK, l).standard_normal((w.B, w.H, w.S, w.d), dtype=np.float32)
            k *= np.float32(w.act_std)
            if w.salience:
                k[:, :, :, 0] = (self.salience()[:, None, :w.S] * np.sqrt(w.d)).astype(np.float32)
            ks.append(self._store(k))
            vs.append(self._normal((w.B, w.H, w.S, w.d), w.act_std, _T_PV, l))
        return np.stack(ks), np.stack(vs)

    def step_qkv(self, n: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """q, k_new, v_new for the token at position n: each [L, B, H, d]."""
        w = self.w
        qs, ks, vs = [], [], []
        for l in range(w.L):
            q = self._normal((w.B, w.H, w.d), w.act_std, _T_Q, l, n, storage=False)
            k = self._normal((w.B, w.H, w.d), w.act_std, _T_K, l, n, storage=False)
            if w.salience:
                q[:, :, 0] = 1.0
                k[:, :, 0] = (self.salience()[:, None, n] * np.sqrt(w.d)).astype(np.float32)
            qs.append(self._store(q))
            ks.append(self._store(k))
            vs.append(self._normal((w.B, w.H, w.d), w.act_std, _T_V, l, n))
        return np.stack(qs), np.stack(ks), np.stack(vs)


class DeviceNormals:
    """Large tensors drawn on the GPU from one seeded torch generator (tens of GB, which the host generator above
    would take minutes to produce).  N(0, std) rounded to the storage type; draws come in a fixed order, in
    pieces, so the temporaries stay bounded."""

    def __init__(self, seed: int, device: str):
        import torch
        self.torch = torch
        self.device = device
        self.g = torch.Generator(device=device)
        self.g.manual_seed(seed)

    def normal(self, shape, std, dtype):
        torch = self.torch
        out = torch.empty(shape, dtype=dtype, device=self.device)
        flat = out.view(-1)
        piece = 1 << 28
        for i in range(0, flat.numel(), piece):
            n = min(piece, flat.numel() - i)
            flat[i:i + n] = (torch.randn(n, generator=self.g, device=self.device, dtype=torch.float32) * std).to(dtype)
        return out
