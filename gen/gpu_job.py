"""Device-side twin of a workload: the seeded inputs uploaded byte for byte and one decode job on them, driven
through the C-ABI binding.  Used by the GPU tests (next to the oracle) and by bench.py (alone); nothing here knows
the oracle, and nothing of the method is computed here."""
import numpy as np
import torch

from gen.synthetic import SyntheticInputs, Workload
from paper_2407_02328_amd import Adore, make_config

DEV = "cuda:0"


def storage_dtype(w: Workload):
    return torch.bfloat16 if w.dtype == "bf16" else torch.float32


def to_dev(a: np.ndarray, dtype) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV).to(dtype).contiguous()


def adore_config(w: Workload):
    return make_config(layers=w.L, batch=w.B, heads=w.H, head_dim=w.d, hidden=w.D, cache_slots=w.K,
                       rebuild_budget=w.R, max_positions=w.N_max, ctrl_hidden=w.dprime, dtype=w.dtype,
                       pos_scale=w.pos_scale, score_mode=2 if w.h2o else 1 if w.rescore else 0, rope_base=w.rope_base)


def device_weights(w: Workload, wts):
    st = storage_dtype(w)
    return {k: to_dev(v, st if k in ("w_kv", "gru_w_ih", "gru_w_hh") else torch.float32) for k, v in wts.items()}


class GpuJob:
    """Device-side twin of an oracle run: same workload, same inputs, uploaded byte for byte."""

    def __init__(self, w: Workload, inp: SyntheticInputs = None, wts=None, hidden=None, prompt=None, ordered=True):
        self.w = w
        self.ordered = ordered     # False: inputs are complete in memory at every call (synchronised first)
        self.inp = inp or SyntheticInputs(w)
        self.wts = wts if wts is not None else self.inp.weights()
        st = storage_dtype(w)
        self.st = st
        self.adore = Adore(adore_config(w), device_weights(w, self.wts), DEV)
        if not ordered:
            self.adore.set_input_order(False)
        self.hidden_np = self.inp.hidden_store() if hidden is None else hidden
        self.hidden = to_dev(self.hidden_np, st)
        self.prompt_np = self.inp.prompt_kv() if prompt is None else prompt
        self.out = torch.empty((w.L, w.B, w.H, w.d), dtype=torch.float32, device=DEV)
        self.slot_map = torch.empty((w.B, w.H, w.K), dtype=torch.int32, device=DEV)
        self.released = torch.empty((w.B, w.H, w.R + 1), dtype=torch.int32, device=DEV)
        self.rebuilt = torch.empty((w.B, max(w.R, 1)), dtype=torch.int32, device=DEV)
        self.state = self.adore.empty_state()

    def init(self, score_override=None):
        w = self.w
        pk, pv = self.prompt_np
        ov = None if score_override is None else to_dev(score_override, torch.float32)
        self.adore.init_cache(to_dev(pk, self.st), to_dev(pv, self.st), self.hidden,
                              self.hidden[0][:, :w.S].contiguous(), ov, w.S)
        torch.cuda.synchronize()

    def step(self, n, qkv=None, override=None, whole=False, x_n=None):
        """One step through the fine-grained calls, or (whole, L = 1) through adore_decode_step, which reports
        the slot map only.  x_n: a device buffer to pass as the controller input instead of a fresh copy of the
        token's row.  Returns numpy (out, slot_map, released, rebuilt, score_n)."""
        w = self.w
        q, k, v = self.inp.step_qkv(n) if qkv is None else qkv
        qd, kd, vd = (to_dev(a, self.st) for a in (q, k, v))
        ov = None if override is None else to_dev(np.asarray(override, dtype=np.float32), torch.float32)
        if x_n is None:
            x_n = self.hidden[0][:, n].contiguous()  # a copy kernel on the stream the context is bound to
        if not self.ordered:
            torch.cuda.synchronize()
        if whole:
            self.adore.decode_step(qd[0], kd[0], vd[0], self.hidden[0], x_n, ov, self.out[0], self.slot_map)
        else:
            for l in range(w.L):
                self.adore.attend(l, qd[l], kd[l], vd[l], self.out[l])
            self.adore.schedule(x_n, ov, self.slot_map, self.released, self.rebuilt)
            for l in range(w.L):
                self.adore.rebuild(l, self.hidden[l])
        # the scores, and the caches as the step leaves them (device copies: adopt_rebuilt_rows reads rows of them)
        self.adore.get_state(scores=self.state["scores"], cache_k=self.state["cache_k"], cache_v=self.state["cache_v"])
        torch.cuda.synchronize()
        sc = self.state["scores"]     # H2O: [B,H,N_max], every held token's score moves at every step
        score_n = sc[..., :n + 1].cpu().numpy() if (w.rescore or w.h2o) else sc[:, n].cpu().numpy()
        return (self.out.cpu().numpy().astype(np.float64), self.slot_map.cpu().numpy(),
                self.released.cpu().numpy(), self.rebuilt.cpu().numpy()[:, :w.R], score_n)

    def snapshot(self):
        self.adore.get_state(**self.state)
        torch.cuda.synchronize()
        return {k: v.float().cpu().numpy() if v.dtype.is_floating_point else v.cpu().numpy()
                for k, v in self.state.items()}
