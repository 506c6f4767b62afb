"""Shared test plumbing: build an oracle for a workload, parse the golden trajectory."""
import os

import numpy as np

from gen import SyntheticInputs, Workload
from oracle.adore_oracle import AdoreOracle, OracleConfig

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def oracle_config(w: Workload) -> OracleConfig:
    return OracleConfig(L=w.L, B=w.B, H=w.H, d=w.d, D=w.D, K=w.K, R=w.R, N_max=w.N_max,
                        dprime=w.dprime, dtype=w.dtype, pos_scale=w.pos_scale, rescore=w.rescore,
                        rope_base=w.rope_base)


def make_oracle(w: Workload, weights=None):
    inp = SyntheticInputs(w)
    wts = inp.weights() if weights is None else weights
    return AdoreOracle(oracle_config(w), wts), inp, wts


def small_workload(**kw) -> Workload:
    base = dict(name="small", L=1, B=2, H=2, d=16, D=32, K=12, R=3, S=20, T=24, dtype="f32",
                dprime=8, act_std=1.0, w_std=0.2)
    base.update(kw)
    return Workload(**base)


def parse_trajectory(path):
    """Returns (init_scores, after_init, steps) from a golden slot-trajectory file."""
    init_scores, steps, after_init = [], [], None

    def ints(s):
        return [int(t) for t in s.split()]

    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split("|")]
            head = parts[0].split()
            if head[0] == "init":
                init_scores.append(float(head[2]))
            elif head[0] == "after_init":
                after_init = dict(slot_map=ints(parts[1]), rebuilt=ints(parts[3]))
            elif head[0] == "step":
                steps.append(dict(n=int(head[1]), score=float(head[2]), slot_map=ints(parts[1]),
                                  released=ints(parts[2]), rebuilt=ints(parts[3])))
    return np.array(init_scores, dtype=np.float32), after_init, steps
