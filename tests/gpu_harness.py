"""Runs the HIP path (through the C-ABI binding) next to the oracle on the same seeded inputs."""
import numpy as np
import torch

from gen import SyntheticInputs, Workload
from paper_2407_02328_amd import Adore, make_config
from tests.helpers import make_oracle

DEV = "cuda:0"


def storage_dtype(w: Workload):
    return torch.bfloat16 if w.dtype == "bf16" else torch.float32


def to_dev(a: np.ndarray, dtype) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV).to(dtype).contiguous()


def adore_config(w: Workload):
    return make_config(layers=w.L, batch=w.B, heads=w.H, head_dim=w.d, hidden=w.D, cache_slots=w.K,
                       rebuild_budget=w.R, max_positions=w.N_max, ctrl_hidden=w.dprime, dtype=w.dtype,
                       pos_scale=w.pos_scale, score_mode=1 if w.rescore else 0, rope_base=w.rope_base)


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
        self.adore.get_state(scores=self.state["scores"])
        torch.cuda.synchronize()
        sc = self.state["scores"]
        score_n = sc[:, :n + 1].cpu().numpy() if w.rescore else sc[:, n].cpu().numpy()
        return (self.out.cpu().numpy().astype(np.float64), self.slot_map.cpu().numpy(),
                self.released.cpu().numpy(), self.rebuilt.cpu().numpy()[:, :w.R], score_n)

    def snapshot(self):
        self.adore.get_state(**self.state)
        torch.cuda.synchronize()
        return {k: v.float().cpu().numpy() if v.dtype.is_floating_point else v.cpu().numpy()
                for k, v in self.state.items()}


def row_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max over rows of  max|got - want| / max|want|  (rows = last axis)."""
    num = np.abs(got - want).max(axis=-1)
    den = np.abs(want).max(axis=-1)
    return float((num / np.maximum(den, 1e-30)).max())


def out_tol(w: Workload) -> float:
    return 2e-3 if w.dtype == "bf16" else 1e-5


def lockstep(w: Workload, steps: int, override=None, check_cache_every=0, wts=None, whole=None, ordered=True,
             full_size_rows=False):
    """Free-running GPU trajectory with the oracle in lockstep.  whole: None = every step through attend /
    schedule / rebuild; otherwise a function of the step index that says which steps go through
    adore_decode_step (released and rebuilt positions are then checked through the slot map only).

    Each step the oracle computes its own sigma_n, which must agree with the GPU's to 1e-5; it then
    adopts the GPU's bits so that both sides select from identical keys.  Slot maps, released and
    rebuilt positions must be identical; outputs within the storage type's tolerance.
    ordered: True / False = the context's input order for the whole run; a function of the step index
    switches it from step to step (inputs are then complete at every call).
    full_size_rows: the row check of the full-size sampled runs (thousands of rebuilt rows per step, of which a
    few per thousand land on the neighbouring storage value; such an entry of a key moves its token's logit by
    q_j * ulp / sqrt(d), which a row whose probability sits on that token shows in full): every row within the
    tolerance + 2^-7, all but 0.5 % within the tolerance.
    """
    orc, inp, wts = make_oracle(w, wts)
    job = GpuJob(w, inp, wts, ordered=ordered if isinstance(ordered, bool) else False)
    hs = job.hidden_np
    pk, pv = job.prompt_np
    job.init(None if override is None else override[:, :w.S])
    snap = job.snapshot()
    # init: the oracle adopts the GPU's prompt scores after checking them
    orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S,
                   score_override=None if override is None else override[:, :w.S])
    gpu_scores = snap["scores"][:, :w.S]
    assert np.abs(gpu_scores.astype(np.float64) - orc.score[:, :w.S].astype(np.float64)).max() < 1e-5
    if override is None and not np.array_equal(gpu_scores, orc.score[:, :w.S]):
        orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S, score_override=gpu_scores)
    assert np.array_equal(snap["slot_pos"], orc.slot_pos), "slot map after init"
    compare_cache(w, snap, orc)
    worst = 0.0
    for t in range(steps):
        n = w.S + t
        qkv = inp.step_qkv(n)
        ov = None if override is None else override[:, n]
        one_call = whole is not None and bool(whole(t))
        if not isinstance(ordered, bool):
            job.adore.set_input_order(bool(ordered(t)))
        out_g, map_g, rel_g, rb_g, score_g = job.step(n, qkv, ov, whole=one_call)
        out_o, map_o, rel_o, rb_o, own = orc.decode_step(*qkv, hs, hs[0][:, n],
                                                         score_override=score_g)
        if w.rescore:     # every score of this step: the oracle's own values against the GPU's, then adopted
            assert np.abs(orc.own_scores - score_g.astype(np.float64)).max() < 1e-5, f"sigma at n={n}"
        elif override is None:
            assert np.abs(own - score_g.astype(np.float64)).max() < 1e-5, f"sigma at n={n}"
        else:
            assert np.array_equal(score_g, ov.astype(np.float32))
        assert np.array_equal(map_g, map_o), f"slot map at n={n}"
        if not one_call:
            assert np.array_equal(rel_g, rel_o), f"released at n={n}"
            assert np.array_equal(rb_g, rb_o), f"rebuilt at n={n}"
        err = row_rel_err(out_g, out_o)
        worst = max(worst, err)
        if full_size_rows:
            e = np.abs(out_g - out_o).max(axis=-1) / np.maximum(np.abs(out_o).max(axis=-1), 1e-30)
            assert e.max() < out_tol(w) + 2.0 ** -7, f"attention output at n={n}: {e.max()}"
            assert (e >= out_tol(w)).mean() <= 0.005, f"attention output at n={n}: {(e >= out_tol(w)).sum()} rows beyond {out_tol(w)}"
        else:
            assert err < out_tol(w), f"attention output at n={n}: {err}"
        if check_cache_every and (t + 1) % check_cache_every == 0:
            compare_cache(w, job.snapshot(), orc)
    return worst, job, orc


def sampled_lockstep(w: Workload, steps: int, seqs, whole=lambda t: True):
    """A workload at its full size on the GPU, the oracle on a few of its sequences.  Sequences do not interact, so
    an oracle built for the sampled sequences alone (same weights, their rows of every input) must agree with those
    rows of the full run: scores within 1e-5 and then adopted, slot maps (released and rebuilt positions where the
    call reports them) identical, outputs and occupied cache rows within the storage type's tolerance."""
    from oracle.adore_oracle import AdoreOracle
    from tests.helpers import oracle_config
    seqs = list(seqs)
    inp = SyntheticInputs(w)
    wts = inp.weights()
    job = GpuJob(w, inp, wts)
    ws = w.scaled(B=len(seqs))
    orc = AdoreOracle(oracle_config(ws), wts)
    hs = job.hidden_np[:, seqs]
    pk, pv = (a[:, seqs] for a in job.prompt_np)
    job.init()

    def sampled_snapshot():
        snap = job.snapshot()
        return {k: (v[:, seqs] if k.startswith("cache") else v[seqs]) for k, v in snap.items()}

    snap = sampled_snapshot()
    orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S)
    gpu_scores = snap["scores"][:, :w.S]
    assert np.abs(gpu_scores.astype(np.float64) - orc.score[:, :w.S].astype(np.float64)).max() < 1e-5
    if not np.array_equal(gpu_scores, orc.score[:, :w.S]):
        orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S, score_override=gpu_scores)
    assert np.array_equal(snap["slot_pos"], orc.slot_pos), "slot map after init"
    compare_cache(ws, snap, orc)
    worst = 0.0
    for t in range(steps):
        n = w.S + t
        qkv = inp.step_qkv(n)
        one_call = bool(whole(t))
        out_g, map_g, rel_g, rb_g, score_g = job.step(n, qkv, whole=one_call)
        out_o, map_o, rel_o, rb_o, own = orc.decode_step(*(a[:, seqs] for a in qkv), hs, hs[0][:, n],
                                                         score_override=score_g[seqs])
        assert np.abs(own - score_g[seqs].astype(np.float64)).max() < 1e-5, f"sigma at n={n}"
        assert np.array_equal(map_g[seqs], map_o), f"slot map at n={n}"
        if not one_call:
            assert np.array_equal(rel_g[seqs], rel_o), f"released at n={n}"
            assert np.array_equal(rb_g[seqs], rb_o), f"rebuilt at n={n}"
        err = row_rel_err(out_g[:, seqs], out_o)
        worst = max(worst, err)
        assert err < out_tol(w), f"attention output at n={n}: {err}"
    compare_cache(ws, sampled_snapshot(), orc)
    return worst, job, orc


def stack_sampled(w: Workload, steps: int, seqs):
    """A layer stack too large for host-side inputs, at its full size: W_kv, hidden states and prompt K/V are drawn
    on the device (gen.DeviceNormals) and only the rows of the sampled sequences (and W_kv) come back for the
    oracle.  Every step through attend x L, schedule, rebuild x L.  Checks as in sampled_lockstep, every layer."""
    from gen import DeviceNormals
    from oracle.adore_oracle import AdoreOracle
    from tests.helpers import oracle_config
    seqs = list(seqs)
    st = storage_dtype(w)
    drawer = DeviceNormals(w.seed, DEV)
    small = SyntheticInputs(w.scaled(L=1, H=1, d=64, B=1)).weights()   # controller tensors do not depend on L, H, d, B
    dev_w = {k: to_dev(v, st if k in ("gru_w_ih", "gru_w_hh") else torch.float32) for k, v in small.items() if k != "w_kv"}
    dev_w["w_kv"] = drawer.normal((w.L, 2 * w.H * w.d, w.D), w.w_std, st)
    hidden = drawer.normal((w.L, w.B, w.N_max, w.D), w.act_std, st)
    prompt_k = drawer.normal((w.L, w.B, w.H, w.S, w.d), w.act_std, st)
    prompt_v = drawer.normal((w.L, w.B, w.H, w.S, w.d), w.act_std, st)
    adore = Adore(adore_config(w), dev_w, DEV)
    adore.init_cache(prompt_k, prompt_v, hidden, hidden[0][:, :w.S].contiguous(), None, w.S)
    state = adore.empty_state()
    out = torch.empty((w.L, w.B, w.H, w.d), dtype=torch.float32, device=DEV)
    slot_map = torch.empty((w.B, w.H, w.K), dtype=torch.int32, device=DEV)
    released = torch.empty((w.B, w.H, w.R + 1), dtype=torch.int32, device=DEV)
    rebuilt = torch.empty((w.B, max(w.R, 1)), dtype=torch.int32, device=DEV)

    def host(t):
        return t.float().cpu().numpy() if t.dtype.is_floating_point else t.cpu().numpy()

    def sampled_state():
        adore.get_state(**state)
        torch.cuda.synchronize()
        return {k: host(v[:, seqs] if k.startswith("cache") else v[seqs]) for k, v in state.items()}

    ws = w.scaled(B=len(seqs))
    wts = dict(small, w_kv=host(dev_w["w_kv"]))
    orc = AdoreOracle(oracle_config(ws), wts)
    hs = host(hidden[:, seqs])
    pk, pv = host(prompt_k[:, seqs]), host(prompt_v[:, seqs])
    snap = sampled_state()
    orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S)
    gpu_scores = snap["scores"][:, :w.S]
    assert np.abs(gpu_scores.astype(np.float64) - orc.score[:, :w.S].astype(np.float64)).max() < 1e-5
    if not np.array_equal(gpu_scores, orc.score[:, :w.S]):
        orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S, score_override=gpu_scores)
    assert np.array_equal(snap["slot_pos"], orc.slot_pos), "slot map after init"
    compare_cache(ws, snap, orc)
    inp = SyntheticInputs(w)
    worst = 0.0
    for t in range(steps):
        n = w.S + t
        q, k, v = inp.step_qkv(n)
        qd, kd, vd = (to_dev(a, st) for a in (q, k, v))
        for l in range(w.L):
            adore.attend(l, qd[l], kd[l], vd[l], out[l])
        adore.schedule(hidden[0][:, n].contiguous(), None, slot_map, released, rebuilt)
        for l in range(w.L):
            adore.rebuild(l, hidden[l])
        adore.get_state(scores=state["scores"])
        torch.cuda.synchronize()
        score_g = state["scores"][:, n].cpu().numpy()
        out_o, map_o, rel_o, rb_o, own = orc.decode_step(q[:, seqs], k[:, seqs], v[:, seqs], hs, hs[0][:, n],
                                                         score_override=score_g[seqs])
        assert np.abs(own - score_g[seqs].astype(np.float64)).max() < 1e-5, f"sigma at n={n}"
        assert np.array_equal(slot_map.cpu().numpy()[seqs], map_o), f"slot map at n={n}"
        assert np.array_equal(released.cpu().numpy()[seqs], rel_o), f"released at n={n}"
        assert np.array_equal(rebuilt.cpu().numpy()[seqs][:, :w.R], rb_o), f"rebuilt at n={n}"
        # Thousands of rows per step.  A rebuilt cache row may differ from the oracle's by one unit in the last place
        # (compare_cache: fp32 against fp64 accumulation, one rounding each), 2^-7 of the entry; a row of the output
        # whose softmax sits on such a row inherits up to that much on top of the attention's own 2e-3.  So: every
        # row within 2e-3 + 2^-7, and all but a handful within 2e-3.
        got = out.cpu().numpy().astype(np.float64)[:, seqs]
        e = np.abs(got - out_o).max(axis=-1) / np.maximum(np.abs(out_o).max(axis=-1), 1e-30)
        worst = max(worst, float(e.max()))
        assert e.max() < out_tol(w) + 2.0 ** -7, f"attention output at n={n}: {e.max()}"
        assert (e >= out_tol(w)).mean() <= 0.005, f"attention output at n={n}: {(e >= out_tol(w)).sum()} rows beyond {out_tol(w)}"
    compare_cache(ws, sampled_state(), orc)
    adore.close()
    return worst


def compare_cache(w: Workload, snap, orc):
    """Occupied rows of the GPU cache against the oracle's: inserted rows are copies (exact);
    rebuilt rows are fp32-accumulated and rounded once, so a value may land on the neighbouring
    storage value (one unit in the last place); entries that cancel to almost zero additionally
    carry the fp32 accumulation error itself, bounded here by 2e-5 of the largest entry.
    With the rotary embedding a key row is the rotation of the rounded projection: where the projection landed
    on the neighbouring storage value, the rotation spreads that unit over the two entries of a plane (at most
    sqrt(2) of it, measured at the row's largest entry) before the second rounding adds its own; such rows are
    rare, so all but 1 % of the entries still have to be within one unit."""
    occ = orc.slot_pos >= 0                                  # [B,H,K]
    for name, ref in (("cache_k", orc.Kc), ("cache_v", orc.Vc)):
        with np.errstate(invalid="ignore"):                 # free slots may hold any bits
            got = snap[name].astype(np.float64)              # [L,B,H,K,d]
        for l in range(w.L):
            g, r = got[l][occ], ref[l][occ]                  # [rows, d]
            if w.dtype == "bf16":
                ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(r), 1e-30))) - 7)
                one = ulp * 1.0001 + 2e-5 * np.abs(r).max()
                if w.rope_base > 0 and name == "cache_k":
                    row_ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(r).max(axis=-1, keepdims=True), 1e-30))) - 7)
                    assert np.all(np.abs(g - r) <= one + 1.5 * row_ulp), name
                    assert (np.abs(g - r) > one).mean() <= 0.01, name
                else:
                    assert np.all(np.abs(g - r) <= one), name
            else:
                assert np.all(np.abs(g - r) <= 2e-6 * np.maximum(np.abs(r).max(), 1e-30)), name


# ---------------------------------------------------------------------------------------------
# rebuild forward through the layer stack
# ---------------------------------------------------------------------------------------------
def forward_tol(w: Workload) -> float:
    """Bound on |got - want| / max|want| per output row of the forward.  Every row of q, k, v, the attention
    output and x' is rounded once to bf16 on both sides; the GPU accumulates in fp32 (and carries the
    probabilities with 16 bits), the oracle in fp64, so a value near a rounding boundary may land on the
    neighbouring bf16 value.  A unit in the last place of a bf16 value v is 2^-7 of v at the bottom of its binade
    and 2^-8 of v at the top (8 significant bits), so at most 2^-7 of the row's largest entry.  Such a flip
    upstream moves an entry of x' by about one unit again, hence one unit per rounding stage that feeds the row:
    L layers and the cache rows written in earlier steps, (L + 1) * 2^-7 of the row's largest entry.  (What
    catches a systematic error is the bound on the mean error the tests put next to this one.)"""
    return (w.L + 1) * 2.0 ** -7


def forward_lockstep(w: Workload, steps: int, override=None, ordered=True):
    """adore_forward_step next to the forward oracle: identical selections (the oracle adopts the GPU's
    sigma bits after checking them), output rows within forward_tol.  Returns (worst, mean) row errors."""
    from oracle.adore_oracle import AdoreForwardOracle
    from tests.helpers import oracle_config
    inp = SyntheticInputs(w)
    wts = dict(inp.weights(), **inp.forward_weights())
    orc = AdoreForwardOracle(oracle_config(w), wts)
    st = storage_dtype(w)
    adore = Adore(adore_config(w), device_weights(w, {k: v for k, v in wts.items() if k not in ("w_q", "w_o")}), DEV)
    if not ordered:
        adore.set_input_order(False)
    wq, wo = to_dev(wts["w_q"], st), to_dev(wts["w_o"], st)
    E = inp.hidden_store_layer(0)
    Ed = to_dev(E, st)
    pk, pv = inp.prompt_kv()
    ov0 = None if override is None else to_dev(override[:, :w.S], torch.float32)
    adore.init_cache(to_dev(pk, st), to_dev(pv, st), None, Ed[:, :w.S].contiguous(), ov0, w.S)
    state = adore.empty_state()
    adore.get_state(slot_pos=state["slot_pos"], scores=state["scores"])
    torch.cuda.synchronize()
    gpu_scores = state["scores"][:, :w.S].cpu().numpy()
    orc.init_cache(pk, pv, None, E[:, :w.S], w.S, score_override=None if override is None else override[:, :w.S])
    assert np.abs(gpu_scores.astype(np.float64) - orc.score[:, :w.S].astype(np.float64)).max() < 1e-5
    if override is None and not np.array_equal(gpu_scores, orc.score[:, :w.S]):
        orc.init_cache(pk, pv, None, E[:, :w.S], w.S, score_override=gpu_scores)
    assert np.array_equal(state["slot_pos"].cpu().numpy(), orc.slot_pos), "slot map after init"
    rows = torch.zeros((w.B, w.R + 1, w.D), dtype=st, device=DEV)
    slot_map = torch.empty((w.B, w.H, w.K), dtype=torch.int32, device=DEV)
    released = torch.empty((w.B, w.H, w.R + 1), dtype=torch.int32, device=DEV)
    rebuilt = torch.empty((w.B, max(w.R, 1)), dtype=torch.int32, device=DEV)
    worst, mean = 0.0, 0.0
    for t in range(steps):
        n = w.S + t
        npend = [len(p) for p in orc.pending]
        ov = None if override is None else to_dev(np.asarray(override[:, n], dtype=np.float32), torch.float32)
        if not ordered:
            torch.cuda.synchronize()
        adore.forward_step(wq, wo, Ed, ov, rows, slot_map, released, rebuilt)
        adore.get_state(scores=state["scores"])
        torch.cuda.synchronize()
        sc = state["scores"]
        score_g = sc[:, :n + 1].cpu().numpy() if w.rescore else sc[:, n].cpu().numpy()
        x_o, rows_o, map_o, rel_o, rb_o, own = orc.forward_step(E, score_override=score_g)
        if w.rescore:     # every score of this step: the oracle's own values against the GPU's, then adopted
            assert np.abs(orc.own_scores - score_g.astype(np.float64)).max() < 1e-5, f"sigma at n={n}"
        elif override is None:
            assert np.abs(own - score_g.astype(np.float64)).max() < 1e-5, f"sigma at n={n}"
        assert np.array_equal(slot_map.cpu().numpy(), map_o), f"slot map at n={n}"
        assert np.array_equal(released.cpu().numpy(), rel_o), f"released at n={n}"
        assert np.array_equal(rebuilt.cpu().numpy()[:, :w.R], rb_o), f"rebuilt at n={n}"
        got = rows.float().cpu().numpy().astype(np.float64)
        for b in range(w.B):
            used = list(range(npend[b])) + [w.R]
            g, want = got[b, used], rows_o[b, used]
            assert np.isfinite(g).all(), f"output rows at n={n}"
            err = np.abs(g - want).max(axis=-1) / np.abs(want).max(axis=-1)
            assert err.max() < forward_tol(w), f"output rows at n={n}, b={b}: {err.max()}"
            worst = max(worst, float(err.max()))
            mean = max(mean, float(np.abs(g - want).mean() / np.abs(want).max()))
    adore.close()
    return worst, mean
