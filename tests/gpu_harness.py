"""Runs the HIP path (through the C-ABI binding) next to the oracle on the same seeded inputs."""
import numpy as np
import torch

from gen import SyntheticInputs, Workload
from gen.gpu_job import DEV, GpuJob, adore_config, device_weights, storage_dtype, to_dev
from paper_2407_02328_amd import Adore, make_config
from tests.helpers import make_oracle


def row_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max over rows of  max|got - want| / max|want|  (rows = last axis)."""
    num = np.abs(got - want).max(axis=-1)
    den = np.abs(want).max(axis=-1)
    return float((num / np.maximum(den, 1e-30)).max())


def out_tol(w: Workload) -> float:
    return 2e-3 if w.dtype == "bf16" else 1e-5


def lockstep(w: Workload, steps: int, override=None, check_cache_every=0, wts=None, whole=None, ordered=True):
    """Free-running GPU trajectory with the oracle in lockstep.  whole: None = every step through attend /
    schedule / rebuild; otherwise a function of the step index that says which steps go through
    adore_decode_step (released and rebuilt positions are then checked through the slot map only).

    Each step the oracle computes its own sigma_n, which must agree with the GPU's to 1e-5; it then
    adopts the GPU's bits so that both sides select from identical keys.  Slot maps, released and
    rebuilt positions must be identical; outputs within the storage type's tolerance.
    The rows a step rebuilds are handled like sigma: checked against the oracle's own (one unit of the storage
    type, see check_cache_rows), then adopted, so that the next step's attention reads identical rows on both
    sides and every output row of every step has to meet the tolerance the benchmark spec states, at every size.
    ordered: True / False = the context's input order for the whole run; a function of the step index
    switches it from step to step (inputs are then complete at every call).
    """
    orc, inp, wts = make_oracle(w, wts)
    job = GpuJob(w, inp, wts, ordered=ordered if isinstance(ordered, bool) else False)
    hs = job.hidden_np
    pk, pv = job.prompt_np
    job.init(None if override is None else override[:, :w.S])
    snap = job.snapshot()
    # init: the oracle adopts the GPU's prompt scores after checking them
    rb0 = orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S,
                         score_override=None if override is None else override[:, :w.S])
    gpu_scores = snap["scores"][:, :w.S]
    assert np.abs(gpu_scores.astype(np.float64) - orc.score[:, :w.S].astype(np.float64)).max() < 1e-5
    if override is None and not np.array_equal(gpu_scores, orc.score[:, :w.S]):
        rb0 = orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S, score_override=gpu_scores)
    assert np.array_equal(snap["slot_pos"], orc.slot_pos), "slot map after init"
    compare_cache(w, snap, orc)
    adopt_rebuilt_rows(w, orc, job.state["cache_k"], job.state["cache_v"], rb0)
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
        assert err < out_tol(w), f"attention output at n={n}: {err}"
        adopt_rebuilt_rows(w, orc, job.state["cache_k"], job.state["cache_v"], rebuilt_lists(rb_o))
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
    rb0 = orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S)
    gpu_scores = snap["scores"][:, :w.S]
    assert np.abs(gpu_scores.astype(np.float64) - orc.score[:, :w.S].astype(np.float64)).max() < 1e-5
    if not np.array_equal(gpu_scores, orc.score[:, :w.S]):
        rb0 = orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S, score_override=gpu_scores)
    assert np.array_equal(snap["slot_pos"], orc.slot_pos), "slot map after init"
    compare_cache(ws, snap, orc)
    adopt_rebuilt_rows(ws, orc, job.state["cache_k"], job.state["cache_v"], rb0, seqs)
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
        adopt_rebuilt_rows(ws, orc, job.state["cache_k"], job.state["cache_v"], rebuilt_lists(rb_o), seqs)
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
    rb0 = orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S)
    gpu_scores = snap["scores"][:, :w.S]
    assert np.abs(gpu_scores.astype(np.float64) - orc.score[:, :w.S].astype(np.float64)).max() < 1e-5
    if not np.array_equal(gpu_scores, orc.score[:, :w.S]):
        rb0 = orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S, score_override=gpu_scores)
    assert np.array_equal(snap["slot_pos"], orc.slot_pos), "slot map after init"
    compare_cache(ws, snap, orc)
    adopt_rebuilt_rows(ws, orc, state["cache_k"], state["cache_v"], rb0, seqs)
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
        adore.get_state(scores=state["scores"], cache_k=state["cache_k"], cache_v=state["cache_v"])
        torch.cuda.synchronize()
        score_g = state["scores"][:, n].cpu().numpy()
        out_o, map_o, rel_o, rb_o, own = orc.decode_step(q[:, seqs], k[:, seqs], v[:, seqs], hs, hs[0][:, n],
                                                         score_override=score_g[seqs])
        assert np.abs(own - score_g[seqs].astype(np.float64)).max() < 1e-5, f"sigma at n={n}"
        assert np.array_equal(slot_map.cpu().numpy()[seqs], map_o), f"slot map at n={n}"
        assert np.array_equal(released.cpu().numpy()[seqs], rel_o), f"released at n={n}"
        assert np.array_equal(rebuilt.cpu().numpy()[seqs][:, :w.R], rb_o), f"rebuilt at n={n}"
        err = row_rel_err(out.cpu().numpy().astype(np.float64)[:, seqs], out_o)
        worst = max(worst, err)
        assert err < out_tol(w), f"attention output at n={n}: {err}"
        adopt_rebuilt_rows(ws, orc, state["cache_k"], state["cache_v"], rebuilt_lists(rb_o), seqs)
    compare_cache(ws, sampled_state(), orc)
    adore.close()
    return worst


def check_cache_rows(w: Workload, name: str, g: np.ndarray, r: np.ndarray):
    """Cache rows [rows, d] of the GPU (g) against the oracle's (r): inserted rows are copies (exact);
    rebuilt rows are fp32-accumulated and rounded once, so a value may land on the neighbouring
    storage value (one unit in the last place); entries that cancel to almost zero additionally
    carry the fp32 accumulation error itself, bounded here by 2e-5 of the largest entry.
    With the rotary embedding a key row is the rotation of the rounded projection: where the projection landed
    on the neighbouring storage value, the rotation spreads that unit over the two entries of a plane (at most
    sqrt(2) of it, measured at the row's largest entry) before the second rounding adds its own; such rows are
    rare, so all but 1 % of the entries still have to be within one unit."""
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


def compare_cache(w: Workload, snap, orc):
    """Every occupied row of the GPU cache against the oracle's (check_cache_rows)."""
    occ = orc.slot_pos >= 0                                  # [B,H,K]
    for name, ref in (("cache_k", orc.Kc), ("cache_v", orc.Vc)):
        with np.errstate(invalid="ignore"):                 # free slots may hold any bits
            got = snap[name].astype(np.float64)              # [L,B,H,K,d]
        for l in range(w.L):
            check_cache_rows(w, name, got[l][occ], ref[l][occ])


def rebuilt_lists(rebuilt_pos: np.ndarray):
    """[B][R] positions padded with -1 -> per sequence the list of the positions chosen, best first."""
    return [[int(p) for p in row if p >= 0] for row in rebuilt_pos]


def adopt_rebuilt_rows(w: Workload, orc, cache_k: torch.Tensor, cache_v: torch.Tensor, rebuilt, seqs=None):
    """The K/V rows a step (or the init) has just rebuilt: the GPU's rows are checked against the oracle's own
    (check_cache_rows: one unit of the storage type, fp32 against fp64 accumulation) and then replace them in the
    oracle's cache, as the GPU's sigma bits replace the oracle's once they have been checked.  From here on both
    sides attend over identical rows, so an output row shows the attention's own error and nothing else.
    cache_k, cache_v: device copies [L][B][H][K][d] of the GPU's caches after the step; rebuilt: per oracle
    sequence the positions just rebuilt; seqs: the GPU's sequences the oracle follows (default: all)."""
    c = orc.cfg
    r = max(len(x) for x in rebuilt)
    if r == 0:
        return
    # (sequences may have chosen different numbers of tokens where the heads decide for themselves: the lists are
    # padded with their own first entry, which is then checked and adopted twice)
    slots = np.empty((c.B, c.H, r), dtype=np.int64)
    for b in range(c.B):
        lst = list(rebuilt[b]) + [rebuilt[b][0]] * (r - len(rebuilt[b])) if rebuilt[b] else None
        for h in range(c.H):
            slot_of = {int(p): k for k, p in enumerate(orc.slot_pos[b, h]) if p >= 0}
            slots[b, h] = [slot_of[p] for p in lst] if lst else int(np.nonzero(orc.slot_pos[b, h] >= 0)[0][0])
    idx = torch.from_numpy(slots).to(cache_k.device)[None, :, :, :, None].expand(c.L, -1, -1, -1, c.d)
    at = slots[None, :, :, :, None]
    for name, dev, ref in (("cache_k", cache_k, orc.Kc), ("cache_v", cache_v, orc.Vc)):
        sub = dev if seqs is None else dev[:, list(seqs)]    # [L, B of the oracle, H, K, d]
        rows = torch.gather(sub, 3, idx).float().cpu().numpy().astype(np.float64)   # [L, B, H, r, d]
        want = np.take_along_axis(ref, at, axis=3)
        for l in range(c.L):
            check_cache_rows(w, name, rows[l].reshape(-1, c.d), want[l].reshape(-1, c.d))
        np.put_along_axis(ref, at, rows, axis=3)


# ---------------------------------------------------------------------------------------------
# H2O(Rebuilt): scores = the attention each head has given a token so far
# ---------------------------------------------------------------------------------------------
def h2o_score_check(own: np.ndarray, got: np.ndarray, what: str):
    """The GPU's accumulated scores against the oracle's: the oracle adds this step's fp64 probability to the fp32
    score both sides started the step from; the GPU adds its fp32 probability in fp32.  So: the softmax's own error
    (1e-5, as for sigma) plus one fp32 rounding of the sum (2^-23 of it; scores grow with the steps)."""
    err = np.abs(own - got.astype(np.float64))
    assert np.all(err <= 1e-5 + 2.0 ** -22 * np.abs(own)), f"{what}: {err.max()}"


def h2o_lockstep(w: Workload, steps: int, score_init=None, whole=None, check_cache_every=0, zero_queries=False):
    """The H2O score mode next to its oracle: after every step the GPU's scores [B,H,n+1] are checked against the
    oracle's own and adopted, then slot maps (one per head), released and rebuilt positions must be identical, outputs
    within the attention tolerance; rebuilt rows are checked and adopted as in lockstep.
    Returns (worst output error, job, oracle, number of steps at which two heads of a sequence held different tokens)."""
    from oracle.adore_oracle import AdoreH2OOracle
    from tests.helpers import oracle_config
    assert w.h2o and w.L == 1
    inp = SyntheticInputs(w)
    wts = inp.weights()
    orc = AdoreH2OOracle(oracle_config(w), wts)
    job = GpuJob(w, inp, wts)
    hs = job.hidden_np
    pk, pv = job.prompt_np
    job.init(score_init)
    snap = job.snapshot()
    rb0 = orc.init_cache(pk, pv, hs, w.S, score_init=score_init)
    assert np.array_equal(snap["scores"][:, :, :w.S], orc.hscore[:, :, :w.S])
    assert np.array_equal(snap["slot_pos"], orc.slot_pos), "slot map after init"
    compare_cache(w, snap, orc)
    adopt_rebuilt_rows(w, orc, job.state["cache_k"], job.state["cache_v"], rb0)
    worst, differ = 0.0, 0
    for t in range(steps):
        n = w.S + t
        q, k, v = inp.step_qkv(n)
        if zero_queries:
            q = np.zeros_like(q)
        one_call = whole is not None and bool(whole(t))
        out_g, map_g, rel_g, rb_g, score_g = job.step(n, (q, k, v), whole=one_call)
        out_o, map_o, rel_o, rb_o = orc.decode_step(q, k, v, hs, score_override=score_g)
        h2o_score_check(orc.own_scores, score_g, f"scores at n={n}")
        assert np.array_equal(map_g, map_o), f"slot map at n={n}"
        if not one_call:
            assert np.array_equal(rel_g, rel_o), f"released at n={n}"
            assert np.array_equal(rb_g, rb_o), f"rebuilt at n={n}"
        err = row_rel_err(out_g, out_o)
        worst = max(worst, err)
        assert err < out_tol(w), f"attention output at n={n}: {err}"
        adopt_rebuilt_rows(w, orc, job.state["cache_k"], job.state["cache_v"], rebuilt_lists(rb_o))
        differ += any(set(map_o[b, h][map_o[b, h] >= 0]) != set(map_o[b, 0][map_o[b, 0] >= 0])
                      for b in range(w.B) for h in range(1, w.H))
        if check_cache_every and (t + 1) % check_cache_every == 0:
            compare_cache(w, job.snapshot(), orc)
    return worst, job, orc, differ


# ---------------------------------------------------------------------------------------------
# rebuild forward through the layer stack
# ---------------------------------------------------------------------------------------------
def forward_row_check(w: Workload, got: np.ndarray, want: np.ndarray, what: str) -> float:
    """Rows [rows, D] leaving one layer of the rebuild forward: the GPU's against the oracle's, both computed from
    the same rows entering the layer and the same K/V rows (forward_lockstep hands the GPU's to the oracle layer
    by layer).  x' = round(x + W_o round(o)): the attention's own tolerance (2e-3 of a row's largest entry, as for
    the decode step; the output projection keeps norms, so it carries over to x'), and the one rounding of x'
    itself, which may land on the neighbouring storage value (fp32 against fp64 accumulation): every entry within
    one unit of its own last place plus 2e-3 of the row's largest entry.  Returns the largest row error
    max|got - want| / max|want| for the report."""
    assert np.isfinite(got).all(), what
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - (7 if w.dtype == "bf16" else 23))
    top = np.abs(want).max(axis=-1, keepdims=True)
    bad = np.abs(got - want) > ulp * 1.0001 + out_tol(w) * top
    assert not bad.any(), f"{what}: {int(bad.sum())} entries, worst {float((np.abs(got - want) / top).max()):.3e} of the row maximum"
    return float((np.abs(got - want).max(axis=-1) / top[..., 0]).max())


def forward_lockstep(w: Workload, steps: int, override=None, ordered=True):
    """adore_forward_step next to the forward oracle: identical selections (the oracle adopts the GPU's
    sigma bits after checking them), and, layer by layer, the K/V rows the step writes (check_cache_rows) and the
    rows leaving the layer (forward_row_check) against the oracle's own, which then takes the GPU's over, so that
    every layer is compared on identical inputs and no bound grows with the depth.
    Returns (worst, mean) row errors over all layers."""
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
    layer_rows = torch.zeros((w.L, w.B, w.R + 1, w.D), dtype=st, device=DEV)
    slot_map = torch.empty((w.B, w.H, w.K), dtype=torch.int32, device=DEV)
    released = torch.empty((w.B, w.H, w.R + 1), dtype=torch.int32, device=DEV)
    rebuilt = torch.empty((w.B, max(w.R, 1)), dtype=torch.int32, device=DEV)
    worst, mean = 0.0, 0.0
    for t in range(steps):
        n = w.S + t
        npend = [len(p) for p in orc.pending]
        assert len(set(npend)) == 1
        r = npend[0]
        used = list(range(r)) + [w.R]                     # where the step's rows sit in [R+1]-row arrays
        # the slots of the step's rows: the tokens chosen by the step before, and the lowest free slot for token n
        slots = np.zeros((w.B, w.H, w.R + 1), dtype=np.int64)
        for b in range(w.B):
            for h in range(w.H):
                slot_of = {int(p): k for k, p in enumerate(orc.slot_pos[b, h]) if p >= 0}
                slots[b, h, used] = [slot_of[p] for p in orc.pending[b]] + [int(np.nonzero(orc.slot_pos[b, h] < 0)[0][0])]
        ov = None if override is None else to_dev(np.asarray(override[:, n], dtype=np.float32), torch.float32)
        if not ordered:
            torch.cuda.synchronize()
        adore.forward_step(wq, wo, Ed, ov, rows, slot_map, released, rebuilt, layer_rows=layer_rows)
        adore.get_state(scores=state["scores"], cache_k=state["cache_k"], cache_v=state["cache_v"])
        torch.cuda.synchronize()
        sc = state["scores"]
        score_g = sc[:, :n + 1].cpu().numpy() if w.rescore else sc[:, n].cpu().numpy()
        idx = torch.from_numpy(slots).to(DEV)[None, :, :, :, None].expand(w.L, -1, -1, -1, w.d)
        adopt = dict(x=layer_rows.float().cpu().numpy().astype(np.float64),
                     k=torch.gather(state["cache_k"], 3, idx).float().cpu().numpy().astype(np.float64),
                     v=torch.gather(state["cache_v"], 3, idx).float().cpu().numpy().astype(np.float64))
        x_o, rows_o, map_o, rel_o, rb_o, own = orc.forward_step(E, score_override=score_g, adopt=adopt)
        if w.rescore:     # every score of this step: the oracle's own values against the GPU's, then adopted
            assert np.abs(orc.own_scores - score_g.astype(np.float64)).max() < 1e-5, f"sigma at n={n}"
        elif override is None:
            assert np.abs(own - score_g.astype(np.float64)).max() < 1e-5, f"sigma at n={n}"
        assert np.array_equal(slot_map.cpu().numpy(), map_o), f"slot map at n={n}"
        assert np.array_equal(released.cpu().numpy(), rel_o), f"released at n={n}"
        assert np.array_equal(rebuilt.cpu().numpy()[:, :w.R], rb_o), f"rebuilt at n={n}"
        assert torch.equal(layer_rows[w.L - 1][:, used], rows[:, used]), "the last layer's rows in both outputs"
        for l in range(w.L):
            for name in ("k", "v"):
                check_cache_rows(w, "cache_" + name, adopt[name][l][:, :, used].reshape(-1, w.d),
                                 orc.own[name][l][:, :, used].reshape(-1, w.d))
            g, want = adopt["x"][l][:, used].reshape(-1, w.D), orc.own["x"][l][:, used].reshape(-1, w.D)
            worst = max(worst, forward_row_check(w, g, want, f"rows leaving layer {l} at n={n}"))
            mean = max(mean, float(np.abs(g - want).mean() / np.abs(want).max()))
    adore.close()
    return worst, mean
