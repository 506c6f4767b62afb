"""Pins for the CPU oracle: each checks it against something other than itself.

Library routines (torch CPU GRUCell / Linear / matmul, scipy softmax), closed
forms, brute force over subsets, invariants, a hand-worked trajectory.  None of
these touches the GPU.
"""
import itertools
import os

import numpy as np
import pytest
import scipy.special
import torch

from gen import SyntheticInputs, Workload
from oracle import adore_oracle as O
from tests.helpers import GOLDEN, make_oracle, oracle_config, parse_trajectory, small_workload


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------
def test_round_bf16_matches_torch_on_fp32_values():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float64).numpy()
    got = O.round_to_storage(a.astype(np.float64), "bf16")
    assert np.array_equal(got, want)


def test_round_bf16_ties_and_single_rounding():
    ulp = 2.0 ** -7                      # bf16 spacing in [1, 2)
    cases = {
        1.0 + ulp / 2: 1.0,              # tie -> even significand
        1.0 + 3 * ulp / 2: 1.0 + 2 * ulp,
        1.0 + ulp / 2 + 2.0 ** -30: 1.0 + ulp,   # just above the tie: a detour through fp32 would give 1.0
        -(1.0 + ulp / 2): -1.0,
        0.0: 0.0,
        3.0e-39: 3.0e-39 if False else None,     # subnormal range: checked below
    }
    for a, want in cases.items():
        if want is None:
            continue
        assert O.round_to_storage(np.array([a]), "bf16")[0] == want
    # subnormal spacing of bf16 is 2**-133
    sub = O.round_to_storage(np.array([3.0e-39]), "bf16")[0]
    assert sub == np.rint(3.0e-39 / 2.0 ** -133) * 2.0 ** -133


def test_round_f32_is_numpy_cast():
    a = np.random.default_rng(1).standard_normal(1000)
    assert np.array_equal(O.round_to_storage(a, "f32"), a.astype(np.float32).astype(np.float64))


# --------------------------------------------------------------------------
# attention (Sec. 2.1, Eq. 1)
# --------------------------------------------------------------------------
def test_softmax_rows_sum_to_one_and_shift_invariance():
    rng = np.random.default_rng(2)
    for rows in (1, 2, 7, 64, 513):
        q = rng.standard_normal(32)
        Km = rng.standard_normal((rows, 32)) * 3.0
        Vm = rng.standard_normal((rows, 32))
        out, p = O.attention_row(q, Km, Vm)
        assert abs(p.sum() - 1.0) < 1e-12
        assert np.all(p >= 0)
        # library softmax on the same logits
        want_p = scipy.special.softmax(Km @ q / np.sqrt(32.0))
        np.testing.assert_allclose(p, want_p, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(out, want_p @ Vm, rtol=1e-12, atol=1e-14)
        # adding a constant to every logit (a key component along q) leaves the output unchanged
        shift = 5.0 * q / (q @ q) * np.sqrt(32.0)
        out2, _ = O.attention_row(q, Km + shift[None, :], Vm)
        np.testing.assert_allclose(out2, out, rtol=1e-9, atol=1e-12)


def test_single_row_attention_returns_that_value_row():
    rng = np.random.default_rng(3)
    q, k, v = rng.standard_normal(16), rng.standard_normal((1, 16)), rng.standard_normal((1, 16))
    out, p = O.attention_row(q, k, v)
    assert p[0] == 1.0 and np.array_equal(out, v[0])


def test_scale_uses_head_dim():
    # with q = k = ones(d) the logit is d / sqrt(d) = sqrt(d); two rows, second key zero
    d = 64
    q = np.ones(d)
    Km = np.stack([np.ones(d), np.zeros(d)])
    Vm = np.stack([np.ones(d), -np.ones(d)])
    out, p = O.attention_row(q, Km, Vm)
    want_p0 = 1.0 / (1.0 + np.exp(-np.sqrt(d)))
    assert abs(p[0] - want_p0) < 1e-15


def test_slicing_matrix_identity():
    """Sec. 2.4: S_j K equals K with row j removed, so a release is just a dropped row."""
    rng = np.random.default_rng(4)
    Km = rng.standard_normal((9, 5))
    for j in range(9):
        assert np.array_equal(O.slice_rows_by_matmul(Km, j), np.delete(Km, j, axis=0))


# --------------------------------------------------------------------------
# controller (Sec. 2.2, Eq. 2)
# --------------------------------------------------------------------------
def test_gru_cell_matches_torch_grucell():
    torch.manual_seed(0)
    D, dp = 48, 12
    cell = torch.nn.GRUCell(D, dp).double()
    x = torch.randn(5, D, dtype=torch.float64)
    h = torch.randn(5, dp, dtype=torch.float64)
    want = cell(x, h).detach().numpy()
    W_ih, W_hh = cell.weight_ih.detach().numpy(), cell.weight_hh.detach().numpy()
    b_ih, b_hh = cell.bias_ih.detach().numpy(), cell.bias_hh.detach().numpy()
    for i in range(5):
        got = O.gru_cell(x[i].numpy(), h[i].numpy(), W_ih, W_hh, b_ih, b_hh)
        np.testing.assert_allclose(got, want[i], rtol=1e-12, atol=1e-13)


def test_gru_sequence_matches_torch_gru_from_zero_state():
    torch.manual_seed(1)
    D, dp, S = 20, 6, 9
    gru = torch.nn.GRU(D, dp, num_layers=1, batch_first=True, bidirectional=False).double()
    xs = torch.randn(1, S, D, dtype=torch.float64)
    want, _ = gru(xs)
    h = np.zeros(dp)
    for i in range(S):
        h = O.gru_cell(xs[0, i].numpy(), h, gru.weight_ih_l0.detach().numpy(),
                       gru.weight_hh_l0.detach().numpy(), gru.bias_ih_l0.detach().numpy(),
                       gru.bias_hh_l0.detach().numpy())
        np.testing.assert_allclose(h, want[0, i].detach().numpy(), rtol=1e-11, atol=1e-12)


def test_keep_probability_matches_torch_layers():
    torch.manual_seed(2)
    dp = 10
    pos = torch.nn.Linear(1, dp).double()
    inter = torch.nn.Linear(dp, dp).double()
    outl = torch.nn.Linear(dp, 1).double()
    z = torch.randn(dp, dtype=torch.float64)
    for delta in (0.0, 0.25, 3.0):
        want = torch.sigmoid(outl(torch.tanh(inter(pos(torch.tensor([delta], dtype=torch.float64)) + z))))
        wts = dict(pos_w=pos.weight.detach().numpy()[:, 0], pos_b=pos.bias.detach().numpy(),
                   mlp_w1=inter.weight.detach().numpy(), mlp_b1=inter.bias.detach().numpy(),
                   out_w=outl.weight.detach().numpy()[0], out_b=outl.bias.detach().numpy())
        got = O.keep_probability(z.numpy(), delta, wts)
        assert abs(got - want.item()) < 1e-14


def test_oracle_scores_follow_gru_then_mlp_over_a_prompt():
    """The stateful path feeds positions i * pos_scale and carries z across tokens."""
    w = small_workload(B=1, S=7, T=2)
    orc, inp, wts = make_oracle(w)
    hs = inp.hidden_store()
    pk, pv = inp.prompt_kv()
    orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S)
    cell = torch.nn.GRUCell(w.D, w.dprime).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(wts["gru_w_ih"].astype(np.float64)))
        cell.weight_hh.copy_(torch.from_numpy(wts["gru_w_hh"].astype(np.float64)))
        cell.bias_ih.copy_(torch.from_numpy(wts["gru_b_ih"].astype(np.float64)))
        cell.bias_hh.copy_(torch.from_numpy(wts["gru_b_hh"].astype(np.float64)))
        h = torch.zeros(1, w.dprime, dtype=torch.float64)
        for i in range(w.S):
            h = cell(torch.from_numpy(hs[0][0, i].astype(np.float64))[None], h)
            p = torch.from_numpy(wts["pos_w"].astype(np.float64)) * (i * w.pos_scale) + \
                torch.from_numpy(wts["pos_b"].astype(np.float64))
            u = torch.tanh(torch.from_numpy(wts["mlp_w1"].astype(np.float64)) @ (p + h[0]) +
                           torch.from_numpy(wts["mlp_b1"].astype(np.float64)))
            s = torch.sigmoid(torch.from_numpy(wts["out_w"].astype(np.float64)) @ u + float(wts["out_b"][0]))
            assert abs(float(orc.score[0, i]) - s.item()) < 1e-6     # score is stored as fp32
    np.testing.assert_allclose(orc.z[0], h[0].numpy(), rtol=1e-11, atol=1e-12)


# --------------------------------------------------------------------------
# selections (Sec. 2.2 release, Sec. 2.3 rebuild choice): brute force
# --------------------------------------------------------------------------
def _better(i, j, score):
    """i ranks above j."""
    return score[i] > score[j] or (score[i] == score[j] and i < j)


def test_release_is_the_unique_lowest_set_by_brute_force():
    rng = np.random.default_rng(5)
    K = 8
    for trial in range(150):
        npos = 14
        score = rng.choice(np.array([0.1, 0.3, 0.3, 0.5, 0.7, 0.7, 0.9], dtype=np.float32), npos)
        occ = rng.integers(3, K + 1)
        slots = rng.permutation(K)[:occ]
        positions = rng.permutation(npos)[:occ]
        slot_pos = np.full(K, -1, dtype=np.int32)
        slot_pos[slots] = positions
        current = int(positions[rng.integers(occ)])
        m = int(rng.integers(1, occ + 1))
        got = O.release_lowest(slot_pos, score, current, m)
        x = max(0, occ - m)
        assert len(got) == x and got == sorted(got)
        cands = [int(s) for s in slots if slot_pos[s] != current]
        # exactly one subset of size x has every member ranked below every non-member
        hits = []
        for sub in itertools.combinations(sorted(cands), x):
            rest = [s for s in cands if s not in sub]
            if all(_better(slot_pos[r], slot_pos[s], score) for s in sub for r in rest):
                hits.append(list(sub))
        assert hits == [got]


def test_rebuild_choice_by_brute_force():
    rng = np.random.default_rng(6)
    for trial in range(150):
        n = int(rng.integers(3, 11))
        score = rng.choice(np.array([0.2, 0.4, 0.4, 0.6, 0.8], dtype=np.float32), n + 1)
        resident = list(rng.permutation(n + 1)[:rng.integers(1, n + 1)])
        R = int(rng.integers(0, 5))
        got = O.rebuild_choice(resident, n, score, R)
        pool = [p for p in range(n + 1) if p not in resident]
        r = min(R, len(pool))
        assert len(got) == r and set(got) <= set(pool)
        # best first, and nothing left in the pool beats a chosen token
        for a, b in zip(got, got[1:]):
            assert _better(a, b, score)
        for p in pool:
            if p not in got:
                assert all(_better(g, p, score) for g in got)


# --------------------------------------------------------------------------
# whole path
# --------------------------------------------------------------------------
def _run(orc, inp, w, steps, override=None, collect=None):
    hs = inp.hidden_store()
    pk, pv = inp.prompt_kv()
    orc.init_cache(pk, pv, hs, hs[0][:, :w.S], w.S,
                   score_override=None if override is None else override[:, :w.S])
    outs = []
    for t in range(steps):
        n = w.S + t
        q, k, v = inp.step_qkv(n)
        res = orc.decode_step(q, k, v, hs, hs[0][:, n], None if override is None else override[:, n])
        outs.append(res)
        if collect is not None:
            collect(n, res)
    return outs, hs, pk, pv


@pytest.mark.parametrize("name,K,R", [("slot_trajectory_K4_R1.txt", 4, 1), ("slot_trajectory_K7_R3.txt", 7, 3)])
def test_hand_worked_trajectory(name, K, R):
    """Slot maps worked out by hand from the rules.  The second file rebuilds three tokens per step into free
    slots that are not neighbours, so the order in which the ranks take the free slots (rank rho -> rho-th
    lowest free slot) decides every line of it."""
    init_scores, after_init, steps = parse_trajectory(os.path.join(GOLDEN, name))
    S = len(init_scores)
    w = Workload("golden", L=1, B=1, H=2, d=4, D=8, K=K, R=R, S=S, T=len(steps), dtype="f32", dprime=4)
    orc, inp, _ = make_oracle(w)
    hs = inp.hidden_store()
    pk, pv = inp.prompt_kv()
    rb = orc.init_cache(pk, pv, hs, hs[0][:, :S], S, score_override=init_scores[None, :])
    for h in range(w.H):
        assert orc.slot_pos[0, h].tolist() == after_init["slot_map"]
    assert rb[0] == after_init["rebuilt"]
    for st in steps:
        q, k, v = inp.step_qkv(st["n"])
        out, slot_map, released, rebuilt, _ = orc.decode_step(
            q, k, v, hs, hs[0][:, st["n"]], np.array([st["score"]], dtype=np.float32))
        for h in range(w.H):
            assert slot_map[0, h].tolist() == st["slot_map"], st
            assert released[0, h].tolist() == st["released"], st
        assert rebuilt[0].tolist() == st["rebuilt"], st


def test_no_release_when_cache_holds_everything_equals_full_attention():
    """K - R - 1 >= N_max: nothing is ever released, slot k holds position k, output = Eq. 1 over all rows."""
    for R in (0, 3):
        w = small_workload(S=6, T=10, K=6 + 10 + R + 1, R=R, H=3)
        orc, inp, _ = make_oracle(w)
        outs, hs, pk, pv = _run(orc, inp, w, w.T)
        Kall = [pk[0][:, :, i] for i in range(w.S)]
        Vall = [pv[0][:, :, i] for i in range(w.S)]
        for t, (out, slot_map, released, rebuilt, _) in enumerate(outs):
            n = w.S + t
            q, k, v = inp.step_qkv(n)
            Kall.append(k[0]); Vall.append(v[0])
            Km = np.stack(Kall, axis=2).astype(np.float64)      # [B,H,n+1,d]
            Vm = np.stack(Vall, axis=2).astype(np.float64)
            logits = np.einsum("bhd,bhnd->bhn", q[0].astype(np.float64), Km) / np.sqrt(w.d)
            want = np.einsum("bhn,bhnd->bhd", scipy.special.softmax(logits, axis=-1), Vm)
            np.testing.assert_allclose(out[0], want, rtol=1e-11, atol=1e-13)
            expect_map = np.full(w.K, -1); expect_map[:n + 1] = np.arange(n + 1)
            assert np.all(slot_map == expect_map[None, None, :])
            assert np.all(released == -1) and np.all(rebuilt == -1)


def test_static_scores_closed_form():
    """With fixed scores, after step n: persistent rows = {n} + best (m-1) of the older tokens,
    rebuilt rows = the next R in rank."""
    w = small_workload(B=2, H=2, K=12, R=3, S=20, T=24)
    rng = np.random.default_rng(7)
    override = rng.choice(np.linspace(0.05, 0.95, 13).astype(np.float32), (w.B, w.N_max))   # many ties
    orc, inp, _ = make_oracle(w)

    def check(n, res):
        out, slot_map, released, rebuilt, _ = res
        for b in range(w.B):
            older = np.arange(n)
            order = older[np.lexsort((older, -override[b, :n].astype(np.float64)))]    # best first
            persistent = set(order[:w.m - 1].tolist()) | {n}
            want_rebuilt = order[w.m - 1:w.m - 1 + w.R].tolist()
            assert rebuilt[b].tolist() == want_rebuilt
            for h in range(w.H):
                held = [int(p) for p in slot_map[b, h] if p >= 0]
                assert len(held) == len(set(held)) == w.K - 1
                assert set(held) == persistent | set(want_rebuilt)

    _run(orc, inp, w, w.T, override=override, collect=check)


def test_invariants_with_controller_scores():
    w = small_workload(B=2, H=3, K=10, R=2, S=5, T=30)
    orc, inp, _ = make_oracle(w)
    state = {"prev_occ": min(w.S, w.m) + min(w.R, w.S - min(w.S, w.m))}

    def check(n, res):
        out, slot_map, released, rebuilt, own = res
        for b in range(w.B):
            # uniform policy: every head of a sequence holds the same map
            for h in range(1, w.H):
                assert np.array_equal(slot_map[b, h], slot_map[b, 0])
                assert np.array_equal(released[b, h], released[b, 0])
            held = [int(p) for p in slot_map[b, 0] if p >= 0]
            assert len(held) == len(set(held)) <= w.K - 1          # one slot stays free
            assert n in held                                        # current token survives its step
            rb = [int(p) for p in rebuilt[b] if p >= 0]
            rel = [int(p) for p in released[b, 0] if p >= 0]
            assert set(rb) <= set(held)
            occ_before_release = state["prev_occ"] + 1
            assert occ_before_release == min(n + 1, w.K) or n < w.K
            assert len(rel) == max(0, occ_before_release - w.m)
            pool = set(range(n + 1)) - (set(held) - set(rb))
            assert len(rb) == min(w.R, len(pool))
            assert 0.0 < own[b] < 1.0 and orc.score[b, n] == np.float32(own[b])
        state["prev_occ"] = len(held)
        # attention probabilities of every row sum to one
        for (valid, p) in orc.last_probs.values():
            assert abs(p.sum() - 1.0) < 1e-12

    _run(orc, inp, w, w.T, collect=check)


# --------------------------------------------------------------------------
# rescore mode (every token scored again at every step, with its distance to the current token)
# --------------------------------------------------------------------------
def test_rescore_without_position_dependence_is_the_static_policy():
    """With a zero position layer weight the score cannot depend on the distance, so scoring every token
    again gives back the values of the static mode: both modes must walk the same trajectory.  Fails if the
    stored state z_i is off by one token, if scores land on the wrong positions, or if the selections read
    stale values."""
    w_static = small_workload(B=2, H=2, K=12, R=3, S=20, T=24)
    w_re = w_static.scaled(rescore=True)
    wts = SyntheticInputs(w_static).weights()
    wts = dict(wts, pos_w=np.zeros_like(wts["pos_w"]))
    a, inp, _ = make_oracle(w_static, wts)
    b, _, _ = make_oracle(w_re, wts)
    ra = _run(a, inp, w_static, w_static.T)[0]
    rb = _run(b, inp, w_re, w_re.T)[0]
    for (oa, ma, rla, rba, sa), (ob, mb, rlb, rbb, sb) in zip(ra, rb):
        assert np.array_equal(ma, mb) and np.array_equal(rla, rlb) and np.array_equal(rba, rbb)
        assert np.array_equal(oa, ob)
        assert np.allclose(sa, sb, rtol=0, atol=1e-15)
    assert np.array_equal(a.score, b.score)


def test_rescore_with_pure_recency_scores_is_a_sliding_window():
    """GRU weights zero (z_i = 0 for every token), identity interaction layer, positive output weights and
    a negative position weight: the score is a strictly decreasing function of the distance n - i alone,
    so the policy must keep exactly the m most recent tokens and rebuild the R before them, most recent
    first -- window attention.  Absolute positions, a flipped sign of the distance or an off-by-one in
    it all break this."""
    w = small_workload(B=2, H=2, K=12, R=3, S=20, T=24, rescore=True, pos_scale=2.0 ** -6)
    wts = SyntheticInputs(w).weights()
    dp = w.dprime
    wts = dict(wts, gru_w_ih=np.zeros_like(wts["gru_w_ih"]), gru_w_hh=np.zeros_like(wts["gru_w_hh"]),
               gru_b_ih=np.zeros_like(wts["gru_b_ih"]), gru_b_hh=np.zeros_like(wts["gru_b_hh"]),
               pos_w=np.full(dp, -1.0, dtype=np.float32), pos_b=np.zeros(dp, dtype=np.float32),
               mlp_w1=np.eye(dp, dtype=np.float32), mlp_b1=np.zeros(dp, dtype=np.float32),
               out_w=np.ones(dp, dtype=np.float32), out_b=np.zeros(1, dtype=np.float32))
    orc, inp, _ = make_oracle(w, wts)

    def check(n, res):
        out, slot_map, released, rebuilt, _ = res
        want_rebuilt = [n - w.m - j for j in range(w.R)]
        window = set(range(n - w.m + 1, n + 1))
        for b in range(w.B):
            assert rebuilt[b].tolist() == want_rebuilt
            for h in range(w.H):
                held = {int(p) for p in slot_map[b, h] if p >= 0}
                assert held == window | set(want_rebuilt)
            assert np.all(np.diff(orc.score[b, :n + 1].astype(np.float64)) > 0)     # newer = higher

    _run(orc, inp, w, w.T, collect=check)


def test_rescore_invariants_and_promotion_of_rebuilt_tokens():
    """Random controller weights in rescore mode: the counting invariants of the static mode still hold
    (one free slot, current token kept, released count, rebuilt = top of the pool by this step's scores),
    and scores do change between steps, so that a rebuilt token can stay as a resident (a promotion)."""
    w = small_workload(B=2, H=3, K=10, R=2, S=12, T=40, rescore=True, pos_scale=2.0 ** -3)
    orc, inp, _ = make_oracle(w)
    seen = {"changed": False, "promoted": False, "prev_rb": [set() for _ in range(w.B)], "prev": None}

    def check(n, res):
        out, slot_map, released, rebuilt, own = res
        for b in range(w.B):
            for h in range(1, w.H):
                assert np.array_equal(slot_map[b, h], slot_map[b, 0])
            held = [int(p) for p in slot_map[b, 0] if p >= 0]
            assert len(held) == len(set(held)) == min(n + 1, w.K - 1) and n in held
            rb = [int(p) for p in rebuilt[b] if p >= 0]
            rel = [int(p) for p in released[b, 0] if p >= 0]
            assert len(rel) == max(0, min(n + 1, w.K) - w.m)
            sc = orc.score[b, :n + 1]
            assert np.allclose(sc, orc.own_scores[b], rtol=0, atol=1e-7)
            pool = sorted(set(range(n + 1)) - (set(held) - set(rb)), key=lambda p: (-float(sc[p]), p))
            assert rb == pool[:min(w.R, len(pool))]
            persistent = set(held) - set(rb)
            if seen["prev_rb"][b] & persistent:
                seen["promoted"] = True          # rebuilt last step, resident now
            seen["prev_rb"][b] = set(rb)
        if seen["prev"] is not None and not np.array_equal(seen["prev"], orc.score[:, :n]):
            seen["changed"] = True
        seen["prev"] = orc.score[:, :n + 1].copy()

    _run(orc, inp, w, w.T, collect=check)
    assert seen["changed"] and seen["promoted"]
    # the value itself: torch layers applied to the stored GRU states (a torch GRU over the same inputs)
    # with the distance to the last token as position feature.  Catches an offset in the distance.
    wt = {k: torch.tensor(np.asarray(v, dtype=np.float64)) for k, v in orc.w64.items()}
    gru = torch.nn.GRU(w.D, w.dprime, batch_first=True).double()
    with torch.no_grad():
        gru.weight_ih_l0.copy_(wt["gru_w_ih"]); gru.weight_hh_l0.copy_(wt["gru_w_hh"])
        gru.bias_ih_l0.copy_(wt["gru_b_ih"]); gru.bias_hh_l0.copy_(wt["gru_b_hh"])
        x = torch.tensor(inp.hidden_store()[0].astype(np.float64))             # [B, N_max, D]
        z_all, _ = gru(x)
        n = w.N_max - 1
        dist = torch.tensor((n - np.arange(n + 1)).astype(np.float32) * np.float32(w.pos_scale), dtype=torch.float64)
        p = dist[:, None] * wt["pos_w"][None, :] + wt["pos_b"][None, :]       # [n+1, d']
        u = torch.tanh((p[None] + z_all[:, :n + 1]) @ wt["mlp_w1"].T + wt["mlp_b1"])
        want = torch.sigmoid(u @ wt["out_w"] + wt["out_b"][0]).numpy()
    assert np.abs(want - orc.own_scores).max() < 1e-12


# --------------------------------------------------------------------------
# rebuild forward through a layer stack (Sec. 2.3 in full)
# --------------------------------------------------------------------------
def _forward_oracle(w, wts=None):
    inp = SyntheticInputs(w)
    wts = dict(inp.weights(), **inp.forward_weights()) if wts is None else wts
    return O.AdoreForwardOracle(oracle_config(w), wts), inp, wts


def _rotate_complex(t, base):
    """Rotary embedding written with complex numbers (torch): the pair (x[j], x[j + d/2]) is the complex
    number x[j] + i x[j + d/2], multiplied by exp(i pos base^(-2j/d)).  t: [..., N, d], positions 0..N-1."""
    N, d = t.shape[-2], t.shape[-1]
    freq = torch.tensor(float(base), dtype=torch.float64) ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
    ang = torch.arange(N, dtype=torch.float64)[:, None] * freq[None, :]
    z = torch.complex(t[..., :d // 2], t[..., d // 2:]) * torch.polar(torch.ones_like(ang), ang)
    return torch.cat([z.real, z.imag], dim=-1)


def _causal_stack_reference(E, wts, w):
    """Textbook decoder stack of attention-only layers over the whole sequence, torch fp64:
    x' = x + W_o . causal_attention(W_q x, W_k x, W_v x), q and k rotated by their positions when the
    workload asks for the rotary embedding.  Returns (X_L [B,N,D], K [L,B,H,N,d], V)."""
    X = torch.tensor(E.astype(np.float64))
    B, N, _ = X.shape
    Hd = w.H * w.d
    Ks, Vs = [], []
    for l in range(w.L):
        Wq = torch.tensor(wts["w_q"][l].astype(np.float64))
        Wkv = torch.tensor(wts["w_kv"][l].astype(np.float64))
        Wo = torch.tensor(wts["w_o"][l].astype(np.float64))
        heads = lambda t: t.reshape(B, N, w.H, w.d).transpose(1, 2)       # [B,H,N,d]
        Q, K, V = heads(X @ Wq.T), heads(X @ Wkv[:Hd].T), heads(X @ Wkv[Hd:].T)
        if w.rope_base > 0:
            Q, K = _rotate_complex(Q, w.rope_base), _rotate_complex(K, w.rope_base)
        A = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True)
        X = X + A.transpose(1, 2).reshape(B, N, Hd) @ Wo.T
        Ks.append(K.numpy()); Vs.append(V.numpy())
    return X.numpy(), np.stack(Ks), np.stack(Vs)


@pytest.mark.parametrize("rope_base", [0.0, 50.0])
def test_forward_with_every_released_token_rebuilt_is_a_causal_decoder_stack(rope_base):
    """When R covers the whole pool, every token is in the cache at every step (as a resident or rebuilt), so
    the rebuild forward must give what a plain causal decoder stack gives: the output row of the current
    token, and the rows of the rebuilt tokens at their own positions.  This fixes the mask among the R+1
    query rows (a rebuilt token that saw later tokens would get another state from layer 2 on), the residual,
    the head layout of W_q / W_o, the order of the rows and the slot each K/V row lands in."""
    w = Workload("fwd", L=3, B=2, H=2, d=8, D=16, K=17, R=8, S=10, T=6, dtype="f32", dprime=8,
                 act_std=1.0, w_std=0.25, rope_base=rope_base)
    orc, inp, wts = _forward_oracle(w)
    E = inp.hidden_store_layer(0)                                         # [B, N_max, D] embeddings
    XL, Kref, Vref = _causal_stack_reference(E, wts, w)
    pk = O.round_to_storage(Kref[:, :, :, :w.S], "f32"); pv = O.round_to_storage(Vref[:, :, :, :w.S], "f32")
    orc.init_cache(pk, pv, None, E[:, :w.S], w.S)
    scale = np.abs(XL).max()
    for t in range(w.T):
        n = w.S + t
        pending = [list(p) for p in orc.pending]
        x_out, rows, slot_map, released, rebuilt, own = orc.forward_step(E)
        assert np.abs(x_out - XL[:, n]).max() < 1e-5 * scale
        for b in range(w.B):
            held = {int(p) for p in slot_map[b, 0] if p >= 0}
            assert held == set(range(n + 1))                              # nobody is missing
            for rho, pos in enumerate(pending[b]):
                assert np.abs(rows[b, rho] - XL[b, pos]).max() < 1e-5 * scale
    # and the cache rows themselves are the reference K/V of their positions, layer by layer
    for l in range(w.L):
        for b in range(w.B):
            for h in range(w.H):
                for k, pos in enumerate(orc.slot_pos[b, h]):
                    if pos >= 0 and pos not in orc.pending[b]:
                        assert np.abs(orc.Kc[l, b, h, k] - Kref[l, b, h, pos]).max() < 1e-5 * np.abs(Kref).max()
                        assert np.abs(orc.Vc[l, b, h, k] - Vref[l, b, h, pos]).max() < 1e-5 * np.abs(Vref).max()


def test_forward_without_rebuild_budget_is_the_single_query_step():
    """R = 0, one layer: the forward is the pinned single-query step with q, k, v = the projections of the
    current token's embedding, followed by the residual output projection."""
    w = small_workload(B=2, H=2, K=9, R=0, S=12, T=10, L=1)
    fwd, inp, wts = _forward_oracle(w)
    base, _, _ = make_oracle(w, wts)
    E = inp.hidden_store_layer(0)
    pk, pv = inp.prompt_kv()
    fwd.init_cache(pk, pv, None, E[:, :w.S], w.S)
    base.init_cache(pk, pv, inp.hidden_store(), E[:, :w.S], w.S)
    Hd = w.H * w.d
    Wq, Wkv, Wo = (wts[k][0].astype(np.float64) for k in ("w_q", "w_kv", "w_o"))
    for t in range(w.T):
        n = w.S + t
        x = E[:, n].astype(np.float64)
        q = O.round_to_storage(x @ Wq.T, w.dtype).reshape(1, w.B, w.H, w.d)
        kv = O.round_to_storage(x @ Wkv.T, w.dtype)
        k = kv[:, :Hd].reshape(1, w.B, w.H, w.d); v = kv[:, Hd:].reshape(1, w.B, w.H, w.d)
        out, map_b, rel_b, rb_b, own_b = base.decode_step(q, k, v, inp.hidden_store(), E[:, n])
        x_out, rows, map_f, rel_f, rb_f, own_f = fwd.forward_step(E)
        want = O.round_to_storage(x + O.round_to_storage(out[0].reshape(w.B, Hd), w.dtype) @ Wo.T, w.dtype)
        assert np.array_equal(map_b, map_f) and np.array_equal(rel_b, rel_f)
        assert np.allclose(x_out, want, rtol=0, atol=1e-12)


def test_forward_adoption_hook_leaves_the_arithmetic_alone():
    """forward_step(adopt=...) hands given per-layer rows and K/V on instead of its own.  Fed its own values
    (found pass by pass: with a guess adopted, the first pass gives the right K/V of the first layer, the second
    its rows, the third the K/V of the second layer, ...) it must return exactly what the plain step returns,
    and report those values as its own."""
    import copy
    w = Workload("fwd_adopt", L=3, B=2, H=2, d=8, D=16, K=10, R=3, S=14, T=4, dtype="bf16", dprime=8, w_std=0.25,
                 rope_base=100.0)
    orc, inp, wts = _forward_oracle(w)
    E = inp.hidden_store_layer(0)
    pk, pv = inp.prompt_kv()
    orc.init_cache(pk, pv, None, E[:, :w.S], w.S)
    for t in range(w.T):
        guess = dict(x=np.zeros((w.L, w.B, w.R + 1, w.D)), k=np.zeros((w.L, w.B, w.H, w.R + 1, w.d)),
                     v=np.zeros((w.L, w.B, w.H, w.R + 1, w.d)))
        for _ in range(2 * w.L + 1):
            twin = copy.deepcopy(orc)
            got = twin.forward_step(E, adopt=guess)
            guess = twin.own
        want = orc.forward_step(E)
        for g, r in zip(got, want):
            assert np.array_equal(g, r)
        assert np.array_equal(twin.Kc, orc.Kc) and np.array_equal(twin.Vc, orc.Vc)
        assert np.array_equal(twin.own["x"][w.L - 1], want[1])


def test_forward_invariants_with_a_small_budget():
    """R smaller than the pool: counts and residency as in the base step; the tokens rebuilt in a step are
    the ones chosen in the step before; every output is finite."""
    w = Workload("fwd2", L=2, B=2, H=3, d=8, D=16, K=10, R=2, S=14, T=12, dtype="bf16", dprime=8, w_std=0.25)
    orc, inp, wts = _forward_oracle(w)
    E = inp.hidden_store_layer(0)
    pk, pv = inp.prompt_kv()
    first = orc.init_cache(pk, pv, None, E[:, :w.S], w.S)
    prev = [list(r) for r in first]
    for t in range(w.T):
        n = w.S + t
        assert [list(p) for p in orc.pending] == prev
        x_out, rows, slot_map, released, rebuilt, own = orc.forward_step(E)
        assert np.isfinite(x_out).all()
        for b in range(w.B):
            for h in range(1, w.H):
                assert np.array_equal(slot_map[b, h], slot_map[b, 0])
            held = [int(p) for p in slot_map[b, 0] if p >= 0]
            assert len(held) == len(set(held)) == w.K - 1 and n in held
            assert np.all(rows[b, len(prev[b]):w.R] == 0)
        prev = [[int(p) for p in rebuilt[b] if p >= 0] for b in range(w.B)]


@pytest.mark.parametrize("rope_base", [0.0, 10000.0])
def test_rebuilt_rows_equal_original_rows_and_full_attention_when_everything_fits(rope_base):
    """If the supplied K/V are the projections of the hidden states (the keys turned to their positions when
    the rotary embedding is on, here by torch complex arithmetic), a rebuilt row is identical to the row that
    was released; while |pool| <= R every token is present, so the output is Eq. 1 over all tokens."""
    w = small_workload(B=1, H=2, K=12, R=5, S=4, T=7, dtype="f32", rope_base=rope_base)   # m = 6; pool <= 5 up to n = 10
    orc, inp, wts = make_oracle(w)
    hs = inp.hidden_store()
    W = wts["w_kv"][0].astype(np.float64)
    kv_all = hs[0].astype(np.float64) @ W.T                                            # [B,N,2Hd]
    Hd = w.H * w.d
    k_all = kv_all[:, :, :Hd].reshape(w.B, w.N_max, w.H, w.d).transpose(0, 2, 1, 3)    # [B,H,N,d]
    v_all = kv_all[:, :, Hd:].reshape(w.B, w.N_max, w.H, w.d).transpose(0, 2, 1, 3)
    k_all = k_all.astype(np.float32).astype(np.float64)
    v_all = v_all.astype(np.float32).astype(np.float64)
    if rope_base > 0:       # rounded projection, turned, rounded again
        k_all = _rotate_complex(torch.tensor(np.ascontiguousarray(k_all)), rope_base).numpy()
        k_all = k_all.astype(np.float32).astype(np.float64)
    orc.init_cache(k_all[None, :, :, :w.S], v_all[None, :, :, :w.S], hs, hs[0][:, :w.S], w.S)
    for n in range(w.S, w.S + w.T):
        q, _, _ = inp.step_qkv(n)
        out, slot_map, released, rebuilt, _ = orc.decode_step(
            q, k_all[None, :, :, n], v_all[None, :, :, n], hs, hs[0][:, n])
        logits = np.einsum("bhd,bhnd->bhn", q[0].astype(np.float64), k_all[:, :, :n + 1]) / np.sqrt(w.d)
        want = np.einsum("bhn,bhnd->bhd", scipy.special.softmax(logits, axis=-1), v_all[:, :, :n + 1])
        np.testing.assert_allclose(out[0], want, rtol=1e-10, atol=1e-12)
        for h in range(w.H):
            for s in range(w.K):
                p = slot_map[0, h, s]
                if p >= 0:      # with the rotation two fp64 evaluation orders meet: equal up to the fp32 rounding
                    assert np.abs(orc.Kc[0, 0, h, s] - k_all[0, h, p]).max() <= (2e-7 * np.abs(k_all).max() if rope_base else 0)
                    assert np.array_equal(orc.Vc[0, 0, h, s], v_all[0, h, p])
    assert (rebuilt >= 0).sum() == 5        # the last step did rebuild R tokens


def test_projection_matches_triple_loop_and_torch_matmul():
    w = small_workload(B=1, H=2, d=4, D=6, dtype="bf16")
    orc, inp, wts = make_oracle(w)
    x = inp.hidden_store()[0, 0, :3]
    got = orc._project(0, x, [0, 1, 2])
    W = wts["w_kv"][0]
    naive = np.zeros((3, 2 * w.H * w.d))
    for i in range(3):
        for j in range(2 * w.H * w.d):
            acc = 0.0
            for t in range(w.D):
                acc += float(x[i, t]) * float(W[j, t])
            naive[i, j] = acc
    lib = (torch.from_numpy(x.astype(np.float64)) @ torch.from_numpy(W.astype(np.float64)).T).numpy()
    np.testing.assert_allclose(naive, lib, rtol=1e-13, atol=1e-15)
    assert np.array_equal(got, O.round_to_storage(lib, "bf16"))
    # every result is a bf16 value
    assert np.array_equal(got, torch.from_numpy(got).to(torch.bfloat16).to(torch.float64).numpy())


def test_oracle_rejects_bad_budget_and_overrun():
    w = small_workload(K=4, R=3)
    with pytest.raises(ValueError):
        make_oracle(w)
    w = small_workload(S=3, T=1)
    orc, inp, _ = make_oracle(w)
    _run(orc, inp, w, 1)
    q, k, v = inp.step_qkv(w.S)
    with pytest.raises(RuntimeError):
        orc.decode_step(q, k, v, inp.hidden_store(), inp.hidden_store()[0][:, 0])


# --------------------------------------------------------------------------
# rotary position embedding (optional reading, see the oracle's header)
# --------------------------------------------------------------------------
def test_rotary_is_identity_at_position_zero_and_keeps_lengths():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((4, 3, 16))
    out = O.rotary(x, [0, 1, 7, 1000], 10000.0)
    assert np.array_equal(out[0], x[0])
    np.testing.assert_allclose(np.linalg.norm(out, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    assert np.abs(out[1:] - x[1:]).max() > 0.1


def test_rotary_in_two_dimensions_is_the_plane_rotation_by_the_position():
    x = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, -3.0]])
    out = O.rotary(x, [1, 2, 5], 77.0)                   # d = 2: one plane, frequency base^0 = 1
    for row, p, got in zip(x, [1, 2, 5], out):
        Rm = np.array([[np.cos(p), -np.sin(p)], [np.sin(p), np.cos(p)]])
        np.testing.assert_allclose(got, Rm @ row, rtol=0, atol=1e-15)


def test_rotary_matches_complex_multiplication_in_torch():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((9, 2, 3, 12))               # positions 0..8, two head axes
    want = _rotate_complex(torch.tensor(x).permute(1, 2, 0, 3), 500.0).permute(2, 0, 1, 3).numpy()
    np.testing.assert_allclose(O.rotary(x, list(range(9)), 500.0), want, rtol=0, atol=1e-14)


def test_rotary_products_depend_on_the_distance_only():
    """<rot(q, m), rot(k, n)> = <rot(q, m + s), rot(k, n + s)>: the property the embedding exists for."""
    rng = np.random.default_rng(7)
    q, k = rng.standard_normal((1, 32)), rng.standard_normal((1, 32))
    base = 10000.0
    ref = float(O.rotary(q, [9], base)[0] @ O.rotary(k, [4], base)[0])
    for s in (1, 13, 700):
        assert abs(float(O.rotary(q, [9 + s], base)[0] @ O.rotary(k, [4 + s], base)[0]) - ref) < 1e-11
    assert abs(float(O.rotary(q, [9], base)[0] @ O.rotary(k, [5], base)[0]) - ref) > 1e-3


def test_decode_oracle_rotates_only_the_rebuilt_keys():
    """Same job with and without the embedding: value rows, supplied rows and all selections are the same;
    a rebuilt key row is the unrotated projection turned to its token's position."""
    w0 = small_workload(B=1, H=2, K=10, R=3, S=12, T=6, dtype="f32")
    w1 = w0.scaled(rope_base=100.0)
    a, inp, wts = make_oracle(w0)
    b, _, _ = make_oracle(w1, wts)
    pk, pv = inp.prompt_kv()
    hs = inp.hidden_store()
    for o in (a, b):
        o.init_cache(pk, pv, hs, hs[0][:, :w0.S], w0.S)
    seen = 0
    for n in range(w0.S, w0.S + w0.T):
        q, k, v = inp.step_qkv(n)
        ra = a.decode_step(q, k, v, hs, hs[0][:, n])
        rb = b.decode_step(q, k, v, hs, hs[0][:, n])
        assert np.array_equal(ra[1], rb[1]) and np.array_equal(ra[3], rb[3])
        assert np.array_equal(a.Vc, b.Vc)
        for h in range(w0.H):
            for s, pos in enumerate(a.slot_pos[0, h]):
                if pos in ra[3][0]:
                    raw = hs[0, 0, pos].astype(np.float64) @ wts["w_kv"][0][h * w0.d:(h + 1) * w0.d].astype(np.float64).T
                    want = O.rotary(raw.astype(np.float32)[None], [int(pos)], 100.0)[0].astype(np.float32)
                    assert np.array_equal(b.Kc[0, 0, h, s], want.astype(np.float64))
                    seen += 1
                elif pos >= 0 and not np.array_equal(a.Kc[0, 0, h, s], b.Kc[0, 0, h, s]):
                    # rebuilt in an earlier step and still resident
                    assert pos < n
    assert seen > 0


# --------------------------------------------------------------------------
# top-K attention over a whole sequence
# --------------------------------------------------------------------------
def test_topk_attention_with_k_covering_the_sequence_is_causal_attention():
    rng = np.random.default_rng(11)
    q, k, v = (rng.standard_normal((3, 19, 8)) for _ in range(3))
    want = torch.nn.functional.scaled_dot_product_attention(torch.tensor(q), torch.tensor(k), torch.tensor(v),
                                                            is_causal=True).numpy()
    for top_k in (19, 64):
        got, kept = O.topk_attention(q, k, v, top_k)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
        assert np.array_equal(kept, np.broadcast_to(np.tril(np.ones((19, 19), dtype=bool)), kept.shape))


def test_topk_attention_with_k_one_returns_the_value_of_the_largest_weight():
    rng = np.random.default_rng(12)
    q, k, v = (rng.standard_normal((2, 15, 4)) for _ in range(3))
    got, kept = O.topk_attention(q, k, v, 1)
    for r in range(2):
        for i in range(15):
            j = int(np.argmax(k[r, :i + 1] @ q[r, i]))
            assert np.array_equal(got[r, i], v[r, j]) and kept[r, i].sum() == 1 and kept[r, i, j]


def test_topk_attention_by_brute_force_over_subsets():
    """Tiny case: of all subsets of top_k past keys, the kept one has the largest sum of weights (that is the
    top-K set when no two weights are equal), and the output is the softmax over exactly that subset."""
    rng = np.random.default_rng(13)
    S, d, top_k = 7, 3, 3
    q, k, v = (rng.standard_normal((1, S, d)) for _ in range(3))
    got, kept = O.topk_attention(q, k, v, top_k)
    for i in range(S):
        w = k[0, :i + 1] @ q[0, i]
        size = min(top_k, i + 1)
        best = max(itertools.combinations(range(i + 1), size), key=lambda c: sum(w[list(c)]))
        assert sorted(best) == list(np.nonzero(kept[0, i])[0])
        p = scipy.special.softmax(w[list(best)] / np.sqrt(d))
        np.testing.assert_allclose(got[0, i], p @ v[0, list(best)], rtol=1e-12, atol=1e-13)


def test_topk_attention_rows_sum_to_one_and_ties_go_to_the_lower_position():
    rng = np.random.default_rng(14)
    S, d, top_k = 12, 4, 5
    k, v = rng.standard_normal((1, S, d)), rng.standard_normal((1, S, d))
    ones = np.ones((1, S, d))
    q = rng.standard_normal((1, S, d))
    got, _ = O.topk_attention(q, k, ones, top_k)            # softmax weights sum to 1
    np.testing.assert_allclose(got, ones, rtol=1e-13)
    got, kept = O.topk_attention(np.zeros((1, S, d)), k, v, top_k)      # all weights equal: the first top_k positions
    for i in range(S):
        n = min(top_k, i + 1)
        assert list(np.nonzero(kept[0, i])[0]) == list(range(n))
        np.testing.assert_allclose(got[0, i], v[0, :n].mean(axis=0), rtol=1e-13, atol=1e-14)
    # two equal weights at the cut: keys 2 and 6 are identical, K = 2 and the best key is 9 -> 9 and 2 stay
    k2 = rng.standard_normal((1, S, d)) * 0.01
    qv = np.array([1.0, 0.0, 0.0, 0.0])
    k2[0, 2] = k2[0, 6] = 2 * qv
    k2[0, 9] = 3 * qv
    _, kept = O.topk_attention(np.broadcast_to(qv, (1, S, d)), k2, v, 2)
    assert list(np.nonzero(kept[0, 11])[0]) == [2, 9]
