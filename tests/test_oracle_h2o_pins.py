"""Pins for the H2O(Rebuilt) oracle (Sec. 3.1, baselines 6 and 7): each checks it against something other than
itself: a closed form under uniform attention, a library softmax summed up independently, brute-force order
checks of both selections, a one-head job that must equal a job whose heads are copies, invariants when the
heads disagree, and Eq. 1 over all tokens when nothing is ever evicted."""
import numpy as np
import pytest
import scipy.special

from gen import SyntheticInputs, Workload
from oracle import adore_oracle as O
from tests.helpers import oracle_config


def _job(w, wts=None):
    inp = SyntheticInputs(w)
    wts = inp.weights() if wts is None else wts
    return O.AdoreH2OOracle(oracle_config(w), wts), inp


def _w(**kw):
    base = dict(name="h2o", L=1, B=2, H=3, d=16, D=32, K=16, R=3, S=40, T=20, dtype="f32", dprime=8, act_std=1.0, w_std=0.2)
    base.update(kw)
    return Workload(**base)


def test_uniform_attention_gives_the_closed_form():
    """q = 0: every held row gets 1 / (rows held) at every step.  From zero prompt scores and a prompt longer than
    the cache, ties put the lowest positions into the cache; from then on the rows that are attended keep growing
    at the same rate, so nothing ever overtakes them: each head holds tokens 0 .. m-2 and the current one for good,
    tokens m-1 .. m+R-2 are rebuilt at every step, a generated token is attended twice (in its own step, where it is
    exempt, and in the next), and the scores are step counts over K (exact in fp32: K = 16)."""
    w = _w(K=16, R=3, S=40, T=25)
    orc, inp = _job(w)
    hs = inp.hidden_store()
    pk, pv = inp.prompt_kv()
    rb = orc.init_cache(pk, pv, hs, w.S)
    m = w.K - w.R - 1
    assert all(r == list(range(m - 1, m - 1 + w.R)) for r in rb)
    for t in range(w.T):
        n = w.S + t
        q, k, v = inp.step_qkv(n)
        out, slot_map, released, rebuilt = orc.decode_step(np.zeros_like(q), k, v, hs)
        for b in range(w.B):
            assert rebuilt[b].tolist() == list(range(m - 1, m - 1 + w.R))
            for h in range(w.H):
                held = sorted(int(p) for p in slot_map[b, h] if p >= 0)
                assert held == list(range(m - 1 + w.R)) + [n]
                want = np.zeros(n + 1)
                want[:m - 1 + w.R] = (t + 1) / w.K          # attended at every step so far
                want[w.S - 1] = 1.0 / w.K                   # the last prompt token: attended once, then evicted
                want[w.S:n] = 2.0 / w.K                     # a generated token stays for its own step (exempt) and the next
                want[n] = 1.0 / w.K
                assert np.array_equal(orc.hscore[b, h, :n + 1].astype(np.float64), want)
    assert orc.n == w.S + w.T


def test_scores_are_the_library_softmax_summed_by_position():
    """The accumulated score of (head, token) against an independent tally: at every step scipy's softmax of the
    logits of the rows the head holds (read from the oracle's cache before the step), added up by position."""
    w = _w(B=1, H=2, K=12, R=2, S=20, T=30, act_std=0.7)
    orc, inp = _job(w)
    hs = inp.hidden_store()
    pk, pv = inp.prompt_kv()
    rng = np.random.default_rng(5)
    init = rng.random((w.B, w.H, w.S)).astype(np.float32)
    orc.init_cache(pk, pv, hs, w.S, score_init=init)
    tally = np.zeros((w.H, w.N_max))
    tally[:, :w.S] = init[0]
    for t in range(w.T):
        n = w.S + t
        q, k, v = inp.step_qkv(n)
        before = orc.slot_pos.copy()
        Kc = orc.Kc.copy()
        orc.decode_step(q, k, v, hs)
        for h in range(w.H):
            pos = [int(p) for p in before[0, h] if p >= 0] + [n]
            rows = np.concatenate([Kc[0, 0, h][before[0, h] >= 0], k[0, 0, h][None, :]])
            p = scipy.special.softmax(rows @ q[0, 0, h] / np.sqrt(float(w.d)))
            for pos_i, p_i in zip(pos, p):
                tally[h, pos_i] += p_i
        assert np.abs(orc.hscore[0, :, :n + 1] - tally[:, :n + 1]).max() < 1e-5 * (1 + t)   # fp32 storage
        assert abs(orc.own_scores[0].sum() - (init.sum() + (t + 1) * w.H)) < 1e-3          # one unit per head and step


def test_both_selections_by_brute_force_order_checks():
    """Per head: every evicted token ranks below every token that stays (the current one aside).  Per sequence:
    the candidates are exactly the tokens some head is missing, and every chosen one ranks above every other
    candidate on the fp32 sum over heads; ties (scores on a coarse grid) go to the lower position."""
    w = _w(B=2, H=3, K=10, R=3, S=14, T=40)
    orc, inp = _job(w)
    hs = inp.hidden_store()
    pk, pv = inp.prompt_kv()
    rng = np.random.default_rng(9)
    grid = lambda shape: (rng.integers(0, 4, size=shape) / 2.0).astype(np.float32)
    orc.init_cache(pk, pv, hs, w.S, score_init=grid((w.B, w.H, w.S)))
    m = w.K - w.R - 1
    beats = lambda sc, i, j: sc[i] > sc[j] or (sc[i] == sc[j] and i < j)
    for t in range(w.T):
        n = w.S + t
        q, k, v = inp.step_qkv(n)
        before = orc.slot_pos.copy()
        forced = np.zeros((w.B, w.H, n + 1), dtype=np.float32)
        forced[:, :, :n] = orc.hscore[:, :, :n]
        forced += grid(forced.shape) * (rng.random(forced.shape) < 0.2)      # scores move, stay on the grid
        out, slot_map, released, rebuilt = orc.decode_step(q, k, v, hs, score_override=forced)
        for b in range(w.B):
            after_release = []
            for h in range(w.H):
                had = [int(p) for p in before[b, h] if p >= 0] + [n]
                gone = [int(p) for p in released[b, h] if p >= 0]
                assert len(gone) == max(0, len(had) - m) and n not in gone and set(gone) <= set(had)
                stay = [p for p in had if p not in gone]
                after_release.append(set(stay))
                sc = forced[b, h]
                assert all(beats(sc, s_, g) for s_ in stay if s_ != n for g in gone)
            pool = [i for i in range(n + 1) if any(i not in s_ for s_ in after_release)]
            agg = np.zeros(n + 1, dtype=np.float32)
            for h in range(w.H):
                agg = agg + forced[b, h]
            chosen = [int(p) for p in rebuilt[b] if p >= 0]
            assert len(chosen) == min(w.R, len(pool)) and set(chosen) <= set(pool)
            assert all(beats(agg, chosen[i], chosen[i + 1]) for i in range(len(chosen) - 1))
            assert all(beats(agg, c_, u) for c_ in chosen for u in pool if u not in chosen)
            for h in range(w.H):
                held = [int(p) for p in slot_map[b, h] if p >= 0]
                assert len(held) == len(set(held))
                assert set(held) == after_release[h] | set(chosen)
                # a head keeps the row of a chosen token it still holds; the others take the lowest free slots in rank order
                free = [k_ for k_ in range(w.K) if before[b, h, k_] < 0 or int(before[b, h, k_]) in
                        [int(p) for p in released[b, h] if p >= 0]]
                free = sorted(set(free) - {int(np.nonzero(before[b, h] < 0)[0][0])})      # minus the current token's slot
                new = [c_ for c_ in chosen if c_ not in after_release[h]]
                assert [int(slot_map[b, h, s_]) for s_ in free[:len(new)]] == new


def test_heads_that_are_copies_behave_like_one_head():
    """Three identical heads against a one-head job on the same data: every head's slot map equals the single
    head's, and the per-sequence choice on the sum over heads equals the choice on the single score."""
    w1 = _w(B=2, H=1, K=12, R=3, S=30, T=25, act_std=0.8)
    w3 = w1.scaled(H=3)
    inp1 = SyntheticInputs(w1)
    wts1 = inp1.weights()
    Hd = w1.d
    wkv = wts1["w_kv"]                                                  # [1, 2*d, D]
    wts3 = dict(wts1, w_kv=np.concatenate([np.tile(wkv[:, :Hd], (1, 3, 1)), np.tile(wkv[:, Hd:], (1, 3, 1))], axis=1))
    o1 = O.AdoreH2OOracle(oracle_config(w1), wts1)
    o3 = O.AdoreH2OOracle(oracle_config(w3), wts3)
    hs = inp1.hidden_store()
    pk, pv = inp1.prompt_kv()
    rep = lambda a, ax: np.repeat(a, 3, axis=ax)
    o1.init_cache(pk, pv, hs, w1.S)
    o3.init_cache(rep(pk, 2), rep(pv, 2), hs, w1.S)
    for t in range(w1.T):
        q, k, v = inp1.step_qkv(w1.S + t)
        r1 = o1.decode_step(q, k, v, hs)
        r3 = o3.decode_step(rep(q, 2), rep(k, 2), rep(v, 2), hs)
        for h in range(3):
            assert np.array_equal(r3[1][:, h], r1[1][:, 0]) and np.array_equal(r3[2][:, h], r1[2][:, 0])
            assert np.allclose(r3[0][0][:, h], r1[0][0][:, 0], rtol=0, atol=1e-12)
        assert np.array_equal(r3[3], r1[3])


def test_heads_that_attend_differently_hold_different_tokens():
    """Head 0's queries point at the key of one old token, head 1's at another: the heads keep different tokens,
    every position sits at most once in a head, and a rebuilt token ends up in every head."""
    w = _w(B=1, H=2, K=10, R=2, S=30, T=20, act_std=0.5)
    orc, inp = _job(w)
    hs = inp.hidden_store()
    pk, pv = inp.prompt_kv()
    orc.init_cache(pk, pv, hs, w.S)
    differ = 0
    for t in range(w.T):
        n = w.S + t
        q, k, v = inp.step_qkv(n)
        q = q.copy()
        for h, target in ((0, 0), (1, 1)):                  # each head's query = a multiple of one resident key
            slot = int(np.nonzero(orc.slot_pos[0, h] == target)[0][0])
            q[0, 0, h] = 6.0 * orc.Kc[0, 0, h, slot]
        out, slot_map, released, rebuilt = orc.decode_step(q, k, v, hs)
        sets = [set(int(p) for p in slot_map[0, h] if p >= 0) for h in range(w.H)]
        differ += sets[0] != sets[1]
        for h in range(w.H):
            held = [int(p) for p in slot_map[0, h] if p >= 0]
            assert len(held) == len(set(held)) <= w.K - 1
            assert all(int(p) in sets[h] for p in rebuilt[0] if p >= 0)
        assert 0 in sets[0] and 1 in sets[1]                 # the token a head keeps looking at stays in it
    assert differ > 0
    assert orc.hscore[0, 0, 0] > 5 * orc.hscore[0, 1, 0] and orc.hscore[0, 1, 1] > 5 * orc.hscore[0, 0, 1]


def test_rebuilt_rows_are_the_projections_of_their_tokens():
    """Consistency case: the supplied K/V of every token are the rounded projections of its hidden state (torch
    matmul), so whatever the oracle rebuilds must reproduce the row the token had: every occupied row of every
    head equals its token's projection, head slice by head slice."""
    import torch
    w = _w(B=2, H=3, K=10, R=3, S=16, T=25, dtype="bf16")
    orc, inp = _job(w)
    wts = inp.weights()
    hs = inp.hidden_store()
    Hd = w.H * w.d
    proj = torch.from_numpy(hs[0].astype(np.float64)) @ torch.from_numpy(wts["w_kv"][0].astype(np.float64)).T   # [B,N,2Hd]
    proj = O.round_to_storage(proj.numpy(), w.dtype)
    Kall = proj[..., :Hd].reshape(w.B, w.N_max, w.H, w.d).transpose(0, 2, 1, 3)        # [B,H,N,d]
    Vall = proj[..., Hd:].reshape(w.B, w.N_max, w.H, w.d).transpose(0, 2, 1, 3)
    orc.init_cache(Kall[None, :, :, :w.S], Vall[None, :, :, :w.S], hs, w.S)
    for t in range(w.T):
        n = w.S + t
        q, _, _ = inp.step_qkv(n)
        orc.decode_step(q, Kall[None, :, :, n], Vall[None, :, :, n], hs)
        for b in range(w.B):
            for h in range(w.H):
                for s_, p_ in enumerate(orc.slot_pos[b, h]):
                    if p_ >= 0:
                        assert np.array_equal(orc.Kc[0, b, h, s_], Kall[b, h, p_]) and np.array_equal(orc.Vc[0, b, h, s_], Vall[b, h, p_])


def test_a_cache_that_holds_everything_is_full_attention():
    w = _w(B=1, H=2, K=64, R=2, S=20, T=10)
    assert w.K - w.R - 1 >= w.N_max
    orc, inp = _job(w)
    hs = inp.hidden_store()
    pk, pv = inp.prompt_kv()
    orc.init_cache(pk, pv, hs, w.S)
    Kall = [pk[0, 0, h] for h in range(w.H)]
    Vall = [pv[0, 0, h] for h in range(w.H)]
    for t in range(w.T):
        q, k, v = inp.step_qkv(w.S + t)
        out, slot_map, released, rebuilt = orc.decode_step(q, k, v, hs)
        Kall = [np.concatenate([Kall[h], k[0, 0, h][None]]) for h in range(w.H)]
        Vall = [np.concatenate([Vall[h], v[0, 0, h][None]]) for h in range(w.H)]
        want = O.full_attention(q[0, 0], np.stack(Kall), np.stack(Vall))
        assert np.allclose(out[0, 0], want, rtol=0, atol=1e-12)
        assert (released < 0).all() and (rebuilt < 0).all()
        assert (slot_map[0, :, :w.S + t + 1] == np.arange(w.S + t + 1)).all()


def test_h2o_oracle_takes_one_layer_only():
    with pytest.raises(ValueError):
        _job(_w(L=2))
