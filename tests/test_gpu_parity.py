"""Parity of the HIP path (called through the C-ABI) with the CPU oracle on the same seeded inputs.

Slot maps, released and rebuilt positions must be identical; attention outputs within 1e-5 (fp32)
or 2e-3 (bf16) of the oracle, measured per row as max|diff| / max|ref|; the controller's sigma
within 1e-5.  Both sides rank tokens from the same fp32 sigma bits (the oracle checks its own
value against the GPU's, then adopts the GPU's bits).
"""
import os
from dataclasses import replace

import numpy as np
import pytest
import torch

from gen import SyntheticInputs, Workload, workload
from oracle import adore_oracle as O
from tests.helpers import GOLDEN, parse_trajectory, small_workload

pytestmark = pytest.mark.gpu


def _harness():
    from tests import gpu_harness
    return gpu_harness


def test_tiny_full_trajectory():
    """The tiny workload end to end: prompt 128, all 256 decode steps, fp32."""
    h = _harness()
    w = workload("tiny")
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=64)
    print(f"tiny: worst output error {worst:.3e}")
    job.adore.close()


def test_bf16_trajectory_spanning_tiles_with_ragged_sizes():
    """bf16, d=128: K=200 is not a multiple of the 64-slot tile, B*R=15 rows leave the GEMM tile ragged,
    the attention splits each row over several workgroups."""
    h = _harness()
    w = Workload("bf16_small", L=1, B=3, H=4, d=128, D=512, K=200, R=5, S=260, T=40, dtype="bf16")
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=10)
    assert job.adore.cfg.cache_slots == 200
    print(f"bf16_small: worst output error {worst:.3e}")
    job.adore.close()


def test_bf16_head_dim_64_and_two_layers():
    h = _harness()
    w = Workload("bf16_d64", L=2, B=2, H=4, d=64, D=256, K=96, R=8, S=120, T=24, dtype="bf16")
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=8)
    job.adore.close()


def test_fp32_head_dim_128():
    h = _harness()
    w = Workload("f32_d128", L=1, B=2, H=2, d=128, D=128, K=80, R=4, S=100, T=16, dtype="f32",
                 act_std=0.3, w_std=0.1)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=8)
    job.adore.close()


def test_warm_up_from_a_short_prompt():
    """S < m: the cache fills up first (nothing released, nothing rebuilt), then reaches steady state."""
    h = _harness()
    w = small_workload(B=2, H=2, d=64, D=64, K=20, R=4, S=3, T=40, dtype="f32", dprime=16)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=5)
    job.adore.close()


def test_no_rebuild_budget():
    h = _harness()
    w = small_workload(B=1, H=2, d=64, D=64, K=16, R=0, S=30, T=20, dtype="f32", dprime=16)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=5)
    job.adore.close()


def test_maximum_slots_and_single_token_prompt():
    h = _harness()
    w = Workload("k1024", L=1, B=1, H=2, d=64, D=64, K=1024, R=30, S=1, T=12, dtype="bf16", dprime=16)
    worst, job, _ = h.lockstep(w, steps=w.T)
    job.adore.close()
    w = Workload("k1024_full", L=1, B=1, H=2, d=64, D=64, K=1024, R=1022, S=1500, T=6, dtype="bf16", dprime=16)
    worst, job, _ = h.lockstep(w, steps=w.T)
    job.adore.close()


def test_injected_ties_are_broken_by_position():
    """Scores drawn from 7 values: most comparisons are ties."""
    h = _harness()
    w = small_workload(B=2, H=2, d=64, D=64, K=24, R=5, S=70, T=30, dtype="f32", dprime=16)
    rng = np.random.default_rng(11)
    override = rng.choice(np.array([0.0, -0.0, 0.25, 0.5, 0.5, 0.75, 1.0], dtype=np.float32), (w.B, w.N_max))
    worst, job, _ = h.lockstep(w, steps=w.T, override=override, check_cache_every=10)
    job.adore.close()


@pytest.mark.parametrize("name,K,R", [("slot_trajectory_K4_R1.txt", 4, 1), ("slot_trajectory_K7_R3.txt", 7, 3)])
def test_hand_worked_trajectory_on_gpu(name, K, R):
    """The slot maps worked out by hand; the second file pins which free slot each rebuilt rank takes."""
    h = _harness()
    init_scores, after_init, steps = parse_trajectory(os.path.join(GOLDEN, name))
    S = len(init_scores)
    w = Workload("golden", L=1, B=1, H=2, d=64, D=64, K=K, R=R, S=S, T=len(steps), dtype="f32", dprime=16)
    job = h.GpuJob(w)
    job.init(init_scores[None, :])
    snap = job.snapshot()
    for hh in range(w.H):
        assert snap["slot_pos"][0, hh].tolist() == after_init["slot_map"]
    for st in steps:
        out, slot_map, released, rebuilt, score = job.step(st["n"], override=np.array([st["score"]], np.float32))
        for hh in range(w.H):
            assert slot_map[0, hh].tolist() == st["slot_map"], st
            assert released[0, hh].tolist() == st["released"], st
        assert rebuilt[0].tolist() == st["rebuilt"], st
    job.adore.close()


def test_decode_step_entry_point_and_determinism():
    """adore_decode_step (L = 1) gives the same result as attend + schedule + rebuild, and a second run
    from the same inputs reproduces slot maps and outputs bit for bit."""
    h = _harness()
    w = Workload("ds", L=1, B=2, H=4, d=128, D=256, K=72, R=6, S=90, T=10, dtype="bf16")
    inp = SyntheticInputs(w)
    results = []
    for rep in range(2):
        job = h.GpuJob(w, inp)
        job.init()
        maps, outs = [], []
        for n in range(w.S, w.S + w.T):
            q, k, v = (h.to_dev(a[0], job.st) for a in inp.step_qkv(n))
            if rep == 0:
                job.adore.decode_step(q, k, v, job.hidden[0], job.hidden[0][:, n].contiguous(), None,
                                      job.out[0], job.slot_map)
            else:
                job.adore.attend(0, q, k, v, job.out[0])
                job.adore.schedule(job.hidden[0][:, n].contiguous(), None, job.slot_map, None, None)
                job.adore.rebuild(0, job.hidden[0])
            torch.cuda.synchronize()
            maps.append(job.slot_map.cpu().numpy().copy())
            outs.append(job.out.cpu().numpy().copy())
        results.append((maps, outs, job.snapshot()))
        job.adore.close()
    for a, b in zip(results[0][0], results[1][0]):
        assert np.array_equal(a, b)
    for a, b in zip(results[0][1], results[1][1]):
        assert np.array_equal(a, b)
    for key in ("cache_k", "cache_v", "scores", "z", "slot_pos"):
        s0, s1 = results[0][2][key], results[1][2][key]
        if key == "scores":
            s0, s1 = s0[:, :w.S + w.T], s1[:, :w.S + w.T]
        if key in ("cache_k", "cache_v"):
            occ = results[0][2]["slot_pos"] >= 0
            s0, s1 = s0[0][occ], s1[0][occ]
        assert np.array_equal(s0, s1), key


def test_two_contexts_interleaved_do_not_disturb_each_other():
    """Contexts are independent: a job stepped alone and the same job stepped in turns with a second context of
    another shape (same stream, one with the whole-step call, one with the fine-grained calls, no synchronisation
    between them) give the same bits."""
    h = _harness()
    wa = Workload("ctx_a", L=1, B=2, H=4, d=128, D=256, K=72, R=6, S=90, T=10, dtype="bf16", dprime=128)
    wb = Workload("ctx_b", L=2, B=3, H=2, d=64, D=128, K=40, R=9, S=30, T=10, dtype="bf16", dprime=32)
    ia, ib = SyntheticInputs(wa), SyntheticInputs(wb)

    def step_a(job, n):
        q, k, v = (h.to_dev(a[0], job.st) for a in ia.step_qkv(n))
        job.adore.decode_step(q, k, v, job.hidden[0], job.hidden[0][:, n].contiguous(), None, job.out[0], job.slot_map)

    def step_b(job, n):
        q, k, v = (h.to_dev(a, job.st) for a in ib.step_qkv(n))
        for l in range(wb.L):
            job.adore.attend(l, q[l], k[l], v[l], job.out[l])
        job.adore.schedule(job.hidden[0][:, n].contiguous(), None, job.slot_map, job.released, job.rebuilt)
        for l in range(wb.L):
            job.adore.rebuild(l, job.hidden[l])

    alone = h.GpuJob(wa, ia)
    alone.init()
    for t in range(wa.T):
        step_a(alone, wa.S + t)
    want = alone.snapshot()
    want_out = alone.out.cpu().numpy().copy()
    alone.adore.close()

    a, b = h.GpuJob(wa, ia), h.GpuJob(wb, ib)
    a.init()
    b.init()
    for t in range(wa.T):
        step_a(a, wa.S + t)
        step_b(b, wb.S + t)
    got = a.snapshot()
    assert np.array_equal(a.out.cpu().numpy(), want_out)
    occ = want["slot_pos"] >= 0
    assert np.array_equal(got["slot_pos"], want["slot_pos"])
    assert np.array_equal(got["scores"][:, :wa.S + wa.T], want["scores"][:, :wa.S + wa.T])
    assert np.array_equal(got["z"], want["z"])
    for key in ("cache_k", "cache_v"):
        assert np.array_equal(got[key][0][occ], want[key][0][occ]), key
    # and the second context followed its own oracle meanwhile: its trajectory alone, for comparison
    b2 = h.GpuJob(wb, ib)
    b2.init()
    for t in range(wb.T):
        step_b(b2, wb.S + t)
    sb, sb2 = b.snapshot(), b2.snapshot()
    assert np.array_equal(sb["slot_pos"], sb2["slot_pos"])
    assert np.array_equal(b.out.cpu().numpy(), b2.out.cpu().numpy())
    for j in (a, b, b2):
        j.adore.close()


def test_state_snapshot_and_restore():
    h = _harness()
    w = Workload("snap", L=1, B=2, H=2, d=64, D=128, K=40, R=4, S=60, T=12, dtype="bf16", dprime=32)
    inp = SyntheticInputs(w)
    job = h.GpuJob(w, inp)
    job.init()
    for n in range(w.S, w.S + 4):
        job.step(n)
    saved = {k: v.clone() for k, v in job.state.items()}
    step = job.adore.get_state(**saved)
    torch.cuda.synchronize()
    assert step == w.S + 4
    ref = [job.step(n) for n in range(w.S + 4, w.S + 8)]
    job.adore.set_state(saved["slot_pos"], saved["scores"], saved["z"], saved["cache_k"], saved["cache_v"], step)
    again = [job.step(n) for n in range(w.S + 4, w.S + 8)]
    for a, b in zip(ref, again):
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    job.adore.close()


def test_state_machine_on_device():
    h = _harness()
    from paper_2407_02328_amd import AdoreError
    w = Workload("sm", L=2, B=1, H=2, d=64, D=64, K=16, R=2, S=20, T=2, dtype="f32", dprime=16)
    inp = SyntheticInputs(w)
    job = h.GpuJob(w, inp)
    job.init()
    q, k, v = (h.to_dev(a, job.st) for a in inp.step_qkv(w.S))
    x = job.hidden[0][:, w.S].contiguous()
    with pytest.raises(AdoreError) as e:
        job.adore.schedule(x)                       # no layer attended yet
    assert e.value.code == -2
    job.adore.attend(0, q[0], k[0], v[0], job.out[0])
    with pytest.raises(AdoreError):
        job.adore.attend(0, q[0], k[0], v[0], job.out[0])      # twice
    with pytest.raises(AdoreError):
        job.adore.schedule(x)                       # layer 1 missing
    with pytest.raises(AdoreError):
        job.adore.rebuild(0, job.hidden[0])         # before schedule
    job.adore.attend(1, q[1], k[1], v[1], job.out[1])
    job.adore.schedule(x)
    with pytest.raises(AdoreError):
        job.adore.schedule(x)
    job.adore.rebuild(1, job.hidden[1])
    with pytest.raises(AdoreError):
        job.adore.rebuild(1, job.hidden[1])
    with pytest.raises(AdoreError):
        job.adore.get_state()                       # mid-step
    job.adore.rebuild(0, job.hidden[0])
    assert job.adore.get_state() == w.S + 1
    # one more step reaches N_max; the next attend is refused
    q, k, v = (h.to_dev(a, job.st) for a in inp.step_qkv(w.S + 1))
    for l in range(2):
        job.adore.attend(l, q[l], k[l], v[l], job.out[l])
    job.adore.schedule(job.hidden[0][:, w.S + 1].contiguous())
    for l in range(2):
        job.adore.rebuild(l, job.hidden[l])
    with pytest.raises(AdoreError) as e:
        job.adore.attend(0, q[0], k[0], v[0], job.out[0])
    assert e.value.code == -2
    with pytest.raises(ValueError):
        job.adore.attend(0, q[0].float().double(), k[0], v[0], job.out[0])   # wrong dtype caught by the binding
    torch.cuda.synchronize()
    job.adore.close()


@pytest.mark.parametrize("ordered", [True, False])
def test_init_again_restarts_the_context(ordered):
    """adore_init_cache may be called again: after some steps a second init over the same prompt (enqueued right
    behind the last step, no synchronisation) starts the same trajectory again, bit for bit, and a third over a
    shorter prompt gives what a context that has seen nothing else gives."""
    h = _harness()
    w = Workload("restart", **dict(ORDER_W, T=12))
    inp = SyntheticInputs(w)
    job = h.GpuJob(w, inp, ordered=ordered)
    job.init()
    first = [job.step(w.S + t, whole=t % 2 == 0) for t in range(w.T)]
    st = job.st
    pk, pv = (h.to_dev(a, st) for a in job.prompt_np)
    job.adore.init_cache(pk, pv, job.hidden, job.hidden[0][:, :w.S].contiguous(), None, w.S)
    second = [job.step(w.S + t, whole=t % 2 == 0) for t in range(w.T)]
    def same(a_run, b_run, whole_steps, when):
        for t, (a, b) in enumerate(zip(a_run, b_run)):
            for x, y, what in zip(a, b, ("output", "slot map", "released", "rebuilt", "score")):
                if what in ("released", "rebuilt") and t % 2 == whole_steps:
                    continue        # the whole-step call reports the slot map only
                assert np.array_equal(x, y), f"{what} at step {t} {when}"

    same(first, second, 0, "after the second init")
    # a third init over a shorter prompt, in the same context: nothing of the longer runs is left behind (the same
    # steps in a context that has seen nothing else give the same bits)
    S2 = 50
    pk2, pv2 = (t[:, :, :, :S2].contiguous() for t in (pk, pv))

    def short_run(j):
        j.adore.init_cache(pk2, pv2, j.hidden, j.hidden[0][:, :S2].contiguous(), None, S2)
        return [j.step(S2 + t, whole=t % 2 == 1) for t in range(w.T)]

    third = short_run(job)
    job.adore.close()
    fresh = h.GpuJob(w, inp, ordered=ordered)
    want = short_run(fresh)
    fresh.adore.close()
    same(third, want, 1, "after the init over the shorter prompt")


@pytest.mark.parametrize("split,waves", [(1, 4), (1, 16), (2, 8), (4, 4), (3, 16)])
def test_attention_launch_shapes(split, waves, monkeypatch):
    """Every split count / workgroup width of the attention kernel gives the oracle's result."""
    h = _harness()
    monkeypatch.setenv("ADORE_ATTEND_SPLIT", str(split))
    monkeypatch.setenv("ADORE_ATTEND_WAVES", str(waves))
    w = Workload("shapes", L=1, B=2, H=3, d=128, D=256, K=300, R=7, S=400, T=6, dtype="bf16", dprime=32)
    worst, job, _ = h.lockstep(w, steps=w.T)
    assert job.adore.cfg.cache_slots == 300
    job.adore.close()


def test_full_attention_cache_holds_every_token():
    """K - R - 1 >= N_max: nothing is ever released, the step is the full attention of Eq. 1 over a cache of
    more than 1024 slots (the no-release kernel walks the row in chunks), and the slot map stays the identity."""
    h = _harness()
    w = Workload("full", L=1, B=2, H=2, d=128, D=256, K=1500, R=4, S=1100, T=5, dtype="bf16", dprime=32)
    worst, job, orc = h.lockstep(w, steps=w.T)
    sm = job.slot_map.cpu().numpy()
    n_last = w.S + w.T - 1
    assert (sm[..., :n_last + 1] == np.arange(n_last + 1)).all() and (sm[..., n_last + 1:] == -1).all()
    job.adore.close()


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4])
def test_rebuild_gemm_tile_shapes(tile, monkeypatch):
    """Every output-tile shape of the re-projection kernel (256x256 ... 128x32) gives the oracle's cache rows
    and outputs: M = B*R = 3*45 = 135 rows is a ragged tile in each of them, d = 64 puts up to four head
    slices into one tile row, and D = 448 leaves a guarded tail in every pipeline depth."""
    h = _harness()
    monkeypatch.setenv("ADORE_GEMM_TILE", str(tile))
    w = Workload("tiles", L=1, B=3, H=8, d=64, D=448, K=128, R=45, S=200, T=5, dtype="bf16", dprime=32)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=1)
    job.adore.close()


def test_llama7b_layer_full_size_steps():
    """The benchmark workload at its full size and in the launch configuration bench.py times
    (B16 H32 d128 D4096 K512 R32, prompt 1024): init plus six free-running steps, every slot map,
    every output row and every occupied cache row against the oracle."""
    h = _harness()
    w = workload("llama7b_layer").scaled(T=8)
    worst, job, _ = h.lockstep(w, steps=6, check_cache_every=3)
    print(f"llama7b_layer: worst output error {worst:.3e}")
    job.adore.close()


@pytest.mark.timeout(600)
def test_llama7b_layer_full_size_many_steps_sampled_sequences():
    """The benchmark workload at full size over 72 steps of adore_decode_step (several times round the rings of
    per-step lists, across a 64-token boundary of the controller's scratch); the oracle follows sequences 3 and 12."""
    h = _harness()
    w = workload("llama7b_layer").scaled(T=80)
    worst, job, _ = h.sampled_lockstep(w, steps=72, seqs=[3, 12])
    print(f"llama7b_layer (full size, 72 steps, 2 of 16 sequences): worst output error {worst:.3e}")
    job.adore.close()


def test_long_context_reduced_with_salience():
    """The long-context recipe (Zipf salience in key dimension 0 and in the controller input, K = 1024,
    rows split over several workgroups) at a prompt the oracle finishes in seconds."""
    h = _harness()
    w = workload("long_context").scaled(B=1, H=4, S=2048, T=12)
    worst, job, _ = h.lockstep(w, steps=10, check_cache_every=5)
    assert job.adore.cfg.cache_slots == 1024
    print(f"long_context (reduced): worst output error {worst:.3e}")
    job.adore.close()


def test_high_batch_reduced():
    """The high-batch recipe (K = 256, R = 16) with 8 of its 128 sequences."""
    h = _harness()
    w = workload("high_batch").scaled(B=8, T=10)
    worst, job, _ = h.lockstep(w, steps=8, check_cache_every=4)
    job.adore.close()


@pytest.mark.timeout(300)
def test_high_batch_full_size_sampled_sequences():
    """high_batch at its full size (B128 H32 d128 D4096 K256 R16, prompt 512) through adore_decode_step and, every
    third step, the fine-grained calls; the oracle follows sequences 0, 77 and 127."""
    h = _harness()
    w = workload("high_batch").scaled(T=8)
    worst, job, _ = h.sampled_lockstep(w, steps=6, seqs=[0, 77, 127], whole=lambda t: t % 3 != 2)
    print(f"high_batch (full size, 3 of 128 sequences): worst output error {worst:.3e}")
    job.adore.close()


@pytest.mark.timeout(300)
def test_long_context_full_size_sampled_sequences():
    """long_context at its full size (B4 H32 d128 D4096 K1024 R32, prompt 8192, Zipf salience): sixteen prompt
    chunks through the scan, 8000 candidates for the rebuild choice; the oracle follows sequences 1 and 3."""
    h = _harness()
    w = workload("long_context").scaled(T=8)
    worst, job, _ = h.sampled_lockstep(w, steps=5, seqs=[1, 3], whole=lambda t: t % 2 == 0)
    print(f"long_context (full size, 2 of 4 sequences): worst output error {worst:.3e}")
    job.adore.close()


@pytest.mark.timeout(900)
def test_stack32_full_size_sampled_sequences():
    """stack32 at its full size (L32 B32 H32 d128 D4096 K512 R32, prompt 2048: 9 GB of cache, 21 GB of hidden
    states, offsets beyond 32 bits in every layer-indexed tensor), inputs drawn on the device; the oracle follows
    sequences 5 and 31 through every layer."""
    h = _harness()
    w = workload("stack32").scaled(T=3)
    worst = h.stack_sampled(w, steps=2, seqs=[5, 31])
    print(f"stack32 (full size, 2 of 32 sequences): worst output error {worst:.3e}")


def test_stack32_reduced_all_layers():
    """The 32-layer stack (attend x 32, one schedule, rebuild x 32 through the fine-grained calls) with small
    heads and hidden size: every layer's outputs, slot maps and cache rows over eight steps, so that a wrong
    per-layer offset into the cache, W_kv or the hidden store shows on the layer it belongs to."""
    h = _harness()
    w = workload("stack32").scaled(B=2, H=2, D=256, K=64, R=8, S=100, T=10, dprime=32)
    assert w.L == 32
    worst, job, _ = h.lockstep(w, steps=8, check_cache_every=4)
    job.adore.close()


# ---- rescore mode: every token scored again at every step, relative position --------------------
def test_rescore_mode_fp32_trajectory():
    """d' = 128 (the specialised cell kernel keeps W_1 (z_i + pos_b) + b_1 per token), fp32: every score of
    every step within 1e-5 of the oracle's, then identical slot maps, released and rebuilt positions."""
    h = _harness()
    w = Workload("rescore32", L=1, B=2, H=2, d=64, D=256, K=48, R=6, S=80, T=30, dtype="f32", dprime=128,
                 act_std=0.125, w_std=0.125, pos_scale=2.0 ** -6, rescore=True)
    worst, job, orc = h.lockstep(w, steps=w.T, check_cache_every=10)
    assert np.array_equal(orc.score[:, :w.N_max], job.snapshot()["scores"][:, :w.N_max])
    job.adore.close()


def test_rescore_mode_bf16_generic_controller_and_warm_up():
    """Any-d' cell kernel (d' = 32), bf16 storage, a prompt shorter than the cache so that the first steps
    release nothing, 37 tokens per sequence at the end (the last workgroup of the rescore kernel is ragged)."""
    h = _harness()
    w = Workload("rescore16", L=2, B=3, H=2, d=128, D=256, K=24, R=4, S=9, T=28, dtype="bf16", dprime=32,
                 pos_scale=2.0 ** -5, rescore=True)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=14)
    job.adore.close()


def test_rescore_mode_recency_weights_give_a_sliding_window_on_gpu():
    """Zero GRU, identity interaction layer, negative position weight: the score falls with the distance to
    the current token only, and the cache must hold exactly the last m tokens plus the R before them."""
    h = _harness()
    w = Workload("window", L=1, B=2, H=2, d=64, D=128, K=20, R=3, S=30, T=12, dtype="bf16", dprime=32,
                 pos_scale=2.0 ** -6, rescore=True)
    wts = SyntheticInputs(w).weights()
    dp = w.dprime
    wts = dict(wts, gru_w_ih=np.zeros_like(wts["gru_w_ih"]), gru_w_hh=np.zeros_like(wts["gru_w_hh"]),
               gru_b_ih=np.zeros_like(wts["gru_b_ih"]), gru_b_hh=np.zeros_like(wts["gru_b_hh"]),
               pos_w=np.full(dp, -1.0, dtype=np.float32), pos_b=np.zeros(dp, dtype=np.float32),
               mlp_w1=np.eye(dp, dtype=np.float32), mlp_b1=np.zeros(dp, dtype=np.float32),
               out_w=np.ones(dp, dtype=np.float32), out_b=np.zeros(1, dtype=np.float32))
    worst, job, _ = h.lockstep(w, steps=w.T, wts=wts)
    sm = job.slot_map.cpu().numpy()
    n = w.S + w.T - 1
    want = set(range(n - w.m - w.R + 1, n + 1))
    for b in range(w.B):
        for hh in range(w.H):
            assert {int(p) for p in sm[b, hh] if p >= 0} == want
    job.adore.close()


def test_rescore_mode_rejects_overrides_and_restore():
    h = _harness()
    w = Workload("rescore_api", L=1, B=1, H=2, d=64, D=128, K=16, R=2, S=20, T=4, dtype="bf16", dprime=32,
                 rescore=True)
    job = h.GpuJob(w)
    from paper_2407_02328_amd import AdoreError
    with pytest.raises(AdoreError) as e:
        job.init(score_override=np.zeros((w.B, w.S), dtype=np.float32))
    assert e.value.code == -1
    job.init()
    q, k, v = (h.to_dev(a[0], job.st) for a in job.inp.step_qkv(w.S))
    ov = torch.zeros(w.B, dtype=torch.float32, device="cuda:0")
    with pytest.raises(AdoreError) as e:
        job.adore.decode_step(q, k, v, job.hidden[0], job.hidden[0][:, w.S].contiguous(), ov, job.out[0], None)
    assert e.value.code == -1
    with pytest.raises(AdoreError) as e:
        job.adore.set_state(job.state["slot_pos"], None, None, None, None, w.S)
    assert e.value.code == -3
    job.adore.decode_step(q, k, v, job.hidden[0], job.hidden[0][:, w.S].contiguous(), None, job.out[0], None)
    torch.cuda.synchronize()
    job.adore.close()


# ---------------------------------------------------------------------------------------------
# rebuild forward through the layer stack (R+1 query rows per layer)
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,kw", [
    # one 16-row query block, head_dim 64, three layers, a prompt shorter than the cache (rebuild set grows from 0)
    ("r8_d64", dict(L=3, B=2, H=4, d=64, D=256, K=64, R=8, S=40, T=40)),
    # 33 rows (three query blocks, the last with one row), head_dim 128, a slot count that is no multiple of 128
    ("r32_d128", dict(L=2, B=2, H=4, d=128, D=512, K=160, R=32, S=200, T=12)),
    # two and four query blocks
    ("r20_d64", dict(L=1, B=3, H=2, d=64, D=128, K=96, R=20, S=100, T=10)),
    ("r63_d128", dict(L=1, B=1, H=2, d=128, D=256, K=200, R=63, S=260, T=6)),
    # no rebuild budget: the forward is the single-query step with projections around it
    ("r0", dict(L=2, B=2, H=2, d=64, D=128, K=48, R=0, S=60, T=10)),
    # more than 16 sequences: two blocks of current-token rows, the second nearly empty
    ("b18", dict(L=2, B=18, H=2, d=128, D=256, K=64, R=4, S=70, T=5)),
])
def test_forward_step_matches_the_forward_oracle(name, kw):
    h = _harness()
    w = Workload("fwd_" + name, dtype="bf16", dprime=32, w_std=0.06, **kw)
    worst, mean = h.forward_lockstep(w, w.T)
    print(f"forward {name}: worst row error {worst:.2e}, mean {mean:.2e}", flush=True)
    assert mean < 2.0 ** -10


@pytest.mark.parametrize("name,dtype,kw", [
    # fp32 storage (the 1e-5 parity point of the forward): the projections and the attention as plain kernels
    ("f32_r8_d64", "f32", dict(L=3, B=2, H=4, d=64, D=256, K=64, R=8, S=40, T=40)),
    ("f32_r20_d128", "f32", dict(L=2, B=3, H=2, d=128, D=128, K=96, R=20, S=130, T=10)),
    ("f32_r0", "f32", dict(L=2, B=2, H=2, d=64, D=128, K=48, R=0, S=60, T=10)),
    ("f32_rope", "f32", dict(L=2, B=2, H=2, d=64, D=128, K=72, R=10, S=90, T=12, rope_base=10000.0)),
    # bf16 with a model width that is no multiple of 128: plain projections around the matrix-core attention
    ("bf16_D200", "bf16", dict(L=2, B=2, H=3, d=64, D=200, K=80, R=12, S=100, T=12)),
    # bf16 with more than 64 rows per sequence: plain attention between matrix-core projections
    ("bf16_r70", "bf16", dict(L=1, B=2, H=2, d=64, D=128, K=160, R=70, S=200, T=6)),
])
def test_forward_step_on_the_plain_kernels(name, dtype, kw):
    """Configurations the matrix-core kernels of the forward do not take run the same arithmetic as one wave per
    output element; fp32 storage is held to 1e-5."""
    h = _harness()
    w = Workload("fwdp_" + name, dtype=dtype, dprime=32, w_std=0.96 / np.sqrt(kw["D"]), **kw)
    worst, mean = h.forward_lockstep(w, w.T)
    print(f"forward {name}: worst row error {worst:.2e}, mean {mean:.2e}", flush=True)
    assert mean < (2.0 ** -10 if dtype == "bf16" else 1e-6)


def test_forward_step_tiny_config_fp32():
    """The fp32 configuration of the parity suite through the rebuild forward (it had no forward path before)."""
    h = _harness()
    w = replace(workload("tiny"), L=2, T=24)
    worst, mean = h.forward_lockstep(w, w.T)
    print(f"forward tiny fp32 x2: worst row error {worst:.2e}, mean {mean:.2e}", flush=True)
    assert worst < 1e-5


def test_forward_step_with_the_current_rows_in_a_launch_of_their_own(monkeypatch):
    """Widths that are multiples of 256 let the current tokens' rows ride in the tile launches (the cases above
    with H*d = 256 and 512; r20_d64 and r0 do not); here they are kept out of them at such a width."""
    monkeypatch.setenv("ADORE_FWD_CUR_SEPARATE", "1")
    h = _harness()
    w = Workload("fwd_sep", dtype="bf16", dprime=32, w_std=0.06, L=2, B=2, H=4, d=128, D=512, K=160, R=32, S=200, T=6)
    worst, mean = h.forward_lockstep(w, w.T)
    assert mean < 2.0 ** -10


def test_forward_step_llama7b_layer_full_size():
    """The rebuild forward at the benchmark shape and in the launch configuration `bench.py --forward` times
    (B16 H32 d128 D4096 K512 R32, prompt 1024: 33 rows per sequence, 512 + 16 rows per projection), two
    layers: init plus three steps, every selection and every output row against the forward oracle."""
    h = _harness()
    w = workload("llama7b_layer").scaled(L=2, T=4)
    worst, mean = h.forward_lockstep(w, 3)
    print(f"forward llama7b_layer x2: worst row error {worst:.2e}, mean {mean:.2e}", flush=True)
    assert mean < 2.0 ** -10


def test_forward_step_with_rescoring_controller():
    """The rebuild forward with the controller that rates every token again at every step (relative
    position): promotions and demotions change which tokens are rebuilt from step to step."""
    h = _harness()
    w = Workload("fwd_rescore", L=2, B=2, H=4, d=64, D=256, K=48, R=6, S=60, T=24, dtype="bf16", dprime=32,
                 w_std=0.06, rescore=True)
    worst, mean = h.forward_lockstep(w, w.T)
    assert mean < 2.0 ** -10


def test_forward_step_with_injected_ties():
    """Scores given from outside with many equal values: ties go to the lower position in the forward too."""
    h = _harness()
    w = Workload("fwd_ties", L=1, B=2, H=2, d=64, D=128, K=40, R=5, S=50, T=16, dtype="bf16", dprime=32, w_std=0.06)
    rng = np.random.default_rng(7)
    override = rng.integers(0, 4, size=(w.B, w.N_max)).astype(np.float32) / 4.0
    worst, mean = h.forward_lockstep(w, w.T, override=override)
    assert mean < 2.0 ** -10


# ---- adore_decode_step: the selections ride in the attention launch --------------------------------
@pytest.mark.parametrize("name,kw,steps", [
    ("tiny", None, 40),                                                                        # fp32, d = 64, K = 64
    ("bf16_k200", dict(L=1, B=3, H=4, d=128, D=512, K=200, R=5, S=260, T=30, dtype="bf16"), 30),  # ragged K, split rows
    ("bf16_h9", dict(L=1, B=2, H=9, d=64, D=256, K=130, R=12, S=20, T=40, dtype="bf16", dprime=32), 40),  # warm-up from a
    # short prompt (x = 0, then r < R), 9 heads = one full and one nearly empty release workgroup per sequence
    ("bf16_k1024", dict(L=1, B=1, H=4, d=128, D=256, K=1024, R=40, S=1100, T=8, dtype="bf16", dprime=32), 8),
])
def test_decode_step_call_matches_the_oracle(name, kw, steps):
    """Every step through adore_decode_step: slot maps, outputs and cache rows against the oracle."""
    h = _harness()
    w = workload("tiny") if kw is None else Workload("ds_" + name, **kw)
    worst, job, _ = h.lockstep(w, steps=steps, check_cache_every=5, whole=lambda t: True)
    job.adore.close()


@pytest.mark.parametrize("H,K", [(9, 130), (6, 256), (17, 40)])
def test_decode_step_call_with_four_heads_to_a_wave(H, K, monkeypatch):
    """Large batches of short rows let a wave of the riding selections release four heads one after the other (as the
    full-size high-batch run does); here that path is forced on small shapes whose head counts leave waves with
    four, some and no heads."""
    monkeypatch.setenv("ADORE_RIDE_HPW", "4")
    h = _harness()
    w = Workload("ds_hpw", L=1, B=2, H=H, d=64, D=128, K=K, R=7, S=K + 30, T=20, dtype="bf16", dprime=32)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=5, whole=lambda t: True)
    job.adore.close()


def test_decode_step_call_on_long_sequences():
    """Beyond about 4500 positions a sequence's scores and ranking keys no longer fit the LDS of the riding selections,
    and adore_decode_step goes through the selection kernels on the side stream.  5000-token prompts, rows of 300
    slots, 9 heads; whole-step calls mixed with the fine-grained ones."""
    h = _harness()
    w = Workload("ds_long", L=1, B=2, H=9, d=64, D=128, K=300, R=20, S=5000, T=10, dtype="bf16", dprime=32)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=5, whole=lambda t: t % 4 != 3)
    job.adore.close()


@pytest.mark.parametrize("S", [9000, 40000])
def test_rebuild_choice_over_sequences_beyond_the_key_cache(S):
    """The per-sequence choice keeps the ranking keys of a sequence in LDS up to about 7000 tokens, a copy of the
    scores up to about 33000, and reads the scores from memory in every pass beyond: one short-headed job on either
    side of the second limit (the first tier is what every other test runs)."""
    h = _harness()
    w = Workload(f"choice_{S}", L=1, B=2, H=2, d=64, D=64, K=40, R=6, S=S, T=6, dtype="f32", dprime=16)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=3, whole=lambda t: t % 2 == 0)
    job.adore.close()


def test_decode_step_call_mixed_with_fine_grained_calls():
    """Steps alternate in blocks between adore_decode_step and attend / schedule / rebuild: the reserved slot is
    handed over correctly in both directions and the side stream catches up when the selections move back to it."""
    h = _harness()
    w = Workload("ds_mixed", L=1, B=2, H=4, d=128, D=256, K=96, R=8, S=120, T=36, dtype="bf16", dprime=32)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=4, whole=lambda t: (t // 3) % 2 == 0)
    job.adore.close()
    rng = np.random.default_rng(11)
    ties = rng.integers(0, 3, size=(w.B, w.N_max)).astype(np.float32) / 2.0
    worst, job, _ = h.lockstep(w, steps=20, override=ties, whole=lambda t: t % 2 == 1)
    job.adore.close()


@pytest.mark.parametrize("ordered", [True, False])
def test_decode_step_call_at_the_benchmark_shape(ordered):
    """llama7b_layer at full size through adore_decode_step, the call bench.py times, in both input orders."""
    h = _harness()
    w = workload("llama7b_layer").scaled(T=8)
    worst, job, _ = h.lockstep(w, steps=6, check_cache_every=3, whole=lambda t: True, ordered=ordered)
    job.adore.close()


# ---- input order: adore_set_input_order --------------------------------------------------------------
ORDER_W = dict(L=1, B=2, H=4, d=128, D=256, K=96, R=8, S=120, T=36, dtype="bf16", dprime=32)


@pytest.mark.parametrize("calls", ["whole", "fine", "mixed"])
def test_inputs_complete_at_call_time(calls):
    """With the input order switched off the side stream runs ahead of the caller's stream (its lists are rings);
    the trajectory is the oracle's all the same.  The harness synchronises before every call, as that mode asks."""
    h = _harness()
    w = Workload("order_" + calls, **ORDER_W)
    whole = {"whole": lambda t: True, "fine": None, "mixed": lambda t: (t // 3) % 2 == 0}[calls]
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=4, whole=whole, ordered=False)
    job.adore.close()


@pytest.mark.parametrize("ordered", [True, False])
def test_context_bound_to_a_stream_of_the_callers(ordered):
    """Everything above runs on the default stream.  A context created while another stream is current is bound to
    that stream (default priority): its inputs are produced there, its side streams order themselves against it,
    and the trajectory is the oracle's all the same, through the whole-step call and the fine-grained ones."""
    h = _harness()
    w = Workload("own_stream", **ORDER_W)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=4, whole=lambda t: (t // 3) % 2 == 0, ordered=ordered)
        assert job.adore.stream.cuda_stream == stream.cuda_stream != 0
        job.adore.close()
    torch.cuda.synchronize()


def test_input_order_switched_between_steps():
    h = _harness()
    w = Workload("order_switch", **ORDER_W)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=4, whole=lambda t: (t // 3) % 2 == 0,
                               ordered=lambda t: (t // 5) % 2 == 0)
    job.adore.close()


def test_inputs_complete_at_call_time_two_layers_rescore_and_forward():
    h = _harness()
    w = Workload("order_l2", L=2, B=2, H=4, d=64, D=128, K=72, R=6, S=90, T=20, dtype="bf16", dprime=32)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=5, ordered=False)
    job.adore.close()
    w = Workload("order_rescore", L=1, B=2, H=2, d=64, D=64, K=40, R=4, S=50, T=20, dtype="f32", dprime=16,
                 pos_scale=2.0 ** -5, rescore=True)
    worst, job, _ = h.lockstep(w, steps=w.T, ordered=False)
    job.adore.close()
    w = Workload("order_fwd", L=2, B=2, H=2, d=128, D=256, K=64, R=7, S=80, T=10, dtype="bf16", dprime=32)
    h.forward_lockstep(w, w.T, ordered=False)


@pytest.mark.parametrize("env", ["ADORE_NO_RIDE", "ADORE_NO_OVERLAP"])
@pytest.mark.parametrize("ordered", [True, False])
def test_decode_step_call_with_the_selections_as_kernels_of_their_own(env, ordered, monkeypatch):
    """adore_decode_step with the riding switched off (selections and controller on the side stream) and with the
    side stream switched off (everything on the caller's stream), mixed with the fine-grained calls."""
    monkeypatch.setenv(env, "1")
    h = _harness()
    w = Workload("ds_" + env.lower(), **ORDER_W)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=4, whole=lambda t: (t // 3) % 2 == 0, ordered=ordered)
    job.adore.close()


@pytest.mark.parametrize("ordered", [True, False])
def test_decode_step_call_with_the_rescoring_controller(ordered):
    """RESCORE mode never rides (every score changes at every step): adore_decode_step enqueues the side chain
    first, then the attention, then the rebuild."""
    h = _harness()
    w = Workload("ds_rescore", L=1, B=2, H=2, d=64, D=256, K=48, R=6, S=60, T=24, dtype="bf16", dprime=128,
                 pos_scale=2.0 ** -6, rescore=True)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=6, whole=lambda t: t % 3 != 2, ordered=ordered)
    job.adore.close()


def test_inputs_produced_on_the_stream_are_waited_for():
    """Default input order: x_n and score_override may be written by work that is still queued on the context's
    stream when the call is made.  One job gets its inputs complete; its twin gets them from copies enqueued
    behind milliseconds of other work into buffers that hold NaN until then.  Same bits in both."""
    import torch
    h = _harness()
    w = Workload("order_lazy", **dict(ORDER_W, T=12))
    ref = h.GpuJob(w)
    lazy = h.GpuJob(w, ref.inp, ref.wts)
    ref.init()
    lazy.init()
    rng = np.random.default_rng(5)
    busy = torch.randn((4096, 4096), device=h.DEV)
    x_buf = torch.empty((w.B, w.D), dtype=ref.st, device=h.DEV)
    for t in range(w.T):
        n = w.S + t
        whole = t % 2 == 0
        want = ref.step(n, whole=whole)
        x_buf.fill_(float("nan"))
        torch.cuda.synchronize()
        for _ in range(4):
            busy = torch.tanh(busy @ busy)          # a few milliseconds on the context's stream
        x_buf.copy_(lazy.hidden[0][:, n])
        got = lazy.step(n, whole=whole, x_n=x_buf)
        for g, r, what in zip(got, want, ("out", "slot map", "released", "rebuilt", "sigma")):
            if what in ("released", "rebuilt") and whole:
                continue                            # not reported by adore_decode_step
            assert np.array_equal(g, r), f"{what} at n={n}"
    ref.adore.close()
    lazy.adore.close()


@pytest.mark.parametrize("calls", ["whole", "fine"])
def test_first_steps_without_a_synchronise_after_the_init_when_inputs_are_not_ordered(calls):
    """Input order off (the side streams wait for nothing of a step's own): adore_init_cache and the first steps
    enqueued back to back with no synchronisation in between, every input prepared beforehand and every step with
    output buffers of its own.  The controller of the first step must still start behind the prompt scan (it reads
    the GRU state the scan leaves and reuses its scratch).  Same bits as the run that synchronises after every call."""
    h = _harness()
    w = Workload("order_init", **dict(ORDER_W, S=900, T=8))      # two prompt chunks: the scan alone takes ~0.7 ms
    inp = SyntheticInputs(w)
    ref = h.GpuJob(w, inp)
    ref.init()
    want = [ref.step(w.S + t, whole=calls == "whole") for t in range(w.T)]
    want_state = ref.snapshot()
    ref.adore.close()

    job = h.GpuJob(w, inp, ordered=False)
    st = job.st
    pk, pv = (h.to_dev(a, st) for a in job.prompt_np)
    ctrl = job.hidden[0][:, :w.S].contiguous()
    qkv = [[h.to_dev(a[0], st) for a in inp.step_qkv(w.S + t)] for t in range(w.T)]
    xs = [job.hidden[0][:, w.S + t].contiguous() for t in range(w.T)]
    outs = [torch.empty((w.B, w.H, w.d), dtype=torch.float32, device=h.DEV) for _ in range(w.T)]
    maps = [torch.empty((w.B, w.H, w.K), dtype=torch.int32, device=h.DEV) for _ in range(w.T)]
    torch.cuda.synchronize()
    job.adore.init_cache(pk, pv, job.hidden, ctrl, None, w.S)
    for t in range(w.T):
        q, k, v = qkv[t]
        if calls == "whole":
            job.adore.decode_step(q, k, v, job.hidden[0], xs[t], None, outs[t], maps[t])
        else:
            job.adore.attend(0, q, k, v, outs[t])
            job.adore.schedule(xs[t], None, maps[t], None, None)
            job.adore.rebuild(0, job.hidden[0])
    torch.cuda.synchronize()
    for t in range(w.T):
        assert np.array_equal(maps[t].cpu().numpy(), want[t][1]), f"slot map at step {t}"
        assert np.array_equal(outs[t].cpu().numpy().astype(np.float64), want[t][0][0]), f"output at step {t}"
    got_state = job.snapshot()
    assert np.array_equal(got_state["scores"][:, :w.S + w.T], want_state["scores"][:, :w.S + w.T])
    assert np.array_equal(got_state["z"], want_state["z"])
    job.adore.close()


@pytest.mark.parametrize("name,ordered,steps", [
    ("llama7b_layer", False, 48), ("llama7b_layer", True, 48), ("high_batch", False, 24), ("long_context", False, 24)])
def test_free_running_steps_as_the_benchmark_times_them(name, ordered, steps):
    """What bench.py times is a run of steps enqueued back to back with no synchronisation, at full size, most of
    them in the order-off mode: the side streams then run ahead through the rings of per-step lists and catch up at
    their periodic waits.  Here the same is done with every step keeping its outputs: the init and `steps` steps
    (several times round the rings) without a synchronisation in between must leave, step for step, the bits of a
    run that synchronises after every call (which is the run the oracle follows in the tests above)."""
    h = _harness()
    w = workload(name)
    inp = SyntheticInputs(w)
    st = h.storage_dtype(w)
    qkv = [[h.to_dev(a, st) for a in inp.step_qkv(w.S + t)] for t in range(steps)]

    def run(sync_every_call):
        job = h.GpuJob(w, inp, ordered=ordered)
        pk, pv = (h.to_dev(a, st) for a in job.prompt_np)
        ctrl = job.hidden[0][:, :w.S].contiguous()
        xs = [job.hidden[0][:, w.S + t].contiguous() for t in range(steps)]
        outs = [torch.empty((w.L, w.B, w.H, w.d), dtype=torch.float32, device=h.DEV) for _ in range(steps)]
        maps = [torch.empty((w.B, w.H, w.K), dtype=torch.int32, device=h.DEV) for _ in range(steps)]
        torch.cuda.synchronize()
        job.adore.init_cache(pk, pv, job.hidden, ctrl, None, w.S)
        for t in range(steps):
            if sync_every_call:
                torch.cuda.synchronize()
            q, k, v = qkv[t]
            if w.L == 1:
                job.adore.decode_step(q[0], k[0], v[0], job.hidden[0], xs[t], None, outs[t][0], maps[t])
            else:
                for l in range(w.L):
                    job.adore.attend(l, q[l], k[l], v[l], outs[t][l])
                job.adore.schedule(xs[t], None, maps[t], None, None)
                for l in range(w.L):
                    job.adore.rebuild(l, job.hidden[l])
        torch.cuda.synchronize()
        state = job.snapshot()
        result = ([o.cpu().numpy() for o in outs], [m.cpu().numpy() for m in maps], state)
        job.adore.close()
        return result

    want = run(True)
    got = run(False)
    for t in range(steps):
        assert np.array_equal(got[1][t], want[1][t]), f"slot map at step {t}"
        assert np.array_equal(got[0][t], want[0][t]), f"output at step {t}"
    assert np.array_equal(got[2]["slot_pos"], want[2]["slot_pos"])
    assert np.array_equal(got[2]["scores"][:, :w.S + steps], want[2]["scores"][:, :w.S + steps])
    occ = want[2]["slot_pos"] >= 0
    for key in ("cache_k", "cache_v"):
        for l in range(w.L):
            assert np.array_equal(got[2][key][l][occ], want[2][key][l][occ]), key


@pytest.mark.parametrize("ordered", [False, True])
def test_free_running_forward_steps_as_the_benchmark_times_them(ordered):
    """The same for adore_forward_step (bench.py --forward): two layers of the benchmark shape, 20 steps back to
    back against 20 steps with a synchronisation before each."""
    h = _harness()
    w = workload("llama7b_layer").scaled(L=2)
    steps = 20
    inp = SyntheticInputs(w)
    st = h.storage_dtype(w)
    wts = dict(inp.weights(), **inp.forward_weights())
    wq, wo = h.to_dev(wts["w_q"], st), h.to_dev(wts["w_o"], st)
    Ed = h.to_dev(inp.hidden_store_layer(0), st)
    pk, pv = (h.to_dev(a, st) for a in inp.prompt_kv())
    dev_w = h.device_weights(w, {k: v for k, v in wts.items() if k not in ("w_q", "w_o")})

    def run(sync_every_call):
        from paper_2407_02328_amd.binding import Adore
        adore = Adore(h.adore_config(w), dev_w, h.DEV)
        if not ordered:
            adore.set_input_order(False)
        rows = [torch.zeros((w.B, w.R + 1, w.D), dtype=st, device=h.DEV) for _ in range(steps)]
        maps = [torch.empty((w.B, w.H, w.K), dtype=torch.int32, device=h.DEV) for _ in range(steps)]
        rebuilt = [torch.empty((w.B, w.R), dtype=torch.int32, device=h.DEV) for _ in range(steps)]
        torch.cuda.synchronize()
        adore.init_cache(pk, pv, None, Ed[:, :w.S].contiguous(), None, w.S)
        for t in range(steps):
            if sync_every_call:
                torch.cuda.synchronize()
            adore.forward_step(wq, wo, Ed, None, rows[t], maps[t], None, rebuilt[t])
        torch.cuda.synchronize()
        state = adore.empty_state()
        adore.get_state(**state)
        torch.cuda.synchronize()
        result = ([r.float().cpu().numpy() for r in rows], [m.cpu().numpy() for m in maps],
                  [r.cpu().numpy() for r in rebuilt], {k: v.float().cpu().numpy() if v.dtype.is_floating_point else v.cpu().numpy()
                                                       for k, v in state.items()})
        adore.close()
        return result

    want = run(True)
    got = run(False)
    for t in range(steps):
        assert np.array_equal(got[1][t], want[1][t]), f"slot map at step {t}"
        assert np.array_equal(got[2][t], want[2][t]), f"rebuilt positions at step {t}"
        assert np.array_equal(got[0][t], want[0][t]), f"rows at step {t}"
    assert np.array_equal(got[3]["slot_pos"], want[3]["slot_pos"])
    occ = want[3]["slot_pos"] >= 0
    for key in ("cache_k", "cache_v"):
        for l in range(w.L):
            assert np.array_equal(got[3][key][l][occ], want[3][key][l][occ]), key


# ---- a sweep of random small shapes ----------------------------------------------------------------------
def _random_workloads(count, seed):
    """Small shapes drawn at random within what the library documents as supported: every axis ragged against the
    kernels' tiles (K against 64 slots per wave, B against 16 sequences per controller tile, H against 4 heads per
    release workgroup, R + 1 against the free list, S on both sides of the cache size)."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        d = int(rng.choice([64, 128]))
        dtype = str(rng.choice(["bf16", "bf16", "f32"]))
        K = int(rng.integers(4, 260))
        R = int(rng.integers(0, min(K - 2, 40) + 1))
        L = int(rng.choice([1, 1, 2, 3]))
        S = int(rng.integers(1, 2 * K + 2))
        kw = dict(L=L, B=int(rng.integers(1, 6)), H=int(rng.integers(1, 7)), d=d,
                  D=int(rng.choice([64, 128, 192, 256, 384])), K=K, R=R, S=S, T=int(rng.integers(6, 14)),
                  dtype=dtype, dprime=int(rng.choice([8, 32, 128])))
        out.append((f"rand{i}", kw, str(rng.choice(["fine", "whole", "mixed"])) if L == 1 else "fine",
                    bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("name,kw,calls,ordered", _random_workloads(64, 20240702))
def test_random_small_configurations(name, kw, calls, ordered):
    h = _harness()
    w = Workload(name, **kw)
    whole = {"fine": None, "whole": lambda t: True, "mixed": lambda t: t % 3 != 1}[calls]
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=3, whole=whole, ordered=ordered)
    job.adore.close()


def _random_rescore_workloads(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        K = int(rng.integers(6, 120))
        out.append((f"rrand{i}", dict(L=int(rng.choice([1, 2])), B=int(rng.integers(1, 4)), H=int(rng.integers(1, 5)),
                                      d=int(rng.choice([64, 128])), D=int(rng.choice([64, 128, 256])), K=K,
                                      R=int(rng.integers(0, min(K - 2, 12) + 1)), S=int(rng.integers(1, 2 * K)),
                                      T=int(rng.integers(6, 12)), dtype=str(rng.choice(["bf16", "f32"])),
                                      dprime=int(rng.choice([8, 32, 128])), pos_scale=2.0 ** -int(rng.integers(3, 8)),
                                      rescore=True)))
    return out


@pytest.mark.parametrize("name,kw", _random_rescore_workloads(12, 7))
def test_random_small_configurations_rescore(name, kw):
    h = _harness()
    w = Workload(name, **kw)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=4, whole=(lambda t: t % 2 == 0) if w.L == 1 else None)
    job.adore.close()


def _random_forward_workloads(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        d = int(rng.choice([64, 128]))
        H = int(rng.choice([2, 4, 6] if d == 64 else [1, 2, 3, 4]))
        K = int(rng.integers(8, 220))
        out.append((f"frand{i}", dict(L=int(rng.choice([1, 2, 3])), B=int(rng.integers(1, 20)), H=H, d=d,
                                      D=int(rng.choice([128, 256, 384, 512])), K=K,
                                      R=int(rng.integers(0, min(K - 2, 63) + 1)), S=int(rng.integers(1, 2 * K)),
                                      T=int(rng.integers(4, 9)))))
    return out


@pytest.mark.parametrize("name,kw", _random_forward_workloads(16, 11))
def test_random_small_configurations_forward(name, kw):
    h = _harness()
    # weights scaled with the width (each projection about norm-preserving, as in the fixed cases above at D = 256):
    # with larger ones the rows grow from layer to layer, the softmax sharpens, and what the test then measures is
    # how three layers amplify a one-unit rounding difference, not whether a layer is computed correctly
    w = Workload(name, dtype="bf16", dprime=32, w_std=0.96 / np.sqrt(kw["D"]), **kw)
    worst, mean = h.forward_lockstep(w, w.T)
    assert mean < 2.0 ** -10


def _random_medium_workloads(count, seed):
    """Shapes between the small cases and the benchmark's: several GEMM tiles per axis (all five tile shapes get
    picked across the sweep), rows of up to 1024 slots, more than 16 sequences."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        K = int(rng.integers(200, 1025))
        R = int(rng.integers(8, 49))
        out.append((f"mrand{i}", dict(L=1, B=int(rng.integers(1, 25)), H=int(rng.integers(4, 17)), d=128,
                                      D=int(rng.choice([512, 1024, 2048])), K=K, R=R,
                                      S=int(rng.integers(K // 2, 2 * K)), T=5, dtype="bf16", dprime=128),
                    str(rng.choice(["fine", "whole", "mixed"])), bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("name,kw,calls,ordered", _random_medium_workloads(10, 3))
def test_random_medium_configurations(name, kw, calls, ordered):
    h = _harness()
    w = Workload(name, **kw)
    whole = {"fine": None, "whole": lambda t: True, "mixed": lambda t: t % 3 != 1}[calls]
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=2, whole=whole, ordered=ordered)
    job.adore.close()


# ---- rotary position embedding on the keys (and forward queries) the library makes ------------------
@pytest.mark.parametrize("name,kw,calls", [
    # fp32, one wave per output element, head_dim 64
    ("f32_d64", dict(L=1, B=2, H=2, d=64, D=128, K=40, R=6, S=50, T=20, dtype="f32", dprime=16), "fine"),
    # fp32, head_dim 128, the whole-step call
    ("f32_d128", dict(L=1, B=2, H=2, d=128, D=128, K=80, R=4, S=100, T=16, dtype="f32", act_std=0.3, w_std=0.1), "whole"),
    # bf16 on the tile kernel, ragged tiles, two layers through the fine-grained calls
    ("bf16_d64_l2", dict(L=2, B=2, H=4, d=64, D=256, K=96, R=8, S=120, T=24, dtype="bf16", dprime=32), "fine"),
    # bf16, d = 128, the whole-step call with the selections riding; positions beyond 1000
    ("bf16_d128", dict(L=1, B=3, H=4, d=128, D=512, K=200, R=20, S=1050, T=20, dtype="bf16", dprime=32), "whole"),
    # a prompt shorter than the cache: the rebuild set grows from nothing
    ("bf16_warm", dict(L=1, B=2, H=9, d=64, D=256, K=130, R=12, S=20, T=40, dtype="bf16", dprime=32), "whole"),
])
def test_rotary_embedding_on_rebuilt_keys(name, kw, calls):
    """rope_base = 10000: every rebuilt key row is the rounded projection turned to its token's position; slot
    maps, outputs and cache rows against the oracle (its rotation is pinned on the CPU)."""
    h = _harness()
    w = Workload("rope_" + name, rope_base=10000.0, **kw)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=4, whole=(lambda t: True) if calls == "whole" else None)
    print(f"rope {name}: worst output error {worst:.3e}", flush=True)
    job.adore.close()


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("d", [64, 128])
def test_rotary_embedding_with_every_tile_shape(tile, d, monkeypatch):
    """The key tiles turn their rows themselves when a tile holds whole heads (256- to 64-wide tiles at d = 64,
    256- and 128-wide ones at d = 128); narrower tiles leave it to the pass that follows.  Both give the same rows."""
    h = _harness()
    monkeypatch.setenv("ADORE_GEMM_TILE", str(tile))
    w = Workload("rope_tiles", L=1, B=3, H=512 // d, d=d, D=448, K=128, R=45, S=200, T=4, dtype="bf16", dprime=32,
                 rope_base=10000.0)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=1)
    job.adore.close()


def test_rotary_embedding_changes_the_keys_and_nothing_else():
    """The same job with and without the embedding on the GPU: selections and value rows agree, rebuilt key
    rows differ (so the tests above do not pass by the rotation being skipped on both sides)."""
    h = _harness()
    kw = dict(L=1, B=2, H=4, d=128, D=256, K=96, R=8, S=120, T=10, dtype="bf16", dprime=32)
    snaps = []
    for base in (0.0, 500.0):
        w = Workload("rope_onoff", rope_base=base, **kw)
        worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=5)
        snaps.append(job.snapshot())
        job.adore.close()
    a, b = snaps
    assert np.array_equal(a["slot_pos"], b["slot_pos"]) and np.array_equal(a["cache_v"], b["cache_v"])
    assert not np.array_equal(a["cache_k"], b["cache_k"])


@pytest.mark.parametrize("name,kw", [
    ("r8_d64", dict(L=3, B=2, H=4, d=64, D=256, K=64, R=8, S=40, T=30)),
    ("r32_d128", dict(L=2, B=2, H=4, d=128, D=512, K=160, R=32, S=200, T=10)),
    ("r0", dict(L=2, B=2, H=2, d=64, D=128, K=48, R=0, S=60, T=8)),
    ("b18", dict(L=2, B=18, H=2, d=128, D=256, K=64, R=4, S=70, T=5)),
])
def test_forward_step_with_rotary_embedding(name, kw):
    """Rebuild forward with rope_base = 10000: queries and keys of the R+1 rows of every layer are turned to
    their positions (rebuilt tokens: their own; current token: n)."""
    h = _harness()
    w = Workload("fwd_rope_" + name, dtype="bf16", dprime=32, w_std=0.06, rope_base=10000.0, **kw)
    worst, mean = h.forward_lockstep(w, w.T)
    print(f"forward rope {name}: worst row error {worst:.2e}, mean {mean:.2e}", flush=True)
    assert mean < 2.0 ** -10


def test_rotary_embedding_at_the_benchmark_shape():
    """llama7b_layer with the embedding on, in the launch configuration bench.py times: init and four steps
    through adore_decode_step, everything against the oracle (16384 rebuilt key rows per step)."""
    h = _harness()
    w = workload("llama7b_layer").scaled(T=6, rope_base=10000.0)
    worst, job, _ = h.lockstep(w, steps=4, check_cache_every=2, whole=lambda t: True)
    print(f"rope llama7b_layer: worst output error {worst:.3e}", flush=True)
    job.adore.close()


def test_rotary_embedding_in_a_context_restored_without_an_init():
    """A snapshot taken from one context and restored into a fresh one (adore_set_state with no adore_init_cache
    before it): the next steps give the same bits, so the angle table is there although no init made it."""
    h = _harness()
    w = Workload("rope_snap", L=1, B=2, H=2, d=64, D=128, K=40, R=4, S=60, T=12, dtype="bf16", dprime=32,
                 rope_base=10000.0)
    inp = SyntheticInputs(w)
    job = h.GpuJob(w, inp)
    job.init()
    for n in range(w.S, w.S + 4):
        job.step(n)
    saved = {k: v.clone() for k, v in job.state.items()}
    step = job.adore.get_state(**saved)
    torch.cuda.synchronize()
    ref = [job.step(n) for n in range(w.S + 4, w.S + 8)]
    ref_k = job.snapshot()["cache_k"]
    fresh = h.GpuJob(w, inp)
    fresh.adore.set_state(saved["slot_pos"], saved["scores"], saved["z"], saved["cache_k"], saved["cache_v"], step)
    again = [fresh.step(n) for n in range(w.S + 4, w.S + 8)]
    for a, b in zip(ref, again):
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    occ = job.snapshot()["slot_pos"] >= 0
    assert np.array_equal(ref_k[0][occ], fresh.snapshot()["cache_k"][0][occ])
    job.adore.close(); fresh.adore.close()


# ---- the sweeps of random shapes again with the rotary embedding on --------------------------------
@pytest.mark.parametrize("name,kw,calls,ordered", _random_workloads(24, 515))
def test_random_small_configurations_with_rotary_embedding(name, kw, calls, ordered):
    h = _harness()
    w = Workload(name, rope_base=float(10 ** (2 + len(name) % 3)), **kw)        # bases 100, 1000, 10000
    whole = {"fine": None, "whole": lambda t: True, "mixed": lambda t: t % 3 != 1}[calls]
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=3, whole=whole, ordered=ordered)
    job.adore.close()


@pytest.mark.parametrize("name,kw", _random_rescore_workloads(6, 99))
def test_random_small_configurations_rescore_with_rotary_embedding(name, kw):
    h = _harness()
    w = Workload(name, rope_base=10000.0, **kw)
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=4, whole=(lambda t: t % 2 == 0) if w.L == 1 else None)
    job.adore.close()


@pytest.mark.parametrize("name,kw", _random_forward_workloads(12, 23))
def test_random_small_configurations_forward_with_rotary_embedding(name, kw):
    """Widths H*d that are multiples of 256 turn the current tokens' rows inside the projection launch (whole heads
    per workgroup, or not: then the pass of its own), the others go through the pass; tiles wide and narrow."""
    h = _harness()
    w = Workload(name, dtype="bf16", dprime=32, w_std=0.96 / np.sqrt(kw["D"]), rope_base=10000.0, **kw)
    worst, mean = h.forward_lockstep(w, w.T)
    assert mean < 2.0 ** -10


@pytest.mark.parametrize("name,kw,calls,ordered", _random_medium_workloads(4, 41))
def test_random_medium_configurations_with_rotary_embedding(name, kw, calls, ordered):
    h = _harness()
    w = Workload(name, rope_base=10000.0, **kw)
    whole = {"fine": None, "whole": lambda t: True, "mixed": lambda t: t % 3 != 1}[calls]
    worst, job, _ = h.lockstep(w, steps=w.T, check_cache_every=2, whole=whole, ordered=ordered)
    job.adore.close()
