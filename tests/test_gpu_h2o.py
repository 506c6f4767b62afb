"""GPU parity of the H2O(Rebuilt) score mode (Sec. 3.1, baselines 6 and 7) against its oracle: the scores every
head accumulates from its own attention within tolerance and then adopted; per-head slot maps, released and
rebuilt positions bit-exact; outputs within the attention tolerance; rebuilt rows within one storage unit."""
import numpy as np
import pytest

from gen import Workload, workload

pytestmark = pytest.mark.gpu


def _harness():
    from tests import gpu_harness
    return gpu_harness


@pytest.mark.parametrize("name,kw,calls", [
    # fp32, d = 64, a prompt longer than the cache
    ("f32_d64", dict(B=2, H=3, d=64, D=128, K=24, R=4, S=40, T=40, dtype="f32", dprime=16), "fine"),
    # bf16, d = 128, ragged K, the GEMM tile ragged, whole-step calls
    ("bf16_d128", dict(B=3, H=4, d=128, D=512, K=200, R=5, S=260, T=30, dtype="bf16", dprime=32), "whole"),
    # a prompt shorter than the cache: nothing is evicted at first, then heads start to differ
    ("warm", dict(B=2, H=9, d=64, D=256, K=40, R=6, S=5, T=70, dtype="bf16", dprime=32), "mixed"),
    # the largest row the release takes, rows split over several workgroups
    ("k1024", dict(B=1, H=4, d=128, D=256, K=1024, R=40, S=1100, T=8, dtype="bf16", dprime=32), "whole"),
    # no rebuild budget: plain H2O
    ("r0", dict(B=2, H=2, d=64, D=64, K=16, R=0, S=30, T=20, dtype="f32", dprime=16), "fine"),
])
def test_h2o_trajectory_matches_the_oracle(name, kw, calls):
    h = _harness()
    w = Workload("h2o_" + name, L=1, h2o=True, **kw)
    rng = np.random.default_rng(3)
    init = rng.random((w.B, w.H, w.S)).astype(np.float32)        # what the prompt's own attention would have left
    whole = {"fine": None, "whole": lambda t: True, "mixed": lambda t: t % 3 != 1}[calls]
    worst, job, orc, differ = h.h2o_lockstep(w, w.T, score_init=init, whole=whole, check_cache_every=5)
    print(f"h2o {name}: worst output error {worst:.2e}, heads held different tokens at {differ} of {w.T} steps", flush=True)
    if w.H > 1 and w.T >= 20:
        assert differ > 0          # the slot maps really are per head
    job.adore.close()


def test_h2o_uniform_attention_closed_form_on_gpu():
    """q = 0 from zero prompt scores: every probability is 1 / (rows held), all sums tie exactly, and the tie rule
    alone decides: each head holds tokens 0 .. m-2 and the current one, tokens m-1 .. m+R-2 are rebuilt at every
    step (the closed form the oracle is pinned with)."""
    h = _harness()
    w = Workload("h2o_uniform", L=1, B=2, H=3, d=64, D=128, K=16, R=3, S=40, T=25, dtype="f32", dprime=16, h2o=True)
    worst, job, orc, differ = h.h2o_lockstep(w, w.T, zero_queries=True)
    m = w.K - w.R - 1
    sm = job.slot_map.cpu().numpy()
    n = w.S + w.T - 1
    for b in range(w.B):
        for hh in range(w.H):
            assert sorted(int(p) for p in sm[b, hh] if p >= 0) == list(range(m - 1 + w.R)) + [n]
    assert differ == 0
    job.adore.close()


def test_h2o_ties_on_a_coarse_grid_of_prompt_scores():
    """Prompt scores drawn from four values: the first releases and choices are decided by position."""
    h = _harness()
    w = Workload("h2o_ties", L=1, B=2, H=4, d=64, D=128, K=24, R=5, S=70, T=12, dtype="f32", dprime=16, h2o=True)
    rng = np.random.default_rng(17)
    init = (rng.integers(0, 4, size=(w.B, w.H, w.S)) / 4.0).astype(np.float32)
    worst, job, orc, differ = h.h2o_lockstep(w, w.T, score_init=init, check_cache_every=4)
    job.adore.close()


def test_h2o_at_the_benchmark_shape():
    """llama7b_layer (B16 H32 d128 D4096 K512 R32, prompt 1024) in H2O mode: init and five steps through
    adore_decode_step, 512 slot maps of 512 slots each, every output row and every rebuilt row against the oracle."""
    h = _harness()
    w = workload("llama7b_layer").scaled(T=6, h2o=True)
    rng = np.random.default_rng(23)
    init = rng.random((w.B, w.H, w.S)).astype(np.float32)
    worst, job, orc, differ = h.h2o_lockstep(w, 5, score_init=init, whole=lambda t: True)
    print(f"h2o llama7b_layer: worst output error {worst:.2e}, heads differ at {differ} of 5 steps", flush=True)
    assert differ == 5
    job.adore.close()


def _random_h2o_workloads(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        K = int(rng.integers(4, 260))
        R = int(rng.integers(0, min(K - 2, 40) + 1))
        kw = dict(B=int(rng.integers(1, 5)), H=int(rng.integers(1, 10)), d=int(rng.choice([64, 128])),
                  D=int(rng.choice([64, 128, 256])), K=K, R=R, S=int(rng.integers(1, 2 * K + 2)), T=int(rng.integers(6, 14)),
                  dtype=str(rng.choice(["bf16", "f32"])), dprime=16)
        out.append((f"hrand{i}", kw, str(rng.choice(["fine", "whole", "mixed"]))))
    return out


@pytest.mark.parametrize("name,kw,calls", _random_h2o_workloads(24, 2024))
def test_h2o_random_small_configurations(name, kw, calls):
    h = _harness()
    w = Workload(name, L=1, h2o=True, **kw)
    rng = np.random.default_rng(len(name) + w.K)
    init = rng.random((w.B, w.H, w.S)).astype(np.float32) if w.K % 2 else None
    whole = {"fine": None, "whole": lambda t: True, "mixed": lambda t: t % 3 != 1}[calls]
    worst, job, orc, differ = h.h2o_lockstep(w, w.T, score_init=init, whole=whole, check_cache_every=3)
    job.adore.close()


def test_h2o_mode_rejects_what_it_does_not_take():
    h = _harness()
    import torch
    from paper_2407_02328_amd import AdoreError
    w = Workload("h2o_api", L=1, B=1, H=2, d=64, D=64, K=16, R=2, S=20, T=4, dtype="f32", dprime=16, h2o=True)
    job = h.GpuJob(w)
    job.init()
    q, k, v = (h.to_dev(a[0], job.st) for a in job.inp.step_qkv(w.S))
    ov = torch.zeros(w.B, dtype=torch.float32, device="cuda:0")
    with pytest.raises(AdoreError) as e:        # scores come from the attention: no override in a step
        job.adore.decode_step(q, k, v, job.hidden[0], None, ov, job.out[0], None)
    assert e.value.code == -1
    with pytest.raises(AdoreError) as e:
        job.adore.set_state(job.state["slot_pos"], None, None, None, None, w.S)
    assert e.value.code == -3
    job.adore.decode_step(q, k, v, job.hidden[0], None, None, job.out[0], None)     # x_n is not read in this mode
    torch.cuda.synchronize()
    job.adore.close()
