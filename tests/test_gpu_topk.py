"""GPU parity of adore_topk_attention (top-K attention over a whole sequence) against the oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _mods():
    import torch
    from oracle import adore_oracle as O
    from paper_2407_02328_amd import topk_attention
    return torch, O, topk_attention


def _to_gpu(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0").to(torch.bfloat16).contiguous()


def _bf16_values(torch, a):
    """The values a bf16 tensor holds, as fp64 (so that the oracle sees what the GPU sees)."""
    return _to_gpu(torch, a).float().cpu().numpy().astype(np.float64)


def _row_err(got, want):
    return np.abs(got - want).max(axis=-1) / np.maximum(np.abs(want).max(axis=-1), 1e-30)


BAND = 1e-3      # weights closer than this may change places between fp32 and fp64 accumulation (a hundred times the
                 # fp32 error of a d-term sum of products of unit-variance values)
TOL = 2e-3 + 2.0 ** -8      # the attention tolerance + the rounding of the bf16 output


def _check_rows_allowing_swaps_at_the_cut(O, q, k, v, got, top_k, what):
    """q, k, v, got: [rows, S, d] fp64.  The GPU decides on fp32 weights, the oracle on fp64 ones.  A query whose
    K-th and (K+1)-th largest weights are more than BAND apart has one kept set, and its row must meet TOL against
    the oracle's.  For the others the kept sets a decision on weights perturbed by less than BAND / 2 can reach are
    listed: a key stays for certain if fewer than K others come within BAND of it from above, goes for certain if K
    others beat it by more than BAND, and the keys in between fill the remaining places in every combination; the
    GPU's row must meet TOL against the oracle's softmax and value sum over ONE of these sets."""
    import itertools
    rows, S, d = q.shape
    want, _ = O.topk_attention(q, k, v, top_k)
    e = _row_err(got, want)
    unclear, worst_unclear = 0, 0.0
    for r in range(rows):
        for i in range(top_k, S):
            w = k[r, :i + 1] @ q[r, i]
            srt = np.sort(w)[::-1]
            if srt[top_k - 1] - srt[top_k] > BAND:
                assert e[r, i] < TOL, f"{what}: row {r} query {i}: {e[r, i]}"
                continue
            unclear += 1
            n_ge = lambda x: int(np.searchsorted(-srt, -x, side="right"))       # how many weights are >= x
            n_gt = lambda x: int(np.searchsorted(-srt, -x, side="left"))        # ... > x
            sure = [j for j in range(i + 1) if n_ge(w[j] - BAND) <= top_k]
            band = [j for j in range(i + 1) if n_ge(w[j] - BAND) > top_k and n_gt(w[j] + BAND) < top_k]
            need = top_k - len(sure)
            assert 0 <= need <= len(band) and len(band) <= 12, (len(sure), len(band))
            best = np.inf
            for comb in itertools.combinations(band, need):
                sel = np.array(sorted(sure + list(comb)))
                out = O.softmax_row(w[sel] / np.sqrt(np.float64(d))) @ v[r, sel]
                best = min(best, float(np.abs(got[r, i] - out).max() / np.abs(out).max()))
            worst_unclear = max(worst_unclear, best)
            assert best < TOL, f"{what}: row {r} query {i}: no kept set within the band gives the GPU's row ({best})"
        for i in range(min(top_k, S)):
            assert e[r, i] < TOL, f"{what}: row {r} query {i}: {e[r, i]}"
    print(f"{what}: worst row {e.max():.2e} against the oracle's own sets; {unclear} queries with a tie within {BAND} at "
          f"the cut, worst of them against their best admissible set {worst_unclear:.2e}", flush=True)
    assert unclear <= 0.1 * rows * S


GRID_CASES = [
    # rows, S, d, top_k
    (2, 1, 64, 1),            # a single token
    (3, 17, 64, 5),           # one ragged query block
    (2, 100, 128, 1),         # K = 1: the value row of the largest weight
    (2, 100, 128, 32),
    (1, 257, 128, 96),        # ragged tail of one query and one key
    (2, 600, 64, 96),         # several query blocks, every wave has several key blocks
    (1, 300, 128, 1000),      # K beyond the sequence: plain causal attention
    (1, 1024, 128, 96),       # the longest rows a lane holds as 16 keys
    (1, 1100, 64, 200),       # 32 keys per lane
    (1, 2048, 128, 300),      # the longest sequence whose weights stay in LDS
    (1, 2049, 64, 300),       # one more: the weights of a query block go through the workspace
    (2, 3000, 128, 96),       # ... several 64-key groups per lane pass, a ragged last one
    (2, 200, 64, 64),         # K a multiple of the wave: the cut falls on a lane boundary
    (11, 70, 64, 20),         # one whole group of 8 rows (one per XCD) and a tail of 3
]


@pytest.mark.parametrize("rows,S,d,top_k", GRID_CASES)
def test_topk_attention_on_exactly_representable_weights(rows, S, d, top_k):
    """q and k on a grid of quarters in [-2, 2]: every product sum is exact in fp32 and in fp64, so both sides
    select from identical weights, equal weights abound (the tie rule decides many rows) and the kept sets are
    the same; the outputs then differ by the arithmetic of the softmax and the second product only."""
    torch, O, topk_attention = _mods()
    rng = np.random.default_rng(1000 * S + top_k)
    q = rng.integers(-8, 9, size=(rows, S, d)) / 4.0
    k = rng.integers(-8, 9, size=(rows, S, d)) / 4.0
    v = _bf16_values(torch, rng.standard_normal((rows, S, d)))
    want, kept = O.topk_attention(q, k, v, top_k)
    got = topk_attention(_to_gpu(torch, q), _to_gpu(torch, k), _to_gpu(torch, v), top_k)
    torch.cuda.synchronize()
    e = _row_err(got.float().cpu().numpy().astype(np.float64), want)
    print(f"grid rows={rows} S={S} d={d} K={top_k}: worst row error {e.max():.2e}", flush=True)
    assert e.max() < TOL


@pytest.mark.parametrize("rows,S,d,top_k", [(2, 500, 128, 96), (2, 333, 64, 48), (1, 1500, 128, 512), (1, 2600, 128, 700)])
def test_topk_attention_on_gaussian_inputs(rows, S, d, top_k):
    """Gaussian q, k, v.  The GPU takes its decision on fp32 weights, the oracle on fp64 ones: where the K-th and
    the (K+1)-th largest weight of a query are further apart than the fp32 accumulation error can bridge, the kept
    sets are the same and the output must agree to the attention tolerance; for the few other queries the GPU's row
    must be the oracle's attention over one of the kept sets that differ only in keys within that distance of the cut."""
    torch, O, topk_attention = _mods()
    rng = np.random.default_rng(7 * S + top_k)
    q, k, v = (_bf16_values(torch, rng.standard_normal((rows, S, d))) for _ in range(3))
    got = topk_attention(_to_gpu(torch, q), _to_gpu(torch, k), _to_gpu(torch, v), top_k).float().cpu().numpy().astype(np.float64)
    torch.cuda.synchronize()
    _check_rows_allowing_swaps_at_the_cut(O, q, k, v, got, top_k, f"gauss rows={rows} S={S} K={top_k}")


def test_topk_attention_at_the_benchmark_shape_sampled_rows():
    """B16 x H32 rows of 1024 tokens, head_dim 128, K = 96 (the paper's fine-tuning setting), as bench.py
    --topk-attention times it: eight rows checked in full against the oracle, Gaussian inputs drawn on the device."""
    torch, O, topk_attention = _mods()
    from gen import DeviceNormals
    rows, S, d, top_k = 512, 1024, 128, 96
    drawer = DeviceNormals(20240702, "cuda:0")
    q, k, v = (drawer.normal((rows, S, d), 1.0, torch.bfloat16) for _ in range(3))
    got = topk_attention(q, k, v, top_k)
    torch.cuda.synchronize()
    pick = [0, 1, 63, 200, 255, 256, 400, 511]
    sel = torch.tensor(pick, device="cuda:0")
    q64, k64, v64 = (t[sel].float().cpu().numpy().astype(np.float64) for t in (q, k, v))
    _check_rows_allowing_swaps_at_the_cut(O, q64, k64, v64, got[sel].float().cpu().numpy().astype(np.float64), top_k,
                                          "benchmark shape")


def test_topk_attention_rejects_what_it_does_not_take():
    torch, O, topk_attention = _mods()
    from paper_2407_02328_amd import AdoreError
    q = torch.zeros((1, 8, 96), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(AdoreError):
        topk_attention(q, q, q, 4)                      # head_dim 96
    q = torch.zeros((1, 32769, 64), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(AdoreError):
        topk_attention(q, q, q, 4)                      # sequence longer than the entry point takes
    q = torch.zeros((1, 8, 64), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(AdoreError):
        topk_attention(q, q, q, 0)
    with pytest.raises(AdoreError):
        topk_attention(q, q, q, 4, workspace=torch.empty(16, dtype=torch.uint8, device="cuda:0"))


def _random_topk_cases(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        S = int(rng.integers(1, 700))
        out.append((int(rng.integers(1, 12)), S, int(rng.choice([64, 128])), int(rng.integers(1, S + 40)),
                    int(rng.choice([1, 2, 4, 8]))))
    return out


@pytest.mark.parametrize("rows,S,d,top_k,levels", _random_topk_cases(24, 2407))
def test_topk_attention_random_shapes_on_exactly_representable_weights(rows, S, d, top_k, levels):
    """Random shapes; q and k on grids of `levels` steps per unit (coarse grids: most weights of a query tie, so
    the cut among equal weights decides nearly every row; fine grids: few ties)."""
    torch, O, topk_attention = _mods()
    rng = np.random.default_rng(rows * 100003 + S * 17 + top_k)
    q = rng.integers(-2 * levels, 2 * levels + 1, size=(rows, S, d)) / float(levels)
    k = rng.integers(-2 * levels, 2 * levels + 1, size=(rows, S, d)) / float(levels)
    if levels == 1:                        # very coarse: make whole runs of keys identical
        k[:, ::3] = k[:, :1]
    v = _bf16_values(torch, rng.standard_normal((rows, S, d)))
    want, kept = O.topk_attention(q, k, v, top_k)
    got = topk_attention(_to_gpu(torch, q), _to_gpu(torch, k), _to_gpu(torch, v), top_k)
    torch.cuda.synchronize()
    e = _row_err(got.float().cpu().numpy().astype(np.float64), want)
    assert e.max() < TOL, f"rows={rows} S={S} d={d} K={top_k} levels={levels}: {e.max()}"


@pytest.mark.timeout(900)
def test_topk_attention_at_the_long_context_shape_sampled_rows():
    """B4 x H32 rows of 8192 tokens (the long-context workload's prompts), K = 96: the weights of a query block go
    through the workspace, one piece per workgroup in flight (0.3 GB in all).  Two rows that sit on different XCDs
    checked in full against the oracle."""
    torch, O, topk_attention = _mods()
    from gen import DeviceNormals
    from paper_2407_02328_amd import load_library
    rows, S, d, top_k = 128, 8192, 128, 96
    assert load_library().adore_topk_attention_workspace_bytes(rows, S, d) < (1 << 30)
    drawer = DeviceNormals(20240703, "cuda:0")
    q, k, v = (drawer.normal((rows, S, d), 1.0, torch.bfloat16) for _ in range(3))
    got = topk_attention(q, k, v, top_k)
    torch.cuda.synchronize()
    pick = [77, 122]
    sel = torch.tensor(pick, device="cuda:0")
    q64, k64, v64 = (t[sel].float().cpu().numpy().astype(np.float64) for t in (q, k, v))
    _check_rows_allowing_swaps_at_the_cut(O, q64, k64, v64, got[sel].float().cpu().numpy().astype(np.float64), top_k,
                                          "long-context shape")
