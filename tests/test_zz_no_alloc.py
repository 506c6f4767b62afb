"""The top-K attention entry point that allocates nothing (adore_topk_attention_static) against the one that
takes a workspace: same bits, on two calls in a row, the second with a smaller input (so whatever the first call
left in the library's fixed scratch array is still there when the second runs)."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _raw_static_call(lib, q, k, v, out, top_k, stream):
    rows, seq, d = q.shape
    return lib.adore_topk_attention_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), rows, seq, d,
                                           top_k, stream)


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    import torch
    from gen import DeviceNormals
    from oracle import adore_oracle as O
    from paper_2407_02328_amd import load_library, topk_attention
    lib = load_library()
    dev = "cuda:0"
    drawer = DeviceNormals(2407, dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    # (rows, seq, head_dim, top_k): the first fills 60 MiB of the 64 MiB array, the second is smaller and ragged
    for rows, S, d, top_k in [(240, 1000, 128, 96), (3, 333, 64, 48)]:
        q, k, v = (drawer.normal((rows, S, d), 1.0, torch.bfloat16) for _ in range(3))
        want = topk_attention(q, k, v, top_k)
        got = torch.full_like(q, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated(dev)
        assert _raw_static_call(lib, q, k, v, got, top_k, stream) == 0
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated(dev) == before
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (rows, S, d, top_k)
        # and against the oracle, on the rows it finishes in seconds (the bar of the other top-K tests)
        sel = [0, rows - 1]
        q64, k64, v64 = (t[sel].float().cpu().numpy().astype(np.float64) for t in (q, k, v))
        from tests.test_gpu_topk import _check_rows_allowing_swaps_at_the_cut
        _check_rows_allowing_swaps_at_the_cut(O, q64, k64, v64, got[sel].float().cpu().numpy().astype(np.float64), top_k,
                                              f"static rows={rows} S={S}")


def test_static_scratch_entry_point_rejects_what_exceeds_its_array():
    import torch
    from paper_2407_02328_amd import load_library
    lib = load_library()
    dev = "cuda:0"
    stream = torch.cuda.current_stream(dev).cuda_stream
    t = torch.zeros((1, 2049, 64), dtype=torch.bfloat16, device=dev)          # needs the quadratic row buffer
    assert _raw_static_call(lib, t, t, t, torch.empty_like(t), 4, stream) == -4
    t = torch.zeros((300, 1024, 128), dtype=torch.bfloat16, device=dev)        # 75 MiB transposed copy
    assert _raw_static_call(lib, t, t, t, torch.empty_like(t), 4, stream) == -4
    t = torch.zeros((2, 16, 64), dtype=torch.bfloat16, device=dev)
    assert _raw_static_call(lib, t, t, t, torch.empty_like(t), 0, stream) == -1
    assert lib.adore_topk_attention_static(None, t.data_ptr(), t.data_ptr(), t.data_ptr(), 2, 16, 64, 4, stream) == -1
    torch.cuda.synchronize()
