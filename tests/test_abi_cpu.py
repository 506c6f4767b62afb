"""Host-side checks of the C-ABI library that need no GPU: it loads, exports what the header
declares, sizes its workspace, and rejects bad arguments and out-of-order calls before touching
any device memory (the pointers used here are never dereferenced on the host)."""
import ctypes
import os
import re

import pytest

from gen import workload
from paper_2407_02328_amd import EXPORTS, LIB_PATH, load_library
from paper_2407_02328_amd.binding import AdoreConfig, AdoreWeights, make_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000       # 256-byte aligned, never dereferenced


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB_PATH):
        from paper_2407_02328_amd.build import build_library
        build_library()
    return load_library()


def cfg_for(w, **kw):
    base = dict(layers=w.L, batch=w.B, heads=w.H, head_dim=w.d, hidden=w.D, cache_slots=w.K,
                rebuild_budget=w.R, max_positions=w.N_max, ctrl_hidden=w.dprime, dtype=w.dtype,
                pos_scale=w.pos_scale)
    base.update(kw)
    return make_config(**base)


def fake_weights():
    w = AdoreWeights()
    for name, _ in AdoreWeights._fields_:
        setattr(w, name, FAKE)
    return w


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "adore.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(adore_[a-z_]+)\s*\(", text))
    assert declared == set(EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.adore_abi_version() == 10


def test_workspace_bytes(lib):
    w = workload("llama7b_layer")
    c = cfg_for(w)
    n = lib.adore_workspace_bytes(ctypes.byref(c))
    cache = 2 * w.L * w.B * w.H * w.K * w.d * 2
    assert cache <= n < cache + (64 << 20)
    assert n % 256 == 0
    bad = cfg_for(w, rebuild_budget=w.K - 1)
    assert lib.adore_workspace_bytes(ctypes.byref(bad)) == 0
    assert lib.adore_workspace_bytes(None) == 0


def test_create_rejects_bad_arguments(lib):
    w = workload("tiny")
    c, wt = cfg_for(w), fake_weights()
    h = ctypes.c_void_p()
    n = lib.adore_workspace_bytes(ctypes.byref(c))
    assert lib.adore_create(None, ctypes.byref(wt), FAKE, n, None, ctypes.byref(h)) == -1
    assert lib.adore_create(ctypes.byref(c), None, FAKE, n, None, ctypes.byref(h)) == -1
    assert lib.adore_create(ctypes.byref(c), ctypes.byref(wt), None, n, None, ctypes.byref(h)) == -1
    assert lib.adore_create(ctypes.byref(c), ctypes.byref(wt), FAKE, n - 1, None, ctypes.byref(h)) == -4
    assert lib.adore_create(ctypes.byref(c), ctypes.byref(wt), FAKE + 16, n, None, ctypes.byref(h)) == -4
    for kw in (dict(rebuild_budget=w.K - 1), dict(batch=0), dict(dtype=7), dict(rebuild_budget=-1),
               dict(cache_slots=1, rebuild_budget=0)):
        bad = cfg_for(w, **kw)
        assert lib.adore_create(ctypes.byref(bad), ctypes.byref(wt), FAKE, n, None, ctypes.byref(h)) == -1, kw
    for kw in (dict(head_dim=96), dict(cache_slots=2048, max_positions=4096), dict(hidden=260)):
        uns = cfg_for(w, **kw)
        big = lib.adore_workspace_bytes(ctypes.byref(uns))
        assert lib.adore_create(ctypes.byref(uns), ctypes.byref(wt), FAKE, big, None, ctypes.byref(h)) == -3, kw
    # more than 1024 slots are fine when the cache never has to release: K - R - 1 >= N_max (full attention)
    full = cfg_for(w, cache_slots=2048, max_positions=2048 - w.R - 1)
    big = lib.adore_workspace_bytes(ctypes.byref(full))
    assert lib.adore_create(ctypes.byref(full), ctypes.byref(wt), FAKE, big, None, ctypes.byref(h)) == 0
    assert lib.adore_destroy(h) == 0
    over = cfg_for(w, cache_slots=2048, max_positions=2048 - w.R)
    big = lib.adore_workspace_bytes(ctypes.byref(over))
    assert lib.adore_create(ctypes.byref(over), ctypes.byref(wt), FAKE, big, None, ctypes.byref(h)) == -3
    # rescore mode: unknown mode value, d' not a multiple of 4, no overrides, no set_state
    assert lib.adore_create(ctypes.byref(cfg_for(w, score_mode=3)), ctypes.byref(wt), FAKE, n, None, ctypes.byref(h)) == -1
    # H2O mode: scores per head (a larger workspace), one layer, no rotary embedding, a bounded number of positions,
    # no override in a step, no set_state, x_n not needed
    h2o = cfg_for(w, score_mode=2)
    big = lib.adore_workspace_bytes(ctypes.byref(h2o))
    assert big >= n + (w.H - 1) * w.B * w.N_max * 4
    for kw in (dict(layers=2), dict(rope_base=100.0), dict(max_positions=8000), dict(heads=256)):
        uns = cfg_for(w, score_mode=2, **kw)
        assert lib.adore_create(ctypes.byref(uns), ctypes.byref(wt), FAKE, lib.adore_workspace_bytes(ctypes.byref(uns)),
                                None, ctypes.byref(h)) == -3, kw
    assert lib.adore_create(ctypes.byref(h2o), ctypes.byref(wt), FAKE, big, None, ctypes.byref(h)) == 0
    assert lib.adore_schedule(h, None, FAKE, None, None, None, None) == -1        # an override
    assert lib.adore_schedule(h, None, None, None, None, None) == -2              # (valid arguments; no init yet)
    assert lib.adore_set_state(h, FAKE, None, None, None, None, 5) == -3
    assert lib.adore_init_cache(h, FAKE, FAKE, None, FAKE, None, 4) == -3         # no rebuild forward in this mode
    assert lib.adore_destroy(h) == 0
    odd = cfg_for(w, score_mode=1, ctrl_hidden=6)
    big = lib.adore_workspace_bytes(ctypes.byref(odd))
    assert lib.adore_create(ctypes.byref(odd), ctypes.byref(wt), FAKE, big, None, ctypes.byref(h)) == -3
    re = cfg_for(w, score_mode=1)
    big = lib.adore_workspace_bytes(ctypes.byref(re))
    assert big > n                                   # one d'-vector per token on top of the static layout
    assert lib.adore_create(ctypes.byref(re), ctypes.byref(wt), FAKE, big, None, ctypes.byref(h)) == 0
    assert lib.adore_schedule(h, FAKE, FAKE, None, None, None, None) == -1
    assert lib.adore_decode_step(h, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None) == -1
    assert lib.adore_set_state(h, FAKE, None, None, None, None, 5) == -3
    assert lib.adore_destroy(h) == 0
    # rotary embedding: a negative or non-finite base is invalid; a positive one adds the angle table
    for bad_base in (-1.0, float("nan"), float("inf")):
        assert lib.adore_workspace_bytes(ctypes.byref(cfg_for(w, rope_base=bad_base))) == 0
        assert lib.adore_create(ctypes.byref(cfg_for(w, rope_base=bad_base)), ctypes.byref(wt), FAKE, n, None,
                                ctypes.byref(h)) == -1
    rp = cfg_for(w, rope_base=10000.0)
    big = lib.adore_workspace_bytes(ctypes.byref(rp))
    assert n + w.N_max * (w.d // 2) * 24 <= big < n + w.N_max * (w.d // 2) * 24 + 512
    assert lib.adore_create(ctypes.byref(rp), ctypes.byref(wt), FAKE, n, None, ctypes.byref(h)) == -4
    assert lib.adore_create(ctypes.byref(rp), ctypes.byref(wt), FAKE, big, None, ctypes.byref(h)) == 0
    assert lib.adore_destroy(h) == 0
    wt2 = fake_weights()
    wt2.out_b = None
    assert lib.adore_create(ctypes.byref(c), ctypes.byref(wt2), FAKE, n, None, ctypes.byref(h)) == -1


def test_calls_out_of_order_are_state_errors(lib):
    w = workload("tiny")
    c, wt = cfg_for(w), fake_weights()
    h = ctypes.c_void_p()
    n = lib.adore_workspace_bytes(ctypes.byref(c))
    assert lib.adore_create(ctypes.byref(c), ctypes.byref(wt), FAKE, n, None, ctypes.byref(h)) == 0
    try:
        # nothing may run before init_cache; none of these reaches a kernel launch
        assert lib.adore_attend(h, 0, FAKE, FAKE, FAKE, FAKE) == -2
        assert lib.adore_schedule(h, FAKE, None, None, None, None) == -2
        assert lib.adore_rebuild(h, 0, FAKE) == -2
        assert lib.adore_decode_step(h, FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, None) == -2
        step = ctypes.c_int32()
        assert lib.adore_get_state(h, None, None, None, None, None, ctypes.byref(step)) == -2
        # argument errors come first
        assert lib.adore_attend(h, 1, FAKE, FAKE, FAKE, FAKE) == -1
        assert lib.adore_attend(h, 0, None, FAKE, FAKE, FAKE) == -1
        assert lib.adore_init_cache(h, FAKE, FAKE, FAKE, FAKE, None, 0) == -1
        assert lib.adore_init_cache(h, FAKE, FAKE, FAKE, FAKE, None, w.N_max) == -1
        assert lib.adore_init_cache(h, None, FAKE, FAKE, FAKE, None, 4) == -1
        assert lib.adore_set_state(h, None, None, None, None, None, 5) == -1
        assert lib.adore_set_state(h, FAKE, None, None, None, None, 0) == -1
        # the input-order switch is host state only until a GPU call has made the side stream
        assert lib.adore_set_input_order(None, 0) == -1
        assert lib.adore_set_input_order(h, 0) == 0
        assert lib.adore_set_input_order(h, 1) == 0
        # the rebuild forward: null arguments, a context not initialised for it -- all caught on the host
        from paper_2407_02328_amd.binding import AdoreForwardWeights
        fw = AdoreForwardWeights(FAKE, FAKE)
        assert lib.adore_forward_step(h, None, FAKE, None, FAKE, None, None, None, None) == -1
        assert lib.adore_forward_step(h, ctypes.byref(fw), None, None, FAKE, None, None, None, None) == -1
        assert lib.adore_forward_step(h, ctypes.byref(fw), FAKE, None, None, None, None, None, None) == -1
        assert lib.adore_forward_step(h, ctypes.byref(AdoreForwardWeights(None, FAKE)), FAKE, None, FAKE, None, None, None, None) == -1
        assert lib.adore_forward_step(h, ctypes.byref(fw), FAKE, None, FAKE, None, None, None, None) == -2
    finally:
        assert lib.adore_destroy(h) == 0
    # a cache of more than 8192 slots (one that never releases) has no forward path: caught on the host
    wide = cfg_for(w, cache_slots=9000, max_positions=9000 - w.R - 1)
    h2 = ctypes.c_void_p()
    assert lib.adore_create(ctypes.byref(wide), ctypes.byref(wt), FAKE, lib.adore_workspace_bytes(ctypes.byref(wide)),
                            None, ctypes.byref(h2)) == 0
    assert lib.adore_init_cache(h2, FAKE, FAKE, None, FAKE, None, 4) == -3
    assert lib.adore_destroy(h2) == 0
    assert lib.adore_destroy(None) == -1


def test_guard_word_layout_on_the_host(lib, monkeypatch):
    """ADORE_GUARD_WORDS=1: the workspace grows by 256 bytes per region, create takes it, and a context that has
    not touched the GPU reports that it has no guard words to count yet."""
    w = workload("tiny")
    c, wt = cfg_for(w), fake_weights()
    plain = lib.adore_workspace_bytes(ctypes.byref(c))
    monkeypatch.setenv("ADORE_GUARD_WORDS", "1")
    guarded = lib.adore_workspace_bytes(ctypes.byref(c))
    assert guarded > plain and (guarded - plain) % 256 == 0 and guarded - plain >= 20 * 256
    h = ctypes.c_void_p()
    assert lib.adore_create(ctypes.byref(c), ctypes.byref(wt), FAKE, plain, None, ctypes.byref(h)) == -4
    assert lib.adore_create(ctypes.byref(c), ctypes.byref(wt), FAKE, guarded, None, ctypes.byref(h)) == 0
    bad = ctypes.c_int32(7)
    assert lib.adore_check_guards(None, ctypes.byref(bad)) == -1
    assert lib.adore_check_guards(h, None) == -1
    assert lib.adore_check_guards(h, ctypes.byref(bad)) == 0 and bad.value == -1
    assert lib.adore_destroy(h) == 0


def test_strerror_and_kernel_names(lib):
    seen = set()
    for code in (0, -1, -2, -3, -4, -5, -99):
        s = lib.adore_strerror(code).decode()
        assert s
        seen.add(s)
    assert len(seen) == 7
    from paper_2407_02328_amd import KERNELS
    assert [lib.adore_kernel_name(i).decode() for i in range(len(KERNELS))] == KERNELS


def test_topk_attention_host_checks(lib):
    ws = lib.adore_topk_attention_workspace_bytes
    assert ws(0, 8, 64) == 0 and ws(1, 0, 64) == 0
    assert ws(3, 100, 128) == 3 * 128 * 128 * 2          # keys padded to a multiple of 32
    assert ws(1, 33, 64) % 256 == 0 and ws(1, 33, 64) >= 64 * 64 * 2
    call = lib.adore_topk_attention
    n = ws(2, 64, 64)
    assert call(None, FAKE, FAKE, FAKE, FAKE, n, 2, 64, 64, 4, None) == -1
    assert call(FAKE, FAKE, FAKE, FAKE, FAKE, n, 2, 64, 64, 0, None) == -1
    assert call(FAKE, FAKE, FAKE, FAKE, FAKE, n, 0, 64, 64, 4, None) == -1
    assert call(FAKE, FAKE, FAKE, FAKE, FAKE, n, 2, 64, 96, 4, None) == -3
    assert call(FAKE, FAKE, FAKE, FAKE, FAKE, 1 << 40, 2, 40000, 64, 4, None) == -3
    # beyond 2048 tokens the weights of a query block live in the workspace: one piece of 16 rows per workgroup of
    # the launch, which has at most 512 of them (fewer when there are fewer query blocks)
    long = ws(2, 4096, 64)
    assert long >= 2 * 64 * 4096 * 2 + 2 * 256 * 16 * 4096 * 4
    big = ws(128, 8192, 128)
    assert 128 * 128 * 8192 * 2 + 512 * 16 * 8192 * 4 <= big < 128 * 128 * 8192 * 2 + 512 * 16 * 8192 * 4 + (4 << 20)
    assert call(FAKE, FAKE, FAKE, FAKE, FAKE, long - 1, 2, 4096, 64, 4, None) == -4
    assert call(FAKE, FAKE, FAKE, FAKE, FAKE, n - 1, 2, 64, 64, 4, None) == -4
    assert call(FAKE, FAKE, FAKE, FAKE, FAKE + 16, n, 2, 64, 64, 4, None) == -4
