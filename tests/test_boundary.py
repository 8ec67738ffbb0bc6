"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, rejects bad
arguments on the host before touching a device, and its host budget allocator agrees with the
oracle's.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import lava_oracle as O
from paper_2509_09754_amd import lava

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "lava.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lava_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert "lava_window_scores" in names and "lava_compact_kv" in names and len(names) >= 9
    dll = ctypes.CDLL(lava.LIB_PATH)
    for n in names:
        assert hasattr(dll, n), f"{n} declared in lava.h but not exported"
    assert sorted(lava.EXPORTS) == names


def test_status_strings():
    assert lava.status_string(lava.LAVA_OK) == "ok"
    assert "budget" in lava.status_string(lava.LAVA_ERR_BUDGET)
    assert lava.lib.lava_prof_kernel_count() >= 8
    assert lava.lib.lava_prof_kernel_name(0) == b"vnorm"


def test_tuning_round_trip_and_validation():
    try:
        lava.set_tuning(sweep_shape="narrow", sweep_workgroups=300, decode_rows_per_unit=256, barrier_spin_limit=7)
        t = lava.get_tuning()
        assert (t.sweep_shape, t.sweep_workgroups, t.decode_rows_per_unit, t.barrier_spin_limit) == (2, 300, 256, 7)
        bad = lava.Tuning(3, 0, 0, 0, 0)
        assert lava.lib.lava_set_tuning(ctypes.byref(bad)) == lava.LAVA_ERR_INVALID_ARG
        bad = lava.Tuning(0, 0, 4, 0, 0)                        # schedules are 0..3
        assert lava.lib.lava_set_tuning(ctypes.byref(bad)) == lava.LAVA_ERR_INVALID_ARG
        bad = lava.Tuning(0, 0, 0, 64, 0)                       # fewer rows than one round of the decode wavefronts
        assert lava.lib.lava_set_tuning(ctypes.byref(bad)) == lava.LAVA_ERR_INVALID_ARG
        bad = lava.Tuning(0, 0, 0, 0, 0)
        bad.reserved[1] = 1
        assert lava.lib.lava_set_tuning(ctypes.byref(bad)) == lava.LAVA_ERR_INVALID_ARG
        assert lava.get_tuning().sweep_workgroups == 300        # a rejected setting changes nothing
        assert lava.lib.lava_get_tuning(None) == lava.LAVA_ERR_INVALID_ARG
        # the decode unit size is part of the workspace layout: the size query follows the tuning
        d = _desc()
        small_units = lava.lava_decode_workspace_bytes(d, 4, 65536, 0)
        lava.set_tuning(decode_rows_per_unit=1024)
        assert lava.lava_decode_workspace_bytes(d, 4, 65536, 0) < small_units
    finally:
        assert lava.lib.lava_set_tuning(None) == lava.LAVA_OK
    t = lava.get_tuning()
    assert (t.sweep_shape, t.sweep_workgroups, t.sweep_schedule, t.decode_rows_per_unit, t.barrier_spin_limit) == (0,) * 5


def test_no_environment_variable_is_read_by_the_library():
    src = os.path.join(ROOT, "paper_2509_09754_amd", "csrc")
    for name in sorted(os.listdir(src)):
        assert "getenv" not in open(os.path.join(src, name)).read(), name


def _desc(**kw):
    base = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, window=32, dtype="bf16")
    base.update(kw)
    return lava.LayerDesc.make(**base)


FAKE = ctypes.c_void_p(0x10000)       # never dereferenced: every case below fails validation first


def _ws(desc, lens, **over):
    lens = np.asarray(lens, dtype=np.int64)
    args = dict(q=FAKE, k=FAKE, v=FAKE, scores=FAKE, vbar=FAKE, stat=FAKE, ws=FAKE, ws_bytes=1 << 40)
    args.update(over)
    return lava.lib.lava_window_scores(ctypes.byref(desc), len(lens), lens.ctypes.data_as(ctypes.c_void_p),
                                       args["q"], args["k"], args["v"], None, args["scores"], args["vbar"],
                                       args["stat"], args["ws"], args["ws_bytes"], None)


def test_window_scores_argument_errors():
    good = _desc()
    assert _ws(_desc(n_q_heads=30), [4096]) == lava.LAVA_ERR_SHAPE            # H % H_kv != 0
    assert _ws(_desc(head_dim=96), [4096]) == lava.LAVA_ERR_SHAPE
    assert _ws(_desc(window=65), [4096]) == lava.LAVA_ERR_SHAPE
    assert _ws(_desc(n_q_heads=8 * 17), [4096]) == lava.LAVA_ERR_SHAPE         # G = 17
    assert lava.lava_window_scores_workspace_bytes(_desc(window=64, n_q_heads=8 * 16), 1, 4096) > 0
    assert _ws(_desc(pool_kernel=4), [4096]) == lava.LAVA_ERR_SHAPE
    assert _ws(_desc(window=0), [4096]) == lava.LAVA_ERR_INVALID_ARG
    assert _ws(_desc(dtype=lava.LAVA_BF16), [32]) == lava.LAVA_ERR_SHAPE      # N must exceed w
    d = _desc()
    d.dtype = 7
    assert _ws(d, [4096]) == lava.LAVA_ERR_INVALID_ARG
    assert _ws(good, [4096], k=None) == lava.LAVA_ERR_INVALID_ARG
    assert _ws(good, [4096], k=ctypes.c_void_p(0x10008)) == lava.LAVA_ERR_INVALID_ARG   # misaligned
    assert _ws(good, [4096], ws=None) == lava.LAVA_ERR_WORKSPACE
    assert _ws(good, [4096], ws_bytes=16) == lava.LAVA_ERR_WORKSPACE
    assert _ws(good, [4096], ws=ctypes.c_void_p(0x10010)) == lava.LAVA_ERR_WORKSPACE
    lens = np.asarray([4096, 9000], dtype=np.int64)
    prm = lambda sws, swsb: lava.lib.lava_window_scores_primed(
        ctypes.byref(good), 2, lens.ctypes.data_as(ctypes.c_void_p), FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, FAKE,
        1 << 40, sws, swsb, None)
    need = lava.lava_select_batch_workspace_bytes(2, 8 * 9000)  # one region per sequence, sized for the longest
    assert prm(None, need) == lava.LAVA_ERR_WORKSPACE
    assert prm(FAKE, need - 1) == lava.LAVA_ERR_WORKSPACE
    assert prm(ctypes.c_void_p(0x10010), need) == lava.LAVA_ERR_WORKSPACE
    assert lava.lava_window_scores_workspace_bytes(good, 1, 4096) > 8 * 4064 * 4
    assert lava.lava_window_scores_workspace_bytes(_desc(head_dim=100), 1, 4096) == 0
    # a budget plan is validated before anything is launched
    one = np.asarray([4096], dtype=np.int64)
    def planned(plan):
        return lava.lib.lava_window_scores_planned(
            ctypes.byref(good), 1, one.ctypes.data_as(ctypes.c_void_p), FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, None,
            0, None, 0, ctypes.byref(plan), None)
    fake = FAKE.value
    assert planned(lava.BudgetPlan(4, 1, fake, fake, fake, fake, fake)) == lava.LAVA_ERR_WORKSPACE   # plan accepted
    assert planned(lava.BudgetPlan(0, 0, fake, fake, fake, fake, fake)) == lava.LAVA_ERR_INVALID_ARG
    assert planned(lava.BudgetPlan(lava.LAVA_PLAN_MAX_LAYERS + 1, 0, fake, fake, fake, fake, fake)) == lava.LAVA_ERR_INVALID_ARG
    assert planned(lava.BudgetPlan(4, 4, fake, fake, fake, fake, fake)) == lava.LAVA_ERR_INVALID_ARG
    assert planned(lava.BudgetPlan(4, -1, fake, fake, fake, fake, fake)) == lava.LAVA_ERR_INVALID_ARG
    for missing in range(5):
        ptrs = [fake] * 5
        ptrs[missing] = None
        assert planned(lava.BudgetPlan(4, 1, *ptrs)) == lava.LAVA_ERR_INVALID_ARG


def test_workspace_size_never_shrinks_with_length():
    # a batch shares one workspace sized for its longest sequence; every shorter one must fit
    for d in (_desc(), _desc(n_q_heads=8, n_kv_heads=2, head_dim=64, window=8, dtype="f32"),
              _desc(n_q_heads=16, n_kv_heads=2)):
        prev = 0
        for n in list(range(40, 20000, 13)) + list(range(20000, 700000, 4999)):
            b = lava.lava_window_scores_workspace_bytes(d, 1, n)
            assert b >= prev > -1 and b % 256 == 0
            prev = b


def test_select_and_compact_argument_errors():
    L = lava.lib
    big = 1 << 40
    call = lambda nh, total, budget, ws=FAKE, wsb=big, sc=FAKE: L.lava_select_topk(
        nh, sc, None, total, budget, None, FAKE, FAKE, FAKE, None, ws, wsb, None)
    assert call(8, 8 * 1024, 8 * 1024 + 1) == lava.LAVA_ERR_BUDGET
    assert call(8, 8 * 1024, -1) == lava.LAVA_ERR_BUDGET
    assert call(0, 1024, 10) == lava.LAVA_ERR_INVALID_ARG
    assert call(65, 65 * 16, 10) == lava.LAVA_ERR_SHAPE
    assert call(8, 1001, 10) == lava.LAVA_ERR_SHAPE             # equal segments need total % heads == 0
    assert call(8, 1024, 10, sc=None) == lava.LAVA_ERR_INVALID_ARG
    assert call(8, 1024, 10, ws=None) == lava.LAVA_ERR_WORKSPACE
    assert call(8, 1024, 10, wsb=8) == lava.LAVA_ERR_WORKSPACE
    primed = lambda nh, total, budget, ws=FAKE, wsb=big: L.lava_select_topk_primed(
        nh, FAKE, total, budget, None, FAKE, FAKE, FAKE, None, ws, wsb, None)
    assert primed(8, 1001, 10) == lava.LAVA_ERR_SHAPE           # a prepared workspace serves equal segments
    assert primed(8, 1024, 2000) == lava.LAVA_ERR_BUDGET
    assert primed(8, 1024, 10, wsb=8) == lava.LAVA_ERR_WORKSPACE
    assert lava.lava_select_workspace_bytes(1 << 20) >= 3 * 2048 * 4
    assert lava.lava_select_workspace_bytes(0) == 0
    assert L.lava_select_status(None, 1024, None) == lava.LAVA_ERR_INVALID_ARG
    assert L.lava_select_status(FAKE, 0, None) == lava.LAVA_ERR_INVALID_ARG
    d = _desc()
    cc = lambda n, cap, k=FAKE: L.lava_compact_kv(ctypes.byref(d), n, k, FAKE, FAKE, FAKE, cap, FAKE, FAKE, None)
    assert cc(1024, 8 * 1024 + 1) == lava.LAVA_ERR_BUDGET
    assert cc(1024, -1) == lava.LAVA_ERR_INVALID_ARG
    assert cc(1024, 16, k=None) == lava.LAVA_ERR_INVALID_ARG
    assert cc(1024, 0) == lava.LAVA_OK                          # nothing to move, nothing launched


def test_host_budgets_match_oracle():
    r = np.random.Generator(np.random.PCG64(21))
    for trial in range(200):
        L = int(r.integers(1, 40))
        e = (r.random(L) * (r.random(L) < 0.85)).astype(np.float32)
        lo = r.integers(0, 300, L)
        hi = lo + r.integers(0, 5000, L)
        total = int(r.integers(lo.sum(), hi.sum() + 1))
        got = lava.lava_layer_budgets(e, [total], lo, hi)[0]
        ref = O.layer_budgets(e.astype(np.float64), total, lo, hi)
        assert got.tolist() == ref, (trial, e, lo, hi, total)
    # the stack configuration: 32 layers, bounds H_kv*w and H_kv*N
    e = r.random(32).astype(np.float32) * 1e-5
    got = lava.lava_layer_budgets(e, [131072], [256] * 32, [262144] * 32)[0]
    assert got.sum() == 131072 and got.tolist() == O.layer_budgets(e.astype(np.float64), 131072, [256] * 32, [262144] * 32)
    # batch of two sequences with different totals
    e2 = r.random((2, 5)).astype(np.float32)
    got = lava.lava_layer_budgets(e2, [100, 777], np.zeros((2, 5)), np.full((2, 5), 1000))
    for b, tot in enumerate([100, 777]):
        assert got[b].tolist() == O.layer_budgets(e2[b].astype(np.float64), tot, [0] * 5, [1000] * 5)


def test_host_budgets_errors():
    with pytest.raises(lava.LavaError) as ei:
        lava.lava_layer_budgets(np.ones(2, np.float32), [5], [3, 3], [9, 9])
    assert ei.value.status == lava.LAVA_ERR_BUDGET
    with pytest.raises(lava.LavaError):
        lava.lava_layer_budgets(np.ones(2, np.float32), [50], [3, 3], [9, 9])


def test_decode_argument_errors():
    L = lava.lib
    d = _desc()
    big = 1 << 40

    def call(desc=d, batch=1, q=FAKE, kh=FAKE, vh=FAKE, offs=FAKE, cap=1024, kt=None, vt=None, tail=0, tcap=0,
             out=FAKE, ws=FAKE, wsb=big):
        return L.lava_decode_attention(ctypes.byref(desc), batch, q, kh, vh, offs, None, cap, kt, vt, tail, tcap,
                                       out, None, ws, wsb, None)

    assert call(q=None) == lava.LAVA_ERR_INVALID_ARG
    assert call(offs=None) == lava.LAVA_ERR_INVALID_ARG
    assert call(out=None) == lava.LAVA_ERR_INVALID_ARG
    assert call(kh=None) == lava.LAVA_ERR_INVALID_ARG                    # rows but no packed cache
    assert call(cap=-1) == lava.LAVA_ERR_INVALID_ARG
    assert call(tail=4, tcap=4) == lava.LAVA_ERR_INVALID_ARG             # tail rows but no tail buffers
    assert call(kt=FAKE, vt=FAKE, tail=5, tcap=4) == lava.LAVA_ERR_INVALID_ARG
    assert call(kh=ctypes.c_void_p(0x10004)) == lava.LAVA_ERR_INVALID_ARG
    assert call(batch=0) == lava.LAVA_ERR_INVALID_ARG
    assert call(desc=_desc(head_dim=96)) == lava.LAVA_ERR_SHAPE
    assert call(desc=_desc(n_q_heads=72, n_kv_heads=8)) == lava.LAVA_ERR_SHAPE   # G = 9
    assert call(ws=None) == lava.LAVA_ERR_WORKSPACE
    assert call(wsb=64) == lava.LAVA_ERR_WORKSPACE
    # window and pool_kernel of the descriptor are ignored by the decode step
    odd = _desc(window=32)
    odd.window, odd.pool_kernel = 999, 4
    assert lava.lava_decode_workspace_bytes(odd, 2, 8192, 16) > 0
    assert lava.lava_decode_workspace_bytes(d, 0, 8192, 0) == 0
    prev = 0
    for cap in range(0, 200000, 777):        # enough for every smaller capacity of the same batch
        b = lava.lava_decode_workspace_bytes(d, 4, cap, 0)
        assert b % 256 == 0 and b > 0


def test_cascade_and_packed_compaction_argument_errors():
    L = lava.lib
    d = _desc()
    cp = lambda src=FAKE, rows=1000, cap=10, k=FAKE: L.lava_compact_packed(
        ctypes.byref(d), src, rows, k, FAKE, None, FAKE, FAKE, cap, FAKE, FAKE, None, None)
    assert cp(src=None) == lava.LAVA_ERR_INVALID_ARG
    assert cp(k=None) == lava.LAVA_ERR_INVALID_ARG
    assert cp(rows=0) == lava.LAVA_ERR_INVALID_ARG
    assert cp(cap=1001) == lava.LAVA_ERR_BUDGET
    assert cp(cap=0) == lava.LAVA_OK                              # nothing to move, nothing launched

    state = lava.CascadeStateStruct()
    for i in range(2):
        state.k[i] = state.v[i] = state.pos[i] = state.scores[i] = 0x10000
        state.head_offsets[i] = state.layer_start[i] = 0x10000
    state.head_counts = state.kept_idx = 0x10000
    state.capacity, state.max_layers, state.cur = 8192, 4, 0
    n = 4096
    step = lambda st=state, layer_idx=0, total=8192, ws=FAKE, wsb=1 << 40, nn=n: L.lava_cascade_step(
        ctypes.byref(d), layer_idx, nn, FAKE, FAKE, FAKE, FAKE, total, ctypes.byref(st), FAKE, ws, wsb, None)
    assert step(total=8 * 32 - 1) == lava.LAVA_ERR_BUDGET         # below H_kv * w per layer
    assert step(total=8 * n + 1) == lava.LAVA_ERR_BUDGET          # more than the layers seen so far hold
    assert step(nn=32) == lava.LAVA_ERR_SHAPE
    assert step(layer_idx=4, total=5 * 8192) == lava.LAVA_ERR_SHAPE        # beyond max_layers
    assert step(ws=None) == lava.LAVA_ERR_WORKSPACE
    assert step(wsb=16) == lava.LAVA_ERR_WORKSPACE
    assert step(layer_idx=1, total=8193) == lava.LAVA_ERR_BUDGET  # the arenas hold `capacity` rows in all
    broken = lava.CascadeStateStruct.from_buffer_copy(state)
    broken.layer_start[1] = None
    assert step(st=broken) == lava.LAVA_ERR_INVALID_ARG
    broken = lava.CascadeStateStruct.from_buffer_copy(state)
    broken.cur = 2
    assert step(st=broken) == lava.LAVA_ERR_INVALID_ARG
    one = lava.lava_select_workspace_bytes(8 * n)
    assert lava.lava_cascade_workspace_bytes(d, n, 1, 8192) == one + 512      # + the in-place gather's barrier words
    assert lava.lava_cascade_workspace_bytes(d, n, 5, 8192) == 5 * one + 512
    assert lava.lava_cascade_workspace_bytes(d, 16, 1, 8192) == 0
    assert lava.lava_cascade_workspace_bytes(d, n, 0, 8192) == 0
    assert step(layer_idx=0, wsb=one - 1) == lava.LAVA_ERR_WORKSPACE
    # K and V share one arena (the state above: every pointer equal) -> the barrier words are needed too
    assert step(layer_idx=0, wsb=one) == lava.LAVA_ERR_WORKSPACE
    # ... and both of them share it, or neither
    mixed = lava.CascadeStateStruct.from_buffer_copy(state)
    mixed.v[1] = 0x20000
    assert step(st=mixed) == lava.LAVA_ERR_INVALID_ARG
    two = lava.CascadeStateStruct.from_buffer_copy(state)
    two.k[1] = two.v[1] = 0x20000
    assert step(st=two, layer_idx=0, wsb=one - 1) == lava.LAVA_ERR_WORKSPACE


def test_batch_select_and_compact_argument_errors():
    L = lava.lib
    big = 1 << 40
    good = lava.SelectProblem(0x10000, None, 8 * 1024, 100, None, 0x10000, 0x10000, 0x10000, None, None, None)
    seg_primed = lava.SelectProblem(0x10000, 0x10000, 8 * 1024, 100, None, 0x10000, 0x10000, 0x10000, None, None, None,
                                    None, 1)

    def sel(problems, nh=8, widest=8 * 1024, ws=FAKE, wsb=big):
        table = (lava.SelectProblem * max(len(problems), 1))(*problems)
        return L.lava_select_topk_batch(nh, len(problems), ctypes.cast(table, ctypes.c_void_p), widest, ws, wsb, None)

    def changed(**kw):
        p = lava.SelectProblem.from_buffer_copy(good)
        for k, v in kw.items():
            setattr(p, k, v)
        return p

    assert sel([]) == lava.LAVA_ERR_INVALID_ARG
    assert L.lava_select_topk_batch(8, 1, None, 1024, FAKE, big, None) == lava.LAVA_ERR_INVALID_ARG
    assert sel([good, changed(budget=8 * 1024 + 1)]) == lava.LAVA_ERR_BUDGET       # any row of the table is checked
    assert sel([good, changed(scores=None)]) == lava.LAVA_ERR_INVALID_ARG
    assert sel([good, changed(total_entries=1001)]) == lava.LAVA_ERR_SHAPE         # equal segments
    assert sel([good, changed(total_entries=16 * 1024)]) == lava.LAVA_ERR_SHAPE    # wider than the stated maximum
    assert sel([good], nh=65) == lava.LAVA_ERR_SHAPE
    assert sel([good, seg_primed]) == lava.LAVA_ERR_INVALID_ARG                    # prepared + explicit segments
    assert sel([good, good], ws=None) == lava.LAVA_ERR_WORKSPACE
    one = lava.lava_select_workspace_bytes(8 * 1024)
    assert lava.lava_select_batch_workspace_bytes(3, 8 * 1024) == 3 * one
    assert lava.lava_select_batch_workspace_bytes(0, 8 * 1024) == 0
    assert sel([good, good, good], wsb=3 * one - 1) == lava.LAVA_ERR_WORKSPACE
    assert L.lava_select_batch_status(None, 2, 1024, None) == lava.LAVA_ERR_INVALID_ARG
    assert L.lava_select_batch_status(FAKE, 0, 1024, None) == lava.LAVA_ERR_INVALID_ARG

    d = _desc()
    okc = lava.CompactProblem(1024, None, 0x10000, 0x10000, None, 0x10000, 0x10000, 0, 0x10000, 0x10000, None, None,
                              None)

    def cmp(problems):
        table = (lava.CompactProblem * max(len(problems), 1))(*problems)
        return L.lava_compact_batch(ctypes.byref(d), len(problems), ctypes.cast(table, ctypes.c_void_p), None)

    def cchanged(**kw):
        p = lava.CompactProblem.from_buffer_copy(okc)
        for k, v in kw.items():
            setattr(p, k, v)
        return p

    assert cmp([]) == lava.LAVA_ERR_INVALID_ARG
    assert cmp([okc, okc]) == lava.LAVA_OK                                          # capacities 0: nothing launched
    assert cmp([okc, cchanged(capacity=8 * 1024 + 1)]) == lava.LAVA_ERR_BUDGET      # dense source: H_kv * n rows
    assert cmp([okc, cchanged(src_offsets=0x10000, capacity=1025)]) == lava.LAVA_ERR_BUDGET   # packed source: pool rows
    assert cmp([okc, cchanged(k_out=None)]) == lava.LAVA_ERR_INVALID_ARG
    assert cmp([okc, cchanged(k_src=0x10008)]) == lava.LAVA_ERR_INVALID_ARG         # rows move as 16-byte words
    assert cmp([okc, cchanged(src_rows=0)]) == lava.LAVA_ERR_INVALID_ARG
