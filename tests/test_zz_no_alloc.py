"""lava_select_topk_static (the selection on the library's built-in scratch array, for callers that
cannot allocate) against lava_select_topk on the same inputs, through the C ABI: bit-exact, on
two calls in a row, the second with a smaller input, so that whatever the first call left in the
shared array must not leak into the second.  The oracle is consulted as well."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import lava_oracle as O
from paper_2509_09754_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lava():
    from paper_2509_09754_amd import lava as mod
    assert torch.cuda.is_available()
    return mod


_CALLS = [0]


def _outputs(nh, cap):
    return (torch.full((nh,), -7, dtype=torch.int32, device="cuda"),
            torch.full((nh + 1,), -7, dtype=torch.int64, device="cuda"),
            torch.full((cap + 8,), -7, dtype=torch.int32, device="cuda"),
            torch.full((cap + 8,), -7.0, dtype=torch.float32, device="cuda"))


def _raw_static(lava, nh, sc, seg, budget, bd, outs):
    """Straight through ctypes.CDLL: no helper of the binding between the test and the C ABI."""
    p = lambda t: None if t is None else ctypes.c_void_p(t.data_ptr())
    return lava.lib.lava_select_topk_static(nh, p(sc), p(seg), sc.numel(), budget, p(bd), p(outs[0]), p(outs[1]),
                                            p(outs[2]), p(outs[3]),
                                            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))


def _compare(lava, scores_f32, nh, budget, seg_offsets=None, budget_dev=None):
    flat = np.ascontiguousarray(scores_f32, dtype=np.float32).ravel()
    sc = torch.from_numpy(flat).cuda()
    seg = None if seg_offsets is None else torch.tensor(seg_offsets, dtype=torch.int64, device="cuda")
    bd = None if budget_dev is None else torch.tensor([budget_dev], dtype=torch.int64, device="cuda")
    cap = max(budget, 1)
    want = _outputs(nh, cap)
    lava.lava_select_topk(nh, sc, budget, seg_offsets=seg, budget_dev=bd, head_counts=want[0], head_offsets=want[1],
                          kept_idx=want[2], kept_scores=want[3])
    got = _outputs(nh, cap)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    assert _raw_static(lava, nh, sc, seg, budget, bd, got) == lava.LAVA_OK
    torch.cuda.synchronize()
    # free device memory as the driver reports it: unchanged by the call (the very first call in a
    # process may load the library's code object, so it is exempt)
    if _CALLS[0] > 0:
        assert torch.cuda.mem_get_info()[0] >= free_before
    _CALLS[0] += 1
    for a, b in zip(got, want):
        assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a,
                           b.view(torch.int32) if b.dtype == torch.float32 else b)
    # and the oracle, on what is unique: counts, offsets, kept positions, kept score bits
    eff = budget if budget_dev is None else max(0, min(budget, budget_dev))
    offs_ref = seg_offsets if seg_offsets is not None else [g * (flat.size // nh) for g in range(nh + 1)]
    rc, ro, ri, rs = O.select_topk(flat.astype(np.float64), offs_ref, eff)
    assert np.array_equal(got[0].cpu().numpy(), rc) and np.array_equal(got[1].cpu().numpy(), ro)
    assert np.array_equal(got[2].cpu().numpy()[:eff], ri)
    assert np.array_equal(got[3].cpu().numpy()[:eff].view(np.uint32), rs.astype(np.float32).view(np.uint32))


def test_static_scratch_selection_matches_workspace_selection(lava):
    print("static select: 8 x 40000 then 4 x 3000", flush=True)
    big = O.flat_layer_scores(synth.random_scores(8, 40000 - 32, 31).astype(np.float64), 40000).astype(np.float32)
    _compare(lava, big, 8, 8 * 512)                       # 20 workgroups, plateaus, +inf window entries
    small = synth.random_scores(4, 3000, 32)
    _compare(lava, small, 4, 777)                          # one workgroup: most of the array still holds the first call's words
    print("static select: segments, device budget, ties", flush=True)
    seg = [0, 100, 100, 4500, 9000, 9000, 9001, 12345]
    _compare(lava, synth.random_scores(1, seg[-1], 33).ravel(), len(seg) - 1, 5000, seg_offsets=seg, budget_dev=1234)
    _compare(lava, np.full((4, 3000), 0.25, dtype=np.float32), 4, 3001)
    print("static select: 8 x 131072 then 2 x 1024", flush=True)
    full = O.flat_layer_scores(synth.random_scores(8, 131072 - 32, 34).astype(np.float64), 131072).astype(np.float32)
    _compare(lava, full, 8, 8192)
    _compare(lava, synth.random_scores(2, 1024, 35), 2, 256)


def test_static_scratch_selection_multi_launch_path_then_small(lava):
    # 2.4 M entries run the selection's phases as separate launches over the same array
    print("static select: 8 x 300000 (separate launches) then 3 x 777", flush=True)
    n = 300000
    full = O.flat_layer_scores(synth.random_scores(8, n - 32, 36).astype(np.float64), n).astype(np.float32)
    _compare(lava, full, 8, 8 * 1024)
    _compare(lava, synth.random_scores(3, 777, 37), 3, 100)


def test_static_scratch_selection_rejects_what_the_array_cannot_hold(lava):
    nh = 8
    sc = torch.zeros(8, dtype=torch.float32, device="cuda")          # never read: the size check comes first
    outs = _outputs(nh, 8)
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    too_many = lava.SELECT_STATIC_MAX_ENTRIES + nh
    st = lava.lib.lava_select_topk_static(nh, p(sc), None, too_many, 8, None, p(outs[0]), p(outs[1]), p(outs[2]),
                                          p(outs[3]), None)
    assert st == lava.LAVA_ERR_WORKSPACE
    assert lava.lib.lava_select_topk_static(nh, p(sc), None, 8, 9, None, p(outs[0]), p(outs[1]), p(outs[2]),
                                            p(outs[3]), None) == lava.LAVA_ERR_BUDGET
    torch.cuda.synchronize()
    assert all(bool((t == -7).all()) for t in outs)                   # nothing was launched
