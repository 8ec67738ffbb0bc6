"""Algorithm 2 as a driver on the GPU against the oracle's literal cascade.

Selection is integer work and rows are bit copies, so after every outer iteration the state of
every layer (head offsets, token positions, retained scores, packed K / V rows) and the budget
vector must equal the oracle's exactly, provided both sides rank the same float32 scores and
allocate from the same float32 statistics.
"""
import dataclasses

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


def say(*a):
    print(*a, flush=True)


def check_state(lava, state, t, ref_state, k_store, v_store, dtype, tag):
    offs_ref, pos_ref, sc_ref = ref_state
    cur = state.current(t)
    offs = cur["head_offsets"].cpu().numpy()
    assert np.array_equal(offs, offs_ref), (tag, offs, offs_ref)
    kept = int(offs[-1])
    assert cur["pos"].shape[0] == kept, tag                      # the layer's extent in the arena is exactly what it holds
    assert np.array_equal(cur["pos"][:kept].cpu().numpy(), pos_ref), tag
    assert np.array_equal(cur["scores"][:kept].cpu().numpy().view(np.uint32),
                          sc_ref.astype(np.float32).view(np.uint32)), tag
    assert np.array_equal(cur["head_counts"].cpu().numpy(), np.diff(offs_ref)), tag
    # rows: bit copies of the original cache rows at the retained positions
    kh = lava.to_host_bits(cur["k_hat"][:kept])
    vh = lava.to_host_bits(cur["v_hat"][:kept])
    for g in range(len(offs) - 1):
        a, b = int(offs[g]), int(offs[g + 1])
        assert np.array_equal(kh[a:b], k_store[g][pos_ref[a:b]]), (tag, g)
        assert np.array_equal(vh[a:b], v_store[g][pos_ref[a:b]]), (tag, g)


# every cascade runs twice: K and V in two arenas (out-of-place gathers), and in one arena that the step
# re-compacts in place
ARENAS = pytest.mark.parametrize("in_place", [False, True], ids=["two-arenas", "one-arena-in-place"])


def run_cascade(lava, shape, n_layers, total_budget, seeds, use_gpu_scores, in_place=False):
    H, Hkv, d, N, w = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.n, shape.window
    desc = lava.LayerDesc.make(H, Hkv, d, w, shape.dtype, pool_kernel=shape.pool_kernel)
    state = lava.CascadeState(desc, n_layers, total_budget, in_place=in_place)   # arenas of `total_budget` rows, whatever the depth
    layer_scores, ents, stores = [], [], []
    ws = None
    for l in range(n_layers):
        inp = synth.gen_layer(dataclasses.replace(shape, heavy_frac=float(seeds["fracs"][l])), seeds["base"] + l)
        k_dev, v_dev = lava.to_device(inp.k, shape.dtype), lava.to_device(inp.v, shape.dtype)
        if use_gpu_scores:
            q_dev = lava.to_device(inp.q_win, shape.dtype)
            sc_dev, _, _ = lava.lava_window_scores(desc, [N], q_dev, k_dev, v_dev, layer_stat=state.e[l: l + 1])
            torch.cuda.synchronize()
            sc = sc_dev.cpu().numpy().reshape(Hkv, N)
            e_l = float(state.e[l].item())
        else:
            q, k, v = inp.f64()
            s, _ = O.lava_scores(q, k, v, w, shape.pool_kernel)
            sc = O.flat_layer_scores(s, N).astype(np.float32)
            e_l = float(np.float32(O.layer_entropy(s)))
            state.e[l] = e_l
            sc_dev = torch.from_numpy(sc.ravel()).cuda()
        layer_scores.append(sc.astype(np.float64))
        ents.append(e_l)
        stores.append((inp.k, inp.v))
        ws = lava.lava_cascade_step(desc, l, N, k_dev, v_dev, sc_dev, state, total_budget, workspace=ws)
        torch.cuda.synchronize()
        # oracle: the literal algorithm on the layers seen so far, same scores, same statistics
        ref_state, history = O.cascade(layer_scores, N, total_budget, w, entropies=ents)
        assert state.budgets[: l + 1].cpu().numpy().tolist() == history[-1], (l, history[-1])
        starts = state.layer_start[state.cur][: l + 2].cpu().numpy()
        assert starts[0] == 0 and np.array_equal(np.diff(starts), [int(r[0][-1]) for r in ref_state])   # back to back
        for t in range(l + 1):
            check_state(lava, state, t, ref_state[t], stores[t][0], stores[t][1], shape.dtype, f"step {l} layer {t}")
    return state, history


@ARENAS
def test_cascade_small_f32_matches_oracle(lava, in_place):
    say("cascade: 5 layers, f32, N=1024 (config 1 shape), oracle scores")
    shape = synth.config(1)
    fr = synth.stack_heavy_fracs(5, 3)
    state, history = run_cascade(lava, shape, 5, 5 * 256, dict(base=100, fracs=fr), use_gpu_scores=False,
                                 in_place=in_place)
    assert sum(history[-1]) == 5 * 256
    # budgets shrink as layers arrive (the memory is shared with more layers)
    say("  final budgets", history[-1])


@ARENAS
def test_cascade_bf16_gpu_scores(lava, in_place):
    say("cascade: 4 layers, bf16 32q/8kv d128, N=4096+5, scores and statistics from the GPU")
    shape = synth.config(2, n=4096 + 5, budget=1024)
    fr = synth.stack_heavy_fracs(4, 5)
    state, history = run_cascade(lava, shape, 4, 4 * 1024, dict(base=200, fracs=fr), use_gpu_scores=True,
                                 in_place=in_place)
    assert sum(history[-1]) == 4 * 1024
    say("  final budgets", history[-1])


@ARENAS
def test_cascade_many_layers_tight_budget(lava, in_place):
    say("cascade: 14 layers, f32, N=300, total barely above the lower bounds -> many layers pinned at H_kv * w")
    shape = synth.config(1, n=300)
    fr = synth.stack_heavy_fracs(14, 11)
    total = 14 * shape.n_kv_heads * shape.window + 90          # 16 per layer is the floor
    state, history = run_cascade(lava, shape, 14, total, dict(base=500, fracs=fr), use_gpu_scores=False,
                                 in_place=in_place)
    assert sum(history[-1]) == total and min(history[-1]) >= shape.n_kv_heads * shape.window


@ARENAS
def test_cascade_first_layer_takes_everything(lava, in_place):
    say("cascade: total budget = one layer's size -> the first layer is kept whole, then shrinks")
    shape = synth.config(1, n=600)
    fr = synth.stack_heavy_fracs(3, 9)
    total = shape.n_kv_heads * 600             # the first step evicts nothing
    run_cascade(lava, shape, 3, total, dict(base=300, fracs=fr), use_gpu_scores=False, in_place=in_place)
    desc = lava.LayerDesc.make(shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.window, shape.dtype)
    state = lava.CascadeState(desc, 1, total + 1, in_place=in_place)
    arenas = 1 if in_place else 2
    assert state.bytes() < (arenas + 0.5) * (total + 1) * (2 * shape.head_dim * 4 + 12)   # arenas + scratch, not per layer
    dummy = torch.zeros(shape.n_kv_heads * 600 * shape.head_dim, dtype=torch.float32, device="cuda")
    with pytest.raises(lava.LavaError) as ei:   # more than the layers seen so far can hold: infeasible, as in the oracle
        lava.lava_cascade_step(desc, 0, 600, dummy, dummy, dummy[: shape.n_kv_heads * 600], state, total + 1)
    assert ei.value.status == lava.LAVA_ERR_BUDGET


def test_compact_packed_matches_oracle(lava):
    say("compact_packed: gather from a packed source with positions")
    rng = np.random.Generator(np.random.PCG64(5))
    Hkv, d = 4, 64
    desc = lava.LayerDesc.make(8, Hkv, d, 8, "bf16")
    src_counts = np.array([300, 0, 17, 1000])
    src_offs = np.concatenate([[0], np.cumsum(src_counts)]).astype(np.int64)
    rows = int(src_offs[-1])
    k_src = synth.store(rng.standard_normal((rows + 9, d), dtype=np.float32), "bf16")
    v_src = synth.store(rng.standard_normal((rows + 9, d), dtype=np.float32), "bf16")
    pos_src = rng.integers(0, 100000, rows + 9).astype(np.int32)
    keep = [np.sort(rng.choice(c, size=min(c, m), replace=False)) for c, m in zip(src_counts, [100, 0, 17, 3])]
    new_offs = np.concatenate([[0], np.cumsum([len(x) for x in keep])]).astype(np.int64)
    idx = np.concatenate(keep).astype(np.int32)
    cap = int(new_offs[-1])
    k_out = torch.full((cap + 4, d), 3.0, dtype=torch.bfloat16, device="cuda")
    v_out = torch.full((cap + 4, d), 3.0, dtype=torch.bfloat16, device="cuda")
    pos_out = torch.full((cap + 4,), -9, dtype=torch.int32, device="cuda")
    lava.lava_compact_packed(desc, torch.from_numpy(src_offs).cuda(), lava.to_device(k_src, "bf16"),
                             lava.to_device(v_src, "bf16"), torch.from_numpy(new_offs).cuda(),
                             torch.from_numpy(idx).cuda(), cap, pos_src=torch.from_numpy(pos_src).cuda(),
                             k_out=k_out, v_out=v_out, pos_out=pos_out)
    torch.cuda.synchronize()
    src_row = np.concatenate([src_offs[g] + keep[g] for g in range(Hkv)])
    assert np.array_equal(lava.to_host_bits(k_out[:cap]), k_src[src_row])
    assert np.array_equal(lava.to_host_bits(v_out[:cap]), v_src[src_row])
    assert np.array_equal(pos_out[:cap].cpu().numpy(), pos_src[src_row])
    assert torch.all(k_out[cap:] == 3.0) and torch.all(pos_out[cap:] == -9)       # nothing past the survivors


def test_select_reads_total_from_segment_offsets(lava):
    say("select: total_entries is an upper bound when segment offsets are given")
    nh = 4
    s = synth.random_scores(1, 5000, 8).ravel()
    offs = np.array([0, 1000, 1000, 2600, 3100], dtype=np.int64)                  # 3100 of 5000 entries exist
    sc = torch.from_numpy(s).cuda()
    counts, o, idx, ks = lava.lava_select_topk(nh, sc, 700, seg_offsets=torch.from_numpy(offs).cuda())
    torch.cuda.synchronize()
    rc, ro, ri, rs = O.select_topk(s[:3100].astype(np.float64), offs, 700)
    assert np.array_equal(counts.cpu().numpy(), rc) and np.array_equal(o.cpu().numpy(), ro)
    assert np.array_equal(idx.cpu().numpy()[:700], ri)
    # budget above what exists: everything that exists is kept
    counts, o, idx, ks = lava.lava_select_topk(nh, sc, 4000, seg_offsets=torch.from_numpy(offs).cuda())
    torch.cuda.synchronize()
    assert counts.cpu().numpy().tolist() == [1000, 0, 1600, 500] and int(o[-1]) == 3100


@ARENAS
def test_decode_reads_a_cascade_layer_in_place(lava, in_place):
    say("cascade: decode attention over layer 1 of a 3-layer state, straight from the arena")
    shape = synth.config(2, n=2048 + 9, budget=512)
    fr = synth.stack_heavy_fracs(3, 2)
    state, _ = run_cascade(lava, shape, 3, 3 * 512, dict(base=400, fracs=fr), use_gpu_scores=True, in_place=in_place)
    H, Hkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    desc = lava.LayerDesc.make(H, Hkv, d, shape.window, shape.dtype)
    r = np.random.Generator(np.random.PCG64(8))
    q_new = synth.store(r.standard_normal((1, H, d), dtype=np.float32), shape.dtype)
    args = state.decode_args(1)
    out, lse = lava.lava_decode_attention(desc, 1, lava.to_device(q_new, shape.dtype), args["k_hat"], args["v_hat"],
                                          args["head_offsets"], args["rows_capacity"], seq_base=args["seq_base"])
    torch.cuda.synchronize()
    cur = state.current(1)
    want, want_lse = O.decode_attention(synth.load_f64(q_new, shape.dtype)[0],
                                        synth.load_f64(lava.to_host_bits(cur["k_hat"]), shape.dtype),
                                        synth.load_f64(lava.to_host_bits(cur["v_hat"]), shape.dtype),
                                        cur["head_offsets"].cpu().numpy())
    got = out.cpu().numpy()[0]
    for h in range(H):
        assert np.abs(got[h] - want[h]).max() <= 2e-5 * np.abs(want[h]).max()
    assert np.allclose(lse.cpu().numpy()[0], want_lse, rtol=1e-5, atol=1e-5)


def test_in_place_step_with_a_wait_that_gives_up_marks_the_state(lava, tuning):
    """The waits of a step are bounded (the selections' and the in-place gather's grid barriers).  With the
    bound at a single poll, set from the host, every kernel still runs to its end and the state's error word
    is set; the same steps with the default bound leave it clear."""
    say("cascade in place: forced give-up of the bounded waits")
    shape = synth.config(2, n=16384 + 3, budget=0)
    H, Hkv, d, N, w = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.n, shape.window
    desc = lava.LayerDesc.make(H, Hkv, d, w, shape.dtype)
    total = 3 * 24000
    for spin, expect in ((0, 0), (1, 1)):
        state = lava.CascadeState(desc, 3, total, in_place=True)
        ws = None
        for l in range(3):
            inp = synth.gen_layer(shape, 700 + l)
            q_dev, k_dev, v_dev = (lava.to_device(a, shape.dtype) for a in (inp.q_win, inp.k, inp.v))
            sc_dev, _, _ = lava.lava_window_scores(desc, [N], q_dev, k_dev, v_dev, layer_stat=state.e[l: l + 1])
            if l == 2:
                tuning(barrier_spin_limit=spin)
            ws = lava.lava_cascade_step(desc, l, N, k_dev, v_dev, sc_dev, state, total, workspace=ws)
            torch.cuda.synchronize()
            tuning()
        assert int(state.error[0]) == expect, spin
        if not expect:
            starts = state.layer_start[state.cur].cpu().numpy()
            assert starts[0] == 0 and starts[3] == total
