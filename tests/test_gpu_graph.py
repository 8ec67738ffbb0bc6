"""The whole path is capturable in a HIP graph: the library allocates nothing, synchronises nothing
and records no memset nodes, so one layer's calls (scores -> device budgets -> selection with a
device-side budget -> compaction -> a decode step over the result) can be replayed as one graph.
Every replay is checked against the eager result, with eager work in between."""
import numpy as np
import pytest
import torch

from paper_2509_09754_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lava():
    from paper_2509_09754_amd import lava as mod
    assert torch.cuda.is_available()
    return mod


@pytest.mark.parametrize("composed", [False, True], ids=["plain-calls", "prepared-selection-and-planned-budget"])
def test_layer_eviction_replays_from_a_graph(lava, composed):
    """composed: the scores call prepares the selection's workspace and forms the budget itself (four
    launches for the eviction instead of seven); the clearing those calls rely on is done by kernels, so
    the sequence is as capturable as the plain one."""
    print(f"graph: capture one layer's eviction + decode (composed={composed}), replay 4 times on changing inputs",
          flush=True)
    sh = synth.config(2, n=8192 + 40, budget=2048)
    H, Hkv, d, N, w, B = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.n, sh.window, sh.budget
    desc = lava.LayerDesc.make(H, Hkv, d, w, sh.dtype)
    dev = "cuda"
    layers = [synth.gen_layer(sh, seed) for seed in (0, 1, 2)]
    q, k, v = (lava.to_device(a, sh.dtype, dev).clone() for a in (layers[0].q_win, layers[0].k, layers[0].v))
    q_new = torch.randn(1, H, d, device=dev).to(desc.torch_dtype)

    bufs = dict(
        ws_scores=torch.empty(lava.lava_window_scores_workspace_bytes(desc, 1, N), dtype=torch.uint8, device=dev),
        ws_sel=torch.empty(lava.lava_select_workspace_bytes(Hkv * N), dtype=torch.uint8, device=dev),
        ws_dec=torch.empty(lava.lava_decode_workspace_bytes(desc, 1, B), dtype=torch.uint8, device=dev),
        scores=torch.empty(Hkv * N, dtype=torch.float32, device=dev),
        vbar=torch.empty(1, Hkv, dtype=torch.float32, device=dev),
        stat=torch.empty(1, dtype=torch.float32, device=dev),
        budgets=torch.empty(1, 1, dtype=torch.int64, device=dev),
        total=torch.tensor([B - 100], dtype=torch.int64, device=dev),
        lo=torch.tensor([[Hkv * w]], dtype=torch.int64, device=dev),
        hi=torch.tensor([[Hkv * N]], dtype=torch.int64, device=dev),
        counts=torch.empty(Hkv, dtype=torch.int32, device=dev),
        offs=torch.empty(1, Hkv + 1, dtype=torch.int64, device=dev),
        idx=torch.full((B,), -1, dtype=torch.int32, device=dev),
        kept=torch.empty(B, dtype=torch.float32, device=dev),
        k_hat=torch.zeros(B, d, dtype=desc.torch_dtype, device=dev),
        v_hat=torch.zeros(B, d, dtype=desc.torch_dtype, device=dev),
        out=torch.empty(1, H, d, dtype=torch.float32, device=dev),
        lse=torch.empty(1, H, dtype=torch.float32, device=dev),
    )

    e_table = torch.zeros(1, 1, dtype=torch.float32, device=dev)
    plan = lava.make_budget_plan(e_table, 0, bufs["total"], bufs["lo"], bufs["hi"], bufs["budgets"]) if composed else None

    def step():
        b = bufs
        lava.lava_window_scores(desc, [N], q, k, v, scores=b["scores"], vbar=b["vbar"], layer_stat=b["stat"],
                                workspace=b["ws_scores"], select_workspace=b["ws_sel"] if composed else None,
                                budget_plan=plan)
        if not composed:
            lava.lava_layer_budgets(b["stat"].view(1, 1), b["total"], b["lo"], b["hi"], budgets=b["budgets"])
        lava.lava_select_topk(Hkv, b["scores"], B, budget_dev=b["budgets"].view(-1), head_counts=b["counts"],
                              head_offsets=b["offs"].view(-1), kept_idx=b["idx"], kept_scores=b["kept"],
                              workspace=b["ws_sel"], primed=composed)
        lava.lava_compact_kv(desc, N, k, v, b["offs"].view(-1), b["idx"], B, k_out=b["k_hat"], v_out=b["v_hat"])
        lava.lava_decode_attention(desc, 1, q_new, b["k_hat"], b["v_hat"], b["offs"], B, out=b["out"], lse=b["lse"],
                                   workspace=b["ws_dec"])

    def snapshot():
        torch.cuda.synchronize()
        return {n: bufs[n].clone() for n in ("scores", "stat", "budgets", "counts", "offs", "idx", "kept", "k_hat",
                                             "v_hat", "out", "lse")}

    step()                                   # eager warm-up (also loads every kernel before capture)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)

    for rep in range(4):
        src = layers[rep % 3]
        for dst, arr in ((q, src.q_win), (k, src.k), (v, src.v)):
            dst.copy_(lava.to_device(arr, sh.dtype, dev))
        step()
        want = snapshot()
        for name in ("scores", "idx", "kept", "k_hat", "out"):   # scribble over outputs: the replay must rewrite them
            bufs[name].fill_(0)
        bufs["budgets"].fill_(-5)
        (torch.rand(1 << 20, device=dev) * 2).sum().item()      # unrelated eager work and a synchronisation in between
        graph.replay()
        got = snapshot()
        kept = int(want["offs"][0, -1])
        assert kept == B - 100
        for name in want:
            a, b = want[name], got[name]
            if name in ("idx", "kept", "k_hat", "v_hat"):
                a, b = a[:kept], b[:kept]
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (rep, name)
        assert lava.lava_select_status(bufs["ws_sel"], Hkv * N) == lava.LAVA_OK


@pytest.mark.parametrize("in_place", [False, True], ids=["two-arenas", "one-arena-in-place"])
def test_cascade_of_three_layers_replays_from_a_graph(lava, in_place):
    print(f"graph: capture three cascade steps (scores + step per layer, in_place={in_place}), replay 3 times", flush=True)
    sh = synth.config(2, n=4096 + 21, budget=0)
    H, Hkv, d, N, w = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.n, sh.window
    L, total = 3, 3 * 700
    desc = lava.LayerDesc.make(H, Hkv, d, w, sh.dtype)
    dev = "cuda"
    inps = [[synth.gen_layer(sh, 10 * r + l) for l in range(L)] for r in range(2)]
    q = [lava.to_device(inps[0][l].q_win, sh.dtype, dev).clone() for l in range(L)]
    k = [lava.to_device(inps[0][l].k, sh.dtype, dev).clone() for l in range(L)]
    v = [lava.to_device(inps[0][l].v, sh.dtype, dev).clone() for l in range(L)]
    state = lava.CascadeState(desc, L, total, device=dev, in_place=in_place)
    scores = torch.empty(L, Hkv * N, dtype=torch.float32, device=dev)
    vbar = torch.empty(L, Hkv, dtype=torch.float32, device=dev)
    ws_s = torch.empty(lava.lava_window_scores_workspace_bytes(desc, 1, N), dtype=torch.uint8, device=dev)
    ws_c = torch.empty(lava.lava_cascade_workspace_bytes(desc, N, L, total), dtype=torch.uint8, device=dev)

    def run():
        state.reset()
        for l in range(L):
            lava.lava_window_scores(desc, [N], q[l], k[l], v[l], scores=scores[l], vbar=vbar[l: l + 1],
                                    layer_stat=state.e[l: l + 1], workspace=ws_s)
            lava.lava_cascade_step(desc, l, N, k[l], v[l], scores[l], state, total, workspace=ws_c)

    def snapshot():
        torch.cuda.synchronize()
        c = state.cur
        return [t.clone() for t in (state.budgets, state.layer_start[c], state.head_offsets[c], state.head_counts,
                                    state.pos[c][:total], state.scores[c][:total], state.k[c][:total], state.v[c][:total])]

    run()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.current_stream().wait_stream(side)
    final_cur = state.cur                                   # an odd number of steps: the state ends in arena 1
    for rep in range(3):
        src = inps[rep % 2]
        for l in range(L):
            q[l].copy_(lava.to_device(src[l].q_win, sh.dtype, dev))
            k[l].copy_(lava.to_device(src[l].k, sh.dtype, dev))
            v[l].copy_(lava.to_device(src[l].v, sh.dtype, dev))
        run()
        want = snapshot()
        assert state.cur == final_cur and int(want[1][-1]) == total
        for i in range(2):                                   # scribble over both arenas: the replay must rewrite them
            state.k[i].fill_(0), state.pos[i].fill_(-1), state.scores[i].fill_(0)
        (torch.rand(1 << 20, device=dev) * 2).sum().item()
        graph.replay()
        got = snapshot()
        for a, b in zip(want, got):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), rep
