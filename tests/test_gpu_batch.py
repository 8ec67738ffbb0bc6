"""Tables of selections / compactions (lava_select_topk_batch, lava_compact_batch) against the oracle.

Every problem of a table is one Alg.-1 selection or compaction, so each must equal the oracle's
result for that problem alone, bit for bit, whatever else shares the launch.
"""
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


def run_select_table(lava, nh, cases, seed):
    """cases: list of (entries per head, budget, explicit segments?, device budget?)."""
    dev = "cuda"
    keep, probs, refs = [], [], []
    widest = 0
    for i, (n, budget, ragged, dev_budget) in enumerate(cases):
        s = synth.random_scores(nh, n, seed + i).ravel()
        total = s.size
        if ragged:
            r = np.random.Generator(np.random.PCG64(seed + 100 + i))
            cuts = np.sort(r.integers(0, total + 1, nh - 1))
            offs = np.concatenate([[0], cuts, [total]]).astype(np.int64)
        else:
            offs = (np.arange(nh + 1) * n).astype(np.int64)
        cap = budget
        bd = None
        if dev_budget:                       # the device value wins; the host value is the capacity of the outputs
            cap = min(total, budget + 50)
            bd = torch.tensor([budget], dtype=torch.int64, device=dev)
        sc = torch.from_numpy(s).to(dev)
        t = dict(scores=sc, counts=torch.full((nh,), -7, dtype=torch.int32, device=dev),
                 offs=torch.full((nh + 1,), -7, dtype=torch.int64, device=dev),
                 idx=torch.full((max(cap, 1),), -7, dtype=torch.int32, device=dev),
                 ks=torch.full((max(cap, 1),), -7.0, dtype=torch.float32, device=dev),
                 seg=torch.from_numpy(offs).to(dev) if ragged else None, bd=bd)
        keep.append(t)
        probs.append(lava.select_problem(sc, cap, t["counts"], t["offs"], t["idx"], t["ks"], seg_offsets=t["seg"],
                                         budget_dev=bd))
        refs.append((O.select_topk(s.astype(np.float64), offs, budget), s, budget))
        widest = max(widest, total)
    ws = lava.lava_select_topk_batch(nh, probs, widest)
    torch.cuda.synchronize()
    assert lava.lava_select_batch_status(ws, len(probs), widest) == lava.LAVA_OK
    for i, (t, ((rc, ro, ri, rs), s, budget)) in enumerate(zip(keep, refs)):
        assert np.array_equal(t["counts"].cpu().numpy(), rc), i
        assert np.array_equal(t["offs"].cpu().numpy(), ro), i
        assert np.array_equal(t["idx"].cpu().numpy()[:budget], ri), i
        assert np.array_equal(t["ks"].cpu().numpy()[:budget].view(np.uint32),
                              np.asarray(rs, dtype=np.float32).view(np.uint32)), i
        if budget < t["idx"].numel():
            assert torch.all(t["idx"][budget:] == -7), i        # nothing past the survivors
    return keep


def test_select_table_mixed_sizes(lava):
    say("select batch: 7 problems of mixed size, segments and budget sources in one launch")
    cases = [(1000, 300, False, False), (17, 17 * 4, False, False), (5000, 1, True, True), (40000, 12345, True, False),
             (1, 0, False, False), (16384 * 2 + 3, 4000, False, True), (300, 1200, True, False)]
    run_select_table(lava, 4, cases, 11)


def test_select_table_more_problems_than_one_launch_holds(lava):
    say("select batch: 40 problems (two tables), then problems wide enough to need several launches")
    r = np.random.Generator(np.random.PCG64(3))
    cases = [(int(r.integers(1, 3000)), 0, bool(i % 2), bool(i % 3 == 0)) for i in range(40)]
    cases = [(n, int(r.integers(0, 8 * n + 1)), rg, db) for (n, _, rg, db) in cases]
    run_select_table(lava, 8, cases, 50)
    # 6 problems of 64 workgroups each and one of a single workgroup: more than one launch's share
    wide = [(131072, 4096 + 100 * i, bool(i % 2), True) for i in range(6)] + [(100, 37, False, False)]
    run_select_table(lava, 8, wide, 70)


def test_select_table_equals_single_calls(lava):
    say("select batch: results identical to one lava_select_topk call per problem, ties included")
    nh = 8
    dev = "cuda"
    r = np.random.Generator(np.random.PCG64(9))
    probs, outs, singles = [], [], []
    for i in range(5):
        n = 3000 + 700 * i
        s = np.round(r.standard_normal(nh * n) * 4).astype(np.float32)          # heavy ties
        sc = torch.from_numpy(s).to(dev)
        budget = 500 + 333 * i
        o = [torch.empty(nh, dtype=torch.int32, device=dev), torch.empty(nh + 1, dtype=torch.int64, device=dev),
             torch.empty(budget, dtype=torch.int32, device=dev), torch.empty(budget, dtype=torch.float32, device=dev)]
        probs.append(lava.select_problem(sc, budget, *o))
        outs.append((sc, o))
        singles.append(lava.lava_select_topk(nh, sc, budget))
    lava.lava_select_topk_batch(nh, probs)
    torch.cuda.synchronize()
    for (sc, o), single in zip(outs, singles):
        for a, b in zip(o, single):
            assert torch.equal(a, b)


def test_compact_table_matches_oracle(lava):
    say("compact batch: dense and packed sources of different sizes in one launch")
    dev = "cuda"
    Hkv, d = 4, 128
    desc = lava.LayerDesc.make(8, Hkv, d, 8, "bf16")
    r = np.random.Generator(np.random.PCG64(21))
    probs, checks, hold = [], [], []
    for i, n in enumerate([700, 64, 5000, 1]):
        dense = i % 2 == 0
        if dense:
            src_counts = np.full(Hkv, n)
            src_offs = None
        else:
            src_counts = r.integers(0, n + 1, Hkv)
            src_offs = np.concatenate([[0], np.cumsum(src_counts)]).astype(np.int64)
        rows = int(src_counts.sum())
        pool = max(rows, 1) + 3
        k_src = synth.store(r.standard_normal((pool, d), dtype=np.float32), "bf16")
        v_src = synth.store(r.standard_normal((pool, d), dtype=np.float32), "bf16")
        pos_src = r.integers(0, 1 << 20, pool).astype(np.int32)
        kept = [np.sort(r.choice(c, size=int(r.integers(0, c + 1)), replace=False)) if c else np.zeros(0, dtype=np.int64)
                for c in src_counts]
        new_offs = np.concatenate([[0], np.cumsum([len(x) for x in kept])]).astype(np.int64)
        idx = np.concatenate(kept).astype(np.int32) if new_offs[-1] else np.zeros(1, dtype=np.int32)
        cap = int(new_offs[-1])
        starts = np.arange(Hkv) * n if dense else src_offs[:-1]
        src_row = np.concatenate([starts[g] + kept[g] for g in range(Hkv)]).astype(np.int64)
        t = dict(k=lava.to_device(k_src, "bf16", dev), v=lava.to_device(v_src, "bf16", dev),
                 pos=torch.from_numpy(pos_src).to(dev), offs=torch.from_numpy(new_offs).to(dev),
                 idx=torch.from_numpy(idx).to(dev),
                 src=None if dense else torch.from_numpy(src_offs).to(dev),
                 ko=torch.full((cap + 2, d), 5.0, dtype=torch.bfloat16, device=dev),
                 vo=torch.full((cap + 2, d), 5.0, dtype=torch.bfloat16, device=dev),
                 po=torch.full((cap + 2,), -3, dtype=torch.int32, device=dev))
        hold.append(t)
        probs.append(lava.compact_problem(desc, n if dense else pool, t["k"], t["v"], t["offs"], t["idx"], cap, t["ko"],
                                          t["vo"], src_offsets=t["src"], pos_src=None if dense else t["pos"],
                                          pos_out=t["po"]))
        want_pos = np.concatenate(kept).astype(np.int32) if dense else pos_src[src_row]
        checks.append((cap, k_src[src_row], v_src[src_row], want_pos))
    lava.lava_compact_batch(desc, probs)
    torch.cuda.synchronize()
    for i, (t, (cap, wk, wv, wp)) in enumerate(zip(hold, checks)):
        assert np.array_equal(lava.to_host_bits(t["ko"][:cap]), wk), i
        assert np.array_equal(lava.to_host_bits(t["vo"][:cap]), wv), i
        assert np.array_equal(t["po"][:cap].cpu().numpy(), wp), i
        assert torch.all(t["ko"][cap:] == 5.0) and torch.all(t["po"][cap:] == -3), i


def test_ragged_batch_full_size_one_layer(lava):
    """The batched serving configuration at full size (16 sequences of 4K-64K tokens, one layer), in the
    launch configuration the benchmark times: one lava_window_scores call for the batch, device budgets,
    one table of selections and one of compactions.  Scores and statistics against the oracle per
    sequence; selection and compaction bit-exact on the scores the GPU produced."""
    lens = [int(x) for x in synth.ragged_lengths(16, 0)]
    say(f"ragged batch, full size: lengths {lens}")
    base = synth.config(5)
    H, Hkv, d, w = base.n_q_heads, base.n_kv_heads, base.head_dim, base.window
    B = 4096
    desc = lava.LayerDesc.make(H, Hkv, d, w, base.dtype)
    dev = "cuda"
    inps = [synth.gen_layer(synth.config(5, n=n, budget=B), 900 + b) for b, n in enumerate(lens)]
    q = torch.cat([lava.to_device(i.q_win, "bf16").reshape(-1) for i in inps])
    k = torch.cat([lava.to_device(i.k, "bf16").reshape(-1) for i in inps])
    v = torch.cat([lava.to_device(i.v, "bf16").reshape(-1) for i in inps])
    scores, vbar, stat = lava.lava_window_scores(desc, lens, q, k, v)
    nb = len(lens)
    total_b = torch.full((nb,), B, dtype=torch.int64, device=dev)
    lo = torch.full((nb, 1), Hkv * w, dtype=torch.int64, device=dev)
    hi = torch.tensor([[Hkv * n] for n in lens], dtype=torch.int64, device=dev)
    budgets = lava.lava_layer_budgets(stat.view(-1, 1), total_b, lo, hi)
    counts = torch.empty(nb, Hkv, dtype=torch.int32, device=dev)
    offs = torch.empty(nb, Hkv + 1, dtype=torch.int64, device=dev)
    idx = torch.empty(nb, B, dtype=torch.int32, device=dev)
    k_hat = torch.empty(nb, B, d, dtype=torch.bfloat16, device=dev)
    v_hat = torch.empty(nb, B, d, dtype=torch.bfloat16, device=dev)
    starts = np.concatenate([[0], np.cumsum(lens)])
    sel, cmp = [], []
    for b, n in enumerate(lens):
        a0, a1 = int(starts[b]) * Hkv, int(starts[b + 1]) * Hkv
        sel.append(lava.select_problem(scores[a0:a1], B, counts[b], offs[b], idx[b], budget_dev=budgets[b]))
        cmp.append(lava.compact_problem(desc, n, k.view(-1, d)[a0:a1], v.view(-1, d)[a0:a1], offs[b], idx[b], B,
                                        k_hat[b], v_hat[b]))
    ws = lava.lava_select_topk_batch(Hkv, sel, Hkv * max(lens))
    lava.lava_compact_batch(desc, cmp)
    torch.cuda.synchronize()
    assert lava.lava_select_batch_status(ws, nb, Hkv * max(lens)) == lava.LAVA_OK
    assert budgets.cpu().numpy().ravel().tolist() == [B] * nb          # one layer: the whole budget
    s_host, vb_host, e_host = scores.cpu().numpy(), vbar.cpu().numpy(), stat.cpu().numpy()
    worst, least = 0.0, 1.0
    for b, (n, inp) in enumerate(zip(lens, inps)):
        qq, kk, vv = inp.f64()
        ref_s, ref_vbar = O.lava_scores(qq, kk, vv, w, 7)
        got = s_host[Hkv * starts[b]: Hkv * starts[b + 1]].reshape(Hkv, n)
        Np = n - w
        assert np.all(np.isposinf(got[:, Np:]))
        mask = ref_s > 1e-30 * ref_s.max()
        rel = np.abs(got[:, :Np].astype(np.float64)[mask] - ref_s[mask]) / ref_s[mask]
        worst = max(worst, float(rel.max()))
        assert rel.max() < 1e-3, (b, rel.max())
        np.testing.assert_allclose(vb_host[b], ref_vbar, rtol=1e-5)
        ref_e = O.layer_entropy(ref_s)
        assert abs(float(e_host[b]) - ref_e) <= 1e-4 * ref_e + 2e-5 / ref_s.size
        # selection: exact on the GPU's own scores; kept set against the oracle's scores
        uniform = (np.arange(Hkv + 1) * n).astype(np.int64)
        rc, ro, ri, _ = O.select_topk(got.astype(np.float64).ravel(), uniform, B)
        assert np.array_equal(counts[b].cpu().numpy(), rc) and np.array_equal(offs[b].cpu().numpy(), ro)
        assert np.array_equal(idx[b].cpu().numpy(), ri)
        flat_ref = O.flat_layer_scores(ref_s, n)
        oc, oo, oi, _ = O.select_topk(flat_ref.ravel(), uniform, B)
        mine = set(int(g * n + p) for g in range(Hkv) for p in ri[ro[g]:ro[g + 1]])
        theirs = set(int(g * n + p) for g in range(Hkv) for p in oi[oo[g]:oo[g + 1]])
        least = min(least, len(mine & theirs) / B)
        assert np.all(rc >= w)
        # compaction: bit copies of the selected rows
        assert np.array_equal(lava.to_host_bits(k_hat[b]), O.compact(inp.k, ro, ri))
        assert np.array_equal(lava.to_host_bits(v_hat[b]), O.compact(inp.v, ro, ri))
    say(f"   worst score error {worst:.2e}, least kept-set overlap {least:.5f}")
    assert least >= 0.999


def test_ragged_batch_several_layers_dynamic_budgets(lava):
    """The batched serving configuration as a stack: 16 ragged sequences (one of them only w + 1 tokens
    long) x 4 layers, every sequence with its own total budget split over its layers by the layer
    statistics (batched lava_layer_budgets on the device), then one table of selections and one of
    compactions over all (sequence, layer) pairs.  The expected values come from the oracle alone, per
    sequence, from the raw inputs: statistics -> budgets -> kept sets; the GPU's budgets may differ from
    them by one unit per layer (fp32 statistics on a rounding boundary), selections are bit-exact on the
    scores the GPU produced, kept sets overlap the oracle's >= 99.9 %, rows are bit copies."""
    L = 4
    base = synth.config(5)
    H, Hkv, d, w = base.n_q_heads, base.n_kv_heads, base.head_dim, base.window
    lens = [int(x) for x in synth.ragged_lengths(15, 3)]
    lens.insert(6, w + 1)                                       # one prefix token per head
    nb = len(lens)
    per_layer = Hkv * 256
    totals = [min(L * per_layer, L * Hkv * n - (L if n > w + 1 else 8)) for n in lens]
    say(f"ragged stack: {L} layers, lengths {lens}, totals {totals}")
    desc = lava.LayerDesc.make(H, Hkv, d, w, base.dtype)
    dev = "cuda"
    starts = np.concatenate([[0], np.cumsum(lens)])
    tok = int(starts[-1])
    stat = torch.zeros(nb, L, dtype=torch.float32, device=dev)
    scores = torch.empty(L, Hkv * tok, dtype=torch.float32, device=dev)
    k_dev = torch.empty(L, Hkv * tok, d, dtype=torch.bfloat16, device=dev)
    v_dev = torch.empty(L, Hkv * tok, d, dtype=torch.bfloat16, device=dev)
    ref_e = np.zeros((nb, L))
    ref_scores = [[None] * L for _ in range(nb)]
    host_rows = [[None] * L for _ in range(nb)]
    ws = torch.empty(lava.lava_window_scores_workspace_bytes(desc, nb, tok), dtype=torch.uint8, device=dev)
    for l in range(L):
        inps = [synth.gen_layer(synth.config(5, n=n, budget=Hkv * w), 7000 + 100 * l + b) for b, n in enumerate(lens)]
        q = torch.cat([lava.to_device(i.q_win, "bf16").reshape(-1) for i in inps])
        k_dev[l] = torch.cat([lava.to_device(i.k, "bf16").reshape(-1, d) for i in inps])
        v_dev[l] = torch.cat([lava.to_device(i.v, "bf16").reshape(-1, d) for i in inps])
        e_l = torch.empty(nb, dtype=torch.float32, device=dev)
        lava.lava_window_scores(desc, lens, q, k_dev[l], v_dev[l], scores=scores[l], layer_stat=e_l, workspace=ws)
        stat[:, l] = e_l
        for b, inp in enumerate(inps):
            qq, kk, vv = inp.f64()
            ref_scores[b][l], _ = O.lava_scores(qq, kk, vv, w, 7)
            ref_e[b, l] = O.layer_entropy(ref_scores[b][l])
            host_rows[b][l] = (inp.k, inp.v)
        say(f"   layer {l}: generated, scored on the GPU and by the oracle")
    torch.cuda.synchronize()
    e_host = stat.cpu().numpy()
    for b in range(nb):
        for l in range(L):
            assert abs(float(e_host[b, l]) - ref_e[b, l]) <= 1e-4 * ref_e[b, l] + 2e-5 / ref_scores[b][l].size, (b, l)

    total_t = torch.tensor(totals, dtype=torch.int64, device=dev)
    lo = torch.full((nb, L), Hkv * w, dtype=torch.int64, device=dev)
    hi = torch.tensor([[Hkv * n] * L for n in lens], dtype=torch.int64, device=dev)
    budgets = lava.lava_layer_budgets(stat, total_t, lo, hi)
    cap = [min(totals[b], Hkv * lens[b]) for b in range(nb)]
    counts = torch.empty(nb, L, Hkv, dtype=torch.int32, device=dev)
    offs = torch.empty(nb, L, Hkv + 1, dtype=torch.int64, device=dev)
    idx = [[torch.full((cap[b] + 4,), -7, dtype=torch.int32, device=dev) for _ in range(L)] for b in range(nb)]
    k_hat = [[torch.full((cap[b] + 1, d), 3.0, dtype=torch.bfloat16, device=dev) for _ in range(L)] for b in range(nb)]
    v_hat = [[torch.full((cap[b] + 1, d), 3.0, dtype=torch.bfloat16, device=dev) for _ in range(L)] for b in range(nb)]
    err = torch.zeros(1, dtype=torch.int32, device=dev)
    sel, cmp = [], []
    for b, n in enumerate(lens):
        a0, a1 = int(starts[b]) * Hkv, int(starts[b + 1]) * Hkv
        for l in range(L):
            sel.append(lava.select_problem(scores[l][a0:a1], cap[b], counts[b, l], offs[b, l], idx[b][l],
                                           budget_dev=budgets[b, l: l + 1], error_dev=err))
            cmp.append(lava.compact_problem(desc, n, k_dev[l][a0:a1], v_dev[l][a0:a1], offs[b, l], idx[b][l], cap[b],
                                            k_hat[b][l], v_hat[b][l]))
    lava.lava_select_topk_batch(Hkv, sel, Hkv * max(lens))
    lava.lava_compact_batch(desc, cmp)
    torch.cuda.synchronize()
    assert int(err[0]) == 0
    got_budgets = budgets.cpu().numpy()
    s_host = scores.cpu().numpy()
    counts_h, offs_h = counts.cpu().numpy(), offs.cpu().numpy()
    least, worst_delta = 1.0, 0
    for b, n in enumerate(lens):
        want = O.layer_budgets(ref_e[b], totals[b], [Hkv * w] * L, [Hkv * n] * L)
        assert int(got_budgets[b].sum()) == totals[b] == sum(want)
        assert np.all(got_budgets[b] >= Hkv * w) and np.all(got_budgets[b] <= Hkv * n)
        worst_delta = max(worst_delta, int(np.abs(got_budgets[b] - np.asarray(want)).max()))
        # the same allocation rule on the statistics the GPU produced: exact
        assert got_budgets[b].tolist() == O.layer_budgets(e_host[b].astype(np.float64), totals[b], [Hkv * w] * L,
                                                          [Hkv * n] * L)
        uniform = (np.arange(Hkv + 1) * n).astype(np.int64)
        a0, a1 = int(starts[b]) * Hkv, int(starts[b + 1]) * Hkv
        for l in range(L):
            B_gpu, B_ref = int(got_budgets[b, l]), int(want[l])
            got = s_host[l][a0:a1].reshape(Hkv, n)
            assert np.all(np.isposinf(got[:, n - w:]))
            mask = ref_scores[b][l] > 1e-30 * ref_scores[b][l].max()
            rel = np.abs(got[:, : n - w].astype(np.float64)[mask] - ref_scores[b][l][mask]) / ref_scores[b][l][mask]
            assert rel.max() < 1e-3, (b, l, rel.max())
            rc, ro, ri, _ = O.select_topk(got.astype(np.float64).ravel(), uniform, B_gpu)
            i_h = idx[b][l].cpu().numpy()
            assert np.array_equal(counts_h[b, l], rc) and np.array_equal(offs_h[b, l], ro), (b, l)
            assert np.array_equal(i_h[:B_gpu], ri) and np.all(i_h[cap[b]:] == -7), (b, l)
            assert np.all(rc >= w) and rc.sum() == B_gpu                     # Eq. 1
            oc, oo, oi, _ = O.select_topk(O.flat_layer_scores(ref_scores[b][l], n).ravel(), uniform, B_ref)
            mine = set(int(g * n + p) for g in range(Hkv) for p in ri[ro[g]:ro[g + 1]])
            theirs = set(int(g * n + p) for g in range(Hkv) for p in oi[oo[g]:oo[g + 1]])
            least = min(least, len(mine & theirs) / min(B_gpu, B_ref))
            kk, vv = host_rows[b][l]
            assert np.array_equal(lava.to_host_bits(k_hat[b][l][:B_gpu]), O.compact(kk, ro, ri)), (b, l)
            assert np.array_equal(lava.to_host_bits(v_hat[b][l][:B_gpu]), O.compact(vv, ro, ri)), (b, l)
            assert bool((k_hat[b][l][B_gpu:] == 3.0).all()), (b, l)
    say(f"   budgets vs the oracle's: max |difference| {worst_delta}; least kept-set overlap {least:.5f}")
    assert worst_delta <= 1 and least >= 0.999


def test_tables_with_device_side_offsets(lava):
    """Problems whose data sit back to back in shared buffers at offsets only the device knows (the layout
    of the cascade's pools): selection reads / writes at the offsets, compaction gathers from and to them."""
    say("select + compact batch: packed inputs and outputs addressed through device-side offsets")
    dev = "cuda"
    Hkv, d = 4, 64
    desc = lava.LayerDesc.make(8, Hkv, d, 8, "bf16")
    r = np.random.Generator(np.random.PCG64(33))
    held = [900, 40, 3000]                                    # rows each source layer holds
    budgets = [300, 40, 1111]
    src_start = np.concatenate([[0], np.cumsum(held)]).astype(np.int64)
    out_start = np.concatenate([[0], np.cumsum(budgets)]).astype(np.int64)
    pool = int(src_start[-1]) + 7
    k_src = synth.store(r.standard_normal((pool, d), dtype=np.float32), "bf16")
    v_src = synth.store(r.standard_normal((pool, d), dtype=np.float32), "bf16")
    pos_src = r.integers(0, 1 << 20, pool).astype(np.int32)
    sc_src = synth.random_scores(1, pool, 5).ravel()
    seg = []
    for h in held:
        cuts = np.sort(r.integers(0, h + 1, Hkv - 1))
        seg.append(np.concatenate([[0], cuts, [h]]).astype(np.int64))
    out_rows = int(out_start[-1])
    t = dict(k=lava.to_device(k_src, "bf16", dev), v=lava.to_device(v_src, "bf16", dev),
             pos=torch.from_numpy(pos_src).to(dev), sc=torch.from_numpy(sc_src).to(dev),
             src_start=torch.from_numpy(src_start).to(dev), out_start=torch.from_numpy(out_start).to(dev),
             seg=[torch.from_numpy(x).to(dev) for x in seg],
             counts=torch.zeros(3, Hkv, dtype=torch.int32, device=dev),
             offs=torch.zeros(3, Hkv + 1, dtype=torch.int64, device=dev),
             idx=torch.full((out_rows + 3,), -7, dtype=torch.int32, device=dev),
             ks=torch.full((out_rows + 3,), -7.0, dtype=torch.float32, device=dev),
             ko=torch.full((out_rows + 3, d), 5.0, dtype=torch.bfloat16, device=dev),
             vo=torch.full((out_rows + 3, d), 5.0, dtype=torch.bfloat16, device=dev),
             po=torch.full((out_rows + 3,), -3, dtype=torch.int32, device=dev))
    sel, cmp = [], []
    for i in range(3):
        sel.append(lava.select_problem(t["sc"], budgets[i], t["counts"][i], t["offs"][i], t["idx"], t["ks"],
                                       seg_offsets=t["seg"][i], total_entries=held[i],
                                       in_offset_dev=t["src_start"][i: i + 1], out_offset_dev=t["out_start"][i: i + 1]))
        cmp.append(lava.compact_problem(desc, pool, t["k"], t["v"], t["offs"][i], t["idx"], out_rows, t["ko"], t["vo"],
                                        src_offsets=t["seg"][i], pos_src=t["pos"], pos_out=t["po"],
                                        src_offset_dev=t["src_start"][i: i + 1], out_offset_dev=t["out_start"][i: i + 1]))
    lava.lava_select_topk_batch(Hkv, sel, max(held))
    lava.lava_compact_batch(desc, cmp)
    torch.cuda.synchronize()
    idx, ks = t["idx"].cpu().numpy(), t["ks"].cpu().numpy()
    for i in range(3):
        a, b = int(src_start[i]), int(src_start[i + 1])
        rc, ro, ri, rs = O.select_topk(sc_src[a:b].astype(np.float64), seg[i], budgets[i])
        o0 = int(out_start[i])
        assert np.array_equal(t["counts"][i].cpu().numpy(), rc) and np.array_equal(t["offs"][i].cpu().numpy(), ro), i
        assert np.array_equal(idx[o0: o0 + budgets[i]], ri), i
        assert np.array_equal(ks[o0: o0 + budgets[i]].view(np.uint32), np.asarray(rs, np.float32).view(np.uint32)), i
        rows = np.concatenate([a + seg[i][g] + ri[ro[g]: ro[g + 1]] for g in range(Hkv)]).astype(np.int64)
        assert np.array_equal(lava.to_host_bits(t["ko"][o0: o0 + budgets[i]]), k_src[rows]), i
        assert np.array_equal(lava.to_host_bits(t["vo"][o0: o0 + budgets[i]]), v_src[rows]), i
        assert np.array_equal(t["po"][o0: o0 + budgets[i]].cpu().numpy(), pos_src[rows]), i
    assert np.all(idx[out_rows:] == -7) and torch.all(t["ko"][out_rows:] == 5.0) and torch.all(t["po"][out_rows:] == -3)


def test_compact_table_larger_than_one_launch_table(lava):
    say("compact batch: 35 small problems (the per-launch table holds 32)")
    dev = "cuda"
    Hkv, d = 2, 64
    desc = lava.LayerDesc.make(4, Hkv, d, 4, "f32")
    r = np.random.Generator(np.random.PCG64(55))
    probs, hold, want = [], [], []
    for i in range(35):
        n = int(r.integers(1, 90))
        k_src = r.standard_normal((Hkv, n, d)).astype(np.float32)
        v_src = r.standard_normal((Hkv, n, d)).astype(np.float32)
        kept = [np.sort(r.choice(n, size=int(r.integers(0, n + 1)), replace=False)) for _ in range(Hkv)]
        offs = np.concatenate([[0], np.cumsum([len(x) for x in kept])]).astype(np.int64)
        idx = np.concatenate(kept).astype(np.int32) if offs[-1] else np.zeros(1, dtype=np.int32)
        cap = int(offs[-1])
        t = dict(k=torch.from_numpy(k_src).to(dev), v=torch.from_numpy(v_src).to(dev),
                 offs=torch.from_numpy(offs).to(dev), idx=torch.from_numpy(idx).to(dev),
                 ko=torch.full((cap + 1, d), 9.0, dtype=torch.float32, device=dev),
                 vo=torch.full((cap + 1, d), 9.0, dtype=torch.float32, device=dev))
        hold.append(t)
        probs.append(lava.compact_problem(desc, n, t["k"].view(-1, d), t["v"].view(-1, d), t["offs"], t["idx"], cap,
                                          t["ko"], t["vo"]))
        want.append((cap, O.compact(k_src, offs, idx), O.compact(v_src, offs, idx)))
    lava.lava_compact_batch(desc, probs)
    torch.cuda.synchronize()
    for i, (t, (cap, wk, wv)) in enumerate(zip(hold, want)):
        assert np.array_equal(t["ko"][:cap].cpu().numpy(), wk) and np.array_equal(t["vo"][:cap].cpu().numpy(), wv), i
        assert torch.all(t["ko"][cap:] == 9.0), i
