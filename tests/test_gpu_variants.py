"""Score and budget variants (the paper's ablations and the score rows of its Table 4) against the
oracle: the attention-only score, per-head top-k (uniform head budgets) realised with one selection
per head, and fixed layer-budget patterns through lava_layer_budgets."""
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


@pytest.mark.parametrize("cfg,over", [(1, {}), (2, dict(n=4096 + 77))])
def test_attention_only_score(lava, cfg, over):
    say(f"variant: attention-only score, config {cfg} {over}")
    sh = synth.config(cfg, **over)
    inp = synth.gen_layer(sh, 4)
    desc = lava.LayerDesc.make(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.window, sh.dtype,
                               pool_kernel=sh.pool_kernel, score_kind=lava.LAVA_SCORE_ATTENTION)
    q, k, v = (lava.to_device(a, sh.dtype) for a in (inp.q_win, inp.k, inp.v))
    scores, vbar, stat = lava.lava_window_scores(desc, [sh.n], q, k, v)
    torch.cuda.synchronize()
    qf, kf, vf = inp.f64()
    want, _ = O.lava_scores(qf, kf, vf, sh.window, sh.pool_kernel, use_value_norm=False)
    got = scores.cpu().numpy().reshape(sh.n_kv_heads, sh.n)
    assert np.all(np.isinf(got[:, sh.n_prefix:])) and np.all(vbar.cpu().numpy() == 1.0)
    got = got[:, : sh.n_prefix].astype(np.float64)
    mask = want > 1e-30 * want.max()
    assert np.max(np.abs(got[mask] - want[mask]) / want[mask]) <= 1e-3
    assert abs(float(stat[0]) - O.layer_entropy(want)) <= 1e-4 * O.layer_entropy(want) + 2e-5 / want.size
    # the value factor is the only difference from the LAVa score: same array up to the per-head scale
    full, vb = O.lava_scores(qf, kf, vf, sh.window, sh.pool_kernel)
    np.testing.assert_allclose(full, want * vb[:, None], rtol=1e-12)


TOKEN_NORM_CASES = [
    ("cfg1", synth.config(1), None),
    ("cfg2-4k", synth.config(2, n=4096 + 77), None),
    ("cfg2-9k-narrow", synth.config(2, n=9000 + 5), "narrow"),
    ("bf16-G8-two-chunks", synth.LayerShape(16, 2, 128, 2100, 32, "bf16", 300), None),
    ("f32-d128", synth.LayerShape(8, 2, 128, 1111, 32, "f32", 300), None),
    ("bf16-d64-pool3", synth.LayerShape(8, 4, 64, 3000, 16, "bf16", 400, pool_kernel=3), None),
]


@pytest.mark.parametrize("name,sh,shape", TOKEN_NORM_CASES, ids=[c[0] for c in TOKEN_NORM_CASES])
def test_token_norm_score(lava, name, sh, shape, tuning):
    say(f"variant: per-token value-norm score, {name}")
    if shape:
        tuning(sweep_shape=shape)
    inp = synth.gen_layer(sh, 6)
    desc = lava.LayerDesc.make(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.window, sh.dtype,
                               pool_kernel=sh.pool_kernel, score_kind=lava.LAVA_SCORE_TOKEN_NORM)
    q, k, v = (lava.to_device(a, sh.dtype) for a in (inp.q_win, inp.k, inp.v))
    scores, vbar, stat = lava.lava_window_scores(desc, [sh.n], q, k, v)
    torch.cuda.synchronize()
    qf, kf, vf = inp.f64()
    want, want_vbar = O.token_norm_scores(qf, kf, vf, sh.window, sh.pool_kernel)
    got = scores.cpu().numpy().reshape(sh.n_kv_heads, sh.n)
    assert np.all(np.isposinf(got[:, sh.n_prefix:]))
    np.testing.assert_allclose(vbar.cpu().numpy()[0], want_vbar, rtol=1e-5)
    got = got[:, : sh.n_prefix].astype(np.float64)
    mask = want > 1e-30 * want.max()
    assert np.max(np.abs(got[mask] - want[mask]) / want[mask]) <= 1e-3
    assert np.all(got[~mask] <= 1e-29 * want.max())
    assert abs(float(stat[0]) - O.layer_entropy(want)) <= 1e-4 * O.layer_entropy(want) + 2e-5 / want.size


def test_token_norm_score_ragged_batch(lava):
    say("variant: per-token value-norm score, ragged batch of three sequences")
    shapes = [synth.config(2, n=n, budget=8 * 64) for n in (1500, 6000 + 3, 33 + 32)]
    inps = [synth.gen_layer(s, 70 + i) for i, s in enumerate(shapes)]
    sh0 = shapes[0]
    desc = lava.LayerDesc.make(sh0.n_q_heads, sh0.n_kv_heads, sh0.head_dim, sh0.window, sh0.dtype,
                               score_kind=lava.LAVA_SCORE_TOKEN_NORM)
    q = torch.cat([lava.to_device(i.q_win, "bf16").reshape(-1) for i in inps])
    k = torch.cat([lava.to_device(i.k, "bf16").reshape(-1) for i in inps])
    v = torch.cat([lava.to_device(i.v, "bf16").reshape(-1) for i in inps])
    scores, vbar, stat = lava.lava_window_scores(desc, [s.n for s in shapes], q, k, v)
    torch.cuda.synchronize()
    s_host, tok = scores.cpu().numpy(), 0
    for b, (sh, inp) in enumerate(zip(shapes, inps)):
        qf, kf, vf = inp.f64()
        want, _ = O.token_norm_scores(qf, kf, vf, sh.window, 7)
        got = s_host[8 * tok: 8 * (tok + sh.n)].reshape(8, sh.n)[:, : sh.n_prefix].astype(np.float64)
        mask = want > 1e-30 * want.max()
        assert np.max(np.abs(got[mask] - want[mask]) / want[mask]) <= 1e-3, b
        assert abs(float(stat[b]) - O.layer_entropy(want)) <= 1e-4 * O.layer_entropy(want) + 2e-5 / want.size
        tok += sh.n


def test_per_head_topk_with_one_selection_per_head(lava):
    say("variant: uniform head budgets = one top-k per head (n_heads = 1 on each head's segment)")
    nh, n, w, per_head = 8, 4096 + 13, 32, 300
    s = synth.random_scores(nh, n - w, 6)
    full = O.flat_layer_scores(s.astype(np.float64), n).astype(np.float32)
    dev = torch.from_numpy(full).cuda()
    for g in range(nh):
        counts, offs, idx, ks = lava.lava_select_topk(1, dev[g], per_head)
        torch.cuda.synchronize()
        rc, ro, ri, rs = O.select_topk(full[g].astype(np.float64), [0, n], per_head)
        assert counts.cpu().numpy().tolist() == [per_head] and np.array_equal(idx.cpu().numpy(), ri)
        assert np.array_equal(ks.cpu().numpy().view(np.uint32), rs.astype(np.float32).view(np.uint32))
        assert np.all(ri[-w:] == np.arange(n - w, n))           # the window is always retained


def test_fixed_layer_budget_patterns(lava):
    say("variant: uniform and pyramid layer budgets are lava_layer_budgets with fixed weights")
    L, total = 32, 32 * 1024
    lo, hi = np.full(L, 8 * 32), np.full(L, 8 * 32768)
    dev = lambda a, dt: torch.from_numpy(np.asarray(a, dtype=dt)).cuda()
    uniform = lava.lava_layer_budgets(dev(np.ones((1, L)), np.float32), dev([total], np.int64), dev(lo[None], np.int64),
                                      dev(hi[None], np.int64))
    torch.cuda.synchronize()
    assert uniform.cpu().numpy().ravel().tolist() == [1024] * L
    weights = np.linspace(1.75, 0.25, L).astype(np.float32)       # more budget for lower layers
    pyramid = lava.lava_layer_budgets(dev(weights[None], np.float32), dev([total], np.int64), dev(lo[None], np.int64),
                                      dev(hi[None], np.int64))
    torch.cuda.synchronize()
    got = pyramid.cpu().numpy().ravel().tolist()
    assert got == O.layer_budgets(weights.astype(np.float64), total, lo, hi) and sum(got) == total
    assert all(a >= b for a, b in zip(got, got[1:]))
