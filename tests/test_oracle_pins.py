"""Pins for the CPU oracle: each check compares it with something other than itself —
pure-Python brute force on tiny inputs, closed forms, library routines in special cases, the
lemma / theorem / identity the paper proves, and invariants of the optimisation problem.
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.ndimage
import scipy.special
import scipy.stats

from oracle import lava_oracle as O
from paper_2509_09754_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ----------------------------------------------------------------- brute force helpers
def brute_attention(q, k, scale):
    """Pure-Python softmax rows, written with explicit loops and math.exp."""
    H, w, d = len(q), len(q[0]), len(q[0][0])
    Hkv, N = len(k), len(k[0])
    G = H // Hkv
    A = [[[0.0] * N for _ in range(w)] for _ in range(H)]
    for h in range(H):
        g = h // G
        for r in range(w):
            last = N - w + r
            logit = []
            for i in range(last + 1):
                acc = 0.0
                for c in range(d):
                    acc += q[h][r][c] * k[g][i][c]
                logit.append(acc * scale)
            m = max(logit)
            ex = [math.exp(x - m) for x in logit]
            z = sum(ex)
            for i in range(last + 1):
                A[h][r][i] = ex[i] / z
    return A


def brute_scores(q, k, v, w, pool):
    """LAVa score by the book with loops: Eq. 3, GQA max (Sec. 4.3), max-pool 7 (Sec. 5.1)."""
    H, Hkv, N, d = len(q), len(k), len(k[0]), len(k[0][0])
    G, Np = H // Hkv, N - w
    A = brute_attention(q, k, 1.0 / math.sqrt(d))
    vbar = [max(sum(abs(x) for x in v[g][i]) for i in range(N)) for g in range(Hkv)]
    sg = [[0.0] * Np for _ in range(Hkv)]
    for g in range(Hkv):
        for i in range(Np):
            best = -1.0
            for h in range(g * G, (g + 1) * G):
                s = vbar[g] / w * sum(A[h][r][i] for r in range(w))
                best = max(best, s)
            sg[g][i] = best
    half = pool // 2
    out = [[max(sg[g][max(0, i - half): min(Np, i + half + 1)]) for i in range(Np)] for g in range(Hkv)]
    return out, vbar


# ----------------------------------------------------------------- attention rows (Sec. 2)
@pytest.mark.parametrize("H,Hkv,w,d,N", [(2, 2, 1, 3, 5), (4, 2, 3, 4, 9), (6, 2, 2, 5, 7)])
def test_attention_rows_brute_force(H, Hkv, w, d, N):
    r = rng(H * 100 + N)
    q, k = r.standard_normal((H, w, d)), r.standard_normal((Hkv, N, d))
    A = O.window_attention(q, k)
    B = np.array(brute_attention(q.tolist(), k.tolist(), 1.0 / math.sqrt(d)))
    np.testing.assert_allclose(A, B, rtol=1e-13, atol=1e-15)
    # each row is a distribution over the keys it may see, zero beyond (causal in the window)
    np.testing.assert_allclose(A.sum(axis=2), 1.0, rtol=1e-13)
    for rr in range(w):
        assert np.all(A[:, rr, N - w + rr + 1:] == 0.0)
        assert np.all(A[:, rr, : N - w + rr + 1] > 0.0)


def test_attention_single_query_is_textbook_softmax():
    r = rng(3)
    q, k = r.standard_normal((3, 1, 8)), r.standard_normal((3, 11, 8))
    A = O.window_attention(q, k)
    for h in range(3):
        ref = scipy.special.softmax(k[h] @ q[h, 0] / math.sqrt(8))
        np.testing.assert_allclose(A[h, 0], ref, rtol=1e-13)


def test_attention_gqa_head_to_group_map():
    # consecutive query heads share a KV head: changing one key of group 1 moves heads 2,3 only
    r = rng(4)
    q, k = r.standard_normal((4, 2, 4)), r.standard_normal((2, 6, 4))
    A0 = O.window_attention(q, k)
    k2 = k.copy()
    k2[1, 2] += 1.0
    A1 = O.window_attention(q, k2)
    assert np.array_equal(A0[:2], A1[:2]) and not np.allclose(A0[2:], A1[2:])


def test_window_lse_matches_rows():
    r = rng(5)
    q, k = r.standard_normal((4, 3, 8)), r.standard_normal((2, 10, 8))
    lse = O.window_lse(q, k)
    A = O.window_attention(q, k)
    for h in range(4):
        for rr in range(3):
            i = 2
            logit = q[h, rr] @ k[h // 2, i] / math.sqrt(8)
            assert math.isclose(math.exp(logit - lse[h, rr]), A[h, rr, i], rel_tol=1e-12)


# ----------------------------------------------------------------- Lemma 1 and the proof's identity
def _masked_softmax_row(q, K, keep):
    logit = K @ q / math.sqrt(len(q))
    logit = np.where(keep, logit, -np.inf)         # -inf on evicted keys before the softmax
    return scipy.special.softmax(logit)


def test_lemma1_masking_equals_renormalisation_and_l1_identity():
    r = rng(6)
    d, N = 6, 9
    q, K = r.standard_normal((1, 1, d)), r.standard_normal((1, N, d))
    A = O.window_attention(q, K)[0, 0]
    for trial in range(20):
        keep = r.random(N) < 0.6
        keep[-1] = True
        Ahat = _masked_softmax_row(q[0, 0], K[0], keep)
        renorm = A * keep / np.sum(A * keep)
        np.testing.assert_allclose(Ahat, renorm, rtol=1e-12, atol=1e-16)        # Lemma 1
        lhs = np.abs(A - renorm).sum()                                         # ||A - A^||_1
        assert math.isclose(lhs, 2.0 * A[~keep].sum(), rel_tol=1e-11, abs_tol=1e-15)


# ----------------------------------------------------------------- Theorem 1 (w = 1, MHA, no pooling)
def _layer_output(A, V, WO):
    return np.concatenate([A[h] @ V[h] for h in range(A.shape[0])]) @ WO


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_theorem1_bound_and_greedy_optimality(seed):
    r = rng(100 + seed)
    H, d, N, B = 2, 3, 6, 5                       # N' = 5 prefix entries per head, budget 5 of 12
    q, K, V = r.standard_normal((H, 1, d)), r.standard_normal((H, N, d)), r.standard_normal((H, N, d))
    V[0] *= 3.0                                    # make the head-dependent factor matter
    WO = r.standard_normal((H * d, 4))
    A = O.window_attention(q, K)[:, 0, :]          # [H, N]
    vbar = np.array([np.abs(V[h]).sum(axis=1).max() for h in range(H)])
    C = np.abs(WO).sum(axis=1).max()               # ||W_O^T||_1: largest row abs-sum of W_O
    y = _layer_output(A, V, WO)

    best, best_masks = None, []
    prefix = [(h, i) for h in range(H) for i in range(N - 1)]
    for kept in itertools.combinations(prefix, B - H):          # window entry of each head is kept
        I = np.zeros((H, N))
        I[:, N - 1] = 1.0
        for h, i in kept:
            I[h, i] = 1.0
        Ahat = A * I / (A * I).sum(axis=1, keepdims=True)
        loss = np.abs(y - _layer_output(Ahat, V, WO)).sum()
        bound = 2.0 * C * sum(vbar[h] * (A[h] * (1 - I[h])).sum() for h in range(H))
        assert loss <= bound * (1 + 1e-12)                      # Theorem 1 for every mask
        if best is None or bound < best - 1e-15:
            best, best_masks = bound, [I]
        elif abs(bound - best) <= 1e-15:
            best_masks.append(I)

    out = O.layer_evict(q, K, V, window=1, budget=B, pool_kernel=1)
    I = np.zeros((H, N))
    for h in range(H):
        for t in range(out["head_offsets"][h], out["head_offsets"][h + 1]):
            I[h, out["kept_idx"][t]] = 1.0
    assert I.sum() == B and np.all(I[:, N - 1] == 1.0)
    assert any(np.array_equal(I, m) for m in best_masks)        # the oracle's mask minimises the bound
    # dropping the value factor picks a different (worse-bound) mask on this input at least once
    np.testing.assert_allclose(out["vbar"], vbar, rtol=1e-14)


def test_value_factor_changes_cross_head_ranking():
    # Two heads with identical attention; head 0 has 10x larger values -> all prefix budget goes there.
    r = rng(7)
    d, N = 4, 8
    q = np.repeat(r.standard_normal((1, 1, d)), 2, axis=0)
    K = np.repeat(r.standard_normal((1, N, d)), 2, axis=0)
    V = r.standard_normal((2, N, d))
    V[0] = V[1] * 10.0
    out = O.layer_evict(q, K, V, window=1, budget=2 + 4, pool_kernel=1)
    assert list(out["head_counts"]) == [5, 1]


# ----------------------------------------------------------------- value norm (App. C)
def test_value_norm_is_matrix_one_norm_of_transpose():
    V = rng(8).standard_normal((3, 17, 5))
    got = O.value_norm_max(V)
    for g in range(3):
        assert math.isclose(got[g], np.linalg.norm(V[g].T, 1), rel_tol=1e-14)
    # the maximum runs over all N rows, window rows included
    V[1, -1] = 100.0
    assert math.isclose(O.value_norm_max(V)[1], 500.0)


# ----------------------------------------------------------------- full score vs brute force
@pytest.mark.parametrize("H,Hkv,w,d,N,pool", [(4, 2, 3, 4, 14, 7), (2, 2, 2, 3, 6, 7), (6, 3, 2, 4, 12, 3), (4, 1, 4, 2, 20, 1)])
def test_scores_brute_force(H, Hkv, w, d, N, pool):
    r = rng(H + 7 * N)
    q, k, v = r.standard_normal((H, w, d)), r.standard_normal((Hkv, N, d)), r.standard_normal((Hkv, N, d))
    s, vbar = O.lava_scores(q, k, v, w, pool)
    bs, bv = brute_scores(q.tolist(), k.tolist(), v.tolist(), w, pool)
    np.testing.assert_allclose(s, np.array(bs), rtol=1e-12)
    np.testing.assert_allclose(vbar, np.array(bv), rtol=1e-14)


def test_special_case_reduces_to_window_mean_attention():
    # unit value factor, no pooling, MHA: the score is the plain recent-attention mean (Table 1)
    r = rng(9)
    q, k, v = r.standard_normal((2, 4, 8)), r.standard_normal((2, 30, 8)), r.standard_normal((2, 30, 8))
    s, _ = O.lava_scores(q, k, v, 4, 1, use_value_norm=False)
    ref = np.zeros((2, 26))
    for h in range(2):
        for rr in range(4):
            last = 30 - 4 + rr
            ref[h] += scipy.special.softmax(k[h, : last + 1] @ q[h, rr] / math.sqrt(8))[:26]
    np.testing.assert_allclose(s, ref / 4, rtol=1e-12)


# ----------------------------------------------------------------- the per-token value-norm score (VATP ablation)
@pytest.mark.parametrize("H,Hkv,w,d,N,pool", [(4, 2, 3, 4, 14, 7), (2, 2, 2, 3, 9, 3), (6, 3, 2, 4, 12, 1)])
def test_token_norm_scores_brute_force(H, Hkv, w, d, N, pool):
    r = rng(31 * H + N)
    q, k, v = r.standard_normal((H, w, d)), r.standard_normal((Hkv, N, d)), r.standard_normal((Hkv, N, d))
    s, vbar = O.token_norm_scores(q, k, v, w, pool)
    A = brute_attention(q.tolist(), k.tolist(), 1.0 / math.sqrt(d))
    G, Np, half = H // Hkv, N - w, pool // 2
    for g in range(Hkv):
        att = [max(sum(A[h][rr][i] for rr in range(w)) / w for h in range(g * G, (g + 1) * G)) for i in range(Np)]
        for i in range(Np):
            pooled = max(att[max(0, i - half): min(Np, i + half + 1)])
            norm = sum(abs(x) for x in v[g, i].tolist())
            assert math.isclose(s[g, i], norm * pooled, rel_tol=1e-12)
        assert math.isclose(vbar[g], max(sum(abs(x) for x in row) for row in v[g].tolist()), rel_tol=1e-14)


def test_token_norm_scores_reduce_to_lava_scores_for_equal_norms():
    # rows of equal L1 norm inside a head (signed permutations of one vector): the token's own norm
    # and the head's maximum coincide, so the two scores are the same array
    r = rng(77)
    H, Hkv, w, d, N = 4, 2, 3, 6, 40
    q, k = r.standard_normal((H, w, d)), r.standard_normal((Hkv, N, d))
    v = np.empty((Hkv, N, d))
    for g in range(Hkv):
        proto = r.standard_normal(d)
        for i in range(N):
            v[g, i] = r.permutation(proto) * r.choice([-1.0, 1.0], d)
    a, va = O.token_norm_scores(q, k, v, w, 7)
    b, vb = O.lava_scores(q, k, v, w, 7)
    np.testing.assert_allclose(a, b, rtol=1e-13)
    np.testing.assert_allclose(va, vb, rtol=1e-14)
    # scaling one value row scales that entry's score alone, by the same factor
    v2 = v.copy()
    v2[1, 5] *= -3.0
    c, _ = O.token_norm_scores(q, k, v2, w, 7)
    assert math.isclose(c[1, 5], 3.0 * a[1, 5], rel_tol=1e-13)
    c[1, 5] = a[1, 5]
    assert np.array_equal(c, a)


# ----------------------------------------------------------------- pooling
@pytest.mark.parametrize("n,kernel", [(1, 7), (3, 7), (6, 7), (7, 7), (50, 7), (50, 3), (50, 1), (9, 9)])
def test_maxpool_vs_library_and_loop(n, kernel):
    s = rng(n * 10 + kernel).random((3, n))
    got = O.maxpool(s, kernel)
    ref = scipy.ndimage.maximum_filter1d(s, size=kernel, axis=1, mode="constant", cval=-np.inf)
    assert np.array_equal(got, ref)
    half = kernel // 2
    for g in range(3):
        for i in range(n):
            assert got[g, i] == max(s[g, max(0, i - half): i + half + 1])


def test_pool_commutes_with_group_max_and_scaling():
    r = rng(10)
    sh = r.random((6, 40))
    a = O.maxpool(O.group_max(sh, 3), 7)
    b = O.group_max(O.maxpool(sh, 7), 3)
    assert np.array_equal(a, b)
    assert np.array_equal(O.maxpool(3.7 * sh, 7), 3.7 * O.maxpool(sh, 7))


# ----------------------------------------------------------------- entropy statistic (Eq. 4-5)
def test_entropy_vs_scipy_and_closed_forms():
    s = rng(11).random((4, 33)) + 0.01
    e = O.layer_entropy(s)
    assert math.isclose(e, scipy.stats.entropy(s.ravel()) / s.size, rel_tol=1e-12)
    # closed form ln S - T/S
    S, T = s.sum(), (s * np.log(s)).sum()
    assert math.isclose(e * s.size, math.log(S) - T / S, rel_tol=1e-12)
    # uniform scores: maximal entropy ln(M)
    u = np.full((2, 50), 0.37)
    assert math.isclose(O.layer_entropy(u), math.log(100) / 100, rel_tol=1e-12)
    # a single non-zero score: zero entropy; zeros contribute 0 ln 0 = 0
    z = np.zeros((2, 10))
    z[1, 3] = 5.0
    assert O.layer_entropy(z) == 0.0
    # scale invariance (the value factor of a single-head layer cancels)
    assert math.isclose(O.layer_entropy(7.0 * s), e, rel_tol=1e-12)
    assert O.layer_entropy(np.zeros((2, 4))) == 0.0


# ----------------------------------------------------------------- layer budgets (Alg. 2)
def test_budgets_proportional_and_invariants():
    e = [0.1, 0.2, 0.3, 0.4]
    b = O.layer_budgets(e, 1000, [0] * 4, [1000] * 4)
    assert b == [100, 200, 300, 400]
    # equal statistics -> uniform split, leftovers to lower layers
    assert O.layer_budgets([0.5] * 3, 10, [0] * 3, [10] * 3) == [4, 3, 3]
    # invariant to a common scale (log base, normaliser of Eq. 5)
    e2 = rng(12).random(32)
    b1 = O.layer_budgets(e2, 131072, [256] * 32, [262144] * 32)
    b2 = O.layer_budgets(e2 * 8.0, 131072, [256] * 32, [262144] * 32)
    assert b1 == b2 and sum(b1) == 131072
    # exact proportionality up to rounding
    q = e2 / e2.sum() * 131072
    b3 = O.layer_budgets(e2, 131072, [0] * 32, [262144] * 32)
    assert max(abs(bi - qi) for bi, qi in zip(b3, q)) < 1.0 + 1e-9
    assert all(b >= 256 for b in b1)


def test_budgets_clamping():
    # first cascade step: one layer would take everything, but cannot exceed H_kv * N
    assert O.layer_budgets([0.3], 100, [8], [100]) == [100]
    b = O.layer_budgets([0.9, 0.05, 0.05], 100, [10, 10, 10], [60, 100, 100])
    assert sum(b) == 100 and b[0] == 60 and min(b) >= 10
    b = O.layer_budgets([0.98, 0.01, 0.01], 100, [10, 10, 10], [100, 100, 100])
    assert b == [80, 10, 10]
    with pytest.raises(ValueError):
        O.layer_budgets([1, 1], 5, [3, 3], [9, 9])
    # all-zero statistics fall back to a uniform split
    assert O.layer_budgets([0.0, 0.0], 9, [0, 0], [9, 9]) == [5, 4]


def test_budgets_random_invariants():
    r = rng(13)
    for trial in range(300):
        L = int(r.integers(1, 12))
        e = r.random(L) * (r.random(L) < 0.8)
        lo = r.integers(0, 20, L)
        hi = lo + r.integers(0, 200, L)
        total = int(r.integers(lo.sum(), hi.sum() + 1))
        b = O.layer_budgets(e, total, lo, hi)
        assert sum(b) == total
        assert all(l <= x <= h for l, x, h in zip(lo, b, hi))


# ----------------------------------------------------------------- selection (Alg. 1)
def _offsets(Hkv, n):
    return [g * n for g in range(Hkv + 1)]


@pytest.mark.parametrize("seed", range(4))
def test_select_vs_lexsort_and_invariants(seed):
    Hkv, n, w = 3, 200, 4
    s = synth.random_scores(Hkv, n - w, seed).astype(np.float64)
    full = O.flat_layer_scores(s, n).ravel()
    for B in [Hkv * w, Hkv * w + 1, 57, 300, Hkv * n]:
        counts, offs, idx, kept_s = O.select_topk(full, _offsets(Hkv, n), B)
        flat_idx = np.arange(full.size)
        ref = np.sort(np.lexsort((flat_idx, -full))[:B])
        got = np.concatenate([g * n + idx[offs[g]:offs[g + 1]] for g in range(Hkv)])
        assert np.array_equal(got, ref)
        assert counts.sum() == B and np.all(counts >= w)            # Eq. 1 constraints
        assert np.array_equal(np.diff(offs), counts)
        for g in range(Hkv):                                        # window always retained, ascending
            seg = idx[offs[g]:offs[g + 1]]
            assert np.all(np.diff(seg) > 0)
            assert set(range(n - w, n)) <= set(seg.tolist())
        keep = np.zeros(full.size, bool)
        keep[got] = True
        if B < full.size:
            thr = full[keep].min()
            assert thr >= full[~keep].max()
            # among entries tied with the threshold, the kept ones have the smallest flat indices
            tied = np.flatnonzero(full == thr)
            k_tied = tied[keep[tied]]
            assert np.array_equal(k_tied, tied[: k_tied.size])
        assert np.array_equal(kept_s, full[got])


def test_select_tiny_exhaustive():
    # every score vector over {0, 1, 2} of length 5, two heads: compare with a selection loop
    for vals in itertools.product([0.0, 1.0, 2.0], repeat=5):
        sc = np.array(vals)
        for B in range(6):
            _, offs, idx, _ = O.select_topk(sc, [0, 2, 5], B)
            remaining = list(range(5))
            chosen = []
            for _ in range(B):
                best = max(remaining, key=lambda p: (sc[p], -p))
                chosen.append(best)
                remaining.remove(best)
            got = [p for p in idx[: offs[1]]] + [2 + p for p in idx[offs[1]:]]
            assert sorted(chosen) == [int(x) for x in got]


def test_compact_is_take():
    r = rng(14)
    x = r.integers(0, 2 ** 16, size=(3, 20, 8)).astype(np.uint16)
    counts, offs, idx, _ = O.select_topk(r.random(60), _offsets(3, 20), 17)
    out = O.compact(x, offs, idx)
    ref = np.concatenate([np.take(x[g], idx[offs[g]:offs[g + 1]], axis=0) for g in range(3)])
    assert out.dtype == x.dtype and np.array_equal(out, ref)


# ----------------------------------------------------------------- whole layer + cascade
def test_layer_evict_on_config1_invariants():
    shape = synth.config(1)
    inp = synth.gen_layer(shape, 0)
    q, k, v = inp.f64()
    out = O.layer_evict(q, k, v, shape.window, shape.budget, k_store=inp.k, v_store=inp.v)
    assert out["head_counts"].sum() == shape.budget and np.all(out["head_counts"] >= shape.window)
    assert out["k_hat"].shape == (shape.budget, shape.head_dim) and out["k_hat"].dtype == inp.k.dtype
    # the sink (token 0) and its pooled neighbours survive in both heads
    for g in range(shape.n_kv_heads):
        seg = out["kept_idx"][out["head_offsets"][g]:out["head_offsets"][g + 1]]
        assert 0 in seg
    # dynamic head budgets: planted heavy keys are spread unevenly, so are the survivors
    assert out["entropy"] > 0


def test_cascade_equals_single_shot():
    r = rng(15)
    Hkv, n, w, L, total = 2, 60, 3, 5, 5 * 2 * 12
    layers = []
    for l in range(L):
        s = synth.random_scores(Hkv, n - w, 50 + l, plateau=3).astype(np.float64) * (1 + l)
        layers.append(O.flat_layer_scores(s, n))
    state, history = O.cascade(layers, n, total, w)
    ent = [O.layer_entropy(x[:, : n - w]) for x in layers]
    final = O.layer_budgets(ent, total, [Hkv * w] * L, [Hkv * n] * L)
    assert history[-1] == final and sum(final) == total
    for l in range(L):
        smallest = min(h[l] for h in history[l:])            # nested top-k: the tightest budget wins
        _, offs, idx, kept_s = O.select_topk(layers[l].ravel(), _offsets(Hkv, n), smallest)
        assert np.array_equal(state[l][0], offs) and np.array_equal(state[l][1], idx)
        assert np.array_equal(state[l][2], kept_s)
        # budgets shrink as more layers share the memory (Sec. 4.2), up to integer rounding
        seq = [h[l] for h in history[l:]]
        assert all(b2 <= b1 + 1 for b1, b2 in zip(seq, seq[1:]))


def test_cascade_with_given_statistics():
    """cascade(entropies=...) allocates from the statistics it is handed and is otherwise the same
    algorithm: handed its own statistics it reproduces the plain run; handed constant weights it
    reproduces the uniform split (every step: total / layers so far, up to rounding), and the final
    state is again a single top-k per layer with the tightest budget of the layer's history; the
    scores' own entropies play no role then (scaling a layer's scores changes nothing)."""
    Hkv, n, w, L, total = 3, 50, 4, 4, 4 * 3 * 10
    layers = []
    for l in range(L):
        s = synth.random_scores(Hkv, n - w, 70 + l, plateau=2).astype(np.float64)
        layers.append(O.flat_layer_scores(s, n))
    own = [O.layer_entropy(x[:, : n - w]) for x in layers]
    plain_state, plain_hist = O.cascade(layers, n, total, w)
    given_state, given_hist = O.cascade(layers, n, total, w, entropies=own)
    assert plain_hist == given_hist
    for a, b in zip(plain_state, given_state):
        assert all(np.array_equal(x, y) for x, y in zip(a, b))
    const_state, const_hist = O.cascade(layers, n, total, w, entropies=[0.25] * L)
    for l, h in enumerate(const_hist):
        assert sum(h) == total and max(h) - min(h) <= 1 and len(h) == l + 1
        assert h == sorted(h, reverse=True)                   # leftover units go to the lower layers first
    scaled = [x * (3.0 ** l) for l, x in enumerate(layers)]
    scaled_state, scaled_hist = O.cascade(scaled, n, total, w, entropies=[0.25] * L)
    assert scaled_hist == const_hist
    for l in range(L):
        tightest = min(h[l] for h in const_hist[l:])
        _, offs, idx, kept = O.select_topk(layers[l].ravel(), _offsets(Hkv, n), tightest)
        assert np.array_equal(const_state[l][0], offs) and np.array_equal(const_state[l][1], idx)
        assert np.array_equal(const_state[l][2], kept)
        assert np.array_equal(scaled_state[l][1], idx)        # same positions: a positive factor keeps the order
    # a skewed hand-made statistic: budgets follow it in proportion (exact here: 120 * 1/8, 1/8, 2/8, 4/8)
    skew_state, skew_hist = O.cascade(layers, n, total, w, entropies=[1.0, 1.0, 2.0, 4.0])
    assert skew_hist[-1] == [15, 15, 30, 60]
    assert [int(st[0][-1]) for st in skew_state] == [15, 15, 30, 60]


# ----------------------------------------------------------------- numbers the paper prints (App. D)
def test_paper_cost_model_numbers():
    vals = {}
    with open(os.path.join(GOLDEN, "paper_cost_model.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                key, val = line.split("=")
                vals[key.strip()] = float(val)
    ec = O.extra_compute_ratio(10000, 128, 32)
    em = O.extra_memory_ratio(32, 32, 1024, 128, 10000)
    # the paper rounds to one significant digit ("approximately 0.01%", "0.6%")
    assert round(ec * 100, 2) == vals["extra_compute_percent"]
    assert round(em * 100, 1) == vals["extra_memory_percent"]


# ----------------------------------------------------------------- generator sanity (not the oracle)
def test_generator_structure_and_determinism():
    shape = synth.config(1)
    a, b = synth.gen_layer(shape, 3), synth.gen_layer(shape, 3)
    assert np.array_equal(a.k, b.k) and np.array_equal(a.v, b.v) and np.array_equal(a.q_win, b.q_win)
    assert not np.array_equal(a.k, synth.gen_layer(shape, 4).k)
    x = rng(16).standard_normal(1000).astype(np.float32)
    bits = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(bits)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(synth.f32_to_bf16_bits(back), bits)
    import torch
    assert np.array_equal(torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16), bits)
    big = synth.gen_layer(synth.config(2, n=2048, budget=8 * 64), 0)
    assert big.k.dtype == np.uint16 and big.k.shape == (8, 2048, 128)


# ----------------------------------------------------------------- decode attention (Sec. 2 / Sec. 3)
def _full_and_kept(seed, Hkv=2, G=3, N=40, d=8, keep=0.4):
    r = rng(seed)
    q = r.standard_normal((Hkv * G, d))
    k = r.standard_normal((Hkv, N, d))
    v = r.standard_normal((Hkv, N, d)) * np.exp(0.5 * r.standard_normal((Hkv, N, 1)))
    mask = r.random((Hkv, N)) < keep
    mask[:, -3:] = True
    offs = np.concatenate([[0], np.cumsum(mask.sum(1))])
    k_hat = np.concatenate([k[g][mask[g]] for g in range(Hkv)])
    v_hat = np.concatenate([v[g][mask[g]] for g in range(Hkv)])
    return q, k, v, mask, offs, k_hat, v_hat


def test_decode_is_masked_renormalised_full_attention():
    # Sec. 3: eviction = masking; the compressed cache gives A*I / ||A*I||_1 applied to V
    for seed in range(4):
        q, k, v, mask, offs, k_hat, v_hat = _full_and_kept(seed)
        out, lse = O.decode_attention(q, k_hat, v_hat, offs)
        G = q.shape[0] // k.shape[0]
        for h in range(q.shape[0]):
            g = h // G
            A = scipy.special.softmax(k[g] @ q[h] / math.sqrt(q.shape[1]))
            Am = A * mask[g]
            want = (Am / Am.sum()) @ v[g]
            np.testing.assert_allclose(out[h], want, rtol=1e-12, atol=1e-14)
            logits = (k[g] @ q[h] / math.sqrt(q.shape[1]))[mask[g]]
            assert abs(lse[h] - scipy.special.logsumexp(logits)) < 1e-12


def test_decode_brute_force_tiny():
    q, k, v, mask, offs, k_hat, v_hat = _full_and_kept(11, Hkv=2, G=2, N=9, d=3, keep=0.5)
    out, _ = O.decode_attention(q, k_hat, v_hat, offs, scale=0.7)
    for h in range(4):
        g = h // 2
        rows = range(int(offs[g]), int(offs[g + 1]))
        ws = [math.exp(0.7 * sum(q[h][c] * k_hat[i][c] for c in range(3))) for i in rows]
        for c in range(3):
            want = sum(wt * v_hat[i][c] for wt, i in zip(ws, rows)) / sum(ws)
            assert abs(out[h][c] - want) < 1e-12


def test_decode_closed_forms():
    r = rng(5)
    # identical keys -> uniform attention -> the mean of the value rows
    k_hat = np.tile(r.standard_normal((1, 6)), (10, 1))
    v_hat = r.standard_normal((10, 6))
    q = r.standard_normal((2, 6))
    out, lse = O.decode_attention(q, k_hat, v_hat, [0, 4, 10])
    np.testing.assert_allclose(out[0], v_hat[:4].mean(0), rtol=1e-12)
    np.testing.assert_allclose(out[1], v_hat[4:].mean(0), rtol=1e-12)
    assert abs(lse[0] - (k_hat[0] @ q[0] / math.sqrt(6) + math.log(4))) < 1e-12
    # one overwhelming key -> its value row; an empty head -> zeros and -inf
    k2 = np.zeros((5, 6)); k2[3] = 500 * q[0]
    out, lse = O.decode_attention(q[:1], k2, v_hat[:5], [0, 5])
    np.testing.assert_allclose(out[0], v_hat[3], atol=1e-9)
    out, lse = O.decode_attention(q, k_hat, v_hat, [0, 0, 10])
    assert np.all(out[0] == 0) and lse[0] == -np.inf and np.isfinite(lse[1])
    # the order of the retained rows inside a head does not matter
    perm = np.concatenate([r.permutation(4), 4 + r.permutation(6)])
    kk = r.standard_normal((10, 6))
    o2, _ = O.decode_attention(q, kk, v_hat, [0, 4, 10])
    o3, _ = O.decode_attention(q, kk[perm], v_hat[perm], [0, 4, 10])
    np.testing.assert_allclose(o2, o3, rtol=1e-11, atol=1e-13)


def test_decode_tail_equals_appended_rows():
    # Sec. 2: the cache grows by Cat[K, K^N]; a dense tail must act like rows appended to each head
    q, k, v, mask, offs, k_hat, v_hat = _full_and_kept(7)
    r = rng(8)
    Hkv = k.shape[0]
    kt, vt = r.standard_normal((Hkv, 5, 8)), r.standard_normal((Hkv, 5, 8))
    out, lse = O.decode_attention(q, k_hat, v_hat, offs, kt, vt)
    k_app = np.concatenate([np.concatenate([k_hat[offs[g]:offs[g + 1]], kt[g]]) for g in range(Hkv)])
    v_app = np.concatenate([np.concatenate([v_hat[offs[g]:offs[g + 1]], vt[g]]) for g in range(Hkv)])
    offs2 = [int(offs[g]) + 5 * g for g in range(Hkv + 1)]
    out2, lse2 = O.decode_attention(q, k_app, v_app, offs2)
    np.testing.assert_allclose(out, out2, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, lse2, rtol=1e-12)


def test_decode_loss_obeys_theorem_bound():
    # Thm. 1 per head: || (A - A') V ||_1 <= 2 * Vbar * (evicted attention mass)
    for seed in range(6):
        q, k, v, mask, offs, k_hat, v_hat = _full_and_kept(20 + seed, keep=0.6)
        Hkv, N, d = k.shape
        full_offs = [g * N for g in range(Hkv + 1)]
        o_full, _ = O.decode_attention(q, k.reshape(-1, d), v.reshape(-1, d), full_offs)
        o_kept, _ = O.decode_attention(q, k_hat, v_hat, offs)
        G = q.shape[0] // Hkv
        for h in range(q.shape[0]):
            g = h // G
            A = scipy.special.softmax(k[g] @ q[h] / math.sqrt(d))
            eps = A[~mask[g]].sum()
            vbar = np.abs(v[g]).sum(1).max()
            assert np.abs(o_full[h] - o_kept[h]).sum() <= 2 * vbar * eps * (1 + 1e-9) + 1e-14
