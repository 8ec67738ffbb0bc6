"""CPU oracle for the LAVa prefill-end eviction path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, single-threaded numpy in float64, written from the paper's definitions so
that it can be checked against them by eye.  Nothing here is tuned, blocked or fused, and
nothing here is shared with, imported by, or imports the HIP path.  Only tests, the smoke
check and the benchmark's cpu_baseline leg may call it.

LAVa is a heuristic (a scoring function followed by greedy selection), so the oracle is the
algorithm step by step in the paper's order.  Steps and the passage each follows:

  attention rows      A^j_{l,h} = Softmax(Q^j K^T / sqrt(d_h)), each window row normalised
                      over all keys up to and including itself             (Sec. 2)
  window mean         (1/w) sum over the w window rows                     (Def. 1, Eq. 3)
  value norm          Vbar_{l,h} = max_k ||V_{l,h}[k]||_1 over all N rows  (Thm. 1; App. C)
  head score          s_{l,h}[i] = Vbar_{l,h} * window mean                (Def. 1, Eq. 3)
  GQA group score     max over the query heads of a KV group               (Sec. 4.3)
  pooling             max-pool, kernel 7, stride 1, over the token axis    (Sec. 5.1)
  layer statistic     normalised entropy of the layer's scores             (Eq. 4, Eq. 5)
  layer budgets       B_l = e_l / sum_l e_l * total budget                 (Alg. 2)
  selection           the B_l largest entries over all heads of the layer  (Alg. 1)
  head budgets        number of survivors that fall in each head           (Sec. 4.1)
  compaction          K^, V^ = the surviving rows                          (Alg. 1)
  decode attention    one new token attends to the retained entries only:
                      A = Softmax(q K^T / sqrt(d_h)) over them, y = A V    (Sec. 2; Sec. 3 mask)

Readings taken where the paper is silent or inconsistent (each is listed with its reason in
the design notes): exactly w window rows (the paper's sum has w+1 terms but divides by w);
budgets count the window entries, which are forced to be kept (Eq. 1's constraints), realised
as score +inf; pooling sees prefix positions only and clips at both ends; the entropy is
taken over the same pooled, group-level array the selection consumes, natural log, divided
by H_kv * N'; ties are broken by lower flat index g*N + i; kept rows are stored in ascending
position inside each head.

Parity unpinned (no worked example is printed anywhere in the paper; only invariants
constrain them): which array the entropy is taken over, the integer rounding of layer
budgets (largest remainder), and whether budgets include the window entries.
"""
from __future__ import annotations

import math

import numpy as np


# ------------------------------------------------------------------ attention (Sec. 2)
def window_attention(q_win: np.ndarray, k: np.ndarray, scale: float | None = None) -> np.ndarray:
    """A[h, r, i]: how much window row r (token position N-w+r) of head h attends to key i.

    q_win [H, w, d], k [H_kv, N, d] in float64.  Query head h reads KV head h // (H/H_kv).
    Row r is a softmax over keys 0 .. N-w+r (causal inside the window); entries beyond are 0.
    """
    H, w, d = q_win.shape
    Hkv, N, _ = k.shape
    G = H // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    A = np.zeros((H, w, N), dtype=np.float64)
    for h in range(H):
        logits = (q_win[h] @ k[h // G].T) * scale          # [w, N]
        for r in range(w):
            last = N - w + r                               # position of this query token
            row = logits[r, : last + 1]
            p = np.exp(row - row.max())
            A[h, r, : last + 1] = p / p.sum()
    return A


def window_lse(q_win: np.ndarray, k: np.ndarray, scale: float | None = None) -> np.ndarray:
    """Natural-log log-sum-exp of each window row's logits, [H, w] (what a prefill attention
    kernel would hand over; used to exercise the optional LSE input of the scoring call)."""
    H, w, d = q_win.shape
    Hkv, N, _ = k.shape
    G = H // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros((H, w), dtype=np.float64)
    for h in range(H):
        logits = (q_win[h] @ k[h // G].T) * scale
        for r in range(w):
            row = logits[r, : N - w + r + 1]
            m = row.max()
            out[h, r] = m + math.log(np.exp(row - m).sum())
    return out


# ------------------------------------------------------------------ LAVa score (Eq. 3)
def window_mean(A: np.ndarray) -> np.ndarray:
    """a[h, i] = (1/w) * sum_r A[h, r, i] for prefix positions i < N - w."""
    H, w, N = A.shape
    return A[:, :, : N - w].sum(axis=1) / w


def value_norm_max(v: np.ndarray) -> np.ndarray:
    """Vbar[g] = max over all N rows of the row's L1 norm.  v [H_kv, N, d]."""
    return np.abs(v).sum(axis=2).max(axis=1)


def value_norm_rows(v: np.ndarray) -> np.ndarray:
    """L1 norm of every value row.  v [H_kv, N, d] -> [H_kv, N]."""
    return np.abs(v).sum(axis=2)


def head_scores(a: np.ndarray, vbar: np.ndarray, group: int) -> np.ndarray:
    """s_head[h, i] = Vbar[h // G] * a[h, i]."""
    H = a.shape[0]
    return np.stack([vbar[h // group] * a[h] for h in range(H)])


def group_max(s_head: np.ndarray, group: int) -> np.ndarray:
    """GQA rule: score of a cache entry = max over the query heads sharing that KV head."""
    H, Np = s_head.shape
    return s_head.reshape(H // group, group, Np).max(axis=1)


def maxpool(s: np.ndarray, kernel: int = 7) -> np.ndarray:
    """Max-pool along the last axis, stride 1, same length, window clipped at both ends."""
    if kernel == 1:
        return s.copy()
    if kernel < 1 or kernel % 2 == 0:
        raise ValueError("pool kernel must be odd")
    half = kernel // 2
    n = s.shape[-1]
    out = s.copy()
    for delta in range(1, half + 1):
        if delta >= n:
            break
        out[..., delta:] = np.maximum(out[..., delta:], s[..., : n - delta])   # neighbour i-delta
        out[..., : n - delta] = np.maximum(out[..., : n - delta], s[..., delta:])  # neighbour i+delta
    return out


def lava_scores(q_win, k, v, window: int, pool_kernel: int = 7, scale=None, use_value_norm: bool = True):
    """Pooled group-level LAVa scores s[g, i], i in the prefix, plus Vbar[g].  Inputs float64."""
    H, Hkv = q_win.shape[0], k.shape[0]
    if q_win.shape[1] != window:
        raise ValueError("q_win must hold exactly w rows")
    G = H // Hkv
    A = window_attention(q_win, k, scale)
    a = window_mean(A)
    vbar = value_norm_max(v)
    s_head = head_scores(a, vbar if use_value_norm else np.ones_like(vbar), G)
    s = maxpool(group_max(s_head, G), pool_kernel)
    return s, vbar


def token_norm_scores(q_win, k, v, window: int, pool_kernel: int = 7, scale=None):
    """The comparison score of the paper's VATP ablation (appendix paragraph "VATP", Table 4 row
    "recent attention scores + value vectors"): every token's own value norm times its attention
    score, where LAVa uses one factor per head.  The attention score is the pooled, group-level
    window mean (the rule is applied on top of the pooled SnapKV score in that ablation):
        s[g, i] = ||V[g, i]||_1 * maxpool(max_{h in g} a[h, i]).
    Returns (s, Vbar) like lava_scores."""
    H, Hkv = q_win.shape[0], k.shape[0]
    if q_win.shape[1] != window:
        raise ValueError("q_win must hold exactly w rows")
    G = H // Hkv
    a = window_mean(window_attention(q_win, k, scale))
    pooled = maxpool(group_max(a, G), pool_kernel)
    norms = value_norm_rows(v)
    return norms[:, : pooled.shape[1]] * pooled, norms.max(axis=1)


# ------------------------------------------------------------------ layer statistic (Eq. 4-5)
def layer_entropy(s: np.ndarray) -> float:
    """e_l = -sum(s^ ln s^) / (number of entries), s^ = s / sum(s); 0 ln 0 := 0.
    An all-zero score array (only possible when every value row is zero) gives 0."""
    total = float(s.sum())
    if not total > 0.0:
        return 0.0
    p = (s / total).ravel()
    p = p[p > 0.0]
    return float(-(p * np.log(p)).sum() / s.size)


# ------------------------------------------------------------------ layer budgets (Alg. 2)
def _largest_remainder(weights, total):
    """Integers proportional to weights that sum to total: floor the real quotas, then hand
    the leftover units to the largest fractional parts (ties: lower index)."""
    n = len(weights)
    wsum = 0.0
    for x in weights:                      # sequential sum, index order
        wsum += float(x)
    if not wsum > 0.0:
        weights = [1.0] * n
        wsum = float(n)
    quota = [(float(x) / wsum) * float(total) for x in weights]
    base = [int(math.floor(q)) for q in quota]
    left = int(total) - sum(base)
    order = sorted(range(n), key=lambda i: (-(quota[i] - base[i]), i))
    # float rounding can leave `left` slightly outside [0, n); cycle so the sum is exact
    j = 0
    while left > 0:
        base[order[j % n]] += 1
        left -= 1
        j += 1
    j = 0
    while left < 0:
        i = order[n - 1 - (j % n)]
        if base[i] > 0:
            base[i] -= 1
            left += 1
        j += 1
    return base


def layer_budgets(e, total: int, lo, hi):
    """B_l = e_l / sum(e) * total as integers with sum(B) == total and lo_l <= B_l <= hi_l.

    Proportional split by largest remainder over the layers not yet pinned to a bound; after
    each split the layers that violate a bound are pinned (upper violators when their excess
    is at least the lower violators' deficit, else the lower violators) and the rest is split
    again.  Requires sum(lo) <= total <= sum(hi).
    """
    L = len(e)
    lo = [int(x) for x in lo]
    hi = [int(x) for x in hi]
    if sum(lo) > total or sum(hi) < total or any(a > b for a, b in zip(lo, hi)):
        raise ValueError("infeasible budget bounds")
    out = [0] * L
    free = list(range(L))
    remaining = int(total)
    while free:
        part = _largest_remainder([e[i] for i in free], remaining)
        over = [(i, b) for i, b in zip(free, part) if b > hi[i]]
        under = [(i, b) for i, b in zip(free, part) if b < lo[i]]
        if not over and not under:
            for i, b in zip(free, part):
                out[i] = b
            break
        excess = sum(b - hi[i] for i, b in over)
        deficit = sum(lo[i] - b for i, b in under)
        if over and excess >= deficit:
            for i, _ in over:
                out[i] = hi[i]
                remaining -= hi[i]
            pinned = {i for i, _ in over}
        else:
            for i, _ in under:
                out[i] = lo[i]
                remaining -= lo[i]
            pinned = {i for i, _ in under}
        free = [i for i in free if i not in pinned]
    return out


# ------------------------------------------------------------------ selection (Alg. 1)
def flat_layer_scores(s: np.ndarray, n: int) -> np.ndarray:
    """The layer's flattened score array [H_kv, N]: prefix scores, then +inf for the w window
    entries of every head (they are always retained, Eq. 1 last constraint)."""
    Hkv, Np = s.shape
    full = np.full((Hkv, n), np.inf, dtype=s.dtype)
    full[:, :Np] = s
    return full


def select_topk(scores, offsets, budget: int):
    """Keep the `budget` entries that come first under (score descending, flat index
    ascending) over the concatenated per-head segments.

    scores: 1-D array, heads concatenated; offsets: H+1 segment starts.  Returns
    (head_counts [H], head_offsets [H+1], kept_idx [budget] = position inside its head,
    ascending per head, heads concatenated, kept_scores [budget]).
    """
    scores = np.asarray(scores).ravel()
    offsets = [int(x) for x in offsets]
    nheads = len(offsets) - 1
    total = offsets[-1]
    if not 0 <= budget <= total:
        raise ValueError("budget out of range")
    order = np.argsort(-scores[:total], kind="stable")      # ties keep ascending index
    kept_flat = np.sort(order[:budget])
    head_counts = np.zeros(nheads, dtype=np.int64)
    kept_idx = np.zeros(budget, dtype=np.int64)
    for t, p in enumerate(kept_flat):
        g = 0
        while not (offsets[g] <= p < offsets[g + 1]):
            g += 1
        head_counts[g] += 1
        kept_idx[t] = p - offsets[g]
    head_offsets = np.concatenate([[0], np.cumsum(head_counts)]).astype(np.int64)
    return head_counts, head_offsets, kept_idx, scores[kept_flat].copy()


def compact(x: np.ndarray, head_offsets, kept_idx) -> np.ndarray:
    """Packed survivors: out[head_offsets[g] + t] = x[g, kept_idx[head_offsets[g] + t]]."""
    Hkv = x.shape[0]
    rows = []
    for g in range(Hkv):
        for t in range(int(head_offsets[g]), int(head_offsets[g + 1])):
            rows.append(x[g, int(kept_idx[t])])
    if not rows:
        return np.zeros((0,) + x.shape[2:], dtype=x.dtype)
    return np.stack(rows)


# ------------------------------------------------------------------ decode step (Sec. 2, Sec. 3)
def decode_attention(q, k_hat, v_hat, head_offsets, k_tail=None, v_tail=None, scale=None):
    """Attention of ONE new token over a compressed layer cache.

    Sec. 2: A_h = Softmax(q_h K_h^T / sqrt(d_h)), output A_h V_h.  Sec. 3: eviction is a mask,
    i.e. the softmax runs over the retained entries only.  Query head h reads KV head
    g = h // (H / H_kv), whose retained rows are k_hat / v_hat[head_offsets[g] : head_offsets[g+1]]
    followed by the rows appended since the eviction, k_tail / v_tail[g] (Cat[K, K^N] of Sec. 2).

    q [H, d]; k_hat, v_hat [R, d]; head_offsets [H_kv + 1]; k_tail, v_tail [H_kv, T, d] or None.
    Returns (out [H, d], lse [H]); a head with no entries gives zeros and -inf.
    """
    H, d = q.shape
    Hkv = len(head_offsets) - 1
    G = H // Hkv
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.zeros((H, d), dtype=np.float64)
    lse = np.full(H, -np.inf, dtype=np.float64)
    for h in range(H):
        g = h // G
        lo, hi = int(head_offsets[g]), int(head_offsets[g + 1])
        keys, vals = k_hat[lo:hi], v_hat[lo:hi]
        if k_tail is not None and k_tail.shape[1] > 0:
            keys = np.concatenate([keys, k_tail[g]], axis=0)
            vals = np.concatenate([vals, v_tail[g]], axis=0)
        if keys.shape[0] == 0:
            continue
        logits = (keys @ q[h]) * scale
        m = logits.max()
        p = np.exp(logits - m)
        z = p.sum()
        out[h] = (p / z) @ vals
        lse[h] = m + math.log(z)
    return out, lse


def layer_evict(q_win, k, v, window: int, budget: int, pool_kernel: int = 7, scale=None,
                k_store=None, v_store=None):
    """Algorithm 1 for one layer.  q_win, k, v float64; k_store / v_store (optional) are the
    arrays in their storage dtype whose rows are copied bit for bit into the packed cache."""
    Hkv, N, _ = k.shape
    s, vbar = lava_scores(q_win, k, v, window, pool_kernel, scale)
    e = layer_entropy(s)
    full = flat_layer_scores(s, N)
    counts, offs, idx, kept_s = select_topk(full.ravel(), [g * N for g in range(Hkv + 1)], budget)
    ks = k if k_store is None else k_store
    vs = v if v_store is None else v_store
    return dict(scores=full, vbar=vbar, entropy=e, head_counts=counts, head_offsets=offs,
                kept_idx=idx, kept_scores=kept_s, k_hat=compact(ks, offs, idx), v_hat=compact(vs, offs, idx))


# ------------------------------------------------------------------ Algorithm 2, literally
def cascade(layer_scores, n: int, total_budget: int, window: int, entropies=None):
    """Run Algorithm 2 on precomputed per-layer flat score arrays [H_kv, N] (window = +inf):
    after layer l arrives every layer <= l is re-evicted from what it still retains, with the
    budget e_l / sum(e so far) * total.  Returns per layer (head_offsets, kept positions,
    retained scores) and the list of budget vectors used at each step.  `entropies`, if given,
    replaces the statistics computed here (so that a caller can allocate from the exact values
    another implementation saw); the algorithm is unchanged."""
    L = len(layer_scores)
    Hkv = layer_scores[0].shape[0]
    lo, hi = Hkv * window, Hkv * n
    ent, state, history = [], [], []
    for l in range(L):
        ent.append(layer_entropy(layer_scores[l][:, : n - window]) if entropies is None else float(entropies[l]))
        offs = np.array([g * n for g in range(Hkv + 1)], dtype=np.int64)
        pos = np.concatenate([np.arange(n, dtype=np.int64)] * Hkv)
        state.append((offs, pos, layer_scores[l].ravel().copy()))
        budgets = layer_budgets(ent, total_budget, [lo] * (l + 1), [hi] * (l + 1))
        history.append(budgets)
        for t in range(l + 1):
            offs, pos, sc = state[t]
            b = min(budgets[t], int(offs[-1]))
            counts, new_offs, idx, kept_s = select_topk(sc, offs, b)
            new_pos = np.zeros(b, dtype=np.int64)
            for g in range(Hkv):
                a0, a1 = int(new_offs[g]), int(new_offs[g + 1])
                new_pos[a0:a1] = pos[int(offs[g]) + idx[a0:a1]]
            state[t] = (new_offs, new_pos, kept_s)
    return state, history


# ------------------------------------------------------------------ the paper's cost model (App. D)
def extra_compute_ratio(n: int, d_h: int, h: int) -> float:
    """Extra work of LAVa over SnapKV relative to the layer's prefill attention:
    H N (d_h + log2 H) / (H N^2 d_h)."""
    return (h * n * (d_h + math.log2(h))) / (h * n * n * d_h)


def extra_memory_ratio(n_layers: int, h: int, b_lh: int, d_h: int, n: int) -> float:
    """Retained scores relative to SnapKV's peak: L H B / (H N d_h + L H B d_h)."""
    return (n_layers * h * b_lh) / (h * n * d_h + n_layers * h * b_lh * d_h)
