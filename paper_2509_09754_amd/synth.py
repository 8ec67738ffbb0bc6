"""Seeded synthetic layer inputs (Q window, K, V) shaped like the paper's workloads.

This module holds no arithmetic of the eviction method itself: it only draws random
tensors, plants structure in them (an attention sink, a few keys aligned with window
queries, log-normal value-row norms) and rounds them once to the storage dtype.  The
CPU oracle and the HIP path both consume the arrays produced here, byte for byte.

The paper evaluates on LongBench / Needle-in-a-Haystack / Ruler / InfiniteBench prompts
run through Mistral-7B, Qwen2.5 and Llama-3-8B (Sec. 5.1); neither those prompts nor the
weights are available, so these tensors stand in for the K/V cache and the last-w queries
at the end of prefill: same shapes (GQA head counts, head_dim, context lengths, budgets),
and the qualitative structure eviction methods rely on (a sink token, a small set of
strongly attended keys, local burstiness that motivates pooling).
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

F32 = "f32"
BF16 = "bf16"


# --------------------------------------------------------------------------- dtype I/O
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 -> bfloat16 (round-to-nearest-even), returned as uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    # NaN never occurs in generated data; plain RNE on the upper 16 bits.
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float array once to the storage dtype: float32 array, or uint16 bf16 bits."""
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == BF16:
        return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))
    raise ValueError(f"unknown dtype {dtype!r}")


def load_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 view of stored values (what the oracle computes on)."""
    if dtype == F32:
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == BF16:
        return bf16_bits_to_f32(a).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype!r}")


def itemsize(dtype: str) -> int:
    return 4 if dtype == F32 else 2


# --------------------------------------------------------------------------- configs
@dataclasses.dataclass(frozen=True)
class LayerShape:
    """One layer of one sequence.  Names follow the paper's notation (Sec. 2, App. A)."""
    n_q_heads: int      # H
    n_kv_heads: int     # H_kv (GQA, Sec. 4.3)
    head_dim: int       # d_h
    n: int              # N, cached tokens
    window: int         # w, observation window
    dtype: str          # storage dtype of Q, K, V
    budget: int         # B_l, entries kept in this layer (window entries included)
    heavy_frac: float = 0.01      # fraction of prefix entries planted as strongly attended
    heavy_count: Optional[int] = None   # overrides heavy_frac when set
    burst: int = 1      # heavy keys come in runs of this many consecutive tokens
    pool_kernel: int = 7

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_prefix(self) -> int:
        return self.n - self.window


def config(idx: int, **over) -> LayerShape:
    """The single-layer shapes of the benchmark configurations (1-based, as listed)."""
    if idx == 1:
        s = LayerShape(8, 2, 64, 1024, 8, F32, 256, heavy_count=16)
    elif idx == 2:
        s = LayerShape(32, 8, 128, 32768, 32, BF16, 8 * 512)
    elif idx == 3:   # one layer of the 32-layer stack; heavy_frac is redrawn per layer
        s = LayerShape(32, 8, 128, 32768, 32, BF16, 8 * 512)
    elif idx == 4:
        s = LayerShape(32, 8, 128, 131072, 32, BF16, 8 * 1024, burst=64)
    elif idx == 5:   # one sequence of the ragged batch; n is redrawn per sequence
        s = LayerShape(32, 8, 128, 65536, 32, BF16, 8 * 256)
    else:
        raise ValueError("config index must be 1..5")
    return dataclasses.replace(s, **over) if over else s


@dataclasses.dataclass
class LayerInputs:
    shape: LayerShape
    q_win: np.ndarray   # [H, w, d]      storage dtype (float32 or uint16 bf16 bits)
    k: np.ndarray       # [H_kv, N, d]
    v: np.ndarray       # [H_kv, N, d]

    def f64(self):
        """(q_win, k, v) widened exactly to float64."""
        dt = self.shape.dtype
        return load_f64(self.q_win, dt), load_f64(self.k, dt), load_f64(self.v, dt)


# --------------------------------------------------------------------------- generator
def _unit(x: np.ndarray) -> np.ndarray:
    nrm = np.sqrt(np.sum(x.astype(np.float64) ** 2, axis=-1, keepdims=True))
    return (x / np.maximum(nrm, 1e-30)).astype(np.float32)


def gen_layer(shape: LayerShape, seed: int) -> LayerInputs:
    """Draw one layer.  Recipe (all draws from numpy PCG64(seed), float32, rounded once):

    * Q_win, K ~ N(0,1);  V[g,i,:] ~ N(0,1) * exp(0.5 z_{g,i}), z ~ N(0,1)
      (log-normal row norms, sigma = 0.5);
    * sink: K[:,0,:] *= 4;
    * heavy keys: `heavy_count` (or heavy_frac * H_kv * N') entries drawn uniformly over the
      flattened prefix (g, i), i in [1, N'), so heads receive different numbers of them;
      with burst > 1 the draw picks burst starts and marks `burst` consecutive tokens.
      Each heavy key is replaced by |K[g,i]| * (0.8 q^ + 0.6 u^) with q^ the direction of a
      window query of a random head of the group and u^ a unit vector orthogonal to q^,
      i.e. cosine 0.8 to that query before rounding.
    """
    H, Hkv, d, N, w = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.n, shape.window
    if H % Hkv or w < 1 or N <= w:
        raise ValueError("bad layer shape")
    G, Np = H // Hkv, N - w
    rng = np.random.Generator(np.random.PCG64(seed))
    q = rng.standard_normal((H, w, d), dtype=np.float32)
    k = rng.standard_normal((Hkv, N, d), dtype=np.float32)
    v = rng.standard_normal((Hkv, N, d), dtype=np.float32)
    z = rng.standard_normal((Hkv, N, 1), dtype=np.float32)
    v *= np.exp(np.float32(0.5) * z)
    del z
    k[:, 0, :] *= np.float32(4.0)

    n_heavy = shape.heavy_count if shape.heavy_count is not None else int(round(shape.heavy_frac * Hkv * Np))
    burst = max(1, shape.burst)
    if n_heavy > 0 and Np > 1:
        n_starts = max(1, n_heavy // burst)
        flat = rng.integers(0, Hkv * (Np - 1), size=n_starts)
        g0, i0 = flat // (Np - 1), 1 + flat % (Np - 1)
        g = np.repeat(g0, burst)
        i = np.repeat(i0, burst) + np.tile(np.arange(burst), n_starts)
        keep = i < Np
        g, i = g[keep], i[keep]
        # drop duplicates so each planted key is written once (order-independent result)
        _, first = np.unique(g * N + i, return_index=True)
        g, i = g[np.sort(first)], i[np.sort(first)]
        m = g.shape[0]
        h = g * G + rng.integers(0, G, size=m)
        r = rng.integers(0, w, size=m)
        qhat = _unit(q[h, r])                                   # [m, d]
        u = rng.standard_normal((m, d), dtype=np.float32)
        u = u - np.sum(u * qhat, axis=-1, keepdims=True) * qhat  # orthogonal to qhat
        uhat = _unit(u)
        nrm = np.sqrt(np.sum(k[g, i].astype(np.float64) ** 2, axis=-1, keepdims=True)).astype(np.float32)
        k[g, i] = nrm * (np.float32(0.8) * qhat + np.float32(0.6) * uhat)

    dt = shape.dtype
    return LayerInputs(shape, store(q, dt), store(k, dt), store(v, dt))


def stack_heavy_fracs(n_layers: int, seed: int, lo: float = 0.002, hi: float = 0.03) -> np.ndarray:
    """Per-layer heavy-key fractions U[lo, hi] for the multi-layer stack configuration."""
    rng = np.random.Generator(np.random.PCG64(seed + 7919))
    return rng.uniform(lo, hi, size=n_layers)


def ragged_lengths(batch: int, seed: int, lo: int = 4096, hi: int = 65536) -> np.ndarray:
    """Per-sequence prefix lengths U{lo..hi} for the batched serving configuration."""
    rng = np.random.Generator(np.random.PCG64(seed + 104729))
    return rng.integers(lo, hi + 1, size=batch).astype(np.int64)


def random_scores(n_heads: int, n: int, seed: int, plateau: int = 7, zero_frac: float = 0.05) -> np.ndarray:
    """A float32 score array [n_heads, n] with the structure selection must cope with:
    runs of bit-identical values (as max-pooling produces), exact zeros, a heavy tail."""
    rng = np.random.Generator(np.random.PCG64(seed + 15485863))
    base = np.exp(rng.standard_normal((n_heads, (n + plateau - 1) // plateau)) * 2.0).astype(np.float32)
    base[rng.random(base.shape) < zero_frac] = 0.0
    s = np.repeat(base, plateau, axis=1)[:, :n]
    return np.ascontiguousarray(s, dtype=np.float32)


# --------------------------------------------------------------------------- decode-step inputs
@dataclasses.dataclass
class DecodeInputs:
    dtype: str
    q: np.ndarray             # [batch, H, d]                 storage dtype
    k_hat: np.ndarray         # [batch * rows_capacity, d]    packed rows, sequence b at b * rows_capacity
    v_hat: np.ndarray
    head_offsets: np.ndarray  # [batch, H_kv + 1] int64
    rows_capacity: int
    k_tail: np.ndarray        # [batch, H_kv, tail_capacity, d]
    v_tail: np.ndarray
    tail_len: int


def head_split(rows: int, n_heads: int, rng, kind: str = "skewed") -> np.ndarray:
    """Offsets [n_heads + 1] that split `rows` packed rows among heads: 'uniform', or 'skewed'
    (the uneven head budgets a layer-wide selection produces: a few heads take most rows, some
    may get none)."""
    if kind == "uniform":
        cnt = np.full(n_heads, rows // n_heads, dtype=np.int64)
        cnt[: rows - cnt.sum()] += 1
    else:
        wgt = np.exp(1.5 * rng.standard_normal(n_heads))
        wgt[rng.random(n_heads) < 0.15] = 0.0
        if wgt.sum() == 0.0:
            wgt[0] = 1.0
        cnt = np.floor(wgt / wgt.sum() * rows).astype(np.int64)
        cnt[int(np.argmax(wgt))] += rows - cnt.sum()
    return np.concatenate([[0], np.cumsum(cnt)]).astype(np.int64)


def gen_decode(n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: str, rows, seed: int,
               rows_capacity: int | None = None, tail_len: int = 0, tail_capacity: int | None = None,
               split: str = "skewed", heavy_frac: float = 0.01) -> DecodeInputs:
    """A compressed layer cache as the eviction leaves it, plus one new query token per sequence.

    rows[b] packed rows for sequence b, split among the KV heads by `head_split`; q, K ~ N(0,1),
    V ~ N(0,1) * log-normal row scale (sigma 0.5) as in gen_layer; a fraction `heavy_frac` of the
    rows are turned towards the query of a random head of their group (cosine 0.8), which is what
    retained entries look like: they were kept because recent queries attend to them."""
    rng = np.random.Generator(np.random.PCG64(seed + 7919))
    rows = np.asarray(rows, dtype=np.int64)
    batch = rows.shape[0]
    cap = int(rows.max()) if rows_capacity is None else int(rows_capacity)
    tcap = tail_len if tail_capacity is None else int(tail_capacity)
    G, d = n_q_heads // n_kv_heads, head_dim
    q = rng.standard_normal((batch, n_q_heads, d), dtype=np.float32)
    k = rng.standard_normal((batch * cap, d), dtype=np.float32)
    v = rng.standard_normal((batch * cap, d), dtype=np.float32)
    v *= np.exp(np.float32(0.5) * rng.standard_normal((batch * cap, 1), dtype=np.float32))
    kt = rng.standard_normal((batch, n_kv_heads, max(tcap, 1), d), dtype=np.float32)
    vt = rng.standard_normal((batch, n_kv_heads, max(tcap, 1), d), dtype=np.float32)
    offs = np.zeros((batch, n_kv_heads + 1), dtype=np.int64)
    for b in range(batch):
        offs[b] = head_split(int(rows[b]), n_kv_heads, rng, split)
        n_heavy = int(round(heavy_frac * rows[b]))
        if n_heavy == 0:
            continue
        r = rng.integers(0, int(rows[b]), size=n_heavy)
        r = np.unique(r)
        g = np.searchsorted(offs[b], r, side="right") - 1
        h = g * G + rng.integers(0, G, size=r.shape[0])
        qhat = _unit(q[b, h])
        u = rng.standard_normal((r.shape[0], d), dtype=np.float32)
        u = u - np.sum(u * qhat, axis=-1, keepdims=True) * qhat
        rr = b * cap + r
        nrm = np.sqrt(np.sum(k[rr].astype(np.float64) ** 2, axis=-1, keepdims=True)).astype(np.float32)
        k[rr] = nrm * (np.float32(0.8) * qhat + np.float32(0.6) * _unit(u))
    return DecodeInputs(dtype, store(q, dtype), store(k, dtype), store(v, dtype), offs, cap,
                        store(kt, dtype), store(vt, dtype), int(tail_len))
