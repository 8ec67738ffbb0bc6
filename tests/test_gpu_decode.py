"""Parity of lava_decode_attention (one new token over the compressed cache) against the oracle.

Bar: fp32 accumulation of exact products -> |out - ref| <= DEC_TOL * max|ref| per head (the
probabilities sum to one, so the output error is relative to the value scale), log-sum-exp within
1e-5 absolute + relative.
"""
import math

import numpy as np
import pytest
import torch

from oracle import lava_oracle as O
from paper_2509_09754_amd import synth

pytestmark = pytest.mark.gpu

DEC_TOL = 2e-5


@pytest.fixture(scope="module")
def lava():
    from paper_2509_09754_amd import lava as mod
    assert torch.cuda.is_available()
    return mod


def say(*a):
    print(*a, flush=True)


def run_gpu(lava, di, H, Hkv, d, scale=0.0, seq_base=None, use_tail=True):
    desc = lava.LayerDesc.make(H, Hkv, d, 1, di.dtype, softmax_scale=scale)
    batch = di.q.shape[0]
    dev = "cuda"
    q = lava.to_device(di.q, di.dtype, dev)
    kh = lava.to_device(di.k_hat, di.dtype, dev) if di.k_hat.shape[0] else None
    vh = lava.to_device(di.v_hat, di.dtype, dev) if di.v_hat.shape[0] else None
    offs = torch.from_numpy(di.head_offsets).to(dev)
    tail = di.tail_len if use_tail else 0
    kt = lava.to_device(di.k_tail, di.dtype, dev) if tail else None
    vt = lava.to_device(di.v_tail, di.dtype, dev) if tail else None
    sb = None if seq_base is None else torch.tensor(seq_base, dtype=torch.int64, device=dev)
    out = torch.full((batch, H, d), 777.0, dtype=torch.float32, device=dev)
    lse = torch.full((batch, H), 777.0, dtype=torch.float32, device=dev)
    lava.lava_decode_attention(desc, batch, q, kh, vh, offs, di.rows_capacity, seq_base=sb, k_tail=kt, v_tail=vt,
                               tail_len=tail, tail_capacity=di.k_tail.shape[2], out=out, lse=lse)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


def run_oracle(di, scale=None, seq_base=None, use_tail=True):
    q = synth.load_f64(di.q, di.dtype)
    k = synth.load_f64(di.k_hat, di.dtype)
    v = synth.load_f64(di.v_hat, di.dtype)
    kt = synth.load_f64(di.k_tail, di.dtype)[:, :, : di.tail_len]
    vt = synth.load_f64(di.v_tail, di.dtype)[:, :, : di.tail_len]
    outs, lses = [], []
    for b in range(q.shape[0]):
        base = b * di.rows_capacity if seq_base is None else int(seq_base[b])
        rows = int(di.head_offsets[b, -1])
        o, l = O.decode_attention(q[b], k[base: base + rows], v[base: base + rows], di.head_offsets[b],
                                  kt[b] if use_tail and di.tail_len else None,
                                  vt[b] if use_tail and di.tail_len else None, scale)
        outs.append(o)
        lses.append(l)
    return np.stack(outs), np.stack(lses)


def compare(out, lse, ref, ref_lse, tol=DEC_TOL):
    assert out.shape == ref.shape
    worst = 0.0
    for b in range(ref.shape[0]):
        for h in range(ref.shape[1]):
            scale = max(np.abs(ref[b, h]).max(), 1e-30)
            err = np.abs(out[b, h] - ref[b, h]).max() / scale
            worst = max(worst, err)
            if np.isinf(ref_lse[b, h]):
                assert np.all(out[b, h] == 0.0) and lse[b, h] == -np.inf
            else:
                assert err <= tol, (b, h, err)
                assert abs(lse[b, h] - ref_lse[b, h]) <= 1e-5 * (1 + abs(ref_lse[b, h])), (b, h)
    return worst


CASES = [
    # H, Hkv, d, dtype, rows per sequence, tail_len
    (32, 8, 128, "bf16", [8192], 0),
    (32, 8, 128, "bf16", [1000, 4097, 31], 5),
    (8, 2, 64, "f32", [256], 0),
    (8, 2, 64, "f32", [300, 77], 40),
    (8, 4, 64, "bf16", [513, 2000], 3),
    (4, 4, 128, "f32", [700], 129),
    (6, 2, 128, "bf16", [900, 64], 0),          # G = 3 (padded to 4)
    (10, 2, 64, "bf16", [1500], 1),             # G = 5 (padded to 8)
    (16, 2, 128, "bf16", [2100, 1], 33),        # G = 8
    (28, 4, 128, "bf16", [3000], 0),            # G = 7
    (2, 2, 128, "bf16", [1, 2, 0], 0),          # single rows; an empty sequence
    (64, 64, 64, "bf16", [4000, 333], 2),       # 64 KV heads (MHA): the largest head count the step takes
    (128, 64, 128, "bf16", [2500], 0),          # 64 KV heads, G = 2
]


@pytest.mark.parametrize("H,Hkv,d,dtype,rows,tail", CASES)
@pytest.mark.parametrize("seed", [0, 1])
def test_decode_matches_oracle(lava, H, Hkv, d, dtype, rows, tail, seed):
    say(f"decode H={H} Hkv={Hkv} d={d} {dtype} rows={rows} tail={tail} seed={seed}")
    di = synth.gen_decode(H, Hkv, d, dtype, rows, seed, tail_len=tail, tail_capacity=tail + 3 if tail else 0)
    out, lse = run_gpu(lava, di, H, Hkv, d)
    ref, ref_lse = run_oracle(di)
    worst = compare(out, lse, ref, ref_lse)
    say(f"  worst relative error {worst:.2e}")


def test_decode_uniform_split_scale_and_seq_base(lava):
    say("decode: uniform split, explicit scale, explicit sequence bases in reverse order")
    H, Hkv, d = 8, 2, 128
    di = synth.gen_decode(H, Hkv, d, "bf16", [640, 640, 640], 5, rows_capacity=700, split="uniform")
    base = [1400, 700, 0]
    # reorder the sequences' rows in the pool to match the bases
    k2, v2 = di.k_hat.copy(), di.v_hat.copy()
    for b in range(3):
        k2[base[b]: base[b] + 700] = di.k_hat[b * 700: (b + 1) * 700]
        v2[base[b]: base[b] + 700] = di.v_hat[b * 700: (b + 1) * 700]
    di.k_hat, di.v_hat = k2, v2
    out, lse = run_gpu(lava, di, H, Hkv, d, scale=0.05, seq_base=base)
    ref, ref_lse = run_oracle(di, scale=0.05, seq_base=base)
    compare(out, lse, ref, ref_lse)


def test_decode_is_deterministic_and_leaves_neighbours_alone(lava):
    say("decode: determinism")
    H, Hkv, d = 32, 8, 128
    di = synth.gen_decode(H, Hkv, d, "bf16", [5000, 3000], 9, tail_len=7)
    a, la = run_gpu(lava, di, H, Hkv, d)
    b, lb = run_gpu(lava, di, H, Hkv, d)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32)) and np.array_equal(la.view(np.uint32), lb.view(np.uint32))


def test_decode_reports_offsets_beyond_capacity(lava):
    say("decode: offsets beyond the stated capacity give NaN, nothing is read out of bounds")
    H, Hkv, d = 8, 2, 64
    di = synth.gen_decode(H, Hkv, d, "bf16", [200, 200], 3)
    di.head_offsets[1, -1] = 201          # claims one row more than the capacity
    out, lse = run_gpu(lava, di, H, Hkv, d)
    assert np.all(np.isnan(out[1])) and np.all(np.isnan(lse[1]))
    ref, ref_lse = run_oracle(synth.gen_decode(H, Hkv, d, "bf16", [200, 200], 3))
    compare(out[:1], lse[:1], ref[:1], ref_lse[:1])
    di.head_offsets[1] = [0, 150, 100]    # decreasing
    out, lse = run_gpu(lava, di, H, Hkv, d)
    assert np.all(np.isnan(out[1]))


def test_decode_full_cache_equals_full_attention(lava):
    say("decode over an unevicted cache (offsets g*N) == plain attention of the new token")
    sh = synth.config(2, n=4096 + 37)
    inp = synth.gen_layer(sh, 3)
    H, Hkv, d, N = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.n
    q = inp.q_win[:, -1, :][None]                                    # the last window query as the new token
    di = synth.DecodeInputs(sh.dtype, np.ascontiguousarray(q), inp.k.reshape(-1, d), inp.v.reshape(-1, d),
                            np.array([[g * N for g in range(Hkv + 1)]], dtype=np.int64), Hkv * N,
                            np.zeros((1, Hkv, 1, d), dtype=inp.k.dtype), np.zeros((1, Hkv, 1, d), dtype=inp.k.dtype), 0)
    out, lse = run_gpu(lava, di, H, Hkv, d)
    qf, kf, vf = inp.f64()
    G = H // Hkv
    for h in range(H):
        logits = kf[h // G] @ qf[h, -1] / math.sqrt(d)
        p = np.exp(logits - logits.max())
        want = (p / p.sum()) @ vf[h // G]
        assert np.abs(out[0, h] - want).max() <= DEC_TOL * np.abs(want).max()


def test_decode_after_eviction_end_to_end(lava):
    say("evict a layer on the GPU, then decode over the packed cache it wrote")
    sh = synth.config(2, n=8192 + 11, budget=1024)
    inp = synth.gen_layer(sh, 1)
    H, Hkv, d = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    desc = lava.LayerDesc.make(H, Hkv, d, sh.window, sh.dtype)
    dev = "cuda"
    qw, k, v = (lava.to_device(a, sh.dtype, dev) for a in (inp.q_win, inp.k, inp.v))
    res = lava.evict_layer(desc, sh.n, qw, k, v, sh.budget)
    torch.cuda.synchronize()
    r = np.random.Generator(np.random.PCG64(77))
    q_new = synth.store(r.standard_normal((1, H, d), dtype=np.float32), sh.dtype)
    out, lse = lava.lava_decode_attention(desc, 1, lava.to_device(q_new, sh.dtype, dev), res["k_hat"], res["v_hat"],
                                          res["head_offsets"].view(1, -1).contiguous(), sh.budget)
    torch.cuda.synchronize()
    offs = res["head_offsets"].cpu().numpy()
    assert offs[-1] == sh.budget and np.all(np.diff(offs) >= sh.window)
    want, want_lse = O.decode_attention(synth.load_f64(q_new, sh.dtype)[0],
                                        synth.load_f64(lava.to_host_bits(res["k_hat"]), sh.dtype),
                                        synth.load_f64(lava.to_host_bits(res["v_hat"]), sh.dtype), offs)
    compare(out.cpu().numpy(), lse.cpu().numpy(), want[None], want_lse[None])


def test_decode_large_batch_sampled(lava):
    say("decode: batch 64 x 8192 rows (the benchmarked shape), sampled sequences against the oracle")
    H, Hkv, d = 32, 8, 128
    di = synth.gen_decode(H, Hkv, d, "bf16", [8192] * 64, 4, tail_len=16)
    out, lse = run_gpu(lava, di, H, Hkv, d)
    ref, ref_lse = run_oracle(di)
    worst = compare(out, lse, ref, ref_lse)
    say(f"  worst relative error {worst:.2e}")
