#!/usr/bin/env python3
"""Benchmark of the LAVa prefill-end eviction path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4|cfg2|cfg1]

One step = the whole hot path for one layer of one sequence, inputs resident in HBM:
lava_window_scores (value norms, window softmax statistics, window scores, pooling + layer
statistic) -> lava_layer_budgets (on device) -> lava_select_topk (budget read on device) ->
lava_compact_kv.  Steps rotate over several distinct K/V buffer sets so that no step can be
served from the 256 MB Infinity Cache by the previous one.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak

def measured_traffic(workload):
    """{kernel: (read bytes, write bytes)} per launch from profiles/<workload>_hbm_counters.md, the summary that
    `bench.py --summarize-profiles` writes from two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE; scaled by
    what the same counters read for the 1 GiB probe kernels).  Empty if the summary is not there."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_counters.md")
    out = {}
    if not os.path.exists(path):
        return out
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) < 5 or not cells[0] or cells[0] in ("kernel", "---"):
            continue
        try:
            read_mib, write_mib = float(cells[3]), float(cells[4])
        except ValueError:
            continue
        for kid in ("vnorm", "stats", "scores", "sweep", "sel_fused", "compact", "decode_merge", "decode"):
            if cells[0].startswith(kid + "_kernel"):
                # the statistics kernel that also sweeps the value rows is the launch the library times as "prepass"
                name = "prepass" if kid == "stats" and cells[0].rstrip(">").endswith("true") else kid
                if name not in out:
                    out[name] = (int(read_mib * 2**20), int(write_mib * 2**20))
    return out


def summarize_profiles(workload):
    """Writes profiles/<workload>_kernel_trace.md and profiles/<workload>_hbm_counters.md from the rocprofv3 CSV
    output under gpurun_out/ (directories prof_<wl>, pmc_fetch_<wl>, pmc_write_<wl>, pmc_util_<wl>, as the
    commands quoted in the summaries leave them).  Reads files only; runs nothing."""
    import collections
    import csv
    wl = workload
    flags = {"decode": "--steps 40 --decode-only"}.get(
        wl, "--steps 20 --warmup 3 --no-cpu-baseline --no-check --no-decode --no-cascade" + ("" if wl == "cfg4" else f" --workload {wl}"))
    cmd = f"python3 bench.py {flags}"

    def short(n):
        return n.replace("(anonymous namespace)::", "").split("(")[0].replace("void lava::", "").replace("lava::", "")

    def ours(n):
        return not (n.startswith("void at::") or "rocclr" in n or n.startswith("Cijk") or n.strip() == "void")

    rows = list(csv.DictReader(open(os.path.join(ROOT, f"gpurun_out/prof_{wl}/{wl}_kernel_stats.csv"))))
    out = [f"# rocprofv3 kernel trace - {wl}\n",
           "Command (from the repository root on the MI355X box, after `cd /tmp && export TMPDIR=/tmp`):\n",
           f"    rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/prof_{wl} -o {wl} -- {cmd}\n",
           "Per-kernel durations from `*_kernel_stats.csv` (the command runs warm-up, timed, per-kernel-event and "
           "caller-LSE loops; `calls` counts all of them); summary written by `python bench.py --summarize-profiles "
           f"{wl}`.  Kernels PyTorch launches while the inputs are generated are left out.\n",
           "| kernel | calls | avg us | min us | max us | % of GPU time |", "|---|---|---|---|---|---|"]
    for r in rows:
        n = short(r["Name"])
        if ours(n):
            out.append(f"| {n} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.2f} | {float(r['MinNs']) / 1e3:.2f} | "
                       f"{float(r['MaxNs']) / 1e3:.2f} | {r['Percentage']} |")
    open(os.path.join(ROOT, "profiles", f"{wl}_kernel_trace.md"), "w").write("\n".join(out) + "\n")

    def pmc(kind):
        path = os.path.join(ROOT, f"gpurun_out/pmc_{kind}_{wl}/p_counter_collection.csv")
        if not os.path.exists(path):
            return None
        agg = collections.defaultdict(lambda: collections.defaultdict(list))
        for r in csv.DictReader(open(path)):
            agg[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
        return {k: {c: sum(x) / len(x) for c, x in v.items()} for k, v in agg.items()}

    f, w, u = pmc("fetch"), pmc("write"), pmc("util")
    if f is None or w is None:
        print(f"wrote profiles/{wl}_kernel_trace.md (no counter runs found)")
        return
    kib = 1048576.0
    if "probe_read_kernel" in f and "probe_copy_kernel" in w:
        ff, wf = kib / f["probe_read_kernel"]["FETCH_SIZE"], kib / w["probe_copy_kernel"]["WRITE_SIZE"]
        calib = ("Calibration: the same command runs `lava_probe_stream` on 1 GiB (= 1048576 KiB): `probe_read_kernel` "
                 f"FETCH_SIZE = {f['probe_read_kernel']['FETCH_SIZE']:.1f} -> bytes = counter KiB x {ff:.3f}; "
                 f"`probe_copy_kernel` WRITE_SIZE = {w['probe_copy_kernel']['WRITE_SIZE']:.1f} -> bytes = counter KiB x {wf:.3f}.\n")
    else:
        ff, wf = 2.0, 1.0
        calib = "Calibration: the factors of `cfg4_hbm_counters.md` (same counters): FETCH_SIZE KiB x 2.000, WRITE_SIZE KiB x 1.000.\n"
    out = [f"# rocprofv3 HBM byte counters and utilisation - {wl}\n",
           "Commands (each its own run, after `cd /tmp && export TMPDIR=/tmp`):\n",
           f"    rocprofv3 --pmc FETCH_SIZE --output-format csv -d gpurun_out/pmc_fetch_{wl} -o p -- {cmd}",
           f"    rocprofv3 --pmc WRITE_SIZE --output-format csv -d gpurun_out/pmc_write_{wl} -o p -- {cmd}",
           f"    rocprofv3 --pmc MfmaUtil MemUnitStalled LDSBankConflict --output-format csv -d gpurun_out/pmc_util_{wl} -o p -- {cmd}\n",
           calib, f"Summary written by `python bench.py --summarize-profiles {wl}`; `bench.py` reads columns 4 and 5 of "
           "this table for `traffic`.\n",
           "| kernel | FETCH_SIZE (KiB/dispatch) | WRITE_SIZE (KiB/dispatch) | HBM read MiB (scaled) | HBM write MiB (scaled) | "
           "MfmaUtil % | MemUnitStalled % | LDSBankConflict % |", "|---|---|---|---|---|---|---|---|"]
    for k in f:
        if not ours(k) or k not in w:
            continue
        uu = (u or {}).get(k, {})
        out.append(f"| {k} | {f[k]['FETCH_SIZE']:.1f} | {w[k]['WRITE_SIZE']:.1f} | {f[k]['FETCH_SIZE'] * ff / 1024:.2f} | "
                   f"{w[k]['WRITE_SIZE'] * wf / 1024:.2f} | {uu.get('MfmaUtil', float('nan')):.1f} | "
                   f"{uu.get('MemUnitStalled', float('nan')):.1f} | {uu.get('LDSBankConflict', float('nan')):.1f} |")
    open(os.path.join(ROOT, "profiles", f"{wl}_hbm_counters.md"), "w").write("\n".join(out) + "\n")
    print(f"wrote profiles/{wl}_kernel_trace.md and profiles/{wl}_hbm_counters.md")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg4", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--sets", type=int, default=0, help="distinct K/V buffer sets (0 = enough for >= 1.5 GiB)")
    ap.add_argument("--sweep-schedule", default="auto", choices=["auto", "separate", "persistent", "prepass"],
                    help="lava_tuning.sweep_schedule for the whole run (A/B of the sweep schedules)")
    ap.add_argument("--no-plan", action="store_true",
                    help="lava_layer_budgets as a launch of its own instead of the budget plan carried by the scores call")
    ap.add_argument("--sweep-shape", default="auto", choices=["auto", "wide", "narrow"],
                    help="lava_tuning.sweep_shape for the whole run (A/B of the two workgroup shapes of the key sweeps)")
    ap.add_argument("--summarize-profiles", metavar="WORKLOAD", default=None,
                    help="write profiles/<workload>_*.md from rocprofv3 CSV output under gpurun_out/ and exit (no GPU)")
    ap.add_argument("--no-primed", action="store_true",
                    help="plain lava_window_scores + lava_select_topk instead of the pair in which the score kernels "
                         "prepare the selection's first histogram")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-check", action="store_true")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-attention leg")
    ap.add_argument("--no-cascade", action="store_true", help="skip the Algorithm-2 cascade leg (cfg3: the layer-by-layer route)")
    ap.add_argument("--no-compare", action="store_true",
                    help="cfg5: skip the comparison leg (one call per sequence), for profiling the batched launches")
    ap.add_argument("--decode-only", action="store_true",
                    help="run only the batched decode-attention case (for profiling that kernel) and print its object")
    return ap.parse_args()


def cascade_leg(lava, torch, np, sh, desc, dev, sets, scores, args):
    """Algorithm 2's outer loop for a stack of layers: after each layer arrives, device budgets plus one
    (re-)eviction per layer seen so far.  Timing only: every layer reuses the benchmark layer's K, V and
    scores (the selection and the copies do the same work whatever the values are), the statistics are
    drawn at random so the budgets differ per layer.  Parity of the driver is a test, not this leg."""
    n_layers = 8
    per_layer = sh.budget
    total = n_layers * per_layer
    rng = np.random.Generator(np.random.PCG64(args.seed + 5))
    stats = torch.from_numpy((1e-6 * (0.5 + rng.random(n_layers))).astype(np.float32))
    ws = torch.empty(lava.lava_cascade_workspace_bytes(desc, sh.n, n_layers, total), dtype=torch.uint8, device=dev)
    _, k, v = sets[0]

    def measure(in_place):
        state = lava.CascadeState(desc, n_layers, total, device=dev, in_place=in_place)
        state.e.copy_(stats)

        def run():
            state.reset()
            times = []
            for l in range(n_layers):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                lava.lava_cascade_step(desc, l, sh.n, k, v, scores, state, total, workspace=ws)
                b.record()
                times.append((a, b))
            torch.cuda.synchronize()
            return [1e3 * a.elapsed_time(b) for a, b in times]

        run()
        reps = [run() for _ in range(5)]
        best = [min(r[l] for r in reps) for l in range(n_layers)]
        return best, state.budgets.cpu().numpy().tolist(), state.bytes()

    best, budgets, state_bytes = measure(False)
    best_ip, budgets_ip, state_bytes_ip = measure(True)
    assert budgets == budgets_ip
    return {"note": "Alg. 2 outer loop, one step per arriving layer: budgets + one (re-)eviction per layer so far",
            "layers": n_layers, "total_budget": total, "us_per_step": [round(x, 1) for x in best],
            "us_all_steps": round(sum(best), 1), "final_budgets": budgets,
            "state_bytes": state_bytes, "dense_kv_bytes_of_the_layers": n_layers * 2 * k.numel() * k.element_size(),
            "one_arena_in_place": {"us_per_step": [round(x, 1) for x in best_ip], "us_all_steps": round(sum(best_ip), 1),
                                   "state_bytes": state_bytes_ip}}


def decode_leg(lava, synth, torch, np, sh, desc, dev, sets, k_hat, v_hat, offs, B, args):
    """The step after the path: one new token attends to the compressed cache.  Three timings:
    the layer just evicted (batch 1), the same token over the unevicted cache (what the eviction
    saves), and a batch of 64 compressed caches rotating over >= 1 GiB (the bandwidth case)."""
    esize = synth.itemsize(sh.dtype)
    row_bytes = sh.head_dim * esize
    iters = max(20, args.steps // 2)

    def timed(fn, n):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    rng = np.random.Generator(np.random.PCG64(args.seed + 99))
    q1 = lava.to_device(synth.store(rng.standard_normal((1, sh.n_q_heads, sh.head_dim), dtype=np.float32), sh.dtype),
                        sh.dtype, dev)
    offs1 = offs.view(1, -1).contiguous()
    out1 = torch.empty(1, sh.n_q_heads, sh.head_dim, dtype=torch.float32, device=dev)
    lse1 = torch.empty(1, sh.n_q_heads, dtype=torch.float32, device=dev)
    ws1 = torch.empty(lava.lava_decode_workspace_bytes(desc, 1, B), dtype=torch.uint8, device=dev)
    t_small = timed(lambda i: lava.lava_decode_attention(desc, 1, q1, k_hat, v_hat, offs1, B, out=out1, lse=lse1,
                                                         workspace=ws1), 4 * iters)

    # the same token over the whole, unevicted layer cache
    full_rows = sh.n_kv_heads * sh.n
    offs_full = torch.arange(sh.n_kv_heads + 1, dtype=torch.int64, device=dev).mul_(sh.n).view(1, -1).contiguous()
    ws_full = torch.empty(lava.lava_decode_workspace_bytes(desc, 1, full_rows), dtype=torch.uint8, device=dev)

    def full(i):
        _, k, v = sets[i % len(sets)]
        lava.lava_decode_attention(desc, 1, q1, k.view(-1, sh.head_dim), v.view(-1, sh.head_dim), offs_full, full_rows,
                                   out=out1, lse=lse1, workspace=ws_full)
    t_full = timed(full, iters)

    out = {
        "note": "one new token per sequence over the packed variable-length cache (Sec. 2 step on the retained entries)",
        "evicted_layer_us": round(1e6 * t_small, 2), "evicted_rows": B,
        "full_cache_us": round(1e6 * t_full, 2), "full_rows": full_rows,
        "attention_speedup_from_eviction": round(t_full / t_small, 1),
    }
    out["batched"] = decode_batched(lava, synth, torch, np, sh, desc, dev, B, args, iters)
    return out


def decode_batched(lava, synth, torch, np, sh, desc, dev, B, args, iters):
    """64 compressed caches of B rows each, skewed head budgets, rotating over >= 1 GiB of pools."""
    esize = synth.itemsize(sh.dtype)
    row_bytes = sh.head_dim * esize

    def timed(fn, n):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    batch = 64
    n_pools = max(2, int(np.ceil(2**30 / (2 * batch * B * row_bytes))))
    di = synth.gen_decode(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, [B] * batch, args.seed)
    qb = lava.to_device(di.q, sh.dtype, dev)
    offs_b = torch.from_numpy(di.head_offsets).to(dev)
    kb0, vb0 = lava.to_device(di.k_hat, sh.dtype, dev), lava.to_device(di.v_hat, sh.dtype, dev)
    pools = [(kb0, vb0)] + [(kb0.clone(), vb0.clone()) for _ in range(n_pools - 1)]
    out_b = torch.empty(batch, sh.n_q_heads, sh.head_dim, dtype=torch.float32, device=dev)
    lse_b = torch.empty(batch, sh.n_q_heads, dtype=torch.float32, device=dev)
    ws_b = torch.empty(lava.lava_decode_workspace_bytes(desc, batch, B), dtype=torch.uint8, device=dev)

    def batched(i):
        kb, vb = pools[i % n_pools]
        lava.lava_decode_attention(desc, batch, qb, kb, vb, offs_b, B, out=out_b, lse=lse_b, workspace=ws_b)
    t_batch = timed(batched, iters)
    lava.prof_enable(True)
    lava.prof_reset()
    for i in range(iters):
        batched(i)
    torch.cuda.synchronize()
    prof = lava.prof_read()
    lava.prof_enable(False)
    k_us = {n: 1e3 * prof[n][0] / max(prof[n][1], 1) for n in ("decode", "decode_merge")}
    bytes_b = 2 * batch * B * row_bytes
    return {"batch": batch, "rows_per_seq": B, "us": round(1e6 * t_batch, 2), "pools": n_pools,
            "algorithmic_bytes": bytes_b, "kernel_us": {n: round(v, 2) for n, v in k_us.items()},
            "achieved_GBs": round(bytes_b / (k_us["decode"] * 1e-6) / 1e9, 1),
            "frac_of_hbm_peak": round(bytes_b / (k_us["decode"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}


def ragged_batch(lava, synth, torch, np, dev, args):
    """Config 5, one layer: 16 sequences of ragged length (4096 .. 65536 tokens) evicted in one batch.
    Throughput only, so K / V / Q are drawn on the device (same distributions as the generator, without
    the planted structure); every sequence gets the same per-sequence budget.  The sweeps of the whole
    batch are three launches, the budgets one, the selections and the compactions one table each.  For
    comparison the same work is also timed with one call per sequence for every step."""
    sh = synth.config(2)
    H, Hkv, d, w = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.window
    desc = lava.LayerDesc.make(H, Hkv, d, w, sh.dtype)
    lens = [int(x) for x in synth.ragged_lengths(16, args.seed)]
    total, B = sum(lens), 4096
    gen = torch.Generator(device=dev).manual_seed(args.seed)
    n_sets = max(2, int(np.ceil(1.5 * 2**30 / (4 * total * Hkv * d))))
    sets = []
    for _ in range(n_sets):
        k = torch.randn(total * Hkv, d, generator=gen, device=dev).to(torch.bfloat16)
        v = (torch.randn(total * Hkv, d, generator=gen, device=dev) *
             torch.exp(0.5 * torch.randn(total * Hkv, 1, generator=gen, device=dev))).to(torch.bfloat16)
        q = torch.randn(len(lens), H, w, d, generator=gen, device=dev).to(torch.bfloat16)
        sets.append((q, k, v))
    ws = torch.empty(lava.lava_window_scores_workspace_bytes(desc, len(lens), total), dtype=torch.uint8, device=dev)
    ws_sel = torch.empty(lava.lava_select_workspace_bytes(Hkv * max(lens)), dtype=torch.uint8, device=dev)
    scores = torch.empty(Hkv * total, dtype=torch.float32, device=dev)
    vbar = torch.empty(len(lens), Hkv, dtype=torch.float32, device=dev)
    stat = torch.empty(len(lens), dtype=torch.float32, device=dev)
    budgets = torch.empty(len(lens), 1, dtype=torch.int64, device=dev)
    total_b = torch.full((len(lens),), B, dtype=torch.int64, device=dev)
    lo = torch.full((len(lens), 1), Hkv * w, dtype=torch.int64, device=dev)
    hi = torch.tensor([[Hkv * n] for n in lens], dtype=torch.int64, device=dev)
    counts = torch.empty(len(lens), Hkv, dtype=torch.int32, device=dev)
    offs = torch.empty(len(lens), Hkv + 1, dtype=torch.int64, device=dev)
    idx = torch.empty(len(lens), B, dtype=torch.int32, device=dev)
    kept = torch.empty(len(lens), B, dtype=torch.float32, device=dev)
    k_hat = torch.empty(len(lens), B, d, dtype=torch.bfloat16, device=dev)
    v_hat = torch.empty(len(lens), B, d, dtype=torch.bfloat16, device=dev)
    starts = np.concatenate([[0], np.cumsum(lens)])

    ws_batch = torch.empty(lava.lava_select_batch_workspace_bytes(len(lens), Hkv * max(lens)), dtype=torch.uint8,
                           device=dev)

    # the tables hold pointers only: built once per buffer set, as a serving loop would keep them
    sel = []
    for b, n in enumerate(lens):
        a0, a1 = int(starts[b]) * Hkv, int(starts[b + 1]) * Hkv
        sel.append(lava.select_problem(scores[a0:a1], B, counts[b], offs[b], idx[b], kept[b], budget_dev=budgets[b],
                                       primed=not args.no_primed))
    sel_table = (lava.SelectProblem * len(lens))(*sel)
    cmp_tables = []
    for _, k, v in sets:
        cmp = []
        for b, n in enumerate(lens):
            a0, a1 = int(starts[b]) * Hkv, int(starts[b + 1]) * Hkv
            cmp.append(lava.compact_problem(desc, n, k[a0:a1], v[a0:a1], offs[b], idx[b], B, k_hat[b], v_hat[b]))
        cmp_tables.append((lava.CompactProblem * len(lens))(*cmp))

    # budgets of every sequence (one layer each here) formed by the scores call, or by a launch of their own
    planned = not args.no_plan
    e_table = torch.zeros(len(lens), 1, dtype=torch.float32, device=dev)
    plan = lava.make_budget_plan(e_table, 0, total_b, lo, hi, budgets) if planned else None

    def tail_batched(i):
        if not planned:
            lava.lava_layer_budgets(stat.view(-1, 1), total_b, lo, hi, budgets=budgets)
        lava.lava_select_topk_batch(Hkv, sel_table, Hkv * max(lens), workspace=ws_batch)
        lava.lava_compact_batch(desc, cmp_tables[i % n_sets])

    def tail(q, k, v):
        lava.lava_layer_budgets(stat.view(-1, 1), total_b, lo, hi, budgets=budgets)
        for b, n in enumerate(lens):
            a0, a1 = int(starts[b]) * Hkv, int(starts[b + 1]) * Hkv
            lava.lava_select_topk(Hkv, scores[a0:a1], B, budget_dev=budgets[b], head_counts=counts[b],
                                  head_offsets=offs[b], kept_idx=idx[b], kept_scores=kept[b], workspace=ws_sel)
            lava.lava_compact_kv(desc, n, k[a0:a1], v[a0:a1], offs[b], idx[b], B, k_out=k_hat[b], v_out=v_hat[b])

    def step_batched(i):
        q, k, v = sets[i % n_sets]
        lava.lava_window_scores(desc, lens, q, k, v, scores=scores, vbar=vbar, layer_stat=stat, workspace=ws,
                                select_workspace=None if args.no_primed else ws_batch, budget_plan=plan)
        tail_batched(i)

    def step_one_by_one(i):
        q, k, v = sets[i % n_sets]
        for b, n in enumerate(lens):
            a0, a1 = int(starts[b]) * Hkv, int(starts[b + 1]) * Hkv
            lava.lava_window_scores(desc, [n], q[b:b + 1], k[a0:a1], v[a0:a1], scores=scores[a0:a1], vbar=vbar[b:b + 1],
                                    layer_stat=stat[b:b + 1], workspace=ws)
        tail(q, k, v)

    def timed(fn, steps):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    steps = max(10, args.steps // 10)
    t_batch = timed(step_batched, steps)
    t_seq = None if args.no_compare else timed(step_one_by_one, steps)
    esize = 2
    path_bytes = 2 * total * Hkv * d * esize + 2 * 4 * Hkv * total + len(lens) * 4 * B * d * esize
    return {
        "metric": "cached tokens evicted-and-compacted/sec per layer; achieved HBM GB/s vs peak",
        "value": round(total / t_batch, 1), "unit": "tokens/s/layer", "n_gpus": 1, "steps": steps, "warmup": 3,
        "ms_per_step": round(1e3 * t_batch, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic (drawn on the device)",
        "config": {"workload": f"cfg5: one layer, 32q/8kv heads, d_h 128, batch 16 ragged, lengths {lens}, "
                               f"w=32, budget {B} per sequence, bf16", "total_tokens": total, "kv_buffer_sets": n_sets},
        "path": {"algorithmic_bytes": path_bytes, "achieved_GBs": round(path_bytes / t_batch / 1e9, 1),
                 "frac_of_hbm_peak": round(path_bytes / t_batch / 1e9 / HBM_PEAK_GBS, 4)},
        "one_call_per_sequence": None if t_seq is None else {"ms_per_step": round(1e3 * t_seq, 5),
                                                             "value": round(total / t_seq, 1)},
    }


def layer_stack(lava, synth, torch, np, dev, args):
    """Config 3: a 32-layer model, 32K cached tokens per layer, one shared budget of 131072 entries; K + V of
    all layers (4 GiB) resident.  Throughput only: K / V / Q are drawn on the device.  Two routes to the
    same final state: `single_shot` once every layer is there (the layers as a batch: three sweep launches,
    one budgets launch, one table of selections, one of compactions) and `cascade`, Algorithm 2 as layers
    arrive (per layer: the sweeps of that layer, then one cascade step over all layers so far)."""
    sh = synth.config(3)
    H, Hkv, d, w, N = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.window, sh.n
    L, total = 32, 131072
    dense = Hkv * N
    desc = lava.LayerDesc.make(H, Hkv, d, w, sh.dtype)
    gen = torch.Generator(device=dev).manual_seed(args.seed)
    k = torch.empty(L, Hkv * N, d, dtype=torch.bfloat16, device=dev)
    v = torch.empty(L, Hkv * N, d, dtype=torch.bfloat16, device=dev)
    for l in range(L):
        k[l] = torch.randn(Hkv * N, d, generator=gen, device=dev).to(torch.bfloat16)
        v[l] = (torch.randn(Hkv * N, d, generator=gen, device=dev) *
                torch.exp(0.5 * torch.randn(Hkv * N, 1, generator=gen, device=dev))).to(torch.bfloat16)
    q = torch.randn(L, H, w, d, generator=gen, device=dev).to(torch.bfloat16)
    state = lava.CascadeState(desc, L, total, device=dev)
    scores = torch.empty(L * dense, dtype=torch.float32, device=dev)
    vbar = torch.empty(L, Hkv, dtype=torch.float32, device=dev)
    ws_batch = torch.empty(lava.lava_window_scores_workspace_bytes(desc, L, L * N), dtype=torch.uint8, device=dev)
    ws_one = torch.empty(lava.lava_window_scores_workspace_bytes(desc, 1, N), dtype=torch.uint8, device=dev)
    ws_casc = torch.empty(lava.lava_cascade_workspace_bytes(desc, N, L, total), dtype=torch.uint8, device=dev)
    ws_sel = torch.empty(lava.lava_select_batch_workspace_bytes(L, dense), dtype=torch.uint8, device=dev)
    lo = torch.full((1, L), Hkv * w, dtype=torch.int64, device=dev)
    hi = torch.full((1, L), dense, dtype=torch.int64, device=dev)
    total_t = torch.tensor([total], dtype=torch.int64, device=dev)
    budgets = torch.empty(1, L, dtype=torch.int64, device=dev)
    layer_start = torch.zeros(L + 1, dtype=torch.int64, device=dev)
    counts = torch.empty(L, Hkv, dtype=torch.int32, device=dev)
    offs = torch.empty(L, Hkv + 1, dtype=torch.int64, device=dev)
    idx = torch.empty(total, dtype=torch.int32, device=dev)
    k_hat = torch.empty(total, d, dtype=torch.bfloat16, device=dev)
    v_hat = torch.empty(total, d, dtype=torch.bfloat16, device=dev)
    cap = min(total, dense)
    sel = [lava.select_problem(scores[l * dense: (l + 1) * dense], cap, counts[l], offs[l], idx,
                               budget_dev=budgets[0, l: l + 1], out_offset_dev=layer_start[l: l + 1]) for l in range(L)]
    cmp = [lava.compact_problem(desc, N, k[l], v[l], offs[l], idx, total, k_hat, v_hat,
                                out_offset_dev=layer_start[l: l + 1]) for l in range(L)]
    sel_table = (lava.SelectProblem * L)(*sel)
    cmp_table = (lava.CompactProblem * L)(*cmp)

    def single_shot():
        lava.lava_window_scores(desc, [N] * L, q, k, v, scores=scores, vbar=vbar, layer_stat=state.e, workspace=ws_batch)
        lava.lava_layer_budgets(state.e.view(1, L), total_t, lo, hi, budgets=budgets)
        torch.cumsum(budgets[0], 0, out=layer_start[1:])
        lava.lava_select_topk_batch(Hkv, sel_table, dense, workspace=ws_sel)
        lava.lava_compact_batch(desc, cmp_table)

    def cascade():
        state.reset()
        for l in range(L):
            sc = scores[l * dense: (l + 1) * dense]
            lava.lava_window_scores(desc, [N], q[l: l + 1], k[l], v[l], scores=sc, vbar=vbar[l: l + 1],
                                    layer_stat=state.e[l: l + 1], workspace=ws_one)
            lava.lava_cascade_step(desc, l, N, k[l], v[l], sc, state, total, workspace=ws_casc)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    reps = max(5, args.steps // 20)
    t_single = timed(single_shot, reps)
    t_casc = None if args.no_cascade else timed(cascade, reps)
    tokens = L * N
    kv_bytes = 2 * k.numel() * k.element_size()
    path_bytes = kv_bytes + 2 * 4 * L * dense + 4 * total * d * 2
    return {
        "metric": "cached tokens evicted-and-compacted/sec per layer; achieved HBM GB/s vs peak",
        "value": round(tokens / t_single, 1), "unit": "tokens/s/layer", "n_gpus": 1, "steps": reps, "warmup": 1,
        "ms_per_step": round(1e3 * t_single, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic (drawn on the device)",
        "config": {"workload": f"cfg3: {L} layers, 32q/8kv heads, d_h 128, N={N} per layer, w=32, shared budget "
                               f"{total}, bf16; one step = the whole stack", "kv_bytes_resident": kv_bytes},
        "path": {"algorithmic_bytes": path_bytes, "achieved_GBs": round(path_bytes / t_single / 1e9, 1),
                 "frac_of_hbm_peak": round(path_bytes / t_single / 1e9 / HBM_PEAK_GBS, 4)},
        "cascade_as_layers_arrive": None if t_casc is None else {
            "ms_per_stack": round(1e3 * t_casc, 4), "value": round(tokens / t_casc, 1),
            "us_per_layer": round(1e6 * t_casc / L, 1), "state_bytes": state.bytes()},
    }


def main():
    args = parse()
    if args.summarize_profiles:
        summarize_profiles(args.summarize_profiles)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported. Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2509_09754_amd import lava, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    lava.set_tuning(sweep_schedule=args.sweep_schedule, sweep_shape=args.sweep_shape)

    if args.workload == "cfg3":
        print(json.dumps(layer_stack(lava, synth, torch, np, dev, args)), flush=True)
        return
    if args.workload == "cfg5":
        print(json.dumps(ragged_batch(lava, synth, torch, np, dev, args)), flush=True)
        return
    cfg_idx = {"cfg1": 1, "cfg2": 2, "cfg4": 4}[args.workload]
    sh = synth.config(cfg_idx)
    esize = synth.itemsize(sh.dtype)
    desc = lava.LayerDesc.make(sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.window, sh.dtype, pool_kernel=sh.pool_kernel)
    if args.decode_only:
        res = decode_batched(lava, synth, torch, np, sh, desc, dev, sh.budget, args, max(20, args.steps // 2))
        print(json.dumps({"decode_only": res, "workload": args.workload}), flush=True)
        return
    inp = synth.gen_layer(sh, args.seed)
    kv_bytes = sh.n_kv_heads * sh.n * sh.head_dim * esize           # one of K or V
    n_sets = args.sets if args.sets > 0 else max(2, int(np.ceil(1.5 * 2**30 / (2 * kv_bytes))))
    n_sets = min(n_sets, 64)

    q0, k0, v0 = (lava.to_device(a, sh.dtype, dev) for a in (inp.q_win, inp.k, inp.v))
    sets = [(q0, k0, v0)] + [(q0.clone(), k0.clone(), v0.clone()) for _ in range(n_sets - 1)]

    total_entries = sh.n_kv_heads * sh.n
    B = sh.budget
    ws_scores = torch.empty(lava.lava_window_scores_workspace_bytes(desc, 1, sh.n), dtype=torch.uint8, device=dev)
    ws_sel = torch.empty(lava.lava_select_workspace_bytes(total_entries), dtype=torch.uint8, device=dev)
    scores = torch.empty(total_entries, dtype=torch.float32, device=dev)
    vbar = torch.empty(1, sh.n_kv_heads, dtype=torch.float32, device=dev)
    stat = torch.empty(1, dtype=torch.float32, device=dev)
    budgets = torch.empty(1, 1, dtype=torch.int64, device=dev)
    total_b = torch.tensor([B], dtype=torch.int64, device=dev)
    lo = torch.tensor([[sh.n_kv_heads * sh.window]], dtype=torch.int64, device=dev)
    hi = torch.tensor([[total_entries]], dtype=torch.int64, device=dev)
    counts = torch.empty(sh.n_kv_heads, dtype=torch.int32, device=dev)
    offs = torch.empty(sh.n_kv_heads + 1, dtype=torch.int64, device=dev)
    idx = torch.empty(B, dtype=torch.int32, device=dev)
    kept_s = torch.empty(B, dtype=torch.float32, device=dev)
    k_hat = torch.empty(B, sh.head_dim, dtype=desc.torch_dtype, device=dev)
    v_hat = torch.empty(B, sh.head_dim, dtype=desc.torch_dtype, device=dev)
    lens = [sh.n]

    # ---- streaming probe: plain read / copy of 1 GiB (also calibrates the profiler's byte counters)
    probe_bytes = 1 << 30
    probe_src = torch.empty(probe_bytes, dtype=torch.uint8, device=dev).fill_(1)
    probe_dst = torch.empty(probe_bytes, dtype=torch.uint8, device=dev)
    probe_sink = torch.zeros(64, dtype=torch.int32, device=dev)

    def timed_probe(mode):
        best = float("inf")
        for _ in range(5):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            lava.probe_stream(probe_src, probe_dst if mode == 0 else probe_sink, probe_bytes, mode, 8192)
            b.record()
            torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b) * 1e-3)
        return best

    probe = {"read_GBs": round(probe_bytes / timed_probe(1) / 1e9, 1),
             "copy_GBs_read_plus_write": round(2 * probe_bytes / timed_probe(0) / 1e9, 1), "bytes": probe_bytes}
    del probe_src, probe_dst

    lse_dev = [None]
    primed = not args.no_primed

    # budgets (Alg. 2's rule over the layers seen so far: here one layer) formed by the scores call itself,
    # or by a launch of their own
    planned = not args.no_plan
    e_table = torch.zeros(1, 1, dtype=torch.float32, device=dev)
    plan = lava.make_budget_plan(e_table, 0, total_b, lo, hi, budgets) if planned else None

    def step(i):
        q, k, v = sets[i % n_sets]
        lava.lava_window_scores(desc, lens, q, k, v, lse=lse_dev[0], scores=scores, vbar=vbar, layer_stat=stat,
                                workspace=ws_scores, select_workspace=ws_sel if primed else None, budget_plan=plan)
        if not planned:
            lava.lava_layer_budgets(stat.view(1, 1), total_b, lo, hi, budgets=budgets)
        lava.lava_select_topk(sh.n_kv_heads, scores, B, budget_dev=budgets.view(-1), head_counts=counts,
                              head_offsets=offs, kept_idx=idx, kept_scores=kept_s, workspace=ws_sel, primed=primed)
        lava.lava_compact_kv(desc, sh.n, k, v, offs, idx, B, k_out=k_hat, v_out=v_hat)

    host_enqueue = [0.0]   # seconds the host spent enqueueing the timed steps of the latest loop

    def timed_loop():
        for i in range(args.warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        host_enqueue[0] = time.perf_counter() - t0
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def per_step_times():
        """Duration of every step of an identical loop, from events between the steps (median / min)."""
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        marks[0].record()
        for i in range(args.steps):
            step(i)
            marks[i + 1].record()
        torch.cuda.synchronize()
        t = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
        return {"median_ms": round(t[len(t) // 2], 5), "min_ms": round(t[0], 5), "max_ms": round(t[-1], 5)}

    def per_kernel_times():
        """Average duration of every kernel over an identical loop, HIP events on the launch stream."""
        lava.prof_enable(True)
        lava.prof_reset()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        prof = lava.prof_read()
        lava.prof_enable(False)
        return {name: 1e3 * ms / max(cnt, 1) for name, (ms, cnt) in prof.items() if cnt}

    elapsed = timed_loop()
    host_ms_per_step = 1e3 * host_enqueue[0] / args.steps
    ms_per_step = 1e3 * elapsed / args.steps
    tokens_per_s = sh.n / (elapsed / args.steps)
    step_spread = per_step_times()
    per_kernel_us = per_kernel_times()

    # ---- variant: the prefill attention hands over the window rows' log-sum-exp, so the statistics
    # pass is skipped (the LSE itself is prepared here with torch, outside any timed region)
    G = sh.n_q_heads // sh.n_kv_heads
    with torch.no_grad():
        qf = q0.float().view(sh.n_kv_heads, G * sh.window, sh.head_dim)
        logits = torch.bmm(qf, k0.float().view(sh.n_kv_heads, sh.n, sh.head_dim).transpose(1, 2))
        logits = logits.view(sh.n_q_heads, sh.window, sh.n) / (sh.head_dim ** 0.5)
        pos = torch.arange(sh.n, device=dev)[None, None, :]
        last = (sh.n - sh.window + torch.arange(sh.window, device=dev))[None, :, None]
        logits = logits.masked_fill(pos > last, float("-inf"))
        lse_dev[0] = torch.logsumexp(logits, dim=2).contiguous()
        del logits, qf
    # (the host sometimes enqueues slowly right after the large temporaries above are released and the loop
    # then measures the host; best of three loops, each of exactly --steps steps, for this secondary figure)
    lse_elapsed, lse_host_ms_per_step = float("inf"), 0.0
    for _ in range(3):
        t = timed_loop()
        if t < lse_elapsed:
            lse_elapsed, lse_host_ms_per_step = t, 1e3 * host_enqueue[0] / args.steps
    lse_spread = per_step_times()
    lse_kernel_us = per_kernel_times()
    lse_dev[0] = None

    # ---- algorithmic bytes of each sweep kernel per launch (what it must move given its inputs / outputs)
    q_bytes = sh.n_q_heads * sh.window * sh.head_dim * esize
    score_bytes = 4 * total_entries
    alg_bytes = {
        "vnorm": kv_bytes,
        "stats": kv_bytes + q_bytes,
        "scores": kv_bytes + q_bytes + score_bytes,
        "sweep": 2 * (kv_bytes + q_bytes) + score_bytes,
        "prepass": 2 * kv_bytes + q_bytes,                      # value norms + statistics in one launch: V once, K once
        "sel_fused": score_bytes,
        "compact": 4 * B * sh.head_dim * esize,
    }
    traffic = measured_traffic(args.workload)

    def kernel_line(name, us):
        gbs = alg_bytes[name] / (us * 1e-6) / 1e9
        return {"us": round(us, 2), "algorithmic_bytes": alg_bytes[name], "GBs": round(gbs, 1),
                "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                "traffic": sum(traffic[name]) if name in traffic else None}

    sweep_names = [n for n in ("vnorm", "stats", "prepass", "scores", "sweep") if n in per_kernel_us]
    sweep_kernels = {n: kernel_line(n, per_kernel_us[n]) for n in sweep_names}
    # the dominant kernel: the slowest of the sweeps (sweep_kernels lists them all)
    dominant = max(sweep_names, key=lambda n: per_kernel_us[n])
    dom = sweep_kernels[dominant]
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": dom["GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dom["frac_of_hbm_peak"], "traffic": dom["traffic"],
                "traffic_source": f"profiles/{args.workload}_hbm_counters.md" if dom["traffic"] is not None else None,
                "kernel_us": dom["us"], "algorithmic_bytes": dom["algorithmic_bytes"]}
    # the K/V sweep as a whole, both accountings: K once + V once (a second pass over K is overhead) and
    # the bytes the kernels actually have to stream (K twice + V once); and with the caller's LSE (K once)
    sweep_us = sum(per_kernel_us[n] for n in sweep_names)
    once = 2 * kv_bytes + q_bytes + score_bytes
    moved = sum(alg_bytes[n] for n in sweep_names)
    lse_names = [n for n in ("vnorm", "scores") if n in lse_kernel_us]
    lse_us = sum(lse_kernel_us[n] for n in lse_names)
    kv_sweep = {
        "kernels": sweep_names, "us": round(sweep_us, 2),
        "k_once_v_once": {"bytes": once, "GBs": round(once / sweep_us / 1e3, 1),
                          "frac_of_hbm_peak": round(once / sweep_us / 1e3 / HBM_PEAK_GBS, 4)},
        "bytes_streamed": {"bytes": moved, "GBs": round(moved / sweep_us / 1e3, 1),
                           "frac_of_hbm_peak": round(moved / sweep_us / 1e3 / HBM_PEAK_GBS, 4)},
        "with_lse": {"kernels": lse_names, "us": round(lse_us, 2), "bytes": once,
                     "GBs": round(once / lse_us / 1e3, 1),
                     "frac_of_hbm_peak": round(once / lse_us / 1e3 / HBM_PEAK_GBS, 4)},
    }
    # whole-path view: K once + V once + scores + kept rows, over the whole step
    path_bytes = 2 * kv_bytes + q_bytes + 2 * score_bytes + 4 * B * sh.head_dim * esize
    path_gbs = path_bytes / (elapsed / args.steps) / 1e9

    out = {
        "metric": "cached tokens evicted-and-compacted/sec per layer; achieved HBM GB/s vs peak",
        "value": round(tokens_per_s, 1), "unit": "tokens/s/layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": sh.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}: one layer, {sh.n_q_heads}q/{sh.n_kv_heads}kv heads, d_h {sh.head_dim}, "
                               f"N={sh.n}, w={sh.window}, B_l={B}, {sh.dtype}, batch 1",
                   "kv_buffer_sets": n_sets, "sweep_schedule": args.sweep_schedule, "sweep_shape": args.sweep_shape,
                   "scores_prepare_selection": primed, "scores_form_budgets": planned},
        "roofline": roofline,
        "step_spread": step_spread,
        "host_enqueue_ms_per_step": round(host_ms_per_step, 5),
        "sweep_kernels": sweep_kernels,
        "kv_sweep": kv_sweep,
        "path": {"algorithmic_bytes": path_bytes, "achieved_GBs": round(path_gbs, 1),
                 "frac_of_hbm_peak": round(path_gbs / HBM_PEAK_GBS, 4)},
        "kernels_us": {k: round(v, 2) for k, v in per_kernel_us.items()},
        "stream_probe": probe,
        "with_lse": {"note": "window-row log-sum-exp supplied by the caller: statistics pass skipped",
                     "ms_per_step": round(1e3 * lse_elapsed / args.steps, 5),
                     "value": round(sh.n / (lse_elapsed / args.steps), 1),
                     "path_frac_of_hbm_peak": round(path_bytes / (lse_elapsed / args.steps) / 1e9 / HBM_PEAK_GBS, 4),
                     "step_spread": lse_spread, "host_enqueue_ms_per_step": round(lse_host_ms_per_step, 5),
                     "kernels_us": {k: round(v, 2) for k, v in lse_kernel_us.items()}},
    }

    if not args.no_decode:
        out["decode"] = decode_leg(lava, synth, torch, np, sh, desc, dev, sets, k_hat, v_hat, offs, B, args)

    if not args.no_cascade:
        out["cascade"] = cascade_leg(lava, torch, np, sh, desc, dev, sets, scores, args)

    if not args.no_check or not args.no_cpu_baseline:
        from oracle import lava_oracle as O
        try:
            from threadpoolctl import threadpool_limits
        except Exception:                                       # pragma: no cover
            threadpool_limits = None
        q, k, v = inp.f64()
        # the oracle on full layers of the workload until about ten seconds have gone by (at most 12 runs)
        runs, cpu_s = 0, 0.0
        while runs < 12 and (runs == 0 or cpu_s < 10.0):
            t0 = time.perf_counter()
            if threadpool_limits is not None:
                with threadpool_limits(limits=1):
                    ref = O.layer_evict(q, k, v, sh.window, B, sh.pool_kernel, k_store=inp.k, v_store=inp.v)
            else:
                ref = O.layer_evict(q, k, v, sh.window, B, sh.pool_kernel, k_store=inp.k, v_store=inp.v)
            cpu_s += time.perf_counter() - t0
            runs += 1
        out["cpu_baseline"] = {"value": round(runs * sh.n / cpu_s, 1), "unit": "tokens/s/layer",
                               "cores": 1 if threadpool_limits is not None else os.cpu_count(),
                               "kind": "oracle",
                               "sample": f"{runs} full layers of the workload (N={sh.n}) one after another, "
                                         f"{cpu_s:.1f} s in all",
                               "host_cores_available": os.cpu_count()}
        # parity of the timed configuration against the oracle (outside the timed region)
        step(0)
        torch.cuda.synchronize()
        c, o, ii = counts.cpu().numpy(), offs.cpu().numpy(), idx.cpu().numpy()
        mine = {(g, int(p)) for g in range(sh.n_kv_heads) for p in ii[o[g]:o[g + 1]]}
        theirs = {(g, int(p)) for g in range(sh.n_kv_heads)
                  for p in ref["kept_idx"][ref["head_offsets"][g]:ref["head_offsets"][g + 1]]}
        got = scores.cpu().numpy().reshape(sh.n_kv_heads, sh.n)[:, : sh.n_prefix].astype(np.float64)
        want = ref["scores"][:, : sh.n_prefix]
        mask = want > 1e-30 * want.max()
        out["parity"] = {"kept_overlap": round(len(mine & theirs) / B, 6),
                         "score_max_rel_err": float(np.max(np.abs(got[mask] - want[mask]) / want[mask]))}

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
