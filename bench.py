#!/usr/bin/env python3
"""Benchmark of the KeyDiff block-prefill step on one MI355X.

One bench *step* = one steady-state block step (cache full at N, B new tokens:
append, attention, anchor, score, select, compact) through every layer of the
workload, each layer on its own cache with its own seeded data.  The metric is
prompt tokens/s per layer: B / (time of one layer's block step).

Prints ONE JSON line (see the keys below) and nothing else on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from synth import get_config, make_layer  # noqa: E402

PEAK_BF16_MFMA_TFLOPS = 2500.0   # dense bf16, MI355X
PEAK_HBM_GBPS = 8000.0
CALIBRATION_COPY_BYTES = 256 << 20


def measured_traffic(workload: str, layout: str):
    """HBM bytes per step_main launch from the committed counter summary of this workload, or None.

    The figure comes from two rocprofv3 --pmc runs of this script (FETCH_SIZE, WRITE_SIZE), each
    scaled by the same counter's reading for the calibration copy; it cannot be measured from
    inside the process."""
    import re
    path = os.path.join(ROOT, "profiles", f"step_main_{workload}_{layout}_hbm_traffic.txt")
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def to_blocks(bits: np.ndarray, B: int):
    """token-major [T][H][d] uint16 -> torch bf16 [T/B][1][H][B][d] on the GPU."""
    import torch
    T, H, d = bits.shape
    t = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return t.view(T // B, B, H, d).permute(0, 2, 1, 3).contiguous().unsqueeze(1)


def bench_decode(args, w):
    """The generation phase (block size 1): a batch of sequences, caches at the budget, one token and
    one eviction per sequence, KV head and step.  HBM-bound: K and V cross it once per step."""
    import torch

    import paper_2504_15364_amd as kd
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    N, D, Hq, Hkv, batch = w.budget_N, w.head_dim, w.n_q_heads, w.n_kv_heads, w.batch
    n_steps = args.warmup + args.steps + args.profile_steps + (0 if args.no_cpu_baseline else args.cpu_steps)
    t0 = time.time()
    with ThreadPoolExecutor(min(16, os.cpu_count() or 1)) as ex:
        seqs = list(ex.map(lambda s_: make_layer(w, seed=args.seed + 1000 * 5, seq=s_, t1=N + n_steps), range(batch)))
    log(f"[bench] generated {batch} sequences x {N + n_steps} tokens in {time.time() - t0:.1f}s")

    def dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)

    def token(t):   # [batch][heads][1][d] bit patterns of token t of every sequence
        return tuple(np.stack([s_[x][t][:, None, :] for s_ in seqs]) for x in ("q", "k", "v"))

    cache = kd.KeyDiffCache(kd.KeyDiffConfig(batch, Hq, Hkv, D, N, 1, layout=kd.LAYOUT_FILL))
    K0 = np.stack([s_["k"][:N].transpose(1, 0, 2) for s_ in seqs])
    V0 = np.stack([s_["v"][:N].transpose(1, 0, 2) for s_ in seqs])
    P0 = np.broadcast_to(np.arange(N, dtype=np.int32), (batch, Hkv, N)).copy()
    cache.load(dev(K0), dev(V0), torch.from_numpy(P0).cuda())
    toks = [tuple(dev(x) for x in token(N + i)) for i in range(args.warmup + args.steps + args.profile_steps)]
    out = torch.empty((batch, Hq, 1, D), dtype=torch.bfloat16, device="cuda")
    i = 0
    for _ in range(args.warmup):
        cache.decode_step(*toks[i], N + i, out=out)
        i += 1
    if args.pmc_calibration:
        src = torch.empty(CALIBRATION_COPY_BYTES, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads and writes CALIBRATION_COPY_BYTES each
        del src, dst
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        cache.decode_step(*toks[i], N + i, out=out)
        i += 1
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    us_step = elapsed / args.steps * 1e6

    kernels = {}
    if args.profile_steps > 0:
        cache.profile_enable(True)
        for _ in range(args.profile_steps):
            cache.decode_step(*toks[i], N + i, out=out)
            i += 1
        torch.cuda.synchronize()
        tot = {k: list(v) for k, v in cache.profile_read().items()}
        cache.profile_enable(False)
        pair = tot.pop("event_pair", [0.0, 0])
        pair_us = pair[0] / pair[1] * 1e3 if pair[1] else 0.0
        bracket_sum_us = sum(v[0] for v in tot.values()) * 1e3 / args.profile_steps
        launches = sum(v[1] for v in tot.values()) / args.profile_steps
        overhead_us = min(pair_us, max(0.0, (bracket_sum_us - us_step) / launches))   # see the prefill path
        kernels = {k: {"avg_us": v[0] / v[1] * 1e3 - overhead_us, "launches": v[1],
                       "event_bracket_us": v[0] / v[1] * 1e3, "event_overhead_us": overhead_us,
                       "empty_event_pair_us": pair_us} for k, v in tot.items() if v[1]}
    assert cache.status() == 0

    n = N + 1
    kv_bytes = 2.0 * batch * Hkv * n * D * 2                       # K and V once
    bytes_step = kv_bytes + 2 * batch * Hq * D * 2 + batch * Hkv * n * 4 + 4 * batch * Hkv * D * 2
    roofline = None
    if "step_main" in kernels:
        t_main = kernels["step_main"]["avg_us"] * 1e-6
        achieved = kv_bytes / t_main / 1e9
        roofline = {"bound": "hbm", "kernel": "step_main_kernel (helper waves, alternating tiles)", "achieved": achieved,
                    "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBPS,
                    "traffic": measured_traffic(w.name, "fill"), "bytes_per_launch": kv_bytes,
                    "avg_launch_us": kernels["step_main"]["avg_us"]}
    t_min = bytes_step / (PEAK_HBM_GBPS * 1e9)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        from synth import bf16_bits_to_f32
        oc = oracle.OracleCache(batch, Hq, Hkv, D, N, 1)
        oc.load(K0, V0, P0)
        ref = kd.KeyDiffCache(kd.KeyDiffConfig(batch, Hq, Hkv, D, N, 1, layout=kd.LAYOUT_FILL))
        ref.load(dev(K0), dev(V0), torch.from_numpy(P0).cuda())
        tc, worst = 0.0, 0.0
        for s_ in range(args.cpu_steps):
            q, k, v = token(N + s_)
            t1 = time.perf_counter()
            o_ref, _, _ = oc.decode_step(q, k, v, N + s_)
            tc += time.perf_counter() - t1
            got = ref.decode_step(dev(q), dev(k), dev(v), N + s_)
            worst = max(worst, float(np.abs(bf16_bits_to_f32(got.view(torch.int16).cpu().numpy().view(np.uint16)) - o_ref).max()))
            assert np.array_equal(np.sort(ref.positions().cpu().numpy(), axis=-1), oc.positions()), "retained set differs"
        cpu = {"value": batch * args.cpu_steps / tc, "unit": "tokens/s/layer",
               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "kind": "oracle",
               "sample": f"{args.cpu_steps} decode steps of the {batch} sequences (fp64, OpenMP over heads x rows)",
               "us_per_step": tc / args.cpu_steps * 1e6, "max_abs_attention_diff_vs_gpu": worst,
               "retained_sets_identical": True}

    print(json.dumps({
        "metric": f"generated tokens/sec per layer (KeyDiff decode step, batch {batch}) at N={N}",
        "value": batch / (us_step * 1e-6), "unit": "tokens/s/layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": us_step * 1e-3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D, "budget_N": N,
                   "block_B": 1, "batch": batch, "layers": 1, "layout": "fill", "tokens_per_step": batch,
                   "step": "one decode step of every sequence of the batch on one layer"},
        "us_per_layer_step": us_step,
        "step_roofline": {"binding": "hbm", "t_min_us": t_min * 1e6, "frac": t_min / (us_step * 1e-6),
                          "bytes": bytes_step},
        "roofline": roofline, "kernels": kernels, "cpu_baseline": cpu,
    }))


def decode_record(args, steps=24, warmup=6):
    """A short run of the generation phase (decode_8b: batch 16, N = 8192, B = 1) for the default line."""
    import torch

    import paper_2504_15364_amd as kd
    w = get_config("decode_8b")
    N, D, Hq, Hkv, batch = w.budget_N, w.head_dim, w.n_q_heads, w.n_kv_heads, w.batch
    total = warmup + steps + 8
    with ThreadPoolExecutor(min(16, os.cpu_count() or 1)) as ex:
        seqs = list(ex.map(lambda s_: make_layer(w, seed=args.seed + 1000 * 5, seq=s_, t1=N + total), range(batch)))

    def dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)
    cache = kd.KeyDiffCache(kd.KeyDiffConfig(batch, Hq, Hkv, D, N, 1, layout=kd.LAYOUT_FILL))
    K0 = np.stack([s_["k"][:N].transpose(1, 0, 2) for s_ in seqs])
    V0 = np.stack([s_["v"][:N].transpose(1, 0, 2) for s_ in seqs])
    P0 = np.broadcast_to(np.arange(N, dtype=np.int32), (batch, Hkv, N)).copy()
    cache.load(dev(K0), dev(V0), torch.from_numpy(P0).cuda())
    toks = [tuple(dev(np.stack([s_[x][N + i][:, None, :] for s_ in seqs])) for x in ("q", "k", "v")) for i in range(total)]
    out = torch.empty((batch, Hq, 1, D), dtype=torch.bfloat16, device="cuda")
    i = 0
    for _ in range(warmup):
        cache.decode_step(*toks[i], N + i, out=out)
        i += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        cache.decode_step(*toks[i], N + i, out=out)
        i += 1
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / steps * 1e6
    cache.profile_enable(True)
    for _ in range(8):
        cache.decode_step(*toks[i], N + i, out=out)
        i += 1
    torch.cuda.synchronize()
    prof = {k: v[0] / v[1] * 1e3 for k, v in cache.profile_read().items() if v[1] and k != "event_pair"}
    assert cache.status() == 0
    cache.close()
    kv_bytes = 2.0 * batch * Hkv * (N + 1) * D * 2
    t_min_us = (kv_bytes + 2 * batch * Hq * D * 2 + batch * Hkv * (N + 1) * 4) / (PEAK_HBM_GBPS * 1e9) * 1e6
    return {"workload": "decode_8b", "batch": batch, "budget_N": N, "steps": steps, "us_per_step": us,
            "tokens_per_s_per_layer": batch / (us * 1e-6), "kv_bytes_per_step": kv_bytes,
            "step_GBps": kv_bytes / us / 1e3, "frac_of_hbm_roofline": t_min_us / us,
            "event_bracket_us": prof}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=48)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="llama31_8b")
    ap.add_argument("--layers", type=int, default=0, help="0 = the workload's layer count")
    ap.add_argument("--budget", type=int, default=0,
                    help="cache budget N (a multiple of the block size); 0 = the workload's (the paper's budgets: 2K-8K)")
    ap.add_argument("--layout", choices=["fill", "ordered"], default="fill")
    ap.add_argument("--eviction", choices=["deferred", "immediate"], default="deferred",
                    help="deferred: the selection and compaction of layer l runs inside the attention launch "
                         "of layer l + 1 (keydiff_prefill_block_deferred); immediate: inside layer l's own step")
    ap.add_argument("--profile-steps", type=int, default=8, help="extra steps timed per kernel with HIP events")
    ap.add_argument("--seed", type=int, default=20250415)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=4)
    ap.add_argument("--no-whole-prompt", action="store_true",
                    help="skip the whole-prompt run (every block of the prompt through every layer from empty "
                         "caches: the fill steps and every evicting step)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the secondary measurements (the other eviction mode and row layout, the keydiff_scores "
                         "pass, the decode step): with it, and --no-whole-prompt, every launch of the process is a "
                         "steady-state block step of the headline mode -- what the rocprofv3 summaries are taken from")
    ap.add_argument("--mode-steps", type=int, default=12, help="timed steps of each secondary mode")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also launch plain device copies of a known size (untimed), so that a rocprofv3 "
                         "--pmc run of this command holds the counter's reading for a known byte count")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    w = get_config(args.workload)
    if args.budget:
        if args.budget % w.block_B or args.budget < w.block_B:
            sys.exit(f"--budget must be a positive multiple of the block size {w.block_B}")
        w = w.small(budget_N=args.budget, prompt_T=max(w.prompt_T, 4 * args.budget))
    if w.block_B == 1:
        return bench_decode(args, w)
    L = args.layers or w.n_layers
    B, N, D, Hq, Hkv = w.block_B, w.budget_N, w.head_dim, w.n_q_heads, w.n_kv_heads
    fill_blocks = N // B
    n_steps = args.warmup + args.steps + args.profile_steps
    T_need = (fill_blocks + max(n_steps, 0 if args.no_extras else 7 + args.mode_steps)) * B
    if T_need > w.prompt_T:
        sys.exit(f"--warmup + --steps + --profile-steps = {n_steps} exceeds the {w.prompt_T // B - fill_blocks} "
                 f"evicting steps of a {w.prompt_T}-token prompt")

    # ---- seeded host data, one fresh seed per layer (threads: numpy releases the GIL)
    t0 = time.time()
    workers = min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(workers) as ex:
        layers = list(ex.map(lambda l: make_layer(w, seed=args.seed + 100 * 3 + l, layer=l, t1=T_need), range(L)))
    log(f"[bench] generated {L} layers x {T_need} tokens in {time.time() - t0:.1f}s")

    import torch

    import paper_2504_15364_amd as kd
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    layout = kd.LAYOUT_FILL if args.layout == "fill" else kd.LAYOUT_ORDERED
    caches, dq, dk, dv, outs = [], [], [], [], []
    for l in range(L):
        caches.append(kd.KeyDiffCache(kd.KeyDiffConfig(w.batch, Hq, Hkv, D, N, B, layout=layout)))
        dq.append(to_blocks(layers[l]["q"], B))
        dk.append(to_blocks(layers[l]["k"], B))
        dv.append(to_blocks(layers[l]["v"], B))
        outs.append(torch.empty_like(dq[l][0]))

    deferred = args.eviction == "deferred" and L > 1

    def run_block(i):
        if deferred:   # one call: layer l takes along the eviction layer l - 1 left pending (layer 0: the last layer's)
            kd.prefill_block_layers(caches, [t[i] for t in dq], [t[i] for t in dk], [t[i] for t in dv], i * B, out=outs)
            return
        for l in range(L):
            caches[l].prefill_block(dq[l][i], dk[l][i], dv[l][i], i * B, out=outs[l])

    def finish_all():   # the one eviction still pending belongs to the timed work
        if deferred:
            caches[L - 1].finish()

    def load_first_N(cache, l):
        # while n <= N nothing is evicted, so after the first N tokens the cache IS those tokens in
        # order: load that state directly, so every attention launch of this process is a
        # steady-state one (the rocprofv3 average and the live HIP-event average then cover the
        # same launches)
        k0 = dk[l][:fill_blocks, 0].permute(1, 0, 2, 3).reshape(1, Hkv, N, D).contiguous()
        v0 = dv[l][:fill_blocks, 0].permute(1, 0, 2, 3).reshape(1, Hkv, N, D).contiguous()
        p0 = torch.arange(N, dtype=torch.int32, device="cuda").repeat(1, Hkv, 1).contiguous()
        cache.load(k0, v0, p0)

    # ---- untimed: bring every cache to the budget, then warm up in steady state
    for l in range(L):
        load_first_N(caches[l], l)
    torch.cuda.synchronize()
    assert all(c.len == N for c in caches)
    i = fill_blocks
    for _ in range(args.warmup):
        run_block(i)
        i += 1
    finish_all()
    if args.pmc_calibration:
        src = torch.empty(CALIBRATION_COPY_BYTES, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads and writes CALIBRATION_COPY_BYTES each
        del src, dst
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for _ in range(args.steps):
        run_block(i)
        i += 1
    finish_all()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed / args.steps * 1e3
    us_per_layer_step = elapsed / (args.steps * L) * 1e6
    tokens_per_s_per_layer = B / (elapsed / (args.steps * L))

    # ---- per-kernel durations, HIP events recorded by the library on its launch stream
    kernels = {}
    if args.profile_steps > 0:
        for c in caches:
            c.profile_enable(True)
        for _ in range(args.profile_steps):
            run_block(i)
            i += 1
        finish_all()
        torch.cuda.synchronize()
        tot = {}
        for c in caches:
            for name, (ms, cnt) in c.profile_read().items():
                a = tot.setdefault(name, [0.0, 0])
                a[0] += ms
                a[1] += cnt
            c.profile_enable(False)
        # What the two event records of a bracket add to it is not known a priori.  An event pair with
        # nothing between it (the library records one per profiled step) is an upper bound: two
        # back-to-back records serialise, while next to a kernel most of their processing hides
        # behind it -- taking the whole pair off makes the kernels shorter than rocprofv3 sees them
        # and leaves gaps between them that its trace does not show.  The brackets of a step's
        # launches, back to back on one stream, must add up to the step's wall-clock time measured
        # above without any event: the excess, split evenly over the launches, is the overhead
        # taken off (never more than the empty pair).
        pair = tot.pop("event_pair", [0.0, 0])
        pair_us = pair[0] / pair[1] * 1e3 if pair[1] else 0.0
        layer_steps = args.profile_steps * L
        bracket_sum_us = sum(v[0] for v in tot.values()) * 1e3 / layer_steps    # per layer-step
        launches_per_layer_step = sum(v[1] for v in tot.values()) / layer_steps
        overhead_us = min(pair_us, max(0.0, (bracket_sum_us - us_per_layer_step) / launches_per_layer_step))
        kernels = {k: {"avg_us": v[0] / v[1] * 1e3 - overhead_us, "launches": v[1],
                       "event_bracket_us": v[0] / v[1] * 1e3, "event_overhead_us": overhead_us,
                       "empty_event_pair_us": pair_us}
                   for k, v in tot.items() if v[1]}
    assert all(c.status() == 0 for c in caches)

    # ---- secondary: the same steady-state steps with the eviction inside the step (keydiff_prefill_block,
    # two launches per layer) and in the stable row layout, on fresh caches with the same data; the
    # keydiff_scores pass over a full cache
    plan = caches[0].plan()
    modes, scores_pass, ordered_kernels = None, None, None
    if not args.no_extras:
        first = fill_blocks + args.warmup
        def run_mode(lay, defer):
            cs = [kd.KeyDiffCache(kd.KeyDiffConfig(w.batch, Hq, Hkv, D, N, B, layout=lay)) for _ in range(L)]
            for l in range(L):
                load_first_N(cs[l], l)
            def blk(i):
                if defer and L > 1:
                    kd.prefill_block_layers(cs, [t[i] for t in dq], [t[i] for t in dk], [t[i] for t in dv], i * B, out=outs)
                else:
                    for l in range(L):
                        cs[l].prefill_block(dq[l][i], dk[l][i], dv[l][i], i * B, out=outs[l])
            for i in range(fill_blocks, fill_blocks + 3):
                blk(i)
            cs[L - 1].finish()
            torch.cuda.synchronize()
            t0_ = time.perf_counter()
            for i in range(fill_blocks + 3, fill_blocks + 3 + args.mode_steps):
                blk(i)
            cs[L - 1].finish()
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0_) / (args.mode_steps * L) * 1e6
            prof = None
            if lay == kd.LAYOUT_ORDERED and not defer:  # per-kernel times of the stable layout (HIP events; deferred, the shift rides in the merge launch)
                for c in cs:
                    c.profile_enable(True)
                for i in range(fill_blocks + 3 + args.mode_steps, fill_blocks + 7 + args.mode_steps):
                    blk(i)
                cs[L - 1].finish()
                torch.cuda.synchronize()
                tot = {}
                for c in cs:
                    for name, (ms, cnt) in c.profile_read().items():
                        a = tot.setdefault(name, [0.0, 0])
                        a[0] += ms
                        a[1] += cnt
                pair = tot.pop("event_pair", [0.0, 0])
                prof = {k: {"event_bracket_us": v[0] / v[1] * 1e3, "launches": v[1]} for k, v in tot.items() if v[1]}
            assert all(c.status() == 0 for c in cs)
            for c in cs:
                c.close()
            return us, prof
        modes = {"deferred_fill": us_per_layer_step if deferred and args.layout == "fill" else None}
        for key, lay, defer in (("deferred_fill", kd.LAYOUT_FILL, True), ("immediate_fill", kd.LAYOUT_FILL, False),
                                ("deferred_ordered", kd.LAYOUT_ORDERED, True), ("immediate_ordered", kd.LAYOUT_ORDERED, False)):
            if modes.get(key) is None:
                modes[key], prof = run_mode(lay, defer)
                if prof is not None:
                    ordered_kernels = prof
        modes = {k: {"us_per_layer_step": v, "tokens_per_s_per_layer": B / (v * 1e-6),
                     "frac_of_step_roofline": None} for k, v in modes.items()}
        # keydiff_scores on the caches of all layers in turn, back to back (each cache is at the budget:
        # N rows of d bf16 per head in, a float per row out; 32 caches of 17 MB each, so the keys of a
        # launch come from HBM, not from a cache that still holds them)
        for c in caches:
            c.scores()
        torch.cuda.synchronize()
        reps = 4
        sc_out = torch.empty((w.batch, Hkv, N), dtype=torch.float32, device="cuda")
        lib, stream_ptr = kd.load_library(), torch.cuda.current_stream().cuda_stream
        calls = [(c._h, sc_out.data_ptr(), stream_ptr) for c in caches] * reps   # the bare C calls: the host must keep ahead
        t0_ = time.perf_counter()
        for a in calls:
            lib.keydiff_scores(*a)
        torch.cuda.synchronize()
        sc_us = (time.perf_counter() - t0_) / (reps * L) * 1e6
        sc_bytes = w.batch * Hkv * N * (D * 2 + 4)
        scores_pass = {"kernel": "step_score_kernel", "bytes": sc_bytes, "us": sc_us,
                       "GBps": sc_bytes / (sc_us * 1e-6) / 1e9, "frac_of_hbm_peak": sc_bytes / (sc_us * 1e-6) / 1e9 / PEAK_HBM_GBPS,
                       "note": f"wall clock over {reps * L} back-to-back launches on {L} different caches (launch gaps included)"}

    # algorithmic work of one steady-state block step of one layer
    n = N + B
    flops_attn = 4.0 * Hq * B * D * (N + B / 2.0)
    bytes_step = (2 * Hkv * n * D * 2 + 2 * Hq * B * D * 2 + 2 * Hkv * B * D * 2 + Hkv * n * 4
                  + 2 * 2 * Hkv * B * D * 2)        # K+V once, Q in/O out, new rows, scores, <= B moved rows r+w
    roofline = None
    if "step_main" in kernels:
        t_attn = kernels["step_main"]["avg_us"] * 1e-6
        achieved = flops_attn / t_attn / 1e12
        # with deferred eviction nearly every launch of the class is the carrying variant of the kernel
        roofline = {"bound": "mfma", "kernel": "step_main_carry_kernel" if deferred else "step_main_kernel",
                    "achieved": achieved,
                    "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_MFMA_TFLOPS,
                    "traffic": measured_traffic(w.name, args.layout), "flops_per_launch": flops_attn,
                    "avg_launch_us": kernels["step_main"]["avg_us"]}
    t_min = max(flops_attn / (PEAK_BF16_MFMA_TFLOPS * 1e12), bytes_step / (PEAK_HBM_GBPS * 1e9))
    step_frac = t_min / (us_per_layer_step * 1e-6)

    # ---- the oracle on the host cores, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        from synth import bf16_bits_to_f32, block_of
        data = layers[0]
        oc = oracle.OracleCache(1, Hq, Hkv, D, N, B)
        for b in range(fill_blocks):          # reach the steady state without attention (keys decide the trace)
            oc.prefill_block(None, block_of(data["k"], b * B, B)[None], block_of(data["v"], b * B, B)[None], b * B)
        tc, worst = 0.0, 0.0
        ref_cache = kd.KeyDiffCache(kd.KeyDiffConfig(w.batch, Hq, Hkv, D, N, B, layout=layout))
        load_first_N(ref_cache, 0)
        for s in range(args.cpu_steps):
            b = fill_blocks + s
            q, k, v = (block_of(data[x], b * B, B)[None] for x in ("q", "k", "v"))
            t1 = time.perf_counter()
            ref, _, _ = oc.prefill_block(q, k, v, b * B)
            tc += time.perf_counter() - t1
            got = ref_cache.prefill_block(dq[0][b], dk[0][b], dv[0][b], b * B)
            got = bf16_bits_to_f32(got.view(torch.int16).cpu().numpy().view(np.uint16))
            worst = max(worst, float(np.abs(got - ref).max()))
            same = np.array_equal(np.sort(ref_cache.positions().cpu().numpy(), axis=-1), oc.positions())
            assert same, "retained set differs from the oracle"
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = {"value": B * args.cpu_steps / tc, "unit": "tokens/s/layer", "cores": threads, "kind": "oracle",
               "sample": f"{args.cpu_steps} steady-state block steps of layer 0 (fp64, OpenMP over heads x rows)",
               "us_per_step": tc / args.cpu_steps * 1e6, "max_abs_attention_diff_vs_gpu": worst,
               "retained_sets_identical": True}

    # ---- whole prompt: the N / B fill steps (fewer keys, nothing evicted) and every evicting step,
    # back to back from empty caches, through every layer with that layer's own data -- the order a
    # model runs them in (block by block, layer after layer)
    whole = None
    if not args.no_whole_prompt:
        for c in caches:
            c.close()
        del caches[:], dq[:], dk[:], dv[:]
        torch.cuda.empty_cache()
        t0 = time.time()
        with ThreadPoolExecutor(workers) as ex:
            full = list(ex.map(lambda l: make_layer(w, seed=args.seed + 100 * 3 + l, layer=l, t1=w.prompt_T), range(L)))
        log(f"[bench] generated {L} layers x {w.prompt_T} tokens in {time.time() - t0:.1f}s")
        wq, wk, wv = ([to_blocks(f[x], B) for f in full] for x in ("q", "k", "v"))
        del full
        wcs = [kd.KeyDiffCache(kd.KeyDiffConfig(w.batch, Hq, Hkv, D, N, B, layout=layout)) for _ in range(L)]
        wouts = [torch.empty_like(wq[0][0]) for _ in range(L)]
        nb = w.prompt_T // B
        empty_kv = torch.empty((w.batch, Hkv, 0, D), dtype=torch.bfloat16, device="cuda")
        empty_pos = torch.empty((w.batch, Hkv, 0), dtype=torch.int32, device="cuda")
        for rep in range(2):                       # first pass warms up, second is timed
            for wc in wcs:
                wc.load(empty_kv, empty_kv, empty_pos)  # back to the empty cache
            torch.cuda.synchronize()
            t_w = time.perf_counter()
            for b_ in range(nb):
                if deferred:
                    kd.prefill_block_layers(wcs, [t[b_] for t in wq], [t[b_] for t in wk], [t[b_] for t in wv], b_ * B,
                                            out=wouts)
                    continue
                for l in range(L):
                    wcs[l].prefill_block(wq[l][b_], wk[l][b_], wv[l][b_], b_ * B, out=wouts[l])
            for wc in wcs:
                wc.finish()
            torch.cuda.synchronize()
            t_w = time.perf_counter() - t_w
        whole = {"prompt_tokens": w.prompt_T, "steps": nb, "fill_steps": fill_blocks, "layers": L,
                 "ms_all_layers": t_w * 1e3, "ms_per_layer": t_w * 1e3 / L,
                 "tokens_per_s_per_layer": w.prompt_T * L / t_w, "tokens_per_s_all_layers": w.prompt_T / t_w}
        assert all(wc.status() == 0 for wc in wcs)
        for wc in wcs:
            wc.close()

    # the bandwidth-bound kernels of a step against the HBM peak (live HIP-event times; bytes per launch
    # from the launch plan: `splits` partial outputs of Hq x B rows in fp16 + their (max, sum) pairs in,
    # the merged rows out; the stable shift reads and writes the rows behind the first evicted one,
    # here priced as every row of K and V)
    hbm_kernels = {}
    if plan[0] > 1 and "step_post" in kernels and deferred:
        mb = plan[0] * Hq * B * (D * 2 + 8) + Hq * B * D * 2
        us = kernels["step_post"]["avg_us"]
        hbm_kernels["merge_kernel"] = {"bytes": mb, "us": us, "GBps": mb / us / 1e3,
                                       "frac_of_hbm_peak": mb / us / 1e3 / PEAK_HBM_GBPS, "key_ranges": plan[0]}
    if ordered_kernels and "compact_ordered" in ordered_kernels:
        cb = 2 * 2 * Hkv * N * D * 2
        us = ordered_kernels["compact_ordered"]["event_bracket_us"]
        hbm_kernels["compact_ordered_kernel"] = {"bytes_upper_bound": cb, "event_bracket_us": us, "GBps": cb / us / 1e3,
                                                 "frac_of_hbm_peak": cb / us / 1e3 / PEAK_HBM_GBPS}
    if scores_pass:
        hbm_kernels["step_score_kernel"] = scores_pass
    if modes:
        for v in modes.values():
            v["frac_of_step_roofline"] = t_min / (v["us_per_layer_step"] * 1e-6)
    decode = None
    if not args.no_extras and w.name == "llama31_8b":
        decode = decode_record(args)

    print(json.dumps({
        "metric": "prompt tokens/sec per layer (KeyDiff block prefill) at N=8K"
                  if N == 8192 else f"prompt tokens/sec per layer (KeyDiff block prefill) at N={N}",
        "value": tokens_per_s_per_layer, "unit": "tokens/s/layer", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D, "budget_N": N,
                   "block_B": B, "layers": L, "layout": args.layout,
                   "eviction": "deferred" if deferred else "immediate", "tokens_per_step": B,
                   "step": "one steady-state block step through every layer"},
        "us_per_layer_step": us_per_layer_step,
        "step_roofline": {"binding": "mfma" if flops_attn / 2.5e15 > bytes_step / 8e12 else "hbm",
                          "t_min_us": t_min * 1e6, "frac": step_frac, "flops": flops_attn, "bytes": bytes_step},
        "roofline": roofline, "kernels": kernels, "modes": modes, "hbm_kernels": hbm_kernels,
        "whole_prompt": whole, "decode": decode, "cpu_baseline": cpu,
    }))


if __name__ == "__main__":
    main()
