"""Phase timeline of step_main (and of the selection it carries) from in-kernel wall-clock stamps.

Needs the profiling build of the library (`python -m paper_2504_15364_amd.build --timeline`), which
stamps the 100 MHz wall clock at named points of every workgroup; this script runs steady-state block
steps of a workload through several layers with the eviction deferred (the launch bench.py times),
collects the stamps of every launch and prints, per phase, when it ends (microseconds after the
launch's first workgroup started; mean / min / max over workgroups and launches).

    python -m paper_2504_15364_amd.timeline [--workload llama31_8b] [--layers 8] [--steps 6]
"""
from __future__ import annotations

import argparse
import ctypes as C
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
os.environ["KEYDIFF_LIBRARY"] = os.path.join(HERE, "libkeydiff_timeline.so")
sys.path.insert(0, os.path.dirname(HERE))

ATTN_PHASES = [
    (13, "  arguments read, key range known"),
    (14, "  block rows and first K tile requested"),
    (15, "  queries requested"),
    (1, "first two tiles + queries requested"),
    (2, "block rows landed, summed (fp64) and folded"),
    (3, "queries and first K tile landed"),
    (4, "queries in registers"),
    (5, "first barrier passed"),
    (6, "anchor formed"),
    (7, "logits of first tile ready (loop starts)"),
    (16, "  step 3: barrier passed"),
    (17, "  step 3: stage A done (S^T of next tile)"),
    (18, "  step 3: stage B done (O^T += V^T P^T)"),
    (19, "  step 3: tile scored"),
    (20, "  step 4: barrier passed"),
    (21, "  step 4: stage A done"),
    (22, "  step 4: stage B done"),
    (23, "  step 4: tile scored"),
    (8, "all steps but the last done"),
    (9, "last tile done"),
    (10, "partials / output stores issued"),
    (11, "append stored, scores flushed"),
    (12, "stores acknowledged (workgroup ends)"),
]
SEL_PHASES = [
    (1, "loads issued (scores, positions, key sum, tail rows)"),
    (3, "scores arrived and binned"),
    (4, "threshold bin known"),
    (5, "candidates collected"),
    (6, "ranking done"),
    (7, "lists written"),
    (8, "evicted rows read, key sum stored"),
    (9, "moves issued"),
    (12, "stores acknowledged (workgroup ends)"),
]
TICK_US = 0.01   # wall_clock64 counts a constant 100 MHz clock


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="llama31_8b")
    ap.add_argument("--layers", type=int, default=8)
    ap.add_argument("--steps", type=int, default=6)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--seed", type=int, default=20250415)
    ap.add_argument("--eviction", choices=["deferred", "immediate"], default="deferred",
                    help="immediate: keydiff_prefill_block per layer; the selection then runs in step_post, after the attention")
    args = ap.parse_args()

    import torch

    import paper_2504_15364_amd as kd
    from synth import get_config, make_layer

    lib = kd.load_library()
    if not hasattr(lib, "keydiff_timeline_buffer"):
        sys.exit("the loaded library is not the profiling build")
    lib.keydiff_timeline_buffer.argtypes = [C.c_void_p, C.c_size_t]
    lib.keydiff_timeline_buffer.restype = C.c_long

    w = get_config(args.workload)
    L, B, N, D, Hq, Hkv = args.layers, w.block_B, w.budget_N, w.head_dim, w.n_q_heads, w.n_kv_heads
    fill = N // B
    nsteps = args.warmup + args.steps
    T = (fill + nsteps) * B
    # one seeded token stream per (layer, sequence of the batch)
    layers = [[make_layer(w, seed=args.seed + 300 + l, layer=l, seq=sq, t1=T) for sq in range(w.batch)] for l in range(L)]

    def to_blocks(seqs, name):   # -> [block][batch][heads][B][d]
        bits = np.stack([sq[name] for sq in seqs])                       # [batch][T][heads][d]
        t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)
        nb, Tn, H, d = bits.shape
        return t.view(nb, Tn // B, B, H, d).permute(1, 0, 3, 2, 4).contiguous()

    caches, dq, dk, dv, outs = [], [], [], [], []
    for l in range(L):
        caches.append(kd.KeyDiffCache(kd.KeyDiffConfig(w.batch, Hq, Hkv, D, N, B, layout=kd.LAYOUT_FILL)))
        dq.append(to_blocks(layers[l], "q"))
        dk.append(to_blocks(layers[l], "k"))
        dv.append(to_blocks(layers[l], "v"))
        outs.append(torch.empty_like(dq[l][0]))
        # the first N tokens of every sequence, [batch][heads][N][d]
        k0 = dk[l][:fill].permute(1, 2, 0, 3, 4).reshape(w.batch, Hkv, N, D).contiguous()
        v0 = dv[l][:fill].permute(1, 2, 0, 3, 4).reshape(w.batch, Hkv, N, D).contiguous()
        p0 = torch.arange(N, dtype=torch.int32, device="cuda").repeat(w.batch, Hkv, 1).contiguous()
        caches[l].load(k0, v0, p0)

    def run_block(i):
        if args.eviction == "deferred":
            kd.prefill_block_layers(caches, [t[i] for t in dq], [t[i] for t in dk], [t[i] for t in dv], i * B, out=outs)
        else:
            for l in range(L):
                caches[l].prefill_block(dq[l][i], dk[l][i], dv[l][i], i * B, out=outs[l])

    for i in range(fill, fill + args.warmup):
        run_block(i)
    torch.cuda.synchronize()
    slots = L * args.steps * (1 if args.eviction == "deferred" else 2)   # immediate: step_main, then step_post
    WGS = 512
    buf = torch.zeros(slots * WGS * 32, dtype=torch.int64, device="cuda")
    got = lib.keydiff_timeline_buffer(buf.data_ptr(), buf.numel() * 8)
    assert got == slots, (got, slots)
    for i in range(fill + args.warmup, fill + nsteps):
        run_block(i)
    torch.cuda.synchronize()
    lib.keydiff_timeline_buffer(None, 0)
    rec = buf.cpu().numpy().reshape(slots, WGS, 32)
    for c in caches:
        assert c.status() == 0
        c.close()

    def summarise(kind, phases, title):
        rows = {i: [] for i, _ in phases}
        starts, ntl = [], []
        n_wg = 0
        for s in range(slots):
            r = rec[s]
            live = r[r[:, 31] != 0]
            if live.size == 0:
                continue
            t_launch = live[:, 0].min()            # first workgroup of the launch to start
            mine = live[live[:, 31] == kind]
            n_wg = max(n_wg, len(mine))
            starts.extend(((mine[:, 0] - t_launch) * TICK_US).tolist())
            ntl.extend(mine[:, 30].tolist())
            for i, _ in phases:
                ok = mine[:, i] != 0
                rows[i].extend(((mine[ok, i] - t_launch) * TICK_US).tolist())
        if not starts:
            return
        print(f"\n{title}: {n_wg} workgroups per launch, {len(starts) // max(n_wg, 1)} launches")
        if kind == 1:
            print(f"  key tiles per workgroup: mean {np.mean(ntl):.2f}, min {int(np.min(ntl))}, max {int(np.max(ntl))}")
        print(f"  {'phase ends (us after the first workgroup of the launch started)':66s} {'mean':>7s} {'min':>7s} {'max':>7s}   +mean")
        print(f"  {'workgroup starts':66s} {np.mean(starts):7.2f} {np.min(starts):7.2f} {np.max(starts):7.2f}")
        prev = float(np.mean(starts))
        for i, name in phases:
            if not rows[i]:
                continue
            m = float(np.mean(rows[i]))
            delta = "" if name.startswith("  ") else f"{m - prev:+7.2f}"
            print(f"  {name:66s} {m:7.2f} {np.min(rows[i]):7.2f} {np.max(rows[i]):7.2f}   {delta}")
            if not name.startswith("  "):
                prev = m

    print(f"# workload {w.name}: {L} layers, {args.steps} recorded block steps, eviction {args.eviction} "
          f"({'step_main_carry_kernel' if args.eviction == 'deferred' else 'step_main_kernel, then step_post_kernel'})")
    print("# stamps: thread 0 of every workgroup, constant 100 MHz clock (0.01 us resolution)")
    summarise(1, ATTN_PHASES, "attention workgroups")
    summarise(2, SEL_PHASES, "carried selection workgroups" if args.eviction == "deferred"
              else "selection workgroups of step_post (a launch of its own after the attention)")
    summarise(4, [(12, "partials merged, output stored and acknowledged (workgroup ends)")],
              "merging workgroups of step_post")
    # when the attention workgroups end, by position in the grid: key split (workgroups of a split take
    # consecutive key tiles; the last split holds the block's own rows) and KV head
    BH = w.batch * Hkv
    mtiles = (w.group * B + 255) // 256
    by_split, by_head, by_start = {}, {}, []
    for s in range(slots):
        r = rec[s]
        idx = np.nonzero(r[:, 31] == 1)[0]
        if idx.size == 0:
            continue
        t_launch = r[r[:, 31] != 0][:, 0].min()
        first = idx.min()
        for i in idx:
            wg = i - first
            end = (r[i, 12] - t_launch) * TICK_US
            by_split.setdefault(wg // (BH * mtiles), []).append((end, r[i, 30], (r[i, 0] - t_launch) * TICK_US))
            by_head.setdefault(wg % BH, []).append(end)
    if by_split:
        print("\nattention workgroups by key split: tiles, start, end (us, mean over launches, heads and row tiles)")
        for sp in sorted(by_split):
            v = np.array(by_split[sp])
            print(f"  split {sp:2d}: tiles {v[:, 1].mean():5.2f}  start {v[:, 2].mean():5.2f}  end {v[:, 0].mean():6.2f}  (max {v[:, 0].max():6.2f})")
        print("  by KV head (end, mean): " + "  ".join(f"{np.mean(by_head[h]):.2f}" for h in sorted(by_head)))
    ends = []
    for s in range(slots):
        live = rec[s][rec[s][:, 31] != 0]
        if live.size:
            ends.append((live[:, 12].max() - live[:, 0].min()) * TICK_US)
    print(f"\nfirst workgroup start -> last workgroup end, per launch: mean {np.mean(ends):.2f} us, "
          f"min {np.min(ends):.2f}, max {np.max(ends):.2f}")


if __name__ == "__main__":
    main()
