"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The retained position set of every KV head is compared with the oracle after
EVERY block step of the prompt (the eviction trace needs keys only, so the oracle
runs it without attention); attention is compared on sampled steps, for which the
oracle is in the bit-identical cache state.
"""
import numpy as np
import pytest

import oracle
import paper_2504_15364_amd as kd
from helpers import ATTN_ATOL, SCORE_ATOL, SCORE_RTOL, bf16_out_to_f32, rows_by_position, to_dev
from synth import block_of, get_config, make_layer

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def dev_blocks(bits, B):
    T, H, d = bits.shape
    t = to_dev(bits)
    return t.view(T // B, B, H, d).permute(0, 2, 1, 3).contiguous().unsqueeze(1)


def run_full(name, layout, T=None, attn_steps=(), seed=77, layer=0, **kw):
    """The whole prompt of one layer through keydiff_prefill_block: retained sets against the oracle
    after every step, attention on the steps named, K/V rows at the end.  kw: anchor_mode, window_W."""
    w = get_config(name)
    T = T or w.prompt_T
    B, N = w.block_B, w.budget_N
    data = make_layer(w, seed=seed, layer=layer, t1=T)
    dq, dk, dv = (dev_blocks(data[x], B) for x in ("q", "k", "v"))
    cache = kd.KeyDiffCache(kd.KeyDiffConfig(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B, layout=layout, **kw))
    oc = oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B, **kw)
    nsteps = T // B
    attn_steps = {s % nsteps for s in attn_steps}
    evicting = 0
    for i in range(nsteps):
        want_attn = i in attn_steps
        q = block_of(data["q"], i * B, B)[None] if want_attn else None
        out = cache.prefill_block(dq[i], dk[i], dv[i], i * B)
        ref, _, ev = oc.prefill_block(q, block_of(data["k"], i * B, B)[None], block_of(data["v"], i * B, B)[None], i * B)
        evicting += ev > 0
        pos = np.sort(cache.positions().cpu().numpy(), axis=-1)
        assert np.array_equal(pos, oc.positions()), f"{name}: retained set differs after step {i}"
        if want_attn:
            err = float(np.abs(bf16_out_to_f32(out) - ref).max())
            assert err <= ATTN_ATOL, f"{name}: attention error {err} at step {i}"
    # the K/V row behind every retained position, bit for bit
    pos, K, V = rows_by_position(cache)
    assert np.array_equal(K, oc.keys()) and np.array_equal(V, oc.values())
    assert cache.status() == 0
    assert evicting == nsteps - N // B
    if layout == kd.LAYOUT_ORDERED:
        assert np.all(np.diff(cache.positions().cpu().numpy(), axis=-1) > 0), "rows not in position order"
    cache.close()


def test_llama31_8b_shape_whole_prompt_fill_layout():
    # the headline workload as bench.py launches it (FILL layout), all 256 steps of one layer
    run_full("llama31_8b", kd.LAYOUT_FILL, attn_steps=(3, 64, 255))


def test_llama31_8b_shape_whole_prompt_ordered_layout():
    # the stable in-place layout over all 256 steps (192 of them shift rows)
    run_full("llama31_8b", kd.LAYOUT_ORDERED, attn_steps=(100, -1), layer=5)


def test_llama31_8b_shape_whole_prompt_sliding_window():
    # Method, "KeyDiff with Sliding Window": 10 % of the budget reserved for the most recent tokens
    run_full("llama31_8b", kd.LAYOUT_FILL, attn_steps=(200,), layer=2, window_W=819)


def test_llama31_8b_shape_whole_prompt_unit_key_anchor():
    # Eq. 7 as printed: the anchor is the mean of the unit keys
    run_full("llama31_8b", kd.LAYOUT_FILL, attn_steps=(130,), layer=3, anchor_mode=kd.ANCHOR_MEAN_UNIT_KEY)


def test_llama32_3b_shape_whole_prompt():
    run_full("llama32_3b", kd.LAYOUT_FILL, attn_steps=(40, 127))


def test_qwen25_7b_shape_whole_prompt():
    # G = 7, B = 256, heavy channel outliers: all 128 steps (96 evicting)
    run_full("qwen25_7b", kd.LAYOUT_FILL, attn_steps=(31, 77, -1))


def test_decode_8b_shape_batch16_all_steps():
    # full budget, batch of 16 sequences, one token and one eviction per sequence, head and step, for
    # all 1024 steps.  The retained sets are compared after every step (the oracle runs the eviction
    # trace without attention, one host thread per sequence: the sequences are independent); attention
    # on sampled steps, where the oracle is in the bit-identical cache state.
    from concurrent.futures import ThreadPoolExecutor
    w = get_config("decode_8b")
    N, steps = w.budget_N, w.decode_steps
    assert steps == 1024
    sampled = {0, 1, 63, 200, 511, 777, 1000, 1023}
    with ThreadPoolExecutor(16) as ex:
        seqs = list(ex.map(lambda s: make_layer(w, seed=55, seq=s, t1=N + steps), range(w.batch)))
        cfg = kd.KeyDiffConfig(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, N, 1, layout=kd.LAYOUT_FILL)
        cache = kd.KeyDiffCache(cfg)
        ocs = [oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, 1) for _ in range(w.batch)]
        K0 = np.stack([s["k"][:N].transpose(1, 0, 2) for s in seqs])          # [batch][Hkv][N][d]
        V0 = np.stack([s["v"][:N].transpose(1, 0, 2) for s in seqs])
        P0 = np.broadcast_to(np.arange(N, dtype=np.int32), (w.batch, w.n_kv_heads, N)).copy()
        cache.load(to_dev(K0), to_dev(V0), torch.from_numpy(P0).cuda())
        for b, oc in enumerate(ocs):
            oc.load(K0[b:b + 1], V0[b:b + 1], P0[b:b + 1])
        toks = {x: to_dev(np.stack([s[x][N:] for s in seqs]).transpose(1, 0, 2, 3)[:, :, :, None, :])
                for x in ("q", "k", "v")}                                     # [step][batch][heads][1][d]
        for i in range(steps):
            t = N + i
            out = cache.decode_step(toks["q"][i], toks["k"][i], toks["v"][i], t)
            want = i in sampled

            def one(b):
                q, k, v = (seqs[b][x][t][None, :, None, :] for x in ("q", "k", "v"))
                ref, _, ev = ocs[b].decode_step(q if want else None, k, v, t)
                assert ev == 1
                return ref, ocs[b].positions()[0]
            res = list(ex.map(one, range(w.batch)))
            got_pos = np.sort(cache.positions().cpu().numpy(), axis=-1)
            assert np.array_equal(got_pos, np.stack([r[1] for r in res])), f"retained set differs after step {i}"
            if want:
                ref = np.concatenate([r[0] for r in res])
                err = float(np.abs(bf16_out_to_f32(out) - ref).max())
                assert err <= ATTN_ATOL, f"attention error {err} at step {i}"
    got = cache.scores().cpu().numpy()
    order = np.argsort(cache.positions().cpu().numpy(), axis=-1, kind="stable")
    want_sc = np.concatenate([oc.scores() for oc in ocs])
    assert np.allclose(np.take_along_axis(got, order, -1), want_sc, rtol=SCORE_RTOL, atol=SCORE_ATOL)
    pos, K, V = rows_by_position(cache)
    assert np.array_equal(K, np.concatenate([oc.keys() for oc in ocs]))
    assert np.array_equal(V, np.concatenate([oc.values() for oc in ocs]))
    assert cache.status() == 0
    cache.close()


BENCH_SEED = 20250415 + 100 * 3     # bench.py: --seed + 100 * (config number) + layer


def test_llama31_8b_shape_whole_prompt_through_the_layers_call_with_the_bench_seeds():
    # What bench.py times, from empty caches over the whole prompt: keydiff_prefill_block_layers on
    # the first four layers with the benchmark's own seeds, every layer's eviction carried by the
    # next layer's attention launch.  Retained sets of layers 0-2 are compared with the oracle after
    # every block (reading them forces nothing: their evictions have ridden already); the last
    # layer's eviction is still pending after a call, and reading its positions would run it in a
    # launch of its own, so it is read every 16th block and at the end -- both ways of finishing an
    # eviction then occur.  Attention on sampled (block, layer) pairs.
    from concurrent.futures import ThreadPoolExecutor
    w = get_config("llama31_8b")
    B, N, T, L = w.block_B, w.budget_N, w.prompt_T, 4
    nb = T // B
    with ThreadPoolExecutor(L) as ex:
        layers = list(ex.map(lambda l: make_layer(w, seed=BENCH_SEED + l, layer=l, t1=T), range(L)))
        caches = [kd.KeyDiffCache(kd.KeyDiffConfig(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B, layout=kd.LAYOUT_FILL))
                  for _ in range(L)]
        ocs = [oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B) for _ in range(L)]
        dq, dk, dv = ([dev_blocks(d[x], B) for d in layers] for x in ("q", "k", "v"))
        for c in caches:
            c.profile_enable(True)
        sampled = {(5, 0), (64, 1), (65, 3), (150, 2), (255, 0), (255, 3)}
        for i in range(nb):
            outs = kd.prefill_block_layers(caches, [t[i] for t in dq], [t[i] for t in dk], [t[i] for t in dv], i * B)

            def one(l):
                q = block_of(layers[l]["q"], i * B, B)[None] if (i, l) in sampled else None
                ref, _, _ = ocs[l].prefill_block(q, block_of(layers[l]["k"], i * B, B)[None],
                                                 block_of(layers[l]["v"], i * B, B)[None], i * B)
                return ref
            refs = list(ex.map(one, range(L)))
            for l in range(L):
                if refs[l] is not None:
                    err = float(np.abs(bf16_out_to_f32(outs[l]) - refs[l]).max())
                    assert err <= ATTN_ATOL, f"attention error {err}, block {i}, layer {l}"
                if l < L - 1 or i % 16 == 15 or i == nb - 1:
                    pos = np.sort(caches[l].positions().cpu().numpy(), axis=-1)
                    assert np.array_equal(pos, ocs[l].positions()), f"retained set differs: block {i}, layer {l}"
    rode = alone = 0
    for l in range(L):
        pos, K, V = rows_by_position(caches[l])
        assert np.array_equal(pos, ocs[l].positions())
        assert np.array_equal(K, ocs[l].keys()) and np.array_equal(V, ocs[l].values()), f"rows of layer {l} differ"
        assert caches[l].status() == 0
        alone += caches[l].profile_read()["select_alone"][1]
        caches[l].close()
    evicting = nb - N // B
    assert alone == evicting // 16, f"{alone} evictions ran alone; expected the {evicting // 16} the test forced"


def test_llama31_8b_shape_ordered_layout_through_the_layers_call():
    # the ORDERED layout the way bench.py's "deferred_ordered" mode runs it: caches loaded at the budget,
    # steady-state blocks through four layers in one call per block; the row shift of layer l rides in the
    # attention launch of layer l + 2 (56 workgroups next to 192 of the attention and 8 of a selection)
    w = get_config("llama31_8b")
    B, N, L, steps = w.block_B, w.budget_N, 4, 6
    T = N + steps * B
    caches, ocs, datas, dev = [], [], [], []
    for l in range(L):
        data = make_layer(w, seed=BENCH_SEED + l, layer=l, t1=T)
        cache = kd.KeyDiffCache(kd.KeyDiffConfig(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B, layout=kd.LAYOUT_ORDERED))
        oc = oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B)
        K0 = data["k"][:N].transpose(1, 0, 2)[None].copy()
        V0 = data["v"][:N].transpose(1, 0, 2)[None].copy()
        P0 = np.broadcast_to(np.arange(N, dtype=np.int32), (1, w.n_kv_heads, N)).copy()
        cache.load(to_dev(K0), to_dev(V0), torch.from_numpy(P0).cuda())
        oc.load(K0, V0, P0)
        caches.append(cache), ocs.append(oc), datas.append(data)
        dev.append(tuple(dev_blocks(data[x][N:], B) for x in ("q", "k", "v")))
    sampled = {(0, 0), (1, 2), (3, 1), (steps - 1, L - 1)}
    hosted = 0
    for i in range(steps):
        t = N + i * B
        outs = kd.prefill_block_layers(caches, [d[0][i] for d in dev], [d[1][i] for d in dev], [d[2][i] for d in dev], t)
        plans = [c.plan() for c in caches]
        hosted += sum(1 for pl in plans if pl[3] & 2)
        if i >= 1:
            assert all(pl[3] & 2 for pl in plans), f"block {i}: a launch took no row shift along: {plans}"
            assert all(pl[0] == 12 for pl in plans), plans     # 12 key ranges x 16 + 8 + 56 workgroups = 256
        for l in range(L):
            q = block_of(datas[l]["q"], t, B)[None] if (i, l) in sampled else None
            ref, _, ev = ocs[l].prefill_block(q, block_of(datas[l]["k"], t, B)[None], block_of(datas[l]["v"], t, B)[None], t)
            assert ev == B
            if q is not None:
                err = float(np.abs(bf16_out_to_f32(outs[l]) - ref).max())
                assert err <= ATTN_ATOL, f"attention error {err}, step {i}, layer {l}"
    for l in range(L):
        pos, K, V = rows_by_position(caches[l])   # finishes what is still pending
        assert np.array_equal(pos, ocs[l].positions()), f"retained set of layer {l} differs"
        assert np.array_equal(K, ocs[l].keys()) and np.array_equal(V, ocs[l].values())
        assert np.all(np.diff(caches[l].positions().cpu().numpy(), axis=-1) > 0), "rows not in position order"
        assert caches[l].status() == 0
        caches[l].close()
    assert hosted >= (steps - 1) * L


@pytest.mark.parametrize("layout", [kd.LAYOUT_FILL, kd.LAYOUT_ORDERED], ids=["fill", "ordered"])
def test_llama31_8b_shape_deferred_eviction_across_layers(layout):
    # the headline workload the way bench.py runs it by default: caches loaded at the budget, then
    # steady-state block steps through several layers, every layer's eviction carried by the next
    # layer's attention launch.  Attention is checked on sampled calls, the caches at the end.
    w = get_config("llama31_8b")
    B, N, L, steps = w.block_B, w.budget_N, 3, 5
    T = N + steps * B
    layers = []
    for l in range(L):
        data = make_layer(w, seed=91, layer=l, t1=T)
        cache = kd.KeyDiffCache(kd.KeyDiffConfig(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B, layout=layout))
        oc = oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B)
        K0 = data["k"][:N].transpose(1, 0, 2)[None].copy()
        V0 = data["v"][:N].transpose(1, 0, 2)[None].copy()
        P0 = np.broadcast_to(np.arange(N, dtype=np.int32), (1, w.n_kv_heads, N)).copy()
        cache.load(to_dev(K0), to_dev(V0), torch.from_numpy(P0).cuda())
        oc.load(K0, V0, P0)
        cache.profile_enable(True)
        layers.append((data, cache, oc, *(dev_blocks(data[x][N:], B) for x in ("q", "k", "v"))))
    sampled = {(0, 0), (2, 1), (steps - 1, L - 1)}
    for i in range(steps):
        for l, (data, cache, oc, dq, dk, dv) in enumerate(layers):
            t = N + i * B
            out = cache.prefill_block_deferred(dq[i], dk[i], dv[i], t, carry=layers[l - 1][1])
            q = block_of(data["q"], t, B)[None] if (i, l) in sampled else None
            ref, _, ev = oc.prefill_block(q, block_of(data["k"], t, B)[None], block_of(data["v"], t, B)[None], t)
            assert ev == B
            if q is not None:
                err = float(np.abs(bf16_out_to_f32(out) - ref).max())
                assert err <= ATTN_ATOL, f"attention error {err}, step {i}, layer {l}"
    alone = 0
    for l, (data, cache, oc, *_rest) in enumerate(layers):
        pos, K, V = rows_by_position(cache)   # finishes what is still pending (the last layer's last eviction)
        assert np.array_equal(pos, oc.positions()), f"retained set of layer {l} differs"
        assert np.array_equal(K, oc.keys()) and np.array_equal(V, oc.values())
        if layout == kd.LAYOUT_ORDERED:
            assert np.all(np.diff(cache.positions().cpu().numpy(), axis=-1) > 0), "rows not in position order"
        assert cache.status() == 0
        cnt = cache.profile_read()
        alone += cnt["select_alone"][1]
        cache.close()
    assert alone == 1, f"{alone} evictions ran in a launch of their own; only the very last one should"
