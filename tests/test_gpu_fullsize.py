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


def run_full(name, layout, T=None, attn_steps=(), seed=77, layer=0):
    w = get_config(name)
    T = T or w.prompt_T
    B, N = w.block_B, w.budget_N
    data = make_layer(w, seed=seed, layer=layer, t1=T)
    dq, dk, dv = (dev_blocks(data[x], B) for x in ("q", "k", "v"))
    cache = kd.KeyDiffCache(kd.KeyDiffConfig(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B, layout=layout))
    oc = oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B)
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
    cache.close()


def test_llama31_8b_shape_whole_prompt_fill_layout():
    # the headline workload as bench.py launches it (FILL layout), all 256 steps of one layer
    run_full("llama31_8b", kd.LAYOUT_FILL, attn_steps=(3, 64, 255))


def test_llama31_8b_shape_ordered_layout():
    run_full("llama31_8b", kd.LAYOUT_ORDERED, T=8192 + 24 * 128, attn_steps=(-1,), layer=5)


def test_llama32_3b_shape_whole_prompt():
    run_full("llama32_3b", kd.LAYOUT_FILL, attn_steps=(40, 127))


def test_qwen25_7b_shape():
    # G = 7, B = 256, heavy channel outliers
    run_full("qwen25_7b", kd.LAYOUT_FILL, T=8192 + 24 * 256, attn_steps=(31, -1))


def test_decode_8b_shape_batch16():
    # full budget, batch of 16 sequences, one token and one eviction per step
    w = get_config("decode_8b")
    N, steps = w.budget_N, 32
    seqs = [make_layer(w, seed=55, seq=s, t1=N + steps) for s in range(w.batch)]
    cfg = kd.KeyDiffConfig(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, N, 1, layout=kd.LAYOUT_FILL)
    cache = kd.KeyDiffCache(cfg)
    oc = oracle.OracleCache(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, N, 1)
    K0 = np.stack([s["k"][:N].transpose(1, 0, 2) for s in seqs])          # [batch][Hkv][N][d]
    V0 = np.stack([s["v"][:N].transpose(1, 0, 2) for s in seqs])
    P0 = np.broadcast_to(np.arange(N, dtype=np.int32), (w.batch, w.n_kv_heads, N)).copy()
    cache.load(to_dev(K0), to_dev(V0), torch.from_numpy(P0).cuda())
    oc.load(K0, V0, P0)
    for t in range(N, N + steps):
        q, k, v = (np.stack([s[x][t][:, None, :] for s in seqs]) for x in ("q", "k", "v"))
        out = cache.decode_step(to_dev(q), to_dev(k), to_dev(v), t)
        ref, _, ev = oc.decode_step(q, k, v, t)
        assert ev == 1
        assert np.abs(bf16_out_to_f32(out) - ref).max() <= ATTN_ATOL, t
        assert np.array_equal(np.sort(cache.positions().cpu().numpy(), axis=-1), oc.positions()), t
    got = cache.scores().cpu().numpy()
    order = np.argsort(cache.positions().cpu().numpy(), axis=-1, kind="stable")
    assert np.allclose(np.take_along_axis(got, order, -1), oc.scores(), rtol=SCORE_RTOL, atol=SCORE_ATOL)
    assert cache.status() == 0


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
