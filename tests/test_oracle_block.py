"""Pins for the oracle's attention and block prompt processing (CPU only)."""
import os

import numpy as np
import pytest

import oracle
from synth import bf16_bits_to_f64, block_of, f32_to_bf16_bits, get_config, make_layer

torch = pytest.importorskip("torch")


def bits(x):
    return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def full_causal_reference(q, k, v, G):
    """Plain causal attention over the whole prompt with a library routine.
    q [T][hq][d], k/v [T][hkv][d] bits -> float64 [T][hq][d]."""
    qd = torch.from_numpy(bf16_bits_to_f64(q)).permute(1, 0, 2)            # [hq][T][d]
    kd = torch.from_numpy(bf16_bits_to_f64(k)).permute(1, 0, 2).repeat_interleave(G, dim=0)
    vd = torch.from_numpy(bf16_bits_to_f64(v)).permute(1, 0, 2).repeat_interleave(G, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(qd, kd, vd, is_causal=True)
    return o.permute(1, 0, 2).numpy()


def run_blocks(w, data, B, N, with_q=True, **kw):
    oc = oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B, **kw)
    outs, trace = [], []
    T = data["k"].shape[0]
    for t in range(0, T, B):
        Bt = min(B, T - t)
        q = block_of(data["q"], t, Bt)[None] if with_q else None
        o, _, ev = oc.prefill_block(q, block_of(data["k"], t, Bt)[None], block_of(data["v"], t, Bt)[None], t)
        if with_q:
            outs.append(o[0].transpose(1, 0, 2))                             # [Bt][hq][d]
        trace.append((oc.len, ev, oc.positions().copy()))
    return (np.concatenate(outs) if with_q else None), trace, oc


SMALL = get_config("toy").small(n_q_heads=6, n_kv_heads=2, head_dim=16, prompt_T=45)


@pytest.mark.parametrize("B", [45, 16, 7, 1])
def test_blockwise_attention_without_eviction_is_one_shot_causal_attention(B):
    # Background, block prompt processing: one block of the whole prompt (B = T) is one-shot
    # processing; with N >= T nothing is evicted, so the same holds for every B, and B = 1 is
    # the generation phase (Eq. 2).
    data = make_layer(SMALL, seed=3)
    ref = full_causal_reference(data["q"], data["k"], data["v"], SMALL.group)
    got, trace, _ = run_blocks(SMALL, data, B, N=64)
    assert np.allclose(got, ref, rtol=1e-5, atol=1e-6)        # oracle emits float32
    assert all(ev == 0 for _, ev, _ in trace)


def test_gqa_head_mapping_and_softmax_scale():
    # values that identify their KV head: with G = 3, query heads 0-2 read head 0 and 3-5 head 1
    hq, hkv, d, n = 6, 2, 8, 5
    K = bits(np.random.default_rng(0).standard_normal((hkv, n, d)))
    V = bits(np.stack([np.full((n, d), 1.0), np.full((n, d), -2.0)]))
    q = bits(np.random.default_rng(1).standard_normal((hq, 1, d)))
    out = oracle.attention(q, K, V, length=n - 1, Bt=1)
    assert np.allclose(out[:3], 1.0) and np.allclose(out[3:], -2.0)       # rows of P sum to one
    # scale 1/sqrt(d): compare one row against the definition written with library calls
    kd, qd = bf16_bits_to_f64(K[1]), bf16_bits_to_f64(q[4, 0])
    Vr = bits(np.random.default_rng(2).standard_normal((hkv, n, d)))
    p = torch.softmax(torch.from_numpy(kd @ qd) / np.sqrt(d), dim=0).numpy()
    out = oracle.attention(q, K, Vr, length=n - 1, Bt=1)
    assert np.allclose(out[4, 0], p @ bf16_bits_to_f64(Vr[1]), rtol=1e-6, atol=1e-7)


def test_causal_mask_inside_the_block():
    # one cached row, a block of three: block query j must ignore block rows > j.
    hq = hkv = 1
    d = 4
    K = bits(np.zeros((1, 4, d)))                    # all logits equal -> uniform weights
    V = bits(np.array([[[8, 0, 0, 0], [0, 8, 0, 0], [0, 0, 8, 0], [0, 0, 0, 8]]], dtype=np.float32))
    q = bits(np.ones((1, 3, d)))
    out = oracle.attention(q, K, V, length=1, Bt=3)[0]
    assert np.allclose(out[0], [4, 4, 0, 0])
    assert np.allclose(out[1], [8 / 3, 8 / 3, 8 / 3, 0])
    assert np.allclose(out[2], [2, 2, 2, 2])


def test_fig1_shape_example():
    path = os.path.join(os.path.dirname(__file__), "golden", "fig1_block_processing.txt")
    g = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            key, *vals = line.split()
            g[key] = [int(v) for v in vals]
    T, N, B = g["prompt_T"][0], g["budget_N"][0], g["block_B"][0]
    w = get_config("toy").small(n_q_heads=2, n_kv_heads=1, head_dim=8, prompt_T=T)
    data = make_layer(w, seed=1)
    _, trace, _ = run_blocks(w, data, B, N)
    assert len(trace) == g["blocks"][0]
    assert [ln for ln, _, _ in trace] == g["cache_len_after"]
    assert [ev for _, ev, _ in trace] == g["evicted_per_step"]


def test_trace_invariants_and_independence_from_queries_and_values():
    w = get_config("toy").small(prompt_T=320, head_dim=32)
    N, B = 96, 32
    data = make_layer(w, seed=11)
    _, trace, oc = run_blocks(w, data, B, N)
    # budget never exceeded; exactly N kept once n > N; positions ascending and unique
    for i, (ln, ev, pos) in enumerate(trace):
        n_before = min(N, i * B) + B
        assert ln == min(n_before, N) and ev == max(0, n_before - N)
        assert np.all(np.diff(pos[0], axis=-1) > 0)
    # the trace depends on keys only: other queries/values, or no attention at all
    other = make_layer(w, seed=12)
    swapped = dict(data, q=other["q"], v=other["v"])
    _, trace2, _ = run_blocks(w, swapped, B, N)
    _, trace3, oc3 = run_blocks(w, data, B, N, with_q=False)
    for a, b, c in zip(trace, trace2, trace3):
        assert np.array_equal(a[2], b[2]) and np.array_equal(a[2], c[2])
    # every retained position carries its original K and V row, bit for bit
    pos = oc.positions()[0]
    for g in range(w.n_kv_heads):
        assert np.array_equal(oc.keys()[0, g], data["k"][pos[g], g])
        assert np.array_equal(oc.values()[0, g], data["v"][pos[g], g])


def test_each_step_keeps_the_brute_force_lowest_scores():
    # replay one evicting step by hand: library mean/cosine on the rows, full argsort
    w = get_config("toy").small(prompt_T=160, head_dim=16)
    N, B = 64, 32
    data = make_layer(w, seed=21)
    oc = oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, w.head_dim, N, B)
    for t in range(0, 160, B):
        before_pos = oc.positions()[0, 0] if oc.len else np.zeros(0, np.int32)
        rows_pos = np.concatenate([before_pos, np.arange(t, t + B, dtype=np.int32)])
        _, sc, ev = oc.prefill_block(None, block_of(data["k"], t, B)[None], block_of(data["v"], t, B)[None], t,
                                     want_scores=True)
        if ev == 0:
            continue
        x = torch.from_numpy(bf16_bits_to_f64(data["k"][rows_pos, 0]))
        cos = torch.nn.functional.cosine_similarity(x.mean(0)[None], x, dim=1).numpy()
        assert np.allclose(sc[0, 0], cos, rtol=1e-6, atol=1e-7)
        order = np.lexsort((rows_pos, cos.astype(np.float32)))[:N]
        assert np.array_equal(np.sort(rows_pos[order]), oc.positions()[0, 0])


def test_budget_at_least_prompt_never_evicts():
    w = get_config("toy").small(prompt_T=40, head_dim=16)
    data = make_layer(w, seed=31)
    _, trace, oc = run_blocks(w, data, 8, N=40)
    assert oc.len == 40 and all(ev == 0 for _, ev, _ in trace)
    assert np.array_equal(oc.positions()[0, 0], np.arange(40))


def test_decode_step_is_eq2_for_one_token_and_evicts_the_most_anchor_similar_key():
    # B = 1 is the generation phase.  Every step is replayed by hand on a cache tracked in numpy:
    # the new token attends to [K || k_new], [V || v_new] (Eq. 2) written with library calls, and
    # once the budget is exceeded the one key with the highest cosine to the mean key leaves
    # (full argsort by (score, position), last element).
    w = get_config("toy").small(n_q_heads=4, n_kv_heads=2, head_dim=16, prompt_T=40)
    G, N, d = 2, 12, 16
    data = make_layer(w, seed=31)
    oc = oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, d, N, 1)
    held = [np.zeros(0, np.int64) for _ in range(w.n_kv_heads)]     # positions cached per KV head
    for t in range(40):
        q, k, v = (block_of(data[x], t, 1)[None] for x in ("q", "k", "v"))
        out, _, ev = oc.decode_step(q, k, v, t)
        assert ev == (1 if t >= N else 0)
        for g in range(w.n_kv_heads):
            rows = np.concatenate([held[g], [t]])
            Kd = torch.from_numpy(bf16_bits_to_f64(data["k"][rows, g]))
            Vd = torch.from_numpy(bf16_bits_to_f64(data["v"][rows, g]))
            for h in range(g * G, (g + 1) * G):
                qd = torch.from_numpy(bf16_bits_to_f64(data["q"][t, h]))
                ref = torch.softmax(Kd @ qd / np.sqrt(d), dim=0) @ Vd
                assert np.allclose(out[0, h, 0], ref.numpy(), rtol=1e-6, atol=1e-7)
            if len(rows) > N:
                cos = torch.nn.functional.cosine_similarity(Kd.mean(0)[None], Kd, dim=1).numpy().astype(np.float32)
                gone = np.lexsort((rows, cos))[-1]
                rows = np.delete(rows, gone)
            held[g] = rows
            assert np.array_equal(oc.positions()[0, g], held[g])


def test_scores_of_the_cache_are_the_cosine_to_the_mean_cached_key():
    # several KV heads and a cache shorter than its capacity: a wrong head stride, or the capacity
    # taken for the length, would move the rows the anchor and the scores are taken over
    w = get_config("toy").small(n_q_heads=6, n_kv_heads=3, head_dim=16, prompt_T=96)
    data = make_layer(w, seed=41)
    _, _, oc = run_blocks(w, data, 32, N=48, with_q=False)
    assert oc.len == 48 and oc.cap == 80
    got = oc.scores()
    assert got.shape == (1, 3, 48)
    for g in range(3):
        rows = oc.keys()[0, g]
        assert np.array_equal(rows, data["k"][oc.positions()[0, g], g])
        x = torch.from_numpy(bf16_bits_to_f64(rows))
        cos = torch.nn.functional.cosine_similarity(x.mean(0)[None], x, dim=1).numpy()
        assert np.allclose(got[0, g], cos, rtol=1e-6, atol=1e-7)
        _, s32 = oracle.scores(rows)          # the free function, pinned on its own in test_oracle_scores
        assert np.array_equal(got[0, g], s32)
    # a cache still filling (len < N) scores exactly the rows it holds
    oc_part = oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, w.head_dim, 48, 32)
    oc_part.prefill_block(None, block_of(data["k"], 0, 20)[None], block_of(data["v"], 0, 20)[None], 0)
    x = torch.from_numpy(bf16_bits_to_f64(data["k"][:20, 1]))
    cos = torch.nn.functional.cosine_similarity(x.mean(0)[None], x, dim=1).numpy()
    assert np.allclose(oc_part.scores()[0, 1], cos, rtol=1e-6, atol=1e-7)


def test_teacher_forced_load_restores_rows_positions_and_the_next_step():
    w = get_config("toy").small(prompt_T=128, head_dim=16)
    data = make_layer(w, seed=41)
    oc = oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, w.head_dim, 48, 32)
    for t in range(0, 96, 32):
        oc.prefill_block(None, block_of(data["k"], t, 32)[None], block_of(data["v"], t, 32)[None], t)
    oc2 = oracle.OracleCache(1, w.n_q_heads, w.n_kv_heads, w.head_dim, 48, 32)
    oc2.load(oc.keys(), oc.values(), oc.positions())
    pos = oc.positions()[0, 0]
    assert oc2.len == 48 and np.array_equal(oc2.positions()[0, 0], pos)
    assert np.array_equal(oc2.keys()[0, 0], data["k"][pos, 0]) and np.array_equal(oc2.values()[0, 0], data["v"][pos, 0])
    # the step after the load, replayed by hand from the loaded rows
    k, v = block_of(data["k"], 96, 32)[None], block_of(data["v"], 96, 32)[None]
    oc2.prefill_block(None, k, v, 96)
    rows = np.concatenate([pos, np.arange(96, 128)])
    x = torch.from_numpy(bf16_bits_to_f64(data["k"][rows, 0]))
    cos = torch.nn.functional.cosine_similarity(x.mean(0)[None], x, dim=1).numpy().astype(np.float32)
    keep = np.sort(rows[np.lexsort((rows, cos))[:48]])
    assert np.array_equal(oc2.positions()[0, 0], keep)
